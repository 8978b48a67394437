// Chunk-based pre-filling attention, software-pipelined form: 4 waves per workgroup (one per
// SIMD, more than 256 registers each), 64 query rows (two 32-row blocks) per wave, 256 rows per
// workgroup.  Every K/V operand read from LDS feeds two matrix instructions (one per row block),
// which halves the LDS traffic per FLOP of the 32-rows-per-wave kernels, and the overlap of
// vector and matrix work is arranged inside one instruction stream instead of being left to two
// waves of a SIMD drifting apart.  The loop body handles the two 32-key halves of a tile; each of
// its four phases pairs the matrix work of a neighbouring half with the vector work of the
// current one,
//
//     A0:  O += P(t-1, half 1) . V        |  row maxima of S(t, half 0)
//     B0:  S(t, half 1)   = K . Q^T       |  exponentials of S(t, half 0)   -> P(t, half 0)
//     A1:  O += P(t, half 0) . V          |  row maxima of S(t, half 1)
//     B1:  S(t+1, half 0) = K . Q^T       |  exponentials of S(t, half 1)   -> P(t, half 1)
//
// and every phase is written as slices (one operand read for the next slice, two matrix
// instructions, a share of the vector work) separated by scheduling fences, so the interleaving
// is the source order.  The (rare, wave-uniform) rescale of the running reference sits between A
// and B, where O holds exactly the products of all earlier halves.
//
// Only tiles that need no mask run through the pipeline.  The ring serves the tiles in the order
// [full history tiles][own tiles][ragged last history tile]; a wave pipelines the full history
// tiles and the own tiles that lie entirely below its rows, and handles its diagonal tile(s) and
// the ragged history tile one after the other in a plain sequential form (the order of the tiles
// does not matter to the online softmax).
//
// Tiles stream through a 4-stage LDS ring of direct global->LDS loads: tile t+2 is issued at the
// top of step t, after the one workgroup barrier per tile that (a) makes tile t+1 visible and (b)
// proves every wave has finished with tile t-2, whose stage is refilled.  Every wait on the ring
// is vmcnt(0).  The score products (builtins) land in ordinary vector registers, where the vector
// ALU needs them; the output accumulators are kept in the accumulation registers by issuing their
// matrix instructions from inline assembly.  Work distribution (persistent workgroups, queues
// per KV-head group) is that of prefill_dma_kernel.
#include <math.h>

#include <algorithm>
#include <type_traits>

#include "vxl_internal.h"
#include "vxl_mfma.h"

namespace vxl {

namespace {

// Measurement builds only (VXL_PIPE_ABL in the environment of the build script): bit 0 leaves out
// the exponentials, bit 1 the exponent / maximum / row-sum work, bit 2 the ring loads inside the
// loop -- the results are then wrong, all accesses stay in bounds -- and bit 5 adds up the clock
// ticks of the four phases and the barrier per wave and stores the totals behind the LSE array
// (which the caller must then make 64 floats longer).
#ifndef VXL_PIPE_ABL
#define VXL_PIPE_ABL 0
#endif

template <int D>
struct PipeCfg {
    static constexpr int WAVES = 4;
    static constexpr int BM = 64 * WAVES;                     // query rows per workgroup
    static constexpr int NS = 4;                              // ring stages
    static constexpr int TILE = kKeyTile * D;                 // elements of one unpadded K (or V) tile
    static constexpr int STAGE = 2 * TILE;                    // K tile then V tile
    static constexpr int LDS_BYTES = NS * STAGE * 2 + 16;     // the ring and the slot of the work index
    static constexpr int PPR = D / 8;                         // 16-byte pieces per row
    static constexpr int RPI = 64 / PPR;                      // rows per load instruction (1 KiB)
    static constexpr int NI = kKeyTile / RPI;                 // instructions per tile per matrix
    static constexpr int IPW = NI / WAVES;                    // ... per wave
    static constexpr int KS = D / 16;                         // 16-wide d steps of S = K.Q^T
    static constexpr int DB = D / 32;                         // 32-wide d blocks of O
};

typedef __attribute__((address_space(3))) const char* lds_cptr;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// All matrix products go through the compiler's builtins (at one wave per SIMD their results are
// placed in the accumulation registers; the vector ALU reads the scores from there).
__device__ __forceinline__ void mfma_acc(f32x16& o, const bf16x8& a, const bf16x8& b) {
    o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, o, 0, 0, 0);
}
__device__ __forceinline__ void settle_acc(f32x16&) {}

// K operand of the 16-wide d step ks for the 32 keys kb*32.. of the tile at LDS byte offset `tile`.
// koff: this lane's byte offset of its piece for ks = 0 in key block 0; the XOR swizzle of the
// 16-byte pieces commutes with the d step (bits 5..), so the other steps are one XOR away, and
// the key block and the tile only add multiples of 256.
template <int D>
__device__ __forceinline__ bf16x8 read_k(lds_cptr ring, uint32_t tile, uint32_t koff, int kb, int ks) {
    return *(const __attribute__((address_space(3))) bf16x8*)(ring + ((tile + koff) ^ (uint32_t)(ks << 5)) +
                                                               kb * 32 * D * 2);
}
// V^T operand (transposing LDS read) of the 16-key step (kb, j) and the 32-wide d block db; voff:
// this lane's byte offset for db = 0 in the first 16-key step (the swizzle of the 64-byte chunks
// commutes with db in the same way).
template <int D>
__device__ __forceinline__ bf16x8 read_vt(lds_cptr ring, uint32_t tile, uint32_t voff, int kb, int j, int db) {
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    lds_cptr p = ring + ((tile + voff) ^ (uint32_t)(db << 6)) + (kb * 32 + j * 16) * D * 2;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
    const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 8 * D * 2));   // row + 8: same swizzle
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
}

template <int D>
__global__ __launch_bounds__(256, 1) void prefill_pipe_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    const uint16_t* __restrict__ Kctx, const uint16_t* __restrict__ Vctx, uint16_t* __restrict__ O,
    float* __restrict__ LSE, const Segment* __restrict__ segs, const WorkItem* __restrict__ work,
    int n_tokens, int n_q_heads, int group, int ctx_rows_pad, float scale, int n_items, int xpg,
    int* __restrict__ queue) {
    using C = PipeCfg<D>;
    constexpr int NS = C::NS, KS = C::KS, DB = C::DB;
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds;
    lds_cptr ring = (lds_cptr)(__attribute__((address_space(3))) void*)lds;
    int* next_slot = (int*)(lds + NS * C::STAGE);

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int qid = xpg > 0 ? (int)(blockIdx.x & 7) / xpg : 0;            // this workgroup's queue
    const int q_len_items = xpg > 0 ? n_items * group : n_items * n_q_heads;
    const float c2 = scale * kLog2e;
    const int r_in = lane / C::PPR, pp = lane % C::PPR;

    // this lane's operand offsets (bytes) inside a stage: its K piece of d step 0 in key block 0,
    // its V^T piece of d block 0 in the first 16-key step
    const uint32_t koff = (uint32_t)k_tile_off<D>(l32, hi) * 2;
    uint32_t voff;
    {
        const int dhalf = (lane >> 4) & 1, sl = lane & 15;
        const int row = 4 * hi + (sl >> 2);
        constexpr int CPR = D * 2 / 64, RPL = D == 128 ? 1 : 2;
        voff = (uint32_t)(C::TILE + row * D + (((row / RPL) & (CPR - 1)) << 5) + dhalf * 16 + 4 * (sl & 3)) * 2;
    }

    if (tid == 0) next_slot[0] = atomicAdd(queue + qid, 1);
    __syncthreads();
    int j = __builtin_amdgcn_readfirstlane(next_slot[0]);
  for (int par = 1; j < q_len_items; par ^= 1) {
    const int item = xpg > 0 ? j / group : j / n_q_heads;
    const int h = xpg > 0 ? qid * group + j % group : j % n_q_heads;
    const int g = h / group;
    const WorkItem wi = work[item];
    const Segment sg = segs[wi.seg];
    const int m0 = wi.m_tile * C::BM;
    const int wrow0 = m0 + wave * 64;                         // first query row (segment-relative) of this wave
    const int last_row = min(m0 + C::BM, sg.q_len) - 1;
    // ring order: full history tiles, own tiles (keys start `back` rows before the segment), then
    // the ragged last history tile
    const int n_full = sg.ctx_len / kKeyTile;
    const int n_own = (last_row + sg.back) / kKeyTile + 1;
    const bool has_rag = (sg.ctx_len % kKeyTile) != 0;
    const int n_t = n_full + n_own + (has_rag ? 1 : 0);
    const bool wave_rows = wrow0 < sg.q_len;
    // pipelined: the full history tiles and the own tiles entirely visible to the wave's first row
    const int n_pipe = wave_rows ? n_full + min((wrow0 + sg.back + 1) / kKeyTile, n_own) : 0;
    // sequential: own tiles from there up to the diagonal of the wave's last row, and the ragged tile
    const int own_end = wave_rows ? n_full + (min(wrow0 + 63, sg.q_len - 1) + sg.back) / kKeyTile + 1 : 0;

    const char* kctx_g = (const char*)(Kctx + (size_t)g * ctx_rows_pad * D);
    const char* vctx_g = (const char*)(Vctx + (size_t)g * ctx_rows_pad * D);
    const char* kown = (const char*)(K + ((size_t)g * n_tokens + sg.q_start - sg.back) * D);
    const char* vown = (const char*)(V + ((size_t)g * n_tokens + sg.q_start - sg.back) * D);

    // Source of ring tile t (stage t % NS): pointers to its first K and V row, last valid row.
    struct TileSrc { const char* kb; const char* vb; int rlim; uint32_t st; };
    auto tile_src = [&](int t) -> TileSrc {
        const bool own = t >= n_full && t < n_full + n_own;
        const int row0 = own ? (t - n_full) * kKeyTile : min(t, n_full) * kKeyTile;
        TileSrc ts;
        ts.rlim = own ? min(kKeyTile - 1, sg.back + sg.q_len - 1 - row0) : kKeyTile - 1;
        ts.kb = (own ? kown : kctx_g) + (size_t)row0 * (D * 2);
        ts.vb = (own ? vown : vctx_g) + (size_t)row0 * (D * 2);
        ts.st = lds_base + (uint32_t)(t % NS) * (C::STAGE * 2);
        return ts;
    };
    // The i-th of the 2*IPW loads this wave contributes to a tile (instruction slots wave, wave + 4,
    // ...; even i: K, odd i: V).  Rows beyond rlim are clamped to it.
    auto issue_one = [&](const TileSrc& ts, int i) {
        const int slot = wave + (i >> 1) * C::WAVES;
        const int row = slot * C::RPI + r_in;
        const uint32_t roff = (uint32_t)min(row, ts.rlim) * (D * 2);
        if ((i & 1) == 0) {
            const int kp = pp ^ ((row / (16 / C::PPR)) & (C::PPR - 1));
            dma16(ts.kb, roff + kp * 16, ts.st + slot * 1024);
        } else {
            constexpr int CPR = D * 2 / 64, RPL = D == 128 ? 1 : 2;
            const int vp = (((pp >> 2) ^ ((row / RPL) & (CPR - 1))) << 2) | (pp & 3);
            dma16(ts.vb, roff + vp * 16, ts.st + C::TILE * 2 + slot * 1024);
        }
    };
    auto issue = [&](int t) {
        const TileSrc ts = tile_src(t);
#pragma unroll
        for (int i = 0; i < 2 * C::IPW; ++i) issue_one(ts, i);
    };
    // The one workgroup barrier of step t: behind it tile t+1 is in LDS for everybody (every wave
    // has waited for its own loads of it; only the loads of tile t+2, requested during this step,
    // may still be in flight) and everybody is done with tile t-1's K and tile t-2 (so the stage of
    // tile t-2 may be refilled with tile t+2 in step t+1... and is, at its start).  A pipelined
    // wave places it before its last phase (the first to touch tile t+1), a sequential wave at
    // the end of its step.
    constexpr int NLD = 2 * C::IPW;                           // ring loads per wave and tile
    auto step_barrier = [&]() {
        wait_vmcnt<NLD>();
        __builtin_amdgcn_s_barrier();
    };
    auto stage_of = [&](int t) -> uint32_t { return (uint32_t)(t % NS) * (C::STAGE * 2); };

    f32x16 o[2][DB];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int db = 0; db < DB; ++db) o[qb][db] = zero16();
    // running reference of a row in the exp2 domain (scaled logit * log2 e) and this lane's half
    // of the running sum
    float m2[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};

    issue(0);
    issue(min(1, n_t - 1));

    // Query rows: loaded after the ring has been started and forced complete here; the compiler's
    // wait for them covers the older ring loads as well.
    bf16x8 qreg[2][KS];
    {
        const char* qbase = (const char*)(Q + ((size_t)h * n_tokens + sg.q_start) * D);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const uint32_t qoff = (uint32_t)min(wrow0 + qb * 32 + l32, sg.q_len - 1) * (D * 2) + hi * 16;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                qreg[qb][ks] = __builtin_bit_cast(bf16x8, *(const uint4*)(qbase + qoff + ks * 32));
        }
        // the index of the item after this one is fetched in the same wait and read when this item is done
        if (tid == 0) next_slot[par] = atomicAdd(queue + qid, 1);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
                asm volatile("" :: "v"(__builtin_bit_cast(u32x4, qreg[qb][ks])));
                asm volatile("" : "+a"(qreg[qb][ks]));       // the queries stay in the accumulation registers
            }
    }
    __builtin_amdgcn_s_barrier();                             // tiles 0 and 1 are in LDS for everybody
    __builtin_amdgcn_sched_barrier(0);

    // s0 / s1: the two halves of a tile -- raw scores when a phase B has written them, exponents
    // x = score*c2 - reference once a phase A has gone over them.  p0 / p1: their probabilities,
    // per row block and 16-key step.
    f32x16 s0[2], s1[2];
    bf16x8 p0[2][2], p1[2][2];
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};

    // A lane asks for a raise of the running reference when one of its own exponents exceeds 8
    // (probabilities stay below 2^8, which fp32 and bf16 carry at unchanged relative precision) or
    // when the row has no reference yet; the decision is wave-uniform (ballot), so the common path
    // has no cross-lane traffic.  The raise itself is exact: O, l and the exponents at hand are
    // moved to the new reference.
    auto wants_raise = [&](const float (&mx)[2]) -> bool {
        return mx[0] > 8.f || mx[1] > 8.f || (m2[0] == -INFINITY && mx[0] > -INFINITY) ||
               (m2[1] == -INFINITY && mx[1] > -INFINITY);
    };
    auto raise = [&](const float (&mx)[2], f32x16 (&x)[2]) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
            for (int db = 0; db < DB; ++db) settle_acc(o[qb][db]);
            const float row_mx = fmaxf(mx[qb], __shfl_xor(mx[qb], 32));
            const float old_g = m2[qb] == -INFINITY ? 0.f : m2[qb];
            const float m_new = fmaxf(m2[qb], old_g + row_mx);
            const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m2[qb] - m_new);
            const float shift = (m_new == -INFINITY ? 0.f : m_new) - old_g;
            l_run[qb] *= alpha;
            m2[qb] = m_new;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[qb][db][r] *= alpha;
#pragma unroll
            for (int r = 0; r < 16; ++r) x[qb][r] -= shift;
        }
    };

    // Operand queue of the pipelined phases: the operands of a phase's slices 0 and 1 are requested
    // by the last two slices of the phase before it.
    struct OpQ { bf16x8 c, n; };
    constexpr int NA = 2 * DB;                                // slices of a phase A (2 or 4 matrix instruction pairs per 16-key step)
    static_assert(NA == 2 * C::IPW, "one ring load per slice of a phase A");

    // Phase A: O += P . V (32 keys kb*32.. of the tile at tv; P = p, whose row sums are added to l
    // here) in 2*NA slices of ONE matrix instruction each: a wave issues in order, so two matrix
    // instructions in a row would stall it for the length of the first, and the vector work is
    // spread evenly between them instead.  Per slice: a share of s -> exponents x = s*c2 - reference
    // with their lane maxima, a share of the row sums, and (DMA) one of this wave's ring loads of
    // tile ts.  The last slices request the first operands of the phase B that follows (tile tk, key
    // block kbk).  Then the raise of the reference: rare, except in the first half of an item
    // (PV = false: no product is owed yet), where every row gets its reference.
    auto phase_a = [&](auto pv_c, auto dma_c, uint32_t tv, int kb, const bf16x8 (&p)[2][2], f32x16 (&s)[2],
                       OpQ& q, uint32_t tk, int kbk, const TileSrc& ts) {
        constexpr bool PV = decltype(pv_c)::value, DMA = decltype(dma_c)::value;
        constexpr int VPS = 16 / NA;                          // score registers per operand step and row block
        float mx[2] = {-INFINITY, -INFINITY}, sum[2] = {0.f, 0.f};
        const float nmc[2] = {m2[0] == -INFINITY ? 0.f : -m2[0], m2[1] == -INFINITY ? 0.f : -m2[1]};
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int jj = i / DB, db = i % DB;
            bf16x8 nxt;
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                if (qb == 0) {
                    if (i + 2 < NA) { if constexpr (PV) nxt = read_vt<D>(ring, tv, voff, kb, (i + 2) / DB, (i + 2) % DB); }
                    else nxt = read_k<D>(ring, tk, koff, kbk, i + 2 - NA);
                }
                if constexpr (PV) mfma_acc(o[qb][db], q.c, p[qb][jj]);
                if constexpr (DMA && !(VXL_PIPE_ABL & 4)) { if (qb == 1) issue_one(ts, i); }
                if constexpr (!(VXL_PIPE_ABL & 2)) {
#pragma unroll
                    for (int r = i * VPS; r < (i + 1) * VPS; ++r) {
                        s[qb][r] = fmaf(s[qb][r], c2, nmc[qb]);
                        mx[qb] = fmaxf(mx[qb], s[qb][r]);
                    }
                    if constexpr (PV) {
                        // row sums of p[qb]: 8 dwords (2 steps x 4), 8 / NA per slice
#pragma unroll
                        for (int w = i * (8 / NA); w < (i + 1) * (8 / NA); ++w) {
                            typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
                            const u32x4 pw = __builtin_bit_cast(u32x4, p[qb][w >> 2]);
                            const int dw = w & 3;
                            const unsigned one_dw = dw == 0 ? pw.x : dw == 1 ? pw.y : dw == 2 ? pw.z : pw.w;
                            sum[qb] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, one_dw), ones, sum[qb], false);
                        }
                    }
                } else if (i == 0) {
                    mx[qb] = s[qb][0];
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            q.c = q.n;
            q.n = nxt;
        }
        if constexpr (PV) {
            l_run[0] += sum[0];
            l_run[1] += sum[1];
            // every row has its reference by now (set at the item's first half)
            if (__builtin_amdgcn_ballot_w64(fmaxf(mx[0], mx[1]) > 8.f) != 0) raise(mx, s);
        } else {
            raise(mx, s);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    // Phase B: s_dst = K(32 keys kb*32.. of the tile at tk) . Q^T in 2*KS slices of one matrix
    // instruction, with the exponentials of x -> p_dst (bf16, B-operand order) spread over the
    // slices.  The last slices request the first operands of the phase A that follows (tile tv, key
    // block kbv).
    auto phase_b = [&](uint32_t tk, int kb, f32x16 (&s_dst)[2], const f32x16 (&x)[2], bf16x8 (&p_dst)[2][2],
                       OpQ& q, uint32_t tv, int kbv) {
        constexpr int VPS = 16 / KS;                          // score registers per d step and row block (2 or 4)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bf16x8 nxt;
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                if (qb == 0) {
                    if (ks + 2 < KS) nxt = read_k<D>(ring, tk, koff, kb, ks + 2);
                    else nxt = read_vt<D>(ring, tv, voff, kbv, (ks + 2 - KS) / DB, (ks + 2 - KS) % DB);
                }
                if (ks == 0) s_dst[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q.c, qreg[qb][ks], zero16(), 0, 0, 0);
                else s_dst[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q.c, qreg[qb][ks], s_dst[qb], 0, 0, 0);
                if constexpr (!(VXL_PIPE_ABL & 1)) {
#pragma unroll
                    for (int r = ks * VPS; r < (ks + 1) * VPS; r += 2) {
                        p_dst[qb][r >> 3][r & 7] = (__bf16)__builtin_amdgcn_exp2f(x[qb][r]);
                        p_dst[qb][r >> 3][(r & 7) + 1] = (__bf16)__builtin_amdgcn_exp2f(x[qb][r + 1]);
                    }
                } else if (ks == 0) {
                    asm volatile("" : "+v"(p_dst[qb][0]) : "v"(x[qb]));
                    asm volatile("" : "+v"(p_dst[qb][1]));
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            q.c = q.n;
            q.n = nxt;
        }
    };
    typedef std::integral_constant<bool, true> yes;
    typedef std::integral_constant<bool, false> no;

    int t = 0;
    if (n_pipe > 0) {
        // first pipelined tile: S(0, half 0) computed up front, nothing is owed to O yet
        {
            const uint32_t tk = stage_of(0);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 a = read_k<D>(ring, tk, koff, 0, ks);
                if (ks == 0) {
                    s0[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[0][ks], zero16(), 0, 0, 0);
                    s0[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[1][ks], zero16(), 0, 0, 0);
                } else {
                    s0[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[0][ks], s0[0], 0, 0, 0);
                    s0[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[1][ks], s0[1], 0, 0, 0);
                }
            }
        }
        OpQ q;
        {
            const TileSrc ts = tile_src(min(2, n_t - 1));
            phase_a(no(), yes(), 0u, 0, p1, s0, q, stage_of(0), 1, ts);
        }
        phase_b(stage_of(0), 1, s1, s0, p0, q, stage_of(0), 0);
        phase_a(yes(), no(), stage_of(0), 0, p0, s1, q, stage_of(1), 0, TileSrc());
        step_barrier();
        phase_b(stage_of(1), 0, s0, s1, p1, q, stage_of(0), 1);
#if VXL_PIPE_ABL & 32
        unsigned long long pc[7] = {0, 0, 0, 0, 0, 0, 0};     // measurement build: cycles per phase
#define VXL_TICK(k_) do { const unsigned long long n_ = clock64(); pc[k_] += n_ - tk_; tk_ = n_; } while (0)
#else
#define VXL_TICK(k_) do {} while (0)
#endif
        for (t = 1; t < n_pipe; ++t) {
#if VXL_PIPE_ABL & 32
            unsigned long long tk_ = clock64();
#endif
            const TileSrc ts = tile_src(min(t + 2, n_t - 1));
            VXL_TICK(0);
            phase_a(yes(), yes(), stage_of(t - 1), 1, p1, s0, q, stage_of(t), 1, ts);
            VXL_TICK(1);
            phase_b(stage_of(t), 1, s1, s0, p0, q, stage_of(t), 0);
            VXL_TICK(2);
            phase_a(yes(), no(), stage_of(t), 0, p0, s1, q, stage_of(t + 1), 0, ts);
            VXL_TICK(3);
            step_barrier();
            VXL_TICK(4);
            phase_b(stage_of(t + 1), 0, s0, s1, p1, q, stage_of(t), 1);
            VXL_TICK(5);
#if VXL_PIPE_ABL & 32
            pc[6] += 1;
#endif
        }
#if VXL_PIPE_ABL & 32
        if (LSE && lane == 0)
            for (int k_ = 0; k_ < 7; ++k_) atomicAdd((unsigned long long*)(LSE + (size_t)n_q_heads * n_tokens) + k_, pc[k_]);
#endif
#undef VXL_TICK
        // the last half's product (its first two operands are in the queue)
        {
            const uint32_t tv = stage_of(n_pipe - 1);
            float sum[2] = {0.f, 0.f};
#pragma unroll
            for (int i = 0; i < NA; ++i) {
                const int jj = i / DB, db = i % DB;
                const bf16x8 a = i == 0 ? q.c : (i == 1 ? q.n : read_vt<D>(ring, tv, voff, 1, jj, db));
                mfma_acc(o[0][db], a, p1[0][jj]);
                mfma_acc(o[1][db], a, p1[1][jj]);
            }
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int st = 0; st < 2; ++st)
#pragma unroll
                    for (int dw = 0; dw < 4; ++dw) {
                        bf16x2 pr;
                        pr[0] = p1[qb][st][2 * dw];
                        pr[1] = p1[qb][st][2 * dw + 1];
                        sum[qb] = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, sum[qb], false);
                    }
            l_run[0] += sum[0];
            l_run[1] += sum[1];
        }
    }
    // the remaining steps: masked tiles one after the other, other tiles only pass through the ring
    for (; t < n_t; ++t) {
        issue(min(t + 2, n_t - 1));
        const bool own = t >= n_full && t < n_full + n_own;
        const bool mine = wave_rows && (own ? t < own_end : true);     // (not own => the ragged history tile)
        if (!mine) { step_barrier(); continue; }
        const int key0 = own ? (t - n_full) * kKeyTile : n_full * kKeyTile;
        const uint32_t tile = stage_of(t);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            f32x16 (&s)[2] = s0;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 a = read_k<D>(ring, tile, koff, kb, ks);
                if (ks == 0) {
                    s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[0][ks], zero16(), 0, 0, 0);
                    s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[1][ks], zero16(), 0, 0, 0);
                } else {
                    s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[0][ks], s[0], 0, 0, 0);
                    s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[1][ks], s[1], 0, 0, 0);
                }
            }
            float mx[2];
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                // tile-relative key kt is visible iff kt <= lim
                const int lim = own ? wrow0 + sg.back + qb * 32 + l32 - key0 : sg.ctx_len - key0 - 1;
                const float nmc = m2[qb] == -INFINITY ? 0.f : -m2[qb];
                mx[qb] = -INFINITY;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    s[qb][r] = acc_key(kb, r, hi) <= lim ? fmaf(s[qb][r], c2, nmc) : -INFINITY;
                    mx[qb] = fmaxf(mx[qb], s[qb][r]);
                }
            }
            if (__builtin_amdgcn_ballot_w64(wants_raise(mx)) != 0) raise(mx, s);
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                float sum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    bf16x2 pr;
                    pr[0] = (__bf16)__builtin_amdgcn_exp2f(s[qb][r]);
                    pr[1] = (__bf16)__builtin_amdgcn_exp2f(s[qb][r + 1]);
                    sum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, sum, false);
                    p0[qb][r >> 3][r & 7] = pr[0];
                    p0[qb][r >> 3][(r & 7) + 1] = pr[1];
                }
                l_run[qb] += sum;
            }
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const bf16x8 a = read_vt<D>(ring, tile, voff, kb, jj, db);
                    mfma_acc(o[0][db], a, p0[0][jj]);
                    mfma_acc(o[1][db], a, p0[1][jj]);
                }
        }
        step_barrier();
    }
    wait_vmcnt<0>();                                          // drain the refills before the next item

#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
        for (int db = 0; db < DB; ++db) settle_acc(o[qb][db]);
        const int q_off = wrow0 + qb * 32 + l32;
        const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32);
        if (q_off < sg.q_len) {
            const float inv = 1.f / l_tot;
            char* obase = (char*)(O + ((size_t)h * n_tokens + sg.q_start) * D);
            const uint32_t ooff = (uint32_t)q_off * (D * 2) + hi * 8;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    bf16x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (__bf16)(o[qb][db][rq * 4 + e] * inv);
                    *(bf16x4*)(obase + ooff + (db * 32 + rq * 8) * 2) = v;
                }
            if (LSE && hi == 0)
                (LSE + (size_t)h * n_tokens + sg.q_start)[q_off] = m2[qb] * kLn2 + logf(l_tot);
        }
    }
    __syncthreads();                    // every wave is done with this item's tiles; next_slot[par] is written
    j = __builtin_amdgcn_readfirstlane(next_slot[par]);
  }
}

}  // namespace

template <int D>
static vxl_status run_prefill_pipe(const vxl_layout* L, const vxl_attn_desc* d, float scale, const void* Q,
                                   const void* K, const void* V, const uint16_t* kctx, const uint16_t* vctx,
                                   void* O, float* LSE, int* queue, hipStream_t s) {
    using C = PipeCfg<D>;
    static bool attr_done = false;
    if (!attr_done) {
        VXL_HIP_TRY(hipFuncSetAttribute((const void*)prefill_pipe_kernel<D>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
        attr_done = true;
    }
    static int n_cus = 0;                                     // one persistent workgroup per compute unit
    if (n_cus == 0) {
        int dev = 0;
        VXL_HIP_TRY(hipGetDevice(&dev));
        VXL_HIP_TRY(hipDeviceGetAttribute(&n_cus, hipDeviceAttributeMultiprocessorCount, dev));
        if (n_cus < 8) n_cus = 8;
    }
    const int group = d->n_q_heads / d->n_kv_heads;
    const int xpg = 8 % d->n_kv_heads == 0 ? 8 / d->n_kv_heads : 0;
    const long long n_pairs = (long long)L->n_work[1] * d->n_q_heads;
    const unsigned n_blocks = (unsigned)std::min<long long>(n_cus / 8 * 8, xpg ? (n_pairs + 7) / 8 * 8 : n_pairs);
    hipLaunchKernelGGL((prefill_pipe_kernel<D>), dim3(n_blocks), dim3(256), C::LDS_BYTES, s, (const uint16_t*)Q,
                       (const uint16_t*)K, (const uint16_t*)V, kctx, vctx, (uint16_t*)O, LSE, L->d_segs,
                       L->d_work[1], L->n_tokens, d->n_q_heads, group, L->n_ctx_tiles * kKeyTile, scale,
                       L->n_work[1], xpg, queue);
    VXL_HIP_TRY(hipGetLastError());
    return VXL_OK;
}

vxl_status launch_prefill_pipe_main(const vxl_layout* L, const vxl_attn_desc* d, float scale, const void* Q,
                                    const void* K, const void* V, const uint16_t* kctx, const uint16_t* vctx,
                                    void* O, float* LSE, int* queue, hipStream_t s) {
    return d->head_dim == 128 ? run_prefill_pipe<128>(L, d, scale, Q, K, V, kctx, vctx, O, LSE, queue, s)
                              : run_prefill_pipe<64>(L, d, scale, Q, K, V, kctx, vctx, O, LSE, queue, s);
}

}  // namespace vxl
