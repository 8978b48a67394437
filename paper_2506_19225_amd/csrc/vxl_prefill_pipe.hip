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

// The output accumulators live in the accumulation registers: their matrix instructions are
// issued from inline assembly.  The compiler does not know these instructions' latency, so every
// vector-ALU read of an accumulator is preceded by settle_acc (the rare rescale and the final
// store; the matrix pipe itself orders dependent accumulations).
__device__ __forceinline__ void mfma_acc(f32x16& o, const bf16x8& a, const bf16x8& b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(o) : "v"(a), "v"(b));
}
__device__ __forceinline__ void settle_acc(f32x16& o) {
    asm volatile("s_nop 15\n\ts_nop 15" : "+a"(o));
}

// K operand of the 16-wide d step ks for the 32 keys kb*32.. of the tile at LDS byte address `tile`
// (koff: this lane's byte offsets of its pieces in key block 0).
template <int D>
__device__ __forceinline__ bf16x8 read_k(lds_cptr ring, uint32_t tile, const uint32_t (&koff)[D / 16], int kb,
                                         int ks) {
    return *(const __attribute__((address_space(3))) bf16x8*)(ring + (tile + koff[ks]) + kb * 32 * D * 2);
}
// V^T operand (transposing LDS read) of the 16-key step (kb, j) and the 32-wide d block db.
template <int D>
__device__ __forceinline__ bf16x8 read_vt(lds_cptr ring, uint32_t tile, const uint32_t (&voff)[D / 32], int kb,
                                          int j, int db) {
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    lds_cptr p = ring + (tile + voff[db]) + (kb * 32 + j * 16) * D * 2;
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

    // this lane's operand offsets (bytes) inside a stage: K pieces of key block 0, V^T pieces of
    // the first 16-key step
    uint32_t koff[KS], voff[DB];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) koff[ks] = (uint32_t)k_tile_off<D>(l32, ks * 2 + hi) * 2;
    {
        const int dhalf = (lane >> 4) & 1, sl = lane & 15;
        const int row = 4 * hi + (sl >> 2);
        constexpr int CPR = D * 2 / 64, RPL = D == 128 ? 1 : 2;
#pragma unroll
        for (int db = 0; db < DB; ++db)
            voff[db] = (uint32_t)(C::TILE + row * D + ((db ^ ((row / RPL) & (CPR - 1))) << 5) + dhalf * 16 +
                                  4 * (sl & 3)) * 2;
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

    // Tile t -> stage t % NS.  Every wave issues 2*IPW loads: instruction slots wave, wave + 4, ...
    auto issue = [&](int t) {
        const bool own = t >= n_full && t < n_full + n_own;
        const int row0 = own ? (t - n_full) * kKeyTile : min(t, n_full) * kKeyTile;
        const int rlim = own ? min(kKeyTile - 1, sg.back + sg.q_len - 1 - row0) : kKeyTile - 1;
        const char* kb = (own ? kown : kctx_g) + (size_t)row0 * (D * 2);
        const char* vb = (own ? vown : vctx_g) + (size_t)row0 * (D * 2);
        const uint32_t st = lds_base + (uint32_t)(t % NS) * (C::STAGE * 2);
#pragma unroll
        for (int i = 0; i < C::IPW; ++i) {
            const int slot = wave + i * C::WAVES;
            const int row = slot * C::RPI + r_in;
            const uint32_t roff = (uint32_t)min(row, rlim) * (D * 2);
            const int kp = pp ^ ((row / (16 / C::PPR)) & (C::PPR - 1));
            constexpr int CPR = D * 2 / 64, RPL = D == 128 ? 1 : 2;
            const int vp = (((pp >> 2) ^ ((row / RPL) & (CPR - 1))) << 2) | (pp & 3);
            dma16(kb, roff + kp * 16, st + slot * 1024);
            dma16(vb, roff + vp * 16, st + C::TILE * 2 + slot * 1024);
        }
    };
    // top of step t: tile t+1 lands, everyone is done with tile t-2, tile t+2 is requested
    auto step_top = [&](int t) {
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        issue(min(t + 2, n_t - 1));
    };
    auto stage_of = [&](int t) -> uint32_t { return (uint32_t)(t % NS) * (C::STAGE * 2); };

    f32x16 o[2][DB];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int db = 0; db < DB; ++db) o[qb][db] = zero16();
    float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};

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
            }
    }
    __builtin_amdgcn_sched_barrier(0);

    f32x16 s0[2], s1[2];                                      // scores of the two halves of a tile
    bf16x8 p0[2][2], p1[2][2];                                // their probabilities, per row block and 16-key step

    // The rare raise of the running reference for both row blocks (exact: O and l are rescaled
    // with it), taken when some lane of the wave sees a logit more than 2^8 above its reference.
    auto raise = [&](const float (&mx)[2]) {
        const bool grow = (mx[0] - m_run[0]) * c2 > 8.f || (mx[1] - m_run[1]) * c2 > 8.f;   // true for a first finite logit
        if (__builtin_amdgcn_ballot_w64(grow) != 0) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
                for (int db = 0; db < DB; ++db) settle_acc(o[qb][db]);
                const float m_new = fmaxf(m_run[qb], mx[qb]);
                const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f((m_run[qb] - m_new) * c2);
                l_run[qb] *= alpha;
                m_run[qb] = m_new;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[qb][db][r] *= alpha;
            }
        }
    };

    // Phase A: O += P(prev half) . V in NA slices of two matrix instructions, with the row maxima of
    // s (both row blocks) spread over the slices; then the rare raise.  PV = false: maxima only.
    auto phase_a = [&](auto pv_c, uint32_t tile, int kb, const bf16x8 (&p)[2][2], const f32x16 (&s)[2]) {
        constexpr int NA = 2 * DB, VPS = 16 / NA;             // slices; score registers per slice and row block
        float mx[2] = {s[0][0], s[1][0]};
        bf16x8 a_cur, a_nxt;
        if constexpr (decltype(pv_c)::value) a_cur = read_vt<D>(ring, tile, voff, kb, 0, 0);
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int jj = i / DB, db = i % DB;
            if constexpr (decltype(pv_c)::value) {
                if (i + 1 < NA) a_nxt = read_vt<D>(ring, tile, voff, kb, (i + 1) / DB, (i + 1) % DB);
                mfma_acc(o[0][db], a_cur, p[0][jj]);
                mfma_acc(o[1][db], a_cur, p[1][jj]);
            }
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int r = i * VPS; r < (i + 1) * VPS; ++r) mx[qb] = fmaxf(mx[qb], s[qb][r]);
            if constexpr (decltype(pv_c)::value) {
                __builtin_amdgcn_sched_barrier(0);
                a_cur = a_nxt;
            }
        }
        mx[0] = fmaxf(mx[0], __shfl_xor(mx[0], 32));
        mx[1] = fmaxf(mx[1], __shfl_xor(mx[1], 32));
        raise(mx);
        __builtin_amdgcn_sched_barrier(0);
    };
    // Phase B: s_dst = K(32 keys) . Q^T in KS slices of two matrix instructions, with the
    // exponentials of s_src -> p_dst (bf16, B-operand order) spread over the slices.
    auto phase_b = [&](uint32_t tile, int kb, f32x16 (&s_dst)[2], const f32x16 (&s_src)[2], bf16x8 (&p_dst)[2][2]) {
        constexpr int VPS = 16 / KS;                          // score registers per slice and row block (2 or 4)
        const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
        float mc[2], sum[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) mc[qb] = (m_run[qb] == -INFINITY ? 0.f : m_run[qb]) * c2;
        bf16x8 a_cur = read_k<D>(ring, tile, koff, kb, 0), a_nxt;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ks + 1 < KS) a_nxt = read_k<D>(ring, tile, koff, kb, ks + 1);
            if (ks == 0) {
                s_dst[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_cur, qreg[0][ks], zero16(), 0, 0, 0);
                s_dst[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_cur, qreg[1][ks], zero16(), 0, 0, 0);
            } else {
                s_dst[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_cur, qreg[0][ks], s_dst[0], 0, 0, 0);
                s_dst[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_cur, qreg[1][ks], s_dst[1], 0, 0, 0);
            }
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int r = ks * VPS; r < (ks + 1) * VPS; r += 2) {
                    bf16x2 pr;
                    pr[0] = (__bf16)__builtin_amdgcn_exp2f(fmaf(s_src[qb][r], c2, -mc[qb]));
                    pr[1] = (__bf16)__builtin_amdgcn_exp2f(fmaf(s_src[qb][r + 1], c2, -mc[qb]));
                    sum[qb][(r >> 1) & 1] = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, sum[qb][(r >> 1) & 1], false);
                    p_dst[qb][r >> 3][r & 7] = pr[0];
                    p_dst[qb][r >> 3][(r & 7) + 1] = pr[1];
                }
            __builtin_amdgcn_sched_barrier(0);
            a_cur = a_nxt;
        }
        l_run[0] += sum[0][0] + sum[0][1];
        l_run[1] += sum[1][0] + sum[1][1];
        __builtin_amdgcn_sched_barrier(0);
    };
    typedef std::integral_constant<bool, true> yes;
    typedef std::integral_constant<bool, false> no;

    int t = 0;
    if (n_pipe > 0) {
        // first pipelined tile: nothing is owed to O yet
        step_top(0);
        // S(0, half 0)
        {
            bf16x8 a_cur = read_k<D>(ring, stage_of(0), koff, 0, 0);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                bf16x8 a_nxt = a_cur;
                if (ks + 1 < KS) a_nxt = read_k<D>(ring, stage_of(0), koff, 0, ks + 1);
                if (ks == 0) {
                    s0[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_cur, qreg[0][ks], zero16(), 0, 0, 0);
                    s0[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_cur, qreg[1][ks], zero16(), 0, 0, 0);
                } else {
                    s0[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_cur, qreg[0][ks], s0[0], 0, 0, 0);
                    s0[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_cur, qreg[1][ks], s0[1], 0, 0, 0);
                }
                a_cur = a_nxt;
            }
        }
        phase_a(no(), 0u, 0, p1, s0);
        phase_b(stage_of(0), 1, s1, s0, p0);
        phase_a(yes(), stage_of(0), 0, p0, s1);
        phase_b(stage_of(1), 0, s0, s1, p1);                  // (operands are whatever the stage holds if n_pipe == 1)
        for (t = 1; t < n_pipe; ++t) {
            step_top(t);
            phase_a(yes(), stage_of(t - 1), 1, p1, s0);
            phase_b(stage_of(t), 1, s1, s0, p0);
            phase_a(yes(), stage_of(t), 0, p0, s1);
            phase_b(stage_of(t + 1), 0, s0, s1, p1);
        }
        // the last half's product
        {
            const uint32_t tile = stage_of(n_pipe - 1);
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const bf16x8 a = read_vt<D>(ring, tile, voff, 1, jj, db);
                    mfma_acc(o[0][db], a, p1[0][jj]);
                    mfma_acc(o[1][db], a, p1[1][jj]);
                }
        }
    }
    // the remaining steps: masked tiles one after the other, other tiles only pass through the ring
    for (; t < n_t; ++t) {
        step_top(t);
        const bool own = t >= n_full && t < n_full + n_own;
        const bool mine = wave_rows && (own ? t < own_end : true);     // (not own => the ragged history tile)
        if (!mine) continue;
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
#pragma unroll
                for (int r = 0; r < 16; ++r) s[qb][r] = acc_key(kb, r, hi) <= lim ? s[qb][r] : -INFINITY;
                mx[qb] = s[qb][0];
#pragma unroll
                for (int r = 1; r < 16; ++r) mx[qb] = fmaxf(mx[qb], s[qb][r]);
                mx[qb] = fmaxf(mx[qb], __shfl_xor(mx[qb], 32));
            }
            raise(mx);
            const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                const float mc = (m_run[qb] == -INFINITY ? 0.f : m_run[qb]) * c2;
                float sum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    bf16x2 pr;
                    pr[0] = (__bf16)__builtin_amdgcn_exp2f(fmaf(s[qb][r], c2, -mc));
                    pr[1] = (__bf16)__builtin_amdgcn_exp2f(fmaf(s[qb][r + 1], c2, -mc));
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
                (LSE + (size_t)h * n_tokens + sg.q_start)[q_off] = m_run[qb] * scale + logf(l_tot);
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
