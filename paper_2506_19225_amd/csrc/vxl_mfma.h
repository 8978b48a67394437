// Device building blocks of the matrix-core attention kernels (gfx950, wave64).
//
// Both kernels compute the scores transposed, S^T = K.Q^T with v_mfma_f32_32x32x16_bf16:
//   A operand (K tile, from LDS): lane (l32, hi) holds K[key = l32][d = 16*ks + 8*hi .. +7]
//   B operand (Q, in registers):  lane (l32, hi) holds Q[query = l32][d = 16*ks + 8*hi .. +7]
//   accumulator: lane (l32, hi), register r holds S^T[key = 8*(r/4) + 4*hi + r%4][query = l32]
// so a lane owns one query column (its partner lane ^ 32 owns the other half of the keys) and
// the softmax statistics need one cross-lane exchange.  The probabilities then feed the second
// product O^T = V^T.P^T directly as its B operand: for the 16-key step j of a 32-key block the
// registers r = 8j .. 8j+7 of a lane are the keys 16j + 4*hi + {0,1,2,3, 8,9,10,11}.  The A
// operand V^T[d][those keys] is produced from a row-major V tile in LDS by the transposing LDS
// read (ds_read_b64_tr_b16): inside a group of 16 lanes, lane i receives element (i % 4) of the
// 8-byte pieces addressed by lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4.
#pragma once

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

namespace vxl {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// LDS row strides (in elements) of the row-major K and V tiles.  Measured on gfx950, the LDS
// behaves as 32 banks of 8 bytes, each half-wave (lanes 0-31, lanes 32-63) served separately:
// an access pattern runs at full rate when the 8-byte pieces touched by the 32 lanes of a
// half-wave fall into distinct banks.  The K operand read (lane = row, 16 bytes at a common
// column) needs an odd stride in 8-byte units: D*2 + 8 bytes.  The transposing V read (4 rows x
// 64 contiguous bytes per half-wave) needs the stride to be 8 or 24 (mod 32) units: 320 bytes
// for D = 128, 192 bytes for D = 64.
template <int D> struct LdsRows {
    static constexpr int K = D;                       // unpadded; pieces are XOR-swizzled instead
    static constexpr int V = D == 128 ? 160 : 96;
};

// Element offset of 16-byte piece `piece` of row `row` in the K tile.  Rows are unpadded (so
// every piece stays 16-byte aligned) and the piece index is XOR-ed with the row's position
// inside a group of 16 256-byte lines: the 32 rows a half-wave reads at one logical piece then
// cover every bank exactly twice, which is the full rate of a 16-byte access.
template <int D>
__device__ __forceinline__ int k_tile_off(int row, int piece) {
    constexpr int PPR = D / 8;                        // pieces per row
    constexpr int RPL = 16 / PPR;                     // rows per 256-byte line
    return row * D + ((piece ^ ((row / RPL) & (PPR - 1))) << 3);
}

// Register staging of one 64-key K tile and V tile by a 256-thread workgroup: every thread
// carries D/32 16-byte pieces of each.  The pieces are named members, not an array: they have to
// live in VGPRs across a scheduling fence between the global loads and the LDS stores.
template <int D, int VROW>
struct TileRegs {
    static constexpr int LD = D / 32;
    static constexpr int RPP = 256 / (D / 8);         // rows covered by one pass of the 256 threads
    uint4 k0, k1, k2, k3, v0, v1, v2, v3;

    // kb / vb: wave-uniform byte pointers to row 0 of the tile; rows beyond rlim are clamped to it
    // (the caller masks their scores; a clamped V row is finite, so 0 * v stays 0).
    __device__ __forceinline__ void fetch(const char* kb, const char* vb, int ld_r, int ld_part, int rlim) {
#define VXL_TILE_OFF(i_) ((uint32_t)min(ld_r + (i_) * RPP, rlim) * (D * 2) + ld_part * 16)
        k0 = *(const uint4*)(kb + VXL_TILE_OFF(0));
        v0 = *(const uint4*)(vb + VXL_TILE_OFF(0));
        k1 = *(const uint4*)(kb + VXL_TILE_OFF(1));
        v1 = *(const uint4*)(vb + VXL_TILE_OFF(1));
        if constexpr (LD > 2) {
            k2 = *(const uint4*)(kb + VXL_TILE_OFF(2));
            v2 = *(const uint4*)(vb + VXL_TILE_OFF(2));
            k3 = *(const uint4*)(kb + VXL_TILE_OFF(3));
            v3 = *(const uint4*)(vb + VXL_TILE_OFF(3));
        }
#undef VXL_TILE_OFF
    }
    // The same for rows reached through a row map: tile row r is token src[r] of the dense tensors
    // (rows kv_tok_bytes apart from kd / vd) or, if src[r] < 0, row -1 - src[r] of the sparse
    // buffers (rows D * 2 bytes apart, ks_delta / vs_delta bytes from kd / vd).  The map entries of a
    // tile are requested one tile before its rows (load_map), so that the two dependent loads of a
    // row do not both fall into one tile's arithmetic.  src points at the tile's first entry.
    int m0_, m1_, m2_, m3_;
    __device__ __forceinline__ void load_map(const int32_t* src, int ld_r, int rlim) {
        m0_ = src[min(ld_r, rlim)];
        m1_ = src[min(ld_r + RPP, rlim)];
        if constexpr (LD > 2) {
            m2_ = src[min(ld_r + 2 * RPP, rlim)];
            m3_ = src[min(ld_r + 3 * RPP, rlim)];
        }
    }
    __device__ __forceinline__ void fetch_mapped(const char* kd, const char* vd, long long ks_delta,
                                                 long long vs_delta, long long kv_tok_bytes, int ld_part) {
#define VXL_TILE_ROW(t_, k_, v_)                                                                      \
        do {                                                                                          \
            const long long r_ = (t_) >= 0 ? (long long)(t_) * kv_tok_bytes : (long long)(-1 - (t_)) * (D * 2); \
            k_ = *(const uint4*)(kd + ((t_) >= 0 ? 0 : ks_delta) + r_ + ld_part * 16);                \
            v_ = *(const uint4*)(vd + ((t_) >= 0 ? 0 : vs_delta) + r_ + ld_part * 16);                \
        } while (0)
        VXL_TILE_ROW(m0_, k0, v0);
        VXL_TILE_ROW(m1_, k1, v1);
        if constexpr (LD > 2) {
            VXL_TILE_ROW(m2_, k2, v2);
            VXL_TILE_ROW(m3_, k3, v3);
        }
#undef VXL_TILE_ROW
    }
    __device__ __forceinline__ void stage(uint16_t* kt, uint16_t* vt, int ld_r, int ld_part) const {
        *(uint4*)(kt + k_tile_off<D>(ld_r, ld_part)) = k0;
        *(uint4*)(vt + ld_r * VROW + ld_part * 8) = v0;
        *(uint4*)(kt + k_tile_off<D>(ld_r + RPP, ld_part)) = k1;
        *(uint4*)(vt + (ld_r + RPP) * VROW + ld_part * 8) = v1;
        if constexpr (LD > 2) {
            *(uint4*)(kt + k_tile_off<D>(ld_r + 2 * RPP, ld_part)) = k2;
            *(uint4*)(vt + (ld_r + 2 * RPP) * VROW + ld_part * 8) = v2;
            *(uint4*)(kt + k_tile_off<D>(ld_r + 3 * RPP, ld_part)) = k3;
            *(uint4*)(vt + (ld_r + 3 * RPP) * VROW + ld_part * 8) = v3;
        }
    }
};

constexpr int kKeyTileRows = 64;                    // keys per tile (same as kKeyTile)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int r = 0; r < 16; ++r) z[r] = 0.f;
    return z;
}

// Tile-relative key index of accumulator register r of key block kb for lane half hi.
__device__ __forceinline__ constexpr int acc_key(int kb, int r, int hi) {
    return kb * 32 + 8 * (r >> 2) + 4 * hi + (r & 3);
}

// S^T[qb][kb] = K tile (64 keys, row-major in LDS, pieces placed by k_tile_off) times Q^T.
template <int D, int QB, int KROW, int KB = 2>
__device__ __forceinline__ void qk_tile(const uint16_t* kt, const bf16x8 (&qreg)[QB][D / 16], int l32,
                                        int hi, f32x16 (&s)[QB][KB]) {
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) s[qb][kb] = zero16();
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const bf16x8 a = *(const bf16x8*)(kt + k_tile_off<D>(kb * 32 + l32, ks * 2 + hi));
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
                s[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[qb][ks], s[qb][kb], 0, 0, 0);
        }
}

// The same product for one row block with the K operands requested AHEAD steps before the matrix
// instructions that use them, the order pinned for the scheduler: (AHEAD + 1) x 2 operand reads,
// then per step two matrix instructions followed by the two reads of step + AHEAD + 1.  Left to
// itself the compiler reads an operand pair right before its two instructions and, depending on
// unrelated code, waits for both reads before the first instruction.
template <int D, int AHEAD>
__device__ __forceinline__ void qk_tile_ahead(const uint16_t* kt, const bf16x8 (&qreg)[1][D / 16], int l32, int hi,
                                              f32x16 (&s)[1][2]) {
    constexpr int NK = D / 16;
    s[0][0] = zero16();
    s[0][1] = zero16();
    bf16x8 a[NK][2];
#pragma unroll
    for (int ks = 0; ks < NK; ++ks)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) a[ks][kb] = *(const bf16x8*)(kt + k_tile_off<D>(kb * 32 + l32, ks * 2 + hi));
#pragma unroll
    for (int ks = 0; ks < NK; ++ks)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
            s[0][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks][kb], qreg[0][ks], s[0][kb], 0, 0, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * (AHEAD + 1), 0);          // LDS reads
#pragma unroll
    for (int ks = 0; ks < NK; ++ks) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                    // matrix instructions
        if (ks + AHEAD + 1 < NK) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    }
}

// Online-softmax update of one query block.  m_run is the reference logit of the running
// exponentials (raw units), l_run this lane's half of the running sum, c2 = softmax_scale*log2(e).
// The reference is raised -- and l_run and the output accumulators rescaled -- only when some
// lane of the wave sees a logit more than 2^8 above its reference (in the exp2 domain), a
// wave-uniform decision: until then the probabilities stay below 2^8, which fp32 and bf16
// represent with unchanged relative precision, and the final division by l_run is the same.
// The sum is taken over the bf16-rounded probabilities (the weights the second product uses).
template <int DB, int KB = 2>
__device__ __forceinline__ void softmax_tile(f32x16 (&s)[KB], float c2, float& m_run, float& l_run,
                                             f32x16 (&o)[DB], bf16x8 (&pb)[KB][2]) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    float mx = s[0][0];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
    // The test is made on this lane's half of the keys (the two lanes of a row keep equal
    // references, and the ballot covers both), so the common path has no cross-lane traffic; the
    // row maximum is only formed when the reference is raised.
    const bool grow = (mx - m_run) * c2 > 8.f;              // also true for the first finite logit
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f((m_run - m_new) * c2);
        l_run *= alpha;
        m_run = m_new;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
    }
    const float mc = (m_run == -INFINITY ? 0.f : m_run) * c2;
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    float sum0 = 0.f, sum1 = 0.f;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            bf16x2 pr;
            pr[0] = (__bf16)__builtin_amdgcn_exp2f(fmaf(s[kb][r], c2, -mc));
            pr[1] = (__bf16)__builtin_amdgcn_exp2f(fmaf(s[kb][r + 1], c2, -mc));
            if (((kb * 8 + r / 2) & 1) == 0) sum0 = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, sum0, false);
            else sum1 = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, sum1, false);
            pb[kb][r >> 3][r & 7] = pr[0];
            pb[kb][r >> 3][(r & 7) + 1] = pr[1];
        }
    l_run += sum0 + sum1;
}

// Element offset of 16-byte piece `piece` of row `row` in an UNPADDED V tile (row stride D).
// The 64-byte chunks of a row are XOR-ed with the row's index inside a group of four 256-byte
// lines, so the four rows a half-wave touches in one transposing read fall into distinct banks.
template <int D>
__device__ __forceinline__ int v_tile_off(int row, int piece) {
    constexpr int CPR = D * 2 / 64;                   // 64-byte chunks per row
    constexpr int RPL = D == 128 ? 1 : 2;             // rows per 256-byte line
    return row * D + ((((piece >> 2) ^ ((row / RPL) & (CPR - 1))) << 2 | (piece & 3)) << 3);
}

// A operand of the second product for the 16-key step (kb, j) and the 32-wide d block db, read
// transposed from a row-major V tile in LDS: row stride VROW elements when VROW > D (padded
// layout), or the unpadded swizzled layout of v_tile_off when VROW == D.
template <int D, int VROW>
__device__ __forceinline__ bf16x8 load_vt_operand(const uint16_t* vt, int kb, int j, int db, int lane) {
    const int hi = lane >> 5, dhalf = (lane >> 4) & 1, s = lane & 15;
    const int row = kb * 32 + j * 16 + 4 * hi + (s >> 2);
    const uint16_t* p;
    if constexpr (VROW == D) {
        constexpr int CPR = D * 2 / 64, RPL = D == 128 ? 1 : 2;
        p = vt + row * D + ((db ^ ((row / RPL) & (CPR - 1))) << 5) + dhalf * 16 + 4 * (s & 3);
    } else {
        p = vt + row * VROW + db * 32 + dhalf * 16 + 4 * (s & 3);
    }
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
    const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 8 * VROW));   // row + 8: same swizzle
    const s16x8 both = __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

// Direct global -> LDS copy of one ROWS-key K tile and V tile by ONE wave (global_load_lds_dwordx4:
// lane i's 16 bytes land at the LDS base + 16*i, so one instruction fills 1 KiB of consecutive
// LDS and the swizzles are applied on the global side: a lane fetches the piece that belongs at
// its LDS position).  kt / vt are the unpadded swizzled tiles (k_tile_off / v_tile_off); rows
// beyond rlim are clamped to it.  Completion is tracked by vmcnt.
template <int D, int ROWS = 64>
__device__ __forceinline__ void dma_tile_wave(const char* kb, const char* vb, uint16_t* kt, uint16_t* vt,
                                              int lane, int rlim) {
    constexpr int PPR = D / 8;                        // 16-byte pieces per row
    constexpr int RPI = 64 / PPR;                     // rows per instruction (1 KiB)
    typedef const __attribute__((address_space(1))) void* gptr;
    typedef __attribute__((address_space(3))) void* lptr;
    const int r_in = lane / PPR, pp = lane % PPR;
#pragma unroll
    for (int i = 0; i < ROWS / RPI; ++i) {
        const int row = i * RPI + r_in;
        const int src_row = min(row, rlim);
        // logical piece that lives at physical position pp of this row
        const int kp = pp ^ ((row / (16 / PPR)) & (PPR - 1));
        constexpr int CPR = D * 2 / 64, RPL = D == 128 ? 1 : 2;
        const int vp = (((pp >> 2) ^ ((row / RPL) & (CPR - 1))) << 2) | (pp & 3);
        __builtin_amdgcn_global_load_lds((gptr)(kb + (size_t)src_row * (D * 2) + kp * 16),
                                         (lptr)(kt + i * RPI * D), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((gptr)(vb + (size_t)src_row * (D * 2) + vp * 16),
                                         (lptr)(vt + i * RPI * D), 16, 0, 0);
    }
}

// Pieces of a hand-kept ring of direct global -> LDS loads (kernels that count vmcnt themselves).
// wait_vmcnt<N>: wait until at most N vector-memory operations of this wave are outstanding.
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70);
}
// Wait until no vector-memory operation and no LDS (or scalar-memory) operation of this wave is
// outstanding: what a wave owes the workgroup before a bare s_barrier when it has stored to LDS
// something the others read right behind that barrier.  (The barrier instruction itself waits
// for nothing; an LDS store still queued behind other traffic of its SIMD can be overtaken by
// another SIMD's load.)
__device__ __forceinline__ void wait_vmcnt0_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0x0070); }
// 16 bytes per lane from (uniform base + per-lane offset) to LDS byte offset lds_off + 16*lane.
// Issued from inline assembly so that the compiler neither counts it nor orders LDS reads of
// other ring stages behind it.  The statement overwrites m0 (the LDS base of the load), which the
// compiler reserves and does not accept on a clobber list: kernels that use dma16 must therefore
// contain no m0 use of the compiler's own, which the build checks in their generated assembly.
__device__ __forceinline__ void dma16(const void* base, uint32_t off, uint32_t lds_off) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_off), "v"(off), "s"(base) : "memory");
}

// The same from a per-lane 64-bit address (rows gathered from anywhere in memory).
__device__ __forceinline__ void dma16_addr(const void* addr, uint32_t lds_off) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(lds_off), "v"(addr) : "memory");
}

// Byte offset (from the dense K or V base of the KV head) of the row a map entry names: entry e >= 0
// is dense token e (rows tok_bytes apart); e < 0 is row -1 - e of the sparse buffer, which starts
// sp_delta bytes from the dense base (rows row_bytes apart).  One multiplication and two selects, so
// that a per-lane mix of the two kinds does not become divergent control flow.
__device__ __forceinline__ long long mapped_row_offset(int e, long long tok_bytes, int row_bytes, long long sp_delta) {
    const bool dense = e >= 0;
    const long long idx = dense ? e : ~e;
    return idx * (dense ? tok_bytes : (long long)row_bytes) + (dense ? 0ll : sp_delta);
}

// A 32-bit global load issued from inline assembly: it enters the hand-kept vmcnt count like a direct
// load, and its result is valid only behind a vmcnt wait that covers it (see settle_i32).
__device__ __forceinline__ int load_i32_hidden(const int32_t* p) {
    int v;
    asm volatile("global_load_dword %0, %1, off" : "=&v"(v) : "v"(p) : "memory");
    return v;
}
// Marks the point behind the wait from which a hidden load's result may be used.
__device__ __forceinline__ void settle_i32(int& v) { asm volatile("" : "+v"(v)); }

// N 32-bit LDS reads issued and awaited inside inline assembly.  For kernels that keep their own
// vmcnt count: an LDS read the compiler can see, placed after a hand-issued direct load (whose
// statement clobbers memory), makes it wait for vmcnt(0) first, which empties the ring.
template <int N>
__device__ __forceinline__ void lds_read_i32_hidden(uint32_t byte_addr, uint32_t stride_bytes, int (&v)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i)
        asm volatile("ds_read_b32 %0, %1" : "=v"(v[i]) : "v"(byte_addr + i * stride_bytes) : "memory");
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+v"(v[i]));       // uses stay behind the wait
}

// O^T[qb][db] += V^T . P^T over the 64 keys of the tile.
template <int D, int QB, int VROW, int KB = 2>
__device__ __forceinline__ void pv_tile(const uint16_t* vt, const bf16x8 (&pb)[QB][KB][2], int lane,
                                        f32x16 (&o)[QB][D / 32]) {
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                const bf16x8 a = load_vt_operand<D, VROW>(vt, kb, j, db, lane);
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[qb][kb][j], o[qb][db], 0, 0, 0);
            }
}

// The second product for one row block with its LDS operand reads pinned AHEAD matrix
// instructions before their use (two transposing reads per instruction).  The vector work the
// compiler weaves in between (exponentials of later keys) is left where it puts it: a fixed share
// after every matrix instruction measured 5 % slower.
template <int D, int AHEAD>
__device__ __forceinline__ void pv_tile_ahead(const uint16_t* vt, const bf16x8 (&pb)[1][2][2], int lane,
                                              f32x16 (&o)[1][D / 32]) {
    constexpr int NM = 4 * (D / 32);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                const bf16x8 a = load_vt_operand<D, D>(vt, kb, j, db, lane);
                o[0][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[0][kb][j], o[0][db], 0, 0, 0);
            }
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * (AHEAD + 1), 1);
#pragma unroll
    for (int i = 0; i < NM; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
        if (i + AHEAD + 1 < NM) __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
    }
}

}  // namespace vxl
