// Measurement kernels behind the hooks of vxl_debug.h: what this chip attains on the two rooflines
// with nothing in the way.  Nothing here is on the path of an operation.
#include "vxl_internal.h"
#include "vxl_mfma.h"

namespace vxl {

// A register-resident stream of the matrix instruction the kernels use (four
// independent accumulators per wave, 8 waves per workgroup, one workgroup per compute unit,
// `iters` x 4 instructions per wave), for reading kernel rates against an attained peak.
namespace {
__global__ __launch_bounds__(512, 2) void mfma_stream_kernel(float* __restrict__ out, int iters, float seed) {
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = zero16();
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)(seed + (float)e);
        b[e] = (__bf16)(seed * 0.5f + (float)(threadIdx.x & 7));
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < 4; ++m) acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[m], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) t += acc[i][r];
    out[(size_t)blockIdx.x * 512 + threadIdx.x] = t;
}
// The same stream fed with operands as the attention kernels see them: eight register sets of
// pseudo-random bf16 values in (-1, 1), a different pair in every instruction.  The chip holds its
// clock under the stream above (few mantissa bits set, the same operands every time) and lowers it
// under this one, so this is the rate a matrix-bound kernel on real data can be read against.
__global__ __launch_bounds__(512, 2) void mfma_stream_random_kernel(float* __restrict__ out, int iters, uint32_t seed) {
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = zero16();
    bf16x8 r[8];
    uint32_t x = seed ^ (threadIdx.x * 0x9E3779B9u) ^ (blockIdx.x * 0x85EBCA6Bu);
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            x ^= x << 13; x ^= x >> 17; x ^= x << 5;              // xorshift32
            r[j][e] = (__bf16)((float)(int32_t)x * (1.0f / 2147483648.0f));
        }
    for (int it = 0; it < iters; it += 2) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(r[j], r[(j + 3) & 7], acc[j & 3], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int q = 0; q < 16; ++q) t += acc[i][q];
    out[(size_t)blockIdx.x * 512 + threadIdx.x] = t;
}
}  // namespace
extern "C" double vxl_debug_mfma_stream_random(float* out, int n_workgroups, int iters, void* stream) {
    if (!out || n_workgroups <= 0 || iters <= 0 || (iters & 1)) return 0.0;
    hipLaunchKernelGGL(mfma_stream_random_kernel, dim3(n_workgroups), dim3(512), 0, (hipStream_t)stream, out, iters,
                       0x2545F491u);
    if (hipGetLastError() != hipSuccess) return 0.0;
    return (double)n_workgroups * 8.0 * iters * 4.0 * 2.0 * 32 * 32 * 16;
}

// out: device float [n_workgroups * 512]; returns the number of floating-point operations launched
// (0 on a bad argument).
extern "C" double vxl_debug_mfma_stream(float* out, int n_workgroups, int iters, void* stream) {
    if (!out || n_workgroups <= 0 || iters <= 0) return 0.0;
    hipLaunchKernelGGL(mfma_stream_kernel, dim3(n_workgroups), dim3(512), 0, (hipStream_t)stream, out, iters, 1.0f);
    if (hipGetLastError() != hipSuccess) return 0.0;
    return (double)n_workgroups * 8.0 * iters * 4.0 * 2.0 * 32 * 32 * 16;
}


// ------------------------------------------------------------------------------------------
// A measured alternative, used by the tile-loop kernel below only: the tile arithmetic of vxl_mfma.h
// on v_mfma_f32_16x16x32_bf16 (half the outputs and twice the reduction
// depth per instruction: fewer accumulator writes per flop).  Lane (g = lane / 16, m = lane % 16):
//   A operand: A[row m][k = 8g .. 8g+7];  B operand: B[k = 8g .. 8g+7][column m];
//   accumulator register r: D[row 4g + r][column m].
// A wave still owns 32 query rows, as two column blocks qb of 16: S^T[key][query] = K.Q^T gives a
// lane the scores of query 16*qb + m for the keys 16*kb + 4g + r of key block kb (4 blocks of 16 per
// tile), and the probabilities feed O^T = V^T.P^T as its B operand directly: for the 32-key step
// `step` the k slots 8g + e of a lane are the keys 32*step + 4g + e (e < 4) and
// 32*step + 16 + 4g + e - 4 (e >= 4), and the A operand V^T[d][those keys] is gathered from the
// row-major V tile by two transposing reads.
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ f32x4 zero4() { f32x4 z = {0.f, 0.f, 0.f, 0.f}; return z; }

// Element offset of 16-byte piece `piece` of row `row` in the V tile of the 16x16x32 kernels: rows
// unpadded, the 32-byte segments of a row XOR-ed with the row's index among eight rows, so that the
// eight rows x 32 bytes a half-wave touches in one transposing read cover every bank once.
template <int D>
__device__ __forceinline__ int v16_piece(int row, int piece) {
    constexpr int SPR = D * 2 / 32;                   // 32-byte segments per row
    constexpr int RPL = D == 128 ? 1 : 2;             // rows per 256-byte line
    return (((piece >> 1) ^ ((row / RPL) & (SPR - 1))) << 1) | (piece & 1);
}

// Tile-relative key of accumulator register r of key block kb (16 keys) for lane group g.
__device__ __forceinline__ constexpr int acc16_key(int kb, int r, int g) { return kb * 16 + 4 * g + r; }

template <int D>
__device__ __forceinline__ void qk16_tile(const uint16_t* kt, const bf16x8 (&q)[2][D / 32], int g, int m,
                                          f32x4 (&s)[2][4]) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) s[qb][kb] = zero4();
#pragma unroll
    for (int ks = 0; ks < D / 32; ++ks)
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
            const bf16x8 a = *(const bf16x8*)(kt + k_tile_off<D>(kb * 16 + m, ks * 4 + g));
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
                s[qb][kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, q[qb][ks], s[qb][kb], 0, 0, 0);
        }
}

// The same with the order pinned: the K operand of a pair of matrix instructions is read AHEAD pairs
// before them.
template <int D, int AHEAD>
__device__ __forceinline__ void qk16_tile_ahead(const uint16_t* kt, const bf16x8 (&q)[2][D / 32], int g, int m,
                                                f32x4 (&s)[2][4]) {
    qk16_tile<D>(kt, q, g, m, s);
    constexpr int NP = 4 * (D / 32);                  // operand reads = pairs of matrix instructions
    __builtin_amdgcn_sched_group_barrier(0x100, AHEAD + 1, 2);
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 2);
        if (i + AHEAD + 1 < NP) __builtin_amdgcn_sched_group_barrier(0x100, 1, 2);
    }
}

// Online-softmax update of the two query blocks of a wave (see softmax_tile for the lazy reference).
// m_run / l_run: per query block, this lane's query; l_run is the lane's quarter of the running sum.
template <int DB16>
__device__ __forceinline__ void softmax16_tile(f32x4 (&s)[2][4], float c2, float (&m_run)[2], float (&l_run)[2],
                                               f32x4 (&o)[2][DB16], bf16x8 (&pb)[2][2]) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    float mx[2];
    bool grow = false;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        mx[qb] = s[qb][0][0];
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
            for (int r = 0; r < 4; ++r) mx[qb] = fmaxf(mx[qb], s[qb][kb][r]);
        grow = grow || (mx[qb] - m_run[qb]) * c2 > 8.f;
    }
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            float v = fmaxf(mx[qb], __shfl_xor(mx[qb], 16));
            v = fmaxf(v, __shfl_xor(v, 32));
            const float m_new = fmaxf(m_run[qb], v);
            const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f((m_run[qb] - m_new) * c2);
            l_run[qb] *= alpha;
            m_run[qb] = m_new;
#pragma unroll
            for (int db = 0; db < DB16; ++db)
#pragma unroll
                for (int r = 0; r < 4; ++r) o[qb][db][r] *= alpha;
        }
    }
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const float mc = (m_run[qb] == -INFINITY ? 0.f : m_run[qb]) * c2;
        float sum0 = 0.f, sum1 = 0.f;
#pragma unroll
        for (int step = 0; step < 2; ++step)
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const int kb = 2 * step + (e >> 2), r = e & 3;
                bf16x2 pr;
                pr[0] = (__bf16)__builtin_amdgcn_exp2f(fmaf(s[qb][kb][r], c2, -mc));
                pr[1] = (__bf16)__builtin_amdgcn_exp2f(fmaf(s[qb][kb][r + 1], c2, -mc));
                if ((e & 2) == 0) sum0 = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, sum0, false);
                else sum1 = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, sum1, false);
                pb[qb][step][e] = pr[0];
                pb[qb][step][e + 1] = pr[1];
            }
        l_run[qb] += sum0 + sum1;
    }
}

// A operand of the second product for the 32-key step `step` and the 16-wide d block db.
template <int D>
__device__ __forceinline__ bf16x8 load_vt16_operand(const uint16_t* vt, int step, int db, int g, int m) {
    const int row = step * 32 + 4 * g + (m >> 2);
    constexpr int SPR = D * 2 / 32, RPL = D == 128 ? 1 : 2;
    const uint16_t* p = vt + row * D + ((db ^ ((row / RPL) & (SPR - 1))) << 4) + 4 * (m & 3);
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
    const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 16 * D));   // row + 16: same swizzle
    const s16x8 both = __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

template <int D>
__device__ __forceinline__ void pv16_tile(const uint16_t* vt, const bf16x8 (&pb)[2][2], int g, int m,
                                          f32x4 (&o)[2][D / 16]) {
#pragma unroll
    for (int step = 0; step < 2; ++step)
#pragma unroll
        for (int db = 0; db < D / 16; ++db) {
            const bf16x8 a = load_vt16_operand<D>(vt, step, db, g, m);
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
                o[qb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pb[qb][step], o[qb][db], 0, 0, 0);
        }
}

// The same with the two transposing reads of an operand AHEAD operands before its pair of matrix
// instructions; the vector work the compiler weaves in between is left where it puts it.
template <int D, int AHEAD>
__device__ __forceinline__ void pv16_tile_ahead(const uint16_t* vt, const bf16x8 (&pb)[2][2], int g, int m,
                                                f32x4 (&o)[2][D / 16]) {
    pv16_tile<D>(vt, pb, g, m, o);
    constexpr int NP = 2 * (D / 16);
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * (AHEAD + 1), 3);
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 3);
        if (i + AHEAD + 1 < NP) __builtin_amdgcn_sched_group_barrier(0x100, 2, 3);
    }
}

// The tile loop of the pre-filling kernel on its own: the kernel's tile functions (score product
// with the K operands from LDS, online softmax, second product with the transposed V operands from
// LDS) over a ring of four LDS-resident 64-key tiles, 8 waves x 32 rows, one meeting per two tiles
// -- no work items, no masks, no query / output traffic.  What is left in or taken out by `mode`
// prices the ingredients of a tile against the bare matrix-instruction stream on the same data:
//   0  matrix instructions only (32 per wave and tile, operands = the query registers)
//   1  the full tile code on resident tiles
//   2  1 + the ring refilled two tiles ahead by direct global->LDS loads (source resident in L2)
//   3  1 without the softmax arithmetic (weights = converted scores)
//   4  1 with both operand streams taken from registers instead of LDS
//   5  the full tile code in its v_mfma_f32_16x16x32_bf16 form     6  5 + ring refills
//   7  matrix instructions only, v_mfma_f32_16x16x32_bf16 (64 per wave and tile)
namespace {
template <int MODE>
__global__ __launch_bounds__(512, 1) void tile_loop_kernel(const uint16_t* __restrict__ kv, float* __restrict__ out,
                                                           int n_tiles, float c2) {
    constexpr int D = 128, NS = 4, TILE = kKeyTile * D, STAGE = 2 * TILE;
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int i = tid; i < NS * STAGE / 8; i += 512) ((uint4*)lds)[i] = ((const uint4*)kv)[i + blockIdx.x * 64];
    __syncthreads();
    bf16x8 qreg[1][D / 16];
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) qreg[0][ks] = __builtin_bit_cast(bf16x8, ((const uint4*)kv)[tid * 16 + ks]);
    f32x16 o[1][D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db) o[0][db] = zero16();
    float m_run = -INFINITY, l_run = 0.f;
    // (the 16x16x32 form: two query blocks of 16 per wave)
    const int g16 = lane >> 4, m16 = lane & 15;
    bf16x8 q16[2][D / 32];
    f32x4 o16[2][D / 16];
    float m16_run[2] = {-INFINITY, -INFINITY}, l16_run[2] = {0.f, 0.f};
    if (MODE >= 5) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int ks = 0; ks < D / 32; ++ks) q16[qb][ks] = qreg[0][qb * 4 + ks];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int db = 0; db < D / 16; ++db) o16[qb][db] = zero4();
    }
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds;
    const char* gbase = (const char*)kv + (size_t)blockIdx.x * 4096;
    auto issue = [&](int t) {                                  // 4 loads of 1 KiB per wave: its share of a K and a V tile
        const uint32_t st = lds_base + (uint32_t)(t % NS) * (STAGE * 2);
        const uint32_t goff = (uint32_t)(t & 63) * (STAGE * 2);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int slot = wave + i * 8;
            dma16(gbase, goff + slot * 1024 + lane * 16, st + slot * 1024);
            dma16(gbase, goff + TILE * 2 + slot * 1024 + lane * 16, st + TILE * 2 + slot * 1024);
        }
    };
    if (MODE == 2 || MODE == 6) { issue(0); issue(1); }
    auto process = [&](int ti) {
        const uint16_t* kt = lds + (ti % NS) * STAGE;
        const uint16_t* vt = kt + TILE;
        if (MODE == 7) {
#pragma unroll
            for (int j = 0; j < 64; ++j)
                o16[j & 1][(j >> 1) & 7] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qreg[0][j & 7], qreg[0][(j + 3) & 7],
                                                                                  o16[j & 1][(j >> 1) & 7], 0, 0, 0);
            return;
        }
        if (MODE >= 5) {
            f32x4 s16[2][4];
            qk16_tile_ahead<D, 2>(kt, q16, g16, m16, s16);
            bf16x8 pb16[2][2];
            softmax16_tile<D / 16>(s16, c2, m16_run, l16_run, o16, pb16);
            pv16_tile_ahead<D, 2>(vt, pb16, g16, m16, o16);
            return;
        }
        if (MODE == 0) {
#pragma unroll
            for (int j = 0; j < 32; ++j)
                o[0][j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qreg[0][j & 7], qreg[0][(j + 3) & 7], o[0][j & 3], 0, 0, 0);
            return;
        }
        f32x16 s[1][2];
        if (MODE == 4) {
            s[0][0] = zero16();
            s[0][1] = zero16();
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
                    s[0][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qreg[0][(ks + kb + 1) & 7], qreg[0][ks], s[0][kb], 0, 0, 0);
        } else {
            qk_tile_ahead<D, 1>(kt, qreg, l32, hi, s);
        }
        bf16x8 pb[1][2][2];
        if (MODE == 3) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int e = 0; e < 8; ++e) pb[0][kb][j][e] = (__bf16)s[0][kb][j * 8 + e];
        } else {
            softmax_tile<D / 32>(s[0], c2, m_run, l_run, o[0], pb[0]);
        }
        if (MODE == 4) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int db = 0; db < D / 32; ++db)
                        o[0][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qreg[0][(kb * 2 + j + db) & 7], pb[0][kb][j], o[0][db], 0, 0, 0);
        } else {
            pv_tile_ahead<D, 2>(vt, pb, lane, o);
        }
    };
    for (int t0 = 0; t0 < n_tiles; t0 += 2) {
        wait_vmcnt0_lgkmcnt0();
        __builtin_amdgcn_s_barrier();
        if (MODE == 2 || MODE == 6) issue(t0 + 2);
        process(t0);
        if (MODE == 2 || MODE == 6) issue(t0 + 3);
        process(t0 + 1);
    }
    wait_vmcnt<0>();
    float r = l_run + m_run;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int q = 0; q < 16; ++q) r += o[0][db][q];
    if (MODE >= 5) {
        r = l16_run[0] + l16_run[1] + m16_run[0] + m16_run[1];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int db = 0; db < D / 16; ++db)
#pragma unroll
                for (int q = 0; q < 4; ++q) r += o16[qb][db][q];
    }
    out[(size_t)blockIdx.x * 512 + tid] = r;
}
}  // namespace
// kv: device bf16 values, at least vxl_debug_tile_loop_bytes(n_workgroups) bytes; out: device float
// [n_workgroups * 512].  Returns the floating-point operations of the matrix instructions launched
// (n_workgroups x 8 waves x n_tiles x 32 instructions), 0 on a bad argument or a failed launch.
extern "C" size_t vxl_debug_tile_loop_bytes(int n_workgroups) {
    return n_workgroups <= 0 ? 0 : (size_t)66 * (2 * kKeyTile * 128 * 2) + (size_t)n_workgroups * 4096 + 16384;
}
extern "C" double vxl_debug_tile_loop(int mode, const void* kv, float* out, int n_workgroups, int n_tiles,
                                      void* stream) {
    if (!kv || !out || n_workgroups <= 0 || n_tiles <= 0 || (n_tiles & 1) || mode < 0 || mode > 7) return 0.0;
    constexpr int lds_bytes = 4 * 2 * kKeyTile * 128 * 2;
    static PerDeviceOnce attr;
    const vxl_status ast = attr.run([] {
        VXL_HIP_TRY(hipFuncSetAttribute((const void*)tile_loop_kernel<0>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
        VXL_HIP_TRY(hipFuncSetAttribute((const void*)tile_loop_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
        VXL_HIP_TRY(hipFuncSetAttribute((const void*)tile_loop_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
        VXL_HIP_TRY(hipFuncSetAttribute((const void*)tile_loop_kernel<3>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
        VXL_HIP_TRY(hipFuncSetAttribute((const void*)tile_loop_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
        VXL_HIP_TRY(hipFuncSetAttribute((const void*)tile_loop_kernel<5>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
        VXL_HIP_TRY(hipFuncSetAttribute((const void*)tile_loop_kernel<6>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
        VXL_HIP_TRY(hipFuncSetAttribute((const void*)tile_loop_kernel<7>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
        return VXL_OK;
    });
    if (ast != VXL_OK) return 0.0;
    const float c2 = 0.0883883f * kLog2e;
#define VXL_TL(M) hipLaunchKernelGGL(tile_loop_kernel<M>, dim3(n_workgroups), dim3(512), lds_bytes, (hipStream_t)stream, \
                                     (const uint16_t*)kv, out, n_tiles, c2)
    switch (mode) {
        case 0: VXL_TL(0); break;
        case 1: VXL_TL(1); break;
        case 2: VXL_TL(2); break;
        case 3: VXL_TL(3); break;
        case 4: VXL_TL(4); break;
        case 5: VXL_TL(5); break;
        case 6: VXL_TL(6); break;
        default: VXL_TL(7); break;
    }
#undef VXL_TL
    if (hipGetLastError() != hipSuccess) return 0.0;
    return (double)n_workgroups * 8.0 * n_tiles * 32.0 * 2.0 * 32 * 32 * 16;
}

// A bare streaming read: `n_workgroups` workgroups of 256 threads read `bytes` (a multiple of 16) of
// `src` once, 16 bytes per thread and step, eight loads in flight per thread, and write one float
// per thread (a sum that keeps the loads alive).  The time of one launch over a buffer of a decode
// call's size is what a split-KV kernel could at best take for it.
namespace {
__global__ __launch_bounds__(256) void read_stream_kernel(const uint4* __restrict__ src, size_t n_vec,
                                                          float* __restrict__ out) {
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    unsigned acc = 0;
    for (; i + 7 * stride < n_vec; i += 8 * stride) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[i + u * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < n_vec; i += stride) {
        const uint4 v = src[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = (float)acc;
}
}  // namespace
extern "C" int vxl_debug_read_stream(const void* src, size_t bytes, float* out, int n_workgroups, void* stream) {
    if (!src || !out || bytes == 0 || bytes % 16 != 0 || n_workgroups <= 0) return VXL_ERR_INVALID_ARG;
    hipLaunchKernelGGL(read_stream_kernel, dim3(n_workgroups), dim3(256), 0, (hipStream_t)stream, (const uint4*)src,
                       bytes / 16, out);
    return hipGetLastError() == hipSuccess ? VXL_OK : VXL_ERR_HIP;
}

}  // namespace vxl
