// Softmax attention-mass relevance score (the second reading of the attention-score relevance
// oracle of "Bi-level KVs Decoding"): score[b, c] = mean over (t, h) of the softmax probability
// mass that query token t of head h puts on the dense keys of chunk c, the softmax running over
// ALL tokens (prefix and every chunk).
//
// One pass over the dense keys.  The token range is cut into items (the prefix and every chunk,
// each in pieces of at most kMassPiece keys; table built with the layout).  A workgroup owns one
// (item, KV head, row tile, query b) and produces for each of its stacked query rows
// rho = t*G + hg the pair (m, l): m = the largest scaled logit of the item in base-2 units,
// l = sum over the item's keys of 2^(logit2 - m).  Two small kernels then combine the items of a
// row (M = max m, L = sum l*2^(m-M)) and add up, per chunk, l*2^(m-M)/L over the rows; both use
// fixed summation orders, so equal inputs give equal scores.  The selection is the same LDS
// bitonic sort as in the mean-logit mode.
#include <math.h>

#include <algorithm>

#include "vxl_internal.h"
#include "vxl_mfma.h"

namespace vxl {

namespace {

__device__ __forceinline__ float ldf(const float* p) { return *p; }
__device__ __forceinline__ float ldf(const uint16_t* p) { return __uint_as_float((uint32_t)(*p) << 16); }

// Register staging of one 64-key K tile by a 256-thread workgroup (D/32 16-byte pieces per thread).
template <int D>
struct KTileRegs {
    static constexpr int LD = D / 32;
    static constexpr int RPP = 256 / (D / 8);         // rows covered by one pass of the 256 threads
    uint4 k0, k1, k2, k3;
    // kb: wave-uniform byte pointer to row 0 of the tile; rows beyond rlim are clamped to it (the
    // caller masks their scores).
    __device__ __forceinline__ void fetch(const char* kb, int ld_r, int ld_part, int rlim, uint32_t row_bytes) {
#define VXL_TILE_OFF(i_) ((uint32_t)min(ld_r + (i_) * RPP, rlim) * row_bytes + ld_part * 16)
        k0 = *(const uint4*)(kb + VXL_TILE_OFF(0));
        k1 = *(const uint4*)(kb + VXL_TILE_OFF(1));
        if constexpr (LD > 2) {
            k2 = *(const uint4*)(kb + VXL_TILE_OFF(2));
            k3 = *(const uint4*)(kb + VXL_TILE_OFF(3));
        }
#undef VXL_TILE_OFF
    }
    __device__ __forceinline__ void stage(uint16_t* kt, int ld_r, int ld_part) const {
        *(uint4*)(kt + k_tile_off<D>(ld_r, ld_part)) = k0;
        *(uint4*)(kt + k_tile_off<D>(ld_r + RPP, ld_part)) = k1;
        if constexpr (LD > 2) {
            *(uint4*)(kt + k_tile_off<D>(ld_r + 2 * RPP, ld_part)) = k2;
            *(uint4*)(kt + k_tile_off<D>(ld_r + 3 * RPP, ld_part)) = k3;
        }
    }
};

constexpr int kMassRowTile = 128;                     // stacked query rows per workgroup (4 waves x 32)

// bf16, matrix cores: S^T = K.Q^T per 64-key tile, running (m, l) per query column.
template <int D>
__global__ __launch_bounds__(256, 2) void mass_partial_kernel(
    const uint16_t* __restrict__ Qd, const uint16_t* __restrict__ K, const MassItem* __restrict__ items,
    float* __restrict__ part_m, float* __restrict__ part_l, int T_q, int n_q_heads, int n_kv_heads, int group,
    long long kv_head, long long kv_tok, int n_items, float scale) {   // K strides in elements
    __shared__ __attribute__((aligned(16))) uint16_t Ks[2][kKeyTile * D];
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int item = blockIdx.x;
    const int g = blockIdx.y % n_kv_heads, rt = blockIdx.y / n_kv_heads;
    const int b = blockIdx.z;
    const int n_rows = group * T_q;
    const int k_lo = items[item].key_lo, k_hi = items[item].key_hi;
    const int wrow0 = rt * kMassRowTile + wave * 32;
    const bool wave_active = wrow0 < n_rows;          // waves without rows only help with the copies

    bf16x8 qreg[1][D / 16];
    {
        const int rho = min(wrow0 + l32, n_rows - 1);
        const int t = rho / group, hg = rho % group;
        const uint4* src = (const uint4*)(Qd + (((size_t)b * T_q + t) * n_q_heads + g * group + hg) * D);
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) qreg[0][ks] = __builtin_bit_cast(bf16x8, src[ks * 2 + hi]);
    }
    float m_run = -INFINITY, l_run = 0.f;
    const float c2 = scale * kLog2e;

    const char* kbase = (const char*)(K + (size_t)g * kv_head);
    const uint32_t row_bytes = (uint32_t)kv_tok * 2;
    const int ld_r = tid / (D / 8), ld_part = tid % (D / 8);
    KTileRegs<D> tr;
    const int n_t = (k_hi - k_lo + kKeyTile - 1) / kKeyTile;
    tr.fetch(kbase + (size_t)k_lo * row_bytes, ld_r, ld_part, min(kKeyTile - 1, k_hi - 1 - k_lo), row_bytes);
    tr.stage(Ks[0], ld_r, ld_part);
    __syncthreads();
    for (int ti = 0; ti < n_t; ++ti) {
        const int buf = ti & 1;
        const int key0 = k_lo + ti * kKeyTile;
        {   // next tile (the last iteration re-reads its own), in flight during the arithmetic
            const int nk0 = k_lo + min(ti + 1, n_t - 1) * kKeyTile;
            tr.fetch(kbase + (size_t)nk0 * row_bytes, ld_r, ld_part, min(kKeyTile - 1, k_hi - 1 - nk0), row_bytes);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (wave_active) {
            f32x16 s[1][2];
            qk_tile<D, 1, D>(Ks[buf], qreg, l32, hi, s);
            if (key0 + kKeyTile > k_hi) {
                const int lim = k_hi - key0 - 1;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        s[0][kb][r] = acc_key(kb, r, hi) <= lim ? s[0][kb][r] : -INFINITY;
            }
            float mx = s[0][0][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[0][kb][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));       // every tile holds at least one valid key
            const float m_new = fmaxf(m_run, mx);
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c2);   // 0 on the first tile
            const float mc = m_new * c2;
            float sum[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    sum[r & 3] += __builtin_amdgcn_exp2f(fmaf(s[0][kb][r], c2, -mc));
            l_run = fmaf(l_run, alpha, (sum[0] + sum[1]) + (sum[2] + sum[3]));
            m_run = m_new;
        }
        tr.stage(Ks[buf ^ 1], ld_r, ld_part);
        __syncthreads();
    }
    if (!wave_active) return;
    const int rho = wrow0 + l32;
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (rho < n_rows && hi == 0) {
        const size_t idx = (((size_t)b * n_kv_heads + g) * n_items + item) * (size_t)n_rows + rho;
        part_m[idx] = m_run * c2;
        part_l[idx] = l_tot;
    }
}

__device__ __forceinline__ float wave_max(float v) {
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Vector-ALU form (fp32 arithmetic): one wavefront per query row, a lane per key.  Serves the F32
// storage dtype and, for BF16, an on-device cross-check of the matrix-core kernel.
template <typename T, int D>
__global__ __launch_bounds__(256) void mass_partial_simple_kernel(
    const T* __restrict__ Qd, const T* __restrict__ K, const MassItem* __restrict__ items,
    float* __restrict__ part_m, float* __restrict__ part_l, int T_q, int n_q_heads, int n_kv_heads, int group,
    long long kv_head, long long kv_tok, int n_items, float scale) {   // K strides in elements
    __shared__ float q_lds[4][D];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int item = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int n_rows = group * T_q;
    const int k_lo = items[item].key_lo, k_hi = items[item].key_hi;
    const float c2 = scale * kLog2e;
    const T* kbase = K + (size_t)g * kv_head;
    for (int rho = wave; rho < n_rows; rho += 4) {
        const int t = rho / group, hg = rho % group;
        const T* qrow = Qd + (((size_t)b * T_q + t) * n_q_heads + g * group + hg) * D;
#pragma unroll
        for (int x = 0; x < D / 64; ++x) q_lds[wave][lane + 64 * x] = ldf(qrow + lane + 64 * x);
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        float m = -INFINITY, l = 0.f;
        for (int base = k_lo; base < k_hi; base += 64) {
            const int j = base + lane;
            const bool valid = j < k_hi;
            float s = -INFINITY;
            if (valid) {
                const T* kp = kbase + (size_t)j * kv_tok;
                float a = 0.f;
#pragma unroll 8
                for (int d = 0; d < D; ++d) a = fmaf(q_lds[wave][d], ldf(kp + d), a);
                s = a * c2;
            }
            const float m_new = fmaxf(m, wave_max(s));
            const float p = valid ? exp2f(s - m_new) : 0.f;
            l = l * exp2f(m - m_new) + wave_sum(p);
            m = m_new;
        }
        if (lane == 0) {
            const size_t idx = (((size_t)b * n_kv_heads + g) * n_items + item) * (size_t)n_rows + rho;
            part_m[idx] = m;
            part_l[idx] = l;
        }
        __builtin_amdgcn_wave_barrier();               // q_lds[wave] is rewritten by the next row
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

// Per stacked row (b, g, rho): M = max over the items of m, 1/L with L = sum l * 2^(m - M).  A block
// handles 32 consecutive rows of one (b, g) with 8 item groups: thread (ig, r) folds the items
// ig, ig + 8, ... of row r into a running (M, L) in that order (loads coalesced over the rows),
// and the eight partial pairs of a row are folded in group order -- a fixed summation order.
__global__ __launch_bounds__(256) void mass_rowstat_kernel(const float* __restrict__ part_m,
                                                           const float* __restrict__ part_l,
                                                           float* __restrict__ row_m, float* __restrict__ row_il,
                                                           int n_items, int n_rows) {
    __shared__ float sm[8][32], sl[8][32];
    const int r = threadIdx.x & 31, ig = threadIdx.x >> 5;
    const int rho = blockIdx.x * 32 + r;
    const size_t bg = blockIdx.y;
    float M = -INFINITY, L = 0.f;
    if (rho < n_rows) {
        const size_t base = bg * n_items * n_rows + rho;
        for (int it = ig; it < n_items; it += 8) {
            const float m = part_m[base + (size_t)it * n_rows], l = part_l[base + (size_t)it * n_rows];
            const float Mn = fmaxf(M, m);
            L = L * exp2f(M - Mn) + l * exp2f(m - Mn);         // (M = -inf: L = 0 and 2^-inf = 0)
            M = Mn;
        }
    }
    sm[ig][r] = M;
    sl[ig][r] = L;
    __syncthreads();
    if (ig == 0 && rho < n_rows) {
#pragma unroll
        for (int k = 1; k < 8; ++k) {
            const float m = sm[k][r], l = sl[k][r];
            if (m == -INFINITY) continue;                      // a group without items
            const float Mn = fmaxf(M, m);
            L = L * exp2f(M - Mn) + l * exp2f(m - Mn);
            M = Mn;
        }
        row_m[bg * n_rows + rho] = M;
        row_il[bg * n_rows + rho] = 1.f / L;
    }
}

// One block per (chunk c, query b): score = (1 / (T * Hq)) * sum over the stacked rows of all KV
// heads of [sum over the items of c of l * 2^(m - M_row)] / L_row.  A thread adds its rows
// r = tid, tid + 256, ... in that order; the 256 partial sums are added in a fixed tree.
__global__ __launch_bounds__(256) void mass_chunk_kernel(const float* __restrict__ part_m,
                                                         const float* __restrict__ part_l,
                                                         const float* __restrict__ row_m,
                                                         const float* __restrict__ row_il,
                                                         const int32_t* __restrict__ item_off,
                                                         float* __restrict__ scores, int n_items, int n_rows,
                                                         int n_kv_heads, int n_chunks, float inv_count) {
    __shared__ float wsum[4];
    const int c = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int i0 = item_off[c], i1 = item_off[c + 1];
    const int total = n_kv_heads * n_rows;
    float acc = 0.f;
    for (int r = tid; r < total; r += 256) {
        const int g = r / n_rows, rho = r % n_rows;
        const size_t bg = (size_t)b * n_kv_heads + g;
        const float M = row_m[bg * n_rows + rho];
        float a = 0.f;
        for (int it = i0; it < i1; ++it) {
            const size_t idx = (bg * n_items + it) * (size_t)n_rows + rho;
            a = fmaf(part_l[idx], exp2f(part_m[idx] - M), a);
        }
        acc = fmaf(a, row_il[bg * n_rows + rho], acc);
    }
    acc = wave_sum(acc);
    if ((tid & 63) == 0) wsum[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0) scores[(size_t)b * n_chunks + c] = ((wsum[0] + wsum[1]) + (wsum[2] + wsum[3])) * inv_count;
}

}  // namespace

MassPlan mass_plan(const vxl_layout* L, const vxl_attn_desc* d, int batch, int T) {
    MassPlan p{};
    const size_t rows = (size_t)(d->n_q_heads / d->n_kv_heads) * T;
    const size_t bg = (size_t)batch * d->n_kv_heads;
    size_t off = 0;
    p.part_m = off;  off += align_up(bg * L->n_mass_items * rows * sizeof(float), 256);
    p.part_l = off;  off += align_up(bg * L->n_mass_items * rows * sizeof(float), 256);
    p.row_m = off;   off += align_up(bg * rows * sizeof(float), 256);
    p.row_il = off;  off += align_up(bg * rows * sizeof(float), 256);
    p.scores = off;  off += align_up((size_t)batch * std::max(1, L->n_chunks) * sizeof(float), 256);
    p.total = off;
    return p;
}

vxl_status launch_score_mass(const vxl_layout* L, const vxl_attn_desc* d, float scale, const void* Qd,
                             int batch, int T, const void* K, float* scores, void* ws, bool force_simple,
                             hipStream_t s) {
    const MassPlan p = mass_plan(L, d, batch, T);
    float* part_m = (float*)((char*)ws + p.part_m);
    float* part_l = (float*)((char*)ws + p.part_l);
    float* row_m = (float*)((char*)ws + p.row_m);
    float* row_il = (float*)((char*)ws + p.row_il);
    const int group = d->n_q_heads / d->n_kv_heads;
    const int n_rows = group * T;
    const int n_items = L->n_mass_items;
    const TokStrides ts = tok_strides(d, L->n_tokens);
    if (d->dtype == VXL_BF16 && !force_simple) {
        const int n_rt = (n_rows + kMassRowTile - 1) / kMassRowTile;
        const dim3 grid(n_items, n_rt * d->n_kv_heads, batch);
#define VXL_LAUNCH(D)                                                                                   \
    hipLaunchKernelGGL((mass_partial_kernel<D>), grid, dim3(256), 0, s, (const uint16_t*)Qd,            \
                       (const uint16_t*)K, L->d_mass_items, part_m, part_l, T, d->n_q_heads,            \
                       d->n_kv_heads, group, ts.kh, ts.kt, n_items, scale)
        if (d->head_dim == 64) VXL_LAUNCH(64); else VXL_LAUNCH(128);
#undef VXL_LAUNCH
    } else {
        const dim3 grid(n_items, d->n_kv_heads, batch);
#define VXL_LAUNCH(T_, D)                                                                               \
    hipLaunchKernelGGL((mass_partial_simple_kernel<T_, D>), grid, dim3(256), 0, s, (const T_*)Qd,       \
                       (const T_*)K, L->d_mass_items, part_m, part_l, T, d->n_q_heads, d->n_kv_heads,   \
                       group, ts.kh, ts.kt, n_items, scale)
        if (d->dtype == VXL_F32) { if (d->head_dim == 64) VXL_LAUNCH(float, 64); else VXL_LAUNCH(float, 128); }
        else { if (d->head_dim == 64) VXL_LAUNCH(uint16_t, 64); else VXL_LAUNCH(uint16_t, 128); }
#undef VXL_LAUNCH
    }
    VXL_HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(mass_rowstat_kernel, dim3((n_rows + 31) / 32, batch * d->n_kv_heads), dim3(256), 0, s,
                       part_m, part_l, row_m, row_il, n_items, n_rows);
    VXL_HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(mass_chunk_kernel, dim3(L->n_chunks, batch), dim3(256), 0, s, part_m, part_l, row_m,
                       row_il, L->d_mass_off, scores, n_items, n_rows, d->n_kv_heads, L->n_chunks,
                       1.f / ((float)T * (float)d->n_q_heads));
    VXL_HIP_TRY(hipGetLastError());
    return VXL_OK;
}

}  // namespace vxl
