// Plain vector-ALU kernels: one 64-lane wavefront per query row, fp32 arithmetic throughout.
// They serve the F32 storage dtype (whose 1e-5 tolerance rules out bf16 matrix-core inputs)
// and, for BF16 storage, an on-device cross-check of the matrix-core kernels that shares none
// of their tiling, compaction or transposition.
#include <math.h>

#include "vxl_internal.h"

namespace vxl {

namespace {

__device__ __forceinline__ float ld(const float* p) { return *p; }
__device__ __forceinline__ float ld(const uint16_t* p) { return __uint_as_float((uint32_t)(*p) << 16); }
__device__ __forceinline__ void st(float* p, float v) { *p = v; }
__device__ __forceinline__ void st(uint16_t* p, float v) {
    uint32_t b = __float_as_uint(v);
    if ((b & 0x7fffffffu) > 0x7f800000u) { *p = 0x7fc0; return; }
    b += 0x7fffu + ((b >> 16) & 1u);
    *p = (uint16_t)(b >> 16);
}

__device__ __forceinline__ float wave_max(float v) {
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Softmax attention of one query row over n_keys keys; krow(slot) / vrow(slot) return the K and
// the V row of key `slot`.  q_lds: this wave's D floats of LDS.
template <typename T, int D, typename KRowFn, typename VRowFn>
__device__ __forceinline__ void attend_row(const T* qrow, KRowFn krow, VRowFn vrow, int n_keys, float scale,
                                           float* q_lds, T* orow, float* lse_out) {
    const int lane = threadIdx.x & 63;
    constexpr int X = D / 64;
#pragma unroll
    for (int x = 0; x < X; ++x) q_lds[lane + 64 * x] = ld(qrow + lane + 64 * x);
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    float m = -INFINITY, l = 0.f, acc[X];
#pragma unroll
    for (int x = 0; x < X; ++x) acc[x] = 0.f;
    for (int base = 0; base < n_keys; base += 64) {
        const int slot = base + lane;
        const bool valid = slot < n_keys;
        float s = -INFINITY;
        if (valid) {
            const T* kp = krow(slot);
            float a = 0.f;
#pragma unroll 8
            for (int d = 0; d < D; ++d) a = fmaf(q_lds[d], ld(kp + d), a);
            s = a * scale;
        }
        const float m_new = fmaxf(m, wave_max(s));
        const float p = valid ? expf(s - m_new) : 0.f;
        const float alpha = expf(m - m_new);
        l = l * alpha + wave_sum(p);
#pragma unroll
        for (int x = 0; x < X; ++x) acc[x] *= alpha;
        const int cnt = min(64, n_keys - base);
        for (int j = 0; j < cnt; ++j) {
            const float pj = __shfl(p, j);
            const T* vp = vrow(base + j);
#pragma unroll
            for (int x = 0; x < X; ++x) acc[x] = fmaf(pj, ld(vp + lane + 64 * x), acc[x]);
        }
        m = m_new;
    }
    const float inv = 1.f / l;
#pragma unroll
    for (int x = 0; x < X; ++x) st(orow + lane + 64 * x, acc[x] * inv);
    if (lse_out && lane == 0) *lse_out = m + logf(l);
}

template <typename T, int D>
__global__ __launch_bounds__(256) void prefill_simple_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, T* __restrict__ O,
    float* __restrict__ LSE, const int32_t* __restrict__ bounds, const int32_t* __restrict__ soff,
    const int32_t* __restrict__ sidx, int n_tokens, int n_prefix, int n_chunks, int group,
    float scale, int window, long long q_head, long long q_tok, long long kv_head_stride, long long kv_tok) {
    __shared__ float q_lds[4][D];
    const int wave = threadIdx.x >> 6;
    const int i = blockIdx.x * 4 + wave;
    const int h = blockIdx.y;
    if (i >= n_tokens) return;
    const int g = h / group;
    int own_start = 0, n_hist = 0;
    if (i >= n_prefix) {
        int lo = 0, hi = n_chunks;          // last chunk c with bounds[c] <= i
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (bounds[mid] <= i) lo = mid; else hi = mid;
        }
        // dense range starts `window` tokens before the chunk (not inside the prefix); kept tokens
        // of earlier chunks count as history only if they lie before that range
        own_start = max(n_prefix, bounds[lo] - window);
        int a = 0, b = soff[lo];            // first kept index (of the earlier chunks) >= own_start
        while (a < b) {
            const int mid = (a + b) >> 1;
            if (sidx[mid] < own_start) a = mid + 1; else b = mid;
        }
        n_hist = n_prefix + a;
    }
    const int n_keys = n_hist + (i - own_start + 1);
    auto key = [=](int slot) -> size_t {
        int tok;
        if (slot < n_hist) tok = slot < n_prefix ? slot : sidx[slot - n_prefix];
        else tok = own_start + (slot - n_hist);
        return (size_t)tok * kv_tok;
    };
    const T* kh = K + (size_t)g * kv_head_stride;
    const T* vh = V + (size_t)g * kv_head_stride;
    const size_t q_off = (size_t)h * q_head + (size_t)i * q_tok;
    attend_row<T, D>(Q + q_off, [=](int slot) { return kh + key(slot); }, [=](int slot) { return vh + key(slot); },
                     n_keys, scale, q_lds[wave], O + q_off, LSE ? LSE + (size_t)h * n_tokens + i : nullptr);
}

template <typename T, int D>
__global__ __launch_bounds__(256) void decode_simple_kernel(
    const T* __restrict__ Qd, const T* __restrict__ Kmix, const T* __restrict__ Vmix,
    T* __restrict__ O, float* __restrict__ LSE, const int32_t* __restrict__ mix_len, int batch, int T_q,
    int n_q_heads, int group, int l_cap, float scale) {
    __shared__ float q_lds[4][D];
    const int wave = threadIdx.x >> 6;
    const long row = (long)blockIdx.x * 4 + wave;           // (b, t, h) flattened
    const long n_rows = (long)batch * T_q * n_q_heads;
    if (row >= n_rows) return;
    const int h = (int)(row % n_q_heads);
    const int b = (int)(row / ((long)T_q * n_q_heads));
    const int g = h / group;
    const int n_kv = n_q_heads / group;
    const int n_keys = min(max(mix_len[b], 0), l_cap);
    auto key = [=](int slot) -> size_t { return (size_t)slot * D; };
    const size_t kv_off = ((size_t)b * n_kv + g) * (size_t)l_cap * D;
    if (n_keys == 0) {
        const int lane = threadIdx.x & 63;
        for (int x = 0; x < D / 64; ++x) st(O + row * D + lane + 64 * x, 0.f);
        if (LSE && lane == 0) LSE[row] = -INFINITY;
        return;
    }
    const T* kh = Kmix + kv_off;
    const T* vh = Vmix + kv_off;
    attend_row<T, D>(Qd + row * D, [=](int slot) { return kh + key(slot); }, [=](int slot) { return vh + key(slot); },
                     n_keys, scale, q_lds[wave], O + row * D, LSE ? LSE + row : nullptr);
}

// The same over the mixed KV set read in place: mixed row `slot` of query b is token src_idx[b, slot]
// of K / V, or (src < 0) row -1 - src of the sparse buffers Ksp / Vsp [Hkv, S_total, D].
template <typename T, int D>
__global__ __launch_bounds__(256) void decode_inplace_simple_kernel(
    const T* __restrict__ Qd, const T* __restrict__ K, const T* __restrict__ V, const T* __restrict__ Ksp,
    const T* __restrict__ Vsp, const int32_t* __restrict__ src_idx, T* __restrict__ O, float* __restrict__ LSE,
    const int32_t* __restrict__ mix_len, int batch, int T_q, int n_q_heads, int group, int l_cap, int s_total,
    long long kv_head_stride, long long kv_tok, float scale) {
    __shared__ float q_lds[4][D];
    const int wave = threadIdx.x >> 6;
    const long row = (long)blockIdx.x * 4 + wave;           // (b, t, h) flattened
    const long n_rows = (long)batch * T_q * n_q_heads;
    if (row >= n_rows) return;
    const int h = (int)(row % n_q_heads);
    const int b = (int)(row / ((long)T_q * n_q_heads));
    const int g = h / group;
    const int n_keys = min(max(mix_len[b], 0), l_cap);
    if (n_keys == 0) {
        const int lane = threadIdx.x & 63;
        for (int x = 0; x < D / 64; ++x) st(O + row * D + lane + 64 * x, 0.f);
        if (LSE && lane == 0) LSE[row] = -INFINITY;
        return;
    }
    const int32_t* src = src_idx + (size_t)b * l_cap;
    const T* kh = K + (size_t)g * kv_head_stride;
    const T* vh = V + (size_t)g * kv_head_stride;
    const T* ksh = Ksp ? Ksp + (size_t)g * s_total * D : nullptr;
    const T* vsh = Vsp ? Vsp + (size_t)g * s_total * D : nullptr;
    auto krow = [=](int slot) { const int t = src[slot]; return t >= 0 ? kh + (size_t)t * kv_tok : ksh + (size_t)(-1 - t) * D; };
    auto vrow = [=](int slot) { const int t = src[slot]; return t >= 0 ? vh + (size_t)t * kv_tok : vsh + (size_t)(-1 - t) * D; };
    attend_row<T, D>(Qd + row * D, krow, vrow, n_keys, scale, q_lds[wave], O + row * D, LSE ? LSE + row : nullptr);
}

}  // namespace

vxl_status launch_prefill_simple(const vxl_layout* L, const vxl_attn_desc* d, float scale,
                                 const void* Q, const void* K, const void* V, void* O, float* LSE,
                                 hipStream_t s) {
    const dim3 grid((L->n_tokens + 3) / 4, d->n_q_heads), block(256);
    const int group = d->n_q_heads / d->n_kv_heads;
    const TokStrides ts = tok_strides(d, L->n_tokens);
#define VXL_LAUNCH(T, D)                                                                          \
    hipLaunchKernelGGL((prefill_simple_kernel<T, D>), grid, block, 0, s, (const T*)Q, (const T*)K, \
                       (const T*)V, (T*)O, LSE, L->d_bounds, L->d_soff, L->d_sidx, L->n_tokens,   \
                       L->n_prefix, L->n_chunks, group, scale, L->window, ts.qh, ts.qt, ts.kh, ts.kt)
    if (d->dtype == VXL_F32) { if (d->head_dim == 64) VXL_LAUNCH(float, 64); else VXL_LAUNCH(float, 128); }
    else { if (d->head_dim == 64) VXL_LAUNCH(uint16_t, 64); else VXL_LAUNCH(uint16_t, 128); }
#undef VXL_LAUNCH
    VXL_HIP_TRY(hipGetLastError());
    return VXL_OK;
}

vxl_status launch_decode_simple(const vxl_attn_desc* d, float scale, const void* Qd, int batch, int T,
                                const void* Kmix, const void* Vmix, int l_cap, const int32_t* mix_len,
                                void* O, float* LSE, hipStream_t s) {
    const long n_rows = (long)batch * T * d->n_q_heads;
    const dim3 grid((unsigned)((n_rows + 3) / 4)), block(256);
    const int group = d->n_q_heads / d->n_kv_heads;
#define VXL_LAUNCH(T_, D)                                                                            \
    hipLaunchKernelGGL((decode_simple_kernel<T_, D>), grid, block, 0, s, (const T_*)Qd,              \
                       (const T_*)Kmix, (const T_*)Vmix, (T_*)O, LSE, mix_len, batch, T, d->n_q_heads, \
                       group, l_cap, scale)
    if (d->dtype == VXL_F32) { if (d->head_dim == 64) VXL_LAUNCH(float, 64); else VXL_LAUNCH(float, 128); }
    else { if (d->head_dim == 64) VXL_LAUNCH(uint16_t, 64); else VXL_LAUNCH(uint16_t, 128); }
#undef VXL_LAUNCH
    VXL_HIP_TRY(hipGetLastError());
    return VXL_OK;
}

vxl_status launch_decode_inplace_simple(const vxl_layout* L, const vxl_attn_desc* d, float scale, const void* Qd,
                                        int batch, int T, const void* K, const void* V, const void* Ksp,
                                        const void* Vsp, const int32_t* src_idx, int l_cap,
                                        const int32_t* mix_len, void* O, float* LSE, hipStream_t s) {
    const long n_rows = (long)batch * T * d->n_q_heads;
    const dim3 grid((unsigned)((n_rows + 3) / 4)), block(256);
    const int group = d->n_q_heads / d->n_kv_heads;
    const TokStrides ts = tok_strides(d, L->n_tokens);
#define VXL_LAUNCH(T_, D)                                                                                    \
    hipLaunchKernelGGL((decode_inplace_simple_kernel<T_, D>), grid, block, 0, s, (const T_*)Qd, (const T_*)K,  \
                       (const T_*)V, (const T_*)Ksp, (const T_*)Vsp, src_idx, (T_*)O, LSE, mix_len, batch, T,   \
                       d->n_q_heads, group, l_cap, L->s_total, ts.kh, ts.kt, scale)
    if (d->dtype == VXL_F32) { if (d->head_dim == 64) VXL_LAUNCH(float, 64); else VXL_LAUNCH(float, 128); }
    else { if (d->head_dim == 64) VXL_LAUNCH(uint16_t, 64); else VXL_LAUNCH(uint16_t, 128); }
#undef VXL_LAUNCH
    VXL_HIP_TRY(hipGetLastError());
    return VXL_OK;
}

}  // namespace vxl
