// Bi-level KV decoding, the integer / bandwidth-bound steps: per-chunk mean keys, relevance
// scores + top-k selection (LDS bitonic sort), and the dense/sparse gather into the mixed KV.
#include <math.h>

#include <algorithm>

#include "vxl_internal.h"

namespace vxl {

namespace {

__device__ __forceinline__ float ld(const float* p) { return *p; }
__device__ __forceinline__ float ld(const uint16_t* p) { return __uint_as_float((uint32_t)(*p) << 16); }

// ------------------------------------------------------------------------------------------
// kbar[g, c, :] = mean of the dense key rows of chunk c.  One block per (chunk, kv head).
// A thread owns one 16-byte column piece and the rows rg, rg + RG, ... of the chunk, which it
// sums in row order (four independent accumulators: rows 0,4,8.. / 1,5,9.. of its sequence);
// the RG partial sums are then added in group order.  The summation tree depends only on the
// values and their offsets inside the chunk: two chunks with equal contents get bit-identical
// means, hence exactly tied scores.
// ------------------------------------------------------------------------------------------
// qbar[b, g, :] = mean over the T query tokens and the query heads of KV head g of Qd[b, t, h, :].
// One block per (b, g): a thread owns one 16-byte column piece of one head and adds its T tokens in
// token order (16 loads in flight at a time); the heads of the group are then added in head order.
template <typename T, int D>
__device__ __forceinline__ void query_mean_block(const T* __restrict__ Qd, float* __restrict__ qbar, int b, int g,
                                                 int T_q, int n_q_heads, int n_kv_heads, float* hsum /*[group][D]*/) {
    constexpr int EPC = 16 / (int)sizeof(T);
    constexpr int PPR = D / EPC;
    const int group = n_q_heads / n_kv_heads, tid = threadIdx.x;
    const T* qb = Qd + (size_t)b * T_q * n_q_heads * D;
    const int row_pieces = n_q_heads * PPR;
    for (int p = tid; p < group * PPR; p += 256) {
        const int gp = g * group * PPR + p;                    // piece index inside a token's [Hq*D] row
        float acc[EPC];
#pragma unroll
        for (int i = 0; i < EPC; ++i) acc[i] = 0.f;
        for (int t0 = 0; t0 < T_q; t0 += 16) {
            uint4 v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int t = t0 + u < T_q ? t0 + u : T_q - 1;      // clamped rows are not added below
                v[u] = ((const uint4*)qb)[(size_t)t * row_pieces + gp];
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                if (t0 + u < T_q) {
                    const T* e = (const T*)&v[u];
#pragma unroll
                    for (int i = 0; i < EPC; ++i) acc[i] += ld(e + i);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < EPC; ++i) hsum[p * EPC + i] = acc[i];
    }
    __syncthreads();
    for (int dd = tid; dd < D; dd += 256) {
        float a = 0.f;
        for (int hg = 0; hg < group; ++hg) a += hsum[hg * D + dd];
        qbar[((size_t)b * n_kv_heads + g) * D + dd] = a / (float)(T_q * group);
    }
}

// Blocks x < n_chunks summarise chunk x; blocks x >= n_chunks (when Qd is given) form the mean
// query of query x - n_chunks: both feed the scoring kernel, one launch serves both.
template <typename T, int D>
__global__ __launch_bounds__(256) void chunk_summarize_kernel(const T* __restrict__ K,
                                                              const int32_t* __restrict__ bounds,
                                                              float* __restrict__ kbar, long long kv_head_u4,
                                                              long long kv_tok_u4,   // K strides, 16-byte units
                                                              int n_chunks, const T* __restrict__ Qd,
                                                              float* __restrict__ qbar, int T_q, int n_q_heads,
                                                              int n_kv_heads) {
    constexpr int EPC = 16 / (int)sizeof(T);        // elements per 16-byte piece
    constexpr int PPR = D / EPC;                    // pieces per row
    constexpr int RG = 256 / PPR;                   // row groups
    extern __shared__ float dyn[];                  // [group][D] for the query blocks
    __shared__ float part[RG][D];
    if ((int)blockIdx.x >= n_chunks) {
        query_mean_block<T, D>(Qd, qbar, blockIdx.x - n_chunks, blockIdx.y, T_q, n_q_heads, n_kv_heads, dyn);
        return;
    }
    const int c = blockIdx.x, g = blockIdx.y;
    const int piece = threadIdx.x % PPR, rg = threadIdx.x / PPR;
    const int lo = bounds[c], hi = bounds[c + 1];
    const uint4* base = (const uint4*)K + (size_t)g * kv_head_u4 + piece;
    float acc[4][EPC];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < EPC; ++i) acc[u][i] = 0.f;
    int r = lo + rg;
    for (; r + 3 * RG < hi; r += 4 * RG) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = base[(size_t)(r + u * RG) * kv_tok_u4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const T* e = (const T*)&v[u];
#pragma unroll
            for (int i = 0; i < EPC; ++i) acc[u][i] += ld(e + i);
        }
    }
    for (int u = 0; r < hi; r += RG, ++u) {
        const uint4 v = base[(size_t)r * kv_tok_u4];
        const T* e = (const T*)&v;
#pragma unroll
        for (int i = 0; i < EPC; ++i) {
            if (u == 0) acc[0][i] += ld(e + i);
            else if (u == 1) acc[1][i] += ld(e + i);
            else acc[2][i] += ld(e + i);
        }
    }
#pragma unroll
    for (int i = 0; i < EPC; ++i) part[rg][piece * EPC + i] = (acc[0][i] + acc[1][i]) + (acc[2][i] + acc[3][i]);
    __syncthreads();
    if (threadIdx.x < D) {
        float s = part[0][threadIdx.x];
#pragma unroll
        for (int i = 1; i < RG; ++i) s += part[i][threadIdx.x];
        kbar[((size_t)g * n_chunks + c) * D + threadIdx.x] = s / (float)(hi - lo);
    }
}

// ------------------------------------------------------------------------------------------
// One block per query b: mean query per kv head, scores of all chunks, bitonic sort of
// (score, chunk id) in LDS, top-k ids + dense mask.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ bool ranks_before(float sa, int ia, float sb, int ib) {
    return sa > sb || (sa == sb && ia < ib);     // score descending, ties to the lower chunk id
}

// Bitonic sort of (score, chunk id) in LDS, best first (s_val / s_idx hold n_sort entries, a power
// of two, padding = (-inf, INT_MAX)), then the ids of the k best and the membership mask of query b.
// Called by all 256 threads of the block after a barrier.
__device__ __forceinline__ void sort_select(float* s_val, int* s_idx, int n_sort, int n_chunks, int k, int b,
                                            int32_t* __restrict__ topk_idx, uint8_t* __restrict__ dense_mask) {
    const int tid = threadIdx.x;
    if (n_sort <= 1024) {
        // Up to 1024 chunks: every thread ranks its chunks (tid, tid + 256, ...) by counting the
        // chunks that come before them in the order (score descending, id ascending) -- a total
        // order, so the ranks are a permutation -- instead of the barrier-per-step sort below
        // (n^2 / 256 comparisons per thread: 4 us at 640 chunks, where the 55 barrier steps of
        // the sort took 25).
        for (int c = tid; c < n_chunks; c += 256) {
            const float sc = s_val[c];
            int rank = 0;
            for (int o = 0; o < n_chunks; ++o) rank += ranks_before(s_val[o], o, sc, c) ? 1 : 0;
            if (rank < k) topk_idx[(size_t)b * k + rank] = c;
            dense_mask[(size_t)b * n_chunks + c] = (uint8_t)(rank < k ? 1 : 0);
        }
        return;
    }
    // bitonic sort, best first
    for (int size = 2; size <= n_sort; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int i = tid; i < n_sort / 2; i += 256) {
                const int lo = 2 * i - (i & (stride - 1));
                const int hi = lo + stride;
                const bool up = ((lo & size) == 0);
                const float va = s_val[lo], vb = s_val[hi];
                const int ia = s_idx[lo], ib = s_idx[hi];
                const bool a_first = ranks_before(va, ia, vb, ib);
                if (a_first != up) { s_val[lo] = vb; s_val[hi] = va; s_idx[lo] = ib; s_idx[hi] = ia; }
            }
            __syncthreads();
        }
    }
    // membership flags in LDS (the sorted scores are no longer needed), then one coalesced
    // write of the mask
    int* flag = (int*)s_val;
    for (int c = tid; c < n_sort; c += 256) flag[c] = 0;
    __syncthreads();
    for (int i = tid; i < k; i += 256) {
        const int c = s_idx[i];
        topk_idx[(size_t)b * k + i] = c;
        if (c < n_chunks) flag[c] = 1;       // (a NaN score could surface a padding slot)
    }
    __syncthreads();
    for (int c = tid; c < n_chunks; c += 256) dense_mask[(size_t)b * n_chunks + c] = (uint8_t)flag[c];
}

// The scores alone, 32 chunks per block (grid: chunk groups x queries): the same lanes, slices and
// add tree as score_topk_kernel, so a chunk's score does not depend on which of the two computed it.
template <int D>
__global__ __launch_bounds__(256) void chunk_score_kernel(const float* __restrict__ qbar_g,
                                                          const float* __restrict__ kbar, int n_kv_heads,
                                                          int n_chunks, float scale, float* __restrict__ scores) {
    extern __shared__ unsigned char smem[];
    float* qbar = (float*)smem;                               // [Hkv][D]
    const int b = blockIdx.y, tid = threadIdx.x;
    for (int e = tid; e < n_kv_heads * D; e += 256) qbar[e] = qbar_g[(size_t)b * n_kv_heads * D + e];
    __syncthreads();
    const int part = tid & 7, c = blockIdx.x * 32 + (tid >> 3);
    const int slice = n_kv_heads * D / 8;
    float a0 = 0.f;
    if (c < n_chunks) {
#pragma unroll 8
        for (int x = 0; x < slice; x += 4) {
            const int e = part * slice + x, g = e / D, dd = e % D;
            const float4 kv = *(const float4*)(kbar + ((size_t)g * n_chunks + c) * D + dd);
            const float* qg = qbar + e;
            a0 = fmaf(qg[0], kv.x, a0);
            a0 = fmaf(qg[1], kv.y, a0);
            a0 = fmaf(qg[2], kv.z, a0);
            a0 = fmaf(qg[3], kv.w, a0);
        }
    }
    a0 += __shfl_xor(a0, 1);
    a0 += __shfl_xor(a0, 2);
    a0 += __shfl_xor(a0, 4);
    if (part == 0 && c < n_chunks) scores[(size_t)b * n_chunks + c] = a0 * (scale / (float)n_kv_heads);
}

template <int D>
__global__ __launch_bounds__(256) void score_topk_kernel(
    const float* __restrict__ qbar_g, const float* __restrict__ kbar, int n_kv_heads, int n_chunks, int k,
    int n_sort, float scale, int32_t* __restrict__ topk_idx, uint8_t* __restrict__ dense_mask,
    float* __restrict__ scores) {
    extern __shared__ unsigned char smem[];
    float* qbar = (float*)smem;                               // [Hkv][D]
    float* s_val = qbar + n_kv_heads * D;                     // [n_sort]
    int* s_idx = (int*)(s_val + n_sort);                      // [n_sort]
    const int b = blockIdx.x, tid = threadIdx.x;
    for (int e = tid; e < n_kv_heads * D; e += 256) qbar[e] = qbar_g[(size_t)b * n_kv_heads * D + e];
    __syncthreads();
    // Scores: 8 consecutive lanes share a chunk; lane `part` takes the part-th eighth of the
    // flattened (kv head, d) index range, and the eight partial dot products are added in a fixed
    // tree.  Every thread works on two chunks at a time so that their loads overlap.
    {
        const int part = tid & 7, cl = tid >> 3;              // 32 chunk slots per pass and half
        const int slice = n_kv_heads * D / 8;                 // elements per part (a multiple of 4)
        for (int base = 0; base < n_sort; base += 64) {
            float pg[2] = {0.f, 0.f};
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int c = base + u * 32 + cl;
                if (c < n_chunks) {
                    float a0 = 0.f;
#pragma unroll 8
                    for (int x = 0; x < slice; x += 4) {
                        const int e = part * slice + x, g = e / D, dd = e % D;
                        const float4 kv = *(const float4*)(kbar + ((size_t)g * n_chunks + c) * D + dd);
                        const float* qg = qbar + e;
                        a0 = fmaf(qg[0], kv.x, a0);
                        a0 = fmaf(qg[1], kv.y, a0);
                        a0 = fmaf(qg[2], kv.z, a0);
                        a0 = fmaf(qg[3], kv.w, a0);
                    }
                    pg[u] = a0;
                }
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                float a0 = pg[u];
                a0 += __shfl_xor(a0, 1);
                a0 += __shfl_xor(a0, 2);
                a0 += __shfl_xor(a0, 4);
                const int c = base + u * 32 + cl;
                if (part == 0 && c < n_sort) {
                    float a = -INFINITY;
                    if (c < n_chunks) {
                        a = a0 * (scale / (float)n_kv_heads);
                        if (scores) scores[(size_t)b * n_chunks + c] = a;
                    }
                    s_val[c] = a;
                    s_idx[c] = c < n_chunks ? c : 0x7fffffff;
                }
            }
        }
    }
    __syncthreads();
    sort_select(s_val, s_idx, n_sort, n_chunks, k, b, topk_idx, dense_mask);
}

// Selection alone, from scores some other kernel has written: one block per query.
__global__ __launch_bounds__(256) void topk_from_scores_kernel(const float* __restrict__ scores, int n_chunks,
                                                               int k, int n_sort, int32_t* __restrict__ topk_idx,
                                                               uint8_t* __restrict__ dense_mask) {
    extern __shared__ unsigned char smem[];
    float* s_val = (float*)smem;                              // [n_sort]
    int* s_idx = (int*)(s_val + n_sort);                      // [n_sort]
    const int b = blockIdx.x;
    for (int c = threadIdx.x; c < n_sort; c += 256) {
        s_val[c] = c < n_chunks ? scores[(size_t)b * n_chunks + c] : -INFINITY;
        s_idx[c] = c < n_chunks ? c : 0x7fffffff;
    }
    __syncthreads();
    sort_select(s_val, s_idx, n_sort, n_chunks, k, b, topk_idx, dense_mask);
}

// ------------------------------------------------------------------------------------------
// Pooled sparse KVs: chunk c (len rows) is cut into cnt = soff[c+1] - soff[c] consecutive groups,
// group m = rows [floor(m*len/cnt), floor((m+1)*len/cnt)); pooled row soff[c] + m is the mean of
// the group's rows, K and V alike.  LPR lanes per pooled row (a 16-byte piece each), fp32 sums in
// row order, one division, one rounding to the storage dtype.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void st_round(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_round(uint16_t* p, float v) {
    uint32_t b = __float_as_uint(v);
    if ((b & 0x7fffffffu) > 0x7f800000u) { *p = 0x7fc0; return; }
    b += 0x7fffu + ((b >> 16) & 1u);
    *p = (uint16_t)(b >> 16);
}

template <typename T, int D>
__global__ __launch_bounds__(256) void pool_sparse_kernel(const T* __restrict__ K, const T* __restrict__ V,
                                                          const int32_t* __restrict__ bounds,
                                                          const int32_t* __restrict__ soff, int n_chunks,
                                                          long long kv_head_u4, long long kv_tok_u4,
                                                          int s_total, T* __restrict__ Ksp,
                                                          T* __restrict__ Vsp) {
    constexpr int EPC = 16 / (int)sizeof(T);        // elements per 16-byte piece
    constexpr int LPR = D / EPC;                    // lanes per row
    constexpr int ROWS = 256 / LPR;
    const int r = blockIdx.x * ROWS + threadIdx.x / LPR, part = threadIdx.x % LPR, g = blockIdx.y;
    if (r >= s_total) return;
    int c = 0, hi_c = n_chunks;                     // last chunk with soff[c] <= r (its range holds r)
    while (hi_c - c > 1) {
        const int mid = (c + hi_c) >> 1;
        if (soff[mid] <= r) c = mid; else hi_c = mid;
    }
    const long long len = bounds[c + 1] - bounds[c], cnt = soff[c + 1] - soff[c], m = r - soff[c];
    const int lo = bounds[c] + (int)((m * len) / cnt), hi = bounds[c] + (int)(((m + 1) * len) / cnt);
    float ak[EPC], av[EPC];
#pragma unroll
    for (int i = 0; i < EPC; ++i) ak[i] = av[i] = 0.f;
    const uint4* kp = (const uint4*)K + (size_t)g * kv_head_u4 + part;   // (K, V strides in 16-byte units)
    const uint4* vp = (const uint4*)V + (size_t)g * kv_head_u4 + part;
    for (int t = lo; t < hi; ++t) {
        const uint4 kq = kp[(size_t)t * kv_tok_u4], vq = vp[(size_t)t * kv_tok_u4];
        const T* ke = (const T*)&kq;
        const T* ve = (const T*)&vq;
#pragma unroll
        for (int i = 0; i < EPC; ++i) { ak[i] += ld(ke + i); av[i] += ld(ve + i); }
    }
    const float n = (float)(hi - lo);
    T* ko = Ksp + ((size_t)g * s_total + r) * D + part * EPC;
    T* vo = Vsp + ((size_t)g * s_total + r) * D + part * EPC;
#pragma unroll
    for (int i = 0; i < EPC; ++i) { st_round(ko + i, ak[i] / n); st_round(vo + i, av[i] / n); }
}

// ------------------------------------------------------------------------------------------
// Gather, one launch.  Every block first forms, in LDS, the exclusive scan of the rows every chunk
// of its query contributes (its length if dense, its sparse-row count otherwise) -- C <= 4096
// entries, a few hundred nanoseconds, cheaper than a launch of its own -- and then copies its
// share of the mixed rows: a group of LPR lanes per row (all KV heads, K and V, 16-byte
// accesses), the source row found by binary search in the scanned offsets.  A block handles
// `groups` consecutive passes of 256 / LPR rows (chosen by the host so that small gathers still
// fill the chip and large ones amortise the scan).  Block 0 of a query writes mix_len; a query whose
// mixed set does not fit l_cap gets mix_len = -(rows needed) and none of its rows is copied.
// With Kmix == nullptr nothing is copied at all: the call only writes mix_len and src_idx (the row
// map the in-place decode reads the dense and sparse rows through).
// ------------------------------------------------------------------------------------------
template <int ROW_BYTES>
__global__ __launch_bounds__(256) void gather_kernel(
    const uint4* __restrict__ K, const uint4* __restrict__ V, const uint8_t* __restrict__ dense_mask,
    const int32_t* __restrict__ bounds, const int32_t* __restrict__ soff, const int32_t* __restrict__ sidx,
    int n_chunks, int n_prefix, long long kv_head_u4, long long kv_tok_u4,   // K, V strides in 16-byte units
    int n_kv_heads, int l_cap, int groups, uint4* __restrict__ Kmix,
    uint4* __restrict__ Vmix, int32_t* __restrict__ mix_len, int32_t* __restrict__ src_idx,
    const uint4* __restrict__ Ksp, const uint4* __restrict__ Vsp, int s_total) {
    constexpr int LPR = ROW_BYTES / 16;                       // lanes per row
    constexpr int ROWS = 256 / LPR;                           // rows per pass
    extern __shared__ int off[];                              // [n_chunks + 1] first mixed row of every chunk
    __shared__ int wave_tot[4];
    __shared__ int carry;
    const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint8_t* mask = dense_mask + (size_t)b * n_chunks;
    if (tid == 0) carry = n_prefix;
    __syncthreads();
    // The rows every chunk contributes, four 256-chunk passes at a time: their loads are all
    // requested before the first scan (one memory round trip per 1024 chunks, not per 256).
    for (int base4 = 0; base4 < n_chunks; base4 += 1024) {
        int v4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = base4 + u * 256 + tid;
            v4[u] = 0;
            if (c < n_chunks) v4[u] = mask[c] ? bounds[c + 1] - bounds[c] : soff[c + 1] - soff[c];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int base = base4 + u * 256;
            if (base >= n_chunks) break;                      // (uniform)
            const int c = base + tid;
            const int v = v4[u];
            int inc = v;                                      // inclusive scan inside the wave
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_up(inc, o);
                if (lane >= o) inc += t;
            }
            if (lane == 63) wave_tot[wave] = inc;
            __syncthreads();
            int before = carry;
            for (int w = 0; w < wave; ++w) before += wave_tot[w];
            if (c < n_chunks) off[c] = before + inc - v;
            __syncthreads();
            if (tid == 0) carry += wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
            __syncthreads();
        }
    }
    if (tid == 0) {
        off[n_chunks] = carry;
        // a mixed set that does not fit l_cap is reported, not truncated: minus the rows it needs
        if (blockIdx.x == 0) mix_len[b] = carry <= l_cap ? carry : -carry;
    }
    __syncthreads();
    const int len = off[n_chunks] <= l_cap ? off[n_chunks] : 0;
    const int part = tid % LPR;
    for (int gi = 0; gi < groups; ++gi) {
        const int r = (blockIdx.x * groups + gi) * ROWS + tid / LPR;
        if (r >= len) break;                                  // (rows ascend with gi)
        int src;                                              // token id, or -1 - pooled row
        if (r < n_prefix) {
            src = r;
        } else {
            int lo = 0, hi = n_chunks;                        // last chunk with off[c] <= r
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (off[mid] <= r) lo = mid; else hi = mid;
            }
            const int o = r - off[lo];
            if (mask[lo]) src = bounds[lo] + o;
            else src = Ksp ? -1 - (soff[lo] + o) : sidx[soff[lo] + o];
        }
        if (src_idx && part == 0) src_idx[(size_t)b * l_cap + r] = src;
        if (!Kmix) continue;                                  // index-only call: no rows are copied
        const uint4* ks = src >= 0 ? K : Ksp;
        const uint4* vs = src >= 0 ? V : Vsp;
        // the pooled rows are dense [Hkv, S_total, D]; K and V have the caller's strides
        const size_t head_u4 = src >= 0 ? (size_t)kv_head_u4 : (size_t)s_total * LPR;
        const size_t row_u4 = src >= 0 ? (size_t)src * kv_tok_u4 : (size_t)(-1 - src) * LPR;
        for (int g = 0; g < n_kv_heads; ++g) {
            const size_t s_off = g * head_u4 + row_u4 + part;
            const size_t d_off = (((size_t)b * n_kv_heads + g) * l_cap + r) * LPR + part;
            const uint4 kv = ks[s_off];
            const uint4 vv = vs[s_off];
            Kmix[d_off] = kv;
            Vmix[d_off] = vv;
        }
    }
}

}  // namespace

// kbar (n_chunks blocks per KV head; skipped when do_chunks is false) and qbar (batch blocks per KV
// head) in one launch.
vxl_status launch_summaries(const vxl_layout* L, const vxl_attn_desc* d, const void* K, float* kbar,
                            bool do_chunks, const void* Qd, int batch, int T, float* qbar, hipStream_t s) {
    const int nc = do_chunks ? L->n_chunks : 0;
    const dim3 grid(nc + batch, d->n_kv_heads), block(256);
    const size_t smem = (size_t)(d->n_q_heads / d->n_kv_heads) * d->head_dim * sizeof(float);
    const TokStrides ts = tok_strides(d, L->n_tokens);
    const long long epc = d->dtype == VXL_BF16 ? 8 : 4;       // elements per 16 bytes
#define VXL_LAUNCH(T_, D)                                                                         \
    hipLaunchKernelGGL((chunk_summarize_kernel<T_, D>), grid, block, smem, s, (const T_*)K, L->d_bounds, \
                       kbar, ts.kh / epc, ts.kt / epc, nc, (const T_*)Qd, qbar, T, d->n_q_heads,   \
                       d->n_kv_heads)
    if (d->dtype == VXL_F32) { if (d->head_dim == 64) VXL_LAUNCH(float, 64); else VXL_LAUNCH(float, 128); }
    else { if (d->head_dim == 64) VXL_LAUNCH(uint16_t, 64); else VXL_LAUNCH(uint16_t, 128); }
#undef VXL_LAUNCH
    VXL_HIP_TRY(hipGetLastError());
    return VXL_OK;
}

vxl_status launch_score_topk(const vxl_layout* L, const vxl_attn_desc* d, float scale, int batch, int k,
                             const float* qbar, const float* kbar, int32_t* topk_idx, uint8_t* dense_mask,
                             float* scores, float* scores_ws, hipStream_t s) {
    int n_sort = 2;
    while (n_sort < L->n_chunks) n_sort <<= 1;
    // Beyond 128 chunks one block per query is a serial chain (90 us at 640 chunks): the scores are
    // then formed by 32 chunks per block and the selection reads them back.
    if (L->n_chunks > 128) {
        float* sc = scores ? scores : scores_ws;
        const size_t smem_q = (size_t)d->n_kv_heads * d->head_dim * 4;
        const dim3 grid((L->n_chunks + 31) / 32, batch);
        if (d->head_dim == 64)
            hipLaunchKernelGGL((chunk_score_kernel<64>), grid, dim3(256), smem_q, s, qbar, kbar, d->n_kv_heads,
                               L->n_chunks, scale, sc);
        else
            hipLaunchKernelGGL((chunk_score_kernel<128>), grid, dim3(256), smem_q, s, qbar, kbar, d->n_kv_heads,
                               L->n_chunks, scale, sc);
        VXL_HIP_TRY(hipGetLastError());
        return launch_topk_from_scores(L, sc, batch, k, topk_idx, dense_mask, s);
    }
    const size_t smem = (size_t)d->n_kv_heads * d->head_dim * 4 + (size_t)n_sort * 8;
    if (smem > 64 * 1024) return VXL_ERR_UNSUPPORTED;
    const dim3 grid(batch), block(256);
    if (d->head_dim == 64)
        hipLaunchKernelGGL((score_topk_kernel<64>), grid, block, smem, s, qbar, kbar, d->n_kv_heads, L->n_chunks, k,
                           n_sort, scale, topk_idx, dense_mask, scores);
    else
        hipLaunchKernelGGL((score_topk_kernel<128>), grid, block, smem, s, qbar, kbar, d->n_kv_heads, L->n_chunks, k,
                           n_sort, scale, topk_idx, dense_mask, scores);
    VXL_HIP_TRY(hipGetLastError());
    return VXL_OK;
}

vxl_status launch_topk_from_scores(const vxl_layout* L, const float* scores, int batch, int k,
                                   int32_t* topk_idx, uint8_t* dense_mask, hipStream_t s) {
    int n_sort = 2;
    while (n_sort < L->n_chunks) n_sort <<= 1;
    hipLaunchKernelGGL(topk_from_scores_kernel, dim3(batch), dim3(256), (size_t)n_sort * 8, s, scores,
                       L->n_chunks, k, n_sort, topk_idx, dense_mask);
    VXL_HIP_TRY(hipGetLastError());
    return VXL_OK;
}

vxl_status launch_pool_sparse(const vxl_layout* L, const vxl_attn_desc* d, const void* K, const void* V,
                              void* Ksp, void* Vsp, hipStream_t s) {
    if (L->s_total == 0) return VXL_OK;
    const int epc = d->dtype == VXL_BF16 ? 8 : 4;
    const int rows = 256 / (d->head_dim / epc);
    const dim3 grid((L->s_total + rows - 1) / rows, d->n_kv_heads), block(256);
    const TokStrides ts = tok_strides(d, L->n_tokens);
#define VXL_LAUNCH(T, D)                                                                            \
    hipLaunchKernelGGL((pool_sparse_kernel<T, D>), grid, block, 0, s, (const T*)K, (const T*)V,      \
                       L->d_bounds, L->d_soff, L->n_chunks, ts.kh / epc, ts.kt / epc, L->s_total,   \
                       (T*)Ksp, (T*)Vsp)
    if (d->dtype == VXL_F32) { if (d->head_dim == 64) VXL_LAUNCH(float, 64); else VXL_LAUNCH(float, 128); }
    else { if (d->head_dim == 64) VXL_LAUNCH(uint16_t, 64); else VXL_LAUNCH(uint16_t, 128); }
#undef VXL_LAUNCH
    VXL_HIP_TRY(hipGetLastError());
    return VXL_OK;
}

vxl_status launch_gather(const vxl_layout* L, const vxl_attn_desc* d, const void* K, const void* V,
                         const void* Ksp, const void* Vsp, const uint8_t* dense_mask, int batch, void* Kmix,
                         void* Vmix, int l_cap, int32_t* mix_len, int32_t* src_idx, hipStream_t s) {
    const int row_bytes = d->head_dim * (d->dtype == VXL_BF16 ? 2 : 4);
    const size_t smem = (size_t)(L->n_chunks + 1) * sizeof(int);
    const TokStrides ts = tok_strides(d, L->n_tokens);
    const long long epc = d->dtype == VXL_BF16 ? 8 : 4;
#define VXL_LAUNCH(RB)                                                                             \
    do {                                                                                           \
        constexpr int rows = 256 / (RB / 16);                                                      \
        const long passes = (l_cap + rows - 1) / rows;                                             \
        const int groups = (int)std::max<long>(1, std::min<long>(8, passes * batch / 512));        \
        const dim3 grid((unsigned)((passes + groups - 1) / groups), batch);                        \
        hipLaunchKernelGGL((gather_kernel<RB>), grid, dim3(256), smem, s, (const uint4*)K,         \
                           (const uint4*)V, dense_mask, L->d_bounds, L->d_soff, L->d_sidx,         \
                           L->n_chunks, L->n_prefix, ts.kh / epc, ts.kt / epc, d->n_kv_heads,      \
                           l_cap, groups,                                                         \
                           (uint4*)Kmix, (uint4*)Vmix, mix_len, src_idx, (const uint4*)Ksp,        \
                           (const uint4*)Vsp, L->s_total);                                         \
    } while (0)
    if (row_bytes == 128) VXL_LAUNCH(128);
    else if (row_bytes == 256) VXL_LAUNCH(256);
    else VXL_LAUNCH(512);
#undef VXL_LAUNCH
    VXL_HIP_TRY(hipGetLastError());
    return VXL_OK;
}

}  // namespace vxl
