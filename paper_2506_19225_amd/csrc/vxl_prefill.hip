// Chunk-based pre-filling attention on the gfx950 matrix cores (bf16 inputs, fp32 accumulate).
//
// Pre-pass (once per call): the K rows every later chunk may see -- the prefix rows followed by
// the kept rows of all chunks in chunk order -- are compacted into one buffer, so the history of
// chunk c is simply its first P + sparse_offsets[c] rows; V is re-laid out as key-major tiles
// V^T[d][64 keys] (history tiles and own-segment tiles) because the P.V product contracts over
// keys and an MFMA operand needs its contraction index contiguous per lane.
//
// Main kernel: one workgroup = one query-row tile of one query head of one segment (the prefix
// or a chunk).  It walks the key tiles  history[0, ctx_len)  then  own segment[0, diagonal]  with
// an online softmax.  Scores are computed transposed, S^T = K.Q^T (32x32x16 bf16 MFMA), so that
// a lane owns one query column: row max / row sum need a single cross-lane exchange, and the
// probabilities are already in the B-operand layout of the second product O^T = V^T.P^T.
#include <math.h>

#include "vxl_internal.h"

namespace vxl {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ uint4 zero4() { return make_uint4(0u, 0u, 0u, 0u); }

// ------------------------------------------------------------------------------------------
// Pre-pass 1: Kctx[g, r, :] = K[g, tile_src[r], :] (zero rows where tile_src is -1).
// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void compact_k_kernel(const uint4* __restrict__ K,
                                                        const int32_t* __restrict__ tile_src,
                                                        uint4* __restrict__ Kctx, int n_rows_pad,
                                                        int n_tokens) {
    constexpr int LPR = D * 2 / 16, ROWS = 256 / LPR;
    const int r = blockIdx.x * ROWS + threadIdx.x / LPR, part = threadIdx.x % LPR, g = blockIdx.y;
    if (r >= n_rows_pad) return;
    const int src = tile_src[r];
    const uint4 v = src >= 0 ? K[((size_t)g * n_tokens + src) * LPR + part] : zero4();
    Kctx[((size_t)g * n_rows_pad + r) * LPR + part] = v;
}

// Position of key `kappa` (0..15) inside a 16-key group of a V^T tile.  The second product
// feeds probabilities straight from the accumulator layout of the first: for a 16-key step the
// lanes 0..31 hold keys {0-3, 8-11} and the lanes 32..63 hold keys {4-7, 12-15}, so the tile
// stores each half contiguously: position p holds key 4*(p/8) + 8*((p%8)/4) + p%4.
__device__ __forceinline__ int key_of_pos(int p) { return 4 * (p >> 3) + 8 * ((p & 7) >> 2) + (p & 3); }

// ------------------------------------------------------------------------------------------
// Pre-pass 2: Vt[g, tile, d, pos] = V[g, tile_src[tile*64 + key(pos)], d]  (zero where -1).
// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void transpose_v_kernel(const uint4* __restrict__ V,
                                                          const int32_t* __restrict__ tile_src,
                                                          uint4* __restrict__ Vt, int n_tiles,
                                                          int n_tokens) {
    constexpr int LPR = D * 2 / 16;
    constexpr int ROW = D + 2;                                // odd word stride: conflict-free columns
    __shared__ uint16_t tile[64 * ROW];
    const int t = blockIdx.x, g = blockIdx.y, tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 64 * LPR / 256; ++i) {
        const int idx = tid + 256 * i, r = idx / LPR, part = idx % LPR;
        const int src = tile_src[t * 64 + r];
        const uint4 v = src >= 0 ? V[((size_t)g * n_tokens + src) * LPR + part] : zero4();
        uint32_t* dst = (uint32_t*)(tile + r * ROW + part * 8);
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    }
    __syncthreads();
    uint4* out = Vt + ((size_t)g * n_tiles + t) * (D * 8);
#pragma unroll
    for (int i = 0; i < D * 8 / 256; ++i) {
        const int idx = tid + 256 * i, d = idx / 8, cc = idx % 8;
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int p0 = cc * 8 + 2 * e, p1 = p0 + 1;
            const int k0 = (p0 & ~15) + key_of_pos(p0 & 15), k1 = (p1 & ~15) + key_of_pos(p1 & 15);
            w[e] = (uint32_t)tile[k0 * ROW + d] | ((uint32_t)tile[k1 * ROW + d] << 16);
        }
        out[idx] = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// ------------------------------------------------------------------------------------------
// Main kernel.
// ------------------------------------------------------------------------------------------
template <int D, int QB>
struct PrefillCfg {
    static constexpr int BM = 128 * QB;          // query rows per workgroup (4 waves x QB x 32)
    static constexpr int KS = D / 16;            // k-steps of the first product
    static constexpr int DB = D / 32;            // 32-wide d blocks of the second product
    static constexpr int KROW = D + 8;           // LDS row strides (elements): +16 bytes so that
    static constexpr int VROW = kKeyTile + 8;    // 8 consecutive rows fall into distinct banks
    static constexpr int K_ELEMS = kKeyTile * KROW;
    static constexpr int V_ELEMS = D * VROW;
    static constexpr int LDS_BYTES = 2 * (K_ELEMS + V_ELEMS) * 2;
    static constexpr int LD = D / 32;            // 16-byte loads per thread per K (and per V) tile
};

template <int D, int QB>
__global__ __launch_bounds__(256, (QB == 1 ? 2 : 1)) void prefill_mfma_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ Kctx,
    const uint16_t* __restrict__ Vt, uint16_t* __restrict__ O, float* __restrict__ LSE,
    const Segment* __restrict__ segs, const WorkItem* __restrict__ work, int n_tokens, int n_q_heads,
    int group, int n_ctx_tiles, int n_tiles_all, float scale) {
    using C = PrefillCfg<D, QB>;
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    uint16_t* Ks = lds;                          // [2][64][KROW]
    uint16_t* Vs = lds + 2 * C::K_ELEMS;         // [2][D][VROW]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hi = lane >> 5;
    const int item = blockIdx.x / n_q_heads, h = blockIdx.x % n_q_heads, g = h / group;
    const WorkItem wi = work[item];
    const Segment sg = segs[wi.seg];
    const int m0 = wi.m_tile * C::BM;
    const int wrow0 = m0 + wave * 32 * QB;       // first query row (segment-relative) of this wave

    const int n_ctx_t = (sg.ctx_len + kKeyTile - 1) / kKeyTile;
    const int last_row = min(m0 + C::BM, sg.q_len) - 1;
    const int n_t = n_ctx_t + last_row / kKeyTile + 1;
    const size_t ctx_rows_pad = (size_t)n_ctx_tiles * kKeyTile;

    // ---- this wave's queries, in B-operand layout: lane (l32, hi) holds 8 consecutive d ----
    bf16x8 qreg[QB][C::KS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int row = sg.q_start + min(wrow0 + qb * 32 + l32, sg.q_len - 1);
        const uint4* src = (const uint4*)(Q + ((size_t)h * n_tokens + row) * D);
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) qreg[qb][ks] = __builtin_bit_cast(bf16x8, src[ks * 2 + hi]);
    }

    f32x16 o[C::DB][QB];
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[db][qb][r] = 0.f;
    }
    const float c2 = scale * 1.4426950408889634f;

    uint4 kreg[C::LD], vreg[C::LD];
    auto fetch = [&](int ti) {
        const bool is_ctx = ti < n_ctx_t;
        const int j = ti - n_ctx_t;
#pragma unroll
        for (int i = 0; i < C::LD; ++i) {
            const int idx = tid + 256 * i, r = idx / (D / 8), part = idx % (D / 8);
            const uint16_t* rowp =
                is_ctx ? Kctx + ((size_t)g * ctx_rows_pad + (size_t)ti * kKeyTile + r) * D
                       : K + ((size_t)g * n_tokens + sg.q_start + min(j * kKeyTile + r, sg.q_len - 1)) * D;
            kreg[i] = ((const uint4*)rowp)[part];
        }
        const int vt_tile = is_ctx ? ti : n_ctx_tiles + sg.tile_base + j;
        const uint4* vsrc = (const uint4*)(Vt + ((size_t)g * n_tiles_all + vt_tile) * (size_t)(D * kKeyTile));
#pragma unroll
        for (int i = 0; i < C::LD; ++i) vreg[i] = vsrc[tid + 256 * i];
    };
    auto stage = [&](int buf) {
        uint16_t* kd = Ks + buf * C::K_ELEMS;
        uint16_t* vd = Vs + buf * C::V_ELEMS;
#pragma unroll
        for (int i = 0; i < C::LD; ++i) {
            const int idx = tid + 256 * i;
            *(uint4*)(kd + (idx / (D / 8)) * C::KROW + (idx % (D / 8)) * 8) = kreg[i];
            *(uint4*)(vd + (idx / 8) * C::VROW + (idx % 8) * 8) = vreg[i];
        }
    };

    fetch(0);
    stage(0);
    __syncthreads();

    for (int ti = 0; ti < n_t; ++ti) {
        const int buf = ti & 1;
        if (ti + 1 < n_t) fetch(ti + 1);

        const bool is_ctx = ti < n_ctx_t;
        const int key0 = is_ctx ? ti * kKeyTile : (ti - n_ctx_t) * kKeyTile;   // tile start in its space
        // own tiles entirely above this wave's rows contribute nothing
        const bool skip = !is_ctx && key0 > wrow0 + 32 * QB - 1;
        if (!skip) {
            const uint16_t* kt = Ks + buf * C::K_ELEMS;
            const uint16_t* vt = Vs + buf * C::V_ELEMS;
            // ---- S^T = K . Q^T : [64 keys] x [32*QB queries] ----
            f32x16 s[2][QB];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[kb][qb][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const bf16x8 a = *(const bf16x8*)(kt + (kb * 32 + l32) * C::KROW + ks * 16 + hi * 8);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        s[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[qb][ks], s[kb][qb], 0, 0, 0);
                }
            }
            // ---- mask (ragged last history tile, causal own tiles) ----
            const bool need_mask = is_ctx ? (key0 + kKeyTile > sg.ctx_len) : (key0 + kKeyTile - 1 > wrow0);
            if (need_mask) {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    // key (tile-relative) kt_ is visible iff kt_ <= lim
                    const int lim = is_ctx ? sg.ctx_len - key0 - 1 : wrow0 + qb * 32 + l32 - key0;
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int kt_ = kb * 32 + 8 * (r >> 2) + 4 * hi + (r & 3);
                            s[kb][qb][r] = kt_ <= lim ? s[kb][qb][r] : -INFINITY;
                        }
                }
            }
            // ---- online softmax; a lane and its partner (lane ^ 32) share a query column ----
            bf16x8 pb[2][2][QB];                  // [key block][16-key step][query block]
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                float mx = s[0][qb][0];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][qb][r]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_run[qb], mx);
                const float m_use = m_new == -INFINITY ? 0.f : m_new;
                const float alpha = __builtin_amdgcn_exp2f((m_run[qb] - m_use) * c2);
                const float mc = m_use * c2;
                float sum = 0.f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float p = __builtin_amdgcn_exp2f(fmaf(s[kb][qb][r], c2, -mc));
                        sum += p;
                        pb[kb][r >> 3][qb][r & 7] = (__bf16)p;
                    }
                }
                l_run[qb] = l_run[qb] * alpha + sum;
                m_run[qb] = m_new;
#pragma unroll
                for (int db = 0; db < C::DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[db][qb][r] *= alpha;
            }
            // ---- O^T += V^T . P^T ----
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int db = 0; db < C::DB; ++db) {
                        const bf16x8 a = *(const bf16x8*)(vt + (db * 32 + l32) * C::VROW + kb * 32 + j * 16 + hi * 8);
#pragma unroll
                        for (int qb = 0; qb < QB; ++qb)
                            o[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[kb][j][qb], o[db][qb], 0, 0, 0);
                    }
        }
        if (ti + 1 < n_t) stage(buf ^ 1);
        __syncthreads();
    }

    // ---- normalise and store: lane owns query column l32; 4 consecutive d per register quad ----
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int q_off = wrow0 + qb * 32 + l32;
        const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32);
        if (q_off >= sg.q_len) continue;
        const float inv = 1.f / l_tot;
        const size_t tok = (size_t)h * n_tokens + sg.q_start + q_off;
        uint16_t* orow = O + tok * D;
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                bf16x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (__bf16)(o[db][qb][rq * 4 + e] * inv);
                *(bf16x4*)(orow + db * 32 + rq * 8 + hi * 4) = v;
            }
        if (LSE && hi == 0) LSE[tok] = m_run[qb] * scale + logf(l_tot);
    }
}

template <typename F>
vxl_status enable_big_lds(F kernel, int bytes) {
    VXL_HIP_TRY(hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    return VXL_OK;
}

}  // namespace

static int g_prefill_qb = 1;
static hipEvent_t g_ev_start = nullptr, g_ev_stop = nullptr;
extern "C" void vxl_debug_prefill_rows_per_wave(int blocks) { g_prefill_qb = blocks == 2 ? 2 : 1; }
// Measurement hook: when both events are set, every vxl_chunk_prefill records them on its stream
// immediately before and after the main attention kernel (the pre-pass is outside the bracket).
extern "C" void vxl_debug_prefill_events(void* start, void* stop) {
    g_ev_start = (hipEvent_t)start;
    g_ev_stop = (hipEvent_t)stop;
}

template <int D, int QB>
static vxl_status run_prefill(const vxl_layout* L, const vxl_attn_desc* d, float scale, const void* Q,
                              const void* K, const void* V, void* O, float* LSE, void* ws, hipStream_t s) {
    using C = PrefillCfg<D, QB>;
    const PrefillWorkspace w = prefill_workspace(L, d);
    uint16_t* kctx = (uint16_t*)((char*)ws + w.kctx);
    uint16_t* vt = (uint16_t*)((char*)ws + w.vt);
    const int n_tiles_all = L->n_ctx_tiles + L->n_own_tiles;
    if (L->n_ctx_tiles > 0) {
        constexpr int rows = 256 / (D * 2 / 16);
        const int n_rows_pad = L->n_ctx_tiles * kKeyTile;
        hipLaunchKernelGGL((compact_k_kernel<D>), dim3((n_rows_pad + rows - 1) / rows, d->n_kv_heads),
                           dim3(256), 0, s, (const uint4*)K, L->d_tile_src, (uint4*)kctx, n_rows_pad,
                           L->n_tokens);
        VXL_HIP_TRY(hipGetLastError());
    }
    hipLaunchKernelGGL((transpose_v_kernel<D>), dim3(n_tiles_all, d->n_kv_heads), dim3(256), 0, s,
                       (const uint4*)V, L->d_tile_src, (uint4*)vt, n_tiles_all, L->n_tokens);
    VXL_HIP_TRY(hipGetLastError());

    static bool attr_done = false;
    if (!attr_done) {
        vxl_status st = enable_big_lds(prefill_mfma_kernel<D, QB>, C::LDS_BYTES);
        if (st != VXL_OK) return st;
        attr_done = true;
    }
    const int v = QB - 1;
    const bool timed = g_ev_start && g_ev_stop;
    if (timed) VXL_HIP_TRY(hipEventRecord(g_ev_start, s));
    const unsigned n_blocks = (unsigned)L->n_work[v] * (unsigned)d->n_q_heads;
    hipLaunchKernelGGL((prefill_mfma_kernel<D, QB>), dim3(n_blocks), dim3(256), C::LDS_BYTES, s,
                       (const uint16_t*)Q, (const uint16_t*)K, kctx, vt, (uint16_t*)O, LSE, L->d_segs,
                       L->d_work[v], L->n_tokens, d->n_q_heads, d->n_q_heads / d->n_kv_heads,
                       L->n_ctx_tiles, n_tiles_all, scale);
    VXL_HIP_TRY(hipGetLastError());
    if (timed) VXL_HIP_TRY(hipEventRecord(g_ev_stop, s));
    return VXL_OK;
}

vxl_status launch_prefill_bf16(const vxl_layout* L, const vxl_attn_desc* d, float scale, const void* Q,
                               const void* K, const void* V, void* O, float* LSE, void* ws, hipStream_t s) {
    if (d->head_dim == 128)
        return g_prefill_qb == 2 ? run_prefill<128, 2>(L, d, scale, Q, K, V, O, LSE, ws, s)
                                 : run_prefill<128, 1>(L, d, scale, Q, K, V, O, LSE, ws, s);
    return g_prefill_qb == 2 ? run_prefill<64, 2>(L, d, scale, Q, K, V, O, LSE, ws, s)
                             : run_prefill<64, 1>(L, d, scale, Q, K, V, O, LSE, ws, s);
}

}  // namespace vxl
