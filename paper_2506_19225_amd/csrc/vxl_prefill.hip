// Chunk-based pre-filling attention on the gfx950 matrix cores (bf16 inputs, fp32 accumulate).
//
// Pre-pass (once per call): the K and V rows every later chunk may see -- the prefix rows
// followed by the kept rows of all chunks in chunk order -- are compacted into two contiguous
// buffers, so the history of chunk c is simply their first P + sparse_offsets[c] rows.
//
// Main kernel (prefill_dma_kernel): a persistent workgroup takes bands of query rows of one
// segment (the prefix or a chunk) and walks 64-key tiles  history[0, ctx_len)  then  own
// segment[0, diagonal]  with an online softmax; the arithmetic is in vxl_mfma.h.  256 rows and 8
// waves per workgroup, tiles streamed into an LDS ring by direct global-to-LDS loads.  A second
// instance of the same template (128 rows, 4 waves, two workgroups per compute unit) is kept as
// an on-device cross-check.
#include <math.h>

#include <algorithm>
#include <atomic>

#include "vxl_internal.h"
#include "vxl_mfma.h"

namespace vxl {

namespace {

__device__ __forceinline__ uint4 zero4() { return make_uint4(0u, 0u, 0u, 0u); }

// ------------------------------------------------------------------------------------------
// Pre-pass: Kctx[g, r, :] = K[g, tile_src[r], :], same for V (zero rows where tile_src is -1).
// Its first workgroup also zeroes the work-queue counters of the persistent main kernel (when
// `queue` is given), which saves that kernel's callers a launch of their own.
// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void compact_kv_kernel(const uint4* __restrict__ K, const uint4* __restrict__ V,
                                                         const int32_t* __restrict__ tile_src,
                                                         uint4* __restrict__ Kctx, uint4* __restrict__ Vctx,
                                                         int n_rows_pad, long long kv_head_u4, long long kv_tok_u4,
                                                         int* __restrict__ queue) {
    constexpr int LPR = D * 2 / 16, ROWS = 256 / LPR;
    if (queue && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < 8) queue[threadIdx.x] = 0;
    const int r = blockIdx.x * ROWS + threadIdx.x / LPR, part = threadIdx.x % LPR, g = blockIdx.y;
    if (r >= n_rows_pad) return;
    const int src = tile_src[r];
    const size_t so = (size_t)g * kv_head_u4 + (size_t)max(src, 0) * kv_tok_u4 + part;   // (strides in 16-byte units)
    const size_t dk = ((size_t)g * n_rows_pad + r) * LPR + part;
    Kctx[dk] = src >= 0 ? K[so] : zero4();
    Vctx[dk] = src >= 0 ? V[so] : zero4();
}

// ------------------------------------------------------------------------------------------
// Main kernel: 8 waves = 256 query rows per workgroup (one workgroup per
// compute unit, two waves per SIMD), K/V tiles brought in by direct global->LDS loads into a ring
// of NS stages, two tiles ahead of the arithmetic: the staging stays out of the VALU/VGPR budget
// and the memory latency hides behind several tiles of arithmetic.
//
// The loads are issued from inline assembly: the compiler cannot see them, so it neither orders
// them against the LDS reads of other stages nor counts them in its own vmcnt bookkeeping; the
// kernel does both by hand (every wave issues the same number of loads per tile, and waits with
// vmcnt = loads still allowed in flight).  No compiler-visible vector memory operation may be
// outstanding while the ring runs: the query registers are forced complete before the first ring
// load, and the kernel must not spill (the build refuses a compile of it that uses scratch).
// ------------------------------------------------------------------------------------------
template <int D, int NS, int NW = 8>
struct PrefillDmaCfg {
    static constexpr int WAVES = NW;                          // 8 (one workgroup per compute unit) or 4 (two)
    static constexpr int BM = 32 * WAVES;
    static constexpr int TILE = kKeyTile * D;                 // elements of one unpadded K (or V) tile
    static constexpr int STAGE = 2 * TILE;                    // K tile then V tile
    static constexpr int LDS_BYTES = NS * STAGE * 2 + 16;     // the ring and the slot of the work index
    static constexpr int PPR = D / 8;                         // 16-byte pieces per row
    static constexpr int RPI = 64 / PPR;                      // rows per load instruction (1 KiB)
    static constexpr int NI = kKeyTile / RPI;                 // instructions per tile per matrix
    static constexpr int IPW = NI / WAVES;                    // ... per wave
    static constexpr int GROUP = 2 * IPW;                     // loads per wave per tile (K and V)
};

// The kernel is persistent: the grid is one workgroup per compute unit, and every workgroup keeps
// taking the next (band of query rows, part of its row-block x head grid) pair of its queue from a
// counter in global memory until the queue is empty.  The work list is sorted heaviest first, so this is greedy longest-first
// scheduling without gaps between workgroups.  With xpg > 0 there is one queue per KV head group,
// served by the xpg XCDs (blockIdx.x % 8, the order workgroups are dealt out in) whose L2 then
// holds that group's K and V; otherwise a single queue.  The counters must be zero at launch.
template <int D, int NS, bool STRIDED, int NW = 8>
__global__ __launch_bounds__(NW * 64, 2) void prefill_dma_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    const uint16_t* __restrict__ Kctx, const uint16_t* __restrict__ Vctx, uint16_t* __restrict__ O,
    float* __restrict__ LSE, const Segment* __restrict__ segs, const WorkItem* __restrict__ work,
    int n_tokens, int n_q_heads, int group, int ctx_rows_pad, float scale, int n_items, int xpg,
    int* __restrict__ queue, long long q_head_arg, int q_tok_arg, long long kv_head_arg, int kv_tok_arg) {
    using C = PrefillDmaCfg<D, NS, NW>;
    // Element strides of Q/O and K/V rows: the arguments, or (STRIDED false, the dense head-major
    // layout) constants, so that the dense instance carries no stride arithmetic or registers.
    const long long q_head = STRIDED ? q_head_arg : (long long)n_tokens * D;
    const long long kv_head = STRIDED ? kv_head_arg : (long long)n_tokens * D;
    const int q_tok = STRIDED ? q_tok_arg : D;
    const int kv_tok = STRIDED ? kv_tok_arg : D;
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds;
    int* next_slot = (int*)(lds + NS * C::STAGE);

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int qid = xpg > 0 ? (int)(blockIdx.x & 7) / xpg : 0;            // this workgroup's queue
    const int q_len_items = xpg > 0 ? n_items * group : n_items * n_q_heads;
    const float c2 = scale * kLog2e;
    const int r_in = lane / C::PPR, pp = lane % C::PPR;

    // Lane-constant parts of the refill addresses of a full tile: row and (swizzled) 16-byte piece
    // of this lane in each of the wave's load instructions -- for the compact history tiles
    // (rows D elements apart) and for the own tiles, read in place (rows kv_tok elements apart).
    uint32_t koff_ctx[C::IPW], voff_ctx[C::IPW], koff_own[C::IPW], voff_own[C::IPW];
#pragma unroll
    for (int i = 0; i < C::IPW; ++i) {
        const int row = (wave + i * C::WAVES) * C::RPI + r_in;
        const int kp = pp ^ ((row / (16 / C::PPR)) & (C::PPR - 1));
        constexpr int CPR = D * 2 / 64, RPL = D == 128 ? 1 : 2;
        const int vp = (((pp >> 2) ^ ((row / RPL) & (CPR - 1))) << 2) | (pp & 3);
        koff_ctx[i] = (uint32_t)row * (D * 2) + kp * 16;
        voff_ctx[i] = (uint32_t)row * (D * 2) + vp * 16;
        koff_own[i] = STRIDED ? (uint32_t)row * (uint32_t)(kv_tok * 2) + kp * 16 : koff_ctx[i];
        voff_own[i] = STRIDED ? (uint32_t)row * (uint32_t)(kv_tok * 2) + vp * 16 : voff_ctx[i];
    }

    if (tid == 0) next_slot[0] = atomicAdd(queue + qid, 1);
    __syncthreads();
    int j = __builtin_amdgcn_readfirstlane(next_slot[0]);
    // The descriptors of an item (two dependent scalar loads) are fetched while the item before it
    // runs, as soon as its index is known.
    auto item_of = [&](int jj) { return xpg > 0 ? jj / group : jj / n_q_heads; };
    WorkItem wi_next = {0, 0};
    Segment sg_next = {0, 0, 0, 0, 0};
    if (j < q_len_items) {
        wi_next = work[item_of(j)];
        sg_next = segs[wi_next.seg];
    }
  for (int par = 1; j < q_len_items; par ^= 1) {
    // A list entry is a band of C::BM query rows of a segment; with the `group` query heads that
    // share a KV head it makes a grid of (up to 8 row blocks of 32) x group cells, which is cut
    // row block major into `group` parts of 8 cells, one per wave.  A part spans few row blocks
    // (all heads of one or two of them), so all its waves stop at about the same own tile, and
    // the cells of a ragged last band fill as few parts as possible: cut head by head, every
    // part of such a band would run with most of its waves idle (variable chunk lengths: +11 %).
    // Parts left without cells walk one tile and write nothing.
    const int part_id = xpg > 0 ? qid * group + j % group : j % n_q_heads;
    const int g = part_id / group;                            // KV head
    const int part = part_id - g * group;
    const WorkItem wi = wi_next;
    const Segment sg = sg_next;
    const int m0 = wi.m_tile * C::BM;
    const int band_blocks = min(C::WAVES, (sg.q_len - m0 + 31) / 32);
    const int cell = part * C::WAVES + wave;
    const int rb = cell / group;                              // this wave's row block and head
    const int h = g * group + (cell - rb * group);
    const bool idle = rb >= band_blocks;                      // (the grid of a ragged last band is smaller)
    const int wrow0 = m0 + rb * 32;
    const int n_ctx_t = (sg.ctx_len + kKeyTile - 1) / kKeyTile;
    const int rb_last = min(band_blocks - 1, (part * C::WAVES + C::WAVES - 1) / group);
    const int last_row = min(m0 + (rb_last + 1) * 32, sg.q_len) - 1;
    // own keys start `back` rows early; a part without cells still walks one tile (every wave idle)
    const int n_t = part * C::WAVES < band_blocks * group ? n_ctx_t + (last_row + sg.back) / kKeyTile + 1 : 1;

    const char* kctx_g = (const char*)(Kctx + (size_t)g * ctx_rows_pad * D);
    const char* vctx_g = (const char*)(Vctx + (size_t)g * ctx_rows_pad * D);
    const char* kown = (const char*)(K + (size_t)g * kv_head + (size_t)(sg.q_start - sg.back) * kv_tok);
    const char* vown = (const char*)(V + (size_t)g * kv_head + (size_t)(sg.q_start - sg.back) * kv_tok);

    // Tile t -> stage t % NS.  Every wave issues GROUP loads: instruction slots wave, wave + 8, ...
    auto issue = [&](int t) {
        const bool ctx = t < n_ctx_t;
        const int row0 = ctx ? t * kKeyTile : (t - n_ctx_t) * kKeyTile;
        const int rlim = ctx ? kKeyTile - 1 : min(kKeyTile - 1, sg.back + sg.q_len - 1 - row0);
        const uint32_t row_bytes = ctx ? D * 2 : (uint32_t)kv_tok * 2;
        const char* kb = (ctx ? kctx_g : kown) + (size_t)row0 * row_bytes;
        const char* vb = (ctx ? vctx_g : vown) + (size_t)row0 * row_bytes;
        const uint32_t st = lds_base + (uint32_t)(t % NS) * (C::STAGE * 2);
        if (STRIDED && ctx) {
#pragma unroll
            for (int i = 0; i < C::IPW; ++i) {
                const int slot = wave + i * C::WAVES;
                dma16(kb, koff_ctx[i], st + slot * 1024);
                dma16(vb, voff_ctx[i], st + C::TILE * 2 + slot * 1024);
            }
        } else if (rlim == kKeyTile - 1) {
#pragma unroll
            for (int i = 0; i < C::IPW; ++i) {
                const int slot = wave + i * C::WAVES;
                dma16(kb, koff_own[i], st + slot * 1024);
                dma16(vb, voff_own[i], st + C::TILE * 2 + slot * 1024);
            }
        } else {                                              // rows past the segment's last key repeat it
#pragma unroll
            for (int i = 0; i < C::IPW; ++i) {
                const int slot = wave + i * C::WAVES;
                const int row = slot * C::RPI + r_in;
                const uint32_t back_rows = (uint32_t)(row - min(row, rlim)) * row_bytes;
                dma16(kb, koff_own[i] - back_rows, st + slot * 1024);
                dma16(vb, voff_own[i] - back_rows, st + C::TILE * 2 + slot * 1024);
            }
        }
    };

    f32x16 o[1][D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db) o[0][db] = zero16();
    float m_run = -INFINITY, l_run = 0.f;

    // The ring is used as two groups of TPB stages: while the tiles of one group are consumed the
    // other group is refilled, and the workgroup meets at ONE barrier per TPB tiles (fewer
    // meetings let the waves drift apart, which is what overlaps one wave's vector work with
    // another's matrix work).  Tile indices beyond the last are clamped to it, so that every wave
    // always issues the same number of loads; a clamped issue rewrites the last tile's own stage
    // with the same bytes, which is harmless.
    constexpr int TPB = NS / 2;                               // tiles per workgroup barrier: 2, or 1 with a 2-stage ring
    static_assert(NS == 2 * TPB && (TPB == 1 || TPB == 2), "two groups of TPB stages");
#pragma unroll
    for (int t = 0; t < TPB; ++t) issue(min(t, n_t - 1));

    // The query rows are loaded after the ring has been started (both latencies then overlap) and
    // forced complete here: the compiler's wait for them covers the older ring loads as well, and
    // from here on no load it knows of is outstanding.
    bf16x8 qreg[1][D / 16];
    {
        // uniform base + 32-bit lane offset: the address stays out of the vector registers
        const char* qbase = (const char*)(Q + (size_t)h * q_head + (size_t)sg.q_start * q_tok);
        const uint32_t qoff = (uint32_t)min(wrow0 + l32, sg.q_len - 1) * (uint32_t)(q_tok * 2) + hi * 16;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks)
            qreg[0][ks] = __builtin_bit_cast(bf16x8, *(const uint4*)(qbase + qoff + ks * 32));
        // the index of the item after this one is fetched in the same wait and read when this item is done
        if (tid == 0) next_slot[par] = atomicAdd(queue + qid, 1);
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
            typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
            asm volatile("" :: "v"(__builtin_bit_cast(u32x4, qreg[0][ks])));
        }
    }
    __builtin_amdgcn_sched_barrier(0);

    auto process = [&](int ti) {
        const bool is_ctx = ti < n_ctx_t;
        const int key0 = is_ctx ? ti * kKeyTile : (ti - n_ctx_t) * kKeyTile;
        const bool skip = idle || (!is_ctx && key0 > wrow0 + sg.back + 31);   // the tile lies above this wave's rows
        if (!skip) {
            const uint16_t* kt = lds + (ti % NS) * C::STAGE;
            const uint16_t* vt = kt + C::TILE;
            f32x16 s[1][2];
            qk_tile_ahead<D, 1>(kt, qreg, l32, hi, s);
            const bool need_mask = is_ctx ? (key0 + kKeyTile > sg.ctx_len) : (key0 + kKeyTile - 1 > wrow0 + sg.back);
            if (need_mask) {
                const int lim = is_ctx ? sg.ctx_len - key0 - 1 : wrow0 + sg.back + l32 - key0;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        s[0][kb][r] = acc_key(kb, r, hi) <= lim ? s[0][kb][r] : -INFINITY;
            }
            bf16x8 pb[1][2][2];
            softmax_tile<D / 32>(s[0], c2, m_run, l_run, o[0], pb[0]);
            pv_tile_ahead<D, 2>(vt, pb, lane, o);
        }
    };
    for (int t0 = 0; t0 < n_t; t0 += TPB) {
        // this wave's parts of tiles t0, t0+1 have landed -- and, at the item's first meeting, the
        // next item's index (an LDS store of wave 0, read by everybody right behind the barrier)
        wait_vmcnt0_lgkmcnt0();
        __builtin_amdgcn_s_barrier();                         // ... and everyone's; the other group is free
        if (t0 == 0) {                                        // the next item's index was written before this barrier
            const int jn = __builtin_amdgcn_readfirstlane(next_slot[par]);
            if (jn < q_len_items) {
                wi_next = work[item_of(jn)];
                sg_next = segs[wi_next.seg];
            }
        }
        if (t0 + TPB < n_t) issue(t0 + TPB);                  // (all waits are vmcnt(0): nothing is issued past the last tile,
        process(t0);                                          //  so the item does not end waiting for loads nobody reads)
        if constexpr (TPB == 2) {
            if (t0 + TPB + 1 < n_t) issue(t0 + TPB + 1);      // the second refill between the two tiles
            if (t0 + 1 < n_t) process(t0 + 1);
        }
    }
    wait_vmcnt<0>();                                          // nothing of the ring is in flight when the item ends

    {
        const int q_off = wrow0 + l32;
        const float l_tot = l_run + __shfl_xor(l_run, 32);
        if (q_off < sg.q_len && !idle) {
            const float inv = 1.f / l_tot;
            // uniform bases + 32-bit lane offsets, as for the query loads
            char* obase = (char*)(O + (size_t)h * q_head + (size_t)sg.q_start * q_tok);
            const uint32_t ooff = (uint32_t)q_off * (uint32_t)(q_tok * 2) + hi * 8;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    bf16x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (__bf16)(o[0][db][rq * 4 + e] * inv);
                    *(bf16x4*)(obase + ooff + (db * 32 + rq * 8) * 2) = v;
                }
            if (LSE && hi == 0) (LSE + (size_t)h * n_tokens + sg.q_start)[q_off] = m_run * scale + logf(l_tot);
        }
    }
    __syncthreads();                    // every wave is done with this item's tiles; next_slot[par] is written
    j = __builtin_amdgcn_readfirstlane(next_slot[par]);
  }
}

// Zeroes the queue counters of the persistent kernel (a kernel, not a memset: the call may be
// captured into a graph).
__global__ void reset_queue_kernel(int* queue) {
    if (threadIdx.x < 8) queue[threadIdx.x] = 0;
}

template <typename F>
vxl_status enable_big_lds(F kernel, int bytes) {
    VXL_HIP_TRY(hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    return VXL_OK;
}

}  // namespace

static std::atomic<int> g_prefill_variant{0};
static std::atomic<hipEvent_t> g_ev_start{nullptr}, g_ev_stop{nullptr};
// Cross-check only (declared in vxl_debug.h): 0 = the default instance (8 waves, 256-row bands, one
// workgroup per compute unit); 1 = the same kernel as two independent 4-wave workgroups per compute
// unit (128-row bands, a 2-stage ring each, one meeting per tile).
extern "C" void vxl_debug_prefill_variant(int v) { g_prefill_variant = v == 1 ? 1 : 0; }
// Measurement hook (declared in vxl_debug.h): when both events are set, every vxl_chunk_prefill
// records them on its stream immediately before and after the main attention kernel (the pre-pass
// is outside the bracket).
extern "C" void vxl_debug_prefill_events(void* start, void* stop) {
    g_ev_start = (hipEvent_t)start;
    g_ev_stop = (hipEvent_t)stop;
}

template <int D, int NS, int NW = 8>
static vxl_status run_prefill_dma(const vxl_layout* L, const vxl_attn_desc* d, float scale, const void* Q,
                                  const void* K, const void* V, void* O, float* LSE, void* ws, hipStream_t s) {
    using C = PrefillDmaCfg<D, NS, NW>;
    const TokStrides ts = tok_strides(d, L->n_tokens);
    // 32-bit byte offsets inside a segment's rows (longest segment plus its look-back)
    long long max_rows = 0;
    for (const Segment& sg : L->segs) max_rows = std::max<long long>(max_rows, (long long)sg.q_len + sg.back);
    if (max_rows * std::max(ts.qt, ts.kt) * 2 >= (1ll << 32) || ts.qt >= (1ll << 30) || ts.kt >= (1ll << 30))
        return VXL_ERR_UNSUPPORTED;
    const PrefillWorkspace w = prefill_workspace(L, d);
    uint16_t* kctx = (uint16_t*)((char*)ws + w.kctx);
    uint16_t* vctx = (uint16_t*)((char*)ws + w.vctx);
    int* queue = (int*)((char*)ws + w.queue);
    const int n_rows_pad = L->n_ctx_tiles * kKeyTile;
    if (L->n_ctx_tiles > 0) {
        constexpr int rows = 256 / (D * 2 / 16);
        hipLaunchKernelGGL((compact_kv_kernel<D>), dim3((n_rows_pad + rows - 1) / rows, d->n_kv_heads),
                           dim3(256), 0, s, (const uint4*)K, (const uint4*)V, L->d_tile_src, (uint4*)kctx,
                           (uint4*)vctx, n_rows_pad, ts.kh / 8, ts.kt / 8, queue);
    } else {
        hipLaunchKernelGGL(reset_queue_kernel, dim3(1), dim3(64), 0, s, queue);
    }
    VXL_HIP_TRY(hipGetLastError());
    static PerDeviceOnce attr;
    vxl_status st = attr.run([] {
        const vxl_status a = enable_big_lds(prefill_dma_kernel<D, NS, false, NW>, C::LDS_BYTES);
        return a != VXL_OK ? a : enable_big_lds(prefill_dma_kernel<D, NS, true, NW>, C::LDS_BYTES);
    });
    if (st != VXL_OK) return st;
    int n_cus = 0;                                            // one persistent workgroup per compute unit
    st = device_cu_count(&n_cus);
    if (st != VXL_OK) return st;
    hipEvent_t ev_start = g_ev_start, ev_stop = g_ev_stop;
    const bool timed = ev_start && ev_stop;
    if (timed) VXL_HIP_TRY(hipEventRecord(ev_start, s));
    const int group = d->n_q_heads / d->n_kv_heads;
    const int xpg = 8 % d->n_kv_heads == 0 ? 8 / d->n_kv_heads : 0;
    constexpr int wl_i = NW == 8 ? 1 : 0;                     // the work list cut in bands of 32 * NW rows
    constexpr int per_cu = 8 / NW;                            // workgroups per compute unit
    const long long n_pairs = (long long)L->n_work[wl_i] * d->n_q_heads;
    // no more workgroups than pairs (rounded up to whole rounds over the 8 XCDs when queues are per XCD group)
    const unsigned n_blocks = (unsigned)std::min<long long>((long long)per_cu * (n_cus / 8 * 8),
                                                            xpg ? (n_pairs + 7) / 8 * 8 : n_pairs);
#define VXL_LAUNCH(STRIDED_)                                                                             \
    hipLaunchKernelGGL((prefill_dma_kernel<D, NS, STRIDED_, NW>), dim3(n_blocks), dim3(NW * 64),          \
                       C::LDS_BYTES, s, (const uint16_t*)Q, (const uint16_t*)K, (const uint16_t*)V, kctx,  \
                       vctx, (uint16_t*)O, LSE, L->d_segs, L->d_work[wl_i], L->n_tokens, d->n_q_heads,     \
                       group, n_rows_pad, scale, L->n_work[wl_i], xpg, queue, ts.qh, (int)ts.qt, ts.kh,    \
                       (int)ts.kt)
    if (dense_layout(d)) VXL_LAUNCH(false); else VXL_LAUNCH(true);
#undef VXL_LAUNCH
    VXL_HIP_TRY(hipGetLastError());
    if (timed) VXL_HIP_TRY(hipEventRecord(ev_stop, s));
    return VXL_OK;
}

vxl_status device_cu_count(int* n_cus) {
    static std::mutex mu;
    static int count[kMaxDevices] = {};
    int dev = 0;
    VXL_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return VXL_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (count[dev] == 0) {
        int n = 0;
        VXL_HIP_TRY(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
        count[dev] = n < 8 ? 8 : n;
    }
    *n_cus = count[dev];
    return VXL_OK;
}

vxl_status launch_prefill_bf16(const vxl_layout* L, const vxl_attn_desc* d, float scale, const void* Q,
                               const void* K, const void* V, void* O, float* LSE, void* ws, hipStream_t s) {
    if (g_prefill_variant == 1)
        return d->head_dim == 128 ? run_prefill_dma<128, 2, 4>(L, d, scale, Q, K, V, O, LSE, ws, s)
                                  : run_prefill_dma<64, 2, 4>(L, d, scale, Q, K, V, O, LSE, ws, s);
    return d->head_dim == 128 ? run_prefill_dma<128, 4>(L, d, scale, Q, K, V, O, LSE, ws, s)
                              : run_prefill_dma<64, 4>(L, d, scale, Q, K, V, O, LSE, ws, s);
}

}  // namespace vxl
