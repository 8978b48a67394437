// Host side of the C ABI: argument validation, the layout handle (device copies of the
// chunking and the pre-filling tile schedule), workspace planning and kernel dispatch.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <numeric>

#include "vxl_internal.h"

namespace vxl {

static thread_local char g_last_error[512] = "";
static std::atomic<int> g_force_simple{0};

void set_last_error(const char* what, hipError_t e) {
    snprintf(g_last_error, sizeof(g_last_error), "%s: %s", what, hipGetErrorString(e));
}

static bool desc_ok(const vxl_attn_desc* d, vxl_status* st) {
    if (!d) { *st = VXL_ERR_INVALID_ARG; return false; }
    if (d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->n_q_heads % d->n_kv_heads != 0 ||
        !(d->softmax_scale >= 0.0f) || !std::isfinite(d->softmax_scale)) {
        *st = VXL_ERR_INVALID_ARG; return false;
    }
    if ((d->dtype != VXL_F32 && d->dtype != VXL_BF16) || (d->head_dim != 64 && d->head_dim != 128)) {
        *st = VXL_ERR_UNSUPPORTED; return false;
    }
    const int64_t sv[4] = {d->q_stride_head, d->q_stride_tok, d->kv_stride_head, d->kv_stride_tok};
    const bool any = sv[0] || sv[1] || sv[2] || sv[3];
    if (any) {                                                // all set, 16-byte multiples, rows of head_dim fit
        const int64_t unit = d->dtype == VXL_BF16 ? 8 : 4;
        for (int64_t v : sv)
            if (v <= 0 || v % unit != 0) { *st = VXL_ERR_INVALID_ARG; return false; }
        if (d->q_stride_tok < d->head_dim || d->kv_stride_tok < d->head_dim) { *st = VXL_ERR_INVALID_ARG; return false; }
    }
    if (d->reserved != 0) { *st = VXL_ERR_INVALID_ARG; return false; }
    return true;
}

static float resolve_scale(const vxl_attn_desc* d) {
    return d->softmax_scale > 0.0f ? d->softmax_scale : 1.0f / std::sqrt((float)d->head_dim);
}

static size_t elem_bytes(const vxl_attn_desc* d) { return d->dtype == VXL_BF16 ? 2 : 4; }

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

PrefillWorkspace prefill_workspace(const vxl_layout* L, const vxl_attn_desc* d) {
    PrefillWorkspace w{};
    if (d->dtype != VXL_BF16) { w.total = 0; return w; }
    size_t off = 0;
    w.kctx = off;
    off += align_up((size_t)d->n_kv_heads * L->n_ctx_tiles * kKeyTile * d->head_dim * 2, 256);
    w.vctx = off;
    off += align_up((size_t)d->n_kv_heads * L->n_ctx_tiles * kKeyTile * d->head_dim * 2, 256);
    w.queue = off;
    off += 256;
    w.total = off;
    return w;
}

static std::atomic<int> g_decode_step_waves{0};     // cross-check hook (vxl_debug.h): 0 = choose, 4 or 8 = force
extern "C" void vxl_debug_decode_step_waves(int w) { g_decode_step_waves = (w == 4 || w == 8) ? w : 0; }

DecodePlan decode_plan(const vxl_attn_desc* d, int batch, int T, int l_cap, bool gathered) {
    DecodePlan p{};
    if (d->dtype != VXL_BF16) { p.n_split = 1; p.split_len = l_cap; p.total = 0; return p; }
    const int rows = (d->n_q_heads / d->n_kv_heads) * T;
    const int tiles = (l_cap + kKeyTile - 1) / kKeyTile;
    // 129-256 stacked rows fit one 256-row workgroup of the ring kernel or two 128-row workgroups
    // of the 4-wave kernel.  The ring kernel streams better, but only when its launch covers the
    // chip; at short mixed sets the split cap below leaves it a fraction of the compute units
    // (measured at 224 rows: 64 and 120 workgroups, 4-wave kernel 9 % and 5 % faster; 176 and
    // 256 workgroups, ring kernel 5 % and 8 % faster).
    bool ring = rows > 128;
    if (ring && rows <= 256) {
        const long blocks = (long)batch * d->n_kv_heads;
        const long splits = std::max<long>(1, std::min<long>(std::min<long>((256 + blocks - 1) / blocks, (long)l_cap / rows), tiles));
        const int per = (int)((tiles + splits - 1) / splits);
        ring = blocks * ((tiles + per - 1) / per) >= 150;
    }
    p.use_ring = ring ? 1 : 0;
    const int row_tile = ring ? 256 : 128;
    const int n_rtile = (rows + row_tile - 1) / row_tile;
    if (rows <= kRowBlock) {
        // Step mode: every wave of a workgroup owns whole 32-key tiles; one workgroup per compute
        // unit (its tile pairs fill the LDS), tiles spread evenly over at most ~256 workgroups.
        constexpr int kTile = 32;
        const int tiles32 = (l_cap + kTile - 1) / kTile;
        const long units = (long)batch * d->n_kv_heads;
        const long max_split = std::max<long>(1, 256 / units);
        // four double-buffered waves (measured equal or faster than eight single-buffered ones at every size)
        const int kWaves = gathered && g_decode_step_waves == 8 ? 8 : 4;
        p.step_waves = kWaves;
        long n_split = std::min<long>((tiles32 + kWaves - 1) / kWaves, max_split);
        // (in-place form: a wave's row map lives in LDS, 32 tiles at most -- more splits instead)
        if (!gathered) n_split = std::max<long>(n_split, (tiles32 + kWaves * 32 - 1) / (kWaves * 32));
        const int tpw = (int)((tiles32 + kWaves * n_split - 1) / (kWaves * n_split));
        n_split = (tiles32 + kWaves * tpw - 1) / (kWaves * tpw);
        p.n_split = (int)n_split;
        p.split_len = kWaves * tpw * kTile;
        size_t off = 0;
        p.part_o = off;
        off += align_up((size_t)batch * d->n_kv_heads * p.n_split * rows * d->head_dim * sizeof(float), 256);
        p.part_ml = off;
        off += align_up((size_t)batch * d->n_kv_heads * p.n_split * rows * sizeof(float), 256);
        p.total = off;
        return p;
    }
    // Split the keys until every compute unit has its workgroups (one of the 8-wave ring kernel,
    // two of the 4-wave kernel), but keep the partial results (fp32 rows per split) below roughly
    // the KV bytes they summarise (measured at 224 rows over 4,096 keys: 16 splits 20.0 us per
    // call, 32 splits 21.3, 22 splits 21.2, 8 splits 24.0).
    const long base_blocks = (long)batch * d->n_kv_heads * n_rtile;
    const long target = ring ? 256 : 512;
    long want = (target + base_blocks - 1) / base_blocks;
    const long cap = std::max<long>(1, (long)l_cap / rows);
    want = std::max<long>(1, std::min<long>(std::min<long>(want, cap), tiles));
    const int tiles_per = (int)((tiles + want - 1) / want);
    p.n_split = (tiles + tiles_per - 1) / tiles_per;
    p.split_len = tiles_per * kKeyTile;
    size_t off = 0;
    p.part_o = off;
    off += align_up((size_t)batch * d->n_kv_heads * p.n_split * rows * d->head_dim * sizeof(float), 256);
    p.part_ml = off;
    off += align_up((size_t)batch * d->n_kv_heads * p.n_split * rows * sizeof(float), 256);
    p.total = off;
    return p;
}

// Workspace of the in-place decode: split-KV partial results, then the row map and the lengths.
InplaceWorkspace inplace_workspace(const vxl_attn_desc* d, int batch, int T, int l_cap) {
    InplaceWorkspace w{};
    // The row map and the lengths come first: their places do not depend on the number of query
    // tokens, so a map survives calls with another n_q_tokens on the same workspace.
    size_t off = 0;
    w.src_idx = off;
    off += align_up((size_t)batch * l_cap * sizeof(int32_t), 256);
    w.mix_len = off;
    off += align_up((size_t)batch * sizeof(int32_t), 256);
    w.partials = off;
    off += align_up(std::max<size_t>(256, decode_plan(d, batch, T, l_cap, false).total), 256);
    w.total = off;
    return w;
}

}  // namespace vxl

using namespace vxl;

extern "C" {

int vxl_version(void) { return 100; }

const char* vxl_status_string(vxl_status s) {
    switch (s) {
        case VXL_OK: return "ok";
        case VXL_ERR_INVALID_ARG: return "invalid argument";
        case VXL_ERR_UNSUPPORTED: return "unsupported dtype, head_dim or chunk count";
        case VXL_ERR_WORKSPACE: return "workspace missing or too small";
        case VXL_ERR_HIP: return "HIP runtime error";
        case VXL_ERR_ALLOC: return "host or device memory allocation failed";
    }
    return "unknown status";
}

const char* vxl_last_error(void) { return g_last_error; }

// Test hook (vxl_debug.h): route BF16 calls through the plain vector-ALU kernels (an on-device
// cross-check of the matrix-core kernels).
void vxl_debug_force_simple(int on) { g_force_simple = on; }

vxl_status vxl_layout_create(int32_t n_tokens, int32_t n_prefix, int32_t n_chunks,
                             const int32_t* chunk_bounds, const int32_t* sparse_offsets,
                             const int32_t* sparse_idx, vxl_stream stream, vxl_layout** out) {
    return vxl_layout_create_windowed(n_tokens, n_prefix, n_chunks, chunk_bounds, sparse_offsets, sparse_idx,
                                      0, stream, out);
}

vxl_status vxl_layout_create_windowed(int32_t n_tokens, int32_t n_prefix, int32_t n_chunks,
                                      const int32_t* chunk_bounds, const int32_t* sparse_offsets,
                                      const int32_t* sparse_idx, int32_t window, vxl_stream stream,
                                      vxl_layout** out) {
    if (!out) return VXL_ERR_INVALID_ARG;
    *out = nullptr;
    if (n_tokens <= 0 || n_prefix < 0 || n_chunks < 0 || window < 0 || !chunk_bounds || !sparse_offsets)
        return VXL_ERR_INVALID_ARG;
    if (n_chunks > VXL_MAX_CHUNKS) return VXL_ERR_UNSUPPORTED;
    if (chunk_bounds[0] != n_prefix || chunk_bounds[n_chunks] != n_tokens || sparse_offsets[0] != 0)
        return VXL_ERR_INVALID_ARG;
    for (int c = 0; c < n_chunks; ++c) {
        if (chunk_bounds[c + 1] <= chunk_bounds[c]) return VXL_ERR_INVALID_ARG;
        if (sparse_offsets[c + 1] < sparse_offsets[c]) return VXL_ERR_INVALID_ARG;
        if (sparse_offsets[c + 1] - sparse_offsets[c] > chunk_bounds[c + 1] - chunk_bounds[c])
            return VXL_ERR_INVALID_ARG;
    }
    const int32_t s_total = sparse_offsets[n_chunks];
    if (s_total > 0 && !sparse_idx) return VXL_ERR_INVALID_ARG;
    for (int c = 0; c < n_chunks; ++c) {
        for (int32_t i = sparse_offsets[c]; i < sparse_offsets[c + 1]; ++i) {
            const int32_t t = sparse_idx[i];
            if (t < chunk_bounds[c] || t >= chunk_bounds[c + 1]) return VXL_ERR_INVALID_ARG;
            if (i > sparse_offsets[c] && t <= sparse_idx[i - 1]) return VXL_ERR_INVALID_ARG;
        }
    }

    vxl_layout* L = new (std::nothrow) vxl_layout();
    if (!L) return VXL_ERR_ALLOC;
    L->n_tokens = n_tokens; L->n_prefix = n_prefix; L->n_chunks = n_chunks; L->s_total = s_total;
    L->window = window;
    L->bounds.assign(chunk_bounds, chunk_bounds + n_chunks + 1);
    L->soff.assign(sparse_offsets, sparse_offsets + n_chunks + 1);
    if (s_total) L->sidx.assign(sparse_idx, sparse_idx + s_total);

    // segments and the closed-form pair count
    int32_t tile_base = 0;
    int64_t pairs = (int64_t)n_prefix * (n_prefix + 1) / 2;
    if (n_prefix > 0) {
        L->segs.push_back({0, n_prefix, 0, tile_base, 0});
        tile_base += (n_prefix + kKeyTile - 1) / kKeyTile;
    }
    for (int c = 0; c < n_chunks; ++c) {
        const int32_t len = chunk_bounds[c + 1] - chunk_bounds[c];
        // dense look-back range [lo, b_c); kept tokens inside it are seen through it, not twice
        const int32_t back = (int32_t)std::min<int64_t>(window, chunk_bounds[c] - n_prefix);
        const int32_t lo = chunk_bounds[c] - back;
        const int32_t* kept_begin = L->sidx.data();
        const int32_t* kept_end = kept_begin + sparse_offsets[c];
        const int32_t n_kept_before = (int32_t)(std::lower_bound(kept_begin, kept_end, lo) - kept_begin);
        const int32_t ctx = n_prefix + n_kept_before;
        L->segs.push_back({chunk_bounds[c], len, ctx, tile_base, back});
        tile_base += (len + kKeyTile - 1) / kKeyTile;
        pairs += (int64_t)len * (ctx + back) + (int64_t)len * (len + 1) / 2;
    }
    L->pair_count = pairs;
    L->n_seg = (int32_t)L->segs.size();
    L->n_own_tiles = tile_base;
    L->l_ctx = n_prefix + s_total;
    L->n_ctx_tiles = (L->l_ctx + kKeyTile - 1) / kKeyTile;

    // source token of every slot of every V tile: history tiles first, then own tiles
    std::vector<int32_t> tile_src((size_t)(L->n_ctx_tiles + L->n_own_tiles) * kKeyTile, -1);
    for (int32_t r = 0; r < L->l_ctx; ++r) tile_src[r] = r < n_prefix ? r : L->sidx[r - n_prefix];
    for (const Segment& sg : L->segs) {
        int32_t* dst = tile_src.data() + (size_t)(L->n_ctx_tiles + sg.tile_base) * kKeyTile;
        for (int32_t r = 0; r < sg.q_len; ++r) dst[r] = sg.q_start + r;
    }

    // work items, heaviest first (cost = key tiles visited)
    std::vector<WorkItem> work[2];
    for (int v = 0; v < 2; ++v) {
        const int bm = 128 << v;
        std::vector<std::pair<int64_t, WorkItem>> items;
        for (int s = 0; s < L->n_seg; ++s) {
            const Segment& sg = L->segs[s];
            const int mt = (sg.q_len + bm - 1) / bm;
            for (int m = 0; m < mt; ++m) {
                const int last = std::min(sg.q_len, (m + 1) * bm) - 1;
                const int64_t cost = (sg.ctx_len + kKeyTile - 1) / kKeyTile + (last + sg.back) / kKeyTile + 1;
                items.push_back({cost, {s, m}});
            }
        }
        std::stable_sort(items.begin(), items.end(),
                         [](const auto& a, const auto& b) { return a.first > b.first; });
        for (auto& it : items) work[v].push_back(it.second);
        L->n_work[v] = (int32_t)work[v].size();
    }

    // items of the attention-mass score: the prefix and every chunk in pieces of kMassPiece keys
    std::vector<MassItem> mass_items;
    std::vector<int32_t> mass_off(n_chunks + 1, 0);
    for (int32_t lo = 0; lo < n_prefix; lo += kMassPiece)
        mass_items.push_back({lo, std::min(lo + kMassPiece, n_prefix), -1});
    for (int c = 0; c < n_chunks; ++c) {
        mass_off[c] = (int32_t)mass_items.size();
        for (int32_t lo = chunk_bounds[c]; lo < chunk_bounds[c + 1]; lo += kMassPiece)
            mass_items.push_back({lo, std::min(lo + kMassPiece, chunk_bounds[c + 1]), c});
    }
    mass_off[n_chunks] = (int32_t)mass_items.size();
    L->n_mass_items = (int32_t)mass_items.size();

    // one device blob
    size_t off = 0;
    auto place = [&](size_t bytes) { size_t o = off; off += align_up(std::max<size_t>(bytes, 4), 256); return o; };
    const size_t o_bounds = place((n_chunks + 1) * 4), o_soff = place((n_chunks + 1) * 4);
    const size_t o_sidx = place((size_t)s_total * 4);
    const size_t o_segs = place(L->segs.size() * sizeof(Segment));
    const size_t o_tsrc = place(tile_src.size() * 4);
    const size_t o_w0 = place(work[0].size() * sizeof(WorkItem));
    const size_t o_w1 = place(work[1].size() * sizeof(WorkItem));
    const size_t o_mi = place(mass_items.size() * sizeof(MassItem));
    const size_t o_mo = place(mass_off.size() * 4);
    L->blob_bytes = off;
    std::vector<char> host(off, 0);
    memcpy(host.data() + o_bounds, L->bounds.data(), (n_chunks + 1) * 4);
    memcpy(host.data() + o_soff, L->soff.data(), (n_chunks + 1) * 4);
    if (s_total) memcpy(host.data() + o_sidx, L->sidx.data(), (size_t)s_total * 4);
    memcpy(host.data() + o_segs, L->segs.data(), L->segs.size() * sizeof(Segment));
    memcpy(host.data() + o_tsrc, tile_src.data(), tile_src.size() * 4);
    if (!work[0].empty()) memcpy(host.data() + o_w0, work[0].data(), work[0].size() * sizeof(WorkItem));
    if (!work[1].empty()) memcpy(host.data() + o_w1, work[1].data(), work[1].size() * sizeof(WorkItem));
    if (!mass_items.empty()) memcpy(host.data() + o_mi, mass_items.data(), mass_items.size() * sizeof(MassItem));
    memcpy(host.data() + o_mo, mass_off.data(), mass_off.size() * 4);

    hipError_t e = hipGetDevice(&L->device);
    if (e == hipSuccess) e = hipMalloc(&L->d_blob, off);
    if (e == hipSuccess) e = hipMemcpyAsync(L->d_blob, host.data(), off, hipMemcpyHostToDevice, (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) {
        set_last_error("vxl_layout_create", e);
        if (L->d_blob) (void)hipFree(L->d_blob);
        delete L;
        return e == hipErrorOutOfMemory ? VXL_ERR_ALLOC : VXL_ERR_HIP;
    }
    char* base = (char*)L->d_blob;
    L->d_bounds = (int32_t*)(base + o_bounds);
    L->d_soff = (int32_t*)(base + o_soff);
    L->d_sidx = (int32_t*)(base + o_sidx);
    L->d_segs = (Segment*)(base + o_segs);
    L->d_tile_src = (int32_t*)(base + o_tsrc);
    L->d_work[0] = (WorkItem*)(base + o_w0);
    L->d_work[1] = (WorkItem*)(base + o_w1);
    L->d_mass_items = (MassItem*)(base + o_mi);
    L->d_mass_off = (int32_t*)(base + o_mo);
    *out = L;
    return VXL_OK;
}

vxl_status vxl_layout_destroy(vxl_layout* L) {
    if (!L) return VXL_OK;
    vxl_status st = VXL_OK;
    if (L->d_blob) {
        hipError_t e = hipFree(L->d_blob);
        if (e != hipSuccess) { set_last_error("hipFree", e); st = VXL_ERR_HIP; }
    }
    delete L;
    return st;
}

int32_t vxl_mixed_kv_capacity(const vxl_layout* L, int32_t k) {
    if (!L) return 0;
    k = std::max(0, std::min(k, L->n_chunks));
    std::vector<int32_t> extra(L->n_chunks);
    for (int c = 0; c < L->n_chunks; ++c)
        extra[c] = (L->bounds[c + 1] - L->bounds[c]) - (L->soff[c + 1] - L->soff[c]);
    std::partial_sort(extra.begin(), extra.begin() + k, extra.end(), std::greater<int32_t>());
    int64_t cap = (int64_t)L->n_prefix + L->s_total;
    for (int i = 0; i < k; ++i) cap += extra[i];
    return (int32_t)cap;
}

int64_t vxl_prefill_pair_count(const vxl_layout* L) { return L ? L->pair_count : 0; }

size_t vxl_workspace_bytes(vxl_op op, const vxl_layout* L, const vxl_attn_desc* d, int32_t batch,
                           int32_t n_q_tokens, int32_t l_cap) {
    vxl_status st;
    if (!desc_ok(d, &st)) return 0;
    switch (op) {
        case VXL_OP_PREFILL:
            if (!L) return 0;
            return std::max<size_t>(256, prefill_workspace(L, d).total);
        case VXL_OP_SCORE_TOPK:     // mean queries [B][Hkv][D], mean keys [Hkv][C][D] (used when no cache is given), scores [B][C]
            if (!L || batch <= 0) return 0;
            return align_up((size_t)batch * d->n_kv_heads * d->head_dim * 4, 256) +
                   align_up((size_t)d->n_kv_heads * std::max(1, L->n_chunks) * d->head_dim * 4, 256) +
                   align_up((size_t)batch * std::max(1, L->n_chunks) * 4, 256);
        case VXL_OP_GATHER:          // the gather keeps its per-query offsets in LDS: no workspace
            return 0;
        case VXL_OP_DECODE:
            if (batch <= 0 || n_q_tokens <= 0 || l_cap <= 0) return 0;
            return std::max<size_t>(256, decode_plan(d, batch, n_q_tokens, l_cap).total);
        case VXL_OP_SCORE_MASS:
            if (!L || batch <= 0 || n_q_tokens <= 0) return 0;
            return std::max<size_t>(256, mass_plan(L, d, batch, n_q_tokens).total);
        case VXL_OP_DECODE_INPLACE:
            if (batch <= 0 || n_q_tokens <= 0 || l_cap <= 0) return 0;
            return inplace_workspace(d, batch, n_q_tokens, l_cap).total;
    }
    return 0;
}

vxl_status vxl_chunk_prefill(const vxl_layout* L, const vxl_attn_desc* d, const void* Q,
                             const void* K, const void* V, void* O, float* LSE, void* workspace,
                             size_t workspace_bytes, vxl_stream stream) {
    vxl_status st;
    if (!L) return VXL_ERR_INVALID_ARG;
    if (!desc_ok(d, &st)) return st;
    if (!Q || !K || !V || !O) return VXL_ERR_INVALID_ARG;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return VXL_ERR_INVALID_ARG;
    if (O == Q || O == K || O == V) return VXL_ERR_INVALID_ARG;
    const float scale = resolve_scale(d);
    if (d->dtype == VXL_BF16 && !g_force_simple) {
        const size_t need = prefill_workspace(L, d).total;
        if (!workspace || workspace_bytes < need || !aligned16(workspace)) return VXL_ERR_WORKSPACE;
        return launch_prefill_bf16(L, d, scale, Q, K, V, O, LSE, workspace, (hipStream_t)stream);
    }
    return launch_prefill_simple(L, d, scale, Q, K, V, O, LSE, (hipStream_t)stream);
}

vxl_status vxl_chunk_score_topk(const vxl_layout* L, const vxl_attn_desc* d, const void* Qd,
                                int32_t batch, int32_t n_q_tokens, const void* K, int32_t k,
                                float* kbar, int32_t kbar_ready, int32_t* topk_idx,
                                uint8_t* dense_mask, float* scores, void* workspace,
                                size_t workspace_bytes, vxl_stream stream) {
    vxl_status st;
    if (!L) return VXL_ERR_INVALID_ARG;
    if (!desc_ok(d, &st)) return st;
    if (!Qd || batch <= 0 || n_q_tokens <= 0 || k < 0 || !dense_mask) return VXL_ERR_INVALID_ARG;
    if (!aligned16(Qd)) return VXL_ERR_INVALID_ARG;
    const int kk = std::min(k, L->n_chunks);
    if (kk > 0 && !topk_idx) return VXL_ERR_INVALID_ARG;
    if (kbar_ready && !kbar) return VXL_ERR_INVALID_ARG;
    if (!kbar_ready && (!K || !aligned16(K))) return VXL_ERR_INVALID_ARG;
    if (L->n_chunks == 0) return VXL_OK;      // nothing to score, nothing to write
    const size_t need = vxl_workspace_bytes(VXL_OP_SCORE_TOPK, L, d, batch, n_q_tokens, 0);
    if (!workspace || workspace_bytes < need || !aligned16(workspace)) return VXL_ERR_WORKSPACE;
    float* qbar = (float*)workspace;
    const size_t o_kbar = align_up((size_t)batch * d->n_kv_heads * d->head_dim * 4, 256);
    const size_t o_sc = o_kbar + align_up((size_t)d->n_kv_heads * std::max(1, L->n_chunks) * d->head_dim * 4, 256);
    float* kb = kbar ? kbar : (float*)((char*)workspace + o_kbar);
    st = launch_summaries(L, d, K, kb, !kbar_ready, Qd, batch, n_q_tokens, qbar, (hipStream_t)stream);
    if (st != VXL_OK) return st;
    return launch_score_topk(L, d, resolve_scale(d), batch, kk, qbar, kb, topk_idx, dense_mask, scores,
                             (float*)((char*)workspace + o_sc), (hipStream_t)stream);
}

vxl_status vxl_chunk_score_topk_mass(const vxl_layout* L, const vxl_attn_desc* d, const void* Qd,
                                     int32_t batch, int32_t n_q_tokens, const void* K, int32_t k,
                                     int32_t* topk_idx, uint8_t* dense_mask, float* scores,
                                     void* workspace, size_t workspace_bytes, vxl_stream stream) {
    vxl_status st;
    if (!L) return VXL_ERR_INVALID_ARG;
    if (!desc_ok(d, &st)) return st;
    if (!Qd || !K || batch <= 0 || n_q_tokens <= 0 || k < 0 || !dense_mask) return VXL_ERR_INVALID_ARG;
    if (!aligned16(Qd) || !aligned16(K)) return VXL_ERR_INVALID_ARG;
    const int kk = std::min(k, L->n_chunks);
    if (kk > 0 && !topk_idx) return VXL_ERR_INVALID_ARG;
    if (L->n_chunks == 0) return VXL_OK;      // nothing to score, nothing to write
    const MassPlan p = mass_plan(L, d, batch, n_q_tokens);
    if (!workspace || workspace_bytes < p.total || !aligned16(workspace)) return VXL_ERR_WORKSPACE;
    float* sc = scores ? scores : (float*)((char*)workspace + p.scores);
    st = launch_score_mass(L, d, resolve_scale(d), Qd, batch, n_q_tokens, K, sc, workspace,
                           g_force_simple != 0, (hipStream_t)stream);
    if (st != VXL_OK) return st;
    return launch_topk_from_scores(L, sc, batch, kk, topk_idx, dense_mask, (hipStream_t)stream);
}

vxl_status vxl_gather_bilevel_kv(const vxl_layout* L, const vxl_attn_desc* d, const void* K,
                                 const void* V, const uint8_t* dense_mask, int32_t batch,
                                 void* Kmix, void* Vmix, int32_t l_cap, int32_t* mix_len,
                                 int32_t* src_idx, vxl_stream stream) {
    vxl_status st;
    if (!L) return VXL_ERR_INVALID_ARG;
    if (!desc_ok(d, &st)) return st;
    if (!K || !V || !Kmix || !Vmix || !mix_len || batch <= 0) return VXL_ERR_INVALID_ARG;
    if (L->n_chunks > 0 && !dense_mask) return VXL_ERR_INVALID_ARG;
    if (!aligned16(K) || !aligned16(V) || !aligned16(Kmix) || !aligned16(Vmix)) return VXL_ERR_INVALID_ARG;
    if (l_cap < vxl_mixed_kv_capacity(L, 0)) return VXL_ERR_INVALID_ARG;
    return launch_gather(L, d, K, V, nullptr, nullptr, dense_mask, batch, Kmix, Vmix, l_cap, mix_len, src_idx,
                         (hipStream_t)stream);
}

vxl_status vxl_pool_sparse_kv(const vxl_layout* L, const vxl_attn_desc* d, const void* K, const void* V,
                              void* Ksp, void* Vsp, vxl_stream stream) {
    vxl_status st;
    if (!L) return VXL_ERR_INVALID_ARG;
    if (!desc_ok(d, &st)) return st;
    if (!K || !V || !aligned16(K) || !aligned16(V)) return VXL_ERR_INVALID_ARG;
    if (L->s_total > 0 && (!Ksp || !Vsp || !aligned16(Ksp) || !aligned16(Vsp))) return VXL_ERR_INVALID_ARG;
    if (Ksp == K || Ksp == V || Vsp == K || Vsp == V || (Ksp && Ksp == Vsp)) return VXL_ERR_INVALID_ARG;
    return launch_pool_sparse(L, d, K, V, Ksp, Vsp, (hipStream_t)stream);
}

vxl_status vxl_gather_bilevel_kv_pooled(const vxl_layout* L, const vxl_attn_desc* d, const void* K,
                                        const void* V, const void* Ksp, const void* Vsp,
                                        const uint8_t* dense_mask, int32_t batch, void* Kmix, void* Vmix,
                                        int32_t l_cap, int32_t* mix_len, int32_t* src_idx,
                                        vxl_stream stream) {
    vxl_status st;
    if (!L) return VXL_ERR_INVALID_ARG;
    if (!desc_ok(d, &st)) return st;
    if (!K || !V || !Kmix || !Vmix || !mix_len || batch <= 0) return VXL_ERR_INVALID_ARG;
    if (L->n_chunks > 0 && !dense_mask) return VXL_ERR_INVALID_ARG;
    if (L->s_total > 0 && (!Ksp || !Vsp || !aligned16(Ksp) || !aligned16(Vsp))) return VXL_ERR_INVALID_ARG;
    if (!aligned16(K) || !aligned16(V) || !aligned16(Kmix) || !aligned16(Vmix)) return VXL_ERR_INVALID_ARG;
    if (l_cap < vxl_mixed_kv_capacity(L, 0)) return VXL_ERR_INVALID_ARG;
    // (a layout without sparse rows never reads the pooled buffers; the kernel takes the pooled
    // path only when they are given)
    return launch_gather(L, d, K, V, L->s_total > 0 ? Ksp : nullptr, L->s_total > 0 ? Vsp : nullptr, dense_mask,
                         batch, Kmix, Vmix, l_cap, mix_len, src_idx, (hipStream_t)stream);
}

vxl_status vxl_bilevel_decode(const vxl_attn_desc* d, const void* Qd, int32_t batch,
                              int32_t n_q_tokens, const void* Kmix, const void* Vmix, int32_t l_cap,
                              const int32_t* mix_len, void* O, float* LSE, void* workspace,
                              size_t workspace_bytes, vxl_stream stream) {
    vxl_status st;
    if (!desc_ok(d, &st)) return st;
    if (!Qd || !Kmix || !Vmix || !mix_len || !O || batch <= 0 || n_q_tokens <= 0 || l_cap <= 0)
        return VXL_ERR_INVALID_ARG;
    if (!aligned16(Qd) || !aligned16(Kmix) || !aligned16(Vmix) || !aligned16(O)) return VXL_ERR_INVALID_ARG;
    const float scale = resolve_scale(d);
    if (d->dtype == VXL_BF16 && !g_force_simple) {
        const size_t need = decode_plan(d, batch, n_q_tokens, l_cap).total;
        if (!workspace || workspace_bytes < need || !aligned16(workspace)) return VXL_ERR_WORKSPACE;
        return launch_decode_bf16(d, scale, Qd, batch, n_q_tokens, Kmix, Vmix, l_cap, mix_len, O,
                                  LSE, workspace, (hipStream_t)stream);
    }
    return launch_decode_simple(d, scale, Qd, batch, n_q_tokens, Kmix, Vmix, l_cap, mix_len, O, LSE,
                                (hipStream_t)stream);
}

vxl_status vxl_bilevel_decode_inplace(const vxl_layout* L, const vxl_attn_desc* d, const void* Qd,
                                      int32_t batch, int32_t n_q_tokens, const void* K, const void* V,
                                      const void* Ksp, const void* Vsp, const uint8_t* dense_mask,
                                      int32_t l_cap, int32_t map_ready, void* O, float* LSE, int32_t* mix_len,
                                      void* workspace, size_t workspace_bytes, vxl_stream stream) {
    vxl_status st;
    if (!L) return VXL_ERR_INVALID_ARG;
    if (!desc_ok(d, &st)) return st;
    if (!Qd || !K || !V || !O || batch <= 0 || n_q_tokens <= 0 || l_cap <= 0) return VXL_ERR_INVALID_ARG;
    if (L->n_chunks > 0 && !dense_mask) return VXL_ERR_INVALID_ARG;
    if ((Ksp == nullptr) != (Vsp == nullptr)) return VXL_ERR_INVALID_ARG;
    if (!aligned16(Qd) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(Ksp) || !aligned16(Vsp))
        return VXL_ERR_INVALID_ARG;
    if (l_cap < vxl_mixed_kv_capacity(L, 0)) return VXL_ERR_INVALID_ARG;
    const InplaceWorkspace w = inplace_workspace(d, batch, n_q_tokens, l_cap);
    if (!workspace || workspace_bytes < w.total || !aligned16(workspace)) return VXL_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    int32_t* src_idx = (int32_t*)((char*)workspace + w.src_idx);
    int32_t* len = mix_len ? mix_len : (int32_t*)((char*)workspace + w.mix_len);
    const bool pooled = Ksp != nullptr && L->s_total > 0;
    if (!map_ready) {           // the row map and the lengths: the gather's index pass, no row is copied
        st = launch_gather(L, d, K, V, pooled ? Ksp : nullptr, pooled ? Vsp : nullptr, dense_mask, batch, nullptr,
                           nullptr, l_cap, len, src_idx, s);
        if (st != VXL_OK) return st;
    }
    const float scale = resolve_scale(d);
    if (d->dtype == VXL_BF16 && !g_force_simple)
        return launch_decode_bf16_inplace(L, d, scale, Qd, batch, n_q_tokens, K, V, Ksp, Vsp, src_idx, l_cap, len, O,
                                          LSE, (char*)workspace + w.partials, s);
    return launch_decode_inplace_simple(L, d, scale, Qd, batch, n_q_tokens, K, V, Ksp, Vsp, src_idx, l_cap, len, O,
                                        LSE, s);
}

vxl_status vxl_bilevel_decode_static(const vxl_attn_desc* d, const void* Qd, int32_t batch,
                                     int32_t n_q_tokens, const void* Kmix, const void* Vmix, int32_t l_cap,
                                     const int32_t* mix_len, void* O, float* LSE, vxl_stream stream) {
    vxl_status st;
    if (!desc_ok(d, &st)) return st;
    if (!Qd || !Kmix || !Vmix || !mix_len || !O || batch <= 0 || n_q_tokens <= 0 || l_cap <= 0)
        return VXL_ERR_INVALID_ARG;
    if (!aligned16(Qd) || !aligned16(Kmix) || !aligned16(Vmix) || !aligned16(O)) return VXL_ERR_INVALID_ARG;
    const float scale = resolve_scale(d);
    if (d->dtype == VXL_BF16 && !g_force_simple) {
        const size_t need = decode_plan(d, batch, n_q_tokens, l_cap).total;
        if (need > (size_t)VXL_STATIC_SCRATCH_BYTES) {
            snprintf(g_last_error, sizeof(g_last_error),
                     "vxl_bilevel_decode_static: the split-KV partial results of this call need %zu bytes, the "
                     "static scratch holds %zu", need, (size_t)VXL_STATIC_SCRATCH_BYTES);
            return VXL_ERR_WORKSPACE;
        }
        void* ws = nullptr;
        st = decode_static_scratch(&ws);
        if (st != VXL_OK) return st;
        return launch_decode_bf16(d, scale, Qd, batch, n_q_tokens, Kmix, Vmix, l_cap, mix_len, O, LSE, ws,
                                  (hipStream_t)stream);
    }
    return launch_decode_simple(d, scale, Qd, batch, n_q_tokens, Kmix, Vmix, l_cap, mix_len, O, LSE,
                                (hipStream_t)stream);
}

}  // extern "C"
