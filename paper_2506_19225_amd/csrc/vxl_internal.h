// Internal declarations shared by the host API layer and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>
#include <vector>

#include "vxl.h"
#include "vxl_debug.h"

namespace vxl {

constexpr int kKeyTile = 64;      // keys per K/V tile of the matrix-core kernels
constexpr int kRowBlock = 32;     // query rows per MFMA block (one 32x32 tile side)

// One pre-filling segment: the prefix (if any) or a chunk.  Queries of a segment attend to the
// first ctx_len rows of the compacted history buffer, to the `back` tokens right before the
// segment (the sliding chunk window's dense look-back range; 0 without a window) and, causally,
// to their own segment: row r of the segment sees the dense rows [q_start - back, q_start + r].
struct Segment {
    int32_t q_start;    // first token id
    int32_t q_len;      // tokens in the segment
    int32_t ctx_len;    // visible history rows: 0 for the prefix; for chunk c, P + the number of
                        // kept tokens of earlier chunks that lie before the look-back range
    int32_t tile_base;  // index of the segment's first own-V tile among the own tiles
    int32_t back;       // dense look-back rows: min(window, b_c - P)
};

struct WorkItem {
    int32_t seg;
    int32_t m_tile;     // query row tile inside the segment
};

// One item of the attention-mass score: a piece (at most kMassPiece keys) of the prefix or of a
// chunk.  The prefix pieces come first, then the pieces of the chunks in chunk order.
constexpr int kMassPiece = 1024;
struct MassItem {
    int32_t key_lo, key_hi;   // token range [key_lo, key_hi)
    int32_t chunk;            // -1 for the prefix
};

}  // namespace vxl

struct vxl_layout {
    int32_t n_tokens = 0, n_prefix = 0, n_chunks = 0, s_total = 0, window = 0;
    std::vector<int32_t> bounds, soff, sidx;          // host copies
    int device = 0;

    // ---- device metadata (single allocation `d_blob`) ----
    void* d_blob = nullptr;
    size_t blob_bytes = 0;
    int32_t* d_bounds = nullptr;      // [C+1]
    int32_t* d_soff = nullptr;        // [C+1]
    int32_t* d_sidx = nullptr;        // [S_total]
    // pre-filling schedule
    int32_t n_seg = 0;
    int32_t l_ctx = 0;                // P + S_total rows of compacted history
    int32_t n_ctx_tiles = 0;          // ceil(l_ctx / 64)
    int32_t n_own_tiles = 0;          // sum over segments of ceil(q_len / 64)
    std::vector<vxl::Segment> segs;   // host copy
    vxl::Segment* d_segs = nullptr;   // [n_seg]
    int32_t* d_tile_src = nullptr;    // [(n_ctx_tiles + n_own_tiles) * 64] source token per
                                      // tile slot, -1 = padding
    vxl::WorkItem* d_work[2] = {nullptr, nullptr};   // heaviest-first items for 128 / 256 rows
    int32_t n_work[2] = {0, 0};
    int64_t pair_count = 0;
    // attention-mass score: item table and, per chunk, its range of items
    int32_t n_mass_items = 0;
    vxl::MassItem* d_mass_items = nullptr;   // [n_mass_items]
    int32_t* d_mass_off = nullptr;           // [C+1]: items of chunk c are [off[c], off[c+1])
};

namespace vxl {

void set_last_error(const char* what, hipError_t e);

#define VXL_HIP_TRY(expr)                                        \
    do {                                                         \
        hipError_t _e = (expr);                                  \
        if (_e != hipSuccess) {                                  \
            ::vxl::set_last_error(#expr, _e);                    \
            return VXL_ERR_HIP;                                  \
        }                                                        \
    } while (0)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// One-time set-up per device (kernel attributes, device properties), safe to reach from several
// host threads: `run(f)` calls f() once for the current device, under a lock, and remembers a
// success; a failure is returned and tried again by the next call.
constexpr int kMaxDevices = 64;
class PerDeviceOnce {
    std::mutex mu_;
    bool done_[kMaxDevices] = {};

  public:
    template <typename F>
    vxl_status run(F&& f) {
        int dev = 0;
        VXL_HIP_TRY(hipGetDevice(&dev));
        if (dev < 0 || dev >= kMaxDevices) return VXL_ERR_UNSUPPORTED;
        std::lock_guard<std::mutex> lock(mu_);
        if (done_[dev]) return VXL_OK;
        const vxl_status st = f();
        if (st == VXL_OK) done_[dev] = true;
        return st;
    }
};
// Compute units of the current device (at least 8), cached per device.
vxl_status device_cu_count(int* n_cus);

// ---- pre-filling ----
// Element strides of the per-layer tensors (the descriptor's, or the dense head-major default).
struct TokStrides {
    long long qh, qt, kh, kt;
};
inline TokStrides tok_strides(const vxl_attn_desc* d, int n_tokens) {
    if (d->q_stride_tok == 0)
        return {(long long)n_tokens * d->head_dim, d->head_dim, (long long)n_tokens * d->head_dim, d->head_dim};
    return {d->q_stride_head, d->q_stride_tok, d->kv_stride_head, d->kv_stride_tok};
}
inline bool dense_layout(const vxl_attn_desc* d) { return d->q_stride_tok == 0; }

struct PrefillWorkspace {      // byte offsets into the caller's workspace (bf16 path)
    size_t kctx;               // [Hkv][n_ctx_tiles*64][D] compacted history keys
    size_t vctx;               // [Hkv][n_ctx_tiles*64][D] compacted history values
    size_t queue;              // 8 int counters: next work index per queue of the persistent kernel
    size_t total;
};
PrefillWorkspace prefill_workspace(const vxl_layout* L, const vxl_attn_desc* d);

vxl_status launch_prefill_bf16(const vxl_layout* L, const vxl_attn_desc* d, float scale,
                               const void* Q, const void* K, const void* V, void* O, float* LSE,
                               void* ws, hipStream_t s);
vxl_status launch_prefill_simple(const vxl_layout* L, const vxl_attn_desc* d, float scale,
                                 const void* Q, const void* K, const void* V, void* O, float* LSE,
                                 hipStream_t s);

// ---- scoring / selection / gather ----
vxl_status launch_summaries(const vxl_layout* L, const vxl_attn_desc* d, const void* K, float* kbar,
                            bool do_chunks, const void* Qd, int batch, int T, float* qbar, hipStream_t s);
vxl_status launch_score_topk(const vxl_layout* L, const vxl_attn_desc* d, float scale, int batch, int k,
                             const float* qbar, const float* kbar, int32_t* topk_idx, uint8_t* dense_mask,
                             float* scores, float* scores_ws /*[B][C], used when scores is null*/, hipStream_t s);
vxl_status launch_topk_from_scores(const vxl_layout* L, const float* scores, int batch, int k,
                                   int32_t* topk_idx, uint8_t* dense_mask, hipStream_t s);

// attention-mass score
struct MassPlan {              // byte offsets into the caller's workspace
    size_t part_m, part_l;     // [B][Hkv][n_mass_items][G*T] per-item maximum (base 2) and sum
    size_t row_m, row_il;      // [B][Hkv][G*T] per-row maximum and reciprocal of the total sum
    size_t scores;             // [B][C] (used when the caller does not ask for the scores)
    size_t total;
};
MassPlan mass_plan(const vxl_layout* L, const vxl_attn_desc* d, int batch, int T);
vxl_status launch_score_mass(const vxl_layout* L, const vxl_attn_desc* d, float scale, const void* Qd,
                             int batch, int T, const void* K, float* scores, void* ws, bool force_simple,
                             hipStream_t s);

// Ksp / Vsp: pooled sparse rows [Hkv, S_total, D] read instead of the kept rows, or null
vxl_status launch_gather(const vxl_layout* L, const vxl_attn_desc* d, const void* K, const void* V,
                         const void* Ksp, const void* Vsp, const uint8_t* dense_mask, int batch, void* Kmix,
                         void* Vmix, int l_cap, int32_t* mix_len, int32_t* src_idx, hipStream_t s);
vxl_status launch_pool_sparse(const vxl_layout* L, const vxl_attn_desc* d, const void* K, const void* V,
                              void* Ksp, void* Vsp, hipStream_t s);

// ---- decode ----
struct DecodePlan {
    int n_split;        // key splits per (batch, kv head)
    int split_len;      // keys per split (multiple of 64)
    int use_ring;          // 129+ stacked rows: 1 = the 256-row ring kernel, 0 = the 128-row 4-wave kernel
    int step_waves;     // step mode: waves per workgroup (8 single-buffered or 4 double-buffered), else 0
    size_t part_o;      // byte offsets into the workspace
    size_t part_ml;
    size_t total;
};
// gathered = false plans the in-place form (always the 4-wave step kernel, splits bounded by its row-map area)
DecodePlan decode_plan(const vxl_attn_desc* d, int batch, int T, int l_cap, bool gathered = true);

struct InplaceWorkspace {      // byte offsets into the caller's workspace (vxl_bilevel_decode_inplace)
    size_t partials;           // the decode plan's partial results
    size_t src_idx;            // [B][l_cap] int32 row map
    size_t mix_len;            // [B] int32 (used when the caller does not ask for the lengths)
    size_t total;
};
InplaceWorkspace inplace_workspace(const vxl_attn_desc* d, int batch, int T, int l_cap);

vxl_status launch_decode_bf16(const vxl_attn_desc* d, float scale, const void* Qd, int batch, int T,
                              const void* Kmix, const void* Vmix, int l_cap, const int32_t* mix_len,
                              void* O, float* LSE, void* ws, hipStream_t s);
vxl_status launch_decode_bf16_inplace(const vxl_layout* L, const vxl_attn_desc* d, float scale, const void* Qd,
                                      int batch, int T, const void* K, const void* V, const void* Ksp,
                                      const void* Vsp, const int32_t* src_idx, int l_cap, const int32_t* mix_len,
                                      void* O, float* LSE, void* ws, hipStream_t s);
vxl_status launch_decode_inplace_simple(const vxl_layout* L, const vxl_attn_desc* d, float scale, const void* Qd,
                                        int batch, int T, const void* K, const void* V, const void* Ksp,
                                        const void* Vsp, const int32_t* src_idx, int l_cap,
                                        const int32_t* mix_len, void* O, float* LSE, hipStream_t s);
// device address of this device's static decode scratch (VXL_STATIC_SCRATCH_BYTES bytes)
vxl_status decode_static_scratch(void** ptr);
vxl_status launch_decode_simple(const vxl_attn_desc* d, float scale, const void* Qd, int batch, int T,
                                const void* Kmix, const void* Vmix, int l_cap, const int32_t* mix_len,
                                void* O, float* LSE, hipStream_t s);

}  // namespace vxl
