// Offline (host-memory) bi-level KV store ("Bi-level KVs Decoding": the dense and the sparse KVs
// of every chunk are kept in an offline memory; for a query, dense KVs are reloaded for the
// relevant chunks and sparse KVs for the others, and concatenated into the mixed KV set).
//
// The store holds pinned host copies of the dense K/V [Hkv, N, D] and of the sparse K/V
// [Hkv, S_total, D] of one layer.  Reloading builds the mixed KV set of every query directly in
// device memory with strided host-to-device copies: rows of one source (dense or sparse) that are
// consecutive in the mixed set form one run, and a run is one 2-D copy over all KV heads (row
// pitch = the head stride of its source / of the mixed buffer).  Everything is asynchronous on the
// caller's stream, so a reload for the next query can run on a side stream beside the decode of
// the current one.
#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "vxl_internal.h"

struct vxl_kv_store {
    int32_t n_tokens = 0, n_prefix = 0, n_chunks = 0, s_total = 0;
    int32_t n_kv_heads = 0, head_dim = 0;
    size_t elem = 0;
    bool strided = false;                  // the device K, V are not dense [Hkv, N, D]
    long long kv_head = 0, kv_tok = 0;     // their strides, in elements
    std::vector<int32_t> bounds, soff;
    // pinned host memory (one allocation): dense K, dense V, sparse K, sparse V
    void* h_blob = nullptr;
    size_t blob_bytes = 0;
    char *h_k = nullptr, *h_v = nullptr, *h_ksp = nullptr, *h_vsp = nullptr;
};

namespace {
// The mixed lengths reach the device as launch arguments of a one-block kernel: the values are
// copied when the call is made, so reloads issued back to back (on one stream or on several) never
// share a host staging buffer.
constexpr int kMaxReloadBatch = 256;     // lengths per launch (1 KiB of kernel arguments)
struct LenArgs { int32_t v[kMaxReloadBatch]; };
__global__ void write_lens_kernel(int32_t* __restrict__ dst, LenArgs a, int n) {
    if ((int)threadIdx.x < n) dst[threadIdx.x] = a.v[threadIdx.x];
}
}

using namespace vxl;

extern "C" {

vxl_status vxl_kv_store_create(const vxl_layout* L, const vxl_attn_desc* d, vxl_kv_store** out) {
    if (!out) return VXL_ERR_INVALID_ARG;
    *out = nullptr;
    if (!L || !d) return VXL_ERR_INVALID_ARG;
    if (d->n_kv_heads <= 0 || (d->head_dim != 64 && d->head_dim != 128) ||
        (d->dtype != VXL_F32 && d->dtype != VXL_BF16))
        return VXL_ERR_UNSUPPORTED;
    if (!dense_layout(d) && (d->kv_stride_head <= 0 || d->kv_stride_tok < d->head_dim)) return VXL_ERR_INVALID_ARG;
    vxl_kv_store* S = new (std::nothrow) vxl_kv_store();
    if (!S) return VXL_ERR_ALLOC;
    S->n_tokens = L->n_tokens; S->n_prefix = L->n_prefix; S->n_chunks = L->n_chunks; S->s_total = L->s_total;
    S->n_kv_heads = d->n_kv_heads; S->head_dim = d->head_dim;
    S->elem = d->dtype == VXL_BF16 ? 2 : 4;
    const TokStrides ts = tok_strides(d, L->n_tokens);
    S->strided = !dense_layout(d);
    S->kv_head = ts.kh; S->kv_tok = ts.kt;
    S->bounds = L->bounds; S->soff = L->soff;
    const size_t dense = align_up((size_t)S->n_kv_heads * S->n_tokens * S->head_dim * S->elem, 256);
    const size_t sparse = align_up((size_t)S->n_kv_heads * std::max(1, S->s_total) * S->head_dim * S->elem, 256);
    S->blob_bytes = 2 * dense + 2 * sparse;
    hipError_t e = hipHostMalloc(&S->h_blob, S->blob_bytes, hipHostMallocDefault);
    if (e != hipSuccess) {
        set_last_error("hipHostMalloc", e);
        delete S;
        return e == hipErrorOutOfMemory ? VXL_ERR_ALLOC : VXL_ERR_HIP;
    }
    char* p = (char*)S->h_blob;
    S->h_k = p; p += dense;
    S->h_v = p; p += dense;
    S->h_ksp = p; p += sparse;
    S->h_vsp = p;
    *out = S;
    return VXL_OK;
}

vxl_status vxl_kv_store_destroy(vxl_kv_store* S) {
    if (!S) return VXL_OK;
    vxl_status st = VXL_OK;
    if (S->h_blob) {
        hipError_t e = hipHostFree(S->h_blob);
        if (e != hipSuccess) { set_last_error("hipHostFree", e); st = VXL_ERR_HIP; }
    }
    delete S;
    return st;
}

size_t vxl_kv_store_host_bytes(const vxl_kv_store* S) { return S ? S->blob_bytes : 0; }

vxl_status vxl_kv_store_offload(vxl_kv_store* S, const void* K, const void* V, const void* Ksp,
                                const void* Vsp, vxl_stream stream) {
    if (!S || !K || !V) return VXL_ERR_INVALID_ARG;
    if (S->s_total > 0 && (!Ksp || !Vsp)) return VXL_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const size_t dense = (size_t)S->n_kv_heads * S->n_tokens * S->head_dim * S->elem;
    const size_t sparse = (size_t)S->n_kv_heads * S->s_total * S->head_dim * S->elem;
    if (!S->strided) {
        VXL_HIP_TRY(hipMemcpyAsync(S->h_k, K, dense, hipMemcpyDeviceToHost, s));
        VXL_HIP_TRY(hipMemcpyAsync(S->h_v, V, dense, hipMemcpyDeviceToHost, s));
    } else {                                                  // the host copy is dense: one strided copy per KV head
        const size_t row = (size_t)S->head_dim * S->elem, head = (size_t)S->n_tokens * row;
        for (int g = 0; g < S->n_kv_heads; ++g) {
            const size_t src = (size_t)g * S->kv_head * S->elem;
            VXL_HIP_TRY(hipMemcpy2DAsync(S->h_k + g * head, row, (const char*)K + src, (size_t)S->kv_tok * S->elem,
                                         row, S->n_tokens, hipMemcpyDeviceToHost, s));
            VXL_HIP_TRY(hipMemcpy2DAsync(S->h_v + g * head, row, (const char*)V + src, (size_t)S->kv_tok * S->elem,
                                         row, S->n_tokens, hipMemcpyDeviceToHost, s));
        }
    }
    if (sparse) {
        VXL_HIP_TRY(hipMemcpyAsync(S->h_ksp, Ksp, sparse, hipMemcpyDeviceToHost, s));
        VXL_HIP_TRY(hipMemcpyAsync(S->h_vsp, Vsp, sparse, hipMemcpyDeviceToHost, s));
    }
    return VXL_OK;
}

vxl_status vxl_kv_store_reload(vxl_kv_store* S, const uint8_t* dense_mask, int32_t batch, void* Kmix,
                               void* Vmix, int32_t l_cap, int32_t* mix_len_host, int32_t* mix_len,
                               vxl_stream stream) {
    if (!S || !Kmix || !Vmix || batch <= 0 || l_cap <= 0) return VXL_ERR_INVALID_ARG;
    if (S->n_chunks > 0 && !dense_mask) return VXL_ERR_INVALID_ARG;
    if (mix_len && batch > kMaxReloadBatch) return VXL_ERR_UNSUPPORTED;
    hipStream_t s = (hipStream_t)stream;
    const size_t row = (size_t)S->head_dim * S->elem;
    const int C = S->n_chunks;
    // lengths first: nothing is copied if a query does not fit
    std::vector<int32_t> lens(batch);
    for (int b = 0; b < batch; ++b) {
        int64_t len = S->n_prefix;
        for (int c = 0; c < C; ++c)
            len += dense_mask[(size_t)b * C + c] ? S->bounds[c + 1] - S->bounds[c] : S->soff[c + 1] - S->soff[c];
        if (len > l_cap) return VXL_ERR_INVALID_ARG;
        lens[b] = (int32_t)len;
    }
    for (int b = 0; b < batch; ++b) {
        char* kd = (char*)Kmix + (size_t)b * S->n_kv_heads * l_cap * row;
        char* vd = (char*)Vmix + (size_t)b * S->n_kv_heads * l_cap * row;
        // one run = consecutive mixed rows that are consecutive rows of one source
        auto copy_run = [&](bool from_dense, int64_t src_row, int64_t dst_row, int64_t n_rows) -> hipError_t {
            if (n_rows <= 0) return hipSuccess;
            const size_t spitch = (size_t)(from_dense ? S->n_tokens : S->s_total) * row;
            const char* ks = (from_dense ? S->h_k : S->h_ksp) + (size_t)src_row * row;
            const char* vs = (from_dense ? S->h_v : S->h_vsp) + (size_t)src_row * row;
            hipError_t e = hipMemcpy2DAsync(kd + (size_t)dst_row * row, (size_t)l_cap * row, ks, spitch,
                                            (size_t)n_rows * row, S->n_kv_heads, hipMemcpyHostToDevice, s);
            if (e != hipSuccess) return e;
            return hipMemcpy2DAsync(vd + (size_t)dst_row * row, (size_t)l_cap * row, vs, spitch,
                                    (size_t)n_rows * row, S->n_kv_heads, hipMemcpyHostToDevice, s);
        };
        // the prefix joins a dense first chunk (token ids continue)
        bool run_dense = true;
        int64_t run_src = 0, run_dst = 0, run_rows = S->n_prefix, dst = S->n_prefix;
        for (int c = 0; c < C; ++c) {
            const bool dn = dense_mask[(size_t)b * C + c] != 0;
            const int64_t src0 = dn ? S->bounds[c] : S->soff[c];
            const int64_t n = dn ? S->bounds[c + 1] - S->bounds[c] : S->soff[c + 1] - S->soff[c];
            if (n == 0) continue;
            if (run_rows > 0 && dn == run_dense && src0 == run_src + run_rows) {
                run_rows += n;
            } else {
                VXL_HIP_TRY(copy_run(run_dense, run_src, run_dst, run_rows));
                run_dense = dn; run_src = src0; run_dst = dst; run_rows = n;
            }
            dst += n;
        }
        VXL_HIP_TRY(copy_run(run_dense, run_src, run_dst, run_rows));
        if (mix_len_host) mix_len_host[b] = lens[b];
    }
    if (mix_len) {
        LenArgs a{};
        std::copy(lens.begin(), lens.end(), a.v);
        hipLaunchKernelGGL(write_lens_kernel, dim3(1), dim3(kMaxReloadBatch), 0, s, mix_len, a, (int)batch);
        VXL_HIP_TRY(hipGetLastError());
    }
    return VXL_OK;
}

}  // extern "C"
