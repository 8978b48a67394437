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
}  // namespace
// out: device float [n_workgroups * 512]; returns the number of floating-point operations launched
// (0 on a bad argument).
extern "C" double vxl_debug_mfma_stream(float* out, int n_workgroups, int iters, void* stream) {
    if (!out || n_workgroups <= 0 || iters <= 0) return 0.0;
    hipLaunchKernelGGL(mfma_stream_kernel, dim3(n_workgroups), dim3(512), 0, (hipStream_t)stream, out, iters, 1.0f);
    if (hipGetLastError() != hipSuccess) return 0.0;
    return (double)n_workgroups * 8.0 * iters * 4.0 * 2.0 * 32 * 32 * 16;
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
