// GQA decode attention over the mixed KV set: split-KV partials on the matrix cores and the
// fixed-order log-sum-exp merge.
#include <math.h>

#include "vxl_internal.h"

namespace vxl {

vxl_status launch_decode_bf16(const vxl_attn_desc* d, float scale, const void* Qd, int batch, int T,
                              const void* Kmix, const void* Vmix, int l_cap, const int32_t* mix_len,
                              void* O, float* LSE, void* ws, hipStream_t s) {
    (void)ws;
    return launch_decode_simple(d, scale, Qd, batch, T, Kmix, Vmix, l_cap, mix_len, O, LSE, s);
}

}  // namespace vxl
