// spd_op_attention_static: the stand-alone single-query attention for callers that cannot
// allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
// forbid hipMalloc).  Same kernels as spd_op_attention; the scratch they need (one arrival
// counter line per head and the per-chunk partial results that the last block of a head
// merges) lives in a file-scope device array instead of a caller-supplied buffer.
//
// Every GPU the library runs on holds its own copy of that array, at its own address, until
// the process ends.  The array's name is only a host-side handle: its device address is looked
// up once per device with hipGetSymbolAddress and that pointer is what kernels and fills get.
// All calls on one GPU share the array: calls that overlap on one GPU (different streams or
// threads) race; calls on one stream are ordered and each clears the counters it needs.
#include "spd_internal.h"

#include <mutex>

namespace {

static __device__ __align__(256) unsigned char scratch[SPD_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
void *scratch_ptr[MAX_DEVICES];   // device address of `scratch` on each device, once looked up
std::mutex scratch_mu;

hipError_t scratch_of_current_device(void **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(scratch_mu);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

extern "C" int spd_op_attention_static(int32_t dtype, const float *q, const void *K, const void *V, float *out,
                                       int32_t n_heads, int32_t n_kv_heads, int32_t d_head, int32_t n_ctx,
                                       int32_t cap_ctx, void *hip_stream) {
    const int rc = spdk::attention_args_status(dtype, q, K, V, out, n_heads, n_kv_heads, d_head, n_ctx, cap_ctx);
    if (rc != SPD_OK) return rc;
    const size_t need = spd_op_attention_scratch_bytes(n_heads, d_head, cap_ctx);
    if (need == 0) return SPD_EINVAL;
    if (need > (size_t)SPD_STATIC_SCRATCH_BYTES) return SPD_EWORKSPACE;   // more heads x chunks than the static array holds
    void *ptr = nullptr;
    if (scratch_of_current_device(&ptr) != hipSuccess) {
        (void)hipGetLastError();
        return SPD_EHIP;
    }
    return spdk::attention_on_scratch((hipStream_t)hip_stream, dtype, q, K, V, out, ptr, n_heads, n_kv_heads, d_head,
                                      n_ctx, cap_ctx);
}
