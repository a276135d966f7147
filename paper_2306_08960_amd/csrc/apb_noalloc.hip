// apb_quantize_forward_static: the quantize + forward step for callers that cannot allocate.  The
// packed activations, which apb_quantize_forward passes through a workspace of the caller, pass
// through a static array in device memory instead.
#include <atomic>
#include <cmath>

#include "apb_internal.h"

namespace {

// One copy per GPU, at an address of its own on each.  In host code the name below only stands for
// the symbol: the device address comes from hipGetSymbolAddress (scratch_of_current_device) and is
// what every kernel argument uses.
static __device__ __align__(256) unsigned char scratch[APB_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device, resolved once per device.
int scratch_of_current_device(void** out) {
    int dev = 0;
    APB_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return APB_ERR_SHAPE;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        APB_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return APB_ERR_HIP;
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // two threads resolve the same address
    }
    *out = p;
    return APB_OK;
}

}  // namespace

using namespace apb;

extern "C" int apb_quantize_forward_static(const apb_layer* layer, const float* X, int M, int bits, float step, float* Y,
                                           void* stream) {
    if (!layer || !X || !Y) return APB_ERR_NULL;
    const LayerDev& d = layer->d;
    if (bad_shape_acts(d.K, M) || (long long)d.N * M >= (1LL << 40)) return APB_ERR_SHAPE;
    if (bits != 1 && bits != 2) return APB_ERR_BITS;
    if (!std::isfinite(step) || !(step > 0.0f)) return APB_ERR_VALUE;
    const size_t Mp = (size_t)kWave * (((size_t)M + kWave - 1) / kWave);
    const size_t need = sizeof(uint32_t) * Mp * ((size_t)bits * d.Kw + 1);    // = apb_acts_bytes(K, M, bits)
    if (need > (size_t)APB_STATIC_SCRATCH_BYTES) return APB_ERR_SCRATCH;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (forward_float_applies(d, M, bits)) return launch_forward_float(d, X, M, bits, step, Y, s);   // one kernel, no scratch
    void* base = nullptr;
    int rc = scratch_of_current_device(&base);
    if (rc != APB_OK) return rc;
    // The quantize kernel overwrites every plane word of this K x M, and every column sum the forward kernel
    // reads (it clears the sums first, with a fill kernel, where it adds to them), so nothing of an earlier
    // call is read.
    uint32_t* planes = static_cast<uint32_t*>(base);
    int32_t* colsum = reinterpret_cast<int32_t*>(planes + (size_t)bits * d.Kw * Mp);
    return launch_quantize_then_forward(d, X, M, bits, step, planes, colsum, Y, s);
}
