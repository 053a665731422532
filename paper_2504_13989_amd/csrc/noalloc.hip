// rq_quant_error_noalloc: rq_quant_error for callers that cannot allocate device memory (code under
// HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  The per-row partial
// sums that rq_quant_error keeps in the caller's workspace live in a static device array instead.
//
// Every GPU the library runs on holds its own copy of the array, at its own address, until the
// process ends.  The array's name is only a host-side stand-in for it: its device address on a given
// GPU is asked for once (hipGetSymbolAddress, with that GPU current) and that address is what the
// kernels receive.  All calls on one GPU share the array: calls that overlap in time on one GPU
// (different streams or host threads) race on it and must be ordered by the caller.
#include <mutex>

#include "rotq_internal.h"

namespace {

static __device__ __align__(256) unsigned char scratch[RQ_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];       // device address of `scratch` per device, nullptr = not yet asked
std::mutex g_scratch_mu;

}  // namespace

void* rq::static_scratch(int dev) {
    if (dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_ptr[dev]) return g_scratch_ptr[dev];
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess || cur != dev) {
        (void)hipGetLastError();
        return nullptr;                 // the address can only be asked for on the device itself
    }
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
        (void)hipGetLastError();
        return nullptr;
    }
    g_scratch_ptr[dev] = p;
    return p;
}

extern "C" int rq_quant_error_noalloc(const rq_hadamard_t* h, const void* X, int dtype, int64_t rows, int d,
                                      int64_t ld, int bits, const float* clips, int n_clips, float* mse,
                                      void* stream) {
    if (!h) return RQ_ERR_ARG;
    const size_t need = rq_quant_error_workspace(rows, n_clips);
    if (need == 0) return RQ_ERR_ARG;                        // rows < 0 or n_clips out of range
    if (need > (size_t)RQ_NOALLOC_SCRATCH_BYTES) return RQ_ERR_TOO_LARGE;
    if (h->device < 0) return RQ_ERR_HIP;
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess || cur != h->device) {
        (void)hipGetLastError();
        return RQ_ERR_HIP;                                   // the handle's tables live on another device
    }
    void* ptr = rq::static_scratch(h->device);               // resolved when the handle was built
    if (!ptr) return RQ_ERR_HIP;
    // every partial sum the reduction reads is written by this call's own row kernel first, so nothing
    // in the array has to start at zero
    return rq::quant_error_impl(h, X, dtype, rows, d, ld, bits, clips, n_clips, mse, ptr,
                                (size_t)RQ_NOALLOC_SCRATCH_BYTES, stream, false);
}
