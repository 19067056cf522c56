// LayerNorm backward for callers that cannot allocate (code under HIP graph capture, tight serving
// loops, harnesses that forbid hipMalloc): the column-reduction partials that bp_op_layernorm_bwd
// takes from a caller-supplied workspace live here in a file-scope device array instead.  Each GPU
// the library runs on holds its own copy of the array, at its own address, until the process ends.
#include <atomic>

#include "bp_host.h"

namespace {

// [row chunks of 32][2][H] floats: 8 MiB covers T*H <= 32 Mi elements (e.g. 4096 x 5120, 8192 x 4096)
constexpr size_t kScratchFloats = (size_t)2 << 20;
static __device__ __align__(256) float scratch[kScratchFloats];

constexpr int kMaxDevices = 64;
// device address of `scratch` on each GPU, looked up once per device with that device current
std::atomic<float*> g_scratch_ptr[kMaxDevices];

int scratch_of_current_device(float** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return bp::fail(BP_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return bp::fail(BP_EINVAL, "device %d outside 0..%d", dev, kMaxDevices - 1);
    float* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        // the array's name is only a host-side handle: the device address comes from the runtime
        e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            return bp::fail(BP_EHIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
        }
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // same value from every thread
    }
    *out = p;
    return BP_OK;
}

}  // namespace

extern "C" {

size_t bp_static_scratch_floats(void) { return kScratchFloats; }

int bp_op_layernorm_bwd_static(int dtype, int T, int H, const void* dout, const void* x, const float* mean,
                               const float* rstd, const float* gamma, const void* residual_grad, void* dx,
                               float* dgamma, float* dbeta, void* stream) {
    if (dtype != BP_F32 && dtype != BP_BF16) return bp::fail(BP_EINVAL, "unknown dtype %d", dtype);
    if (!dout || !x || !mean || !rstd || !gamma || !dx || !dgamma || !dbeta) return bp::fail(BP_EINVAL, "null pointer");
    if (T <= 0 || H <= 0) return bp::fail(BP_EINVAL, "T and H must be positive");
    if (H % 8 || H > 8192) return bp::fail(BP_ESHAPE, "H = %d must be a multiple of 8 and at most 8192", H);
    const size_t need = bp::colsum_chunks(T) * (size_t)H * 2;
    if (need > kScratchFloats)
        return bp::fail(BP_ESHAPE, "T = %d, H = %d needs %zu floats of scratch, the static buffer holds %zu "
                        "(use bp_op_layernorm_bwd with a workspace)", T, H, need, kScratchFloats);
    float* ws = nullptr;
    int rc = scratch_of_current_device(&ws);
    if (rc) return rc;
    // every partial the second reduction kernel reads is written by the first one of this call, so
    // nothing left over from an earlier call has to be cleared
    hipError_t e = bp::launch_colsum(dtype, T, H, dout, x, mean, rstd, dbeta, dgamma, ws, (hipStream_t)stream);
    if (e != hipSuccess) return bp::fail(BP_EHIP, "column reduction: %s", hipGetErrorString(e));
    e = bp::launch_ln_bwd_rows(dtype, T, H, dout, x, mean, rstd, gamma, residual_grad, dx, (hipStream_t)stream);
    if (e != hipSuccess) return bp::fail(BP_EHIP, "row kernel: %s", hipGetErrorString(e));
    return BP_OK;
}

}  // extern "C"
