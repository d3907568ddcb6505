// dmr_qlinear_forward_static: dmr_qlinear_forward for callers that cannot hand over a workspace they
// allocated (code under HIP-graph capture, tight serving loops, harnesses that forbid hipMalloc).  The
// partial sums that the split-K kernels otherwise keep in the caller's workspace live in one array in
// device memory that is part of this library's code object: every GPU the library runs on holds its own
// copy at its own address until the process ends.  Nothing is allocated or freed here or below.
#include <atomic>

#include "common.hpp"

namespace {

constexpr size_t kScratchBytes = DMR_STATIC_SCRATCH_BYTES;

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device, resolved once per device (in host code the array's
// name is only a handle for this lookup, not an address a kernel could use).
dmr_status_t scratch_on_current_device(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DMR_ERR_HIP;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DMR_ERR_HIP;
        g_scratch_ptr[dev].store(p, std::memory_order_release);    // every thread resolves the same address
    }
    *out = p;
    return DMR_OK;
}

}  // namespace

extern "C" {

dmr_status_t dmr_qlinear_forward_static(const dmr_qlinear_t *layer, const uint16_t *d_x, int64_t M, void *d_y,
                                        dmr_out_t out, void *stream) {
    if (!layer) return DMR_ERR_NULL;
    if (M < 0 || M > (int64_t(1) << 22)) return DMR_ERR_SHAPE;
    if (out != DMR_OUT_BF16 && out != DMR_OUT_FP32) return DMR_ERR_UNSUPPORTED;
    if (M == 0) return DMR_OK;
    if (!d_x || !d_y) return DMR_ERR_NULL;
    int64_t K = 0, N = 0;
    if (dmr_qlinear_shape(layer, &K, &N, nullptr) != DMR_OK) return DMR_ERR_NULL;
    const size_t need = dmr_qlinear_bits(layer) == 3 ? dmr_qlinear_w3_workspace_bytes(M, K, N)
                                                     : dmr_qlinear_workspace_bytes(M, K, N);
    if (need > kScratchBytes) return DMR_ERR_WORKSPACE;      // beyond the fixed scratch: use dmr_qlinear_forward
    if (need == 0) return dmr_qlinear_forward(layer, d_x, M, d_y, out, nullptr, 0, stream);
    void *ws = nullptr;
    const dmr_status_t st = scratch_on_current_device(&ws);
    if (st != DMR_OK) return st;
    // The kernels write every partial sum before the reduction pass reads it, so nothing has to be cleared
    // between calls; what the previous call left behind is simply overwritten.
    return dmr_qlinear_forward(layer, d_x, M, d_y, out, ws, kScratchBytes, stream);
}

}  // extern "C"
