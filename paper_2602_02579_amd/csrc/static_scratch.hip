// pkv_query_score_static: the query score for callers that cannot allocate device
// memory (code under graph capture, tight serving loops, harnesses that forbid it).
// The kernels are those of pkv_query_score; their scratch (per-column normalisers,
// per-range partial normalisers, per-block partial column sums) lives in a file-scope
// device array instead of a caller-provided workspace.
//
// Every GPU the library runs on holds its own copy of the array, at its own address,
// until the process ends.  The array's name is only a handle on the host: the address
// kernels and runtime calls need comes from hipGetSymbolAddress, asked once per device
// with that device current, and kept.
#include <atomic>

#include "pkv_common.h"

namespace {

constexpr size_t kScratchBytes = PKV_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of this GPU's copy of `scratch`, resolved on the first call on a device.
pkv_status scratch_address(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return PKV_ERR_LAUNCH;
    if (dev < 0 || dev >= kMaxDevices) return PKV_ERR_UNSUPPORTED;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p)
            return PKV_ERR_LAUNCH;
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // same value from any thread
    }
    *out = p;
    return PKV_OK;
}

}  // namespace

extern "C" pkv_status pkv_query_score_static(const pkv_layer_cfg* cfg, const void* q,
                                             const void* k, float* score, int64_t nq,
                                             int64_t n_ctx, float softmax_scale,
                                             int accumulate, void* stream) {
    // sizes first: a problem whose scratch does not fit the array is refused before
    // anything touches the device
    if (!cfg) return PKV_ERR_NULL;
    if (nq > 0 && n_ctx > 0 &&
        pkv_workspace_bytes(PKV_CALL_QUERY_SCORE, cfg, n_ctx, nq) > kScratchBytes)
        return PKV_ERR_WORKSPACE;
    void* ptr = nullptr;
    const pkv_status st = scratch_address(&ptr);
    if (st != PKV_OK) return st;
    // nothing in the scratch has to start at zero: every kernel writes what the next reads
    return pkv_query_score(cfg, q, k, score, nq, n_ctx, softmax_scale, accumulate, ptr,
                           kScratchBytes, stream);
}
