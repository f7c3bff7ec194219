// masked_argmax for callers that cannot allocate device memory (code under HIP graph capture,
// tight serving loops, harnesses that forbid hipMalloc): the same two kernels as
// fsmidx_masked_argmax, with the slice results -- one 64-bit word per (sequence, slice) -- kept in
// a fixed array of this library's own instead of a caller's workspace.
#include <mutex>

#include "internal.h"

namespace fsmidx {

constexpr int kStaticArgmaxBatch = 4096;      // sequences per call that the fixed array has room for
constexpr size_t kScratchBytes = (size_t)kStaticArgmaxBatch * kArgmaxSplits * sizeof(uint64_t);   // 2 MiB

// Every GPU that this library runs on holds its own copy of this array, at its own address, until
// the process ends.  In host code the name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_lock;
static void *g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU, once looked up

// The address of the current device's copy of `scratch` (looked up on the first call on a device).
static int scratch_address(void **out)
{
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess)
        return fail(FSMIDX_HIP_ERROR, "hipGetDevice: %s", hipGetErrorString(e));
    if (device < 0 || device >= kMaxDevices)
        return fail(FSMIDX_UNSUPPORTED, "device %d: only devices 0..%d are supported", device, kMaxDevices - 1);
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[device]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(FSMIDX_HIP_ERROR, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return FSMIDX_OK;
}

}  // namespace fsmidx

using namespace fsmidx;

extern "C" int fsmidx_masked_argmax_static(const fsmidx_csr *index, const int32_t *states_dev, int32_t batch,
                                           const void *logits, int64_t row_stride, int32_t dtype,
                                           int32_t *tokens_out_dev, int32_t *states_out_dev, void *stream_v)
{
    size_t need = 0;
    if (int rc = check_argmax_call(index, states_dev, batch, logits, row_stride, dtype, tokens_out_dev, states_out_dev,
                                   &need))
        return rc;
    if (batch > kStaticArgmaxBatch)
        return fail(FSMIDX_INVALID_ARG, "batch %d exceeds the %d sequences that the library's own scratch array holds; "
                                        "use fsmidx_masked_argmax with a workspace", batch, kStaticArgmaxBatch);
    if (batch == 0)
        return FSMIDX_OK;
    void *partial = nullptr;
    if (int rc = scratch_address(&partial))
        return rc;
    // Nothing has to start at zero: the first kernel writes every slice word of sequences
    // [0, batch) before the second reads them, and neither touches the words beyond.
    hipError_t e = launch_argmax(*index, states_dev, batch, logits, row_stride, dtype, static_cast<uint64_t *>(partial),
                                 tokens_out_dev, states_out_dev, static_cast<hipStream_t>(stream_v));
    if (e != hipSuccess)
        return fail(FSMIDX_HIP_ERROR, "launch of masked_argmax: %s", hipGetErrorString(e));
    return FSMIDX_OK;
}
