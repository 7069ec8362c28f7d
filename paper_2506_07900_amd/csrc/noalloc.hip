// infllmv2_sparse_attn_decode_noalloc: stage 3 of a decode step for callers that cannot hand over a
// workspace they allocated -- code under HIP graph capture, tight serving loops, harnesses that forbid
// hipMalloc.  The per-block partial results (o, max, sum) of the split-KV attention live in a fixed
// array in device memory that is part of the library's code object; everything else is
// infllmv2_sparse_attn_decode unchanged (the same kernels, the same bits).
#include <atomic>
#include <mutex>

#include "common.h"

using namespace infllmv2;

namespace {

constexpr size_t kScratchBytes = INFLLMV2_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// In host code `scratch` is only a handle for hipGetSymbolAddress: each GPU holds its own copy of the
// array at its own address, looked up once per device (with that device current) and kept here.
constexpr int kMaxDevices = 64;
std::mutex g_lock;
void *g_scratch_ptr[kMaxDevices];
std::atomic<bool> g_have[kMaxDevices];

int scratch_for_current_device(void **ptr) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    if (!g_have[dev].load(std::memory_order_acquire)) {
        std::lock_guard<std::mutex> guard(g_lock);
        if (!g_have[dev].load(std::memory_order_relaxed)) {
            void *p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return (int)e;
            if (!p) return (int)hipErrorInvalidSymbol;
            g_scratch_ptr[dev] = p;
            g_have[dev].store(true, std::memory_order_release);
        }
    }
    *ptr = g_scratch_ptr[dev];
    return 0;
}

}  // namespace

extern "C" int32_t infllmv2_sparse_attn_decode_noalloc(const infllmv2_params *prm, const infllmv2_tensor *q,
                                                        const infllmv2_tensor *k, const infllmv2_tensor *v,
                                                        const int32_t *seqlens, int32_t batch, int32_t max_seqlen,
                                                        const int32_t *block_idx, const infllmv2_tensor *out,
                                                        float *lse, void *stream) {
    Dims dm;
    Tensor tq, tk, tv, tout;
    const int32_t st = validate_attn_decode(prm, q, k, v, seqlens, batch, max_seqlen, block_idx, out, lse, &dm, &tq,
                                            &tk, &tv, &tout);
    if (st != INFLLMV2_OK) return st;
    if (attn_decode_ws_bytes(dm) > kScratchBytes) return INFLLMV2_ERR_UNSUPPORTED;   // beyond the fixed array
    void *ws = nullptr;
    if (scratch_for_current_device(&ws) != 0) return INFLLMV2_ERR_HIP;
    return launch_attn_decode(dm, tq, tk, tv, seqlens, block_idx, nullptr, tout, lse, ws,
                              reinterpret_cast<hipStream_t>(stream)) == 0
               ? INFLLMV2_OK
               : INFLLMV2_ERR_HIP;
}
