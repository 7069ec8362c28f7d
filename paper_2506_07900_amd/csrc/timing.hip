// Measurement entry points of the bench-only build of the library (libinfllmv2_bench.so, every source
// compiled with INFLLMV2_TIMING): per-kernel event timing around each launch of the entry points, and
// the probe kernels.  None of this is in libinfllmv2.so, whose launches carry no timing hooks.
#include "common.h"

#include "../../include/infllmv2_bench.h"

#ifndef INFLLMV2_TIMING
#error "timing.hip belongs to the bench build (-DINFLLMV2_TIMING)"
#endif

namespace {
constexpr int kMaxTimed = 256;
bool g_timing = false;
int g_timed = 0;
hipEvent_t g_ev[2 * kMaxTimed];
bool g_ev_made = false;
const char *g_names[kMaxTimed];
}  // namespace

namespace infllmv2 {
void timing_begin(const char *kernel_name, hipStream_t stream) {
    if (!g_timing || g_timed >= kMaxTimed) return;
    g_names[g_timed] = kernel_name;
    (void)hipEventRecord(g_ev[2 * g_timed], stream);
}
void timing_end(hipStream_t stream) {
    if (!g_timing || g_timed >= kMaxTimed) return;
    (void)hipEventRecord(g_ev[2 * g_timed + 1], stream);
    ++g_timed;
}
}  // namespace infllmv2

extern "C" {

int32_t infllmv2_timing_enable(int32_t enable) {
    if (enable && !g_ev_made) {
        for (int i = 0; i < 2 * kMaxTimed; ++i)
            if (hipEventCreate(&g_ev[i]) != hipSuccess) return INFLLMV2_ERR_HIP;
        g_ev_made = true;
    }
    g_timing = enable != 0;
    g_timed = 0;
    return INFLLMV2_OK;
}

int32_t infllmv2_timing_read(int32_t max_entries, const char **names, float *ms) {
    if (max_entries < 0 || (max_entries > 0 && (!names || !ms))) return INFLLMV2_ERR_INVALID_ARGUMENT;
    const int n = g_timed < max_entries ? g_timed : max_entries;
    for (int i = 0; i < n; ++i) {
        if (hipEventSynchronize(g_ev[2 * i + 1]) != hipSuccess) return INFLLMV2_ERR_HIP;
        if (hipEventElapsedTime(&ms[i], g_ev[2 * i], g_ev[2 * i + 1]) != hipSuccess) return INFLLMV2_ERR_HIP;
        names[i] = g_names[i];
    }
    g_timed = 0;
    return n;
}

int32_t infllmv2_probe_peaks(void *buf, size_t buf_bytes, double *mfma_flops, double *stream_bytes, void *stream) {
    if (!buf || !mfma_flops || !stream_bytes || buf_bytes < (size_t)(8u << 20) ||
        (reinterpret_cast<uintptr_t>(buf) & 255u) != 0)
        return INFLLMV2_ERR_INVALID_ARGUMENT;
    return infllmv2::launch_probes(buf, buf_bytes, mfma_flops, stream_bytes, reinterpret_cast<hipStream_t>(stream)) == 0
               ? INFLLMV2_OK : INFLLMV2_ERR_HIP;
}

int32_t infllmv2_probe_detail(void *buf, size_t buf_bytes, double *work, void *stream) {
    if (!buf || !work || buf_bytes < (size_t)(8u << 20) || (reinterpret_cast<uintptr_t>(buf) & 255u) != 0)
        return INFLLMV2_ERR_INVALID_ARGUMENT;
    return infllmv2::launch_probes_detail(buf, buf_bytes, work, reinterpret_cast<hipStream_t>(stream)) == 0
               ? INFLLMV2_OK : INFLLMV2_ERR_HIP;
}

}  // extern "C"
