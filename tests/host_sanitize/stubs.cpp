// Host-only stand-ins for everything the ABI layer (csrc/cf_api.cpp) calls below itself: the kernel launchers
// and the handful of HIP runtime functions.  Nothing runs on a device; every launch is appended to a log so the
// driver can check the launch sequence a call makes.  Used only by the sanitizer build of the CPU tests.
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "cf_internal.h"

std::vector<std::string> g_launch_log;
bool g_capturing = false;
static void note(const char *what) { g_launch_log.push_back(what); }

extern "C" {
hipError_t hipGetDevice(int *d) { *d = 0; return hipSuccess; }
hipError_t hipGetLastError(void) { return hipSuccess; }
hipError_t hipDeviceGetAttribute(int *v, hipDeviceAttribute_t, int) { *v = 256; return hipSuccess; }
hipError_t hipStreamIsCapturing(hipStream_t, hipStreamCaptureStatus *s)
{
    *s = g_capturing ? hipStreamCaptureStatusActive : hipStreamCaptureStatusNone;
    return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipMemcpy(void *dst, const void *src, size_t n, hipMemcpyKind) { std::memcpy(dst, src, n); return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
}

namespace cf {
// tables really are written (into the host buffer that plays the workspace), so the driver can read them back
hipError_t launch_upload_ptrs(const PtrChunk &chunk, TensorPtrs *dst, int n, hipStream_t)
{
    note("k_upload_ptrs");
    std::memcpy(dst, chunk.p, sizeof(TensorPtrs) * (size_t)n);
    return hipSuccess;
}
hipError_t launch_upload_bytes(const void *src, void *dst, size_t bytes, hipStream_t)
{
    std::memcpy(dst, src, bytes);
    return hipSuccess;
}
hipError_t launch_fill_words(void *dst, uint32_t value, size_t n_words, hipStream_t)
{
    uint32_t *w = static_cast<uint32_t *>(dst);
    for (size_t i = 0; i < n_words; ++i) w[i] = value;
    return hipSuccess;
}
hipError_t launch_fill_item_tensor(const uint32_t *item_prefix, uint32_t *item_tensor, int n_tensors, hipStream_t)
{
    for (int t = 0; t < n_tensors; ++t)
        for (uint32_t i = item_prefix[t]; i < item_prefix[t + 1]; ++i) item_tensor[i] = (uint32_t)t;
    return hipSuccess;
}
hipError_t launch_warmup(const BatchView &, const LaunchRange &, int, hipStream_t) { note("k_warmup"); return hipSuccess; }
hipError_t launch_colreduce(const BatchView &, const LaunchRange &, int, int, hipStream_t) { note("k_colreduce"); return hipSuccess; }
hipError_t launch_finalize(const BatchView &, const LaunchRange &, hipStream_t) { note("k_finalize"); return hipSuccess; }
hipError_t launch_finalize_rank1(const BatchView &, const LaunchRange &, hipStream_t) { note("k_finalize_rank1"); return hipSuccess; }
hipError_t launch_encode(const BatchView &, const LaunchRange &, int, int, bool, hipStream_t) { note("k_encode"); return hipSuccess; }
hipError_t launch_encode_nm(const BatchView &, const LaunchRange &, int, int, bool, bool, hipStream_t) { note("k_encode_nm"); return hipSuccess; }
hipError_t launch_decode(const BatchView &, const LaunchRange &, hipStream_t) { note("k_decode"); return hipSuccess; }
hipError_t launch_lr_orth(const BatchView &, const LaunchRange &, bool, int, hipStream_t) { note("k_lr_orth"); return hipSuccess; }
hipError_t launch_lr_project(const BatchView &, const LaunchRange &, bool, int, hipStream_t) { note("k_lr_project"); return hipSuccess; }
hipError_t launch_lr_backproject(const BatchView &, const LaunchRange &, int, hipStream_t) { note("k_lr_backproject"); return hipSuccess; }
hipError_t launch_lr_quant_u(const BatchView &, const LaunchRange &, hipStream_t) { note("k_lr_quant_u"); return hipSuccess; }
hipError_t launch_lr_encode(const BatchView &, const LaunchRange &, int, bool, hipStream_t) { note("k_lr_apply"); return hipSuccess; }
hipError_t launch_lr_decode(const BatchView &, const LaunchRange &, hipStream_t) { note("k_lr_apply"); return hipSuccess; }
int persistent_max_blocks_per_cu(int, int, bool, bool) { return 2; }
hipError_t launch_single_pass(const BatchView &, const LaunchRange &, int, int, bool, bool, int, bool, bool redo, hipStream_t)
{
    note(redo ? "k_single_pass_redo" : "k_single_pass");
    return hipSuccess;
}
hipError_t launch_reset_partials(const BatchView &, const LaunchRange &, const PtrChunk &chunk, TensorPtrs *dst, int n, hipStream_t)
{
    if (n > 0) note("ptrs_in_reset");       // the call's last batch of pointer sets rides along
    note("k_reset_partials");
    if (n > 0) std::memcpy(dst, chunk.p, sizeof(TensorPtrs) * (size_t)n);
    return hipSuccess;
}
hipError_t static_scratch(void **ptr)
{
    static void *buf = nullptr;
    if (!buf && posix_memalign(&buf, 256, kStaticScratchBytes) != 0) return hipErrorOutOfMemory;
    *ptr = buf;
    return hipSuccess;
}
}  // namespace cf
