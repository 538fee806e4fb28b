// Optional per-kernel-class device timing: HIP event pairs recorded on the stream the kernel is
// launched on.  Off by default; with a class enabled, every launch of that class is bracketed.
#include "tasc_internal.h"
#include <mutex>

namespace {
struct Pair { hipEvent_t a, b; int cls; };
std::mutex g_mu;
uint32_t g_mask = 0;
std::vector<Pair> g_used;
std::vector<Pair> g_free;
}  // namespace

bool tasc_prof_on(int cls) { return (g_mask >> cls) & 1u; }

int tasc_prof_begin(int cls, hipStream_t st) {
    std::lock_guard<std::mutex> lk(g_mu);
    Pair p;
    if (!g_free.empty()) {
        p = g_free.back();
        g_free.pop_back();
    } else {
        if (hipEventCreate(&p.a) != hipSuccess) return -1;
        if (hipEventCreate(&p.b) != hipSuccess) { (void)hipEventDestroy(p.a); return -1; }
    }
    p.cls = cls;
    (void)hipEventRecord(p.a, st);
    g_used.push_back(p);
    return (int)g_used.size() - 1;
}

void tasc_prof_end(int handle, hipStream_t st) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (handle >= 0 && handle < (int)g_used.size()) (void)hipEventRecord(g_used[handle].b, st);
}

extern "C" tasc_status tasc_profile_enable(uint32_t class_mask) {
    std::lock_guard<std::mutex> lk(g_mu);
    g_mask = class_mask & ((1u << TASC_N_KERNEL_CLASSES) - 1);
    return TASC_OK;
}

extern "C" tasc_status tasc_profile_read(double* total_ms, int64_t* launches) {
    TASC_REQUIRE(total_ms && launches, "profile_read: null argument");
    TASC_HIP(hipDeviceSynchronize());
    std::lock_guard<std::mutex> lk(g_mu);
    for (int c = 0; c < TASC_N_KERNEL_CLASSES; ++c) { total_ms[c] = 0.0; launches[c] = 0; }
    for (Pair& p : g_used) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) {
            total_ms[p.cls] += ms;
            launches[p.cls] += 1;
        }
        g_free.push_back(p);
    }
    g_used.clear();
    return TASC_OK;
}

// Plain copy kernel of known size: the reference against which hardware byte counters are scaled.
namespace {
__global__ void k_calibration_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) dst[i] = src[i];
}
}  // namespace

extern "C" tasc_status tasc_calibration_copy(void* dst, const void* src, size_t bytes, void* stream) {
    TASC_REQUIRE(dst && src && bytes % 16 == 0 && ((uintptr_t)dst & 15) == 0 && ((uintptr_t)src & 15) == 0,
                 "calibration_copy: buffers must be 16-byte aligned and a multiple of 16 bytes long");
    k_calibration_copy<<<dim3(4096), dim3(256), 0, (hipStream_t)stream>>>((const uint4*)src, (uint4*)dst, bytes / 16);
    TASC_LAUNCH_CHECK();
    return TASC_OK;
}
