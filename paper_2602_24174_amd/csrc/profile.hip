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
// any class but the whole-step ones, whose brackets sit outside the step's launches
bool tasc_prof_any() { return (g_mask & ~((1u << TASC_KC_VERIFY) | (1u << TASC_KC_DRAFT))) != 0; }

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

extern "C" tasc_status tasc_profile_durations(int32_t cls, double* ms, int64_t cap, int64_t* n) {
    TASC_REQUIRE(n && cap >= 0 && (ms || cap == 0), "profile_durations: null argument");
    TASC_REQUIRE(cls >= 0 && cls < TASC_N_KERNEL_CLASSES, "profile_durations: class %d outside [0, %d)", cls, TASC_N_KERNEL_CLASSES);
    TASC_HIP(hipDeviceSynchronize());
    std::lock_guard<std::mutex> lk(g_mu);
    int64_t k = 0;
    for (Pair& p : g_used) {
        if (p.cls != cls) continue;
        float t = 0.f;
        if (hipEventElapsedTime(&t, p.a, p.b) != hipSuccess) continue;
        if (k < cap) ms[k] = t;
        ++k;
    }
    *n = k;
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

namespace {
typedef __attribute__((ext_vector_type(8))) __bf16 cal_bf16x8;
typedef __attribute__((ext_vector_type(16))) float cal_f32x16;
// 8 independent accumulators of 32 x 32 per wave, operands in registers: nothing but the MFMA pipe is busy
__global__ __launch_bounds__(512) void k_calibration_mfma(int iters, float* sink) {
    cal_bf16x8 a[2], b[4];
    for (int i = 0; i < 2; ++i)
        for (int e = 0; e < 8; ++e) a[i][e] = (__bf16)(float)((threadIdx.x + i + e) & 7);
    for (int i = 0; i < 4; ++i)
        for (int e = 0; e < 8; ++e) b[i][e] = (__bf16)(float)((threadIdx.x * 3 + i + e) & 7);
    cal_f32x16 acc[2][4];
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 4; ++j)
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 4; ++j)
            for (int e = 0; e < 16; ++e) s += acc[i][j][e];
    if (s == -1.0f) sink[0] = s;        // sums of non-negative products: never true, keeps the loop
}
}  // namespace

extern "C" tasc_status tasc_calibration_mfma(int32_t iters, void* stream, double* tflops) {
    TASC_REQUIRE(iters >= 1 && iters <= 100000 && tflops, "calibration_mfma: iters %d outside [1, 100000] or null result", iters);
    hipStream_t st = (hipStream_t)stream;
    int dev = 0, cus = 0;
    TASC_HIP(hipGetDevice(&dev));
    TASC_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    float* sink = nullptr;
    TASC_HIP(hipMalloc((void**)&sink, sizeof(float)));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    float ms = 0.f;
    if (e == hipSuccess) {
        k_calibration_mfma<<<dim3(cus), dim3(512), 0, st>>>(iters, sink);      // warm-up (clocks, code fetch)
        e = hipEventRecord(e0, st);
        k_calibration_mfma<<<dim3(cus), dim3(512), 0, st>>>(iters, sink);
        if (e == hipSuccess) e = hipEventRecord(e1, st);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(sink);
    if (e != hipSuccess) {
        tasc_set_error("calibration_mfma: %s", hipGetErrorString(e));
        return TASC_EHIP;
    }
    // per wave and iteration: 32 MFMAs of 32 x 32 x 16 (2 * 32 * 32 * 16 flop each); 8 waves per workgroup
    *tflops = (double)cus * 8.0 * iters * 32.0 * 32768.0 / (ms * 1e-3) / 1e12;
    return TASC_OK;
}

namespace {
typedef unsigned int cal_u32x4 __attribute__((ext_vector_type(4)));
// read stream: a workgroup of 512 threads takes blocks of 64 KB, 8 independent 16-byte loads per lane, nothing stored
__global__ __launch_bounds__(512) void k_calibration_read(const cal_u32x4* __restrict__ src, size_t n_blocks, size_t steps, unsigned* sink) {
    cal_u32x4 acc = {0, 0, 0, 0};
    for (size_t it = 0; it < steps; ++it) {
        const size_t blk = (it * gridDim.x + blockIdx.x) % n_blocks;
        const cal_u32x4* p = src + blk * 4096 + threadIdx.x;
        cal_u32x4 r[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) r[q] = p[q * 512];
#pragma unroll
        for (int q = 0; q < 8; ++q) acc ^= r[q];
    }
    if (acc[0] == 0x9e3779b9u && acc[1] == 0x7f4a7c15u && acc[2] == 0x94d049bbu && acc[3] == 0xbf58476du) sink[0] = acc[0];   // keeps the loads
}
}  // namespace

extern "C" tasc_status tasc_calibration_read(const void* src, size_t bytes, int32_t passes, void* stream, double* gbps) {
    TASC_REQUIRE(src && gbps && bytes >= 65536 && bytes % 65536 == 0 && ((uintptr_t)src & 15) == 0 && passes >= 1 && passes <= 1000000,
                 "calibration_read: 16-byte aligned buffer of a multiple of 64 KB and 1 .. 1000000 passes needed");
    hipStream_t st = (hipStream_t)stream;
    int dev = 0, cus = 0;
    TASC_HIP(hipGetDevice(&dev));
    TASC_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const size_t n_blocks = bytes / 65536;
    const unsigned wgs = (unsigned)cus;
    const size_t steps = (n_blocks * (size_t)passes + wgs - 1) / wgs;
    TASC_REQUIRE(steps <= ((size_t)1 << 26), "calibration_read: %zu blocks x %d passes is too much work for one launch", n_blocks, passes);
    unsigned* sink = nullptr;
    TASC_HIP(hipMalloc((void**)&sink, sizeof(unsigned)));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    float ms = 0.f;
    if (e == hipSuccess) {
        k_calibration_read<<<dim3(wgs), dim3(512), 0, st>>>((const cal_u32x4*)src, n_blocks, steps < 64 ? steps : 64, sink);   // warm-up
        e = hipEventRecord(e0, st);
        k_calibration_read<<<dim3(wgs), dim3(512), 0, st>>>((const cal_u32x4*)src, n_blocks, steps, sink);
        if (e == hipSuccess) e = hipEventRecord(e1, st);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(sink);
    if (e != hipSuccess) {
        tasc_set_error("calibration_read: %s", hipGetErrorString(e));
        return TASC_EHIP;
    }
    *gbps = (double)wgs * (double)steps * 65536.0 / (ms * 1e-3) / 1e9;
    return TASC_OK;
}

extern "C" tasc_status tasc_calibration_copy(void* dst, const void* src, size_t bytes, void* stream) {
    TASC_REQUIRE(dst && src && bytes % 16 == 0 && ((uintptr_t)dst & 15) == 0 && ((uintptr_t)src & 15) == 0,
                 "calibration_copy: buffers must be 16-byte aligned and a multiple of 16 bytes long");
    k_calibration_copy<<<dim3(4096), dim3(256), 0, (hipStream_t)stream>>>((const uint4*)src, (uint4*)dst, bytes / 16);
    TASC_LAUNCH_CHECK();
    return TASC_OK;
}

// ---------------------------------------------------------------- hand-over latency between resident workgroups
namespace {
constexpr int kHandoverPhases = 200;
constexpr unsigned kHandoverLds = 100 * 1024;      // forces one workgroup per compute unit: every participant is resident

// `n_part` workgroups (ids stride * j) exchange `units` 8-byte words per phase, each writing its contiguous share and
// then reading all of them.  mode 0: "flag in data" -- the words start as a sentinel, readers poll the words themselves
// (agent-scope loads and stores) until none is the sentinel; three buffers are used in turn and an owner resets its
// words once it has seen the next phase complete.  mode 1: the classic way -- data stored (agent scope), stores waited
// for, one arrival flag per participant, one wave polls the flags, then the data is loaded.
__global__ __launch_bounds__(512) void k_calibration_handover(u64* buf, u32* flags, int mode, int units, int stride, int n_part, u32* err, u64* ticks) {
    const int wg = blockIdx.x;
    if (wg % stride != 0 || wg / stride >= n_part) return;
    const int r = wg / stride;
    const int per = (units + n_part - 1) / n_part;
    __shared__ u32 s_w[8];
    u32 acc = 1;
    u64 t0 = 0;
    if (threadIdx.x == 0) t0 = wall_clock64();
    for (int ph = 0; ph < kHandoverPhases; ++ph) {
        u64* b = buf + (size_t)(mode == 0 ? ph % 3 : ph) * units;
        u64* bprev = buf + (size_t)((ph + 2) % 3) * units;
        for (int j = threadIdx.x; j < per; j += 512) {
            const int u = r * per + j;
            if (u < units) __hip_atomic_store(b + u, ((u64)(u32)ph << 32) | (acc & 0xFFFFu), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (mode == 1) {
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            if (threadIdx.x < 64) {
                if (threadIdx.x == 0) __hip_atomic_store(flags + r, (u32)(ph + 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                u32 spins = 0;
                for (int base = 0; base < n_part; base += 64) {
                    for (;;) {
                        u32 f = ph + 1;
                        if (base + (int)threadIdx.x < n_part) f = __hip_atomic_load(flags + base + threadIdx.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        if (__all((int)(f - (u32)(ph + 1)) >= 0)) break;
                        if (++spins > (1u << 16)) { atomicOr(err, 1u); break; }
                    }
                }
            }
            __syncthreads();
        }
        u32 mine = 0;
        for (int u = threadIdx.x; u < units; u += 512) {
            u64 v;
            u32 spins = 0;
            for (;;) {
                v = __hip_atomic_load(b + u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (mode == 1 || v != ~0ull) break;
                if (++spins > (1u << 16)) { atomicOr(err, 1u); break; }
            }
            if ((u32)(v >> 32) != (u32)ph) atomicOr(err, 2u);          // stale or foreign data
            mine += (u32)v;
        }
        for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o);
        if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = mine;
        __syncthreads();
        acc = s_w[0] + s_w[1] + s_w[2] + s_w[3] + s_w[4] + s_w[5] + s_w[6] + s_w[7];
        if (mode == 0 && ph > 0)
            for (int j = threadIdx.x; j < per; j += 512) {
                const int u = r * per + j;
                if (u < units) __hip_atomic_store(bprev + u, ~0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        __syncthreads();
        if (*(volatile u32*)err & 1u) break;
    }
    if (threadIdx.x == 0 && r == 0) { ticks[0] = wall_clock64() - t0; ticks[1] = acc; }
}
__global__ void k_calibration_fill(u64* p, size_t n, u64 v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}
}  // namespace

extern "C" tasc_status tasc_calibration_handover(int32_t n_workgroups, int32_t stride, int32_t bytes, int32_t with_flags, void* stream,
                                                 double* us_per_handover) {
    TASC_REQUIRE(us_per_handover && n_workgroups >= 2 && stride >= 1 && bytes >= 8 && bytes % 8 == 0 && bytes <= (1 << 20),
                 "calibration_handover: 2 or more workgroups, stride >= 1 and 8 .. 2^20 bytes (a multiple of 8) needed");
    hipStream_t st = (hipStream_t)stream;
    int dev = 0, cus = 0;
    TASC_HIP(hipGetDevice(&dev));
    TASC_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    TASC_REQUIRE((long)(n_workgroups - 1) * stride < cus, "calibration_handover: %d workgroups at stride %d do not fit %d compute units",
                 n_workgroups, stride, cus);
    static bool attr = false;
    if (!attr) {
        TASC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_calibration_handover), hipFuncAttributeMaxDynamicSharedMemorySize, kHandoverLds));
        attr = true;
    }
    const int units = bytes / 8, mode = with_flags ? 1 : 0;
    const size_t words = (size_t)kHandoverPhases * units;
    u64* buf = nullptr;
    TASC_HIP(hipMalloc((void**)&buf, words * 8 + 4096 + 64));
    u32* flags = reinterpret_cast<u32*>(buf + words);
    u32* err = flags + 1024 - 16;
    u64* ticks = reinterpret_cast<u64*>(flags + 1024);
    double best = 1e30;
    u32 herr = 0;
    hipError_t e = hipSuccess;
    for (int rep = 0; rep < 3 && e == hipSuccess && !herr; ++rep) {
        k_calibration_fill<<<dim3(256), dim3(256), 0, st>>>(buf, words, ~0ull);
        k_calibration_fill<<<dim3(1), dim3(256), 0, st>>>(reinterpret_cast<u64*>(flags), 512 + 8, 0ull);
        k_calibration_handover<<<dim3(cus), dim3(512), kHandoverLds, st>>>(buf, flags, mode, units, stride, n_workgroups, err, ticks);
        e = hipGetLastError();
        u64 h[2] = {0, 0};
        if (e == hipSuccess) e = hipMemcpyAsync(h, ticks, 16, hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipMemcpyAsync(&herr, err, 4, hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        const double us = (double)h[0] * 0.01 / kHandoverPhases;         // 100 MHz clock
        if (us < best) best = us;
    }
    (void)hipFree(buf);
    if (e != hipSuccess) {
        tasc_set_error("calibration_handover: %s", hipGetErrorString(e));
        return TASC_EHIP;
    }
    if (herr) {
        tasc_set_error("calibration_handover: %s", (herr & 2u) ? "a reader saw stale data" : "a wait timed out (are all workgroups resident?)");
        return TASC_EHIP;
    }
    *us_per_handover = best;
    return TASC_OK;
}
