// Statistics of a finished count table: Shannon entropy, Renyi entropy of order 2 and the number of entries,
// most frequent first, that reach a given share of the total count (paper, "Task-Induced n-Grams Concentration":
// n-gram entropy and unique n-grams attaining 80 % of the CDF; Appendix, "Predicting Model Speedup ... from the
// Data": H_alpha(p) = log(sum p^alpha) / (1 - alpha)).  The distribution is count / total over the table's entries.
//
// Integers stay exact: entry count, total and the coverage count (a radix select over the 32-bit counts, one byte
// per pass, on (entries, mass) histograms).  The two fp64 sums (c ln c and c^2) are taken per workgroup and added
// in workgroup order by one thread, so a table gives the same bits on every run.
#include "tasc_internal.h"

namespace {
constexpr int kStatThreads = 256;
constexpr int kStatBlocksMax = 1024;

struct SelectState {          // device-resident state of the radix select
    u64 need;                 // mass to reach
    u64 above_entries;        // entries with a count above the current prefix range
    u64 above_mass;
    u32 prefix;               // the selected high bytes so far
    u32 done;                 // 1 once the threshold is fixed (need == 0 or nothing to select)
    u64 n_cover;
};

__device__ inline u32 entry_count(const unsigned char* base, size_t stride, u64 i) {
    return *reinterpret_cast<const u32*>(base + i * stride);
}

// per-workgroup partial sums: entries, total (exact), sum c ln c, sum c^2 (fp64)
__global__ __launch_bounds__(kStatThreads) void k_table_moments(const unsigned char* base, size_t stride, u64 n, u64* part_n, u64* part_t,
                                                                double* part_l, double* part_q) {
    u64 cn = 0, ct = 0;
    double cl = 0.0, cq = 0.0;
    for (u64 i = (u64)blockIdx.x * kStatThreads + threadIdx.x; i < n; i += (u64)gridDim.x * kStatThreads) {
        const u32 c = entry_count(base, stride, i);
        if (c) {
            const double x = (double)c;
            cn += 1;
            ct += c;
            cl += x * log(x);
            cq += x * x;
        }
    }
    __shared__ u64 s_n[kStatThreads], s_t[kStatThreads];
    __shared__ double s_l[kStatThreads], s_q[kStatThreads];
    s_n[threadIdx.x] = cn; s_t[threadIdx.x] = ct; s_l[threadIdx.x] = cl; s_q[threadIdx.x] = cq;
    __syncthreads();
    for (int w = kStatThreads / 2; w > 0; w >>= 1) {          // fixed tree: the same order on every run
        if ((int)threadIdx.x < w) {
            s_n[threadIdx.x] += s_n[threadIdx.x + w];
            s_t[threadIdx.x] += s_t[threadIdx.x + w];
            s_l[threadIdx.x] += s_l[threadIdx.x + w];
            s_q[threadIdx.x] += s_q[threadIdx.x + w];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) { part_n[blockIdx.x] = s_n[0]; part_t[blockIdx.x] = s_t[0]; part_l[blockIdx.x] = s_l[0]; part_q[blockIdx.x] = s_q[0]; }
}

// adds the partials in workgroup order; fills the result and the select's starting state
__global__ void k_table_finish(const u64* part_n, const u64* part_t, const double* part_l, const double* part_q, int blocks,
                               int coverage_ppm, tasc_table_entropy* res, SelectState* st) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    u64 n = 0, t = 0;
    double l = 0.0, q = 0.0;
    for (int b = 0; b < blocks; ++b) { n += part_n[b]; t += part_t[b]; l += part_l[b]; q += part_q[b]; }
    res->n_entries = (int64_t)n;
    res->total = (int64_t)t;
    if (t == 0) {
        res->shannon = 0.0;
        res->renyi2 = 0.0;
    } else {
        const double lt = log((double)t);
        res->shannon = lt - l / (double)t;              // -sum p ln p = ln T - (sum c ln c) / T
        res->renyi2 = 2.0 * lt - log(q);                // -ln sum p^2 = 2 ln T - ln sum c^2
    }
    // mass to reach: ceil(total * ppm / 1e6), in 128-bit so that nothing overflows
    const unsigned __int128 prod = (unsigned __int128)t * (unsigned __int128)(u32)coverage_ppm + 999999u;
    st->need = (u64)(prod / 1000000u);
    st->above_entries = 0;
    st->above_mass = 0;
    st->prefix = 0;
    st->done = st->need == 0 ? 1u : 0u;
    st->n_cover = 0;
}

// (entries, mass) per value of byte `pass` (3 = most significant) among the counts whose higher bytes equal the prefix
__global__ __launch_bounds__(kStatThreads) void k_select_hist(const unsigned char* base, size_t stride, u64 n, int pass, const SelectState* st,
                                                              u64* hist_entries, u64* hist_mass) {
    if (st->done) return;                                   // uniform over the grid
    __shared__ u64 s_e[256], s_m[256];
    s_e[threadIdx.x] = 0; s_m[threadIdx.x] = 0;
    __syncthreads();
    const u32 prefix = st->prefix;
    const int shift = 8 * pass;
    for (u64 i = (u64)blockIdx.x * kStatThreads + threadIdx.x; i < n; i += (u64)gridDim.x * kStatThreads) {
        const u32 c = entry_count(base, stride, i);
        if (c && (pass == 3 || (c >> (shift + 8)) == prefix)) {
            const u32 b = (c >> shift) & 255u;
            atomicAdd(reinterpret_cast<unsigned long long*>(&s_e[b]), 1ull);
            atomicAdd(reinterpret_cast<unsigned long long*>(&s_m[b]), (unsigned long long)c);
        }
    }
    __syncthreads();
    if (s_e[threadIdx.x]) {
        atomicAdd(reinterpret_cast<unsigned long long*>(&hist_entries[threadIdx.x]), (unsigned long long)s_e[threadIdx.x]);
        atomicAdd(reinterpret_cast<unsigned long long*>(&hist_mass[threadIdx.x]), (unsigned long long)s_m[threadIdx.x]);
    }
}

// walks the byte values downwards until the mass is reached; clears the histogram for the next pass
__global__ void k_select_pick(int pass, SelectState* st, u64* hist_entries, u64* hist_mass, tasc_table_entropy* res) {
    if (blockIdx.x != 0) return;
    if (threadIdx.x == 0 && !st->done) {
        u64 ae = st->above_entries, am = st->above_mass;
        int b = 255;
        for (; b > 0; --b) {
            if (am + hist_mass[b] >= st->need) break;
            ae += hist_entries[b];
            am += hist_mass[b];
        }
        // b: the byte value inside which the threshold count lies (the total reaches `need`, so some bin does)
        st->above_entries = ae;
        st->above_mass = am;
        st->prefix = (st->prefix << 8) | (u32)b;
        if (pass == 0) {
            // every remaining entry has count == prefix: take as many of them as the missing mass needs
            const u64 c = st->prefix;
            const u64 missing = st->need - am;                     // > 0
            st->n_cover = ae + (c ? (missing + c - 1) / c : 0);
            st->done = 1;
        }
    }
    __syncthreads();
    if (pass == 0 && threadIdx.x == 0) res->n_cover = (int64_t)st->n_cover;
    for (int i = threadIdx.x; i < 256; i += blockDim.x) { hist_entries[i] = 0; hist_mass[i] = 0; }
}
}  // namespace

// which table an order names: base address of the first count, stride between counts, number of slots
struct TableSpan {
    const unsigned char* base;
    size_t stride;
    u64 n;
};
static TableSpan table_span(const tasc_ngram* ng, int order) {
    TableSpan t;
    if (order == 1) {
        t.base = reinterpret_cast<const unsigned char*>(ng->unigram);
        t.stride = sizeof(u32);
        t.n = (u64)ng->view.vocab;
    } else {
        const TascSlot* slots = ng->slots[order][1];
        t.base = reinterpret_cast<const unsigned char*>(slots) + offsetof(TascSlot, a);
        t.stride = sizeof(TascSlot);
        t.n = slots ? ng->view.ord[order].full_mask + 1 : 0;
    }
    if (!t.base || (order != 1 && !ng->slots[order][1])) t.n = 0;
    return t;
}
static int stat_blocks(u64 n) {
    int blocks = (int)((n + kStatThreads - 1) / kStatThreads < (u64)kStatBlocksMax ? (n + kStatThreads - 1) / kStatThreads : (u64)kStatBlocksMax);
    return blocks < 1 ? 1 : blocks;
}
// scratch of one call: partial sums, two 256-bin histograms, the select state and the result
static size_t stat_scratch_bytes(int blocks) {
    return (size_t)blocks * (2 * sizeof(u64) + 2 * sizeof(double)) + 2 * 256 * sizeof(u64) + sizeof(SelectState) + sizeof(tasc_table_entropy);
}
#define STAT_SCRATCH_MAX (kStatBlocksMax * 32 + 2 * 256 * 8 + 64 + 64)

__global__ void k_stat_clear(u64* p, int n_words) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n_words; i += gridDim.x * blockDim.x) p[i] = 0;
}
__global__ void k_stat_result(const tasc_table_entropy* res, tasc_table_entropy* out) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *out = *res;
}

// Enqueues the whole computation on `st`; *res_out = where the result will be (inside `scratch`).  `scratch` must hold
// stat_scratch_bytes(blocks) zero bytes when the first kernel runs: cleared here by a fill kernel (a memset node in a
// captured graph is not safe to replay, a kernel is).
static tasc_status enqueue_entropy(const TableSpan& t, int blocks, int coverage_ppm, unsigned char* scratch, hipStream_t st,
                                   tasc_table_entropy** res_out) {
    u64* part_n = reinterpret_cast<u64*>(scratch);
    u64* part_t = part_n + blocks;
    double* part_l = reinterpret_cast<double*>(part_t + blocks);
    double* part_q = part_l + blocks;
    u64* hist_e = reinterpret_cast<u64*>(part_q + blocks);
    u64* hist_m = hist_e + 256;
    SelectState* state = reinterpret_cast<SelectState*>(hist_m + 256);
    tasc_table_entropy* res = reinterpret_cast<tasc_table_entropy*>(state + 1);
    const int words = (int)(stat_scratch_bytes(blocks) / 8);
    k_stat_clear<<<dim3((words + 255) / 256), dim3(256), 0, st>>>(reinterpret_cast<u64*>(scratch), words);
    k_table_moments<<<dim3(blocks), dim3(kStatThreads), 0, st>>>(t.base, t.stride, t.n, part_n, part_t, part_l, part_q);
    k_table_finish<<<dim3(1), dim3(64), 0, st>>>(part_n, part_t, part_l, part_q, blocks, coverage_ppm, res, state);
    for (int pass = 3; pass >= 0; --pass) {
        k_select_hist<<<dim3(blocks), dim3(kStatThreads), 0, st>>>(t.base, t.stride, t.n, pass, state, hist_e, hist_m);
        k_select_pick<<<dim3(1), dim3(256), 0, st>>>(pass, state, hist_e, hist_m, res);
    }
    TASC_LAUNCH_CHECK();
    *res_out = res;
    return TASC_OK;
}

extern "C" tasc_status tasc_ngram_entropy(const tasc_ngram* ng, int32_t order, int32_t coverage_ppm, tasc_table_entropy* out,
                                          void* stream) {
    TASC_REQUIRE(ng && out, "ngram_entropy: null argument");
    TASC_REQUIRE(order >= 1 && order <= ng->view.n_max, "ngram_entropy: order %d outside [1, %d]", order, ng->view.n_max);
    TASC_REQUIRE(coverage_ppm >= 0 && coverage_ppm <= 1000000, "ngram_entropy: coverage_ppm %d outside [0, 1000000]", coverage_ppm);
    hipStream_t st = (hipStream_t)stream;
    const TableSpan t = table_span(ng, order);
    const int blocks = stat_blocks(t.n);
    unsigned char* scratch = nullptr;
    TASC_HIP(hipMalloc(&scratch, stat_scratch_bytes(blocks)));
    tasc_table_entropy* res = nullptr;
    tasc_status rc = enqueue_entropy(t, blocks, coverage_ppm, scratch, st, &res);
    tasc_table_entropy host;
    if (rc == TASC_OK) {
        hipError_t e = hipMemcpyAsync(&host, res, sizeof(host), hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e != hipSuccess) {
            tasc_set_error("ngram_entropy: read back -> %s", hipGetErrorString(e));
            rc = TASC_EHIP;
        }
    }
    hipError_t ef = hipFree(scratch);
    if (rc == TASC_OK && ef != hipSuccess) {
        tasc_set_error("ngram_entropy: free -> %s", hipGetErrorString(ef));
        rc = TASC_EHIP;
    }
    if (rc == TASC_OK) *out = host;
    return rc;
}

// ---------------------------------------------------------------- the same, allocating nothing
// The scratch of tasc_ngram_entropy in a fixed array that every call on a device shares (each device holds its own copy
// of the array at its own address: the address is looked up once per device and kept).
static __device__ __align__(256) unsigned char scratch[STAT_SCRATCH_MAX];
constexpr int kMaxDevices = 64;
static unsigned char* g_scratch_ptr[kMaxDevices];

extern "C" tasc_status tasc_ngram_entropy_noalloc(const tasc_ngram* ng, int32_t order, int32_t coverage_ppm,
                                                  tasc_table_entropy* out_device, void* stream) {
    TASC_REQUIRE(ng && out_device, "ngram_entropy_noalloc: null argument");
    TASC_REQUIRE(order >= 1 && order <= ng->view.n_max, "ngram_entropy_noalloc: order %d outside [1, %d]", order, ng->view.n_max);
    TASC_REQUIRE(coverage_ppm >= 0 && coverage_ppm <= 1000000, "ngram_entropy_noalloc: coverage_ppm %d outside [0, 1000000]",
                 coverage_ppm);
    hipStream_t st = (hipStream_t)stream;
    const TableSpan t = table_span(ng, order);
    if (t.n > (u64)TASC_ENTROPY_NOALLOC_MAX_SLOTS) {
        tasc_set_error("ngram_entropy_noalloc: the table of order %d has %llu slots, the fixed scratch serves at most %llu", order,
                       (unsigned long long)t.n, (unsigned long long)TASC_ENTROPY_NOALLOC_MAX_SLOTS);
        return TASC_ENOMEM;
    }
    const int blocks = stat_blocks(t.n);
    if (stat_scratch_bytes(blocks) > (size_t)STAT_SCRATCH_MAX) {
        tasc_set_error("ngram_entropy_noalloc: %zu bytes of scratch needed, %d available", stat_scratch_bytes(blocks), STAT_SCRATCH_MAX);
        return TASC_ENOMEM;
    }
    int dev = 0;
    TASC_HIP(hipGetDevice(&dev));
    TASC_REQUIRE(dev >= 0 && dev < kMaxDevices, "ngram_entropy_noalloc: device %d outside [0, %d)", dev, kMaxDevices);
    if (!g_scratch_ptr[dev]) {
        unsigned char* p = nullptr;
        TASC_HIP(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
        TASC_REQUIRE(p != nullptr, "ngram_entropy_noalloc: the scratch array has no device address");
        g_scratch_ptr[dev] = p;
    }
    tasc_table_entropy* res = nullptr;
    tasc_status rc = enqueue_entropy(t, blocks, coverage_ppm, g_scratch_ptr[dev], st, &res);
    if (rc != TASC_OK) return rc;
    k_stat_result<<<dim3(1), dim3(64), 0, st>>>(res, out_device);
    TASC_LAUNCH_CHECK();
    return TASC_OK;
}
