// Corpus n-gram tables on the GPU: counting, pruning, per-context aggregates, export.
//
// Paper, section "Proposed Method: TASC-spec": the drafter is a collection of n-gram models M_n,
// n <= n_max, each derived from the n-gram frequencies in the task corpus and pruned of the
// elements whose frequency is below p_min; the most frequent token is the last resort.
//
// Layout and algorithm (all integer, exact keys):
//   * counting table of one order: open addressing over 8-byte slots {first position + 1 : 32,
//     count : 32}.  A slot names its key by the position of its first occurrence in the corpus,
//     which stays resident, so a slot is claimed and counted with single 64-bit atomics and no
//     multi-word publication is needed.  Probing is linear.
//   * after counting, the kept n-grams (count >= p_min) are re-inserted into two small tables
//     that carry explicit 128-bit keys (32-byte slots, see TascSlot): the full table (context +
//     successor -> count) and the context table (context -> T, most frequent successor).
#include "tasc_internal.h"
#include <algorithm>
#include <string.h>

static thread_local char g_err[512] = "";
void tasc_set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}
extern "C" const char* tasc_last_error(void) { return g_err; }

namespace {

constexpr int kThreads = 256;

// Token histogram.  Corpus tokens follow a steep rank-frequency law, so adding every occurrence straight to the
// global histogram serialises on the few hottest counters.  A workgroup therefore first counts a chunk of
// kUniChunk tokens in an LDS table (open addressing, twice as many slots as tokens, so it cannot fill up) and
// then adds each distinct token's count to the global histogram once.
constexpr int kUniChunk = 2048, kUniSlots = 4096;
__global__ __launch_bounds__(kThreads) void k_unigram(const int32_t* __restrict__ tok, u64 T, int vocab, u32* hist, u32* bad) {
    __shared__ u32 s_key[kUniSlots];
    __shared__ u32 s_cnt[kUniSlots];
    for (int i = threadIdx.x; i < kUniSlots; i += kThreads) { s_key[i] = 0xFFFFFFFFu; s_cnt[i] = 0; }
    __syncthreads();
    for (u64 c0 = (u64)blockIdx.x * kUniChunk; c0 < T; c0 += (u64)gridDim.x * kUniChunk) {
        for (int j = threadIdx.x; j < kUniChunk; j += kThreads) {
            const u64 i = c0 + j;
            if (i >= T) break;
            const int t = tok[i];
            if (t < 0 || t >= vocab) { atomicOr(bad, 1u); continue; }
            u32 h = ((u32)t * 2654435761u) >> 20;                      // top 12 bits: kUniSlots = 4096
            for (;;) {
                const u32 old = atomicCAS(&s_key[h], 0xFFFFFFFFu, (u32)t);
                if (old == 0xFFFFFFFFu || old == (u32)t) { atomicAdd(&s_cnt[h], 1u); break; }
                h = (h + 1) & (kUniSlots - 1);
            }
        }
        __syncthreads();
        for (int i = threadIdx.x; i < kUniSlots; i += kThreads) {
            const u32 k = s_key[i];
            if (k != 0xFFFFFFFFu) {
                atomicAdd(&hist[k], s_cnt[i]);
                s_key[i] = 0xFFFFFFFFu;
                s_cnt[i] = 0;
            }
        }
        __syncthreads();
    }
}

// best[0] = max over tokens of (count << 32) | (0xFFFFFFFF - token): largest count, smallest id
__global__ void k_unigram_argmax(const u32* hist, int vocab, u64* best) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    u64 v = 0;
    for (; i < vocab; i += gridDim.x * blockDim.x) {
        u64 c = ((u64)hist[i] << 32) | (u64)(0xFFFFFFFFu - (u32)i);
        v = c > v ? c : v;
    }
    for (int o = 32; o > 0; o >>= 1) {
        u64 w = __shfl_xor(v, o);
        v = w > v ? w : v;
    }
    if ((threadIdx.x & 63) == 0) atomicMax(best, v);
}

// rem[i] = tokens left in the document from position i on, saturated at 255
__global__ void k_mark_doc_tails(const int64_t* doc_off, int64_t n_docs, int n_max, uint8_t* rem) {
    int64_t d = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (d >= n_docs) return;
    int64_t b = doc_off[d], e = doc_off[d + 1];
    for (int j = 1; j < n_max && e - j >= b; ++j) rem[e - j] = (uint8_t)j;
}

template <int N>
__device__ inline bool same_window(const int32_t* __restrict__ tok, u64 p, const int32_t* w) {
    bool eq = true;
#pragma unroll
    for (int j = 0; j < N; ++j) eq = eq && (tok[p + j] == w[j]);
    return eq;
}

// Counting in two levels.  A workgroup takes chunks of kChunk consecutive corpus positions (coalesced scan,
// the chunk's tokens staged in LDS), counts the chunk's windows in an LDS hash table whose slots name their
// key by a position inside the chunk, and then adds every distinct window of the chunk to the global table
// once, with its chunk count.  Task corpora concentrate on few n-grams (the paper's typical-set argument), so
// the frequent ones would otherwise serialise hundreds of thousands of atomics on one address.
constexpr int kChunk = 2048;
constexpr int kLdsSlots = 4096;

template <int N>
__global__ __launch_bounds__(kThreads) void k_count(const int32_t* __restrict__ tok, const uint8_t* __restrict__ rem, u64 T,
                                                    int bits, u64* slots, u64 mask) {
    __shared__ int32_t s_tok[kChunk + TASC_MAX_ORDER];
    __shared__ u64 s_slot[kLdsSlots];
    const int tid = threadIdx.x;
    for (u64 base = (u64)blockIdx.x * kChunk; base < T; base += (u64)gridDim.x * kChunk) {
        const int n_here = (int)min((u64)(kChunk + N - 1), T - base);
        for (int i = tid; i < n_here; i += kThreads) s_tok[i] = tok[base + i];
        for (int i = tid; i < kLdsSlots; i += kThreads) s_slot[i] = 0;
        __syncthreads();
        const int n_win = (int)min((u64)kChunk, T - base);
        for (int i = tid; i < n_win; i += kThreads) {
            if (rem[base + i] < N) continue;           // the window would leave its document
            u64 lo = 0, hi = 0;
#pragma unroll
            for (int j = 0; j < N; ++j) tasc_key_put(lo, hi, j, bits, (u32)s_tok[i + j]);
            u32 idx = (u32)(tasc_hash_key(lo, hi, N) >> 20) & (kLdsSlots - 1);
            for (int probe = 0; probe < kLdsSlots; ++probe) {
                u64 sl = s_slot[idx];
                if (sl == 0) {
                    const u64 old = atomicCAS(&s_slot[idx], 0ull, ((u64)(i + 1) << 32) | 1ull);
                    if (old == 0) break;
                    sl = old;
                }
                const int p = (int)(sl >> 32) - 1;
                bool eq = true;
#pragma unroll
                for (int j = 0; j < N; ++j) eq = eq && (s_tok[p + j] == s_tok[i + j]);
                if (eq) {
                    atomicAdd(&s_slot[idx], 1ull);
                    break;
                }
                idx = (idx + 1) & (kLdsSlots - 1);
            }
        }
        __syncthreads();
        for (int sidx = tid; sidx < kLdsSlots; sidx += kThreads) {
            const u64 sl = s_slot[sidx];
            if (sl == 0) continue;
            const int p = (int)(sl >> 32) - 1;
            const u64 cnt = sl & 0xFFFFFFFFull;
            int32_t w[N];
            u64 lo = 0, hi = 0;
#pragma unroll
            for (int j = 0; j < N; ++j) {
                w[j] = s_tok[p + j];
                tasc_key_put(lo, hi, j, bits, (u32)w[j]);
            }
            u64 idx = tasc_hash_key(lo, hi, N) & mask;
            for (u64 probe = 0; probe <= mask; ++probe) {
                u64 g = __hip_atomic_load(&slots[idx], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (g == 0) {
                    const u64 old = atomicCAS(&slots[idx], 0ull, ((base + p + 1) << 32) | cnt);
                    if (old == 0) break;
                    g = old;
                }
                if (same_window<N>(tok, (g >> 32) - 1, w)) {
                    atomicAdd(&slots[idx], cnt);
                    break;
                }
                idx = (idx + 1) & mask;
            }
        }
        __syncthreads();
    }
}

// counters[0] = distinct n-grams, counters[1] = kept n-grams
__global__ __launch_bounds__(kThreads) void k_tally(const u64* slots, u64 cap, u32 p_min, u64* counters) {
    __shared__ u32 s_d[kThreads / 64], s_k[kThreads / 64];
    u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    const u64 stride = (u64)gridDim.x * blockDim.x;
    u32 distinct = 0, kept = 0;
    for (; i < cap; i += stride) {
        const u64 s = slots[i];
        distinct += s != 0;
        kept += (s != 0) && ((u32)s >= p_min);
    }
    for (int o = 32; o > 0; o >>= 1) {
        distinct += __shfl_xor(distinct, o);
        kept += __shfl_xor(kept, o);
    }
    if ((threadIdx.x & 63) == 0) { s_d[threadIdx.x >> 6] = distinct; s_k[threadIdx.x >> 6] = kept; }
    __syncthreads();
    if (threadIdx.x == 0) {      // one pair of atomics per workgroup, not per wave
        u64 d = 0, k = 0;
        for (int w = 0; w < kThreads / 64; ++w) { d += s_d[w]; k += s_k[w]; }
        if (d) atomicAdd(&counters[0], d);
        if (k) atomicAdd(&counters[1], k);
    }
}

struct CtxRef {   // context table under construction: key named by a corpus position
    u32 pos1;     // position + 1 of the context's first token, 0 = empty
    u32 total;    // T: sum of kept successor counts
    u64 best;     // max of (count << 32) | (0xFFFFFFFF - successor)
};

template <int N>
__global__ __launch_bounds__(kThreads) void k_keep(const int32_t* __restrict__ tok, const u64* __restrict__ slots,
                                                   u64 cap, u32 p_min, int bits, TascSlot* full, u64 full_mask,
                                                   CtxRef* ctx, u64 ctx_mask) {
    u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= cap) return;
    u64 s = slots[i];
    u32 cnt = (u32)s;
    if (s == 0 || cnt < p_min) return;
    u64 p = (s >> 32) - 1;
    int32_t w[N];
    u64 lo = 0, hi = 0, clo = 0, chi = 0;
#pragma unroll
    for (int j = 0; j < N; ++j) {
        w[j] = tok[p + j];
        tasc_key_put(lo, hi, j, bits, (u32)w[j]);
        if (j < N - 1) tasc_key_put(clo, chi, j, bits, (u32)w[j]);
    }
    // full table: keys are distinct, so claiming a slot (count 0 -> cnt) is all the synchronisation needed
    u64 idx = tasc_hash_key(lo, hi, N) & full_mask;
    for (u64 probe = 0; probe <= full_mask; ++probe) {
        if (atomicCAS(&full[idx].a, 0u, cnt) == 0u) {
            full[idx].lo = lo;
            full[idx].hi = hi;
            break;
        }
        idx = (idx + 1) & full_mask;
    }
    // context table: many kept n-grams share a context
    idx = tasc_hash_key(clo, chi, N - 1) & ctx_mask;
    for (u64 probe = 0; probe <= ctx_mask; ++probe) {
        u32 q = __hip_atomic_load(&ctx[idx].pos1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bool mine = false;
        if (q == 0) {
            u32 old = atomicCAS(&ctx[idx].pos1, 0u, (u32)(p + 1));
            mine = old == 0;
            q = old;
        }
        if (mine || same_window<N - 1>(tok, (u64)q - 1, w)) {
            atomicAdd(&ctx[idx].total, cnt);
            atomicMax(&ctx[idx].best, ((u64)cnt << 32) | (u64)(0xFFFFFFFFu - (u32)w[N - 1]));
            break;
        }
        idx = (idx + 1) & ctx_mask;
    }
}

// gives every context slot its explicit key; same index, so the probe sequences stay valid
__global__ void k_materialize_ctx(const int32_t* __restrict__ tok, const CtxRef* ref, u64 cap, int n_ctx_tok,
                                  int bits, TascSlot* out, u64* n_contexts) {
    u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= cap) return;
    CtxRef r = ref[i];
    TascSlot s = {0, 0, 0, 0, 0, 0};
    if (r.pos1 != 0) {
        for (int j = 0; j < n_ctx_tok; ++j) tasc_key_put(s.lo, s.hi, j, bits, (u32)tok[(u64)r.pos1 - 1 + j]);
        s.a = r.total;
        s.b = 0xFFFFFFFFu - (u32)r.best;
        s.c = (u32)(r.best >> 32);
        atomicAdd(n_contexts, 1ull);
    }
    out[i] = s;
}

u64 pow2_at_least(u64 v) {
    u64 c = 1;
    while (c < v) c <<= 1;
    return c;
}

template <int N>
void launch_count(const int32_t* tok, const uint8_t* rem, u64 T, int bits, u64* slots, u64 mask, hipStream_t st) {
    const u64 chunks = (T + kChunk - 1) / kChunk;
    k_count<N><<<dim3((unsigned)std::min<u64>(chunks, 1u << 20)), dim3(kThreads), 0, st>>>(tok, rem, T, bits, slots, mask);
}
template <int N>
void launch_keep(const int32_t* tok, const u64* slots, u64 cap, u32 p_min, int bits, TascSlot* full, u64 fm,
                 CtxRef* ctx, u64 cm, hipStream_t st) {
    k_keep<N><<<dim3((unsigned)((cap + kThreads - 1) / kThreads)), dim3(kThreads), 0, st>>>(tok, slots, cap, p_min, bits, full,
                                                                                         fm, ctx, cm);
}

struct Cleanup {   // frees temporaries on every exit path
    std::vector<void*> ptrs;
    std::vector<hipEvent_t> evs;
    ~Cleanup() {
        for (void* p : ptrs) (void)hipFree(p);
        for (hipEvent_t e : evs) (void)hipEventDestroy(e);
    }
};

}  // namespace

void tasc_build_cache_free(TascBuildCache* c) {
    for (int i = 0; i < TASC_BUILD_CACHE_SLOTS; ++i) {
        if (c->p[i]) (void)hipFree(c->p[i]);
        c->p[i] = nullptr;
        c->cap[i] = 0;
    }
}

extern "C" tasc_status tasc_ngram_build(const int32_t* tokens, const int64_t* doc_offsets, int64_t n_docs,
                                        int32_t vocab, int32_t n_max, int32_t p_min, tasc_mem where, void* stream,
                                        tasc_ngram** out) {
    return tasc_ngram_build_cached(tokens, doc_offsets, n_docs, vocab, n_max, p_min, where, stream, nullptr, false, out);
}

tasc_status tasc_ngram_build_cached(const int32_t* tokens, const int64_t* doc_offsets, int64_t n_docs, int32_t vocab, int32_t n_max,
                                    int32_t p_min, tasc_mem where, void* stream, TascBuildCache* cache, bool counts_only,
                                    tasc_ngram** out) {
    TASC_REQUIRE(out != nullptr && doc_offsets != nullptr, "ngram_build: null argument");
    TASC_REQUIRE(n_docs >= 0 && vocab >= 1, "ngram_build: n_docs %lld, vocab %d", (long long)n_docs, vocab);
    TASC_REQUIRE(n_max >= 2 && n_max <= TASC_MAX_ORDER, "ngram_build: n_max %d outside [2, %d]", n_max, TASC_MAX_ORDER);
    TASC_REQUIRE(p_min >= 1, "ngram_build: p_min %d < 1", p_min);
    TASC_REQUIRE(where == TASC_MEM_HOST || where == TASC_MEM_DEVICE, "ngram_build: bad memory kind");
    int bits = 1;
    while ((1ll << bits) < vocab) ++bits;
    TASC_REQUIRE(n_max * bits <= 128, "ngram_build: n_max %d x %d bits per token exceeds the 128-bit key", n_max, bits);
    TASC_REQUIRE(doc_offsets[0] == 0, "ngram_build: doc_offsets[0] != 0");
    for (int64_t d = 0; d < n_docs; ++d)
        TASC_REQUIRE(doc_offsets[d + 1] >= doc_offsets[d], "ngram_build: doc_offsets decrease at %lld", (long long)d);
    const u64 T = (u64)doc_offsets[n_docs];
    TASC_REQUIRE(T < 0xFFFFFFFFull, "ngram_build: corpus of %llu tokens is too large", T);
    TASC_REQUIRE(T == 0 || tokens != nullptr, "ngram_build: null tokens");
    hipStream_t st = (hipStream_t)stream;

    Cleanup tmp;
    tasc_ngram* ng = new tasc_ngram();
    memset(&ng->view, 0, sizeof ng->view);
    memset(ng->slots, 0, sizeof ng->slots);
    memset(&ng->stats, 0, sizeof ng->stats);
    ng->unigram = nullptr;
    ng->borrowed = cache != nullptr;
    ng->p_min = p_min;
    ng->view.n_max = n_max;
    ng->view.bits = bits;
    ng->view.vocab = vocab;
    ng->view.fallback = 0;
    ng->stats.n_tokens = (int64_t)T;
    struct Guard {   // destroys the half-built handle unless released
        tasc_ngram* p;
        ~Guard() { if (p) tasc_ngram_destroy(p); }
    } guard{ng};

    // device buffer for call site `site`: from the cache (grown when too small), else a fresh allocation that is
    // either temporary (freed on return) or handed to the handle
    auto get_buf = [&](int site, void** p, size_t bytes, bool temporary) -> tasc_status {
        bytes = bytes ? bytes : 1;
        if (cache) {
            if (cache->cap[site] < bytes) {
                if (cache->p[site]) TASC_HIP(hipFree(cache->p[site]));
                cache->p[site] = nullptr;
                cache->cap[site] = 0;
                const size_t want = bytes + bytes / 8;
                TASC_HIP(hipMalloc(&cache->p[site], want));
                cache->cap[site] = want;
            }
            *p = cache->p[site];
            return TASC_OK;
        }
        TASC_HIP(hipMalloc(p, bytes));
        if (temporary) tmp.ptrs.push_back(*p);
        return TASC_OK;
    };
#define TASC_GET(site, p, bytes, temporary) do { tasc_status _rc = get_buf(site, (void**)(p), bytes, temporary); if (_rc != TASC_OK) return _rc; } while (0)
    hipEvent_t ev0, ev1, evc0, evc1;
    TASC_HIP(hipEventCreate(&ev0)); tmp.evs.push_back(ev0);
    TASC_HIP(hipEventCreate(&ev1)); tmp.evs.push_back(ev1);
    TASC_HIP(hipEventCreate(&evc0)); tmp.evs.push_back(evc0);
    TASC_HIP(hipEventCreate(&evc1)); tmp.evs.push_back(evc1);

    const int32_t* d_tok = tokens;
    if (where == TASC_MEM_HOST && T > 0) {
        void* p;
        TASC_GET(0, &p, T * sizeof(int32_t), true);
        TASC_HIP(hipMemcpyAsync(p, tokens, T * sizeof(int32_t), hipMemcpyHostToDevice, st));
        d_tok = (const int32_t*)p;
    }
    TASC_HIP(hipEventRecord(ev0, st));
    TASC_GET(1, &ng->unigram, (size_t)vocab * sizeof(u32), false);
    TASC_HIP(hipMemsetAsync(ng->unigram, 0, (size_t)vocab * sizeof(u32), st));
    u64* d_counters;   // [0] distinct [1] kept [2] contexts [3] unigram best [4] bad-token flag
    TASC_GET(2, &d_counters, 8 * sizeof(u64), true);
    TASC_HIP(hipMemsetAsync(d_counters, 0, 8 * sizeof(u64), st));
    u64 h_counters[8];

    if (T > 0) {
        unsigned grid = (unsigned)std::min<u64>((T + kUniChunk - 1) / kUniChunk, 2048);
        k_unigram<<<dim3(grid), dim3(kThreads), 0, st>>>(d_tok, T, vocab, ng->unigram, (u32*)&d_counters[4]);
        TASC_LAUNCH_CHECK();
        k_unigram_argmax<<<dim3(64), dim3(kThreads), 0, st>>>(ng->unigram, vocab, &d_counters[3]);
        TASC_LAUNCH_CHECK();
        TASC_HIP(hipMemcpyAsync(h_counters, d_counters, sizeof h_counters, hipMemcpyDeviceToHost, st));
        TASC_HIP(hipStreamSynchronize(st));
        TASC_REQUIRE(h_counters[4] == 0, "ngram_build: corpus holds a token outside [0, %d)", vocab);
        ng->view.fallback = (int32_t)(0xFFFFFFFFu - (u32)h_counters[3]);
    }

    // windows per order, from the document lengths
    u64 windows[TASC_MAX_ORDER + 1] = {0};
    for (int64_t d = 0; d < n_docs; ++d) {
        int64_t len = doc_offsets[d + 1] - doc_offsets[d];
        for (int n = 2; n <= n_max; ++n)
            if (len >= n) windows[n] += (u64)(len - n + 1);
    }
    uint8_t* d_rem = nullptr;
    int64_t* d_off = nullptr;
    u64* d_slots = nullptr;
    u64 slots_cap = 0;
    if (windows[2] > 0) {
        TASC_GET(3, &d_rem, T, true);
        TASC_GET(4, &d_off, (size_t)(n_docs + 1) * sizeof(int64_t), true);
        TASC_HIP(hipMemcpyAsync(d_off, doc_offsets, (size_t)(n_docs + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
        TASC_HIP(hipMemsetAsync(d_rem, 0xFF, T, st));
        k_mark_doc_tails<<<dim3((unsigned)((n_docs + kThreads - 1) / kThreads)), dim3(kThreads), 0, st>>>(d_off, n_docs, n_max, d_rem);
        TASC_LAUNCH_CHECK();
        slots_cap = pow2_at_least(std::max<u64>(1024, windows[2] + windows[2] / 2));
        TASC_GET(5, &d_slots, slots_cap * sizeof(u64), true);
    }

    float count_ms = 0.f;
    for (int n = 2; n <= n_max; ++n) {
        ng->stats.windows[n] = (int64_t)windows[n];
        if (windows[n] == 0) continue;
        const u64 cap = pow2_at_least(std::max<u64>(1024, windows[n] + windows[n] / 2));   // <= slots_cap
        TASC_HIP(hipMemsetAsync(d_slots, 0, cap * sizeof(u64), st));
        TASC_HIP(hipMemsetAsync(d_counters, 0, 3 * sizeof(u64), st));
        TASC_HIP(hipEventRecord(evc0, st));
        switch (n) {
            case 2: launch_count<2>(d_tok, d_rem, T, bits, d_slots, cap - 1, st); break;
            case 3: launch_count<3>(d_tok, d_rem, T, bits, d_slots, cap - 1, st); break;
            case 4: launch_count<4>(d_tok, d_rem, T, bits, d_slots, cap - 1, st); break;
            case 5: launch_count<5>(d_tok, d_rem, T, bits, d_slots, cap - 1, st); break;
            case 6: launch_count<6>(d_tok, d_rem, T, bits, d_slots, cap - 1, st); break;
            case 7: launch_count<7>(d_tok, d_rem, T, bits, d_slots, cap - 1, st); break;
            default: launch_count<8>(d_tok, d_rem, T, bits, d_slots, cap - 1, st); break;
        }
        TASC_LAUNCH_CHECK();
        TASC_HIP(hipEventRecord(evc1, st));
        k_tally<<<dim3((unsigned)std::min<u64>((cap + kThreads - 1) / kThreads, 2048)), dim3(kThreads), 0, st>>>(
            d_slots, cap, (u32)p_min, d_counters);
        TASC_LAUNCH_CHECK();
        TASC_HIP(hipMemcpyAsync(h_counters, d_counters, 3 * sizeof(u64), hipMemcpyDeviceToHost, st));
        TASC_HIP(hipStreamSynchronize(st));
        float ms = 0.f;
        TASC_HIP(hipEventElapsedTime(&ms, evc0, evc1));
        count_ms += ms;
        ng->stats.distinct[n] = (int64_t)h_counters[0];
        ng->stats.kept[n] = (int64_t)h_counters[1];
        const u64 kept = h_counters[1];
        if (kept == 0) continue;
        const u64 fcap = pow2_at_least(std::max<u64>(64, 2 * kept));
        TascSlot *full, *ctx = nullptr;
        CtxRef* ref;
        TASC_GET(8 + 3 * n, &full, fcap * sizeof(TascSlot), false);
        ng->slots[n][1] = full;
        if (!counts_only) {
            TASC_GET(8 + 3 * n + 1, &ctx, fcap * sizeof(TascSlot), false);
            ng->slots[n][0] = ctx;
        }
        TASC_GET(8 + 3 * n + 2, &ref, fcap * sizeof(CtxRef), true);
        TASC_HIP(hipMemsetAsync(full, 0, fcap * sizeof(TascSlot), st));
        TASC_HIP(hipMemsetAsync(ref, 0, fcap * sizeof(CtxRef), st));
        switch (n) {
            case 2: launch_keep<2>(d_tok, d_slots, cap, (u32)p_min, bits, full, fcap - 1, ref, fcap - 1, st); break;
            case 3: launch_keep<3>(d_tok, d_slots, cap, (u32)p_min, bits, full, fcap - 1, ref, fcap - 1, st); break;
            case 4: launch_keep<4>(d_tok, d_slots, cap, (u32)p_min, bits, full, fcap - 1, ref, fcap - 1, st); break;
            case 5: launch_keep<5>(d_tok, d_slots, cap, (u32)p_min, bits, full, fcap - 1, ref, fcap - 1, st); break;
            case 6: launch_keep<6>(d_tok, d_slots, cap, (u32)p_min, bits, full, fcap - 1, ref, fcap - 1, st); break;
            case 7: launch_keep<7>(d_tok, d_slots, cap, (u32)p_min, bits, full, fcap - 1, ref, fcap - 1, st); break;
            default: launch_keep<8>(d_tok, d_slots, cap, (u32)p_min, bits, full, fcap - 1, ref, fcap - 1, st); break;
        }
        TASC_LAUNCH_CHECK();
        if (!counts_only) {
            k_materialize_ctx<<<dim3((unsigned)((fcap + kThreads - 1) / kThreads)), dim3(kThreads), 0, st>>>(
                d_tok, ref, fcap, n - 1, bits, ctx, &d_counters[2]);
            TASC_LAUNCH_CHECK();
        }
        TASC_HIP(hipMemcpyAsync(h_counters, d_counters, 3 * sizeof(u64), hipMemcpyDeviceToHost, st));
        TASC_HIP(hipStreamSynchronize(st));
        ng->stats.contexts[n] = (int64_t)h_counters[2];
        ng->view.ord[n].ctx = ctx;
        ng->view.ord[n].full = full;
        ng->view.ord[n].ctx_mask = ctx ? fcap - 1 : 0;
        ng->view.ord[n].full_mask = fcap - 1;
    }
    TASC_HIP(hipEventRecord(ev1, st));
    TASC_HIP(hipStreamSynchronize(st));
    float ms = 0.f;
    TASC_HIP(hipEventElapsedTime(&ms, ev0, ev1));
    ng->stats.build_ms = ms;
    ng->stats.count_ms = count_ms;
    guard.p = nullptr;
    *out = ng;
    return TASC_OK;
}

extern "C" void tasc_ngram_destroy(tasc_ngram* ng) {
    if (!ng) return;
    if (ng->borrowed) {
        delete ng;
        return;
    }
    for (int n = 0; n <= TASC_MAX_ORDER; ++n)
        for (int j = 0; j < 2; ++j)
            if (ng->slots[n][j]) (void)hipFree(ng->slots[n][j]);
    if (ng->unigram) (void)hipFree(ng->unigram);
    delete ng;
}

namespace {
// downloads the occupied slots of one table, sorted by their token strings
tasc_status fetch_sorted(const tasc_ngram* ng, int order, int which, int ntok, std::vector<TascSlot>& rows) {
    rows.clear();
    const TascSlot* d = ng->slots[order][which];
    if (!d) return TASC_OK;
    u64 cap = (which == 0 ? ng->view.ord[order].ctx_mask : ng->view.ord[order].full_mask) + 1;
    std::vector<TascSlot> all(cap);
    TASC_HIP(hipMemcpy(all.data(), d, cap * sizeof(TascSlot), hipMemcpyDeviceToHost));
    for (const TascSlot& s : all)
        if (s.a != 0) rows.push_back(s);
    const int bits = ng->view.bits;
    std::sort(rows.begin(), rows.end(), [=](const TascSlot& x, const TascSlot& y) {
        for (int j = 0; j < ntok; ++j) {
            u32 a = tasc_key_get(x.lo, x.hi, j, bits), b = tasc_key_get(y.lo, y.hi, j, bits);
            if (a != b) return a < b;
        }
        return false;
    });
    return TASC_OK;
}
}  // namespace

extern "C" tasc_status tasc_ngram_export(const tasc_ngram* ng, int32_t order, int32_t* ctx_next, uint32_t* counts,
                                         int64_t* n_inout) {
    TASC_REQUIRE(ng && n_inout, "ngram_export: null argument");
    TASC_REQUIRE(order >= 2 && order <= ng->view.n_max, "ngram_export: order %d outside [2, %d]", order, ng->view.n_max);
    const int64_t kept = ng->stats.kept[order];
    const int64_t cap = *n_inout;
    *n_inout = kept;
    if (!ctx_next && !counts) return TASC_OK;
    TASC_REQUIRE(ctx_next && counts, "ngram_export: one output array is null");
    if (cap < kept) {
        tasc_set_error("ngram_export: room for %lld rows, %lld needed", (long long)cap, (long long)kept);
        return TASC_ENOMEM;
    }
    std::vector<TascSlot> rows;
    tasc_status rc = fetch_sorted(ng, order, 1, order, rows);
    if (rc != TASC_OK) return rc;
    if ((int64_t)rows.size() != kept) {
        tasc_set_error("ngram_export: table holds %zu rows, expected %lld", rows.size(), (long long)kept);
        return TASC_ESTATE;
    }
    for (size_t i = 0; i < rows.size(); ++i) {
        for (int j = 0; j < order; ++j)
            ctx_next[i * order + j] = (int32_t)tasc_key_get(rows[i].lo, rows[i].hi, j, ng->view.bits);
        counts[i] = rows[i].a;
    }
    return TASC_OK;
}

extern "C" tasc_status tasc_ngram_export_contexts(const tasc_ngram* ng, int32_t order, int32_t* ctx, uint32_t* total,
                                                  int32_t* top, uint32_t* top_count, int64_t* n_inout) {
    TASC_REQUIRE(ng && n_inout, "ngram_export_contexts: null argument");
    TASC_REQUIRE(order >= 2 && order <= ng->view.n_max, "ngram_export_contexts: order %d outside [2, %d]", order,
                 ng->view.n_max);
    const int64_t n = ng->stats.contexts[order];
    const int64_t cap = *n_inout;
    *n_inout = n;
    if (!ctx && !total && !top && !top_count) return TASC_OK;
    TASC_REQUIRE(ctx && total && top && top_count, "ngram_export_contexts: one output array is null");
    if (cap < n) {
        tasc_set_error("ngram_export_contexts: room for %lld rows, %lld needed", (long long)cap, (long long)n);
        return TASC_ENOMEM;
    }
    std::vector<TascSlot> rows;
    tasc_status rc = fetch_sorted(ng, order, 0, order - 1, rows);
    if (rc != TASC_OK) return rc;
    if ((int64_t)rows.size() != n) {
        tasc_set_error("ngram_export_contexts: table holds %zu rows, expected %lld", rows.size(), (long long)n);
        return TASC_ESTATE;
    }
    for (size_t i = 0; i < rows.size(); ++i) {
        for (int j = 0; j < order - 1; ++j)
            ctx[i * (order - 1) + j] = (int32_t)tasc_key_get(rows[i].lo, rows[i].hi, j, ng->view.bits);
        total[i] = rows[i].a;
        top[i] = (int32_t)rows[i].b;
        top_count[i] = rows[i].c;
    }
    return TASC_OK;
}

extern "C" tasc_status tasc_ngram_unigram(const tasc_ngram* ng, int32_t* fallback, uint32_t* counts) {
    TASC_REQUIRE(ng, "ngram_unigram: null handle");
    if (counts) TASC_HIP(hipMemcpy(counts, ng->unigram, (size_t)ng->view.vocab * sizeof(u32), hipMemcpyDeviceToHost));
    if (fallback) *fallback = ng->view.fallback;
    return TASC_OK;
}

extern "C" tasc_status tasc_ngram_get_stats(const tasc_ngram* ng, tasc_ngram_stats* out) {
    TASC_REQUIRE(ng && out, "ngram_get_stats: null argument");
    *out = ng->stats;
    return TASC_OK;
}
