// Counting core of the paper's tokenizer enrichment ("Enriching the Tokenizer": merge reward
// f_merge(t^n) = freq(t^n) (n - 1) and the loop of the algorithm "Tokenizer Enrichment"), without the
// prefix-collision filter, which needs token strings: every step counts the n-grams (2 <= n <= n_max) of the corpus
// as currently tokenised with the ordinary table builder (p_min = 1), picks the n-gram with the largest reward
// (ties: shorter, then smallest token tuple), gives it the next free token id and re-tokenises the corpus on the
// device (left to right, without overlap, inside each output).
#include <vector>

#include "tasc_internal.h"

namespace {
constexpr int kThreads = 256;
constexpr int kScanItems = 16;                       // elements per thread of a scan block
constexpr int kScanBlock = kThreads * kScanItems;    // 4096

struct MergeCand {
    u64 reward;      // freq * (n - 1); 0 = none
    u64 lo, hi;      // packed token tuple
    u32 n, freq;
};

// a before b: larger reward, then shorter n-gram, then lexicographically smaller tuple
__device__ inline bool cand_before(const MergeCand& a, const MergeCand& b, int bits) {
    if (a.reward != b.reward) return a.reward > b.reward;
    if (a.reward == 0) return false;
    if (a.n != b.n) return a.n < b.n;
    for (u32 j = 0; j < a.n; ++j) {
        const u32 ta = tasc_key_get(a.lo, a.hi, (int)j, bits), tb = tasc_key_get(b.lo, b.hi, (int)j, bits);
        if (ta != tb) return ta < tb;
    }
    return false;
}

__device__ inline void block_best(MergeCand& mine, int bits, MergeCand* out) {
    __shared__ MergeCand s_c[kThreads];
    s_c[threadIdx.x] = mine;
    __syncthreads();
    for (int w = kThreads / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w && cand_before(s_c[threadIdx.x + w], s_c[threadIdx.x], bits)) s_c[threadIdx.x] = s_c[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = s_c[0];
}

// best candidate of every workgroup over the full table of one order
__global__ __launch_bounds__(kThreads) void k_best_in_table(const TascSlot* __restrict__ slots, u64 cap, int n, int bits, MergeCand* block_out) {
    MergeCand best{0, 0, 0, 0, 0};
    for (u64 i = (u64)blockIdx.x * kThreads + threadIdx.x; i < cap; i += (u64)gridDim.x * kThreads) {
        const TascSlot s = slots[i];
        if (s.a) {
            MergeCand c{(u64)s.a * (u64)(n - 1), s.lo, s.hi, (u32)n, s.a};
            if (cand_before(c, best, bits)) best = c;
        }
    }
    block_best(best, bits, block_out + blockIdx.x);
}
__global__ __launch_bounds__(kThreads) void k_best_final(const MergeCand* __restrict__ cands, int count, int bits, MergeCand* out) {
    MergeCand best{0, 0, 0, 0, 0};
    for (int i = threadIdx.x; i < count; i += kThreads)
        if (cand_before(cands[i], best, bits)) best = cands[i];
    block_best(best, bits, out);
}

__global__ void k_doc_starts(const int64_t* __restrict__ off, int64_t n_docs, unsigned char* start) {
    const int64_t d = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (d < n_docs && off[d] < off[d + 1]) start[off[d]] = 1;
}

struct Gram { int32_t t[TASC_MAX_ORDER]; };

// mark[i] = 1 iff the n-gram starts at i and lies inside one output (no output starts in (i, i + n - 1])
__global__ void k_mark(const int32_t* __restrict__ tok, const unsigned char* __restrict__ start, u64 T, Gram g, int n, unsigned char* mark) {
    const u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= T) return;
    bool ok = i + (u64)n <= T;
    if (ok) {
        for (int j = 0; j < n; ++j) ok = ok && tok[i + j] == g.t[j] && (j == 0 || !start[i + j]);
    }
    mark[i] = ok ? 1 : 0;
}

// Left-to-right choice among overlapping matches.  A match with no match in the n - 1 positions before it ("head")
// is always taken; from it, one thread walks the run of matches that overlap each other, taking the first match at
// or after the end of the last taken one, and stops when that one is a head itself (its own thread takes it) or lies
// beyond the reach of an overlap.  The walk ends at the latest at the end of the corpus.
__global__ void k_select(const unsigned char* __restrict__ mark, u64 T, int n, unsigned char* sel) {
    const u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= T || !mark[i]) return;
    auto is_head = [&](u64 p) {
        for (int j = 1; j < n; ++j)
            if (p >= (u64)j && mark[p - j]) return false;
        return true;
    };
    if (!is_head(i)) return;
    u64 cur = i;
    for (;;) {
        sel[cur] = 1;
        u64 next = T;
        for (u64 p = cur + n; p < cur + 2 * (u64)n - 1 && p < T; ++p)
            if (mark[p]) { next = p; break; }
        if (next >= T || is_head(next)) break;
        cur = next;
    }
}

// keep[i] = 0 for the positions a taken match swallows (all but its first); val[i] = token after the merge
__global__ void k_keep(const int32_t* __restrict__ tok, const unsigned char* __restrict__ sel, u64 T, int n, int32_t new_id, unsigned char* keep,
                       int32_t* val) {
    const u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= T) return;
    bool inside = false;
    for (int j = 1; j < n; ++j) inside = inside || (i >= (u64)j && sel[i - j]);
    keep[i] = inside ? 0 : 1;
    val[i] = sel[i] ? new_id : tok[i];
}

// exclusive scan of keep[] into pos[0..T] in three steps: per-block sums, scan of the sums (one workgroup), apply
__global__ __launch_bounds__(kThreads) void k_scan_sums(const unsigned char* __restrict__ keep, u64 T, u32* bsum) {
    const u64 base = (u64)blockIdx.x * kScanBlock;
    u32 c = 0;
    for (int j = 0; j < kScanItems; ++j) {
        const u64 i = base + (u64)j * kThreads + threadIdx.x;
        if (i < T) c += keep[i];
    }
    __shared__ u32 s[kThreads];
    s[threadIdx.x] = c;
    __syncthreads();
    for (int w = kThreads / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) s[threadIdx.x] += s[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) bsum[blockIdx.x] = s[0];
}
__global__ __launch_bounds__(kThreads) void k_scan_offsets(u32* bsum, u32 n_blocks) {   // in place: exclusive scan, one workgroup
    __shared__ u32 s[kThreads];
    __shared__ u32 carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (u32 b0 = 0; b0 < n_blocks; b0 += kThreads) {
        const u32 i = b0 + threadIdx.x;
        const u32 v = i < n_blocks ? bsum[i] : 0;
        s[threadIdx.x] = v;
        __syncthreads();
        for (int w = 1; w < kThreads; w <<= 1) {             // inclusive scan of the chunk
            const u32 add = (int)threadIdx.x >= w ? s[threadIdx.x - w] : 0;
            __syncthreads();
            s[threadIdx.x] += add;
            __syncthreads();
        }
        if (i < n_blocks) bsum[i] = carry + s[threadIdx.x] - v;
        __syncthreads();
        if (threadIdx.x == 0) carry += s[kThreads - 1];
        __syncthreads();
    }
}
// thread t of a block owns the kScanItems consecutive elements base + t * kScanItems ..
__global__ __launch_bounds__(kThreads) void k_scan_apply(const unsigned char* __restrict__ keep, const int32_t* __restrict__ val, u64 T,
                                                         const u32* __restrict__ boff, u32* pos, int32_t* out) {
    const u64 base = (u64)blockIdx.x * kScanBlock + (u64)threadIdx.x * kScanItems;
    u32 c = 0;
    for (int j = 0; j < kScanItems; ++j)
        if (base + j < T) c += keep[base + j];
    __shared__ u32 s[kThreads];
    s[threadIdx.x] = c;
    __syncthreads();
    for (int w = 1; w < kThreads; w <<= 1) {
        const u32 add = (int)threadIdx.x >= w ? s[threadIdx.x - w] : 0;
        __syncthreads();
        s[threadIdx.x] += add;
        __syncthreads();
    }
    u32 p = boff[blockIdx.x] + s[threadIdx.x] - c;
    for (int j = 0; j < kScanItems; ++j) {
        const u64 i = base + j;
        if (i < T) {
            pos[i] = p;
            if (keep[i]) { out[p] = val[i]; ++p; }
        }
    }
    if (base <= T && T < base + kScanItems) pos[T] = p;         // the thread whose range holds position T (all its kept ones counted)
}
__global__ void k_new_offsets(const int64_t* __restrict__ off, int64_t n_docs, const u32* __restrict__ pos, int64_t* off_out) {
    const int64_t d = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (d <= n_docs) off_out[d] = (int64_t)pos[off[d]];
}

struct Bufs {
    std::vector<void*> p;
    ~Bufs() { for (void* q : p) (void)hipFree(q); }
    template <class T> tasc_status get(T** out, size_t count) {
        void* q = nullptr;
        TASC_HIP(hipMalloc(&q, (count ? count : 1) * sizeof(T)));
        p.push_back(q);
        *out = (T*)q;
        return TASC_OK;
    }
};
}  // namespace

#define TOK_TRY(expr) do { tasc_status _rc = (expr); if (_rc != TASC_OK) return _rc; } while (0)

extern "C" tasc_status tasc_tok_enrich(const int32_t* tokens, const int64_t* doc_offsets, int64_t n_docs, int32_t vocab, int32_t n_max,
                                       int32_t budget, tasc_mem where, void* stream, int32_t* merges, int64_t* merge_freq,
                                       int64_t* corpus_len, int32_t* out_tokens, int64_t* out_offsets, int32_t* n_merges) {
    TASC_REQUIRE(doc_offsets && merges && merge_freq && corpus_len && out_offsets && n_merges, "tok_enrich: null argument");
    TASC_REQUIRE(n_docs >= 0 && vocab >= 1 && budget >= 0, "tok_enrich: n_docs %lld, vocab %d, budget %d", (long long)n_docs, vocab, budget);
    TASC_REQUIRE(n_max >= 2 && n_max <= TASC_MAX_ORDER, "tok_enrich: n_max %d outside [2, %d]", n_max, TASC_MAX_ORDER);
    TASC_REQUIRE(where == TASC_MEM_HOST || where == TASC_MEM_DEVICE, "tok_enrich: bad memory kind");
    TASC_REQUIRE((int64_t)vocab + budget <= 0x7FFFFFFF, "tok_enrich: vocab + budget overflows int32");
    const int32_t vocab_all = vocab + budget;               // one key width for every step
    int bits = 1;
    while ((1ll << bits) < vocab_all) ++bits;
    TASC_REQUIRE(n_max * bits <= 128, "tok_enrich: n_max %d x %d bits per token exceeds the 128-bit key", n_max, bits);
    TASC_REQUIRE(doc_offsets[0] == 0, "tok_enrich: doc_offsets[0] != 0");
    for (int64_t d = 0; d < n_docs; ++d)
        TASC_REQUIRE(doc_offsets[d + 1] >= doc_offsets[d], "tok_enrich: doc_offsets decrease at %lld", (long long)d);
    const u64 T0 = (u64)doc_offsets[n_docs];
    TASC_REQUIRE(T0 < 0xFFFFFFFFull, "tok_enrich: corpus of %llu tokens is too large", (unsigned long long)T0);
    TASC_REQUIRE(T0 == 0 || (tokens && out_tokens), "tok_enrich: null tokens");
    hipStream_t st = (hipStream_t)stream;

    Bufs bufs;
    int32_t *cur, *nxt, *val;
    unsigned char *start, *mark, *sel, *keep;
    u32 *pos, *bsum;
    int64_t *d_off, *d_off2;
    MergeCand *cands, *best;
    const u32 scan_blocks = (u32)((T0 + kScanBlock) / kScanBlock);          // covers positions 0..T
    const int cand_blocks = 512;
    TOK_TRY(bufs.get(&cur, T0)); TOK_TRY(bufs.get(&nxt, T0)); TOK_TRY(bufs.get(&val, T0));
    TOK_TRY(bufs.get(&start, T0 + TASC_MAX_ORDER)); TOK_TRY(bufs.get(&mark, T0)); TOK_TRY(bufs.get(&sel, T0)); TOK_TRY(bufs.get(&keep, T0));
    TOK_TRY(bufs.get(&pos, T0 + 1)); TOK_TRY(bufs.get(&bsum, scan_blocks));
    TOK_TRY(bufs.get(&d_off, (size_t)n_docs + 1)); TOK_TRY(bufs.get(&d_off2, (size_t)n_docs + 1));
    TOK_TRY(bufs.get(&cands, (size_t)cand_blocks * (TASC_MAX_ORDER + 1))); TOK_TRY(bufs.get(&best, 1));
    if (T0) TASC_HIP(hipMemcpyAsync(cur, tokens, T0 * sizeof(int32_t), where == TASC_MEM_HOST ? hipMemcpyHostToDevice : hipMemcpyDeviceToDevice, st));
    std::vector<int64_t> offs(doc_offsets, doc_offsets + n_docs + 1);
    TASC_HIP(hipMemcpyAsync(d_off, offs.data(), (size_t)(n_docs + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));

    // the builder's buffers are kept across the merges (the corpus only shrinks, so they are allocated once)
    struct CacheOwner {
        TascBuildCache c{};
        ~CacheOwner() { tasc_build_cache_free(&c); }
    } build_cache;
    u64 T = T0;
    corpus_len[0] = (int64_t)T;
    int done = 0;
    for (; done < budget; ++done) {
        if (T == 0) break;
        tasc_ngram* ng = nullptr;
        TOK_TRY(tasc_ngram_build_cached(cur, offs.data(), n_docs, vocab_all, n_max, 1, TASC_MEM_DEVICE, stream, &build_cache.c, true, &ng));
        struct Guard { tasc_ngram* p; ~Guard() { tasc_ngram_destroy(p); } } guard{ng};
        int n_cand = 0;
        for (int n = 2; n <= n_max; ++n) {
            const TascSlot* slots = ng->slots[n][1];
            if (!slots) continue;
            k_best_in_table<<<dim3(cand_blocks), dim3(kThreads), 0, st>>>(slots, ng->view.ord[n].full_mask + 1, n, bits, cands + n_cand);
            TASC_LAUNCH_CHECK();
            n_cand += cand_blocks;
        }
        if (n_cand == 0) break;                                  // no n-gram left in the corpus
        k_best_final<<<dim3(1), dim3(kThreads), 0, st>>>(cands, n_cand, bits, best);
        TASC_LAUNCH_CHECK();
        MergeCand h;
        TASC_HIP(hipMemcpyAsync(&h, best, sizeof h, hipMemcpyDeviceToHost, st));
        TASC_HIP(hipStreamSynchronize(st));
        if (h.reward == 0) break;
        Gram g{};
        const int n = (int)h.n;
        int32_t* row = merges + (size_t)done * (1 + TASC_MAX_ORDER);
        row[0] = n;
        for (int j = 0; j < TASC_MAX_ORDER; ++j) {
            g.t[j] = j < n ? (int32_t)tasc_key_get(h.lo, h.hi, j, bits) : 0;
            row[1 + j] = j < n ? g.t[j] : -1;
        }
        merge_freq[done] = (int64_t)h.freq;
        const int32_t new_id = vocab + done;

        // re-tokenise
        const unsigned gridT = (unsigned)((T + kThreads - 1) / kThreads);
        TASC_HIP(hipMemsetAsync(start, 0, T + TASC_MAX_ORDER, st));
        TASC_HIP(hipMemsetAsync(sel, 0, T, st));
        if (n_docs) {
            k_doc_starts<<<dim3((unsigned)((n_docs + kThreads - 1) / kThreads)), dim3(kThreads), 0, st>>>(d_off, n_docs, start);
            TASC_LAUNCH_CHECK();
        }
        k_mark<<<dim3(gridT), dim3(kThreads), 0, st>>>(cur, start, T, g, n, mark);
        TASC_LAUNCH_CHECK();
        k_select<<<dim3(gridT), dim3(kThreads), 0, st>>>(mark, T, n, sel);
        TASC_LAUNCH_CHECK();
        k_keep<<<dim3(gridT), dim3(kThreads), 0, st>>>(cur, sel, T, n, new_id, keep, val);
        TASC_LAUNCH_CHECK();
        const u32 nb = (u32)((T + kScanBlock) / kScanBlock);      // blocks covering positions 0..T
        k_scan_sums<<<dim3(nb), dim3(kThreads), 0, st>>>(keep, T, bsum);
        TASC_LAUNCH_CHECK();
        k_scan_offsets<<<dim3(1), dim3(kThreads), 0, st>>>(bsum, nb);
        TASC_LAUNCH_CHECK();
        k_scan_apply<<<dim3(nb), dim3(kThreads), 0, st>>>(keep, val, T, bsum, pos, nxt);
        TASC_LAUNCH_CHECK();
        k_new_offsets<<<dim3((unsigned)((n_docs + 1 + kThreads - 1) / kThreads)), dim3(kThreads), 0, st>>>(d_off, n_docs, pos, d_off2);
        TASC_LAUNCH_CHECK();
        TASC_HIP(hipMemcpyAsync(offs.data(), d_off2, (size_t)(n_docs + 1) * sizeof(int64_t), hipMemcpyDeviceToHost, st));
        TASC_HIP(hipStreamSynchronize(st));
        std::swap(cur, nxt);
        std::swap(d_off, d_off2);
        T = (u64)offs[n_docs];
        corpus_len[done + 1] = (int64_t)T;
    }
    *n_merges = done;
    if (T) TASC_HIP(hipMemcpyAsync(out_tokens, cur, T * sizeof(int32_t), where == TASC_MEM_HOST ? hipMemcpyDeviceToHost : hipMemcpyDeviceToDevice, st));
    TASC_HIP(hipStreamSynchronize(st));
    for (int64_t d = 0; d <= n_docs; ++d) out_offsets[d] = offs[d];
    return TASC_OK;
}
