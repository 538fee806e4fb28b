// Internal definitions shared by the translation units of libtasc (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>
#include <vector>
#include "../../include/tasc.h"

typedef unsigned long long u64;
typedef uint32_t u32;

void tasc_set_error(const char* fmt, ...);

#define TASC_HIP(expr)                                                                    \
    do {                                                                                  \
        hipError_t _e = (expr);                                                           \
        if (_e != hipSuccess) {                                                           \
            tasc_set_error("%s:%d: %s -> %s", __FILE__, __LINE__, #expr, hipGetErrorString(_e)); \
            return TASC_EHIP;                                                             \
        }                                                                                 \
    } while (0)

#define TASC_REQUIRE(cond, ...)            \
    do {                                   \
        if (!(cond)) {                     \
            tasc_set_error(__VA_ARGS__);   \
            return TASC_EINVAL;            \
        }                                  \
    } while (0)

#define TASC_LAUNCH_CHECK()                                                          \
    do {                                                                             \
        hipError_t _e = hipGetLastError();                                           \
        if (_e != hipSuccess) {                                                      \
            tasc_set_error("%s:%d: launch -> %s", __FILE__, __LINE__, hipGetErrorString(_e)); \
            return TASC_EHIP;                                                        \
        }                                                                            \
    } while (0)

// ---------------------------------------------------------------- n-gram tables
// One 32-byte slot of a finished (read-only) table.  The key is the packed token string
// (token j at bit j*bits of the 128-bit integer hi:lo).  Context tables: a = T (sum of kept
// successor counts), b = most frequent kept successor, c = its count.  Full tables: a = count.
// a == 0 marks an empty slot.
struct __attribute__((aligned(32))) TascSlot {
    u64 lo, hi;
    u32 a, b, c, d;
};

struct TascOrderTab {
    const TascSlot* ctx;
    const TascSlot* full;
    u64 ctx_mask;   // capacity - 1 (capacity is a power of two); 0 and ctx == nullptr if the order is empty
    u64 full_mask;
};

struct TascNgramView {
    TascOrderTab ord[TASC_MAX_ORDER + 1];   // indexed by n
    int32_t n_max, bits, fallback, vocab;
};

struct tasc_ngram {
    TascNgramView view;
    TascSlot* slots[TASC_MAX_ORDER + 1][2];
    u32* unigram;   // device [vocab]
    int32_t p_min;
    tasc_ngram_stats stats;
    bool borrowed;  // the device buffers belong to a TascBuildCache: tasc_ngram_destroy frees the handle only
};

// Device buffers of a table build kept across builds (repeated builds over a shrinking corpus: every call site
// of the builder has a slot, a buffer is re-allocated only when it is too small).  The owner frees them with
// tasc_build_cache_free once no handle built from them is in use.
#define TASC_BUILD_CACHE_SLOTS (8 + 3 * (TASC_MAX_ORDER + 1))
struct TascBuildCache {
    void* p[TASC_BUILD_CACHE_SLOTS];
    size_t cap[TASC_BUILD_CACHE_SLOTS];
};
void tasc_build_cache_free(TascBuildCache* c);
// tasc_ngram_build with the buffers taken from `cache` (nullptr: allocate and free as usual) and, with
// `counts_only`, without the per-context tables (the n-gram counts of slots[n][1] only)
tasc_status tasc_ngram_build_cached(const int32_t* tokens, const int64_t* doc_offsets, int64_t n_docs, int32_t vocab, int32_t n_max,
                                    int32_t p_min, tasc_mem where, void* stream, TascBuildCache* cache, bool counts_only,
                                    tasc_ngram** out);

__host__ __device__ inline u64 tasc_mix64(u64 x) {
    x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27; x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}
__host__ __device__ inline u64 tasc_hash_key(u64 lo, u64 hi, int ntok) {
    return tasc_mix64(lo ^ tasc_mix64(hi + 0x9E3779B97F4A7C15ull * (u64)(ntok + 1)));
}
// appends token t as element j of a packed key
__host__ __device__ inline void tasc_key_put(u64& lo, u64& hi, int j, int bits, u32 t) {
    int sh = j * bits;
    if (sh < 64) {
        lo |= (u64)t << sh;
        if (sh + bits > 64) hi |= (u64)t >> (64 - sh);
    } else {
        hi |= (u64)t << (sh - 64);
    }
}
__host__ __device__ inline u32 tasc_key_get(u64 lo, u64 hi, int j, int bits) {
    int sh = j * bits;
    u64 v;
    if (sh < 64) {
        v = lo >> sh;
        if (sh + bits > 64) v |= hi << (64 - sh);
    } else {
        v = hi >> (sh - 64);
    }
    return (u32)(v & ((1ull << bits) - 1));
}

// ---------------------------------------------------------------- model
struct TascLayerW {
    const void* wqkv;  // [(H + 2 Hkv) hd, d]: q heads, k heads, v heads
    const void* wo;    // [d, H hd]
    const void* wgu;   // [2F, d]: blocks of 16 gate rows followed by the 16 up rows of the same features
    const void* wd;    // [d, F]
    const float* g1;
    const float* g2;
    // The same four matrices in MFMA-fragment order for the small-batch kernel (nullptr if the model is not
    // eligible): tile (nt, ks) = rows 16 nt .. +16, columns 32 ks .. +32 is one contiguous KB, lane l of a wave
    // owning the 8 elements W[16 nt + (l & 15)][32 ks + 8 (l >> 4) .. +8]; tiles ordered [nt][ks].  A wave
    // instruction that loads one A fragment per lane then reads 8 whole cache lines instead of 16 half lines.
    const void* wqkv_f;
    const void* wo_f;
    const void* wgu_f;
    const void* wd_f;
};

struct tasc_model {
    tasc_model_desc desc;
    void* lm_head_f = nullptr;   // LM head in MFMA-fragment order (rows padded to a multiple of 16), or nullptr
    std::vector<TascLayerW> layers;
    void* embed;
    void* lm_head;
    float* gf;
    float* rope_cos;   // [max_pos, hd/2]
    float* rope_sin;
    int64_t* bias_rowptr;
    int32_t* bias_col;
    float* bias_val;
    float* bias_base;
    TascLayerW* d_layers;   // device copy of `layers`
    std::vector<void*> allocs;
};

// ---------------------------------------------------------------- session
#define TASC_KV_BLOCK 16
#define TASC_MAX_CHAINS 4          // most ranges of sequences the tiled forward runs side by side
#define TASC_DRAFT_MAX_LEN 4096   // longest sequence the draft kernel can hold in LDS
#define TASC_LM_STRIP 128         // vocabulary columns per partial-argmax strip

struct TascSessDev {
    // per-sequence state (device)
    int32_t* tokens;     // [B, max_len] committed tokens: prompt then generated (last one = pending)
    int32_t* n_tok;      // [B] committed tokens
    int32_t* n_prompt;   // [B]
    int32_t* cached;     // [B] positions whose K,V are valid in the cache
    int32_t* n_emit;     // [B] generated tokens so far
    int32_t* block_tab;  // [B, max_blocks]
    // per-forward row metadata
    int32_t* row_tok;    // [M_max] input token of every row (clamped into the vocabulary)
    int32_t* n_rows;     // [B] active rows of the sequence in this forward
    int32_t* pos0;       // [B] position of the sequence's first row
    int32_t* sel_rows;   // [M_max] rows fed to the LM head (negative: none, row 0 is used and ignored)
    int32_t* sel_tok;    // [M_max] input token of every LM-head row (its bias row)
    // counters: [0] sequences that reached max_new, [1] min n_emit scratch, [2] steps, [3] accepted,
    // [4] proposed, [8..8+TASC_MAX_K] accept-length histogram
    u64* counters;
    // activations
    float* x;            // [M_max, d] residual stream
    void* h;             // [M_max, d]   normalised activations, model dtype
    float* qkv;          // [M_max, (H + 2Hkv) hd]
    void* q;             // [M_max, H hd] rotated queries, model dtype
    void* att;           // [M_max, H hd]
    void* act;           // [M_max, F]
    float* part_val;     // [M_max, n_strips]
    int32_t* part_idx;   // [M_max, n_strips]
    int32_t* amax;       // [M_max] argmax token of every LM-head row
    float* att_part;     // attention split partials
    char* small_ws;      // the small-batch kernel's per-phase / per-layer activation buffers (tasc_small_ws_bytes)
    int32_t* drafts;     // [B, TASC_MAX_K] used by tasc_generate
    int32_t* bias_ptr;   // [M_max, n_strips + 1] LM-head bias cursors of the small-batch kernel
};

// one verify step of the tiled kernels, recorded once and replayed: its launches only name buffers of the session and
// the caller's draft / result pointers, which make the key
struct TascStepGraph {
    int32_t k, chains;
    const int32_t* drafts;
    int32_t* accept_len;
    int32_t* emitted;
    int32_t seen;             // eager runs so far (the first run also does the kernels' one-off set-up); -1: capture failed
    hipGraphExec_t exec;      // null until recorded
};

struct tasc_session {
    const tasc_model* model;
    int32_t batch, max_len, max_rows, max_blocks, n_strips;
    int32_t max_new;
    int32_t prefilled;
    void* kv_pool;
    size_t kv_layer_stride;   // elements per layer
    size_t page_elems;        // elements per page (K and V)
    TascSessDev d;
    u64* host_counters;       // pinned
    u32 bar_epoch;            // barriers the layer group's arrival flags (counters[32..63]) have seen so far
    u64 barb_base;            // same for the whole-grid barrier counter (counters[26])
    hipStream_t chain_st[TASC_MAX_CHAINS - 1];   // streams of the second and later chains of the tiled forward
    hipEvent_t chain_fork, chain_join[TASC_MAX_CHAINS - 1];
    bool chain_ready;         // the streams and events above exist
    hipStream_t graph_st;     // the stream verify steps are captured on (a graph may be launched on any stream)
    std::vector<TascStepGraph> step_graphs;   // instantiated verify steps, by their arguments
    int ll_copy;              // which copy of the small-batch activation buffers the next pipeline launch uses
    bool ll_armed;            // both copies hold the "not written yet" pattern wherever the next launch expects it
};

// counters[] slots used beyond the statistics
#define TASC_CTR_FLAGS 32     // 64 32-bit arrival flags of the layer-group barrier (slots 32..63)
#define TASC_N_COUNTERS 64
#define TASC_CTR_BAR_ERR 25   // grid-barrier time-out flag (low 32 bits)
#define TASC_CTR_BARB 26      // whole-grid barrier arrival counter
#define TASC_CTR_XCD_STEPS 28 // steps of the persistent kernel whose layer group used XCD-local barriers
#define TASC_CTR_XCC 27       // XCDs the layer group of the running step found itself on (low 32 bits)

// the tail of a verify step, fused into the forward when the small-batch kernel runs it
struct TascVerifyTail {
    int32_t k;
    const int32_t* drafts;
    int32_t* accept_len;
    int32_t* emitted;
    int32_t* trace_step;
    bool done;                // out: the forward already performed the accept
};

// library-wide options (tasc_config_set)
// Layout of ONE copy of the small-batch kernels' activation buffers (each written once per launch): byte offsets, strides
// in elements, and the size of a copy in bytes.  16 rows throughout.  The workspace holds two copies: the pipeline
// kernel uses them in turn and refills the idle one with its "not written yet" pattern (the barrier kernel uses copy 0).
struct TascSmallWs {
    size_t x_off, x_stride;         // float [2 L + 1][16][D]
    size_t q_off, att_off, q_stride;   // bf16 [L][16][H hd] each
    size_t act_off, act_stride;     // bf16  [L][16][F]
    size_t kvn_off, kvn_stride;     // bf16  [L][16][2 Hkv hd]: the launch's own key and value rows
    size_t pv_off, pi_off;          // float / int32 [16][n_strips]: LM-head strip maxima and their token ids
    size_t bytes;
};
inline TascSmallWs tasc_small_ws_layout(const tasc_model_desc& c) {
    TascSmallWs w;
    const size_t L = c.n_layers, HD = (size_t)c.n_heads * c.head_dim, KD = (size_t)c.n_kv_heads * c.head_dim, al = 256;
    const size_t n_strips = ((size_t)c.vocab + TASC_LM_STRIP - 1) / TASC_LM_STRIP;
    auto up = [&](size_t v) { return (v + al - 1) / al * al; };
    size_t o = 0;
    w.x_off = o; w.x_stride = 16 * (size_t)c.d_model; o += up((2 * L + 1) * w.x_stride * 4);
    w.q_stride = 16 * HD;
    w.q_off = o; o += up(L * w.q_stride * 2);
    w.att_off = o; o += up(L * w.q_stride * 2);
    w.act_off = o; w.act_stride = 16 * (size_t)c.d_ffn; o += up(L * w.act_stride * 2);
    w.kvn_off = o; w.kvn_stride = 16 * 2 * KD; o += up(L * w.kvn_stride * 2);
    w.pv_off = o; o += up(16 * n_strips * 4);
    w.pi_off = o; o += up(16 * n_strips * 4);
    w.bytes = o;
    return w;
}
inline size_t tasc_small_ws_bytes(const tasc_model_desc& c) { return c.dtype == TASC_BF16 ? 2 * tasc_small_ws_layout(c).bytes : 256; }

struct TascConfig {
    int small_path;           // 0: generic kernels only, 1: fused kernel one phase per launch, 2: persistent
    int small_grid;           // workgroups of the persistent kernel (0 = one per compute unit)
    int layer_wgs;            // workgroups of its layer group (0 = default)
    int layer_stride;         // the group's workgroup-id stride (0 = default)
    int tiled_path;           // 1: LDS-tiled MFMA kernels for bf16 forwards of more than 16 rows, 0: generic kernels
    int xcd_local;            // 1 = the layer group may use XCD-local barriers when it sits on one XCD
    int layer_workers;        // members of the layer group that compute in XCD-local mode (0 = all), the rest prefetch
    int small_kernel;         // 1: the spatial-pipeline kernel where the model fits it, 0: the barrier kernel always
    int pipe_share;           // tiles a workgroup of the pipeline kernel takes per layer at least (1..3): fewer, fatter workgroups
    int chains;               // ranges of sequences whose layers run side by side on streams of their own (0 = the library's rule)
    int step_graph;           // 1: verify steps of the tiled kernels are recorded into a graph and replayed, 0: launched one by one
};
extern TascConfig g_tasc_config;

// forward.hip
// fills both copies of the small-batch activation buffers with the pipeline kernel's "not written yet" pattern
tasc_status tasc_pipe_arm(tasc_session* s, hipStream_t st);
// true if a forward of nq rows per sequence of this session takes the tiled kernels (and no fused persistent one)
bool tasc_forward_is_tiled(const tasc_model* m, const tasc_session* s, int32_t nq);
// the chain count forward_tiled would use
int tasc_forward_chains(const tasc_model* m, const tasc_session* s, int32_t nq);
tasc_status tasc_forward_rows(const tasc_model* m, tasc_session* s, int32_t nq, int32_t n_sel,
                              float* logits_dbg, TascVerifyTail* tail, hipStream_t st);

// profile.hip: optional event timing per kernel class
bool tasc_prof_on(int cls);
bool tasc_prof_any();
int tasc_prof_begin(int cls, hipStream_t st);
void tasc_prof_end(int handle, hipStream_t st);
struct TascProfScope {
    int h;
    hipStream_t st;
    TascProfScope(int cls, hipStream_t s) : h(-1), st(s) { if (tasc_prof_on(cls)) h = tasc_prof_begin(cls, s); }
    ~TascProfScope() { if (h >= 0) tasc_prof_end(h, st); }
};
