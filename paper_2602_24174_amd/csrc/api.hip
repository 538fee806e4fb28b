// Model and session handles, the greedy accept step, and the draft-then-verify loop
// (paper, subsection "Speculative Decoding": gamma drafted tokens, one target forward, a prefix of
// k <= gamma tokens accepted; greedy, beam size 1).
#include "tasc_internal.h"
#include <math.h>
#include <string.h>
#include <algorithm>

namespace {

size_t elt_size(int dtype) { return dtype == TASC_F32 ? 4 : 2; }
size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---------------------------------------------------------------- per-forward row metadata
__global__ void k_reset(int B, int max_len, const int32_t* __restrict__ prompts, const int64_t* __restrict__ off,
                        int32_t* tokens, int32_t* n_tok, int32_t* n_prompt, int32_t* cached, int32_t* n_emit, u64* counters) {
    const int b = blockIdx.x;
    const int64_t o = off[b];
    const int P = (int)(off[b + 1] - o);
    for (int i = threadIdx.x; i < P; i += blockDim.x) tokens[(size_t)b * max_len + i] = prompts[o + i];
    if (threadIdx.x == 0) {
        n_tok[b] = P;
        n_prompt[b] = P;
        cached[b] = 0;
        n_emit[b] = 0;
    }
    if (b == 0)
        for (int i = threadIdx.x; i < TASC_N_COUNTERS; i += blockDim.x) counters[i] = 0;
}

__global__ void k_check_prompts(const int32_t* __restrict__ prompts, int64_t n, int vocab, u64* flag) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n && (prompts[i] < 0 || prompts[i] >= vocab)) atomicOr(flag, 1ull);
}

// prompt chunk c of C positions: rows, positions, and which rows feed the LM head
__global__ void k_prepare_prefill(int B, int C, int chunk, int max_len, const int32_t* __restrict__ tokens,
                                  const int32_t* __restrict__ n_prompt, int32_t* row_tok, int32_t* n_rows, int32_t* pos0,
                                  int32_t* sel_rows, int32_t* sel_tok) {
    const int b = blockIdx.x;
    const int P = n_prompt[b], base = chunk * C;
    const int nr = max(0, min(C, P - base));
    for (int i = threadIdx.x; i < C; i += blockDim.x) row_tok[b * C + i] = i < nr ? tokens[(size_t)b * max_len + base + i] : 0;
    if (threadIdx.x == 0) {
        n_rows[b] = nr;
        pos0[b] = base;
        const bool last = P - 1 >= base && P - 1 < base + C;
        sel_rows[b] = last ? b * C + (P - 1 - base) : -1;
        sel_tok[b] = last ? tokens[(size_t)b * max_len + P - 1] : 0;
    }
}

// after a prompt chunk: the cache now covers the chunk; a sequence whose prompt ended in it commits
// the argmax of its last position as generated token #1
__global__ void k_commit_prefill(int B, int C, int chunk, int max_len, int max_new, const int32_t* __restrict__ n_prompt,
                                 const int32_t* __restrict__ sel_rows, const int32_t* __restrict__ amax, int have_lm,
                                 int32_t* tokens, int32_t* n_tok, int32_t* cached, int32_t* n_emit, u64* counters) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int P = n_prompt[b];
    cached[b] = min(P, (chunk + 1) * C);
    if (have_lm && sel_rows[b] >= 0) {
        tokens[(size_t)b * max_len + P] = amax[b];
        n_tok[b] = P + 1;
        n_emit[b] = 1;
        if (max_new <= 1) atomicAdd(&counters[0], 1ull);
    }
}

__global__ void k_prepare_verify(int B, int k, int max_len, int vocab, const int32_t* __restrict__ tokens,
                                 const int32_t* __restrict__ n_tok, const int32_t* __restrict__ cached,
                                 const int32_t* __restrict__ drafts, int32_t* row_tok, int32_t* n_rows, int32_t* pos0,
                                 int32_t* sel_rows, int32_t* sel_tok) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    const int nq = k + 1;
    if (idx >= B * nq) return;
    const int b = idx / nq, i = idx % nq;
    int t;
    if (i == 0) {
        t = tokens[(size_t)b * max_len + n_tok[b] - 1];
        n_rows[b] = nq;
        pos0[b] = cached[b];
    } else {
        t = drafts[b * k + i - 1];
        t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);   // a draft outside the vocabulary can only be rejected
    }
    row_tok[idx] = t;
    sel_rows[idx] = idx;
    sel_tok[idx] = t;
}

// Greedy acceptance (one thread per sequence): longest prefix of the drafts equal to the target's
// argmax, plus the bonus token; rollback = the cached length only grows by the accepted rows.
__global__ void k_accept(int B, int k, int max_len, int max_new, const int32_t* __restrict__ drafts,
                         const int32_t* __restrict__ amax, int32_t* tokens, int32_t* n_tok, int32_t* cached, int32_t* n_emit,
                         u64* counters, int32_t* accept_len, int32_t* emitted, int32_t* trace_step) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int nq = k + 1;
    const int N = n_tok[b];
    const bool frozen = n_emit[b] >= max_new;
    int m = 0;
    if (!frozen) {
        while (m < k && drafts[b * k + m] == amax[b * nq + m]) ++m;
        int32_t* seq = tokens + (size_t)b * max_len;
        for (int i = 0; i < m; ++i) seq[N + i] = drafts[b * k + i];
        seq[N + m] = amax[b * nq + m];
        n_tok[b] = N + m + 1;
        cached[b] += m + 1;
        const int e = n_emit[b] + m + 1;
        n_emit[b] = e;
        if (e >= max_new) atomicAdd(&counters[0], 1ull);
        atomicAdd(&counters[3], (u64)m);
        atomicAdd(&counters[4], (u64)k);
        atomicAdd(&counters[8 + m], 1ull);
    }
    if (accept_len) accept_len[b] = m;
    if (emitted)
        for (int i = 0; i < nq; ++i)
            emitted[b * nq + i] = frozen ? -1 : (i < m ? drafts[b * k + i] : (i == m ? amax[b * nq + m] : -1));
    if (trace_step) {
        int32_t* t = trace_step + (size_t)b * (2 * k + 3);
        t[0] = N;
        for (int i = 0; i < k; ++i) t[1 + i] = drafts[b * k + i];
        for (int i = 0; i < nq; ++i) t[1 + k + i] = amax[b * nq + i];
        t[2 * k + 2] = frozen ? -1 : m;
    }
    if (b == 0) atomicAdd(&counters[2], 1ull);
}

// counters[1] = the fewest tokens any sequence has generated (valid after the kernel; reset before)
__global__ void k_min_emit(int B, const int32_t* __restrict__ n_emit, u64* counters) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) atomicMin(&counters[1], (u64)n_emit[b]);
}
__global__ void k_set_u64(u64* p, u64 v) { *p = v; }

__global__ void k_gather_out(int B, int max_len, int max_new, const int32_t* __restrict__ tokens,
                             const int32_t* __restrict__ n_prompt, int32_t* out) {
    const int b = blockIdx.x;
    for (int i = threadIdx.x; i < max_new; i += blockDim.x) out[(size_t)b * max_new + i] = tokens[(size_t)b * max_len + n_prompt[b] + i];
}

__global__ void k_init_block_tab(int B, int max_blocks, int32_t* bt) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= B * max_blocks) return;
    const int b = idx / max_blocks, j = idx % max_blocks;
    bt[idx] = j * B + b;   // pages of one sequence are interleaved with the other sequences'
}

}  // namespace

// ================================================================ model
// out (MFMA-fragment order, see TascLayerW) <- W [N][K] row-major bf16; rows N .. n_pad read as zero
__global__ void k_repack_frag(const uint16_t* __restrict__ W, int N, int K, int n_pad, uint16_t* __restrict__ out) {
    const int64_t chunk = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;     // one 16-byte chunk per thread
    const int nks = K / 32;
    if (chunk >= (int64_t)(n_pad / 16) * nks * 64) return;
    const int lane = (int)(chunk & 63);
    const int64_t tile = chunk >> 6;
    const int ks = (int)(tile % nks), nt = (int)(tile / nks);
    const int row = nt * 16 + (lane & 15), col = ks * 32 + 8 * (lane >> 4);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row < N) v = *reinterpret_cast<const uint4*>(W + (size_t)row * K + col);
    *reinterpret_cast<uint4*>(out + chunk * 8) = v;
}

extern "C" tasc_status tasc_model_create(const tasc_model_desc* desc, const tasc_weight_ptrs* w, tasc_model** out) {
    TASC_REQUIRE(desc && w && out, "model_create: null argument");
    const tasc_model_desc& c = *desc;
    TASC_REQUIRE(c.dtype == TASC_F32 || c.dtype == TASC_BF16, "model_create: dtype %d", c.dtype);
    TASC_REQUIRE(c.n_layers >= 1 && c.d_model >= 8 && c.n_heads >= 1 && c.n_kv_heads >= 1 && c.head_dim >= 8 && c.d_ffn >= 16 &&
                     c.vocab >= 2 && c.max_pos >= 1,
                 "model_create: non-positive dimension");
    TASC_REQUIRE(c.d_model % 8 == 0 && c.head_dim % 8 == 0 && c.d_ffn % 16 == 0, "model_create: d_model and head_dim must be "
                 "multiples of 8, d_ffn of 16");
    TASC_REQUIRE(c.head_dim <= 256, "model_create: head_dim %d > 256", c.head_dim);
    TASC_REQUIRE(c.n_heads % c.n_kv_heads == 0, "model_create: n_heads %d not a multiple of n_kv_heads %d", c.n_heads,
                 c.n_kv_heads);
    TASC_REQUIRE(w->embed && w->lm_head && w->gf && w->wq && w->wk && w->wv && w->wo && w->wg && w->wu && w->wd && w->g1 && w->g2,
                 "model_create: null weight pointer");
    const bool has_bias = w->bias_rowptr || w->bias_col || w->bias_val || w->bias_base;
    TASC_REQUIRE(!has_bias || (w->bias_rowptr && w->bias_base), "model_create: incomplete bias table");

    tasc_model* m = new tasc_model();
    m->desc = c;
    m->embed = m->lm_head = nullptr;
    m->gf = m->rope_cos = m->rope_sin = nullptr;
    m->bias_rowptr = nullptr; m->bias_col = nullptr; m->bias_val = nullptr; m->bias_base = nullptr;
    struct Guard { tasc_model* p; ~Guard() { if (p) tasc_model_destroy(p); } } guard{m};
    const size_t es = elt_size(c.dtype);
    const size_t D = c.d_model, HD = (size_t)c.n_heads * c.head_dim, KD = (size_t)c.n_kv_heads * c.head_dim, F = c.d_ffn;

    auto dev_alloc = [&](size_t bytes, void** p) -> tasc_status {
        TASC_HIP(hipMalloc(p, std::max<size_t>(bytes, 16)));
        m->allocs.push_back(*p);
        return TASC_OK;
    };
    auto dev_copy = [&](const void* src, size_t bytes, void** p) -> tasc_status {
        tasc_status rc = dev_alloc(bytes, p);
        if (rc != TASC_OK) return rc;
        if (bytes) TASC_HIP(hipMemcpy(*p, src, bytes, hipMemcpyDefault));
        return TASC_OK;
    };
    // fragment-order copies for the small-batch kernel, if the model has the shapes that kernel serves
    const bool frag = c.dtype == TASC_BF16 && c.d_model % 32 == 0 && c.d_model <= 1536 && c.d_ffn % 32 == 0 && c.n_layers <= 48 &&
                      (c.head_dim == 32 || c.head_dim == 64 || c.head_dim == 128);
    auto dev_frag = [&](const void* src, size_t N, size_t K, const void** p) -> tasc_status {
        const size_t n_pad = (N + 15) / 16 * 16;
        void* q;
        tasc_status rc2 = dev_alloc(n_pad * K * 2, &q);
        if (rc2 != TASC_OK) return rc2;
        const int64_t chunks = (int64_t)(n_pad / 16) * (K / 32) * 64;
        k_repack_frag<<<dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, 0>>>((const uint16_t*)src, (int)N, (int)K, (int)n_pad, (uint16_t*)q);
        TASC_LAUNCH_CHECK();
        *p = q;
        return TASC_OK;
    };
    tasc_status rc;
    if ((rc = dev_copy(w->embed, (size_t)c.vocab * D * es, &m->embed)) != TASC_OK) return rc;
    if ((rc = dev_copy(w->lm_head, (size_t)c.vocab * D * es, &m->lm_head)) != TASC_OK) return rc;
    if (frag && (rc = dev_frag(m->lm_head, c.vocab, D, (const void**)&m->lm_head_f)) != TASC_OK) return rc;
    if ((rc = dev_copy(w->gf, D * 4, (void**)&m->gf)) != TASC_OK) return rc;
    m->d_layers = nullptr;
    m->layers.resize(c.n_layers);
    for (int l = 0; l < c.n_layers; ++l) {
        TASC_REQUIRE(w->wq[l] && w->wk[l] && w->wv[l] && w->wo[l] && w->wg[l] && w->wu[l] && w->wd[l] && w->g1[l] && w->g2[l],
                     "model_create: null weight pointer in layer %d", l);
        TascLayerW& L = m->layers[l];
        void* p;
        if ((rc = dev_alloc((HD + 2 * KD) * D * es, &p)) != TASC_OK) return rc;
        TASC_HIP(hipMemcpy(p, w->wq[l], HD * D * es, hipMemcpyDefault));
        TASC_HIP(hipMemcpy((char*)p + HD * D * es, w->wk[l], KD * D * es, hipMemcpyDefault));
        TASC_HIP(hipMemcpy((char*)p + (HD + KD) * D * es, w->wv[l], KD * D * es, hipMemcpyDefault));
        L.wqkv = p;
        if ((rc = dev_copy(w->wo[l], D * HD * es, &p)) != TASC_OK) return rc;
        L.wo = p;
        // gate / up interleaved in blocks of 16 rows
        if ((rc = dev_alloc(2 * F * D * es, &p)) != TASC_OK) return rc;
        const size_t blk = 16 * D * es;
        TASC_HIP(hipMemcpy2D(p, 2 * blk, w->wg[l], blk, blk, F / 16, hipMemcpyDefault));
        TASC_HIP(hipMemcpy2D((char*)p + blk, 2 * blk, w->wu[l], blk, blk, F / 16, hipMemcpyDefault));
        L.wgu = p;
        if ((rc = dev_copy(w->wd[l], D * F * es, &p)) != TASC_OK) return rc;
        L.wd = p;
        if ((rc = dev_copy(w->g1[l], D * 4, &p)) != TASC_OK) return rc;
        L.g1 = (const float*)p;
        if ((rc = dev_copy(w->g2[l], D * 4, &p)) != TASC_OK) return rc;
        L.g2 = (const float*)p;
        L.wqkv_f = L.wo_f = L.wgu_f = L.wd_f = nullptr;
        if (frag) {
            if ((rc = dev_frag(L.wqkv, HD + 2 * KD, D, &L.wqkv_f)) != TASC_OK) return rc;
            if ((rc = dev_frag(L.wo, D, HD, &L.wo_f)) != TASC_OK) return rc;
            if ((rc = dev_frag(L.wgu, 2 * F, D, &L.wgu_f)) != TASC_OK) return rc;
            if ((rc = dev_frag(L.wd, D, F, &L.wd_f)) != TASC_OK) return rc;
        }
    }
    if ((rc = dev_copy(m->layers.data(), sizeof(TascLayerW) * c.n_layers, (void**)&m->d_layers)) != TASC_OK) return rc;
    // RoPE table: angle(p, i) = p * theta^(-2i/hd), double on the host, fp32 on the device
    {
        const int half = c.head_dim / 2;
        std::vector<float> cs((size_t)c.max_pos * half), sn((size_t)c.max_pos * half);
        for (int i = 0; i < half; ++i) {
            const double inv = pow((double)c.rope_theta, -2.0 * i / c.head_dim);
            for (int p = 0; p < c.max_pos; ++p) {
                cs[(size_t)p * half + i] = (float)cos(p * inv);
                sn[(size_t)p * half + i] = (float)sin(p * inv);
            }
        }
        if ((rc = dev_copy(cs.data(), cs.size() * 4, (void**)&m->rope_cos)) != TASC_OK) return rc;
        if ((rc = dev_copy(sn.data(), sn.size() * 4, (void**)&m->rope_sin)) != TASC_OK) return rc;
    }
    if (has_bias) {
        int64_t nnz = 0;
        TASC_HIP(hipMemcpy(&nnz, w->bias_rowptr + c.vocab, sizeof nnz, hipMemcpyDefault));
        TASC_REQUIRE(nnz >= 0 && (nnz == 0 || (w->bias_col && w->bias_val)), "model_create: bias table has %lld entries but no "
                     "column/value arrays", (long long)nnz);
        if ((rc = dev_copy(w->bias_rowptr, (size_t)(c.vocab + 1) * 8, (void**)&m->bias_rowptr)) != TASC_OK) return rc;
        if ((rc = dev_copy(w->bias_col, (size_t)nnz * 4, (void**)&m->bias_col)) != TASC_OK) return rc;
        if ((rc = dev_copy(w->bias_val, (size_t)nnz * 4, (void**)&m->bias_val)) != TASC_OK) return rc;
        if ((rc = dev_copy(w->bias_base, (size_t)c.vocab * 4, (void**)&m->bias_base)) != TASC_OK) return rc;
    }
    TASC_HIP(hipDeviceSynchronize());
    guard.p = nullptr;
    *out = m;
    return TASC_OK;
}

extern "C" void tasc_model_destroy(tasc_model* m) {
    if (!m) return;
    for (void* p : m->allocs) (void)hipFree(p);
    delete m;
}

// ================================================================ session
namespace {
struct WsLayout {
    size_t off[32];
    size_t total;
};
// carves the workspace; order must match bind_workspace
WsLayout ws_layout(const tasc_model_desc& c, int B, int max_len, int max_rows) {
    const size_t M = (size_t)B * max_rows, es = elt_size(c.dtype);
    const size_t HD = (size_t)c.n_heads * c.head_dim, KD = (size_t)c.n_kv_heads * c.head_dim;
    const size_t n_strips = ((size_t)c.vocab + TASC_LM_STRIP - 1) / TASC_LM_STRIP;
    const size_t max_blocks = ((size_t)max_len + TASC_KV_BLOCK - 1) / TASC_KV_BLOCK;
    const size_t sizes[] = {
        (size_t)B * max_len * 4,  // tokens
        (size_t)B * 4, (size_t)B * 4, (size_t)B * 4, (size_t)B * 4,  // n_tok n_prompt cached n_emit
        (size_t)B * max_blocks * 4,                                  // block_tab
        M * 4, (size_t)B * 4, (size_t)B * 4, M * 4, M * 4,           // row_tok n_rows pos0 sel_rows sel_tok
        TASC_N_COUNTERS * 8,                                         // counters (+ barrier flags)
        M * c.d_model * 4,                                           // x
        M * std::max<size_t>(c.d_model, 1) * es,                     // h
        M * (HD + 2 * KD) * 4,                                       // qkv
        M * HD * es, M * HD * es,                                    // q att
        M * (size_t)c.d_ffn * es,                                    // act
        M * n_strips * 4, M * n_strips * 4, M * 4,                   // part_val part_idx amax
        8 * M * std::max<size_t>(HD + 2 * KD, c.d_model) * 4,        // att_part: k-slice partial sums of the narrow GEMMs
        (size_t)B * TASC_MAX_K * 4,                                  // drafts
        M * (n_strips + 1) * 4,                                      // bias_ptr
        tasc_small_ws_bytes(c),                                      // write-once activation buffers of the small-batch kernel
    };
    WsLayout L;
    size_t o = 0;
    int i = 0;
    for (size_t sz : sizes) {
        L.off[i++] = o;
        o += align_up(sz, 256);
    }
    L.total = o;
    return L;
}
}  // namespace

extern "C" size_t tasc_session_kv_bytes(const tasc_model* m, int32_t batch, int32_t max_len) {
    if (!m || batch < 1 || max_len < 1) return 0;
    const tasc_model_desc& c = m->desc;
    const size_t max_blocks = ((size_t)max_len + TASC_KV_BLOCK - 1) / TASC_KV_BLOCK;
    const size_t page = 2 * (size_t)c.n_kv_heads * TASC_KV_BLOCK * c.head_dim;
    return (size_t)c.n_layers * batch * max_blocks * page * elt_size(c.dtype);
}

extern "C" size_t tasc_session_workspace_bytes(const tasc_model* m, int32_t batch, int32_t max_len, int32_t max_rows) {
    if (!m || batch < 1 || max_len < 1 || max_rows < 1) return 0;
    return ws_layout(m->desc, batch, max_len, max_rows).total;
}

extern "C" tasc_status tasc_session_create(const tasc_model* m, int32_t batch, int32_t max_len, int32_t max_rows, void* kv_pool,
                                           size_t kv_bytes, void* workspace, size_t ws_bytes, tasc_session** out) {
    TASC_REQUIRE(m && kv_pool && workspace && out, "session_create: null argument");
    TASC_REQUIRE(batch >= 1 && max_len >= 1 && max_rows >= 1, "session_create: batch %d, max_len %d, max_rows %d", batch, max_len,
                 max_rows);
    TASC_REQUIRE(max_len <= m->desc.max_pos, "session_create: max_len %d exceeds the model's max_pos %d", max_len, m->desc.max_pos);
    TASC_REQUIRE(((uintptr_t)kv_pool & 255) == 0 && ((uintptr_t)workspace & 255) == 0, "session_create: buffers must be 256-byte "
                 "aligned");
    const size_t need_kv = tasc_session_kv_bytes(m, batch, max_len);
    const WsLayout L = ws_layout(m->desc, batch, max_len, max_rows);
    if (kv_bytes < need_kv || ws_bytes < L.total) {
        tasc_set_error("session_create: kv pool %zu of %zu bytes, workspace %zu of %zu bytes", kv_bytes, need_kv, ws_bytes, L.total);
        return TASC_ENOMEM;
    }
    tasc_session* s = new tasc_session();
    s->model = m;
    s->batch = batch;
    s->max_len = max_len;
    s->max_rows = max_rows;
    s->max_blocks = (max_len + TASC_KV_BLOCK - 1) / TASC_KV_BLOCK;
    s->n_strips = (m->desc.vocab + TASC_LM_STRIP - 1) / TASC_LM_STRIP;
    s->max_new = 0;
    s->prefilled = 0;
    s->kv_pool = kv_pool;
    s->page_elems = 2 * (size_t)m->desc.n_kv_heads * TASC_KV_BLOCK * m->desc.head_dim;
    s->kv_layer_stride = (size_t)batch * s->max_blocks * s->page_elems;
    s->host_counters = nullptr;
    s->bar_epoch = 0;
    s->barb_base = 0;
    s->ll_copy = 0;
    s->ll_armed = false;
    s->chain_ready = false;
    s->graph_st = nullptr;
    char* w = (char*)workspace;
    int i = 0;
    TascSessDev& d = s->d;
    d.tokens = (int32_t*)(w + L.off[i++]);
    d.n_tok = (int32_t*)(w + L.off[i++]);
    d.n_prompt = (int32_t*)(w + L.off[i++]);
    d.cached = (int32_t*)(w + L.off[i++]);
    d.n_emit = (int32_t*)(w + L.off[i++]);
    d.block_tab = (int32_t*)(w + L.off[i++]);
    d.row_tok = (int32_t*)(w + L.off[i++]);
    d.n_rows = (int32_t*)(w + L.off[i++]);
    d.pos0 = (int32_t*)(w + L.off[i++]);
    d.sel_rows = (int32_t*)(w + L.off[i++]);
    d.sel_tok = (int32_t*)(w + L.off[i++]);
    d.counters = (u64*)(w + L.off[i++]);
    d.x = (float*)(w + L.off[i++]);
    d.h = (void*)(w + L.off[i++]);
    d.qkv = (float*)(w + L.off[i++]);
    d.q = (void*)(w + L.off[i++]);
    d.att = (void*)(w + L.off[i++]);
    d.act = (void*)(w + L.off[i++]);
    d.part_val = (float*)(w + L.off[i++]);
    d.part_idx = (int32_t*)(w + L.off[i++]);
    d.amax = (int32_t*)(w + L.off[i++]);
    d.att_part = (float*)(w + L.off[i++]);
    d.drafts = (int32_t*)(w + L.off[i++]);
    d.bias_ptr = (int32_t*)(w + L.off[i++]);
    d.small_ws = (char*)(w + L.off[i++]);
    struct Guard { tasc_session* p; ~Guard() { if (p) tasc_session_destroy(p); } } guard{s};
    TASC_HIP(hipHostMalloc((void**)&s->host_counters, 32 * sizeof(u64), hipHostMallocDefault));
    {   // streams (default priority) and events of the tiled forward's chains
        int made_st = 0, made_ev = 0;
        bool ok = hipEventCreateWithFlags(&s->chain_fork, hipEventDisableTiming) == hipSuccess;
        for (int i = 0; ok && i < TASC_MAX_CHAINS - 1; ++i) {
            ok = hipStreamCreateWithFlags(&s->chain_st[i], hipStreamNonBlocking) == hipSuccess;
            if (ok) ++made_st;
            ok = ok && hipEventCreateWithFlags(&s->chain_join[i], hipEventDisableTiming) == hipSuccess;
            if (ok) ++made_ev;
        }
        if (!ok) {
            for (int i = 0; i < made_st; ++i) (void)hipStreamDestroy(s->chain_st[i]);
            for (int i = 0; i < made_ev; ++i) (void)hipEventDestroy(s->chain_join[i]);
            tasc_set_error("session_create: streams of the forward chains -> %s", hipGetErrorString(hipGetLastError()));
            return TASC_EHIP;
        }
        if (hipStreamCreateWithFlags(&s->graph_st, hipStreamNonBlocking) != hipSuccess) {
            s->graph_st = nullptr;
            for (int i = 0; i < made_st; ++i) (void)hipStreamDestroy(s->chain_st[i]);
            for (int i = 0; i < made_ev; ++i) (void)hipEventDestroy(s->chain_join[i]);
            (void)hipEventDestroy(s->chain_fork);
            tasc_set_error("session_create: capture stream -> %s", hipGetErrorString(hipGetLastError()));
            return TASC_EHIP;
        }
        s->chain_ready = true;
    }
    const int n = batch * s->max_blocks;
    k_init_block_tab<<<dim3((n + 255) / 256), dim3(256), 0, 0>>>(batch, s->max_blocks, d.block_tab);
    TASC_LAUNCH_CHECK();
    TASC_HIP(hipMemsetAsync(d.counters, 0, TASC_N_COUNTERS * sizeof(u64), 0));
    // the MFMA attention multiplies masked keys by zero weights: the pool must never hold NaN or Inf patterns
    TASC_HIP(hipMemsetAsync(kv_pool, 0, need_kv, 0));
    TASC_HIP(hipDeviceSynchronize());
    guard.p = nullptr;
    *out = s;
    return TASC_OK;
}

extern "C" void tasc_session_destroy(tasc_session* s) {
    if (!s) return;
    if (s->host_counters) (void)hipHostFree(s->host_counters);
    for (TascStepGraph& e : s->step_graphs)
        if (e.exec) (void)hipGraphExecDestroy(e.exec);
    if (s->chain_ready) {
        (void)hipStreamDestroy(s->graph_st);
        (void)hipEventDestroy(s->chain_fork);
        for (int i = 0; i < TASC_MAX_CHAINS - 1; ++i) {
            (void)hipStreamDestroy(s->chain_st[i]);
            (void)hipEventDestroy(s->chain_join[i]);
        }
    }
    delete s;
}

extern "C" tasc_status tasc_session_prefill(const tasc_model* m, tasc_session* s, const int32_t* prompts,
                                            const int64_t* prompt_offsets, tasc_mem where, int32_t max_new, void* stream) {
    TASC_REQUIRE(m && s && prompts && prompt_offsets, "prefill: null argument");
    TASC_REQUIRE(s->model == m, "prefill: session belongs to another model");
    TASC_REQUIRE(max_new >= 1, "prefill: max_new %d < 1", max_new);
    TASC_REQUIRE(where == TASC_MEM_HOST || where == TASC_MEM_DEVICE, "prefill: bad memory kind");
    TASC_REQUIRE(prompt_offsets[0] == 0, "prefill: prompt_offsets[0] != 0");
    hipStream_t st = (hipStream_t)stream;
    const int B = s->batch, C = s->max_rows;
    int64_t longest = 0;
    for (int b = 0; b < B; ++b) {
        const int64_t P = prompt_offsets[b + 1] - prompt_offsets[b];
        TASC_REQUIRE(P >= 1, "prefill: prompt %d is empty", b);
        // room for the generated tokens, one step of overshoot and the rows a frozen sequence still writes
        TASC_REQUIRE(P + max_new + 2 * (int64_t)s->max_rows <= s->max_len,
                     "prefill: prompt %d (%lld tokens) + max_new %d + 2 x max_rows %d exceeds max_len %d", b, (long long)P, max_new,
                     s->max_rows, s->max_len);
        longest = std::max(longest, P);
    }
    const int64_t total = prompt_offsets[B];
    s->prefilled = 0;
    struct Tmp { std::vector<void*> p; ~Tmp() { for (void* q : p) (void)hipFree(q); } } tmp;
    const int32_t* d_prompts = prompts;
    if (where == TASC_MEM_HOST) {
        void* p;
        TASC_HIP(hipMalloc(&p, total * 4)); tmp.p.push_back(p);
        TASC_HIP(hipMemcpyAsync(p, prompts, total * 4, hipMemcpyHostToDevice, st));
        d_prompts = (const int32_t*)p;
    }
    int64_t* d_off;
    TASC_HIP(hipMalloc((void**)&d_off, (B + 1) * 8)); tmp.p.push_back(d_off);
    TASC_HIP(hipMemcpyAsync(d_off, prompt_offsets, (B + 1) * 8, hipMemcpyHostToDevice, st));
    TascSessDev& d = s->d;
    k_reset<<<dim3(B), dim3(256), 0, st>>>(B, s->max_len, d_prompts, d_off, d.tokens, d.n_tok, d.n_prompt, d.cached, d.n_emit,
                                           d.counters);
    TASC_LAUNCH_CHECK();
    s->bar_epoch = 0;  // k_reset cleared the barrier flags and counters (the time-out flag among them) with the other counters
    s->barb_base = 0;
    s->ll_armed = false;   // a step that timed out may have left its hand-over buffers half written: re-armed at the next launch
    k_check_prompts<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(d_prompts, total, m->desc.vocab, &d.counters[31]);
    TASC_LAUNCH_CHECK();
    TASC_HIP(hipMemcpyAsync(s->host_counters, d.counters, 32 * 8, hipMemcpyDeviceToHost, st));
    TASC_HIP(hipStreamSynchronize(st));
    TASC_REQUIRE(s->host_counters[31] == 0, "prefill: a prompt token lies outside [0, %d)", m->desc.vocab);
    TASC_HIP(hipMemsetAsync(&d.counters[31], 0, 8, st));
    s->max_new = max_new;

    const int n_chunks = (int)((longest + C - 1) / C);
    for (int c = 0; c < n_chunks; ++c) {
        bool any_last = false;
        for (int b = 0; b < B && !any_last; ++b) {
            const int64_t P = prompt_offsets[b + 1] - prompt_offsets[b];
            any_last = P - 1 >= (int64_t)c * C && P - 1 < (int64_t)(c + 1) * C;
        }
        k_prepare_prefill<<<dim3(B), dim3(64), 0, st>>>(B, C, c, s->max_len, d.tokens, d.n_prompt, d.row_tok, d.n_rows, d.pos0,
                                                        d.sel_rows, d.sel_tok);
        TASC_LAUNCH_CHECK();
        tasc_status rc = tasc_forward_rows(m, s, C, any_last ? B : 0, nullptr, nullptr, st);
        if (rc != TASC_OK) return rc;
        k_commit_prefill<<<dim3((B + 63) / 64), dim3(64), 0, st>>>(B, C, c, s->max_len, max_new, d.n_prompt, d.sel_rows, d.amax,
                                                                   any_last ? 1 : 0, d.tokens, d.n_tok, d.cached, d.n_emit,
                                                                   d.counters);
        TASC_LAUNCH_CHECK();
    }
    TASC_HIP(hipStreamSynchronize(st));   // the temporaries above are freed on return
    s->prefilled = 1;
    return TASC_OK;
}

namespace {
// the launches of one verify step on `st`
tasc_status verify_step_enqueue(const tasc_model* m, tasc_session* s, const int32_t* drafts, int32_t k, int32_t* accept_len,
                                int32_t* emitted, float* logits_dbg, int32_t* trace_step, hipStream_t st) {
    const int B = s->batch, nq = k + 1;
    TascSessDev& d = s->d;
    k_prepare_verify<<<dim3((B * nq + 255) / 256), dim3(256), 0, st>>>(B, k, s->max_len, m->desc.vocab, d.tokens, d.n_tok, d.cached,
                                                                       drafts, d.row_tok, d.n_rows, d.pos0, d.sel_rows, d.sel_tok);
    TASC_LAUNCH_CHECK();
    TascVerifyTail tail{k, drafts, accept_len, emitted, trace_step, false};
    tasc_status rc = tasc_forward_rows(m, s, nq, B * nq, logits_dbg, &tail, st);
    if (rc != TASC_OK) return rc;
    if (!tail.done) {
        TascProfScope ps(TASC_KC_ACCEPT, st);
        k_accept<<<dim3((B + 63) / 64), dim3(64), 0, st>>>(B, k, s->max_len, s->max_new, drafts, d.amax, d.tokens, d.n_tok,
                                                           d.cached, d.n_emit, d.counters, accept_len, emitted, trace_step);
    }
    TASC_LAUNCH_CHECK();
    return TASC_OK;
}

// A verify step of the tiled kernels is a few hundred launches whose arguments never change from step to step (row
// counts, positions and tokens live in device memory), so the second step with the same arguments is recorded into a
// graph, on a stream of the session's own, and every later one is a single graph launch on the caller's stream.
tasc_status verify_step_impl(const tasc_model* m, tasc_session* s, const int32_t* drafts, int32_t k, int32_t* accept_len,
                             int32_t* emitted, float* logits_dbg, int32_t* trace_step, hipStream_t st) {
    TascProfScope whole(TASC_KC_VERIFY, st);
    bool graphable = g_tasc_config.step_graph != 0 && s->chain_ready && !logits_dbg && !trace_step && !tasc_prof_any() &&
                     tasc_forward_is_tiled(m, s, k + 1);
    if (graphable) {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(st, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) {
            (void)hipGetLastError();
            graphable = false;                // the caller records this step itself
        }
    }
    if (!graphable) return verify_step_enqueue(m, s, drafts, k, accept_len, emitted, logits_dbg, trace_step, st);
    const int chains = tasc_forward_chains(m, s, k + 1);
    TascStepGraph* g = nullptr;
    for (TascStepGraph& e : s->step_graphs)
        if (e.k == k && e.chains == chains && e.drafts == drafts && e.accept_len == accept_len && e.emitted == emitted) g = &e;
    if (!g) {
        if (s->step_graphs.size() >= 8) {     // a caller that keeps changing its buffers: forget the oldest
            if (s->step_graphs.front().exec) (void)hipGraphExecDestroy(s->step_graphs.front().exec);
            s->step_graphs.erase(s->step_graphs.begin());
        }
        s->step_graphs.push_back(TascStepGraph{k, chains, drafts, accept_len, emitted, 0, nullptr});
        g = &s->step_graphs.back();
    }
    if (!g->exec && g->seen >= 1) {
        hipGraph_t graph = nullptr;
        bool ok = hipStreamBeginCapture(s->graph_st, hipStreamCaptureModeThreadLocal) == hipSuccess;
        if (ok) {
            const tasc_status rc = verify_step_enqueue(m, s, drafts, k, accept_len, emitted, nullptr, nullptr, s->graph_st);
            ok = hipStreamEndCapture(s->graph_st, &graph) == hipSuccess && rc == TASC_OK && graph != nullptr;
        }
        ok = ok && hipGraphInstantiate(&g->exec, graph, nullptr, nullptr, 0) == hipSuccess;
        if (graph) (void)hipGraphDestroy(graph);
        if (!ok) {
            (void)hipGetLastError();
            g->exec = nullptr;
            g->seen = -1;                     // this key stays on plain launches
        }
    }
    if (g->exec) {
        TASC_HIP(hipGraphLaunch(g->exec, st));
        return TASC_OK;
    }
    if (g->seen >= 0) ++g->seen;
    return verify_step_enqueue(m, s, drafts, k, accept_len, emitted, logits_dbg, trace_step, st);
}
}  // namespace

extern "C" tasc_status tasc_verify_step(const tasc_model* m, tasc_session* s, const int32_t* drafts, int32_t k,
                                        int32_t* accept_len, int32_t* emitted, float* logits_dbg, void* stream) {
    TASC_REQUIRE(m && s, "verify_step: null argument");
    TASC_REQUIRE(s->model == m, "verify_step: session belongs to another model");
    TASC_REQUIRE(k >= 0 && k <= TASC_MAX_K && k + 1 <= s->max_rows, "verify_step: k %d outside [0, min(%d, max_rows - 1 = %d)]", k,
                 TASC_MAX_K, s->max_rows - 1);
    TASC_REQUIRE(k == 0 || drafts, "verify_step: null drafts");
    if (!s->prefilled) {
        tasc_set_error("verify_step: session has no prompt yet");
        return TASC_ESTATE;
    }
    return verify_step_impl(m, s, drafts, k, accept_len, emitted, logits_dbg, nullptr, (hipStream_t)stream);
}

extern "C" tasc_status tasc_generate(const tasc_model* m, const tasc_ngram* ng, tasc_session* s, const int32_t* prompts,
                                     const int64_t* prompt_offsets, tasc_mem where, int32_t max_new, const tasc_spec_params* p,
                                     int32_t* out_tokens, int32_t* trace, int32_t trace_steps, tasc_gen_stats* stats,
                                     void* stream) {
    TASC_REQUIRE(m && s && p && out_tokens, "generate: null argument");
    TASC_REQUIRE(p->k >= 0 && p->k <= TASC_MAX_K && p->k + 1 <= s->max_rows, "generate: k %d outside [0, min(%d, max_rows - 1)]",
                 p->k, TASC_MAX_K);
    TASC_REQUIRE(p->k == 0 || ng, "generate: k > 0 needs the n-gram tables");
    TASC_REQUIRE(!trace || trace_steps >= 0, "generate: negative trace capacity");
    hipStream_t st = (hipStream_t)stream;
    struct Ev { hipEvent_t e[3]; int n = 0; ~Ev() { for (int i = 0; i < n; ++i) (void)hipEventDestroy(e[i]); } } ev;
    for (int i = 0; i < 3; ++i) { TASC_HIP(hipEventCreate(&ev.e[i])); ev.n = i + 1; }
    TASC_HIP(hipEventRecord(ev.e[0], st));
    tasc_status rc = tasc_session_prefill(m, s, prompts, prompt_offsets, where, max_new, st);
    if (rc != TASC_OK) return rc;
    TASC_HIP(hipEventRecord(ev.e[1], st));
    const int B = s->batch, k = p->k;
    TascSessDev& d = s->d;
    const size_t trace_stride = (size_t)B * (2 * k + 3);
    int64_t steps = 0;
    int64_t min_emit = 1;
    while (min_emit < max_new) {
        // every step emits at least 1 and at most k + 1 tokens per sequence: this many steps are certainly needed
        const int64_t run = (max_new - min_emit + k) / (k + 1);
        for (int64_t i = 0; i < run; ++i, ++steps) {
            if (k > 0) {
                rc = tasc_draft(ng, s, p, d.drafts, st);
                if (rc != TASC_OK) return rc;
            }
            int32_t* tr = (trace && steps < trace_steps) ? trace + steps * trace_stride : nullptr;
            rc = verify_step_impl(m, s, d.drafts, k, nullptr, nullptr, nullptr, tr, st);
            if (rc != TASC_OK) return rc;
        }
        k_set_u64<<<dim3(1), dim3(1), 0, st>>>(&d.counters[1], ~0ull);
        k_min_emit<<<dim3((B + 255) / 256), dim3(256), 0, st>>>(B, d.n_emit, d.counters);
        TASC_LAUNCH_CHECK();
        TASC_HIP(hipMemcpyAsync(s->host_counters, d.counters, 32 * 8, hipMemcpyDeviceToHost, st));
        TASC_HIP(hipStreamSynchronize(st));
        min_emit = (int64_t)s->host_counters[1];
    }
    k_gather_out<<<dim3(B), dim3(256), 0, st>>>(B, s->max_len, max_new, d.tokens, d.n_prompt, out_tokens);
    TASC_LAUNCH_CHECK();
    TASC_HIP(hipEventRecord(ev.e[2], st));
    TASC_HIP(hipMemcpyAsync(s->host_counters, d.counters, 32 * 8, hipMemcpyDeviceToHost, st));
    TASC_HIP(hipStreamSynchronize(st));
    if (s->host_counters[TASC_CTR_BAR_ERR] != 0) {
        tasc_set_error("generate: a grid barrier of the persistent kernel timed out; the session must be prefilled again");
        return TASC_EHIP;
    }
    if (stats) {
        memset(stats, 0, sizeof *stats);
        stats->steps = steps;
        stats->emitted = (int64_t)B * max_new;
        stats->accepted = (int64_t)s->host_counters[3];
        stats->proposed = (int64_t)s->host_counters[4];
        for (int i = 0; i <= TASC_MAX_K; ++i) stats->accept_hist[i] = (int64_t)s->host_counters[8 + i];
        stats->xcd_local_steps = (int64_t)s->host_counters[TASC_CTR_XCD_STEPS];
        float a = 0.f, b = 0.f;
        TASC_HIP(hipEventElapsedTime(&a, ev.e[0], ev.e[1]));
        TASC_HIP(hipEventElapsedTime(&b, ev.e[1], ev.e[2]));
        stats->prefill_ms = a;
        stats->decode_ms = b;
    }
    return TASC_OK;
}

extern "C" tasc_status tasc_session_status(tasc_session* s, int32_t* timed_out, void* stream) {
    TASC_REQUIRE(s && timed_out, "session_status: null argument");
    hipStream_t st = (hipStream_t)stream;
    TASC_HIP(hipMemcpyAsync(s->host_counters, s->d.counters, 32 * 8, hipMemcpyDeviceToHost, st));
    TASC_HIP(hipStreamSynchronize(st));
    *timed_out = s->host_counters[TASC_CTR_BAR_ERR] != 0 ? 1 : 0;
    return TASC_OK;
}

extern "C" tasc_status tasc_session_get_tokens(const tasc_session* s, int32_t b, int32_t* tokens, int32_t cap, int32_t* n,
                                               void* stream) {
    TASC_REQUIRE(s && n, "get_tokens: null argument");
    TASC_REQUIRE(b >= 0 && b < s->batch, "get_tokens: sequence %d outside [0, %d)", b, s->batch);
    hipStream_t st = (hipStream_t)stream;
    TASC_HIP(hipStreamSynchronize(st));
    int32_t cnt = 0;
    TASC_HIP(hipMemcpy(&cnt, s->d.n_tok + b, 4, hipMemcpyDeviceToHost));
    *n = cnt;
    if (!tokens) return TASC_OK;
    if (cap < cnt) {
        tasc_set_error("get_tokens: room for %d tokens, %d needed", cap, cnt);
        return TASC_ENOMEM;
    }
    TASC_HIP(hipMemcpy(tokens, s->d.tokens + (size_t)b * s->max_len, (size_t)cnt * 4, hipMemcpyDeviceToHost));
    return TASC_OK;
}
