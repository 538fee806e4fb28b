// Draft proposal: k tokens per sequence from the mixture of the corpus drafter and the context
// drafter (paper, section "Proposed Method: TASC-spec":
//     p_mixed(x|c) = lambda p_corp(x|c) + (1 - lambda) p_prompt(x|c),
// each source queried in descending order of n, first match wins, most frequent token if none).
//
// One workgroup per sequence.  The sequence's committed tokens sit in LDS; the context drafter is
// not a stored table but a scan: for the running suffix, every position of the sequence gets the
// length of its match with the suffix, the longest match gives the context's order, and the tokens
// that follow the matching positions are its successor multiset.  Exact integer scores.
#include "tasc_internal.h"

namespace {

constexpr int kThreads = 256;

struct DraftArgs {
    TascNgramView ng;
    const int32_t* tokens;    // [B, max_len]
    const int32_t* n_tok;     // [B]
    const int32_t* n_prompt;  // [B]
    int32_t max_len, k, q16, p_min_ctx, ctx_gen;
    int32_t* drafts;          // [B, k]
};

__device__ inline bool probe(const TascSlot* __restrict__ tab, u64 mask, u64 lo, u64 hi, int ntok, TascSlot& out) {
    u64 idx = tasc_hash_key(lo, hi, ntok) & mask;
    for (u64 p = 0; p <= mask; ++p) {
        TascSlot s = tab[idx];
        if (s.a == 0) return false;
        if (s.lo == lo && s.hi == hi) {
            out = s;
            return true;
        }
        idx = (idx + 1) & mask;
    }
    return false;
}

__global__ __launch_bounds__(kThreads) void k_draft(DraftArgs a) {
    __shared__ int32_t s_tok[TASC_DRAFT_MAX_LEN];
    __shared__ int32_t s_list[TASC_DRAFT_MAX_LEN];   // successors of the matching positions
    __shared__ uint16_t s_cnt[TASC_DRAFT_MAX_LEN];   // multiplicity of s_list[e] within the list
    __shared__ uint8_t s_ml[TASC_DRAFT_MAX_LEN];     // match length of every position with the suffix
    __shared__ int32_t s_suf[TASC_MAX_ORDER];        // s_suf[i] = i-th token from the end of the running context
    __shared__ int32_t s_d[TASC_MAX_K];
    __shared__ int s_mmax, s_m, s_T, s_ncorp, s_x;
    __shared__ u64 s_best;
    __shared__ TascSlot s_hit[TASC_MAX_ORDER + 1];
    __shared__ int s_found[TASC_MAX_ORDER + 1];

    const int b = blockIdx.x, tid = threadIdx.x;
    const int N = a.n_tok[b];
    const int Nctx = a.ctx_gen ? N : min(N, a.n_prompt[b]);   // tokens the context statistics cover
    const int32_t* seq = a.tokens + (size_t)b * a.max_len;
    for (int i = tid; i < N; i += kThreads) s_tok[i] = seq[i];
    const u64 q = (u64)a.q16, qb = (u64)(65536 - a.q16);
    const int n_max = a.ng.n_max, bits = a.ng.bits;
    __syncthreads();

    for (int j = 0; j < a.k; ++j) {
        const int wlen = N + j;
        const int nsuf = min(n_max - 1, wlen);
        if (tid < nsuf) s_suf[tid] = tid < j ? s_d[j - 1 - tid] : s_tok[N - 1 - (tid - j)];
        if (tid == 0) { s_mmax = 0; s_m = 0; s_T = 0; s_ncorp = 0; s_best = 0; s_x = 0x7FFFFFFF; }
        if (tid <= TASC_MAX_ORDER) s_found[tid] = 0;
        __syncthreads();

        // ---- corpus source: all orders probed at once, the highest hit wins.  Issued first: the probes' global round trips
        // then run under the other waves' context scan
        if (q > 0 && tid < n_max - 1) {
            const int n = n_max - tid;                 // n - 1 context tokens
            if (n - 1 <= nsuf && a.ng.ord[n].ctx != nullptr) {
                u64 lo = 0, hi = 0;
                for (int i = 0; i < n - 1; ++i) tasc_key_put(lo, hi, i, bits, (u32)s_suf[n - 2 - i]);
                TascSlot hit;
                if (probe(a.ng.ord[n].ctx, a.ng.ord[n].ctx_mask, lo, hi, n - 1, hit)) {
                    s_hit[n] = hit;
                    s_found[n] = 1;
                }
            }
        }
        // ---- context source: match length of every successor position p (context ends at p - 1)
        int n_ctx = 0, T_ctx = 0;
        if (qb > 0) {
            int lmax = 0;
            for (int p = 1 + tid; p < Nctx; p += kThreads) {
                int ml = 0;
                while (ml < nsuf && p - 1 - ml >= 0 && s_tok[p - 1 - ml] == s_suf[ml]) ++ml;
                s_ml[p] = (uint8_t)ml;
                lmax = max(lmax, ml);
            }
            if (lmax > 0) atomicMax(&s_mmax, lmax);
            __syncthreads();
            const int mmax = s_mmax;
            // back off from the longest matching context until one has a kept successor
            for (int n = mmax + 1; n >= 2; --n) {
                for (int p = 1 + tid; p < Nctx; p += kThreads)
                    if (s_ml[p] >= n - 1) s_list[atomicAdd(&s_m, 1)] = s_tok[p];
                __syncthreads();
                const int m = s_m;
                for (int e = tid; e < m; e += kThreads) {
                    const int x = s_list[e];
                    int c = 0;
                    for (int f = 0; f < m; ++f) c += s_list[f] == x;
                    s_cnt[e] = (uint16_t)min(c, 65535);
                    if (c >= a.p_min_ctx) atomicAdd(&s_T, 1);
                }
                __syncthreads();
                if (s_T > 0) { n_ctx = n; T_ctx = s_T; break; }
                __syncthreads();
                if (tid == 0) s_m = 0;
                __syncthreads();
            }
        }
        const int m_list = n_ctx ? s_m : 0;

        __syncthreads();
        if (tid == 0) {
            int nc = 0;
            for (int n = n_max; n >= 2 && !nc; --n) nc = s_found[n] ? n : 0;
            s_ncorp = nc;
        }
        __syncthreads();
        const int n_corp = s_ncorp;

        // ---- proposal
        int x;
        if (!n_corp && !n_ctx) {
            x = a.ng.fallback;
        } else if (!n_ctx) {
            x = (int)s_hit[n_corp].b;
        } else {
            const u64 T_corp = n_corp ? s_hit[n_corp].a : 0;
            u64 lo0 = 0, hi0 = 0;
            if (n_corp)
                for (int i = 0; i < n_corp - 1; ++i) tasc_key_put(lo0, hi0, i, bits, (u32)s_suf[n_corp - 2 - i]);
            u64 my_score = 0;
            int my_x = 0x7FFFFFFF;
            for (int e = tid; e < m_list; e += kThreads) {
                const int c = s_cnt[e];
                if (c < a.p_min_ctx) continue;
                const int xe = s_list[e];
                u64 sc;
                if (n_corp) {
                    u64 lo = lo0, hi = hi0;
                    tasc_key_put(lo, hi, n_corp - 1, bits, (u32)xe);
                    TascSlot hit;
                    u64 c_corp = probe(a.ng.ord[n_corp].full, a.ng.ord[n_corp].full_mask, lo, hi, n_corp, hit) ? hit.a : 0;
                    sc = q * c_corp * (u64)T_ctx + qb * (u64)c * T_corp;
                } else {
                    sc = (u64)c;
                }
                if (sc > my_score || (sc == my_score && xe < my_x)) { my_score = sc; my_x = xe; }
            }
            if (n_corp && tid == 0) {
                // the corpus' own best successor: scores at least this even if the context never saw it
                const u64 sc = q * (u64)s_hit[n_corp].c * (u64)T_ctx;
                const int xe = (int)s_hit[n_corp].b;
                if (sc > my_score || (sc == my_score && xe < my_x)) { my_score = sc; my_x = xe; }
            }
            if (my_x != 0x7FFFFFFF) atomicMax(&s_best, my_score);
            __syncthreads();
            if (my_x != 0x7FFFFFFF && my_score == s_best) atomicMin(&s_x, my_x);
            __syncthreads();
            x = s_x;
        }
        __syncthreads();
        if (tid == 0) {
            s_d[j] = x;
            a.drafts[(size_t)b * a.k + j] = x;
        }
        __syncthreads();
    }
}

}  // namespace

extern "C" tasc_status tasc_draft(const tasc_ngram* ng, tasc_session* s, const tasc_spec_params* p, int32_t* drafts,
                                  void* stream) {
    TASC_REQUIRE(ng && s && p && drafts, "draft: null argument");
    TASC_REQUIRE(p->k >= 1 && p->k <= TASC_MAX_K, "draft: k %d outside [1, %d]", p->k, TASC_MAX_K);
    TASC_REQUIRE(p->lambda_q16 >= 0 && p->lambda_q16 <= 65536, "draft: lambda_q16 %d outside [0, 65536]", p->lambda_q16);
    TASC_REQUIRE(p->p_min_ctx >= 1, "draft: p_min_ctx %d < 1", p->p_min_ctx);
    TASC_REQUIRE(ng->view.vocab == s->model->desc.vocab, "draft: table vocabulary %d, model vocabulary %d", ng->view.vocab,
                 s->model->desc.vocab);
    if (!s->prefilled) {
        tasc_set_error("draft: session has no prompt yet");
        return TASC_ESTATE;
    }
    TASC_REQUIRE(s->max_len <= TASC_DRAFT_MAX_LEN, "draft: max_len %d exceeds %d", s->max_len, TASC_DRAFT_MAX_LEN);
    DraftArgs a;
    a.ng = ng->view;
    a.tokens = s->d.tokens;
    a.n_tok = s->d.n_tok;
    a.n_prompt = s->d.n_prompt;
    a.max_len = s->max_len;
    a.k = p->k;
    a.q16 = p->lambda_q16;
    a.p_min_ctx = p->p_min_ctx;
    a.ctx_gen = p->ctx_includes_generated;
    a.drafts = drafts;
    {
        TascProfScope ps(TASC_KC_DRAFT, (hipStream_t)stream);
        k_draft<<<dim3(s->batch), dim3(kThreads), 0, (hipStream_t)stream>>>(a);
    }
    TASC_LAUNCH_CHECK();
    return TASC_OK;
}
