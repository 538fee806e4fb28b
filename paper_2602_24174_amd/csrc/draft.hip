// Draft proposal: k tokens per sequence from the mixture of the corpus drafter and the context
// drafter (paper, section "Proposed Method: TASC-spec":
//     p_mixed(x|c) = lambda p_corp(x|c) + (1 - lambda) p_prompt(x|c),
// each source queried in descending order of n, first match wins, most frequent token if none).
//
// One wave per sequence.  The sequence's committed tokens sit in LDS; the context drafter is
// not a stored table but a scan: for the running suffix, every position of the sequence gets the
// length of its match with the suffix, the longest match gives the context's order, and the tokens
// that follow the matching positions are its successor multiset.  Exact integer scores.
#include "tasc_internal.h"

namespace {

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

// One WAVE per sequence: every exchange between lanes is a ballot, a shuffle or an LDS access of the same wave, so
// the k sequential proposals cross no workgroup barrier.  Per proposal:
//   * corpus source: lanes 0 .. n_max-2 request the first slot of one order each, and the answers are only looked at
//     after the context phase, so the round trip runs under it;
//   * context source: the match length of every position with the running suffix is UPDATED from the previous
//     proposal's (a position matches m + 1 tokens iff the token before it is the one just appended and its predecessor
//     matched m): one compare pass over the sequence compacts the matching positions into a list (ballot + prefix
//     count), everything after that touches list entries only.  The positions of the longest match feed their
//     successors into a hash table in LDS (token -> multiplicity; entries carry a generation number, so the table
//     is never cleared), whose distinct entries are the candidates;
//   * the candidates' corpus counts are requested at EVERY order before the corpus context is known (a second round
//     trip that would otherwise wait for the first), and the ones of the matching order are used;
//   * the argmax over (score, smallest token) is a wave reduction.
constexpr int kHashSlots = 2 * TASC_DRAFT_MAX_LEN;        // more than any sequence has successors

__device__ __forceinline__ u64 wave_max_u64(u64 v) {
    for (int o = 32; o > 0; o >>= 1) {
        const u64 w = __shfl_xor(v, o);
        v = w > v ? w : v;
    }
    return v;
}
__device__ __forceinline__ TascSlot slot_load(const TascSlot* p) {
    const uint4 a = reinterpret_cast<const uint4*>(p)[0], b = reinterpret_cast<const uint4*>(p)[1];
    TascSlot s;
    s.lo = (u64)a.x | ((u64)a.y << 32); s.hi = (u64)a.z | ((u64)a.w << 32);
    s.a = b.x; s.b = b.y; s.c = b.z; s.d = b.w;
    return s;
}
// finishes a probe whose first slot `s` (index idx) has been loaded already
__device__ __forceinline__ bool probe_finish(const TascSlot* __restrict__ tab, u64 mask, u64 lo, u64 hi, u64 idx, TascSlot& s) {
    for (u64 p = 0; p <= mask; ++p) {
        if (s.a == 0) return false;
        if (s.lo == lo && s.hi == hi) return true;
        idx = (idx + 1) & mask;
        s = slot_load(tab + idx);
    }
    return false;
}

__global__ __launch_bounds__(64) void k_draft(DraftArgs a) {
    __shared__ int32_t s_tok[TASC_DRAFT_MAX_LEN];
    __shared__ uint8_t s_ml[TASC_DRAFT_MAX_LEN];          // match length of every position with the suffix (0 outside the list)
    __shared__ uint16_t s_pos[2][TASC_DRAFT_MAX_LEN];     // positions with a match length >= 1, ping-pong
    __shared__ u64 s_tab[kHashSlots];                     // {generation : 16, multiplicity : 16, token : 32}
    __shared__ uint16_t s_dl[TASC_DRAFT_MAX_LEN];         // slots of the distinct successors of the current generation
    __shared__ int32_t s_suf[TASC_MAX_ORDER];             // s_suf[i] = i-th token from the end of the running context
    __shared__ int32_t s_d[TASC_MAX_K];                   // the proposals so far
    __shared__ int s_nd;
    __shared__ TascSlot s_hit[TASC_MAX_ORDER + 1];

    const int b = blockIdx.x, lane = threadIdx.x;
    const u64 lt_mask = (1ull << lane) - 1;
    const int N = a.n_tok[b];
    const int Nctx = a.ctx_gen ? N : min(N, a.n_prompt[b]);   // tokens the context statistics cover
    const int32_t* seq = a.tokens + (size_t)b * a.max_len;
    for (int i0 = 0; i0 < N; i0 += 256) {                  // four loads in flight per lane
        int32_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = seq[min(i0 + 64 * u + lane, N - 1)];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i0 + 64 * u + lane < N) s_tok[i0 + 64 * u + lane] = v[u];
    }
    for (int i = lane; i < kHashSlots; i += 64) s_tab[i] = 0;     // generation 0 = never used
    const u64 q = (u64)a.q16, qb = (u64)(65536 - a.q16);
    const int n_max = a.ng.n_max, bits = a.ng.bits;
    u32 gen = 0;
    int cur = 0, n_list = 0;                               // which half of s_pos is current, and its length
    int x_prev = 0, nsuf_prev = -1;
    __builtin_amdgcn_s_waitcnt(0);
    __builtin_amdgcn_wave_barrier();

    for (int j = 0; j < a.k; ++j) {
        const int wlen = N + j;
        const int nsuf = min(n_max - 1, wlen);
        if (lane < nsuf) s_suf[lane] = lane < j ? s_d[j - 1 - lane] : s_tok[N - 1 - (lane - j)];
        __builtin_amdgcn_s_waitcnt(0);
        __builtin_amdgcn_wave_barrier();

        // ---- corpus source: the first slot of every order is requested now and examined after the context phase
        const int my_n = n_max - lane;                     // lane l probes the contexts of n - 1 = n_max - 1 - l tokens
        const bool c_probe = q > 0 && lane < n_max - 1 && my_n - 1 <= nsuf && a.ng.ord[my_n < 2 ? 2 : my_n].ctx != nullptr;
        u64 c_lo = 0, c_hi = 0, c_idx = 0;
        TascSlot c_slot = {0, 0, 0, 0, 0, 0};
        if (c_probe) {
            for (int i = 0; i < my_n - 1; ++i) tasc_key_put(c_lo, c_hi, i, bits, (u32)s_suf[my_n - 2 - i]);
            c_idx = tasc_hash_key(c_lo, c_hi, my_n - 1) & a.ng.ord[my_n].ctx_mask;
            c_slot = slot_load(a.ng.ord[my_n].ctx + c_idx);
        }

        // ---- context source
        int n_ctx = 0, T_ctx = 0, n_dist = 0;
        if (qb > 0) {
            int lmax = 0;
            const int nxt = cur ^ 1;
            int n_new = 0;
            if (j == 0 || nsuf_prev < n_max - 1) {
                // from scratch (the first proposal; or a context still shorter than n_max - 1: a handful of tokens)
                for (int p0 = 0; p0 < Nctx; p0 += 64) {
                    const int p = p0 + lane;
                    int ml = 0;
                    if (p < Nctx)
                        while (ml < nsuf && p - 1 - ml >= 0 && s_tok[p - 1 - ml] == s_suf[ml]) ++ml;
                    if (p < Nctx) s_ml[p] = (uint8_t)ml;
                    const u64 hit = __ballot(ml > 0);
                    if (ml > 0) s_pos[nxt][n_new + __popcll(hit & lt_mask)] = (uint16_t)p;
                    n_new += __popcll(hit);
                    lmax = max(lmax, ml);
                }
            } else {
                // the positions that follow an occurrence of the token just appended: one compare pass, compacted
                uint8_t* s_val = reinterpret_cast<uint8_t*>(s_dl);        // their new match lengths, parked until all old ones are read
                for (int p0 = 1; p0 < Nctx; p0 += 256) {          // 256 positions per round: all their LDS reads in flight together
                    bool hit1[4];
                    int mlp[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int p = min(p0 + 64 * u + lane, Nctx - 1);
                        hit1[u] = p0 + 64 * u + lane < Nctx && s_tok[p - 1] == x_prev;
                        mlp[u] = (int)s_ml[p - 1];
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int p = p0 + 64 * u + lane;
                        const u64 hit = __ballot(hit1[u]);
                        if (hit1[u]) {
                            const int ml = min(mlp[u] + 1, nsuf);
                            const int at = n_new + __popcll(hit & lt_mask);
                            s_pos[nxt][at] = (uint16_t)p;
                            s_val[at] = (uint8_t)ml;
                            lmax = max(lmax, ml);
                        }
                        n_new += __popcll(hit);
                    }
                }
                __builtin_amdgcn_s_waitcnt(0);
                __builtin_amdgcn_wave_barrier();
                for (int e = lane; e < n_list; e += 64) s_ml[s_pos[cur][e]] = 0;          // the old matches go ...
                __builtin_amdgcn_s_waitcnt(0);
                __builtin_amdgcn_wave_barrier();
                for (int e = lane; e < n_new; e += 64) s_ml[s_pos[nxt][e]] = s_val[e];    // ... the new ones come
            }
            cur = nxt;
            n_list = n_new;
            for (int o = 32; o > 0; o >>= 1) lmax = max(lmax, __shfl_xor(lmax, o));
            __builtin_amdgcn_s_waitcnt(0);
            __builtin_amdgcn_wave_barrier();
            // back off from the longest matching context until one has a kept successor
            for (int n = lmax + 1; n >= 2 && !n_ctx; --n) {
                ++gen;
                if (lane == 0) s_nd = 0;
                __builtin_amdgcn_s_waitcnt(0);
                __builtin_amdgcn_wave_barrier();
                for (int e0 = 0; e0 < n_list; e0 += 64) {
                    const int e = e0 + lane;
                    const int p = e < n_list ? s_pos[cur][e] : 0;
                    const bool in = e < n_list && p >= 1 && s_ml[p] >= n - 1;
                    const u32 key = in ? (u32)s_tok[p] : 0u;
                    const u64 act = __ballot(in);
                    if (!act) continue;
                    // a run of one token (every lane the same successor) is added in one go by the first lane
                    const int first = __ffsll((unsigned long long)act) - 1;
                    const u32 k0 = (u32)__shfl((int)key, first);
                    const bool uniform = __ballot(in && key == k0) == act;
                    const bool me = uniform ? lane == first : in;
                    const u64 add = uniform ? (u64)__popcll(act) : 1ull;
                    if (me) {
                        u32 slot = (u32)(tasc_mix64(key) & (kHashSlots - 1));
                        for (;;) {
                            const u64 w = s_tab[slot];
                            if ((u32)(w >> 48) != gen) {
                                // empty for this generation: claim it
                                const u64 neu = ((u64)gen << 48) | (add << 32) | key;
                                if (atomicCAS(reinterpret_cast<unsigned long long*>(&s_tab[slot]), w, neu) == w) {
                                    s_dl[atomicAdd(&s_nd, 1)] = (uint16_t)slot;
                                    break;
                                }
                                continue;                  // somebody else took it: look at it again
                            }
                            if ((u32)w == key) {
                                atomicAdd(reinterpret_cast<unsigned long long*>(&s_tab[slot]), add << 32);
                                break;
                            }
                            slot = (slot + 1) & (kHashSlots - 1);
                        }
                    }
                }
                __builtin_amdgcn_s_waitcnt(0);
                __builtin_amdgcn_wave_barrier();
                n_dist = s_nd;
                int t = 0;
                for (int e = lane; e < n_dist; e += 64) {
                    const int c = (int)((s_tab[s_dl[e]] >> 32) & 0xFFFFu);
                    if (c >= a.p_min_ctx) t += c;
                }
                for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o);
                if (t > 0) { n_ctx = n; T_ctx = t; }
            }
        }

        // ---- the candidates' corpus counts, requested at every order a corpus context could match (pair = candidate x order)
        const int n_ord = n_max - 1;
        const bool spec = q > 0 && n_ctx && n_dist * n_ord <= 64;
        u64 f_lo = 0, f_hi = 0, f_idx = 0;
        TascSlot f_slot = {0, 0, 0, 0, 0, 0};
        int f_n = 0, f_x = 0, f_c = 0;
        if (spec && lane < n_dist * n_ord) {
            const u64 w = s_tab[s_dl[lane / n_ord]];
            f_x = (int)(u32)w;
            f_c = (int)((w >> 32) & 0xFFFFu);
            f_n = n_max - lane % n_ord;
            if (f_c >= a.p_min_ctx && f_n - 1 <= nsuf && a.ng.ord[f_n].full != nullptr) {
                for (int i = 0; i < f_n - 1; ++i) tasc_key_put(f_lo, f_hi, i, bits, (u32)s_suf[f_n - 2 - i]);
                tasc_key_put(f_lo, f_hi, f_n - 1, bits, (u32)f_x);
                f_idx = tasc_hash_key(f_lo, f_hi, f_n) & a.ng.ord[f_n].full_mask;
                f_slot = slot_load(a.ng.ord[f_n].full + f_idx);
            } else {
                f_n = 0;
            }
        }

        // ---- the corpus context: the highest order whose probe hits
        bool found = false;
        if (c_probe && probe_finish(a.ng.ord[my_n].ctx, a.ng.ord[my_n].ctx_mask, c_lo, c_hi, c_idx, c_slot)) {
            s_hit[my_n] = c_slot;
            found = true;
        }
        const u64 found_mask = __ballot(found);
        const int n_corp = found_mask ? n_max - (__ffsll((unsigned long long)found_mask) - 1) : 0;   // lowest lane = highest order
        __builtin_amdgcn_s_waitcnt(0);
        __builtin_amdgcn_wave_barrier();

        // ---- proposal
        int x;
        if (!n_corp && !n_ctx) {
            x = a.ng.fallback;
        } else if (!n_ctx) {
            x = (int)s_hit[n_corp].b;
        } else {
            const u64 T_corp = n_corp ? s_hit[n_corp].a : 0;
            u64 my_score = 0;
            int my_x = 0x7FFFFFFF;
            if (spec) {
                // one lane per (candidate, order): the lanes of the matching order (or, without a corpus match, of the
                // highest order: one per candidate) score
                const bool scorer = lane < n_dist * n_ord && f_c >= a.p_min_ctx && (n_corp ? (n_max - lane % n_ord) == n_corp : lane % n_ord == 0);
                if (scorer) {
                    u64 sc;
                    if (n_corp) {
                        const u64 c_corp = (f_n == n_corp && probe_finish(a.ng.ord[f_n].full, a.ng.ord[f_n].full_mask, f_lo, f_hi, f_idx, f_slot)) ? f_slot.a : 0;
                        sc = q * c_corp * (u64)T_ctx + qb * (u64)f_c * T_corp;
                    } else {
                        sc = (u64)f_c;
                    }
                    my_score = sc;
                    my_x = f_x;
                }
            } else {
                u64 lo0 = 0, hi0 = 0;
                if (n_corp)
                    for (int i = 0; i < n_corp - 1; ++i) tasc_key_put(lo0, hi0, i, bits, (u32)s_suf[n_corp - 2 - i]);
                for (int e = lane; e < n_dist; e += 64) {
                    const u64 w = s_tab[s_dl[e]];
                    const int c = (int)((w >> 32) & 0xFFFFu);
                    if (c < a.p_min_ctx) continue;
                    const int xe = (int)(u32)w;
                    u64 sc;
                    if (n_corp) {
                        u64 lo = lo0, hi = hi0;
                        tasc_key_put(lo, hi, n_corp - 1, bits, (u32)xe);
                        TascSlot hit;
                        const u64 c_corp = probe(a.ng.ord[n_corp].full, a.ng.ord[n_corp].full_mask, lo, hi, n_corp, hit) ? hit.a : 0;
                        sc = q * c_corp * (u64)T_ctx + qb * (u64)c * T_corp;
                    } else {
                        sc = (u64)c;
                    }
                    if (sc > my_score || (sc == my_score && xe < my_x)) { my_score = sc; my_x = xe; }
                }
            }
            if (n_corp && lane == 63) {
                // the corpus' own best successor: scores at least this even if the context never saw it (merged into
                // whatever the lane holds already)
                const u64 sc = q * (u64)s_hit[n_corp].c * (u64)T_ctx;
                const int xe = (int)s_hit[n_corp].b;
                if (sc > my_score || (sc == my_score && xe < my_x)) { my_score = sc; my_x = xe; }
            }
            const u64 best = wave_max_u64(my_x != 0x7FFFFFFF ? my_score : 0);
            int cand = (my_x != 0x7FFFFFFF && my_score == best) ? my_x : 0x7FFFFFFF;
            for (int o = 32; o > 0; o >>= 1) cand = min(cand, __shfl_xor(cand, o));
            x = cand;
        }
        if (lane == 0) {
            s_d[j] = x;
            a.drafts[(size_t)b * a.k + j] = x;
        }
        x_prev = x;
        nsuf_prev = nsuf;
        __builtin_amdgcn_s_waitcnt(0);
        __builtin_amdgcn_wave_barrier();
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
        k_draft<<<dim3(s->batch), dim3(64), 0, (hipStream_t)stream>>>(a);
    }
    TASC_LAUNCH_CHECK();
    return TASC_OK;
}
