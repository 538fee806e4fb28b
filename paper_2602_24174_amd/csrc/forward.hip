// One target forward over M = batch * nq rows against the paged KV cache, ending (optionally) in the
// LM head with fused bias and argmax.  Used by the prompt forward (nq = chunk length) and by the
// verify step (nq = k + 1; paper, subsection "Speculative Decoding": the drafted tokens are verified
// in parallel via a single forward pass).
#include "tasc_internal.h"
#include "kernels_generic.h"

namespace {

template <typename T>
tasc_status forward_rows_t(const tasc_model* m, tasc_session* s, int nq, int n_sel, float* logits_dbg, hipStream_t st) {
    const tasc_model_desc& c = m->desc;
    const TascSessDev& d = s->d;
    const int M = s->batch * nq;
    const int D = c.d_model, H = c.n_heads, Hkv = c.n_kv_heads, hd = c.head_dim, F = c.d_ffn;
    const int nqkv = (H + 2 * Hkv) * hd, nqo = H * hd;
    KvGeom gm{H, Hkv, hd, nq, s->max_blocks, s->page_elems};
    const float scale = 1.0f / sqrtf((float)hd);

    { TascProfScope ps(TASC_KC_PREPARE, st); k_embed<T><<<dim3(M), dim3(64), 0, st>>>((const T*)m->embed, d.row_tok, D, d.x); }
    TASC_LAUNCH_CHECK();
    for (int l = 0; l < c.n_layers; ++l) {
        const TascLayerW& w = m->layers[l];
        T* kv_layer = (T*)s->kv_pool + (size_t)l * s->kv_layer_stride;
        { TascProfScope ps(TASC_KC_NORM, st); k_rmsnorm<T><<<dim3(M), dim3(64), 0, st>>>(d.x, w.g1, nullptr, D, c.rms_eps, (T*)d.h); }
        { TascProfScope ps(TASC_KC_GEMM_QKV, st); k_gemm_generic<T, EPI_STORE><<<dim3((nqkv + 3) / 4), dim3(256), 0, st>>>((const T*)d.h, (const T*)w.wqkv, M, nqkv, D,
                                                                              d.qkv, nullptr); }
        { TascProfScope ps(TASC_KC_ROPE_KV, st); k_rope_kv<T><<<dim3(M), dim3(256), 0, st>>>(d.qkv, m->rope_cos, m->rope_sin, c.max_pos, d.n_rows, d.pos0, d.block_tab,
                                                  gm, (T*)d.q, kv_layer); }
        { TascProfScope ps(TASC_KC_ATTN, st); k_attn_generic<T><<<dim3(s->batch, H), dim3(256), (size_t)nq * hd * sizeof(float), st>>>(
            (const T*)d.q, kv_layer, d.n_rows, d.pos0, d.block_tab, gm, scale, (T*)d.att); }
        { TascProfScope ps(TASC_KC_GEMM_O, st); k_gemm_generic<T, EPI_RESID><<<dim3((D + 3) / 4), dim3(256), 0, st>>>((const T*)d.att, (const T*)w.wo, M, D, nqo, d.x,
                                                                          nullptr); }
        { TascProfScope ps(TASC_KC_NORM, st); k_rmsnorm<T><<<dim3(M), dim3(64), 0, st>>>(d.x, w.g2, nullptr, D, c.rms_eps, (T*)d.h); }
        { TascProfScope ps(TASC_KC_GEMM_GU, st); k_gemm_generic<T, EPI_SWIGLU><<<dim3((F + 3) / 4), dim3(256), 0, st>>>((const T*)d.h, (const T*)w.wgu, M, F, D, nullptr,
                                                                           (T*)d.act); }
        { TascProfScope ps(TASC_KC_GEMM_D, st); k_gemm_generic<T, EPI_RESID><<<dim3((D + 3) / 4), dim3(256), 0, st>>>((const T*)d.act, (const T*)w.wd, M, D, F, d.x,
                                                                          nullptr); }
        TASC_LAUNCH_CHECK();
    }
    if (n_sel > 0) {
        { TascProfScope ps(TASC_KC_NORM, st); k_rmsnorm<T><<<dim3(n_sel), dim3(64), 0, st>>>(d.x, m->gf, d.sel_rows, D, c.rms_eps, (T*)d.h); }
        BiasCsr bias{m->bias_rowptr, m->bias_col, m->bias_val, m->bias_base};
        { TascProfScope ps(TASC_KC_LMHEAD, st); k_lmhead_generic<T><<<dim3(s->n_strips), dim3(256), 0, st>>>((const T*)d.h, (const T*)m->lm_head, d.sel_tok, n_sel,
                                                                  c.vocab, D, bias, d.part_val, d.part_idx, s->n_strips,
                                                                  logits_dbg); }
        { TascProfScope ps(TASC_KC_ACCEPT, st); k_argmax_reduce<<<dim3(n_sel), dim3(64), 0, st>>>(d.part_val, d.part_idx, s->n_strips, d.amax); }
        TASC_LAUNCH_CHECK();
    }
    return TASC_OK;
}

}  // namespace

tasc_status tasc_forward_rows(const tasc_model* m, tasc_session* s, int32_t nq, int32_t n_sel, float* logits_dbg,
                              hipStream_t st) {
    if (m->desc.dtype == TASC_F32) return forward_rows_t<float>(m, s, nq, n_sel, logits_dbg, st);
    return forward_rows_t<BF16>(m, s, nq, n_sel, logits_dbg, st);
}
