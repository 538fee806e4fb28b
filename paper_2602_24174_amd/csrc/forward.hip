// One target forward over M = batch * nq rows against the paged KV cache, ending (optionally) in the
// LM head with fused bias and argmax.  Used by the prompt forward (nq = chunk length) and by the
// verify step (nq = k + 1; paper, subsection "Speculative Decoding": the drafted tokens are verified
// in parallel via a single forward pass).
//
// Which kernels run depends on the model and the session only (dtype, row count of the call), never on
// data, so plain greedy decoding (k = 0) and speculative decoding of the same session shapes reduce
// every row in the same order.
#include "tasc_internal.h"
#include "kernels_generic.h"
#include "kernels_small.h"
#include "kernels_pipe.h"
#include "kernels_tiled.h"

TascConfig g_tasc_config = {/*small_path*/ 2, /*small_grid*/ 0, /*layer_wgs*/ 0, /*layer_stride*/ 0, /*tiled_path*/ 1, /*xcd_local*/ 1,
                             /*layer_workers*/ 0, /*small_kernel*/ 1, /*pipe_share*/ 1, /*chains*/ 0, /*step_graph*/ 1};
// One-time set-up (kernel attributes, the compute-unit count) is kept per device and done under a lock, so that calls
// from several host threads, or sessions on different devices of one process, each find their own device prepared.
#include <mutex>
namespace {
struct DevState { bool tiled_ready = false, small_ready = false, pipe_ready = false; int cu_count = 0; };
DevState g_dev[16];
std::mutex g_dev_mu;
DevState& dev_state() {
    int dev = 0;
    (void)hipGetDevice(&dev);
    return g_dev[dev & 15];
}
}  // namespace
static u64* g_phase_ts = nullptr;
static int64_t g_phase_ts_cap = 0;

extern "C" tasc_status tasc_profile_phases(uint64_t* device_buf, int64_t capacity) {
    TASC_REQUIRE(capacity >= 0 && (device_buf || capacity == 0), "profile_phases: bad buffer");
    g_phase_ts = (u64*)device_buf;
    g_phase_ts_cap = device_buf ? capacity : 0;
    return TASC_OK;
}

extern "C" tasc_status tasc_config_set(int32_t key, int32_t value) {
    if (key == TASC_CFG_SMALL_PATH) {
        TASC_REQUIRE(value >= 0 && value <= 2, "config_set: small path %d outside [0, 2]", value);
        g_tasc_config.small_path = value;
    } else if (key == TASC_CFG_SMALL_GRID) {
        TASC_REQUIRE(value >= 0 && value <= 4096, "config_set: grid %d outside [0, 4096]", value);
        g_tasc_config.small_grid = value;
    } else if (key == TASC_CFG_TILED_PATH) {
        TASC_REQUIRE(value == 0 || value == 1, "config_set: tiled path %d outside [0, 1]", value);
        g_tasc_config.tiled_path = value;
    } else if (key == TASC_CFG_SMALL_LAYER_WGS) {
        TASC_REQUIRE(value >= 0 && value <= 4096, "config_set: layer workgroups %d outside [0, 4096]", value);
        g_tasc_config.layer_wgs = value;
    } else if (key == TASC_CFG_SMALL_LAYER_STRIDE) {
        TASC_REQUIRE(value >= 0 && value <= 64, "config_set: layer stride %d outside [0, 64]", value);
        g_tasc_config.layer_stride = value;
    } else if (key == TASC_CFG_SMALL_LAYER_WORKERS) {
        TASC_REQUIRE(value >= 0 && value <= 64, "config_set: layer workers %d outside [0, 64]", value);
        g_tasc_config.layer_workers = value;
    } else if (key == TASC_CFG_SMALL_KERNEL) {
        TASC_REQUIRE(value == 0 || value == 1, "config_set: small kernel %d outside [0, 1]", value);
        g_tasc_config.small_kernel = value;
    } else if (key == TASC_CFG_STEP_GRAPH) {
        TASC_REQUIRE(value == 0 || value == 1, "config_set: step graph %d outside [0, 1]", value);
        g_tasc_config.step_graph = value;
    } else if (key == TASC_CFG_CHAINS) {
        TASC_REQUIRE(value >= 0 && value <= TASC_MAX_CHAINS, "config_set: chains %d outside [0, %d]", value, TASC_MAX_CHAINS);
        g_tasc_config.chains = value;
    } else if (key == TASC_CFG_PIPE_SHARE) {
        TASC_REQUIRE(value >= 1 && value <= 3, "config_set: pipeline share %d outside [1, 3]", value);
        g_tasc_config.pipe_share = value;
    } else if (key == TASC_CFG_SMALL_XCD_LOCAL) {
        TASC_REQUIRE(value == 0 || value == 1, "config_set: XCD-local switch %d outside [0, 1]", value);
        g_tasc_config.xcd_local = value;
    } else {
        tasc_set_error("config_set: unknown key %d", key);
        return TASC_EINVAL;
    }
    return TASC_OK;
}

namespace {

#define PROF(cls) TascProfScope _ps(cls, st)

template <typename T>
tasc_status forward_generic(const tasc_model* m, tasc_session* s, int nq, int n_sel, float* logits_dbg, hipStream_t st) {
    const tasc_model_desc& c = m->desc;
    const TascSessDev& d = s->d;
    const int M = s->batch * nq;
    const int D = c.d_model, H = c.n_heads, Hkv = c.n_kv_heads, hd = c.head_dim, F = c.d_ffn;
    const int nqkv = (H + 2 * Hkv) * hd, nqo = H * hd;
    KvGeom gm{H, Hkv, hd, nq, s->max_blocks, s->page_elems};
    const float scale = 1.0f / sqrtf((float)hd);
    {
        PROF(TASC_KC_PREPARE);
        k_embed<T><<<dim3(M), dim3(64), 0, st>>>((const T*)m->embed, d.row_tok, D, d.x);
    }
    TASC_LAUNCH_CHECK();
    for (int l = 0; l < c.n_layers; ++l) {
        const TascLayerW& w = m->layers[l];
        T* kv_layer = (T*)s->kv_pool + (size_t)l * s->kv_layer_stride;
        {
            PROF(TASC_KC_NORM);
            k_rmsnorm<T><<<dim3(M), dim3(64), 0, st>>>(d.x, w.g1, nullptr, D, c.rms_eps, (T*)d.h);
        }
        {
            PROF(TASC_KC_GEMM_QKV);
            k_gemm_generic<T, EPI_STORE><<<dim3((nqkv + 3) / 4), dim3(256), 0, st>>>((const T*)d.h, (const T*)w.wqkv, M, nqkv, D,
                                                                                  d.qkv, nullptr);
        }
        {
            PROF(TASC_KC_ROPE_KV);
            k_rope_kv<T><<<dim3(M), dim3(256), 0, st>>>(d.qkv, m->rope_cos, m->rope_sin, c.max_pos, d.n_rows, d.pos0, d.block_tab,
                                                      gm, (T*)d.q, kv_layer);
        }
        {
            PROF(TASC_KC_ATTN);
            k_attn_generic<T><<<dim3(s->batch, H), dim3(256), (size_t)nq * hd * sizeof(float), st>>>(
                (const T*)d.q, kv_layer, d.n_rows, d.pos0, d.block_tab, gm, scale, (T*)d.att);
        }
        {
            PROF(TASC_KC_GEMM_O);
            k_gemm_generic<T, EPI_RESID><<<dim3((D + 3) / 4), dim3(256), 0, st>>>((const T*)d.att, (const T*)w.wo, M, D, nqo, d.x,
                                                                              nullptr);
        }
        {
            PROF(TASC_KC_NORM);
            k_rmsnorm<T><<<dim3(M), dim3(64), 0, st>>>(d.x, w.g2, nullptr, D, c.rms_eps, (T*)d.h);
        }
        {
            PROF(TASC_KC_GEMM_GU);
            k_gemm_generic<T, EPI_SWIGLU><<<dim3((F + 3) / 4), dim3(256), 0, st>>>((const T*)d.h, (const T*)w.wgu, M, F, D, nullptr,
                                                                               (T*)d.act);
        }
        {
            PROF(TASC_KC_GEMM_D);
            k_gemm_generic<T, EPI_RESID><<<dim3((D + 3) / 4), dim3(256), 0, st>>>((const T*)d.act, (const T*)w.wd, M, D, F, d.x,
                                                                              nullptr);
        }
        TASC_LAUNCH_CHECK();
    }
    if (n_sel > 0) {
        {
            PROF(TASC_KC_NORM);
            k_rmsnorm<T><<<dim3(n_sel), dim3(64), 0, st>>>(d.x, m->gf, d.sel_rows, D, c.rms_eps, (T*)d.h);
        }
        BiasCsr bias{m->bias_rowptr, m->bias_col, m->bias_val, m->bias_base};
        {
            PROF(TASC_KC_LMHEAD);
            k_lmhead_generic<T><<<dim3(s->n_strips), dim3(256), 0, st>>>((const T*)d.h, (const T*)m->lm_head, d.sel_tok, n_sel,
                                                                      c.vocab, D, bias, d.part_val, d.part_idx, s->n_strips,
                                                                      logits_dbg);
        }
        {
            PROF(TASC_KC_ACCEPT);
            k_argmax_reduce<<<dim3(n_sel), dim3(64), 0, st>>>(d.part_val, d.part_idx, s->n_strips, d.amax);
        }
        TASC_LAUNCH_CHECK();
    }
    return TASC_OK;
}

// the LDS-tiled MFMA kernels serve bf16 forwards of any row count with these shapes
bool tiled_path_fits(const tasc_model_desc& c) {
    return c.dtype == TASC_BF16 && c.d_model % 64 == 0 && (c.n_heads * c.head_dim) % 64 == 0 && c.d_ffn % 64 == 0 &&
           (c.head_dim == 32 || c.head_dim == 64 || c.head_dim == 128);
}


// tile shapes: 128 x 128 on 4 waves, and 256 x 256 on 8 waves for row counts where the GEMMs are MFMA-bound.
// Both reduce every output element over k in the same order, so the choice may depend on the row count.
#define TILE_SMALL 128, 128, 2, 2
#define TILE_LARGE 256, 256, 2, 4
#define TILE_NARROW 64, 128, 1, 4      // few rows and a narrow output: twice the workgroups of the small tile
#define TILE_MID 256, 192, 4, 2        // 192 rows per tile where that leaves fewer padded rows than 256 (576 = 3 x 192)
constexpr int kLargeTileRows = 384;

template <int EPI>
tasc_status tiled_attrs() {
    TASC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_gemm_tiled<EPI, TILE_SMALL>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 TG_LDS_BYTES(128, 128)));
    TASC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_gemm_tiled<EPI, TILE_LARGE>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 TG_LDS_BYTES(256, 256)));
    TASC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_gemm_tiled<EPI, TILE_MID>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 TG_LDS_BYTES(256, 192)));
    if constexpr (EPI != TEPI_LMHEAD)
        TASC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_gemm_tiled<EPI, TILE_NARROW>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     TG_LDS_BYTES(64, 128)));
    return TASC_OK;
}

// launches out = epilogue(A W^T) with the tile shape that suits M; `slices` > 1 only for TEPI_PARTIAL
template <int EPI>
void launch_gemm(const BF16* A, const void* Wm, int M, int N, int K, float* outf, BF16* outb, const LmEpi& lm, int slices,
                 hipStream_t st, const RopeEpi& rp = RopeEpi{}) {
    // large tiles need enough of them to fill the chip: narrow outputs stay on the small tile (the k order, and so
    // every row's result, is the same for both shapes)
    const long large_wgs = (long)((M + 255) / 256) * ((N + 255) / 256) * slices;
    // ... and a very wide output (the LM head) takes them from 129 rows on: one row tile then reads every weight tile
    // once, and the activations are re-read per 256 instead of per 128 output features
    if ((M >= kLargeTileRows && large_wgs >= 128) || (M > 128 && large_wgs >= 512)) {
        // 192-row tiles where they cover the rows with less padding and no more tiles (the tile shape never changes a
        // row's result)
        const int mt256 = (M + 255) / 256, mt192 = (M + 191) / 192;
        if (mt192 <= mt256 && mt192 * 192 < mt256 * 256) {
            dim3 g((unsigned)(mt192 * ((N + 255) / 256)), (unsigned)slices);
            k_gemm_tiled<EPI, TILE_MID><<<g, dim3(512), TG_LDS_BYTES(256, 192), st>>>(A, (const BF16*)Wm, M, N, K, outf, outb, lm, rp);
            return;
        }
        dim3 g((unsigned)(mt256 * ((N + 255) / 256)), (unsigned)slices);
        k_gemm_tiled<EPI, TILE_LARGE><<<g, dim3(512), TG_LDS_BYTES(256, 256), st>>>(A, (const BF16*)Wm, M, N, K, outf, outb, lm, rp);
    } else {
        const long small_wgs = (long)((M + 127) / 128) * ((N + 127) / 128) * slices;
        if constexpr (EPI != TEPI_LMHEAD) {
            // (the rotation epilogue needs whole heads inside a tile)
            if (small_wgs <= 128 && !(EPI == TEPI_ROPE && rp.gm.hd > 64)) {     // half of the compute units idle: halve the tile's width (a workgroup each, still)
                dim3 g((unsigned)(((M + 127) / 128) * ((N + 63) / 64)), (unsigned)slices);
                k_gemm_tiled<EPI, TILE_NARROW><<<g, dim3(256), TG_LDS_BYTES(64, 128), st>>>(A, (const BF16*)Wm, M, N, K, outf, outb, lm, rp);
                return;
            }
        }
        dim3 g((unsigned)(((M + 127) / 128) * ((N + 127) / 128)), (unsigned)slices);
        k_gemm_tiled<EPI, TILE_SMALL><<<g, dim3(256), TG_LDS_BYTES(128, 128), st>>>(A, (const BF16*)Wm, M, N, K, outf, outb, lm, rp);
    }
}

tasc_status tiled_ready() {
    std::lock_guard<std::mutex> lock(g_dev_mu);
    DevState& ds = dev_state();
    if (ds.tiled_ready) return TASC_OK;
    tasc_status rc;
    if ((rc = tiled_attrs<TEPI_STORE>()) != TASC_OK) return rc;
    if ((rc = tiled_attrs<TEPI_RESID>()) != TASC_OK) return rc;
    if ((rc = tiled_attrs<TEPI_SWIGLU>()) != TASC_OK) return rc;
    if ((rc = tiled_attrs<TEPI_LMHEAD>()) != TASC_OK) return rc;
    if ((rc = tiled_attrs<TEPI_PARTIAL>()) != TASC_OK) return rc;
    if ((rc = tiled_attrs<TEPI_ROPE>()) != TASC_OK) return rc;
    TASC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_attn_staged<2>), hipFuncAttributeMaxDynamicSharedMemorySize, TA_LDS_BYTES(64) + 4 * TA_MAX_BLOCKS));
    TASC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_attn_staged<4>), hipFuncAttributeMaxDynamicSharedMemorySize, TA_LDS_BYTES(128) + 4 * TA_MAX_BLOCKS));
    ds.tiled_ready = true;
    return TASC_OK;
}


// how many ranges of sequences run the layers side by side when the caller leaves the choice to the library
int tiled_auto_chains(const tasc_model_desc& c, int batch, int nq) {
    (void)c; (void)batch; (void)nq;
    return 1;
}

tasc_status forward_tiled(const tasc_model* m, tasc_session* s, int nq, int n_sel, float* logits_dbg, bool decode, hipStream_t st) {
    const tasc_model_desc& c = m->desc;
    const TascSessDev& d = s->d;
    {
        const tasc_status rc = tiled_ready();
        if (rc != TASC_OK) return rc;
    }
    const int M_all = s->batch * nq;
    const int D = c.d_model, H = c.n_heads, Hkv = c.n_kv_heads, hd = c.head_dim, F = c.d_ffn;
    const int nqkv = (H + 2 * Hkv) * hd, nqo = H * hd;
    KvGeom gm{H, Hkv, hd, nq, s->max_blocks, s->page_elems};
    LmEpi none{};
    // Narrow outputs (few column tiles) are computed in k-slices.  The slice count fixes the order in which a row's
    // products are added, so it must be the same for every DECODE forward of a session (a greedy step and a verify step
    // of one session differ in their row count, and speculative decoding must reproduce greedy decoding bit for bit): it
    // depends on N, K and the session's batch only, never on the rows of the call; rows_ref = 5 rows per sequence
    // stands for the verify steps the session is sized for.  A prompt forward is the same computation in the
    // speculative and in the greedy run whatever its slice count, so it takes the count that suits its own rows (its
    // chunks of batch x max_rows rows fill the chip without slices, and every slice is a pass over rows x N partial sums).
    const int rows_ref = decode ? s->batch * 5 : s->batch * nq;
    auto slices = [&](int N, int K) {
        const int n_nt = (N + 127) / 128, nk = K / TG_BK;
        if (n_nt >= 32) return 1;
        // many sequences, short k: the small tiles of one slice already fill the chip, and every slice would cost a
        // pass over rows x N partial sums
        if (nk <= 40 && n_nt * ((rows_ref + 127) / 128) >= 128) return 1;
        int ks;
        if (rows_ref >= kLargeTileRows && nk > 40) {
            // long k on large tiles: as many slices as fit the compute units in one round
            const int tiles = ((rows_ref + 255) / 256) * ((N + 255) / 256);
            ks = 256 / tiles;
        } else {
            // few rows: one slice per 12 k-steps, or enough for about 24 (column tile, slice) pairs if that is more
            // (measured on the qkv / output / down projections of the 0.5B and 1.5B shapes)
            ks = nk / 12 > (24 + n_nt - 1) / n_nt ? nk / 12 : (24 + n_nt - 1) / n_nt;
        }
        // beyond two 128-row tiles every slice's pass over rows x N partial sums costs more than the shorter k loop
        // gains (the 1.5B shape's down projection in the step: 4 slices 4.40 ms per verify step, 8 slices 4.52 ms)
        if (rows_ref > 256 && rows_ref < kLargeTileRows && ks > 4) ks = 4;
        ks = ks < nk / 4 ? ks : nk / 4;                       // slices of at least 4 k-steps
        ks = ks < TG_MAX_SLICES ? ks : TG_MAX_SLICES;
        return ks < 1 ? 1 : ks;
    };
    int att_chunks = 512 / (s->batch * Hkv);          // two workgroups per compute unit in one round,
    att_chunks = att_chunks < 1 ? 1 : (att_chunks > 4 ? 4 : att_chunks);   // but no more than 4 partial results to merge
    {
        PROF(TASC_KC_PREPARE);
        k_embed<BF16><<<dim3(M_all), dim3(64), 0, st>>>((const BF16*)m->embed, d.row_tok, D, d.x);
    }
    TASC_LAUNCH_CHECK();

    // The layers of sequences [b0, b0 + nb) on stream `st`: every kernel below computes a row from that row's own data
    // (and its sequence's cache), in an order fixed by the session, so the layers may run for several ranges of
    // sequences side by side ("chains", each on a stream of its own with its own share of every buffer) without
    // changing a bit of any row.
    auto run_layers = [&](int b0, int nb, hipStream_t st) -> tasc_status {
        const int M = nb * nq;
        const size_t r0 = (size_t)b0 * nq;
        float* const x = d.x + r0 * D;
        BF16* const h = (BF16*)d.h + r0 * D;
        BF16* const q = (BF16*)d.q + r0 * nqo;
        BF16* const att = (BF16*)d.att + r0 * nqo;
        BF16* const act = (BF16*)d.act + r0 * F;
        float* const part = d.att_part + r0 * 8 * (size_t)(nqkv > D ? nqkv : D);   // the scratch is sized per row
        const int32_t* const n_rows = d.n_rows + b0;
        const int32_t* const pos0 = d.pos0 + b0;
        const int32_t* const block_tab = d.block_tab + (size_t)b0 * s->max_blocks;
        // out (+)= A W^T through k-slices and the ordered reduction.  With `norm_g` the RMSNorm of the updated rows (gain
        // norm_g, into h) is fused into the reduction; returns false if the caller still has to run it (no slices).
        auto gemm_sliced = [&](const BF16* A, const void* Wm, int N, int K, float* out, bool resid, const float* norm_g) {
            const int ks = slices(N, K);
            if (ks == 1) {
                if (resid) launch_gemm<TEPI_RESID>(A, Wm, M, N, K, out, nullptr, none, 1, st);
                else launch_gemm<TEPI_STORE>(A, Wm, M, N, K, out, nullptr, none, 1, st);
                return false;
            }
            launch_gemm<TEPI_PARTIAL>(A, Wm, M, N, K, part, nullptr, none, ks, st);
            const size_t mn = (size_t)M * N;
            if (resid && norm_g && N == D && D <= RRN_MAX_D) {
                bool fused = true;
                switch (ks) {
#define RRN_CASE(NS) case NS: k_reduce_resid_norm<NS><<<dim3(M), dim3(256), 0, st>>>(part, mn, out, norm_g, D, c.rms_eps, h); break;
                    RRN_CASE(2) RRN_CASE(3) RRN_CASE(4) RRN_CASE(5) RRN_CASE(6) RRN_CASE(7) RRN_CASE(8)
#undef RRN_CASE
                    default: fused = false;
                }
                if (fused) return true;
            }
            const unsigned blocks = (unsigned)((mn / 4 + 255) / 256);
            if (resid) k_splitk_reduce<true><<<dim3(blocks), dim3(256), 0, st>>>(part, ks, mn, out);
            else k_splitk_reduce<false><<<dim3(blocks), dim3(256), 0, st>>>(part, ks, mn, out);
            return false;
        };
        const int rows_pass = 32;
        const dim3 attn_grid(nb * Hkv, (nq * (H / Hkv) + rows_pass - 1) / rows_pass);
        bool h_ready = false;                 // h already holds the layer's normalised input
        for (int l = 0; l < c.n_layers; ++l) {
            const TascLayerW& w = m->layers[l];
            BF16* kv_layer = (BF16*)s->kv_pool + (size_t)l * s->kv_layer_stride;
            if (!h_ready) {
                PROF(TASC_KC_NORM);
                if (D <= RRN_MAX_D) k_rmsnorm_row<<<dim3(M), dim3(256), 0, st>>>(x, w.g1, D, c.rms_eps, h);
                else k_rmsnorm<BF16><<<dim3(M), dim3(64), 0, st>>>(x, w.g1, nullptr, D, c.rms_eps, h);
            }
            const int ks_qkv = slices(nqkv, D);
            {
                // one slice: rotation and cache append ride in the projection's epilogue
                PROF(TASC_KC_GEMM_QKV);
                if (ks_qkv == 1)
                    launch_gemm<TEPI_ROPE>(h, w.wqkv, M, nqkv, D, nullptr, q, none, 1, st,
                                           RopeEpi{m->rope_cos, m->rope_sin, n_rows, pos0, block_tab, kv_layer, gm, c.max_pos});
                else launch_gemm<TEPI_PARTIAL>(h, w.wqkv, M, nqkv, D, part, nullptr, none, ks_qkv, st);
            }
            if (ks_qkv > 1) {
                // the k-slices of a split projection are added inside the rotation kernel (same order as the reduction kernel)
                PROF(TASC_KC_ROPE_KV);
                k_rope_kv<BF16><<<dim3(M), dim3(256), 0, st>>>(part, m->rope_cos, m->rope_sin, c.max_pos, n_rows,
                                                             pos0, block_tab, gm, q, kv_layer, ks_qkv, (size_t)M * nqkv);
            }
            {
                PROF(TASC_KC_ATTN);
                AttnArgs aa{q, att, kv_layer, n_rows, pos0, block_tab, nb, nq, H, Hkv,
                            s->max_blocks, s->page_elems, 1.0f / sqrtf((float)hd)};
                if (hd == 32 || s->max_blocks > TA_MAX_BLOCKS) {
                    if (hd == 64) k_attn_tiled<2><<<attn_grid, dim3(SMALL_THREADS), 0, st>>>(aa);
                    else if (hd == 128) k_attn_tiled<4><<<attn_grid, dim3(SMALL_THREADS), 0, st>>>(aa);
                    else k_attn_tiled<1><<<attn_grid, dim3(SMALL_THREADS), 0, st>>>(aa);
                } else {
                    // keys and values staged in LDS, 64 rows per pass; the key tiles are dealt to att_chunks workgroups, a
                    // number fixed by the session's batch (it sets the order in which a row's keys are added)
                    const size_t rows_all = (size_t)M;
                    AttnStagedArgs sa{aa, part, part + (size_t)att_chunks * rows_all * H * hd, att_chunks};
                    const dim3 grid(nb * Hkv, (nq * (H / Hkv) + 63) / 64, att_chunks);
                    if (hd == 64) k_attn_staged<2><<<grid, dim3(SMALL_THREADS), TA_LDS_BYTES(64) + 4 * s->max_blocks, st>>>(sa);
                    else k_attn_staged<4><<<grid, dim3(SMALL_THREADS), TA_LDS_BYTES(128) + 4 * s->max_blocks, st>>>(sa);
                    if (att_chunks > 1) {
                        const size_t n = rows_all * H * hd / 4;
                        k_attn_merge<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>(sa.part_o, sa.part_ml, att_chunks, rows_all, H, hd, att);
                    }
                }
            }
            bool normed;
            {
                PROF(TASC_KC_GEMM_O);
                normed = gemm_sliced(att, w.wo, D, nqo, x, true, w.g2);
            }
            if (!normed) {
                PROF(TASC_KC_NORM);
                if (D <= RRN_MAX_D) k_rmsnorm_row<<<dim3(M), dim3(256), 0, st>>>(x, w.g2, D, c.rms_eps, h);
                else k_rmsnorm<BF16><<<dim3(M), dim3(64), 0, st>>>(x, w.g2, nullptr, D, c.rms_eps, h);
            }
            {
                PROF(TASC_KC_GEMM_GU);
                launch_gemm<TEPI_SWIGLU>(h, w.wgu, M, 2 * F, D, nullptr, act, none, 1, st);
            }
            {
                // the next layer's first RMSNorm rides on this reduction
                PROF(TASC_KC_GEMM_D);
                h_ready = gemm_sliced(act, w.wd, D, F, x, true, l + 1 < c.n_layers ? m->layers[l + 1].g1 : nullptr);
            }
            TASC_LAUNCH_CHECK();
        }
        return TASC_OK;
    };

    // chains: few rows leave the layer kernels short of workgroups and bound by their own start-up and dependent
    // memory round trips; ranges of sequences that run side by side fill the compute units.  Each reads the weights
    // again (from the caches when the chains keep pace), so the count stays small.
    const int chains = tasc_forward_chains(m, s, nq);
    if (chains <= 1) {
        const tasc_status rc = run_layers(0, s->batch, st);
        if (rc != TASC_OK) return rc;
    } else {
        TASC_HIP(hipEventRecord(s->chain_fork, st));
        for (int ch = 0; ch < chains; ++ch) {
            const int b0 = (int)((long)s->batch * ch / chains), b1 = (int)((long)s->batch * (ch + 1) / chains);
            hipStream_t cs = ch == 0 ? st : s->chain_st[ch - 1];
            if (ch > 0) TASC_HIP(hipStreamWaitEvent(cs, s->chain_fork, 0));
            const tasc_status rc = run_layers(b0, b1 - b0, cs);
            if (rc != TASC_OK) return rc;
            if (ch > 0) {
                TASC_HIP(hipEventRecord(s->chain_join[ch - 1], cs));
                TASC_HIP(hipStreamWaitEvent(st, s->chain_join[ch - 1], 0));
            }
        }
    }
    if (n_sel > 0) {
        {
            PROF(TASC_KC_NORM);
            k_rmsnorm<BF16><<<dim3(n_sel), dim3(64), 0, st>>>(d.x, m->gf, d.sel_rows, D, c.rms_eps, (BF16*)d.h);
        }
        LmEpi lm{BiasCsr{m->bias_rowptr, m->bias_col, m->bias_val, m->bias_base}, d.sel_tok, d.bias_ptr, d.part_val, d.part_idx,
                 logits_dbg, s->n_strips};
        {
            PROF(TASC_KC_LMHEAD);
            if (m->bias_rowptr) {
                const int n = n_sel * (s->n_strips + 1);
                k_bias_ptr<<<dim3((n + 255) / 256), dim3(256), 0, st>>>(lm.bias, d.sel_tok, n_sel, s->n_strips, d.bias_ptr);
            }
            launch_gemm<TEPI_LMHEAD>((const BF16*)d.h, m->lm_head, n_sel, c.vocab, D, nullptr, nullptr, lm, 1, st);
        }
        {
            PROF(TASC_KC_ACCEPT);
            k_argmax_reduce<<<dim3(n_sel), dim3(64), 0, st>>>(d.part_val, d.part_idx, s->n_strips, d.amax);
        }
        TASC_LAUNCH_CHECK();
    }
    return TASC_OK;
}

// the fused small-batch kernel serves a bf16 forward of at most 16 rows with these shapes
bool small_path_fits(const tasc_model* m, int batch, int nq, int max_blocks) {
    const tasc_model_desc& c = m->desc;
    return m->lm_head_f != nullptr && c.dtype == TASC_BF16 && batch * nq <= SMALL_ROWS && c.n_layers <= SMALL_MAX_LAYERS && batch * max_blocks <= SMALL_MAX_BT && c.d_model <= SMALL_KC && c.d_model % 32 == 0 &&
           (c.head_dim == 32 || c.head_dim == 64 || c.head_dim == 128) && c.d_ffn % 32 == 0 && c.vocab >= 16 &&
           (nq * (c.n_heads / c.n_kv_heads)) >= 1;
}


tasc_status forward_small(const tasc_model* m, tasc_session* s, int nq, int n_sel, float* logits_dbg, TascVerifyTail* tail,
                          hipStream_t st) {
    const tasc_model_desc& c = m->desc;
    const TascSessDev& d = s->d;
    DevState& ds = dev_state();
    if (std::lock_guard<std::mutex> lock(g_dev_mu); !ds.small_ready) {
        int dev = 0, cus = 0;
        TASC_HIP(hipGetDevice(&dev));
        TASC_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        int per_cu = 0;
        TASC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_small_step<1>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     SMALL_LDS_BYTES));
        TASC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_small_step<2>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     SMALL_LDS_BYTES));
        TASC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_small_step<4>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     SMALL_LDS_BYTES));
        TASC_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_small_step<4>, SMALL_THREADS, SMALL_LDS_BYTES));
        if (cus < 1 || per_cu < 1) {
            tasc_set_error("forward: the persistent kernel does not fit the device (%d compute units, %d blocks each)", cus, per_cu);
            return TASC_EHIP;
        }
        ds.cu_count = cus;
        ds.small_ready = true;
    }
    SmallArgs a;
    a.layers = m->d_layers;
    a.embed = (const BF16*)m->embed;
    a.lm_head = (const BF16*)m->lm_head_f;
    a.gf = m->gf;
    a.rope_cos = m->rope_cos;
    a.rope_sin = m->rope_sin;
    a.bias = BiasCsr{m->bias_rowptr, m->bias_col, m->bias_val, m->bias_base};
    a.n_layers = c.n_layers; a.D = c.d_model; a.H = c.n_heads; a.Hkv = c.n_kv_heads; a.hd = c.head_dim; a.F = c.d_ffn;
    a.V = c.vocab; a.max_pos = c.max_pos; a.eps = c.rms_eps; a.scale = 1.0f / sqrtf((float)c.head_dim);
    a.kv_pool = (BF16*)s->kv_pool; a.kv_layer_stride = s->kv_layer_stride; a.page_elems = s->page_elems;
    a.B = s->batch; a.nq = nq; a.M = s->batch * nq; a.max_blocks = s->max_blocks; a.max_len = s->max_len;
    a.n_strips = s->n_strips; a.max_new = s->max_new;
    a.row_tok = d.row_tok; a.n_rows = d.n_rows; a.pos0 = d.pos0; a.block_tab = d.block_tab; a.sel_rows = d.sel_rows;
    a.sel_tok = d.sel_tok; a.n_sel = n_sel;
    {
        const TascSmallWs w = tasc_small_ws_layout(c);
        a.x = (float*)(d.small_ws + w.x_off); a.x_stride = w.x_stride;
        a.q = (BF16*)(d.small_ws + w.q_off); a.att = (BF16*)(d.small_ws + w.att_off); a.q_stride = w.q_stride;
        a.act = (BF16*)(d.small_ws + w.act_off); a.act_stride = w.act_stride;
    }
    a.part_val = d.part_val; a.part_idx = d.part_idx; a.amax = d.amax; a.logits_dbg = logits_dbg;
    a.k = tail ? tail->k : -1;
    a.drafts = tail ? tail->drafts : nullptr;
    a.tokens = d.tokens; a.n_tok = d.n_tok; a.cached = d.cached; a.n_emit = d.n_emit; a.counters = d.counters;
    a.accept_len = tail ? tail->accept_len : nullptr;
    a.emitted = tail ? tail->emitted : nullptr;
    a.trace_step = tail ? tail->trace_step : nullptr;
    a.bar_flags = (u32*)&d.counters[TASC_CTR_FLAGS];
    a.barb_counter = &d.counters[TASC_CTR_BARB];
    a.bar_error = (u32*)&d.counters[TASC_CTR_BAR_ERR];
    a.xcc_mask = (u32*)&d.counters[TASC_CTR_XCC];
    a.xcd_local = g_tasc_config.xcd_local;
    a.bias_ptr = d.bias_ptr;
    const int n_phases = 3 + 5 * c.n_layers, n_lg_phases = 1 + 5 * c.n_layers;
    a.phase_ts = g_phase_ts;
    a.phase_ts_wgs = g_phase_ts ? (int32_t)(g_phase_ts_cap / (2 * (int64_t)n_phases)) : 0;
    const int last = n_sel > 0 ? n_phases : n_lg_phases;   // without LM-head rows the step ends after the last layer
    int grid = g_tasc_config.small_grid > 0 ? g_tasc_config.small_grid : ds.cu_count;
    grid = grid < ds.cu_count ? grid : ds.cu_count;            // every workgroup must be resident: at most one per compute unit
    // Layer group.  The dispatcher deals workgroup ids round-robin over the 8 XCDs, so by default the group is
    // every 8th workgroup, 32 of them: one XCD's worth, which lets the 150 latency-bound layer phases hand
    // their activations over through that XCD's L2 (the kernel checks where it really runs and falls back
    // to agent-scope barriers otherwise).  With XCD-local barriers off, or a grid too small for that, the
    // group is the first 48 workgroups, spread over all XCDs.  The LM head always uses the whole grid.
    const bool one_xcd = g_tasc_config.xcd_local != 0 && g_tasc_config.small_path == 2 && grid >= 8 * 32;
    int stride = g_tasc_config.layer_stride > 0 ? g_tasc_config.layer_stride : (one_xcd ? 8 : 1);
    int lg = g_tasc_config.layer_wgs > 0 ? g_tasc_config.layer_wgs : (one_xcd && g_tasc_config.layer_stride <= 0 ? 32 : 48);
    if (stride > grid) stride = grid;
    if (lg > (grid + stride - 1) / stride) lg = (grid + stride - 1) / stride;
    if (lg > SMALL_MAX_GROUP) lg = SMALL_MAX_GROUP;
    a.lg_stride = stride;
    a.lg_count = lg;
    a.lg_workers = g_tasc_config.layer_workers > 0 ? g_tasc_config.layer_workers : lg;
    a.bar_epoch = s->bar_epoch;
    a.barb_base = s->barb_base;
    s->ll_armed = false;       // this kernel writes the first copy of the buffers the pipeline kernel expects untouched
    PROF(TASC_KC_LAYERS);
    auto launch = [&](int p0, int p1) {
        if (c.head_dim == 32) k_small_step<1><<<dim3(grid), dim3(SMALL_THREADS), SMALL_LDS_BYTES, st>>>(a, p0, p1);
        else if (c.head_dim == 64) k_small_step<2><<<dim3(grid), dim3(SMALL_THREADS), SMALL_LDS_BYTES, st>>>(a, p0, p1);
        else k_small_step<4><<<dim3(grid), dim3(SMALL_THREADS), SMALL_LDS_BYTES, st>>>(a, p0, p1);
    };
    if (g_tasc_config.small_path == 2) {
        launch(0, last);
        s->bar_epoch += (u32)(n_lg_phases - 1);
        s->barb_base += (u64)(last - n_lg_phases) * grid;
    } else {
        for (int ph = 0; ph < last; ++ph) {
            // a launch of one phase crosses no barrier
            launch(ph, ph + 1);
        }
    }
    TASC_LAUNCH_CHECK();
    if (tail) tail->done = n_sel > 0;
    return TASC_OK;
}

// ---------------------------------------------------------------- the spatial-pipeline kernel
__global__ void k_fill_sentinel(u64* p, size_t units16) {
    for (size_t u = (size_t)blockIdx.x * blockDim.x + threadIdx.x; u < units16; u += (size_t)gridDim.x * blockDim.x) {
        p[2 * u] = ~0ull;
        p[2 * u + 1] = ~0ull;
    }
}

// Deals the workgroups of the grid to the five roles: every role gets enough of them that a workgroup's share of the
// role's items (16-feature tiles, or (sequence, head) pairs) stays within what one pass holds in registers.  Returns
// false if the grid is too small for the model.
bool pipe_roles(const tasc_model_desc& c, int batch, int grid, int32_t (&base)[PIPE_N_ROLES], int32_t (&count)[PIPE_N_ROLES]) {
    const bool wide = c.d_model > 768;                     // 6 fragments per tile row and lane: one item per pass
    const int items[PIPE_N_ROLES] = {(c.n_heads + 2 * c.n_kv_heads) * (c.head_dim / 32), batch * c.n_heads, c.d_model / 16,
                                     c.d_ffn / 16, c.d_model / 16};
    const int max_share[PIPE_N_ROLES] = {wide ? 1 : 3, 1 << 20, 3, wide ? 1 : 3, 3};
    int share[PIPE_N_ROLES] = {1, 1, 1, 1, 1};
    for (int r = 0; r < PIPE_N_ROLES; ++r)
        if (r != PIPE_ATTN) share[r] = g_tasc_config.pipe_share > max_share[r] ? max_share[r] : (g_tasc_config.pipe_share < 1 ? 1 : g_tasc_config.pipe_share);
    auto wgs = [&](int r) { return (items[r] + share[r] - 1) / share[r]; };
    share[PIPE_ATTN] = (items[PIPE_ATTN] + 15) / 16;       // at most 16 workgroups on attention
    for (;;) {
        int total = 0;
        for (int r = 0; r < PIPE_N_ROLES; ++r) total += wgs(r);
        if (total <= grid) break;
        int pick = -1;
        for (int r = 0; r < PIPE_N_ROLES; ++r)
            if (share[r] < max_share[r] && (pick < 0 || wgs(r) > wgs(pick))) pick = r;
        if (pick < 0) return false;
        ++share[pick];
    }
    int at = 0;
    for (int r = 0; r < PIPE_N_ROLES; ++r) {
        base[r] = at;
        count[r] = wgs(r);
        at += count[r];
    }
    return true;
}

bool pipe_path_fits(const tasc_model* m, int batch, int nq, int max_blocks, int grid) {
    const tasc_model_desc& c = m->desc;
    int32_t b[PIPE_N_ROLES], n[PIPE_N_ROLES];
    return c.d_model % 64 == 0 && grid >= 8 && pipe_roles(c, batch, grid, b, n);
}

template <int NKS, int WKS>
tasc_status pipe_attr() {
    TASC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_pipe_step<NKS, WKS>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 PIPE_LDS_BYTES));
    return TASC_OK;
}

tasc_status forward_pipe(const tasc_model* m, tasc_session* s, int nq, int n_sel, float* logits_dbg, TascVerifyTail* tail, int grid,
                         hipStream_t st) {
    const tasc_model_desc& c = m->desc;
    const TascSessDev& d = s->d;
    if (std::lock_guard<std::mutex> lock(g_dev_mu); !dev_state().pipe_ready) {
        tasc_status rc;
        if ((rc = pipe_attr<1, 3>()) != TASC_OK || (rc = pipe_attr<2, 3>()) != TASC_OK || (rc = pipe_attr<4, 3>()) != TASC_OK ||
            (rc = pipe_attr<1, 6>()) != TASC_OK || (rc = pipe_attr<2, 6>()) != TASC_OK || (rc = pipe_attr<4, 6>()) != TASC_OK)
            return rc;
        dev_state().pipe_ready = true;
    }
    if (!s->ll_armed) {
        tasc_status rc = tasc_pipe_arm(s, st);
        if (rc != TASC_OK) return rc;
    }
    const TascSmallWs w = tasc_small_ws_layout(c);
    char* cur = d.small_ws + (size_t)s->ll_copy * w.bytes;
    char* other = d.small_ws + (size_t)(1 - s->ll_copy) * w.bytes;
    PipeArgs pa;
    SmallArgs& a = pa.a;
    a.layers = m->d_layers;
    a.embed = (const BF16*)m->embed;
    a.lm_head = (const BF16*)m->lm_head_f;
    a.gf = m->gf;
    a.rope_cos = m->rope_cos;
    a.rope_sin = m->rope_sin;
    a.bias = BiasCsr{m->bias_rowptr, m->bias_col, m->bias_val, m->bias_base};
    a.n_layers = c.n_layers; a.D = c.d_model; a.H = c.n_heads; a.Hkv = c.n_kv_heads; a.hd = c.head_dim; a.F = c.d_ffn;
    a.V = c.vocab; a.max_pos = c.max_pos; a.eps = c.rms_eps; a.scale = 1.0f / sqrtf((float)c.head_dim);
    a.kv_pool = (BF16*)s->kv_pool; a.kv_layer_stride = s->kv_layer_stride; a.page_elems = s->page_elems;
    a.B = s->batch; a.nq = nq; a.M = s->batch * nq; a.max_blocks = s->max_blocks; a.max_len = s->max_len;
    a.n_strips = s->n_strips; a.max_new = s->max_new;
    a.row_tok = d.row_tok; a.n_rows = d.n_rows; a.pos0 = d.pos0; a.block_tab = d.block_tab; a.sel_rows = d.sel_rows;
    a.sel_tok = d.sel_tok; a.n_sel = n_sel;
    a.x = (float*)(cur + w.x_off); a.x_stride = w.x_stride;
    a.q = (BF16*)(cur + w.q_off); a.att = (BF16*)(cur + w.att_off); a.q_stride = w.q_stride;
    a.act = (BF16*)(cur + w.act_off); a.act_stride = w.act_stride;
    pa.kvn = (BF16*)(cur + w.kvn_off); pa.kvn_stride = w.kvn_stride;
    pa.pv = (float*)(cur + w.pv_off); pa.pi = (int32_t*)(cur + w.pi_off);
    a.part_val = d.part_val; a.part_idx = d.part_idx; a.amax = d.amax; a.logits_dbg = logits_dbg;
    a.k = tail ? tail->k : -1;
    a.drafts = tail ? tail->drafts : nullptr;
    a.tokens = d.tokens; a.n_tok = d.n_tok; a.cached = d.cached; a.n_emit = d.n_emit; a.counters = d.counters;
    a.accept_len = tail ? tail->accept_len : nullptr;
    a.emitted = tail ? tail->emitted : nullptr;
    a.trace_step = tail ? tail->trace_step : nullptr;
    a.bar_flags = (u32*)&d.counters[TASC_CTR_FLAGS];
    a.barb_counter = &d.counters[TASC_CTR_BARB];
    a.bar_error = (u32*)&d.counters[TASC_CTR_BAR_ERR];
    a.xcc_mask = (u32*)&d.counters[TASC_CTR_XCC];
    a.xcd_local = 0;
    a.bias_ptr = d.bias_ptr;
    a.lg_stride = 1; a.lg_count = 0; a.lg_workers = 0; a.bar_epoch = 0; a.barb_base = 0;
    const int n_phases = 3 + 5 * c.n_layers, n_lg_phases = 1 + 5 * c.n_layers;
    a.phase_ts = g_phase_ts;
    a.phase_ts_wgs = g_phase_ts ? (int32_t)(g_phase_ts_cap / (2 * (int64_t)n_phases)) : 0;
    if (!pipe_roles(c, s->batch, grid, pa.role_base, pa.role_count)) {
        tasc_set_error("forward: the pipeline kernel does not fit %d workgroups", grid);
        return TASC_EINVAL;
    }
    const int last = n_sel > 0 ? n_phases : n_lg_phases;
    PROF(TASC_KC_LAYERS);
    auto launch = [&](int p0, int p1) {
        pa.rearm = p0 == 0 ? (u64*)other : nullptr;
        pa.rearm_units = p0 == 0 ? w.bytes / 16 : 0;
        const bool wide = c.d_model > 768;
#define PIPE_LAUNCH(NKS)                                                                                                 \
        if (wide) k_pipe_step<NKS, 6><<<dim3(grid), dim3(SMALL_THREADS), PIPE_LDS_BYTES, st>>>(pa, p0, p1);               \
        else k_pipe_step<NKS, 3><<<dim3(grid), dim3(SMALL_THREADS), PIPE_LDS_BYTES, st>>>(pa, p0, p1)
        if (c.head_dim == 32) { PIPE_LAUNCH(1); }
        else if (c.head_dim == 64) { PIPE_LAUNCH(2); }
        else { PIPE_LAUNCH(4); }
#undef PIPE_LAUNCH
    };
    if (g_tasc_config.small_path == 2) {
        launch(0, last);
    } else {
        for (int ph = 0; ph < last; ++ph) launch(ph, ph + 1);
    }
    TASC_LAUNCH_CHECK();
    s->ll_copy = 1 - s->ll_copy;
    if (tail) tail->done = n_sel > 0;
    return TASC_OK;
}

}  // namespace

tasc_status tasc_pipe_arm(tasc_session* s, hipStream_t st) {
    const tasc_model_desc& c = s->model->desc;
    if (c.dtype != TASC_BF16) return TASC_OK;
    const size_t units = tasc_small_ws_bytes(c) / 16;
    k_fill_sentinel<<<dim3(1024), dim3(256), 0, st>>>((u64*)s->d.small_ws, units);
    TASC_LAUNCH_CHECK();
    s->ll_armed = true;
    return TASC_OK;
}

extern "C" tasc_status tasc_calibration_gemm(int32_t M, int32_t N, int32_t K, int32_t epilogue, int32_t slices, int32_t iters,
                                             void* stream, double* us_per_launch) {
    TASC_REQUIRE(us_per_launch && M >= 1 && M <= 65536 && N >= 128 && N <= (1 << 20) && N % 128 == 0 && K >= 64 && K <= 65536 && K % 64 == 0,
                 "calibration_gemm: 1 <= M <= 65536, N a multiple of 128 up to 2^20, K a multiple of 64 up to 65536");
    TASC_REQUIRE(epilogue == TEPI_STORE || epilogue == TEPI_RESID || epilogue == TEPI_SWIGLU || epilogue == TEPI_PARTIAL,
                 "calibration_gemm: epilogue %d is none of store (0), residual add (1), SwiGLU (2), k-slice partial sums (4)", epilogue);
    TASC_REQUIRE(slices >= 1 && slices <= TG_MAX_SLICES && (slices == 1 || epilogue == TEPI_PARTIAL) && K / 64 >= slices,
                 "calibration_gemm: 1 .. %d k-slices, more than one only with the partial-sum epilogue", TG_MAX_SLICES);
    TASC_REQUIRE(iters >= 1 && iters <= 10000, "calibration_gemm: 1 .. 10000 launches");
    hipStream_t st = (hipStream_t)stream;
    tasc_status rc = tiled_ready();
    if (rc != TASC_OK) return rc;
    const size_t a_bytes = (size_t)M * K * 2, w_bytes = (size_t)N * K * 2, o_bytes = (size_t)M * N * 4 * slices;
    struct Tmp { void* p[3] = {nullptr, nullptr, nullptr}; ~Tmp() { for (void* q : p) if (q) (void)hipFree(q); } } t;
    TASC_HIP(hipMalloc(&t.p[0], a_bytes));
    TASC_HIP(hipMalloc(&t.p[1], w_bytes));
    TASC_HIP(hipMalloc(&t.p[2], o_bytes));
    TASC_HIP(hipMemsetAsync(t.p[0], 0x3c, a_bytes, st));       // bf16 0x3c3c = 0.0115: finite sums and SwiGLU arguments
    TASC_HIP(hipMemsetAsync(t.p[1], 0x3c, w_bytes, st));
    TASC_HIP(hipMemsetAsync(t.p[2], 0, o_bytes, st));
    LmEpi none{};
    auto launch = [&]() {
        const BF16* A = (const BF16*)t.p[0];
        if (epilogue == TEPI_STORE) launch_gemm<TEPI_STORE>(A, t.p[1], M, N, K, (float*)t.p[2], nullptr, none, 1, st);
        else if (epilogue == TEPI_RESID) launch_gemm<TEPI_RESID>(A, t.p[1], M, N, K, (float*)t.p[2], nullptr, none, 1, st);
        else if (epilogue == TEPI_SWIGLU) launch_gemm<TEPI_SWIGLU>(A, t.p[1], M, N, K, nullptr, (BF16*)t.p[2], none, 1, st);
        else launch_gemm<TEPI_PARTIAL>(A, t.p[1], M, N, K, (float*)t.p[2], nullptr, none, slices, st);
    };
    struct Ev { hipEvent_t e[2] = {nullptr, nullptr}; ~Ev() { for (hipEvent_t q : e) if (q) (void)hipEventDestroy(q); } } ev;
    TASC_HIP(hipEventCreate(&ev.e[0]));
    TASC_HIP(hipEventCreate(&ev.e[1]));
    for (int i = 0; i < 3; ++i) launch();
    TASC_LAUNCH_CHECK();
    TASC_HIP(hipEventRecord(ev.e[0], st));
    for (int i = 0; i < iters; ++i) launch();
    TASC_HIP(hipEventRecord(ev.e[1], st));
    TASC_LAUNCH_CHECK();
    TASC_HIP(hipEventSynchronize(ev.e[1]));
    float ms = 0.f;
    TASC_HIP(hipEventElapsedTime(&ms, ev.e[0], ev.e[1]));
    *us_per_launch = (double)ms * 1e3 / iters;
    return TASC_OK;
}

int tasc_forward_chains(const tasc_model* m, const tasc_session* s, int32_t nq) {
    int chains = g_tasc_config.chains > 0 ? g_tasc_config.chains : tiled_auto_chains(m->desc, s->batch, nq);
    chains = chains < s->batch ? chains : s->batch;
    chains = chains < TASC_MAX_CHAINS ? chains : TASC_MAX_CHAINS;
    if (tasc_prof_any() || !s->chain_ready) chains = 1;       // the per-class timers bracket launches on one stream
    return chains;
}

bool tasc_forward_is_tiled(const tasc_model* m, const tasc_session* s, int32_t nq) {
    const int decode_rows = s->max_rows < SMALL_ROWS ? s->max_rows : SMALL_ROWS;
    if (g_tasc_config.small_path != 0 && nq <= SMALL_ROWS && small_path_fits(m, s->batch, decode_rows, s->max_blocks)) return false;
    return g_tasc_config.tiled_path != 0 && tiled_path_fits(m->desc);
}

tasc_status tasc_forward_rows(const tasc_model* m, tasc_session* s, int32_t nq, int32_t n_sel, float* logits_dbg,
                              TascVerifyTail* tail, hipStream_t st) {
    if (tail) tail->done = false;
    // The kernel family of a decode step (nq <= 16 rows per sequence) is a property of the session, not of the
    // call's row count, so that a greedy step and a speculative step of one session use the same kernels and
    // reduce every row in the same order.  Prompt chunks of more than 16 rows always take the tiled kernels.
    const int decode_rows = s->max_rows < SMALL_ROWS ? s->max_rows : SMALL_ROWS;
    if (g_tasc_config.small_path != 0 && nq <= SMALL_ROWS && small_path_fits(m, s->batch, decode_rows, s->max_blocks)) {
        if (g_tasc_config.small_kernel != 0) {
            int cus = 0;
            {
                std::lock_guard<std::mutex> lock(g_dev_mu);
                DevState& ds = dev_state();
                if (ds.cu_count == 0) {
                    int dev = 0;
                    TASC_HIP(hipGetDevice(&dev));
                    TASC_HIP(hipDeviceGetAttribute(&ds.cu_count, hipDeviceAttributeMultiprocessorCount, dev));
                }
                cus = ds.cu_count;
            }
            int grid = g_tasc_config.small_grid > 0 ? g_tasc_config.small_grid : cus;
            grid = grid < cus ? grid : cus;      // every workgroup must be resident: at most one per compute unit
            if (pipe_path_fits(m, s->batch, decode_rows, s->max_blocks, grid)) return forward_pipe(m, s, nq, n_sel, logits_dbg, tail, grid, st);
        }
        return forward_small(m, s, nq, n_sel, logits_dbg, tail, st);
    }
    if (g_tasc_config.tiled_path != 0 && tiled_path_fits(m->desc)) return forward_tiled(m, s, nq, n_sel, logits_dbg, tail != nullptr, st);
    if (m->desc.dtype == TASC_F32) return forward_generic<float>(m, s, nq, n_sel, logits_dbg, st);
    return forward_generic<BF16>(m, s, nq, n_sel, logits_dbg, st);
}
