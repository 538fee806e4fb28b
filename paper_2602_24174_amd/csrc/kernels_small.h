// Small-batch (at most 16 rows) bf16 target forward as ONE persistent kernel.
//
// A verify step of k+1 <= 16 rows streams every weight once and does almost no arithmetic, so its
// time is set by launch and dependency latency, not by bandwidth or MFMA rate.  All phases of all
// layers therefore run inside one launch of `k_small_step`: the grid stays resident (one workgroup
// of 8 waves per compute unit at most) and moves from phase to phase through a grid-wide barrier.
//   0                  embedding gather
//   1 + 5l + 0         RMSNorm + fused q/k/v projection + RoPE + KV append
//   1 + 5l + 1         attention of the rows over the paged cache (GQA group packed into the MFMA tile)
//   1 + 5l + 2         output projection + residual
//   1 + 5l + 3         RMSNorm + gate/up projection + SwiGLU
//   1 + 5l + 4         down projection + residual
//   1 + 5L             final RMSNorm + LM head + bias + per-strip argmax
//   2 + 5L             argmax over strips (+ draft compare, accept length, KV rollback when verifying)
// The host may also launch any sub-range of phases (one phase per launch needs no barrier).
//
// GEMMs use v_mfma_f32_16x16x32_bf16 with the WEIGHT tile as the A operand (16 output features x 32 k)
// and the 16 activation rows as the B operand, so a lane ends up with 4 consecutive output features
// of one row.  Inside a phase everything that does not depend on the previous phase (weight tiles,
// RoPE table entries, page addresses) is requested before the activations are staged, so that a phase
// costs about one memory round trip.  Every row's reduction order is fixed by the kernel (k-steps dealt
// round-robin to the 8 waves, partial sums added in wave order), independent of how many rows are valid.
#pragma once
#include "kernels_generic.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// eight bf16 values given as four packed 32-bit words, as an MFMA operand (no trip through memory)
__device__ inline bf16x8 as_bf16x8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    return __builtin_bit_cast(bf16x8, u32x4{a, b, c, d});
}

#define SMALL_ROWS 16
#define SMALL_KC 1536                 // activation columns staged in LDS at a time
#define SMALL_KP (SMALL_KC + 8)       // padded LDS row length (elements)
#define SMALL_THREADS 512
#define SMALL_NW 8                    // waves per workgroup
#define SMALL_WKS 6                   // k-steps of one staged chunk a wave owns at most: KC / 32 / NW
#define SMALL_ATT_SLOT 2048           // floats of one attention combine slot (rows of a pass x head_dim)

// dynamic LDS layout (bytes)
#define SMALL_LDS_ACT 0
#define SMALL_LDS_RED (SMALL_ROWS * SMALL_KP * 2)                 // 49408
#define SMALL_LDS_BYTES (SMALL_LDS_RED + 2 * SMALL_NW * 64 * 16)  // + 16384 = 65792

struct SmallArgs {
    // model
    const TascLayerW* layers;   // device array [n_layers]
    const BF16* embed;
    const BF16* lm_head;
    const float* gf;
    const float* rope_cos;
    const float* rope_sin;
    BiasCsr bias;
    int32_t n_layers, D, H, Hkv, hd, F, V, max_pos;
    float eps, scale;
    // session
    BF16* kv_pool;
    size_t kv_layer_stride, page_elems;
    int32_t B, nq, M, max_blocks, max_len, n_strips, max_new;
    const int32_t* row_tok;
    const int32_t* n_rows;
    const int32_t* pos0;
    const int32_t* block_tab;
    const int32_t* sel_rows;
    const int32_t* sel_tok;
    int32_t n_sel;
    float* x;
    BF16* q;
    BF16* att;
    BF16* act;
    float* part_val;
    int32_t* part_idx;
    int32_t* amax;
    float* logits_dbg;
    // verify-mode tail (accept); k < 0: stop after the argmax
    int32_t k;
    const int32_t* drafts;
    int32_t* tokens;
    int32_t* n_tok;
    int32_t* cached;
    int32_t* n_emit;
    u64* counters;
    int32_t* accept_len;
    int32_t* emitted;
    int32_t* trace_step;
    // Two grid barriers, each a monotone arrival counter plus the value it had when this launch began.
    // Barrier A joins the workgroups of the layer group (the embedding and layer phases), barrier B all
    // workgroups of the grid (before the LM head and before the accept).
    u64* bar_counter;       // A
    u64 bar_base;
    u64* barb_counter;      // B
    u64 barb_base;
    u32* bar_error;
    // layer group: workgroups wg = lg_stride * j, j < lg_count, run the layer phases
    int32_t lg_stride, lg_count;
    // bias cursor table [n_sel][n_strips + 1]: entries of bias row sel_tok[r] with column < strip start
    int32_t* bias_ptr;
    // optional: wall-clock ticks [workgroup][phase][begin, end] of this launch (nullptr = off)
    u64* phase_ts;
    int32_t phase_ts_wgs;   // workgroups the buffer has room for
};

// ---------------------------------------------------------------- grid barrier
// Every workgroup arrives once per barrier; the counter never resets (the host advances bar_base by
// barriers * workgroups per launch).  The workgroup barrier collects the waves' stores, then wave 0
// alone publishes them (agent-scope release), arrives, waits, and acquires for the whole compute unit.
// The wait is bounded: on time-out the error flag is raised and every later barrier falls through,
// so the grid always drains.
__device__ __noinline__ void grid_sync(u64* counter, u64 target, u32* error, int sleep) {
    __syncthreads();
    if (threadIdx.x < 64) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        if (threadIdx.x == 0) {
            __hip_atomic_fetch_add(counter, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            u32 spins = 0;
            while (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
                if (sleep) __builtin_amdgcn_s_sleep(32); else __builtin_amdgcn_s_sleep(1);
                if ((++spins & 1023u) == 0) {
                    if (__hip_atomic_load(error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) break;
                    if (spins > (1u << 22)) {
                        __hip_atomic_fetch_or(error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    __syncthreads();
}

// ---------------------------------------------------------------- staging of the 16 activation rows
// Wave w stages rows w and w + 8: s_act[r][0..D) = bf16(x[r] * g / sqrt(mean(x[r]^2) + eps)) for r < M, zero for
// r >= M.  One pass: the row stays in registers between the sum of squares and the scaling.  D <= 1536.
__device__ inline void stage_normed(const float* __restrict__ x, const float* __restrict__ g, const int32_t* __restrict__ sel,
                                    int M, int D, float eps, uint16_t* s_act) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float4 v[2][6], gg[6];
    float ss[2] = {0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 6; ++t)
        if (4 * (lane + 64 * t) < D) gg[t] = *reinterpret_cast<const float4*>(g + 4 * (lane + 64 * t));
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int r = wave + SMALL_NW * j;
        if (r < M) {
            int src = sel ? sel[r] : r;
            if (src < 0) src = 0;
            const float* xr = x + (size_t)src * D;
#pragma unroll
            for (int t = 0; t < 6; ++t)
                if (4 * (lane + 64 * t) < D) v[j][t] = *reinterpret_cast<const float4*>(xr + 4 * (lane + 64 * t));
        }
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        if (wave + SMALL_NW * j < M) {
#pragma unroll
            for (int t = 0; t < 6; ++t)
                if (4 * (lane + 64 * t) < D)
                    ss[j] += v[j][t].x * v[j][t].x + v[j][t].y * v[j][t].y + v[j][t].z * v[j][t].z + v[j][t].w * v[j][t].w;
        }
        ss[j] = wave_sum(ss[j]);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int r = wave + SMALL_NW * j;
        const float ri = 1.0f / sqrtf(ss[j] / (float)D + eps);
#pragma unroll
        for (int t = 0; t < 6; ++t) {
            const int k = 4 * (lane + 64 * t);
            if (k < D) {
                uint2 o = make_uint2(0, 0);
                if (r < M) {
                    o.x = (uint32_t)f2bf(v[j][t].x * ri * gg[t].x) | ((uint32_t)f2bf(v[j][t].y * ri * gg[t].y) << 16);
                    o.y = (uint32_t)f2bf(v[j][t].z * ri * gg[t].z) | ((uint32_t)f2bf(v[j][t].w * ri * gg[t].w) << 16);
                }
                *reinterpret_cast<uint2*>(s_act + r * SMALL_KP + k) = o;
            }
        }
    }
    __syncthreads();
}

// s_act[r][0..kw) = src[r][kc0..kc0+kw) (bf16 rows of length K), zero for r >= M.
__device__ inline void stage_copy(const BF16* __restrict__ src, int M, int K, int kc0, int kw, uint16_t* s_act) {
    for (int idx = threadIdx.x; idx < SMALL_ROWS * (kw / 8); idx += SMALL_THREADS) {
        const int r = idx / (kw / 8), k = (idx % (kw / 8)) * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (r < M) v = *reinterpret_cast<const uint4*>(src + (size_t)r * K + kc0 + k);
        *reinterpret_cast<uint4*>(s_act + r * SMALL_KP + k) = v;
    }
    __syncthreads();
}

// ---------------------------------------------------------------- MFMA tiles, k-steps dealt to the 8 waves
// Weight fragments of the wave's k-steps (ks = wave, wave + 8, ... of a chunk of nks k-steps).
template <int NT>
__device__ inline void load_w(const BF16* const* wrow, int K, int kc0, int nks, bf16x8 (&w)[NT][SMALL_WKS]) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t woff = (size_t)(lane & 15) * K + kc0 + 8 * (lane >> 4);
#pragma unroll
    for (int u = 0; u < SMALL_WKS; ++u) {
        const int ks = wave + SMALL_NW * u;
        if (ks < nks) {
#pragma unroll
            for (int t = 0; t < NT; ++t) w[t][u] = *reinterpret_cast<const bf16x8*>(wrow[t] + woff + ks * 32);
        }
    }
}
template <int NT>
__device__ inline void mma_w(const bf16x8 (&w)[NT][SMALL_WKS], int nks, const uint16_t* s_act, f32x4* acc) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int aoff = (lane & 15) * SMALL_KP + 8 * (lane >> 4);
#pragma unroll
    for (int u = 0; u < SMALL_WKS; ++u) {
        const int ks = wave + SMALL_NW * u;
        if (ks < nks) {
            const bf16x8 b = *reinterpret_cast<const bf16x8*>(s_act + aoff + ks * 32);
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[t][u], b, acc[t], 0, 0, 0);
        }
    }
}

// Sums the waves' partial tiles in wave order; the result is valid in wave 0.
template <int NT>
__device__ inline void reduce_waves(f32x4* acc, f32x4* s_red) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int t = 0; t < NT; ++t) s_red[(t * SMALL_NW + wave) * 64 + lane] = acc[t];
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            f32x4 s = s_red[(t * SMALL_NW) * 64 + lane];
#pragma unroll
            for (int w = 1; w < SMALL_NW; ++w) s += s_red[(t * SMALL_NW + w) * 64 + lane];
            acc[t] = s;
        }
    }
    __syncthreads();
}

__device__ inline uint2 pack_bf16x4(float a, float b, float c, float d) {
    return make_uint2((uint32_t)f2bf(a) | ((uint32_t)f2bf(b) << 16), (uint32_t)f2bf(c) | ((uint32_t)f2bf(d) << 16));
}

// ---------------------------------------------------------------- phase: RMSNorm + q/k/v + RoPE + KV append
// Item = (head, block of 16 dims of the first half): the tile of dims e0..e0+16 and its RoPE partner
// tile of dims half+e0.. are computed together so the rotation happens in registers.
__device__ __forceinline__ void phase_qkv(const SmallArgs& a, int layer, int wg, int nwg, uint16_t* s_act, f32x4* s_red) {
    const TascLayerW& L = a.layers[layer];
    const int half = a.hd / 2, eb_per_head = half / 16;
    const int n_items = (a.H + 2 * a.Hkv) * eb_per_head;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    BF16* kv_layer = a.kv_pool + (size_t)layer * a.kv_layer_stride;
    const int nks = a.D / 32;
    bool staged = false;
    for (int item = wg; item < n_items; item += nwg) {
        const int head = item / eb_per_head, e0 = (item % eb_per_head) * 16;
        const BF16* W = (const BF16*)L.wqkv;
        const BF16* wrow[2] = {W + (size_t)(head * a.hd + e0) * a.D, W + (size_t)(head * a.hd + half + e0) * a.D};
        bf16x8 w[2][SMALL_WKS];
        load_w<2>(wrow, a.D, 0, nks, w);
        // epilogue operands that do not depend on the product
        const int m = lane & 15, e = e0 + 4 * (lane >> 4);
        bool active = false;
        int pos = 0;
        BF16* page = nullptr;
        float4 cs = make_float4(1, 1, 1, 1), sn = make_float4(0, 0, 0, 0);
        if (wave == 0 && m < a.M) {
            const int b = m / a.nq, i = m % a.nq;
            active = i < a.n_rows[b];
            pos = a.pos0[b] + i;
            const int tpos = pos < a.max_pos ? pos : a.max_pos - 1;
            if (head < a.H + a.Hkv) {
                cs = *reinterpret_cast<const float4*>(a.rope_cos + (size_t)tpos * half + e);
                sn = *reinterpret_cast<const float4*>(a.rope_sin + (size_t)tpos * half + e);
            }
            if (active && head >= a.H)
                page = kv_layer + (size_t)a.block_tab[(size_t)b * a.max_blocks + pos / TASC_KV_BLOCK] * a.page_elems;
        }
        if (!staged) {
            stage_normed(a.x, L.g1, nullptr, a.M, a.D, a.eps, s_act);
            staged = true;
        }
        f32x4 acc[2] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
        mma_w<2>(w, nks, s_act, acc);
        reduce_waves<2>(acc, s_red);
        if (wave == 0 && m < a.M) {
            const float c4[4] = {cs.x, cs.y, cs.z, cs.w}, s4[4] = {sn.x, sn.y, sn.z, sn.w};
            float ra[4], rc[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                ra[u] = acc[0][u] * c4[u] - acc[1][u] * s4[u];
                rc[u] = acc[1][u] * c4[u] + acc[0][u] * s4[u];
            }
            if (head < a.H) {
                BF16* qo = a.q + (size_t)m * a.H * a.hd + head * a.hd;
                *reinterpret_cast<uint2*>(qo + e) = pack_bf16x4(ra[0], ra[1], ra[2], ra[3]);
                *reinterpret_cast<uint2*>(qo + half + e) = pack_bf16x4(rc[0], rc[1], rc[2], rc[3]);
            } else if (active) {
                const int slot = pos % TASC_KV_BLOCK;
                if (head < a.H + a.Hkv) {
                    const int g = head - a.H;
                    BF16* kp = page + (size_t)(g * TASC_KV_BLOCK + slot) * a.hd;
                    *reinterpret_cast<uint2*>(kp + e) = pack_bf16x4(ra[0], ra[1], ra[2], ra[3]);
                    *reinterpret_cast<uint2*>(kp + half + e) = pack_bf16x4(rc[0], rc[1], rc[2], rc[3]);
                } else {
                    const int g = head - a.H - a.Hkv;
                    BF16* vt = page + (size_t)a.Hkv * TASC_KV_BLOCK * a.hd + (size_t)g * a.hd * TASC_KV_BLOCK;
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        vt[(size_t)(e + u) * TASC_KV_BLOCK + slot] = BF16{f2bf(acc[0][u])};
                        vt[(size_t)(half + e + u) * TASC_KV_BLOCK + slot] = BF16{f2bf(acc[1][u])};
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------- phases: projections with residual / SwiGLU
// x[m][n] += sum_k src[m][k] W[n][k]    (output projection, down projection); item = 16 output features
__device__ __forceinline__ void phase_proj_resid(const SmallArgs& a, const BF16* __restrict__ W, const BF16* __restrict__ src, int N, int K,
                                        int wg, int nwg, uint16_t* s_act, f32x4* s_red) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    bool staged = false;
    for (int item = wg; item < N / 16; item += nwg) {
        const BF16* wrow[1] = {W + (size_t)item * 16 * K};
        f32x4 acc[1] = {{0, 0, 0, 0}};
        for (int kc0 = 0; kc0 < K; kc0 += SMALL_KC) {
            const int kw = min(SMALL_KC, K - kc0), nks = kw / 32;
            bf16x8 w[1][SMALL_WKS];
            load_w<1>(wrow, K, kc0, nks, w);
            if (!staged || K > SMALL_KC) {
                if (staged) __syncthreads();
                stage_copy(src, a.M, K, kc0, kw, s_act);
                staged = true;
            }
            mma_w<1>(w, nks, s_act, acc);
        }
        const int m = lane & 15, n = item * 16 + 4 * (lane >> 4);
        float4 xv = make_float4(0, 0, 0, 0);
        float4* xp = reinterpret_cast<float4*>(a.x + (size_t)m * N + n);
        if (wave == 0 && m < a.M) xv = *xp;
        reduce_waves<1>(acc, s_red);
        if (wave == 0 && m < a.M) {
            xv.x += acc[0][0]; xv.y += acc[0][1]; xv.z += acc[0][2]; xv.w += acc[0][3];
            *xp = xv;
        }
    }
}

// act[m][f] = silu(h W_gate[f]) * (h W_up[f]); item = 16 features (gate rows then up rows, interleaved per 16)
__device__ __forceinline__ void phase_gate_up(const SmallArgs& a, int layer, int wg, int nwg, uint16_t* s_act, f32x4* s_red) {
    const TascLayerW& L = a.layers[layer];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nks = a.D / 32;
    bool staged = false;
    for (int item = wg; item < a.F / 16; item += nwg) {
        const BF16* W = (const BF16*)L.wgu + (size_t)item * 32 * a.D;
        const BF16* wrow[2] = {W, W + (size_t)16 * a.D};
        bf16x8 w[2][SMALL_WKS];
        load_w<2>(wrow, a.D, 0, nks, w);
        if (!staged) {
            stage_normed(a.x, L.g2, nullptr, a.M, a.D, a.eps, s_act);
            staged = true;
        }
        f32x4 acc[2] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
        mma_w<2>(w, nks, s_act, acc);
        reduce_waves<2>(acc, s_red);
        if (wave == 0) {
            const int m = lane & 15, f = item * 16 + 4 * (lane >> 4);
            if (m < a.M) {
                float o[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) o[u] = acc[0][u] / (1.0f + __expf(-acc[0][u])) * acc[1][u];
                *reinterpret_cast<uint2*>(a.act + (size_t)m * a.F + f) = pack_bf16x4(o[0], o[1], o[2], o[3]);
            }
        }
    }
}

// ---------------------------------------------------------------- phase: attention
// Item = (sequence b, KV head g).  Query rows of the item: r = i * Gq + jq (i-th row of the sequence,
// jq-th head of the group), processed in passes of 32 rows (16 when head_dim = 128).  Keys are visited
// in tiles of 32 at absolute positions; tile t belongs to wave t mod 8.  S^T = K Q^T and O^T = V^T P^T
// are both MFMA products whose lane layouts chain without a transpose: after S^T a lane holds, for query
// row r = lane mod 16, the scores of keys {4q..4q+3} of each 16-key page (q = lane / 16), which is
// exactly the B-operand slot of the second product when its A operand (V^T) is loaded with the same key
// permutation.  The waves' partial (max, sum, O) are merged pairwise in a fixed tree.
template <int NKS>
__device__ __forceinline__ void phase_attn(const SmallArgs& a, int layer, int wg, int nwg, float* s_buf) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int hd = 32 * NKS, ndt = 2 * NKS;
    constexpr int RT = NKS <= 2 ? 2 : 1, rows_pass = 16 * RT;
    const int Gq = a.H / a.Hkv;
    const int R = a.nq * Gq;
    const BF16* kv_layer = a.kv_pool + (size_t)layer * a.kv_layer_stride;
    const size_t v_off = (size_t)a.Hkv * TASC_KV_BLOCK * hd;
    const int m = lane & 15, qd = lane >> 4;
    float* slot_ml = s_buf + 4 * SMALL_ATT_SLOT;       // [4 slots][rows_pass][2]
    for (int item = wg; item < a.B * a.Hkv; item += nwg) {
        const int b = item / a.Hkv, g = item % a.Hkv;
        const int nr = a.n_rows[b], p0 = a.pos0[b];
        const int32_t* bt = a.block_tab + (size_t)b * a.max_blocks;
        const int L = p0 + nr;                         // keys 0 .. L-1 exist
        const int n_tiles = (L + 31) / 32;
        for (int r0 = 0; r0 < R; r0 += rows_pass) {
            // Q fragments (B operand): row r = r0 + 16 rt + m, dims 32 ks + 8 qd ..
            bf16x8 qf[RT][NKS];
            int qi[RT];
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                const int r = r0 + 16 * rt + m;
                const int i = r / Gq, jq = r % Gq;
                const bool ok = r < R && i < nr;
                qi[rt] = ok ? p0 + i : -1;             // position of the query row, -1 = no such row
                const BF16* qp = a.q + (size_t)(b * a.nq + (ok ? i : 0)) * a.H * hd + (size_t)(g * Gq + (ok ? jq : 0)) * hd;
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) {
                    bf16x8 v = *reinterpret_cast<const bf16x8*>(qp + 32 * ks + 8 * qd);
                    if (!ok) v = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
                    qf[rt][ks] = v;
                }
            }
            float mx[RT], lsum[RT];
            f32x4 o[RT][ndt];                          // O^T tiles: lane holds dims 16 dt + 4 qd .. +4 of row m
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                mx[rt] = -INFINITY;
                lsum[rt] = 0.f;
#pragma unroll
                for (int dt = 0; dt < ndt; ++dt) o[rt][dt] = f32x4{0, 0, 0, 0};
            }
            // Tiles are taken TG at a time: all loads of the group are issued before its arithmetic, so a wave
            // pays about one memory round trip per group instead of one per tile.
            constexpr int TG = NKS <= 2 ? 3 : 1;
            for (int tg = wave; tg < n_tiles; tg += SMALL_NW * TG) {
                bf16x8 kf0[TG][NKS], kf1[TG][NKS];
                bf16x8 vf[TG][ndt];
#pragma unroll
                for (int j = 0; j < TG; ++j) {
                    const int t = tg + j * SMALL_NW;
                    if (t < n_tiles) {
                        const int key0 = t * 32;
                        // the two pages of this tile (the second may lie beyond the sequence)
                        const BF16* pg0 = kv_layer + (size_t)bt[key0 / TASC_KV_BLOCK] * a.page_elems;
                        const bool has1 = key0 + 16 < L;
                        const BF16* pg1 = has1 ? kv_layer + (size_t)bt[key0 / TASC_KV_BLOCK + 1] * a.page_elems : pg0;
#pragma unroll
                        for (int ks = 0; ks < NKS; ++ks) {
                            kf0[j][ks] = *reinterpret_cast<const bf16x8*>(pg0 + (size_t)(g * TASC_KV_BLOCK + m) * hd + 32 * ks + 8 * qd);
                            kf1[j][ks] = *reinterpret_cast<const bf16x8*>(pg1 + (size_t)(g * TASC_KV_BLOCK + m) * hd + 32 * ks + 8 * qd);
                        }
#pragma unroll
                        for (int dt = 0; dt < ndt; ++dt) {
                            const uint2 h0 = *reinterpret_cast<const uint2*>(pg0 + v_off + (size_t)(g * hd + 16 * dt + m) * TASC_KV_BLOCK + 4 * qd);
                            const uint2 h1 = has1 ? *reinterpret_cast<const uint2*>(pg1 + v_off + (size_t)(g * hd + 16 * dt + m) * TASC_KV_BLOCK + 4 * qd)
                                                  : make_uint2(0, 0);
                            vf[j][dt] = as_bf16x8(h0.x, h0.y, h1.x, h1.y);
                        }
                    }
                }
#pragma unroll
                for (int j = 0; j < TG; ++j) {
                    const int t = tg + j * SMALL_NW;
                    if (t < n_tiles) {
                        const int key0 = t * 32;
                        // S^T tiles: A = K rows (key = m within the page), B = Q
                        f32x4 s0[RT], s1[RT];
#pragma unroll
                        for (int rt = 0; rt < RT; ++rt) { s0[rt] = f32x4{0, 0, 0, 0}; s1[rt] = f32x4{0, 0, 0, 0}; }
#pragma unroll
                        for (int ks = 0; ks < NKS; ++ks) {
#pragma unroll
                            for (int rt = 0; rt < RT; ++rt) {
                                s0[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf0[j][ks], qf[rt][ks], s0[rt], 0, 0, 0);
                                s1[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf1[j][ks], qf[rt][ks], s1[rt], 0, 0, 0);
                            }
                        }
                        // online softmax per query row; the lane holds keys key0 + 4qd + u (u<4) and key0 + 16 + 4qd + u
#pragma unroll
                        for (int rt = 0; rt < RT; ++rt) {
                            float sv[8];
                            float tmax = -INFINITY;
#pragma unroll
                            for (int u = 0; u < 8; ++u) {
                                const int key = key0 + (u < 4 ? 4 * qd + u : 16 + 4 * qd + (u - 4));
                                const float sc = (u < 4 ? s0[rt][u] : s1[rt][u - 4]) * a.scale;
                                sv[u] = (key <= qi[rt]) ? sc : -INFINITY;   // causal; also hides keys beyond the sequence
                                tmax = fmaxf(tmax, sv[u]);
                            }
                            tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
                            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
                            const float m_new = fmaxf(mx[rt], tmax);
                            float psum = 0.f, corr = 1.f;
                            uint32_t pw[4] = {0, 0, 0, 0};
                            if (m_new != -INFINITY) {
                                corr = __expf(mx[rt] - m_new);
#pragma unroll
                                for (int u = 0; u < 8; ++u) {
                                    const uint32_t pb = f2bf(__expf(sv[u] - m_new));
                                    pw[u >> 1] |= pb << (16 * (u & 1));
                                    psum += bf2f(pb);                    // the sum uses the rounded weights the product uses
                                }
                            }
                            const bf16x8 pk = as_bf16x8(pw[0], pw[1], pw[2], pw[3]);
                            psum += __shfl_xor(psum, 16);
                            psum += __shfl_xor(psum, 32);
                            lsum[rt] = lsum[rt] * corr + psum;
                            mx[rt] = m_new;
                            // O^T += V^T P^T
#pragma unroll
                            for (int dt = 0; dt < ndt; ++dt) {
                                o[rt][dt] *= corr;
                                o[rt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[j][dt], pk, o[rt][dt], 0, 0, 0);
                            }
                        }
                    }
                }
            }
            // merge the waves pairwise, ((0+1)+(2+3))+((4+5)+(6+7)): a fixed tree through four slots of LDS
            auto merge_round = [&](bool writer, bool reader, int sl) {
                float* so = s_buf + sl * SMALL_ATT_SLOT;
                if (writer) {
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
                        for (int dt = 0; dt < ndt; ++dt)
                            *reinterpret_cast<f32x4*>(so + (size_t)(16 * rt + m) * hd + 16 * dt + 4 * qd) = o[rt][dt];
                        if (qd == 0) {
                            slot_ml[(sl * rows_pass + 16 * rt + m) * 2 + 0] = mx[rt];
                            slot_ml[(sl * rows_pass + 16 * rt + m) * 2 + 1] = lsum[rt];
                        }
                    }
                }
                __syncthreads();
                if (reader) {
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) {
                        const float m2 = slot_ml[(sl * rows_pass + 16 * rt + m) * 2 + 0];
                        const float l2 = slot_ml[(sl * rows_pass + 16 * rt + m) * 2 + 1];
                        const float mn = fmaxf(mx[rt], m2);
                        const float c1 = mn == -INFINITY ? 1.f : __expf(mx[rt] - mn);
                        const float c2 = mn == -INFINITY ? 1.f : __expf(m2 - mn);
                        lsum[rt] = lsum[rt] * c1 + l2 * c2;
                        mx[rt] = mn;
#pragma unroll
                        for (int dt = 0; dt < ndt; ++dt) {
                            const f32x4 o2 = *reinterpret_cast<const f32x4*>(so + (size_t)(16 * rt + m) * hd + 16 * dt + 4 * qd);
                            o[rt][dt] = o[rt][dt] * c1 + o2 * c2;
                        }
                    }
                }
                __syncthreads();
            };
            for (int stride = 1; stride < SMALL_NW; stride <<= 1)
                merge_round((wave & (2 * stride - 1)) == stride, (wave & (2 * stride - 1)) == 0, (wave / (2 * stride)) & 3);
            if (wave == 0) {
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    const int r = r0 + 16 * rt + m;
                    if (r < R) {
                        const int i = r / Gq, jq = r % Gq;
                        const float inv = lsum[rt] > 0.f ? 1.0f / lsum[rt] : 0.f;
                        BF16* op = a.att + (size_t)(b * a.nq + i) * a.H * hd + (size_t)(g * Gq + jq) * hd;
#pragma unroll
                        for (int dt = 0; dt < ndt; ++dt)
                            *reinterpret_cast<uint2*>(op + 16 * dt + 4 * qd) =
                                pack_bf16x4(o[rt][dt][0] * inv, o[rt][dt][1] * inv, o[rt][dt][2] * inv, o[rt][dt][3] * inv);
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------- phase: final norm + LM head + bias + strip argmax
// Item = one strip of TASC_LM_STRIP = 128 vocabulary rows: 8 tiles, one per wave, each over the whole k.
__device__ __forceinline__ void phase_lmhead(const SmallArgs& a, int wg, int nwg, uint16_t* s_act, float* s_best) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, qd = lane >> 4;
    int32_t* s_besti = reinterpret_cast<int32_t*>(s_best + SMALL_NW * SMALL_ROWS);
    const int nks = a.D / 32;
    const size_t woff = (size_t)m * a.D + 8 * qd;
    const int aoff = m * SMALL_KP + 8 * qd;
    bool staged = false;
    for (int strip = wg; strip < a.n_strips; strip += nwg) {
        const int v0 = strip * TASC_LM_STRIP + wave * 16;
        const bool live = v0 < a.V;
        int vr = v0;                                              // a ragged last tile reads the last 16 valid rows
        if (vr + 16 > a.V) vr = a.V - 16;
        const BF16* wrow = a.lm_head + (size_t)(live ? vr : 0) * a.D;
        // first group of weight fragments and the lane's bias cursor, before the activations are staged
        constexpr int WG_KS = 18;
        bf16x8 w[WG_KS];
#pragma unroll
        for (int u = 0; u < WG_KS; ++u)
            if (u < nks) w[u] = *reinterpret_cast<const bf16x8*>(wrow + woff + u * 32);
        const bool own = live && m < a.n_sel;
        int64_t bp = 0, be = 0;
        float base = 0.f;
        if (own && a.bias.rowptr) {
            const int u = a.sel_tok[m];
            const int64_t r0 = a.bias.rowptr[u];
            bp = r0 + a.bias_ptr[(size_t)m * (a.n_strips + 1) + strip];
            be = r0 + a.bias_ptr[(size_t)m * (a.n_strips + 1) + strip + 1];
            base = a.bias.base[u];
        }
        if (!staged) {
            stage_normed(a.x, a.gf, a.sel_rows, a.n_sel, a.D, a.eps, s_act);
            staged = true;
        }
        f32x4 acc = {0, 0, 0, 0};
        for (int ks0 = 0; ks0 < nks; ks0 += WG_KS) {
#pragma unroll
            for (int u = 0; u < WG_KS; ++u) {
                if (ks0 + u < nks) {
                    const bf16x8 bfr = *reinterpret_cast<const bf16x8*>(s_act + aoff + (ks0 + u) * 32);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[u], bfr, acc, 0, 0, 0);
                }
            }
            if (ks0 + WG_KS < nks) {
#pragma unroll
                for (int u = 0; u < WG_KS; ++u)
                    if (ks0 + WG_KS + u < nks) w[u] = *reinterpret_cast<const bf16x8*>(wrow + woff + (ks0 + WG_KS + u) * 32);
            }
        }
        float best = -INFINITY;
        int32_t best_i = 0x7FFFFFFF;
        if (own) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = vr + 4 * qd + u;
                if (c < v0) continue;                              // column belongs to the previous tile
                float z = acc[u];
                if (a.bias.rowptr) {
                    while (bp < be && a.bias.col[bp] < c) ++bp;
                    z += (bp < be && a.bias.col[bp] == c) ? a.bias.val[bp] : base;
                }
                if (a.logits_dbg) a.logits_dbg[(size_t)m * a.V + c] = z;
                if (z > best) { best = z; best_i = c; }
            }
        }
        // best over the 4 lane groups of the row, then over the waves of the strip
        for (int off = 16; off < 64; off <<= 1) {
            const float ov = __shfl_xor(best, off);
            const int32_t oi = __shfl_xor(best_i, off);
            if (ov > best || (ov == best && oi < best_i)) { best = ov; best_i = oi; }
        }
        if (qd == 0) { s_best[wave * SMALL_ROWS + m] = best; s_besti[wave * SMALL_ROWS + m] = best_i; }
        __syncthreads();
        if (threadIdx.x < SMALL_ROWS && threadIdx.x < a.n_sel) {
            const int row = threadIdx.x;
            float bv = s_best[row];
            int32_t bi = s_besti[row];
            for (int w8 = 1; w8 < SMALL_NW; ++w8) {
                const float ov = s_best[w8 * SMALL_ROWS + row];
                const int32_t oi = s_besti[w8 * SMALL_ROWS + row];
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            a.part_val[(size_t)row * a.n_strips + strip] = bv;
            a.part_idx[(size_t)row * a.n_strips + strip] = bi;
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------- phase: argmax over strips, accept, rollback
__device__ __forceinline__ void phase_accept(const SmallArgs& a, int32_t* s_amax) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int r = wave; r < a.n_sel; r += SMALL_NW) {
        float bv = -INFINITY;
        int32_t bi = 0x7FFFFFFF;
        for (int s = lane; s < a.n_strips; s += 64) {
            const float v = a.part_val[(size_t)r * a.n_strips + s];
            const int32_t i = a.part_idx[(size_t)r * a.n_strips + s];
            if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
        }
        for (int o = 32; o > 0; o >>= 1) {
            const float v = __shfl_xor(bv, o);
            const int32_t i = __shfl_xor(bi, o);
            if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
        }
        if (lane == 0) {
            bi = bi == 0x7FFFFFFF ? 0 : bi;
            s_amax[r] = bi;
            a.amax[r] = bi;
        }
    }
    __syncthreads();
    if (a.k < 0) return;
    const int b = threadIdx.x, k = a.k, nq = k + 1;
    if (b >= a.B) return;
    const int N = a.n_tok[b];
    const bool frozen = a.n_emit[b] >= a.max_new;
    int mlen = 0;
    if (!frozen) {
        while (mlen < k && a.drafts[b * k + mlen] == s_amax[b * nq + mlen]) ++mlen;
        int32_t* seq = a.tokens + (size_t)b * a.max_len;
        for (int i = 0; i < mlen; ++i) seq[N + i] = a.drafts[b * k + i];
        seq[N + mlen] = s_amax[b * nq + mlen];
        a.n_tok[b] = N + mlen + 1;
        a.cached[b] += mlen + 1;
        const int e = a.n_emit[b] + mlen + 1;
        a.n_emit[b] = e;
        if (e >= a.max_new) atomicAdd(&a.counters[0], 1ull);
        atomicAdd(&a.counters[3], (u64)mlen);
        atomicAdd(&a.counters[4], (u64)k);
        atomicAdd(&a.counters[8 + mlen], 1ull);
    }
    if (a.accept_len) a.accept_len[b] = mlen;
    if (a.emitted)
        for (int i = 0; i < nq; ++i)
            a.emitted[b * nq + i] = frozen ? -1 : (i < mlen ? a.drafts[b * k + i] : (i == mlen ? s_amax[b * nq + mlen] : -1));
    if (a.trace_step) {
        int32_t* t = a.trace_step + (size_t)b * (2 * k + 3);
        t[0] = N;
        for (int i = 0; i < k; ++i) t[1 + i] = a.drafts[b * k + i];
        for (int i = 0; i < nq; ++i) t[1 + k + i] = s_amax[b * nq + i];
        t[2 * k + 2] = frozen ? -1 : mlen;
    }
    if (b == 0) atomicAdd(&a.counters[2], 1ull);
}

// ---------------------------------------------------------------- the persistent step kernel
// cursor table of the LM-head bias: for every LM-head row r and strip s, how many entries of bias row
// sel_tok[r] have a column below the strip's first column (s = n_strips: all of them)
__device__ inline void build_bias_ptr(const SmallArgs& a, int worker, int n_workers) {
    if (!a.bias.rowptr || a.n_sel <= 0) return;
    const int per_row = a.n_strips + 1;
    for (int idx = worker * SMALL_THREADS + threadIdx.x; idx < a.n_sel * per_row; idx += n_workers * SMALL_THREADS) {
        const int r = idx / per_row, st = idx % per_row;
        const int u = a.sel_tok[r];
        const int64_t r0 = a.bias.rowptr[u];
        int64_t lo = r0, hi = a.bias.rowptr[u + 1];
        const int c_first = st * TASC_LM_STRIP;
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if (a.bias.col[mid] < c_first) lo = mid + 1; else hi = mid;
        }
        a.bias_ptr[idx] = (int32_t)(lo - r0);
    }
}

template <int NKS>
__global__ __launch_bounds__(SMALL_THREADS) void k_small_step(SmallArgs a_in, int phase_begin, int phase_end) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    uint16_t* s_act = reinterpret_cast<uint16_t*>(lds + SMALL_LDS_ACT);
    f32x4* s_red = reinterpret_cast<f32x4*>(lds + SMALL_LDS_RED);
    float* s_attn = reinterpret_cast<float*>(lds);     // attention merge slots alias the staging area
    __shared__ float s_best[2 * SMALL_NW * SMALL_ROWS];
    __shared__ int32_t s_amax[SMALL_ROWS];
    // The phases read their arguments from LDS, and so the small tables every phase consults (layer
    // pointers, row counts, positions, block table): after a grid barrier has invalidated the caches a
    // read of global memory costs a full memory round trip, and these reads would sit in front of the
    // weight and activation loads that depend on them.
    __shared__ SmallArgs s_args;
    __shared__ TascLayerW s_layers[48];
    __shared__ int32_t s_nrows[SMALL_ROWS], s_pos0[SMALL_ROWS];
    __shared__ int32_t s_bt[1024];
    if (threadIdx.x == 0) s_args = a_in;
    if (a_in.n_layers <= 48)
        for (int i = threadIdx.x; i < a_in.n_layers * (int)(sizeof(TascLayerW) / 8); i += SMALL_THREADS)
            reinterpret_cast<u64*>(s_layers)[i] = reinterpret_cast<const u64*>(a_in.layers)[i];
    if (threadIdx.x < a_in.B) {
        s_nrows[threadIdx.x] = a_in.n_rows[threadIdx.x];
        s_pos0[threadIdx.x] = a_in.pos0[threadIdx.x];
    }
    if (a_in.B * a_in.max_blocks <= 1024)
        for (int i = threadIdx.x; i < a_in.B * a_in.max_blocks; i += SMALL_THREADS) s_bt[i] = a_in.block_tab[i];
    __syncthreads();
    if (threadIdx.x == 0) {
        if (a_in.n_layers <= 48) s_args.layers = s_layers;
        s_args.n_rows = s_nrows;
        s_args.pos0 = s_pos0;
        if (a_in.B * a_in.max_blocks <= 1024) s_args.block_tab = s_bt;
    }
    __syncthreads();
    const SmallArgs& a = s_args;
    const int wg = blockIdx.x, nwg = gridDim.x;
    const int n_phases = 3 + 5 * a.n_layers, n_lg_phases = 1 + 5 * a.n_layers;
    const bool member = (wg % a.lg_stride == 0) && (wg / a.lg_stride < a.lg_count);
    const int lw = wg / a.lg_stride, lnw = a.lg_count;
    if (phase_begin == 0) {
        // every workgroup outside the layer group (all of them if there is none) shares the cursor table
        const int outside = nwg - lnw;
        if (outside > 0) {
            if (!member) build_bias_ptr(a, wg - min(lnw, (wg + a.lg_stride - 1) / a.lg_stride), outside);   // rank among the outsiders
        } else {
            build_bias_ptr(a, wg, nwg);
        }
    }
    u32 bar_a = 0, bar_b = 0;
    for (int ph = phase_begin; ph < phase_end && ph < n_phases; ++ph) {
        if (ph < n_lg_phases) {
            if (!member) continue;
            if (ph > phase_begin) {
                if (__hip_atomic_load(a.bar_error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
                grid_sync(a.bar_counter, a.bar_base + (u64)(++bar_a) * lnw, a.bar_error, 0);
            }
        } else if (ph > phase_begin) {
            if (__hip_atomic_load(a.bar_error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
            grid_sync(a.barb_counter, a.barb_base + (u64)(++bar_b) * nwg, a.bar_error, member ? 0 : 1);
        }
        const bool ts = a.phase_ts != nullptr && wg < a.phase_ts_wgs && threadIdx.x == 0;
        if (ts) a.phase_ts[((size_t)wg * n_phases + ph) * 2] = wall_clock64();
        if (ph == 0) {
            for (int r = lw; r < a.M; r += lnw) {
                const BF16* e = a.embed + (size_t)a.row_tok[r] * a.D;
                for (int k = threadIdx.x * 8; k < a.D; k += SMALL_THREADS * 8) {
                    float v[8];
                    load8(e + k, v);
                    float* o = a.x + (size_t)r * a.D + k;
                    *reinterpret_cast<float4*>(o) = make_float4(v[0], v[1], v[2], v[3]);
                    *reinterpret_cast<float4*>(o + 4) = make_float4(v[4], v[5], v[6], v[7]);
                }
            }
        } else if (ph < n_lg_phases) {
            const int layer = (ph - 1) / 5, sub = (ph - 1) % 5;
            const TascLayerW& L = a.layers[layer];
            if (sub == 0) phase_qkv(a, layer, lw, lnw, s_act, s_red);
            else if (sub == 1) phase_attn<NKS>(a, layer, lw, lnw, s_attn);
            else if (sub == 2) phase_proj_resid(a, (const BF16*)L.wo, a.att, a.D, a.H * a.hd, lw, lnw, s_act, s_red);
            else if (sub == 3) phase_gate_up(a, layer, lw, lnw, s_act, s_red);
            else phase_proj_resid(a, (const BF16*)L.wd, a.act, a.D, a.F, lw, lnw, s_act, s_red);
        } else if (ph == n_lg_phases) {
            if (a.n_sel > 0) phase_lmhead(a, wg, nwg, s_act, s_best);
        } else {
            if (a.n_sel > 0 && wg == 0) phase_accept(a, s_amax);
        }
        if (ts) {
            __builtin_amdgcn_s_waitcnt(0);
            a.phase_ts[((size_t)wg * n_phases + ph) * 2 + 1] = wall_clock64();
        }
    }
}
