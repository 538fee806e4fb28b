// Small-batch (at most 16 rows) bf16 target forward as ONE persistent kernel.
//
// A verify step of k+1 <= 16 rows streams every weight once and does almost no arithmetic, so its
// time is set by launch and dependency latency, not by bandwidth or MFMA rate.  All phases of all
// layers therefore run inside one launch of `k_small_step`: the grid stays resident (one workgroup
// per compute unit at most) and moves from phase to phase through a grid-wide barrier.  Phases:
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
// of one row.  Every row's reduction order is fixed by the kernel (k-steps dealt round-robin to the 4
// waves, partial sums added in wave order), independent of how many rows are valid.
#pragma once
#include "kernels_generic.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

#define SMALL_ROWS 16
#define SMALL_KC 1536                 // activation columns staged in LDS at a time
#define SMALL_KP (SMALL_KC + 8)       // padded LDS row length (elements)
#define SMALL_THREADS 256
#define SMALL_MAX_KS ((SMALL_KC / 32 + 3) / 4)   // k-steps of one chunk a wave can own

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
    // grid barrier: monotone arrival counter, value it had when this launch began, error flag
    u64* bar_counter;
    u64 bar_base;
    u32* bar_error;
};

// ---------------------------------------------------------------- grid barrier
// Every workgroup arrives once per barrier; the counter never resets (the host advances bar_base by
// barriers * workgroups per launch).  The wait is bounded: on time-out the error flag is raised and
// every later barrier falls through, so the grid always drains.
__device__ inline void grid_sync(const SmallArgs& a, u32 index, u32 nwg) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __syncthreads();
    if (threadIdx.x == 0) {
        const u64 target = a.bar_base + (u64)(index + 1) * nwg;
        __hip_atomic_fetch_add(a.bar_counter, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        u32 spins = 0;
        while (__hip_atomic_load(a.bar_counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(2);
            if ((++spins & 1023u) == 0) {
                if (__hip_atomic_load(a.bar_error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) break;
                if (spins > (1u << 22)) {
                    __hip_atomic_fetch_or(a.bar_error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
            }
        }
    }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

// ---------------------------------------------------------------- staging of the 16 activation rows
// s_act[r][0..kw) = bf16(x[r][kc0..] * rinv[r] * g[kc0..]) for r < M, zero for r >= M.
__device__ inline void stage_normed(const float* __restrict__ x, const float* __restrict__ g, const int32_t* __restrict__ sel,
                                    int M, int D, float eps, int kc0, int kw, uint16_t* s_act, float* s_rinv) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (kc0 == 0) {
        for (int r = wave; r < SMALL_ROWS; r += 4) {
            float ss = 0.f;
            if (r < M) {
                int src = sel ? sel[r] : r;
                if (src < 0) src = 0;
                const float* xr = x + (size_t)src * D;
                for (int k = lane * 4; k < D; k += 256) {
                    float4 v = *reinterpret_cast<const float4*>(xr + k);
                    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
                }
            }
            ss = wave_sum(ss);
            if (lane == 0) s_rinv[r] = 1.0f / sqrtf(ss / (float)D + eps);
        }
        __syncthreads();
    }
    for (int idx = threadIdx.x; idx < SMALL_ROWS * (kw / 4); idx += SMALL_THREADS) {
        const int r = idx / (kw / 4), k = (idx % (kw / 4)) * 4;
        uint2 o = make_uint2(0, 0);
        if (r < M) {
            int src = sel ? sel[r] : r;
            if (src < 0) src = 0;
            const float4 v = *reinterpret_cast<const float4*>(x + (size_t)src * D + kc0 + k);
            const float4 gg = *reinterpret_cast<const float4*>(g + kc0 + k);
            const float ri = s_rinv[r];
            o.x = (uint32_t)f2bf(v.x * ri * gg.x) | ((uint32_t)f2bf(v.y * ri * gg.y) << 16);
            o.y = (uint32_t)f2bf(v.z * ri * gg.z) | ((uint32_t)f2bf(v.w * ri * gg.w) << 16);
        }
        *reinterpret_cast<uint2*>(s_act + r * SMALL_KP + k) = o;
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

// ---------------------------------------------------------------- MFMA tiles
// Adds to acc[t] the product of weight tile t (rows wrow[t] .. +16 of a [*, K] matrix, columns
// kc0 .. kc0+kw) with the staged rows.  KSPLIT: the chunk's k-steps are dealt round-robin to the 4
// waves (each wave then holds a partial sum); otherwise the calling wave does all of them.
template <int NT, bool KSPLIT>
__device__ inline void mfma_tiles(const BF16* const* wrow, int K, int kc0, int kw, const uint16_t* s_act, f32x4* acc) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nks = kw / 32;
    const int first = KSPLIT ? wave : 0, step = KSPLIT ? 4 : 1;
    const size_t woff = (size_t)(lane & 15) * K + kc0 + 8 * (lane >> 4);
    const int aoff = (lane & 15) * SMALL_KP + 8 * (lane >> 4);
    for (int ks0 = first; ks0 < nks; ks0 += step * 6) {
        bf16x8 w[NT][6];
#pragma unroll
        for (int u = 0; u < 6; ++u) {
            const int ks = ks0 + u * step;
            if (ks < nks) {
#pragma unroll
                for (int t = 0; t < NT; ++t) w[t][u] = *reinterpret_cast<const bf16x8*>(wrow[t] + woff + ks * 32);
            }
        }
#pragma unroll
        for (int u = 0; u < 6; ++u) {
            const int ks = ks0 + u * step;
            if (ks < nks) {
                const bf16x8 b = *reinterpret_cast<const bf16x8*>(s_act + aoff + ks * 32);
#pragma unroll
                for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[t][u], b, acc[t], 0, 0, 0);
            }
        }
    }
}

// Sums the 4 waves' partial tiles in wave order; the result is valid in wave 0.
template <int NT>
__device__ inline void reduce_waves(f32x4* acc, f32x4* s_red) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int t = 0; t < NT; ++t) s_red[(t * 4 + wave) * 64 + lane] = acc[t];
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            f32x4 s = s_red[(t * 4 + 0) * 64 + lane];
            s += s_red[(t * 4 + 1) * 64 + lane];
            s += s_red[(t * 4 + 2) * 64 + lane];
            s += s_red[(t * 4 + 3) * 64 + lane];
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
__device__ inline void phase_qkv(const SmallArgs& a, int layer, int wg, int nwg, uint16_t* s_act, float* s_rinv, f32x4* s_red) {
    const TascLayerW& L = a.layers[layer];
    const int half = a.hd / 2, eb_per_head = half / 16;
    const int n_items = (a.H + 2 * a.Hkv) * eb_per_head;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    BF16* kv_layer = a.kv_pool + (size_t)layer * a.kv_layer_stride;
    bool staged = false;
    for (int item = wg; item < n_items; item += nwg) {
        const int head = item / eb_per_head, e0 = (item % eb_per_head) * 16;
        const BF16* W = (const BF16*)L.wqkv;
        const BF16* wrow[2] = {W + (size_t)(head * a.hd + e0) * a.D, W + (size_t)(head * a.hd + half + e0) * a.D};
        f32x4 acc[2] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
        for (int kc0 = 0; kc0 < a.D; kc0 += SMALL_KC) {
            const int kw = min(SMALL_KC, a.D - kc0);
            if (!staged || a.D > SMALL_KC) {
                if (staged) __syncthreads();
                stage_normed(a.x, L.g1, nullptr, a.M, a.D, a.eps, kc0, kw, s_act, s_rinv);
                staged = true;
            }
            mfma_tiles<2, true>(wrow, a.D, kc0, kw, s_act, acc);
        }
        reduce_waves<2>(acc, s_red);
        if (wave == 0) {
            const int m = lane & 15, e = e0 + 4 * (lane >> 4);
            if (m < a.M) {
                const int b = m / a.nq, i = m % a.nq;
                const bool active = i < a.n_rows[b];
                const int pos = a.pos0[b] + i;
                const int tpos = pos < a.max_pos ? pos : a.max_pos - 1;
                float ra[4], rc[4];
                if (head < a.H + a.Hkv) {
                    const float4 cs = *reinterpret_cast<const float4*>(a.rope_cos + (size_t)tpos * half + e);
                    const float4 sn = *reinterpret_cast<const float4*>(a.rope_sin + (size_t)tpos * half + e);
                    const float c4[4] = {cs.x, cs.y, cs.z, cs.w}, s4[4] = {sn.x, sn.y, sn.z, sn.w};
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        ra[u] = acc[0][u] * c4[u] - acc[1][u] * s4[u];
                        rc[u] = acc[1][u] * c4[u] + acc[0][u] * s4[u];
                    }
                }
                if (head < a.H) {
                    BF16* qo = a.q + (size_t)m * a.H * a.hd + head * a.hd;
                    *reinterpret_cast<uint2*>(qo + e) = pack_bf16x4(ra[0], ra[1], ra[2], ra[3]);
                    *reinterpret_cast<uint2*>(qo + half + e) = pack_bf16x4(rc[0], rc[1], rc[2], rc[3]);
                } else if (active) {
                    BF16* page = kv_layer + (size_t)a.block_tab[(size_t)b * a.max_blocks + pos / TASC_KV_BLOCK] * a.page_elems;
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
}

// ---------------------------------------------------------------- phases: projections with residual / SwiGLU
// x[m][n] += sum_k src[m][k] W[n][k]    (output projection, down projection); item = 16 output features
__device__ inline void phase_proj_resid(const SmallArgs& a, const BF16* __restrict__ W, const BF16* __restrict__ src, int N, int K,
                                        int wg, int nwg, uint16_t* s_act, f32x4* s_red) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    bool staged = false;
    for (int item = wg; item < N / 16; item += nwg) {
        const BF16* wrow[1] = {W + (size_t)item * 16 * K};
        f32x4 acc[1] = {{0, 0, 0, 0}};
        for (int kc0 = 0; kc0 < K; kc0 += SMALL_KC) {
            const int kw = min(SMALL_KC, K - kc0);
            if (!staged || K > SMALL_KC) {
                if (staged) __syncthreads();
                stage_copy(src, a.M, K, kc0, kw, s_act);
                staged = true;
            }
            mfma_tiles<1, true>(wrow, K, kc0, kw, s_act, acc);
        }
        reduce_waves<1>(acc, s_red);
        if (wave == 0) {
            const int m = lane & 15, n = item * 16 + 4 * (lane >> 4);
            if (m < a.M) {
                float4* xp = reinterpret_cast<float4*>(a.x + (size_t)m * N + n);
                float4 v = *xp;
                v.x += acc[0][0]; v.y += acc[0][1]; v.z += acc[0][2]; v.w += acc[0][3];
                *xp = v;
            }
        }
    }
}

// act[m][f] = silu(h W_gate[f]) * (h W_up[f]); item = 16 features (gate rows then up rows, interleaved per 16)
__device__ inline void phase_gate_up(const SmallArgs& a, int layer, int wg, int nwg, uint16_t* s_act, float* s_rinv, f32x4* s_red) {
    const TascLayerW& L = a.layers[layer];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    bool staged = false;
    for (int item = wg; item < a.F / 16; item += nwg) {
        const BF16* W = (const BF16*)L.wgu + (size_t)item * 32 * a.D;
        const BF16* wrow[2] = {W, W + (size_t)16 * a.D};
        f32x4 acc[2] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
        for (int kc0 = 0; kc0 < a.D; kc0 += SMALL_KC) {
            const int kw = min(SMALL_KC, a.D - kc0);
            if (!staged || a.D > SMALL_KC) {
                if (staged) __syncthreads();
                stage_normed(a.x, L.g2, nullptr, a.M, a.D, a.eps, kc0, kw, s_act, s_rinv);
                staged = true;
            }
            mfma_tiles<2, true>(wrow, a.D, kc0, kw, s_act, acc);
        }
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
// jq-th head of the group), processed in passes of at most 64 rows (32 when head_dim > 64).  Keys are
// visited in tiles of 32 at absolute positions; tile t belongs to wave t mod 4.  S^T = K Q^T and
// O^T = V^T P^T are both MFMA products whose lane layouts chain without a transpose: after S^T a lane
// holds, for query row r = lane mod 16, the scores of keys {4q..4q+3} of each 16-key page (q = lane / 16),
// which is exactly the B-operand slot of the second product when its A operand (V^T) is loaded with the
// same key permutation.
template <int NKS>
__device__ inline void phase_attn(const SmallArgs& a, int layer, int wg, int nwg, float* s_buf) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int hd = 32 * NKS, ndt = 2 * NKS, nks = NKS;
    constexpr int rows_pass = hd > 64 ? 32 : 64, RT = rows_pass / 16;
    const int Gq = a.H / a.Hkv;
    const int R = a.nq * Gq;
    const BF16* kv_layer = a.kv_pool + (size_t)layer * a.kv_layer_stride;
    const size_t v_off = (size_t)a.Hkv * TASC_KV_BLOCK * hd;
    const int m = lane & 15, qd = lane >> 4;
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
                if (rt < RT) {
                    const int r = r0 + 16 * rt + m;
                    const int i = r / Gq, jq = r % Gq;
                    const bool ok = r < R && i < nr;
                    qi[rt] = ok ? p0 + i : -1;         // position of the query row, -1 = no such row
                    const BF16* qp = a.q + (size_t)(b * a.nq + (ok ? i : 0)) * a.H * hd + (size_t)(g * Gq + (ok ? jq : 0)) * hd;
#pragma unroll
                    for (int ks = 0; ks < NKS; ++ks) {
                        if (ks < nks) {
                            bf16x8 v = *reinterpret_cast<const bf16x8*>(qp + 32 * ks + 8 * qd);
                            if (!ok) v = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
                            qf[rt][ks] = v;
                        }
                    }
                }
            }
            float mx[RT], lsum[RT];
            f32x4 o[RT][ndt];                          // O^T tiles [rt][dim tile]: lane holds dims 4qd..+4 of row m
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                mx[rt] = -INFINITY;
                lsum[rt] = 0.f;
#pragma unroll
                for (int dt = 0; dt < ndt; ++dt) o[rt][dt] = f32x4{0, 0, 0, 0};
            }
            for (int t = wave; t < n_tiles; t += 4) {
                const int key0 = t * 32;
                // the two pages of this tile (the second may lie beyond the sequence)
                const BF16* pg0 = kv_layer + (size_t)bt[key0 / TASC_KV_BLOCK] * a.page_elems;
                const bool has1 = key0 + 16 < L;
                const BF16* pg1 = has1 ? kv_layer + (size_t)bt[key0 / TASC_KV_BLOCK + 1] * a.page_elems : pg0;
                // S^T tiles: A = K rows (key = m within the page), B = Q
                f32x4 s0[RT], s1[RT];
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) { s0[rt] = f32x4{0, 0, 0, 0}; s1[rt] = f32x4{0, 0, 0, 0}; }
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) {
                    if (ks < nks) {
                        const bf16x8 k0 = *reinterpret_cast<const bf16x8*>(pg0 + (size_t)(g * TASC_KV_BLOCK + m) * hd + 32 * ks + 8 * qd);
                        const bf16x8 k1 = *reinterpret_cast<const bf16x8*>(pg1 + (size_t)(g * TASC_KV_BLOCK + m) * hd + 32 * ks + 8 * qd);
#pragma unroll
                        for (int rt = 0; rt < RT; ++rt) {
                            if (rt < RT) {
                                s0[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, qf[rt][ks], s0[rt], 0, 0, 0);
                                s1[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, qf[rt][ks], s1[rt], 0, 0, 0);
                            }
                        }
                    }
                }
                // online softmax per query row; the lane holds keys key0 + 4qd + u (u<4) and key0 + 16 + 4qd + u
                bf16x8 pf[RT];
                float corr[RT];
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    if (rt < RT) {
                        float sv[8];
                        float tmax = -INFINITY;
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            const int key = key0 + (u < 4 ? 4 * qd + u : 16 + 4 * qd + (u - 4));
                            const float s = (u < 4 ? s0[rt][u] : s1[rt][u - 4]) * a.scale;
                            sv[u] = (key <= qi[rt]) ? s : -INFINITY;     // causal; also hides keys beyond the sequence
                            tmax = fmaxf(tmax, sv[u]);
                        }
                        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
                        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
                        const float m_new = fmaxf(mx[rt], tmax);
                        float psum = 0.f;
                        union { bf16x8 v; uint16_t u16[8]; } pk;
                        if (m_new == -INFINITY) {
                            corr[rt] = 1.f;
#pragma unroll
                            for (int u = 0; u < 8; ++u) pk.u16[u] = 0;
                        } else {
                            corr[rt] = __expf(mx[rt] - m_new);
#pragma unroll
                            for (int u = 0; u < 8; ++u) {
                                const float p = __expf(sv[u] - m_new);
                                const uint16_t pb = f2bf(p);
                                pk.u16[u] = pb;
                                psum += bf2f(pb);                        // the sum uses the rounded weights the product uses
                            }
                        }
                        psum += __shfl_xor(psum, 16);
                        psum += __shfl_xor(psum, 32);
                        lsum[rt] = lsum[rt] * corr[rt] + psum;
                        mx[rt] = m_new;
                        pf[rt] = pk.v;
                    }
                }
                // O^T += V^T P^T : A = V^T rows (dim = 16 dt + m), keys {4qd..+4} of page 0 and of page 1
#pragma unroll
                for (int dt = 0; dt < ndt; ++dt) {
                    if (dt < ndt) {
                        const BF16* v0p = pg0 + v_off + (size_t)(g * hd + 16 * dt + m) * TASC_KV_BLOCK + 4 * qd;
                        const BF16* v1p = pg1 + v_off + (size_t)(g * hd + 16 * dt + m) * TASC_KV_BLOCK + 4 * qd;
                        union { bf16x8 v; uint2 h[2]; } vf;
                        vf.h[0] = *reinterpret_cast<const uint2*>(v0p);
                        vf.h[1] = has1 ? *reinterpret_cast<const uint2*>(v1p) : make_uint2(0, 0);
#pragma unroll
                        for (int rt = 0; rt < RT; ++rt) {
                            if (rt < RT) {
                                o[rt][dt] *= corr[rt];
                                o[rt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf.v, pf[rt], o[rt][dt], 0, 0, 0);
                            }
                        }
                    }
                }
            }
            // combine the 4 waves: (w0 + w1) + (w2 + w3), through LDS; rows_pass * hd floats per slot
            float* slot_o[2] = {s_buf, s_buf + rows_pass * hd};
            float* slot_ml = s_buf + 2 * rows_pass * hd;      // [2][rows_pass][2]
            for (int round = 0; round < 2; ++round) {
                const bool writer = round == 0 ? (wave & 1) : (wave == 2);
                const bool reader = round == 0 ? !(wave & 1) : (wave == 0);
                const int sl = round == 0 ? (wave >> 1) : 0;
                if (writer) {
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) {
                        if (rt < RT) {
#pragma unroll
                            for (int dt = 0; dt < ndt; ++dt)
                                if (dt < ndt)
                                    *reinterpret_cast<f32x4*>(slot_o[sl] + (size_t)(16 * rt + m) * hd + 16 * dt + 4 * qd) = o[rt][dt];
                            if (qd == 0) {
                                slot_ml[(sl * rows_pass + 16 * rt + m) * 2 + 0] = mx[rt];
                                slot_ml[(sl * rows_pass + 16 * rt + m) * 2 + 1] = lsum[rt];
                            }
                        }
                    }
                }
                __syncthreads();
                if (reader) {
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) {
                        if (rt < RT) {
                            const float m2 = slot_ml[(sl * rows_pass + 16 * rt + m) * 2 + 0];
                            const float l2 = slot_ml[(sl * rows_pass + 16 * rt + m) * 2 + 1];
                            const float mn = fmaxf(mx[rt], m2);
                            const float c1 = mn == -INFINITY ? 1.f : __expf(mx[rt] - mn);
                            const float c2 = mn == -INFINITY ? 1.f : __expf(m2 - mn);
                            lsum[rt] = lsum[rt] * c1 + l2 * c2;
                            mx[rt] = mn;
#pragma unroll
                            for (int dt = 0; dt < ndt; ++dt) {
                                if (dt < ndt) {
                                    const f32x4 o2 = *reinterpret_cast<const f32x4*>(slot_o[sl] + (size_t)(16 * rt + m) * hd + 16 * dt + 4 * qd);
                                    o[rt][dt] = o[rt][dt] * c1 + o2 * c2;
                                }
                            }
                        }
                    }
                }
                __syncthreads();
            }
            if (wave == 0) {
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    if (rt < RT) {
                        const int r = r0 + 16 * rt + m;
                        if (r < R) {
                            const int i = r / Gq, jq = r % Gq;
                            const float inv = lsum[rt] > 0.f ? 1.0f / lsum[rt] : 0.f;
                            BF16* op = a.att + (size_t)(b * a.nq + i) * a.H * hd + (size_t)(g * Gq + jq) * hd;
#pragma unroll
                            for (int dt = 0; dt < ndt; ++dt)
                                if (dt < ndt)
                                    *reinterpret_cast<uint2*>(op + 16 * dt + 4 * qd) =
                                        pack_bf16x4(o[rt][dt][0] * inv, o[rt][dt][1] * inv, o[rt][dt][2] * inv, o[rt][dt][3] * inv);
                        }
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------- phase: final norm + LM head + bias + strip argmax
// Item = strip of TASC_LM_STRIP = 128 vocabulary rows = 8 tiles, two per wave (no k-split).
__device__ inline void phase_lmhead(const SmallArgs& a, int wg, int nwg, uint16_t* s_act, float* s_rinv, float* s_best) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, qd = lane >> 4;
    int32_t* s_besti = reinterpret_cast<int32_t*>(s_best + 4 * SMALL_ROWS);
    bool staged = false;
    for (int strip = wg; strip < a.n_strips; strip += nwg) {
        if (!staged) {
            stage_normed(a.x, a.gf, a.sel_rows, a.n_sel, a.D, a.eps, 0, a.D, s_act, s_rinv);
            staged = true;
        }
        float best = -INFINITY;
        int32_t best_i = 0x7FFFFFFF;
        // bias row of this lane's row: entries with column >= the lane's first column of the strip
        int64_t bp = 0, be = 0;
        float base = 0.f;
        const bool own = m < a.n_sel;
        if (own && a.bias.rowptr) {
            const int u = a.sel_tok[m];
            int64_t lo = a.bias.rowptr[u];
            be = a.bias.rowptr[u + 1];
            int64_t hi = be;
            const int c_first = strip * TASC_LM_STRIP + wave * 32;
            while (lo < hi) {
                const int64_t mid = (lo + hi) >> 1;
                if (a.bias.col[mid] < c_first) lo = mid + 1; else hi = mid;
            }
            bp = lo;
            base = a.bias.base[u];
        }
        for (int tt = 0; tt < 2; ++tt) {
            const int v0 = strip * TASC_LM_STRIP + wave * 32 + tt * 16;   // wave's tiles are adjacent: columns ascend
            if (v0 >= a.V) break;
            int vr = v0;                                                   // clamp so a ragged last tile reads valid rows
            if (vr + 16 > a.V) vr = a.V - 16;
            const BF16* wrow[1] = {a.lm_head + (size_t)vr * a.D};
            f32x4 acc[1] = {{0, 0, 0, 0}};
            mfma_tiles<1, false>(wrow, a.D, 0, a.D, s_act, acc);
            if (own) {
                // this lane: columns vr + 4qd + u; bias entries of other lanes' columns are skipped over
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int c = vr + 4 * qd + u;
                    if (c < v0) continue;                                  // column already covered by the previous tile
                    float z = acc[0][u];
                    if (a.bias.rowptr) {
                        while (bp < be && a.bias.col[bp] < c) ++bp;
                        z += (bp < be && a.bias.col[bp] == c) ? a.bias.val[bp] : base;
                    }
                    if (a.logits_dbg) a.logits_dbg[(size_t)m * a.V + c] = z;
                    if (z > best) { best = z; best_i = c; }
                }
            }
        }
        // best over the 4 lane groups of the row, then over the 4 waves
        for (int off = 16; off < 64; off <<= 1) {
            const float ov = __shfl_xor(best, off);
            const int32_t oi = __shfl_xor(best_i, off);
            if (ov > best || (ov == best && oi < best_i)) { best = ov; best_i = oi; }
        }
        if (qd == 0) { s_best[wave * SMALL_ROWS + m] = best; s_besti[wave * SMALL_ROWS + m] = best_i; }
        __syncthreads();
        if (threadIdx.x < SMALL_ROWS && threadIdx.x < a.n_sel) {
            float bv = s_best[threadIdx.x];
            int32_t bi = s_besti[threadIdx.x];
            for (int w = 1; w < 4; ++w) {
                const float ov = s_best[w * SMALL_ROWS + threadIdx.x];
                const int32_t oi = s_besti[w * SMALL_ROWS + threadIdx.x];
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            a.part_val[(size_t)threadIdx.x * a.n_strips + strip] = bv;
            a.part_idx[(size_t)threadIdx.x * a.n_strips + strip] = bi;
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------- phase: argmax over strips, accept, rollback
__device__ inline void phase_accept(const SmallArgs& a, int32_t* s_amax) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int r = wave; r < a.n_sel; r += 4) {
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
union SmallLds {
    uint16_t act[SMALL_ROWS * SMALL_KP];   // staged activation rows
    float attn[2 * 64 * 64 + 2 * 64 * 2];  // attention combine slots (rows_pass * hd = 4096 floats each)
};

__global__ __launch_bounds__(SMALL_THREADS) void k_small_step(SmallArgs a, int phase_begin, int phase_end) {
    __shared__ __attribute__((aligned(16))) SmallLds lds;
    __shared__ __attribute__((aligned(16))) f32x4 s_red[2 * 4 * 64];
    __shared__ float s_rinv[SMALL_ROWS];
    __shared__ float s_best[8 * SMALL_ROWS];
    __shared__ int32_t s_amax[SMALL_ROWS];
    const int wg = blockIdx.x, nwg = gridDim.x;
    const int n_phases = 3 + 5 * a.n_layers;
    u32 bar = 0;
    for (int ph = phase_begin; ph < phase_end && ph < n_phases; ++ph) {
        if (ph > phase_begin) {
            if (__hip_atomic_load(a.bar_error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
            grid_sync(a, bar++, nwg);
        }
        if (ph == 0) {
            for (int r = wg; r < a.M; r += nwg) {
                const BF16* e = a.embed + (size_t)a.row_tok[r] * a.D;
                for (int k = threadIdx.x * 8; k < a.D; k += SMALL_THREADS * 8) {
                    float v[8];
                    load8(e + k, v);
                    float* o = a.x + (size_t)r * a.D + k;
                    *reinterpret_cast<float4*>(o) = make_float4(v[0], v[1], v[2], v[3]);
                    *reinterpret_cast<float4*>(o + 4) = make_float4(v[4], v[5], v[6], v[7]);
                }
            }
        } else if (ph <= 5 * a.n_layers) {
            const int layer = (ph - 1) / 5, sub = (ph - 1) % 5;
            const TascLayerW& L = a.layers[layer];
            if (sub == 0) phase_qkv(a, layer, wg, nwg, lds.act, s_rinv, s_red);
            else if (sub == 1) {
                if (a.hd == 32) phase_attn<1>(a, layer, wg, nwg, lds.attn);
                else if (a.hd == 64) phase_attn<2>(a, layer, wg, nwg, lds.attn);
                else phase_attn<4>(a, layer, wg, nwg, lds.attn);
            }
            else if (sub == 2) phase_proj_resid(a, (const BF16*)L.wo, a.att, a.D, a.H * a.hd, wg, nwg, lds.act, s_red);
            else if (sub == 3) phase_gate_up(a, layer, wg, nwg, lds.act, s_rinv, s_red);
            else phase_proj_resid(a, (const BF16*)L.wd, a.act, a.D, a.F, wg, nwg, lds.act, s_red);
        } else if (ph == 5 * a.n_layers + 1) {
            if (a.n_sel > 0) phase_lmhead(a, wg, nwg, lds.act, s_rinv, s_best);
        } else {
            if (a.n_sel > 0 && wg == 0) phase_accept(a, s_amax);
        }
    }
}
