// Type-generic (fp32 or bf16 storage, fp32 arithmetic) kernels of the target forward.  They are the
// fp32 path and the reference the MFMA kernels are checked against.  Every output row is reduced in
// an order that does not depend on how many rows a launch holds, so a token scored as row i of a
// speculative step gets bit-identical results to the same token scored alone by plain greedy decoding.
#pragma once
#include "tasc_internal.h"

struct BF16 { uint16_t v; };

__device__ inline float bf2f(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
// fp32 -> bf16, round to nearest even: the hardware conversion of gfx950 (v_cvt_pk_bf16_f32), one instruction per pair
typedef __attribute__((ext_vector_type(2))) float tasc_f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 tasc_bf16x2;
__device__ inline uint32_t f2bf_pair(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(tasc_f32x2{lo, hi}, tasc_bf16x2));
}
__device__ inline uint16_t f2bf(float f) { return (uint16_t)(f2bf_pair(f, 0.f) & 0xFFFFu); }
__device__ inline float to_f(float v) { return v; }
__device__ inline float to_f(BF16 v) { return bf2f(v.v); }
template <typename T> __device__ inline T from_f(float f);
template <> __device__ inline float from_f<float>(float f) { return f; }
template <> __device__ inline BF16 from_f<BF16>(float f) { return BF16{f2bf(f)}; }

__device__ inline void load8(const float* __restrict__ p, float* o) {
    float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}
__device__ inline void load8(const BF16* __restrict__ p, float* o) {
    uint4 u = *reinterpret_cast<const uint4*>(p);
    o[0] = bf2f(u.x & 0xFFFFu); o[1] = bf2f(u.x >> 16); o[2] = bf2f(u.y & 0xFFFFu); o[3] = bf2f(u.y >> 16);
    o[4] = bf2f(u.z & 0xFFFFu); o[5] = bf2f(u.z >> 16); o[6] = bf2f(u.w & 0xFFFFu); o[7] = bf2f(u.w >> 16);
}

__device__ inline float wave_sum(float v) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ inline float wave_max(float v) {
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

// ---------------------------------------------------------------- embedding gather
template <typename T>
__global__ void k_embed(const T* __restrict__ E, const int32_t* __restrict__ row_tok, int d, float* __restrict__ x) {
    const int r = blockIdx.x;
    const T* e = E + (size_t)row_tok[r] * d;
    for (int k = threadIdx.x * 8; k < d; k += blockDim.x * 8) {
        float v[8];
        load8(e + k, v);
        float* o = x + (size_t)r * d + k;
        *reinterpret_cast<float4*>(o) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(o + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
}

// ---------------------------------------------------------------- RMSNorm: h = x * g / sqrt(mean(x^2) + eps)
// One wave per row.  `sel` (nullable) gathers rows: output row r reads input row sel[r] (negative -> row 0).
template <typename T>
__global__ __launch_bounds__(64) void k_rmsnorm(const float* __restrict__ x, const float* __restrict__ g,
                                                const int32_t* __restrict__ sel, int d, float eps, T* __restrict__ h) {
    const int r = blockIdx.x, lane = threadIdx.x;
    int src = sel ? sel[r] : r;
    if (src < 0) src = 0;
    const float* xr = x + (size_t)src * d;
    float ss = 0.f;
    for (int k = lane * 4; k < d; k += 256) {
        float4 v = *reinterpret_cast<const float4*>(xr + k);
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    ss = wave_sum(ss);
    const float rinv = 1.0f / sqrtf(ss / (float)d + eps);
    for (int k = lane * 4; k < d; k += 256) {
        float4 v = *reinterpret_cast<const float4*>(xr + k);
        float4 gg = *reinterpret_cast<const float4*>(g + k);
        T* o = h + (size_t)r * d + k;
        o[0] = from_f<T>(v.x * rinv * gg.x);
        o[1] = from_f<T>(v.y * rinv * gg.y);
        o[2] = from_f<T>(v.z * rinv * gg.z);
        o[3] = from_f<T>(v.w * rinv * gg.w);
    }
}

// ---------------------------------------------------------------- generic GEMM  out[M, N] = A[M, K] W[N, K]^T
enum { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2 };

// One wave per output column (per FFN feature for EPI_SWIGLU), rows in chunks of 8.  Every lane sums
// its own k-slices in ascending order, then a butterfly adds the 64 partial sums.
template <typename T, int EPI>
__global__ __launch_bounds__(256) void k_gemm_generic(const T* __restrict__ A, const T* __restrict__ W, int M, int N, int K,
                                                      float* __restrict__ outf, T* __restrict__ outT) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = blockIdx.x * 4 + wave;
    if (col >= N) return;
    const T* w0;
    const T* w1 = nullptr;
    if (EPI == EPI_SWIGLU) {
        w0 = W + (size_t)((col >> 4) * 32 + (col & 15)) * K;
        w1 = w0 + (size_t)16 * K;
    } else {
        w0 = W + (size_t)col * K;
    }
    for (int r0 = 0; r0 < M; r0 += 8) {
        float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0}, acu[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int k = lane * 8; k < K; k += 512) {
            float wv[8], uv[8];
            load8(w0 + k, wv);
            if (EPI == EPI_SWIGLU) load8(w1 + k, uv);
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                if (r0 + r < M) {
                    float av[8];
                    load8(A + (size_t)(r0 + r) * K + k, av);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        acc[r] = fmaf(av[e], wv[e], acc[r]);
                        if (EPI == EPI_SWIGLU) acu[r] = fmaf(av[e], uv[e], acu[r]);
                    }
                }
            }
        }
        float mine = 0.f, mine_u = 0.f;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            float v = wave_sum(acc[r]);
            if (lane == r) mine = v;
            if (EPI == EPI_SWIGLU) {
                float u = wave_sum(acu[r]);
                if (lane == r) mine_u = u;
            }
        }
        const int row = r0 + lane;
        if (lane < 8 && row < M) {
            if (EPI == EPI_STORE) outf[(size_t)row * N + col] = mine;
            if (EPI == EPI_RESID) outf[(size_t)row * N + col] += mine;
            if (EPI == EPI_SWIGLU) outT[(size_t)row * N + col] = from_f<T>(mine / (1.0f + expf(-mine)) * mine_u);
        }
    }
}

// ---------------------------------------------------------------- RoPE + KV append
struct KvGeom {
    int32_t H, Hkv, hd, nq, max_blocks;
    size_t page_elems;   // elements of one page: K [Hkv][16][hd] then V^T [Hkv][hd][16]
};

// Row r = (sequence b, i) sits at position pos0[b] + i.  q is rotated into `q_out`; k is rotated and
// written to the K half of its page, v to the transposed V half.  Rows beyond n_rows[b] write nothing.
// `qkv` may be n_slices partial sums [n_slices][rows][nqkv] (slice_stride elements apart), added here in slice order.
template <typename T>
__global__ void k_rope_kv(const float* __restrict__ qkv, const float* __restrict__ cosT, const float* __restrict__ sinT,
                          int max_pos, const int32_t* __restrict__ n_rows, const int32_t* __restrict__ pos0,
                          const int32_t* __restrict__ block_tab, KvGeom gm, T* __restrict__ q_out, T* __restrict__ kv_layer,
                          int n_slices = 1, size_t slice_stride = 0) {
    const int r = blockIdx.x, b = r / gm.nq, i = r % gm.nq;
    const bool active = i < n_rows[b];
    const int pos = pos0[b] + i;
    const int tpos = pos < max_pos ? pos : max_pos - 1;
    const int half = gm.hd / 2, nqkv = (gm.H + 2 * gm.Hkv) * gm.hd;
    const float* src = qkv + (size_t)r * nqkv;
    T* page = nullptr;
    const int slot = pos % TASC_KV_BLOCK;
    if (active) page = kv_layer + (size_t)block_tab[(size_t)b * gm.max_blocks + pos / TASC_KV_BLOCK] * gm.page_elems;
    for (int idx = threadIdx.x; idx < (gm.H + 2 * gm.Hkv) * half; idx += blockDim.x) {
        const int head = idx / half, e = idx % half;
        float a = src[head * gm.hd + e], c = src[head * gm.hd + e + half];
        for (int sl = 1; sl < n_slices; ++sl) {            // k-slices of a split projection, added in slice order
            a += src[(size_t)sl * slice_stride + head * gm.hd + e];
            c += src[(size_t)sl * slice_stride + head * gm.hd + e + half];
        }
        if (head < gm.H + gm.Hkv) {
            const float cs = cosT[(size_t)tpos * half + e], sn = sinT[(size_t)tpos * half + e];
            const float ra = a * cs - c * sn, rc = c * cs + a * sn;
            if (head < gm.H) {
                q_out[(size_t)r * gm.H * gm.hd + head * gm.hd + e] = from_f<T>(ra);
                q_out[(size_t)r * gm.H * gm.hd + head * gm.hd + e + half] = from_f<T>(rc);
            } else if (active) {
                const int g = head - gm.H;
                page[(size_t)(g * TASC_KV_BLOCK + slot) * gm.hd + e] = from_f<T>(ra);
                page[(size_t)(g * TASC_KV_BLOCK + slot) * gm.hd + e + half] = from_f<T>(rc);
            }
        } else if (active) {
            const int g = head - gm.H - gm.Hkv;
            T* vt = page + (size_t)gm.Hkv * TASC_KV_BLOCK * gm.hd;
            vt[(size_t)(g * gm.hd + e) * TASC_KV_BLOCK + slot] = from_f<T>(a);
            vt[(size_t)(g * gm.hd + e + half) * TASC_KV_BLOCK + slot] = from_f<T>(c);
        }
    }
}

// ---------------------------------------------------------------- generic attention over the paged cache
// One workgroup per (sequence, query head); a wave per query row.  Keys are visited in tiles of 64 at
// absolute positions 0, 64, ...; running max / sum (online softmax) in fp32.
template <typename T>
__global__ __launch_bounds__(256) void k_attn_generic(const T* __restrict__ q, const T* __restrict__ kv_layer,
                                                      const int32_t* __restrict__ n_rows, const int32_t* __restrict__ pos0,
                                                      const int32_t* __restrict__ block_tab, KvGeom gm, float scale,
                                                      T* __restrict__ att) {
    extern __shared__ float s_q[];   // [nq][hd]
    const int b = blockIdx.x, j = blockIdx.y, g = (j * gm.Hkv) / gm.H;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int hd = gm.hd, nr = n_rows[b], p0 = pos0[b];
    const size_t qstride = (size_t)gm.H * hd;
    for (int idx = threadIdx.x; idx < gm.nq * hd; idx += blockDim.x) {
        const int i = idx / hd, e = idx % hd;
        s_q[idx] = to_f(q[(size_t)(b * gm.nq + i) * qstride + j * hd + e]);
    }
    __syncthreads();
    const int32_t* bt = block_tab + (size_t)b * gm.max_blocks;
    const size_t v_off = (size_t)gm.Hkv * TASC_KV_BLOCK * hd;
    for (int i = wave; i < gm.nq; i += 4) {
        T* out = att + (size_t)(b * gm.nq + i) * qstride + j * hd;
        if (i >= nr) {
            for (int e = lane; e < hd; e += 64) out[e] = from_f<T>(0.f);
            continue;
        }
        const float* qi = s_q + i * hd;
        const int L = p0 + i + 1;
        float m = -INFINITY, l = 0.f, acc[4] = {0, 0, 0, 0};
        for (int t0 = 0; t0 < L; t0 += 64) {
            const int key = t0 + lane;
            float s = -INFINITY;
            if (key < L) {
                const T* kp = kv_layer + (size_t)bt[key / TASC_KV_BLOCK] * gm.page_elems +
                              (size_t)(g * TASC_KV_BLOCK + key % TASC_KV_BLOCK) * hd;
                float dot = 0.f;
                for (int e = 0; e < hd; e += 8) {
                    float kvv[8];
                    load8(kp + e, kvv);
#pragma unroll
                    for (int u = 0; u < 8; ++u) dot = fmaf(qi[e + u], kvv[u], dot);
                }
                s = dot * scale;
            }
            const float m_new = fmaxf(m, wave_max(s));
            const float corr = expf(m - m_new);
            const float p = key < L ? expf(s - m_new) : 0.f;
            l = l * corr + wave_sum(p);
            m = m_new;
            const int nk = min(64, L - t0);
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] *= corr;
            for (int kk = 0; kk < nk; ++kk) {
                const float pk = __shfl(p, kk);
                const int kpos = t0 + kk;
                const T* vt = kv_layer + (size_t)bt[kpos / TASC_KV_BLOCK] * gm.page_elems + v_off;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int e = lane + 64 * c;
                    if (e < hd) acc[c] = fmaf(pk, to_f(vt[(size_t)(g * hd + e) * TASC_KV_BLOCK + kpos % TASC_KV_BLOCK]), acc[c]);
                }
            }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int e = lane + 64 * c;
            if (e < hd) out[e] = from_f<T>(acc[c] / l);
        }
    }
}

// ---------------------------------------------------------------- generic LM head with fused bias and partial argmax
struct BiasCsr {
    const int64_t* rowptr;
    const int32_t* col;
    const float* val;
    const float* base;
};

// h: [n_rows, d] normalised hidden rows; row r was fed token tok[r] (bias row).  A workgroup covers a
// strip of TASC_LM_STRIP vocabulary columns, 32 per wave, and leaves, per row, the best (value, index)
// of its strip; index ties go to the lowest column.  logits (nullable) receives every logit.
template <typename T>
__global__ __launch_bounds__(256) void k_lmhead_generic(const T* __restrict__ h, const T* __restrict__ W,
                                                        const int32_t* __restrict__ tok, int n_rows, int V, int d,
                                                        BiasCsr bias, float* __restrict__ part_val,
                                                        int32_t* __restrict__ part_idx, int n_strips,
                                                        float* __restrict__ logits) {
    __shared__ float s_v[4][8];
    __shared__ int32_t s_i[4][8];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int strip = blockIdx.x;
    const int c0 = strip * TASC_LM_STRIP + wave * 32;
    for (int r0 = 0; r0 < n_rows; r0 += 8) {
        const int row = r0 + lane;
        const bool own = lane < 8 && row < n_rows;
        float best = -INFINITY;
        int32_t best_i = 0x7FFFFFFF;
        int64_t bp = 0, be = 0;
        float base = 0.f;
        if (own && bias.rowptr) {
            const int u = tok[row];
            int64_t lo = bias.rowptr[u];
            be = bias.rowptr[u + 1];
            int64_t hi = be;
            while (lo < hi) {   // first entry of the row with column >= c0
                int64_t mid = (lo + hi) >> 1;
                if (bias.col[mid] < c0) lo = mid + 1; else hi = mid;
            }
            bp = lo;
            base = bias.base[u];
        }
        for (int c = c0; c < c0 + 32 && c < V; ++c) {
            const T* w = W + (size_t)c * d;
            float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            for (int k = lane * 8; k < d; k += 512) {
                float wv[8];
                load8(w + k, wv);
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    if (r0 + r < n_rows) {
                        float av[8];
                        load8(h + (size_t)(r0 + r) * d + k, av);
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[r] = fmaf(av[e], wv[e], acc[r]);
                    }
                }
            }
            float mine = 0.f;
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                float v = wave_sum(acc[r]);
                if (lane == r) mine = v;
            }
            if (own) {
                float z = mine;
                if (bias.rowptr) {
                    if (bp < be && bias.col[bp] == c) z += bias.val[bp++];
                    else z += base;
                }
                if (logits) logits[(size_t)row * V + c] = z;
                if (z > best) { best = z; best_i = c; }
            }
        }
        if (lane < 8) { s_v[wave][lane] = best; s_i[wave][lane] = best_i; }
        __syncthreads();
        if (wave == 0 && own) {
            float bv = s_v[0][lane];
            int32_t bi = s_i[0][lane];
            for (int w = 1; w < 4; ++w)
                if (s_v[w][lane] > bv) { bv = s_v[w][lane]; bi = s_i[w][lane]; }
            part_val[(size_t)row * n_strips + strip] = bv;
            part_idx[(size_t)row * n_strips + strip] = bi;
        }
        __syncthreads();
    }
}

// amax[r] = argmax over the strips of row r (lowest index among equal values).  One wave per row.
__global__ __launch_bounds__(64) void k_argmax_reduce(const float* __restrict__ part_val, const int32_t* __restrict__ part_idx,
                                                      int n_strips, int32_t* __restrict__ amax) {
    const int r = blockIdx.x, lane = threadIdx.x;
    float bv = -INFINITY;
    int32_t bi = 0x7FFFFFFF;
    for (int s = lane; s < n_strips; s += 64) {
        const float v = part_val[(size_t)r * n_strips + s];
        const int32_t i = part_idx[(size_t)r * n_strips + s];
        if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
    }
    for (int o = 32; o > 0; o >>= 1) {
        const float v = __shfl_xor(bv, o);
        const int32_t i = __shfl_xor(bi, o);
        if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
    }
    if (lane == 0) amax[r] = bi == 0x7FFFFFFF ? 0 : bi;   // all-NaN row: still a valid token id
}
