// bf16 kernels for forwards of more than 16 rows (batched verify steps, prompt chunks): an LDS-tiled
// MFMA GEMM with fused epilogues (plain store, residual add, SwiGLU, LM-head bias + strip argmax) and a
// paged GQA attention kernel on the same MFMA scheme as the small-batch kernel.
//
// GEMM: out[M, N] = A[M, K] W[N, K]^T, both operands k-contiguous.  A workgroup of 4 waves computes a
// 128 (n) x 128 (m) tile; each wave a 64 x 64 quadrant as 2 x 2 v_mfma_f32_32x32x16_bf16 tiles with the
// WEIGHT rows as the A operand, so a lane ends up with runs of 4 consecutive output features of one row.
// k advances in steps of 64 through double-buffered LDS tiles (global -> registers -> LDS while the MFMAs
// of the previous step run).  A row's result depends only on its own data and the fixed k order, not on
// how many rows the launch holds.  Workgroup ids are remapped so that the workgroups sharing a weight
// tile run on the same XCD and find it in that XCD's L2.
#pragma once
#include "kernels_small.h"

typedef __attribute__((ext_vector_type(16))) float f32x16;

#define TG_BM 128   // rows (m) per workgroup tile
#define TG_BN 128   // output features (n) per workgroup tile
#define TG_BK 64
#define TG_LD (TG_BK + 8)                                     // padded LDS row (elements)
#define TG_LDS_BYTES (2 * (TG_BM + TG_BN) * TG_LD * 2)        // 73728
#define TG_MAX_SLICES 8                                       // most k-slices of a narrow GEMM

// TEPI_PARTIAL: blockIdx.y selects one of gridDim.y slices of k; the slice's sums go to outf[slice][M][N] and
// k_splitk_reduce adds the slices in order (plain store or residual add).  Used where N is too narrow for
// the tile count to fill the chip; the number of slices depends on N and K only.
enum { TEPI_STORE = 0, TEPI_RESID = 1, TEPI_SWIGLU = 2, TEPI_LMHEAD = 3, TEPI_PARTIAL = 4 };

struct LmEpi {            // TEPI_LMHEAD only
    BiasCsr bias;
    const int32_t* sel_tok;   // input token of every row (bias row)
    const int32_t* bias_ptr;  // [M][n_strips + 1] cursor table
    float* part_val;          // [M][n_strips]
    int32_t* part_idx;
    float* logits;            // nullable [M][V]
    int32_t n_strips;
};

// rows of the accumulator a lane holds: element i of a 32x32 tile is output feature 8 (i / 4) + 4 (lane / 32) + i % 4
__device__ inline int tile_row(int i, int lane) { return 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3); }

template <int EPI>
__global__ __launch_bounds__(256) void k_gemm_tiled(const BF16* __restrict__ A, const BF16* __restrict__ W, int M, int N, int K,
                                                    float* __restrict__ outf, BF16* __restrict__ outb, LmEpi lm) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    uint16_t* sW = reinterpret_cast<uint16_t*>(lds);                      // [2][TG_BN][TG_LD]
    uint16_t* sA = sW + 2 * TG_BN * TG_LD;                                // [2][TG_BM][TG_LD]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave >> 1, wm = wave & 1;
    // XCD-aware tile order: the dispatcher deals consecutive workgroup ids to the 8 XCDs in turn; give each
    // XCD a contiguous range of tiles, m fastest, so that the tiles sharing weights share an L2
    const int n_mt = (M + TG_BM - 1) / TG_BM, n_nt = (N + TG_BN - 1) / TG_BN, total = n_mt * n_nt;
    int v = blockIdx.x;
    if (total % 8 == 0) v = (blockIdx.x % 8) * (total / 8) + blockIdx.x / 8;
    const int n0 = (v / n_mt) * TG_BN, m0 = (v % n_mt) * TG_BM;

    // global -> register staging: every thread moves 4 x 16 bytes of each operand tile per k-step
    const int ld_row = tid >> 3, ld_col = (tid & 7) * 8;                  // 32 rows x 64 columns per pass
    uint4 rw[4], ra[4];
    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int r = ld_row + 32 * p;
            const int n = n0 + r, m = m0 + r;
            rw[p] = n < N ? *reinterpret_cast<const uint4*>(W + (size_t)n * K + k0 + ld_col) : make_uint4(0, 0, 0, 0);
            ra[p] = m < M ? *reinterpret_cast<const uint4*>(A + (size_t)m * K + k0 + ld_col) : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int r = ld_row + 32 * p;
            *reinterpret_cast<uint4*>(sW + (size_t)(buf * TG_BN + r) * TG_LD + ld_col) = rw[p];
            *reinterpret_cast<uint4*>(sA + (size_t)(buf * TG_BM + r) * TG_LD + ld_col) = ra[p];
        }
    };
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    int kt_begin = 0, nk = K / TG_BK;
    if (EPI == TEPI_PARTIAL) {
        const int per = (nk + gridDim.y - 1) / gridDim.y;
        kt_begin = blockIdx.y * per;
        nk = min(nk, kt_begin + per);
        outf += (size_t)blockIdx.y * M * N;
    }
    if (kt_begin < nk) {
        load_tiles(kt_begin * TG_BK);
        store_tiles(kt_begin & 1);
    }
    __syncthreads();
    for (int kt = kt_begin; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_tiles((kt + 1) * TG_BK);
        const uint16_t* bw = sW + (size_t)(buf * TG_BN + wn * 64 + (lane & 31)) * TG_LD + 8 * (lane >> 5);
        const uint16_t* ba = sA + (size_t)(buf * TG_BM + wm * 64 + (lane & 31)) * TG_LD + 8 * (lane >> 5);
#pragma unroll
        for (int ks = 0; ks < TG_BK / 16; ++ks) {
            bf16x8 fw[2], fa[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                fw[i] = *reinterpret_cast<const bf16x8*>(bw + (size_t)i * 32 * TG_LD + ks * 16);
                fa[i] = *reinterpret_cast<const bf16x8*>(ba + (size_t)i * 32 * TG_LD + ks * 16);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[i], fa[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) {
            store_tiles(buf ^ 1);     // the other buffer was last read before the previous barrier
            __syncthreads();
        }
    }

    // ---- epilogue: acc[i][j][e] = out[m][n], n = n0 + 64 wn + 32 i + tile_row(e, lane), m = m0 + 64 wm + 32 j + lane % 32
    if (EPI == TEPI_LMHEAD) {
        __shared__ float s_bv[2][TG_BM];
        __shared__ int32_t s_bi[2][TG_BM];
        const int strip = n0 / TASC_LM_STRIP;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int ml = 64 * wm + 32 * j + (lane & 31), m = m0 + ml;
            float best = -INFINITY;
            int32_t best_i = 0x7FFFFFFF;
            if (m < M) {
                float base = 0.f;
                if (lm.bias.rowptr) {
                    const int u = lm.sel_tok[m];
                    base = lm.bias.base[u];
                    const int64_t r0 = lm.bias.rowptr[u];
                    const int64_t bp = r0 + lm.bias_ptr[(size_t)m * (lm.n_strips + 1) + strip];
                    const int64_t be = r0 + lm.bias_ptr[(size_t)m * (lm.n_strips + 1) + strip + 1];
                    // the few seen successors of this row inside the strip: replace `base` by their own bias
                    for (int64_t p = bp; p < be; ++p) {
                        const int nl = lm.bias.col[p] - n0 - 64 * wn;        // row within this wave's 64 features
                        if (nl < 0 || nl >= 64) continue;
                        const float dv = lm.bias.val[p] - base;
#pragma unroll
                        for (int i = 0; i < 2; ++i)
#pragma unroll
                            for (int e = 0; e < 16; ++e)
                                if (32 * i + tile_row(e, lane) == nl) acc[i][j][e] += dv;
                    }
                }
#pragma unroll
                for (int i = 0; i < 2; ++i) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int n = n0 + 64 * wn + 32 * i + tile_row(e, lane);
                        if (n < N) {
                            const float z = acc[i][j][e] + base;
                            if (lm.logits) lm.logits[(size_t)m * N + n] = z;
                            if (z > best || (z == best && n < best_i)) { best = z; best_i = n; }
                        }
                    }
                }
            }
            // the two lane halves hold different features of the same row
            const float ov = __shfl_xor(best, 32);
            const int32_t oi = __shfl_xor(best_i, 32);
            if (ov > best || (ov == best && oi < best_i)) { best = ov; best_i = oi; }
            if (lane < 32) { s_bv[wn][ml] = best; s_bi[wn][ml] = best_i; }
        }
        __syncthreads();
        if (tid < TG_BM && m0 + tid < M) {
            float bv = s_bv[0][tid];
            int32_t bi = s_bi[0][tid];
            if (s_bv[1][tid] > bv || (s_bv[1][tid] == bv && s_bi[1][tid] < bi)) { bv = s_bv[1][tid]; bi = s_bi[1][tid]; }
            lm.part_val[(size_t)(m0 + tid) * lm.n_strips + strip] = bv;
            lm.part_idx[(size_t)(m0 + tid) * lm.n_strips + strip] = bi;
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int m = m0 + 64 * wm + 32 * j + (lane & 31);
        if (m >= M) continue;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if (EPI == TEPI_SWIGLU) {
                // rows 0..15 of the 32-row tile are gate features, rows 16..31 the up rows of the same features
                const int fbase = (n0 + 64 * wn + 32 * i) / 2;
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int f = fbase + 8 * q + 4 * (lane >> 5);
                    if (2 * f < N) {
                        float o[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const float g = acc[i][j][4 * q + u], up = acc[i][j][8 + 4 * q + u];
                            o[u] = g / (1.0f + __expf(-g)) * up;
                        }
                        *reinterpret_cast<uint2*>(outb + (size_t)m * (N / 2) + f) = pack_bf16x4(o[0], o[1], o[2], o[3]);
                    }
                }
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = n0 + 64 * wn + 32 * i + 8 * q + 4 * (lane >> 5);
                    if (n < N) {
                        float4* p = reinterpret_cast<float4*>(outf + (size_t)m * N + n);
                        float4 vv = make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                        if (EPI == TEPI_RESID) {
                            const float4 old = *p;
                            vv.x += old.x; vv.y += old.y; vv.z += old.z; vv.w += old.w;
                        }
                        *p = vv;
                    }
                }
            }
        }
    }
}

// out[i] (+)= part[0][i] + part[1][i] + ... in slice order; 4 elements per thread
template <bool RESID>
__global__ void k_splitk_reduce(const float* __restrict__ part, int n_slices, size_t mn, float* __restrict__ out) {
    const size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= mn) return;
    float4 s = *reinterpret_cast<const float4*>(part + i);
    for (int k = 1; k < n_slices; ++k) {
        const float4 v = *reinterpret_cast<const float4*>(part + (size_t)k * mn + i);
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    float4* o = reinterpret_cast<float4*>(out + i);
    if (RESID) {
        const float4 old = *o;
        s.x += old.x; s.y += old.y; s.z += old.z; s.w += old.w;
    }
    *o = s;
}

// cursor table of the LM-head bias (see LmEpi): one thread per (row, strip boundary)
__global__ void k_bias_ptr(BiasCsr bias, const int32_t* __restrict__ sel_tok, int n_sel, int n_strips, int32_t* __restrict__ out) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    const int per_row = n_strips + 1;
    if (idx >= n_sel * per_row) return;
    const int r = idx / per_row, st = idx % per_row;
    const int u = sel_tok[r];
    const int64_t r0 = bias.rowptr[u];
    int64_t lo = r0, hi = bias.rowptr[u + 1];
    const int c_first = st * TASC_LM_STRIP;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (bias.col[mid] < c_first) lo = mid + 1; else hi = mid;
    }
    out[idx] = (int32_t)(lo - r0);
}

// ---------------------------------------------------------------- paged GQA attention, any number of rows
// One workgroup per (sequence, KV head, pass of 32 query rows (16 when head_dim = 128)); the scheme is the
// attention phase of the small-batch kernel (S^T = K Q^T, O^T = V^T P^T, key tiles of 32 at absolute
// positions dealt to the 8 waves, fixed merge tree), with plain kernel arguments.
struct AttnArgs {
    const BF16* q;            // [B * nq, H * hd]
    BF16* att;                // [B * nq, H * hd]
    const BF16* kv_layer;
    const int32_t* n_rows;
    const int32_t* pos0;
    const int32_t* block_tab;
    int32_t B, nq, H, Hkv, max_blocks;
    size_t page_elems;
    float scale;
};

template <int NKS>
__global__ __launch_bounds__(SMALL_THREADS) void k_attn_tiled(AttnArgs a) {
    __shared__ __attribute__((aligned(16))) float s_buf[4 * SMALL_ATT_SLOT + 4 * 32 * 2];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int hd = 32 * NKS, ndt = 2 * NKS;
    constexpr int RT = NKS <= 2 ? 2 : 1, rows_pass = 16 * RT;
    const int Gq = a.H / a.Hkv;
    const int R = a.nq * Gq;
    const size_t v_off = (size_t)a.Hkv * TASC_KV_BLOCK * hd;
    const int m = lane & 15, qd = lane >> 4;
    float* slot_ml = s_buf + 4 * SMALL_ATT_SLOT;
    const int b = blockIdx.x / a.Hkv, g = blockIdx.x % a.Hkv;
    const int r0 = blockIdx.y * rows_pass;
    const int nr = a.n_rows[b], p0 = a.pos0[b];
    const int32_t* bt = a.block_tab + (size_t)b * a.max_blocks;
    // keys this pass can see: up to the position of its last query row
    const int i_last = min(nr - 1, (min(r0 + rows_pass, R) - 1) / Gq);
    const int L = i_last >= 0 ? p0 + i_last + 1 : 0;
    const int n_tiles = (L + 31) / 32;
    bf16x8 qf[RT][NKS];
    int qi[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int r = r0 + 16 * rt + m;
        const int i = r / Gq, jq = r % Gq;
        const bool ok = r < R && i < nr;
        qi[rt] = ok ? p0 + i : -1;
        const BF16* qp = a.q + (size_t)(b * a.nq + (ok ? i : 0)) * a.H * hd + (size_t)(g * Gq + (ok ? jq : 0)) * hd;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            bf16x8 v = *reinterpret_cast<const bf16x8*>(qp + 32 * ks + 8 * qd);
            if (!ok) v = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            qf[rt][ks] = v;
        }
    }
    float mx[RT], lsum[RT];
    f32x4 o[RT][ndt];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        mx[rt] = -INFINITY;
        lsum[rt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < ndt; ++dt) o[rt][dt] = f32x4{0, 0, 0, 0};
    }
    for (int t = wave; t < n_tiles; t += SMALL_NW) {
        const int key0 = t * 32;
        const BF16* pg0 = a.kv_layer + (size_t)bt[key0 / TASC_KV_BLOCK] * a.page_elems;
        const bool has1 = key0 + 16 < L;
        const BF16* pg1 = has1 ? a.kv_layer + (size_t)bt[key0 / TASC_KV_BLOCK + 1] * a.page_elems : pg0;
        bf16x8 kf0[NKS], kf1[NKS], vf[ndt];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            kf0[ks] = *reinterpret_cast<const bf16x8*>(pg0 + (size_t)(g * TASC_KV_BLOCK + m) * hd + 32 * ks + 8 * qd);
            kf1[ks] = *reinterpret_cast<const bf16x8*>(pg1 + (size_t)(g * TASC_KV_BLOCK + m) * hd + 32 * ks + 8 * qd);
        }
#pragma unroll
        for (int dt = 0; dt < ndt; ++dt) {
            const uint2 h0 = *reinterpret_cast<const uint2*>(pg0 + v_off + (size_t)(g * hd + 16 * dt + m) * TASC_KV_BLOCK + 4 * qd);
            const uint2 h1 = has1 ? *reinterpret_cast<const uint2*>(pg1 + v_off + (size_t)(g * hd + 16 * dt + m) * TASC_KV_BLOCK + 4 * qd)
                                  : make_uint2(0, 0);
            vf[dt] = as_bf16x8(h0.x, h0.y, h1.x, h1.y);
        }
        f32x4 s0[RT], s1[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) { s0[rt] = f32x4{0, 0, 0, 0}; s1[rt] = f32x4{0, 0, 0, 0}; }
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                s0[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf0[ks], qf[rt][ks], s0[rt], 0, 0, 0);
                s1[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf1[ks], qf[rt][ks], s1[rt], 0, 0, 0);
            }
        }
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            float sv[8];
            float tmax = -INFINITY;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int key = key0 + (u < 4 ? 4 * qd + u : 16 + 4 * qd + (u - 4));
                const float sc = (u < 4 ? s0[rt][u] : s1[rt][u - 4]) * a.scale;
                sv[u] = (key <= qi[rt]) ? sc : -INFINITY;
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
                    psum += bf2f(pb);
                }
            }
            const bf16x8 pk = as_bf16x8(pw[0], pw[1], pw[2], pw[3]);
            psum += __shfl_xor(psum, 16);
            psum += __shfl_xor(psum, 32);
            lsum[rt] = lsum[rt] * corr + psum;
            mx[rt] = m_new;
#pragma unroll
            for (int dt = 0; dt < ndt; ++dt) {
                o[rt][dt] *= corr;
                o[rt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dt], pk, o[rt][dt], 0, 0, 0);
            }
        }
    }
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
