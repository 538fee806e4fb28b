// bf16 kernels for forwards of more than 16 rows (batched verify steps, prompt chunks): an LDS-tiled
// MFMA GEMM with fused epilogues (plain store, residual add, SwiGLU, LM-head bias + strip argmax) and a
// paged GQA attention kernel on the same MFMA scheme as the small-batch kernel.
//
// GEMM: out[M, N] = A[M, K] W[N, K]^T, both operands k-contiguous.  A workgroup of 4 waves computes a
// BN (n) x BM (m) tile, 128 x 128 on 4 waves or 256 x 256 on 8; each wave a block of v_mfma_f32_32x32x16_bf16 tiles with the
// WEIGHT rows as the A operand, so a lane ends up with runs of 4 consecutive output features of one row.
// k advances in steps of 64 through double-buffered LDS tiles (global -> registers -> LDS while the MFMAs
// of the previous step run).  A row's result depends only on its own data and the fixed k order, not on
// how many rows the launch holds.  Workgroup ids are remapped so that the workgroups sharing a weight
// tile run on the same XCD and find it in that XCD's L2.
#pragma once
#include "kernels_small.h"

typedef __attribute__((ext_vector_type(16))) float f32x16;
#ifndef IGLP
#define IGLP 0
#endif

#define TG_BK 64
#define TG_LD (TG_BK + 8)                                     // padded LDS row (elements)
#define TG_LDS_BYTES(BN, BM) (2 * ((BN) + (BM)) * TG_LD * 2)   // 73728 for 128 x 128, 147456 for 256 x 256
#define TG_MAX_SLICES 8                                       // most k-slices of a narrow GEMM

// TEPI_PARTIAL: the grid's y extent is the number of slices of k (a workgroup's slice comes from the tile order
// below); the slice's sums go to outf[slice][M][N] and k_splitk_reduce adds the slices in order (plain store or
// residual add).  Used where N is too narrow for the tile count to fill the chip; the number of slices depends on
// N and K only.
// TEPI_ROPE: the fused q/k/v projection of a layer whose output is not sliced: the epilogue rotates the q and k heads (RoPE
// at the row's position), writes q to outb and the new k / v rows straight into the row's cache page.
enum { TEPI_STORE = 0, TEPI_RESID = 1, TEPI_SWIGLU = 2, TEPI_LMHEAD = 3, TEPI_PARTIAL = 4, TEPI_ROPE = 5 };

struct RopeEpi {          // TEPI_ROPE only: what k_rope_kv takes
    const float* cosT;        // [max_pos][hd / 2]
    const float* sinT;
    const int32_t* n_rows;    // [B] active rows of the sequence
    const int32_t* pos0;      // [B] position of the sequence's first row
    const int32_t* block_tab; // [B][max_blocks]
    BF16* kv_layer;           // the layer's pages
    KvGeom gm;
    int32_t max_pos;
};

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

// BN x BM = output features x rows of the workgroup tile; WN x WM waves, each computing a
// (BN / WN) x (BM / WM) block as TI x TJ MFMA tiles of 32 x 32.
template <int EPI, int BN, int BM, int WN, int WM>
__global__ __launch_bounds__(64 * WN * WM) __attribute__((amdgpu_waves_per_eu(1, WN * WM >= 8 ? 2 : 1))) void k_gemm_tiled(const BF16* __restrict__ A, const BF16* __restrict__ W, int M, int N,
                                                             int K, float* __restrict__ outf, BF16* __restrict__ outb, LmEpi lm, RopeEpi rp) {
    constexpr int THREADS = 64 * WN * WM;
    constexpr int SN = BN / WN, SM = BM / WM;          // the wave's span in n and m
    constexpr int TI = SN / 32, TJ = SM / 32;
    constexpr int ROWS_PASS = THREADS / 8;             // tile rows one staging pass covers (8 threads x 16 bytes per row)
    constexpr int PW = BN / ROWS_PASS, PA = BM / ROWS_PASS;
    static_assert(SN % 32 == 0 && SM % 32 == 0 && BN % ROWS_PASS == 0 && BM % ROWS_PASS == 0, "tile shape");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    uint16_t* sW = reinterpret_cast<uint16_t*>(lds);                      // [2][BN][TG_LD]
    uint16_t* sA = sW + 2 * BN * TG_LD;                                   // [2][BM][TG_LD]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave / WM, wm = wave % WM;
    // XCD-aware tile order: the dispatcher deals consecutive workgroup ids (x fastest, then y) to the 8 XCDs in turn.
    // Each XCD gets a contiguous range of (k-slice, tile) pairs, m fastest, then n, then the slice, so that the tiles
    // running on an XCD at the same time share weight and activation panels in its L2.  XCD x holds the ids
    // x, x + 8, ..: all / 8 of them, and one more for x < all % 8.
    const int n_mt = (M + BM - 1) / BM, n_nt = (N + BN - 1) / BN, total = n_mt * n_nt;
    const int lin = blockIdx.y * gridDim.x + blockIdx.x, all = total * gridDim.y;
    const int xcd = lin % 8;
    const int vg = xcd * (all / 8) + min(xcd, all % 8) + lin / 8;
    const int slice = vg / total, v = vg % total;
    const int n0 = (v / n_mt) * BN, m0 = (v % n_mt) * BM;

    // global -> register staging, 16 bytes per thread and pass
    const int ld_row = tid >> 3, ld_col = (tid & 7) * 8;
    // two register sets (0 and 1, separate arrays so that both stay in registers): while step kt is multiplied out
    // of LDS, step kt + 1 waits in one set and step kt + 2 is being fetched into the other, so a global load has two
    // steps' worth of time to arrive
    // (native vector types in plain arrays with compile-time indices: a struct-typed uint4 would be copied through
    // private memory)
    struct StageW { u32x4 w[PW]; } sw0, sw1;   // weights: fetched two steps ahead (HBM latency)
    struct StageA { u32x4 a[PA]; } sa0, sa1;   // activations: two steps ahead as well (an L2 round trip under load takes a step)
    // rows past the matrix are read from its last row (unconditional loads keep the memory pipeline's wait counts
    // exact); what they produce is never stored
    const int wrow_last = N - 1 - n0 - ld_row, arow_last = M - 1 - m0 - ld_row;   // clamp bounds relative to the thread's first row
    const BF16* wbase = W + (size_t)(n0 + ld_row) * K + ld_col;
    const BF16* abase = A + (size_t)(m0 + ld_row) * K + ld_col;
    int woff[PW], aoff[PA];                     // element offsets of the thread's rows (a tile spans < 2^31 elements)
#pragma unroll
    for (int p = 0; p < PW; ++p) woff[p] = min(p * ROWS_PASS, wrow_last) * K;
#pragma unroll
    for (int p = 0; p < PA; ++p) aoff[p] = min(p * ROWS_PASS, arow_last) * K;
    auto load_w = [&](StageW& s, int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < PW; ++p) s.w[p] = *reinterpret_cast<const u32x4*>(wbase + woff[p] + k0);
    };
    auto load_a = [&](StageA& s, int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < PA; ++p) s.a[p] = *reinterpret_cast<const u32x4*>(abase + aoff[p] + k0);
    };
    auto store_wa = [&](const StageW& w, const StageA& a, int buf) __attribute__((always_inline)) {
        uint16_t* dw = sW + (size_t)(buf * BN + ld_row) * TG_LD + ld_col;
        uint16_t* da = sA + (size_t)(buf * BM + ld_row) * TG_LD + ld_col;
#pragma unroll
        for (int p = 0; p < PW; ++p) *reinterpret_cast<u32x4*>(dw + (size_t)p * ROWS_PASS * TG_LD) = w.w[p];
#pragma unroll
        for (int p = 0; p < PA; ++p) *reinterpret_cast<u32x4*>(da + (size_t)p * ROWS_PASS * TG_LD) = a.a[p];
    };
    f32x16 acc[TI][TJ];
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // LM head: the rows' bias cursors (a chain of three dependent loads) are fetched before the main loop
    float lm_base[TJ];
    int64_t lm_cur[TJ], lm_end[TJ];
    if (EPI == TEPI_LMHEAD) {
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
            const int m = m0 + SM * wm + 32 * j + (lane & 31);
            const int strip = (n0 + SN * wn) / TASC_LM_STRIP;
            lm_base[j] = 0.f;
            lm_cur[j] = 0;
            lm_end[j] = 0;
            if (m < M && lm.bias.rowptr && strip < lm.n_strips) {
                const int u = lm.sel_tok[m];
                lm_base[j] = lm.bias.base[u];
                const int64_t r0 = lm.bias.rowptr[u];
                lm_cur[j] = r0 + lm.bias_ptr[(size_t)m * (lm.n_strips + 1) + strip];
                lm_end[j] = r0 + lm.bias_ptr[(size_t)m * (lm.n_strips + 1) + strip + 1];
            }
        }
    }
    // rotation epilogue: where every row of the tile goes (position, cache page and slot) is looked up now, under the main
    // loop, instead of as a chain of dependent loads in the epilogue
    __shared__ int32_t s_rpos[EPI == TEPI_ROPE ? BM : 1];      // table position of the row
    __shared__ int32_t s_rslot[EPI == TEPI_ROPE ? BM : 1];     // slot inside its page, -1 for a row that appends nothing
    __shared__ int32_t s_rpage[EPI == TEPI_ROPE ? BM : 1];     // its page
    if (EPI == TEPI_ROPE && tid < BM) {
        const int m = min(m0 + tid, M - 1);
        const int b = m / rp.gm.nq, ir = m % rp.gm.nq;
        const int pos = rp.pos0[b] + ir;
        const bool active = ir < rp.n_rows[b];
        s_rpos[tid] = pos < rp.max_pos ? pos : rp.max_pos - 1;
        s_rslot[tid] = active ? pos % TASC_KV_BLOCK : -1;
        s_rpage[tid] = active ? rp.block_tab[(size_t)b * rp.gm.max_blocks + pos / TASC_KV_BLOCK] : 0;
    }
    int kt_begin = 0, nk = K / TG_BK;
    if (EPI == TEPI_PARTIAL) {
        const int per = (nk + gridDim.y - 1) / gridDim.y;
        kt_begin = slice * per;
        nk = min(nk, kt_begin + per);
        outf += (size_t)slice * M * N;
    }
    const int k_last = (nk - 1) * TG_BK;
    // One pipeline step = the multiply of LDS buffer `buf` with the refill of the other buffer woven into it, a quarter
    // per 16 of k: the registers that hold the next step's tile (weights fetched two steps ago, activations one step
    // ago) go to the other buffer, which nobody has read since the last barrier, and are then refilled from global
    // memory for the step after that (activations at ka, weights at kw; steps past the last re-read the last one and
    // are never multiplied).  The LDS stores and the fetches so travel under the step's MFMAs instead of ahead of them.
    // Nothing sits under a condition: a conditional load ends in a register copy at the join, which waits for the data.
    static_assert(TG_BK == 64, "the refill is split in four quarters, one per MFMA k-block");
    constexpr int QW = (PW + 3) / 4, QA = (PA + 3) / 4;    // staging passes per quarter
    auto step = [&](int buf, StageW& w, StageA& sa_, int ka, int kw) __attribute__((always_inline)) {
        const uint16_t* bw = sW + (size_t)(buf * BN + wn * SN + (lane & 31)) * TG_LD + 8 * (lane >> 5);
        const uint16_t* ba = sA + (size_t)(buf * BM + wm * SM + (lane & 31)) * TG_LD + 8 * (lane >> 5);
        uint16_t* dw = sW + (size_t)((buf ^ 1) * BN + ld_row) * TG_LD + ld_col;
        uint16_t* da = sA + (size_t)((buf ^ 1) * BM + ld_row) * TG_LD + ld_col;
#pragma unroll
        for (int ks = 0; ks < TG_BK / 16; ++ks) {
            bf16x8 fw[TI], fa[TJ];
#pragma unroll
            for (int i = 0; i < TI; ++i) fw[i] = *reinterpret_cast<const bf16x8*>(bw + (size_t)i * 32 * TG_LD + ks * 16);
#pragma unroll
            for (int j = 0; j < TJ; ++j) fa[j] = *reinterpret_cast<const bf16x8*>(ba + (size_t)j * 32 * TG_LD + ks * 16);
#pragma unroll
            for (int t = 0; t < QW; ++t)                                                              // compile-time conditions
                if (ks * QW + t < PW) *reinterpret_cast<u32x4*>(dw + (size_t)(ks * QW + t) * ROWS_PASS * TG_LD) = w.w[ks * QW + t];
#pragma unroll
            for (int t = 0; t < QA; ++t)
                if (ks * QA + t < PA) *reinterpret_cast<u32x4*>(da + (size_t)(ks * QA + t) * ROWS_PASS * TG_LD) = sa_.a[ks * QA + t];
#pragma unroll
            for (int t = 0; t < QA; ++t)
                if (ks * QA + t < PA) sa_.a[ks * QA + t] = *reinterpret_cast<const u32x4*>(abase + aoff[ks * QA + t] + ka);
#pragma unroll
            for (int t = 0; t < QW; ++t)
                if (ks * QW + t < PW) w.w[ks * QW + t] = *reinterpret_cast<const u32x4*>(wbase + woff[ks * QW + t] + kw);
#pragma unroll
            for (int i = 0; i < TI; ++i)
#pragma unroll
                for (int j = 0; j < TJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[i], fa[j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);              // keeps the quarters in this order
        }
    };
    // Prologue: step kt_begin into buffer 0; registers: set 1 = step + 1, set 0 = step + 2.  Step kt multiplies buffer
    // (kt - kt_begin) % 2 and parks set (kt - kt_begin + 1) % 2 in the other one.
    if (kt_begin < nk) {
        load_w(sw0, kt_begin * TG_BK);
        load_a(sa0, kt_begin * TG_BK);
        store_wa(sw0, sa0, 0);
        load_a(sa1, min((kt_begin + 1) * TG_BK, k_last));
        load_w(sw1, min((kt_begin + 1) * TG_BK, k_last));
        load_a(sa0, min((kt_begin + 2) * TG_BK, k_last));
        load_w(sw0, min((kt_begin + 2) * TG_BK, k_last));
    }
    __syncthreads();
    int kt = kt_begin;
    for (; kt + 1 < nk; kt += 2) {                    // pairs of steps: the loop body holds no branch
        step(0, sw1, sa1, min((kt + 3) * TG_BK, k_last), min((kt + 3) * TG_BK, k_last));
        __syncthreads();
        step(1, sw0, sa0, min((kt + 4) * TG_BK, k_last), min((kt + 4) * TG_BK, k_last));
        __syncthreads();
    }
    if (kt < nk) {                                    // odd count: the last step sits in buffer 0; its refill is idle work
        step(0, sw1, sa1, k_last, k_last);
        __syncthreads();
    }

    // ---- epilogue: acc[i][j][e] = out[m][n], n = n0 + SN wn + 32 i + tile_row(e, lane), m = m0 + SM wm + 32 j + lane % 32
    if (EPI == TEPI_LMHEAD) {
        // a strip of TASC_LM_STRIP = 128 features is covered by SPW = 128 / SN consecutive wave rows (or by one)
        constexpr int SPW = SN >= TASC_LM_STRIP ? 1 : TASC_LM_STRIP / SN;
        static_assert(SN <= TASC_LM_STRIP || SN % TASC_LM_STRIP == 0, "wave span vs strip");
        static_assert(SN <= TASC_LM_STRIP, "one strip per wave row at most");
        __shared__ float s_bv[WN][BM];
        __shared__ int32_t s_bi[WN][BM];
        // The seen successors of a row inside the wave's span get their own bias instead of `base`.  A row can have many
        // of them, and which accumulator element holds a given feature is a lane-and-register question, so the wave
        // scatters the differences (bias - base) of its 32 rows into a [32][SN] patch in LDS (the two lanes of a row
        // take alternate groups of 16 entries of the row's list; no load depends on another's value) and every lane
        // then adds the patch elements of its registers.  The tile buffers are free after the loop's last barrier; LDS
        // serves a wave's accesses in program order.
        constexpr int LDP = SN + 1;
        static_assert((size_t)WN * WM * 32 * LDP * 4 <= TG_LDS_BYTES(BN, BM), "bias patches fit the tile buffers");
        float* patch = reinterpret_cast<float*>(lds) + wave * (32 * LDP);
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
            const int ml = SM * wm + 32 * j + (lane & 31), m = m0 + ml;
            float best = -INFINITY;
            int32_t best_i = 0x7FFFFFFF;
            const float base = lm_base[j];
            // (most 32-row blocks have no seen successor inside the wave's span: then there is nothing to patch)
            if (lm.bias.rowptr && __ballot(lm_cur[j] < lm_end[j]) != 0) {
                for (int q = lane; q < 32 * LDP; q += 64) patch[q] = 0.f;
                __builtin_amdgcn_wave_barrier();
                const int lo = n0 + SN * wn;
                const int64_t be = lm_end[j];
                for (int64_t p0 = lm_cur[j] + 16 * (lane >> 5); p0 < be; p0 += 32) {
                    int nl[16];
                    float bv[16];
#pragma unroll
                    for (int q = 0; q < 16; ++q) {           // 32 loads in flight per lane before the first use
                        const int64_t p = p0 + q < be ? p0 + q : be - 1;
                        nl[q] = lm.bias.col[p] - lo;
                        bv[q] = lm.bias.val[p];
                    }
#pragma unroll
                    for (int q = 0; q < 16; ++q)
                        if (p0 + q < be && nl[q] >= 0 && nl[q] < SN) patch[(lane & 31) * LDP + nl[q]] = bv[q] - base;
                }
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int i = 0; i < TI; ++i)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[i][j][e] += patch[(lane & 31) * LDP + 32 * i + tile_row(e, lane)];
                __builtin_amdgcn_wave_barrier();
            }
            if (m < M) {
#pragma unroll
                for (int i = 0; i < TI; ++i) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int n = n0 + SN * wn + 32 * i + tile_row(e, lane);
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
        // one partial per (row, strip): merge the SPW wave rows of every strip of the tile
        for (int idx = tid; idx < BM * (WN / SPW); idx += THREADS) {
            const int ml = idx % BM, sg = idx / BM;
            const int strip = (n0 + SN * sg * SPW) / TASC_LM_STRIP;
            if (m0 + ml < M && strip < lm.n_strips) {
                float bv = s_bv[sg * SPW][ml];
                int32_t bi = s_bi[sg * SPW][ml];
#pragma unroll
                for (int q = 1; q < SPW; ++q) {
                    const float ov = s_bv[sg * SPW + q][ml];
                    const int32_t oi = s_bi[sg * SPW + q][ml];
                    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
                }
                lm.part_val[(size_t)(m0 + ml) * lm.n_strips + strip] = bv;
                lm.part_idx[(size_t)(m0 + ml) * lm.n_strips + strip] = bi;
            }
        }
        return;
    }
    // A lane holds runs of 4 features of 32 different rows, so a direct store would write 16-byte pieces of 32 rows per
    // instruction.  Each wave turns its block around in LDS instead (the tile buffers are free after the loop's last
    // barrier; a region of its own per wave and 32-row block, so waves do not wait for each other): written as
    // [row][feature], read back with consecutive lanes on consecutive 16-byte chunks of one row, so that every store
    // instruction covers whole rows of the wave's block (128 to 512 contiguous bytes each).
    if (EPI == TEPI_SWIGLU) {
        // rows 0..15 of a 32-feature tile are gate features, rows 16..31 the up rows of the same features: SN / 2 outputs
        constexpr int OW = SN / 2;                          // outputs per row of the wave's block (bf16)
        constexpr int LDO = OW * 2 + 16;                    // padded row (bytes)
        constexpr int CH = OW * 2 / 16;                     // 16-byte chunks per row
        constexpr int RPP = 64 / CH;                        // rows per read pass
        static_assert((size_t)WN * WM * TJ * 32 * LDO <= TG_LDS_BYTES(BN, BM) && 64 % CH == 0 && 32 % RPP == 0, "epilogue staging fits the tile buffers");
        unsigned char* reg = lds + (size_t)wave * TJ * 32 * LDO;
        const int Nh = N / 2, fwave = (n0 + SN * wn) / 2;
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
            unsigned char* rj = reg + (size_t)j * 32 * LDO;
#pragma unroll
            for (int i = 0; i < TI; ++i)
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    float o[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const float g = acc[i][j][4 * q + u], up = acc[i][j][8 + 4 * q + u];
                        o[u] = g / (1.0f + __expf(-g)) * up;
                    }
                    *reinterpret_cast<u32x2*>(rj + (size_t)(lane & 31) * LDO + (16 * i + 8 * q + 4 * (lane >> 5)) * 2) = pack_bf16x4(o[0], o[1], o[2], o[3]);
                }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
            const unsigned char* rj = reg + (size_t)j * 32 * LDO;
#pragma unroll
            for (int p = 0; p < 32 / RPP; ++p) {
                const int r = p * RPP + lane / CH, ch = lane % CH;
                const u32x4 v = *reinterpret_cast<const u32x4*>(rj + (size_t)r * LDO + ch * 16);
                const int m = m0 + SM * wm + 32 * j + r, f = fwave + ch * 8;
                if (m < M && f < Nh) *reinterpret_cast<u32x4*>(outb + (size_t)m * Nh + f) = v;
            }
        }
    } else {
        constexpr int LDO = SN * 4 + 16;                    // padded row of the wave's block (bytes, fp32)
        constexpr int CH = SN * 4 / 16;
        constexpr int RPP = 64 / CH;
        static_assert((size_t)WN * WM * 32 * LDO <= TG_LDS_BYTES(BN, BM) && 64 % CH == 0 && 32 % RPP == 0, "epilogue staging fits the tile buffers");
        unsigned char* reg = lds + (size_t)wave * 32 * LDO;
        const int nwave = n0 + SN * wn;
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
            // the reads of the block before are done (LDS serves a wave in order; the rotation also reads other waves' blocks)
            if (EPI == TEPI_ROPE) __syncthreads();
            else if (j > 0) __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int i = 0; i < TI; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<float4*>(reg + (size_t)(lane & 31) * LDO + (32 * i + 8 * q + 4 * (lane >> 5)) * 4) =
                        make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
            if (EPI == TEPI_ROPE) __syncthreads();
            else __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int p = 0; p < 32 / RPP; ++p) {
                const int r = p * RPP + lane / CH, ch = lane % CH;
                float4 vv = *reinterpret_cast<const float4*>(reg + (size_t)r * LDO + ch * 16);
                const int m = m0 + SM * wm + 32 * j + r, n = nwave + ch * 4;
                if (EPI == TEPI_ROPE) {
                    // The lane whose 4 features lie in the first half of a head also takes their partners half a head on
                    // (the same row, this wave's block or the block of a wave further along n: a tile holds whole heads)
                    // and writes both.  Same arithmetic as k_rope_kv.
                    const int hd = rp.gm.hd, half = hd / 2, e = n % hd, head = n / hd;
                    if (m < M && n < N && e < half) {
                        const int nl = SN * wn + ch * 4 + half;                      // partner's feature inside the tile
                        const float4 cc = *reinterpret_cast<const float4*>(lds + (size_t)((nl / SN) * WM + wm) * 32 * LDO + (size_t)r * LDO + (nl % SN) * 4);
                        const int rt = SM * wm + 32 * j + r;                          // row inside the tile
                        const int tpos = s_rpos[rt], slot = s_rslot[rt];
                        const bool active = slot >= 0;
                        BF16* const page = rp.kv_layer + (size_t)s_rpage[rt] * rp.gm.page_elems;
                        const float a4[4] = {vv.x, vv.y, vv.z, vv.w}, c4[4] = {cc.x, cc.y, cc.z, cc.w};
                        if (head < rp.gm.H + rp.gm.Hkv) {
                            const float4 cs = *reinterpret_cast<const float4*>(rp.cosT + (size_t)tpos * half + e);
                            const float4 sn = *reinterpret_cast<const float4*>(rp.sinT + (size_t)tpos * half + e);
                            const float c_[4] = {cs.x, cs.y, cs.z, cs.w}, s_[4] = {sn.x, sn.y, sn.z, sn.w};
                            float ra[4], rc[4];
#pragma unroll
                            for (int u = 0; u < 4; ++u) {
                                ra[u] = a4[u] * c_[u] - c4[u] * s_[u];
                                rc[u] = c4[u] * c_[u] + a4[u] * s_[u];
                            }
                            BF16* dst = nullptr;
                            if (head < rp.gm.H) {
                                dst = outb + (size_t)m * rp.gm.H * hd + head * hd + e;
                            } else if (active) {
                                dst = page + (size_t)((head - rp.gm.H) * TASC_KV_BLOCK + slot) * hd + e;
                            }
                            if (dst) {
                                *reinterpret_cast<u32x2*>(dst) = pack_bf16x4(ra[0], ra[1], ra[2], ra[3]);
                                *reinterpret_cast<u32x2*>(dst + half) = pack_bf16x4(rc[0], rc[1], rc[2], rc[3]);
                            }
                        } else if (active) {
                            uint16_t* vt = reinterpret_cast<uint16_t*>(page) + (size_t)rp.gm.Hkv * TASC_KV_BLOCK * hd +
                                           (size_t)((head - rp.gm.H - rp.gm.Hkv) * hd + e) * TASC_KV_BLOCK + slot;
#pragma unroll
                            for (int u = 0; u < 4; ++u) {
                                vt[(size_t)u * TASC_KV_BLOCK] = f2bf(a4[u]);
                                vt[(size_t)(half + u) * TASC_KV_BLOCK] = f2bf(c4[u]);
                            }
                        }
                    }
                } else if (m < M && n < N) {
                    float4* pp = reinterpret_cast<float4*>(outf + (size_t)m * N + n);
                    if (EPI == TEPI_RESID) {
                        const float4 old = *pp;
                        vv.x += old.x; vv.y += old.y; vv.z += old.z; vv.w += old.w;
                    }
                    *pp = vv;
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

// The ordered reduction with residual add, fused with the RMSNorm that follows it: one workgroup of 256 threads per
// row, a thread per group of 4 features (two groups for d > 1024), every load of a thread issued before the first add.
// x[r] += part[0][r] + part[1][r] + ... (the element order of k_splitk_reduce, so x has the same bits), then
// h[r] = bf16(x[r] * rinv * g); the squares are summed per thread, per wave and over the 4 waves in a fixed order, so
// a row's result does not depend on the launch.  d <= 2048, d % 4 == 0.
#define RRN_MAX_D 2048
template <int NS>
__global__ __launch_bounds__(256) void k_reduce_resid_norm(const float* __restrict__ part, size_t mn, float* __restrict__ x,
                                                           const float* __restrict__ g, int d, float eps, BF16* __restrict__ h) {
    const int r = blockIdx.x, t = threadIdx.x;
    float* xr = x + (size_t)r * d;
    const float* pr = part + (size_t)r * d;
    f32x4 v[2][NS + 1];
    f32x4 gg[2];
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int k = 4 * (t + 256 * u);
        const bool on = k < d;
        const int kc = on ? k : 0;                                  // unconditional loads; the clamped ones are unused
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) v[u][sl] = *reinterpret_cast<const f32x4*>(pr + (size_t)sl * mn + kc);
        v[u][NS] = *reinterpret_cast<const f32x4*>(xr + kc);
        gg[u] = *reinterpret_cast<const f32x4*>(g + kc);
    }
    float ss = 0.f;
    f32x4 s[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        s[u] = v[u][0];
#pragma unroll
        for (int sl = 1; sl < NS; ++sl) s[u] += v[u][sl];
        s[u] += v[u][NS];
        if (4 * (t + 256 * u) < d) {
            *reinterpret_cast<f32x4*>(xr + 4 * (t + 256 * u)) = s[u];
            ss += s[u][0] * s[u][0] + s[u][1] * s[u][1] + s[u][2] * s[u][2] + s[u][3] * s[u][3];
        } else {
            s[u] = zero;
        }
    }
    __shared__ float s_ss[4];
    ss = wave_sum(ss);
    if ((t & 63) == 0) s_ss[t >> 6] = ss;
    __syncthreads();
    ss = ((s_ss[0] + s_ss[1]) + s_ss[2]) + s_ss[3];
    const float rinv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int k = 4 * (t + 256 * u);
        if (k < d)
            *reinterpret_cast<u32x2*>(h + (size_t)r * d + k) =
                pack_bf16x4(s[u][0] * rinv * gg[u][0], s[u][1] * rinv * gg[u][1], s[u][2] * rinv * gg[u][2], s[u][3] * rinv * gg[u][3]);
    }
}

// RMSNorm of whole rows for the tiled path: k_reduce_resid_norm's scheme without the slices (one workgroup of 256
// threads per row, the row in registers between the sum of squares and the scaling).  d <= 2048, d % 4 == 0.
__global__ __launch_bounds__(256) void k_rmsnorm_row(const float* __restrict__ x, const float* __restrict__ g, int d, float eps,
                                                     BF16* __restrict__ h) {
    const int r = blockIdx.x, t = threadIdx.x;
    const float* xr = x + (size_t)r * d;
    f32x4 v[2], gg[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int k = 4 * (t + 256 * u);
        const int kc = k < d ? k : 0;                                // unconditional loads; the clamped ones are unused
        v[u] = *reinterpret_cast<const f32x4*>(xr + kc);
        gg[u] = *reinterpret_cast<const f32x4*>(g + kc);
    }
    float ss = 0.f;
#pragma unroll
    for (int u = 0; u < 2; ++u)
        if (4 * (t + 256 * u) < d) ss += v[u][0] * v[u][0] + v[u][1] * v[u][1] + v[u][2] * v[u][2] + v[u][3] * v[u][3];
    __shared__ float s_ss[4];
    ss = wave_sum(ss);
    if ((t & 63) == 0) s_ss[t >> 6] = ss;
    __syncthreads();
    ss = ((s_ss[0] + s_ss[1]) + s_ss[2]) + s_ss[3];
    const float rinv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int k = 4 * (t + 256 * u);
        if (k < d)
            *reinterpret_cast<u32x2*>(h + (size_t)r * d + k) =
                pack_bf16x4(v[u][0] * rinv * gg[u][0], v[u][1] * rinv * gg[u][1], v[u][2] * rinv * gg[u][2], v[u][3] * rinv * gg[u][3]);
    }
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
// One workgroup per (sequence, KV head, pass of 32 query rows); the scheme is the
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
#define TILED_ATT_SLOT 2048           // floats of one attention combine slot (32 rows x head_dim 64, or 16 rows x 128)
__global__ __launch_bounds__(SMALL_THREADS) void k_attn_tiled(AttnArgs a) {
    __shared__ __attribute__((aligned(16))) float s_buf[4 * TILED_ATT_SLOT + 4 * 32 * 2];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int hd = 32 * NKS, ndt = 2 * NKS;
    constexpr int RT = 2, rows_pass = 16 * RT;
    const int Gq = a.H / a.Hkv;
    const int R = a.nq * Gq;
    const size_t v_off = (size_t)a.Hkv * TASC_KV_BLOCK * hd;
    const int m = lane & 15, qd = lane >> 4;
    float* slot_ml = s_buf + 4 * TILED_ATT_SLOT;
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
    // The wave's tiles (t = wave, wave + 8, ..) alternate between two register sets (head_dim <= 64): while one tile is
    // multiplied, the next one's keys and values are already on their way.  Loads are unconditional: a tile past the end
    // re-reads the last one (never multiplied), a second page beyond the sequence re-reads the first (its keys are
    // masked and the pool holds no NaN patterns).
    struct KV { bf16x8 kf0[NKS], kf1[NKS], vf[ndt]; };
    auto load_tile = [&](KV& kv, int t) __attribute__((always_inline)) {
        const int key0 = min(t, n_tiles - 1) * 32;
        const BF16* pg0 = a.kv_layer + (size_t)bt[key0 / TASC_KV_BLOCK] * a.page_elems;
        const BF16* pg1 = a.kv_layer + (size_t)bt[key0 / TASC_KV_BLOCK + (key0 + 16 < L ? 1 : 0)] * a.page_elems;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            kv.kf0[ks] = *reinterpret_cast<const bf16x8*>(pg0 + (size_t)(g * TASC_KV_BLOCK + m) * hd + 32 * ks + 8 * qd);
            kv.kf1[ks] = *reinterpret_cast<const bf16x8*>(pg1 + (size_t)(g * TASC_KV_BLOCK + m) * hd + 32 * ks + 8 * qd);
        }
#pragma unroll
        for (int dt = 0; dt < ndt; ++dt) {
            const u32x2 h0 = *reinterpret_cast<const u32x2*>(pg0 + v_off + (size_t)(g * hd + 16 * dt + m) * TASC_KV_BLOCK + 4 * qd);
            const u32x2 h1 = *reinterpret_cast<const u32x2*>(pg1 + v_off + (size_t)(g * hd + 16 * dt + m) * TASC_KV_BLOCK + 4 * qd);
            kv.vf[dt] = as_bf16x8(h0[0], h0[1], h1[0], h1[1]);
        }
    };
    auto multiply_tile = [&](const KV& kv, int t) __attribute__((always_inline)) {
        const int key0 = t * 32;
        f32x4 s0[RT], s1[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) { s0[rt] = f32x4{0, 0, 0, 0}; s1[rt] = f32x4{0, 0, 0, 0}; }
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                s0[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kv.kf0[ks], qf[rt][ks], s0[rt], 0, 0, 0);
                s1[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kv.kf1[ks], qf[rt][ks], s1[rt], 0, 0, 0);
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
                o[rt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kv.vf[dt], pk, o[rt][dt], 0, 0, 0);
            }
        }
    };
    if constexpr (NKS <= 2) {
        if (wave < n_tiles) {
            KV kva, kvb;
            load_tile(kva, wave);
            for (int t = wave; t < n_tiles; t += 2 * SMALL_NW) {
                load_tile(kvb, t + SMALL_NW);
                multiply_tile(kva, t);
                load_tile(kva, t + 2 * SMALL_NW);
                if (t + SMALL_NW < n_tiles) multiply_tile(kvb, t + SMALL_NW);
            }
        }
    } else {
        // head_dim 128: one register set (two row tiles of accumulators take the room of the second)
        for (int t = wave; t < n_tiles; t += SMALL_NW) {
            KV kv;
            load_tile(kv, t);
            multiply_tile(kv, t);
        }
    }
    // fixed merge tree ((0+1)+(2+3))+((4+5)+(6+7)) through four LDS slots; a slot holds MRT row tiles, so head_dim 128
    // runs the tree once per row tile
    constexpr int MRT = NKS == 4 ? 1 : RT;
    auto merge_round = [&](bool writer, bool reader, int sl, int rt0) {
        float* so = s_buf + sl * TILED_ATT_SLOT;
        if (writer) {
#pragma unroll
            for (int q = 0; q < MRT; ++q) {
                const int rt = rt0 + q;
#pragma unroll
                for (int dt = 0; dt < ndt; ++dt)
                    *reinterpret_cast<f32x4*>(so + (size_t)(16 * q + m) * hd + 16 * dt + 4 * qd) = o[rt][dt];
                if (qd == 0) {
                    slot_ml[(sl * rows_pass + 16 * q + m) * 2 + 0] = mx[rt];
                    slot_ml[(sl * rows_pass + 16 * q + m) * 2 + 1] = lsum[rt];
                }
            }
        }
        __syncthreads();
        if (reader) {
#pragma unroll
            for (int q = 0; q < MRT; ++q) {
                const int rt = rt0 + q;
                const float m2 = slot_ml[(sl * rows_pass + 16 * q + m) * 2 + 0];
                const float l2 = slot_ml[(sl * rows_pass + 16 * q + m) * 2 + 1];
                const float mn = fmaxf(mx[rt], m2);
                const float c1 = mn == -INFINITY ? 1.f : __expf(mx[rt] - mn);
                const float c2 = mn == -INFINITY ? 1.f : __expf(m2 - mn);
                lsum[rt] = lsum[rt] * c1 + l2 * c2;
                mx[rt] = mn;
#pragma unroll
                for (int dt = 0; dt < ndt; ++dt) {
                    const f32x4 o2 = *reinterpret_cast<const f32x4*>(so + (size_t)(16 * q + m) * hd + 16 * dt + 4 * qd);
                    o[rt][dt] = o[rt][dt] * c1 + o2 * c2;
                }
            }
        }
        __syncthreads();
    };
#pragma unroll
    for (int rt0 = 0; rt0 < RT; rt0 += MRT)
        for (int stride = 1; stride < SMALL_NW; stride <<= 1)
            merge_round((wave & (2 * stride - 1)) == stride, (wave & (2 * stride - 1)) == 0, (wave / (2 * stride)) & 3, rt0);
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
                    *reinterpret_cast<u32x2*>(op + 16 * dt + 4 * qd) =
                        pack_bf16x4(o[rt][dt][0] * inv, o[rt][dt][1] * inv, o[rt][dt][2] * inv, o[rt][dt][3] * inv);
            }
        }
    }
}

// ---------------------------------------------------------------- paged GQA attention with keys and values staged in LDS
// One workgroup per (sequence, KV head, pass of 64 query rows, key chunk c of C).  Key tiles of 64 at absolute
// positions 64 t; chunk c owns the tiles t = c, c + C, ..., so which tiles a workgroup sees does not depend on the
// launch's row count, and a tile past a row's position contributes exactly nothing to that row.  The 8 waves load a tile
// (keys [64][hd], values [hd][64]) from the pages into registers while the previous one is multiplied out of LDS, so the
// tile is read once for all 64 rows.  Wave w multiplies row tile w % 4 (16 rows) by the 32 keys w / 4 of the tile
// (S^T = K Q^T, O^T = V^T P^T with 16x16x32 MFMAs; the key rows are parked in the order that leaves a lane with 8
// consecutive keys, so the values come as one 16-byte LDS read per lane and tile of 16 dims); the two key halves of a
// row tile are merged through LDS at the end.  C == 1: the result goes to `att`; C > 1: unnormalised sums, running maxima and
// denominators go to part_o / part_ml for k_attn_merge, which adds the chunks in the order c = 0, 1, ...
struct AttnStagedArgs {
    AttnArgs a;
    float* part_o;            // [C][B * nq][H * hd]
    float* part_ml;           // [C][B * nq][H][2]
    int32_t C;
};
#define TA_KPAD 8             // bf16 elements of padding per key row / value row in LDS
#define TA_LDS_BYTES(hd) (2 * (64 * ((hd) + TA_KPAD) + (hd) * (64 + TA_KPAD)) * 2)
#define TA_MAX_BLOCKS 2048    // page ids of one sequence kept in LDS (sequences of up to 32,768 tokens)

template <int NKS>
__global__ __launch_bounds__(SMALL_THREADS) __attribute__((amdgpu_waves_per_eu(4, 4))) void k_attn_staged(AttnStagedArgs aa) {
    constexpr int hd = 32 * NKS, ndt = 2 * NKS;
    constexpr int KLD = hd + TA_KPAD, VLD = 64 + TA_KPAD;
    constexpr int LPT = hd / 64;                      // 16-byte loads per thread for the keys of a tile, and for the values
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    uint16_t* sK = reinterpret_cast<uint16_t*>(lds);                 // [2][64][KLD]
    uint16_t* sV = sK + 2 * 64 * KLD;                                // [2][hd][VLD]
    int32_t* s_bt = reinterpret_cast<int32_t*>(lds + TA_LDS_BYTES(hd));   // [max_blocks]: the sequence's page ids
    const AttnArgs& a = aa.a;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 15, qd = lane >> 4;
    const int rt = wave & 3, par = wave >> 2;
    const int Gq = a.H / a.Hkv, R = a.nq * Gq;
    const int b = blockIdx.x / a.Hkv, g = blockIdx.x % a.Hkv;
    const int r0 = blockIdx.y * 64, c = blockIdx.z, C = aa.C;
    const int nr = a.n_rows[b], p0 = a.pos0[b];
    const int32_t* bt = a.block_tab + (size_t)b * a.max_blocks;
    const size_t v_off = (size_t)a.Hkv * TASC_KV_BLOCK * hd;
    const int i_last = min(nr - 1, (min(r0 + 64, R) - 1) / Gq);
    const int L = i_last >= 0 ? p0 + i_last + 1 : 0;                 // keys this pass can see
    const int n_macro = (L + 63) / 64;
    const int n_my = n_macro > c ? (n_macro - c + C - 1) / C : 0;    // tiles c, c + C, ..
    // page ids into LDS once: a tile's fetch then starts without a dependent global load
    for (int i = tid; i < min(4 * n_macro, a.max_blocks); i += SMALL_THREADS) s_bt[i] = bt[i];
    __syncthreads();
    const int pg_last = min(4 * n_macro, a.max_blocks) - 1;

    // the wave's 16 query rows
    const int r = r0 + 16 * rt + m;
    const int qi_row = r / Gq, jq = r % Gq;
    const bool row_ok = r < R && qi_row < nr;
    const int qi = row_ok ? p0 + qi_row : -1;
    const bool tile_rows = r0 + 16 * rt < R;                         // the wave has rows at all
    bf16x8 qf[NKS];
    {
        const BF16* qp = a.q + (size_t)(b * a.nq + (row_ok ? qi_row : 0)) * a.H * hd + (size_t)(g * Gq + (row_ok ? jq : 0)) * hd;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            bf16x8 v = *reinterpret_cast<const bf16x8*>(qp + 32 * ks + 8 * qd);
            if (!row_ok) v = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            qf[ks] = v;
        }
    }
    float mx = -INFINITY, lsum = 0.f;
    f32x4 o[ndt];
#pragma unroll
    for (int dt = 0; dt < ndt; ++dt) o[dt] = f32x4{0, 0, 0, 0};

    // staging: thread -> LPT chunks of 16 bytes of the keys and LPT of the values, consecutive threads on consecutive
    // chunks of a page (a page holds 16 tokens: keys [16][hd] per KV head, values [hd][16])
    u32x4 rk[LPT], rv[LPT];
    auto fetch = [&](int idx) __attribute__((always_inline)) {
        const int t = c + min(idx, n_my - 1) * C;                    // past the end: the last tile again (unconditional loads)
#pragma unroll
        for (int u = 0; u < LPT; ++u) {
            const int q = tid + SMALL_THREADS * u;                   // chunk of the tile's keys: key q / (hd / 8), dims 8 (q % (hd / 8))
            const int key = q / (hd / 8), dch = q % (hd / 8);
            const int pg = min(4 * t + key / TASC_KV_BLOCK, pg_last);
            const BF16* page = a.kv_layer + (size_t)s_bt[pg] * a.page_elems;
            rk[u] = *reinterpret_cast<const u32x4*>(page + (size_t)(g * TASC_KV_BLOCK + key % TASC_KV_BLOCK) * hd + 8 * dch);
            // chunk of the tile's values: page q / (2 hd), dim (q % (2 hd)) / 2, tokens 8 (q % 2) ..
            const int vp = q / (2 * hd), dim = (q % (2 * hd)) / 2, half = q % 2;
            const int pgv = min(4 * t + vp, pg_last);
            const BF16* pagev = a.kv_layer + (size_t)s_bt[pgv] * a.page_elems;
            rv[u] = *reinterpret_cast<const u32x4*>(pagev + v_off + (size_t)(g * hd + dim) * TASC_KV_BLOCK + 8 * half);
        }
    };
    auto park = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < LPT; ++u) {
            const int q = tid + SMALL_THREADS * u;
            const int key = q / (hd / 8), dch = q % (hd / 8);
            // LDS row of a key: within its half of 32, keys 8 j .. 8 j + 3 go to rows 4 j .. 4 j + 3 and keys 8 j + 4 .. 8 j + 7
            // to rows 16 + 4 j ..: the two S^T tiles of a wave then leave lane group j with the scores of keys 8 j .. 8 j + 7,
            // the order in which the second product takes its k index, and a lane's 8 values are one 16-byte LDS read
            const int krow = (key & 32) + 16 * ((key >> 2) & 1) + 4 * ((key >> 3) & 3) + (key & 3);
            *reinterpret_cast<u32x4*>(sK + (size_t)(buf * 64 + krow) * KLD + 8 * dch) = rk[u];
            const int vp = q / (2 * hd), dim = (q % (2 * hd)) / 2, half = q % 2;
            *reinterpret_cast<u32x4*>(sV + (size_t)(buf * hd + dim) * VLD + TASC_KV_BLOCK * vp + 8 * half) = rv[u];
        }
    };
    auto multiply = [&](int buf, int t) __attribute__((always_inline)) {
        const int key0 = 64 * t + 32 * par;
        const uint16_t* kb = sK + (size_t)(buf * 64 + 32 * par + m) * KLD + 8 * qd;
        const uint16_t* vb = sV + (size_t)(buf * hd + m) * VLD + 32 * par + 8 * qd;
        f32x4 s0 = f32x4{0, 0, 0, 0}, s1 = f32x4{0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const bf16x8 k0 = *reinterpret_cast<const bf16x8*>(kb + 32 * ks);
            const bf16x8 k1 = *reinterpret_cast<const bf16x8*>(kb + (size_t)16 * KLD + 32 * ks);
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, qf[ks], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, qf[ks], s1, 0, 0, 0);
        }
        float sv[8];
        float tmax = -INFINITY;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int key = key0 + 8 * qd + u;                       // see the row order in park()
            const float sc = (u < 4 ? s0[u] : s1[u - 4]) * a.scale;
            sv[u] = (key <= qi) ? sc : -INFINITY;
            tmax = fmaxf(tmax, sv[u]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(mx, tmax);
        float psum = 0.f, corr = 1.f;
        uint32_t pw[4] = {0, 0, 0, 0};
        if (m_new != -INFINITY) {
            corr = __expf(mx - m_new);
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
        lsum = lsum * corr + psum;
        mx = m_new;
#pragma unroll
        for (int dt = 0; dt < ndt; ++dt) {
            const bf16x8 vf = *reinterpret_cast<const bf16x8*>(vb + (size_t)16 * dt * VLD);
            o[dt] *= corr;
            o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pk, o[dt], 0, 0, 0);
        }
    };
    if (n_my > 0) {
        fetch(0);
        park(0);
        __syncthreads();
        for (int idx = 0; idx < n_my; ++idx) {
            fetch(idx + 1);
            const int t = c + idx * C;
            if (tile_rows && 64 * t + 32 * par < L) multiply(idx & 1, t);
            park((idx + 1) & 1);
            __syncthreads();
        }
    }
    // merge the two key halves of every row tile: waves 4..7 hand theirs to waves 0..3 through LDS (the tile buffers are free)
    float* so = reinterpret_cast<float*>(lds) + (size_t)rt * (16 * hd + 32);
    if (par == 1) {
#pragma unroll
        for (int dt = 0; dt < ndt; ++dt) *reinterpret_cast<f32x4*>(so + (size_t)m * hd + 16 * dt + 4 * qd) = o[dt];
        if (qd == 0) { so[16 * hd + 2 * m] = mx; so[16 * hd + 2 * m + 1] = lsum; }
    }
    __syncthreads();
    if (par == 0 && tile_rows) {
        const float m2 = so[16 * hd + 2 * m], l2 = so[16 * hd + 2 * m + 1];
        const float mn = fmaxf(mx, m2);
        const float c1 = mn == -INFINITY ? 1.f : __expf(mx - mn);
        const float c2 = mn == -INFINITY ? 1.f : __expf(m2 - mn);
        lsum = lsum * c1 + l2 * c2;
        mx = mn;
#pragma unroll
        for (int dt = 0; dt < ndt; ++dt) {
            const f32x4 o2 = *reinterpret_cast<const f32x4*>(so + (size_t)m * hd + 16 * dt + 4 * qd);
            o[dt] = o[dt] * c1 + o2 * c2;
        }
        if (r < R && qi_row < a.nq) {
            const size_t row = (size_t)(b * a.nq + qi_row), head = (size_t)(g * Gq + jq);
            if (C == 1) {
                const float inv = lsum > 0.f ? 1.0f / lsum : 0.f;
                BF16* op = a.att + (row * a.H + head) * hd;
#pragma unroll
                for (int dt = 0; dt < ndt; ++dt)
                    *reinterpret_cast<u32x2*>(op + 16 * dt + 4 * qd) = pack_bf16x4(o[dt][0] * inv, o[dt][1] * inv, o[dt][2] * inv, o[dt][3] * inv);
            } else {
                const size_t rows_all = (size_t)a.B * a.nq;
                float* po = aa.part_o + (((size_t)c * rows_all + row) * a.H + head) * hd;
#pragma unroll
                for (int dt = 0; dt < ndt; ++dt) *reinterpret_cast<f32x4*>(po + 16 * dt + 4 * qd) = o[dt];
                if (qd == 0) {
                    float* pm = aa.part_ml + (((size_t)c * rows_all + row) * a.H + head) * 2;
                    pm[0] = mx;
                    pm[1] = lsum;
                }
            }
        }
    }
}

// adds the key chunks of k_attn_staged in the order c = 0, 1, ..: one thread per (row, head, 4 dims)
__global__ __launch_bounds__(256) void k_attn_merge(const float* __restrict__ part_o, const float* __restrict__ part_ml, int C, size_t rows_all,
                                                    int H, int hd, BF16* __restrict__ att) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t per_row = (size_t)H * hd / 4;
    if (idx >= rows_all * per_row) return;
    const size_t row = idx / per_row, rem = idx % per_row;
    const int head = (int)(rem / (hd / 4)), d4 = (int)(rem % (hd / 4));
    float mx = -INFINITY, lsum = 0.f;
    f32x4 o = f32x4{0, 0, 0, 0};
    for (int c = 0; c < C; ++c) {
        const size_t rh = ((size_t)c * rows_all + row) * H + head;
        const float m2 = part_ml[rh * 2], l2 = part_ml[rh * 2 + 1];
        const f32x4 o2 = *reinterpret_cast<const f32x4*>(part_o + rh * hd + 4 * d4);
        const float mn = fmaxf(mx, m2);
        const float c1 = mn == -INFINITY ? 1.f : __expf(mx - mn);
        const float c2 = mn == -INFINITY ? 1.f : __expf(m2 - mn);
        lsum = lsum * c1 + l2 * c2;
        o = o * c1 + o2 * c2;
        mx = mn;
    }
    const float inv = lsum > 0.f ? 1.0f / lsum : 0.f;
    *reinterpret_cast<u32x2*>(att + (row * H + head) * hd + 4 * d4) = pack_bf16x4(o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv);
}
