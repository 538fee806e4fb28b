// Small-batch (at most 16 rows) bf16 target forward as ONE persistent kernel.
//
// A verify step of k+1 <= 16 rows streams every weight once and does almost no arithmetic, so its
// time is set by launch and dependency latency, not by bandwidth or MFMA rate.  All phases of all
// layers therefore run inside one launch of `k_small_step`: the grid stays resident (one workgroup
// of 8 waves per compute unit at most) and moves from phase to phase through barriers.
//   0                  embedding gather
//   1 + 5l + 0         RMSNorm + fused q/k/v projection + RoPE + KV append
//   1 + 5l + 1         attention of the rows over the paged cache
//   1 + 5l + 2         output projection + residual
//   1 + 5l + 3         RMSNorm + gate/up projection + SwiGLU
//   1 + 5l + 4         down projection + residual
//   1 + 5L             final RMSNorm + LM head + bias + per-strip argmax
//   2 + 5L             argmax over strips (+ draft compare, accept length, KV rollback when verifying)
// The host may also launch any sub-range of phases (one phase per launch needs no barrier).
//
// The embedding and layer phases run on a "layer group" of workgroups; by default the group is one XCD's
// worth (32 workgroups whose ids are 8 apart), so that the ~150 dependent hand-overs of a step go through
// that XCD's L2 instead of through memory.  The LM head uses the whole grid.
//
// GEMMs use v_mfma_f32_16x16x32_bf16 with the WEIGHT tile as the A operand (16 output features x 32 k)
// and the 16 activation rows as the B operand, so a lane ends up with 4 consecutive output features
// of one row.  A workgroup takes all its work items of a phase in ONE pass (up to 6 weight tiles), the 8
// waves split the k-steps, and everything that does not depend on the previous phase (weight tiles, RoPE
// table entries, page addresses, the residual) is requested before the activations are staged, so that
// a phase costs about one memory round trip.  Every row's reduction order is fixed by the kernel (k-steps
// dealt round-robin to the 8 waves, partial sums added in wave order), independent of how many rows are
// valid, of how many workgroups share the phase and of the barrier flavour.
#pragma once
#include "kernels_generic.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// eight bf16 values given as four packed 32-bit words, as an MFMA operand (no trip through memory)
__device__ inline bf16x8 as_bf16x8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    return __builtin_bit_cast(bf16x8, u32x4{a, b, c, d});
}

// The kernel keeps its argument block in LDS, so the compiler cannot tell where a pointer read from it
// points and would use FLAT instructions for it; a flat access counts against the LDS counter as well as
// the vector-memory counter, so waiting for any LDS read would also wait for every weight load in flight.
// Every pointer to device memory is therefore converted once to the global address space (gptr) and all
// accesses go through typed global pointers (gld / gst).
#define GAS __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ GAS T* gptr(T* p) {
    return (GAS T*)p;
}
template <class V, class T>
__device__ __forceinline__ V gld(const GAS T* p) {
    return *reinterpret_cast<const GAS V*>(p);
}
template <class V, class T>
__device__ __forceinline__ void gst(GAS T* p, V v) {
    *reinterpret_cast<GAS V*>(p) = v;
}
// the wave's index within the workgroup, as a value the compiler knows to be uniform (scalar branches,
// not lane masks, around the loads it guards)
__device__ __forceinline__ int wave_id() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }

// Sum over the 64 lanes with DPP row operations (a few cycles each; the ds_bpermute path of __shfl_xor costs an LDS
// round trip per step).  The lanes are added in a fixed order, the same for every call.
__device__ __forceinline__ float wave_sum_dpp(float v) {
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, false));    // quad_perm [1,0,3,2]
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, false));    // quad_perm [2,3,0,1]
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, false));   // row_half_mirror
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, false));   // row_mirror
    // every lane now holds the sum of its row of 16; rows 0..3 are lanes 0-15, 16-31, 32-47, 48-63
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
    return (r0 + r1) + (r2 + r3);
}

#define SMALL_ROWS 16
#define SMALL_KC 1536                 // activation columns staged in LDS at a time
#define SMALL_KP (SMALL_KC + 8)       // padded LDS row length (elements)
#define SMALL_THREADS 512
#define SMALL_NW 8                    // waves per workgroup
#define SMALL_MAX_TILES 6             // weight tiles (16 output features each) a workgroup multiplies in one pass
#define SMALL_MAX_LAYERS 48           // layer-pointer table held in LDS
#define SMALL_MAX_BT 4096             // block-table entries held in LDS
#define SMALL_MAX_GROUP 64            // workgroups of the layer group (one wave polls their flags)

// dynamic LDS layout (bytes): staged activations, then the waves' partial tiles; the attention phase
// lays its merge slots (8 waves x 16 rows x head_dim floats, then 8 x 16 x (max, sum)) over both
#define SMALL_LDS_ACT 0
#define SMALL_LDS_RED (SMALL_ROWS * SMALL_KP * 2)                                   // 49408
#define SMALL_LDS_BYTES (SMALL_LDS_RED + SMALL_MAX_TILES * SMALL_NW * 64 * 16)      // + 49152 = 98560

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
    // Activations handed from phase to phase.  Every buffer is written ONCE per launch, before anything reads it: the
    // residual stream has a buffer per phase that updates it (x + i x_stride: i = 0 after the embedding, 2l + 1 after
    // layer l's attention block, 2l + 2 after its MLP), q / the attention output / the MLP activation a buffer per
    // layer.  A compute unit's L1 can therefore never hold a line from before the write (it is empty at launch), and
    // the readers use ordinary 16-byte loads even when the producers' stores only went as far as the XCD's L2.
    float* x;           // [2 L + 1][16][D]
    BF16* q;            // [L][16][H hd]
    BF16* att;          // [L][16][H hd]
    BF16* act;          // [L][16][F]
    size_t x_stride, q_stride, act_stride;     // elements
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
    // Barrier of the layer group (the embedding and layer phases): one arrival flag per member, holding
    // the number of the last barrier the member has reached; bar_epoch is that number before this launch.
    u32* bar_flags;         // [SMALL_MAX_GROUP]
    u32 bar_epoch;
    // Barrier of the whole grid (before the LM head and before the accept): a monotone arrival counter
    // plus the value it had when this launch began.
    u64* barb_counter;
    u64 barb_base;
    u32* bar_error;
    // Set of XCDs the layer group's workgroups found themselves on (bit per XCD id), gathered before the
    // group's first barrier and cleared by workgroup 0 at the end of the launch; xcd_local = 0 keeps the
    // group on agent-scope fences whatever the set says.
    u32* xcc_mask;
    int32_t xcd_local;
    // layer group: workgroups wg = lg_stride * j, j < lg_count <= SMALL_MAX_GROUP, run the layer phases; with XCD-local
    // barriers only the first lg_workers of them compute and the others prefetch (see prefetch_ahead)
    int32_t lg_stride, lg_count, lg_workers;
    // bias cursor table [n_sel][n_strips + 1]: entries of bias row sel_tok[r] with column < strip start
    int32_t* bias_ptr;
    // optional: wall-clock ticks [workgroup][phase][begin, end] of this launch (nullptr = off)
    u64* phase_ts;
    int32_t phase_ts_wgs;   // workgroups the buffer has room for
};

// The small tables every phase consults live in LDS and are handed to the phases directly (not through
// the argument block), so that reading them is an LDS read.
struct SmallTabs {
    const TascLayerW* layers;   // [n_layers]
    const int32_t* n_rows;      // [B]
    const int32_t* pos0;        // [B]
    const int32_t* block_tab;   // [B][max_blocks]
};

// ---------------------------------------------------------------- barriers
// Whole-grid barrier.  Every workgroup arrives once per barrier; the counter never resets (the host advances
// barb_base by barriers * workgroups per launch).  The workgroup barrier collects the waves' stores, then wave
// 0 alone publishes them (agent-scope release), arrives, waits, and acquires for the whole compute unit.
// The wait is bounded: on time-out the error flag is raised and every later barrier falls through, so the
// grid always drains.
__device__ __noinline__ void grid_sync(GAS u64* counter, u64 target, GAS u32* error, int sleep) {
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

// Barrier of the layer group: member `me` publishes `epoch` in its flag, the lanes of wave 0 watch one flag
// each until every member shows at least that epoch.  Same bounded wait as above.
//   local = false  wave 0 brackets the exchange with agent-scope release / acquire fences (L2 write-back and
//                  invalidate), which is right wherever the members run.
//   local = true   all members run on one XCD.  Its compute units share one L2 and their vector L1 caches
//                  write through, so a store is visible to the group as soon as the L2 has acknowledged it:
//                  every wave waits for its own stores, nobody writes the L2 back or invalidates anything.
//                  The readers' half of the contract: no address is read before it has been written in this
//                  launch (see SmallArgs), so no L1 holds a stale line.
__device__ __noinline__ void group_sync(GAS u32* flags, int me, int n, u32 epoch, GAS u32* error, bool local) {
    if (local) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        if (!local) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        if (lane == 0) __hip_atomic_store(flags + me, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        u32 spins = 0;
        for (;;) {
            u32 f = epoch;
            if (lane < n) f = __hip_atomic_load(flags + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (__all((int32_t)(f - epoch) >= 0)) break;
            __builtin_amdgcn_s_sleep(1);
            if ((++spins & 1023u) == 0) {
                if (__hip_atomic_load(error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) break;
                if (spins > (1u << 22)) {
                    if (lane == 0) __hip_atomic_fetch_or(error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
            }
        }
        if (!local) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    __syncthreads();
}

__device__ inline u32 xcc_id() {
    u32 v;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(v));
    return v & 15u;
}

// ---------------------------------------------------------------- staging of the 16 activation rows
// Wave w stages rows w and w + 8: s_act[r][0..D) = bf16(x[r] * g / sqrt(mean(x[r]^2) + eps)) for r < M, zero for
// r >= M.  One pass: the row stays in registers between the sum of squares and the scaling.  D <= 256 NTC.
// The loads are issued first (stage_normed_issue), so that a phase can queue them AHEAD of its weight loads: the
// memory pipeline serves a compute unit's requests in order, and the short L2 round trip of the activations must
// not wait behind ~100 KB of weights.  Every load is unconditional (rows and columns beyond the data are clamped
// and masked afterwards).
template <int NTC>
struct NormRegs {
    f32x4 v[2][NTC], g[NTC];
};
template <int NTC>
__device__ __forceinline__ void stage_normed_issue(const GAS float* x, const GAS float* g, const GAS int32_t* sel, int M, int D,
                                                   NormRegs<NTC>& rg) {
    const int lane = threadIdx.x & 63, wave = wave_id();
    const int nt = (D + 255) / 256;             // float4 columns a lane owns
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int r = wave + SMALL_NW * j;
        int src = r < M ? r : 0;
        if (sel) {
            src = sel[src];
            if (src < 0) src = 0;
        }
        const GAS float* xr = x + (size_t)src * D;
#pragma unroll
        for (int t = 0; t < NTC; ++t) {
            const int c = 4 * (lane + 64 * t);
            rg.v[j][t] = gld<f32x4>(xr + (c < D ? c : D - 4));        // unconditional, see load_w
        }
    }
#pragma unroll
    for (int t = 0; t < NTC; ++t) {
        const int c = 4 * (lane + 64 * t);
        rg.g[t] = gld<f32x4>(g + (c < D ? c : D - 4));
    }
}
template <int NTC>
__device__ __forceinline__ void stage_normed_finish(const NormRegs<NTC>& rg, int M, int D, float eps, uint16_t* s_act) {
    const int lane = threadIdx.x & 63, wave = wave_id();
    const int nt = (D + 255) / 256;
    float ss[2] = {0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
        for (int t = 0; t < NTC; ++t)
            if (t < nt) {
                const f32x4 v = rg.v[j][t];
                const float s4 = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
                ss[j] += 4 * (lane + 64 * t) < D ? s4 : 0.f;
            }
        ss[j] = wave_sum_dpp(ss[j]);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int r = wave + SMALL_NW * j;
        const float ri = __builtin_amdgcn_rsqf(ss[j] / (float)D + eps);      // v_rsq_f32: 1 ulp, one instruction
#pragma unroll
        for (int t = 0; t < NTC; ++t) {
            const int c = 4 * (lane + 64 * t);
            if (t < nt && c < D) {
                const f32x4 v = rg.v[j][t], gg = rg.g[t];
                u32x2 o = {0, 0};
                if (r < M) {
                    o[0] = f2bf_pair(v[0] * ri * gg[0], v[1] * ri * gg[1]);
                    o[1] = f2bf_pair(v[2] * ri * gg[2], v[3] * ri * gg[3]);
                }
                *reinterpret_cast<u32x2*>(s_act + r * SMALL_KP + c) = o;
            }
        }
    }
    __syncthreads();
}

// s_act[r][0..kw) = src[r][kc0..kc0+kw) (bf16 rows of length K), zero for r >= M; kw <= 256 NC.  Issue / finish as above.
template <int NC>
struct CopyRegs {
    bf16x8 v[NC];
};
template <int NC>
__device__ __forceinline__ void stage_copy_issue(const GAS BF16* src, int M, int K, int kc0, int kw, CopyRegs<NC>& rg) {
    const int per_row = kw / 8, total = SMALL_ROWS * per_row;
#pragma unroll
    for (int u = 0; u < NC; ++u) {
        const int idx = min((int)threadIdx.x + u * SMALL_THREADS, total - 1);
        const int r = idx / per_row, k = (idx % per_row) * 8;
        rg.v[u] = gld<bf16x8>(src + (size_t)(r < M ? r : 0) * K + kc0 + k);
    }
}
template <int NC>
__device__ __forceinline__ void stage_copy_finish(const CopyRegs<NC>& rg, int M, int kw, uint16_t* s_act) {
    const int per_row = kw / 8, total = SMALL_ROWS * per_row;
#pragma unroll
    for (int u = 0; u < NC; ++u) {
        const int idx = (int)threadIdx.x + u * SMALL_THREADS;
        if (idx < total) {
            const int r = idx / per_row, k = (idx % per_row) * 8;
            *reinterpret_cast<bf16x8*>(s_act + r * SMALL_KP + k) = r < M ? rg.v[u] : bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        }
    }
    __syncthreads();
}

// Requests one dword of every 128-byte line of the part-th of `parts` shares of [p, p + bytes): a software
// prefetch into the XCD's L2 of what a later phase will stream (a missed line is filled whole).  The caller folds
// the returned value into something it eventually stores, which is what keeps the loads alive.
__device__ __forceinline__ u32 touch_lines(const GAS void* p, size_t bytes, int part, int parts) {
    const int lines = (int)((bytes + 127) >> 7);
    const int per = (lines + parts - 1) / parts;
    const int l0 = per * part, l1 = min(l0 + per, lines);
    u32 s = 0;
    for (int lb = l0; lb < l1; lb += 4 * SMALL_THREADS) {
        u32 v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int l = min(lb + SMALL_THREADS * j + (int)threadIdx.x, l1 - 1);
            v[j] = gld<u32>(reinterpret_cast<const GAS u32*>(p) + (size_t)l * 32);
        }
        s ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    return s;
}

// ---------------------------------------------------------------- MFMA tiles, k-steps dealt to the 8 waves
// Weight fragments of the wave's k-steps (ks = wave, wave + 8, ... of a chunk of nks k-steps starting at column
// kc0) of NT tiles; wtile[t] points at tile row t's first fragment (fragment-order matrix, see TascLayerW).
template <int NT, int WKS>
__device__ __forceinline__ void load_w(const GAS BF16* (&wtile)[NT], int kc0, int nks, bf16x8 (&w)[NT][WKS]) {
    const int lane = threadIdx.x & 63, wave = wave_id();
    const size_t woff = (size_t)(kc0 / 32) * 512 + lane * 8;
    // No load sits under a condition (a conditional load ends in a register copy at the join, and the copy waits
    // for the data: the loads would complete one by one): a slot beyond the chunk reloads the wave's first k-step,
    // which its L1 already holds or is fetching.
#pragma unroll
    for (int u = 0; u < WKS; ++u) {
        const int ks = wave + SMALL_NW * u;
        const int ksc = ks < nks ? ks : (wave < nks ? wave : 0);
#pragma unroll
        for (int t = 0; t < NT; ++t) w[t][u] = gld<bf16x8>(wtile[t] + woff + (size_t)ksc * 512);
    }
}
template <int NT, int WKS>
__device__ __forceinline__ void mma_w(const bf16x8 (&w)[NT][WKS], int nks, const uint16_t* s_act, f32x4 (&acc)[NT]) {
    const int lane = threadIdx.x & 63, wave = wave_id();
    const int aoff = (lane & 15) * SMALL_KP + 8 * (lane >> 4);
#pragma unroll
    for (int u = 0; u < WKS; ++u) {
        const int ks = wave + SMALL_NW * u;
        if (ks < nks) {
            const bf16x8 b = *reinterpret_cast<const bf16x8*>(s_act + aoff + ks * 32);
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[t][u], b, acc[t], 0, 0, 0);
        }
    }
}
// The waves' partial tiles go to LDS; tile t is then summed in wave order by whichever wave calls sum_tile.
template <int NT>
__device__ __forceinline__ void put_partials(const f32x4 (&acc)[NT], f32x4* s_red) {
    const int lane = threadIdx.x & 63, wave = wave_id();
#pragma unroll
    for (int t = 0; t < NT; ++t) s_red[(t * SMALL_NW + wave) * 64 + lane] = acc[t];
    __syncthreads();
}
__device__ __forceinline__ f32x4 sum_tile(const f32x4* s_red, int t) {
    const int lane = threadIdx.x & 63;
    f32x4 s = s_red[(t * SMALL_NW) * 64 + lane];
#pragma unroll
    for (int w = 1; w < SMALL_NW; ++w) s += s_red[(t * SMALL_NW + w) * 64 + lane];
    return s;
}

__device__ __forceinline__ u32x2 pack_bf16x4(float a, float b, float c, float d) {
    return u32x2{f2bf_pair(a, b), f2bf_pair(c, d)};
}

// ---------------------------------------------------------------- phase: RMSNorm + q/k/v + RoPE + KV append
// Item = (head, block of 16 dims of the first half): the tile of dims e0..e0+16 and its RoPE partner
// tile of dims half+e0.. are computed together so the rotation happens in registers.  A pass takes NI items
// (wg, wg + nwg, ...); item j of the pass is finished (summed, rotated, stored) by wave j.
template <int NI, int WKS, class PF>
__device__ __forceinline__ u32 phase_qkv(const SmallArgs& a, const SmallTabs& tb, int layer, int wg, int nwg, uint16_t* s_act, f32x4* s_red,
                                         PF prefetch) {
    const TascLayerW& L = tb.layers[layer];
    const int half = a.hd / 2, eb_per_head = half / 16;
    const int n_items = (a.H + 2 * a.Hkv) * eb_per_head;
    const int lane = threadIdx.x & 63, wave = wave_id();
    const GAS BF16* W = gptr((const BF16*)L.wqkv_f);
    const size_t tile_row = (size_t)(a.D / 32) * 512;     // elements of one tile row (16 features, all k)
    GAS BF16* kv_layer = gptr(a.kv_pool) + (size_t)layer * a.kv_layer_stride;
    const GAS float* rope_cos = gptr(a.rope_cos);
    const GAS float* rope_sin = gptr(a.rope_sin);
    GAS BF16* q_out = gptr(a.q) + (size_t)layer * a.q_stride;
    const int nks = a.D / 32;
    const int m = lane & 15;
    u32 sink = 0;
    NormRegs<WKS> xr;                             // WKS = 3: D <= 768; WKS = 6: D <= 1536
    stage_normed_issue<WKS>(gptr(a.x) + (size_t)(2 * layer) * a.x_stride, gptr(L.g1), nullptr, a.M, a.D, xr);
    __builtin_amdgcn_s_barrier();                 // every wave's activation loads are queued before any weight load
    bool staged = false;
    for (int base = wg; base < n_items; base += nwg * NI) {
        const GAS BF16* wrow[2 * NI];
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int item = min(base + j * nwg, n_items - 1);       // a missing item repeats the last one and is dropped below
            const int head = item / eb_per_head, e0 = (item % eb_per_head) * 16;
            wrow[2 * j] = W + (size_t)((head * a.hd + e0) / 16) * tile_row;
            wrow[2 * j + 1] = W + (size_t)((head * a.hd + half + e0) / 16) * tile_row;
        }
        bf16x8 w[2 * NI][WKS];
        load_w<2 * NI, WKS>(wrow, 0, nks, w);
        // epilogue operands of the wave's own item that do not depend on the product; lanes without a row of
        // their own compute (and load) those of row 0 of the pass's first item, so that no load is predicated
        const int my_item = base + wave * nwg;
        const bool mine = wave < NI && my_item < n_items && m < a.M;
        const int it = mine ? my_item : base, mr = mine ? m : 0;
        const int head = it / eb_per_head, e0 = (it % eb_per_head) * 16;
        const int e = e0 + 4 * (lane >> 4);
        const int b = mr / a.nq, i = mr % a.nq;
        const bool active = mine && i < tb.n_rows[b];
        const int pos = tb.pos0[b] + i;
        const int tpos = pos < a.max_pos ? (pos > 0 ? pos : 0) : a.max_pos - 1;
        f32x4 cs = gld<f32x4>(rope_cos + (size_t)tpos * half + e);
        f32x4 sn = gld<f32x4>(rope_sin + (size_t)tpos * half + e);
        if (head >= a.H + a.Hkv) {                               // value heads are not rotated
            cs = f32x4{1, 1, 1, 1};
            sn = f32x4{0, 0, 0, 0};
        }
        GAS BF16* page = kv_layer;
        if (active && head >= a.H)
            page = kv_layer + (size_t)tb.block_tab[(size_t)b * a.max_blocks + pos / TASC_KV_BLOCK] * a.page_elems;
        if (!staged) {
            sink ^= prefetch();
            stage_normed_finish<WKS>(xr, a.M, a.D, a.eps, s_act);
            staged = true;
        }
        f32x4 acc[2 * NI];
#pragma unroll
        for (int t = 0; t < 2 * NI; ++t) acc[t] = f32x4{0, 0, 0, 0};
        mma_w<2 * NI, WKS>(w, nks, s_act, acc);
        put_partials<2 * NI>(acc, s_red);
        if (mine) {
            const f32x4 a0 = sum_tile(s_red, 2 * wave), a1 = sum_tile(s_red, 2 * wave + 1);
            float ra[4], rc[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                ra[u] = a0[u] * cs[u] - a1[u] * sn[u];
                rc[u] = a1[u] * cs[u] + a0[u] * sn[u];
            }
            if (head < a.H) {
                GAS BF16* qo = q_out + (size_t)m * a.H * a.hd + head * a.hd;
                gst(qo + e, pack_bf16x4(ra[0], ra[1], ra[2], ra[3]));
                gst(qo + half + e, pack_bf16x4(rc[0], rc[1], rc[2], rc[3]));
            } else if (active) {
                const int slot = pos % TASC_KV_BLOCK;
                if (head < a.H + a.Hkv) {
                    const int g = head - a.H;
                    GAS BF16* kp = page + (size_t)(g * TASC_KV_BLOCK + slot) * a.hd;
                    gst(kp + e, pack_bf16x4(ra[0], ra[1], ra[2], ra[3]));
                    gst(kp + half + e, pack_bf16x4(rc[0], rc[1], rc[2], rc[3]));
                } else {
                    const int g = head - a.H - a.Hkv;
                    GAS BF16* vt = page + (size_t)a.Hkv * TASC_KV_BLOCK * a.hd + (size_t)g * a.hd * TASC_KV_BLOCK;
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        gst(vt + (size_t)(e + u) * TASC_KV_BLOCK + slot, f2bf(a0[u]));
                        gst(vt + (size_t)(half + e + u) * TASC_KV_BLOCK + slot, f2bf(a1[u]));
                    }
                }
            }
        }
        __syncthreads();                      // s_red is free again
    }
    return sink;
}

// ---------------------------------------------------------------- phases: projections with residual / SwiGLU
// x[m][n] += sum_k src[m][k] W[n][k]    (output projection, down projection); item = 16 output features
template <int NI, int WKS, class PF>
__device__ __forceinline__ u32 phase_proj_resid(const SmallArgs& a, const GAS BF16* W, const GAS BF16* src, const GAS float* x_in,
                                                GAS float* x_out, int N, int K, int wg, int nwg, uint16_t* s_act, f32x4* s_red, PF prefetch) {
    const int lane = threadIdx.x & 63, wave = wave_id();
    const int n_items = N / 16;
    const int m = lane & 15;
    u32 sink = 0;
    CopyRegs<WKS> cr;                             // WKS = 3: chunks of at most 768 columns; WKS = 6: 1536
    stage_copy_issue<WKS>(src, a.M, K, 0, min(SMALL_KC, K), cr);
    __builtin_amdgcn_s_barrier();                 // every wave's activation loads are queued before any weight load
    bool staged = false;
    for (int base = wg; base < n_items; base += nwg * NI) {
        const GAS BF16* wrow[NI];
#pragma unroll
        for (int j = 0; j < NI; ++j) wrow[j] = W + (size_t)min(base + j * nwg, n_items - 1) * (K / 32) * 512;
        const int my_item = base + wave * nwg;
        const bool mine = wave < NI && my_item < n_items && m < a.M;
        const size_t xoff = (size_t)(mine ? m : 0) * N + (mine ? my_item : 0) * 16 + 4 * (lane >> 4);
        f32x4 xv = {0, 0, 0, 0};
        f32x4 acc[NI];
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[j] = f32x4{0, 0, 0, 0};
        for (int kc0 = 0; kc0 < K; kc0 += SMALL_KC) {
            const int kw = min(SMALL_KC, K - kc0), nks = kw / 32;
            bf16x8 w[NI][WKS];
            load_w<NI, WKS>(wrow, kc0, nks, w);
            if (kc0 == 0) xv = gld<f32x4>(x_in + xoff);       // unpredicated: lanes without an output read row 0
            if (!staged) {
                sink ^= prefetch();
                stage_copy_finish<WKS>(cr, a.M, kw, s_act);
                staged = true;
            } else if (K > SMALL_KC) {
                __syncthreads();
                stage_copy_issue<WKS>(src, a.M, K, kc0, kw, cr);
                stage_copy_finish<WKS>(cr, a.M, kw, s_act);
            }
            mma_w<NI, WKS>(w, nks, s_act, acc);
        }
        put_partials<NI>(acc, s_red);
        if (mine) {
            xv += sum_tile(s_red, wave);
            gst(x_out + xoff, xv);
        }
        __syncthreads();
    }
    return sink;
}

// act[m][f] = silu(h W_gate[f]) * (h W_up[f]); item = 16 features (gate rows then up rows, interleaved per 16)
template <int NI, int WKS, class PF>
__device__ __forceinline__ u32 phase_gate_up(const SmallArgs& a, const SmallTabs& tb, int layer, int wg, int nwg, uint16_t* s_act, f32x4* s_red,
                                             PF prefetch) {
    const TascLayerW& L = tb.layers[layer];
    const int lane = threadIdx.x & 63, wave = wave_id();
    const GAS BF16* Wgu = gptr((const BF16*)L.wgu_f);
    const size_t tile_row = (size_t)(a.D / 32) * 512;
    GAS BF16* act = gptr(a.act) + (size_t)layer * a.act_stride;
    const int nks = a.D / 32;
    const int n_items = a.F / 16;
    const int m = lane & 15;
    u32 sink = 0;
    NormRegs<WKS> xr;
    stage_normed_issue<WKS>(gptr(a.x) + (size_t)(2 * layer + 1) * a.x_stride, gptr(L.g2), nullptr, a.M, a.D, xr);
    __builtin_amdgcn_s_barrier();                 // every wave's activation loads are queued before any weight load
    bool staged = false;
    for (int base = wg; base < n_items; base += nwg * NI) {
        const GAS BF16* wrow[2 * NI];
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const GAS BF16* Wi = Wgu + (size_t)min(base + j * nwg, n_items - 1) * 2 * tile_row;
            wrow[2 * j] = Wi;
            wrow[2 * j + 1] = Wi + tile_row;
        }
        bf16x8 w[2 * NI][WKS];
        load_w<2 * NI, WKS>(wrow, 0, nks, w);
        if (!staged) {
            sink ^= prefetch();
            stage_normed_finish<WKS>(xr, a.M, a.D, a.eps, s_act);
            staged = true;
        }
        f32x4 acc[2 * NI];
#pragma unroll
        for (int t = 0; t < 2 * NI; ++t) acc[t] = f32x4{0, 0, 0, 0};
        mma_w<2 * NI, WKS>(w, nks, s_act, acc);
        put_partials<2 * NI>(acc, s_red);
        const int my_item = base + wave * nwg;
        if (wave < NI && my_item < n_items && m < a.M) {
            const f32x4 gt = sum_tile(s_red, 2 * wave), up = sum_tile(s_red, 2 * wave + 1);
            float o[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) o[u] = gt[u] / (1.0f + __expf(-gt[u])) * up[u];
            gst(act + (size_t)m * a.F + my_item * 16 + 4 * (lane >> 4), pack_bf16x4(o[0], o[1], o[2], o[3]));
        }
        __syncthreads();
    }
    return sink;
}

// ---------------------------------------------------------------- phase: attention
// Item = (sequence b, query head h): the sequence's rows are the 16 columns of one MFMA tile.  Keys are
// visited in tiles of 32 at absolute positions; tile t belongs to wave t mod 8.  S^T = K Q^T and O^T = V^T P^T
// are both MFMA products whose lane layouts chain without a transpose: after S^T a lane holds, for query row
// i = lane mod 16, the scores of keys {4q..4q+3} of each 16-key page (q = lane / 16), which is exactly the
// B-operand slot of the second product when its A operand (V^T) is loaded with the same key permutation.
// All loads of a group of TG tiles are issued together and unconditionally (tiles beyond the sequence repeat
// the last one and are skipped by the arithmetic).  The waves' partial (max, sum, O) meet in LDS and are
// combined in wave order by all threads at once.
template <int NKS>
__device__ __forceinline__ void phase_attn(const SmallArgs& a, const SmallTabs& tb, int layer, int wg, int nwg, float* s_buf) {
    const int lane = threadIdx.x & 63, wave = wave_id();
    constexpr int hd = 32 * NKS, ndt = 2 * NKS;
    constexpr int TG = NKS <= 2 ? 3 : 1;
    const int Gq = a.H / a.Hkv;
    const GAS BF16* kv_layer = gptr(a.kv_pool) + (size_t)layer * a.kv_layer_stride;
    const GAS BF16* q_in = gptr(a.q) + (size_t)layer * a.q_stride;
    GAS BF16* att_out = gptr(a.att) + (size_t)layer * a.q_stride;
    const size_t v_off = (size_t)a.Hkv * TASC_KV_BLOCK * hd;
    const int m = lane & 15, qd = lane >> 4;
    float* slot_o = s_buf;                                   // [wave][row][hd]
    float* slot_ml = s_buf + SMALL_NW * SMALL_ROWS * hd;     // [wave][row][max, sum]
    for (int item = wg; item < a.B * a.H; item += nwg) {
        const int b = item / a.H, h = item % a.H, g = h / Gq;
        const int nr = tb.n_rows[b], p0 = tb.pos0[b];
        const int32_t* bt = tb.block_tab + (size_t)b * a.max_blocks;
        const int L = p0 + nr;                               // keys 0 .. L-1 exist
        const int n_tiles = (L + 31) / 32;
        // Q fragments (B operand): query row m, dims 32 ks + 8 qd ..
        const bool okq = m < nr;
        const int qi = okq ? p0 + m : -1;                    // position of the query row, -1 = no such row
        const GAS BF16* qp = q_in + (size_t)(b * a.nq + (okq ? m : 0)) * a.H * hd + (size_t)h * hd;
        bf16x8 qf[NKS];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const bf16x8 v = gld<bf16x8>(qp + 32 * ks + 8 * qd);
            qf[ks] = okq ? v : bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        }
        float mx = -INFINITY, lsum = 0.f;
        f32x4 o[ndt];                                        // O^T tiles: lane holds dims 16 dt + 4 qd .. +4 of row m
#pragma unroll
        for (int dt = 0; dt < ndt; ++dt) o[dt] = f32x4{0, 0, 0, 0};
        for (int tg = wave; tg < n_tiles; tg += SMALL_NW * TG) {
            bf16x8 kf0[TG][NKS], kf1[TG][NKS];
            bf16x8 vf[TG][ndt];
#pragma unroll
            for (int j = 0; j < TG; ++j) {
                const int t = min(tg + j * SMALL_NW, n_tiles - 1);
                const int key0 = t * 32;
                // the two pages of this tile (the second may lie beyond the sequence: then the first again)
                const GAS BF16* pg0 = kv_layer + (size_t)bt[key0 / TASC_KV_BLOCK] * a.page_elems;
                const GAS BF16* pg1 = kv_layer + (size_t)bt[key0 / TASC_KV_BLOCK + (key0 + 16 < L ? 1 : 0)] * a.page_elems;
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) {
                    kf0[j][ks] = gld<bf16x8>(pg0 + (size_t)(g * TASC_KV_BLOCK + m) * hd + 32 * ks + 8 * qd);
                    kf1[j][ks] = gld<bf16x8>(pg1 + (size_t)(g * TASC_KV_BLOCK + m) * hd + 32 * ks + 8 * qd);
                }
#pragma unroll
                for (int dt = 0; dt < ndt; ++dt) {
                    const u32x2 h0 = gld<u32x2>(pg0 + v_off + (size_t)(g * hd + 16 * dt + m) * TASC_KV_BLOCK + 4 * qd);
                    const u32x2 h1 = gld<u32x2>(pg1 + v_off + (size_t)(g * hd + 16 * dt + m) * TASC_KV_BLOCK + 4 * qd);
                    vf[j][dt] = as_bf16x8(h0[0], h0[1], h1[0], h1[1]);
                }
            }
#pragma unroll
            for (int j = 0; j < TG; ++j) {
                const int t = tg + j * SMALL_NW;
                if (t < n_tiles) {
                    const int key0 = t * 32;
                    // S^T tiles: A = K rows (key = m within the page), B = Q
                    f32x4 s0 = {0, 0, 0, 0}, s1 = {0, 0, 0, 0};
#pragma unroll
                    for (int ks = 0; ks < NKS; ++ks) {
                        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf0[j][ks], qf[ks], s0, 0, 0, 0);
                        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf1[j][ks], qf[ks], s1, 0, 0, 0);
                    }
                    // online softmax per query row; the lane holds keys key0 + 4qd + u (u<4) and key0 + 16 + 4qd + u
                    float sv[8];
                    float tmax = -INFINITY;
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int key = key0 + (u < 4 ? 4 * qd + u : 16 + 4 * qd + (u - 4));
                        const float sc = (u < 4 ? s0[u] : s1[u - 4]) * a.scale;
                        sv[u] = (key <= qi) ? sc : -INFINITY;      // causal; also hides keys beyond the sequence
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
                            psum += bf2f(pb);                      // the sum uses the rounded weights the product uses
                        }
                    }
                    const bf16x8 pk = as_bf16x8(pw[0], pw[1], pw[2], pw[3]);
                    psum += __shfl_xor(psum, 16);
                    psum += __shfl_xor(psum, 32);
                    lsum = lsum * corr + psum;
                    mx = m_new;
                    // O^T += V^T P^T
#pragma unroll
                    for (int dt = 0; dt < ndt; ++dt) {
                        o[dt] *= corr;
                        o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[j][dt], pk, o[dt], 0, 0, 0);
                    }
                }
            }
        }
        // the waves' partial results meet in LDS ...
#pragma unroll
        for (int dt = 0; dt < ndt; ++dt)
            *reinterpret_cast<f32x4*>(slot_o + (size_t)(wave * SMALL_ROWS + m) * hd + 16 * dt + 4 * qd) = o[dt];
        if (qd == 0) {
            slot_ml[(wave * SMALL_ROWS + m) * 2 + 0] = mx;
            slot_ml[(wave * SMALL_ROWS + m) * 2 + 1] = lsum;
        }
        __syncthreads();
        // ... and thread (row r, dims d0 .. d0 + PER) combines them in wave order
        {
            constexpr int PER = hd / 32;
            const int r = threadIdx.x / 32, d0 = (threadIdx.x % 32) * PER;
            float mall = -INFINITY;
#pragma unroll
            for (int w = 0; w < SMALL_NW; ++w) mall = fmaxf(mall, slot_ml[(w * SMALL_ROWS + r) * 2]);
            float den = 0.f, num[PER];
#pragma unroll
            for (int u = 0; u < PER; ++u) num[u] = 0.f;
#pragma unroll
            for (int w = 0; w < SMALL_NW; ++w) {
                const float mw = slot_ml[(w * SMALL_ROWS + r) * 2];
                const float c = mw == -INFINITY ? 0.f : __expf(mw - mall);
                den += c * slot_ml[(w * SMALL_ROWS + r) * 2 + 1];
#pragma unroll
                for (int u = 0; u < PER; ++u) num[u] += c * slot_o[(size_t)(w * SMALL_ROWS + r) * hd + d0 + u];
            }
            if (r < nr) {
                const float inv = den > 0.f ? 1.0f / den : 0.f;
                GAS BF16* op = att_out + (size_t)(b * a.nq + r) * a.H * hd + (size_t)h * hd + d0;
                if constexpr (PER == 1) {
                    gst(op, f2bf(num[0] * inv));
                } else if constexpr (PER == 2) {
                    gst(op, (uint32_t)f2bf(num[0] * inv) | ((uint32_t)f2bf(num[1] * inv) << 16));
                } else {
                    gst(op, pack_bf16x4(num[0] * inv, num[1] * inv, num[2] * inv, num[3] * inv));
                }
            }
        }
        __syncthreads();                      // the slots are free again (next item, or the next phase's staging)
    }
}

// ---------------------------------------------------------------- phase: final norm + LM head + bias + strip argmax
// Item = one strip of TASC_LM_STRIP = 128 vocabulary rows: 8 tiles, one per wave, each over the whole k.
__device__ __forceinline__ void phase_lmhead(const SmallArgs& a, int wg, int nwg, uint16_t* s_act, float* s_best) {
    const int lane = threadIdx.x & 63, wave = wave_id();
    const int m = lane & 15, qd = lane >> 4;
    int32_t* s_besti = reinterpret_cast<int32_t*>(s_best + SMALL_NW * SMALL_ROWS);
    const int nks = a.D / 32;
    const int aoff = m * SMALL_KP + 8 * qd;
    const GAS BF16* lm_head = gptr(a.lm_head);              // fragment order, rows padded to a multiple of 16
    const GAS int32_t* sel_tok = gptr(a.sel_tok);
    const GAS int32_t* bias_ptr = gptr(a.bias_ptr);
    const bool has_bias = a.bias.rowptr != nullptr;
    const GAS int64_t* b_rowptr = gptr(a.bias.rowptr);
    const GAS int32_t* b_col = gptr(a.bias.col);
    const GAS float* b_val = gptr(a.bias.val);
    const GAS float* b_base = gptr(a.bias.base);
    const bool dbg = a.logits_dbg != nullptr;
    GAS float* logits_dbg = gptr(a.logits_dbg);
    GAS float* part_val = gptr(a.part_val);
    GAS int32_t* part_idx = gptr(a.part_idx);
    bool staged = false;
    for (int strip = wg; strip < a.n_strips; strip += nwg) {
        const int v0 = strip * TASC_LM_STRIP + wave * 16;
        const bool live = v0 < a.V;
        const GAS BF16* wrow = lm_head + (size_t)(live ? v0 / 16 : 0) * nks * 512 + lane * 8;
        // first group of weight fragments and the lane's bias cursor, before the activations are staged
        constexpr int WG_KS = 18;
        bf16x8 w[WG_KS];
#pragma unroll
        for (int u = 0; u < WG_KS; ++u)
            w[u] = gld<bf16x8>(wrow + (size_t)min(u, nks - 1) * 512);   // unconditional, see load_w
        const bool own = live && m < a.n_sel;
        int64_t bp = 0, be = 0;
        float base = 0.f;
        if (own && has_bias) {
            const int u = sel_tok[m];
            const int64_t r0 = b_rowptr[u];
            bp = r0 + bias_ptr[(size_t)m * (a.n_strips + 1) + strip];
            be = r0 + bias_ptr[(size_t)m * (a.n_strips + 1) + strip + 1];
            base = b_base[u];
        }
        if (!staged) {
            NormRegs<6> xr;
            stage_normed_issue<6>(gptr(a.x) + (size_t)(2 * a.n_layers) * a.x_stride, gptr(a.gf), gptr(a.sel_rows), a.n_sel, a.D, xr);
            stage_normed_finish<6>(xr, a.n_sel, a.D, a.eps, s_act);
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
                for (int u = 0; u < WG_KS; ++u) w[u] = gld<bf16x8>(wrow + (size_t)min(ks0 + WG_KS + u, nks - 1) * 512);
            }
        }
        float best = -INFINITY;
        int32_t best_i = 0x7FFFFFFF;
        if (own) {
            if (has_bias) {
                // the lane's first feature inside the row's sorted list: a binary search, not a walk from the strip's start
                // (a frequent token has tens of seen successors per strip, and every step is a dependent load)
                const int c0 = v0 + 4 * qd;
                int64_t lo = bp, hi = be;
                while (lo < hi) {
                    const int64_t mid = (lo + hi) >> 1;
                    if (b_col[mid] < c0) lo = mid + 1; else hi = mid;
                }
                bp = lo;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = v0 + 4 * qd + u;
                if (c >= a.V) continue;                            // padding rows of a ragged last tile
                float z = acc[u];
                if (has_bias) {
                    while (bp < be && b_col[bp] < c) ++bp;
                    z += (bp < be && b_col[bp] == c) ? b_val[bp] : base;
                }
                if (dbg) logits_dbg[(size_t)m * a.V + c] = z;
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
            part_val[(size_t)row * a.n_strips + strip] = bv;
            part_idx[(size_t)row * a.n_strips + strip] = bi;
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------- phase: argmax over strips, accept, rollback
__device__ __forceinline__ void phase_accept(const SmallArgs& al, int32_t* s_amax) {
    const int lane = threadIdx.x & 63, wave = wave_id();
    // a view of the arguments this phase uses, pointers pinned to global memory
    const GAS float* part_val = gptr(al.part_val);
    const GAS int32_t* part_idx = gptr(al.part_idx);
    GAS int32_t* amax = gptr(al.amax);
    GAS int32_t* n_tok = gptr(al.n_tok);
    GAS int32_t* n_emit = gptr(al.n_emit);
    const GAS int32_t* drafts = gptr(al.drafts);
    GAS int32_t* tokens = gptr(al.tokens);
    GAS int32_t* cached = gptr(al.cached);
    GAS u64* counters = gptr(al.counters);
    GAS int32_t* accept_len = gptr(al.accept_len);
    GAS int32_t* emitted = gptr(al.emitted);
    GAS int32_t* trace_step = gptr(al.trace_step);
    const bool has_accept_len = al.accept_len != nullptr, has_emitted = al.emitted != nullptr, has_trace = al.trace_step != nullptr;
    const int n_sel = al.n_sel, n_strips = al.n_strips, k = al.k, B = al.B, max_new = al.max_new, max_len = al.max_len;
    for (int r = wave; r < n_sel; r += SMALL_NW) {
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
        if (lane == 0) {
            bi = bi == 0x7FFFFFFF ? 0 : bi;
            s_amax[r] = bi;
            amax[r] = bi;
        }
    }
    __syncthreads();
    if (k < 0) return;
    const int b = threadIdx.x, nq = k + 1;
    if (b >= B) return;
    const int N = n_tok[b];
    const bool frozen = n_emit[b] >= max_new;
    int mlen = 0;
    if (!frozen) {
        while (mlen < k && drafts[b * k + mlen] == s_amax[b * nq + mlen]) ++mlen;
        GAS int32_t* seq = tokens + (size_t)b * max_len;
        for (int i = 0; i < mlen; ++i) seq[N + i] = drafts[b * k + i];
        seq[N + mlen] = s_amax[b * nq + mlen];
        n_tok[b] = N + mlen + 1;
        cached[b] += mlen + 1;
        const int e = n_emit[b] + mlen + 1;
        n_emit[b] = e;
        if (e >= max_new) __hip_atomic_fetch_add(&counters[0], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add(&counters[3], (u64)mlen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add(&counters[4], (u64)k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add(&counters[8 + mlen], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (has_accept_len) accept_len[b] = mlen;
    if (has_emitted)
        for (int i = 0; i < nq; ++i)
            emitted[b * nq + i] = frozen ? -1 : (i < mlen ? drafts[b * k + i] : (i == mlen ? s_amax[b * nq + mlen] : -1));
    if (has_trace) {
        GAS int32_t* t = trace_step + (size_t)b * (2 * k + 3);
        t[0] = N;
        for (int i = 0; i < k; ++i) t[1 + i] = drafts[b * k + i];
        for (int i = 0; i < nq; ++i) t[1 + k + i] = s_amax[b * nq + i];
        t[2 * k + 2] = frozen ? -1 : mlen;
    }
    if (b == 0) __hip_atomic_fetch_add(&counters[2], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---------------------------------------------------------------- the persistent step kernel
// cursor table of the LM-head bias: for every LM-head row r and strip s, how many entries of bias row
// sel_tok[r] have a column below the strip's first column (s = n_strips: all of them)
__device__ inline void build_bias_ptr(const SmallArgs& a, int worker, int n_workers) {
    if (!a.bias.rowptr || a.n_sel <= 0) return;
    const int per_row = a.n_strips + 1;
    const GAS int32_t* sel_tok = gptr(a.sel_tok);
    const GAS int64_t* b_rowptr = gptr(a.bias.rowptr);
    const GAS int32_t* b_col = gptr(a.bias.col);
    GAS int32_t* bias_ptr = gptr(a.bias_ptr);
    for (int idx = worker * SMALL_THREADS + threadIdx.x; idx < a.n_sel * per_row; idx += n_workers * SMALL_THREADS) {
        const int r = idx / per_row, st = idx % per_row;
        const int u = sel_tok[r];
        const int64_t r0 = b_rowptr[u];
        int64_t lo = r0, hi = b_rowptr[u + 1];
        const int c_first = st * TASC_LM_STRIP;
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if (b_col[mid] < c_first) lo = mid + 1; else hi = mid;
        }
        bias_ptr[idx] = (int32_t)(lo - r0);
    }
}

// With XCD-local barriers the layer group splits into workers, which run the phases, and prefetchers, which
// during phase `ph` pull what the NEXT phase will stream (weights, norm gains, RoPE rows, cached keys and values)
// from memory into the XCD's L2, one dword per 128-byte line.  A compute unit serves its memory requests in
// order and can keep only so many misses in flight, so a unit that streams ~100 KB of cold weights delays
// every later request of its own by microseconds; the workers never miss (what they read was fetched by a
// prefetcher or written by a worker), and the prefetchers have nothing else to do.  L2 capacity (4 MB) bounds
// the look-ahead to one phase.
__device__ __forceinline__ u32 touch_kv(const SmallArgs& a, const SmallTabs& tb, int layer, int part, int parts) {
    const GAS BF16* kv_layer = gptr(a.kv_pool) + (size_t)layer * a.kv_layer_stride;
    const int lpp = (int)(a.page_elems * 2 / 128);                 // 128-byte lines per page
    int total = 0;
    for (int b = 0; b < a.B; ++b) total += (tb.pos0[b] + tb.n_rows[b] + TASC_KV_BLOCK - 1) / TASC_KV_BLOCK * lpp;
    u32 s = 0;
    for (int f0 = part * SMALL_THREADS; f0 < total; f0 += parts * SMALL_THREADS) {
        int rem = min(f0 + (int)threadIdx.x, total - 1), b = 0;
        for (; b < a.B - 1; ++b) {
            const int n = (tb.pos0[b] + tb.n_rows[b] + TASC_KV_BLOCK - 1) / TASC_KV_BLOCK * lpp;
            if (rem < n) break;
            rem -= n;
        }
        const int page = tb.block_tab[(size_t)b * a.max_blocks + rem / lpp];
        s ^= gld<u32>(reinterpret_cast<const GAS u32*>(kv_layer + (size_t)page * a.page_elems) + (size_t)(rem % lpp) * 32);
    }
    return s;
}
// norm gains of layer `layer` (which = 0: before attention, 1: before the MLP) and, for which = 0, the RoPE rows
__device__ __forceinline__ u32 touch_small(const SmallArgs& a, const SmallTabs& tb, int layer, int which) {
    const TascLayerW& L = tb.layers[layer];
    u32 s = touch_lines(gptr(which ? L.g2 : L.g1), (size_t)a.D * 4, 0, 1);
    if (which == 0) {
        const int half = a.hd / 2, m = min((int)threadIdx.x, a.M - 1);
        const int b = m / a.nq, pos = tb.pos0[b] + m % a.nq;
        const int tpos = pos < a.max_pos ? (pos > 0 ? pos : 0) : a.max_pos - 1;
        s ^= gld<u32>(reinterpret_cast<const GAS u32*>(gptr(a.rope_cos) + (size_t)tpos * half));
        s ^= gld<u32>(reinterpret_cast<const GAS u32*>(gptr(a.rope_sin) + (size_t)tpos * half));
        if (half * 4 > 128) {
            s ^= gld<u32>(reinterpret_cast<const GAS u32*>(gptr(a.rope_cos) + (size_t)tpos * half + 32));
            s ^= gld<u32>(reinterpret_cast<const GAS u32*>(gptr(a.rope_sin) + (size_t)tpos * half + 32));
        }
    }
    return s;
}
__device__ __forceinline__ u32 prefetch_ahead(const SmallArgs& a, const SmallTabs& tb, int ph, int part, int parts) {
    const size_t qkv_bytes = (size_t)(a.H + 2 * a.Hkv) * a.hd * a.D * 2;
    if (ph == 0) return touch_lines(gptr(tb.layers[0].wqkv_f), qkv_bytes, part, parts) ^ (part == 0 ? touch_small(a, tb, 0, 0) : 0u);
    const int layer = (ph - 1) / 5, sub = (ph - 1) % 5;
    const TascLayerW& L = tb.layers[layer];
    if (sub == 0) return touch_kv(a, tb, layer, part, parts);
    if (sub == 1) return touch_lines(gptr(L.wo_f), (size_t)a.D * a.H * a.hd * 2, part, parts) ^ (part == 0 ? touch_small(a, tb, layer, 1) : 0u);
    if (sub == 2) return touch_lines(gptr(L.wgu_f), (size_t)2 * a.F * a.D * 2, part, parts);
    if (sub == 3) return touch_lines(gptr(L.wd_f), (size_t)a.D * a.F * 2, part, parts);
    if (layer + 1 < a.n_layers)
        return touch_lines(gptr(tb.layers[layer + 1].wqkv_f), qkv_bytes, part, parts) ^ (part == 0 ? touch_small(a, tb, layer + 1, 0) : 0u);
    return 0;
}

// How many items a workgroup takes per pass: all of its share if the registers allow (NI * tiles * WKS <= 18
// weight fragments per lane), else one at a time.
template <int WKS, class PF>
__device__ __forceinline__ u32 run_qkv(const SmallArgs& a, const SmallTabs& tb, int layer, int lw, int lnw, uint16_t* s_act, f32x4* s_red, PF pf) {
    if constexpr (WKS == 3) {
        const int n_items = (a.H + 2 * a.Hkv) * (a.hd / 32);
        const int share = (n_items + lnw - 1) / lnw;
        if (share >= 3) return phase_qkv<3, 3>(a, tb, layer, lw, lnw, s_act, s_red, pf);
        if (share == 2) return phase_qkv<2, 3>(a, tb, layer, lw, lnw, s_act, s_red, pf);
    }
    return phase_qkv<1, WKS>(a, tb, layer, lw, lnw, s_act, s_red, pf);
}
template <int WKS, class PF>
__device__ __forceinline__ u32 run_gate_up(const SmallArgs& a, const SmallTabs& tb, int layer, int lw, int lnw, uint16_t* s_act, f32x4* s_red,
                                           PF pf) {
    if constexpr (WKS == 3) {
        const int share = (a.F / 16 + lnw - 1) / lnw;
        if (share >= 3) return phase_gate_up<3, 3>(a, tb, layer, lw, lnw, s_act, s_red, pf);
        if (share == 2) return phase_gate_up<2, 3>(a, tb, layer, lw, lnw, s_act, s_red, pf);
    }
    return phase_gate_up<1, WKS>(a, tb, layer, lw, lnw, s_act, s_red, pf);
}
template <class PF>
__device__ __forceinline__ u32 run_proj(const SmallArgs& a, const GAS BF16* W, const GAS BF16* src, const GAS float* x_in, GAS float* x_out,
                                        int N, int K, int lw, int lnw, uint16_t* s_act, f32x4* s_red, PF pf) {
    const int share = (N / 16 + lnw - 1) / lnw;
    if (K <= 768) {
        if (share >= 3) return phase_proj_resid<3, 3>(a, W, src, x_in, x_out, N, K, lw, lnw, s_act, s_red, pf);
        if (share == 2) return phase_proj_resid<2, 3>(a, W, src, x_in, x_out, N, K, lw, lnw, s_act, s_red, pf);
        return phase_proj_resid<1, 3>(a, W, src, x_in, x_out, N, K, lw, lnw, s_act, s_red, pf);
    }
    if (share >= 3) return phase_proj_resid<3, 6>(a, W, src, x_in, x_out, N, K, lw, lnw, s_act, s_red, pf);
    if (share == 2) return phase_proj_resid<2, 6>(a, W, src, x_in, x_out, N, K, lw, lnw, s_act, s_red, pf);
    return phase_proj_resid<1, 6>(a, W, src, x_in, x_out, N, K, lw, lnw, s_act, s_red, pf);
}

template <int NKS>
__global__ __launch_bounds__(SMALL_THREADS) void k_small_step(SmallArgs a_in, int phase_begin, int phase_end) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    uint16_t* s_act = reinterpret_cast<uint16_t*>(lds + SMALL_LDS_ACT);
    f32x4* s_red = reinterpret_cast<f32x4*>(lds + SMALL_LDS_RED);
    float* s_attn = reinterpret_cast<float*>(lds);     // attention merge slots lie over the staging area and the partial tiles
    __shared__ float s_best[2 * SMALL_NW * SMALL_ROWS];
    __shared__ int32_t s_amax[SMALL_ROWS];
    // The phases read their arguments from LDS, and so the small tables every phase consults (layer
    // pointers, row counts, positions, block table): after a grid barrier has invalidated the caches a
    // read of global memory costs a full memory round trip, and these reads would sit in front of the
    // weight and activation loads that depend on them.  The host checks that the tables fit.
    __shared__ SmallArgs s_args;
    __shared__ TascLayerW s_layers[SMALL_MAX_LAYERS];
    __shared__ int32_t s_nrows[SMALL_ROWS], s_pos0[SMALL_ROWS];
    __shared__ int32_t s_bt[SMALL_MAX_BT];
    __shared__ int s_local;
    if (threadIdx.x == 0) s_args = a_in;
    for (int i = threadIdx.x; i < a_in.n_layers * (int)(sizeof(TascLayerW) / 8); i += SMALL_THREADS)
        reinterpret_cast<u64*>(s_layers)[i] = reinterpret_cast<const u64*>(a_in.layers)[i];
    if (threadIdx.x < a_in.B) {
        s_nrows[threadIdx.x] = a_in.n_rows[threadIdx.x];
        s_pos0[threadIdx.x] = a_in.pos0[threadIdx.x];
    }
    for (int i = threadIdx.x; i < a_in.B * a_in.max_blocks; i += SMALL_THREADS) s_bt[i] = a_in.block_tab[i];
    __syncthreads();
    const SmallTabs tb = {s_layers, s_nrows, s_pos0, s_bt};
    const SmallArgs& a = s_args;
    const int wg = blockIdx.x, nwg = gridDim.x;
    const int n_phases = 3 + 5 * a.n_layers, n_lg_phases = 1 + 5 * a.n_layers;
    const bool member = (wg % a.lg_stride == 0) && (wg / a.lg_stride < a.lg_count);
    const int lw = wg / a.lg_stride, lnw = a.lg_count;
    GAS u32* bar_error = gptr(a.bar_error);
    GAS u64* phase_ts = gptr(a.phase_ts);
    if (phase_begin == 0) {
        // every workgroup outside the layer group (all of them if there is none) shares the cursor table
        const int outside = nwg - lnw;
        if (outside > 0) {
            if (!member) build_bias_ptr(a, wg - min(lnw, (wg + a.lg_stride - 1) / a.lg_stride), outside);   // rank among the outsiders
        } else {
            build_bias_ptr(a, wg, nwg);
        }
    }
    // A launch that runs the whole step may keep the layer group's traffic inside one XCD: every member
    // reports the XCD it runs on before the group's first barrier (always an agent-scope one), and if they
    // all name the same one the later barriers of the group are the XCD-local kind.
    const bool probe_xcd = a.xcd_local != 0 && member && phase_begin == 0 && phase_end >= n_lg_phases;
    if (probe_xcd && threadIdx.x == 0)
        __hip_atomic_fetch_or(gptr(a.xcc_mask), 1u << xcc_id(), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    bool local = false;
    int nwk = lnw;                                 // members that compute; the others (XCD-local mode only) prefetch
    u32 sink = 0;                                  // folds the prefetch loads' values (see touch_lines)
    u32 bar_a = 0, bar_b = 0;
    for (int ph = phase_begin; ph < phase_end && ph < n_phases; ++ph) {
        if (ph < n_lg_phases) {
            if (!member) continue;
            if (ph > phase_begin) {
                if (__hip_atomic_load(bar_error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
                group_sync(gptr(a.bar_flags), lw, lnw, a.bar_epoch + (++bar_a), bar_error, local);
                if (probe_xcd && bar_a == 1) {
                    if (threadIdx.x == 0) {
                        const u32 mask = __hip_atomic_load(gptr(a.xcc_mask), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        s_local = __popc(mask) == 1;
                    }
                    __syncthreads();
                    local = s_local != 0;
                    if (local && a.lg_workers > 0 && a.lg_workers < lnw) nwk = a.lg_workers;
                }
            }
        } else if (ph > phase_begin) {
            if (__hip_atomic_load(bar_error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
            grid_sync(gptr(a.barb_counter), a.barb_base + (u64)(++bar_b) * nwg, bar_error, member ? 0 : 1);
        }
        const bool ts = a.phase_ts != nullptr && wg < a.phase_ts_wgs && threadIdx.x == 0;
        if (ts) phase_ts[((size_t)wg * n_phases + ph) * 2] = wall_clock64();
        auto pf = []() { return 0u; };
        if (ph == 0) {
            const GAS BF16* embed = gptr(a.embed);
            const GAS int32_t* row_tok = gptr(a.row_tok);
            GAS float* x = gptr(a.x);
            for (int r = lw; r < a.M; r += lnw) {
                const GAS BF16* e = embed + (size_t)row_tok[r] * a.D;
                for (int k = threadIdx.x * 8; k < a.D; k += SMALL_THREADS * 8) {
                    const u32x4 u = gld<u32x4>(e + k);
                    GAS float* o = x + (size_t)r * a.D + k;
                    gst(o, f32x4{bf2f(u[0] & 0xFFFFu), bf2f(u[0] >> 16), bf2f(u[1] & 0xFFFFu), bf2f(u[1] >> 16)});
                    gst(o + 4, f32x4{bf2f(u[2] & 0xFFFFu), bf2f(u[2] >> 16), bf2f(u[3] & 0xFFFFu), bf2f(u[3] >> 16)});
                }
            }
        } else if (ph < n_lg_phases && lw >= nwk) {
            sink ^= prefetch_ahead(a, tb, ph, lw - nwk, lnw - nwk);
        } else if (ph < n_lg_phases) {
            const int layer = (ph - 1) / 5, sub = (ph - 1) % 5;
            const TascLayerW& L = tb.layers[layer];
            const int lnw = nwk;                   // the phases share their items among the workers
            if (sub == 0) {
                if (a.D <= 768) sink ^= run_qkv<3>(a, tb, layer, lw, lnw, s_act, s_red, pf);
                else sink ^= run_qkv<6>(a, tb, layer, lw, lnw, s_act, s_red, pf);
            } else if (sub == 1) {
                phase_attn<NKS>(a, tb, layer, lw, lnw, s_attn);
            } else if (sub == 3) {
                if (a.D <= 768) sink ^= run_gate_up<3>(a, tb, layer, lw, lnw, s_act, s_red, pf);
                else sink ^= run_gate_up<6>(a, tb, layer, lw, lnw, s_act, s_red, pf);
            } else {
                const bool o_proj = sub == 2;
                // residual stream: read buffer 2l (+1 for the down projection), write the next one
                const GAS float* x_in = gptr(a.x) + (size_t)(2 * layer + (o_proj ? 0 : 1)) * a.x_stride;
                GAS float* x_out = gptr(a.x) + (size_t)(2 * layer + (o_proj ? 1 : 2)) * a.x_stride;
                const GAS BF16* src = o_proj ? gptr(a.att) + (size_t)layer * a.q_stride : gptr(a.act) + (size_t)layer * a.act_stride;
                sink ^= run_proj(a, gptr((const BF16*)(o_proj ? L.wo_f : L.wd_f)), src, x_in, x_out, a.D, o_proj ? a.H * a.hd : a.F, lw, lnw,
                                 s_act, s_red, pf);
            }
        } else if (ph == n_lg_phases) {
            if (a.n_sel > 0) phase_lmhead(a, wg, nwg, s_act, s_best);
        } else {
            if (a.n_sel > 0 && wg == 0) phase_accept(a, s_amax);
        }
        if (ts) {
            __builtin_amdgcn_s_waitcnt(0);
            phase_ts[((size_t)wg * n_phases + ph) * 2 + 1] = wall_clock64();
        }
    }
    // every member read the set right after the group's first barrier, and workgroup 0 has passed later ones
    if (probe_xcd && wg == 0 && threadIdx.x == 0) {
        __hip_atomic_store(gptr(a.xcc_mask), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (local) gptr(a.counters)[TASC_CTR_XCD_STEPS] += 1;     // only this thread of this launch touches the slot
    }
    if (sink == 0x9E3779B9u && a.phase_ts != nullptr && threadIdx.x == 0) phase_ts[0] = sink;   // never the point: see touch_lines
}
