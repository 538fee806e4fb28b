// Small-batch (at most 16 rows) bf16 target forward as a SPATIAL PIPELINE: one persistent launch per verify step in
// which every workgroup owns one kind of work for ALL layers.
//
// A verify step of k+1 <= 16 rows is a chain of 5 dependent phases per layer (q/k/v projection, attention, output
// projection, gate/up, down) whose arithmetic is negligible: its duration is the number of hand-overs times the cost of
// one.  Two things set that cost, and this kernel removes both from the chain:
//   * weights.  A workgroup has a ROLE (one of the five phases) and the same few output tiles of that phase in every
//     layer, a share small enough for registers (<= 18 MFMA fragments per lane).  Right after finishing layer l it
//     requests its tiles of layer l + 1, four hand-overs before it needs them: the weight stream (all of the model,
//     spread over every compute unit of the chip) runs beside the dependency chain instead of inside it.
//   * barriers.  Activations travel "flag in data": every hand-over buffer is written once per launch and holds a
//     sentinel (all ones, a NaN pattern no arithmetic here produces) until then.  A consumer polls the very words it
//     needs, with loads and stores that bypass the non-coherent caches (agent scope: straight to the memory side, the
//     only place the 8 XCDs share), and goes on when none of them is the sentinel: one store latency plus one load
//     latency per hand-over, no arrival counters, no fences, no second trip for the data.
// The buffers exist twice; a launch uses one copy and re-arms the other (fills it with the sentinel) for the next
// launch, so nothing has to be cleared between the last read and the next write of a buffer inside a launch.
//
// The arithmetic is that of kernels_small.h, tile for tile (same k-step dealing over the 8 waves, same wave-order sums,
// same attention tiling at absolute key positions), so every row's result is bit-identical to that kernel's and
// independent of the row count of the call.
//
// Every wait is bounded: a poll that does not complete raises the session's error flag, after which every poll of every
// workgroup returns at once, so the grid always drains.
#pragma once
#include "kernels_small.h"

#define PIPE_SENT 0xFFFFFFFFu
#ifndef PIPE_POLL_DEPTH
#define PIPE_POLL_DEPTH 1        // polls of a staging wait kept in flight (more of them slow every hand-over down: see pipe_wait_hint)
#endif
// dynamic LDS: the staging layout of kernels_small.h, or the attention role's merge slots + tail image (head_dim 128:
// 8 x 16 x 128 floats + 8 x 16 x 2 floats + 64 x 136 + 128 x 72 bf16), whichever is larger
#define PIPE_LDS_BYTES (65536 + 1024 + 17408 + 18432)
#define PIPE_SPIN_LIMIT (1u << 19)     // polls of about a microsecond each: half a second

enum { PIPE_QKV = 0, PIPE_ATTN = 1, PIPE_O = 2, PIPE_GU = 3, PIPE_DOWN = 4, PIPE_N_ROLES = 5 };

struct PipeArgs {
    SmallArgs a;                       // model, session, activations (the copy this launch uses), verify tail
    BF16* kvn;                         // [L][16][2 Hkv hd] the launch's new key (rotated) and value rows, row-major
    size_t kvn_stride;                 // elements per layer
    float* pv;                         // [16][n_strips] LM-head strip maxima
    int32_t* pi;                       // [16][n_strips] and their token ids
    int32_t role_base[PIPE_N_ROLES];   // workgroups role_base[r] .. + role_count[r] have role r; the others only serve the LM head
    int32_t role_count[PIPE_N_ROLES];
    u64* rearm;                        // the OTHER copy of the hand-over buffers, filled with the sentinel by this launch
    size_t rearm_units;                // ... in 16-byte units (0: nothing to re-arm, e.g. a launch that does not begin a step)
};

// ---------------------------------------------------------------- flag-in-data loads and stores
__device__ __forceinline__ u64 ll_ld(const GAS void* p) {
    return __hip_atomic_load(reinterpret_cast<const GAS u64*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void ll_st(GAS void* p, u64 v) {
    __hip_atomic_store(reinterpret_cast<GAS u64*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void ll_st32(GAS void* p, u32 v) {
    __hip_atomic_store(reinterpret_cast<GAS u32*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u32 ll_ld32(const GAS void* p) {
    return __hip_atomic_load(reinterpret_cast<const GAS u32*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ bool ll_ok(u64 v) { return (u32)v != PIPE_SENT && (u32)(v >> 32) != PIPE_SENT; }
__device__ __forceinline__ u64 pack_u64(u32 lo, u32 hi) { return (u64)lo | ((u64)hi << 32); }
__device__ __forceinline__ void ll_st_f4(GAS float* p, f32x4 v) {
    ll_st(p, pack_u64(__float_as_uint(v[0]), __float_as_uint(v[1])));
    ll_st(p + 2, pack_u64(__float_as_uint(v[2]), __float_as_uint(v[3])));
}
__device__ __forceinline__ void ll_st_b4(GAS BF16* p, u32x2 v) { ll_st(p, pack_u64(v[0], v[1])); }

// One round of a poll has failed: count it, give up when the flag is up or the limit is reached.  Returns true to stop.
__device__ __forceinline__ bool ll_give_up(u32& spins, GAS u32* err) {
    ++spins;
    if ((spins & 63u) != 0) return false;
    if (__hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return true;
    if (spins > PIPE_SPIN_LIMIT) {
        __hip_atomic_fetch_or(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return true;
    }
    return false;
}

// Every poll of an unwritten buffer is a round trip to the memory side, and 200 workgroups polling at full rate for
// inputs that are four hand-overs away slow down the one hand-over that is in progress (measured: the more polls in
// flight, the longer every hand-over).  So a workgroup first waits, with ONE thread and pauses between its loads, for a
// word that gets written one phase before its producers run (its producers' own input), and only then starts to poll
// its inputs in earnest.  `word` = nullptr: no such word (the first phase of a launch).
__device__ __forceinline__ void pipe_wait_hint(const GAS void* word, GAS u32* err) {
    if (word != nullptr && threadIdx.x == 0) {
        u32 spins = 0;
        while (!ll_ok(ll_ld(word)) && !ll_give_up(spins, err)) __builtin_amdgcn_s_sleep(8);
    }
    __syncthreads();
}

// ---------------------------------------------------------------- staging through polls
// stage_normed_issue of kernels_small.h with the rows read through the poll (gains are weights: plain loads, done by
// the caller ahead of time into rg.g)
// DEPTH polls are kept in flight: an agent-scope load takes over a microsecond, and a phase goes on only when the
// slowest of its pollers has seen the data, so the sampling interval of a poller is on the critical path.
template <int NTC, int DEPTH>
__device__ __forceinline__ u32 pipe_poll_rows(const GAS float* x, const GAS int32_t* sel, int M, int D, NormRegs<NTC>& rg, GAS u32* err) {
    const int lane = threadIdx.x & 63, wave = wave_id();
    const GAS float* xr[2];
    bool live[2];                                  // rows beyond M are not polled (the staging zeroes them); uniform per wave
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int r = wave + SMALL_NW * j;
        live[j] = r < M;
        int src = r < M ? r : 0;
        if (sel) {
            src = sel[src];
            if (src < 0) src = 0;
        }
        xr[j] = x + (size_t)src * D;
    }
    struct Round { u64 v[2][NTC][2]; };
    auto issue = [&](Round& q) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
            if (live[j]) {
#pragma unroll
                for (int t = 0; t < NTC; ++t) {
                    const int c = 4 * (lane + 64 * t);
                    const GAS float* p = xr[j] + (c < D ? c : D - 4);
                    q.v[j][t][0] = ll_ld(p);
                    q.v[j][t][1] = ll_ld(p + 2);
                }
            }
    };
    auto take = [&](const Round& q) {
        u32 bad = 0;
#pragma unroll
        for (int j = 0; j < 2; ++j)
            if (live[j]) {
#pragma unroll
                for (int t = 0; t < NTC; ++t) bad |= (u32)!ll_ok(q.v[j][t][0]) | (u32)!ll_ok(q.v[j][t][1]);
            }
        if (bad) return false;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int t = 0; t < NTC; ++t)
                rg.v[j][t] = f32x4{__uint_as_float((u32)q.v[j][t][0]), __uint_as_float((u32)(q.v[j][t][0] >> 32)),
                                   __uint_as_float((u32)q.v[j][t][1]), __uint_as_float((u32)(q.v[j][t][1] >> 32))};
        return true;
    };
    u32 spins = 0;
    Round q[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) issue(q[d]);
    for (bool out = false; !out;) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            if (!out) {
                out = take(q[d]) || ll_give_up(spins, err);
                if (!out) issue(q[d]);
            }
        }
    }
    return spins;
}
template <int NTC>
__device__ __forceinline__ void pipe_load_gains(const GAS float* g, int D, NormRegs<NTC>& rg) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int t = 0; t < NTC; ++t) {
        const int c = 4 * (lane + 64 * t);
        rg.g[t] = gld<f32x4>(g + (c < D ? c : D - 4));
    }
}

// stage_copy_issue of kernels_small.h through the poll (two polls in flight, as above)
template <int NC>
__device__ __forceinline__ void pipe_poll_copy(const GAS BF16* src, int M, int K, int kc0, int kw, CopyRegs<NC>& rg, GAS u32* err) {
    const int per_row = kw / 8, total = SMALL_ROWS * per_row;
    const GAS BF16* p[NC];
    bool live[NC];                                 // rows beyond M are not polled (the staging zeroes them)
#pragma unroll
    for (int u = 0; u < NC; ++u) {
        const int idx = (int)threadIdx.x + u * SMALL_THREADS;
        const int ic = min(idx, total - 1);
        const int r = ic / per_row, k = (ic % per_row) * 8;
        live[u] = idx < total && r < M;
        p[u] = src + (size_t)(r < M ? r : 0) * K + kc0 + k;
    }
    struct Round { u64 v[NC][2]; };
    auto issue = [&](Round& q) {
#pragma unroll
        for (int u = 0; u < NC; ++u) {
            q.v[u][0] = 0;
            q.v[u][1] = 0;
            if (live[u]) {
                q.v[u][0] = ll_ld(p[u]);
                q.v[u][1] = ll_ld(p[u] + 4);
            }
        }
    };
    auto take = [&](const Round& q) {
        u32 bad = 0;
#pragma unroll
        for (int u = 0; u < NC; ++u) bad |= (u32)!ll_ok(q.v[u][0]) | (u32)!ll_ok(q.v[u][1]);
        if (bad) return false;
#pragma unroll
        for (int u = 0; u < NC; ++u)
            rg.v[u] = as_bf16x8((u32)q.v[u][0], (u32)(q.v[u][0] >> 32), (u32)q.v[u][1], (u32)(q.v[u][1] >> 32));
        return true;
    };
    u32 spins = 0;
    constexpr int DEPTH = NC <= 3 ? PIPE_POLL_DEPTH : 2;
    Round q[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) issue(q[d]);
    for (bool out = false; !out;) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            if (!out) {
                out = take(q[d]) || ll_give_up(spins, err);
                if (!out) issue(q[d]);
            }
        }
    }
}
__device__ __forceinline__ f32x4 pipe_poll_f4(const GAS float* p, GAS u32* err) {
    u32 spins = 0;
    u64 a, b;
    for (;;) {
        a = ll_ld(p);
        b = ll_ld(p + 2);
        if ((ll_ok(a) && ll_ok(b)) || ll_give_up(spins, err)) break;
    }
    return f32x4{__uint_as_float((u32)a), __uint_as_float((u32)(a >> 32)), __uint_as_float((u32)b), __uint_as_float((u32)(b >> 32))};
}

// per-phase time stamps (optional): [workgroup][phase][inputs complete, outputs stored]
struct PipeStamp {
    GAS u64* ts;
    int n_phases;
    bool on;
    __device__ __forceinline__ void ready(int ph) const { if (on) ts[(size_t)ph * 2] = wall_clock64(); }
    __device__ __forceinline__ void done(int ph) const { if (on) ts[(size_t)ph * 2 + 1] = wall_clock64(); }
};

// layers [l0, l1) of the phase `sub` that fall into the launch's phase range [p0, p1) (phase = 1 + 5 l + sub)
__device__ __forceinline__ void pipe_layer_range(int sub, int n_layers, int p0, int p1, int& l0, int& l1) {
    const int lo = p0 - 1 - sub, hi = p1 - 1 - sub;          // layers with lo <= 5 l < hi
    l0 = lo <= 0 ? 0 : (lo + 4) / 5;
    l1 = hi <= 0 ? 0 : (hi + 4) / 5;
    if (l1 > n_layers) l1 = n_layers;
    if (l0 > l1) l0 = l1;
}

// ---------------------------------------------------------------- role: RMSNorm + q/k/v + RoPE + KV append
// Items as in phase_qkv (head, block of 16 dims of the first half, with its RoPE partner tile); the workgroup's NI
// items are lw, lw + lnw, ...; item j is finished by wave j.
template <int NI, int WKS>
__device__ __forceinline__ void role_qkv(const PipeArgs& pa, const SmallTabs& tb, int lw, int lnw, int l0, int l1, uint16_t* s_act,
                                         f32x4* s_red, const PipeStamp& st) {
    const SmallArgs& a = pa.a;
    if (l0 >= l1) return;
    GAS u32* err = gptr(a.bar_error);
    const int half = a.hd / 2, eb_per_head = half / 16;
    const int n_items = (a.H + 2 * a.Hkv) * eb_per_head;
    const int lane = threadIdx.x & 63, wave = wave_id();
    const size_t tile_row = (size_t)(a.D / 32) * 512;
    const int nks = a.D / 32;
    const int m = lane & 15;
    // what does not depend on the layer: the wave's own item, its row's position, rotation factors, page
    const int my_item = lw + wave * lnw;
    const bool mine = wave < NI && my_item < n_items && m < a.M;
    const int it = mine ? my_item : lw, mr = mine ? m : 0;
    const int head = it / eb_per_head, e0 = (it % eb_per_head) * 16;
    const int e = e0 + 4 * (lane >> 4);
    const int b = mr / a.nq, i = mr % a.nq;
    const bool active = mine && i < tb.n_rows[b];
    const int pos = tb.pos0[b] + i;
    const int tpos = pos < a.max_pos ? (pos > 0 ? pos : 0) : a.max_pos - 1;
    f32x4 cs = gld<f32x4>(gptr(a.rope_cos) + (size_t)tpos * half + e);
    f32x4 sn = gld<f32x4>(gptr(a.rope_sin) + (size_t)tpos * half + e);
    if (head >= a.H + a.Hkv) {                               // value heads are not rotated
        cs = f32x4{1, 1, 1, 1};
        sn = f32x4{0, 0, 0, 0};
    }
    const size_t page_off = (active && head >= a.H) ? (size_t)tb.block_tab[(size_t)b * a.max_blocks + pos / TASC_KV_BLOCK] * a.page_elems : 0;
    size_t wofs[2 * NI];
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        const int item = min(lw + j * lnw, n_items - 1);      // a missing item repeats the last one and is dropped below
        const int hj = item / eb_per_head, ej = (item % eb_per_head) * 16;
        wofs[2 * j] = (size_t)((hj * a.hd + ej) / 16) * tile_row;
        wofs[2 * j + 1] = (size_t)((hj * a.hd + half + ej) / 16) * tile_row;
    }
    bf16x8 w[2 * NI][WKS];
    NormRegs<WKS> xr;
    auto fetch = [&](int layer) {
        const TascLayerW& L = tb.layers[layer];
        const GAS BF16* W = gptr((const BF16*)L.wqkv_f);
        const GAS BF16* wrow[2 * NI];
#pragma unroll
        for (int t = 0; t < 2 * NI; ++t) wrow[t] = W + wofs[t];
        load_w<2 * NI, WKS>(wrow, 0, nks, w);
        pipe_load_gains<WKS>(gptr(L.g1), a.D, xr);
    };
    fetch(l0);
    for (int layer = l0; layer < l1; ++layer) {
        const int ph = 1 + 5 * layer + PIPE_QKV;
        pipe_wait_hint(layer > 0 ? gptr(a.act) + (size_t)(layer - 1) * a.act_stride : nullptr, err);
        pipe_poll_rows<WKS, (WKS == 3 ? PIPE_POLL_DEPTH : 1)>(gptr(a.x) + (size_t)(2 * layer) * a.x_stride, nullptr, a.M, a.D, xr, err);
        st.ready(ph);
        stage_normed_finish<WKS>(xr, a.M, a.D, a.eps, s_act);
        f32x4 acc[2 * NI];
#pragma unroll
        for (int t = 0; t < 2 * NI; ++t) acc[t] = f32x4{0, 0, 0, 0};
        mma_w<2 * NI, WKS>(w, nks, s_act, acc);
        put_partials<2 * NI>(acc, s_red);
        if (mine) {
            GAS BF16* kv_layer = gptr(a.kv_pool) + (size_t)layer * a.kv_layer_stride;
            GAS BF16* q_out = gptr(a.q) + (size_t)layer * a.q_stride;
            GAS BF16* kvn = gptr(pa.kvn) + (size_t)layer * pa.kvn_stride + (size_t)m * 2 * a.Hkv * a.hd;
            const f32x4 a0 = sum_tile(s_red, 2 * wave), a1 = sum_tile(s_red, 2 * wave + 1);
            float ra[4], rc[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                ra[u] = a0[u] * cs[u] - a1[u] * sn[u];
                rc[u] = a1[u] * cs[u] + a0[u] * sn[u];
            }
            const u32x2 lo = pack_bf16x4(ra[0], ra[1], ra[2], ra[3]), hi = pack_bf16x4(rc[0], rc[1], rc[2], rc[3]);
            if (head < a.H) {
                GAS BF16* qo = q_out + (size_t)m * a.H * a.hd + head * a.hd;
                ll_st_b4(qo + e, lo);
                ll_st_b4(qo + half + e, hi);
            } else {
                // to this launch's attention through the hand-over buffer (rows without a position too: they are polled
                // by nobody, but a buffer is either written whole or not at all), to later launches through the cache
                GAS BF16* kn = kvn + (size_t)(head - a.H) * a.hd;
                ll_st_b4(kn + e, lo);
                ll_st_b4(kn + half + e, hi);
                if (active) {
                    GAS BF16* page = kv_layer + page_off;
                    const int slot = pos % TASC_KV_BLOCK;
                    if (head < a.H + a.Hkv) {
                        const int g = head - a.H;
                        GAS BF16* kp = page + (size_t)(g * TASC_KV_BLOCK + slot) * a.hd;
                        gst(kp + e, lo);
                        gst(kp + half + e, hi);
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
        }
        st.done(ph);
        // The next layer's tiles, requested four hand-overs before they are needed -- and only once every wave is past the
        // result stores: a compute unit serves its memory requests in order, so a cold weight stream queued ahead of the
        // stores (by the waves that have nothing to store) would hold them back.
        // (The last layer asks for its own tiles again: no load sits under a condition.)
        __syncthreads();                      // s_red and s_act are free again; and no wave requests weights before the stores are out
        fetch(min(layer + 1, l1 - 1));
    }
}

// ---------------------------------------------------------------- roles: output / down projection with residual
// x_out[m][n] = x_in[m][n] + sum_k src[m][k] W[n][k]; items of 16 output features lw, lw + lnw, ... (NI of them)
template <int NI, int WKS>
__device__ __forceinline__ void role_proj(const PipeArgs& pa, const SmallTabs& tb, bool o_proj, int lw, int lnw, int l0, int l1,
                                          uint16_t* s_act, f32x4* s_red, const PipeStamp& st) {
    const SmallArgs& a = pa.a;
    if (l0 >= l1) return;
    GAS u32* err = gptr(a.bar_error);
    const int lane = threadIdx.x & 63, wave = wave_id();
    const int N = a.D, K = o_proj ? a.H * a.hd : a.F;
    const int n_items = N / 16;
    const int m = lane & 15;
    // the workgroup's items are neighbours (lw NI, lw NI + 1, ..): together they cover whole 128-byte lines of the output
    // rows where NI allows, so that a line has one writer
    const int my_item = lw * NI + wave;
    const bool mine = wave < NI && my_item < n_items && m < a.M;
    const size_t xoff = (size_t)(mine ? m : 0) * N + (mine ? my_item : 0) * 16 + 4 * (lane >> 4);
    size_t wofs[NI];
#pragma unroll
    for (int j = 0; j < NI; ++j) wofs[j] = (size_t)min(lw * NI + j, n_items - 1) * (K / 32) * 512;
    const int kw0 = min(SMALL_KC, K), nks0 = kw0 / 32;
    bf16x8 w[NI][WKS];
    auto fetch = [&](int layer, int kc0, int nks) {
        const TascLayerW& L = tb.layers[layer];
        const GAS BF16* W = gptr((const BF16*)(o_proj ? L.wo_f : L.wd_f));
        const GAS BF16* wrow[NI];
#pragma unroll
        for (int j = 0; j < NI; ++j) wrow[j] = W + wofs[j];
        load_w<NI, WKS>(wrow, kc0, nks, w);
    };
    fetch(l0, 0, nks0);
    for (int layer = l0; layer < l1; ++layer) {
        const int ph = 1 + 5 * layer + (o_proj ? PIPE_O : PIPE_DOWN);
        const GAS float* x_in = gptr(a.x) + (size_t)(2 * layer + (o_proj ? 0 : 1)) * a.x_stride;
        GAS float* x_out = gptr(a.x) + (size_t)(2 * layer + (o_proj ? 1 : 2)) * a.x_stride;
        const GAS BF16* src = o_proj ? gptr(a.att) + (size_t)layer * a.q_stride : gptr(a.act) + (size_t)layer * a.act_stride;
        f32x4 acc[NI];
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[j] = f32x4{0, 0, 0, 0};
        pipe_wait_hint(o_proj ? (const GAS void*)(gptr(a.q) + (size_t)layer * a.q_stride) : (const GAS void*)x_in, err);
        // the residual comes through the same kind of buffer; it was written a phase before the producer of `src` began,
        // so this poll ends long before the next one
        const f32x4 xv0 = pipe_poll_f4(x_in + xoff, err);
        for (int kc0 = 0; kc0 < K; kc0 += SMALL_KC) {
            const int kw = min(SMALL_KC, K - kc0), nks = kw / 32;
            if (kc0 > 0) {
                __syncthreads();                          // the previous chunk's fragments have been read
                fetch(layer, kc0, nks);
            }
            CopyRegs<WKS> cr;
            pipe_poll_copy<WKS>(src, a.M, K, kc0, kw, cr, err);
            if (kc0 == 0) st.ready(ph);
            stage_copy_finish<WKS>(cr, a.M, kw, s_act);
            mma_w<NI, WKS>(w, nks, s_act, acc);
        }
        put_partials<NI>(acc, s_red);
        if (mine) {
            const f32x4 xv = xv0 + sum_tile(s_red, wave);
            ll_st_f4(x_out + xoff, xv);
        }
        st.done(ph);
        __syncthreads();
        fetch(min(layer + 1, l1 - 1), 0, nks0);       // after the result stores of every wave: see role_qkv
    }
}

// ---------------------------------------------------------------- role: RMSNorm + gate/up + SwiGLU
template <int NI, int WKS>
__device__ __forceinline__ void role_gate_up(const PipeArgs& pa, const SmallTabs& tb, int lw, int lnw, int l0, int l1, uint16_t* s_act,
                                             f32x4* s_red, const PipeStamp& st) {
    const SmallArgs& a = pa.a;
    if (l0 >= l1) return;
    GAS u32* err = gptr(a.bar_error);
    const int lane = threadIdx.x & 63, wave = wave_id();
    const size_t tile_row = (size_t)(a.D / 32) * 512;
    const int nks = a.D / 32;
    const int n_items = a.F / 16;
    const int m = lane & 15;
    const int my_item = lw * NI + wave;               // neighbouring items: see role_proj
    const bool mine = wave < NI && my_item < n_items && m < a.M;
    size_t wofs[NI];
#pragma unroll
    for (int j = 0; j < NI; ++j) wofs[j] = (size_t)min(lw * NI + j, n_items - 1) * 2 * tile_row;
    bf16x8 w[2 * NI][WKS];
    NormRegs<WKS> xr;
    auto fetch = [&](int layer) {
        const TascLayerW& L = tb.layers[layer];
        const GAS BF16* Wgu = gptr((const BF16*)L.wgu_f);
        const GAS BF16* wrow[2 * NI];
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            wrow[2 * j] = Wgu + wofs[j];
            wrow[2 * j + 1] = Wgu + wofs[j] + tile_row;
        }
        load_w<2 * NI, WKS>(wrow, 0, nks, w);
        pipe_load_gains<WKS>(gptr(L.g2), a.D, xr);
    };
    fetch(l0);
    for (int layer = l0; layer < l1; ++layer) {
        const int ph = 1 + 5 * layer + PIPE_GU;
        GAS BF16* act = gptr(a.act) + (size_t)layer * a.act_stride;
        pipe_wait_hint(gptr(a.att) + (size_t)layer * a.q_stride, err);
        pipe_poll_rows<WKS, (WKS == 3 ? PIPE_POLL_DEPTH : 1)>(gptr(a.x) + (size_t)(2 * layer + 1) * a.x_stride, nullptr, a.M, a.D, xr, err);
        st.ready(ph);
        stage_normed_finish<WKS>(xr, a.M, a.D, a.eps, s_act);
        f32x4 acc[2 * NI];
#pragma unroll
        for (int t = 0; t < 2 * NI; ++t) acc[t] = f32x4{0, 0, 0, 0};
        mma_w<2 * NI, WKS>(w, nks, s_act, acc);
        put_partials<2 * NI>(acc, s_red);
        if (mine) {
            const f32x4 gt = sum_tile(s_red, 2 * wave), up = sum_tile(s_red, 2 * wave + 1);
            float o[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) o[u] = gt[u] / (1.0f + __expf(-gt[u])) * up[u];
            ll_st_b4(act + (size_t)m * a.F + my_item * 16 + 4 * (lane >> 4), pack_bf16x4(o[0], o[1], o[2], o[3]));
        }
        st.done(ph);
        __syncthreads();
        fetch(min(layer + 1, l1 - 1));                // after the result stores of every wave: see role_qkv
    }
}

// ---------------------------------------------------------------- role: attention
// phase_attn of kernels_small.h, item for item and tile for tile.  The cached keys and values (positions below the
// sequence's cached length) come from the paged cache with ordinary loads; the rows of THIS launch come from the
// hand-over buffer: they are polled, parked in LDS, and patched into the fragments of the (at most two) key tiles that
// reach beyond the cached length, so the tiling at absolute key positions -- and with it every row's summation order
// -- is the same whether a key was cached by an earlier launch or produced by this one.
template <int NKS>
__device__ __forceinline__ void role_attn(const PipeArgs& pa, const SmallTabs& tb, int lw, int lnw, int l0, int l1, float* s_buf,
                                          const PipeStamp& st) {
    const SmallArgs& a = pa.a;
    GAS u32* err = gptr(a.bar_error);
    const int lane = threadIdx.x & 63, wave = wave_id();
    constexpr int hd = 32 * NKS, ndt = 2 * NKS;
    constexpr int TG = NKS <= 2 ? 3 : 1;
    const int Gq = a.H / a.Hkv;
    const size_t v_off = (size_t)a.Hkv * TASC_KV_BLOCK * hd;
    const int m = lane & 15, qd = lane >> 4;
    float* slot_o = s_buf;                                   // [wave][row][hd]
    float* slot_ml = s_buf + SMALL_NW * SMALL_ROWS * hd;     // [wave][row][max, sum]
    // image of the 64 keys from the tile that holds the first row of this launch: K rows and V^T rows, padded against
    // bank conflicts; cached keys are copied in from the paged cache, this launch's rows from the hand-over buffer
    constexpr int KT = hd + 8, VT = 64 + 8;
    uint16_t* s_kt = reinterpret_cast<uint16_t*>(slot_ml + SMALL_NW * SMALL_ROWS * 2);   // [64][KT]
    uint16_t* s_vt = s_kt + 64 * KT;                                                      // [hd][VT]
    const int n_items = a.B * a.H;
    const int my_items = lw < n_items ? (n_items - lw + lnw - 1) / lnw : 0;
    const int n_units = (l1 - l0) * my_items;                // unit u = (layer l0 + u / my_items, item lw + (u % my_items) lnw)
    if (n_units <= 0) return;
    // fragments of one group of TG key tiles (tiles tg, tg + 8, ..) of a unit, from the paged cache.  Every load is
    // unconditional: tiles beyond the sequence repeat the last one and are skipped by the arithmetic.
    bf16x8 kf0[TG][NKS], kf1[TG][NKS];
    bf16x8 vf[TG][ndt];
    auto load_group = [&](int u, int tg) {
        const int layer = l0 + u / my_items, item = lw + (u % my_items) * lnw;
        const int b = item / a.H, g = (item % a.H) / Gq;
        const int L = tb.pos0[b] + tb.n_rows[b];
        const int n_tiles = (L + 31) / 32;
        const int32_t* bt = tb.block_tab + (size_t)b * a.max_blocks;
        const GAS BF16* kv_layer = gptr(a.kv_pool) + (size_t)layer * a.kv_layer_stride;
#pragma unroll
        for (int j = 0; j < TG; ++j) {
            const int t = max(0, min(tg + j * SMALL_NW, n_tiles - 1));
            const int key0 = t * 32;
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
    };
    // The cached keys and values do not depend on this launch's rows: the first group of a unit is requested when the
    // unit before it ends (a whole layer ahead when the workgroup has one item), and sits in registers during the poll.
    load_group(0, wave);
    for (int u = 0; u < n_units; ++u) {
        const int layer = l0 + u / my_items, item = lw + (u % my_items) * lnw;
        const int ph = 1 + 5 * layer + PIPE_ATTN;
        const GAS BF16* q_in = gptr(a.q) + (size_t)layer * a.q_stride;
        const GAS BF16* kvn = gptr(pa.kvn) + (size_t)layer * pa.kvn_stride;
        GAS BF16* att_out = gptr(a.att) + (size_t)layer * a.q_stride;
        const int b = item / a.H, h = item % a.H, g = h / Gq;
        const int nr = tb.n_rows[b], p0 = tb.pos0[b];
        const int L = p0 + nr;                               // keys 0 .. L-1 exist
        const int n_tiles = (L + 31) / 32;
        // ---- the tail image: first the cached part (whole pages, stale slots included: overwritten below) ...
        const int tail0 = (p0 / 32) * 32;
        pipe_wait_hint(gptr(a.x) + (size_t)(2 * layer) * a.x_stride, err);
        {
            const GAS BF16* kv_layer = gptr(a.kv_pool) + (size_t)layer * a.kv_layer_stride;
            const int32_t* bt = tb.block_tab + (size_t)b * a.max_blocks;
            constexpr int kch = hd / 8;                          // 16-byte chunks per key row
            for (int c = threadIdx.x; c < 2 * 64 * kch; c += SMALL_THREADS) {
                const bool is_v = c >= 64 * kch;
                const int cc = is_v ? c - 64 * kch : c;
                // K: chunk cc = (key, part); V^T: chunk cc = (page, dim, half)
                const int key = is_v ? (cc / (2 * hd)) * 16 : cc / kch;
                const int pg = min((tail0 + key) / TASC_KV_BLOCK, a.max_blocks - 1);
                const GAS BF16* page = kv_layer + (size_t)bt[pg] * a.page_elems;
                if (!is_v) {
                    const int part = cc % kch;
                    const bf16x8 v = gld<bf16x8>(page + (size_t)(g * TASC_KV_BLOCK + key % 16) * hd + 8 * part);
                    *reinterpret_cast<bf16x8*>(s_kt + key * KT + 8 * part) = v;
                } else {
                    const int d = (cc % (2 * hd)) / 2, half = cc % 2;
                    const bf16x8 v = gld<bf16x8>(page + v_off + (size_t)(g * hd + d) * TASC_KV_BLOCK + 8 * half);
                    *reinterpret_cast<bf16x8*>(s_vt + d * VT + key + 8 * half) = v;
                }
            }
        }
        __syncthreads();
        // ---- ... then this launch's key and value rows of the sequence (KV head g)
        {
            const int upr = hd / 4;                          // 8-byte units per row and matrix
            const int t = threadIdx.x;
            const bool need = t < nr * upr;
            const int r = need ? t / upr : 0, c = need ? (t % upr) * 4 : 0;
            const GAS BF16* kp = kvn + (size_t)(b * a.nq + r) * 2 * a.Hkv * hd + (size_t)g * hd + c;
            const GAS BF16* vp = kp + (size_t)a.Hkv * hd;
            if (need) {
                u64 kv8, vv8;
                u32 spins = 0;
                for (;;) {
                    kv8 = ll_ld(kp);
                    vv8 = ll_ld(vp);
                    if ((ll_ok(kv8) && ll_ok(vv8)) || ll_give_up(spins, err)) break;
                }
                const int slot = p0 - tail0 + r;             // < 48
                *reinterpret_cast<u64*>(s_kt + slot * KT + c) = kv8;
#pragma unroll
                for (int e = 0; e < 4; ++e) s_vt[(c + e) * VT + slot] = (uint16_t)(vv8 >> (16 * e));
            }
        }
        // ---- Q fragments (B operand): query row m, dims 32 ks + 8 qd ..
        const bool okq = m < nr;
        const int qi = okq ? p0 + m : -1;                    // position of the query row, -1 = no such row
        const GAS BF16* qp = q_in + (size_t)(b * a.nq + (okq ? m : 0)) * a.H * hd + (size_t)h * hd;
        bf16x8 qf[NKS];
        {
            u32 spins = 0;
            for (;;) {
                u64 v[NKS][2];
                bool ok = true;
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) {
                    v[ks][0] = ll_ld(qp + 32 * ks + 8 * qd);
                    v[ks][1] = ll_ld(qp + 32 * ks + 8 * qd + 4);
                }
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) {
                    ok = ok && ll_ok(v[ks][0]) && ll_ok(v[ks][1]);
                    const bf16x8 f = as_bf16x8((u32)v[ks][0], (u32)(v[ks][0] >> 32), (u32)v[ks][1], (u32)(v[ks][1] >> 32));
                    qf[ks] = okq ? f : bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
                }
                if (ok || nr == 0 || ll_give_up(spins, err)) break;
            }
        }
        __syncthreads();                                     // the new rows are in LDS
        if (u % my_items == 0) st.ready(ph);
        float mx = -INFINITY, lsum = 0.f;
        f32x4 o[ndt];                                        // O^T tiles: lane holds dims 16 dt + 4 qd .. +4 of row m
#pragma unroll
        for (int dt = 0; dt < ndt; ++dt) o[dt] = f32x4{0, 0, 0, 0};
        for (int tg = wave; tg < n_tiles; tg += SMALL_NW * TG) {
            if (tg != wave) load_group(u, tg);               // long sequences: the later groups on demand
#pragma unroll
            for (int j = 0; j < TG; ++j) {
                const int t = tg + j * SMALL_NW;
                if (t < n_tiles) {
                    const int key0 = t * 32;
                    if (key0 >= tail0) {
                        // the tile lies in the tail image: fragments from LDS
                        const int k0 = key0 - tail0;
#pragma unroll
                        for (int ks = 0; ks < NKS; ++ks) {
                            kf0[j][ks] = *reinterpret_cast<const bf16x8*>(s_kt + (k0 + m) * KT + 32 * ks + 8 * qd);
                            kf1[j][ks] = *reinterpret_cast<const bf16x8*>(s_kt + (k0 + 16 + m) * KT + 32 * ks + 8 * qd);
                        }
#pragma unroll
                        for (int dt = 0; dt < ndt; ++dt) {
                            const u32x2 h0 = *reinterpret_cast<const u32x2*>(s_vt + (16 * dt + m) * VT + k0 + 4 * qd);
                            const u32x2 h1 = *reinterpret_cast<const u32x2*>(s_vt + (16 * dt + m) * VT + k0 + 16 + 4 * qd);
                            vf[j][dt] = as_bf16x8(h0[0], h0[1], h1[0], h1[1]);
                        }
                    }
                    // S^T tiles: A = K rows (key = m within the page), B = Q
                    f32x4 s0 = {0, 0, 0, 0}, s1 = {0, 0, 0, 0};
#pragma unroll
                    for (int ks = 0; ks < NKS; ++ks) {
                        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf0[j][ks], qf[ks], s0, 0, 0, 0);
                        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf1[j][ks], qf[ks], s1, 0, 0, 0);
                    }
                    float sv[8];
                    float tmax = -INFINITY;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int key = key0 + (e < 4 ? 4 * qd + e : 16 + 4 * qd + (e - 4));
                        const float sc = (e < 4 ? s0[e] : s1[e - 4]) * a.scale;
                        sv[e] = (key <= qi) ? sc : -INFINITY;      // causal; also hides keys beyond the sequence
                        tmax = fmaxf(tmax, sv[e]);
                    }
                    tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
                    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
                    const float m_new = fmaxf(mx, tmax);
                    float psum = 0.f, corr = 1.f;
                    uint32_t pw[4] = {0, 0, 0, 0};
                    if (m_new != -INFINITY) {
                        corr = __expf(mx - m_new);
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const uint32_t pb = f2bf(__expf(sv[e] - m_new));
                            pw[e >> 1] |= pb << (16 * (e & 1));
                            psum += bf2f(pb);                      // the sum uses the rounded weights the product uses
                        }
                    }
                    const bf16x8 pk = as_bf16x8(pw[0], pw[1], pw[2], pw[3]);
                    psum += __shfl_xor(psum, 16);
                    psum += __shfl_xor(psum, 32);
                    lsum = lsum * corr + psum;
                    mx = m_new;
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
        // ... and thread (row r, dims d0 .. d0 + PER) combines them in wave order.  Every row of the sequence's nq rows
        // is stored (zeros beyond the rows it has), in units of at least 4 bytes: a consumer takes a word for written
        // as soon as it differs from the sentinel.
        {
            constexpr int PER = hd >= 64 ? hd / 32 : 2;
            constexpr int TPR = hd / PER;                        // threads per row
            const int r = threadIdx.x / TPR, d0 = (threadIdx.x % TPR) * PER;
            if (r < SMALL_ROWS) {
                float mall = -INFINITY;
#pragma unroll
                for (int w8 = 0; w8 < SMALL_NW; ++w8) mall = fmaxf(mall, slot_ml[(w8 * SMALL_ROWS + r) * 2]);
                float den = 0.f, num[PER];
#pragma unroll
                for (int e = 0; e < PER; ++e) num[e] = 0.f;
#pragma unroll
                for (int w8 = 0; w8 < SMALL_NW; ++w8) {
                    const float mw = slot_ml[(w8 * SMALL_ROWS + r) * 2];
                    const float c = mw == -INFINITY ? 0.f : __expf(mw - mall);
                    den += c * slot_ml[(w8 * SMALL_ROWS + r) * 2 + 1];
#pragma unroll
                    for (int e = 0; e < PER; ++e) num[e] += c * slot_o[(size_t)(w8 * SMALL_ROWS + r) * hd + d0 + e];
                }
                if (r < a.nq) {
                    const float inv = (r < nr && den > 0.f) ? 1.0f / den : 0.f;
                    GAS BF16* op = att_out + (size_t)(b * a.nq + r) * a.H * hd + (size_t)h * hd + d0;
                    if constexpr (PER == 2) {
                        ll_st32(op, (uint32_t)f2bf(num[0] * inv) | ((uint32_t)f2bf(num[1] * inv) << 16));
                    } else {
                        ll_st_b4(op, pack_bf16x4(num[0] * inv, num[1] * inv, num[2] * inv, num[3] * inv));
                    }
                }
            }
        }
        if (u % my_items == my_items - 1) st.done(ph);
        __syncthreads();                                     // the slots are free again
        load_group(min(u + 1, n_units - 1), wave);           // after the result stores of every wave: see role_qkv
    }
}

// ---------------------------------------------------------------- final norm + LM head + bias + strip argmax
// phase_lmhead of kernels_small.h over the strips wg, wg + nwg, ...; the rows arrive through the poll, the bias
// cursors are found by binary search in the row's own list, the strip results leave through the hand-over buffer.
// The lane's place in its row's bias list for the workgroup's first two strips, found at the start of the launch: a
// binary search is a dozen dependent loads from memory, which at the end of the step would sit on the critical path.
struct PipeBias {
    int64_t first[2];      // index of the first list entry with a column >= the lane's first feature, per strip pass
    int64_t end;
    float base;
};
__device__ __forceinline__ int64_t pipe_bias_search(const GAS int32_t* b_col, int64_t lo, int64_t hi, int c0) {
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (b_col[mid] < c0) lo = mid + 1; else hi = mid;
    }
    return lo;
}
__device__ __forceinline__ PipeBias pipe_bias_cursors(const PipeArgs& pa, int wg, int nwg) {
    const SmallArgs& a = pa.a;
    PipeBias pb = {{0, 0}, 0, 0.f};
    const int lane = threadIdx.x & 63, wave = wave_id();
    const int m = lane & 15, qd = lane >> 4;
    if (a.bias.rowptr != nullptr && a.n_sel > 0 && m < a.n_sel) {
        const GAS int64_t* b_rowptr = gptr(a.bias.rowptr);
        const GAS int32_t* b_col = gptr(a.bias.col);
        const int u = gptr(a.sel_tok)[m];
        const int64_t lo = b_rowptr[u];
        pb.end = b_rowptr[u + 1];
        pb.base = gptr(a.bias.base)[u];
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int strip = wg + pass * nwg;
            pb.first[pass] = pipe_bias_search(b_col, lo, pb.end, strip * TASC_LM_STRIP + wave * 16 + 4 * qd);
        }
    }
    return pb;
}

__device__ __forceinline__ void pipe_lmhead(const PipeArgs& pa, int wg, int nwg, uint16_t* s_act, float* s_best, const PipeStamp& st,
                                            int ph, const PipeBias& pb) {
    const SmallArgs& a = pa.a;
    GAS u32* err = gptr(a.bar_error);
    const int lane = threadIdx.x & 63, wave = wave_id();
    const int m = lane & 15, qd = lane >> 4;
    int32_t* s_besti = reinterpret_cast<int32_t*>(s_best + SMALL_NW * SMALL_ROWS);
    const int nks = a.D / 32;
    const int aoff = m * SMALL_KP + 8 * qd;
    const GAS BF16* lm_head = gptr(a.lm_head);
    const bool has_bias = a.bias.rowptr != nullptr;
    const GAS int32_t* b_col = gptr(a.bias.col);
    const GAS float* b_val = gptr(a.bias.val);
    const bool dbg = a.logits_dbg != nullptr;
    GAS float* logits_dbg = gptr(a.logits_dbg);
    GAS float* pv = gptr(pa.pv);
    GAS int32_t* pi = gptr(pa.pi);
    const int64_t row_hi = pb.end;
    const float base = pb.base;
    bool staged = false;
    for (int strip = wg; strip < a.n_strips; strip += nwg) {
        const int v0 = strip * TASC_LM_STRIP + wave * 16;
        const bool live = v0 < a.V;
        const GAS BF16* wrow = lm_head + (size_t)(live ? v0 / 16 : 0) * nks * 512 + lane * 8;
        constexpr int WG_KS = 18;
        bf16x8 w[WG_KS];
#pragma unroll
        for (int u = 0; u < WG_KS; ++u) w[u] = gld<bf16x8>(wrow + (size_t)min(u, nks - 1) * 512);
        const bool own = live && m < a.n_sel;
        const int pass = (strip - wg) / nwg;
        int64_t bp = pass == 0 ? pb.first[0] : pb.first[1];
        const int64_t be = row_hi;
        if (own && has_bias && pass >= 2) bp = pipe_bias_search(b_col, pb.first[1], row_hi, v0 + 4 * qd);   // more than two strips per workgroup: small grids only
        if (!staged) {
            NormRegs<6> xr;
            pipe_wait_hint(gptr(a.act) + (size_t)(a.n_layers - 1) * a.act_stride, err);
            pipe_load_gains<6>(gptr(a.gf), a.D, xr);
            pipe_poll_rows<6, 1>(gptr(a.x) + (size_t)(2 * a.n_layers) * a.x_stride, gptr(a.sel_rows), a.n_sel, a.D, xr, err);
            st.ready(ph);
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
            // a NaN maximum would read as "not written yet": it becomes -inf (such a row has no meaningful argmax anyway)
            if (!(bv == bv)) bv = -INFINITY;
            ll_st32(pv + (size_t)row * a.n_strips + strip, __float_as_uint(bv));
            ll_st32(pi + (size_t)row * a.n_strips + strip, (u32)bi);
        }
        __syncthreads();
    }
    st.done(ph);
}

// ---------------------------------------------------------------- argmax over strips, accept, rollback (one workgroup)
__device__ __forceinline__ void pipe_accept(const PipeArgs& pa, int32_t* s_amax, const PipeStamp& st, int ph) {
    const SmallArgs& al = pa.a;
    GAS u32* err = gptr(al.bar_error);
    const int lane = threadIdx.x & 63, wave = wave_id();
    const GAS float* pv = gptr(pa.pv);
    const GAS int32_t* pi = gptr(pa.pi);
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
    pipe_wait_hint(gptr(al.x) + (size_t)(2 * al.n_layers) * al.x_stride, err);
    for (int r = wave; r < n_sel; r += SMALL_NW) {
        float bv = -INFINITY;
        int32_t bi = 0x7FFFFFFF;
        for (int s = lane; s < n_strips; s += 64) {
            u32 vb, ib, spins = 0;
            for (;;) {
                vb = ll_ld32(pv + (size_t)r * n_strips + s);
                ib = ll_ld32(pi + (size_t)r * n_strips + s);
                if ((vb != PIPE_SENT && ib != PIPE_SENT) || ll_give_up(spins, err)) break;
            }
            const float v = __uint_as_float(vb);
            const int32_t i = (int32_t)ib;
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
    st.ready(ph);
    if (k < 0) return;
    const int b = threadIdx.x, nq = k + 1;
    if (b < B) {
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
    st.done(ph);
}

// ---------------------------------------------------------------- the step kernel
// NKS = head_dim / 32.  WKS = 3 serves d_model <= 768, WKS = 6 up to 1536.  Phases [phase_begin, phase_end) of the step
// run (numbering of kernels_small.h); a launch of the whole step is the product path, launches of single phases exist
// for the tests (same results, bit for bit).
template <int NKS, int WKS>
__global__ __launch_bounds__(SMALL_THREADS) void k_pipe_step(PipeArgs pa_in, int phase_begin, int phase_end) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    uint16_t* s_act = reinterpret_cast<uint16_t*>(lds + SMALL_LDS_ACT);
    f32x4* s_red = reinterpret_cast<f32x4*>(lds + SMALL_LDS_RED);
    float* s_attn = reinterpret_cast<float*>(lds);
    __shared__ float s_best[2 * SMALL_NW * SMALL_ROWS];
    __shared__ int32_t s_amax[SMALL_ROWS];
    __shared__ PipeArgs s_args;
    __shared__ TascLayerW s_layers[SMALL_MAX_LAYERS];
    __shared__ int32_t s_nrows[SMALL_ROWS], s_pos0[SMALL_ROWS];
    __shared__ int32_t s_bt[SMALL_MAX_BT];
    if (threadIdx.x == 0) s_args = pa_in;
    for (int i = threadIdx.x; i < pa_in.a.n_layers * (int)(sizeof(TascLayerW) / 8); i += SMALL_THREADS)
        reinterpret_cast<u64*>(s_layers)[i] = reinterpret_cast<const u64*>(pa_in.a.layers)[i];
    if (threadIdx.x < pa_in.a.B) {
        s_nrows[threadIdx.x] = pa_in.a.n_rows[threadIdx.x];
        s_pos0[threadIdx.x] = pa_in.a.pos0[threadIdx.x];
    }
    for (int i = threadIdx.x; i < pa_in.a.B * pa_in.a.max_blocks; i += SMALL_THREADS) s_bt[i] = pa_in.a.block_tab[i];
    __syncthreads();
    const SmallTabs tb = {s_layers, s_nrows, s_pos0, s_bt};
    const PipeArgs& pa = s_args;
    const SmallArgs& a = pa.a;
    const int wg = blockIdx.x, nwg = gridDim.x;
    const int n_phases = 3 + 5 * a.n_layers, n_lg_phases = 1 + 5 * a.n_layers;
    PipeStamp st;
    st.on = a.phase_ts != nullptr && wg < a.phase_ts_wgs && threadIdx.x == 0;
    st.n_phases = n_phases;
    st.ts = gptr(a.phase_ts) + (size_t)wg * n_phases * 2;
    int role = -1, lw = 0, lnw = 1;
#pragma unroll
    for (int r = 0; r < PIPE_N_ROLES; ++r)
        if (wg >= pa.role_base[r] && wg < pa.role_base[r] + pa.role_count[r]) {
            role = r;
            lw = wg - pa.role_base[r];
            lnw = pa.role_count[r];
        }
    int l0 = 0, l1 = 0;
    if (role >= 0) pipe_layer_range(role, a.n_layers, phase_begin, phase_end, l0, l1);
    // ---- embedding (phase 0), by the workgroups of the down projection: they are the last to be needed
    if (phase_begin == 0 && phase_end > 0 && role == PIPE_DOWN) {
        const GAS BF16* embed = gptr(a.embed);
        const GAS int32_t* row_tok = gptr(a.row_tok);
        GAS float* x = gptr(a.x);
        for (int r = lw; r < a.M; r += lnw) {
            const GAS BF16* e = embed + (size_t)row_tok[r] * a.D;
            for (int k = threadIdx.x * 8; k < a.D; k += SMALL_THREADS * 8) {
                const u32x4 u = gld<u32x4>(e + k);
                GAS float* o = x + (size_t)r * a.D + k;
                ll_st_f4(o, f32x4{bf2f(u[0] & 0xFFFFu), bf2f(u[0] >> 16), bf2f(u[1] & 0xFFFFu), bf2f(u[1] >> 16)});
                ll_st_f4(o + 4, f32x4{bf2f(u[2] & 0xFFFFu), bf2f(u[2] >> 16), bf2f(u[3] & 0xFFFFu), bf2f(u[3] >> 16)});
            }
        }
    }
    // ---- the other copy of the hand-over buffers gets its sentinels back for the next launch (nobody reads it now)
    if (pa.rearm_units > 0) {
        GAS u64* p = gptr(pa.rearm);
        for (size_t u = (size_t)wg * SMALL_THREADS + threadIdx.x; u < pa.rearm_units; u += (size_t)nwg * SMALL_THREADS) {
            gst(p + 2 * u, u32x4{PIPE_SENT, PIPE_SENT, PIPE_SENT, PIPE_SENT});
        }
    }
    PipeBias bias_at = {{0, 0}, 0, 0.f};
    if (a.n_sel > 0 && phase_begin <= n_lg_phases && phase_end > n_lg_phases) bias_at = pipe_bias_cursors(pa, wg, nwg);
    // ---- the layers
    if (role == PIPE_QKV) {
        const int share = ((a.H + 2 * a.Hkv) * (a.hd / 32) + lnw - 1) / lnw;
        if constexpr (WKS == 3) {
            if (share >= 3) role_qkv<3, 3>(pa, tb, lw, lnw, l0, l1, s_act, s_red, st);
            else if (share == 2) role_qkv<2, 3>(pa, tb, lw, lnw, l0, l1, s_act, s_red, st);
            else role_qkv<1, 3>(pa, tb, lw, lnw, l0, l1, s_act, s_red, st);
        } else {
            role_qkv<1, WKS>(pa, tb, lw, lnw, l0, l1, s_act, s_red, st);
        }
    } else if (role == PIPE_ATTN) {
        role_attn<NKS>(pa, tb, lw, lnw, l0, l1, s_attn, st);
    } else if (role == PIPE_GU) {
        const int share = (a.F / 16 + lnw - 1) / lnw;
        if constexpr (WKS == 3) {
            if (share >= 3) role_gate_up<3, 3>(pa, tb, lw, lnw, l0, l1, s_act, s_red, st);
            else if (share == 2) role_gate_up<2, 3>(pa, tb, lw, lnw, l0, l1, s_act, s_red, st);
            else role_gate_up<1, 3>(pa, tb, lw, lnw, l0, l1, s_act, s_red, st);
        } else {
            role_gate_up<1, WKS>(pa, tb, lw, lnw, l0, l1, s_act, s_red, st);
        }
    } else if (role == PIPE_O || role == PIPE_DOWN) {
        const bool o_proj = role == PIPE_O;
        const int K = o_proj ? a.H * a.hd : a.F;
        const int share = (a.D / 16 + lnw - 1) / lnw;
        if (K <= 768) {
            if (share >= 3) role_proj<3, 3>(pa, tb, o_proj, lw, lnw, l0, l1, s_act, s_red, st);
            else if (share == 2) role_proj<2, 3>(pa, tb, o_proj, lw, lnw, l0, l1, s_act, s_red, st);
            else role_proj<1, 3>(pa, tb, o_proj, lw, lnw, l0, l1, s_act, s_red, st);
        } else {
            if (share >= 3) role_proj<3, 6>(pa, tb, o_proj, lw, lnw, l0, l1, s_act, s_red, st);
            else if (share == 2) role_proj<2, 6>(pa, tb, o_proj, lw, lnw, l0, l1, s_act, s_red, st);
            else role_proj<1, 6>(pa, tb, o_proj, lw, lnw, l0, l1, s_act, s_red, st);
        }
    }
    // ---- LM head on every workgroup, accept on the last one (a workgroup without a role: it polls from early on)
    if (a.n_sel > 0 && phase_begin <= n_lg_phases && phase_end > n_lg_phases) pipe_lmhead(pa, wg, nwg, s_act, s_best, st, n_lg_phases, bias_at);
    if (a.n_sel > 0 && wg == nwg - 1 && phase_begin <= n_lg_phases + 1 && phase_end > n_lg_phases + 1)
        pipe_accept(pa, s_amax, st, n_lg_phases + 1);
}
