// gfx950 kernels for decode-step attention over a paged KV cache with shared
// prefixes (paper §3.1: a branch attends to shared prefix ++ own tokens; all
// branches of a request are served from one set of prefix pages).
//
// Everything is computed in "transposed" form so that no operand ever has to be
// shuffled between lanes.  With 16x16x32 bf16 MFMA (A: 16 x 32, B: 32 x 16,
// C: 16 x 16; lane l supplies A[l%16][8*(l/16)..+7], B[8*(l/16)..+7][l%16] and
// receives C[4*(l/16)..+3][l%16]):
//   S^T (tokens x rows) = K (tokens x d) * Q^T (d x rows)      A = K tile, B = Q^T
//   O^T (d x rows)      = V^T (d x tokens) * P^T (tokens x rows) A = V^T,   B = P^T
// The C fragment of S^T (lane: query row l%16, tokens 4*(l/16)..+3) is, after
// exp and rounding, already the B fragment of P^T: the 32 tokens of an MFMA
// k-step are two pages, lane group l/16 holding tokens 4*(l/16)..+3 of each.  The
// pool layout (K in groups of 8 dims, V^T in groups of 4 tokens) makes the A
// fragments contiguous 16-byte / 8-byte pieces with unit stride across lanes.
//
// Softmax state per query row (one lane column): running max m in log2 units
// (scale*log2(e) folded in), running sum l, unnormalised O.  Partials of the KV
// chunks of a sequence are combined through their (m, l) by the workgroup that
// delivers the sequence's last partial (merge_rows).
#include "taper_internal.h"

#include <algorithm>

namespace taper {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));

#define DEV __device__ __forceinline__

DEV f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0); }
DEV float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
DEV bf16x8 cat(bf16x4 a, bf16x4 b) { return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7); }
// KV is read exactly once per launch: stream it past the caches (measurably faster than cached loads)
template <typename T>
DEV T stream_load(const T* p) { return __builtin_nontemporal_load(p); }
DEV float max4(f32x4 v) { return fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])); }

// Scores of invalid tokens of a chunk's last 32-token block -> -inf.
// sx: tokens 4*qd+i of the block's first page, sy: of its second page.
DEV void mask_tail(f32x4& sx, f32x4& sy, int qd, int n_valid) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (4 * qd + i >= n_valid) sx[i] = -INFINITY;
        if (16 + 4 * qd + i >= n_valid) sy[i] = -INFINITY;
    }
}

// Online softmax over one 32-token block for one 16-row tile.  Every block passed
// in holds at least one valid token, so the new max is finite.
template <int DT>
DEV bf16x8 softmax_block(f32x4 sx, f32x4 sy, float c, float& m, float& l, f32x4 (&O)[DT]) {
    float mx = fmaxf(max4(sx), max4(sy));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float mn = fmaxf(m, mx * c);
    if (__any(mn > m)) {  // wave-uniform: rescale only when some row's max moved
        const float alpha = fast_exp2(m - mn);
        l *= alpha;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) O[dt] *= alpha;
        m = mn;
    }
    f32x8 p;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        p[i] = fast_exp2(fmaf(sx[i], c, -m));
        p[4 + i] = fast_exp2(fmaf(sy[i], c, -m));
    }
    l += ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
    return __builtin_convertvector(p, bf16x8);
}

DEV float sum_lane_groups(float v) {
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}


// Partials travel between workgroups inside one launch.  Workgroups may sit on
// different XCDs, whose L2s are not kept coherent for ordinary cached accesses,
// and a device-scope fence per workgroup (L2 write-back + invalidate) is far too
// slow.  So every partial word is written and read with device-scope atomic
// accesses (write-through stores, cache-bypassing loads, 8 bytes each), and the
// only ordering needed is "my stores have completed before I count myself in".
DEV void coherent_store2(float* p, float x, float y) {
    unsigned long long v = ((unsigned long long)__float_as_uint(y) << 32) | __float_as_uint(x);
    __hip_atomic_store((unsigned long long*)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
DEV float2 coherent_load2(const float* p) {
    const unsigned long long v = __hip_atomic_load((const unsigned long long*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_float2(__uint_as_float((unsigned)v), __uint_as_float((unsigned)(v >> 32)));
}
DEV void coherent_store4(float* p, f32x4 v) {
    coherent_store2(p, v[0], v[1]);
    coherent_store2(p + 2, v[2], v[3]);
}
DEV f32x4 coherent_load4(const float* p) {
    const float2 a = coherent_load2(p), b = coherent_load2(p + 2);
    f32x4 r = {a.x, a.y, b.x, b.y};
    return r;
}
// all of this thread's earlier stores have completed (no cache maintenance)
DEV void stores_done() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup"); }

// Log-sum-exp merge of all partials of (sequence s, kv head hk) -- its request's
// prefix chunks and its own private chunks -- then normalisation and rounding to
// bf16.  Threads idx0, idx0+stride, ... each own one float4 of the g x D result;
// a thread works on U of them at once and takes the entries four at a time, so
// that 4*U independent loads are in flight per round (the loads bypass the caches
// and cost a full memory latency each).  Entries are taken in plan order, so the
// result does not depend on which workgroup happens to run this.
template <int D, int U>
DEV void merge_rows(const StepArgs& a, const int s, const int hk, const int idx0, const int stride) {
    const int g = a.gqa;
    const int total = g * (D / 4);
    const int e0 = a.merge_start[s], e1 = a.merge_start[s + 1];
    for (int base = idx0; base < total; base += stride * U) {
        float M[U], L[U];
        f32x4 acc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            M[u] = -INFINITY;
            L[u] = 0.f;
            acc[u] = (f32x4)(0.f);
        }
        for (int e = e0; e < e1; e += 4) {
            float2 ml[U][4];
            f32x4 o[U][4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const bool have = e + k < e1;
                const taper_merge_entry me = a.merge[have ? e + k : e];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int idx = base + u * stride;
                    const bool ok = have && idx < total;
                    const int j = ok ? idx / (D / 4) : 0, d4 = ok ? idx % (D / 4) : 0;
                    const int64_t rowi = (int64_t)me.first_row + (int64_t)hk * me.rows_per_head + j;
                    ml[u][k] = coherent_load2((const float*)(a.ws_ml + rowi));
                    o[u][k] = coherent_load4(a.ws_o + rowi * D + 4 * d4);
                    if (!ok) ml[u][k] = make_float2(-INFINITY, 0.f);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float mn = fmaxf(fmaxf(M[u], fmaxf(ml[u][0].x, ml[u][1].x)), fmaxf(ml[u][2].x, ml[u][3].x));
                const float keep = fast_exp2(M[u] - mn);  // first round: exp2(-inf) = 0
                L[u] *= keep;
                acc[u] *= keep;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float w = fast_exp2(ml[u][k].x - mn);
                    L[u] += w * ml[u][k].y;
                    acc[u] += w * o[u][k];
                }
                M[u] = mn;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int idx = base + u * stride;
            if (idx < total) {
                const int j = idx / (D / 4), d4 = idx % (D / 4);
                const int h = hk * g + j;
                const f32x4 r = acc[u] * (1.0f / L[u]);
                *(bf16x4*)((__bf16*)a.out + ((int64_t)s * a.n_q_heads + h) * D + 4 * d4) = __builtin_convertvector(r, bf16x4);
                if (a.lse && d4 == 0) a.lse[(int64_t)s * a.n_q_heads + h] = (M[u] + __log2f(L[u])) * 0.6931471805599453f;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// The work queue.  A unit is a run of tokens of one segment (a request's shared
// prefix, or one sequence's private tokens).  Workgroups are persistent: each
// streams a unit, writes a partial, and goes on with the next unit it holds.
// ---------------------------------------------------------------------------
struct Unit {  // wave-uniform view of a queue entry
    const int32_t* row;  // block-table entries of its pages
    int seq0, n_branch, n_tok, part_base;
    int kind;  // 0 shared, 1 private, -1 none (past the end of the queue)
};

DEV Unit fetch_unit(const StepArgs& a, int u) {
    u = __builtin_amdgcn_readfirstlane(u);
    Unit d;
    d.row = a.bt;
    d.seq0 = d.n_branch = d.n_tok = d.part_base = 0;
    d.kind = -1;
    if (u >= 0 && u < a.n_items) {
        const taper_work_item it = a.items[u];
        d.row = a.bt + (int64_t)it.seq0 * a.bt_stride + it.page0;
        d.seq0 = it.seq0;
        d.n_branch = it.n_branch;
        d.n_tok = it.n_tokens;
        d.part_base = it.part_base;
        d.kind = it.kind;
    }
    return d;
}

// What a workgroup carries from unit to unit.  Closing a unit must not stall the
// streaming, so it is spread over three closes: when unit A is closed its partial
// rows are stored (and not waited for); at the next close, once every wave has seen
// its own stores complete, A's arrivals are announced with atomics whose results are
// not waited for either; at the close after that the results are looked at and the
// sequences that A completed are merged.  The claim of a further unit from the
// head's queue travels the same way (issued at one close, used at the next).
struct Flow {
    Unit cur, next;   // the unit being computed and the one after it (known, so loads can run ahead into it)
    int n_closed;     // units closed so far; its parity selects the LDS buffers of a close
    int b_seq0, b_n;  // sequences of the unit closed last: partial rows stored, arrivals not yet announced
    int c_seq0, c_n;  // sequences of the unit closed before: arrivals announced, results in pend_old
    int pend_claim;   // thread 0: queue index its last claim returned
    int pend_old;     // thread t < c_n: arrival count of sequence c_seq0 + t before this workgroup's increment
    int since;        // vector memory instructions this wave has issued since it last stored partial rows
#ifdef TAPER_WG_TRACE
    long long t_close;  // clock ticks spent closing units
    long long t_bar, t_comb;  // ... of which up to the barrier, and in combine + stores
    int n_close;
#endif
};

struct HandoffSmem {
    int claim;
    int last[64];
};

// Thread side of an arrival whose atomic has returned `old`: the workgroup that
// delivered the last partial of (s, hk) must merge; every other partial has then
// been written through (each writer saw its stores complete before its increment).
// The counter is left at zero for the next launch.
DEV bool settle_arrival(const StepArgs& a, const int s, const int hk, const int old) {
    const int n_entries = a.merge_start[s + 1] - a.merge_start[s];
    const bool last = old == n_entries - 1;
    if (last) a.counters[(int64_t)s * a.n_kv_heads + hk] = 0;
    return last;
}

// Vector memory operations of a wave complete in the order they were issued, so
// "at most KEEP outstanding" means everything but the youngest KEEP has completed.
// Waits until this wave's partial-row stores have completed while leaving up to
// KEEP younger loads (the block fetched ahead) in flight.
template <int KEEP>
DEV void own_stores_done(const int since) {
    static_assert(KEEP == 8 || KEEP == 12 || KEEP == 16 || KEEP == 24, "add the s_waitcnt form");
    if (since >= KEEP) {
        if (KEEP == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        if (KEEP == 12) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
        if (KEEP == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        if (KEEP == 24) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
    } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
}

// First half of a close, before the workgroup barrier: this wave's stores of the
// unit closed last are complete, and the results of the atomics issued at the last
// close go to LDS.
template <int KEEP>
DEV void close_publish(const StepArgs& a, const int hk, Flow& f, HandoffSmem* hs2) {
    const int tid = threadIdx.x;
    HandoffSmem& hs = hs2[f.n_closed & 1];
    own_stores_done<KEEP>(f.since);
    if (tid == 0) hs.claim = f.pend_claim;
    if (tid < f.c_n) hs.last[tid] = settle_arrival(a, f.c_seq0 + tid, hk, f.pend_old);
}

// Second half, after the barrier and after this unit's partial rows have been
// stored: the atomics of this close, the merges the published results call for, and
// the move to the next unit.
template <int D>
DEV void close_advance(const StepArgs& a, const int hk, Flow& f, HandoffSmem* hs2) {
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const HandoffSmem& hs = hs2[f.n_closed & 1];
    f.since = 0;
    if (tid == 0) f.pend_claim = 2 * a.wgs_per_head + atomicAdd(a.queue + hk, 1);
    int old = 0;
    if (tid < f.b_n) old = atomicAdd(a.counters + (int64_t)(f.b_seq0 + tid) * a.n_kv_heads + hk, 1);
    if (f.c_n == 1) {
        if (hs.last[0]) merge_rows<D, 1>(a, f.c_seq0, hk, tid, 256);
    } else {
        for (int b = wave; b < f.c_n; b += 4)
            if (hs.last[b]) merge_rows<D, 2>(a, f.c_seq0 + b, hk, tid & 63, 64);
    }
    f.pend_old = old;
    f.c_seq0 = f.b_seq0;
    f.c_n = f.b_n;
    f.b_seq0 = f.cur.seq0;
    f.b_n = f.cur.n_branch;
    f.cur = f.next;
    f.next = fetch_unit(a, hs.claim);
    f.n_closed++;
}

// After the last unit: announce what is still unannounced and merge what that completes.
template <int D>
DEV void drain(const StepArgs& a, const int hk, Flow& f, HandoffSmem* hs2) {
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int round = 0; round < 2; ++round) {
        HandoffSmem& hs = hs2[f.n_closed & 1];
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (tid < f.c_n) hs.last[tid] = settle_arrival(a, f.c_seq0 + tid, hk, f.pend_old);
        __syncthreads();
        int old = 0;
        if (tid < f.b_n) old = atomicAdd(a.counters + (int64_t)(f.b_seq0 + tid) * a.n_kv_heads + hk, 1);
        if (f.c_n == 1) {
            if (hs.last[0]) merge_rows<D, 1>(a, f.c_seq0, hk, tid, 256);
        } else {
            for (int b = wave; b < f.c_n; b += 4)
                if (hs.last[b]) merge_rows<D, 2>(a, f.c_seq0 + b, hk, tid & 63, 64);
        }
        f.pend_old = old;
        f.c_seq0 = f.b_seq0;
        f.c_n = f.b_n;
        f.b_n = 0;
        f.n_closed++;
    }
}

#define INLINE_LAMBDA __attribute__((always_inline))
#ifdef TAPER_RUNS_AS_CALLS
#define RUN_FN __device__ __attribute__((noinline))
#else
#define RUN_FN __device__ __forceinline__
#endif

// ---------------------------------------------------------------------------
// Private / serial units: one sequence's g query rows (one 16-row tile, rows
// >= g idle).  No reuse across waves, so K/V go straight from HBM into MFMA
// operand registers; the four waves of a workgroup take alternate 32-token
// blocks, each wave keeping two blocks in flight, and combine through LDS when a
// unit is closed.  A wave's loads run ahead into the next unit, so the memory
// pipeline is not drained at unit boundaries.
// ---------------------------------------------------------------------------
template <int D>
struct KVRegs {
    bf16x8 kx[D / 32], ky[D / 32];
    bf16x4 va[D / 16], vb[D / 16];
};

template <int D>
struct PrivateSmem {  // the four waves' states of a unit being closed, double buffered over closes
    float o[2][4][16][D + 4];
    float2 ml[2][4][16];
};

template <int D, int WAVES_PER_SIMD>
RUN_FN void private_run(
    const StepArgs& a, const int hk, Flow& f_io, PrivateSmem<D>& sm, HandoffSmem* hs) {
    Flow f = f_io;
    constexpr int KS = D / 32, DT = D / 16, TILE = 16 * D;
    constexpr int BLOCK_LOADS = 2 * KS + 2 * DT;  // vector loads of one block per wave
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, qd = lane >> 4;
    const int Hkv = a.n_kv_heads, g = a.gqa;
    const __bf16* __restrict__ kvb = (const __bf16*)a.kv;
    const int64_t page_elems = 2LL * Hkv * TILE;
    const float c = a.scale_log2e;
    const int koff = lane * 8, voff = qd * (4 * D) + n * 4;

    bf16x8 qf[KS];
    auto load_q = [&](const Unit& un, bf16x8 (&q)[KS]) INLINE_LAMBDA {
        const __bf16* qrow = (const __bf16*)a.q + ((int64_t)un.seq0 * a.n_q_heads + hk * g + (n < g ? n : 0)) * D;
#pragma unroll
        for (int j = 0; j < KS; ++j) {
            bf16x8 v = *(const bf16x8*)(qrow + 8 * (4 * j + qd));
            if (n >= g) v = (bf16x8)(0);
            q[j] = v;
        }
    };
    load_q(f.cur, qf);
    float m = -INFINITY, l = 0.f;
    f32x4 O[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) O[dt] = (f32x4)(0.f);

    // This wave's blocks of a unit are wave, wave+4, ...  While one register set is computed the
    // other is in flight; when the unit has no further block for this wave, the set is filled
    // with the wave's first block of the next unit instead, so a load is in flight across the
    // close of a unit too.
    auto issue = [&](const Unit& un, const int b, KVRegs<D>& r) INLINE_LAMBDA {
        const int n_pages = (un.n_tok + 15) >> 4;
        const int64_t pa = un.row[2 * b], pb = un.row[2 * b + 1 < n_pages ? 2 * b + 1 : 2 * b];
        const __bf16* ka = kvb + pa * page_elems + (int64_t)hk * TILE;
        const __bf16* kb = kvb + pb * page_elems + (int64_t)hk * TILE;
        const __bf16* va = ka + (int64_t)Hkv * TILE;
        const __bf16* vb = kb + (int64_t)Hkv * TILE;
#pragma unroll
        for (int j = 0; j < KS; ++j) {
            r.kx[j] = stream_load((const bf16x8*)(ka + koff + j * 512));
            r.ky[j] = stream_load((const bf16x8*)(kb + koff + j * 512));
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            r.va[dt] = stream_load((const bf16x4*)(va + voff + dt * 64));
            r.vb[dt] = stream_load((const bf16x4*)(vb + voff + dt * 64));
        }
        f.since += BLOCK_LOADS;
    };
    auto compute = [&](const KVRegs<D>& r, const int b) INLINE_LAMBDA {
        f32x4 sx = (f32x4)(0.f), sy = (f32x4)(0.f);
#pragma unroll
        for (int j = 0; j < KS; ++j) {
            sx = mfma16(r.kx[j], qf[j], sx);
            sy = mfma16(r.ky[j], qf[j], sy);
        }
        const int nv = f.cur.n_tok - 32 * b;
        if (nv < 32) mask_tail(sx, sy, qd, nv);
        const bf16x8 pf = softmax_block<DT>(sx, sy, c, m, l, O);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) O[dt] = mfma16(cat(r.va[dt], r.vb[dt]), pf, O[dt]);
    };
    auto close_unit = [&]() INLINE_LAMBDA {
#ifdef TAPER_WG_TRACE
        const long long t_in = wall_clock64();
#endif
        const int par = f.n_closed & 1;
        l = sum_lane_groups(l);
        if (n < g) {
            if (qd == 0) sm.ml[par][wave][n] = make_float2(m, l);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) *(f32x4*)&sm.o[par][wave][n][16 * dt + 4 * qd] = O[dt];
        }
        close_publish<BLOCK_LOADS>(a, hk, f, hs);
        // q of the unit that becomes current (qf is dead: every block of f.cur is computed)
        if (f.next.kind == 1) load_q(f.next, qf);
        __syncthreads();
#ifdef TAPER_WG_TRACE
        const long long t_b = wall_clock64();
        f.t_bar += t_b - t_in;
#endif
        for (int idx = tid; idx < g * (D / 4); idx += 256) {
            const int r = idx / (D / 4), d4 = idx % (D / 4);
            float mw[4], M = -INFINITY;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                mw[w] = sm.ml[par][w][r].x;
                M = fmaxf(M, mw[w]);
            }
            float L = 0.f;
            f32x4 acc = (f32x4)(0.f);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float wg = mw[w] == -INFINITY ? 0.f : fast_exp2(mw[w] - M);  // a wave may have had no block
                L += wg * sm.ml[par][w][r].y;
                acc += wg * *(const f32x4*)&sm.o[par][w][r][4 * d4];
            }
            const int64_t slot = (int64_t)f.cur.part_base + hk * g + r;
            coherent_store4(a.ws_o + slot * D + 4 * d4, acc);
            if (d4 == 0) coherent_store2((float*)(a.ws_ml + slot), M, L);
        }
#ifdef TAPER_WG_TRACE
        f.t_comb += wall_clock64() - t_b;
#endif
        close_advance<D>(a, hk, f, hs);
        m = -INFINITY;
        l = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) O[dt] = (f32x4)(0.f);
#ifdef TAPER_WG_TRACE
        f.t_close += wall_clock64() - t_in;
        f.n_close++;
#endif
    };

    int b = wave;        // this wave's current block of f.cur
    bool ahead = false;  // the set about to be computed already holds (or is receiving) block b
    // One step: `cur` holds block b of f.cur (if the unit has one for this wave), `other` is free.
    // Returns false when the run is over.
    auto step = [&](KVRegs<D>& cur, KVRegs<D>& other) INLINE_LAMBDA -> bool {
        if (32 * b < f.cur.n_tok) {
            if (!ahead) issue(f.cur, b, cur);
            const int b1 = b + 4;
            ahead = true;
            if (32 * b1 < f.cur.n_tok)
                issue(f.cur, b1, other);
            else if (f.next.kind == 1 && 32 * wave < f.next.n_tok)
                issue(f.next, wave, other);  // the next unit's first block for this wave
            else
                ahead = false;
            compute(cur, b);
            b = b1;
        }
        if (32 * b >= f.cur.n_tok) {
            close_unit();
            b = wave;
            if (f.cur.kind != 1) return false;
        }
        return true;
    };
    KVRegs<D> r0, r1;
    for (;;) {
        if (!step(r0, r1)) break;
        if (!step(r1, r0)) break;
    }
    f_io = f;
}

// ---------------------------------------------------------------------------
// Shared-prefix units: a request's prefix pages are staged in LDS once (64
// tokens per iteration, double buffered) and multiplied against the query rows
// of all n_branch admitted branches x g heads.  16-row tiles are dealt
// round-robin to the four waves, up to NTW tiles per wave.  Staging runs ahead
// into the next unit.
// ---------------------------------------------------------------------------
template <int D>
struct SharedSmem {
    static constexpr int TILE = 16 * D;
    static constexpr int QE = 4 * D;        // elements of one 4-token quarter of a V tile
    static constexpr int VQ = QE + 64;      // padded quarter: odd multiple of 128 B -> quarters alternate bank halves
    static constexpr int PAGE_LDS = TILE + 4 * VQ;
    static constexpr int BUF = 4 * PAGE_LDS;  // 4 pages = 64 tokens
    __bf16 kv[2 * BUF];
};

template <int D, int NTW>
RUN_FN void shared_run(
    const StepArgs& a, const int hk, Flow& f_io, SharedSmem<D>& sm, HandoffSmem* hs) {
    Flow f = f_io;
    constexpr int KS = D / 32, DT = D / 16, TILE = 16 * D;
    constexpr int QE = SharedSmem<D>::QE, VQ = SharedSmem<D>::VQ, PAGE_LDS = SharedSmem<D>::PAGE_LDS,
                  BUF = SharedSmem<D>::BUF;
    __bf16* lds = sm.kv;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, qd = lane >> 4;
    const int Hkv = a.n_kv_heads, g = a.gqa;
    const __bf16* __restrict__ kvb = (const __bf16*)a.kv;
    const int64_t page_elems = 2LL * Hkv * TILE;
    const float c = a.scale_log2e;
    const int se = tid * 8;                       // staging: this thread's element offset inside a tile
    const bool stager = se < TILE;
    const int sv = (se / QE) * VQ + se % QE;      // ... and inside the padded V tile in LDS
    const int koff = lane * 8;
    const int voff = TILE + qd * VQ + n * 4;

    int R = 0, n_act = 0;  // query rows of f.cur and how many of this wave's tiles hold some
    bf16x8 qf[NTW][KS];
    float m[NTW], l[NTW];
    f32x4 O[NTW][DT];
    auto open_unit = [&](const Unit& un, bool with_q) INLINE_LAMBDA {
        R = un.n_branch * g;
        const int tiles = (R + 15) >> 4;
        n_act = (tiles - wave + 3) >> 2;  // tiles wave, wave+4, ...
        n_act = n_act < 0 ? 0 : (n_act > NTW ? NTW : n_act);
#pragma unroll
        for (int k = 0; k < NTW; ++k) {
            if (with_q) {
                const int r = 16 * (wave + 4 * k) + n;
                const bool ok = k < n_act && r < R;
                const int rr = ok ? r : 0;
                const __bf16* qrow = (const __bf16*)a.q + ((int64_t)(un.seq0 + rr / g) * a.n_q_heads + hk * g + rr % g) * D;
#pragma unroll
                for (int j = 0; j < KS; ++j) {
                    bf16x8 v = *(const bf16x8*)(qrow + 8 * (4 * j + qd));
                    if (!ok) v = (bf16x8)(0);
                    qf[k][j] = v;
                }
            }
            m[k] = -INFINITY;
            l[k] = 0.f;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) O[k][dt] = (f32x4)(0.f);
        }
    };
    open_unit(f.cur, true);

    // compute cursor: 64-token block bC of f.cur.  Load cursor: block bL of f.cur or of f.next.
    int bC = 0, bL = 0;
    bool L_in_next = false, have_pages = false;
    int pg[4] = {0, 0, 0, 0};
    auto seek = [&]() INLINE_LAMBDA {
        for (;;) {
            const Unit& un = L_in_next ? f.next : f.cur;
            const int n_pages = (un.n_tok + 15) >> 4;
            if (4 * bL < n_pages) {
#pragma unroll
                for (int i = 0; i < 4; ++i) pg[i] = un.row[4 * bL + i < n_pages ? 4 * bL + i : n_pages - 1];
                have_pages = true;
                return;
            }
            if (L_in_next || f.next.kind != 0) return;
            L_in_next = true;
            bL = 0;
        }
    };
    auto fetch = [&](bf16x8 (&stg)[8]) INLINE_LAMBDA -> bool {
        if (!have_pages) seek();
        if (!have_pages) return false;
        if (stager) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const __bf16* kp = kvb + (int64_t)pg[i] * page_elems + (int64_t)hk * TILE + se;
                stg[2 * i] = stream_load((const bf16x8*)kp);
                stg[2 * i + 1] = stream_load((const bf16x8*)(kp + (int64_t)Hkv * TILE));
            }
            f.since += 8;
        }
        ++bL;
        have_pages = false;
        seek();
        return true;
    };
    auto stage_store = [&](int buf, const bf16x8 (&stg)[8]) INLINE_LAMBDA {
        if (stager) {
            __bf16* base = lds + buf * BUF;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                *(bf16x8*)(base + i * PAGE_LDS + se) = stg[2 * i];
                *(bf16x8*)(base + i * PAGE_LDS + TILE + sv) = stg[2 * i + 1];
            }
        }
    };
    auto close_unit = [&]() INLINE_LAMBDA {
#ifdef TAPER_WG_TRACE
        const long long t_in = wall_clock64();
#endif
        close_publish<16>(a, hk, f, hs);
        __syncthreads();
#pragma unroll
        for (int k = 0; k < NTW; ++k) {
            if (k < n_act) {
                const float lt = sum_lane_groups(l[k]);
                const int r = 16 * (wave + 4 * k) + n;
                if (r < R) {
                    const int64_t slot = (int64_t)f.cur.part_base + (int64_t)hk * R + r;
                    if (qd == 0) coherent_store2((float*)(a.ws_ml + slot), m[k], lt);
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) coherent_store4(a.ws_o + slot * D + 16 * dt + 4 * qd, O[k][dt]);
                }
            }
        }
        const bool more = f.next.kind == 0;
        if (more) open_unit(f.next, true);  // its q loads overlap the rest of the close
        close_advance<D>(a, hk, f, hs);
        if (!more) open_unit(f.cur, false);
        bC = 0;
        if (L_in_next) {
            L_in_next = false;
        } else {
            bL = 0;
            have_pages = false;
        }
#ifdef TAPER_WG_TRACE
        f.t_close += wall_clock64() - t_in;
        f.n_close++;
#endif
    };
    auto consume = [&](int buf) INLINE_LAMBDA {
        while (64 * bC >= f.cur.n_tok) close_unit();  // the staged block belongs to a later unit
        if (n_act > 0) {
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const int nv = f.cur.n_tok - (64 * bC + 32 * hf);
                if (nv <= 0) break;
                const __bf16* pa = lds + buf * BUF + (2 * hf) * PAGE_LDS;
                const __bf16* pb = pa + PAGE_LDS;
                bf16x8 kx[KS], ky[KS];
#pragma unroll
                for (int j = 0; j < KS; ++j) {
                    kx[j] = *(const bf16x8*)(pa + koff + j * 512);
                    ky[j] = *(const bf16x8*)(pb + koff + j * 512);
                }
                bf16x8 pf[NTW];
#pragma unroll
                for (int k = 0; k < NTW; ++k) {
                    if (k < n_act) {
                        f32x4 sx = (f32x4)(0.f), sy = (f32x4)(0.f);
#pragma unroll
                        for (int j = 0; j < KS; ++j) {
                            sx = mfma16(kx[j], qf[k][j], sx);
                            sy = mfma16(ky[j], qf[k][j], sy);
                        }
                        if (nv < 32) mask_tail(sx, sy, qd, nv);
                        pf[k] = softmax_block<DT>(sx, sy, c, m[k], l[k], O[k]);
                    }
                }
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const bf16x8 vf = cat(*(const bf16x4*)(pa + voff + dt * 64), *(const bf16x4*)(pb + voff + dt * 64));
#pragma unroll
                    for (int k = 0; k < NTW; ++k)
                        if (k < n_act) O[k][dt] = mfma16(vf, pf[k], O[k][dt]);
                }
            }
        }
        ++bC;
    };

    bf16x8 stgA[8], stgB[8];
    for (;;) {
        // nothing staged here, and no wave is still reading LDS
        bool a0 = fetch(stgA);
        if (!a0) {
            close_unit();
            if (f.cur.kind != 0) {
                f_io = f;
                return;
            }
            continue;
        }
        bool a1 = fetch(stgB);
        stage_store(0, stgA);
        __syncthreads();
        for (;;) {
            // block t in LDS buffer 0, block t+1 (if any) in stgB
            a0 = a1 && fetch(stgA);
            consume(0);
            if (!a1) break;
            stage_store(1, stgB);
            __syncthreads();
            // block t+1 in LDS buffer 1, block t+2 (if any) in stgA
            a1 = a0 && fetch(stgB);
            consume(1);
            if (!a0) break;
            stage_store(0, stgA);
            __syncthreads();
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// One launch per layer.  Workgroups are persistent and bound to a KV head
// (blockIdx % n_kv_heads, which with round-robin dispatch also keeps a head's
// partials inside one XCD's L2).  Workgroup w of a head starts with units w and
// 2W - 1 - w of the plan's queue (W = workgroups per head) and afterwards takes
// the next unclaimed unit from the head's counter.
// ---------------------------------------------------------------------------
template <int D, int NTW>  // NTW = 0: the queue holds no shared-prefix unit
__global__ __launch_bounds__(256, (NTW <= 2 ? 2 : 1)) void decode_kernel(StepArgs a) {
    union Smem {
        SharedSmem<D> sh;
        PrivateSmem<D> pr;
    };
    __shared__ __attribute__((aligned(16))) char smem_raw[sizeof(Smem)];
    __shared__ HandoffSmem hs[2];
    const int hk = blockIdx.x % a.n_kv_heads;
    const int W = a.wgs_per_head;
    const int w = blockIdx.x / a.n_kv_heads;
#ifdef TAPER_WG_TRACE  // development builds only: per-workgroup start/end clock into the lse buffer
    long long* trace = (long long*)a.lse;
    a.lse = nullptr;
    if (threadIdx.x == 0) trace[3 * blockIdx.x] = wall_clock64();
#endif
    Flow f;
    f.cur = fetch_unit(a, w);
    f.next = fetch_unit(a, 2 * W - 1 - w);  // the second round in reverse, since units shrink along the queue
    f.n_closed = f.b_seq0 = f.b_n = f.c_seq0 = f.c_n = f.pend_claim = f.pend_old = f.since = 0;
#ifdef TAPER_WG_TRACE
    f.t_close = f.t_bar = f.t_comb = 0;
    f.n_close = 0;
#endif
    if (f.cur.kind >= 0) {
        if (threadIdx.x == 0) f.pend_claim = 2 * W + atomicAdd(a.queue + hk, 1);
        while (f.cur.kind >= 0) {
            if constexpr (NTW > 0) {
                if (f.cur.kind == 0) {
                    shared_run<D, (NTW > 0 ? NTW : 1)>(a, hk, f, *reinterpret_cast<SharedSmem<D>*>(smem_raw), hs);
                    continue;
                }
            }
            private_run<D, (NTW <= 2 ? 2 : 1)>(a, hk, f, *reinterpret_cast<PrivateSmem<D>*>(smem_raw), hs);
        }
        drain<D>(a, hk, f, hs);
    }
#ifdef TAPER_WG_TRACE
    if (threadIdx.x == 0) {
        trace[3 * blockIdx.x + 1] = wall_clock64();
        trace[3 * blockIdx.x + 2] = f.t_close * 1000 + f.n_close;
        trace[3 * gridDim.x + 2 * blockIdx.x] = f.t_bar;
        trace[3 * gridDim.x + 2 * blockIdx.x + 1] = f.t_comb;
    }
#endif
    // the last workgroup to leave puts the queue back to zero for the next launch
    if (threadIdx.x == 0 && atomicAdd(a.queue + a.n_kv_heads, 1) == (int)gridDim.x - 1) {
        for (int h = 0; h <= a.n_kv_heads; ++h) a.queue[h] = 0;
    }
}

// ---------------------------------------------------------------------------
// Queues that hold private units only: three waves of a workgroup stream, the
// fourth is the workgroup's control wave.  Everything with a long latency that
// is not KV streaming (claims from the queue, combining the streaming waves'
// states, storing partial rows and waiting for the stores, arrival atomics,
// merges) is the control wave's business, so the streaming waves never wait for
// anything but their own KV loads.  The waves talk through LDS only:
//   ring[k % RING]   unit number k of this workgroup, published by the control wave
//   blk[k % RING]    next unclaimed 32-token block of unit k (streaming waves take blocks as they go)
//   done[k % RING]   streaming waves that have left unit k and dumped their state
//   consumed         units whose states the control wave has combined (their state slots are free)
// No workgroup barrier is used.  Every wait is a bounded spin on an LDS word that
// another wave is certain to write; if a spin ever ran out, the wave raises the
// error word and leaves.
// ---------------------------------------------------------------------------
constexpr int RING = 4;
constexpr int STREAM_WAVES = 3;
constexpr int SPIN_LIMIT = 1 << 22;  // x s_sleep(1) of 64 clocks: seconds, far beyond any legitimate wait

struct RingUnit {
    long long row_off;  // elements from the block table's base to the unit's first entry
    int seq0, n_tok, part_base, kind;
};

template <int D>
struct SpecSmem {
    float o[2][STREAM_WAVES][16][D + 4];
    float2 ml[2][STREAM_WAVES][16];
    RingUnit ring[RING];
    int blk[RING];
    int done[RING];
    int published;  // units (and the end marker) published so far
    int consumed;
    int failed;
};

DEV int lds_load_acquire(const int* p) { return __hip_atomic_load(p, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP); }
DEV void lds_store_release(int* p, int v) { __hip_atomic_store(p, v, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP); }

// Spins until *p >= want (or the workgroup has failed).  Returns false on failure.
DEV bool spin_until_at_least(const StepArgs& a, int* failed, const int* p, const int want) {
    for (int i = 0; i < SPIN_LIMIT; ++i) {
        if (lds_load_acquire(p) >= want) return true;
        if (lds_load_acquire(failed)) return false;
        __builtin_amdgcn_s_sleep(1);
    }
    lds_store_release(failed, 1);
    a.queue[a.n_kv_heads + 1] = 1;  // error word, checked by the host after synchronising
    return false;
}

template <int D>
DEV void stream_wave(const StepArgs& a, const int hk, SpecSmem<D>& sm, const int wave) {
    constexpr int KS = D / 32, DT = D / 16, TILE = 16 * D;
    const int lane = threadIdx.x & 63;
    const int n = lane & 15, qd = lane >> 4;
    const int Hkv = a.n_kv_heads, g = a.gqa;
    const __bf16* __restrict__ kvb = (const __bf16*)a.kv;
    const int64_t page_elems = 2LL * Hkv * TILE;
    const float c = a.scale_log2e;
    const int koff = lane * 8, voff = qd * (4 * D) + n * 4;

    auto read_ring = [&](const int k, RingUnit& u) INLINE_LAMBDA {
        const RingUnit& r = sm.ring[k % RING];
        u.row_off = ((long long)__builtin_amdgcn_readfirstlane((int)(r.row_off >> 32)) << 32) |
                    (unsigned)__builtin_amdgcn_readfirstlane((int)r.row_off);
        u.seq0 = __builtin_amdgcn_readfirstlane(r.seq0);
        u.n_tok = __builtin_amdgcn_readfirstlane(r.n_tok);
        u.part_base = __builtin_amdgcn_readfirstlane(r.part_base);
        u.kind = __builtin_amdgcn_readfirstlane(r.kind);
    };
    bf16x8 qf[KS], qn[KS];  // q of the unit being computed / of the unit the loads have run ahead into
    auto load_q = [&](const RingUnit& un, bf16x8 (&q)[KS]) INLINE_LAMBDA {
        const __bf16* qrow = (const __bf16*)a.q + ((int64_t)un.seq0 * a.n_q_heads + hk * g + (n < g ? n : 0)) * D;
#pragma unroll
        for (int j = 0; j < KS; ++j) {
            bf16x8 v = *(const bf16x8*)(qrow + 8 * (4 * j + qd));
            if (n >= g) v = (bf16x8)(0);
            q[j] = v;
        }
    };
    float m = -INFINITY, l = 0.f;
    f32x4 O[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) O[dt] = (f32x4)(0.f);

    int kC = 0, kL = 0;  // this wave computes unit kC; it claims blocks of unit kL (kC or kC + 1)
    RingUnit uC, uL;
    if (!spin_until_at_least(a, &sm.failed, &sm.published, 1)) return;
    read_ring(0, uC);
    if (uC.kind != 1) return;
    uL = uC;
    load_q(uC, qf);
#pragma unroll
    for (int j = 0; j < KS; ++j) qn[j] = qf[j];

    // The block this wave loads next is claimed one step before its loads are issued, together
    // with its page ids, so neither the LDS round trip nor the block-table fetch delays the loads.
    int nu = -1, nb = 0;       // claimed block: unit number (< 0: none) and block index
    int64_t npa = 0, npb = 0;  // its pages
    auto claim = [&]() INLINE_LAMBDA {
        for (;;) {
            int got = 0;
            if (lane == 0) got = __hip_atomic_fetch_add(&sm.blk[kL % RING], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            const int b = __builtin_amdgcn_readfirstlane(got);
            if (32 * b < uL.n_tok) {
                const int32_t* row = a.bt + uL.row_off;
                const int n_pages = (uL.n_tok + 15) >> 4;
                npa = row[2 * b];
                npb = row[2 * b + 1 < n_pages ? 2 * b + 1 : 2 * b];
                nu = kL;
                nb = b;
                return;
            }
            // unit kL has no block left: run ahead into the next unit if it is there, one unit at most
            if (kL > kC || lds_load_acquire(&sm.published) <= kL + 1) return;
            RingUnit nx;
            read_ring(kL + 1, nx);
            if (nx.kind != 1) return;
            ++kL;
            uL = nx;
            load_q(uL, qn);  // long before the first block of that unit is computed
        }
    };
    auto issue = [&](KVRegs<D>& r) INLINE_LAMBDA {
        const __bf16* ka = kvb + npa * page_elems + (int64_t)hk * TILE;
        const __bf16* kb = kvb + npb * page_elems + (int64_t)hk * TILE;
        const __bf16* va = ka + (int64_t)Hkv * TILE;
        const __bf16* vb = kb + (int64_t)Hkv * TILE;
#pragma unroll
        for (int j = 0; j < KS; ++j) {
            r.kx[j] = stream_load((const bf16x8*)(ka + koff + j * 512));
            r.ky[j] = stream_load((const bf16x8*)(kb + koff + j * 512));
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            r.va[dt] = stream_load((const bf16x4*)(va + voff + dt * 64));
            r.vb[dt] = stream_load((const bf16x4*)(vb + voff + dt * 64));
        }
    };
    // Leaves unit kC: this wave's state goes to the unit's LDS slot for the control wave to combine.
    auto leave_unit = [&]() INLINE_LAMBDA -> bool {
        if (!spin_until_at_least(a, &sm.failed, &sm.consumed, kC - 1)) return false;  // slot of unit kC-2 is free
        const int par = kC & 1;
        l = sum_lane_groups(l);
        if (n < g) {
            if (qd == 0) sm.ml[par][wave][n] = make_float2(m, l);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) *(f32x4*)&sm.o[par][wave][n][16 * dt + 4 * qd] = O[dt];
        }
        if (lane == 0) __hip_atomic_fetch_add(&sm.done[kC % RING], 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        m = -INFINITY;
        l = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) O[dt] = (f32x4)(0.f);
        ++kC;
        return true;
    };
    auto compute = [&](const KVRegs<D>& r, const int b) INLINE_LAMBDA {
        f32x4 sx = (f32x4)(0.f), sy = (f32x4)(0.f);
#pragma unroll
        for (int j = 0; j < KS; ++j) {
            sx = mfma16(r.kx[j], qf[j], sx);
            sy = mfma16(r.ky[j], qf[j], sy);
        }
        const int nv = uC.n_tok - 32 * b;
        if (nv < 32) mask_tail(sx, sy, qd, nv);
        const bf16x8 pf = softmax_block<DT>(sx, sy, c, m, l, O);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) O[dt] = mfma16(cat(r.va[dt], r.vb[dt]), pf, O[dt]);
    };

    // (uX, bX): unit number and block held by register set X, uX < 0 when it holds none
    int u0 = -1, b0 = 0, u1 = -1, b1 = 0;
    KVRegs<D> r0, r1;
    // One step: start the loads of the claimed block into `other` if that set is empty, claim the
    // block after it, then compute `cur` if it holds a block.
    // Returns 0 to go on, 1 when neither set holds a block, -1 on failure.
    auto step = [&](KVRegs<D>& cur, int& uc, const int bc, KVRegs<D>& other, int& uo, int& bo) INLINE_LAMBDA -> int {
        if (uo < 0) {
            if (nu < 0) claim();
            if (nu >= 0) {
                issue(other);
                uo = nu;
                bo = nb;
                nu = -1;
#ifndef NO_PRECLAIM
                claim();
#endif
            }
        }
        if (uc >= 0) {
            if (uc != kC) {  // the block belongs to the next unit (kL == kC + 1, its q is in qn)
                if (!leave_unit()) return -1;
                uC = uL;
#pragma unroll
                for (int j = 0; j < KS; ++j) qf[j] = qn[j];
            }
            compute(cur, bc);
            uc = -1;
            return 0;
        }
        return uo < 0 ? 1 : 0;
    };
    for (;;) {
        int st = step(r0, u0, b0, r1, u1, b1);
        if (st == 0) st = step(r1, u1, b1, r0, u0, b0);
        if (st < 0) return;
        if (st == 0) continue;
        // Neither set holds a block and none could be claimed: unit kC has none left for this
        // wave, and the wave could not run ahead (next unit not published yet, not private, or
        // itself without a block left).
        if (!leave_unit()) return;
        if (kL < kC) {
            if (!spin_until_at_least(a, &sm.failed, &sm.published, kC + 1)) return;
            read_ring(kC, uL);
            kL = kC;
            if (uL.kind != 1) return;
            load_q(uL, qn);
        }
        uC = uL;
#pragma unroll
        for (int j = 0; j < KS; ++j) qf[j] = qn[j];
    }
}

// The control wave of a workgroup.  In order of priority it (1) publishes the next unit when
// the streaming waves are about to run out of blocks (claiming it from the queue only then, so
// a workgroup never sits on unstarted work when the queue runs dry), (2) combines the states of
// a unit all streaming waves have left and stores its partial rows, (3) advances a merge by one
// round of entries.  A unit's arrival is announced when the next unit is combined (its stores
// have completed by then) and the atomic's result is looked at later still, so the wave never
// waits for an operation it has just issued, except for the claim.
template <int D>
DEV void control_wave(const StepArgs& a, const int hk, SpecSmem<D>& sm, const int w) {
    constexpr int PUBLISH_AHEAD_BLOCKS = 16;  // publish the next unit when so few blocks of the last one are unclaimed
    const int lane = threadIdx.x & 63;
    const int g = a.gqa;
    const int W = a.wgs_per_head;
    const int total = g * (D / 4);  // float4 pieces of one (sequence, kv head) result; each lane owns up to 4 of them
    int n_pub = 0, n_cons = 0, n_units = 0;  // ring entries published, units combined, units among the published entries
    bool end_published = false;
    int seq0_of[RING], base_of[RING], ntok_of[RING];  // of the units published and not yet combined
#pragma unroll
    for (int i = 0; i < RING; ++i) seq0_of[i] = base_of[i] = ntok_of[i] = 0;
    int seq_stored = -1;              // sequence whose partial rows were stored at the last combine
    int seq_announced = -1, old = 0;  // sequence whose arrival has been announced; lane 0: the counter before
    // merge in progress: sequence, next entry, end entry, and the running state of this lane's pieces
    int mg_seq = -1, mg_e = 0, mg_e1 = 0;
    float mg_M[4], mg_L[4];
    f32x4 mg_acc[4];
    auto merge_round = [&]() INLINE_LAMBDA {  // two entries of the merge in progress
        taper_merge_entry me[2];
        bool have[2];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            have[k] = mg_e + k < mg_e1;
            me[k] = a.merge[have[k] ? mg_e + k : mg_e];
        }
        float2 ml[4][2];
        f32x4 o[4][2];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = lane + 64 * u;
            const bool in = idx < total;
            const int j = in ? idx / (D / 4) : 0, d4 = in ? idx % (D / 4) : 0;
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int64_t rowi = (int64_t)me[k].first_row + (int64_t)hk * me[k].rows_per_head + j;
                ml[u][k] = coherent_load2((const float*)(a.ws_ml + rowi));
                o[u][k] = coherent_load4(a.ws_o + rowi * D + 4 * d4);
                if (!have[k] || !in) ml[u][k] = make_float2(-INFINITY, 0.f);
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float mn = fmaxf(mg_M[u], fmaxf(ml[u][0].x, ml[u][1].x));
            const float keep = mg_M[u] == -INFINITY ? 0.f : fast_exp2(mg_M[u] - mn);
            mg_L[u] *= keep;
            mg_acc[u] *= keep;
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const float wk = ml[u][k].x == -INFINITY ? 0.f : fast_exp2(ml[u][k].x - mn);
                mg_L[u] += wk * ml[u][k].y;
                mg_acc[u] += wk * o[u][k];
            }
            mg_M[u] = mn;
        }
        mg_e += 2;
        if (mg_e >= mg_e1) {  // normalise, round, write
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int idx = lane + 64 * u;
                if (idx < total) {
                    const int j = idx / (D / 4), d4 = idx % (D / 4);
                    const int h = hk * g + j;
                    const f32x4 r = mg_acc[u] * (1.0f / mg_L[u]);
                    *(bf16x4*)((__bf16*)a.out + ((int64_t)mg_seq * a.n_q_heads + h) * D + 4 * d4) = __builtin_convertvector(r, bf16x4);
                    if (a.lse && d4 == 0) a.lse[(int64_t)mg_seq * a.n_q_heads + h] = (mg_M[u] + __log2f(mg_L[u])) * 0.6931471805599453f;
                }
            }
            mg_seq = -1;
        }
    };
    auto settle = [&]() INLINE_LAMBDA {  // looks at the announced arrival's result; may start a merge
        const int s = seq_announced;
        const int e0 = a.merge_start[s], e1 = a.merge_start[s + 1];
        if (__builtin_amdgcn_readfirstlane(old) == e1 - e0 - 1) {
            if (lane == 0) a.counters[(int64_t)s * a.n_kv_heads + hk] = 0;
            mg_seq = s;
            mg_e = e0;
            mg_e1 = e1;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                mg_M[u] = -INFINITY;
                mg_L[u] = 0.f;
                mg_acc[u] = (f32x4)(0.f);
            }
        }
        seq_announced = -1;
    };
    for (int idle = 0;;) {
        // (1) publish
        bool gate = !end_published && n_pub - n_cons < RING - 1;
        if (gate && n_pub > 0) {
            int last_tok = 0;
#pragma unroll
            for (int i = 0; i < RING; ++i)
                if (i == (n_pub - 1) % RING) last_tok = ntok_of[i];
            gate = lds_load_acquire(&sm.blk[(n_pub - 1) % RING]) + PUBLISH_AHEAD_BLOCKS >= ((last_tok + 31) >> 5);
        }
        if (gate) {
            int id;
            if (n_pub == 0) id = w;
            else if (n_pub == 1) id = 2 * W - 1 - w;
            else {
                int got = 0;
                if (lane == 0) got = atomicAdd(a.queue + hk, 1);
                id = 2 * W + __builtin_amdgcn_readfirstlane(got);
            }
            const Unit un = fetch_unit(a, id);
            const int slot = n_pub % RING;
            if (lane == 0) {
                sm.ring[slot].row_off = un.row - a.bt;
                sm.ring[slot].seq0 = un.seq0;
                sm.ring[slot].n_tok = un.n_tok;
                sm.ring[slot].part_base = un.part_base;
                sm.ring[slot].kind = un.kind;
                sm.blk[slot] = 0;
                sm.done[slot] = 0;
            }
#pragma unroll
            for (int i = 0; i < RING; ++i)
                if (i == slot) {
                    seq0_of[i] = un.seq0;
                    base_of[i] = un.part_base;
                    ntok_of[i] = un.n_tok;
                }
            ++n_pub;
            if (un.kind == 1) ++n_units;
            else end_published = true;
            if (lane == 0) lds_store_release(&sm.published, n_pub);
            idle = 0;
            continue;
        }
        // (2) combine a unit all streaming waves have left; needs the announce slot free
        if (n_cons < n_units && seq_announced < 0 && lds_load_acquire(&sm.done[n_cons % RING]) == STREAM_WAVES) {
            const int slot = n_cons % RING, par = n_cons & 1;
            int seq0 = 0, part_base = 0;
#pragma unroll
            for (int i = 0; i < RING; ++i)
                if (i == slot) {
                    seq0 = seq0_of[i];
                    part_base = base_of[i];
                }
            if (seq_stored >= 0) {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's earlier stores are written through
                if (lane == 0) old = atomicAdd(a.counters + (int64_t)seq_stored * a.n_kv_heads + hk, 1);
                seq_announced = seq_stored;
            }
            for (int idx = lane; idx < total; idx += 64) {
                const int r = idx / (D / 4), d4 = idx % (D / 4);
                float mw[STREAM_WAVES], M = -INFINITY;
#pragma unroll
                for (int v = 0; v < STREAM_WAVES; ++v) {
                    mw[v] = sm.ml[par][v][r].x;
                    M = fmaxf(M, mw[v]);
                }
                float L = 0.f;
                f32x4 acc = (f32x4)(0.f);
#pragma unroll
                for (int v = 0; v < STREAM_WAVES; ++v) {
                    const float wg = mw[v] == -INFINITY ? 0.f : fast_exp2(mw[v] - M);  // a wave may have had no block
                    L += wg * sm.ml[par][v][r].y;
                    acc += wg * *(const f32x4*)&sm.o[par][v][r][4 * d4];
                }
                const int64_t row = (int64_t)part_base + hk * g + r;
                coherent_store4(a.ws_o + row * D + 4 * d4, acc);
                if (d4 == 0) coherent_store2((float*)(a.ws_ml + row), M, L);
            }
            seq_stored = seq0;
            ++n_cons;
            if (lane == 0) lds_store_release(&sm.consumed, n_cons);  // the slot has been read
            idle = 0;
            continue;
        }
        // (3) merges
        if (mg_seq >= 0) {
            merge_round();
            idle = 0;
            continue;
        }
        if (seq_announced >= 0) {
            settle();
            idle = 0;
            continue;
        }
        if (end_published && n_cons == n_units) {
            if (seq_stored < 0) break;
            // the last unit: announce it, then come round again to settle and merge
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if (lane == 0) old = atomicAdd(a.counters + (int64_t)seq_stored * a.n_kv_heads + hk, 1);
            seq_announced = seq_stored;
            seq_stored = -1;
            continue;
        }
        if (lds_load_acquire(&sm.failed)) return;
        if (++idle >= SPIN_LIMIT) {
            lds_store_release(&sm.failed, 1);
            a.queue[a.n_kv_heads + 1] = 1;
            return;
        }
        __builtin_amdgcn_s_sleep(1);
    }
}

template <int D>
__global__ __launch_bounds__(256, 2) void decode_private_kernel(StepArgs a) {
    __shared__ __attribute__((aligned(16))) SpecSmem<D> sm;
    const int hk = blockIdx.x % a.n_kv_heads;
    const int w = blockIdx.x / a.n_kv_heads;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
#ifdef TAPER_WG_TRACE
    long long* trace = (long long*)a.lse;
    a.lse = nullptr;
    if (threadIdx.x == 0) trace[3 * blockIdx.x] = wall_clock64();
#endif
    if (threadIdx.x == 0) {
        sm.published = 0;
        sm.consumed = 0;
        sm.failed = 0;
    }
    __syncthreads();
    if (wave == STREAM_WAVES)
        control_wave<D>(a, hk, sm, w);
    else
        stream_wave<D>(a, hk, sm, wave);
    __syncthreads();
#ifdef TAPER_WG_TRACE
    if (threadIdx.x == 0) {
        trace[3 * blockIdx.x + 1] = wall_clock64();
        trace[3 * blockIdx.x + 2] = 0;
    }
#endif
    // the last workgroup to leave puts the queue back to zero for the next launch
    if (threadIdx.x == 0 && atomicAdd(a.queue + a.n_kv_heads, 1) == (int)gridDim.x - 1) {
        for (int h = 0; h <= a.n_kv_heads; ++h) a.queue[h] = 0;
    }
}

// Physical slot of every logical position, from the device copy of the plan.
__global__ __launch_bounds__(256) void resolve_slots_kernel(StepArgs a, int64_t* slots, int64_t stride) {
    const int s = blockIdx.x;
    const int64_t t = (int64_t)blockIdx.y * 256 + threadIdx.x;
    if (t >= stride) return;
    int64_t v = -1;
    if (t < a.ctx_len[s]) {
        const int32_t* row = a.bt + (int64_t)s * a.bt_stride;
        const int pl = a.prefix_len[s];
        if (t < pl) {
            v = (int64_t)row[t >> 4] * 16 + (t & 15);
        } else {
            const int64_t jj = t - pl;
            v = (int64_t)row[a.n_prefix_pages[s] + (jj >> 4)] * 16 + (jj & 15);
        }
    }
    slots[(int64_t)s * stride + t] = v;
}

// ---------------------------------------------------------------------------
hipError_t launch_decode(const StepArgs& a, hipStream_t s) {
    if (a.n_items == 0) return hipSuccess;
    const dim3 grid(a.wgs_per_head * a.n_kv_heads), block(256);
    const int ntw = (a.max_row_tiles_shared + 3) / 4;
    if (a.head_dim == 128) {
        if (ntw == 0) hipLaunchKernelGGL((decode_private_kernel<128>), grid, block, 0, s, a);
        else if (ntw == 1) hipLaunchKernelGGL((decode_kernel<128, 1>), grid, block, 0, s, a);
        else if (ntw == 2) hipLaunchKernelGGL((decode_kernel<128, 2>), grid, block, 0, s, a);
        else if (ntw == 3) hipLaunchKernelGGL((decode_kernel<128, 3>), grid, block, 0, s, a);
        else return hipErrorInvalidValue;
    } else if (a.head_dim == 64) {
        if (ntw == 0) hipLaunchKernelGGL((decode_private_kernel<64>), grid, block, 0, s, a);
        else if (ntw == 1) hipLaunchKernelGGL((decode_kernel<64, 1>), grid, block, 0, s, a);
        else if (ntw == 2) hipLaunchKernelGGL((decode_kernel<64, 2>), grid, block, 0, s, a);
        else if (ntw == 3) hipLaunchKernelGGL((decode_kernel<64, 3>), grid, block, 0, s, a);
        else return hipErrorInvalidValue;
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// Workgroups the device keeps resident at once, per kernel variant (1, 2, 3 row tiles per wave).
hipError_t query_resident_wgs(int device, int head_dim, int out[3]) {
    hipDeviceProp_t prop;
    hipError_t e = hipGetDeviceProperties(&prop, device);
    if (e != hipSuccess) return e;
    for (int i = 0; i < 3; ++i) {
        int per_cu = 0;
        const void* f = head_dim == 128 ? (i == 0   ? (const void*)decode_kernel<128, 1>
                                           : i == 1 ? (const void*)decode_kernel<128, 2>
                                                    : (const void*)decode_kernel<128, 3>)
                                        : (i == 0   ? (const void*)decode_kernel<64, 1>
                                           : i == 1 ? (const void*)decode_kernel<64, 2>
                                                    : (const void*)decode_kernel<64, 3>);
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, f, 256, 0);
        if (e != hipSuccess) return e;
        out[i] = std::max(1, per_cu) * prop.multiProcessorCount;
    }
    return hipSuccess;
}

hipError_t launch_resolve_slots(const StepArgs& a, int64_t* slots, int64_t stride, hipStream_t s) {
    if (stride <= 0) return hipSuccess;
    const dim3 grid(a.n_seqs, (unsigned)((stride + 255) / 256)), block(256);
    hipLaunchKernelGGL(resolve_slots_kernel, grid, block, 0, s, a, slots, stride);
    return hipGetLastError();
}

}  // namespace taper
