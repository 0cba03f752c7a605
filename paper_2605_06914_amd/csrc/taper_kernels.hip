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
// chunks of a sequence (m, l in fp32; O / l in fp32 or, by default, in half precision with a
// per-row power-of-two scale) are combined through their (m, l) by the workgroup that delivers
// the sequence's last partial (merge_rows).
#include <type_traits>

#include "taper_internal.h"

namespace taper {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

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
    const int t = n_valid - 4 * qd;  // this lane's tokens i (first page) and 16 + i (second page) are valid below t
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (i >= t) sx[i] = -INFINITY;
        if (16 + i >= t) sy[i] = -INFINITY;
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

// The accumulator a block's last matrix instruction wrote must not be read by a vector instruction
// before the matrix pipeline has delivered it (eight passes; the hardware does not interlock, the
// compiler inserts the wait states).  On a path that leaves the block's code through two branches
// and starts with register copies of the accumulators, the compiler was seen to leave too few: the
// last 16 dims of long private items came out wrong, in one build and not in another.  So a block
// ends with the wait states written out, fenced so that the scheduler leaves them where they are.
DEV void settle() {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 11");
    __builtin_amdgcn_sched_barrier(0);
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
// The accumulator part of a partial row travels normalised (divided by the row's own sum, so that
// it is a weighted mean of V rows), in one of two formats (taper_partial_format):
//   PF_F32   fp32, two 8-byte accesses per four values;
//   PF_F16S  half precision after division by a power of two that brings the row's largest
//            magnitude into [0.5, 1): one 8-byte access per four values, 11 bits of mantissa
//            relative to the row's largest element beside the 8 the bf16 result keeps, and no
//            limit on the magnitude of V.  The power of two sits beside (m, l) in the row's
//            statistics record and is multiplied back in by the merge.
constexpr int PF_F16S = TAPER_PARTIAL_F16_SCALED, PF_F32 = TAPER_PARTIAL_F32;
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
template <int PF>
struct PartialRaw {
    unsigned long long w[PF == PF_F32 ? 2 : 1];
};
template <int PF>
DEV void partial_store4(void* rows, int64_t elem, f32x4 v) {
    if constexpr (PF == PF_F32) {
        float* p = (float*)rows + elem;
        coherent_store2(p, v[0], v[1]);
        coherent_store2(p + 2, v[2], v[3]);
    } else {
        const f16x4 h = __builtin_convertvector(v, f16x4);
        __hip_atomic_store((unsigned long long*)((uint16_t*)rows + elem), __builtin_bit_cast(unsigned long long, h),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}
// (the reader addresses a row by a 32-bit element offset from the workspace's base, which is the same for every
// lane and stays in scalar registers: one address register per row instead of two per load.  The plan
// keeps the partial rows of a step below 2^31 bytes.)
template <int PF>
DEV PartialRaw<PF> partial_load4_raw(const void* rows, int elem) {
    PartialRaw<PF> r;
    if constexpr (PF == PF_F32) {
        const unsigned long long* p = (const unsigned long long*)((const char*)rows + elem * 4);
        r.w[0] = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        r.w[1] = __hip_atomic_load(p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        r.w[0] = __hip_atomic_load((const unsigned long long*)((const char*)rows + elem * 2), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
    }
    return r;
}
template <int PF>
DEV f32x4 partial_unpack4(const PartialRaw<PF>& r) {
    if constexpr (PF == PF_F32) {
        f32x4 v;
        v[0] = __uint_as_float((unsigned)r.w[0]);
        v[1] = __uint_as_float((unsigned)(r.w[0] >> 32));
        v[2] = __uint_as_float((unsigned)r.w[1]);
        v[3] = __uint_as_float((unsigned)(r.w[1] >> 32));
        return v;
    } else {
        return __builtin_convertvector(__builtin_bit_cast(f16x4, r.w[0]), f32x4);
    }
}
// The power of two 2^e that brings a row whose largest magnitude is `maxabs` into [0.5, 1), as
// (2^e, 2^-e); e is kept inside [-126, 126] so that both are normal numbers (an all-zero row, or one
// that holds Inf, is multiplied by some power of two all the same: it stays what it is).
DEV float2 row_scale(float maxabs) {
    int e = (int)((__float_as_uint(maxabs) >> 23) & 0xff) - 126;
    e = e < -126 ? -126 : (e > 126 ? 126 : e);
    return make_float2(__uint_as_float((unsigned)(127 + e) << 23), __uint_as_float((unsigned)(127 - e) << 23));
}
DEV float maxabs4(f32x4 v) { return fmaxf(fmaxf(fabsf(v[0]), fabsf(v[1])), fmaxf(fabsf(v[2]), fabsf(v[3]))); }
// Statistics record of a partial row: (running max in log2 units, sum) and, for PF_F16S, (row scale, unused).
template <int PF>
DEV void stats_store(float4* rec, float m, float l, float scale) {
    coherent_store2((float*)rec, m, l);
    if constexpr (PF == PF_F16S) coherent_store2((float*)rec + 2, scale, 0.f);
}
// Every earlier vector memory operation of this wave has completed, in particular its
// write-through stores of partial rows.  (A workgroup-scope release fence does not wait for
// global stores on this target, and nothing weaker than a full wait orders the stores
// before the arrival counter's increment for a reader on another compute unit.)
DEV void stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// What the end of an item needs from the plan, fetched when the item starts so that no
// dependent load is left for the end, where each one costs a loaded memory latency:
// merge_start[seq0 + b] for the item's sequences and the first kMetaWindow merge entries from
// merge_start[seq0] on (the sequences' entry lists are adjacent).
constexpr int kMetaWindow = 128;
struct MergeMeta {
    int ms[65];
    taper_merge_entry me[kMetaWindow];
};
struct MetaRegs {
    int ms;
    taper_merge_entry me;
};
// A per-lane value the compiler must not reason about: whatever is derived from it is
// computed where it is used instead of being hoisted out of the item loop, where it would
// sit in registers (or, worse, in scratch) for the whole kernel.
DEV int opaque(int v) {
    asm volatile("" : "+v"(v));
    return v;
}
// V of the invalid tokens of a chunk's last 32-token block -> 0, so that whatever bits an
// unwritten slot holds (NaN, Inf) meet their zero weight as 0 * 0.  A lane's values are tokens
// 4*qd+i of the first page (va) and of the second (vb), two per dword.  The comparisons are made
// again for every dword pair (from `opaque`) rather than kept: this runs once per chunk, in
// code that has no register to spare.
DEV unsigned keep_pair(unsigned w, int t) {  // both halves if t >= 2, the low one if t == 1, none below
    const unsigned lo = __builtin_amdgcn_ubfe(w, 0, 16);  // (no 32-bit literal: those get hoisted into registers)
    return t > 1 ? w : (t > 0 ? lo : 0u);
}
DEV bf16x4 keep_tail(bf16x4 v, int t) {  // tokens i < t of the four
    u32x2 w = __builtin_bit_cast(u32x2, v);
    w[0] = keep_pair(w[0], t);
    w[1] = keep_pair(w[1], t - 2);
    return __builtin_bit_cast(bf16x4, w);
}
template <int DT>
DEV void zero_tail(bf16x4 (&va)[DT], bf16x4 (&vb)[DT], int qd, int n_valid) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
        const int t = opaque(n_valid - 4 * qd);
        va[dt] = keep_tail(va[dt], t);
        vb[dt] = keep_tail(vb[dt], t - 16);
    }
}

DEV MetaRegs meta_load(const StepArgs& a, const taper_work_item& item, const int tid_) {
    const int tid = opaque(tid_);
    MetaRegs r;
    r.ms = 0;
    r.me.first_row = 0;
    r.me.rows_per_head = 0;
    if (tid <= item.n_branch) r.ms = a.merge_start[item.seq0 + tid];
    if (tid < kMetaWindow && item.merge0 + tid < a.n_merge) r.me = a.merge[item.merge0 + tid];
    return r;
}
DEV void meta_store(MergeMeta& mm, const MetaRegs& r, const int n_branch, const int tid_) {
    const int tid = opaque(tid_);
    if (tid <= n_branch) mm.ms[tid] = r.ms;
    if (tid < kMetaWindow) mm.me[tid] = r.me;
}
DEV taper_merge_entry merge_entry(const StepArgs& a, const MergeMeta& mm, const int e) {
    const int t = e - mm.ms[0];
    if (t < kMetaWindow) return mm.me[t];
    return a.merge[e];
}

// Log-sum-exp merge of all partials of (sequence s, kv head hk) -- its request's
// prefix chunks and its own private chunks, entries [e0, e1) of the merge map -- then
// normalisation and rounding to bf16.  Entries are taken in plan order, so the result
// does not depend on which workgroup happens to run this.  The loads bypass the caches
// and cost a full memory latency per round, so a round keeps R entries in flight.
//
// A group of n_thr consecutive lanes (a workgroup, a wave or half a wave) merges one sequence;
// groups of one wave may work on different sequences side by side.  Lane idx of the group owns
// float4 columns c, c + LPR, ... (U of them) of one row, where LPR = D/4/U lanes cover a row;
// n_thr / LPR rows are merged per pass.
//
// ALL: every round issues R loads per column whatever is left of the list -- past the sequence's last
// entry that entry once more, with weight zero -- so that a round has no branches (what the compiler
// makes of R conditional loads needs many more registers; the callers that run half-waves side by
// side have none to spare).  Otherwise only the entries that exist are loaded: every load here is a
// full trip to memory through a saturated memory system, and the slowest one ends the round.
template <int D, int U, int R, int PF, bool ALL>
DEV void merge_rows(const StepArgs& a, const MergeMeta& mm, const int s, const int hk, const int e0, const int e1,
                    const int idx_, const int n_thr) {
    constexpr int LPR = D / 4 / U;
    const int g = a.gqa;
    const int idx = opaque(idx_);
    const int jr = idx / LPR, c0 = idx % LPR;
    for (int j0 = 0; j0 < g; j0 += n_thr / LPR) {
        const int j = j0 + jr;
        const bool okr = j < g;
        float M = -INFINITY, L = 0.f;
        f32x4 acc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u] = (f32x4)(0.f);
        for (int e = e0; e < e1; e += R) {
            float2 ml[R];
            float sc[R];
            PartialRaw<PF> o[R][U];  // unpacked when they are used
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const bool real = e + k < e1;
                ml[k] = make_float2(-INFINITY, 0.f);
                sc[k] = 1.f;
#pragma unroll
                for (int u = 0; u < U; ++u) o[k][u] = PartialRaw<PF>{};
                if (ALL || real) {
                    const taper_merge_entry me = merge_entry(a, mm, real ? e + k : e1 - 1);
                    const int row = me.first_row + hk * me.rows_per_head + (okr ? j : 0);
                    const float* rec = (const float*)((const char*)a.ws_ml + row * 16);
                    const float2 v = coherent_load2(rec);
                    if (real && okr) ml[k] = v;
                    if constexpr (PF == PF_F16S) sc[k] = coherent_load2(rec + 2).x;
#pragma unroll
                    for (int u = 0; u < U; ++u) o[k][u] = partial_load4_raw<PF>(a.ws_o, row * D + 4 * (c0 + LPR * u));
                }
            }
            float mn = M;
#pragma unroll
            for (int k = 0; k < R; ++k) mn = fmaxf(mn, ml[k].x);
            const float keep = fast_exp2(M - mn);  // first round: exp2(-inf) = 0
            L *= keep;
#pragma unroll
            for (int u = 0; u < U; ++u) acc[u] *= keep;
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const float w = fast_exp2(ml[k].x - mn) * ml[k].y;  // (the row was stored divided by its sum)
                L += w;
                const float ws = PF == PF_F16S ? w * sc[k] : w;
#pragma unroll
                for (int u = 0; u < U; ++u) acc[u] += ws * partial_unpack4<PF>(o[k][u]);
            }
            M = mn;
        }
        if (okr) {
            const int h = hk * g + j;
            const float inv = 1.0f / L;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const f32x4 r = acc[u] * inv;
                *(bf16x4*)((__bf16*)a.out + ((int64_t)s * a.n_q_heads + h) * D + 4 * (c0 + LPR * u)) = __builtin_convertvector(r, bf16x4);
            }
            if (a.lse && c0 == 0) a.lse[(int64_t)s * a.n_q_heads + h] = (M + __log2f(L)) * 0.6931471805599453f;
        }
    }
}

// A workgroup that has written a partial of (sequence s, kv head hk), one of n_entries,
// announces it.  Returns true to the one caller that arrives last: every other partial of
// that (s, hk) has then been written through (each writer waited for its stores before
// its increment) and the caller must merge.  The counter is left at zero for the next launch
// (by a device-scope store, like every other access to it).
DEV bool arrive_last(const StepArgs& a, const int s, const int hk, const int n_entries) {
    int* c = a.counters + (int64_t)s * a.n_kv_heads + hk;
    const bool last = atomicAdd(c, 1) == n_entries - 1;
    if (last) __hip_atomic_store(c, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return last;
}

// End of a shared-prefix item: every branch announces the item's partial; the branches whose set
// is now complete are merged side by side, a wave each for up to four of them, else half a wave.
// (One after the other they cost two to three memory round trips each, at the very end of a
// launch's longest workgroups.)  Called by all threads after the partial rows have been stored
// and waited for; `todo` and `n_todo` are workgroup-shared.
template <int D, int PF>
DEV void arrive_and_merge(const StepArgs& a, const MergeMeta& mm, int* todo, int* n_todo, const taper_work_item& item,
                          const int hk, const int tid) {
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (wave == 0) {  // (an item has at most 64 branches)
        const bool mine = lane < item.n_branch && arrive_last(a, item.seq0 + lane, hk, mm.ms[lane + 1] - mm.ms[lane]);
        const unsigned long long mask = __ballot(mine);
        if (mine) todo[__popcll(mask & ((1ull << lane) - 1))] = lane;
        if (lane == 0) *n_todo = __popcll(mask);
    }
    __syncthreads();
    const int n = *n_todo;
    // entries in flight per round: as many as leave the launch free of register spills (the streaming loops
    // of the callers are at the limit of the register file, and any scratch use costs microseconds per launch)
    constexpr int R64 = 6, R32 = PF == PF_F32 ? 2 : 4;
    if (n <= 4) {
        if (wave < n) {
            const int b = todo[wave];
            merge_rows<D, D / 32, R64, PF, false>(a, mm, item.seq0 + b, hk, mm.ms[b], mm.ms[b + 1], lane, 64);
        }
    } else {
        for (int i = tid >> 5; i < n; i += 8) {
            const int b = todo[i];
            merge_rows<D, D / 16, R32, PF, true>(a, mm, item.seq0 + b, hk, mm.ms[b], mm.ms[b + 1], tid & 31, 32);
        }
    }
}

// ---------------------------------------------------------------------------
// Private / serial kernel: one sequence's g query rows (one 16-row tile, rows
// >= g idle) against a chunk of that sequence's own pages.  No reuse across
// waves, so K/V go straight from HBM into MFMA operand registers; the four
// waves of a workgroup take alternate 32-token blocks and combine through LDS.
// ---------------------------------------------------------------------------
template <int D>
struct KVRegs {
    bf16x8 kx[D / 32], ky[D / 32];
    bf16x4 va[D / 16], vb[D / 16];
};

template <int D>
struct PrivateSmem {
    float o[4][16][D + 4];
    float2 ml[4][16];
    int last;
    int pick;  // pool item a workgroup has taken
    MergeMeta meta;
};

// One private item: a chunk of one sequence's own tokens, for kv head hk.
// SOLO: the item is run by the calling wave alone (short sequences that are a single item:
// four of them proceed side by side in a workgroup, with no barrier and no LDS); otherwise the
// four waves of the workgroup share the item's blocks.
// SB: the block-table row is read through the constant address space from a pointer the compiler knows to
// be the same in all lanes.  Its entries then come by scalar loads, which do not wait for the KV loads in
// flight (a vector load of a page id completes in order, behind everything issued before it: one block in
// flight per wave).  That deeper pipeline pays on steps without shared-prefix work; next to shared-prefix
// workgroups it takes bandwidth from them, and those launches keep the vector loads.
template <int D, bool SOLO, int PF, bool SB>
DEV void private_item(const StepArgs& a, const int it, const int hk, PrivateSmem<D>& sm) {
    constexpr int KS = D / 32, DT = D / 16, TILE = 16 * D;
    auto& sm_o = sm.o;
    auto& sm_ml = sm.ml;
    const int lane = opaque(threadIdx.x) & 63;  // (opaque: per-lane constants are recomputed per item, not kept for the whole kernel)
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, qd = lane >> 4;
    const int Hkv = a.n_kv_heads, g = a.gqa;
    const __bf16* __restrict__ kvb = (const __bf16*)a.kv;
    const int64_t page_elems = 2LL * Hkv * TILE;
    const float c = a.scale_log2e;
    const int koff = lane * 8, voff = qd * (4 * D) + n * 4;
    {
        const taper_work_item item = a.items[it];
        typedef const __attribute__((address_space(4))) int32_t* scalar_row;
        typedef const int32_t* __restrict__ vector_row;
        typename std::conditional<SB, scalar_row, vector_row>::type row;
        if constexpr (SB)
            row = (scalar_row)(a.bt + (int64_t)__builtin_amdgcn_readfirstlane(item.seq0) * a.bt_stride +
                               __builtin_amdgcn_readfirstlane(item.page0));
        else
            row = a.bt + (int64_t)item.seq0 * a.bt_stride + item.page0;
        const int n_tok = item.n_tokens;
        const int n_pages = (n_tok + 15) >> 4;
        const int n_blocks = (n_tok + 31) >> 5;
        const bool sole = SOLO || item.kind >= 2;  // the sequence's whole context: no partial, no arrival, no merge
        MetaRegs mr = {};
        if (!sole) mr = meta_load(a, item, threadIdx.x);

        bf16x8 qf[KS];
        {
            const __bf16* qrow = (const __bf16*)a.q + ((int64_t)item.seq0 * a.n_q_heads + hk * g + (n < g ? n : 0)) * D;
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                bf16x8 v = *(const bf16x8*)(qrow + 8 * (4 * j + qd));
                if (n >= g) v = (bf16x8)(0);
                qf[j] = v;
            }
        }
        float m = -INFINITY, l = 0.f;
        f32x4 O[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) O[dt] = (f32x4)(0.f);

        auto load_block = [&](int b, KVRegs<D>& r) {
            const int ia = 2 * b, ib = (2 * b + 1 < n_pages) ? 2 * b + 1 : ia;
            const int64_t pa = row[ia], pb = row[ib];
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
        };
        auto compute_block = [&](int b, KVRegs<D>& r) {
            f32x4 sx = (f32x4)(0.f), sy = (f32x4)(0.f);
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                sx = mfma16(r.kx[j], qf[j], sx);
                sy = mfma16(r.ky[j], qf[j], sy);
            }
            const int nv = n_tok - 32 * b;
            if (nv < 32) mask_tail(sx, sy, qd, nv);
            const bf16x8 pf = softmax_block<DT>(sx, sy, c, m, l, O);
            if (nv < 32) zero_tail(r.va, r.vb, qd, nv);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) O[dt] = mfma16(cat(r.va[dt], r.vb[dt]), pf, O[dt]);
            // (at head_dim 128 the same statement here costs this loop a few spilled registers, and the code
            // the compiler makes for it keeps the distance by itself; a build check scans every kernel for it)
            if constexpr (D == 64) settle();
        };

        KVRegs<D> r0, r1;
        constexpr int STEP = SOLO ? 1 : 4;  // blocks wave, wave + 4, ... of a shared item; all blocks of a solo one
        int b = SOLO ? 0 : wave;
        if (b < n_blocks) load_block(b, r0);
        while (b < n_blocks) {
            const int b1 = b + STEP;
            if (b1 < n_blocks) load_block(b1, r1);
            compute_block(b, r0);
            if (b1 >= n_blocks) break;
            const int b2 = b1 + STEP;
            if (b2 < n_blocks) load_block(b2, r0);
            compute_block(b1, r1);
            b = b2;
        }

        if constexpr (SOLO) {  // this wave holds the whole result: normalise and write it
            l = sum_lane_groups(l);
            if (n < g) {
                const int h = hk * g + n;
                const float inv = 1.0f / l;
                __bf16* orow = (__bf16*)a.out + ((int64_t)item.seq0 * a.n_q_heads + h) * D;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) *(bf16x4*)(orow + 16 * dt + 4 * qd) = __builtin_convertvector(O[dt] * inv, bf16x4);
                if (a.lse && qd == 0) a.lse[(int64_t)item.seq0 * a.n_q_heads + h] = (m + __log2f(l)) * 0.6931471805599453f;
            }
            return;
        }

        // combine the four waves' states
        l = sum_lane_groups(l);
        if (n < g) {
            if (qd == 0) sm_ml[wave][n] = make_float2(m, l);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) *(f32x4*)&sm_o[wave][n][16 * dt + 4 * qd] = O[dt];
        }
        __syncthreads();
        if (!sole) meta_store(sm.meta, mr, 1, threadIdx.x);  // (after the barrier: nobody still merges the previous item)
        for (int idx = threadIdx.x; idx < g * (D / 4); idx += 256) {
            const int r = idx / (D / 4), d4 = idx % (D / 4);
            float mw[4], M = -INFINITY;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                mw[w] = sm_ml[w][r].x;
                M = fmaxf(M, mw[w]);
            }
            float L = 0.f;
            f32x4 acc = (f32x4)(0.f);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float wg = fast_exp2(mw[w] - M);
                L += wg * sm_ml[w][r].y;
                acc += wg * *(const f32x4*)&sm_o[w][r][4 * d4];
            }
            if (sole) {
                const int h = hk * g + r;
                const f32x4 res = acc * (1.0f / L);
                *(bf16x4*)((__bf16*)a.out + ((int64_t)item.seq0 * a.n_q_heads + h) * D + 4 * d4) = __builtin_convertvector(res, bf16x4);
                if (a.lse && d4 == 0) a.lse[(int64_t)item.seq0 * a.n_q_heads + h] = (M + __log2f(L)) * 0.6931471805599453f;
                continue;
            }
            const int64_t slot = (int64_t)item.part_base + hk * g + r;
            f32x4 row = acc * (1.0f / L);
            float2 sc = make_float2(1.f, 1.f);
            if constexpr (PF == PF_F16S) {  // the row's D/4 lanes are neighbours inside one wave, all of them in this loop
                float mx = maxabs4(row);
#pragma unroll
                for (int o = 1; o < D / 4; o *= 2) mx = fmaxf(mx, __shfl_xor(mx, o));
                sc = row_scale(mx);
                row *= sc.y;
            }
            partial_store4<PF>(a.ws_o, slot * D + 4 * d4, row);
            if (d4 == 0) stats_store<PF>(a.ws_ml + slot, M, L, sc.x);
        }
        if (sole) {
            __syncthreads();  // the combine buffers are free for the next item
            return;
        }
        // publish the partial; whoever completes the sequence's set merges it
        stores_done();
        __syncthreads();
        if (threadIdx.x == 0) sm.last = arrive_last(a, item.seq0, hk, sm.meta.ms[1] - sm.meta.ms[0]);
        __syncthreads();
#ifdef TAPER_WG_TRACE
        const long long t_m0 = wall_clock64();
#endif
        if (sm.last) merge_rows<D, 1, 8, PF, false>(a, sm.meta, item.seq0, hk, sm.meta.ms[0], sm.meta.ms[1], threadIdx.x, 256);
#ifdef TAPER_WG_TRACE
        if (threadIdx.x == 0 && a.trace) a.trace[4 * blockIdx.x + 3] += wall_clock64() - t_m0;
#endif
    }
}

// The private items of a workgroup: those of its share [it0, it1) in order, then whatever it
// can take from its kv head's pool.  Every workgroup makes exactly one claim past the end of
// the pool; the one that makes the last of those puts the counter back to zero for the next
// launch.
template <int D, int PF, bool SB>
DEV void private_items(const StepArgs& a, int it0, const int it1, const int hk, PrivateSmem<D>& sm) {
    const int wgs_per_head = a.n_parts_shared + a.n_parts_private;  // = gridDim.x / n_kv_heads
#ifdef TAPER_WG_TRACE
    bool turned = false;
#endif
    for (;;) {
        int it = it0;
        if (it0 < it1) {
            ++it0;
        } else {
            if (a.n_pool_items == 0) return;
#ifdef TAPER_WG_TRACE
            if (threadIdx.x == 0 && a.trace && !turned) a.trace[4 * blockIdx.x + 1] = wall_clock64();  // own share done
            turned = true;
#endif
            if (threadIdx.x == 0) sm.pick = atomicAdd(a.pool_ctr + hk, 1);
            __syncthreads();
            const int i = sm.pick;
            __syncthreads();
            if (i >= a.n_pool_items) {
                if (threadIdx.x == 0 && i == a.n_pool_items + wgs_per_head - 1)
                    __hip_atomic_store(a.pool_ctr + hk, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                return;
            }
            it = a.pool_first + i;
        }
        if (a.items[it].kind == 3) {  // a run of solo items of this share: dealt to the waves, no barrier inside
            int end = it + 1;
            while (end < it1 && a.items[end].kind == 3) ++end;
            const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
            for (int k = it + wave; k < end; k += 4) private_item<D, true, PF, SB>(a, k, hk, sm);
            it0 = end;
            __syncthreads();
            continue;
        }
        private_item<D, false, PF, SB>(a, it, hk, sm);
    }
}

// ---------------------------------------------------------------------------
// Shared-prefix kernel: a chunk of one request's prefix pages is staged in LDS
// once (64 tokens per iteration, double buffered) and multiplied against the
// query rows of all n_branch admitted branches x g heads.  16-row tiles are
// dealt round-robin to the four waves, up to NTW tiles per wave.
// ---------------------------------------------------------------------------
template <int D>
struct SharedSmem {
    static constexpr int TILE = 16 * D;
    static constexpr int QE = 4 * D;        // elements of one 4-token quarter of a V tile
    static constexpr int VQ = QE + 64;      // padded quarter: odd multiple of 128 B -> quarters alternate bank halves
    static constexpr int PAGE_LDS = TILE + 4 * VQ;
    static constexpr int BUF = 4 * PAGE_LDS;  // 4 pages = 64 tokens
    __bf16 kv[2 * BUF];
    int todo[64];  // branches of the current item whose partials are complete
    int n_todo;
    MergeMeta meta;
};

// The partial rows of a shared-prefix item: tile k of this wave holds row 16 * (wave + 4k) + n of the
// item's R rows in lane column n, 4 values per 16-dim group and lane group.
template <int D, int NTW, int PF>
DEV void store_shared_partials(const StepArgs& a, const taper_work_item& item, const int hk, const int R, const int n_act,
                               const int wave, const int n, const int qd, const float (&m)[NTW], const float (&l)[NTW],
                               const f32x4 (&O)[NTW][D / 16]) {
    constexpr int DT = D / 16;
#pragma unroll
    for (int k = 0; k < NTW; ++k) {
        if (k < n_act) {
            const float lt = sum_lane_groups(l[k]);
            const float inv = 1.0f / lt;
            float2 sc = make_float2(1.f, 1.f);
            if constexpr (PF == PF_F16S) {  // (all 64 lanes are here: k < n_act is wave-uniform)
                float mx = 0.f;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) mx = fmaxf(mx, maxabs4(O[k][dt]));
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                sc = row_scale(mx * inv);
            }
            const int r = 16 * (wave + 4 * k) + n;
            if (r < R) {
                const int64_t slot = (int64_t)item.part_base + (int64_t)hk * R + r;
                if (qd == 0) stats_store<PF>(a.ws_ml + slot, m[k], lt, sc.x);
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    f32x4 v = O[k][dt] * inv;
                    if constexpr (PF == PF_F16S) v *= sc.y;
                    partial_store4<PF>(a.ws_o, slot * D + 16 * dt + 4 * qd, v);
                }
            }
        }
    }
}

template <int D, int NTW, int PF>
DEV void shared_path(const StepArgs& a, const int part, const int hk, SharedSmem<D>& sm) {
    constexpr int KS = D / 32, DT = D / 16, TILE = 16 * D;
    constexpr int QE = SharedSmem<D>::QE, VQ = SharedSmem<D>::VQ, PAGE_LDS = SharedSmem<D>::PAGE_LDS,
                  BUF = SharedSmem<D>::BUF;
    __bf16* lds = sm.kv;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int Hkv = a.n_kv_heads, g = a.gqa;
    const __bf16* __restrict__ kvb = (const __bf16*)a.kv;
    const int64_t page_elems = 2LL * Hkv * TILE;
    const float c = a.scale_log2e;

    const int it0 = a.part_start[part], it1 = a.part_start[part + 1];
    for (int it = it0; it < it1; ++it) {
        // per-lane constants are derived inside the loop from an opaque thread id, so that they are
        // not kept alive across the item's end (the merge wants the registers)
        const int tid = opaque(threadIdx.x);
        const int lane = tid & 63;
        const int n = lane & 15, qd = lane >> 4;
        const int se = tid * 8;                       // staging: this thread's element offset inside a tile
        const bool stager = se < TILE;
        const int sv = (se / QE) * VQ + se % QE;      // ... and inside the padded V tile in LDS
        const int koff = lane * 8;
        const int voff = TILE + qd * VQ + n * 4;
        const taper_work_item item = a.items[it];
        const int32_t* __restrict__ row = a.bt + (int64_t)item.seq0 * a.bt_stride + item.page0;
        const int n_tok = item.n_tokens;
        const int n_pages = (n_tok + 15) >> 4;
        const int n_blocks = (n_tok + 63) >> 6;
        const int R = item.n_branch * g;           // query rows
        const int tiles = (R + 15) >> 4;
        int n_act = (tiles - wave + 3) >> 2;       // tiles wave, wave+4, ...
        n_act = n_act < 0 ? 0 : (n_act > NTW ? NTW : n_act);
        meta_store(sm.meta, meta_load(a, item, tid), item.n_branch, tid);

        bf16x8 qf[NTW][KS];
        float m[NTW], l[NTW];
        f32x4 O[NTW][DT];
#pragma unroll
        for (int k = 0; k < NTW; ++k) {
            const int r = 16 * (wave + 4 * k) + n;
            const bool ok = k < n_act && r < R;
            const int rr = ok ? r : 0;
            const __bf16* qrow = (const __bf16*)a.q + ((int64_t)(item.seq0 + rr / g) * a.n_q_heads + hk * g + rr % g) * D;
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                bf16x8 v = *(const bf16x8*)(qrow + 8 * (4 * j + qd));
                if (!ok) v = (bf16x8)(0);
                qf[k][j] = v;
            }
            m[k] = -INFINITY;
            l[k] = 0.f;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) O[k][dt] = (f32x4)(0.f);
        }

        // Register sets for staging: while block b is computed from LDS, the next blocks are in flight.
        bf16x8 stgA[8], stgB[8];
        auto stage_load = [&](int b, bf16x8 (&stg)[8]) {
            if (stager && b < n_blocks) {
#pragma unroll
                for (int pg = 0; pg < 4; ++pg) {
                    const int ip = 4 * b + pg < n_pages ? 4 * b + pg : n_pages - 1;
                    const int64_t pid = row[ip];
                    const __bf16* kp = kvb + pid * page_elems + (int64_t)hk * TILE + se;
                    stg[2 * pg] = stream_load((const bf16x8*)kp);
                    stg[2 * pg + 1] = stream_load((const bf16x8*)(kp + (int64_t)Hkv * TILE));
                }
            }
        };
        auto stage_store = [&](int b, const bf16x8 (&stg)[8]) {
            if (stager && b < n_blocks) {
                __bf16* base = lds + (b & 1) * BUF;
#pragma unroll
                for (int pg = 0; pg < 4; ++pg) {
                    *(bf16x8*)(base + pg * PAGE_LDS + se) = stg[2 * pg];
                    *(bf16x8*)(base + pg * PAGE_LDS + TILE + sv) = stg[2 * pg + 1];
                }
            }
        };
        auto compute = [&](int b, int buf) {
            if (n_act == 0) return;
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const int nv = n_tok - (64 * b + 32 * hf);
                if (nv <= 0) break;
                const __bf16* pa = lds + buf * BUF + (2 * hf) * PAGE_LDS;
                const __bf16* pb = pa + PAGE_LDS;
                bf16x8 pf[NTW];
                if constexpr (NTW == 1) {
                    // one tile per wave: every K fragment is used once, so the two pages' fragments take turns
                    // in one set of registers (this variant has none to spare beside its three staging sets)
                    f32x4 sx = (f32x4)(0.f), sy = (f32x4)(0.f);
                    bf16x8 kf[KS];
#pragma unroll
                    for (int j = 0; j < KS; ++j) kf[j] = *(const bf16x8*)(pa + koff + j * 512);
#pragma unroll
                    for (int j = 0; j < KS; ++j) sx = mfma16(kf[j], qf[0][j], sx);
#pragma unroll
                    for (int j = 0; j < KS; ++j) kf[j] = *(const bf16x8*)(pb + koff + j * 512);
#pragma unroll
                    for (int j = 0; j < KS; ++j) sy = mfma16(kf[j], qf[0][j], sy);
                    if (nv < 32) mask_tail(sx, sy, qd, nv);
                    pf[0] = softmax_block<DT>(sx, sy, c, m[0], l[0], O[0]);
                } else {
                    bf16x8 kx[KS], ky[KS];
#pragma unroll
                    for (int j = 0; j < KS; ++j) {
                        kx[j] = *(const bf16x8*)(pa + koff + j * 512);
                        ky[j] = *(const bf16x8*)(pb + koff + j * 512);
                    }
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
                }
                // (four V fragment pairs at a time, then one branch for the ragged tail: a branch per
                // fragment would keep the compiler from issuing the LDS reads ahead of the matrix
                // instructions; all eight pairs at once do not fit the registers of two tiles per wave)
#pragma unroll
                for (int h = 0; h < DT / 4; ++h) {
                    bf16x4 va[4], vb[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        va[i] = *(const bf16x4*)(pa + voff + (4 * h + i) * 64);
                        vb[i] = *(const bf16x4*)(pb + voff + (4 * h + i) * 64);
                    }
                    if (nv < 32) zero_tail(va, vb, qd, nv);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const bf16x8 vf = cat(va[i], vb[i]);
#pragma unroll
                        for (int k = 0; k < NTW; ++k)
                            if (k < n_act) O[k][4 * h + i] = mfma16(vf, pf[k], O[k][4 * h + i]);
                    }
                }
                settle();
            }
        };

        if constexpr (NTW == 1) {
            // registers to spare: a third set, so that three blocks are in flight while one is computed
            // (a workgroup's share of a saturated memory system grows with what it keeps in flight)
            bf16x8 stgC[8];
            stage_load(0, stgA);
            stage_load(1, stgB);
            stage_load(2, stgC);
            stage_store(0, stgA);
            __syncthreads();
            for (int b = 0; b < n_blocks; b += 3) {
                stage_load(b + 3, stgA);
                compute(b, b & 1);
                stage_store(b + 1, stgB);
                __syncthreads();
                if (b + 1 >= n_blocks) break;
                stage_load(b + 4, stgB);
                compute(b + 1, (b + 1) & 1);
                stage_store(b + 2, stgC);
                __syncthreads();
                if (b + 2 >= n_blocks) break;
                stage_load(b + 5, stgC);
                compute(b + 2, b & 1);
                stage_store(b + 3, stgA);
                __syncthreads();
            }
        } else {
            stage_load(0, stgA);
            stage_load(1, stgB);
            stage_store(0, stgA);
            __syncthreads();
            for (int b = 0; b < n_blocks; b += 2) {
                stage_load(b + 2, stgA);
                compute(b, b & 1);
                stage_store(b + 1, stgB);
                __syncthreads();
                if (b + 1 >= n_blocks) break;
                stage_load(b + 3, stgB);
                compute(b + 1, (b + 1) & 1);
                stage_store(b + 2, stgA);
                __syncthreads();
            }
        }

        // (lane coordinates are derived afresh: shared with the ones above, they would stay live through the streaming loop)
        const int tid_e = opaque(threadIdx.x);
        store_shared_partials<D, NTW, PF>(a, item, hk, R, n_act, wave, tid_e & 15, (tid_e & 63) >> 4, m, l, O);
        // publish the partials; merge every branch whose set is now complete
        stores_done();
        __syncthreads();
#ifdef TAPER_WG_TRACE
        const long long t_m0 = wall_clock64();
#endif
        arrive_and_merge<D, PF>(a, sm.meta, sm.todo, &sm.n_todo, item, hk, tid_e);
#ifdef TAPER_WG_TRACE
        __syncthreads();
        if (tid == 0 && a.trace) a.trace[4 * blockIdx.x + 3] += wall_clock64() - t_m0;
#endif
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// Shared-prefix kernel for requests wider than 8 row tiles (9 to 12: up to 24 branches at
// 8 query heads per KV head), head_dim 128.  Three tiles per wave leave no registers for
// staging sets, so KV goes from global memory straight into LDS: every wave-level 16-byte
// load lands as 1 KiB at a wave-uniform LDS address, lane after lane, which is exactly one
// quarter of a K tile or one (padded) quarter of a V tile.  Four 32-token buffers: one is
// computed from while three are in flight.
//
// The compiler does not see which buffer an LDS read touches and would wait for every
// outstanding load before each one, so the fragment reads are written out (with their own
// wait), and the barrier is the bare instruction behind an explicit wait: "all but the
// loads of the blocks after this one have landed, and my LDS reads are done".
// ---------------------------------------------------------------------------
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;
DEV unsigned lds_address(const void* p) { return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const char*)p; }
// Two block-table entries through the scalar cache.  (The compiler reads the table with vector
// loads once direct-to-LDS loads are in the loop, and a vector load's completion waits for
// every load issued before it: the pipeline would drain at each one.)  The wait is part of
// the statement: the compiler may copy the results right after it.
DEV void page_ids_fetch(const int32_t* px, const int32_t* py, int& x, int& y) {
    asm volatile("s_load_dword %0, %2, 0x0\n\ts_load_dword %1, %3, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=&s"(x), "=&s"(y) : "s"(px), "s"(py));
}
template <int N>
DEV void wait_loads_but() { asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(N)); }

// K fragments of a 32-token block: four 16-byte reads per page, 1 KiB apart; PB = bytes from one page to the next
template <int PB>
DEV void lds_read_k(unsigned addr, bf16x8 (&kx)[4], bf16x8 (&ky)[4]) {
    asm volatile(
        "ds_read_b128 %0, %8\n\t"
        "ds_read_b128 %1, %8 offset:1024\n\t"
        "ds_read_b128 %2, %8 offset:2048\n\t"
        "ds_read_b128 %3, %8 offset:3072\n\t"
        "ds_read_b128 %4, %8 offset:%9\n\t"
        "ds_read_b128 %5, %8 offset:%10\n\t"
        "ds_read_b128 %6, %8 offset:%11\n\t"
        "ds_read_b128 %7, %8 offset:%12\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(kx[0]), "=&v"(kx[1]), "=&v"(kx[2]), "=&v"(kx[3]), "=&v"(ky[0]), "=&v"(ky[1]), "=&v"(ky[2]), "=&v"(ky[3])
        : "v"(addr), "n"(PB), "n"(PB + 1024), "n"(PB + 2048), "n"(PB + 3072));
}
// V fragments of four consecutive 16-dim groups (128 bytes apart), both pages
template <int PB>
DEV void lds_read_v(unsigned addr, bf16x4 (&va)[4], bf16x4 (&vb)[4]) {
    asm volatile(
        "ds_read_b64 %0, %8\n\t"
        "ds_read_b64 %1, %8 offset:128\n\t"
        "ds_read_b64 %2, %8 offset:256\n\t"
        "ds_read_b64 %3, %8 offset:384\n\t"
        "ds_read_b64 %4, %8 offset:%9\n\t"
        "ds_read_b64 %5, %8 offset:%10\n\t"
        "ds_read_b64 %6, %8 offset:%11\n\t"
        "ds_read_b64 %7, %8 offset:%12\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(va[0]), "=&v"(va[1]), "=&v"(va[2]), "=&v"(va[3]), "=&v"(vb[0]), "=&v"(vb[1]), "=&v"(vb[2]), "=&v"(vb[3])
        : "v"(addr), "n"(PB), "n"(PB + 128), "n"(PB + 256), "n"(PB + 384));
}

template <int D, int PF>
DEV void shared_path_wide(const StepArgs& a, const int part, const int hk, SharedSmem<D>& sm) {
    static_assert(D == 128, "a wave's 64 x 16 bytes must be one quarter of a tile");
    constexpr int NTW = 3, KS = D / 32, DT = D / 16, TILE = 16 * D;
    constexpr int QE = SharedSmem<D>::QE, VQ = SharedSmem<D>::VQ, PAGE_LDS = SharedSmem<D>::PAGE_LDS;
    constexpr int BLK = 2 * PAGE_LDS;  // one 32-token buffer; sm.kv holds four
    constexpr int PB = 2 * PAGE_LDS;   // bytes per page in LDS
    __bf16* lds = sm.kv;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int Hkv = a.n_kv_heads, g = a.gqa;
    const __bf16* __restrict__ kvb = (const __bf16*)a.kv;
    const int64_t page_elems = 2LL * Hkv * TILE;
    const float c = a.scale_log2e;

    const int it0 = a.part_start[part], it1 = a.part_start[part + 1];
    for (int it = it0; it < it1; ++it) {
        const int tid = opaque(threadIdx.x);
        const int lane = tid & 63;
        const int n = lane & 15, qd = lane >> 4;
        const int se = tid * 8;  // this thread's 8 elements of every tile it stages
        const taper_work_item item = a.items[it];
        const int32_t* __restrict__ row = a.bt + (int64_t)item.seq0 * a.bt_stride + item.page0;
        const int n_tok = item.n_tokens;
        const int n_pages = (n_tok + 15) >> 4;
        const int n_blocks = (n_tok + 31) >> 5;
        const int R = item.n_branch * g;
        const int tiles = (R + 15) >> 4;
        int n_act = (tiles - wave + 3) >> 2;
        n_act = n_act < 0 ? 0 : (n_act > NTW ? NTW : n_act);
        meta_store(sm.meta, meta_load(a, item, tid), item.n_branch, tid);

        bf16x8 qf[NTW][KS];
        float m[NTW], l[NTW];
        f32x4 O[NTW][DT];
#pragma unroll
        for (int k = 0; k < NTW; ++k) {
            const int r = 16 * (wave + 4 * k) + n;
            const bool ok = k < n_act && r < R;
            const int rr = ok ? r : 0;
            const __bf16* qrow = (const __bf16*)a.q + ((int64_t)(item.seq0 + rr / g) * a.n_q_heads + hk * g + rr % g) * D;
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                bf16x8 v = *(const bf16x8*)(qrow + 8 * (4 * j + qd));
                if (!ok) v = (bf16x8)(0);
                qf[k][j] = v;
            }
            m[k] = -INFINITY;
            l[k] = 0.f;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) O[k][dt] = (f32x4)(0.f);
        }

        // 4 loads of 16 bytes per thread and block: K and V quarter `wave` of both pages
        int pid0, pid1;  // the pool pages of the block staged next (wave-uniform)
        auto fetch_ids = [&](int b) {  // past the last page (an odd count's second page, a block that does not exist): the last page
            const int i0 = 2 * b < n_pages ? 2 * b : n_pages - 1, i1 = 2 * b + 1 < n_pages ? 2 * b + 1 : n_pages - 1;
            page_ids_fetch(row + i0, row + i1, pid0, pid1);
        };
        auto stage = [&](int b) {
            __bf16* buf = lds + (b & 3) * BLK;
#pragma unroll
            for (int pg = 0; pg < 2; ++pg) {
                const int64_t pid = pg ? pid1 : pid0;
                const __bf16* kp = kvb + pid * page_elems + (int64_t)hk * TILE + se;
                __builtin_amdgcn_global_load_lds((global_void_ptr)kp, (lds_void_ptr)(buf + pg * PAGE_LDS + wave * QE), 16, 0, 2);
                __builtin_amdgcn_global_load_lds((global_void_ptr)(kp + (int64_t)Hkv * TILE),
                                                 (lds_void_ptr)(buf + pg * PAGE_LDS + TILE + wave * VQ), 16, 0, 2);
            }
        };
        auto compute = [&](int b) {
            const int nv = n_tok - 32 * b;
            const unsigned base = lds_address(lds + (b & 3) * BLK);
            bf16x8 kx[KS], ky[KS];
            lds_read_k<PB>(base + lane * 16, kx, ky);
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
            for (int h = 0; h < DT / 4; ++h) {
                bf16x4 va[4], vb[4];
                lds_read_v<PB>(base + 2 * (TILE + qd * VQ + n * 4) + h * 512, va, vb);
                if (nv < 32) zero_tail(va, vb, qd, nv);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const bf16x8 vf = cat(va[i], vb[i]);
#pragma unroll
                    for (int k = 0; k < NTW; ++k)
                        if (k < n_act) O[k][4 * h + i] = mfma16(vf, pf[k], O[k][4 * h + i]);
                }
            }
            settle();
        };

        // (the previous item's LDS reads of these buffers ended before its closing barriers)
        for (int b = 0; b < 3; ++b) {
            fetch_ids(b);
            if (b < n_blocks) stage(b);
        }
        fetch_ids(3);
        for (int b = 0; b < n_blocks; ++b) {
            const int after = n_blocks - 1 - b;  // blocks staged behind this one: 12, 8 or 4 loads may stay in flight
            if (after >= 2) wait_loads_but<8>();
            else if (after == 1) wait_loads_but<4>();
            else wait_loads_but<0>();
            __builtin_amdgcn_s_barrier();  // block b is in LDS for every wave; everyone is done with block b - 1
            if (b + 3 < n_blocks) stage(b + 3);  // into the buffer block b - 1 was computed from
            if (n_act > 0) compute(b);
            fetch_ids(b + 4);  // for the next iteration's stage: its latency overlaps the wait for block b + 1
        }

        const int tid_e = opaque(threadIdx.x);
        store_shared_partials<D, NTW, PF>(a, item, hk, R, n_act, wave, tid_e & 15, (tid_e & 63) >> 4, m, l, O);
        stores_done();
        __syncthreads();
        arrive_and_merge<D, PF>(a, sm.meta, sm.todo, &sm.n_todo, item, hk, tid_e);
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// One launch per layer: workgroup (share, kv head).  Shares below n_parts_shared
// stream shared prefixes, the others private tokens; both kinds run side by side.
// ---------------------------------------------------------------------------
// ALLP: a launch without shared-prefix work (no shared path in the kernel, block-table rows by scalar loads).
template <int D, int NTW, int PF, bool ALLP>
__global__ __launch_bounds__(256, (NTW <= 2 || D == 128 ? 2 : 1)) void decode_kernel(StepArgs a) {
    union Smem {
        SharedSmem<D> sh;
        PrivateSmem<D> pr;
    };
    __shared__ __attribute__((aligned(16))) char smem_raw[sizeof(Smem)];
    const int part = blockIdx.x / a.n_kv_heads;
    const int hk = blockIdx.x % a.n_kv_heads;
#ifdef TAPER_WG_TRACE  // trace builds only (wg_trace.py): per-workgroup clocks -- start, own share done, left, time in merges
    long long* trace = a.trace;
    if (threadIdx.x == 0 && trace) trace[4 * blockIdx.x] = wall_clock64();
#endif
    int it0 = 0, it1 = 0;  // private items of this workgroup's share
    if constexpr (ALLP) {
        it0 = a.part_start[part];
        it1 = a.part_start[part + 1];
    } else if (part < a.n_parts_shared) {
        if constexpr (NTW == 3 && D == 128)
            shared_path_wide<D, PF>(a, part, hk, *reinterpret_cast<SharedSmem<D>*>(smem_raw));
        else
            shared_path<D, NTW, PF>(a, part, hk, *reinterpret_cast<SharedSmem<D>*>(smem_raw));
        __syncthreads();
    } else {
        it0 = a.part_start[part];
        it1 = a.part_start[part + 1];
    }
#ifdef TAPER_WG_TRACE
    if (threadIdx.x == 0 && trace) trace[4 * blockIdx.x + 1] = wall_clock64();  // shared share done (a private share: overwritten when it is done)
#endif
    private_items<D, PF, ALLP>(a, it0, it1, hk, *reinterpret_cast<PrivateSmem<D>*>(smem_raw));
#ifdef TAPER_WG_TRACE
    if (threadIdx.x == 0 && trace) trace[4 * blockIdx.x + 2] = wall_clock64();
#endif
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
            int64_t jj = t - pl;
            int k = a.seg_start[s];
            while (jj >= a.seg_len[k]) jj -= a.seg_len[k++];  // t < ctx_len: k stays inside the sequence's segments
            v = (int64_t)row[a.seg_page0[k] + (jj >> 4)] * 16 + (jj & 15);
        }
    }
    slots[(int64_t)s * stride + t] = v;
}

// KV append: the new key and value rows of every sequence (bf16 [S][Hkv][D]) go to
// slot[s] = page * 16 + token of the pool, in the tile layouts the attention kernels read:
// K element d at (d/8)*128 + tok*8 + d%8 (16-byte groups of 8 dims), V element d at
// (tok/4)*4D + d*4 + tok%4.  One workgroup per sequence, thread = (kv head, group of 8 dims).
__global__ __launch_bounds__(256) void kv_append_kernel(const __bf16* __restrict__ k_new, const __bf16* __restrict__ v_new,
                                                        const int64_t* __restrict__ slot, __bf16* __restrict__ kv,
                                                        const int n_kv_heads, const int D) {
    const int s = blockIdx.x;
    const int64_t sl = slot[s];
    const int64_t page = sl >> 4;
    const int tok = (int)(sl & 15);
    const int groups = D / 8;
    const int64_t tile = 16LL * D;
    for (int i = threadIdx.x; i < n_kv_heads * groups; i += blockDim.x) {
        const int hk = i / groups, d8 = i % groups;
        const int64_t src = ((int64_t)s * n_kv_heads + hk) * D + 8 * d8;
        const bf16x8 kx = *(const bf16x8*)(k_new + src);
        const bf16x8 vx = *(const bf16x8*)(v_new + src);
        __bf16* kt = kv + ((page * 2 + 0) * n_kv_heads + hk) * tile;
        __bf16* vt = kv + ((page * 2 + 1) * n_kv_heads + hk) * tile;
        *(bf16x8*)(kt + d8 * 128 + tok * 8) = kx;
#pragma unroll
        for (int j = 0; j < 8; ++j) vt[(tok >> 2) * (4 * D) + (8 * d8 + j) * 4 + (tok & 3)] = vx[j];
    }
}

// ---------------------------------------------------------------------------
hipError_t launch_kv_append(const void* k_new, const void* v_new, const int64_t* slot, void* kv, int n_seqs, int n_kv_heads,
                            int head_dim, hipStream_t s) {
    if (n_seqs == 0) return hipSuccess;
    hipLaunchKernelGGL(kv_append_kernel, dim3(n_seqs), dim3(256), 0, s, (const __bf16*)k_new, (const __bf16*)v_new, slot,
                       (__bf16*)kv, n_kv_heads, head_dim);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Measurement aid, not a step of the path: a plain streaming read.  Every workgroup reads a
// contiguous slice in 4 KiB pieces, 16 bytes per lane, nontemporal, two pieces per wave in
// flight; nothing is computed but an XOR that keeps the loads alive.  What this reaches on the
// same bytes and launch shape is the rate the machine leaves for any read-bound kernel.
// ---------------------------------------------------------------------------
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ base, int64_t pieces_per_wg, unsigned* sink) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const u32x4* mine = base + (int64_t)blockIdx.x * pieces_per_wg * 256;  // 256 x 16 B = one 4 KiB piece
    u32x4 acc = {0, 0, 0, 0};
    for (int64_t i = 2 * wave; i < pieces_per_wg; i += 8) {
        u32x4 v[2][4];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int64_t piece = i + u < pieces_per_wg ? i + u : i;
#pragma unroll
            for (int k = 0; k < 4; ++k) v[u][k] = __builtin_nontemporal_load(mine + piece * 256 + 64 * k + lane);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int k = 0; k < 4; ++k) acc ^= v[u][k];
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u && sink) sink[0] = 1;  // (practically never: the loads must not be dropped)
}

hipError_t launch_stream_read(const void* base, int64_t pieces_per_wg, int n_workgroups, unsigned* sink, hipStream_t s) {
    hipLaunchKernelGGL(stream_read_kernel, dim3(n_workgroups), dim3(256), 0, s, (const u32x4*)base, pieces_per_wg, sink);
    return hipGetLastError();
}

template <int D, int PF>
static hipError_t launch_decode_as(const StepArgs& a, const dim3 grid, const int ntw, hipStream_t s) {
    const dim3 block(256);
    if (a.n_parts_shared == 0) hipLaunchKernelGGL((decode_kernel<D, 1, PF, true>), grid, block, 0, s, a);
    else if (ntw <= 1) hipLaunchKernelGGL((decode_kernel<D, 1, PF, false>), grid, block, 0, s, a);
    else if (ntw == 2) hipLaunchKernelGGL((decode_kernel<D, 2, PF, false>), grid, block, 0, s, a);
    else if (ntw == 3) hipLaunchKernelGGL((decode_kernel<D, 3, PF, false>), grid, block, 0, s, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_decode(const StepArgs& a, hipStream_t s) {
    const int n_parts = a.n_parts_shared + a.n_parts_private;
    if (n_parts == 0) return hipSuccess;
    const dim3 grid(n_parts * a.n_kv_heads);
    const int ntw = a.n_parts_shared ? (a.max_row_tiles_shared + 3) / 4 : 1;
    const bool f32 = a.partial_format == PF_F32;
    if (a.head_dim == 128) return f32 ? launch_decode_as<128, PF_F32>(a, grid, ntw, s) : launch_decode_as<128, PF_F16S>(a, grid, ntw, s);
    if (a.head_dim == 64) return f32 ? launch_decode_as<64, PF_F32>(a, grid, ntw, s) : launch_decode_as<64, PF_F16S>(a, grid, ntw, s);
    return hipErrorInvalidValue;
}

hipError_t launch_resolve_slots(const StepArgs& a, int64_t* slots, int64_t stride, hipStream_t s) {
    if (stride <= 0) return hipSuccess;
    const dim3 grid(a.n_seqs, (unsigned)((stride + 255) / 256)), block(256);
    hipLaunchKernelGGL(resolve_slots_kernel, grid, block, 0, s, a, slots, stride);
    return hipGetLastError();
}

}  // namespace taper
