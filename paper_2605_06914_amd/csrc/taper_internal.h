// Interface between the C-ABI layer and the HIP kernels (device pointers only).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "taper_attn.h"

namespace taper {

// Device-resident integer metadata of one step plus the tensors of one layer.
struct StepArgs {
    const void* q;             // bf16 [S][Hq][D]
    const void* kv;            // bf16 pool
    void* out;                 // bf16 [S][Hq][D]
    float* lse;                // f32 [S][Hq] or null
    const int32_t* bt;         // [S][bt_stride]
    const taper_work_item* items;
    const int32_t* part_start;
    const int32_t* merge_start;
    const taper_merge_entry* merge;
    const int32_t* prefix_len;
    const int32_t* seg_start;      // [n_seqs + 1] private segments of each sequence
    const int32_t* seg_len;        // tokens of each private segment
    const int32_t* seg_page0;      // block-table entry each private segment starts at
    const int32_t* ctx_len;
    float4* ws_ml;             // [n_partial_rows] (running max in log2 units, sum, row scale, unused)
    void* ws_o;                // [n_partial_rows][D] partial rows, each divided by its own sum: fp32, or half
                               // precision times the row's power-of-two scale (taper_partial_format)
    int32_t* counters;         // [n_seqs][n_kv_heads] partials delivered so far; zero between launches
    int32_t* pool_ctr;         // [n_kv_heads] pool items taken so far; zero between launches
    int32_t pool_first, n_pool_items;  // the pool: items [pool_first, pool_first + n_pool_items)
    int32_t bt_stride;
    int32_t n_seqs;
    int32_t n_merge;           // entries in `merge`
    int32_t n_q_heads, n_kv_heads, gqa, head_dim;
    int32_t n_parts_shared, n_parts_private;
    int32_t max_row_tiles_shared;
    float scale_log2e;         // scale * log2(e)
    int32_t partial_format;    // taper_partial_format of ws_o
#ifdef TAPER_WG_TRACE
    long long* trace;          // [4 * workgroups] clocks of a trace build (see wg_trace.py), or null
#endif
};


// Device memory that belongs to no context: the scratch array of taper_decode_step_attention_static.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
// Address of the calling device's copy of the array (looked up once per device; `device` must be current).
hipError_t static_scratch(int device, void** ptr);
hipError_t launch_zero_words(int32_t* p, int64_t n, hipStream_t s);

hipError_t launch_decode(const StepArgs& a, hipStream_t s);
hipError_t launch_kv_append(const void* k_new, const void* v_new, const int64_t* slot, void* kv, int n_seqs, int n_kv_heads,
                            int head_dim, hipStream_t s);
hipError_t launch_stream_read(const void* base, int64_t pieces_per_wg, int n_workgroups, unsigned* sink, hipStream_t s);
hipError_t launch_resolve_slots(const StepArgs& a, int64_t* slots, int64_t stride, hipStream_t s);

}  // namespace taper
