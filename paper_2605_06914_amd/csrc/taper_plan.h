// Host-side index resolution for one decode step: validation, request CSR,
// KV chunk list, workgroup shares and merge map.  Pure integer C++, no HIP.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "taper_attn.h"

namespace taper {

constexpr int kPrivateBlockTokens = 32;  // tokens one wave of the private kernel consumes per iteration
constexpr int kSharedBlockTokens = 64;   // tokens one workgroup of the shared kernel stages per iteration
constexpr int kSoloMinRun = 4;           // shortest run of short single-item sequences handed to single waves
constexpr int kMaxRowTilesPerItem = 12;  // 16-row query tiles one shared-kernel workgroup can hold (4 waves x 3)

struct HostPlan {
    int n_seqs = 0, n_groups = 0, bt_stride = 0;
    int64_t n_pool_pages = 0;
    std::vector<int32_t> block_table;  // [n_seqs * bt_stride], entries past a row's pages set to -1
    std::vector<int32_t> prefix_len, suffix_len, ctx_len, n_prefix_pages, n_suffix_pages;
    std::vector<int32_t> seg_start, seg_len, seg_page0;  // private segments: CSR [n_seqs + 1], tokens, first block-table entry
    std::vector<int32_t> group_start;  // [n_groups + 1]
    std::vector<taper_work_item> items;
    int n_parts_shared = 0, n_parts_private = 0;
    int n_pool_items = 0;  // items after the shares' items, owned by no share
    std::vector<int32_t> part_start;  // [n_parts + 1]
    std::vector<int32_t> merge_start; // [n_seqs + 1]
    std::vector<taper_merge_entry> merge;
    int64_t n_partial_rows = 0;
    int64_t tokens_unique = 0, tokens_logical = 0;
    int max_row_tiles_shared = 0;  // over shared items: ceil(n_branch * gqa / 16)
};

// Returns TAPER_OK or a negative status; `err` receives a message on failure.
int build_host_plan(const taper_attn_config& cfg, int n_seqs, const int32_t* block_table, int bt_row_stride,
                    const int32_t* branch_group, const int32_t* prefix_len, const int32_t* suffix_len,
                    int64_t n_pool_pages, const taper_plan_options* opts, HostPlan* out, std::string* err);

// The general form: sequence s sees its prefix and then the private segments seg_len[seg_start[s] .. seg_start[s+1]),
// each on pages of its own (suffix_len / n_suffix_pages of the plan are then totals over the segments).
int build_host_plan_segments(const taper_attn_config& cfg, int n_seqs, const int32_t* block_table, int bt_row_stride,
                             const int32_t* branch_group, const int32_t* prefix_len, const int32_t* seg_start,
                             const int32_t* seg_len, int64_t n_pool_pages, const taper_plan_options* opts,
                             HostPlan* out, std::string* err);

int validate_config(const taper_attn_config& cfg, std::string* err);

void resolve_slots_host(const HostPlan& p, int page_size, int64_t* slots, int64_t stride);

}  // namespace taper
