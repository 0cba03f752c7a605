// Host-side index resolution for one decode step (see taper_plan.h).
//
// Which KV each query row reads follows the visibility rule (paper §3.1): the
// request's shared prefix, then the sequence's own private tokens.  The shared
// prefix of a request with several admitted branches becomes "shared" work
// (read once, multiplied against all branches' query rows); everything else is
// "private" work (one sequence's rows).
#include "taper_plan.h"

#include <algorithm>
#include <cstdio>
#include <cstring>

namespace taper {

static std::string fmt(const char* f, long long a = 0, long long b = 0, long long c = 0) {
    char buf[256];
    std::snprintf(buf, sizeof buf, f, a, b, c);
    return buf;
}

int validate_config(const taper_attn_config& cfg, std::string* err) {
    if (cfg.n_q_heads < 1 || cfg.n_kv_heads < 1 || cfg.n_q_heads % cfg.n_kv_heads != 0) {
        *err = "n_q_heads must be a positive multiple of n_kv_heads";
        return TAPER_EINVAL;
    }
    int g = cfg.n_q_heads / cfg.n_kv_heads;
    if (g > 16) {
        *err = "at most 16 query heads per KV head are supported";
        return TAPER_EINVAL;
    }
    if (cfg.head_dim != 64 && cfg.head_dim != 128) {
        *err = "head_dim must be 64 or 128";
        return TAPER_EINVAL;
    }
    if (cfg.page_size != 16) {
        *err = "page_size must be 16";
        return TAPER_EINVAL;
    }
    if (!(cfg.scale > 0.0f) || !(cfg.scale < 1e30f)) {
        *err = "scale must be positive and finite";
        return TAPER_EINVAL;
    }
    if (cfg.partial_format != TAPER_PARTIAL_F16_SCALED && cfg.partial_format != TAPER_PARTIAL_F32) {
        *err = "unknown partial_format";
        return TAPER_EINVAL;
    }
    return TAPER_OK;
}

namespace {

constexpr int64_t kPieceCostTokens = 200;   // what one more piece of a cut sequence costs, in tokens' streaming time
constexpr int64_t kOnePerUnitLossPct = 3;   // what one workgroup per compute unit instead of two costs, percent

struct Segment {
    int32_t seq0, n_branch, page0, n_tokens, kind;
    int32_t ends_seq = 0;  // private: the last tokens of its sequence in plan order (whoever streams them usually merges)
    int32_t whole_seq = 0;  // private: the sequence's whole context
    int32_t siblings = 0;   // shared: this and the next siblings - 1 segments stream the same prefix (one request, cut into sub-groups)
};

// Cost model of a workgroup share, in units of one private token's streaming time: an item of
// n tokens costs fixed + n * per_token_pct / 100, `fixed` covering what an item costs beyond
// streaming its tokens (query load, pipeline fill, partial rows, arrival, merges).
struct Cost {
    int64_t per_token_pct, fixed;
    int64_t merge = 0;  // extra cost of the item that ends a sequence: it arrives last as a rule and merges the partials
};

// Cuts `segs` into workgroup shares of about `quota` cost units, at multiples of `blk` tokens
// from each segment's start: shares are filled one after the other, a segment going on into the
// next share where one is full.  Appends items (tagged with part ids starting at part_id0) and
// returns the number of shares used.
int partition_fill(const std::vector<Segment>& segs, int64_t quota, int blk, const Cost cost, int part_id0,
                   std::vector<taper_work_item>* items) {
    int64_t total_tokens = 0;
    for (const Segment& s : segs) total_tokens += s.n_tokens;
    if (total_tokens == 0) return 0;
    quota = std::max<int64_t>(1, quota);
    const int64_t blk_cost = std::max<int64_t>(1, blk * cost.per_token_pct / 100);
    // a piece is only worth an item of its own if its streaming outweighs the item's fixed cost
    const int64_t min_blocks = std::max<int64_t>(1, (cost.fixed + blk_cost - 1) / blk_cost);
    const int64_t cap = std::max<int64_t>(1, (quota - cost.fixed) / blk_cost);  // blocks of an item with a share to itself
    int part = 0;
    int64_t fill = 0;
    for (const Segment& s : segs) {
        int64_t remaining = (s.n_tokens + blk - 1) / blk, off = 0;  // blocks
        while (remaining > 0) {
            const int64_t room = (quota - fill - cost.fixed) / blk_cost;  // blocks that still fit this share
            if (fill > 0 && room < remaining && room < min_blocks) {        // start the next share instead
                ++part;
                fill = 0;
                continue;
            }
            int64_t take = std::min(remaining, std::max<int64_t>(room, 1));
            // A sequence much shorter than a share is not cut: cutting would turn one item that needs no
            // partial rows at all into two with a merge.  It goes whole into this share if at least half of
            // it fits, else into the next.
            if (s.whole_seq && off == 0 && take < remaining && remaining * 4 <= cap) {
                if (fill > 0 && room * 2 < remaining) {
                    ++part;
                    fill = 0;
                    continue;
                }
                take = remaining;
            }
            if (remaining - take > 0 && remaining - take < min_blocks) take = remaining;  // no sliver left behind
            taper_work_item it;
            std::memset(&it, 0, sizeof it);
            it.seq0 = s.seq0;
            it.n_branch = s.n_branch;
            it.page0 = s.page0 + (int32_t)(off * blk / 16);
            it.n_tokens = (int32_t)std::min<int64_t>(take * blk, s.n_tokens - off * blk);
            it.kind = s.kind;
            it.part = part_id0 + part;
            items->push_back(it);
            fill += cost.fixed + take * blk_cost;
            off += take;
            remaining -= take;
            if (remaining == 0 && s.ends_seq) fill += cost.merge;
            if (fill >= quota) {
                ++part;
                fill = 0;
            }
        }
    }
    return fill > 0 ? part + 1 : part;
}

// The same for items with a large fixed cost (shared-prefix items).  A segment that does not
// fit what is left of the current share tops it up (if that is worth an item); what then
// remains, if it is more than one share, is cut into equal items with a share each rather than
// into full shares and a remainder (which would either be a short item paying the full fixed
// cost or make the last item much longer than the others).  The last of those items is
// `tail_discount` blocks shorter: the workgroup that finishes a shared prefix usually finds the
// request's branches complete and has to merge them all.
int partition_even(const std::vector<Segment>& segs, int64_t quota, int blk, const Cost cost, int64_t tail_discount,
                   int part_id0, std::vector<taper_work_item>* items) {
    quota = std::max<int64_t>(1, quota);
    const int64_t blk_cost = std::max<int64_t>(1, blk * cost.per_token_pct / 100);
    const int64_t min_blocks = std::max<int64_t>(1, (cost.fixed + blk_cost - 1) / blk_cost);
    const int64_t cap = std::max<int64_t>(min_blocks, (quota - cost.fixed) / blk_cost);  // blocks of an item with a share to itself
    int part = 0;
    int64_t fill = 0;
    auto emit = [&](const Segment& s, int64_t off, int64_t take) {
        taper_work_item it;
        std::memset(&it, 0, sizeof it);
        it.seq0 = s.seq0;
        it.n_branch = s.n_branch;
        it.page0 = s.page0 + (int32_t)(off * blk / 16);
        it.n_tokens = (int32_t)std::min<int64_t>(take * blk, s.n_tokens - off * blk);
        it.kind = s.kind;
        it.part = part_id0 + part;
        items->push_back(it);
        fill += cost.fixed + take * blk_cost;
    };
    auto close = [&]() {
        if (fill > 0) ++part;
        fill = 0;
    };
    for (size_t si = 0; si < segs.size(); ++si) {
        const Segment& s = segs[si];
        if (s.siblings >= 2) {
            // Sub-groups of one request read the same pages.  They get the same cuts, every item a share of its
            // own and therefore the launch's start as its start, in workgroups next to each other: the sub-groups
            // then stream the prefix in step, and what the first one fetched is still in the L2 of the XCD (one
            // per kv head) when the others ask for it.  Shares that come out short take from the pool.
            close();
            const int64_t blocks = (s.n_tokens + blk - 1) / blk;
            const int64_t spread = blocks + tail_discount;
            const int64_t k = blocks <= cap + min_blocks / 2 ? 1 : std::max<int64_t>(1, (spread + cap - 1) / cap);
            int64_t remaining = blocks, off = 0;
            for (int64_t i = 0; i < k; ++i) {
                int64_t take = spread / k + (i < spread % k ? 1 : 0);
                take = i + 1 < k ? std::max<int64_t>(1, std::min(take, remaining - (k - 1 - i))) : remaining;
                for (int j = 0; j < s.siblings; ++j) {
                    emit(segs[si + j], off, take);
                    close();
                }
                off += take;
                remaining -= take;
            }
            si += s.siblings - 1;
            continue;
        }
        int64_t remaining = (s.n_tokens + blk - 1) / blk, off = 0;  // blocks
        int64_t room = (quota - fill - cost.fixed) / blk_cost;      // blocks that still fit the current share
        if (fill > 0 && room < remaining && room < min_blocks) {    // not worth an item: start the next share
            close();
            room = cap;
        }
        if (remaining > room && fill > 0) {  // top the current share up
            emit(s, 0, room);
            close();
            off = room;
            remaining -= room;
        }
        if (remaining <= cap + min_blocks / 2) {  // one item; the next segment may top its share up
            emit(s, off, remaining);
            if (fill >= quota) close();
            continue;
        }
        const int64_t spread = remaining + tail_discount;
        const int64_t k = std::max<int64_t>(1, (spread + cap - 1) / cap);
        for (int64_t i = 0; i < k; ++i) {
            int64_t take = spread / k + (i < spread % k ? 1 : 0);
            take = i + 1 < k ? std::max<int64_t>(1, std::min(take, remaining - (k - 1 - i))) : remaining;
            emit(s, off, take);
            close();
            off += take;
            remaining -= take;
        }
    }
    close();
    return part;
}

}  // namespace

int build_host_plan(const taper_attn_config& cfg, int n_seqs, const int32_t* block_table, int bt_row_stride,
                    const int32_t* branch_group, const int32_t* prefix_len, const int32_t* suffix_len,
                    int64_t n_pool_pages, const taper_plan_options* opts, HostPlan* out, std::string* err) {
    if (!suffix_len || n_seqs < 1) {
        *err = "null argument";
        return TAPER_EINVAL;
    }
    std::vector<int32_t> seg_start(n_seqs + 1);
    for (int s = 0; s <= n_seqs; ++s) seg_start[s] = s;  // one private segment per sequence
    return build_host_plan_segments(cfg, n_seqs, block_table, bt_row_stride, branch_group, prefix_len, seg_start.data(),
                                    suffix_len, n_pool_pages, opts, out, err);
}

static int build_for_grid(const taper_attn_config& cfg, int n_seqs, const int32_t* block_table, int bt_row_stride,
                          const int32_t* branch_group, const int32_t* prefix_len, const int32_t* seg_start,
                          const int32_t* seg_len, int64_t n_pool_pages, const taper_plan_options* opts,
                          HostPlan* out, std::string* err) {
    int st = validate_config(cfg, err);
    if (st != TAPER_OK) return st;
    if (!block_table || !branch_group || !prefix_len || !seg_start || !out) {
        *err = "null argument";
        return TAPER_EINVAL;
    }
    if (n_seqs < 1 || bt_row_stride < 1 || n_pool_pages < 1) {
        *err = "n_seqs, bt_row_stride and n_pool_pages must be positive";
        return TAPER_EINVAL;
    }
    if (n_pool_pages > (int64_t)1 << 31) {
        *err = "n_pool_pages exceeds the int32 page id range";
        return TAPER_EINVAL;
    }
    const int P = cfg.page_size;
    const int g = cfg.n_q_heads / cfg.n_kv_heads;
    int target_wgs = opts && opts->target_workgroups > 0 ? opts->target_workgroups : 512;
    const bool share_prefix = opts ? opts->share_prefix != 0 : true;
    // A shared item holds up to 12 row tiles.  At head_dim 128 the kernel for 9 to 12 tiles loads
    // straight into LDS and still runs two workgroups per compute unit; at 64 it stages through
    // registers and runs one, so requests are cut at 8 tiles unless asked otherwise.
    // 64: per-branch flags of the shared kernel.
    const int hard_cap = std::min(64, std::max(2, kMaxRowTilesPerItem * 16 / g));
    int cap_branches = std::min(hard_cap, std::max(2, (cfg.head_dim == 128 ? kMaxRowTilesPerItem : 8) * 16 / g));
    if (opts && opts->max_branches_per_item > 0) cap_branches = std::max(1, std::min(hard_cap, opts->max_branches_per_item));

    HostPlan& p = *out;
    p = HostPlan();
    p.n_seqs = n_seqs;
    p.bt_stride = bt_row_stride;
    p.n_pool_pages = n_pool_pages;
    p.prefix_len.assign(prefix_len, prefix_len + n_seqs);
    // private segments: CSR per sequence, lengths, and the block-table entry each one starts at
    if (seg_start[0] != 0) {
        *err = "seg_start[0] must be 0";
        return TAPER_EINVAL;
    }
    for (int s = 0; s < n_seqs; ++s)
        if (seg_start[s + 1] < seg_start[s]) {
            *err = fmt("sequence %lld: seg_start must not decrease", s);
            return TAPER_EINVAL;
        }
    if (seg_start[n_seqs] > 0 && !seg_len) {
        *err = "null argument";
        return TAPER_EINVAL;
    }
    p.seg_start.assign(seg_start, seg_start + n_seqs + 1);
    p.seg_len.assign(seg_len, seg_len + seg_start[n_seqs]);
    p.seg_page0.assign(seg_start[n_seqs], 0);
    p.suffix_len.assign(n_seqs, 0);
    p.ctx_len.resize(n_seqs);
    p.n_prefix_pages.resize(n_seqs);
    p.n_suffix_pages.resize(n_seqs);
    p.block_table.assign((size_t)n_seqs * bt_row_stride, -1);

    // ---- validation + per-sequence integers
    for (int s = 0; s < n_seqs; ++s) {
        const int64_t pl = prefix_len[s];
        int64_t sl = 0, nsp = 0;
        if (pl < 0) {
            *err = fmt("sequence %lld: negative length", s);
            return TAPER_ELEN;
        }
        const int64_t npp = (pl + P - 1) / P;
        for (int k = seg_start[s]; k < seg_start[s + 1]; ++k) {
            if (seg_len[k] < 0) {
                *err = fmt("sequence %lld: negative length", s);
                return TAPER_ELEN;
            }
            p.seg_page0[k] = (int32_t)std::min<int64_t>(npp + nsp, INT32_MAX);
            sl += seg_len[k];
            nsp += (seg_len[k] + P - 1) / P;
        }
        if (pl + sl < 1) {
            *err = fmt("sequence %lld: empty context", s);
            return TAPER_ELEN;
        }
        if (pl + sl > (1 << 30)) {
            *err = fmt("sequence %lld: context too long", s);
            return TAPER_ELEN;
        }
        p.suffix_len[s] = (int32_t)sl;
        if (npp + nsp > bt_row_stride) {
            *err = fmt("sequence %lld: needs %lld block-table entries, row has %lld", s, npp + nsp, bt_row_stride);
            return TAPER_ELEN;
        }
        p.ctx_len[s] = (int32_t)(pl + sl);
        p.n_prefix_pages[s] = (int32_t)npp;
        p.n_suffix_pages[s] = (int32_t)nsp;
        const int32_t* row = block_table + (size_t)s * bt_row_stride;
        for (int j = 0; j < npp + nsp; ++j) {
            if (row[j] < 0 || row[j] >= n_pool_pages) {
                *err = fmt("sequence %lld entry %lld: page %lld outside the pool", s, j, row[j]);
                return TAPER_EBLOCK;
            }
            p.block_table[(size_t)s * bt_row_stride + j] = row[j];
        }
        p.tokens_logical += pl + sl;
    }
    // ---- request CSR
    for (int s = 0; s < n_seqs; ++s) {
        if (s == 0) {
            if (branch_group[0] != 0) {
                *err = "branch_group must start at 0";
                return TAPER_EGROUP;
            }
            p.group_start.push_back(0);
        } else if (branch_group[s] == branch_group[s - 1] + 1) {
            p.group_start.push_back(s);
        } else if (branch_group[s] != branch_group[s - 1]) {
            *err = fmt("sequence %lld: branch_group must be non-decreasing in steps of 1", s);
            return TAPER_EGROUP;
        }
    }
    p.n_groups = (int)p.group_start.size();
    p.group_start.push_back(n_seqs);
    for (int gi = 0; gi < p.n_groups; ++gi) {
        const int a = p.group_start[gi], b = p.group_start[gi + 1];
        for (int s = a + 1; s < b; ++s) {
            if (prefix_len[s] != prefix_len[a]) {
                *err = fmt("sequence %lld: prefix_len differs from its request's first member", s);
                return TAPER_EGROUP;
            }
            if (std::memcmp(block_table + (size_t)s * bt_row_stride, block_table + (size_t)a * bt_row_stride,
                            sizeof(int32_t) * p.n_prefix_pages[a]) != 0) {
                *err = fmt("sequence %lld: prefix pages differ from its request's first member", s);
                return TAPER_EGROUP;
            }
        }
    }

    // ---- segments of KV to stream
    std::vector<Segment> shared, priv;
    for (int gi = 0; gi < p.n_groups; ++gi) {
        const int a = p.group_start[gi], b = p.group_start[gi + 1], B = b - a;
        const int pl = prefix_len[a];
        p.tokens_unique += pl;
        if (pl > 0) {
            if (B >= 2 && share_prefix) {
                const int n_sub = (B + cap_branches - 1) / cap_branches;
                const size_t first = shared.size();
                for (int k = 0; k < n_sub; ++k) {  // balanced sub-groups of at most cap_branches
                    const int lo = a + (int)((int64_t)B * k / n_sub), hi = a + (int)((int64_t)B * (k + 1) / n_sub);
                    if (hi - lo >= 2)
                        shared.push_back({lo, hi - lo, 0, pl, 0});
                    else if (hi - lo == 1)
                        priv.push_back({lo, 1, 0, pl, 1});
                }
                if (shared.size() - first >= 2 && !(opts && opts->scatter_sub_groups)) shared[first].siblings = (int32_t)(shared.size() - first);
            } else {
                for (int s = a; s < b; ++s) priv.push_back({s, 1, 0, pl, 1});
            }
        }
        for (int s = a; s < b; ++s) {
            p.tokens_unique += p.suffix_len[s];
            for (int k = seg_start[s]; k < seg_start[s + 1]; ++k)
                if (seg_len[k] > 0) priv.push_back({s, 1, p.seg_page0[k], seg_len[k], 1});
            if (!priv.empty() && priv.back().seq0 == s) priv.back().ends_seq = 1;
        }
    }

    {  // private segments that are their sequence's whole context
        std::vector<int32_t> pieces(n_seqs, 0);
        for (const Segment& s : shared)
            for (int b = 0; b < s.n_branch; ++b) pieces[s.seq0 + b] += 2;
        for (const Segment& s : priv) pieces[s.seq0] += 1;
        for (Segment& s : priv) s.whole_seq = pieces[s.seq0] == 1;
    }

    // ---- workgroup shares: both kinds run in one launch and should finish together.  A workgroup of
    // the shared kind keeps fewer bytes in flight than one of the private kind and so gets a smaller
    // slice of a saturated memory system: its tokens are weighted by shared_cost_pct / 100.  Every
    // item also has a fixed cost (a shared item's is large: rows of several branches to store, and
    // the merges of all branches it completes).
    int widest = 0;  // row tiles of the widest shared item: up to 4, the kernel stages with three register sets,
                     // up to 8 with two, above that straight into LDS (measured weights for each)
    for (const Segment& s : shared) widest = std::max(widest, (s.n_branch * g + 15) / 16);
    const Cost cost_shared = {opts && opts->shared_cost_pct > 0 ? opts->shared_cost_pct : (widest <= 4 ? 160 : (widest <= 8 || cfg.head_dim != 128) ? 200 : 140),
                              opts && opts->shared_item_cost > 0 ? opts->shared_item_cost : 800};
    const Cost cost_priv = {100, opts && opts->private_item_cost > 0 ? opts->private_item_cost : 128,
                            opts && opts->private_merge_cost != 0 ? std::max(0, opts->private_merge_cost)
                                                                  : (shared.empty() ? 0 : 192)};
    const int64_t shared_tail_discount = 3;  // blocks: about what merging a request's branches costs
    int64_t cost_total = 0;
    for (const Segment& s : shared) {
        cost_total += cost_shared.fixed + (int64_t)s.n_tokens * cost_shared.per_token_pct / 100;
    }
    for (const Segment& s : priv) {
        cost_total += cost_priv.fixed + s.n_tokens + (s.ends_seq ? cost_priv.merge : 0);
    }
    const int parts_total = std::max(1, target_wgs / cfg.n_kv_heads);
    // ---- the pool: private tokens no share owns.  No cost model predicts the shares' running times
    // to better than some ten percent (the kinds' speeds depend on the mix, page placement matters),
    // so the shares are cut a little short and every workgroup that finishes its share takes items
    // from the pool until it is empty.  Pool items are small: the last one bounds the tail.
    // Without shared-prefix work the shares are alike and end within a few percent of each other:
    // a pool would only add items.
    const int pool_pct = opts && opts->pool_pct != 0 ? std::max(0, std::min(90, opts->pool_pct)) : (shared.empty() ? 0 : 25);
    const int pool_item_opt = opts && opts->pool_item_tokens > 0 ? opts->pool_item_tokens : 0;
    std::vector<Segment> pool;
    {
        int64_t tok_priv = 0;
        for (const Segment& s : priv) tok_priv += s.n_tokens;
        int64_t want = tok_priv * pool_pct / 100;
        while (want >= kPrivateBlockTokens && !priv.empty()) {
            Segment& s = priv.back();
            if (s.n_tokens <= want + kPrivateBlockTokens) {  // the whole segment
                want -= s.n_tokens;
                cost_total -= cost_priv.fixed + s.n_tokens + (s.ends_seq ? cost_priv.merge : 0);
                pool.push_back(s);
                priv.pop_back();
            } else {  // its tail, from a block boundary
                const int keep = (int)((s.n_tokens - want + kPrivateBlockTokens - 1) / kPrivateBlockTokens * kPrivateBlockTokens);
                if (keep < s.n_tokens) {
                    pool.push_back({s.seq0, s.n_branch, s.page0 + keep / 16, s.n_tokens - keep, s.kind, s.ends_seq, 0});
                    s.whole_seq = 0;
                    cost_total -= s.n_tokens - keep + (s.ends_seq ? cost_priv.merge : 0);
                    s.n_tokens = keep;
                    s.ends_seq = 0;
                }
                want = 0;
            }
        }
        std::reverse(pool.begin(), pool.end());
    }
    // A small step is not cut as finely as the grid allows: below a few hundred tokens per share the
    // time goes into the item ends, and a sequence cut into many partials pays a merge round per eight.
    int64_t longest = 0;
    for (const Segment& s : priv) longest = std::max<int64_t>(longest, s.n_tokens);
    const int64_t min_share =
        (opts && opts->min_share_tokens > 0 ? opts->min_share_tokens : std::max<int64_t>(256, longest / 16)) + cost_priv.fixed;
    int64_t quota = std::max<int64_t>(std::max<int64_t>(kSharedBlockTokens, min_share), (cost_total + parts_total - 1) / parts_total);
    for (;;) {  // never more shares than asked for: an extra one would run after all the others
        p.items.clear();
        p.n_parts_shared = partition_even(shared, quota, kSharedBlockTokens, cost_shared, shared_tail_discount, 0, &p.items);
        p.n_parts_private = partition_fill(priv, quota, kPrivateBlockTokens, cost_priv, p.n_parts_shared, &p.items);
        if (p.n_parts_shared + p.n_parts_private <= parts_total || quota >= cost_total * 2 + 4096) break;
        quota += std::max<int64_t>(16, quota / 256);
    }
    const int n_parts = p.n_parts_shared + p.n_parts_private;
    p.part_start.assign(n_parts + 1, 0);
    for (const taper_work_item& it : p.items) p.part_start[it.part + 1]++;
    for (int i = 0; i < n_parts; ++i) p.part_start[i + 1] += p.part_start[i];
    // size of the pool's items: a quarter of a share, between 512 and 1536 tokens, unless the caller says otherwise
    const int pool_item_tokens = std::max<int>(
        kPrivateBlockTokens,
        (pool_item_opt ? pool_item_opt : (int)std::min<int64_t>(1536, std::max<int64_t>(512, quota / 4))) / kPrivateBlockTokens * kPrivateBlockTokens);
    for (const Segment& s : pool) {  // pool items follow the shares' items; their `part` is n_parts
        const int k = (s.n_tokens + pool_item_tokens - 1) / pool_item_tokens;
        const int piece = ((s.n_tokens + k - 1) / k + kPrivateBlockTokens - 1) / kPrivateBlockTokens * kPrivateBlockTokens;
        for (int off = 0; off < s.n_tokens; off += piece) {
            taper_work_item it;
            std::memset(&it, 0, sizeof it);
            it.seq0 = s.seq0;
            it.n_branch = 1;
            it.page0 = s.page0 + off / 16;
            it.n_tokens = std::min(piece, s.n_tokens - off);
            it.kind = 1;
            it.part = n_parts;
            p.items.push_back(it);
        }
    }
    p.n_pool_items = (int)p.items.size() - p.part_start[n_parts];
    // longest first: the launch's last claims are then the shortest items
    std::stable_sort(p.items.begin() + p.part_start[n_parts], p.items.end(),
                     [](const taper_work_item& x, const taper_work_item& y) { return x.n_tokens > y.n_tokens; });

    // ---- partial rows and merge map
    std::vector<std::vector<taper_merge_entry>> per_seq(n_seqs);
    int64_t rows = 0;
    for (taper_work_item& it : p.items) {
        // (the merge addresses partial rows by 32-bit byte offsets: fp32 rows of a step stay below 2^31 bytes)
        if ((rows + (int64_t)it.n_branch * cfg.n_q_heads) * cfg.head_dim * 4 > INT32_MAX) {
            *err = "too many partial rows";
            return TAPER_EINVAL;
        }
        it.part_base = (int32_t)rows;
        const int rph = it.n_branch * g;
        if (it.kind == 0) p.max_row_tiles_shared = std::max(p.max_row_tiles_shared, (rph + 15) / 16);
        for (int b = 0; b < it.n_branch; ++b) per_seq[it.seq0 + b].push_back({it.part_base + b * g, rph});
        rows += (int64_t)rph * cfg.n_kv_heads;
    }
    p.n_partial_rows = rows;
    p.merge_start.assign(n_seqs + 1, 0);
    for (int s = 0; s < n_seqs; ++s) {
        p.merge_start[s + 1] = p.merge_start[s] + (int32_t)per_seq[s].size();
        p.merge.insert(p.merge.end(), per_seq[s].begin(), per_seq[s].end());
    }
    for (taper_work_item& it : p.items) {
        it.merge0 = p.merge_start[it.seq0];
        // a private item that is its sequence's whole context needs no partial rows: the kernel writes the result
        if (it.kind == 1 && p.merge_start[it.seq0 + 1] - p.merge_start[it.seq0] == 1) it.kind = 2;
    }
    // Runs of short such items inside one share are worked on by single waves, four items side by side
    // (a 128-token item gives a wave one block to do when four waves share it: all latency, no streaming).
    const int solo_tokens = opts && opts->solo_item_tokens != 0 ? opts->solo_item_tokens : 512;
    const int n_parts_all = p.n_parts_shared + p.n_parts_private;
    for (int part = p.n_parts_shared; part < n_parts_all && solo_tokens > 0; ++part) {
        int i = p.part_start[part];
        const int end = p.part_start[part + 1];
        while (i < end) {
            int j = i;
            while (j < end && p.items[j].kind == 2 && p.items[j].n_tokens <= solo_tokens) ++j;
            if (j - i >= kSoloMinRun)
                for (int k = i; k < j; ++k) p.items[k].kind = 3;
            i = std::max(j, i + 1);
        }
    }
    return TAPER_OK;
}

// Cutting a sequence costs: every piece writes partial rows, announces them, and one workgroup reads them all back
// (three dependent trips through a loaded memory system, some 200 tokens' streaming time per piece).  A step
// without shared-prefix work whose shares are short is therefore also cut for half the grid -- one workgroup per
// compute unit instead of two, which alone reads 1 to 4 % slower -- and that plan is taken when it saves enough
// pieces to pay for it.  (32 requests of 1024-4096 tokens: 86 pieces become 54 and the launch 2.5 % faster;
// 32 equal requests: no piece at all, 5-10 % faster; a large step has few pieces per share either way.)
int build_host_plan_segments(const taper_attn_config& cfg, int n_seqs, const int32_t* block_table, int bt_row_stride,
                             const int32_t* branch_group, const int32_t* prefix_len, const int32_t* seg_start,
                             const int32_t* seg_len, int64_t n_pool_pages, const taper_plan_options* opts,
                             HostPlan* out, std::string* err) {
    int st = build_for_grid(cfg, n_seqs, block_table, bt_row_stride, branch_group, prefix_len, seg_start, seg_len,
                            n_pool_pages, opts, out, err);
    if (st != TAPER_OK || !opts || opts->small_step_grid <= 0) return st;
    const int grid = opts->target_workgroups > 0 ? opts->target_workgroups : 512;
    const int parts_full = std::max(1, grid / cfg.n_kv_heads);
    if (out->n_parts_shared != 0 || out->n_pool_items != 0 || out->n_parts_private < parts_full || parts_full < 2) return st;
    auto pieces = [](const HostPlan& h) {
        int64_t n = 0;
        for (const taper_work_item& it : h.items) n += it.kind == 1;
        return n;
    };
    const int64_t pieces_full = pieces(*out);
    if (pieces_full * kPieceCostTokens * 100 <= out->tokens_unique * kOnePerUnitLossPct) return st;  // cannot pay even if all went
    taper_plan_options half = *opts;
    half.target_workgroups = grid / 2;
    HostPlan alt;
    std::string err2;
    if (build_for_grid(cfg, n_seqs, block_table, bt_row_stride, branch_group, prefix_len, seg_start, seg_len, n_pool_pages,
                       &half, &alt, &err2) != TAPER_OK)
        return st;
    if ((pieces_full - pieces(alt)) * kPieceCostTokens * 100 > out->tokens_unique * kOnePerUnitLossPct) *out = std::move(alt);
    return st;
}

void resolve_slots_host(const HostPlan& p, int P, int64_t* slots, int64_t stride) {
    for (int s = 0; s < p.n_seqs; ++s) {
        const int32_t* row = p.block_table.data() + (size_t)s * p.bt_stride;
        for (int64_t t = 0; t < stride; ++t) {
            int64_t v = -1;
            if (t < p.ctx_len[s]) {
                if (t < p.prefix_len[s]) {
                    v = (int64_t)row[t / P] * P + t % P;
                } else {
                    int64_t j = t - p.prefix_len[s];
                    int k = p.seg_start[s];
                    while (j >= p.seg_len[k]) j -= p.seg_len[k++];
                    v = (int64_t)row[p.seg_page0[k] + j / P] * P + j % P;
                }
            }
            slots[(size_t)s * stride + t] = v;
        }
    }
}

}  // namespace taper
