// C-ABI layer: context / plan lifetime, device copies of the plan, launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "taper_attn.h"
#include "taper_internal.h"
#include "taper_plan.h"
#ifdef TAPER_WG_TRACE
#include "taper_trace.h"
#endif

namespace {
thread_local std::string g_last_error;

int fail(int code, const std::string& msg) {
    g_last_error = msg;
    return code;
}
int fail_hip(hipError_t e, const char* what) {
    g_last_error = std::string(what) + ": " + hipGetErrorString(e);
    return TAPER_EHIP;
}
#define HIP_TRY(expr)                                  \
    do {                                               \
        hipError_t e_ = (expr);                        \
        if (e_ != hipSuccess) return fail_hip(e_, #expr); \
    } while (0)

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
// largest plan image taper_decode_step_attention_static uploads (block table and work lists of one step)
constexpr size_t kStaticImageBytes = (size_t)8 << 20;
}  // namespace

namespace taper {
int set_error(int code, const std::string& msg) { return fail(code, msg); }
}  // namespace taper

// Device + pinned-host buffers of a plan.  They are recycled through the context
// so that a steady-state decode loop neither allocates nor frees (hipFree would
// synchronise the device once per step).
struct PlanBuffers {
    void* dev = nullptr;      // one device allocation holding every integer array
    void* staging = nullptr;  // pinned host image of `dev`
    size_t bytes = 0;
    hipEvent_t uploaded = nullptr;  // recorded after the host-to-device copy
};

// Partial rows and counters of launches: [counters] int32 | [rows] float4 (m, l, row scale, -) | [rows][D] rows.
// A plan is bound to one workspace for its whole life, and a workspace lives at least as long as
// the plans bound to it: launches in flight and captured graphs keep valid addresses whatever
// is built later.
struct Workspace {
    void* base = nullptr;  // null on a host-only context (bookkeeping only)
    int64_t rows = 0, counters = 0;
    size_t ml_off = 0, o_off = 0, bytes = 0;
    int refs = 0;  // live plans bound to it
    int id = 0;
};

// Where the device arrays of a plan sit (inside a plan's own buffer, or inside the static scratch array).
struct DeviceImage {
    const int32_t* bt = nullptr;
    const taper_work_item* items = nullptr;
    const int32_t* part_start = nullptr;
    const int32_t* merge_start = nullptr;
    const taper_merge_entry* merge = nullptr;
    const int32_t* prefix_len = nullptr;
    const int32_t* seg_start = nullptr;
    const int32_t* seg_len = nullptr;
    const int32_t* seg_page0 = nullptr;
    const int32_t* ctx_len = nullptr;
};

struct taper_ctx {
    taper_attn_config cfg;
    bool host_only = false;
    std::vector<Workspace*> workspaces;  // the last one is current; earlier ones wait for their plans to go
    int next_workspace_id = 1;
    bool counters_suspect = false;  // a call reported a HIP error: clear every workspace's counters before the next launch
    std::vector<PlanBuffers> free_buffers;
    int default_workgroups = 0;  // two resident workgroups per compute unit of the device (0: the builder's own default)
    // for taper_decode_step_attention_static: the device's copy of the library's scratch array, and a pinned
    // image of the plan that is uploaded into it (made at taper_create: the call itself allocates nothing)
    void* static_scratch = nullptr;
    std::string static_error;  // why static_scratch is null
    void* static_staging = nullptr;
    hipEvent_t static_uploaded = nullptr;
#ifdef TAPER_WG_TRACE
    long long* trace = nullptr;
#endif
};

struct taper_plan {
    taper_ctx* ctx = nullptr;
    taper::HostPlan host;
    PlanBuffers buf;
    DeviceImage img;
    Workspace* ws = nullptr;
};

namespace {

void destroy_buffers(PlanBuffers& b) {
    if (b.uploaded) {
        (void)hipEventSynchronize(b.uploaded);
        (void)hipEventDestroy(b.uploaded);
    }
    if (b.dev) (void)hipFree(b.dev);
    if (b.staging) (void)hipHostFree(b.staging);
    b = PlanBuffers();
}

// Takes a recycled buffer set of at least `bytes`, or allocates one.
int acquire_buffers(taper_ctx* ctx, size_t bytes, PlanBuffers* out) {
    for (size_t i = 0; i < ctx->free_buffers.size(); ++i) {
        if (ctx->free_buffers[i].bytes >= bytes) {
            *out = ctx->free_buffers[i];
            ctx->free_buffers.erase(ctx->free_buffers.begin() + i);
            // the pinned image is about to be overwritten: its last copy must have finished
            hipError_t e = hipEventSynchronize(out->uploaded);
            if (e != hipSuccess) return fail_hip(e, "hipEventSynchronize");
            return TAPER_OK;
        }
    }
    PlanBuffers b;
    b.bytes = align_up(bytes + bytes / 2, 4096);
    hipError_t e = hipHostMalloc(&b.staging, b.bytes, hipHostMallocDefault);
    if (e == hipSuccess) e = hipMalloc(&b.dev, b.bytes);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&b.uploaded, hipEventDisableTiming);
    if (e != hipSuccess) {
        g_last_error = std::string("plan allocation: ") + hipGetErrorString(e);
        destroy_buffers(b);
        return TAPER_ENOMEM;
    }
    *out = b;
    return TAPER_OK;
}

// The arrays of a host plan as one image: bt | items | part_start | merge_start | merge | prefix_len |
// seg_start | ctx_len | seg_len | seg_page0, each piece 256-byte aligned.
struct ImagePiece {
    const void* src;
    size_t bytes, off;
};
size_t layout_image(const taper::HostPlan& h, ImagePiece (&pieces)[10]) {
    const ImagePiece init[10] = {
        {h.block_table.data(), h.block_table.size() * sizeof(int32_t), 0},
        {h.items.data(), h.items.size() * sizeof(taper_work_item), 0},
        {h.part_start.data(), h.part_start.size() * sizeof(int32_t), 0},
        {h.merge_start.data(), h.merge_start.size() * sizeof(int32_t), 0},
        {h.merge.data(), h.merge.size() * sizeof(taper_merge_entry), 0},
        {h.prefix_len.data(), h.prefix_len.size() * sizeof(int32_t), 0},
        {h.seg_start.data(), h.seg_start.size() * sizeof(int32_t), 0},
        {h.ctx_len.data(), h.ctx_len.size() * sizeof(int32_t), 0},
        {h.seg_len.data(), h.seg_len.size() * sizeof(int32_t), 0},
        {h.seg_page0.data(), h.seg_page0.size() * sizeof(int32_t), 0},
    };
    size_t total = 0;
    for (int i = 0; i < 10; ++i) {
        pieces[i] = init[i];
        pieces[i].off = total;
        total += align_up(std::max<size_t>(pieces[i].bytes, 16), 256);
    }
    return total;
}
void write_image(const ImagePiece (&pieces)[10], void* host_dst) {
    for (const ImagePiece& p : pieces)
        if (p.bytes) std::memcpy((char*)host_dst + p.off, p.src, p.bytes);
}
DeviceImage bind_image(const ImagePiece (&pieces)[10], void* dev_base) {
    char* d = (char*)dev_base;
    DeviceImage m;
    m.bt = (const int32_t*)(d + pieces[0].off);
    m.items = (const taper_work_item*)(d + pieces[1].off);
    m.part_start = (const int32_t*)(d + pieces[2].off);
    m.merge_start = (const int32_t*)(d + pieces[3].off);
    m.merge = (const taper_merge_entry*)(d + pieces[4].off);
    m.prefix_len = (const int32_t*)(d + pieces[5].off);
    m.seg_start = (const int32_t*)(d + pieces[6].off);
    m.ctx_len = (const int32_t*)(d + pieces[7].off);
    m.seg_len = (const int32_t*)(d + pieces[8].off);
    m.seg_page0 = (const int32_t*)(d + pieces[9].off);
    return m;
}

size_t partial_row_bytes(const taper_attn_config& cfg) {
    return (size_t)cfg.head_dim * (cfg.partial_format == TAPER_PARTIAL_F32 ? sizeof(float) : sizeof(uint16_t));
}
// Offsets of the three parts of a workspace of `rows` partial rows and `counters` counters; returns its size.
size_t layout_workspace(const taper_attn_config& cfg, int64_t rows, int64_t counters, size_t* ml_off, size_t* o_off) {
    *ml_off = align_up((size_t)counters * sizeof(int32_t), 256);
    *o_off = *ml_off + align_up((size_t)rows * sizeof(float4), 256);
    return *o_off + align_up((size_t)rows * partial_row_bytes(cfg), 256);
}
int64_t counters_needed(const taper_attn_config& cfg, int n_seqs) { return ((int64_t)n_seqs + 1) * cfg.n_kv_heads; }

void release_workspace(Workspace* w) {
    if (w->base) (void)hipFree(w->base);
    delete w;
}

// The context's current workspace if it holds `rows` partial rows and `counters` counters, else a new,
// larger one beside it (the old one stays for the plans bound to it).
int current_workspace(taper_ctx* ctx, int64_t rows, int64_t counters, bool headroom, Workspace** out) {
    Workspace* cur = ctx->workspaces.empty() ? nullptr : ctx->workspaces.back();
    if (cur && rows <= cur->rows && counters <= cur->counters) {
        *out = cur;
        return TAPER_OK;
    }
    if (cur) {  // never smaller than what it replaces
        rows = std::max(rows, cur->rows);
        counters = std::max(counters, cur->counters);
    }
    // growth: the only moment anything is freed (workspaces, the current one included, that no plan is bound to)
    bool synced = false;
    for (size_t i = 0; i < ctx->workspaces.size();) {
        Workspace* w = ctx->workspaces[i];
        if (w->refs > 0) {
            ++i;
            continue;
        }
        if (w->base && !synced) {  // launches of plans already freed may still be running
            HIP_TRY(hipDeviceSynchronize());
            synced = true;
        }
        release_workspace(w);
        ctx->workspaces.erase(ctx->workspaces.begin() + i);
    }
    Workspace* w = new (std::nothrow) Workspace();
    if (!w) return fail(TAPER_ENOMEM, "host allocation failed");
    w->rows = headroom ? rows + rows / 4 + 1024 : rows;  // head-room so that slowly growing steps do not reallocate
    w->counters = headroom ? counters + counters / 4 + 1024 : counters;
    w->bytes = layout_workspace(ctx->cfg, w->rows, w->counters, &w->ml_off, &w->o_off);
    w->id = ctx->next_workspace_id++;
    if (!ctx->host_only) {
        hipError_t e = hipSetDevice(ctx->cfg.device);
        if (e == hipSuccess) e = hipMalloc(&w->base, w->bytes);
        if (e == hipSuccess) e = hipMemset(w->base, 0, w->ml_off);  // counters start at zero
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e != hipSuccess) {
            g_last_error = std::string("workspace allocation: ") + hipGetErrorString(e);
            release_workspace(w);
            return TAPER_ENOMEM;
        }
    }
    ctx->workspaces.push_back(w);
    *out = w;
    return TAPER_OK;
}

// After a HIP error the counters of a workspace may have been left non-zero by a launch that did not
// finish; every later launch would then merge too early or never.  Clears them on `s`.
int recover_counters(taper_ctx* ctx, hipStream_t s) {
    if (!ctx->counters_suspect || ctx->host_only) return TAPER_OK;
    for (Workspace* w : ctx->workspaces)
        if (w->base) HIP_TRY(hipMemsetAsync(w->base, 0, w->ml_off, s));
    ctx->counters_suspect = false;
    return TAPER_OK;
}

taper::StepArgs make_args(const taper_ctx* ctx, const taper::HostPlan& h, const DeviceImage& img, void* ws_base,
                          size_t ml_off, size_t o_off, const void* q, const void* kv, void* out, float* lse) {
    taper::StepArgs a;
    std::memset(&a, 0, sizeof a);
    a.q = q;
    a.kv = kv;
    a.out = out;
    a.lse = lse;
    a.bt = img.bt;
    a.items = img.items;
    a.part_start = img.part_start;
    a.merge_start = img.merge_start;
    a.merge = img.merge;
    a.prefix_len = img.prefix_len;
    a.seg_start = img.seg_start;
    a.seg_len = img.seg_len;
    a.seg_page0 = img.seg_page0;
    a.ctx_len = img.ctx_len;
    a.counters = (int32_t*)ws_base;
    a.pool_ctr = a.counters + (int64_t)h.n_seqs * ctx->cfg.n_kv_heads;
    a.pool_first = h.part_start[h.n_parts_shared + h.n_parts_private];
    a.n_pool_items = h.n_pool_items;
    a.ws_ml = (float4*)((char*)ws_base + ml_off);
    a.ws_o = (char*)ws_base + o_off;
    a.bt_stride = h.bt_stride;
    a.n_seqs = h.n_seqs;
    a.n_merge = (int32_t)h.merge.size();
    a.n_q_heads = ctx->cfg.n_q_heads;
    a.n_kv_heads = ctx->cfg.n_kv_heads;
    a.gqa = ctx->cfg.n_q_heads / ctx->cfg.n_kv_heads;
    a.head_dim = ctx->cfg.head_dim;
    a.n_parts_shared = h.n_parts_shared;
    a.n_parts_private = h.n_parts_private;
    a.max_row_tiles_shared = h.max_row_tiles_shared;
    a.scale_log2e = ctx->cfg.scale * 1.4426950408889634f;
    a.partial_format = ctx->cfg.partial_format;
#ifdef TAPER_WG_TRACE
    a.trace = ctx->trace;
#endif
    return a;
}
taper::StepArgs make_args(const taper_ctx* ctx, const taper_plan* plan, const void* q, const void* kv, void* out,
                          float* lse) {
    return make_args(ctx, plan->host, plan->img, plan->ws->base, plan->ws->ml_off, plan->ws->o_off, q, kv, out, lse);
}

int check_step(const taper_ctx* ctx, const taper_plan* plan) {
    if (!ctx || !plan) return fail(TAPER_EINVAL, "null ctx or plan");
    if (plan->ctx != ctx) return fail(TAPER_EINVAL, "plan was built on another context");
    if (ctx->host_only || !plan->buf.dev || !plan->ws || !plan->ws->base)
        return fail(TAPER_EHIP, "host-only context: no device work possible");
    if (plan->host.n_partial_rows > plan->ws->rows || counters_needed(ctx->cfg, plan->host.n_seqs) > plan->ws->counters)
        return fail(TAPER_EINVAL, "workspace smaller than the plan needs");
    return TAPER_OK;
}

// A failed call may have left a launch unfinished: the next launch clears the counters first.
int hip_failed(taper_ctx* ctx, hipError_t e, const char* what) {
    ctx->counters_suspect = true;
    return fail_hip(e, what);
}

int enqueue_step(taper_ctx* ctx, const taper::StepArgs& a, hipStream_t s) {
    int st = recover_counters(ctx, s);
    if (st != TAPER_OK) return st;
    hipError_t e = taper::launch_decode(a, s);
    if (e != hipSuccess) return hip_failed(ctx, e, "decode kernel launch");
    return TAPER_OK;
}

}  // namespace

extern "C" {

const char* taper_strerror(int status) {
    switch (status) {
        case TAPER_OK: return "ok";
        case TAPER_EINVAL: return "invalid argument";
        case TAPER_EBLOCK: return "block-table entry outside the pool";
        case TAPER_EGROUP: return "malformed request grouping";
        case TAPER_ELEN: return "bad sequence length";
        case TAPER_EHIP: return "HIP runtime error";
        case TAPER_ENOMEM: return "out of memory";
        default: return "unknown status";
    }
}

const char* taper_last_error(void) { return g_last_error.c_str(); }

#ifdef TAPER_WG_TRACE
int taper_wg_trace_buffer(taper_ctx* ctx, long long* buf) {
    if (!ctx) return fail(TAPER_EINVAL, "null argument");
    ctx->trace = buf;
    return TAPER_OK;
}
#endif

int taper_append_slots(int n_seqs, const int32_t* block_table, int bt_row_stride, const int32_t* prefix_len,
                       const int32_t* seg_start, const int32_t* seg_len, int page_size, int64_t n_pool_pages,
                       int64_t* slots, int32_t* opens_page) {
    if (!block_table || !prefix_len || !seg_start || !seg_len || !slots) return fail(TAPER_EINVAL, "null argument");
    if (n_seqs < 0 || bt_row_stride < 1 || page_size < 1 || n_pool_pages < 1) return fail(TAPER_EINVAL, "bad argument");
    const int64_t P = page_size;
    for (int s = 0; s < n_seqs; ++s) {
        if (seg_start[s + 1] <= seg_start[s])
            return fail(TAPER_EINVAL, "sequence " + std::to_string(s) + " has no private segment to append to");
        if (prefix_len[s] < 0) return fail(TAPER_ELEN, "negative length");
        int64_t entry = (prefix_len[s] + P - 1) / P;
        for (int k = seg_start[s]; k < seg_start[s + 1] - 1; ++k) {
            if (seg_len[k] < 0) return fail(TAPER_ELEN, "negative length");
            entry += (seg_len[k] + P - 1) / P;
        }
        const int64_t last = seg_len[seg_start[s + 1] - 1];
        if (last < 0) return fail(TAPER_ELEN, "negative length");
        entry += last / P;
        if (entry >= bt_row_stride)
            return fail(TAPER_ELEN, "sequence " + std::to_string(s) + ": block-table row has no entry for the new token's page");
        const int64_t page = block_table[(size_t)s * bt_row_stride + entry];
        if (page < 0 || page >= n_pool_pages)
            return fail(TAPER_EBLOCK, "sequence " + std::to_string(s) + ": page of the new token is outside the pool");
        slots[s] = page * P + last % P;
        if (opens_page) opens_page[s] = last % P == 0;
    }
    return TAPER_OK;
}

int taper_kv_append(taper_ctx* ctx, int n_seqs, const void* k_new, const void* v_new, const int64_t* slots, void* kv_pages,
                    void* hip_stream) {
    if (!ctx || !k_new || !v_new || !slots || !kv_pages || n_seqs < 0) return fail(TAPER_EINVAL, "bad argument");
    if (ctx->host_only) return fail(TAPER_EHIP, "host-only context: no device work possible");
    HIP_TRY(taper::launch_kv_append(k_new, v_new, slots, kv_pages, n_seqs, ctx->cfg.n_kv_heads, ctx->cfg.head_dim,
                                    (hipStream_t)hip_stream));
    return TAPER_OK;
}

int64_t taper_branch_blocks(int64_t branch_local_tokens, int page_size) {
    if (branch_local_tokens <= 0 || page_size < 1) return 0;
    return (branch_local_tokens + page_size - 1) / page_size;
}

int taper_create(const taper_attn_config* cfg, taper_ctx** out_ctx) {
    if (!cfg || !out_ctx) return fail(TAPER_EINVAL, "null argument");
    std::string err;
    int st = taper::validate_config(*cfg, &err);
    if (st != TAPER_OK) return fail(st, err);
    taper_ctx* ctx = new (std::nothrow) taper_ctx();
    if (!ctx) return fail(TAPER_ENOMEM, "host allocation failed");
    ctx->cfg = *cfg;
    ctx->host_only = cfg->device < 0;
    if (!ctx->host_only) {
        int n = 0;
        hipError_t e = hipGetDeviceCount(&n);
        if (e != hipSuccess || cfg->device >= n) {
            delete ctx;
            return fail(TAPER_EHIP, "no such HIP device");
        }
        e = hipSetDevice(cfg->device);
        if (e != hipSuccess) {
            delete ctx;
            return fail_hip(e, "hipSetDevice");
        }
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, cfg->device) == hipSuccess && cus > 0)
            ctx->default_workgroups = 2 * cus;  // the decode kernel keeps two workgroups resident per compute unit
        // set-up of the entry point that allocates nothing (cfg->device is current)
        e = taper::static_scratch(cfg->device, &ctx->static_scratch);
        if (e == hipSuccess) e = hipHostMalloc(&ctx->static_staging, kStaticImageBytes, hipHostMallocDefault);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->static_uploaded, hipEventDisableTiming);
        if (e != hipSuccess) {  // the other entry points do not need it: the static one reports this
            ctx->static_error = std::string("static scratch set-up: ") + hipGetErrorString(e);
            ctx->static_scratch = nullptr;
            (void)hipGetLastError();
        }
    }
    *out_ctx = ctx;
    return TAPER_OK;
}

void taper_destroy(taper_ctx* ctx) {
    if (!ctx) return;
    if (!ctx->host_only) (void)hipDeviceSynchronize();
    for (Workspace* w : ctx->workspaces) release_workspace(w);
    for (PlanBuffers& b : ctx->free_buffers) destroy_buffers(b);
    if (ctx->static_uploaded) (void)hipEventDestroy(ctx->static_uploaded);
    if (ctx->static_staging) (void)hipHostFree(ctx->static_staging);
    delete ctx;
}

int taper_reserve(taper_ctx* ctx, int max_seqs, int64_t max_partial_rows) {
    if (!ctx) return fail(TAPER_EINVAL, "null argument");
    if (max_seqs < 0 || max_partial_rows < 0) return fail(TAPER_EINVAL, "negative size");
    Workspace* w = nullptr;
    return current_workspace(ctx, max_partial_rows, counters_needed(ctx->cfg, max_seqs), false, &w);
}

int taper_plan_build(taper_ctx* ctx, int n_seqs, const int32_t* block_table, int bt_row_stride,
                     const int32_t* branch_group, const int32_t* prefix_len, const int32_t* suffix_len,
                     int64_t n_pool_pages, const taper_plan_options* opts, void* hip_stream, taper_plan** out_plan) {
    if (!suffix_len || n_seqs < 1) return fail(TAPER_EINVAL, "null argument");
    std::vector<int32_t> seg_start((size_t)n_seqs + 1);
    for (int s = 0; s <= n_seqs; ++s) seg_start[s] = s;  // one private segment per sequence
    return taper_plan_build_segments(ctx, n_seqs, block_table, bt_row_stride, branch_group, prefix_len, seg_start.data(),
                                     suffix_len, n_pool_pages, opts, hip_stream, out_plan);
}

int taper_plan_build_segments(taper_ctx* ctx, int n_seqs, const int32_t* block_table, int bt_row_stride,
                              const int32_t* branch_group, const int32_t* prefix_len, const int32_t* seg_start,
                              const int32_t* seg_len, int64_t n_pool_pages, const taper_plan_options* opts,
                              void* hip_stream, taper_plan** out_plan) {
    if (!ctx || !out_plan) return fail(TAPER_EINVAL, "null argument");
    taper_plan* plan = new (std::nothrow) taper_plan();
    if (!plan) return fail(TAPER_ENOMEM, "host allocation failed");
    plan->ctx = ctx;
    std::string err;
    taper_plan_options o;
    std::memset(&o, 0, sizeof o);
    o.share_prefix = 1;
    if (opts) o = *opts;
    if (o.small_step_grid == 0) o.small_step_grid = o.target_workgroups <= 0 ? 1 : -1;  // the rule is for grids left to the library
    if (o.target_workgroups <= 0) o.target_workgroups = ctx->default_workgroups;  // (0 on a host-only context: 512)
    int st = taper::build_host_plan_segments(ctx->cfg, n_seqs, block_table, bt_row_stride, branch_group, prefix_len,
                                             seg_start, seg_len, n_pool_pages, &o, &plan->host, &err);
    if (st != TAPER_OK) {
        delete plan;
        return fail(st, err);
    }
    const taper::HostPlan& h = plan->host;
    if (ctx->host_only) {  // bookkeeping only: which workspace the plan would be bound to
        st = current_workspace(ctx, h.n_partial_rows, counters_needed(ctx->cfg, h.n_seqs), true, &plan->ws);
        if (st != TAPER_OK) {
            delete plan;
            return st;
        }
        plan->ws->refs++;
        *out_plan = plan;
        return TAPER_OK;
    }
    ImagePiece pieces[10];
    const size_t total = layout_image(h, pieces);
    hipError_t e = hipSetDevice(ctx->cfg.device);
    if (e != hipSuccess) {
        delete plan;
        return fail_hip(e, "hipSetDevice");
    }
    st = acquire_buffers(ctx, total, &plan->buf);
    if (st != TAPER_OK) {
        delete plan;
        return st;
    }
    write_image(pieces, plan->buf.staging);
    hipStream_t s = (hipStream_t)hip_stream;
    e = hipMemcpyAsync(plan->buf.dev, plan->buf.staging, total, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipEventRecord(plan->buf.uploaded, s);
    if (e != hipSuccess) {
        std::string msg = std::string("plan upload: ") + hipGetErrorString(e);
        taper_plan_free(plan);
        return fail(TAPER_EHIP, msg);
    }
    plan->img = bind_image(pieces, plan->buf.dev);
    st = current_workspace(ctx, h.n_partial_rows, counters_needed(ctx->cfg, h.n_seqs), true, &plan->ws);
    if (st == TAPER_OK) {
        plan->ws->refs++;
        st = recover_counters(ctx, s);
    }
    if (st != TAPER_OK) {
        std::string keep = g_last_error;
        taper_plan_free(plan);
        return fail(st, keep);
    }
    *out_plan = plan;
    return TAPER_OK;
}

void taper_plan_free(taper_plan* plan) {
    if (!plan) return;
    // Buffers go back to the context.  Work already enqueued that reads them stays
    // valid: a later plan's upload into the same memory is ordered behind it on the
    // stream (one stream per context).
    if (plan->buf.dev) plan->ctx->free_buffers.push_back(plan->buf);
    // The workspace stays (launches of this plan may still be running); one that has been superseded
    // and has no plan left is released at the context's next growth or destruction.
    if (plan->ws) plan->ws->refs--;
    delete plan;
}

int taper_plan_export(const taper_plan* plan, taper_plan_view* v) {
    if (!plan || !v) return fail(TAPER_EINVAL, "null argument");
    const taper::HostPlan& h = plan->host;
    std::memset(v, 0, sizeof *v);
    v->n_seqs = h.n_seqs;
    v->n_groups = h.n_groups;
    v->ctx_len = h.ctx_len.data();
    v->n_prefix_pages = h.n_prefix_pages.data();
    v->n_suffix_pages = h.n_suffix_pages.data();
    v->group_start = h.group_start.data();
    v->seg_start = h.seg_start.data();
    v->seg_len = h.seg_len.data();
    v->seg_page0 = h.seg_page0.data();
    v->n_items = (int32_t)h.items.size();
    v->items = h.items.data();
    v->n_pool_items = h.n_pool_items;
    v->n_parts_shared = h.n_parts_shared;
    v->n_parts_private = h.n_parts_private;
    v->part_start = h.part_start.data();
    v->merge_start = h.merge_start.data();
    v->merge = h.merge.data();
    v->n_partial_rows = h.n_partial_rows;
    v->tokens_unique = h.tokens_unique;
    v->tokens_logical = h.tokens_logical;
    v->workspace_id = plan->ws ? plan->ws->id : 0;
    v->workspace_rows = plan->ws ? plan->ws->rows : 0;
    return TAPER_OK;
}

int taper_plan_resolve_slots_host(const taper_plan* plan, int64_t* slots, int64_t stride) {
    if (!plan || !slots || stride < 0) return fail(TAPER_EINVAL, "bad argument");
    taper::resolve_slots_host(plan->host, plan->ctx->cfg.page_size, slots, stride);
    return TAPER_OK;
}

int taper_plan_resolve_slots(taper_ctx* ctx, const taper_plan* plan, int64_t* slots, int64_t stride,
                             void* hip_stream) {
    int st = check_step(ctx, plan);
    if (st != TAPER_OK) return st;
    if (!slots || stride < 0) return fail(TAPER_EINVAL, "bad argument");
    taper::StepArgs a = make_args(ctx, plan, nullptr, nullptr, nullptr, nullptr);
    HIP_TRY(taper::launch_resolve_slots(a, slots, stride, (hipStream_t)hip_stream));
    return TAPER_OK;
}

int taper_decode_step_attention(taper_ctx* ctx, const taper_plan* plan, const void* q, const void* kv_pages,
                                void* out, float* lse, void* hip_stream) {
    int st = check_step(ctx, plan);
    if (st != TAPER_OK) return st;
    if (!q || !kv_pages || !out) return fail(TAPER_EINVAL, "null tensor pointer");
    return enqueue_step(ctx, make_args(ctx, plan, q, kv_pages, out, lse), (hipStream_t)hip_stream);
}

int taper_decode_step_attention_simple(taper_ctx* ctx, int n_seqs, const void* q, const void* kv_pages,
                                       int64_t n_pool_pages, const int32_t* block_table, int bt_row_stride,
                                       const int32_t* branch_group, const int32_t* prefix_len,
                                       const int32_t* suffix_len, void* out, void* hip_stream) {
    taper_plan* plan = nullptr;
    int st = taper_plan_build(ctx, n_seqs, block_table, bt_row_stride, branch_group, prefix_len, suffix_len,
                              n_pool_pages, nullptr, hip_stream, &plan);
    if (st != TAPER_OK) return st;
    st = taper_decode_step_attention(ctx, plan, q, kv_pages, out, nullptr, hip_stream);
    if (st == TAPER_OK) {
        hipError_t e = hipStreamSynchronize((hipStream_t)hip_stream);
        if (e != hipSuccess) st = hip_failed(ctx, e, "hipStreamSynchronize");
    }
    taper_plan_free(plan);
    return st;
}

int taper_decode_step_attention_static(taper_ctx* ctx, int n_seqs, const void* q, const void* kv_pages,
                                       int64_t n_pool_pages, const int32_t* block_table, int bt_row_stride,
                                       const int32_t* branch_group, const int32_t* prefix_len,
                                       const int32_t* suffix_len, void* out, void* hip_stream) {
    if (!ctx || !q || !kv_pages || !out || !suffix_len || n_seqs < 1) return fail(TAPER_EINVAL, "null argument");
    if (ctx->host_only) return fail(TAPER_EHIP, "host-only context: no device work possible");
    if (!ctx->static_scratch) return fail(TAPER_EHIP, ctx->static_error.empty() ? "static scratch unavailable" : ctx->static_error);
    // the plan, on the host (host memory only)
    taper::HostPlan h;
    std::string err;
    taper_plan_options o;
    std::memset(&o, 0, sizeof o);
    o.share_prefix = 1;
    o.target_workgroups = ctx->default_workgroups;
    o.small_step_grid = 1;
    int st = taper::build_host_plan(ctx->cfg, n_seqs, block_table, bt_row_stride, branch_group, prefix_len, suffix_len,
                                    n_pool_pages, &o, &h, &err);
    if (st != TAPER_OK) return fail(st, err);
    // layout inside the array: plan image | counters | statistics | partial rows
    ImagePiece pieces[10];
    const size_t image = layout_image(h, pieces);
    size_t ml_off = 0, o_off = 0;
    const int64_t counters = counters_needed(ctx->cfg, h.n_seqs);
    const size_t ws_bytes = layout_workspace(ctx->cfg, h.n_partial_rows, counters, &ml_off, &o_off);
    if (image > kStaticImageBytes || image + ws_bytes > taper::kStaticScratchBytes)
        return fail(TAPER_EINVAL, "step too large for the static scratch array: plan image " + std::to_string(image) +
                                      " bytes (limit " + std::to_string(kStaticImageBytes) + "), image + workspace " +
                                      std::to_string(image + ws_bytes) + " bytes (limit " +
                                      std::to_string(taper::kStaticScratchBytes) + ")");
    hipStream_t s = (hipStream_t)hip_stream;
    HIP_TRY(hipSetDevice(ctx->cfg.device));
    HIP_TRY(hipEventSynchronize(ctx->static_uploaded));  // the previous call's upload has read the pinned image
    write_image(pieces, ctx->static_staging);
    char* base = (char*)ctx->static_scratch;
    HIP_TRY(hipMemcpyAsync(base, ctx->static_staging, image, hipMemcpyHostToDevice, s));
    HIP_TRY(hipEventRecord(ctx->static_uploaded, s));
    // the array keeps the last call's contents: what must start at zero is cleared (the counters)
    char* ws = base + image;
    HIP_TRY(taper::launch_zero_words((int32_t*)ws, counters, s));
    const taper::StepArgs a = make_args(ctx, h, bind_image(pieces, base), ws, ml_off, o_off, q, kv_pages, out, nullptr);
    HIP_TRY(taper::launch_decode(a, s));
    return TAPER_OK;
}

int taper_step_latency_probe(taper_ctx* ctx, const taper_plan* plan, int n_layers, const void* const* q_per_layer,
                             const void* const* kv_per_layer, void* const* out_per_layer, int warmup, int iters,
                             void* hip_stream, taper_probe_result* res) {
    int st = check_step(ctx, plan);
    if (st != TAPER_OK) return st;
    if (n_layers < 1 || iters < 1 || warmup < 0 || !q_per_layer || !kv_per_layer || !out_per_layer || !res)
        return fail(TAPER_EINVAL, "bad probe argument");
    for (int l = 0; l < n_layers; ++l)
        if (!q_per_layer[l] || !kv_per_layer[l] || !out_per_layer[l]) return fail(TAPER_EINVAL, "null layer pointer");
    hipStream_t s = (hipStream_t)hip_stream;
    std::vector<hipEvent_t> ev(2 * (size_t)iters, nullptr);
    for (auto& e : ev) HIP_TRY(hipEventCreate(&e));
    int rc = TAPER_OK;
    for (int i = 0; i < warmup + iters && rc == TAPER_OK; ++i) {
        const int k = i - warmup;
        if (k >= 0 && hipEventRecord(ev[2 * k], s) != hipSuccess) rc = fail(TAPER_EHIP, "hipEventRecord");
        for (int l = 0; l < n_layers && rc == TAPER_OK; ++l)
            rc = enqueue_step(ctx, make_args(ctx, plan, q_per_layer[l], kv_per_layer[l], out_per_layer[l], nullptr), s);
        if (k >= 0 && rc == TAPER_OK && hipEventRecord(ev[2 * k + 1], s) != hipSuccess)
            rc = fail(TAPER_EHIP, "hipEventRecord");
    }
    hipError_t es = hipStreamSynchronize(s);
    if (rc == TAPER_OK && es != hipSuccess) rc = hip_failed(ctx, es, "hipStreamSynchronize");
    std::vector<double> us;
    if (rc == TAPER_OK) {
        for (int k = 0; k < iters; ++k) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, ev[2 * k], ev[2 * k + 1]) != hipSuccess) {
                rc = fail(TAPER_EHIP, "hipEventElapsedTime");
                break;
            }
            us.push_back(ms * 1000.0);
        }
    }
    for (auto& e : ev) (void)hipEventDestroy(e);
    if (rc != TAPER_OK) return rc;
    std::sort(us.begin(), us.end());
    double sum = 0;
    for (double u : us) sum += u;
    std::memset(res, 0, sizeof *res);
    res->us_min = us.front();
    res->us_median = (us.size() % 2) ? us[us.size() / 2] : 0.5 * (us[us.size() / 2 - 1] + us[us.size() / 2]);
    res->us_mean = sum / us.size();
    res->n_tokens = plan->host.n_seqs;
    res->n_layers = n_layers;
    res->l_context = plan->host.tokens_logical;
    const int64_t bpt = 2LL * ctx->cfg.n_kv_heads * ctx->cfg.head_dim * 2;
    res->kv_bytes_unique = plan->host.tokens_unique * bpt;
    res->kv_bytes_logical = plan->host.tokens_logical * bpt;
    res->gbps_unique = (double)res->kv_bytes_unique * n_layers / (res->us_median * 1e-6) / 1e9;
    res->gbps_logical = (double)res->kv_bytes_logical * n_layers / (res->us_median * 1e-6) / 1e9;
    return TAPER_OK;
}

int taper_kernel_times(taper_ctx* ctx, const taper_plan* plan, const void* q, const void* kv_pages, void* out,
                       int warmup, int iters, void* hip_stream, double us[2]) {
    if (!q || !kv_pages || !out) return fail(TAPER_EINVAL, "bad argument");
    return taper_kernel_times_layers(ctx, plan, 1, &q, &kv_pages, &out, warmup, iters, hip_stream, us);
}

int taper_kernel_times_layers(taper_ctx* ctx, const taper_plan* plan, int n_layers, const void* const* q_per_layer,
                              const void* const* kv_per_layer, void* const* out_per_layer, int warmup, int iters,
                              void* hip_stream, double us[2]) {
    int st = check_step(ctx, plan);
    if (st != TAPER_OK) return st;
    if (!q_per_layer || !kv_per_layer || !out_per_layer || !us || n_layers < 1 || iters < 1 || warmup < 0)
        return fail(TAPER_EINVAL, "bad argument");
    for (int l = 0; l < n_layers; ++l)
        if (!q_per_layer[l] || !kv_per_layer[l] || !out_per_layer[l]) return fail(TAPER_EINVAL, "null layer pointer");
    hipStream_t s = (hipStream_t)hip_stream;
    std::vector<hipEvent_t> ev(2 * (size_t)iters, nullptr);
    for (auto& e : ev) HIP_TRY(hipEventCreate(&e));
    int rc = TAPER_OK;
    for (int i = 0; i < warmup + iters && rc == TAPER_OK; ++i) {
        const int k = i - warmup, l = i % n_layers;
        const taper::StepArgs a = make_args(ctx, plan, q_per_layer[l], kv_per_layer[l], out_per_layer[l], nullptr);
        hipError_t e = hipSuccess;
        if (k >= 0) e = hipEventRecord(ev[2 * k], s);
        if (e == hipSuccess) e = taper::launch_decode(a, s);
        if (k >= 0 && e == hipSuccess) e = hipEventRecord(ev[2 * k + 1], s);
        if (e != hipSuccess) rc = hip_failed(ctx, e, "kernel timing enqueue");
    }
    hipError_t es = hipStreamSynchronize(s);
    if (rc == TAPER_OK && es != hipSuccess) rc = hip_failed(ctx, es, "hipStreamSynchronize");
    double sum = 0, mn = 1e300;
    if (rc == TAPER_OK) {
        for (int k = 0; k < iters; ++k) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, ev[2 * k], ev[2 * k + 1]) != hipSuccess) {
                rc = fail(TAPER_EHIP, "hipEventElapsedTime");
                break;
            }
            sum += ms * 1000.0;
            mn = std::min(mn, ms * 1000.0);
        }
    }
    for (auto& e : ev) (void)hipEventDestroy(e);
    if (rc != TAPER_OK) return rc;
    us[0] = sum / iters;
    us[1] = mn;
    return TAPER_OK;
}

int taper_stream_read_probe(taper_ctx* ctx, const void* buf, int64_t buf_bytes, int64_t pass_bytes, int n_workgroups,
                            int warmup, int iters, void* hip_stream, double us[2]) {
    if (!ctx || !buf || !us) return fail(TAPER_EINVAL, "null argument");
    if (ctx->host_only) return fail(TAPER_EHIP, "context was created without a device");
    if (n_workgroups < 1 || n_workgroups > 65536 || iters < 1 || warmup < 0) return fail(TAPER_EINVAL, "bad argument");
    const int64_t unit = (int64_t)n_workgroups * 4096;
    if (pass_bytes < unit || pass_bytes % unit != 0 || buf_bytes < pass_bytes)
        return fail(TAPER_EINVAL, "pass_bytes must be a positive multiple of n_workgroups * 4096 and fit the buffer");
    if (((uintptr_t)buf & 15) != 0) return fail(TAPER_EINVAL, "buffer must be 16-byte aligned");
    HIP_TRY(hipSetDevice(ctx->cfg.device));
    hipStream_t s = (hipStream_t)hip_stream;
    const int64_t n_regions = buf_bytes / pass_bytes, pieces_per_wg = pass_bytes / unit;
    unsigned* sink = nullptr;
    HIP_TRY(hipMalloc((void**)&sink, 256));
    std::vector<hipEvent_t> ev(2 * (size_t)iters, nullptr);
    int rc = TAPER_OK;
    for (auto& e : ev)
        if (rc == TAPER_OK && hipEventCreate(&e) != hipSuccess) rc = fail(TAPER_EHIP, "hipEventCreate");
    for (int i = 0; i < warmup + iters && rc == TAPER_OK; ++i) {
        const int k = i - warmup;
        const char* base = (const char*)buf + (i % n_regions) * pass_bytes;
        hipError_t e = hipSuccess;
        if (k >= 0) e = hipEventRecord(ev[2 * k], s);
        if (e == hipSuccess) e = taper::launch_stream_read(base, pieces_per_wg, n_workgroups, sink, s);
        if (k >= 0 && e == hipSuccess) e = hipEventRecord(ev[2 * k + 1], s);
        if (e != hipSuccess) rc = fail_hip(e, "read probe enqueue");
    }
    hipError_t es = hipStreamSynchronize(s);
    if (rc == TAPER_OK && es != hipSuccess) rc = fail_hip(es, "hipStreamSynchronize");
    double sum = 0, mn = 1e300;
    if (rc == TAPER_OK) {
        for (int k = 0; k < iters; ++k) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, ev[2 * k], ev[2 * k + 1]) != hipSuccess) {
                rc = fail(TAPER_EHIP, "hipEventElapsedTime");
                break;
            }
            sum += ms * 1000.0;
            mn = std::min(mn, ms * 1000.0);
        }
    }
    for (auto& e : ev)
        if (e) (void)hipEventDestroy(e);
    (void)hipFree(sink);
    if (rc != TAPER_OK) return rc;
    us[0] = sum / iters;
    us[1] = mn;
    return TAPER_OK;
}

}  // extern "C"
