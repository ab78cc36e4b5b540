// Context, workspace and the two GPU entry points of libspin (spin_verify_attn, spin_accept).
// Host code only; the kernels are in spin_attn.hip and spin_accept.hip.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <string>

#include "spin_device.h"

namespace {

constexpr int kStages = 8;   // pinned staging buffers (and device copies of the tables) cycled between calls
// A device copy of the tables may be overwritten only after the kernels that read it have finished.  An event
// record between two kernels holds the second one up for several microseconds, so the library does not record
// one behind every attention call: every kMarkEvery-th call leaves a marker on its stream, and an upload waits
// for the first marker that lies behind the last reader of its slot (recording one on the spot if there is none).
constexpr int kMarks = 4;
constexpr int kMarkEvery = 4;

inline size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

}  // namespace

// The tables of the most recent attention call, as staged for the GPU, and what they were made for:
// a call with the same request table, decomposition and geometry (the other layers of the same
// step) launches from them again without re-planning or re-uploading.
struct StagedPlan {
    bool valid = false;
    int slot = -1;                  // ring slot holding the tables; kept out of the rotation while valid
    bool in_place = false;          // small tables: passed to the kernels in their arguments, not copied to the device
    size_t bytes = 0;               // size of the staged tables
    // key
    int32_t page_size = 0, n_kv_heads = 0, head_dim = 0, n_pages = 0, n_q_heads = 0, n_sub = -1;
    int32_t waves[3] = {0, 0, 0};
    bool has_subs = false, has_tree = false;
    std::vector<int32_t> prefix, draft, q_off, pt_off, pages;
    std::vector<spin_subreq> subs;
    std::vector<uint64_t> tree;
    // launch data
    size_t off_pieces = 0, off_waves[3] = {0, 0, 0}, off_first[3] = {0, 0, 0}, off_queues = 0, off_ppos = 0, off_strips = 0, off_qoff = 0,
           off_tasks = 0, off_pt = 0, off_tree = 0;
    int32_t n_waves_launch[3] = {0, 0, 0}, n_queued[3] = {0, 0, 0}, class_piece_begin[3] = {0, 0, 0};
    int32_t n_tasks = 0, max_pairs = 0;
};

struct spin_ctx {
    int device = 0;
    std::string err;
    int waves_override = 0;           // 0: as many wavefronts as the device holds
    int resident[2][3] = {{0, 0, 0}, {0, 0, 0}};   // resident wavefronts per head dim (64, 128) and tile class
    // reserved capacities and what the last refused call needed
    int64_t cap_req = 0, cap_rows = 0, cap_pages = 0, cap_items = 0, cap_slots = 0;
    int64_t need_req = 0, need_rows = 0, need_pages = 0, need_items = 0, need_slots = 0;
    // device workspace
    char* d_blob[kStages] = {};   // tables of a call (items, orders, offsets, page table)
    size_t blob_bytes = 0;
    hipStream_t copy_stream = nullptr;   // table uploads run here, beside the previous call's kernels
    int64_t gen = 0;                       // attention calls launched from a device copy of their tables, so far
    int64_t slot_gen[kStages];             // the latest of them that read d_blob[s] (-1: none) ...
    hipStream_t slot_stream[kStages] = {}; // ... and the stream its kernels run on
    hipEvent_t ev_mark[kMarks] = {};       // markers: all calls up to mark_gen[k] launched on mark_stream[k] have finished
    int64_t mark_gen[kMarks];
    hipStream_t mark_stream[kMarks] = {};
    int64_t n_marks = 0;                   // markers recorded so far (the next one goes to n_marks % kMarks)
    int64_t marked_gen = -1;               // the latest call behind which a marker was recorded
    uint16_t* d_part_o = nullptr;
    float* d_part_ml = nullptr;
    float* d_row_max = nullptr;    // acceptance row statistics
    double* d_row_sum = nullptr;
    int32_t* d_row_arg = nullptr;
    int32_t* d_arrive = nullptr;   // per-request arrival counters of the acceptance kernels: zero between launches
    double* d_draw_runs = nullptr; // run masses and last ids of the next-token draw
    int32_t* d_draw_last = nullptr;
    // pinned staging ring
    char* h_stage[kStages] = {};
    hipEvent_t ev[kStages] = {};
    bool ev_pending[kStages] = {};
    int stage = 0;
    std::vector<int64_t> slot_host;   // destination slots of spin_append_kv when they travel in the kernel's arguments
    StagedPlan staged;
    bool reuse_plans = true;
    spin::Plan plan;
    std::vector<int32_t> row_off_host;
    // kernel timing (spin_profile_begin / _end): three events per timed call
    std::vector<hipEvent_t> prof_attn, prof_accept;        // four per timed call: start and end of its two kernels
    std::vector<uint8_t> prof_attn_second, prof_accept_second;   // the call launched a second kernel
    int prof_attn_used = 0, prof_accept_used = 0;
    int64_t prof_attn_seen = 0, prof_accept_seen = 0;   // calls seen while armed
    int32_t prof_every = 1;                              // every n-th of them is timed
    bool prof_on = false;
};

namespace {

int fail(spin_ctx* ctx, int code, const std::string& text) {
    if (ctx) ctx->err = text;
    return code;
}

int fail_hip(spin_ctx* ctx, hipError_t e, const char* where) {
    if (ctx) ctx->err = std::string(where) + ": " + hipGetErrorString(e);
    return SPIN_EHIP;
}

void free_profile(spin_ctx* c) {
    for (hipEvent_t e : c->prof_attn) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->prof_accept) (void)hipEventDestroy(e);
    c->prof_attn.clear();
    c->prof_accept.clear();
    c->prof_attn_used = c->prof_accept_used = 0;
    c->prof_on = false;
}

// Events of the next timed call, or null when the context is not armed / has run out of slots.
hipEvent_t* prof_slot(spin_ctx* c, std::vector<hipEvent_t>& pool, int& used, int64_t& seen) {
    if (!c->prof_on || (seen++ % c->prof_every) != 0 || (size_t)(used + 1) * 4 > pool.size()) return nullptr;
    hipEvent_t* p = pool.data() + (size_t)used * 4;
    ++used;
    return p;
}

void free_workspace(spin_ctx* c) {
    c->staged.valid = false;
    for (int s = 0; s < kStages; ++s)
        if (c->d_blob[s]) (void)hipFree(c->d_blob[s]);
    if (c->d_part_o) (void)hipFree(c->d_part_o);
    if (c->d_part_ml) (void)hipFree(c->d_part_ml);
    if (c->d_row_max) (void)hipFree(c->d_row_max);
    if (c->d_row_sum) (void)hipFree(c->d_row_sum);
    if (c->d_row_arg) (void)hipFree(c->d_row_arg);
    if (c->d_arrive) (void)hipFree(c->d_arrive);
    if (c->d_draw_runs) (void)hipFree(c->d_draw_runs);
    if (c->d_draw_last) (void)hipFree(c->d_draw_last);
    for (int s = 0; s < kStages; ++s)
        if (c->h_stage[s]) (void)hipHostFree(c->h_stage[s]);
    c->d_part_o = nullptr;
    c->d_part_ml = c->d_row_max = nullptr;
    c->d_row_sum = nullptr;
    c->d_row_arg = nullptr;
    c->d_arrive = nullptr;
    c->d_draw_runs = nullptr;
    c->d_draw_last = nullptr;
    for (int s = 0; s < kStages; ++s) c->h_stage[s] = c->d_blob[s] = nullptr;
}

constexpr size_t kInPlaceBytes = spin::kInlineTableBytes;   // tables up to this size travel in the kernel arguments
constexpr int kMaxWaves = 16384;   // wavefronts per launch the staging buffers are sized for

// pieces | per-class wavefront ranges | (strip, head) piece ranges | strip ranges | row offsets | tasks | page table
size_t blob_size(int64_t req, int64_t rows, int64_t pages, int64_t items) {
    // every share holds at least one piece, so there are at most `items` share boundaries in all
    return align16(items * sizeof(spin::Piece)) + align16(items * 4) + align16(items * 40) + 6 * 32 + 2 * align16(items * 8) +
           2 * align16((req + 1) * 4) + align16(pages * 4) + align16(rows * 16) + 128;
}

// Leave a marker on `stream` behind everything launched so far.
hipError_t record_marker(spin_ctx* c, hipStream_t stream, hipEvent_t* out) {
    const int k = (int)(c->n_marks % kMarks);
    hipError_t e = hipEventRecord(c->ev_mark[k], stream);
    if (e != hipSuccess) return e;
    c->mark_gen[k] = c->gen - 1;
    c->mark_stream[k] = stream;
    c->marked_gen = c->gen - 1;
    ++c->n_marks;
    if (out) *out = c->ev_mark[k];
    return hipSuccess;
}

// Make the upload stream wait until the kernels that read d_blob[slot] have finished.
hipError_t wait_for_readers(spin_ctx* c, int slot) {
    const int64_t g0 = c->slot_gen[slot];
    if (g0 < 0) return hipSuccess;
    hipEvent_t m = nullptr;
    int64_t best = INT64_MAX;
    for (int k = 0; k < kMarks; ++k)   // the earliest marker behind that call, on its stream
        if (c->mark_gen[k] >= g0 && c->mark_gen[k] < best && c->mark_stream[k] == c->slot_stream[slot]) {
            best = c->mark_gen[k];
            m = c->ev_mark[k];
        }
    if (!m) {
        hipError_t e = record_marker(c, c->slot_stream[slot], &m);
        if (e != hipSuccess) {
            // (the stream is gone: whatever ran on it is waited for the plain way)
            (void)hipGetLastError();
            c->slot_gen[slot] = -1;
            return hipDeviceSynchronize();
        }
    }
    c->slot_gen[slot] = -1;
    return hipStreamWaitEvent(c->copy_stream, m, 0);
}

// Next pinned staging buffer; waits until the copy that last used it has left the host.
int next_stage(spin_ctx* c, char** out) {
    c->stage = (c->stage + 1) % kStages;
    if (c->staged.valid && c->stage == c->staged.slot) c->stage = (c->stage + 1) % kStages;   // holds a reusable plan
    const int s = c->stage;
    if (c->ev_pending[s]) {
        hipError_t e = hipEventSynchronize(c->ev[s]);
        if (e != hipSuccess) return fail_hip(c, e, "hipEventSynchronize");
        c->ev_pending[s] = false;
    }
    *out = c->h_stage[s];
    return SPIN_OK;
}

}  // namespace

extern "C" {

int spin_create(spin_ctx** out, int device_id) {
    if (!out) return SPIN_EINVAL;
    *out = nullptr;
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess || device_id < 0 || device_id >= n) return SPIN_EHIP;
    e = hipSetDevice(device_id);
    if (e != hipSuccess) return SPIN_EHIP;
    spin_ctx* c = new spin_ctx();
    c->device = device_id;
    bool ok = hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking) == hipSuccess;
    for (int s = 0; s < kStages; ++s) c->slot_gen[s] = -1;
    for (int k = 0; k < kMarks; ++k) c->mark_gen[k] = -1;
    for (int s = 0; s < kStages && ok; ++s) ok = hipEventCreateWithFlags(&c->ev[s], hipEventDisableTiming) == hipSuccess;
    for (int k = 0; k < kMarks && ok; ++k) ok = hipEventCreateWithFlags(&c->ev_mark[k], hipEventDisableTiming) == hipSuccess;
    ok = ok && spin::resolve_static_scratch() == hipSuccess;
    if (!ok) {
        spin_destroy(c);
        return SPIN_EHIP;
    }
    *out = c;
    return SPIN_OK;
}

void spin_destroy(spin_ctx* ctx) {
    if (!ctx) return;
    (void)hipSetDevice(ctx->device);
    (void)hipDeviceSynchronize();
    free_workspace(ctx);
    free_profile(ctx);
    for (int s = 0; s < kStages; ++s)
        if (ctx->ev[s]) (void)hipEventDestroy(ctx->ev[s]);
    for (int k = 0; k < kMarks; ++k)
        if (ctx->ev_mark[k]) (void)hipEventDestroy(ctx->ev_mark[k]);
    if (ctx->copy_stream) (void)hipStreamDestroy(ctx->copy_stream);
    delete ctx;
}

int spin_last_error(spin_ctx* ctx, char* buf, size_t n) {
    if (!ctx || !buf || n == 0) return SPIN_EINVAL;
    snprintf(buf, n, "%s", ctx->err.c_str());
    return SPIN_OK;
}

int spin_set_waves(spin_ctx* ctx, int32_t n_waves) {
    if (!ctx) return SPIN_EINVAL;
    if (n_waves < 0 || n_waves > kMaxWaves) return fail(ctx, SPIN_EINVAL, "n_waves must be 0 (automatic) or 1..16384");
    ctx->waves_override = n_waves;
    return SPIN_OK;
}

int spin_required(spin_ctx* ctx, int64_t* req, int64_t* rows, int64_t* pages, int64_t* items, int64_t* part_slots) {
    if (!ctx) return SPIN_EINVAL;
    if (req) *req = ctx->need_req;
    if (rows) *rows = ctx->need_rows;
    if (pages) *pages = ctx->need_pages;
    if (items) *items = ctx->need_items;
    if (part_slots) *part_slots = ctx->need_slots;
    return SPIN_OK;
}

int spin_reserve(spin_ctx* ctx, int64_t max_req, int64_t max_rows, int64_t max_pages, int64_t max_items,
                 int64_t max_part_slots) {
    if (!ctx) return SPIN_EINVAL;
    if (max_req < 0 || max_rows < 0 || max_pages < 0 || max_items < 0 || max_part_slots < 0)
        return fail(ctx, SPIN_EINVAL, "negative size");
    max_req = std::max(max_req, ctx->cap_req);
    max_rows = std::max(max_rows, ctx->cap_rows);
    max_pages = std::max(max_pages, ctx->cap_pages);
    max_items = std::max(max_items, ctx->cap_items);
    max_part_slots = std::max(max_part_slots, ctx->cap_slots);
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return fail_hip(ctx, e, "hipSetDevice");
    e = hipDeviceSynchronize();
    if (e != hipSuccess) return fail_hip(ctx, e, "hipDeviceSynchronize");
    free_workspace(ctx);
    for (int s = 0; s < kStages; ++s) {   // (the device has just been synchronised: nothing reads the old copies)
        ctx->ev_pending[s] = false;
        ctx->slot_gen[s] = -1;
    }
    ctx->cap_req = ctx->cap_rows = ctx->cap_pages = ctx->cap_items = ctx->cap_slots = 0;
    const size_t blob = blob_size(max_req, max_rows, max_pages, max_items);
    const int64_t stat_rows = 2 * max_rows + max_req + 1;
#define SPIN_TRY(call)                                   \
    do {                                                 \
        e = (call);                                      \
        if (e != hipSuccess) {                           \
            free_workspace(ctx);                         \
            return fail_hip(ctx, e, #call);              \
        }                                                \
    } while (0)
    for (int s = 0; s < kStages; ++s) SPIN_TRY(hipMalloc((void**)&ctx->d_blob[s], blob));
    SPIN_TRY(hipMalloc((void**)&ctx->d_part_o, std::max<size_t>(16, (size_t)max_part_slots * spin::kPartRow * 2)));
    SPIN_TRY(hipMalloc((void**)&ctx->d_part_ml, std::max<size_t>(16, (size_t)max_part_slots * 2 * 4)));
    SPIN_TRY(hipMalloc((void**)&ctx->d_row_max, (size_t)stat_rows * 4));
    SPIN_TRY(hipMalloc((void**)&ctx->d_row_sum, (size_t)stat_rows * 8));
    SPIN_TRY(hipMalloc((void**)&ctx->d_row_arg, (size_t)stat_rows * 4));
    SPIN_TRY(hipMalloc((void**)&ctx->d_arrive, (size_t)(max_req + 1) * 4));
    SPIN_TRY(hipMemset(ctx->d_arrive, 0, (size_t)(max_req + 1) * 4));
    size_t last_bytes = 0;
    const size_t runs_bytes = spin::accept_draw_scratch_bytes(max_req + 1, &last_bytes);
    SPIN_TRY(hipMalloc((void**)&ctx->d_draw_runs, runs_bytes));
    SPIN_TRY(hipMalloc((void**)&ctx->d_draw_last, last_bytes));
    for (int s = 0; s < kStages; ++s) SPIN_TRY(hipHostMalloc((void**)&ctx->h_stage[s], blob, hipHostMallocMapped | hipHostMallocPortable));
#undef SPIN_TRY
    ctx->blob_bytes = blob;
    ctx->cap_req = max_req;
    ctx->cap_rows = max_rows;
    ctx->cap_pages = max_pages;
    ctx->cap_items = max_items;
    ctx->cap_slots = max_part_slots;
    return SPIN_OK;
}

}  // extern "C"

namespace {

// What every call that takes a K/V descriptor demands of it (the attention kernels further restrict head_dim).
int check_kv_desc(spin_ctx* ctx, const spin_kv_desc* kv) {
    if (kv->dtype != SPIN_DTYPE_BF16 && kv->dtype != SPIN_DTYPE_F16) return fail(ctx, SPIN_EUNSUPPORTED, "K/V must be bf16 or fp16");
    if (kv->head_dim < 8 || kv->head_dim % 8) return fail(ctx, SPIN_EUNSUPPORTED, "head_dim must be a multiple of 8");
    if (kv->page_size < 1 || (kv->page_size & (kv->page_size - 1)))
        return fail(ctx, SPIN_EUNSUPPORTED, "page_size must be a power of two");
    if (kv->n_kv_heads < 1) return fail(ctx, SPIN_EINVAL, "n_kv_heads < 1");
    if (kv->n_pages < 0 || kv->token_stride < kv->head_dim || kv->token_stride % 8 || kv->page_stride % 8 ||
        kv->head_stride % 8 || kv->page_stride < 0 || kv->head_stride < 0)
        return fail(ctx, SPIN_EINVAL, "bad K/V strides (must be non-negative multiples of 8 elements)");
    // the kernels keep per-lane byte offsets of up to 15 token pitches in 32 bits
    if (kv->token_stride > (1 << 24)) return fail(ctx, SPIN_EUNSUPPORTED, "token_stride above 2^24 elements");
    return SPIN_OK;
}

// Both attention entry points; tree_mask is null for linear drafts.
int verify_attn_impl(spin_ctx* ctx, const spin_kv_desc* kv, const spin_req_table* table, const spin_subreq* subs,
                     int32_t n_sub, const uint64_t* tree_mask, const void* q_dev, void* o_dev, int32_t n_q_heads,
                     float softmax_scale, void* hip_stream) {
    if (!ctx) return SPIN_EINVAL;
    if (!kv || !table) return fail(ctx, SPIN_EINVAL, "kv descriptor or request table is null");
    if (kv->head_dim != 64 && kv->head_dim != 128) return fail(ctx, SPIN_EUNSUPPORTED, "head_dim must be 64 or 128");
    int rc = check_kv_desc(ctx, kv);
    if (rc) return rc;
    if (n_q_heads < 1 || n_q_heads % kv->n_kv_heads)
        return fail(ctx, SPIN_EINVAL, "n_q_heads must be a positive multiple of n_kv_heads");
    const int group = n_q_heads / kv->n_kv_heads;
    if (group > spin::kMaxTileRows) return fail(ctx, SPIN_EUNSUPPORTED, "more than 64 query heads per KV head");
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return fail_hip(ctx, e, "hipSetDevice");
    hipStream_t stream = (hipStream_t)hip_stream;
    // wavefronts per launch: what the device keeps resident for each kernel variant, unless overridden
    int32_t waves[3];
    const int di = kv->head_dim == 128 ? 1 : 0;
    for (int c = 0; c < 3; ++c) {
        if (ctx->resident[di][c] == 0) {
            int n = 0;
            e = spin::attn_resident_waves(kv->head_dim, c, &n);
            if (e != hipSuccess) return fail_hip(ctx, e, "occupancy query");
            ctx->resident[di][c] = std::min(n, kMaxWaves);
        }
        waves[c] = ctx->waves_override > 0 ? ctx->waves_override : ctx->resident[di][c];
    }
    StagedPlan& sp = ctx->staged;
    std::string err;

    // ---- the same tables as last time?  (compared by content: the caller's arrays may have been rewritten)
    bool hit = false;
    if (ctx->reuse_plans && sp.valid && table->n_req > 0 && table->prefix_len && table->draft_len && table->q_offset &&
        table->pt_offset && table->page_table && (size_t)table->n_req == sp.prefix.size() &&
        sp.page_size == kv->page_size && sp.n_kv_heads == kv->n_kv_heads && sp.head_dim == kv->head_dim &&
        sp.n_pages == kv->n_pages && sp.n_q_heads == n_q_heads && sp.waves[0] == waves[0] && sp.waves[1] == waves[1] &&
        sp.waves[2] == waves[2] && sp.has_subs == (subs != nullptr) && sp.n_sub == n_sub && sp.has_tree == (tree_mask != nullptr)) {
        const size_t n = sp.prefix.size();
        hit = !memcmp(sp.prefix.data(), table->prefix_len, n * 4) && !memcmp(sp.draft.data(), table->draft_len, n * 4) &&
              !memcmp(sp.q_off.data(), table->q_offset, (n + 1) * 4) && !memcmp(sp.pt_off.data(), table->pt_offset, (n + 1) * 4) &&
              !memcmp(sp.pages.data(), table->page_table, sp.pages.size() * 4) &&
              (!subs || !memcmp(sp.subs.data(), subs, sp.subs.size() * sizeof(spin_subreq))) &&
              (!tree_mask || !memcmp(sp.tree.data(), tree_mask, sp.tree.size() * 8));
    }
    if (hit && (!kv->k_pool || !kv->v_pool || !q_dev || !o_dev)) return fail(ctx, SPIN_EINVAL, "null device pointer");
    if (((uintptr_t)kv->k_pool | (uintptr_t)kv->v_pool | (uintptr_t)q_dev | (uintptr_t)o_dev) & 15)
        return fail(ctx, SPIN_EINVAL, "K/V pools, Q and O must be 16-byte aligned");
    if (std::isnan(softmax_scale) || std::isinf(softmax_scale)) return fail(ctx, SPIN_EINVAL, "softmax_scale is not finite");

    if (!hit) {
        rc = spin::validate_table(table, kv->page_size, kv->n_pages, true, err);
        if (rc) return fail(ctx, rc, err);
        if (table->n_req == 0) return SPIN_OK;
        if (!kv->k_pool || !kv->v_pool || !q_dev || !o_dev) return fail(ctx, SPIN_EINVAL, "null device pointer");
        if (subs || n_sub != 0) {
            rc = spin::check_tiling(table, subs, n_sub, err);
            if (rc) return fail(ctx, rc, err);
        }
        const int64_t n_req = table->n_req, n_rows = table->q_offset[n_req], n_pages_used = table->pt_offset[n_req];
        if (tree_mask) {
            // draft tokens come in an order that puts every ancestor before its descendants, so row t may
            // see draft keys 0..t only, and always itself
            for (int32_t i = 0; i < table->n_req; ++i) {
                const int32_t g = table->draft_len[i];
                if (g > 64) return fail(ctx, SPIN_ETABLE, "request " + std::to_string(i) + ": a draft tree holds at most 64 tokens");
                for (int32_t t = 0; t < g; ++t) {
                    const uint64_t m = tree_mask[table->q_offset[i] + t];
                    if (!((m >> t) & 1) || (t < 63 && (m >> (t + 1))))
                        return fail(ctx, SPIN_ETABLE, "request " + std::to_string(i) + ", draft row " + std::to_string(t) +
                                                          ": tree mask must hold the row itself and no later token");
                }
            }
        }
        rc = spin::build_plan(table, subs, n_sub, kv->page_size, group, kv->n_kv_heads, waves, ctx->plan, err);
        if (rc) return fail(ctx, rc, err);
        const spin::Plan& plan = ctx->plan;
        const int64_t n_items = (int64_t)plan.pieces.size();
        if (n_req > ctx->cap_req || n_rows > ctx->cap_rows || n_pages_used > ctx->cap_pages || n_items > ctx->cap_items ||
            plan.part_slots > ctx->cap_slots) {
            ctx->need_req = n_req;
            ctx->need_rows = n_rows;
            ctx->need_pages = n_pages_used;
            ctx->need_items = n_items;
            ctx->need_slots = plan.part_slots;
            return fail(ctx, SPIN_ENOSPC, "reserved workspace too small for this batch (see spin_required)");
        }

        // ---- stage the tables (the slot of the previous plan goes back into the rotation)
        sp.valid = false;
        char* h = nullptr;
        rc = next_stage(ctx, &h);
        if (rc) return rc;
        size_t off = 0;
        bool overflow = false;   // a table that would not fit is not copied; checked after the last one
        auto put = [&](const void* src, size_t bytes) {
            const size_t at = off;
            if (off + bytes > ctx->blob_bytes) overflow = true;
            else if (bytes) memcpy(h + off, src, bytes);
            off = align16(off + bytes);
            return at;
        };
        sp.off_pieces = put(plan.pieces.data(), n_items * sizeof(spin::Piece));
        for (int c = 0; c < 3; ++c) {
            const int32_t n_shares = plan.wave_begin[c].empty() ? 0 : (int32_t)plan.wave_begin[c].size() - 1;
            sp.n_waves_launch[c] = plan.n_static[c];
            sp.n_queued[c] = n_shares - plan.n_static[c];
            sp.class_piece_begin[c] = plan.class_piece_begin[c];
            sp.off_waves[c] = put(plan.wave_begin[c].data(), plan.wave_begin[c].size() * 4);
            sp.off_first[c] = put(plan.share_first[c].data(), plan.share_first[c].size() * 4);
        }
        const int32_t zero_queues[4] = {0, 0, 0, 0};   // the chunk queues start at zero
        sp.off_queues = put(zero_queues, sizeof zero_queues);
        sp.off_ppos = put(plan.ppos.data(), plan.ppos.size() * 4);
        sp.off_strips = put(plan.strip_begin.data(), (n_req + 1) * 4);
        sp.off_qoff = put(table->q_offset, (n_req + 1) * 4);
        sp.off_tasks = put(plan.tasks.data(), plan.tasks.size() * 4);
        sp.off_pt = put(table->page_table, n_pages_used * 4);
        sp.off_tree = off;
        if (overflow) return fail(ctx, SPIN_ENOSPC, "internal: staging buffer too small");
        if (tree_mask) {
            if (off + (size_t)n_rows * 16 > ctx->blob_bytes) return fail(ctx, SPIN_ENOSPC, "internal: staging buffer too small");
            uint32_t* rec = (uint32_t*)(h + off);
            for (int64_t i = 0; i < n_req; ++i)
                for (int64_t r = table->q_offset[i]; r < table->q_offset[i + 1]; ++r, rec += 4) {
                    rec[0] = (uint32_t)tree_mask[r];
                    rec[1] = (uint32_t)(tree_mask[r] >> 32);
                    rec[2] = (uint32_t)table->prefix_len[i];
                    rec[3] = 0;
                }
            off = align16(off + (size_t)n_rows * 16);
        }
        if (off > ctx->blob_bytes) return fail(ctx, SPIN_ENOSPC, "internal: staging buffer too small");
        sp.n_tasks = (int32_t)(plan.tasks.size() / 2);
        int32_t max_draft = 1;
        for (int64_t i = 0; i < n_req; ++i) max_draft = std::max(max_draft, table->draft_len[i]);
        sp.max_pairs = max_draft * group;
        // Upload on the context's own stream so that it runs beside the kernels of earlier calls; the
        // caller's stream only waits for it.  d_blob[slot] is free once the kernels of the call that
        // last used it are done.
        // Small tables (a few requests) are not copied at all: they go into the kernels' arguments, which
        // saves the host four runtime calls, the stream a dependency on another stream and the kernels
        // their first round trips to memory -- what counts when the whole step takes tens of microseconds.
        sp.slot = ctx->stage;
        sp.bytes = off;
        sp.in_place = off <= kInPlaceBytes && sp.n_queued[0] + sp.n_queued[1] + sp.n_queued[2] == 0;
        if (!sp.in_place) {
            e = wait_for_readers(ctx, sp.slot);
            if (e != hipSuccess) return fail_hip(ctx, e, "waiting for the previous readers of the table copy");
            e = hipMemcpyAsync(ctx->d_blob[sp.slot], h, off, hipMemcpyHostToDevice, ctx->copy_stream);
            if (e != hipSuccess) return fail_hip(ctx, e, "hipMemcpyAsync");
            e = hipEventRecord(ctx->ev[sp.slot], ctx->copy_stream);
            if (e != hipSuccess) return fail_hip(ctx, e, "hipEventRecord");
            ctx->ev_pending[sp.slot] = true;
        }
        // remember what these tables were made for
        if (ctx->reuse_plans) {
            sp.page_size = kv->page_size;
            sp.n_kv_heads = kv->n_kv_heads;
            sp.head_dim = kv->head_dim;
            sp.n_pages = kv->n_pages;
            sp.n_q_heads = n_q_heads;
            sp.n_sub = n_sub;
            for (int c = 0; c < 3; ++c) sp.waves[c] = waves[c];
            sp.has_subs = subs != nullptr;
            sp.has_tree = tree_mask != nullptr;
            sp.prefix.assign(table->prefix_len, table->prefix_len + n_req);
            sp.draft.assign(table->draft_len, table->draft_len + n_req);
            sp.q_off.assign(table->q_offset, table->q_offset + n_req + 1);
            sp.pt_off.assign(table->pt_offset, table->pt_offset + n_req + 1);
            sp.pages.assign(table->page_table, table->page_table + n_pages_used);
            sp.subs.assign(subs ? subs : nullptr, subs ? subs + n_sub : nullptr);
            sp.tree.assign(tree_mask ? tree_mask : nullptr, tree_mask ? tree_mask + n_rows : nullptr);
            sp.valid = true;
        }
    } else if (!sp.in_place && sp.n_queued[0] + sp.n_queued[1] + sp.n_queued[2] > 0) {
        // the previous launch from these tables used up the chunk queues
        e = hipMemsetAsync(ctx->d_blob[sp.slot] + sp.off_queues, 0, 16, stream);
        if (e != hipSuccess) return fail_hip(ctx, e, "hipMemsetAsync");
    }

    // ---- launch
    const int slot = sp.slot;
    // (with inline tables the table pointers below are offsets into the kernels' inline-table argument)
    const uintptr_t blob = sp.in_place ? 0 : (uintptr_t)ctx->d_blob[slot];
    if (!sp.in_place && ctx->ev_pending[slot]) {
        // The upload must have landed before the kernels start.  The host waits for it here (some ten
        // microseconds, while the GPU is busy with earlier calls) instead of making the stream wait: a wait
        // for another stream's event, put between two kernels, holds the second one up for several microseconds
        // even when the event has long passed.
        e = hipEventSynchronize(ctx->ev[slot]);
        if (e != hipSuccess) return fail_hip(ctx, e, "hipEventSynchronize");
        ctx->ev_pending[slot] = false;
    }
    int pshift = 0;
    while ((1 << pshift) < kv->page_size) ++pshift;
    const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / std::sqrt((float)kv->head_dim);
    spin::AttnParams ap = {};
    ap.k_pool = (const uint16_t*)kv->k_pool;
    ap.v_pool = (const uint16_t*)kv->v_pool;
    ap.q = (const uint16_t*)q_dev;
    ap.pieces = nullptr;
    ap.wave_begin = nullptr;
    ap.queue = nullptr;
    ap.n_queued = 0;
    ap.page_table = (const int32_t*)(blob + sp.off_pt);
    ap.part_o = ctx->d_part_o;
    ap.part_ml = ctx->d_part_ml;
    ap.o = (uint16_t*)o_dev;
    ap.page_stride = kv->page_stride;
    ap.head_stride = kv->head_stride;
    ap.token_stride = kv->token_stride;
    ap.n_q_heads = n_q_heads;
    ap.n_kv_heads = kv->n_kv_heads;
    ap.group = group;
    ap.page_shift = pshift;
    ap.tree_rows = tree_mask ? (const uint32_t*)(blob + sp.off_tree) : nullptr;
    ap.scale_log2 = scale * 1.4426950408889634f;
    ap.inline_tables = sp.in_place ? 1 : 0;

    const spin::Piece* pieces_dev[3];
    const int32_t* waves_dev[3];
    const int32_t* first_dev[3];
    for (int c = 0; c < 3; ++c) {
        pieces_dev[c] = (const spin::Piece*)(blob + sp.off_pieces) + sp.class_piece_begin[c];
        waves_dev[c] = (const int32_t*)(blob + sp.off_waves[c]);
        first_dev[c] = (const int32_t*)(blob + sp.off_first[c]);
    }
    spin::JoinParams jp = {};
    jp.pieces = (const spin::Piece*)(blob + sp.off_pieces);
    jp.ppos = (const int32_t*)(blob + sp.off_ppos);
    jp.strip_begin = (const int32_t*)(blob + sp.off_strips);
    jp.q_offset = (const int32_t*)(blob + sp.off_qoff);
    jp.tasks = (const int32_t*)(blob + sp.off_tasks);
    jp.part_o = ctx->d_part_o;
    jp.part_ml = ctx->d_part_ml;
    jp.o = (uint16_t*)o_dev;
    jp.n_q_heads = n_q_heads;
    jp.n_kv_heads = kv->n_kv_heads;
    jp.group = group;
    jp.n_tasks = sp.n_tasks;
    jp.max_pairs = sp.max_pairs;
    jp.inline_tables = sp.in_place ? 1 : 0;
    hipEvent_t* pe = prof_slot(ctx, ctx->prof_attn, ctx->prof_attn_used, ctx->prof_attn_seen);
    spin::LaunchTiming timing = {};
    if (pe) memcpy(timing.ev, pe, sizeof timing.ev);
    e = spin::launch_attn(kv->head_dim, kv->dtype == SPIN_DTYPE_F16, ap, pieces_dev, waves_dev, first_dev, sp.n_waves_launch, sp.n_queued,
                          (int32_t*)(blob + sp.off_queues), jp, sp.in_place ? ctx->h_stage[slot] : nullptr, sp.bytes, stream,
                          pe ? &timing : nullptr);
    if (e != hipSuccess) return fail_hip(ctx, e, "attention launch");
    if (pe) ctx->prof_attn_second[ctx->prof_attn_used - 1] = timing.second;
    if (!sp.in_place) {   // (tables passed in the arguments were copied at the launch: nothing on the device to protect)
        if (ctx->slot_gen[slot] >= 0 && ctx->slot_stream[slot] != stream) {
            // The same copy was last read on another stream (a reused plan): that stream gets a marker and this one
            // waits for it, so that the markers of this stream stand for the earlier readers as well.
            hipEvent_t m = nullptr;
            e = record_marker(ctx, ctx->slot_stream[slot], &m);
            if (e == hipSuccess) e = hipStreamWaitEvent(stream, m, 0);
            if (e != hipSuccess) return fail_hip(ctx, e, "ordering two streams that read the same tables");
        }
        ctx->slot_gen[slot] = ctx->gen++;
        ctx->slot_stream[slot] = stream;
        if (ctx->gen - 1 - ctx->marked_gen >= kMarkEvery) {
            e = record_marker(ctx, stream, nullptr);
            if (e != hipSuccess) return fail_hip(ctx, e, "hipEventRecord");
        }
    }
    return SPIN_OK;
}

}  // namespace

extern "C" {

int spin_verify_attn(spin_ctx* ctx, const spin_kv_desc* kv, const spin_req_table* table, const spin_subreq* subs,
                     int32_t n_sub, const void* q_dev, void* o_dev, int32_t n_q_heads, float softmax_scale,
                     void* hip_stream) {
    return verify_attn_impl(ctx, kv, table, subs, n_sub, nullptr, q_dev, o_dev, n_q_heads, softmax_scale, hip_stream);
}

int spin_verify_attn_tree(spin_ctx* ctx, const spin_kv_desc* kv, const spin_req_table* table, const spin_subreq* subs,
                          int32_t n_sub, const uint64_t* tree_mask, const void* q_dev, void* o_dev, int32_t n_q_heads,
                          float softmax_scale, void* hip_stream) {
    if (!ctx) return SPIN_EINVAL;
    if (!tree_mask && table && table->n_req > 0 && table->q_offset && table->q_offset[table->n_req] > 0)
        return fail(ctx, SPIN_EINVAL, "tree mask is null");
    return verify_attn_impl(ctx, kv, table, subs, n_sub, tree_mask, q_dev, o_dev, n_q_heads, softmax_scale, hip_stream);
}

int spin_append_kv(spin_ctx* ctx, const spin_kv_desc* kv, const spin_req_table* table, const void* k_new_dev,
                   const void* v_new_dev, void* hip_stream) {
    if (!ctx) return SPIN_EINVAL;
    if (!kv || !table) return fail(ctx, SPIN_EINVAL, "kv descriptor or request table is null");
    int rc = check_kv_desc(ctx, kv);
    if (rc) return rc;
    std::string err;
    rc = spin::validate_table(table, kv->page_size, kv->n_pages, true, err);
    if (rc) return fail(ctx, rc, err);
    if (table->n_req == 0) return SPIN_OK;
    if (!kv->k_pool || !kv->v_pool || !k_new_dev || !v_new_dev) return fail(ctx, SPIN_EINVAL, "null device pointer");
    if (((uintptr_t)kv->k_pool | (uintptr_t)kv->v_pool | (uintptr_t)k_new_dev | (uintptr_t)v_new_dev) & 15)
        return fail(ctx, SPIN_EINVAL, "K/V pools and new rows must be 16-byte aligned");
    const int64_t n_req = table->n_req, n_rows = table->q_offset[n_req];
    if (n_req > ctx->cap_req || n_rows > ctx->cap_rows) {
        ctx->need_req = std::max<int64_t>(n_req, ctx->cap_req);
        ctx->need_rows = std::max<int64_t>(n_rows, ctx->cap_rows);
        ctx->need_pages = ctx->cap_pages;
        ctx->need_items = ctx->cap_items;
        ctx->need_slots = ctx->cap_slots;
        return fail(ctx, SPIN_ENOSPC, "reserved workspace too small for this batch (see spin_required)");
    }
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return fail_hip(ctx, e, "hipSetDevice");
    hipStream_t stream = (hipStream_t)hip_stream;
    // Destination slot of every packed row.  Small batches carry them in the kernel's arguments; otherwise the
    // kernel reads them from a pinned, device-mapped staging buffer, which needs an event behind the kernel before
    // it is reused (and an event record on the stream costs the attention kernel that follows several microseconds).
    const bool inline_slots = n_rows <= spin::kInlineAppendRows * spin::kInlineAppendLaunches &&
                              (int64_t)kv->n_pages * kv->page_size <= INT32_MAX;
    char* h = nullptr;
    if (inline_slots) {
        ctx->slot_host.resize((size_t)n_rows);
    } else {
        rc = next_stage(ctx, &h);
        if (rc) return rc;
    }
    int64_t* dst = inline_slots ? ctx->slot_host.data() : (int64_t*)h;
    for (int64_t i = 0; i < n_req; ++i) {
        const int32_t* pt = table->page_table + table->pt_offset[i];
        for (int32_t t = 0; t < table->draft_len[i]; ++t) {
            const int64_t pos = (int64_t)table->prefix_len[i] + t;
            dst[table->q_offset[i] + t] = (int64_t)pt[pos / kv->page_size] * kv->page_size + pos % kv->page_size;
        }
    }
    void* dst_dev = nullptr;
    if (!inline_slots) {
        e = hipHostGetDevicePointer(&dst_dev, h, 0);
        if (e != hipSuccess) return fail_hip(ctx, e, "hipHostGetDevicePointer");
    }
    const int slot = ctx->stage;
    spin::AppendParams p = {};
    p.dst_slot = (const int64_t*)dst_dev;
    p.k_new = (const uint16_t*)k_new_dev;
    p.v_new = (const uint16_t*)v_new_dev;
    p.k_pool = (uint16_t*)kv->k_pool;
    p.v_pool = (uint16_t*)kv->v_pool;
    p.page_stride = kv->page_stride;
    p.head_stride = kv->head_stride;
    p.token_stride = kv->token_stride;
    p.n_rows = (int32_t)n_rows;
    p.n_kv_heads = kv->n_kv_heads;
    p.head_dim = kv->head_dim;
    int pshift = 0;
    while ((1 << pshift) < kv->page_size) ++pshift;
    p.page_shift = pshift;
    e = spin::launch_append(p, inline_slots ? dst : nullptr, stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "append launch");
    if (!inline_slots) {
        e = hipEventRecord(ctx->ev[slot], stream);
        if (e != hipSuccess) return fail_hip(ctx, e, "hipEventRecord");
        ctx->ev_pending[slot] = true;
    }
    return SPIN_OK;
}

int spin_accept(spin_ctx* ctx, int32_t mode, int32_t n_req, const int32_t* draft_len_host,
                const int32_t* draft_tokens_dev, const float* target_logits_dev, const float* draft_logits_dev,
                int32_t vocab, const double* u_accept_dev, const double* u_sample_dev, int32_t* n_accepted_dev,
                int32_t* next_token_dev, void* hip_stream) {
    if (!ctx) return SPIN_EINVAL;
    if (mode != SPIN_ACCEPT_GREEDY && mode != SPIN_ACCEPT_REJECTION) return fail(ctx, SPIN_EINVAL, "unknown mode");
    if (n_req < 0 || vocab < 1) return fail(ctx, SPIN_EINVAL, "n_req < 0 or vocab < 1");
    if (vocab > spin::kMaxVocab) return fail(ctx, SPIN_EUNSUPPORTED, "vocabulary larger than 1048576 ids");
    if (n_req == 0) return SPIN_OK;
    if (!draft_len_host) return fail(ctx, SPIN_EINVAL, "draft_len is null");
    ctx->row_off_host.resize(n_req + 1);
    int64_t rows = 0;
    int32_t max_draft = 1;
    for (int32_t i = 0; i < n_req; ++i) {
        if (draft_len_host[i] < 1) return fail(ctx, SPIN_EINVAL, "draft_len < 1");
        ctx->row_off_host[i] = (int32_t)rows;
        rows += draft_len_host[i];
        max_draft = std::max(max_draft, draft_len_host[i]);
        if (rows > INT32_MAX / 2) return fail(ctx, SPIN_EINVAL, "too many draft rows");
    }
    ctx->row_off_host[n_req] = (int32_t)rows;
    if (!draft_tokens_dev || !target_logits_dev || !n_accepted_dev || !next_token_dev)
        return fail(ctx, SPIN_EINVAL, "null device pointer");
    if (mode == SPIN_ACCEPT_REJECTION && (!draft_logits_dev || !u_accept_dev || !u_sample_dev))
        return fail(ctx, SPIN_EINVAL, "rejection mode needs draft logits and both uniform arrays");
    if (n_req > ctx->cap_req || rows > ctx->cap_rows) {
        ctx->need_req = std::max<int64_t>(n_req, ctx->cap_req);
        ctx->need_rows = std::max<int64_t>(rows, ctx->cap_rows);
        ctx->need_pages = ctx->cap_pages;
        ctx->need_items = ctx->cap_items;
        ctx->need_slots = ctx->cap_slots;
        return fail(ctx, SPIN_ENOSPC, "reserved workspace too small for this batch (see spin_required)");
    }
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return fail_hip(ctx, e, "hipSetDevice");
    hipStream_t stream = (hipStream_t)hip_stream;

    spin::AcceptParams p = {};
    p.draft_tokens = draft_tokens_dev;
    p.target_logits = target_logits_dev;
    p.draft_logits = draft_logits_dev;
    p.u_accept = u_accept_dev;
    p.u_sample = u_sample_dev;
    p.row_max = ctx->d_row_max;
    p.row_sum = ctx->d_row_sum;
    p.row_arg = ctx->d_row_arg;
    p.arrive = ctx->d_arrive;
    p.draw_runs = ctx->d_draw_runs;
    p.draw_last = ctx->d_draw_last;
    p.n_accepted = n_accepted_dev;
    p.next_token = next_token_dev;
    p.n_req = n_req;
    p.n_rows = (int32_t)rows;
    p.vocab = vocab;
    p.mode = mode;
    // The per-request row offsets travel in the kernels' arguments where the kernels take them there (batches
    // of up to 959 requests on the usual paths).  Otherwise the kernels read them (two ints per workgroup)
    // straight from a pinned, device-mapped staging buffer, which is reused only after an event recorded behind
    // the kernels has passed -- an event record on the stream costs the next kernel several microseconds, which
    // is why the first form goes without.
    int slot = -1;
    if (spin::accept_reads_row_off(p, max_draft)) {
        char* h = nullptr;
        int rc = next_stage(ctx, &h);
        if (rc) return rc;
        memcpy(h, ctx->row_off_host.data(), (size_t)(n_req + 1) * 4);
        void* row_off_dev = nullptr;
        e = hipHostGetDevicePointer(&row_off_dev, h, 0);
        if (e != hipSuccess) return fail_hip(ctx, e, "hipHostGetDevicePointer");
        p.row_off = (const int32_t*)row_off_dev;
        slot = ctx->stage;
    }
    hipEvent_t* pe = prof_slot(ctx, ctx->prof_accept, ctx->prof_accept_used, ctx->prof_accept_seen);
    spin::LaunchTiming timing = {};
    if (pe) memcpy(timing.ev, pe, sizeof timing.ev);
    e = spin::launch_accept(p, max_draft, ctx->row_off_host.data(), stream, pe ? &timing : nullptr);
    if (e != hipSuccess) return fail_hip(ctx, e, "acceptance launch");
    if (pe) ctx->prof_accept_second[ctx->prof_accept_used - 1] = timing.second;
    if (slot >= 0) {
        e = hipEventRecord(ctx->ev[slot], stream);
        if (e != hipSuccess) return fail_hip(ctx, e, "hipEventRecord");
        ctx->ev_pending[slot] = true;
    }
    return SPIN_OK;
}

int spin_accept_tree(spin_ctx* ctx, int32_t mode, int32_t n_req, const int32_t* draft_len_host,
                     const int32_t* parent_host, const int32_t* draft_tokens_dev, const float* target_logits_dev,
                     const float* draft_logits_dev, int32_t vocab, const double* u_accept_dev,
                     const double* u_sample_dev, int32_t* n_accepted_dev, int32_t* path_dev, int32_t* next_token_dev,
                     void* hip_stream) {
    if (!ctx) return SPIN_EINVAL;
    if (mode != SPIN_ACCEPT_GREEDY && mode != SPIN_ACCEPT_REJECTION) return fail(ctx, SPIN_EINVAL, "unknown mode");
    if (n_req < 0 || vocab < 1) return fail(ctx, SPIN_EINVAL, "n_req < 0 or vocab < 1");
    if (mode == SPIN_ACCEPT_REJECTION && vocab > spin::kMaxVocab)
        return fail(ctx, SPIN_EUNSUPPORTED, "vocabulary larger than 1048576 ids");
    if (n_req == 0) return SPIN_OK;
    if (!draft_len_host || !parent_host) return fail(ctx, SPIN_EINVAL, "draft_len or parent is null");
    ctx->row_off_host.resize(n_req + 1);
    int64_t rows = 0;
    for (int32_t i = 0; i < n_req; ++i) {
        const int32_t g = draft_len_host[i];
        if (g < 1) return fail(ctx, SPIN_EINVAL, "draft_len < 1");
        if (g > 64) return fail(ctx, SPIN_ETABLE, "request " + std::to_string(i) + ": a draft tree holds at most 64 tokens");
        for (int32_t t = 0; t < g; ++t) {
            const int32_t par = parent_host[rows + t];
            if (par < -1 || par >= t)
                return fail(ctx, SPIN_ETABLE, "request " + std::to_string(i) + ", draft token " + std::to_string(t) +
                                                  ": the parent must be an earlier token of the request or -1");
        }
        ctx->row_off_host[i] = (int32_t)rows;
        rows += g;
        if (rows > INT32_MAX / 2) return fail(ctx, SPIN_EINVAL, "too many draft rows");
    }
    ctx->row_off_host[n_req] = (int32_t)rows;
    if (!draft_tokens_dev || !target_logits_dev || !n_accepted_dev || !path_dev || !next_token_dev)
        return fail(ctx, SPIN_EINVAL, "null device pointer");
    if (mode == SPIN_ACCEPT_REJECTION && (!draft_logits_dev || !u_accept_dev || !u_sample_dev))
        return fail(ctx, SPIN_EINVAL, "rejection mode needs draft logits and both uniform arrays");
    if (n_req > ctx->cap_req || rows > ctx->cap_rows) {
        ctx->need_req = std::max<int64_t>(n_req, ctx->cap_req);
        ctx->need_rows = std::max<int64_t>(rows, ctx->cap_rows);
        ctx->need_pages = ctx->cap_pages;
        ctx->need_items = ctx->cap_items;
        ctx->need_slots = ctx->cap_slots;
        return fail(ctx, SPIN_ENOSPC, "reserved workspace too small for this batch (see spin_required)");
    }
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return fail_hip(ctx, e, "hipSetDevice");
    hipStream_t stream = (hipStream_t)hip_stream;
    // row offsets and parents are read by the kernels from the pinned, device-mapped staging buffer
    char* h = nullptr;
    int rc = next_stage(ctx, &h);
    if (rc) return rc;
    const size_t off_parent = align16((size_t)(n_req + 1) * 4);
    memcpy(h, ctx->row_off_host.data(), (size_t)(n_req + 1) * 4);
    memcpy(h + off_parent, parent_host, (size_t)rows * 4);
    void* mapped = nullptr;
    e = hipHostGetDevicePointer(&mapped, h, 0);
    if (e != hipSuccess) return fail_hip(ctx, e, "hipHostGetDevicePointer");
    const int slot = ctx->stage;
    spin::AcceptParams p = {};
    p.row_off = (const int32_t*)mapped;
    p.draft_tokens = draft_tokens_dev;
    p.target_logits = target_logits_dev;
    p.draft_logits = draft_logits_dev;
    p.u_accept = u_accept_dev;
    p.u_sample = u_sample_dev;
    p.row_max = ctx->d_row_max;
    p.row_sum = ctx->d_row_sum;
    p.row_arg = ctx->d_row_arg;
    p.n_accepted = n_accepted_dev;
    p.next_token = next_token_dev;
    p.n_req = n_req;
    p.n_rows = (int32_t)rows;
    p.vocab = vocab;
    p.mode = mode;
    e = spin::launch_accept_tree(p, (const int32_t*)((char*)mapped + off_parent), path_dev, stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "tree acceptance launch");
    e = hipEventRecord(ctx->ev[slot], stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "hipEventRecord");
    ctx->ev_pending[slot] = true;
    return SPIN_OK;
}

int spin_set_plan_reuse(spin_ctx* ctx, int32_t enable) {
    if (!ctx) return SPIN_EINVAL;
    ctx->reuse_plans = enable != 0;
    if (!enable) ctx->staged.valid = false;
    return SPIN_OK;
}

int spin_profile_every(spin_ctx* ctx, int32_t n) {
    if (!ctx || n < 1) return SPIN_EINVAL;
    ctx->prof_every = n;
    return SPIN_OK;
}

int spin_profile_begin(spin_ctx* ctx, int32_t max_calls) {
    if (!ctx || max_calls < 0) return SPIN_EINVAL;
    ctx->prof_attn_seen = ctx->prof_accept_seen = 0;
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return fail_hip(ctx, e, "hipSetDevice");
    free_profile(ctx);
    for (int k = 0; k < 2; ++k) {
        std::vector<hipEvent_t>& pool = k ? ctx->prof_accept : ctx->prof_attn;
        (k ? ctx->prof_accept_second : ctx->prof_attn_second).assign((size_t)max_calls, 0);
        for (int64_t i = 0; i < (int64_t)max_calls * 4; ++i) {
            hipEvent_t ev;
            e = hipEventCreate(&ev);
            if (e != hipSuccess) {
                free_profile(ctx);
                return fail_hip(ctx, e, "hipEventCreate");
            }
            pool.push_back(ev);
        }
    }
    ctx->prof_on = true;
    return SPIN_OK;
}

int spin_profile_end(spin_ctx* ctx, double ms[4], int32_t calls[2]) {
    if (!ctx || !ms || !calls) return SPIN_EINVAL;
    for (int k = 0; k < 4; ++k) ms[k] = 0.0;
    calls[0] = ctx->prof_attn_used;
    calls[1] = ctx->prof_accept_used;
    int rc = SPIN_OK;
    for (int k = 0; k < 2 && rc == SPIN_OK; ++k) {
        std::vector<hipEvent_t>& pool = k ? ctx->prof_accept : ctx->prof_attn;
        const int used = k ? ctx->prof_accept_used : ctx->prof_attn_used;
        const std::vector<uint8_t>& second = k ? ctx->prof_accept_second : ctx->prof_attn_second;
        for (int i = 0; i < used; ++i) {
            hipEvent_t* p = pool.data() + (size_t)i * 4;
            hipError_t e = hipEventSynchronize(second[i] ? p[3] : p[1]);
            float a = 0.f, b = 0.f;
            if (e == hipSuccess) e = hipEventElapsedTime(&a, p[0], p[1]);
            if (e == hipSuccess && second[i]) e = hipEventElapsedTime(&b, p[2], p[3]);
            if (e != hipSuccess) { rc = fail_hip(ctx, e, "reading profile events"); break; }
            ms[2 * k] += a;
            ms[2 * k + 1] += b;
        }
    }
    free_profile(ctx);
    return rc;
}

}  // extern "C"
