// Kernel parameter blocks and launch entry points shared by the HIP translation units of
// libspin.  Internal; the C ABI is include/spin.h.
#ifndef SPIN_DEVICE_H
#define SPIN_DEVICE_H

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "spin_internal.h"

namespace spin {

// Elements (IEEE half precision) per partial output row, whatever the head dim; head dim 64 uses the first 64.
constexpr int kPartRow = 128;

// Tables of a small call (a handful of requests) travel in the kernel arguments instead of device memory:
// the pointer fields marked (*) then hold byte offsets into this block, which follows the parameter block in
// the argument segment, and the kernels turn them into addresses there.
constexpr size_t kInlineTableBytes = 3840;
struct alignas(16) InlineTables {
    char bytes[kInlineTableBytes];
};

struct AttnParams {
    const uint16_t* k_pool;
    const uint16_t* v_pool;
    const uint16_t* q;
    const Piece* pieces;         // (*) pieces of one column-tile class, in streaming order
    const int32_t* wave_begin;   // (*) [n_shares + 1] pieces of each share: gridDim.x per-wavefront shares, then queued chunks
    const int32_t* share_first;  // (*) first block of each share: page ids of its 16-key halves (two; eight for the grouped-query
                                 // kernel's blocks), KV head, first key (-1: the block is not requested ahead)
    int32_t* queue;              // next queued chunk to hand out (zero at launch)
    int32_t n_queued;
    const int32_t* page_table;   // (*)
    uint16_t* part_o;            // [slots][kPartRow] partial rows, each normalised by its own sum, half precision
    float* part_ml;              // [slots][2]: running max (log2 domain), sum
    uint16_t* o;                 // final rows of pieces flagged direct
    const uint32_t* tree_rows;   // (*) tree-shaped drafts only, else null: [R][4] = ancestor mask (low, high), prefix length, 0
    int64_t page_stride, head_stride, token_stride;   // elements
    int32_t n_q_heads, n_kv_heads, group, page_shift;
    float scale_log2;            // softmax scale * log2(e)
    int32_t inline_tables;       // the (*) fields are offsets into the InlineTables argument
};

struct JoinParams {
    const Piece* pieces;         // (*) all classes
    const int32_t* ppos;         // (*) [n_strips * n_kv_heads][2] first piece and count of each (strip, KV head)
    const int32_t* strip_begin;  // (*) [n_req + 1]
    const int32_t* q_offset;     // (*) [n_req + 1]
    const int32_t* tasks;        // (*) [n_tasks][2] (request, KV head)
    const uint16_t* part_o;
    const float* part_ml;
    uint16_t* o;
    int32_t n_q_heads, n_kv_heads, group, n_tasks;
    int32_t max_pairs;           // largest (draft rows x group) of any request
    int32_t inline_tables;       // the (*) fields are offsets into the InlineTables argument
};

// Timing of one call's kernels: the first kernel's start and end are written to ev[0], ev[1], the second kernel's
// -- when the call launches one, which `second` then says -- to ev[2], ev[3].  The time stamps are those of the kernels'
// own dispatch records (events handed to the launch itself): nothing extra is put on the stream.
struct LaunchTiming {
    hipEvent_t ev[4];
    bool second;
};

// Wavefronts of the attention kernel of class `cls` (0, 1, 2) and head dim that fit on the device at once.
hipError_t attn_resident_waves(int head_dim, int cls, int* n_waves);

// n_waves[c] wavefronts stream the pieces of class c; timing (may be null) receives the time stamps of the
// attention kernel (first) and the join kernel (second).  inline_tables (may be null): the tables themselves, at most
// kInlineTableBytes of them, to be passed in the kernel arguments (base.inline_tables / jp.inline_tables set).
hipError_t launch_attn(int head_dim, bool f16, const AttnParams& base, const Piece* const pieces_dev[3],
                       const int32_t* const wave_begin_dev[3], const int32_t* const share_first_dev[3],
                       const int32_t n_waves[3], const int32_t n_queued[3],
                       int32_t* queues_dev, const JoinParams& jp, const void* inline_tables, size_t inline_bytes,
                       hipStream_t stream, LaunchTiming* timing);

struct AppendParams {
    const int64_t* dst_slot;   // [R] page * page_size + slot of every packed row
    const uint16_t* k_new;     // [R][n_kv_heads][head_dim]
    const uint16_t* v_new;
    uint16_t* k_pool;
    uint16_t* v_pool;
    int64_t page_stride, head_stride, token_stride;
    int32_t n_rows, n_kv_heads, head_dim, page_shift;
};

// Batches of up to kInlineAppendRows * kInlineAppendLaunches draft rows whose slots fit 32 bits bring their
// destination slots in the kernel arguments, kInlineAppendRows per launch (dst_slot_host: the slots as the host
// holds them; p.dst_slot may then be null); larger ones are read by the kernel from p.dst_slot.
constexpr int kInlineAppendRows = 960;
constexpr int kInlineAppendLaunches = 4;
hipError_t launch_append(const AppendParams& p, const int64_t* dst_slot_host, hipStream_t stream);

struct AcceptParams {
    const int32_t* row_off;        // [n_req+1] first draft row of each request (device)
    const int32_t* draft_tokens;   // [R]
    const float* target_logits;    // [R+n_req][V]
    const float* draft_logits;     // [R][V] or null
    const double* u_accept;        // [R]
    const double* u_sample;        // [n_req]
    float* row_max;                // [2R+n_req] target rows first, then draft rows
    double* row_sum;
    int32_t* row_arg;
    int32_t* arrive;               // [n_req] arrival counters (zero between launches), or null: the plain two-launch form
    double* draw_runs;             // [n_req][512] run masses of the next-token draw, or null
    int32_t* draw_last;            // [n_req][8] last id with mass of every part of the vocabulary
    int32_t* n_accepted;
    int32_t* next_token;
    int32_t n_req, n_rows, vocab, mode;
    int32_t draw_parts;            // parts the vocabulary is cut into by the next-token draw (set by launch_accept)
};

// Largest vocabulary the next-token search handles (its per-run sums live in LDS).
constexpr int kMaxVocab = 1 << 20;

// Small vocabularies (with arrival counters p.arrive and the longest draft of the batch, max_draft >= 1): one
// launch.  Otherwise the row statistics, then -- rejection mode with counters and the run table p.draw_runs --
// the next-token draw spread over eight workgroups per request, else one workgroup per request.
// row_off_host (may be null): the offsets p.row_off points at, as the host holds them; small batches pass
// them to the kernel by value.  timing (may be null) receives the time stamps of the first and the second kernel.
hipError_t launch_accept(const AcceptParams& p, int max_draft, const int32_t* row_off_host, hipStream_t stream,
                         LaunchTiming* timing);

// Whether the kernels launch_accept would launch for p read p.row_off (else the offsets travel in the kernel
// arguments and p.row_off may be null).
bool accept_reads_row_off(const AcceptParams& p, int max_draft);

// Bytes of p.draw_runs (returned) and p.draw_last for batches of up to n_req requests.
size_t accept_draw_scratch_bytes(int64_t n_req, size_t* last_bytes);

// Look up, for the current device, the address of the static scratch array of spin_accept_noalloc (done by
// spin_create so that the entry point's first call on a device finds it ready).
hipError_t resolve_static_scratch();

// Greedy walk down token trees; p is the (greedy-mode) parameter block of the row statistics, parent
// [R] (device) the index of every draft token's parent within its request (-1: the last prefix token),
// path [R] (device) receives the accepted nodes.
hipError_t launch_accept_tree(const AcceptParams& p, const int32_t* parent, int32_t* path, hipStream_t stream);

}  // namespace spin
#endif
