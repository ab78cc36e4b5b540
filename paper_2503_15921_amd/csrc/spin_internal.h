// Internal declarations shared by the host scheduler and the HIP kernels of libspin.
// Nothing here is part of the C ABI (see include/spin.h for that).
#ifndef SPIN_INTERNAL_H
#define SPIN_INTERNAL_H

#include <stdint.h>

#include <string>
#include <vector>

#include "spin.h"

namespace spin {

// Rows of the (draft row x query head of one KV group) tile one wavefront works on: up to 4 MFMA
// column tiles of 16.
constexpr int kMaxTileRows = 64;
// Keys per wavefront and streaming block of the attention kernels.
constexpr int kBlockKeys = 32;
// Keys per streaming block of the kernel that serves column-tile class c: classes 0 and 1 (one or two
// tiles) run on single wavefronts, class 2 (up to four tiles) on workgroups with four streaming wavefronts.
constexpr int block_keys(int cls) { return cls == 2 ? 4 * kBlockKeys : kBlockKeys; }
// Page ids one piece may touch (cached in LDS by the attention kernel).
constexpr int kMaxPiecePages = 136;
// A wavefront is given at least this many blocks before another wavefront is used.
constexpr int kMinBlocksPerWave = 4;
// Share of the blocks (percent) that is handed out from a queue at the end instead of up front, the
// size range of the queued chunks in keys, and the launch and share sizes from which queueing is used.
constexpr int kDynamicPercent = 10;
constexpr int kMinChunkKeys = 512;
constexpr int kMaxChunkKeys = 1024;
constexpr int kMinDynamicWaves = 64;
constexpr int kMinKeysForQueue = 6144;   // keys per share below which queueing does not pay

// Shares of at most kSnapShareBlocks blocks have their boundaries moved to the end of a (strip, head)
// when one lies within kSnapBlocks blocks.
constexpr int kSnapShareBlocks = 8;
constexpr int kSnapBlocks = 4;

constexpr int32_t kPieceHeadMask = 0xffff;
constexpr int32_t kPieceCarryIn = 1 << 16;   // accumulators continue from the wavefront's previous piece
constexpr int32_t kPieceCarryOut = 1 << 17;  // nothing is written; the next piece continues
constexpr int32_t kPieceDirect = 1 << 18;    // this piece ends a strip-head held by one wavefront: write final rows

// A strip: draft rows [q_begin, q_begin+q_len) of `parent` against keys [k0, k1), at most
// kMaxTileRows / group rows, clipped at its last row's causal edge.
struct Strip {
    int32_t parent, q_begin, q_len, k0, k1;
    int32_t cls;            // column-tile class: 0, 1, 2 for 1, 2, 4 tiles of 16 rows
    int32_t row_complete;   // holds every key its rows may see (k0 == 0 and k1 at the causal edge)
};

// One run of consecutive blocks of one (strip, KV head), streamed by one wavefront: draft rows
// [q_row0, q_row0+n_q) (packed row numbers) against keys [k0, k1); row t sees keys below
// min(k1, causal0 + t).  32 bytes, fetched by the kernel with scalar loads.
struct Piece {
    int32_t head_flags;   // KV head | kPiece* flags
    int32_t q_row0;
    int32_t n_q;
    int32_t causal0;
    int32_t k0, k1;
    int32_t pt_base;      // first page-table entry of the parent
    int32_t out_base;     // first partial-result slot (n_q * group slots) unless carried out or direct
};

struct Plan {
    std::vector<Strip> strips;            // sorted by parent
    std::vector<int32_t> strip_begin;     // [n_req+1] strips of each request
    std::vector<Piece> pieces;            // class 0 | class 1 | class 2, each in streaming order
    std::vector<int32_t> piece_strip;     // strip of each piece
    std::vector<int32_t> piece_wave;      // wavefront (within its class) of each piece
    int32_t class_piece_begin[4] = {0, 0, 0, 0};
    std::vector<int32_t> wave_begin[3];   // [n_shares+1] pieces (index within the class) of each share:
                                          // first the n_static per-wavefront shares, then the queued chunks
    int32_t n_static[3] = {0, 0, 0};
    std::vector<int32_t> share_first[3];  // first block of each share: page ids of its 16-key halves (2, or 8 for class 2),
                                          // KV head, first key (-1: not a whole block on a 32-key boundary, or pages under 16 tokens)
    std::vector<int64_t> bounds;
    std::vector<int64_t> unit_ends;       // scratch: cumulative block count at the end of every (strip, head)
    std::vector<int32_t> ppos;            // [n_strips * n_kv_heads][2]: first piece (global index) and count
    std::vector<int32_t> tasks;           // [n_tasks][2]: (request, KV head) pairs that have partial results to join
    int64_t part_slots = 0;
    int64_t class_blocks[3] = {0, 0, 0};
    // scratch reused between calls
    std::vector<spin_subreq> rects;
    std::vector<uint8_t> need_join;
};

// Table checks shared by every entry point. n_pages < 0 skips the page-id range check.
int validate_table(const spin_req_table* t, int page_size, int64_t n_pages, bool need_pages,
                   std::string& err);
int check_tiling(const spin_req_table* t, const spin_subreq* subs, int32_t n_sub, std::string& err);
// n_waves[c]: wavefronts available to column-tile class c.
int build_plan(const spin_req_table* t, const spin_subreq* subs, int32_t n_sub, int page_size,
               int group, int n_kv_heads, const int32_t n_waves[3], Plan& plan, std::string& err);

}  // namespace spin

#endif
