// Internal declarations shared by the host scheduler and the HIP kernels of libspin.
// Nothing here is part of the C ABI (see include/spin.h for that).
#ifndef SPIN_INTERNAL_H
#define SPIN_INTERNAL_H

#include <stdint.h>

#include <string>
#include <vector>

#include "spin.h"

namespace spin {

// Rows of the (draft row x query head of one KV group) tile one wave works on: up to 4 MFMA
// column tiles of 16.
constexpr int kMaxTileRows = 64;
// Page ids one work item may touch (cached in LDS by the attention kernel).
constexpr int kMaxItemPages = 136;
// Default / maximum number of keys per work item.
constexpr int kDefaultChunk = 1024;
constexpr int kMaxChunk = 2048;

// One unit of attention work: draft rows [q_row0, q_row0+n_q) (packed row numbers) of `parent`
// against its keys [k0, k1); row t of the item sees keys below min(k1, causal0 + t).
struct Item {
    int32_t parent;
    int32_t q_row0;
    int32_t n_q;
    int32_t causal0;
    int32_t k0, k1;
    int32_t pt_base;    // first page-table entry of the parent
    int32_t part_base;  // first partial-result slot; the item owns n_q * n_q_heads slots
};

struct Plan {
    std::vector<Item> items;           // sorted by parent (then k0, then row)
    std::vector<int32_t> order[3];     // launch order per column-tile class (1, 2, 4 tiles): longest first
    std::vector<int32_t> item_begin;   // [n_req+1] range of items of each parent
    std::vector<int32_t> row_req;      // [R] request of each packed row
    int64_t part_slots = 0;
    // scratch reused between calls
    std::vector<spin_subreq> rects, tmp;
};

// Table checks shared by every entry point. n_pages < 0 skips the page-id range check.
int validate_table(const spin_req_table* t, int page_size, int64_t n_pages, bool need_pages,
                   std::string& err);
int check_tiling(const spin_req_table* t, const spin_subreq* subs, int32_t n_sub, std::string& err);
int build_plan(const spin_req_table* t, const spin_subreq* subs, int32_t n_sub, int page_size,
               int group, int n_q_heads, int chunk, Plan& plan, std::string& err);

}  // namespace spin

#endif
