// Host side of libspin that needs no GPU: table checks, request decomposition (Sec. V-A),
// the tiling check and the work scheduler.  Integers only.
#include <algorithm>
#include <cstring>
#include <iterator>
#include <map>
#include <string>
#include <vector>

#include "spin_internal.h"

namespace spin {

static std::string fmt(const char* what, long long a, long long b = 0) {
    char buf[256];
    snprintf(buf, sizeof buf, what, a, b);
    return buf;
}

int validate_table(const spin_req_table* t, int page_size, int64_t n_pages, bool need_pages,
                   std::string& err) {
    if (!t || t->n_req < 0) { err = "request table is null or n_req < 0"; return SPIN_EINVAL; }
    if (t->n_req == 0) return SPIN_OK;
    if (!t->prefix_len || !t->draft_len) { err = "prefix_len / draft_len is null"; return SPIN_EINVAL; }
    for (int32_t i = 0; i < t->n_req; ++i) {
        if (t->prefix_len[i] < 0) { err = fmt("request %lld: prefix_len < 0", i); return SPIN_EINVAL; }
        if (t->draft_len[i] < 1) { err = fmt("request %lld: draft_len < 1", i); return SPIN_EINVAL; }
        if ((int64_t)t->prefix_len[i] + t->draft_len[i] > (int64_t)INT32_MAX / 2) {
            err = fmt("request %lld: too long", i); return SPIN_EINVAL;
        }
    }
    if (t->q_offset) {
        if (t->q_offset[0] != 0) { err = "q_offset[0] != 0"; return SPIN_ETABLE; }
        for (int32_t i = 0; i < t->n_req; ++i)
            if (t->q_offset[i + 1] - t->q_offset[i] != t->draft_len[i]) {
                err = fmt("request %lld: q_offset does not advance by draft_len", i);
                return SPIN_ETABLE;
            }
    } else if (need_pages) { err = "q_offset is null"; return SPIN_EINVAL; }
    if (!need_pages) return SPIN_OK;
    if (!t->pt_offset || !t->page_table) { err = "pt_offset / page_table is null"; return SPIN_EINVAL; }
    if (page_size < 1) { err = "page_size < 1"; return SPIN_EINVAL; }
    if (t->pt_offset[0] < 0) { err = "pt_offset[0] < 0"; return SPIN_ETABLE; }
    for (int32_t i = 0; i < t->n_req; ++i) {
        int64_t have = (int64_t)t->pt_offset[i + 1] - t->pt_offset[i];
        int64_t need = ((int64_t)t->prefix_len[i] + t->draft_len[i] + page_size - 1) / page_size;
        if (have < need) {
            err = fmt("request %lld: page table holds %lld entries, too few", i, have);
            return SPIN_ETABLE;
        }
        if (n_pages >= 0) {
            const int32_t* pt = t->page_table + t->pt_offset[i];
            for (int64_t c = 0; c < need; ++c)
                if (pt[c] < 0 || pt[c] >= n_pages) {
                    err = fmt("request %lld: page id %lld outside the pool", i, pt[c]);
                    return SPIN_ETABLE;
                }
        }
    }
    return SPIN_OK;
}

// Number of visible cells of rectangle s of a parent with prefix p.
static int64_t visible_cells(const spin_subreq& s, int64_t p) {
    int64_t n = 0;
    for (int64_t t = s.q_begin; t < (int64_t)s.q_begin + s.q_len; ++t) {
        int64_t hi = std::min<int64_t>((int64_t)s.kv_begin + s.kv_len, p + t + 1);
        if (hi > s.kv_begin) n += hi - s.kv_begin;
    }
    return n;
}

int check_tiling(const spin_req_table* t, const spin_subreq* subs, int32_t n_sub, std::string& err) {
    if (n_sub < 0 || (n_sub > 0 && !subs)) { err = "sub-request array is null or n_sub < 0"; return SPIN_EINVAL; }
    std::vector<int32_t> idx(n_sub);
    for (int32_t k = 0; k < n_sub; ++k) {
        const spin_subreq& s = subs[k];
        if (s.parent < 0 || s.parent >= t->n_req) { err = fmt("sub-request %lld: parent out of range", k); return SPIN_ETABLE; }
        int64_t p = t->prefix_len[s.parent], g = t->draft_len[s.parent];
        if (s.q_begin < 0 || s.q_len < 1 || (int64_t)s.q_begin + s.q_len > g ||
            s.kv_begin < 0 || s.kv_len < 1 || (int64_t)s.kv_begin + s.kv_len > p + g) {
            err = fmt("sub-request %lld: rectangle outside its parent", k); return SPIN_ETABLE;
        }
        idx[k] = k;
    }
    std::sort(idx.begin(), idx.end(), [&](int32_t a, int32_t b) {
        if (subs[a].parent != subs[b].parent) return subs[a].parent < subs[b].parent;
        return a < b;
    });
    // Per request: the pieces' visible cells must add up to the request's, and no two pieces may share a
    // visible cell; with equal areas that makes the cover exact.  Overlaps are found by a sweep over the
    // draft rows (n log n in the pieces of a request): every piece is first cut back to the rows and keys
    // where it has visible cells at all -- keys below its last row's causal edge, rows from the first one
    // that sees its first key -- after which two pieces share a visible cell exactly when their row ranges
    // and their key ranges both intersect.  The pieces alive at a row are kept ordered by first key; they
    // are pairwise disjoint, so a piece that enters need only be compared with its two neighbours.
    struct Event {
        int32_t row, enter, k0, k1;   // leave events (enter = 0) sort before enter events of the same row
    };
    std::vector<Event> events;
    std::map<int32_t, int32_t> alive;  // first key -> end key
    int32_t pos = 0;
    for (int32_t i = 0; i < t->n_req; ++i) {
        int64_t p = t->prefix_len[i], g = t->draft_len[i];
        int64_t want = g * p + g * (g + 1) / 2;   // sum over rows of (p + t + 1)
        int64_t got = 0;
        events.clear();
        alive.clear();
        for (; pos < n_sub && subs[idx[pos]].parent == i; ++pos) {
            const spin_subreq& s = subs[idx[pos]];
            got += visible_cells(s, p);
            const int64_t q_end = (int64_t)s.q_begin + s.q_len;
            const int64_t k_end = std::min<int64_t>((int64_t)s.kv_begin + s.kv_len, p + q_end);
            const int64_t q_first = std::max<int64_t>(s.q_begin, (int64_t)s.kv_begin - p);
            if (k_end <= s.kv_begin || q_first >= q_end) continue;   // nothing visible in it
            events.push_back({(int32_t)q_first, 1, s.kv_begin, (int32_t)k_end});
            events.push_back({(int32_t)q_end, 0, s.kv_begin, (int32_t)k_end});
        }
        std::sort(events.begin(), events.end(), [](const Event& a, const Event& b) {
            if (a.row != b.row) return a.row < b.row;
            return a.enter < b.enter;
        });
        for (const Event& e : events) {
            if (!e.enter) {
                alive.erase(e.k0);
                continue;
            }
            auto next = alive.lower_bound(e.k0);
            bool clash = next != alive.end() && next->first < e.k1;
            if (!clash && next != alive.begin()) clash = std::prev(next)->second > e.k0;
            if (clash) {
                err = fmt("request %lld: sub-requests overlap", i); return SPIN_ETABLE;
            }
            alive.emplace(e.k0, e.k1);
        }
        if (got != want) {
            err = fmt("request %lld: sub-requests cover %lld cells, not all of them", i, got);
            return SPIN_ETABLE;
        }
    }
    return SPIN_OK;
}

// ---- scheduler ---------------------------------------------------------------------------
// A valid decomposition covers every visible cell once, so by Eq. (13) of Sec. V-A any re-cut of
// the same cells gives the same outputs.  The scheduler uses that freedom in both directions:
// pieces that sit side by side are joined again when that costs nothing (so a prefix shared by
// several row bands is streamed once), and long key ranges are cut into chunks so the chip is
// filled evenly.

static void join_along_keys(std::vector<spin_subreq>& r) {
    std::sort(r.begin(), r.end(), [](const spin_subreq& a, const spin_subreq& b) {
        if (a.parent != b.parent) return a.parent < b.parent;
        if (a.q_begin != b.q_begin) return a.q_begin < b.q_begin;
        if (a.q_len != b.q_len) return a.q_len < b.q_len;
        return a.kv_begin < b.kv_begin;
    });
    size_t w = 0;
    for (size_t k = 0; k < r.size(); ++k) {
        if (w > 0) {
            spin_subreq& a = r[w - 1];
            const spin_subreq& b = r[k];
            if (a.parent == b.parent && a.q_begin == b.q_begin && a.q_len == b.q_len &&
                a.kv_begin + a.kv_len == b.kv_begin) {
                a.kv_len += b.kv_len;
                continue;
            }
        }
        r[w++] = r[k];
    }
    r.resize(w);
}

static void join_along_rows(std::vector<spin_subreq>& r, const spin_req_table* t, int max_rows) {
    std::sort(r.begin(), r.end(), [](const spin_subreq& a, const spin_subreq& b) {
        if (a.parent != b.parent) return a.parent < b.parent;
        if (a.kv_begin != b.kv_begin) return a.kv_begin < b.kv_begin;
        return a.q_begin < b.q_begin;
    });
    size_t w = 0;
    for (size_t k = 0; k < r.size(); ++k) {
        if (w > 0) {
            spin_subreq& a = r[w - 1];
            const spin_subreq& b = r[k];
            if (a.parent == b.parent && a.kv_begin == b.kv_begin && a.q_begin + a.q_len == b.q_begin &&
                a.q_len + b.q_len <= max_rows) {
                // Joining must not show any row a key it could not see before: a piece may end
                // early only where its own last row's causal edge is.
                int32_t p = t->prefix_len[a.parent];
                int32_t ea = a.kv_begin + a.kv_len, eb = b.kv_begin + b.kv_len;
                int32_t e = std::max(ea, eb);
                bool ok_a = (ea == e) || (ea == p + a.q_begin + a.q_len);
                bool ok_b = (eb == e) || (eb == p + b.q_begin + b.q_len);
                if (ok_a && ok_b) {
                    a.q_len += b.q_len;
                    a.kv_len = e - a.kv_begin;
                    continue;
                }
            }
        }
        r[w++] = r[k];
    }
    r.resize(w);
}

int build_plan(const spin_req_table* t, const spin_subreq* subs, int32_t n_sub, int page_size,
               int group, int n_kv_heads, const int32_t n_waves[3], Plan& plan, std::string& err) {
    if (group < 1 || group > kMaxTileRows) { err = "query heads per KV head must be 1..64"; return SPIN_EUNSUPPORTED; }
    if (n_kv_heads < 1 || n_kv_heads > kPieceHeadMask) { err = "n_kv_heads out of range"; return SPIN_EUNSUPPORTED; }
    const int max_rows = kMaxTileRows / group;
    // blocks one piece may span: bounded by the page ids a piece may cache
    int64_t window_keys = std::min<int64_t>(2048, (int64_t)(kMaxPiecePages - 2) * page_size);

    std::vector<spin_subreq>& rects = plan.rects;
    rects.clear();
    if (subs) {
        rects.assign(subs, subs + n_sub);
        // pull every piece back to its last row's causal edge: beyond it nothing is visible
        size_t w = 0;
        for (size_t k = 0; k < rects.size(); ++k) {
            spin_subreq s = rects[k];
            int32_t edge = t->prefix_len[s.parent] + s.q_begin + s.q_len;
            if (s.kv_begin >= edge) continue;
            s.kv_len = std::min(s.kv_begin + s.kv_len, edge) - s.kv_begin;
            rects[w++] = s;
        }
        rects.resize(w);
        join_along_keys(rects);
        join_along_rows(rects, t, 1 << 30);
    } else {
        for (int32_t i = 0; i < t->n_req; ++i)
            rects.push_back({i, 0, t->draft_len[i], 0, t->prefix_len[i] + t->draft_len[i]});
    }
    std::sort(rects.begin(), rects.end(), [](const spin_subreq& a, const spin_subreq& b) {
        if (a.parent != b.parent) return a.parent < b.parent;
        if (a.kv_begin != b.kv_begin) return a.kv_begin < b.kv_begin;
        return a.q_begin < b.q_begin;
    });

    // ---- strips: rectangles cut into row bands one wavefront tile can hold
    plan.strips.clear();
    plan.strip_begin.assign(t->n_req + 1, 0);
    for (int c = 0; c < 3; ++c) plan.class_blocks[c] = 0, plan.n_static[c] = 0;
    for (const spin_subreq& s : rects) {
        const int32_t p = t->prefix_len[s.parent];
        for (int32_t qb = s.q_begin; qb < s.q_begin + s.q_len; qb += max_rows) {
            const int32_t ql = std::min(max_rows, s.q_begin + s.q_len - qb);
            const int32_t ke = std::min(s.kv_begin + s.kv_len, p + qb + ql);
            if (s.kv_begin >= ke) continue;
            const int tiles = (ql * group + 15) / 16;
            Strip st{s.parent, qb, ql, s.kv_begin, ke, tiles <= 1 ? 0 : (tiles == 2 ? 1 : 2),
                     (s.kv_begin == 0 && ke == p + qb + ql) ? 1 : 0};
            plan.strips.push_back(st);
            plan.strip_begin[s.parent + 1]++;
        }
    }
    // One launch per call: every strip runs in the kernel instance of the widest strip (a single
    // wavefront for one or two column tiles, a workgroup of eight wavefronts beyond that).
    int call_cls = 0;
    for (const Strip& st : plan.strips) call_cls = std::max(call_cls, st.cls);
    const int bk = block_keys(call_cls);
    const int window_blocks = (int)std::max<int64_t>(1, window_keys / bk);
    for (Strip& st : plan.strips) {
        st.cls = call_cls;
        plan.class_blocks[call_cls] += (int64_t)((st.k1 - st.k0 + bk - 1) / bk) * n_kv_heads;
    }
    for (int32_t i = 0; i < t->n_req; ++i) plan.strip_begin[i + 1] += plan.strip_begin[i];
    const size_t n_strips = plan.strips.size();
    if ((int64_t)n_strips * n_kv_heads > INT32_MAX / 4) { err = "too many strips"; return SPIN_ENOSPC; }

    // ---- pieces: per class the blocks of all (strip, KV head) pairs form one long sequence (strip,
    // then head, then block); it is cut into equal shares, one per wavefront.  A wavefront keeps its
    // accumulators while it stays inside one (strip, head), so only the cuts cost a partial result.
    plan.pieces.clear();
    plan.piece_strip.clear();
    plan.piece_wave.clear();
    plan.ppos.assign(n_strips * n_kv_heads * 2, 0);
    plan.need_join.assign((size_t)t->n_req * n_kv_heads, 0);
    int64_t slots = 0;
    for (int c = 0; c < 3; ++c) {
        plan.class_piece_begin[c] = (int32_t)plan.pieces.size();
        std::vector<int32_t>& wb = plan.wave_begin[c];
        wb.clear();
        plan.share_first[c].clear();
        const int64_t T = plan.class_blocks[c];
        if (T == 0) continue;
        const int64_t W = std::max<int64_t>(1, std::min<int64_t>(n_waves[c], T / kMinBlocksPerWave));
        // Share boundaries.  The first part of the sequence is cut into W equal shares, one per
        // wavefront.  Wavefronts do not all stream at the same speed, so the last part is cut into
        // small chunks that wavefronts take from a queue as they finish (sizes shrink towards the end).
        std::vector<int64_t>& bounds = plan.bounds;
        bounds.clear();
        // (The grouped-query kernel gets no queue: its workgroups end within a few percent of each other
        // anyway, and the extra cuts cost more in partial results to join than the evening-out saves.)
        const int64_t T_dyn = (c < 2 && W >= kMinDynamicWaves && T / W * bk >= kMinKeysForQueue) ? T * kDynamicPercent / 100 : 0;
        const int64_t T_static = T - T_dyn;
        for (int64_t w = 1; w <= W; ++w) bounds.push_back(w * T_static / W);
        if (T_dyn == 0 && T / W <= kSnapShareBlocks) {
            // Short shares (small batches, where a launch costs as much as the work): a boundary that
            // falls within a few blocks of the end of a (strip, head) moves there, so that many such
            // pairs stay whole, are written directly, and the join kernel may not be needed at all.
            std::vector<int64_t>& ends = plan.unit_ends;
            ends.clear();
            int64_t at = 0;
            for (const Strip& st : plan.strips) {
                if (st.cls != c) continue;
                const int64_t nb = (st.k1 - st.k0 + bk - 1) / bk;
                for (int kvh = 0; kvh < n_kv_heads; ++kvh) ends.push_back(at += nb);
            }
            size_t u = 0, kept = 0;
            for (size_t w = 0; w < bounds.size(); ++w) {
                int64_t b = bounds[w];
                while (u + 1 < ends.size() && ends[u] < b) ++u;       // ends[u]: first pair end at or after b
                const int64_t hi = ends[u], lo = u > 0 ? ends[u - 1] : 0;
                if (hi - b <= kSnapBlocks && hi - b <= b - lo) b = hi;
                else if (b - lo <= kSnapBlocks) b = lo;
                if (b > (kept ? bounds[kept - 1] : 0)) bounds[kept++] = b;   // drop shares left empty
            }
            bounds.resize(kept);
            if (bounds.empty() || bounds.back() != T) bounds.push_back(T);
        }
        plan.n_static[c] = (int32_t)bounds.size();
        for (int64_t at = T_static; at < T;) {
            const int64_t left = T - at;
            const int64_t chunk = std::min<int64_t>(left, std::max<int64_t>(kMinChunkKeys / bk, std::min<int64_t>(kMaxChunkKeys / bk, left / W)));
            at += chunk;
            bounds.push_back(at);
        }
        const int64_t n_shares = (int64_t)bounds.size();
        if (n_shares > INT32_MAX / 2) { err = "too many shares"; return SPIN_ENOSPC; }
        int64_t wave = 0, pos = 0;
        wb.push_back(0);
        for (size_t si = 0; si < n_strips; ++si) {
            const Strip& st = plan.strips[si];
            if (st.cls != c) continue;
            const int32_t nb = (st.k1 - st.k0 + bk - 1) / bk;
            const int32_t p = t->prefix_len[st.parent];
            for (int kvh = 0; kvh < n_kv_heads; ++kvh) {
                const size_t first = plan.pieces.size();
                int32_t b = 0;
                while (b < nb) {
                    while (wave < n_shares - 1 && pos >= bounds[wave]) {
                        ++wave;
                        wb.push_back((int32_t)(plan.pieces.size() - plan.class_piece_begin[c]));
                    }
                    const int64_t seg_end = bounds[wave];
                    const int32_t take = (int32_t)std::min<int64_t>(std::min<int64_t>(nb - b, seg_end - pos), window_blocks);
                    Piece pc;
                    pc.head_flags = kvh;
                    pc.q_row0 = t->q_offset[st.parent] + st.q_begin;
                    pc.n_q = st.q_len;
                    pc.causal0 = p + st.q_begin + 1;
                    pc.k0 = st.k0 + b * bk;
                    pc.k1 = std::min(st.k1, st.k0 + (b + take) * bk);
                    pc.pt_base = t->pt_offset ? t->pt_offset[st.parent] : 0;
                    pc.out_base = 0;
                    plan.pieces.push_back(pc);
                    plan.piece_strip.push_back((int32_t)si);
                    plan.piece_wave.push_back((int32_t)wave);
                    b += take;
                    pos += take;
                }
                // flags: runs of pieces held by the same wavefront carry their accumulators along
                const size_t last = plan.pieces.size();
                const bool one_wave = plan.piece_wave[first] == plan.piece_wave[last - 1];
                for (size_t k = first; k < last; ++k) {
                    Piece& pc = plan.pieces[k];
                    if (k > first && plan.piece_wave[k - 1] == plan.piece_wave[k]) pc.head_flags |= kPieceCarryIn;
                    if (k + 1 < last && plan.piece_wave[k + 1] == plan.piece_wave[k]) {
                        pc.head_flags |= kPieceCarryOut;
                    } else if (one_wave && st.row_complete) {
                        pc.head_flags |= kPieceDirect;
                    } else {
                        if (slots + (int64_t)st.q_len * group > INT32_MAX) { err = "too many partial results"; return SPIN_ENOSPC; }
                        pc.out_base = (int32_t)slots;
                        slots += (int64_t)st.q_len * group;
                        plan.need_join[(size_t)st.parent * n_kv_heads + kvh] = 1;
                    }
                }
                plan.ppos[(si * n_kv_heads + kvh) * 2] = (int32_t)first;
                plan.ppos[(si * n_kv_heads + kvh) * 2 + 1] = (int32_t)(last - first);
            }
        }
        while ((int64_t)wb.size() < n_shares + 1) wb.push_back((int32_t)(plan.pieces.size() - plan.class_piece_begin[c]));
        // What a wavefront needs to request the first K/V block of a share before it has read anything else.
        // Per share: the page ids of the block's 16-key halves (two for the single-wavefront kernels, eight for the
        // grouped-query kernel's block of 128 keys), the KV head and the first key (-1: nothing is requested ahead).
        std::vector<int32_t>& sf = plan.share_first[c];
        const int halves = bk / 16, rec = halves + 2;
        sf.assign((size_t)n_shares * rec, 0);
        for (int64_t s = 0; s < n_shares; ++s) {
            sf[s * rec + halves + 1] = -1;
            if (wb[s] >= wb[s + 1] || !t->pt_offset || !t->page_table || page_size < 16) continue;
            const Piece& pc = plan.pieces[(size_t)plan.class_piece_begin[c] + wb[s]];
            if ((pc.k0 & 31) || pc.k0 + bk > pc.k1) continue;
            for (int h = 0; h < halves; ++h) sf[s * rec + h] = t->page_table[pc.pt_base + (pc.k0 + 16 * h) / page_size];
            sf[s * rec + halves] = pc.head_flags & kPieceHeadMask;
            sf[s * rec + halves + 1] = pc.k0;
        }
    }
    plan.class_piece_begin[3] = (int32_t)plan.pieces.size();
    plan.part_slots = slots;
    plan.tasks.clear();
    for (int32_t i = 0; i < t->n_req; ++i)
        for (int kvh = 0; kvh < n_kv_heads; ++kvh)
            if (plan.need_join[(size_t)i * n_kv_heads + kvh]) {
                plan.tasks.push_back(i);
                plan.tasks.push_back(kvh);
            }
    return SPIN_OK;
}

}  // namespace spin

// ---- C ABI: host-only entry points ---------------------------------------------------------
extern "C" {

const char* spin_strerror(int code) {
    switch (code) {
        case SPIN_OK: return "ok";
        case SPIN_EINVAL: return "invalid argument";
        case SPIN_ETABLE: return "inconsistent request table, page table or sub-request tiling";
        case SPIN_ENOSPC: return "output capacity or reserved workspace too small";
        case SPIN_EUNSUPPORTED: return "unsupported shape or type";
        case SPIN_EHIP: return "HIP runtime error";
        default: return "unknown error code";
    }
}

int spin_kv_padding(const spin_req_table* table, int32_t kv_len, int64_t* n_rows, int64_t* n_pad) {
    std::string err;
    int rc = spin::validate_table(table, 1, -1, false, err);
    if (rc) return rc;
    if (kv_len < 1) return SPIN_EINVAL;
    int64_t rows = 0, pad = 0;
    for (int32_t i = 0; i < table->n_req; ++i) {
        int64_t n = (int64_t)table->prefix_len[i] + table->draft_len[i];
        int64_t r = (n + kv_len - 1) / kv_len;
        rows += r;
        pad += r * kv_len - n;
    }
    if (n_rows) *n_rows = rows;
    if (n_pad) *n_pad = pad;
    return SPIN_OK;
}

int spin_decompose(const spin_req_table* table, const spin_decomp_params* params, spin_subreq* out,
                   int32_t cap, int32_t* n_out, int32_t* kv_len_out) {
    std::string err;
    if (!params || !n_out || cap < 0 || (cap > 0 && !out)) return SPIN_EINVAL;
    int rc = spin::validate_table(table, 1, -1, false, err);
    if (rc) return rc;
    int32_t L = 0, w = 0;
    switch (params->policy) {
        case SPIN_DECOMP_NONE: break;
        case SPIN_DECOMP_Q_SPLIT:
            if (params->q_width < 1) return SPIN_EINVAL;
            w = params->q_width;
            break;
        case SPIN_DECOMP_KV_SPLIT:
            if (params->kv_len < 1) return SPIN_EINVAL;
            L = params->kv_len;
            break;
        case SPIN_DECOMP_KV_SEARCH: {
            if (params->max_subreq < 1 || params->l_step < 1 || params->l_min < 1 ||
                params->l_max < params->l_min) return SPIN_EINVAL;
            // every candidate length is tried: the padding count is not monotone in L (Sec. V-A)
            int64_t best_pad = -1;
            int64_t first = ((int64_t)params->l_min + params->l_step - 1) / params->l_step * params->l_step;
            for (int64_t cand = first; cand <= params->l_max; cand += params->l_step) {
                int64_t rows, pad;
                spin_kv_padding(table, (int32_t)cand, &rows, &pad);
                if (rows <= params->max_subreq && (best_pad < 0 || pad <= best_pad)) {
                    best_pad = pad;
                    L = (int32_t)cand;
                }
            }
            if (kv_len_out) *kv_len_out = L;
            if (L == 0) { *n_out = 0; return SPIN_ENOSPC; }
            break;
        }
        default: return SPIN_EINVAL;
    }
    if (kv_len_out && params->policy == SPIN_DECOMP_KV_SPLIT) *kv_len_out = L;
    int64_t n = 0;
    auto emit = [&](int32_t parent, int32_t qb, int32_t ql, int32_t kb, int32_t kl) {
        if (n < cap) out[n] = {parent, qb, ql, kb, kl};
        ++n;
    };
    for (int32_t i = 0; i < table->n_req; ++i) {
        int32_t p = table->prefix_len[i], g = table->draft_len[i];
        if (w > 0) {
            for (int32_t qb = 0; qb < g; qb += w) {
                int32_t ql = std::min(w, g - qb);
                emit(i, qb, ql, 0, p + qb + ql);
            }
        } else if (L > 0) {
            for (int32_t kb = 0; kb < p + g; kb += L) emit(i, 0, g, kb, std::min(L, p + g - kb));
        } else {
            emit(i, 0, g, 0, p + g);
        }
    }
    if (n > INT32_MAX) return SPIN_ENOSPC;
    *n_out = (int32_t)n;
    return n > cap ? SPIN_ENOSPC : SPIN_OK;
}

int spin_check_tiling(const spin_req_table* table, const spin_subreq* subs, int32_t n_sub) {
    std::string err;
    int rc = spin::validate_table(table, 1, -1, false, err);
    if (rc) return rc;
    return spin::check_tiling(table, subs, n_sub, err);
}

int spin_schedule(const spin_req_table* table, const spin_subreq* subs, int32_t n_sub, int32_t page_size,
                  int32_t group, int32_t n_kv_heads, int32_t n_waves, spin_work_piece* out, int32_t cap,
                  int32_t* n_out) {
    std::string err;
    if (!n_out || cap < 0 || (cap > 0 && !out) || page_size < 1 || n_waves < 1) return SPIN_EINVAL;
    int rc = spin::validate_table(table, 1, -1, false, err);
    if (rc) return rc;
    if (!table->q_offset && table->n_req > 0) return SPIN_EINVAL;
    if (subs || n_sub != 0) {
        rc = spin::check_tiling(table, subs, n_sub, err);
        if (rc) return rc;
    }
    spin::Plan plan;
    spin_req_table t = *table;
    t.pt_offset = nullptr;
    const int32_t waves[3] = {n_waves, n_waves, n_waves};
    rc = spin::build_plan(&t, subs, n_sub, page_size, group, n_kv_heads, waves, plan, err);
    if (rc) return rc;
    *n_out = (int32_t)plan.pieces.size();
    if ((int64_t)plan.pieces.size() > cap) return SPIN_ENOSPC;
    for (size_t k = 0; k < plan.pieces.size(); ++k) {
        const spin::Piece& pc = plan.pieces[k];
        const spin::Strip& st = plan.strips[plan.piece_strip[k]];
        out[k] = {st.parent, st.q_begin, st.q_len, pc.k0, pc.k1 - pc.k0, pc.head_flags & spin::kPieceHeadMask,
                  st.cls, plan.piece_wave[k],
                  ((pc.head_flags & spin::kPieceCarryIn) ? SPIN_PIECE_CARRY_IN : 0) |
                      ((pc.head_flags & spin::kPieceCarryOut) ? SPIN_PIECE_CARRY_OUT : 0) |
                      ((pc.head_flags & spin::kPieceDirect) ? SPIN_PIECE_DIRECT : 0) |
                      (plan.piece_wave[k] >= plan.n_static[st.cls] ? SPIN_PIECE_QUEUED : 0)};
    }
    return SPIN_OK;
}

}  // extern "C"
