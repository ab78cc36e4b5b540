// Host side of libspin that needs no GPU: table checks, request decomposition (Sec. V-A),
// the tiling check and the work scheduler.  Integers only.
#include <algorithm>
#include <cstring>
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
    int32_t pos = 0;
    for (int32_t i = 0; i < t->n_req; ++i) {
        int64_t p = t->prefix_len[i], g = t->draft_len[i];
        int64_t want = g * p + g * (g + 1) / 2;   // sum over rows of (p + t + 1)
        int64_t got = 0;
        int32_t first = pos;
        while (pos < n_sub && subs[idx[pos]].parent == i) got += visible_cells(subs[idx[pos++]], p);
        // No two pieces may share a visible cell; with equal areas this makes the cover exact.
        for (int32_t a = first; a < pos; ++a)
            for (int32_t b = a + 1; b < pos; ++b) {
                const spin_subreq &x = subs[idx[a]], &y = subs[idx[b]];
                int64_t r0 = std::max(x.q_begin, y.q_begin);
                int64_t r1 = std::min((int64_t)x.q_begin + x.q_len, (int64_t)y.q_begin + y.q_len);
                int64_t k0 = std::max(x.kv_begin, y.kv_begin);
                int64_t k1 = std::min((int64_t)x.kv_begin + x.kv_len, (int64_t)y.kv_begin + y.kv_len);
                if (r0 < r1 && k0 < k1 && k0 < p + r1) {
                    err = fmt("request %lld: sub-requests overlap", i); return SPIN_ETABLE;
                }
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
               int group, int n_q_heads, int chunk, Plan& plan, std::string& err) {
    if (group < 1 || group > kMaxTileRows) { err = "query heads per KV head must be 1..64"; return SPIN_EUNSUPPORTED; }
    const int max_rows = kMaxTileRows / group;
    // keys per item: bounded by the chunk and by the page ids one item may cache
    int64_t page_cap = (int64_t)(kMaxItemPages - 2) * page_size;
    int C = (int)std::min<int64_t>(std::min(chunk, kMaxChunk), page_cap);
    C = std::max(C, 1);

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

    plan.items.clear();
    for (int k = 0; k < 3; ++k) plan.order[k].clear();
    plan.item_begin.assign(t->n_req + 1, 0);
    int64_t slots = 0;
    for (const spin_subreq& s : rects) {
        int32_t p = t->prefix_len[s.parent];
        for (int32_t qb = s.q_begin; qb < s.q_begin + s.q_len; qb += max_rows) {
            int32_t ql = std::min(max_rows, s.q_begin + s.q_len - qb);
            int32_t ke = std::min(s.kv_begin + s.kv_len, p + qb + ql);
            for (int32_t c = (s.kv_begin / C) * C; c < ke; c += C) {
                int32_t k0 = std::max(c, s.kv_begin), k1 = std::min(c + C, ke);
                if (k0 >= k1) continue;
                Item it;
                it.parent = s.parent;
                it.q_row0 = t->q_offset[s.parent] + qb;
                it.n_q = ql;
                it.causal0 = p + qb + 1;
                it.k0 = k0;
                it.k1 = k1;
                it.pt_base = t->pt_offset ? t->pt_offset[s.parent] : 0;
                if (slots + (int64_t)ql * n_q_heads > INT32_MAX) { err = "too many partial results"; return SPIN_ENOSPC; }
                it.part_base = (int32_t)slots;
                slots += (int64_t)ql * n_q_heads;
                plan.items.push_back(it);
                plan.item_begin[s.parent + 1]++;
            }
        }
    }
    for (int32_t i = 0; i < t->n_req; ++i) plan.item_begin[i + 1] += plan.item_begin[i];
    plan.part_slots = slots;

    // launch order: per column-tile class, longest items first (counting sort on length)
    std::vector<int32_t>& tmp = plan.row_req;   // borrowed as scratch before it is filled below
    for (int cls = 0; cls < 3; ++cls) {
        tmp.assign(C + 2, 0);
        for (size_t k = 0; k < plan.items.size(); ++k) {
            const Item& it = plan.items[k];
            int tiles = (it.n_q * group + 15) / 16;
            int c = tiles <= 1 ? 0 : (tiles == 2 ? 1 : 2);
            if (c == cls) tmp[C - (it.k1 - it.k0) + 1]++;
        }
        for (int k = 0; k <= C; ++k) tmp[k + 1] += tmp[k];
        plan.order[cls].resize(tmp[C + 1]);
        for (size_t k = 0; k < plan.items.size(); ++k) {
            const Item& it = plan.items[k];
            int tiles = (it.n_q * group + 15) / 16;
            int c = tiles <= 1 ? 0 : (tiles == 2 ? 1 : 2);
            if (c == cls) plan.order[cls][tmp[C - (it.k1 - it.k0)]++] = (int32_t)k;
        }
    }
    int32_t R = t->n_req ? t->q_offset[t->n_req] : 0;
    plan.row_req.resize(R);
    for (int32_t i = 0; i < t->n_req; ++i)
        for (int32_t r = t->q_offset[i]; r < t->q_offset[i + 1]; ++r) plan.row_req[r] = i;
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
                  int32_t group, int32_t keys_per_item, spin_subreq* items_out, int32_t cap,
                  int32_t* n_out) {
    std::string err;
    if (!n_out || cap < 0 || (cap > 0 && !items_out) || page_size < 1 || keys_per_item < 1) return SPIN_EINVAL;
    int rc = spin::validate_table(table, 1, -1, false, err);
    if (rc) return rc;
    if (!table->q_offset && table->n_req > 0) return SPIN_EINVAL;
    if (subs) {
        rc = spin::check_tiling(table, subs, n_sub, err);
        if (rc) return rc;
    }
    spin::Plan plan;
    spin_req_table t = *table;
    t.pt_offset = nullptr;
    rc = spin::build_plan(&t, subs, n_sub, page_size, group, group, keys_per_item, plan, err);
    if (rc) return rc;
    *n_out = (int32_t)plan.items.size();
    if ((int64_t)plan.items.size() > cap) return SPIN_ENOSPC;
    for (size_t k = 0; k < plan.items.size(); ++k) {
        const spin::Item& it = plan.items[k];
        int32_t qb = it.q_row0 - table->q_offset[it.parent];
        items_out[k] = {it.parent, qb, it.n_q, it.k0, it.k1 - it.k0};
    }
    return SPIN_OK;
}

}  // extern "C"
