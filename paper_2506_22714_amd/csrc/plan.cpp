// Host planner: 2D-aware workload distribution (Section 4.2), hybrid load
// balancing (Section 4.3) and format translation (bitmap blocks + residual CSR,
// Section 4.1 item 3) for the SpMM and SDDMM sub-plans.  Pure host C++; windows
// are processed independently on a pool of std::threads and concatenated in
// window order, so the result does not depend on the thread count.
#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <exception>
#include <new>
#include <thread>

#include "plan_internal.h"

using namespace libra;

namespace {

struct Entry {
    uint64_t key;   // col << 32 | csr position  (position order = row order inside a window)
    int32_t r;      // row inside the window
};
struct Vec {
    int32_t col, cnt, first;   // entries [first, first+cnt) of the sorted window
};

// Output of one contiguous range of windows, indices local to the range.
struct Part {
    SubPlan spmm, sddmm;
    int64_t n_vectors = 0, n_vectors_nnz1 = 0;
};

struct Ctx {
    int64_t M, nnz;
    const int32_t *rowptr, *col;
    const uint8_t *val;
    int vsize;
    Resolved o;
    int words;
};

inline void push_val(std::vector<uint8_t> &dst, const Ctx &c, int32_t p) {
    const uint8_t *s = c.val + (size_t)p * c.vsize;
    dst.insert(dst.end(), s, s + c.vsize);
}

// Emit one bitmap block made of the vectors `ids` (slot order) of the current window.
// Returns the mask of window rows that hold a nonzero of the block.
uint32_t emit_block(const Ctx &c, SubPlan &sp, const std::vector<Entry> &ent, const std::vector<Vec> &vecs,
                    const int32_t *ids, int n, std::vector<std::pair<int32_t, int32_t>> &tmp) {
    const int KB = c.o.KB;
    tmp.clear();
    uint32_t rowmask = 0;
    for (int s = 0; s < n; ++s) {
        const Vec &v = vecs[ids[s]];
        sp.blk_cols.push_back(v.col);
        for (int e = v.first; e < v.first + v.cnt; ++e) {
            tmp.emplace_back(ent[e].r * KB + s, (int32_t)(ent[e].key & 0xffffffffu));
            rowmask |= 1u << ent[e].r;
        }
    }
    for (int s = n; s < KB; ++s) sp.blk_cols.push_back(-1);
    std::sort(tmp.begin(), tmp.end());
    size_t w0 = sp.blk_bitmap.size();
    sp.blk_bitmap.resize(w0 + c.words, 0);
    for (auto &bp : tmp) {
        sp.blk_bitmap[w0 + bp.first / 64] |= 1ull << (bp.first % 64);
        sp.dense_perm.push_back(bp.second);
        push_val(sp.dense_val, c, bp.second);
    }
    sp.blk_valptr.push_back((int32_t)sp.dense_perm.size());
    sp.dense_vectors += n;
    sp.pad_slots += KB - n;
    return rowmask;
}

void plan_range(const Ctx &c, int64_t w0, int64_t w1, Part &out) {
    const Resolved &o = c.o;
    const int W = o.W, KB = o.KB;
    std::vector<Entry> ent;
    std::vector<Vec> vecs;
    std::vector<int32_t> ids, cand, resp;
    std::vector<uint8_t> is_dense;
    std::vector<std::pair<int32_t, int32_t>> tmp;
    std::vector<uint32_t> blk_rowmask;
    SubPlan &sa = out.spmm, &sd = out.sddmm;
    sa.win_blkptr.push_back(0);
    sa.blk_valptr.push_back(0);
    sd.win_blkptr.push_back(0);
    sd.blk_valptr.push_back(0);
    sa.win_resptr.push_back(0);

    for (int64_t w = w0; w < w1; ++w) {
        const int64_t r0 = w * W, r1 = std::min<int64_t>(c.M, r0 + W);
        // ---- census: nonzero column vectors of the window (Section 2.2) ----
        ent.clear();
        for (int64_t i = r0; i < r1; ++i)
            for (int32_t p = c.rowptr[i]; p < c.rowptr[i + 1]; ++p)
                ent.push_back({((uint64_t)(uint32_t)c.col[p] << 32) | (uint32_t)p, (int32_t)(i - r0)});
        std::sort(ent.begin(), ent.end(), [](const Entry &a, const Entry &b) { return a.key < b.key; });
        vecs.clear();
        for (int e = 0; e < (int)ent.size();) {
            int32_t cc = (int32_t)(ent[e].key >> 32);
            int f = e;
            while (e < (int)ent.size() && (int32_t)(ent[e].key >> 32) == cc) ++e;
            vecs.push_back({cc, e - f, f});
        }
        out.n_vectors += (int64_t)vecs.size();
        for (auto &v : vecs) out.n_vectors_nnz1 += v.cnt == 1;

        // =================== SpMM sub-plan ===================
        if (o.build_spmm) {
            is_dense.assign(vecs.size(), 0);
            ids.clear();
            if (o.mode != LIBRA_MODE_SCALAR_ONLY) {
                const int tau = o.mode == LIBRA_MODE_DENSE_ONLY ? 1 : o.tau_spmm;
                for (int v = 0; v < (int)vecs.size(); ++v)
                    if (vecs[v].cnt >= tau) ids.push_back(v);           // ascending column
                if (!ids.empty() && o.fill && o.mode == LIBRA_MODE_HYBRID && ids.size() % KB) {
                    // free slots of the last block take scalar-bound vectors, densest first
                    size_t free_slots = KB - ids.size() % KB;
                    cand.clear();
                    for (int v = 0; v < (int)vecs.size(); ++v)
                        if (vecs[v].cnt < tau) cand.push_back(v);
                    std::stable_sort(cand.begin(), cand.end(),
                                     [&](int a, int b) { return vecs[a].cnt > vecs[b].cnt; });
                    for (size_t q = 0; q < cand.size() && q < free_slots; ++q) ids.push_back(cand[q]);
                }
            }
            for (int v : ids) is_dense[v] = 1;
            const int32_t b0 = (int32_t)sa.n_blocks();
            blk_rowmask.clear();
            for (size_t s = 0; s < ids.size(); s += KB)
                blk_rowmask.push_back(emit_block(c, sa, ent, vecs, ids.data() + s,
                                                 (int)std::min<size_t>(KB, ids.size() - s), tmp));
            const int32_t b1 = (int32_t)sa.n_blocks();
            sa.win_blkptr.push_back(b1);
            // residual nonzeros of the window in CSR order, and how many each row keeps
            resp.clear();
            for (int v = 0; v < (int)vecs.size(); ++v)
                if (!is_dense[v])
                    for (int e = vecs[v].first; e < vecs[v].first + vecs[v].cnt; ++e)
                        resp.push_back((int32_t)(ent[e].key & 0xffffffffu));
            std::sort(resp.begin(), resp.end());
            int32_t rlen[32] = {0};
            {
                int64_t i = r0;
                for (int32_t p : resp) {
                    while (p >= c.rowptr[i + 1]) ++i;
                    ++rlen[i - r0];
                }
            }

            // ---- hybrid load balancing (Section 4.3) ----
            uint32_t valid = 0, split_mask = 0, scalar_mask = 0;
            for (int r = 0; r < (int)(r1 - r0); ++r) {
                valid |= 1u << r;
                if (rlen[r] == 0) continue;
                if (rlen[r] < o.short_len) {
                    ++sa.short_rows;
                } else {
                    ++sa.long_rows;
                    if (rlen[r] > o.Cs) split_mask |= 1u << r;
                }
                if (!(split_mask >> r & 1)) scalar_mask |= 1u << r;
            }
            sa.split_rows += __builtin_popcount(split_mask);
            // residual array: rows that are not decomposed first (row order), then the decomposed rows
            auto emit_rows = [&](bool want_split) {
                int64_t i = r0;
                for (int32_t p : resp) {
                    while (p >= c.rowptr[i + 1]) ++i;
                    if ((bool)(split_mask >> (i - r0) & 1) != want_split) continue;
                    sa.res_perm.push_back(p);
                    sa.res_row.push_back((int32_t)i);
                    sa.res_col.push_back(c.col[p]);
                    push_val(sa.res_val, c, p);
                }
            };
            const int32_t q0 = (int32_t)sa.res_perm.size();
            emit_rows(false);
            const int32_t q1 = (int32_t)sa.res_perm.size();
            auto touched = [&](int32_t g0, int32_t g1) {
                uint32_t m = 0;
                for (int32_t b = g0; b < g1; ++b) m |= blk_rowmask[b - b0];
                return m;
            };
            auto cols_in = [&](int32_t g0, int32_t g1) {
                uint32_t n = 0;
                for (int32_t b = g0; b < g1; ++b)
                    for (int s = 0; s < KB; ++s) n += sa.blk_cols[(size_t)b * KB + s] >= 0;
                return n;
            };
            if (b1 - b0 > o.Ts) {
                for (int32_t g0 = b0; g0 < b1; g0 += o.Ts) {
                    int32_t g1 = std::min(b1, g0 + o.Ts);
                    sa.tasks.push_back({LIBRA_TASK_WINDOW, (int32_t)w, g0, g1, q0, q0, 0u, touched(g0, g1), 0u, cols_in(g0, g1)});
                    sa.task_col.push_back(-1);
                }
                if (scalar_mask) {
                    sa.tasks.push_back({LIBRA_TASK_WINDOW, (int32_t)w, b1, b1, q0, q1, scalar_mask, scalar_mask, 0u, (uint32_t)(q1 - q0)});
                    sa.task_col.push_back(-1);
                }
                for (int64_t i = r0; i < r1; ++i) sa.zero_rows.push_back((int32_t)i);
            } else {
                sa.tasks.push_back({LIBRA_TASK_WINDOW, (int32_t)w, b0, b1, q0, q1, scalar_mask, split_mask & touched(b0, b1),
                                    valid & ~split_mask, cols_in(b0, b1) + (uint32_t)(q1 - q0)});
                sa.task_col.push_back(-1);
                for (int r = 0; r < (int)(r1 - r0); ++r)
                    if (split_mask >> r & 1) sa.zero_rows.push_back((int32_t)(r0 + r));
            }
            emit_rows(true);
            {
                int32_t q = q1;
                for (int r = 0; r < (int)(r1 - r0); ++r) {
                    if (!(split_mask >> r & 1)) continue;
                    const int32_t e = q + rlen[r];
                    for (; q < e; q += o.Cs) {
                        int32_t qe = std::min(e, q + o.Cs);
                        sa.tasks.push_back({LIBRA_TASK_CHUNK, (int32_t)(r0 + r), 0, 0, q, qe, 0u, 0u, 0u, (uint32_t)(qe - q)});
                        sa.task_col.push_back(sa.res_col[q]);            // first column of the segment
                    }
                    q = e;
                }
            }
            sa.win_resptr.push_back((int32_t)sa.res_perm.size());
        }

        // =================== SDDMM sub-plan ===================
        if (o.build_sddmm) {
            ids.resize(vecs.size());
            for (int v = 0; v < (int)vecs.size(); ++v) ids[v] = v;
            std::stable_sort(ids.begin(), ids.end(), [&](int a, int b) { return vecs[a].cnt > vecs[b].cnt; });
            const int32_t b0 = (int32_t)sd.n_blocks();
            size_t used = 0;
            if (o.mode != LIBRA_MODE_SCALAR_ONLY) {
                for (size_t s = 0; s < ids.size(); s += KB) {
                    int n = (int)std::min<size_t>(KB, ids.size() - s);
                    int blk_nnz = 0;
                    for (int q = 0; q < n; ++q) blk_nnz += vecs[ids[s + q]].cnt;
                    if (o.mode == LIBRA_MODE_HYBRID && blk_nnz < o.tau_sddmm) break;   // sums never increase: prefix
                    emit_block(c, sd, ent, vecs, ids.data() + s, n, tmp);
                    used = s + n;
                }
            }
            const int32_t b1 = (int32_t)sd.n_blocks();
            sd.win_blkptr.push_back(b1);
            for (int32_t g0 = b0; g0 < b1; g0 += o.sddmm_Ts) {
                int32_t g1 = std::min(b1, g0 + o.sddmm_Ts);
                uint32_t ncols = 0;
                for (int32_t b = g0; b < g1; ++b)
                    for (int s = 0; s < KB; ++s) ncols += sd.blk_cols[(size_t)b * KB + s] >= 0;
                sd.tasks.push_back({LIBRA_TASK_WINDOW, (int32_t)w, g0, g1, 0, 0, 0u, 0u, 0u, ncols + (uint32_t)W});
            }
            resp.clear();
            for (size_t q = used; q < ids.size(); ++q) {
                const Vec &v = vecs[ids[q]];
                for (int e = v.first; e < v.first + v.cnt; ++e) resp.push_back((int32_t)(ent[e].key & 0xffffffffu));
            }
            std::sort(resp.begin(), resp.end());
            int64_t i = r0;
            for (int32_t p : resp) {
                while (p >= c.rowptr[i + 1]) ++i;
                sd.res_perm.push_back(p);
                sd.res_row.push_back((int32_t)i);
                sd.res_col.push_back(c.col[p]);
                push_val(sd.res_val, c, p);
            }
        }
    }
}

template <class T>
void append(std::vector<T> &dst, const std::vector<T> &src) { dst.insert(dst.end(), src.begin(), src.end()); }

// Append `src` (local indices) to `dst` (global indices).
void concat(SubPlan &dst, SubPlan &src, bool spmm) {
    const int32_t blk_base = (int32_t)dst.n_blocks();
    const int32_t val_base = (int32_t)dst.dense_perm.size();
    const int32_t res_base = (int32_t)dst.res_perm.size();
    for (size_t i = 1; i < src.win_blkptr.size(); ++i) dst.win_blkptr.push_back(src.win_blkptr[i] + blk_base);
    for (size_t i = 1; i < src.blk_valptr.size(); ++i) dst.blk_valptr.push_back(src.blk_valptr[i] + val_base);
    append(dst.blk_cols, src.blk_cols);
    append(dst.blk_bitmap, src.blk_bitmap);
    append(dst.dense_perm, src.dense_perm);
    append(dst.dense_val, src.dense_val);
    append(dst.res_perm, src.res_perm);
    append(dst.res_col, src.res_col);
    append(dst.res_row, src.res_row);
    append(dst.res_val, src.res_val);
    append(dst.zero_rows, src.zero_rows);
    append(dst.task_col, src.task_col);
    if (spmm)
        for (size_t i = 1; i < src.win_resptr.size(); ++i) dst.win_resptr.push_back(src.win_resptr[i] + res_base);
    for (libra_task_t t : src.tasks) {
        if (t.kind == LIBRA_TASK_WINDOW) { t.blk_begin += blk_base; t.blk_end += blk_base; }
        if (spmm) { t.res_begin += res_base; t.res_end += res_base; }
        dst.tasks.push_back(t);
    }
    dst.dense_vectors += src.dense_vectors;
    dst.pad_slots += src.pad_slots;
    dst.short_rows += src.short_rows;
    dst.long_rows += src.long_rows;
    dst.split_rows += src.split_rows;
    src = SubPlan();
}

// Sorts packed keys (sort value in the high word, position in the low word) by the high word; keys that come in position
// order leave in (value, position) order, i.e. this is the stable sort of the positions by value.  LSD radix, 11 bits a pass.
void sort_by_high_word(std::vector<uint64_t> &a, uint32_t max_value) {
    std::vector<uint64_t> b(a.size());
    const int bits = 32 - __builtin_clz(max_value | 1u);
    for (int shift = 0; shift < bits; shift += 11) {
        std::vector<size_t> cnt(2049, 0);
        for (uint64_t k : a) cnt[((k >> 32) >> shift & 2047u) + 1]++;
        for (int i = 0; i < 2048; ++i) cnt[i + 1] += cnt[i];
        for (uint64_t k : a) b[cnt[(k >> 32) >> shift & 2047u]++] = k;
        a.swap(b);
    }
}

// The task table that interleaves LIBRA_XCDS queues of positions into tasks[begin, end): entry LIBRA_XCDS*j + x is
// the j-th task of queue x.  Queues of different length are levelled (see below).
void interleave_queues(std::vector<libra_task_t> &tasks, size_t begin, size_t end, std::vector<size_t> (&queue)[LIBRA_XCDS], int noop_kind) {
    // level the queue lengths first: the last (lightest) tasks of a long queue move to the end of the shortest one;
    // what is left to fill with empty tasks is at most one slot per queue
    for (;;) {
        int lo = 0, hi = 0;
        for (int x = 1; x < LIBRA_XCDS; ++x) {
            if (queue[x].size() < queue[lo].size()) lo = x;
            if (queue[x].size() > queue[hi].size()) hi = x;
        }
        if (queue[hi].size() - queue[lo].size() <= 1) break;
        const size_t move = (queue[hi].size() - queue[lo].size()) / 2;
        queue[lo].insert(queue[lo].end(), queue[hi].end() - move, queue[hi].end());
        queue[hi].resize(queue[hi].size() - move);
    }
    size_t maxlen = 0;
    for (auto &q : queue) maxlen = std::max(maxlen, q.size());
    const libra_task_t noop{noop_kind, 0, 0, 0, 0, 0, 0u, 0u, 0u, 0u};
    std::vector<libra_task_t> out;
    out.reserve(maxlen * LIBRA_XCDS);
    for (size_t j = 0; j < maxlen; ++j)
        for (int x = 0; x < LIBRA_XCDS; ++x) out.push_back(j < queue[x].size() ? tasks[begin + queue[x][j]] : noop);
    while (!out.empty() && out.back().cost == 0 && out.back().blk_begin == out.back().blk_end &&
           out.back().res_begin == out.back().res_end && out.back().store_mask == 0 && out.back().atomic_mask == 0)
        out.pop_back();                                             // empty tasks after the last real one
    if (begin == 0 && end == tasks.size()) {
        tasks.swap(out);
    } else {
        tasks.erase(tasks.begin() + begin, tasks.begin() + end);
        tasks.insert(tasks.begin() + begin, out.begin(), out.end());
    }
}

// XCD-aware placement.  Workgroup k of a launch runs on XCD k mod LIBRA_XCDS and every XCD has its own L2, so
// two tasks share fetched rows of the dense operand only if they sit in the same residue class of the task table
// and close to each other.  Tasks of neighbouring windows (they tend to reference the same columns) form a group;
// groups go heaviest first, dealt in snake order to LIBRA_XCDS queues; the table interleaves the queues.  Queues
// of different length are levelled with empty tasks (no blocks, no entries, no output rows).
template <class GroupOf>
void xcd_order(std::vector<libra_task_t> &tasks, size_t begin, size_t end, GroupOf group_of, int noop_kind) {
    const size_t n = end - begin;
    if (n < 2 * LIBRA_XCDS) return;
    std::vector<std::pair<int64_t, size_t>> key(n);                 // (group, position in the heaviest-first list)
    for (size_t i = 0; i < n; ++i) key[i] = {group_of(tasks[begin + i], i), i};
    std::sort(key.begin(), key.end());
    struct Group { uint64_t cost; int64_t gid; size_t first, count; };
    std::vector<Group> groups;
    for (size_t i = 0; i < n;) {
        size_t j = i;
        uint64_t cost = 0;
        while (j < n && key[j].first == key[i].first) cost += tasks[begin + key[j++].second].cost;
        groups.push_back({cost, key[i].first, i, j - i});
        i = j;
    }
    std::stable_sort(groups.begin(), groups.end(), [](const Group &a, const Group &b) { return a.cost > b.cost; });
    std::vector<size_t> queue[LIBRA_XCDS];
    for (size_t r = 0; r < groups.size(); ++r) {
        const size_t round = r / LIBRA_XCDS, x = r % LIBRA_XCDS;
        std::vector<size_t> &q = queue[round & 1 ? LIBRA_XCDS - 1 - x : x];
        for (size_t k = 0; k < groups[r].count; ++k) q.push_back(key[groups[r].first + k].second);
    }
    interleave_queues(tasks, begin, end, queue, noop_kind);
}

// Segments of decomposed rows by column.  A long row's segments are runs of consecutive columns, and they add
// into C with atomics whichever die runs them.  So the segments are sorted by their first column and cut into
// LIBRA_XCDS runs of equal cost, one per die: a die then fetches rows of the dense operand from one column range
// only, in ascending order, instead of from all of it, and its L2 can hold them.  The other tasks are dealt to the
// dies heaviest first as before; each die's queue is merged by cost.
void place_segments_by_column(std::vector<libra_task_t> &tasks, const std::vector<int32_t> &first_col) {
    const size_t n = tasks.size();
    std::vector<size_t> seg, other;
    for (size_t i = 0; i < n; ++i) (tasks[i].kind == LIBRA_TASK_CHUNK ? seg : other).push_back(i);
    if (seg.size() < 8 * LIBRA_XCDS) return;
    {   // by first column, ties in table order (packed keys)
        std::vector<uint64_t> key(seg.size());
        uint32_t top = 0;
        for (size_t k = 0; k < seg.size(); ++k) {
            key[k] = ((uint64_t)(uint32_t)first_col[seg[k]] << 32) | (uint32_t)seg[k];
            top = std::max(top, (uint32_t)first_col[seg[k]]);
        }
        sort_by_high_word(key, top);
        for (size_t k = 0; k < seg.size(); ++k) seg[k] = (size_t)(key[k] & 0xffffffffu);
    }
    uint64_t total = 0;
    for (size_t i : seg) total += tasks[i].cost;
    std::vector<size_t> segq[LIBRA_XCDS], othq[LIBRA_XCDS], queue[LIBRA_XCDS];
    uint64_t run = 0;
    for (size_t i : seg) {
        const size_t x = std::min<uint64_t>(LIBRA_XCDS - 1, run * LIBRA_XCDS / std::max<uint64_t>(total, 1));
        segq[x].push_back(i);
        run += tasks[i].cost;
    }
    for (size_t r = 0; r < other.size(); ++r) {
        const size_t round = r / LIBRA_XCDS, x = r % LIBRA_XCDS;
        othq[round & 1 ? LIBRA_XCDS - 1 - x : x].push_back(other[r]);
    }
    for (int x = 0; x < LIBRA_XCDS; ++x) {
        queue[x].resize(segq[x].size() + othq[x].size());
        std::merge(othq[x].begin(), othq[x].end(), segq[x].begin(), segq[x].end(), queue[x].begin(),
                   [&](size_t a, size_t b) { return tasks[a].cost > tasks[b].cost; });
    }
    interleave_queues(tasks, 0, n, queue, LIBRA_TASK_WINDOW);
}

// The same for the flat residual segments of the SDDMM table (tasks[begin, end), in CSR order): a segment that lies inside
// one row is a run of ascending columns, i.e. it gathers rows of the second dense operand from a narrow column range.
// Those segments are sorted by first column and cut into LIBRA_XCDS equal runs, one per die; the others (several short
// rows each, columns from everywhere) are dealt round-robin as before and follow them in each die's queue.
void place_sddmm_segments_by_column(std::vector<libra_task_t> &tasks, size_t begin, size_t end, const std::vector<int32_t> &seg_col) {
    const size_t n = end - begin;
    std::vector<size_t> placed, other;
    for (size_t i = 0; i < n; ++i) (seg_col.at(i) >= 0 ? placed : other).push_back(i);
    if (placed.size() < 8 * LIBRA_XCDS) return;
    {
        std::vector<uint64_t> key(placed.size());
        uint32_t top = 0;
        for (size_t k = 0; k < placed.size(); ++k) {
            key[k] = ((uint64_t)(uint32_t)seg_col[placed[k]] << 32) | (uint32_t)placed[k];
            top = std::max(top, (uint32_t)seg_col[placed[k]]);
        }
        sort_by_high_word(key, top);
        for (size_t k = 0; k < placed.size(); ++k) placed[k] = (size_t)(key[k] & 0xffffffffu);
    }
    std::vector<size_t> queue[LIBRA_XCDS];
    for (size_t r = 0; r < placed.size(); ++r) queue[r * LIBRA_XCDS / placed.size()].push_back(placed[r]);
    for (size_t r = 0; r < other.size(); ++r) queue[r % LIBRA_XCDS].push_back(other[r]);
    interleave_queues(tasks, begin, end, queue, LIBRA_TASK_CHUNK);
}

// How much neighbouring windows overlap in the columns they reference, on an evenly spaced sample of groups of
// LIBRA_LOCALITY_WINDOWS windows: distinct columns of the group / sum of the distinct columns of its windows.
double neighbour_share(int64_t M, const int32_t *rowptr, const ColumnFetch &cols, int W, int threads) {
    const int64_t rows_per_group = (int64_t)W * LIBRA_LOCALITY_WINDOWS;
    const int64_t ngroups = (M + rows_per_group - 1) / rows_per_group;
    const int64_t nsample = share_samples(ngroups);
    int nthr = threads ? threads : (int)std::thread::hardware_concurrency();
    nthr = (int)std::max<int64_t>(1, std::min<int64_t>(nthr, nsample));
    std::vector<int64_t> together(nthr, 0), apart(nthr, 0);
    // the sampled groups are independent; a hub window's group alone can hold a large share of the nonzeros, so the
    // samples are dealt to the threads one by one rather than in ranges
    auto work = [&](int t) {
        std::vector<uint64_t> keys;
        for (int64_t k = t; k < nsample; k += nthr) {
            const int64_t g = sampled_group(k, ngroups, nsample);
            const int64_t r0 = g * rows_per_group, r1 = std::min(M, r0 + rows_per_group);
            keys.clear();
            const int32_t *col = cols(rowptr[r0], rowptr[r1]) - rowptr[r0];      // indexable by CSR position
            for (int64_t i = r0; i < r1; ++i)
                for (int32_t p = rowptr[i]; p < rowptr[i + 1]; ++p)
                    keys.push_back(((uint64_t)((i - r0) / W) << 32) | (uint32_t)col[p]);
            std::sort(keys.begin(), keys.end());
            apart[t] += std::unique(keys.begin(), keys.end()) - keys.begin();
            for (auto &x : keys) x &= 0xffffffffull;
            std::sort(keys.begin(), keys.end());
            together[t] += std::unique(keys.begin(), keys.end()) - keys.begin();
        }
    };
    if (nthr == 1) {
        work(0);
    } else {
        std::vector<std::exception_ptr> failed(nthr);
        std::vector<std::thread> pool;
        std::exception_ptr start_failed;
        pool.reserve(nthr);
        // a thread that cannot be started must not leave the started ones joinable (their destructor would terminate the
        // process): they are joined first, then the error travels on
        try {
            for (int t = 0; t < nthr; ++t)
                pool.emplace_back([&, t]() {
                    try { work(t); } catch (...) { failed[t] = std::current_exception(); }
                });
        } catch (...) { start_failed = std::current_exception(); }
        for (auto &th : pool) th.join();
        if (start_failed) std::rethrow_exception(start_failed);
        for (auto &f : failed)
            if (f) std::rethrow_exception(f);
    }
    int64_t tg = 0, ap = 0;
    for (int t = 0; t < nthr; ++t) { tg += together[t]; ap += apart[t]; }
    return ap ? (double)tg / (double)ap : 1.0;
}

}  // namespace

int libra::resolve_options(const libra_plan_opts_t *in, int vdt, Resolved &o) {
    libra_plan_opts_t z{};
    if (in) {
        if (in->struct_size != sizeof(libra_plan_opts_t)) return LIBRA_ERR_OPTION;
        z = *in;
    }
    o.mode = z.mode;
    if (o.mode < 0 || o.mode > 2) return LIBRA_ERR_OPTION;
    o.W = z.window_rows ? z.window_rows : 16;
    o.KB = z.block_cols ? z.block_cols : 16;
    o.tau_spmm = z.spmm_min_vec_nnz ? z.spmm_min_vec_nnz : 3;
    o.tau_sddmm = z.sddmm_min_blk_nnz ? z.sddmm_min_blk_nnz : 64;
    o.Ts = z.ts ? z.ts : 16;
    o.Cs = z.cs ? z.cs : 128;
    o.short_len = z.short_len ? z.short_len : 3;
    o.sddmm_Cs = z.sddmm_cs ? z.sddmm_cs : 128;
    o.sddmm_Ts = z.sddmm_ts ? z.sddmm_ts : 4;
    o.sddmm_min_dense_pct = z.sddmm_min_dense_pct;
    if (o.sddmm_min_dense_pct < 0 || o.sddmm_min_dense_pct > 100) return LIBRA_ERR_OPTION;
    o.threads = z.threads;
    if (o.W < 1 || o.W > 32 || o.KB < 1 || o.KB > 64 || o.tau_spmm < 1 || o.tau_sddmm < 1 || o.Ts < 1 ||
        o.Cs < 1 || o.short_len < 1 || o.sddmm_Cs < 1 || o.sddmm_Ts < 1 || o.threads < 0)
        return LIBRA_ERR_OPTION;
    o.fill = !(z.flags & LIBRA_FLAG_NO_FILL_PADDING);
    o.build_spmm = !(z.flags & LIBRA_FLAG_NO_SPMM);
    o.build_sddmm = !(z.flags & LIBRA_FLAG_NO_SDDMM);
    o.heavy_first = !(z.flags & LIBRA_FLAG_NATURAL_ORDER);
    if ((z.flags & LIBRA_FLAG_XCD_ORDER) && (z.flags & LIBRA_FLAG_NO_XCD_ORDER)) return LIBRA_ERR_OPTION;
    o.xcd_order = !o.heavy_first || (z.flags & LIBRA_FLAG_NO_XCD_ORDER) ? 0 : (z.flags & LIBRA_FLAG_XCD_ORDER) ? 1 : -1;
    if ((z.flags & LIBRA_FLAG_SEGMENTS_BY_COLUMN) && (z.flags & LIBRA_FLAG_SEGMENTS_BY_COST)) return LIBRA_ERR_OPTION;
    o.segments_by_column = o.heavy_first && !(z.flags & LIBRA_FLAG_SEGMENTS_BY_COST);
    o.two_kernels = (z.flags & LIBRA_FLAG_TWO_KERNELS) != 0;
    if (z.flags & ~511u) return LIBRA_ERR_OPTION;
    return LIBRA_OK;
}

// Shared tail of the host and the device planner: the flat SDDMM residual segments, the order of the task
// tables and the statistics.  Expects the sub-plans with their tasks in window order.
void libra::finish_plan(libra_plan_t *P, const ColumnFetch &cols, const int64_t *share) {
    const Resolved o = P->o;
    const int64_t M = P->M, nnz = P->nnz;
    const int32_t *rowptr = P->rowptr.data();
    SubPlan &sa = P->spmm, &sd = P->sddmm;
    libra_stats_t &st = P->stats;
    const int64_t nwin = (M + o.W - 1) / o.W;
    int xcd = o.xcd_order;
    const bool trace = std::getenv("LIBRA_TRACE") != nullptr;
    const auto t0 = std::chrono::steady_clock::now();
    auto mark = [&](const char *what) {
        if (trace) std::fprintf(stderr, "[finish_plan] %-34s %8.3f ms\n", what,
                                1e3 * std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count());
    };
    for (int64_t i = 0; i < M; ++i) {       // row lists of the edge softmax
        const int32_t n = rowptr[i + 1] - rowptr[i];
        if (n > LIBRA_SOFTMAX_LONG_ROW) P->long_rows.push_back((int32_t)i);
        else if (n > 64) P->medium_rows.push_back((int32_t)i);
    }
    // longest first: one workgroup takes a long row, and the longest one sets the time of the whole class
    std::stable_sort(P->long_rows.begin(), P->long_rows.end(), [&](int32_t a, int32_t b) {
        return rowptr[a + 1] - rowptr[a] > rowptr[b + 1] - rowptr[b];
    });
    if (!o.build_spmm) sa = SubPlan();
    if (!o.build_sddmm) sd = SubPlan();
    if (P->host_arrays) {
        sa.count_host_arrays();
        sd.count_host_arrays();
    }
    if (o.build_sddmm) {
        // scalar segments over the flat residual list (no atomics needed: each output has one writer)
        const int32_t nres = (int32_t)sd.n.res;
        const size_t nseg = ((size_t)nres + o.sddmm_Cs - 1) / o.sddmm_Cs;
        const bool derive = sd.seg_col.size() != nseg && P->host_arrays;
        if (sd.seg_col.size() != nseg) sd.seg_col.assign(nseg, -1);
        for (int32_t q = 0; q < nres; q += o.sddmm_Cs) {
            int32_t q1 = std::min(nres, q + o.sddmm_Cs);
            sd.tasks.push_back({LIBRA_TASK_CHUNK, 0, 0, 0, q, q1, 0u, 0u, 0u, (uint32_t)(2 * (q1 - q))});
            if (derive && sd.res_row[q] == sd.res_row[q1 - 1]) sd.seg_col[q / o.sddmm_Cs] = sd.res_col[q];
        }
    }
    mark("row lists, sddmm segments");
    // ---- ordering: heaviest first, so that the tail of the launch is made of light tasks ----
    st.neighbour_share = share ? (share[1] ? (double)share[0] / (double)share[1] : 1.0) : neighbour_share(M, rowptr, cols, o.W, o.threads);
    mark("neighbour share");
    if (o.heavy_first) {
        auto heavier = [](const libra_task_t &a, const libra_task_t &b) { return a.cost > b.cost; };
        {
            // heaviest first, the segments' first columns travelling with their tasks
            // (sorted as packed keys: descending cost, then position - i.e. a stable sort - without indirect compares)
            uint32_t top = 0;
            for (const libra_task_t &t : sa.tasks) top = std::max(top, t.cost);
            std::vector<uint64_t> ord(sa.tasks.size());
            for (size_t i = 0; i < ord.size(); ++i) ord[i] = ((uint64_t)(top - sa.tasks[i].cost) << 32) | (uint32_t)i;
            sort_by_high_word(ord, top);
            std::vector<libra_task_t> ts(ord.size());
            std::vector<int32_t> tc(ord.size(), -1);
            for (size_t i = 0; i < ord.size(); ++i) {
                const size_t from = (size_t)(ord[i] & 0xffffffffu);
                ts[i] = sa.tasks[from];
                tc[i] = sa.task_col.at(from);            // both planners fill one entry per task
            }
            sa.tasks.swap(ts);
            sa.task_col.swap(tc);
        }
        mark("spmm heaviest first");
        // SDDMM window tasks first (heaviest first); the flat residual segments stay behind them in order
        auto mid = std::stable_partition(sd.tasks.begin(), sd.tasks.end(),
                                         [](const libra_task_t &t) { return t.kind == LIBRA_TASK_WINDOW; });
        std::stable_sort(sd.tasks.begin(), mid, heavier);
        if (xcd < 0) P->o.xcd_order = xcd = st.neighbour_share <= LIBRA_SHARE_THRESHOLD;
        st.xcd_order = xcd;
        mark("sddmm window tasks first");
        if (!xcd && o.segments_by_column) {
            // the two tables are independent: the SDDMM one is placed on a second thread unless the caller asked for one
            const size_t nwt = (size_t)(mid - sd.tasks.begin());
            auto place_sd = [&]() { place_sddmm_segments_by_column(sd.tasks, nwt, sd.tasks.size(), sd.seg_col); };
            if (o.threads == 1) {
                place_segments_by_column(sa.tasks, sa.task_col);
                place_sd();
            } else {
                std::exception_ptr failed;          // an exception must not leave the thread's function
                std::thread other([&]() {
                    try { place_sd(); } catch (...) { failed = std::current_exception(); }
                });
                try {
                    place_segments_by_column(sa.tasks, sa.task_col);
                } catch (...) {
                    other.join();
                    throw;
                }
                other.join();
                if (failed) std::rethrow_exception(failed);
            }
        }
        if (xcd) {
            const int W = o.W;
            xcd_order(sa.tasks, 0, sa.tasks.size(), [W](const libra_task_t &t, size_t) {
                return (int64_t)(t.kind == LIBRA_TASK_WINDOW ? t.id : t.id / W) / LIBRA_LOCALITY_WINDOWS; }, LIBRA_TASK_WINDOW);
            // SDDMM: window tasks by window; the flat segments (still in CSR order here) in runs of consecutive segments
            const size_t nwt = (size_t)(mid - sd.tasks.begin());
            const size_t nseg = sd.tasks.size() - nwt;
            xcd_order(sd.tasks, nwt, nwt + nseg, [](const libra_task_t &, size_t i) {
                return (int64_t)(i / LIBRA_LOCALITY_SEGMENTS); }, LIBRA_TASK_CHUNK);
            xcd_order(sd.tasks, 0, nwt, [](const libra_task_t &t, size_t) {
                return (int64_t)t.id / LIBRA_LOCALITY_WINDOWS; }, LIBRA_TASK_CHUNK);
        }
    }
    mark("placement done");
    for (SubPlan *sp : {&sa, &sd}) {
        for (auto &t : sp->tasks) (t.kind == LIBRA_TASK_WINDOW ? sp->n_window_tasks : sp->n_chunk_tasks)++;
        sp->n.tasks = (int64_t)sp->tasks.size();
    }

    st.M = M; st.Kc = P->Kc; st.nnz = nnz; st.n_windows = nwin;
    if (o.build_spmm) {
        st.spmm_dense_vectors = sa.dense_vectors; st.spmm_blocks = sa.n.blocks; st.spmm_pad_slots = sa.pad_slots;
        st.spmm_dense_nnz = sa.n.dense; st.spmm_res_nnz = sa.n.res;
        st.spmm_tasks = (int64_t)sa.tasks.size(); st.spmm_chunk_tasks = sa.n_chunk_tasks;
        st.spmm_zero_rows = sa.n.zero_rows;
        st.spmm_short_rows = sa.short_rows; st.spmm_long_rows = sa.long_rows; st.spmm_split_rows = sa.split_rows;
        st.spmm_gather_rows = sa.dense_vectors + st.spmm_res_nnz;
    }
    if (o.build_sddmm) {
        st.sddmm_dense_vectors = sd.dense_vectors; st.sddmm_blocks = sd.n.blocks; st.sddmm_pad_slots = sd.pad_slots;
        st.sddmm_dense_nnz = sd.n.dense; st.sddmm_res_nnz = sd.n.res;
        st.sddmm_tasks = (int64_t)sd.tasks.size();
        st.sddmm_gather_rows = sd.dense_vectors + (int64_t)o.W * sd.n.blocks + 2 * st.sddmm_res_nnz;
    }
}

extern "C" int libra_plan(int64_t M, int64_t Kc, const int32_t *rowptr, const int32_t *col, const void *val,
                          int val_dtype, const libra_plan_opts_t *opts, libra_plan_t **out) {
    if (!out) return LIBRA_ERR_NULL;
    *out = nullptr;
    if (!rowptr) return LIBRA_ERR_NULL;
    if (M < 1 || Kc < 1) return LIBRA_ERR_SHAPE;
    if (M >= (1ll << 31) - 64 || Kc >= (1ll << 31)) return LIBRA_ERR_TOO_LARGE;
    if (val_dtype != LIBRA_F16 && val_dtype != LIBRA_BF16 && val_dtype != LIBRA_F32) return LIBRA_ERR_DTYPE;
    Resolved o{};
    if (int rc = resolve_options(opts, val_dtype, o)) return rc;
    // ---- validate the CSR arrays, O(nnz) ----
    if (rowptr[0] != 0) return LIBRA_ERR_ROWPTR;
    for (int64_t i = 0; i < M; ++i)
        if (rowptr[i + 1] < rowptr[i]) return LIBRA_ERR_ROWPTR;      // int32 rowptr: nnz < 2^31 by type
    const int64_t nnz = rowptr[M];
    if (nnz > 0 && (!col || !val)) return LIBRA_ERR_NULL;
    for (int64_t i = 0; i < M; ++i)
        for (int32_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            if (col[p] < 0 || col[p] >= Kc) return LIBRA_ERR_COLUMN;
            if (p > rowptr[i] && col[p] <= col[p - 1]) return LIBRA_ERR_UNSORTED;
        }

    auto t0 = std::chrono::steady_clock::now();
    libra_plan_t *P = new (std::nothrow) libra_plan_t();
    if (!P) return LIBRA_ERR_NOMEM;
    try {
        P->M = M; P->Kc = Kc; P->nnz = nnz; P->vdt = val_dtype; P->vsize = val_dtype == LIBRA_F32 ? 4 : 2;
        P->o = o;
        P->rowptr.assign(rowptr, rowptr + M + 1);
        Ctx c{M, nnz, rowptr, col, (const uint8_t *)val, P->vsize, o, (o.W * o.KB + 63) / 64};
        const int64_t nwin = (M + o.W - 1) / o.W;
        int nthr = o.threads ? o.threads : (int)std::thread::hardware_concurrency();
        nthr = (int)std::max<int64_t>(1, std::min<int64_t>(nthr, 64));
        // ranges of windows with about equal nnz, a few per thread
        const int64_t nranges = std::max<int64_t>(1, std::min<int64_t>(nwin, (int64_t)nthr * 4));
        std::vector<int64_t> cut(nranges + 1, 0);
        {
            int64_t w = 0;
            for (int64_t r = 1; r < nranges; ++r) {
                int64_t target = nnz / nranges * r;
                while (w < nwin && rowptr[std::min<int64_t>(M, w * o.W)] < target) ++w;
                cut[r] = std::max(cut[r - 1], std::min(w, nwin));
            }
            cut[nranges] = nwin;
        }
        std::vector<Part> parts(nranges);
        std::vector<std::thread> pool;
        std::vector<int> failed(nthr, 0);
        bool start_failed = false;
        pool.reserve(nthr);
        try {               // as above: started threads are joined before a failure to start another one is reported
            for (int t = 0; t < nthr; ++t)
                pool.emplace_back([&, t] {
                    try {
                        for (int64_t r = t; r < nranges; r += nthr) plan_range(c, cut[r], cut[r + 1], parts[r]);
                    } catch (...) { failed[t] = 1; }
                });
        } catch (...) { start_failed = true; }
        for (auto &th : pool) th.join();
        if (start_failed) throw std::bad_alloc();
        for (int f : failed) if (f) throw std::bad_alloc();

        SubPlan &sa = P->spmm, &sd = P->sddmm;
        sa.win_blkptr.push_back(0); sa.blk_valptr.push_back(0); sa.win_resptr.push_back(0);
        sd.win_blkptr.push_back(0); sd.blk_valptr.push_back(0);
        libra_stats_t &st = P->stats;
        for (auto &pt : parts) {
            st.n_vectors += pt.n_vectors;
            st.n_vectors_nnz1 += pt.n_vectors_nnz1;
            if (o.build_spmm) concat(sa, pt.spmm, true);
            if (o.build_sddmm) concat(sd, pt.sddmm, false);
        }
        parts.clear();
        if (o.build_sddmm && share_rule_fires(o, (int64_t)sd.dense_perm.size(), nnz)) {
            // the dense blocks hold too small a share of the nonzeros to pay: every nonzero takes the scalar path, i.e.
            // the sub-plan is what LIBRA_MODE_SCALAR_ONLY builds - the residual list is the matrix in CSR order
            SubPlan all;
            all.win_blkptr.assign((size_t)nwin + 1, 0);
            all.blk_valptr.push_back(0);
            all.res_perm.resize((size_t)nnz);
            all.res_row.resize((size_t)nnz);
            for (int64_t i = 0; i < M; ++i)
                for (int32_t q = rowptr[i]; q < rowptr[i + 1]; ++q) { all.res_perm[q] = q; all.res_row[q] = (int32_t)i; }
            all.res_col.assign(col, col + nnz);
            all.res_val.assign((const uint8_t *)val, (const uint8_t *)val + (size_t)nnz * P->vsize);
            sd = std::move(all);
        }
        finish_plan(P, [col](int64_t p0, int64_t) { return col + p0; });
        st.plan_seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    } catch (...) {
        delete P;
        return LIBRA_ERR_NOMEM;
    }
    *out = P;
    return LIBRA_OK;
}

static void fill_view(const libra_plan_t *P, const SubPlan &sp, bool spmm, libra_subplan_view_t *v) {
    std::memset(v, 0, sizeof *v);
    v->n_windows = (int64_t)sp.win_blkptr.size() - 1;
    v->n_blocks = sp.n_blocks();
    v->n_dense_nnz = (int64_t)sp.dense_perm.size();
    v->n_res_nnz = (int64_t)sp.res_perm.size();
    v->n_tasks = (int64_t)sp.tasks.size();
    v->n_zero_rows = (int64_t)sp.zero_rows.size();
    v->window_rows = P->o.W;
    v->block_cols = P->o.KB;
    v->words_per_block = (P->o.W * P->o.KB + 63) / 64;
    v->value_dtype = P->vdt;
    v->win_blkptr = sp.win_blkptr.data();
    v->blk_cols = sp.blk_cols.data();
    v->blk_bitmap = sp.blk_bitmap.data();
    v->blk_valptr = sp.blk_valptr.data();
    v->dense_val = sp.dense_val.data();
    v->dense_perm = sp.dense_perm.data();
    v->win_resptr = spmm ? sp.win_resptr.data() : nullptr;
    v->res_row = sp.res_row.data();
    v->res_col = sp.res_col.data();
    v->res_val = sp.res_val.data();
    v->res_perm = sp.res_perm.data();
    v->tasks = sp.tasks.data();
    v->zero_rows = sp.zero_rows.data();
}

extern "C" int libra_plan_export(const libra_plan_t *plan, int which, libra_subplan_view_t *view) {
    if (!plan || !view) return LIBRA_ERR_NULL;
    if (!plan->host_arrays) return LIBRA_ERR_NOT_BUILT;      // built on the device without a host copy
    if (which == 0) {
        if (!plan->o.build_spmm) return LIBRA_ERR_NOT_BUILT;
        fill_view(plan, plan->spmm, true, view);
    } else if (which == 1) {
        if (!plan->o.build_sddmm) return LIBRA_ERR_NOT_BUILT;
        fill_view(plan, plan->sddmm, false, view);
    } else {
        return LIBRA_ERR_OPTION;
    }
    return LIBRA_OK;
}

extern "C" int libra_plan_stats(const libra_plan_t *plan, libra_stats_t *stats) {
    if (!plan || !stats) return LIBRA_ERR_NULL;
    *stats = plan->stats;
    return LIBRA_OK;
}

extern "C" void libra_plan_destroy(libra_plan_t *plan) { delete plan; }

extern "C" int libra_version(void) { return LIBRA_VERSION; }

extern "C" const char *libra_strerror(int code) {
    switch (code) {
    case LIBRA_OK: return "ok";
    case LIBRA_ERR_NULL: return "a required pointer is NULL";
    case LIBRA_ERR_SHAPE: return "matrix or operand shape out of range";
    case LIBRA_ERR_ROWPTR: return "rowptr must start at 0 and be non-decreasing";
    case LIBRA_ERR_COLUMN: return "column index outside [0, Kc)";
    case LIBRA_ERR_UNSORTED: return "column indices must be strictly increasing inside a row";
    case LIBRA_ERR_TOO_LARGE: return "size does not fit in 31 bits";
    case LIBRA_ERR_DTYPE: return "unknown value type";
    case LIBRA_ERR_OPTION: return "plan option out of range";
    case LIBRA_ERR_UNSUPPORTED: return "request not supported by the gfx950 kernels";
    case LIBRA_ERR_NOT_UPLOADED: return "plan has no device copy (call libra_plan_upload)";
    case LIBRA_ERR_BUFFER: return "device buffer too small or misaligned";
    case LIBRA_ERR_NOT_BUILT: return "the required sub-plan was not built";
    case LIBRA_ERR_HIP: return "HIP runtime error";
    case LIBRA_ERR_NOMEM: return "host allocation failed";
    default: return "unknown error";
    }
}
