// Host-side graph analysis behind dg4_build_levels (paper Section 3.2):
// validation, logic levels (Eq. 1), the (level, id) order and the cone_k
// neighbour rows with relation codes, plus the upload of the device tables.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <queue>
#include <system_error>
#include <thread>

#include "dg4_internal.h"

namespace {

struct Fanins {
    std::vector<int32_t> src;   // [2n], -1 = absent
    std::vector<uint8_t> inv;   // [2n]
};

int collect_fanins(int64_t n, int64_t e, const int32_t* es, const int32_t* ed, const uint8_t* ei, Fanins& f)
{
    f.src.assign(2 * (size_t)n, -1);
    f.inv.assign(2 * (size_t)n, 0);
    for (int64_t i = 0; i < e; ++i) {
        const int64_t u = es[i], v = ed[i];
        if (u < 0 || u >= n || v < 0 || v >= n) return DG4_ERANGE;
        if (ei[i] > 1) return DG4_EINVAL;
        if (u == v) return DG4_ECYCLE;
        int32_t* slot = &f.src[2 * v];
        if (slot[0] < 0) {
            slot[0] = (int32_t)u; f.inv[2 * v] = ei[i];
        } else if (slot[1] < 0) {
            if (slot[0] == u) return DG4_EFANIN;
            slot[1] = (int32_t)u; f.inv[2 * v + 1] = ei[i];
        } else {
            return DG4_EFANIN;
        }
    }
    return DG4_OK;
}

// Eq. 1 as a longest-path recursion over fanins, run as an explicit-stack
// depth-first search; a node met again while still open closes a cycle.
int longest_path_levels(int64_t n, const Fanins& f, std::vector<int32_t>& level)
{
    enum : uint8_t { NEW = 0, OPEN = 1, DONE = 2 };
    std::vector<uint8_t> state((size_t)n, NEW);
    std::vector<int32_t> stack;
    level.assign((size_t)n, 0);
    for (int64_t root = 0; root < n; ++root) {
        if (state[root] != NEW) continue;
        stack.push_back((int32_t)root);
        while (!stack.empty()) {
            const int32_t v = stack.back();
            if (state[v] == DONE) { stack.pop_back(); continue; }
            state[v] = OPEN;
            bool ready = true;
            int32_t best = -1;
            for (int k = 0; k < 2; ++k) {
                const int32_t u = f.src[2 * (size_t)v + k];
                if (u < 0) continue;
                if (state[u] == DONE) { best = std::max(best, level[u]); continue; }
                if (state[u] == OPEN) return DG4_ECYCLE;
                stack.push_back(u);
                ready = false;
            }
            if (ready) { level[v] = best + 1; state[v] = DONE; stack.pop_back(); }
        }
    }
    return DG4_OK;
}

int check_hint(int64_t n, const Fanins& f, const int32_t* hint)
{
    for (int64_t v = 0; v < n; ++v) {
        if (hint[v] < 0) return DG4_EHINT;
        const bool pi = f.src[2 * v] < 0;
        if (pi && hint[v] != 0) return DG4_EHINT;
        for (int k = 0; k < 2; ++k) {
            const int32_t u = f.src[2 * v + k];
            if (u >= 0 && hint[u] >= hint[v]) return DG4_EHINT;
        }
    }
    return DG4_OK;
}

// cone_j(v) = {v} U cone_{j-1}(fanin0) U cone_{j-1}(fanin1), built hop by hop
// as sorted merges; every entry carries its smallest hop count and, for hop 1,
// the inverter flag of the edge. Rows stay sorted by id throughout.
struct ConeTable {
    int width = 1;                   // slots per node
    std::vector<int32_t> id;         // [n*width], unused slots = -1
    std::vector<uint8_t> hop;        // smallest hop
    std::vector<uint8_t> inv;        // inverter flag where hop == 1
    std::vector<uint8_t> cnt;        // [n]
};

void cone_step(int64_t n, const Fanins& f, const ConeTable& prev, ConeTable& next)
{
    next.width = 2 * prev.width + 1;
    next.id.assign((size_t)n * next.width, -1);
    next.hop.assign((size_t)n * next.width, 0);
    next.inv.assign((size_t)n * next.width, 0);
    next.cnt.assign((size_t)n, 0);
    for (int64_t v = 0; v < n; ++v) {
        int32_t* oid = &next.id[(size_t)v * next.width];
        uint8_t* ohop = &next.hop[(size_t)v * next.width];
        uint8_t* oinv = &next.inv[(size_t)v * next.width];
        int cnt = 0;
        // three sorted streams: {v}, cone(f0) with hops+1, cone(f1) with hops+1
        const int32_t f0 = f.src[2 * v], f1 = f.src[2 * v + 1];
        const int32_t* ida = f0 >= 0 ? &prev.id[(size_t)f0 * prev.width] : nullptr;
        const int32_t* idb = f1 >= 0 ? &prev.id[(size_t)f1 * prev.width] : nullptr;
        const uint8_t* ha = f0 >= 0 ? &prev.hop[(size_t)f0 * prev.width] : nullptr;
        const uint8_t* hb = f1 >= 0 ? &prev.hop[(size_t)f1 * prev.width] : nullptr;
        const int na = f0 >= 0 ? prev.cnt[f0] : 0, nb = f1 >= 0 ? prev.cnt[f1] : 0;
        int ia = 0, ib = 0;
        bool self_out = false;
        while (ia < na || ib < nb || !self_out) {
            int64_t best = INT64_MAX;
            if (ia < na) best = std::min<int64_t>(best, ida[ia]);
            if (ib < nb) best = std::min<int64_t>(best, idb[ib]);
            if (!self_out) best = std::min<int64_t>(best, v);
            uint8_t h = 255, iv = 0;
            if (!self_out && best == v) { h = 0; self_out = true; }
            if (ia < na && ida[ia] == best) {
                const uint8_t hh = (uint8_t)(ha[ia] + 1);
                if (hh < h) { h = hh; iv = hh == 1 ? f.inv[2 * v] : 0; }
                ++ia;
            }
            if (ib < nb && idb[ib] == best) {
                const uint8_t hh = (uint8_t)(hb[ib] + 1);
                if (hh < h) { h = hh; iv = hh == 1 ? f.inv[2 * v + 1] : 0; }
                ++ib;
            }
            oid[cnt] = (int32_t)best; ohop[cnt] = h; oinv[cnt] = iv; ++cnt;
        }
        next.cnt[v] = (uint8_t)cnt;
    }
}

// Cones deeper than three hops (up to 2^(k+1)-1 gates, usually far fewer): one backward search per
// gate over the fanin table, frontier by frontier, so that the first visit fixes the shortest hop;
// a per-gate stamp marks what has been reached. Rows are then sorted by id.
void deep_cones(dg4_graph* g, const Fanins& f)
{
    const int64_t n = g->n;
    // contiguous ranges of gates, one per host thread; the pieces are joined in order
    const int64_t want = std::max<int64_t>(1, std::min<int64_t>(16, (int64_t)std::thread::hardware_concurrency()));
    const int n_parts = (int)std::max<int64_t>(1, std::min<int64_t>(want, n / 4096));
    struct Part { std::vector<int32_t> idx; std::vector<uint8_t> rel; std::vector<int32_t> cnt; bool failed = false; };
    std::vector<Part> parts((size_t)n_parts);
    auto work = [&](int t) {
        Part& out = parts[(size_t)t];
        try {
            const int64_t v0 = n * t / n_parts, v1 = n * (t + 1) / n_parts;
            std::vector<int32_t> seen((size_t)n, -1);
            std::vector<std::pair<int32_t, uint8_t>> row;       // (id, code)
            std::vector<int32_t> frontier, next;
            out.cnt.reserve((size_t)(v1 - v0));
            for (int64_t v = v0; v < v1; ++v) {
                row.clear(); frontier.clear();
                row.emplace_back((int32_t)v, (uint8_t)0);
                seen[v] = (int32_t)v;
                frontier.push_back((int32_t)v);
                for (int hop = 1; hop <= g->hops && !frontier.empty(); ++hop) {
                    next.clear();
                    for (const int32_t w : frontier)
                        for (int i = 0; i < 2; ++i) {
                            const int32_t u = f.src[2 * (size_t)w + i];
                            if (u < 0 || seen[u] == (int32_t)v) continue;
                            seen[u] = (int32_t)v;
                            row.emplace_back(u, hop == 1 ? (uint8_t)(1 + f.inv[2 * (size_t)w + i]) : (uint8_t)3);
                            next.push_back(u);
                        }
                    frontier.swap(next);
                }
                std::sort(row.begin(), row.end());
                for (const auto& r : row) { out.idx.push_back(r.first); out.rel.push_back(r.second); }
                out.cnt.push_back((int32_t)row.size());
            }
        } catch (...) {
            out.failed = true;
        }
    };
    {
        std::vector<std::thread> threads;
        for (int t = 1; t < n_parts; ++t) threads.emplace_back(work, t);
        work(0);
        for (auto& th : threads) th.join();
    }
    for (const Part& part : parts)
        if (part.failed) throw std::bad_alloc();
    g->nbr_ptr.assign((size_t)n + 1, 0);
    size_t total = 0;
    for (const Part& part : parts) total += part.idx.size();
    g->nbr_idx.clear(); g->nbr_rel.clear();
    g->nbr_idx.reserve(total); g->nbr_rel.reserve(total);
    int64_t v = 0;
    for (const Part& part : parts) {
        g->nbr_idx.insert(g->nbr_idx.end(), part.idx.begin(), part.idx.end());
        g->nbr_rel.insert(g->nbr_rel.end(), part.rel.begin(), part.rel.end());
        for (const int32_t c : part.cnt) { g->nbr_ptr[(size_t)v + 1] = g->nbr_ptr[(size_t)v] + c; ++v; }
    }
    g->nnz = (int64_t)g->nbr_idx.size();
}

// Graph partition and updating strategy (Section 3.3, Algorithm 1; Section 3.4, Algorithm 2) turned
// into neighbour rows. Every root gets the running number of its mini-batch (lists by ascending
// level, inside a list the roots of the stride loop, then the unread gates, then the gates left in
// no cone, each part by ascending id); a gate is computed by the smallest number among the cones
// that hold it, and keeps the entries of its cone row that lie in one of that mini-batch's cones
// together with it. Rows of g hold cone_hops(v), ascending id, on entry.
// Algorithm 1's lists (g->cone_root, cone_group_level, cone_group_ptr) and the running number of the
// mini-batch of every root (-1 for gates that root no cone). Returns the number of mini-batches.
int32_t collect_cones(dg4_graph* g, const Fanins& f, int32_t stride, int32_t batch, std::vector<int32_t>& root_stage)
{
    const int64_t n = g->n;
    const int32_t k = g->hops;
    enum : uint8_t { STRIDE = 0, UNREAD = 1, LEFT = 2, NONE = 255 };
    std::vector<uint8_t> kind((size_t)n, NONE), read((size_t)n, 0), covered((size_t)n, 0);
    for (int64_t v = 0; v < n; ++v)
        for (int i = 0; i < 2; ++i)
            if (f.src[2 * (size_t)v + i] >= 0) read[(size_t)f.src[2 * (size_t)v + i]] = 1;
    for (int64_t v = 0; v < n; ++v) {
        const int32_t l = g->level[v];
        if (l >= k && (l - k) % stride == 0) kind[v] = STRIDE;
        else if (!read[v]) kind[v] = UNREAD;
        if (kind[v] != NONE)
            for (int64_t j = g->nbr_ptr[v]; j < g->nbr_ptr[v + 1]; ++j) covered[(size_t)g->nbr_idx[j]] = 1;
    }
    for (int64_t v = 0; v < n; ++v)
        if (!covered[v]) kind[v] = LEFT;
    // the lists, and the mini-batch number of every root
    root_stage.assign((size_t)n, -1);
    int32_t stage = 0;
    for (int32_t l = 0; l <= g->max_level; ++l) {
        const size_t first_cone = g->cone_root.size();
        for (uint8_t part = STRIDE; part <= LEFT; ++part)
            for (int64_t q = g->level_ptr[l]; q < g->level_ptr[l + 1]; ++q)
                if (kind[(size_t)g->order[q]] == part) g->cone_root.push_back(g->order[q]);
        const size_t cones = g->cone_root.size() - first_cone;
        if (!cones) continue;
        g->cone_group_level.push_back(l);
        g->cone_group_ptr.push_back((int64_t)first_cone);
        for (size_t c = 0; c < cones; ++c) root_stage[(size_t)g->cone_root[first_cone + c]] = stage + (int32_t)(c / (size_t)batch);
        stage += (int32_t)((cones + (size_t)batch - 1) / (size_t)batch);
    }
    g->cone_group_ptr.push_back((int64_t)g->cone_root.size());
    g->stride = stride; g->batch_cones = batch;
    return stage;
}

// marks[j] = 1 for the entries j of row(v) that also lie in row(r) (two rows of ascending ids)
inline void mark_common(const dg4_graph* g, int32_t v, int32_t r, uint8_t* marks)
{
    int64_t a = g->nbr_ptr[v], b = g->nbr_ptr[r];
    const int64_t a0 = a, a1 = g->nbr_ptr[v + 1], b1 = g->nbr_ptr[r + 1];
    while (a < a1 && b < b1) {
        const int32_t x = g->nbr_idx[a], y = g->nbr_idx[b];
        if (x == y) { marks[a - a0] = 1; ++a; ++b; }
        else if (x < y) ++a;
        else ++b;
    }
}

void restrict_rows_to_partition(dg4_graph* g, const Fanins& f, int32_t stride, int32_t batch)
{
    const int64_t n = g->n;
    std::vector<int32_t> root_stage;
    collect_cones(g, f, stride, batch, root_stage);
    // the mini-batch that computes a gate: the first one that holds it
    g->stage.assign((size_t)n, INT32_MAX);
    for (const int32_t r : g->cone_root)
        for (int64_t j = g->nbr_ptr[r]; j < g->nbr_ptr[r + 1]; ++j) {
            int32_t& s = g->stage[(size_t)g->nbr_idx[j]];
            s = std::min(s, root_stage[(size_t)r]);
        }
    // entries kept: u in cone(v) and in cone(r), for the roots r of that mini-batch with v in cone(r)
    std::vector<uint8_t> keep((size_t)g->nnz, 0);
    for (const int32_t r : g->cone_root) {
        const int64_t r0 = g->nbr_ptr[r], r1 = g->nbr_ptr[r + 1];
        for (int64_t j = r0; j < r1; ++j) {
            const int32_t v = g->nbr_idx[j];
            if (g->stage[(size_t)v] == root_stage[(size_t)r]) mark_common(g, v, r, &keep[(size_t)g->nbr_ptr[v]]);
        }
    }
    int64_t out = 0;
    for (int64_t v = 0; v < n; ++v) {
        const int64_t lo = g->nbr_ptr[v], hi = g->nbr_ptr[v + 1];
        g->nbr_ptr[v] = out;
        for (int64_t j = lo; j < hi; ++j)
            if (keep[(size_t)j]) { g->nbr_idx[(size_t)out] = g->nbr_idx[(size_t)j]; g->nbr_rel[(size_t)out] = g->nbr_rel[(size_t)j]; ++out; }
    }
    g->nbr_ptr[n] = out; g->nnz = out;
    g->nbr_idx.resize((size_t)out); g->nbr_rel.resize((size_t)out);
}

// (level, id) order of g->level by a counting sort: level_ptr, order, pos
void sort_by_level(dg4_graph* g)
{
    const int64_t n = g->n;
    g->max_level = 0;
    for (int64_t v = 0; v < n; ++v) g->max_level = std::max(g->max_level, g->level[v]);
    g->level_ptr.assign((size_t)g->max_level + 2, 0);
    for (int64_t v = 0; v < n; ++v) ++g->level_ptr[(size_t)g->level[v] + 1];
    for (int32_t l = 0; l <= g->max_level; ++l) g->level_ptr[l + 1] += g->level_ptr[l];
    g->order.resize((size_t)n);
    g->pos.resize((size_t)n);
    std::vector<int64_t> cur(g->level_ptr.begin(), g->level_ptr.end() - 1);
    for (int64_t v = 0; v < n; ++v) {
        const int64_t p = cur[g->level[v]]++;
        g->order[p] = (int32_t)v; g->pos[v] = (int32_t)p;
    }
}

// The ablation without marks (Section 4.4): every mini-batch recomputes all the gates of its cones
// from their initial features, reading nothing from earlier mini-batches, and the last result of a
// gate stands. As a graph: one COPY of a gate per mini-batch that holds it (numbered mini-batch
// after mini-batch, inside one by ascending gate id), whose row holds the copies, in the same
// mini-batch, of the sources that the mini-batch's cones show together with it. g holds the whole
// cone rows of the circuit on entry and the expanded graph on return.
int expand_without_marks(dg4_graph* g, const Fanins& f, int32_t stride, int32_t batch)
{
    const int64_t n = g->n;
    std::vector<int32_t> root_stage;
    const int32_t stages = collect_cones(g, f, stride, batch, root_stage);
    std::vector<int32_t> copy_of, level2, out_and2, out_not2, idx2;
    std::vector<uint8_t> rel2;
    std::vector<int64_t> ptr2(1, 0);
    std::vector<int32_t> last_copy((size_t)n, -1), slot((size_t)n, -1);
    std::vector<int32_t> members;
    std::vector<int64_t> off;                 // start of each member's flags
    std::vector<uint8_t> keep;
    size_t c0 = 0;                            // first cone of the mini-batch
    for (int32_t b = 0; b < stages; ++b) {
        size_t c1 = c0;
        while (c1 < g->cone_root.size() && root_stage[(size_t)g->cone_root[c1]] == b) ++c1;
        members.clear();
        for (size_t c = c0; c < c1; ++c) {
            const int32_t r = g->cone_root[c];
            members.insert(members.end(), g->nbr_idx.begin() + g->nbr_ptr[r], g->nbr_idx.begin() + g->nbr_ptr[r + 1]);
        }
        std::sort(members.begin(), members.end());
        members.erase(std::unique(members.begin(), members.end()), members.end());
        const int64_t first = (int64_t)copy_of.size();
        if (first + (int64_t)members.size() >= (int64_t)0x3FFFFFFF) return DG4_EUNSUPPORTED;
        off.assign(members.size() + 1, 0);
        for (size_t i = 0; i < members.size(); ++i) {
            const int32_t v = members[i];
            slot[(size_t)v] = (int32_t)i;
            off[i + 1] = off[i] + (g->nbr_ptr[v + 1] - g->nbr_ptr[v]);
        }
        keep.assign((size_t)off.back(), 0);
        for (size_t c = c0; c < c1; ++c) {
            const int32_t r = g->cone_root[c];
            for (int64_t j = g->nbr_ptr[r]; j < g->nbr_ptr[r + 1]; ++j) {
                const int32_t v = g->nbr_idx[j];
                mark_common(g, v, r, &keep[(size_t)off[(size_t)slot[(size_t)v]]]);
            }
        }
        for (size_t i = 0; i < members.size(); ++i) {
            const int32_t v = members[i];
            copy_of.push_back(v);
            level2.push_back(g->level[v]);
            out_and2.push_back(g->out_and[v]); out_not2.push_back(g->out_not[v]);
            last_copy[(size_t)v] = (int32_t)(first + (int64_t)i);
            for (int64_t j = g->nbr_ptr[v]; j < g->nbr_ptr[v + 1]; ++j)
                if (keep[(size_t)(off[i] + j - g->nbr_ptr[v])]) {
                    idx2.push_back((int32_t)(first + slot[(size_t)g->nbr_idx[j]]));
                    rel2.push_back(g->nbr_rel[j]);
                }
            ptr2.push_back((int64_t)idx2.size());
        }
        c0 = c1;
    }
    g->n = (int64_t)copy_of.size();
    g->nnz = (int64_t)idx2.size();
    g->level.swap(level2); g->out_and.swap(out_and2); g->out_not.swap(out_not2);
    g->nbr_ptr.swap(ptr2); g->nbr_idx.swap(idx2); g->nbr_rel.swap(rel2);
    if (!g->eq1_level.empty()) {
        std::vector<int32_t> e2(copy_of.size());
        for (size_t c = 0; c < copy_of.size(); ++c) e2[c] = g->eq1_level[(size_t)copy_of[c]];
        g->eq1_level.swap(e2);
    }
    g->copy_of.swap(copy_of); g->last_copy.swap(last_copy);
    g->marks = false;
    sort_by_level(g);
    return DG4_OK;
}

int build_graph(int64_t n, int64_t e, const int32_t* es, const int32_t* ed, const uint8_t* ei, int32_t hops,
                const int32_t* level_hint, int32_t stride, int32_t batch, bool marks, dg4_graph** out);

}  // namespace

extern "C" int dg4_build_levels(int64_t n, int64_t e, const int32_t* es, const int32_t* ed,
                                const uint8_t* ei, int32_t hops, const int32_t* level_hint,
                                dg4_graph** out)
{
    return build_graph(n, e, es, ed, ei, hops, level_hint, 0, 0, true, out);
}

extern "C" int dg4_build_partitioned(int64_t n, int64_t e, const int32_t* es, const int32_t* ed,
                                     const uint8_t* ei, int32_t hops, const int32_t* level_hint,
                                     int32_t stride, int32_t batch_cones, int32_t marks, dg4_graph** out)
{
    if (hops < 1 || hops > DG4_MAX_HOPS) return DG4_EUNSUPPORTED;
    if (stride < 1 || stride >= hops || batch_cones < 1 || (marks != 0 && marks != 1)) return DG4_EINVAL;
    return build_graph(n, e, es, ed, ei, hops, level_hint, stride, batch_cones, marks != 0, out);
}

namespace {

// stride == 0: plain cone rows; else the rows of the partitioned update (without marks: of its copies)
int build_graph(int64_t n, int64_t e, const int32_t* es, const int32_t* ed, const uint8_t* ei, int32_t hops,
                const int32_t* level_hint, int32_t stride, int32_t batch, bool marks, dg4_graph** out)
{
    if (!out || n < 0 || e < 0 || (e > 0 && (!es || !ed || !ei))) return DG4_EINVAL;
    if (hops < 1 || hops > DG4_MAX_HOPS) return DG4_EUNSUPPORTED;
    if (n >= (int64_t)0x3FFFFFFF) return DG4_EUNSUPPORTED;     // 30-bit packed indices
    try {
        Fanins f;
        int rc = collect_fanins(n, e, es, ed, ei, f);
        if (rc != DG4_OK) return rc;
        dg4_graph* g = new dg4_graph();
        std::unique_ptr<dg4_graph> guard(g);
        g->n = n; g->e = e; g->hops = hops;
        rc = longest_path_levels(n, f, g->level);
        if (rc != DG4_OK) return rc;
        if (level_hint) {
            rc = check_hint(n, f, level_hint);
            if (rc != DG4_OK) return rc;
            g->eq1_level = g->level;
            g->level.assign(level_hint, level_hint + n);
        }
        // (level, id) order by a counting sort
        g->max_level = 0;
        for (int64_t v = 0; v < n; ++v) g->max_level = std::max(g->max_level, g->level[v]);
        g->level_ptr.assign((size_t)g->max_level + 2, 0);
        for (int64_t v = 0; v < n; ++v) ++g->level_ptr[(size_t)g->level[v] + 1];
        for (int32_t l = 0; l <= g->max_level; ++l) g->level_ptr[l + 1] += g->level_ptr[l];
        g->order.resize((size_t)n);
        g->pos.resize((size_t)n);
        {
            std::vector<int64_t> cur(g->level_ptr.begin(), g->level_ptr.end() - 1);
            for (int64_t v = 0; v < n; ++v) {
                const int64_t p = cur[g->level[v]]++;
                g->order[p] = (int32_t)v; g->pos[v] = (int32_t)p;
            }
        }
        if (hops > 3) {
            deep_cones(g, f);
        } else {
        // cones, hop by hop
        ConeTable a, b;
        a.width = 1;
        a.id.resize((size_t)n); a.hop.assign((size_t)n, 0); a.inv.assign((size_t)n, 0); a.cnt.assign((size_t)n, 1);
        for (int64_t v = 0; v < n; ++v) a.id[v] = (int32_t)v;
        for (int h = 0; h < hops; ++h) { cone_step(n, f, a, b); std::swap(a, b); }
        g->nbr_ptr.resize((size_t)n + 1);
        int64_t nnz = 0;
        for (int64_t v = 0; v < n; ++v) { g->nbr_ptr[v] = nnz; nnz += a.cnt[v]; }
        g->nbr_ptr[n] = nnz; g->nnz = nnz;
        g->nbr_idx.resize((size_t)nnz);
        g->nbr_rel.resize((size_t)nnz);
        for (int64_t v = 0; v < n; ++v) {
            const size_t base = (size_t)v * a.width;
            for (int j = 0; j < a.cnt[v]; ++j) {
                const uint8_t h = a.hop[base + j];
                g->nbr_idx[g->nbr_ptr[v] + j] = a.id[base + j];
                g->nbr_rel[g->nbr_ptr[v] + j] = h == 0 ? 0 : h == 1 ? (uint8_t)(1 + a.inv[base + j]) : 3;
            }
        }
        }
        // Fanout counts of the structural encoding (Section 3.5, Eq. 2), gathered from the fanin
        // table: a reader with one fanin is a NOT/buffer gate; inverted uses by AND gates share the
        // one inverter of the signal; plain uses by AND gates count one by one.
        g->out_and.assign((size_t)n, 0);
        g->out_not.assign((size_t)n, 0);
        {
            std::vector<uint8_t> inverter((size_t)n, 0);
            for (int64_t v = 0; v < n; ++v) {
                const int32_t a0 = f.src[2 * (size_t)v], a1 = f.src[2 * (size_t)v + 1];
                if (a0 < 0) continue;                                   // primary input
                if (a1 < 0) { ++g->out_not[a0]; continue; }             // v is a NOT / buffer gate
                for (int k = 0; k < 2; ++k) {
                    const int32_t u = f.src[2 * (size_t)v + k];
                    if (f.inv[2 * (size_t)v + k]) inverter[u] = 1; else ++g->out_and[u];
                }
            }
            for (int64_t v = 0; v < n; ++v) g->out_not[v] += inverter[v];
        }
        if (stride > 0 && marks) restrict_rows_to_partition(g, f, stride, batch);
        if (stride > 0 && !marks) {
            rc = expand_without_marks(g, f, stride, batch);
            if (rc != DG4_OK) return rc;
        }
        // the shallower Eq. 1 levelling, if the caller's is deeper
        if (!g->eq1_level.empty()) {
            int32_t deepest = 0;
            for (const int32_t l : g->eq1_level) deepest = std::max(deepest, l);
            if (deepest < g->max_level) {
                g->eq1_level_ptr.assign((size_t)deepest + 2, 0);
                for (const int32_t l : g->eq1_level) ++g->eq1_level_ptr[(size_t)l + 1];
                for (int32_t l = 0; l <= deepest; ++l) g->eq1_level_ptr[l + 1] += g->eq1_level_ptr[l];
            } else {
                g->eq1_level.clear();
            }
        }
        *out = guard.release();
        return DG4_OK;
    } catch (const std::bad_alloc&) {
        return DG4_ENOMEM;
    } catch (...) {
        return DG4_EINVAL;
    }
}

}  // namespace

extern "C" int dg4_graph_array(const dg4_graph* g, int which, const void** host_ptr, int64_t* count)
{
    if (!g || !host_ptr || !count) return DG4_EINVAL;
    switch (which) {
    case DG4_LEVEL: *host_ptr = g->level.data(); *count = g->n; break;
    case DG4_ORDER: *host_ptr = g->order.data(); *count = g->n; break;
    case DG4_LEVEL_PTR: *host_ptr = g->level_ptr.data(); *count = (int64_t)g->level_ptr.size(); break;
    case DG4_NBR_PTR: *host_ptr = g->nbr_ptr.data(); *count = g->n + 1; break;
    case DG4_NBR_IDX: *host_ptr = g->nbr_idx.data(); *count = g->nnz; break;
    case DG4_NBR_REL: *host_ptr = g->nbr_rel.data(); *count = g->nnz; break;
    case DG4_OUT_AND: *host_ptr = g->out_and.data(); *count = g->n; break;
    case DG4_OUT_NOT: *host_ptr = g->out_not.data(); *count = g->n; break;
    case DG4_FLOW_ORDER:
    case DG4_FLOW_TILE_PTR: {
        dg4_graph* m = const_cast<dg4_graph*>(g);            // the schedule is built on first use, under the lock
        std::lock_guard<std::mutex> lock(m->mu);
        if (m->flow_tile_ptr.empty()) {
            const int rc = dg4_flow_schedule(m);
            if (rc != DG4_OK) return rc;
        }
        if (which == DG4_FLOW_ORDER) { *host_ptr = g->flow_order.data(); *count = g->n; }
        else { *host_ptr = g->flow_tile_ptr.data(); *count = (int64_t)g->flow_tile_ptr.size(); }
        break;
    }
    case DG4_PAIR_ORDER:
    case DG4_PAIR_TILE_PTR: {
        dg4_graph* m = const_cast<dg4_graph*>(g);
        std::lock_guard<std::mutex> lock(m->mu);
        if (m->pair_tile_ptr.empty()) {
            const int rc = dg4_pair_schedule(m);
            if (rc != DG4_OK) return rc;
        }
        if (which == DG4_PAIR_ORDER) { *host_ptr = g->pair_order.data(); *count = g->n; }
        else { *host_ptr = g->pair_tile_ptr.data(); *count = (int64_t)g->pair_tile_ptr.size(); }
        break;
    }
    case DG4_CONE_ROOT:
    case DG4_CONE_GROUP_LEVEL:
    case DG4_CONE_GROUP_PTR:
    case DG4_STAGE:
        if (g->stride == 0) return DG4_EINVAL;
        if (which == DG4_STAGE && !g->marks) return DG4_EINVAL;                  // graphs without marks have copies instead
        if (which == DG4_CONE_ROOT) { *host_ptr = g->cone_root.data(); *count = (int64_t)g->cone_root.size(); }
        else if (which == DG4_CONE_GROUP_LEVEL) { *host_ptr = g->cone_group_level.data(); *count = (int64_t)g->cone_group_level.size(); }
        else if (which == DG4_CONE_GROUP_PTR) { *host_ptr = g->cone_group_ptr.data(); *count = (int64_t)g->cone_group_ptr.size(); }
        else { *host_ptr = g->stage.data(); *count = g->n; }
        break;
    case DG4_COPY_OF:
    case DG4_LAST_COPY:
        if (g->stride == 0 || g->marks) return DG4_EINVAL;
        if (which == DG4_COPY_OF) { *host_ptr = g->copy_of.data(); *count = (int64_t)g->copy_of.size(); }
        else { *host_ptr = g->last_copy.data(); *count = (int64_t)g->last_copy.size(); }
        break;
    default: return DG4_EINVAL;
    }
    return DG4_OK;
}

extern "C" int dg4_graph_info(const dg4_graph* g, int64_t* n_nodes, int64_t* n_levels, int64_t* nnz, int32_t* hops)
{
    if (!g) return DG4_EINVAL;
    if (n_nodes) *n_nodes = g->n;
    if (n_levels) *n_levels = (int64_t)g->max_level + 1;
    if (nnz) *nnz = g->nnz;
    if (hops) *hops = g->hops;
    return DG4_OK;
}

// Dataflow order for whole-graph sweeps: list scheduling over the real dependencies. A tile takes
// the (up to) 16 gates that have been ready longest; a gate becomes ready when the tile holding its
// last direct fanin has been filled (every other cone source then sits in an earlier tile too), and
// may go into any later tile; gates that became ready together go by lower level, then lower id.
// Oldest-first keeps as many tiles as possible between a source and its readers, so that the
// source is published before the reader looks for it. Results do not depend on the order; it only
// decides who waits for whom.
// `pairs`: tiles come two at a time (2k and 2k+1, the second possibly empty) with no dependency
// between the two, and count as published together (at the second one): the unit of the sweep
// with the feed-forward sub-block, which runs two tiles through one pass over its weights.
static int flow_schedule(const dg4_graph* g, bool pairs, std::vector<int32_t>& out_order, std::vector<int64_t>& out_tile_ptr)
{
    try {
        std::vector<int64_t> fo_ptr((size_t)g->n + 1, 0);
        std::vector<int32_t> remaining((size_t)g->n, 0);
        // what a gate waits for: its direct fanins (codes 1 and 2; everything else in a whole cone
        // row lies behind them). A row cut by the partition may lack a fanin while keeping a source
        // behind it, so there every source of the row counts.
        auto for_each_fanin = [&](int64_t v, auto&& fn) {
            for (int64_t j = g->nbr_ptr[v]; j < g->nbr_ptr[v + 1]; ++j)
                if (g->stride > 0 ? g->nbr_rel[j] != 0 : (g->nbr_rel[j] == 1 || g->nbr_rel[j] == 2)) fn(g->nbr_idx[j]);
        };
        for (int64_t v = 0; v < g->n; ++v)
            for_each_fanin(v, [&](int32_t u) { ++fo_ptr[(size_t)u + 1]; ++remaining[v]; });
        for (int64_t v = 0; v < g->n; ++v) fo_ptr[v + 1] += fo_ptr[v];
        std::vector<int32_t> fo((size_t)fo_ptr[g->n]);
        {
            std::vector<int64_t> fill(fo_ptr.begin(), fo_ptr.end() - 1);
            for (int64_t v = 0; v < g->n; ++v)
                for_each_fanin(v, [&](int32_t u) { fo[(size_t)fill[u]++] = (int32_t)v; });
        }
        // Gates per tile. A tile is published as a whole and waits for the sources of all its gates, so on a
        // deep, narrow circuit (few gates per dependency level, most compute units idle) small tiles shorten
        // the chain from level to level: a gate then waits for its own sources and little else (medium, 264
        // gates per level, through the register-resident kernel: 6.05 ms with tiles of 16, 5.47 with 4, 4.86
        // with 2, 4.95 with 1). Wide circuits keep 16: there the number of tiles is what costs. Best measured
        // sizes: 2 at 264 and 515 gates per level, 4 at 966, 8 at 1718, 16 at 3092: about one tile per compute
        // unit and level. The width is gates over the depth of the dependencies scheduled here (one pass in
        // topological order).
        int cap_rows = DG4_TILE_ROWS;
        {
            std::vector<int32_t> rem(remaining), depth_of((size_t)g->n, 0), queue;
            queue.reserve((size_t)g->n);
            for (int64_t v = 0; v < g->n; ++v)
                if (rem[v] == 0) queue.push_back((int32_t)v);
            int32_t deepest = 0;
            for (size_t i = 0; i < queue.size(); ++i) {
                const int32_t v = queue[i];
                deepest = std::max(deepest, depth_of[v]);
                for (int64_t j = fo_ptr[v]; j < fo_ptr[v + 1]; ++j) {
                    const int32_t u = fo[(size_t)j];
                    depth_of[u] = std::max(depth_of[u], depth_of[v] + 1);
                    if (--rem[u] == 0) queue.push_back(u);
                }
            }
            const int64_t width = g->n / ((int64_t)deepest + 1);
            if (pairs) {
                // (the dataflow kernel for the other shapes, which takes the tiles of this table one by one on
                // narrow circuits, has the larger fixed cost per tile: 8 gates there, e.g. 105 -> 99 ms for
                // twelve layers on medium; a level of a handful of gates is best left in one tile; three-hop
                // cones, one layer: 8 is best or within 4 % of it from 264 to 1718 gates per level, 16 at 3092)
                if (width >= 64 && width <= 2560) cap_rows = 8;
            } else {
                cap_rows = 2;
                while (cap_rows < DG4_TILE_ROWS && width > (int64_t)cap_rows * DG4_SCHED_TILES_PER_LEVEL) cap_rows *= 2;
            }
        }
        // the ready list is a queue of batches, one per tile, each sorted by (level, id)
        auto before = [&](int32_t a, int32_t b) { return g->level[a] != g->level[b] ? g->level[a] < g->level[b] : a < b; };
        std::vector<int32_t> ready;                 // the queue: taken from `head`, appended at the end
        ready.reserve((size_t)g->n);
        for (int64_t v = 0; v < g->n; ++v)
            if (remaining[v] == 0) ready.push_back((int32_t)v);
        std::sort(ready.begin(), ready.end(), before);
        size_t head = 0;
        std::vector<int32_t> flow((size_t)g->n, 0);
        std::vector<int64_t> tile_ptr(1, 0);
        int64_t q = 0;
        while (head < ready.size()) {
            const int64_t first = q;
            for (int k = 0; k < (pairs ? 2 : 1) * cap_rows && head < ready.size(); ++k) flow[(size_t)q++] = ready[head++];
            if (pairs) tile_ptr.push_back(std::min<int64_t>(first + cap_rows, q));
            tile_ptr.push_back(q);
            const size_t fresh = ready.size();      // eligible from the next tile on
            for (int64_t p = first; p < q; ++p) {
                const int32_t v = flow[(size_t)p];
                for (int64_t j = fo_ptr[v]; j < fo_ptr[v + 1]; ++j) {
                    const int32_t u = fo[(size_t)j];
                    if (--remaining[u] == 0) ready.push_back(u);
                }
            }
            std::sort(ready.begin() + fresh, ready.end(), before);
        }
        if (q != g->n) return DG4_ECYCLE;                      // cannot happen for a validated DAG
        out_order.swap(flow);
        out_tile_ptr.swap(tile_ptr);
    } catch (const std::bad_alloc&) {
        return DG4_ENOMEM;
    }
    return DG4_OK;
}

int dg4_flow_schedule(dg4_graph* g)
{
    if (!g->flow_tile_ptr.empty()) return DG4_OK;          // built once: pointers into it may have been handed out
    return flow_schedule(g, false, g->flow_order, g->flow_tile_ptr);
}

int dg4_pair_schedule(dg4_graph* g)
{
    if (!g->pair_tile_ptr.empty()) return DG4_OK;          // built once: pointers into it may have been handed out
    return flow_schedule(g, true, g->pair_order, g->pair_tile_ptr);
}

// Device tables of the pair schedule (sweeps with the feed-forward sub-block), built on first use.
int dg4_graph_ensure_pairs(dg4_graph* g)
{
    std::lock_guard<std::mutex> lock(g->mu);
    if (g->d_pair_tiles) return DG4_OK;
    if (!g->on_device) return DG4_EINVAL;
    const int w = g->ell_w;
    const size_t rows = (size_t)g->n + DG4_TILE_ROWS;
    try {
        const int rc = dg4_pair_schedule(g);
        if (rc != DG4_OK) return rc;
        const std::vector<int32_t>& order = g->pair_order;
        const std::vector<int64_t>& tile_ptr = g->pair_tile_ptr;
        std::vector<int32_t> padded(rows, 0);
        std::copy(order.begin(), order.end(), padded.begin());
        std::vector<uint2> tiles(tile_ptr.size() - 1);
        for (size_t t = 0; t + 1 < tile_ptr.size(); ++t)
            tiles[t] = make_uint2((uint32_t)tile_ptr[t], (uint32_t)(tile_ptr[t + 1] - tile_ptr[t]));
        std::vector<uint32_t> ell(rows * w, DG4_ELL_PAD);
        std::vector<int32_t> fpos((size_t)g->n, -1);
        for (int64_t q = 0; q < g->n; ++q) fpos[(size_t)order[(size_t)q]] = (int32_t)q;
        for (int64_t v = 0; v < g->n; ++v) {
            const int64_t lo = g->nbr_ptr[v], cnt = g->nbr_ptr[v + 1] - lo;
            uint32_t* r = &ell[(size_t)fpos[v] * w];
            for (int64_t j = 0; j < cnt; ++j)
                r[j] = ((uint32_t)g->nbr_rel[lo + j] << 30) | (uint32_t)fpos[g->nbr_idx[lo + j]];
        }
        uint32_t* d_ell = nullptr; int32_t* d_order = nullptr; uint2* d_tiles = nullptr;
        auto fail = [&](int code) {
            if (d_ell) (void)hipFree(d_ell);
            if (d_order) (void)hipFree(d_order);
            if (d_tiles) (void)hipFree(d_tiles);
            return code;
        };
        if (hipMalloc((void**)&d_ell, rows * w * sizeof(uint32_t)) != hipSuccess) return fail(DG4_ENOMEM);
        if (hipMalloc((void**)&d_order, rows * sizeof(int32_t)) != hipSuccess) return fail(DG4_ENOMEM);
        if (hipMalloc((void**)&d_tiles, std::max<size_t>(tiles.size(), 1) * sizeof(uint2)) != hipSuccess) return fail(DG4_ENOMEM);
        if (hipMemcpy(d_ell, ell.data(), rows * w * sizeof(uint32_t), hipMemcpyHostToDevice) != hipSuccess) return fail(DG4_EHIP);
        if (hipMemcpy(d_order, padded.data(), rows * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess) return fail(DG4_EHIP);
        if (!tiles.empty() && hipMemcpy(d_tiles, tiles.data(), tiles.size() * sizeof(uint2), hipMemcpyHostToDevice) != hipSuccess) return fail(DG4_EHIP);
        g->d_pair_ell = d_ell; g->d_pair_order = d_order; g->d_pair_tiles = d_tiles;
        g->n_pair_tiles = (int64_t)tiles.size();
    } catch (const std::bad_alloc&) {
        return DG4_ENOMEM;
    }
    return DG4_OK;
}

// Device tables: fixed-width packed rows, once by node id (for calls whose
// tensors are indexed by id) and once by position in the (level, id) order
// (for the sweep, whose internal buffers are level sorted).
int dg4_graph_ensure_device(dg4_graph* g)
{
    std::lock_guard<std::mutex> lock(g->mu);
    if (g->on_device) return DG4_OK;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return DG4_EHIP;
    // (one-hop cones get rows of 8 as well: the persistent sweep is laid out for that width; cones
    // deeper than three hops get the longest row, rounded up to four entries)
    int w = std::max(8, 1 << (std::min(g->hops, 3) + 1));
    if (g->hops > 3) {
        int64_t longest = 0;
        for (int64_t v = 0; v < g->n; ++v) longest = std::max(longest, g->nbr_ptr[v + 1] - g->nbr_ptr[v]);
        w = std::max(w, (int)((longest + 3) / 4 * 4));
    }
    const bool with_flow = g->hops <= 2;       // the persistent sweep's tables
    // two tables of rows x w entries are staged in host memory and copied: refuse what cannot fit
    // (a graph of copies without marks at k = 8 can have tens of millions of rows 512 wide)
    if (((size_t)g->n + DG4_TILE_ROWS) * (size_t)w * sizeof(uint32_t) > ((size_t)16 << 30)) return DG4_ENOMEM;
    // one tile of padding: the sweep kernel fetches descriptors of 16 positions at a time
    const size_t rows = (size_t)g->n + DG4_TILE_ROWS;
    try {
        // Processing order of the device kernels. Levels stay in order; INSIDE a level the gates
        // that some gate at most two levels up reads come first (they are published early), and
        // within both groups gates are sorted by the position of their latest-finished source, so
        // that gates whose sources are old share tiles and only the last tiles of a level wait on
        // the levels just before. (The published `order` table keeps (level, id); results do not
        // depend on this.)
        // (three independent derivations, on three threads: the level-sorted tables, the table by node id,
        // the dependency-driven schedule with its table)
        std::vector<int32_t> sweep(rows, 0);
        std::vector<uint32_t> by_id, by_pos, by_flow;
        std::vector<int32_t> flow;
        std::vector<uint2> flow_tiles;
        int rc_job[3] = {DG4_OK, DG4_OK, DG4_OK};
        auto guarded = [&](int slot, auto&& body) {
            try { body(); } catch (const std::bad_alloc&) { rc_job[slot] = DG4_ENOMEM; }
        };
        auto job_levels = [&]() { guarded(0, [&]() {
            std::vector<int32_t> min_reader((size_t)g->n, INT32_MAX);
            for (int64_t v = 0; v < g->n; ++v)
                for (int64_t j = g->nbr_ptr[v]; j < g->nbr_ptr[v + 1]; ++j) {
                    const int32_t u = g->nbr_idx[j];
                    if (u != v) min_reader[u] = std::min(min_reader[u], g->level[v]);
                }
            std::vector<int64_t> key((size_t)g->n, -1);
            for (int32_t l = 0; l <= g->max_level; ++l) {
                const int64_t lo = g->level_ptr[l], hi = g->level_ptr[l + 1];
                for (int64_t q = lo; q < hi; ++q) {
                    const int32_t v = g->order[q];
                    int64_t latest = -1;
                    for (int64_t j = g->nbr_ptr[v]; j < g->nbr_ptr[v + 1]; ++j)
                        if (g->nbr_idx[j] != v) latest = std::max<int64_t>(latest, g->pos[g->nbr_idx[j]]);
                    const int64_t far = (int64_t)min_reader[v] - l > 2 ? 1 : 0;
                    key[v] = (far << 40) + latest + 1;
                    sweep[q] = v;
                }
                std::stable_sort(sweep.begin() + lo, sweep.begin() + hi,
                                 [&](int32_t a, int32_t b) { return key[a] < key[b]; });
                for (int64_t q = lo; q < hi; ++q) g->pos[sweep[q]] = (int32_t)q;   // sources of higher levels see these
            }
            g->sweep_order.assign(sweep.begin(), sweep.begin() + g->n);
            by_pos.assign(rows * w, DG4_ELL_PAD);
            for (int64_t v = 0; v < g->n; ++v) {
                const int64_t lo = g->nbr_ptr[v], cnt = g->nbr_ptr[v + 1] - lo;
                uint32_t* rpos = &by_pos[(size_t)g->pos[v] * w];
                for (int64_t j = 0; j < cnt; ++j)
                    rpos[j] = ((uint32_t)g->nbr_rel[lo + j] << 30) | (uint32_t)g->pos[g->nbr_idx[lo + j]];
            }
        }); };
        // entries stay in ascending-id order in every table, so the summation order of a gate's sources
        // does not depend on the schedule
        auto job_id = [&]() { guarded(1, [&]() {
            by_id.assign(rows * w, DG4_ELL_PAD);
            for (int64_t v = 0; v < g->n; ++v) {
                const int64_t lo = g->nbr_ptr[v], cnt = g->nbr_ptr[v + 1] - lo;
                uint32_t* rid = &by_id[(size_t)v * w];
                for (int64_t j = 0; j < cnt; ++j)
                    rid[j] = ((uint32_t)g->nbr_rel[lo + j] << 30) | (uint32_t)g->nbr_idx[lo + j];
            }
        }); };
        std::vector<uint2> tiles;
        g->level_tile_ptr.assign((size_t)g->max_level + 2, 0);
        for (int32_t l = 0; l <= g->max_level; ++l) {
            g->level_tile_ptr[l] = (int64_t)tiles.size();
            for (int64_t p0 = g->level_ptr[l]; p0 < g->level_ptr[l + 1]; p0 += DG4_TILE_ROWS)
                tiles.push_back(make_uint2((uint32_t)p0, (uint32_t)std::min<int64_t>(DG4_TILE_ROWS, g->level_ptr[l + 1] - p0)));
        }
        g->level_tile_ptr[(size_t)g->max_level + 1] = (int64_t)tiles.size();
        std::vector<uint2> tiles32;
        g->level_tile32_ptr.assign((size_t)g->max_level + 2, 0);
        for (int32_t l = 0; l <= g->max_level; ++l) {
            g->level_tile32_ptr[l] = (int64_t)tiles32.size();
            for (int64_t p0 = g->level_ptr[l]; p0 < g->level_ptr[l + 1]; p0 += 32)
                tiles32.push_back(make_uint2((uint32_t)p0, (uint32_t)std::min<int64_t>(32, g->level_ptr[l + 1] - p0)));
        }
        g->level_tile32_ptr[(size_t)g->max_level + 1] = (int64_t)tiles32.size();
        // Dataflow order for whole-graph sweeps (dg4_flow_schedule)
        auto job_flow = [&]() { guarded(2, [&]() {
            if (!with_flow) return;
            const int rc = dg4_flow_schedule(g);
            if (rc != DG4_OK) { rc_job[2] = rc; return; }
            flow.assign(rows, 0);
            std::copy(g->flow_order.begin(), g->flow_order.end(), flow.begin());
            flow_tiles.resize(g->flow_tile_ptr.size() - 1);
            for (size_t t = 0; t + 1 < g->flow_tile_ptr.size(); ++t)
                flow_tiles[t] = make_uint2((uint32_t)g->flow_tile_ptr[t], (uint32_t)(g->flow_tile_ptr[t + 1] - g->flow_tile_ptr[t]));
            by_flow.assign(rows * w, DG4_ELL_PAD);
            std::vector<int32_t> fpos((size_t)g->n, -1);
            for (int64_t q = 0; q < g->n; ++q) fpos[(size_t)g->flow_order[(size_t)q]] = (int32_t)q;
            for (int64_t v = 0; v < g->n; ++v) {
                const int64_t lo = g->nbr_ptr[v], cnt = g->nbr_ptr[v + 1] - lo;
                uint32_t* r = &by_flow[(size_t)fpos[v] * w];
                for (int64_t j = 0; j < cnt; ++j)
                    r[j] = ((uint32_t)g->nbr_rel[lo + j] << 30) | (uint32_t)fpos[g->nbr_idx[lo + j]];
            }
            g->n_flow_tiles = (int64_t)flow_tiles.size();
        }); };
        {
            std::vector<std::thread> helpers;
            try {
                helpers.emplace_back(job_id);
                helpers.emplace_back(job_flow);
            } catch (const std::system_error&) {}      // no thread to be had: the jobs run here
            job_levels();
            const size_t started = helpers.size();
            for (std::thread& t : helpers) t.join();
            if (started < 1) job_id();
            if (started < 2) job_flow();
        }
        for (int rc : rc_job)
            if (rc != DG4_OK) return rc;
        const size_t bytes = rows * w * sizeof(uint32_t);
        auto fail = [&](int rc) {
            if (g->d_flow_ell) (void)hipFree(g->d_flow_ell);
            if (g->d_flow_order) (void)hipFree(g->d_flow_order);
            if (g->d_flow_tiles) (void)hipFree(g->d_flow_tiles);
            g->d_flow_ell = nullptr; g->d_flow_order = nullptr; g->d_flow_tiles = nullptr;
            if (g->d_ell_id) (void)hipFree(g->d_ell_id);
            if (g->d_ell_pos) (void)hipFree(g->d_ell_pos);
            if (g->d_order) (void)hipFree(g->d_order);
            if (g->d_tiles) (void)hipFree(g->d_tiles);
            if (g->d_tiles32) (void)hipFree(g->d_tiles32);
            g->d_ell_id = g->d_ell_pos = nullptr; g->d_order = nullptr; g->d_tiles = nullptr; g->d_tiles32 = nullptr;
            return rc;
        };
        if (hipMalloc((void**)&g->d_ell_id, bytes) != hipSuccess) return fail(DG4_ENOMEM);
        if (hipMalloc((void**)&g->d_ell_pos, bytes) != hipSuccess) return fail(DG4_ENOMEM);
        if (hipMalloc((void**)&g->d_order, rows * sizeof(int32_t)) != hipSuccess) return fail(DG4_ENOMEM);
        if (hipMalloc((void**)&g->d_tiles, std::max<size_t>(tiles.size(), 1) * sizeof(uint2)) != hipSuccess) return fail(DG4_ENOMEM);
        if (!tiles.empty() &&
            hipMemcpy(g->d_tiles, tiles.data(), tiles.size() * sizeof(uint2), hipMemcpyHostToDevice) != hipSuccess)
            return fail(DG4_EHIP);
        if (hipMalloc((void**)&g->d_tiles32, std::max<size_t>(tiles32.size(), 1) * sizeof(uint2)) != hipSuccess) return fail(DG4_ENOMEM);
        if (!tiles32.empty() &&
            hipMemcpy(g->d_tiles32, tiles32.data(), tiles32.size() * sizeof(uint2), hipMemcpyHostToDevice) != hipSuccess)
            return fail(DG4_EHIP);
        if (hipMemcpy(g->d_ell_id, by_id.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) return fail(DG4_EHIP);
        if (hipMemcpy(g->d_ell_pos, by_pos.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) return fail(DG4_EHIP);
        if (g->n > 0 &&
            hipMemcpy(g->d_order, sweep.data(), rows * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess)
            return fail(DG4_EHIP);
        if (with_flow) {
            if (hipMalloc((void**)&g->d_flow_ell, bytes) != hipSuccess) return fail(DG4_ENOMEM);
            if (hipMalloc((void**)&g->d_flow_order, rows * sizeof(int32_t)) != hipSuccess) return fail(DG4_ENOMEM);
            if (hipMalloc((void**)&g->d_flow_tiles, std::max<size_t>(flow_tiles.size(), 1) * sizeof(uint2)) != hipSuccess) return fail(DG4_ENOMEM);
            if (!flow_tiles.empty() &&
                hipMemcpy(g->d_flow_tiles, flow_tiles.data(), flow_tiles.size() * sizeof(uint2), hipMemcpyHostToDevice) != hipSuccess)
                return fail(DG4_EHIP);
            if (hipMemcpy(g->d_flow_ell, by_flow.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) return fail(DG4_EHIP);
            if (hipMemcpy(g->d_flow_order, flow.data(), rows * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess) return fail(DG4_EHIP);
        }
    } catch (const std::bad_alloc&) {
        return DG4_ENOMEM;
    }
    g->ell_w = w; g->device = dev; g->on_device = true;
    return DG4_OK;
}

// Tiles for the persistent sweep over rows wider than 16 entries: runs of a few positions inside a
// level. The wider the rows, the fewer gates share a tile (and the more lanes walk a gate's row):
// the number depends on the width of the table alone, so that a gate's arithmetic does not depend
// on the range of levels a call covers.
int dg4_graph_ensure_wide_tiles(dg4_graph* g)
{
    std::lock_guard<std::mutex> lock(g->mu);
    if (g->d_tilesw) return DG4_OK;
    if (!g->on_device || g->ell_w <= 16) return DG4_EINVAL;
    const int rows = g->ell_w <= 32 ? 16 : g->ell_w <= 64 ? 8 : g->ell_w <= 128 ? 4 : 2;
    try {
        std::vector<uint2> tiles;
        g->level_tilew_ptr.assign((size_t)g->max_level + 2, 0);
        for (int32_t l = 0; l <= g->max_level; ++l) {
            g->level_tilew_ptr[l] = (int64_t)tiles.size();
            for (int64_t p0 = g->level_ptr[l]; p0 < g->level_ptr[l + 1]; p0 += rows)
                tiles.push_back(make_uint2((uint32_t)p0, (uint32_t)std::min<int64_t>(rows, g->level_ptr[l + 1] - p0)));
        }
        g->level_tilew_ptr[(size_t)g->max_level + 1] = (int64_t)tiles.size();
        uint2* d = nullptr;
        if (hipMalloc((void**)&d, std::max<size_t>(tiles.size(), 1) * sizeof(uint2)) != hipSuccess) return DG4_ENOMEM;
        if (!tiles.empty() && hipMemcpy(d, tiles.data(), tiles.size() * sizeof(uint2), hipMemcpyHostToDevice) != hipSuccess) {
            (void)hipFree(d);
            return DG4_EHIP;
        }
        g->d_tilesw = d; g->wide_tile_rows = rows;
    } catch (const std::bad_alloc&) {
        return DG4_ENOMEM;
    }
    return DG4_OK;
}

// Device tables of the (Eq. 1 level, id) order, see dg4_graph::eq1_level_ptr.
int dg4_graph_ensure_eq1(dg4_graph* g)
{
    std::lock_guard<std::mutex> lock(g->mu);
    if (g->d_ell_eq1) return DG4_OK;
    if (!g->on_device || g->eq1_level_ptr.empty()) return DG4_EINVAL;
    const int w = g->ell_w;
    const size_t rows = (size_t)g->n + DG4_TILE_ROWS;
    try {
        std::vector<int32_t> order(rows, 0), pos((size_t)g->n, 0);
        std::vector<int64_t> cur(g->eq1_level_ptr.begin(), g->eq1_level_ptr.end() - 1);
        for (int64_t v = 0; v < g->n; ++v) {
            const int64_t p = cur[(size_t)g->eq1_level[v]]++;
            order[(size_t)p] = (int32_t)v; pos[(size_t)v] = (int32_t)p;
        }
        std::vector<uint32_t> ell(rows * w, DG4_ELL_PAD);
        for (int64_t v = 0; v < g->n; ++v) {
            const int64_t lo = g->nbr_ptr[v], cnt = g->nbr_ptr[v + 1] - lo;
            uint32_t* r = &ell[(size_t)pos[v] * w];
            for (int64_t j = 0; j < cnt; ++j)
                r[j] = ((uint32_t)g->nbr_rel[lo + j] << 30) | (uint32_t)pos[g->nbr_idx[lo + j]];
        }
        uint32_t* d_ell = nullptr; int32_t* d_order = nullptr;
        if (hipMalloc((void**)&d_ell, rows * w * sizeof(uint32_t)) != hipSuccess) return DG4_ENOMEM;
        if (hipMalloc((void**)&d_order, rows * sizeof(int32_t)) != hipSuccess) { (void)hipFree(d_ell); return DG4_ENOMEM; }
        if (hipMemcpy(d_ell, ell.data(), rows * w * sizeof(uint32_t), hipMemcpyHostToDevice) != hipSuccess ||
            hipMemcpy(d_order, order.data(), rows * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess) {
            (void)hipFree(d_ell); (void)hipFree(d_order);
            return DG4_EHIP;
        }
        g->d_order_eq1 = d_order; g->d_ell_eq1 = d_ell;
    } catch (const std::bad_alloc&) {
        return DG4_ENOMEM;
    }
    return DG4_OK;
}

// level, OutAND, OutNOT of every node as one device table [n][3] for dg4_struct_encode
int dg4_graph_ensure_struct(dg4_graph* g)
{
    std::lock_guard<std::mutex> lock(g->mu);
    if (g->d_struct) return DG4_OK;
    try {
        std::vector<int32_t> t((size_t)std::max<int64_t>(g->n, 1) * 3, 0);
        for (int64_t v = 0; v < g->n; ++v) {
            t[3 * (size_t)v] = g->level[v]; t[3 * (size_t)v + 1] = g->out_and[v]; t[3 * (size_t)v + 2] = g->out_not[v];
        }
        if (hipMalloc((void**)&g->d_struct, t.size() * sizeof(int32_t)) != hipSuccess) return DG4_ENOMEM;
        if (hipMemcpy(g->d_struct, t.data(), t.size() * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess) {
            (void)hipFree(g->d_struct); g->d_struct = nullptr;
            return DG4_EHIP;
        }
    } catch (const std::bad_alloc&) {
        return DG4_ENOMEM;
    }
    return DG4_OK;
}

// Tables for sweeps that keep no K|V store: the frontier of a level is the set of distinct sources
// of its gates (Section 3.4: what has to be pulled from the historical embeddings for one level).
int dg4_graph_ensure_frontier(dg4_graph* g)
{
    std::lock_guard<std::mutex> lock(g->mu);
    if (g->has_frontier) return DG4_OK;
    if (!g->on_device) return DG4_EINVAL;
    const int w = g->ell_w;
    const size_t rows = (size_t)g->n + DG4_TILE_ROWS;
    try {
        const int32_t n_levels = g->max_level + 1;
        std::vector<int64_t> ptr((size_t)n_levels + 1, 0);
        std::vector<int32_t> ids;
        std::vector<uint32_t> ell(rows * w, DG4_ELL_PAD);
        std::vector<int32_t> local((size_t)g->n, -1), seen;
        int64_t largest = 0;
        for (int32_t l = 0; l < n_levels; ++l) {
            seen.clear();
            for (int64_t q = g->level_ptr[l]; q < g->level_ptr[l + 1]; ++q) {
                const int32_t v = g->sweep_order[(size_t)q];
                for (int64_t j = g->nbr_ptr[v]; j < g->nbr_ptr[v + 1]; ++j) {
                    const int32_t u = g->nbr_idx[j];
                    if (u != v && local[u] < 0) { local[u] = 0; seen.push_back(g->pos[u]); }
                }
            }
            std::sort(seen.begin(), seen.end());                    // positions: sources of a level sit close together
            // (sweep order position -> node id through the level-ordered table the device uses)
            for (size_t i = 0; i < seen.size(); ++i) local[g->sweep_order[(size_t)seen[i]]] = (int32_t)i;
            for (int64_t q = g->level_ptr[l]; q < g->level_ptr[l + 1]; ++q) {
                const int32_t v = g->sweep_order[(size_t)q];
                uint32_t* r = &ell[(size_t)q * w];
                const int64_t lo = g->nbr_ptr[v];
                for (int64_t j = lo; j < g->nbr_ptr[v + 1]; ++j) {
                    const int32_t u = g->nbr_idx[j];
                    r[j - lo] = ((uint32_t)g->nbr_rel[j] << 30) | (uint32_t)(u == v ? 0 : local[u]);
                }
            }
            for (int32_t pos : seen) { const int32_t u = g->sweep_order[(size_t)pos]; ids.push_back(u); local[u] = -1; }
            ptr[(size_t)l + 1] = (int64_t)ids.size();
            largest = std::max<int64_t>(largest, (int64_t)seen.size());
        }
        if (hipMalloc((void**)&g->d_front_id, std::max<size_t>(ids.size(), 1) * sizeof(int32_t)) != hipSuccess) return DG4_ENOMEM;
        if (hipMalloc((void**)&g->d_ell_front, rows * w * sizeof(uint32_t)) != hipSuccess) {
            (void)hipFree(g->d_front_id); g->d_front_id = nullptr;
            return DG4_ENOMEM;
        }
        if ((!ids.empty() && hipMemcpy(g->d_front_id, ids.data(), ids.size() * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess) ||
            hipMemcpy(g->d_ell_front, ell.data(), rows * w * sizeof(uint32_t), hipMemcpyHostToDevice) != hipSuccess) {
            (void)hipFree(g->d_front_id); (void)hipFree(g->d_ell_front);
            g->d_front_id = nullptr; g->d_ell_front = nullptr;
            return DG4_EHIP;
        }
        g->front_ptr.swap(ptr);
        g->front_max = largest;
    } catch (const std::bad_alloc&) {
        return DG4_ENOMEM;
    }
    g->has_frontier = true;
    return DG4_OK;
}

extern "C" int dg4_graph_upload(dg4_graph* g)
{
    if (!g) return DG4_EINVAL;
    return dg4_graph_ensure_device(g);
}

extern "C" void dg4_graph_free(dg4_graph* g)
{
    if (!g) return;
    if (g->d_ell_id) (void)hipFree(g->d_ell_id);
    if (g->d_ell_pos) (void)hipFree(g->d_ell_pos);
    if (g->d_order) (void)hipFree(g->d_order);
    if (g->d_tiles) (void)hipFree(g->d_tiles);
    if (g->d_tiles32) (void)hipFree(g->d_tiles32);
    if (g->d_tilesw) (void)hipFree(g->d_tilesw);
    if (g->d_flow_ell) (void)hipFree(g->d_flow_ell);
    if (g->d_flow_order) (void)hipFree(g->d_flow_order);
    if (g->d_flow_tiles) (void)hipFree(g->d_flow_tiles);
    if (g->d_struct) (void)hipFree(g->d_struct);
    if (g->d_front_id) (void)hipFree(g->d_front_id);
    if (g->d_ell_front) (void)hipFree(g->d_ell_front);
    if (g->d_pair_ell) (void)hipFree(g->d_pair_ell);
    if (g->d_pair_order) (void)hipFree(g->d_pair_order);
    if (g->d_pair_tiles) (void)hipFree(g->d_pair_tiles);
    if (g->d_order_eq1) (void)hipFree(g->d_order_eq1);
    if (g->d_ell_eq1) (void)hipFree(g->d_ell_eq1);
    delete g;
}
