// Cache schedule of the resident hop kernel.
//
// The paper's decomposition is "agnostic on nodes" (Section 3.2, Limitation
// paragraph): an edge block is any balanced slice of the list.  For the result that
// is all that matters; for the time a hop takes on this machine it is not, because a
// gathered feature row is only cheap while the XCD that asks for it still holds it
// in its private L2.  This file decides, per plan, in which order destination rows
// are processed and by which XCD, so that rows that draw from the same sources run
// together on one XCD, one column slice at a time (Algorithm 1's column blocks and
// edge blocks, re-used as a cache schedule):
//
//   1. row clusters by synchronous label propagation over the non-zero pattern
//      (a row takes the most frequent label among its sources, ties to the smallest;
//      deterministic, independent of the thread count);
//   2. per column-slice count S, one explicit work list per XCD: records are the
//      plan's segments, cluster by cluster, each (cluster chunk, slice) pair given to
//      the XCD with the least work so far;
//   3. every segment cut into its hot non-zeros (the source is in the row's cluster, or,
//      in a graph without clusters, one of its most popular rows) and the others: as two
//      record lists for the L2s, or as the schedule of the LDS pass, which keeps a list
//      of at most 10,192 rows in a compute unit's LDS one 16-byte strip at a time and
//      orders every lane's reads so that the lanes the LDS serves together never meet
//      on a bank.
//
// Graphs without such structure (one giant cluster and no popular rows worth a pass)
// keep the implicit lists.
#include <algorithm>
#include <atomic>
#include <numeric>

#include "gp_internal.h"

namespace gp {

namespace {

inline uint32_t mix(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

// rows [cut[t], cut[t+1]) hold about the same number of non-zeros for every t
std::vector<int64_t> balanced_row_cuts(const gp_plan& P, int nt)
{
    std::vector<int64_t> cut((size_t)nt + 1, 0);
    for (int t = 1; t < nt; ++t) {
        const int64_t target = P.nnz / nt * t;
        cut[(size_t)t] = std::lower_bound(P.rowptr.begin(), P.rowptr.end(), target) - P.rowptr.begin();
        if (cut[(size_t)t] > P.n) cut[(size_t)t] = P.n;
        if (cut[(size_t)t] < cut[(size_t)t - 1]) cut[(size_t)t] = cut[(size_t)t - 1];
    }
    cut[(size_t)nt] = P.n;
    return cut;
}

}  // namespace

void cluster_rows(const gp_plan& P, RowClusters& C)
{
    const int64_t n = P.n;
    const int nt = (n + P.nnz < (1 << 16)) ? 1 : host_threads();
    const std::vector<int64_t> cut = balanced_row_cuts(P, nt);
    std::vector<int32_t> lab((size_t)n), nxt((size_t)n);
    std::iota(lab.begin(), lab.end(), 0);

    const int max_iter = 10;
    for (int it = 0; it < max_iter; ++it) {
        std::atomic<int64_t> changed{0};
        parallel_run(nt, [&](int t, int) {
            std::vector<int32_t> key, cnt;
            int64_t mine = 0;
            for (int64_t i = cut[(size_t)t]; i < cut[(size_t)t + 1]; ++i) {
                const int64_t s = P.rowptr[i], e = P.rowptr[i + 1];
                if (e == s) {
                    nxt[(size_t)i] = lab[(size_t)i];
                    continue;
                }
                size_t cap = 8;
                while (cap < (size_t)(e - s) * 2) cap *= 2;
                if (key.size() < cap) {
                    key.resize(cap);
                    cnt.resize(cap);
                }
                std::fill(key.begin(), key.begin() + (ptrdiff_t)cap, -1);
                int32_t best = -1, best_cnt = 0;
                for (int64_t k = s; k < e; ++k) {
                    const int32_t l = lab[(size_t)P.col[(size_t)k]];
                    size_t h = mix((uint32_t)l) & (cap - 1);
                    while (key[h] != -1 && key[h] != l) h = (h + 1) & (cap - 1);
                    if (key[h] == -1) {
                        key[h] = l;
                        cnt[h] = 0;
                    }
                    const int32_t c = ++cnt[h];
                    if (c > best_cnt || (c == best_cnt && l < best)) {
                        best = l;
                        best_cnt = c;
                    }
                }
                nxt[(size_t)i] = best;
                mine += best != lab[(size_t)i];
            }
            changed += mine;
        });
        lab.swap(nxt);
        if (changed.load() * 2000 < n) break;
    }

    // renumber: clusters in ascending order of their label
    std::vector<int32_t> rank((size_t)n, 0);
    for (int64_t i = 0; i < n; ++i) rank[(size_t)lab[(size_t)i]] = 1;
    int32_t num = 0;
    for (int64_t i = 0; i < n; ++i) {
        const int32_t present = rank[(size_t)i];
        rank[(size_t)i] = num;
        num += present;
    }
    C.label.resize((size_t)n);
    for (int64_t i = 0; i < n; ++i) C.label[(size_t)i] = rank[(size_t)lab[(size_t)i]];
    C.num = num;

    // how much of the gathering stays inside a row's own cluster, and how many rows the
    // cluster of a typical non-zero has (what an L2 would have to hold)
    std::vector<int64_t> size((size_t)num, 0), weight((size_t)num, 0);
    for (int64_t i = 0; i < n; ++i) {
        ++size[(size_t)C.label[(size_t)i]];
        weight[(size_t)C.label[(size_t)i]] += P.rowptr[i + 1] - P.rowptr[i];
    }
    std::atomic<int64_t> inside{0};
    parallel_run(nt, [&](int t, int) {
        int64_t mine = 0;
        for (int64_t i = cut[(size_t)t]; i < cut[(size_t)t + 1]; ++i) {
            const int32_t li = C.label[(size_t)i];
            for (int64_t k = P.rowptr[i]; k < P.rowptr[i + 1]; ++k) mine += C.label[(size_t)P.col[(size_t)k]] == li;
        }
        inside += mine;
    });
    double wrows = 0.0;
    for (int32_t c = 0; c < num; ++c) wrows += (double)weight[(size_t)c] * (double)size[(size_t)c];
    C.inside_fraction = P.nnz > 0 ? (double)inside.load() / (double)P.nnz : 0.0;
    C.typical_rows = P.nnz > 0 ? wrows / (double)P.nnz : 0.0;
    C.ready = true;
}

// Explicit per-XCD work lists for S column slices of slice_elems elements each.
// Rows are taken cluster by cluster (ascending row inside a cluster) and cut into
// chunks of bounded work; a chunk's segments are listed longest first; every
// (chunk, slice) pair goes, in that order, to the XCD with the least work so far, so
// the slices of one chunk run on different XCDs at about the same time and every XCD
// moves through the clusters at the same pace.
void build_xcd_lists(const gp_plan& P, const std::vector<Segment>& segs, const RowClusters& C, int S, int slice_elems, int d,
                     std::vector<Segment>& recs, int64_t off[9])
{
    const int64_t n = P.n, nsegs = (int64_t)segs.size();
    // rows in (cluster, row) order
    std::vector<int64_t> cstart((size_t)C.num + 1, 0);
    for (int64_t i = 0; i < n; ++i) ++cstart[(size_t)C.label[(size_t)i] + 1];
    for (int32_t c = 0; c < C.num; ++c) cstart[(size_t)c + 1] += cstart[(size_t)c];
    std::vector<int32_t> order((size_t)n);
    {
        std::vector<int64_t> cur(cstart.begin(), cstart.end() - 1);
        for (int64_t i = 0; i < n; ++i) order[(size_t)cur[(size_t)C.label[(size_t)i]]++] = (int32_t)i;
    }
    // chunks: a chunk ends at a cluster boundary once it holds min_rows rows, and inside
    // a cluster when it holds max_work non-zeros
    const int64_t min_rows = 512;
    const int64_t max_work = std::max<int64_t>(P.nnz / 64, 1 << 16);  // in non-zeros of the whole rows
    std::vector<int32_t> chunk_of_row((size_t)n, 0);
    int32_t chunks = 0;
    {
        int64_t rows = 0, work = 0;
        for (int64_t k = 0; k < n; ++k) {
            const int32_t r = order[(size_t)k];
            const bool new_cluster = k > 0 && C.label[(size_t)r] != C.label[(size_t)order[(size_t)k - 1]];
            if (rows > 0 && ((new_cluster && rows >= min_rows) || work >= max_work)) {
                ++chunks;
                rows = work = 0;
            }
            chunk_of_row[(size_t)r] = chunks;
            ++rows;
            work += P.rowptr[(size_t)r + 1] - P.rowptr[(size_t)r] + 1;
        }
        ++chunks;
    }
    // segments by chunk (counting sort), longest first inside a chunk
    std::vector<int64_t> koff((size_t)chunks + 1, 0);
    for (int64_t s = 0; s < nsegs; ++s) ++koff[(size_t)chunk_of_row[(size_t)segs[(size_t)s].row] + 1];
    for (int32_t k = 0; k < chunks; ++k) koff[(size_t)k + 1] += koff[(size_t)k];
    std::vector<int64_t> sidx((size_t)nsegs);
    {
        std::vector<int64_t> cur(koff.begin(), koff.end() - 1);
        for (int64_t s = 0; s < nsegs; ++s) sidx[(size_t)cur[(size_t)chunk_of_row[(size_t)segs[(size_t)s].row]]++] = s;
    }
    const int nt = nsegs < (1 << 16) ? 1 : host_threads();
    parallel_run(nt, [&](int t, int k) {
        for (int32_t c = t; c < chunks; c += k)
            std::stable_sort(sidx.begin() + (ptrdiff_t)koff[(size_t)c], sidx.begin() + (ptrdiff_t)koff[(size_t)c + 1],
                             [&](int64_t a, int64_t b) { return segs[(size_t)a].len > segs[(size_t)b].len; });
    });
    // (chunk, slice) pairs to XCDs
    std::vector<int64_t> chunk_work((size_t)chunks, 0);
    for (int32_t c = 0; c < chunks; ++c)
        for (int64_t j = koff[(size_t)c]; j < koff[(size_t)c + 1]; ++j) chunk_work[(size_t)c] += segs[(size_t)sidx[(size_t)j]].len + 4;
    std::vector<int8_t> owner((size_t)chunks * (size_t)S);
    int64_t load[8] = {0, 0, 0, 0, 0, 0, 0, 0}, count[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int32_t c = 0; c < chunks; ++c)
        for (int s = 0; s < S; ++s) {
            const int width = std::min(slice_elems, d - s * slice_elems);
            int x = 0;
            for (int y = 1; y < 8; ++y)
                if (load[y] < load[x]) x = y;
            owner[(size_t)c * (size_t)S + (size_t)s] = (int8_t)x;
            load[x] += chunk_work[(size_t)c] * (width + 8);
            count[x] += koff[(size_t)c + 1] - koff[(size_t)c];
        }
    off[0] = 0;
    for (int x = 0; x < 8; ++x) off[x + 1] = off[x] + count[x];
    recs.resize((size_t)off[8]);
    int64_t cur[8];
    for (int x = 0; x < 8; ++x) cur[x] = off[x];
    for (int32_t c = 0; c < chunks; ++c)
        for (int s = 0; s < S; ++s) {
            const int x = owner[(size_t)c * (size_t)S + (size_t)s];
            for (int64_t j = koff[(size_t)c]; j < koff[(size_t)c + 1]; ++j) {
                Segment g = segs[(size_t)sidx[(size_t)j]];
                g.slice = (uint8_t)s;
                recs[(size_t)cur[x]++] = g;
            }
        }
}

// Every segment cut in two: the non-zeros whose source lies in the row's own cluster (the
// ones worth a place in the cache) first, the others after them.  out.col is the column
// list with every segment's range reordered that way (stable inside each part); a segment
// with both kinds becomes a hot and a cold record, and a row that ends up with more than one
// record owns consecutive partial-row slots in (segment, hot before cold) order.
HotSets hot_sets_from_clusters(const RowClusters& C)
{
    HotSets H;
    H.num_sets = H.num_lists = C.num;
    H.set_of_row = C.label;
    H.list_of_row = C.label;
    H.list_of_set.resize((size_t)C.num);
    std::iota(H.list_of_set.begin(), H.list_of_set.end(), 0);
    H.hot_fraction = C.inside_fraction;
    return H;
}

// Popularity of a row = how many non-zeros have it as their source.  The `hubs` most popular
// rows (ties to the smaller id) form the one list; rows are cut into sets of consecutive ids.
HotSets hot_sets_from_hubs(const gp_plan& P, int32_t hubs, int64_t rows_per_set)
{
    HotSets H;
    const int64_t n = P.n;
    std::vector<int32_t> uses((size_t)n, 0);
    {
        const int64_t nnz = (int64_t)P.col.size();
        const int nt = nnz < (1 << 20) ? 1 : host_threads();
        parallel_run(nt, [&](int t, int k) {
            for (int64_t e = nnz * t / k; e < nnz * (t + 1) / k; ++e) __atomic_fetch_add(&uses[(size_t)P.col[(size_t)e]], 1, __ATOMIC_RELAXED);
        });
    }
    hubs = (int32_t)std::min<int64_t>(hubs, n);
    std::vector<int32_t> order((size_t)n);
    std::iota(order.begin(), order.end(), 0);
    auto more_popular = [&](int32_t a, int32_t b) { return uses[(size_t)a] != uses[(size_t)b] ? uses[(size_t)a] > uses[(size_t)b] : a < b; };
    if (hubs < n) std::nth_element(order.begin(), order.begin() + hubs, order.end(), more_popular);
    H.list_of_row.assign((size_t)n, -1);
    int64_t hot = 0;
    for (int32_t k = 0; k < hubs; ++k) {
        H.list_of_row[(size_t)order[(size_t)k]] = 0;
        hot += uses[(size_t)order[(size_t)k]];
    }
    H.hot_fraction = P.nnz > 0 ? (double)hot / (double)P.nnz : 0.0;
    H.num_lists = 1;
    H.min_hot = kHubMinHot;
    rows_per_set = std::max<int64_t>(rows_per_set, 64);
    H.num_sets = (int32_t)std::max<int64_t>(1, (n + rows_per_set - 1) / rows_per_set);
    H.list_of_set.assign((size_t)H.num_sets, 0);
    H.set_of_row.resize((size_t)n);
    for (int64_t i = 0; i < n; ++i) H.set_of_row[(size_t)i] = (int32_t)(i / rows_per_set);
    return H;
}

namespace {

// The column list with every segment's hot non-zeros moved to its front (stable on both
// sides), and how many each segment has.
void hot_first(const gp_plan& P, const HotSets& C, std::vector<int32_t>& col, std::vector<int32_t>& hot_len)
{
    const int64_t nsegs = (int64_t)P.segs.size();
    col.resize(P.col.size());
    hot_len.resize((size_t)nsegs);
    const int nt = P.nnz < (1 << 16) ? 1 : host_threads();
    parallel_run(nt, [&](int t, int k) {
        for (int64_t s = nsegs * t / k; s < nsegs * (t + 1) / k; ++s) {
            const Segment& g = P.segs[(size_t)s];
            const int64_t e0 = ((int64_t)g.start_hi << 32) | g.start_lo;
            const int32_t li = C.list_of_set[(size_t)C.set_of_row[(size_t)g.row]];
            int64_t w = e0;
            for (int64_t e = e0; e < e0 + g.len; ++e)
                if (C.list_of_row[(size_t)P.col[(size_t)e]] == li) col[(size_t)w++] = P.col[(size_t)e];
            hot_len[(size_t)s] = (int32_t)(w - e0);
            for (int64_t e = e0; e < e0 + g.len; ++e)
                if (C.list_of_row[(size_t)P.col[(size_t)e]] != li) col[(size_t)w++] = P.col[(size_t)e];
        }
    });
}

}  // namespace

void build_split_schedule(const gp_plan& P, const HotSets& C, SplitSchedule& out)
{
    const int64_t nsegs = (int64_t)P.segs.size();
    std::vector<int32_t> hot_len;
    hot_first(P, C, out.col, hot_len);
    // records per row, in the order the plan lists a row's segments (ascending start)
    std::vector<int32_t> pieces((size_t)P.n, 0);
    for (int64_t s = 0; s < nsegs; ++s) {
        const int32_t h = hot_len[(size_t)s], len = P.segs[(size_t)s].len;
        pieces[(size_t)P.segs[(size_t)s].row] += (h > 0 && h < len) ? 2 : 1;
    }
    out.split.clear();
    std::vector<int64_t> next_slot((size_t)P.n, -1);
    int64_t slot = 0;
    for (int64_t i = 0; i < P.n; ++i)
        if (pieces[(size_t)i] > 1) {
            out.split.push_back(SplitRow{(int32_t)i, pieces[(size_t)i], slot});
            next_slot[(size_t)i] = slot;
            slot += pieces[(size_t)i];
        }
    out.num_slots = slot;
    out.hot.clear();
    out.cold.clear();
    for (int64_t s = 0; s < nsegs; ++s) {
        const Segment& g = P.segs[(size_t)s];
        const int64_t e0 = ((int64_t)g.start_hi << 32) | g.start_lo;
        const int32_t h = hot_len[(size_t)s];
        auto piece = [&](int64_t start, int32_t len) {
            Segment q = g;
            q.start_lo = (uint32_t)(start & 0xFFFFFFFF);
            q.start_hi = (uint8_t)(start >> 32);
            q.len = (uint16_t)len;
            int64_t& ns = next_slot[(size_t)g.row];
            q.slot = ns < 0 ? -1 : (int32_t)ns++;
            return q;
        };
        if (h > 0 || g.len == 0) out.hot.push_back(piece(e0, h));  // a row without non-zeros still owes its zero row
        if (g.len - h > 0) out.cold.push_back(piece(e0 + h, g.len - h));
    }
}

namespace {

// Lanes whose 16-byte LDS reads are served together.  A ds_read_b128 of a wavefront goes
// through the LDS in four passes of 16 lanes, and two lanes of one pass that ask for
// different rows of the same 16 banks cost an extra pass.  Which lanes share a pass was
// measured with a two-lane probe on gfx950: lanes {0-3, 12-15, 20-27} and {4-11, 16-19,
// 28-31} of each half of the wavefront.
inline int lds_pass_of_lane(int l)
{
    const int h = l & 31;
    const bool first = h < 4 || (h >= 12 && h < 16) || (h >= 20 && h < 28);
    return ((l >> 5) << 1) | (first ? 0 : 1);
}

// The reads of the 16 records of one pass group, ordered so that a step asks for 16
// different bank groups (row index mod 16) wherever that can be.  Records and bank groups
// form a bipartite multigraph (one edge per non-zero); with no bank group having more than
// `steps` edges, and padded with reads of zero rows until every record and every bank
// group has `steps` edges, it is regular, and a regular bipartite multigraph is a sum of
// perfect matchings (Hall): each matching is one conflict-free step.
struct PassGroup {
    int32_t count[16][16];               // real reads of record j in bank group r still to place
    std::vector<uint16_t> bucket[16];    // record j's local indices, sorted by bank group, column-list order inside one
    int32_t next[16][16];                // position in bucket[j] of the next unplaced read of bank group r
    int32_t len[16];
    std::vector<uint16_t> table;         // schedule(): the placement, step by step
    std::vector<uint16_t> doubled;       // schedule(): per step, the bank groups that two lanes read

    void load(int j, const int32_t* col, int32_t n, const int32_t* local)
    {
        len[j] = n;
        int32_t start[17] = {0};
        for (int r = 0; r < 16; ++r) count[j][r] = 0;
        for (int32_t e = 0; e < n; ++e) ++count[j][local[col[e]] & 15];
        for (int r = 0; r < 16; ++r) start[r + 1] = start[r] + count[j][r];
        bucket[j].resize((size_t)n);
        for (int r = 0; r < 16; ++r) next[j][r] = start[r];
        int32_t fill[16];
        for (int r = 0; r < 16; ++r) fill[r] = start[r];
        for (int32_t e = 0; e < n; ++e) {
            const uint16_t id = (uint16_t)local[col[e]];
            bucket[j][(size_t)fill[id & 15]++] = id;
        }
    }
    void clear(int j)
    {
        len[j] = 0;
        bucket[j].clear();
        for (int r = 0; r < 16; ++r) count[j][r] = next[j][r] = 0;
    }
    // emit(j, step, local index) for all 16 records and `steps` >= the longest record.  Where a bank group has
    // more reads than there are steps, the surplus is set aside and afterwards takes the place of padding
    // reads of its own record: it then meets another lane's read of the same bank group (a two-way conflict:
    // one more pass for these 16 lanes at that step), which is cheaper than one more step for all 64.
    // (false if no matching was found: cannot happen, checked all the same)
    template <class Emit>
    bool schedule(int32_t steps, uint16_t zero_base, Emit emit)
    {
        int32_t w[16][16];     // reads of record j in bank group r still to place, padding included
        int32_t real[16][16];  // ... of which real ones that take part in the conflict-free placement
        int32_t row_need[16], col_need[16];
        for (int j = 0; j < 16; ++j) {
            if (len[j] > steps) return false;
            row_need[j] = steps - len[j];
            for (int r = 0; r < 16; ++r) real[j][r] = count[j][r];
        }
        for (int r = 0; r < 16; ++r) {
            int32_t sum = 0;
            for (int j = 0; j < 16; ++j) sum += count[j][r];
            for (int j = 0; sum > steps; j = (j + 1) & 15)  // the surplus, taken from the records in turn
                if (real[j][r] > 0) {
                    --real[j][r];
                    ++row_need[j];
                    --sum;
                }
            col_need[r] = steps - sum;
        }
        for (int j = 0; j < 16; ++j)
            for (int r = 0; r < 16; ++r) w[j][r] = real[j][r];
        for (int j = 0, r = 0; j < 16 && r < 16;) {  // padding: any matrix with these margins will do
            const int32_t c = std::min(row_need[j], col_need[r]);
            w[j][r] += c;
            row_need[j] -= c;
            col_need[r] -= c;
            if (row_need[j] == 0) ++j;
            else ++r;
        }
        table.assign((size_t)steps * 16, 0);
        int rec_of[16], grp_of[16];  // the current matching
        for (int i = 0; i < 16; ++i) rec_of[i] = grp_of[i] = -1;
        for (int32_t done = 0; done < steps;) {
            for (int j = 0; j < 16; ++j)
                if (grp_of[j] < 0) {
                    uint32_t seen = 0;
                    if (!augment(j, w, rec_of, grp_of, seen)) return false;
                }
            int32_t c = steps - done;
            for (int j = 0; j < 16; ++j) c = std::min(c, w[j][grp_of[j]]);
            for (int j = 0; j < 16; ++j) {
                const int r = grp_of[j];
                for (int32_t t = 0; t < c; ++t) {
                    uint16_t id = (uint16_t)(zero_base + r);
                    if (real[j][r] > 0) {
                        id = bucket[j][(size_t)next[j][r]++];
                        --real[j][r];
                        --count[j][r];
                    }
                    table[(size_t)(done + t) * 16 + j] = id;
                }
                w[j][r] -= c;
                if (w[j][r] == 0) {
                    rec_of[r] = -1;
                    grp_of[j] = -1;
                }
            }
            done += c;
        }
        // the surplus reads, into padding slots of their own records: a step where the bank group has not
        // been doubled yet if there is one
        doubled.assign((size_t)steps, 0);
        for (int j = 0; j < 16; ++j)
            for (int r = 0; r < 16; ++r)
                for (; count[j][r] > 0; --count[j][r]) {
                    int32_t at = -1;
                    for (int32_t t = 0; t < steps; ++t)
                        if (table[(size_t)t * 16 + j] >= zero_base) {
                            if (at < 0) at = t;
                            if (!(doubled[(size_t)t] >> r & 1)) {
                                at = t;
                                break;
                            }
                        }
                    if (at < 0) return false;
                    table[(size_t)at * 16 + j] = bucket[j][(size_t)next[j][r]++];
                    doubled[(size_t)at] |= (uint16_t)(1u << r);
                }
        for (int32_t t = 0; t < steps; ++t)
            for (int j = 0; j < 16; ++j) emit(j, t, table[(size_t)t * 16 + j]);
        return true;
    }

private:
    static bool augment(int j, const int32_t (&w)[16][16], int (&rec_of)[16], int (&grp_of)[16], uint32_t& seen)
    {
        for (int r = 0; r < 16; ++r) {
            if (w[j][r] <= 0 || (seen >> r & 1)) continue;
            seen |= 1u << r;
            if (rec_of[r] < 0 || augment(rec_of[r], w, rec_of, grp_of, seen)) {
                rec_of[r] = j;
                grp_of[j] = r;
                return true;
            }
        }
        return false;
    }
};

}  // namespace

// The schedule of the LDS pass.  Every segment of the plan is cut into its hot non-zeros
// (source on the list its row's set gathers from) and the others.  Segments are put in an
// order of their own -- set by set, most hot non-zeros first -- and a segment's place in it
// is its *position*.  The LDS launch takes the hot parts, 64 consecutive positions to a
// group (one per lane; every lane walks as many steps as its group needs, so segments of
// like length share a group), and leaves each sum in the plane entry of its position; the
// segment kernel then walks the other parts in position order, adds the plane entry and
// finishes the segment as the plan says (output row or partial-row slot).  Two orders for a
// segment's reads: the column list's, or (where the padding it costs is less than what it
// gains) the conflict-free order of PassGroup.  Either way the order is fixed by the
// schedule, so a sum repeats bit for bit.
bool build_lds_schedule(const gp_plan& P, const HotSets& C, double max_cost, int order, LdsSchedule& out)
{
    const int64_t n = P.n;
    const int32_t num = C.num_sets;
    const int64_t nsegs = (int64_t)P.segs.size();
    if (num <= 0 || C.num_lists <= 0 || nsegs == 0) return false;
    std::vector<int32_t> hot_len;
    hot_first(P, C, out.col, hot_len);
    for (int32_t& h : hot_len)
        if (h < C.min_hot) h = 0;  // (the columns stay reordered: the segment kernel then takes them all)
    // the lists' rows, ascending, and every row's place on its list
    out.member_off.assign((size_t)C.num_lists + 1, 0);
    for (int64_t i = 0; i < n; ++i)
        if (C.list_of_row[(size_t)i] >= 0) ++out.member_off[(size_t)C.list_of_row[(size_t)i] + 1];
    for (int32_t l = 0; l < C.num_lists; ++l) out.member_off[(size_t)l + 1] += out.member_off[(size_t)l];
    out.members.resize((size_t)out.member_off[(size_t)C.num_lists]);
    std::vector<int32_t> local((size_t)n, 0);
    {
        std::vector<int64_t> fill(out.member_off.begin(), out.member_off.end() - 1);
        for (int64_t i = 0; i < n; ++i) {
            const int32_t l = C.list_of_row[(size_t)i];
            if (l < 0) continue;
            local[(size_t)i] = (int32_t)(fill[(size_t)l] - out.member_off[(size_t)l]);
            out.members[(size_t)fill[(size_t)l]++] = (int32_t)i;
        }
    }
    out.list_of_set = C.list_of_set;
    auto members_of_set = [&](int32_t c) {
        const int32_t l = C.list_of_set[(size_t)c];
        return out.member_off[(size_t)l + 1] - out.member_off[(size_t)l];
    };
    // positions: the segments set by set, inside a set most hot non-zeros first (stable)
    std::vector<int64_t> pos_off((size_t)num + 1, 0);
    out.hot_edges = 0;
    for (int64_t s = 0; s < nsegs; ++s) {
        ++pos_off[(size_t)C.set_of_row[(size_t)P.segs[(size_t)s].row] + 1];
        out.hot_edges += hot_len[(size_t)s];
    }
    if (out.hot_edges == 0) return false;
    for (int32_t c = 0; c < num; ++c) pos_off[(size_t)c + 1] += pos_off[(size_t)c];
    std::vector<int64_t> seg_at((size_t)nsegs);  // position -> segment
    {
        std::vector<int64_t> fill(pos_off.begin(), pos_off.end() - 1);
        for (int64_t s = 0; s < nsegs; ++s) seg_at[(size_t)fill[(size_t)C.set_of_row[(size_t)P.segs[(size_t)s].row]]++] = s;
    }
    const int nt = P.nnz < (1 << 16) ? 1 : host_threads();
    parallel_run(nt, [&](int t, int k) {
        for (int32_t c = (int32_t)((int64_t)num * t / k); c < (int32_t)((int64_t)num * (t + 1) / k); ++c)
            std::stable_sort(seg_at.begin() + pos_off[(size_t)c], seg_at.begin() + pos_off[(size_t)c + 1],
                             [&](int64_t a, int64_t b) { return hot_len[(size_t)a] > hot_len[(size_t)b]; });
    });
    // the other parts, in position order, for the segment kernel
    out.cold.resize((size_t)nsegs);
    parallel_run(nt, [&](int t, int k) {
        for (int64_t p = nsegs * t / k; p < nsegs * (t + 1) / k; ++p) {
            const int64_t s = seg_at[(size_t)p];
            Segment q = P.segs[(size_t)s];
            const int64_t start = (((int64_t)q.start_hi << 32) | q.start_lo) + hot_len[(size_t)s];
            q.start_lo = (uint32_t)(start & 0xFFFFFFFF);
            q.start_hi = (uint8_t)(start >> 32);
            q.len = (uint16_t)(q.len - hot_len[(size_t)s]);
            q.slice = hot_len[(size_t)s] > 0 ? kAddPlaneEntry : 0;
            out.cold[(size_t)p] = q;
        }
    });
    // groups: 64 consecutive positions of one set, as far as the set's segments have hot non-zeros
    out.max_members = 0;
    out.group_off.assign((size_t)num + 1, 0);
    std::vector<int32_t> group_set;
    std::vector<int64_t> group_pos;  // first position of the group
    for (int32_t c = 0; c < num; ++c) {
        int64_t with_hot = 0;  // (sorted: they come first)
        while (pos_off[(size_t)c] + with_hot < pos_off[(size_t)c + 1] && hot_len[(size_t)seg_at[(size_t)(pos_off[(size_t)c] + with_hot)]] > 0)
            ++with_hot;
        if (with_hot > 0) {
            if (members_of_set(c) > kLdsMaxMembers) return false;
            out.max_members = (int32_t)std::max<int64_t>(out.max_members, members_of_set(c));
        }
        const int64_t g = (with_hot + 63) / 64;
        if ((int64_t)group_set.size() + g > INT32_MAX) return false;
        for (int64_t i = 0; i < g; ++i) {
            group_set.push_back(c);
            group_pos.push_back(pos_off[(size_t)c] + 64 * i);
        }
        out.group_off[(size_t)c + 1] = (int32_t)group_set.size();
    }
    const int64_t ngroups = (int64_t)group_set.size();
    // lane l of group g: the segment at position group_pos[g] + l, if that is still in the set and has hot non-zeros
    auto segment_of = [&](int64_t g, int lane) -> int64_t {
        const int64_t p = group_pos[(size_t)g] + lane;
        if (p >= pos_off[(size_t)group_set[(size_t)g] + 1]) return -1;
        const int64_t s = seg_at[(size_t)p];
        return hot_len[(size_t)s] > 0 ? s : -1;
    };
    auto hot_start = [&](int64_t s) { return out.col.data() + (((int64_t)P.segs[(size_t)s].start_hi << 32) | P.segs[(size_t)s].start_lo); };
    auto load_pass = [&](PassGroup& pg, int64_t g, int pass, int (&lanes)[16]) {
        int k = 0;
        for (int l = 0; l < 64; ++l)
            if (lds_pass_of_lane(l) == pass) lanes[k++] = l;
        for (int j = 0; j < 16; ++j) {
            const int64_t s = segment_of(g, lanes[j]);
            if (s >= 0) pg.load(j, hot_start(s), hot_len[(size_t)s], local.data());
            else pg.clear(j);
        }
    };
    // steps per group in either order
    std::vector<int32_t> steps_plain((size_t)ngroups), steps_free((size_t)ngroups, 0);
    parallel_run(nt, [&](int t, int k) {
        for (int64_t g = ngroups * t / k; g < ngroups * (t + 1) / k; ++g) {
            steps_plain[(size_t)g] = (hot_len[(size_t)segment_of(g, 0)] + 7) / 8 * 8;
            steps_free[(size_t)g] = steps_plain[(size_t)g];  // (the order with as few conflicts as these steps allow)
        }
    });
    int64_t total_plain = 0, total_free = 0;
    for (int64_t g = 0; g < ngroups; ++g) {
        total_plain += 64 * (int64_t)steps_plain[(size_t)g];
        total_free += 64 * (int64_t)steps_free[(size_t)g];
    }
    // cost of an order = its reads, padding included, a conflict-free read counting 1 / kLdsConflictFreeGain
    const double cost_free = (double)total_free / kLdsConflictFreeGain, cost_plain = (double)total_plain;
    out.conflict_free = order == 2 || (order == 0 && cost_free <= cost_plain);
    const std::vector<int32_t>& steps = out.conflict_free ? steps_free : steps_plain;
    if ((out.conflict_free ? cost_free : cost_plain) > max_cost * (double)out.hot_edges) return false;
    // Staging a strip costs a workgroup some microseconds whatever the set has to read from it: sets
    // with little to read (many tiny clusters) are better served by the L2s.
    if (max_cost < kLdsForcedCost) {
        int64_t busy_sets = 0;
        for (int32_t c = 0; c < num; ++c) busy_sets += out.group_off[(size_t)c + 1] > out.group_off[(size_t)c];
        if ((out.conflict_free ? total_free : total_plain) < kLdsMinReadsPerSet * busy_sets) return false;
    }
    out.groups.resize((size_t)ngroups);
    int64_t id_total = 0;
    for (int64_t g = 0; g < ngroups; ++g) {
        int32_t count = 0;
        while (count < 64 && segment_of(g, count) >= 0) ++count;  // (sorted: the lanes with a segment come first)
        out.groups[(size_t)g] = LdsGroup{id_total, group_pos[(size_t)g], steps[(size_t)g], count};
        id_total += 64 * (int64_t)steps[(size_t)g];
    }
    out.groups.push_back(LdsGroup{id_total, 0, 0, 0});  // sentinel: where the last group's indices end
    out.set_reads.assign((size_t)num, 0);
    for (int32_t c = 0; c < num; ++c)
        out.set_reads[(size_t)c] = out.groups[(size_t)out.group_off[(size_t)c + 1]].id_off - out.groups[(size_t)out.group_off[(size_t)c]].id_off;
    // a set's groups in kWaveCuts runs of about equal cost (a run per wave, or two)
    out.wave_cut.assign((size_t)num * (kWaveCuts + 1), 0);
    for (int32_t c = 0; c < num; ++c) {
        const int32_t g0 = out.group_off[(size_t)c], g1 = out.group_off[(size_t)c + 1];
        // what the groups before g cost a wave: their reads, and per group (its sums stored, the next one's
        // descriptor taken up) about as much as kLdsGroupCostSteps steps
        auto cost_to = [&](int32_t g) {
            return (out.groups[(size_t)g].id_off - out.groups[(size_t)g0].id_off) + 64 * (int64_t)kLdsGroupCostSteps * (int64_t)(g - g0);
        };
        const int64_t all = cost_to(g1);
        int32_t g = g0;
        for (int w = 0; w <= kWaveCuts; ++w) {
            const int64_t target = all * w / kWaveCuts;
            while (g < g1 && cost_to(g) < target) ++g;
            out.wave_cut[(size_t)c * (kWaveCuts + 1) + w] = w == kWaveCuts ? g1 : g;
        }
    }
    out.ids.resize((size_t)id_total);
    std::atomic<bool> ok{true};
    parallel_run(nt, [&](int t, int k) {
        PassGroup pg;
        int lanes[16];
        for (int64_t g = ngroups * t / k; g < ngroups * (t + 1) / k; ++g) {
            const int64_t m = members_of_set(group_set[(size_t)g]);
            const uint16_t zero_base = (uint16_t)((m + 15) / 16 * 16);  // 16 zero rows, one per bank group
            const LdsGroup& G = out.groups[(size_t)g];
            auto slot_of = [&](int lane, int32_t step) -> uint16_t& {
                return out.ids[(size_t)(G.id_off + (int64_t)(step / 8) * 512 + lane * 8 + step % 8)];
            };
            if (out.conflict_free) {
                for (int pass = 0; pass < 4; ++pass) {
                    load_pass(pg, g, pass, lanes);
                    if (!pg.schedule(G.steps, zero_base, [&](int j, int32_t step, uint16_t id) { slot_of(lanes[j], step) = id; }))
                        ok = false;
                }
            } else {
                for (int l = 0; l < 64; ++l) {
                    const int64_t s = segment_of(g, l);
                    const int32_t len = s >= 0 ? hot_len[(size_t)s] : 0;
                    const int32_t* col = s >= 0 ? hot_start(s) : nullptr;
                    for (int32_t st = 0; st < G.steps; ++st) slot_of(l, st) = st < len ? (uint16_t)local[(size_t)col[st]] : zero_base;
                }
            }
        }
    });
    return ok;
}

void deal_lds_octets(const std::vector<int64_t>& set_reads, int strips, std::vector<LdsOctet>& octets, int64_t (&off)[9])
{
    const int per_set = (strips + 7) / 8;
    std::vector<std::vector<LdsOctet>> mine(8);
    double load[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int32_t c = 0; c < (int32_t)set_reads.size(); ++c) {
        if (set_reads[(size_t)c] == 0) continue;
        for (int k = 0; k < per_set; ++k) {
            int x = 0;
            for (int y = 1; y < 8; ++y)
                if (load[y] < load[x]) x = y;
            mine[(size_t)x].push_back(LdsOctet{c, k});
            load[x] += (double)set_reads[(size_t)c] * (double)std::min(8, strips - 8 * k);
        }
    }
    octets.clear();
    for (int x = 0; x < 8; ++x) {
        off[x] = (int64_t)octets.size();
        octets.insert(octets.end(), mine[(size_t)x].begin(), mine[(size_t)x].end());
    }
    off[8] = (int64_t)octets.size();
}

}  // namespace gp
