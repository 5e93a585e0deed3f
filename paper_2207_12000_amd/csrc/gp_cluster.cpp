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
//      the XCD with the least work so far.
//
// Graphs without such structure (one giant cluster, or clusters whose sources do
// not fit an L2 at any useful slice width) keep the implicit lists.
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
void build_split_schedule(const gp_plan& P, const RowClusters& C, SplitSchedule& out)
{
    const int64_t nsegs = (int64_t)P.segs.size();
    out.col.resize(P.col.size());
    std::vector<int32_t> hot_len((size_t)nsegs);
    const int nt = P.nnz < (1 << 16) ? 1 : host_threads();
    parallel_run(nt, [&](int t, int k) {
        for (int64_t s = nsegs * t / k; s < nsegs * (t + 1) / k; ++s) {
            const Segment& g = P.segs[(size_t)s];
            const int64_t e0 = ((int64_t)g.start_hi << 32) | g.start_lo;
            const int32_t li = C.label[(size_t)g.row];
            int64_t w = e0;
            for (int64_t e = e0; e < e0 + g.len; ++e)
                if (C.label[(size_t)P.col[(size_t)e]] == li) out.col[(size_t)w++] = P.col[(size_t)e];
            hot_len[(size_t)s] = (int32_t)(w - e0);
            for (int64_t e = e0; e < e0 + g.len; ++e)
                if (C.label[(size_t)P.col[(size_t)e]] != li) out.col[(size_t)w++] = P.col[(size_t)e];
        }
    });
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

}  // namespace gp
