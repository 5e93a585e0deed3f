// Kernel schedule of a plan: every edge block is cut into segments (runs of
// consecutive non-zeros of one row, at most `segment_edges` long, never crossing
// a block boundary).  A row that ends up as a single segment is written straight
// to the output; a row cut by a block boundary (the case the paper's Limitation
// paragraph of Section 3.2 names: one node's edges may land in different groups)
// or by the length limit becomes several partial rows that a fix-up kernel adds
// in list order (Algorithm 1's accumulation over edge blocks, confined to the
// rows that need it).  Inside a block the segments are ordered longest first so
// the lane groups of a wavefront get similar lengths and long runs start early.
#include <algorithm>
#include <functional>

#include "gp_internal.h"

namespace gp {

namespace {

// P supplies the sorted list (rowptr, nnz, n); the cut into blocks is the caller's.
struct CutPlan {
    const gp_plan& plan;
    const std::vector<int64_t>& block_off;
    const std::vector<int64_t>& rowptr;
    int64_t nnz, n;
    int32_t num_blocks;
    CutPlan(const gp_plan& p, const std::vector<int64_t>& off)
        : plan(p), block_off(off), rowptr(p.rowptr), nnz(p.nnz), n(p.n), num_blocks((int32_t)off.size() - 1)
    {
    }
};

struct Cutter {
    const CutPlan P;
    int64_t L;
    Cutter(const gp_plan& p, const std::vector<int64_t>& off) : P(p, off), L(p.segment_edges) {}

    int32_t block_of(int64_t e) const
    {
        if (e >= P.nnz) return P.num_blocks - 1;
        return (int32_t)(std::upper_bound(P.block_off.begin(), P.block_off.end(), e) - P.block_off.begin() - 1);
    }
    // number of segments row r is cut into, over all blocks (1 for an empty row)
    int64_t pieces(int64_t r) const
    {
        int64_t s = P.rowptr[r];
        const int64_t e = P.rowptr[r + 1];
        if (e == s) return 1;
        int32_t p = block_of(s);
        int64_t total = 0;
        while (s < e) {
            const int64_t hi = std::min(e, P.block_off[p + 1]);
            total += (hi - s + L - 1) / L;
            s = hi;
            ++p;
        }
        return total;
    }
    // pieces of row r that lie in blocks before entry `pos`
    int64_t pieces_before(int64_t r, int64_t pos) const
    {
        int64_t s = P.rowptr[r];
        if (s >= pos) return 0;
        int32_t p = block_of(s);
        int64_t total = 0;
        while (s < pos) {
            const int64_t hi = std::min(pos, P.block_off[p + 1]);
            total += (hi - s + L - 1) / L;
            s = hi;
            ++p;
        }
        return total;
    }
    // first row that block p has work for, and one past the last
    void rows_of_block(int32_t p, int64_t& r0, int64_t& r1) const
    {
        const int64_t lo = P.block_off[p], hi = P.block_off[p + 1];
        const bool last = p == P.num_blocks - 1;
        r0 = std::lower_bound(P.rowptr.begin(), P.rowptr.end() - 1, lo) - P.rowptr.begin();
        if (r0 == P.n || P.rowptr[r0] > lo) --r0;  // the row that straddles lo
        if (r0 < 0) r0 = 0;
        if (last)
            r1 = P.n;
        else
            r1 = std::lower_bound(P.rowptr.begin(), P.rowptr.end() - 1, hi) - P.rowptr.begin();
    }
    // calls emit(row, start, len, piece_index) for every segment of block p
    template <class F>
    void walk(int32_t p, F&& emit) const
    {
        const int64_t lo = P.block_off[p], hi = P.block_off[p + 1];
        int64_t r0, r1;
        rows_of_block(p, r0, r1);
        for (int64_t r = r0; r < r1; ++r) {
            const int64_t rs = P.rowptr[r], re = P.rowptr[r + 1];
            if (rs == re) {
                // an empty row still owes a zero output row; it belongs to the block
                // that holds list position rs (the last block if rs is the end)
                if ((rs >= lo && rs < hi) || (rs >= P.nnz && p == P.num_blocks - 1)) emit(r, rs, 0, 0);
                continue;
            }
            int64_t s = std::max(rs, lo);
            const int64_t e = std::min(re, hi);
            if (s >= e) continue;
            int64_t idx = rs < lo ? pieces_before(r, lo) : 0;
            for (; s < e; s += L, ++idx) emit(r, s, std::min(L, e - s), idx);
        }
    }
};

}  // namespace

gp_status build_schedule(gp_plan* plan)
{
    return cut_schedule(*plan, plan->block_off, plan->segs, plan->seg_off, plan->split, plan->num_slots);
}

gp_status cut_schedule(const gp_plan& plan, const std::vector<int64_t>& block_off, std::vector<Segment>& out_segs,
                       std::vector<int64_t>& out_seg_off, std::vector<SplitRow>& out_split, int64_t& out_num_slots)
{
    const int64_t L = plan.segment_edges;
    if (L < 8 || L > 32768) return fail(GP_ERR_INVALID_ARG, "segment_edges = %lld outside 8 .. 32768", (long long)L);
    if (block_off.size() < 2) return fail(GP_ERR_INVALID_ARG, "a schedule needs at least one block");
    Cutter cut(plan, block_off);
    // the names the body below uses
    struct Out {
        const std::vector<int64_t>& rowptr;
        int64_t n, nnz;
        std::vector<Segment>& segs;
        std::vector<int64_t>& seg_off;
        std::vector<SplitRow>& split;
        int64_t& num_slots;
    } P{plan.rowptr, plan.n, plan.nnz, out_segs, out_seg_off, out_split, out_num_slots};
    const int32_t b = (int32_t)block_off.size() - 1;
    const int nt = (P.n + P.nnz < (1 << 16)) ? 1 : host_threads();

    // split rows and their carry slots, in ascending row order
    {
        std::vector<std::vector<SplitRow>> part((size_t)nt);
        parallel_run(nt, [&](int t, int k) {
            const int64_t lo = P.n * t / k, hi = P.n * (t + 1) / k;
            for (int64_t r = lo; r < hi; ++r) {
                // cheap filter first: a short row strictly inside one block is one piece
                const int64_t s = P.rowptr[r], e = P.rowptr[r + 1];
                if (e - s <= L && (e == s || cut.block_of(s) == cut.block_of(e - 1))) continue;
                const int64_t c = cut.pieces(r);
                if (c > 1) part[t].push_back(SplitRow{(int32_t)r, (int32_t)c, 0});
            }
        });
        P.split.clear();
        int64_t slot = 0;
        for (auto& v : part)
            for (auto& s : v) {
                s.first_slot = slot;
                slot += s.count;
                P.split.push_back(s);
            }
        P.num_slots = slot;
    }
    auto first_slot_of = [&](int32_t row) -> int64_t {
        auto it = std::lower_bound(P.split.begin(), P.split.end(), row,
                                   [](const SplitRow& s, int32_t r) { return s.row < r; });
        return (it != P.split.end() && it->row == row) ? it->first_slot : -1;
    };
    if (P.num_slots > INT32_MAX) return fail(GP_ERR_OVERFLOW, "%lld partial rows exceed int32", (long long)P.num_slots);

    // segments per block
    P.seg_off.assign((size_t)b + 1, 0);
    parallel_run(std::min<int>(nt, b), [&](int t, int k) {
        for (int32_t p = t; p < b; p += k) {
            int64_t c = 0;
            cut.walk(p, [&](int64_t, int64_t, int64_t, int64_t) { ++c; });
            P.seg_off[(size_t)p + 1] = c;
        }
    });
    for (int32_t p = 0; p < b; ++p) P.seg_off[p + 1] += P.seg_off[p];
    P.segs.resize((size_t)P.seg_off[b]);

    parallel_run(std::min<int>(nt, b), [&](int t, int k) {
        std::vector<Segment> tmp;
        std::vector<int64_t> hist;
        for (int32_t p = t; p < b; p += k) {
            tmp.clear();
            cut.walk(p, [&](int64_t r, int64_t s, int64_t len, int64_t idx) {
                Segment g;
                g.start_lo = (uint32_t)(s & 0xFFFFFFFF);
                g.start_hi = (uint8_t)(s >> 32);
                g.slice = 0;
                g.len = (uint16_t)len;
                g.row = (int32_t)r;
                const int64_t fs = first_slot_of((int32_t)r);
                g.slot = fs < 0 ? -1 : (int32_t)(fs + idx);
                tmp.push_back(g);
            });
            // stable counting sort, longest first
            hist.assign((size_t)L + 2, 0);
            for (const Segment& g : tmp) ++hist[(size_t)(L - g.len) + 1];
            for (int64_t i = 0; i <= L; ++i) hist[i + 1] += hist[i];
            Segment* out = P.segs.data() + P.seg_off[p];
            for (const Segment& g : tmp) out[hist[(size_t)(L - g.len)]++] = g;
        }
    });
    return GP_OK;
}

}  // namespace gp
