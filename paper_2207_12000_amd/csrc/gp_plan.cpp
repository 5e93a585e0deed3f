// gp_plan_blocks: host-side edge decomposition (paper Section 3.2, "Precomputation
// on GPU": disjoint balanced edge sets; Eq. 1 for the degree vectors).
//
// Pipeline, all integer work, threaded over row ranges:
//   validate ids -> count candidates per row -> bucket columns by row ->
//   sort + unique inside each row -> degrees / rowptr -> compact -> norms ->
//   equal-count block offsets -> kernel schedule (gp_schedule.cpp).
// Bucketing by row first keeps every sort tiny (one row), so the whole plan is
// two streaming passes over the input plus one pass over the output.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <exception>
#include <functional>
#include <new>
#include <thread>

#include "gp_internal.h"

namespace gp {

int host_threads()
{
    unsigned hw = std::thread::hardware_concurrency();
    if (hw == 0) hw = 1;
    return (int)std::min<unsigned>(hw, 16u);
}

void parallel_run(int nthreads, const std::function<void(int, int)>& fn)
{
    if (nthreads <= 1) {
        fn(0, 1);
        return;
    }
    // an exception inside a worker (e.g. bad_alloc) must reach the caller, not terminate the process
    std::vector<std::thread> th;
    std::vector<std::exception_ptr> err((size_t)nthreads);
    th.reserve(nthreads);
    for (int t = 0; t < nthreads; ++t)
        th.emplace_back([&fn, &err, t, nthreads] {
            try {
                fn(t, nthreads);
            } catch (...) {
                err[(size_t)t] = std::current_exception();
            }
        });
    for (auto& x : th) x.join();
    for (auto& e : err)
        if (e) std::rethrow_exception(e);
}

static inline void chunk_of(int64_t total, int t, int nt, int64_t& lo, int64_t& hi)
{
    lo = total * t / nt;
    hi = total * (t + 1) / nt;
}

}  // namespace gp

using namespace gp;

extern "C" gp_status gp_plan_blocks(const int32_t* src, const int32_t* dst, int64_t m, int64_t n,
                                    int64_t block_budget_edges, uint32_t flags, gp_plan** out_plan)
{
    if (out_plan) *out_plan = nullptr;
    if (!out_plan) return fail(GP_ERR_INVALID_ARG, "out_plan is NULL");
    if (m < 0) return fail(GP_ERR_INVALID_ARG, "m = %lld is negative", (long long)m);
    if (m > 0 && (!src || !dst)) return fail(GP_ERR_INVALID_ARG, "src/dst is NULL with m > 0");
    if (n <= 0 || n > INT32_MAX) return fail(GP_ERR_INVALID_ARG, "n = %lld outside 1 .. 2^31-1", (long long)n);
    if (block_budget_edges <= 0) return fail(GP_ERR_INVALID_ARG, "block budget must be positive");
    if (flags & ~(uint32_t)(GP_SYMMETRISE | GP_ADD_SELF_LOOPS | GP_PLAN_ON_DEVICE))
        return fail(GP_ERR_INVALID_ARG, "unknown plan flag 0x%x", flags);
    const bool sym = flags & GP_SYMMETRISE, loops = flags & GP_ADD_SELF_LOOPS;
    // every candidate count must stay far inside int64 and the 40-bit segment start
    if (m > (INT64_C(1) << 38)) return fail(GP_ERR_OVERFLOW, "m = %lld is too large", (long long)m);

    const int nt = (m + n < (1 << 16)) ? 1 : host_threads();
    gp_plan* plan = nullptr;
    try {
        plan = new gp_plan();
        plan->n = n;
        plan->flags = flags;
        plan->opt = options();

        // 1. validate
        std::atomic<int64_t> bad{-1};
        parallel_run(nt, [&](int t, int k) {
            int64_t lo, hi;
            chunk_of(m, t, k, lo, hi);
            for (int64_t e = lo; e < hi; ++e) {
                const uint32_t s = (uint32_t)src[e], d = (uint32_t)dst[e];
                if (s >= (uint64_t)n || d >= (uint64_t)n) {
                    int64_t expect = -1;
                    bad.compare_exchange_strong(expect, e);
                    return;
                }
            }
        });
        if (bad.load() >= 0) {
            const int64_t e = bad.load();
            gp_plan_destroy(plan);
            return fail(GP_ERR_INDEX_RANGE, "pair %lld = (%d, %d) has a node id outside [0, %lld)", (long long)e,
                        src[e], dst[e], (long long)n);
        }

        if (flags & GP_PLAN_ON_DEVICE) {
            // sort / unique / row pointers on the current GPU; same arrays, bit for bit
            gp_status st = csr_on_device(src, dst, m, n, sym, loops, plan);
            if (st != GP_OK) {
                gp_plan_destroy(plan);
                return st;
            }
        } else {
            // 2. candidates per row (before duplicates collapse)
            std::vector<int64_t> cand_ptr((size_t)n + 1, 0);
            {
                int64_t* cnt = cand_ptr.data() + 1;
                if (loops)
                    for (int64_t i = 0; i < n; ++i) cnt[i] = 1;
                parallel_run(nt, [&](int t, int k) {
                    int64_t lo, hi;
                    chunk_of(m, t, k, lo, hi);
                    for (int64_t e = lo; e < hi; ++e) {
                        const int32_t s = src[e], d = dst[e];
                        if (s == d) continue;
                        __atomic_fetch_add(&cnt[d], 1, __ATOMIC_RELAXED);
                        if (sym) __atomic_fetch_add(&cnt[s], 1, __ATOMIC_RELAXED);
                    }
                });
                for (int64_t i = 0; i < n; ++i) cand_ptr[i + 1] += cand_ptr[i];
            }
            const int64_t ncand = cand_ptr[n];

            // 3. bucket the column ids by row
            std::vector<int32_t> cand((size_t)ncand);
            {
                std::vector<int64_t> cursor(cand_ptr.begin(), cand_ptr.end() - 1);
                if (loops)
                    for (int64_t i = 0; i < n; ++i) cand[cursor[i]++] = (int32_t)i;
                parallel_run(nt, [&](int t, int k) {
                    int64_t lo, hi;
                    chunk_of(m, t, k, lo, hi);
                    for (int64_t e = lo; e < hi; ++e) {
                        const int32_t s = src[e], d = dst[e];
                        if (s == d) continue;
                        cand[__atomic_fetch_add(&cursor[d], 1, __ATOMIC_RELAXED)] = s;
                        if (sym) cand[__atomic_fetch_add(&cursor[s], 1, __ATOMIC_RELAXED)] = d;
                    }
                });
            }

            // 4. sort + unique inside each row; threads own row ranges of similar candidate count
            plan->deg.assign((size_t)n, 0);
            std::vector<int64_t> row_cut((size_t)nt + 1);
            for (int t = 0; t <= nt; ++t) {
                const int64_t target = ncand / nt * t + std::min<int64_t>(t, ncand % nt);
                row_cut[t] = std::lower_bound(cand_ptr.begin(), cand_ptr.end(), target) - cand_ptr.begin();
                if (row_cut[t] > n) row_cut[t] = n;
            }
            row_cut[0] = 0;
            row_cut[nt] = n;
            parallel_run(nt, [&](int t, int) {
                for (int64_t i = row_cut[t]; i < row_cut[t + 1]; ++i) {
                    int32_t* b = cand.data() + cand_ptr[i];
                    int32_t* e = cand.data() + cand_ptr[i + 1];
                    std::sort(b, e);
                    plan->deg[i] = (int32_t)(std::unique(b, e) - b);
                }
            });

            // 5. rowptr and the compacted column list
            plan->rowptr.assign((size_t)n + 1, 0);
            for (int64_t i = 0; i < n; ++i) plan->rowptr[i + 1] = plan->rowptr[i] + plan->deg[i];
            const int64_t nnz = plan->rowptr[n];
            if (nnz >= (INT64_C(1) << 40)) {
                gp_plan_destroy(plan);
                return fail(GP_ERR_OVERFLOW, "non-zero count %lld exceeds the 40-bit list index", (long long)nnz);
            }
            plan->nnz = nnz;
            plan->col.resize((size_t)nnz);
            parallel_run(nt, [&](int t, int) {
                for (int64_t i = row_cut[t]; i < row_cut[t + 1]; ++i)
                    if (plan->deg[i])
                        std::memcpy(plan->col.data() + plan->rowptr[i], cand.data() + cand_ptr[i],
                                    sizeof(int32_t) * (size_t)plan->deg[i]);
            });
            std::vector<int32_t>().swap(cand);
            std::vector<int64_t>().swap(cand_ptr);

        }
        const int64_t nnz = plan->nnz;

        // 6. normalisation vectors: one correctly rounded recipe, fp64 then narrowed once
        //    (the device planner has made them already, by the same recipe)
        if (!plan->norms_on_device) {
            plan->dinv_sqrt.resize((size_t)n);
            plan->dinv.resize((size_t)n);
        }
        if (!plan->norms_on_device) parallel_run(nt, [&](int t, int k) {
            int64_t lo, hi;
            chunk_of(n, t, k, lo, hi);
            for (int64_t i = lo; i < hi; ++i) {
                const int32_t g = plan->deg[i];
                plan->dinv_sqrt[i] = g > 0 ? (float)(1.0 / std::sqrt((double)g)) : 0.0f;
                plan->dinv[i] = g > 0 ? (float)(1.0 / (double)g) : 0.0f;
            }
        });

        // 7. balanced contiguous blocks
        int64_t b = (nnz + block_budget_edges - 1) / block_budget_edges;
        if (b < 1) b = 1;
        if (b > INT32_MAX) {
            gp_plan_destroy(plan);
            return fail(GP_ERR_OVERFLOW, "block count %lld does not fit int32", (long long)b);
        }
        plan->num_blocks = (int32_t)b;
        plan->block_off.resize((size_t)b + 1);
        plan->block_row_lo.assign((size_t)b, 0);
        plan->block_row_hi.assign((size_t)b, -1);
        const int64_t q = nnz / b, r = nnz % b;
        for (int64_t p = 0; p <= b; ++p) plan->block_off[p] = p * q + std::min(p, r);
        if (flags & GP_PLAN_ON_DEVICE) {
            gp_status st = block_rows_on_device(plan);
            if (st != GP_OK) {
                gp_plan_destroy(plan);
                return st;
            }
        }
        for (int64_t p = 0; p < b && !(flags & GP_PLAN_ON_DEVICE); ++p) {
            const int64_t lo = plan->block_off[p], hi = plan->block_off[p + 1];
            if (hi <= lo) continue;
            // row of entry e = (first i with rowptr[i+1] > e)
            auto row_of = [&](int64_t e) {
                return (int32_t)(std::upper_bound(plan->rowptr.begin(), plan->rowptr.end(), e) -
                                 plan->rowptr.begin() - 1);
            };
            plan->block_row_lo[p] = row_of(lo);
            plan->block_row_hi[p] = row_of(hi - 1);
        }

        // Longest run one lane group walks alone.  A run is a serial chain of gathers,
        // so it must stay short against the whole hop: about nnz / 65536, kept within
        // 64 .. 1024 (small graphs: split hubs finely; large graphs: split rarely, so
        // few rows need partial sums).
        int64_t L = plan->opt.segment_edges;
        if (L <= 0) {
            L = 64;
            while (L < 1024 && L * 2 <= nnz / 65536) L *= 2;
        }
        plan->segment_edges = L;
        gp_status st = build_schedule(plan);
        if (st != GP_OK) {
            gp_plan_destroy(plan);
            return st;
        }
    } catch (const std::bad_alloc&) {
        gp_plan_destroy(plan);
        return fail(GP_ERR_OOM_HOST, "host allocation failed while planning (m = %lld, n = %lld)", (long long)m,
                    (long long)n);
    } catch (const std::exception& e) {  // e.g. no more threads: a host resource ran out
        gp_plan_destroy(plan);
        return fail(GP_ERR_OOM_HOST, "planning failed: %s", e.what());
    }
    *out_plan = plan;
    return GP_OK;
}
