// Streamed schedule: X and the hop stack live in pinned host memory and only a
// bounded part of the problem is in HBM at any time (the situation Section 3.2
// is written for: the edge list and the features do not fit on the GPU, Eq. 12).
//
// What stays on the device for the whole call: the two normalisation vectors,
// the list of cut rows, the partial-row buffer, two column slabs of the feature
// matrix (n x w) and two edge-block buffers.  The block count b is fixed by the
// plan; the slab width w (the paper's column blocks, c = ceil(d / w)) is the
// largest that fits the HBM budget.  Unlike Algorithm 1, which re-uploads every
// edge block for every column block of every hop AND moves every slab in and out
// once per hop, a slab here stays in HBM across all K hops (the hops of one
// column slab do not depend on the other slabs), so features cross the host link
// once in and K times out (slab 0 = X is a host-to-host copy done by host threads
// meanwhile), and only the edge blocks are re-sent, c*K times, double-buffered on a
// side stream while the previous block is being computed -- or sent just once and
// kept, when the budget has room for all of them.
#include <algorithm>
#include <cstring>
#include <thread>

#include "gp_internal.h"

namespace gp {

namespace {

struct Streams {
    hipStream_t in = nullptr, cmp = nullptr, out = nullptr;
    std::vector<hipEvent_t> blk_ready, blk_free;  // one pair per edge-block buffer
    hipEvent_t hop_done = nullptr, out_done[2] = {nullptr, nullptr};
    std::vector<void*> dev;

    ~Streams()
    {
        if (in) (void)hipStreamSynchronize(in);
        if (cmp) (void)hipStreamSynchronize(cmp);
        if (out) (void)hipStreamSynchronize(out);
        for (void* p : dev) (void)hipFree(p);
        for (hipEvent_t e : blk_ready) (void)hipEventDestroy(e);
        for (hipEvent_t e : blk_free) (void)hipEventDestroy(e);
        for (hipEvent_t e : {hop_done, out_done[0], out_done[1]})
            if (e) (void)hipEventDestroy(e);
        if (in) (void)hipStreamDestroy(in);
        if (cmp) (void)hipStreamDestroy(cmp);
        if (out) (void)hipStreamDestroy(out);
    }
    gp_status init(int block_buffers)
    {
        // default priority on purpose: all three streams are peers
        GP_HIP(hipStreamCreateWithFlags(&in, hipStreamNonBlocking));
        GP_HIP(hipStreamCreateWithFlags(&cmp, hipStreamNonBlocking));
        GP_HIP(hipStreamCreateWithFlags(&out, hipStreamNonBlocking));
        for (hipEvent_t* e : {&hop_done, &out_done[0], &out_done[1]}) GP_HIP(hipEventCreateWithFlags(e, hipEventDisableTiming));
        for (int i = 0; i < block_buffers; ++i) {
            hipEvent_t a = nullptr, b = nullptr;
            GP_HIP(hipEventCreateWithFlags(&a, hipEventDisableTiming));
            blk_ready.push_back(a);
            GP_HIP(hipEventCreateWithFlags(&b, hipEventDisableTiming));
            blk_free.push_back(b);
        }
        return GP_OK;
    }
    template <class T>
    gp_status alloc(T*& p, size_t bytes)
    {
        p = nullptr;
        if (bytes == 0) return GP_OK;
        void* q = nullptr;
        GP_HIP(hipMalloc(&q, bytes));
        dev.push_back(q);
        p = (T*)q;
        return GP_OK;
    }
};

// pinned mirrors of the two arrays that are streamed block by block
gp_status ensure_pinned(const gp_plan* plan)
{
    std::lock_guard<std::mutex> lk(plan->mu);
    if (!plan->pinned_col && !plan->col.empty()) {
        void* p = nullptr;
        hipError_t e = hipHostMalloc(&p, plan->col.size() * sizeof(int32_t), hipHostMallocDefault);
        if (e != hipSuccess) return fail(GP_ERR_OOM_HOST, "pinned copy of the column list: %s", hipGetErrorString(e));
        std::memcpy(p, plan->col.data(), plan->col.size() * sizeof(int32_t));
        plan->pinned_col = (int32_t*)p;
    }
    if (!plan->pinned_segs && !plan->segs.empty()) {
        void* p = nullptr;
        hipError_t e = hipHostMalloc(&p, plan->segs.size() * sizeof(Segment), hipHostMallocDefault);
        if (e != hipSuccess) return fail(GP_ERR_OOM_HOST, "pinned copy of the segment list: %s", hipGetErrorString(e));
        std::memcpy(p, plan->segs.data(), plan->segs.size() * sizeof(Segment));
        plan->pinned_segs = (Segment*)p;
    }
    if (plan->rows_final.empty() && plan->num_blocks > 0) {
        // first row that a later block still writes to (through any of its segments,
        // empty rows included): everything below it is final once block p is done
        const int32_t b = plan->num_blocks;
        std::vector<int64_t> first((size_t)b, plan->n);
        for (int32_t q = 0; q < b; ++q)
            for (int64_t s = plan->seg_off[q]; s < plan->seg_off[q + 1]; ++s)
                first[(size_t)q] = std::min<int64_t>(first[(size_t)q], plan->segs[(size_t)s].row);
        plan->rows_final.assign((size_t)b, plan->n);
        plan->split_final.assign((size_t)b, (int64_t)plan->split.size());
        int64_t later = plan->n;
        for (int32_t q = b - 1; q >= 0; --q) {
            plan->rows_final[(size_t)q] = later;
            plan->split_final[(size_t)q] =
                std::lower_bound(plan->split.begin(), plan->split.end(), later,
                                 [](const SplitRow& r, int64_t row) { return (int64_t)r.row < row; }) -
                plan->split.begin();
            later = std::min(later, first[(size_t)q]);
        }
    }
    return GP_OK;
}

}  // namespace

void release_pinned(gp_plan* plan)
{
    if (plan->pinned_col) (void)hipHostFree(plan->pinned_col);
    if (plan->pinned_segs) (void)hipHostFree(plan->pinned_segs);
    plan->pinned_col = nullptr;
    plan->pinned_segs = nullptr;
}

namespace {

// n rows of wc elements between a pinned host matrix and a device slab.  A run that
// is contiguous on both sides is one runtime copy in either direction: with rows
// leaving block by block (ranges of ~100 MB) that measured best (config-5 shape at
// 10 % scale: 0.240 s per call against 0.259 s through the row-copy kernel).  A
// strided run (a column slab of a wider matrix) is moved by the row-copy kernel
// reading / writing the pinned host memory directly, on a small grid: pitched
// runtime copies crawl (4 - 13 GB/s here).  Whatever moves the rows out, a hop
// kernel running beside it lasts as long as the copy does (stores to host memory
// queue up in the same memory pipeline the gathers use), so the call is bound by
// the link's outgoing direction either way.  Grid of the kernel, measured on a
// 2.8 GB slab sent whole with the hops beside it: 8 / 16 / 32 / 64 / 128 / 512
// workgroups gave 370 / 309 / 322 / 355 / 358 / 384 ms per 3-hop call.
constexpr int kLinkCopyBlocks = 16;
constexpr int64_t kMinRowsPerCopy = 4096;  // a finished row range smaller than this waits for the next block
gp_status move_rows(void* dst, int64_t ldd, const void* src, int64_t lds, int64_t n, int32_t wc, gp_dtype dtype,
                    hipMemcpyKind kind, hipStream_t stream)
{
    const int es = dtype == GP_F32 ? 4 : 2;
    if (ldd == wc && lds == wc) {
        GP_HIP(hipMemcpyAsync(dst, src, (size_t)n * wc * es, kind, stream));
        return GP_OK;
    }
    return launch_copy_rows(src, lds, dst, ldd, n, wc, dtype, stream, kLinkCopyBlocks);
}

}  // namespace

gp_status propagate_streamed(const gp_plan* plan, const void* X, int64_t ldx, int32_t d, gp_dtype dtype, gp_agg agg,
                             int32_t K, void* out, int64_t ldo)
{
    const int64_t n = plan->n;
    const int32_t b = plan->num_blocks;
    const int es = dtype == GP_F32 ? 4 : 2;
    const int64_t unit = 16 / es;  // slabs are whole 16-byte vectors wide

    gp_status st = ensure_pinned(plan);
    if (st != GP_OK) return st;

    // ---- HBM budget -> slab width (Eq. 12 with b fixed by the plan) ----------------
    int64_t max_edges = 0, max_segs = 0;
    for (int32_t p = 0; p < b; ++p) {
        max_edges = std::max(max_edges, plan->block_off[p + 1] - plan->block_off[p]);
        max_segs = std::max(max_segs, plan->seg_off[p + 1] - plan->seg_off[p]);
    }
    int64_t budget = options().hbm_budget_bytes;
    if (budget <= 0) {
        size_t free_b = 0, total_b = 0;
        GP_HIP(hipMemGetInfo(&free_b, &total_b));
        budget = (int64_t)(free_b / 10 * 8);
    }
    const int64_t fixed = 2 * (max_edges * 4 + max_segs * (int64_t)sizeof(Segment)) + 2 * n * 4 +
                          (int64_t)plan->split.size() * (int64_t)sizeof(SplitRow) + 4096;
    const int64_t per_col = 2 * n * es + plan->num_slots * 4;
    int64_t w = (budget - fixed) / per_col;
    if (w >= d)
        w = d;
    else
        w = w / unit * unit;
    if (w < std::min<int64_t>(unit, d))
        return fail(GP_ERR_OOM_DEVICE,
                    "HBM budget of %lld bytes cannot hold two edge blocks (%lld bytes) plus two column slabs of %lld columns; "
                    "plan with a smaller block budget or raise the HBM budget",
                    (long long)budget, (long long)fixed, (long long)unit);
    const int64_t wpad = (w + 3) / 4 * 4;  // carry rows stay 16-byte aligned
    // Edge-block buffers: two for double buffering; if the budget has room for all b
    // blocks they are uploaded once and stay (on a 288 GB device only what does not fit
    // has to be streamed again every hop).
    const int64_t block_bytes = max_edges * 4 + max_segs * (int64_t)sizeof(Segment);
    int64_t nbuf = 2;
    if (block_bytes > 0) nbuf = std::min<int64_t>(b, 2 + (budget - fixed - per_col * w) / block_bytes);
    if (nbuf < b) nbuf = std::min<int64_t>(b, 2);
    const bool blocks_stay = nbuf >= b;

    Streams S;
    if ((st = S.init((int)nbuf)) != GP_OK) return st;
    float *d_dinv_sqrt, *d_dinv, *d_carry;
    unsigned long long* d_ctrl;
    SplitRow* d_split;
    char* d_slab[2];
    std::vector<int32_t*> d_col((size_t)nbuf, nullptr);
    std::vector<Segment*> d_segs((size_t)nbuf, nullptr);
    if ((st = S.alloc(d_dinv_sqrt, (size_t)n * 4)) != GP_OK || (st = S.alloc(d_dinv, (size_t)n * 4)) != GP_OK ||
        (st = S.alloc(d_split, plan->split.size() * sizeof(SplitRow))) != GP_OK ||
        (st = S.alloc(d_carry, (size_t)plan->num_slots * wpad * 4)) != GP_OK ||
        (st = S.alloc(d_ctrl, kHopCtrlWords * sizeof(unsigned long long))) != GP_OK ||
        (st = S.alloc(d_slab[0], (size_t)n * w * es)) != GP_OK || (st = S.alloc(d_slab[1], (size_t)n * w * es)) != GP_OK)
        return st;
    for (int64_t i = 0; i < nbuf; ++i)
        if ((st = S.alloc(d_col[i], (size_t)max_edges * 4)) != GP_OK ||
            (st = S.alloc(d_segs[i], (size_t)max_segs * sizeof(Segment))) != GP_OK)
            return st;
    GP_HIP(hipMemsetAsync(d_ctrl, 0, kHopCtrlWords * sizeof(unsigned long long), S.cmp));
    // small vectors: pageable sources, so these two copies are synchronous in effect
    GP_HIP(hipMemcpyAsync(d_dinv_sqrt, plan->dinv_sqrt.data(), (size_t)n * 4, hipMemcpyHostToDevice, S.cmp));
    GP_HIP(hipMemcpyAsync(d_dinv, plan->dinv.data(), (size_t)n * 4, hipMemcpyHostToDevice, S.cmp));
    if (!plan->split.empty())
        GP_HIP(hipMemcpyAsync(d_split, plan->split.data(), plan->split.size() * sizeof(SplitRow), hipMemcpyHostToDevice, S.cmp));
    GP_HIP(hipStreamSynchronize(S.cmp));

    const float* edge_w = agg == GP_AGG_SYM ? d_dinv_sqrt : nullptr;
    const float* row_scale = agg == GP_AGG_SYM ? d_dinv_sqrt : agg == GP_AGG_MEAN ? d_dinv : nullptr;
    const int64_t out_slab = n * ldo * es;  // bytes between two hop slabs in the host stack
    std::vector<char> blk_used((size_t)nbuf, 0);
    bool out_used[2] = {false, false};
    int64_t blk_seq = 0;  // running count of block visits: ring position when blocks do not stay

    // slot 0 = X never needs the device: host threads copy it while the GPU works
    std::vector<std::thread> copiers;
    if ((const void*)X != (const void*)out) {
        const int nthreads = (int64_t)n * d * es < (1 << 22) ? 1 : 4;
        for (int t = 0; t < nthreads; ++t)
            copiers.emplace_back([=] {
                const int64_t r0 = n * t / nthreads, r1 = n * (t + 1) / nthreads;
                if (ldx == d && ldo == d) {
                    std::memcpy((char*)out + r0 * d * es, (const char*)X + r0 * d * es, (size_t)(r1 - r0) * d * es);
                } else {
                    for (int64_t r = r0; r < r1; ++r)
                        std::memcpy((char*)out + r * ldo * es, (const char*)X + r * ldx * es, (size_t)d * es);
                }
            });
    }
    struct Joiner {
        std::vector<std::thread>& v;
        ~Joiner()
        {
            for (auto& t : v)
                if (t.joinable()) t.join();
        }
    } joiner{copiers};

    for (int64_t c0 = 0; c0 < d; c0 += w) {
        const int32_t wc = (int32_t)std::min<int64_t>(w, d - c0);
        // X[:, c0 : c0+wc] -> slab 0 (its previous content must have left first)
        if (out_used[0]) GP_HIP(hipStreamWaitEvent(S.cmp, S.out_done[0], 0));
        if ((st = move_rows(d_slab[0], w, (const char*)X + c0 * es, ldx, n, wc, dtype, hipMemcpyHostToDevice, S.cmp)) != GP_OK)
            return st;
        out_used[0] = false;  // nothing leaves from the slab that holds X

        for (int32_t k = 1; k <= K; ++k) {
            const int src = (k - 1) & 1, dst = k & 1;
            // the slab about to be overwritten may still be on its way to the host
            if (out_used[dst]) GP_HIP(hipStreamWaitEvent(S.cmp, S.out_done[dst], 0));
            int64_t rows_done = 0, split_done = 0;
            for (int32_t p = 0; p < b; ++p, ++blk_seq) {
                const int buf = blocks_stay ? p : (int)(blk_seq % nbuf);
                const int64_t e_lo = plan->block_off[p], e_cnt = plan->block_off[p + 1] - e_lo;
                const int64_t s_lo = plan->seg_off[p], s_cnt = plan->seg_off[p + 1] - s_lo;
                if (!(blocks_stay && blk_used[buf])) {  // a block that stays is sent once
                    if (blk_used[buf]) GP_HIP(hipStreamWaitEvent(S.in, S.blk_free[buf], 0));
                    if (e_cnt)
                        GP_HIP(hipMemcpyAsync(d_col[buf], plan->pinned_col + e_lo, (size_t)e_cnt * 4, hipMemcpyHostToDevice, S.in));
                    if (s_cnt)
                        GP_HIP(hipMemcpyAsync(d_segs[buf], plan->pinned_segs + s_lo, (size_t)s_cnt * sizeof(Segment),
                                              hipMemcpyHostToDevice, S.in));
                    GP_HIP(hipEventRecord(S.blk_ready[buf], S.in));
                }
                GP_HIP(hipStreamWaitEvent(S.cmp, S.blk_ready[buf], 0));
                HopArgs a;
                a.segs = d_segs[buf];
                a.num_segs = s_cnt;
                a.col = d_col[buf];
                a.col_base = e_lo;
                a.edge_w = edge_w;
                a.row_scale = row_scale;
                a.xin = d_slab[src];
                a.ldin = w;
                a.xout = d_slab[dst];
                a.ldout = w;
                a.carry = d_carry;
                a.carry_ld = wpad;
                a.ctrl = d_ctrl;
                a.d = wc;
                a.dtype = dtype;
                a.column_slices = plan->opt.column_slices <= 8 ? plan->opt.column_slices : 0;
                a.persistent_blocks = plan->opt.persistent_blocks;
                a.column_tile = plan->opt.column_tile;
                if ((st = hop_passes(a, S.cmp)) != GP_OK) return st;
                GP_HIP(hipEventRecord(S.blk_free[buf], S.cmp));
                blk_used[buf] = 1;
                // Rows that no later block writes to are final now: complete the cut
                // ones among them and send the range home while the next blocks run.
                const int64_t rows_to = plan->rows_final[(size_t)p], split_to = plan->split_final[(size_t)p];
                if (split_to > split_done) {
                    FixupArgs f;
                    f.split = d_split + split_done;
                    f.num_split = split_to - split_done;
                    f.carry = d_carry;
                    f.carry_ld = wpad;
                    f.row_scale = row_scale;
                    f.xout = d_slab[dst];
                    f.ldout = w;
                    f.d = wc;
                    f.dtype = dtype;
                    f.column_tile = plan->opt.column_tile;
                    if ((st = fixup_passes(f, S.cmp)) != GP_OK) return st;
                    split_done = split_to;
                }
                // (small ranges are held back and leave with the next one)
                if (rows_to > rows_done && (rows_to - rows_done >= kMinRowsPerCopy || p == b - 1)) {
                    GP_HIP(hipEventRecord(S.hop_done, S.cmp));
                    GP_HIP(hipStreamWaitEvent(S.out, S.hop_done, 0));
                    if ((st = move_rows((char*)out + (int64_t)k * out_slab + (rows_done * ldo + c0) * es, ldo,
                                        d_slab[dst] + rows_done * w * es, w, rows_to - rows_done, wc, dtype,
                                        hipMemcpyDeviceToHost, S.out)) != GP_OK)
                        return st;
                    rows_done = rows_to;
                }
            }
            GP_HIP(hipEventRecord(S.out_done[dst], S.out));
            out_used[dst] = true;
        }
    }
    GP_HIP(hipStreamSynchronize(S.in));
    GP_HIP(hipStreamSynchronize(S.cmp));
    GP_HIP(hipStreamSynchronize(S.out));
    for (auto& t : copiers) t.join();
    return GP_OK;
}

}  // namespace gp
