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
#include <condition_variable>
#include <cstring>
#include <deque>
#include <thread>

#include "gp_internal.h"

namespace gp {

namespace {

// The blocks and segments the streamed hops walk: the plan's own, or -- when the HBM
// budget asks for more blocks than the plan has (Eq. 12) -- another balanced cut of the
// same sorted list with its own segments, cut rows and partial-row slots.
struct StreamSchedule {
    bool own = false;
    std::vector<int64_t> own_block_off, own_seg_off;
    std::vector<Segment> own_segs;
    std::vector<SplitRow> own_split;
    int64_t own_slots = 0;
    const std::vector<int64_t>* block_off = nullptr;
    const std::vector<int64_t>* seg_off = nullptr;
    const std::vector<Segment>* segs = nullptr;
    const std::vector<SplitRow>* split = nullptr;
    int64_t num_slots = 0;
    int32_t b = 0;
    int64_t max_edges = 0, max_segs = 0;
    // after block p every row below rows_final[p] is complete, and split rows
    // [0, split_final[p]) are the cut rows among them
    std::vector<int64_t> rows_final, split_final;
    Segment* pinned_segs = nullptr;

    void use_plan(const gp_plan* plan)
    {
        own = false;
        block_off = &plan->block_off;
        seg_off = &plan->seg_off;
        segs = &plan->segs;
        split = &plan->split;
        num_slots = plan->num_slots;
        finish();
    }
    gp_status recut(const gp_plan* plan, int64_t blocks)
    {
        own = true;
        own_block_off.resize((size_t)blocks + 1);
        const int64_t q = plan->nnz / blocks, r = plan->nnz % blocks;  // the planner's balanced cut, other count
        for (int64_t p = 0; p <= blocks; ++p) own_block_off[(size_t)p] = p * q + std::min(p, r);
        gp_status st = cut_schedule(*plan, own_block_off, own_segs, own_seg_off, own_split, own_slots);
        if (st != GP_OK) return st;
        block_off = &own_block_off;
        seg_off = &own_seg_off;
        segs = &own_segs;
        split = &own_split;
        num_slots = own_slots;
        finish();
        return GP_OK;
    }
    void finish()
    {
        b = (int32_t)block_off->size() - 1;
        max_edges = max_segs = 0;
        for (int32_t p = 0; p < b; ++p) {
            max_edges = std::max(max_edges, (*block_off)[(size_t)p + 1] - (*block_off)[(size_t)p]);
            max_segs = std::max(max_segs, (*seg_off)[(size_t)p + 1] - (*seg_off)[(size_t)p]);
        }
    }
    // first row that a later block still writes to (through any of its segments, empty
    // rows included): everything below it is final once block p is done
    void final_rows(int64_t n)
    {
        std::vector<int64_t> first((size_t)b, n);
        for (int32_t q = 0; q < b; ++q)
            for (int64_t s = (*seg_off)[(size_t)q]; s < (*seg_off)[(size_t)q + 1]; ++s)
                first[(size_t)q] = std::min<int64_t>(first[(size_t)q], (*segs)[(size_t)s].row);
        rows_final.assign((size_t)b, n);
        split_final.assign((size_t)b, (int64_t)split->size());
        int64_t later = n;
        for (int32_t q = b - 1; q >= 0; --q) {
            rows_final[(size_t)q] = later;
            split_final[(size_t)q] = std::lower_bound(split->begin(), split->end(), later,
                                                       [](const SplitRow& r, int64_t row) { return (int64_t)r.row < row; }) -
                                      split->begin();
            later = std::min(later, first[(size_t)q]);
        }
    }
};

// a large host-to-host copy on several threads (one thread moves 3 - 5 GB/s, the memory system several times that;
// the pinned mirrors of a plan's lists, made on its first streamed call, take 1.22 s on 8 threads and 1.00 s on 16
// at a quarter of config 5; the steady state is bound by the link either way)
void copy_on_threads(void* dst, const void* src, size_t n)
{
    const int nt = n < ((size_t)4 << 20) ? 1 : host_threads();
    parallel_run(nt, [&](int t, int k) {
        const size_t lo = n * (size_t)t / (size_t)k, hi = n * (size_t)(t + 1) / (size_t)k;
        std::memcpy((char*)dst + lo, (const char*)src + lo, hi - lo);
    });
}

// Ordinary (pageable) host memory cannot be the end of an asynchronous copy, and left to
// the runtime its copies are staged one after the other with the enqueuing thread waiting.
// The stager moves such operands through a ring of pinned buffers instead: on the way in,
// host threads fill one buffer while the one before it is on the link; on the way out, a
// drain thread waits for each buffer's copy to land and host threads empty it into the
// caller's memory while the next buffers are on the link.  One stager per plan, kept
// between calls.
class Stager {
public:
    static constexpr int kInSlots = 2, kOutSlots = 6;
    static constexpr size_t kSlotBytes = (size_t)64 << 20;

    ~Stager()
    {
        stop();
        for (int i = 0; i < kInSlots + kOutSlots; ++i) {
            if (ev_[i]) (void)hipEventDestroy(ev_[i]);
            if (buf_[i]) (void)hipHostFree(buf_[i]);
        }
    }
    gp_status init(int device)
    {
        device_ = device;
        for (int i = 0; i < kInSlots + kOutSlots; ++i) {
            hipError_t e = hipHostMalloc(&buf_[i], kSlotBytes, hipHostMallocDefault);
            if (e != hipSuccess) return fail(GP_ERR_OOM_HOST, "pinned staging buffers: %s", hipGetErrorString(e));
            GP_HIP(hipEventCreateWithFlags(&ev_[i], hipEventDisableTiming));
        }
        worker_ = std::thread([this] { drain(); });
        return GP_OK;
    }
    // host (pageable) -> device, in order on `stream`; returns when the last piece is enqueued
    gp_status upload(void* dst, const void* src, size_t bytes, hipStream_t stream)
    {
        for (size_t off = 0, i = 0; off < bytes; off += kSlotBytes, ++i) {
            const int s = (int)(i % kInSlots);
            const size_t n = std::min(kSlotBytes, bytes - off);
            if (in_used_[s]) GP_HIP(hipEventSynchronize(ev_[s]));  // its last piece has left the buffer
            copy_parallel(buf_[s], (const char*)src + off, n);
            GP_HIP(hipMemcpyAsync((char*)dst + off, buf_[s], n, hipMemcpyHostToDevice, stream));
            GP_HIP(hipEventRecord(ev_[s], stream));
            in_used_[s] = true;
        }
        return GP_OK;
    }
    // device -> host (pageable), in order on `stream`; the drain thread finishes the job
    gp_status download(void* dst, const void* src, size_t bytes, hipStream_t stream)
    {
        for (size_t off = 0; off < bytes; off += kSlotBytes) {
            const size_t n = std::min(kSlotBytes, bytes - off);
            int s = -1;
            {
                std::unique_lock<std::mutex> lk(mu_);
                cv_.wait(lk, [&] { return failed_ || !free_.empty(); });
                if (failed_) return fail(GP_ERR_DEVICE, "staging thread: %s", error_.c_str());
                s = free_.front();
                free_.pop_front();
            }
            hipError_t e = hipMemcpyAsync(buf_[s], (const char*)src + off, n, hipMemcpyDeviceToHost, stream);
            if (e == hipSuccess) e = hipEventRecord(ev_[s], stream);
            if (e != hipSuccess) {
                std::lock_guard<std::mutex> lk(mu_);
                free_.push_back(s);
                return fail(GP_ERR_DEVICE, "staged copy to the host: %s", hipGetErrorString(e));
            }
            std::lock_guard<std::mutex> lk(mu_);
            jobs_.push_back(Job{s, (char*)dst + off, n});
            cv_.notify_all();
        }
        return GP_OK;
    }
    // waits until every download has reached the caller's memory
    gp_status finish()
    {
        std::unique_lock<std::mutex> lk(mu_);
        cv_.wait(lk, [&] { return failed_ || (jobs_.empty() && !busy_); });
        for (bool& u : in_used_) u = false;
        if (failed_) {
            const gp_status st = fail(GP_ERR_DEVICE, "staging thread: %s", error_.c_str());
            failed_ = false;  // the next call starts clean (its streams are synchronised by then)
            jobs_.clear();
            free_.clear();
            for (int i = kInSlots; i < kInSlots + kOutSlots; ++i) free_.push_back(i);
            return st;
        }
        return GP_OK;
    }

private:
    struct Job {
        int slot;
        char* dst;
        size_t bytes;
    };
    static void copy_parallel(void* dst, const void* src, size_t n) { copy_on_threads(dst, src, n); }
    void drain()
    {
        (void)hipSetDevice(device_);
        {
            std::lock_guard<std::mutex> lk(mu_);
            for (int i = kInSlots; i < kInSlots + kOutSlots; ++i) free_.push_back(i);
            cv_.notify_all();
        }
        for (;;) {
            Job j;
            {
                std::unique_lock<std::mutex> lk(mu_);
                cv_.wait(lk, [&] { return quit_ || !jobs_.empty(); });
                if (jobs_.empty()) return;  // quit_ and nothing left
                j = jobs_.front();
                jobs_.pop_front();
                busy_ = true;
            }
            hipError_t e = hipEventSynchronize(ev_[j.slot]);
            if (e == hipSuccess) {
                try {
                    copy_parallel(j.dst, buf_[j.slot], j.bytes);
                } catch (const std::exception& ex) {
                    std::lock_guard<std::mutex> lk(mu_);
                    failed_ = true;
                    error_ = ex.what();
                }
            }
            std::lock_guard<std::mutex> lk(mu_);
            if (e != hipSuccess) {
                failed_ = true;
                error_ = hipGetErrorString(e);
            }
            free_.push_back(j.slot);
            busy_ = false;
            cv_.notify_all();
        }
    }
    void stop()
    {
        {
            std::lock_guard<std::mutex> lk(mu_);
            quit_ = true;
            cv_.notify_all();
        }
        if (worker_.joinable()) worker_.join();
    }

    int device_ = 0;
    void* buf_[kInSlots + kOutSlots] = {};
    hipEvent_t ev_[kInSlots + kOutSlots] = {};
    bool in_used_[kInSlots] = {};
    std::mutex mu_;
    std::condition_variable cv_;
    std::deque<int> free_;
    std::deque<Job> jobs_;
    bool busy_ = false, quit_ = false, failed_ = false;
    std::string error_;
    std::thread worker_;
};

// Everything a streamed call needs besides the caller's operands, kept with the plan
// from one call to the next: the schedule, three streams and their events, and the
// device buffers (norm vectors, cut rows, partial rows, cursors, two column slabs, the
// edge-block buffers).  A call whose shape differs (slab width, block count, buffer
// count, element size, device) builds it anew.
struct StreamedState {
    int device = -1;
    int es = 0;
    int64_t w = 0, wpad = 0, nbuf = 0;
    bool blocks_stay = false, blocks_loaded = false;
    int64_t used_b = 0, used_c = 0;  // what the last call ran with (gp_plan_streamed_shape)
    StreamSchedule sched;

    hipStream_t in = nullptr, cmp = nullptr, out = nullptr;
    std::vector<hipEvent_t> blk_ready, blk_free;  // one pair per edge-block buffer
    hipEvent_t hop_done = nullptr, out_done[2] = {nullptr, nullptr};
    std::vector<void*> dev;
    size_t dev_bytes = 0;  // sum of the device allocations below
    float *d_dinv_sqrt = nullptr, *d_dinv = nullptr, *d_carry = nullptr;
    unsigned long long* d_ctrl = nullptr;
    SplitRow* d_split = nullptr;
    char* d_slab[2] = {nullptr, nullptr};
    std::vector<int32_t*> d_col;
    std::vector<Segment*> d_segs;
    Stager* stager = nullptr;  // made by the first call with operands in pageable memory

    ~StreamedState()
    {
        int cur = -1;
        const bool switched = device >= 0 && hipGetDevice(&cur) == hipSuccess && cur != device && hipSetDevice(device) == hipSuccess;
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
        if (sched.pinned_segs) (void)hipHostFree(sched.pinned_segs);
        delete stager;
        if (switched) (void)hipSetDevice(cur);
    }
    gp_status init_streams(int block_buffers)
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
        dev_bytes += bytes;
        p = (T*)q;
        return GP_OK;
    }
};

// pinned mirror of the column list (streamed block by block whatever the cut)
gp_status ensure_pinned_col(const gp_plan* plan)
{
    if (!plan->pinned_col && !plan->col.empty()) {
        void* p = nullptr;
        hipError_t e = hipHostMalloc(&p, plan->col.size() * sizeof(int32_t), hipHostMallocDefault);
        if (e != hipSuccess) return fail(GP_ERR_OOM_HOST, "pinned copy of the column list: %s", hipGetErrorString(e));
        copy_on_threads(p, plan->col.data(), plan->col.size() * sizeof(int32_t));
        plan->pinned_col = (int32_t*)p;
    }
    return GP_OK;
}

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
                    hipMemcpyKind kind, hipStream_t stream, Stager* stager = nullptr)
{
    const int es = dtype == GP_F32 ? 4 : 2;
    if (stager) {  // the host side is pageable memory (contiguous runs only: the caller has checked)
        const size_t bytes = (size_t)n * wc * es;
        return kind == hipMemcpyHostToDevice ? stager->upload(dst, src, bytes, stream) : stager->download(dst, src, bytes, stream);
    }
    if (ldd == wc && lds == wc) {
        GP_HIP(hipMemcpyAsync(dst, src, (size_t)n * wc * es, kind, stream));
        return GP_OK;
    }
    return launch_copy_rows(src, lds, dst, ldd, n, wc, dtype, stream, kLinkCopyBlocks);
}

// HBM bytes of the streamed schedule in the terms of Eq. 12: the edge structure B_S
// (column ids and segment records) is held in two block buffers at a time (beta_S = 2,
// B_S / b each), the feature side B_X (two column slabs and the partial rows, per feature
// column) in slabs of d / c columns (beta_X = 1), and what is neither (two norm vectors,
// the list of cut rows) comes off the budget first.
struct Volumes {
    double B_S, B_X, B_GPU;
    int64_t fixed, per_col;
};
Volumes volumes(int64_t n, int64_t nnz, int64_t nsegs, int64_t slots, int32_t d, int es, int64_t budget)
{
    Volumes v;
    v.fixed = 2 * n * 4 + 16 * slots + 4096;  // a cut row owns at least two slots: 16 B per slot bounds the list
    v.per_col = 2 * n * es + slots * 4;
    v.B_S = 4.0 * (double)nnz + (double)sizeof(Segment) * (double)nsegs;
    v.B_X = (double)v.per_col * (double)d;
    v.B_GPU = (double)(budget - v.fixed);
    return v;
}

}  // namespace

void release_pinned(gp_plan* plan)
{
    delete (StreamedState*)plan->streamed;
    plan->streamed = nullptr;
    if (plan->pinned_col) (void)hipHostFree(plan->pinned_col);
    plan->pinned_col = nullptr;
}

gp_status propagate_streamed(const gp_plan* plan, const void* X, int64_t ldx, int32_t d, gp_dtype dtype, gp_agg agg,
                             int32_t K, void* out, int64_t ldo, bool pageable)
{
    const int64_t n = plan->n;
    const int es = dtype == GP_F32 ? 4 : 2;
    const int64_t unit = 16 / es;  // slabs are whole 16-byte vectors wide
    std::lock_guard<std::mutex> lk(plan->mu);  // one streamed call per plan at a time

    gp_status st = ensure_pinned_col(plan);
    if (st != GP_OK) return st;
    int cur = -1;
    GP_HIP(hipGetDevice(&cur));

    // ---- HBM budget -> block count b and column-block count c (Eq. 12) ----------------
    int64_t budget = options().hbm_budget_bytes;
    if (budget <= 0) {
        size_t free_b = 0, total_b = 0;
        GP_HIP(hipMemGetInfo(&free_b, &total_b));
        // what an earlier call on this plan left on the device counts as free: it is reused or released
        const StreamedState* kept = (const StreamedState*)plan->streamed;
        budget = (int64_t)((free_b + (kept ? kept->dev_bytes : 0)) / 10 * 8);
    }
    const Volumes v = volumes(n, plan->nnz, (int64_t)plan->segs.size(), plan->num_slots, d, es, budget);
    const int64_t max_c = (d + unit - 1) / unit;
    int64_t b_star = 0, c_star = 0;
    if (v.B_GPU <= 0 || gp_solve_aggregation_blocks(v.B_S, v.B_X, v.B_GPU, 2.0, 1.0, max_c, &b_star, &c_star) != GP_OK)
        return fail(GP_ERR_OOM_DEVICE,
                    "HBM budget of %lld bytes cannot hold two edge blocks plus two column slabs of %lld columns at any "
                    "block count; raise the HBM budget",
                    (long long)budget, (long long)unit);

    StreamedState* S = (StreamedState*)plan->streamed;
    // the plan's own blocks serve whenever they are at least as many as the budget asks for
    const bool want_own = b_star > plan->num_blocks;
    const int64_t want_b = want_own ? b_star : plan->num_blocks;
    if (S && (S->device != cur || S->es != es || S->sched.b != want_b || S->sched.own != want_own)) {
        delete S;
        S = nullptr;
        plan->streamed = nullptr;
    }
    StreamSchedule fresh;
    StreamSchedule* sched = S ? &S->sched : &fresh;
    int64_t w = 0, wpad = 0, nbuf = 0;
    for (int attempt = 0;; ++attempt) {
        if (!S) {
            if (want_own) {
                if ((st = fresh.recut(plan, b_star + attempt)) != GP_OK) return st;
            } else {
                fresh.use_plan(plan);
            }
        }
        // slab width: with the plan's blocks the widest that fits beside two of them; with a cut of
        // its own the width Eq. 12's minimiser chose
        const int64_t block_bytes = sched->max_edges * 4 + sched->max_segs * (int64_t)sizeof(Segment);
        const int64_t fixed = 2 * n * 4 + (int64_t)sched->split->size() * (int64_t)sizeof(SplitRow) + 4096;
        const int64_t per_col = 2 * n * es + sched->num_slots * 4;
        w = (budget - fixed - 2 * block_bytes) / per_col;
        if (sched->own) w = std::min<int64_t>(w, ((d + c_star - 1) / c_star + unit - 1) / unit * unit);
        w = w >= d ? d : w / unit * unit;
        if (w >= std::min<int64_t>(unit, d)) {
            wpad = (w + 3) / 4 * 4;  // carry rows stay 16-byte aligned
            // Edge-block buffers: two for double buffering; if the budget has room for all b
            // blocks they are uploaded once and stay (on a 288 GB device only what does not fit
            // has to be streamed again every hop).
            nbuf = 2;
            if (block_bytes > 0) nbuf = std::min<int64_t>(sched->b, (budget - fixed - per_col * w) / block_bytes);
            if (nbuf < sched->b) nbuf = std::min<int64_t>(sched->b, 2);
            break;
        }
        // the cut's own segments and cut rows came out a little larger than the estimate
        if (S || !want_own || attempt >= 8)
            return fail(GP_ERR_OOM_DEVICE,
                        "HBM budget of %lld bytes cannot hold two edge blocks (%lld bytes each) plus two column slabs of "
                        "%lld columns; raise the HBM budget",
                        (long long)budget, (long long)block_bytes, (long long)unit);
    }
    if (S && (S->w != w || S->nbuf != nbuf)) {
        // same schedule, other buffer shape: keep the schedule, rebuild the rest
        fresh = std::move(S->sched);
        S->sched.pinned_segs = nullptr;
        delete S;
        S = nullptr;
        plan->streamed = nullptr;
        fresh.block_off = fresh.own ? &fresh.own_block_off : &plan->block_off;
        fresh.seg_off = fresh.own ? &fresh.own_seg_off : &plan->seg_off;
        fresh.segs = fresh.own ? &fresh.own_segs : &plan->segs;
        fresh.split = fresh.own ? &fresh.own_split : &plan->split;
    }
    if (!S) {
        S = new StreamedState();
        plan->streamed = S;
        S->device = cur;
        S->es = es;
        S->w = w;
        S->wpad = wpad;
        S->nbuf = nbuf;
        S->sched = std::move(fresh);
        StreamSchedule& C = S->sched;
        C.block_off = C.own ? &C.own_block_off : &plan->block_off;
        C.seg_off = C.own ? &C.own_seg_off : &plan->seg_off;
        C.segs = C.own ? &C.own_segs : &plan->segs;
        C.split = C.own ? &C.own_split : &plan->split;
        if (C.rows_final.empty()) C.final_rows(n);
        auto fail_clean = [&](gp_status e) {
            delete S;
            plan->streamed = nullptr;
            return e;
        };
        if (!C.pinned_segs && !C.segs->empty()) {
            void* p = nullptr;
            hipError_t e = hipHostMalloc(&p, C.segs->size() * sizeof(Segment), hipHostMallocDefault);
            if (e != hipSuccess) return fail_clean(fail(GP_ERR_OOM_HOST, "pinned copy of the segment list: %s", hipGetErrorString(e)));
            copy_on_threads(p, C.segs->data(), C.segs->size() * sizeof(Segment));
            C.pinned_segs = (Segment*)p;
        }
        if ((st = S->init_streams((int)nbuf)) != GP_OK) return fail_clean(st);
        S->d_col.assign((size_t)nbuf, nullptr);
        S->d_segs.assign((size_t)nbuf, nullptr);
        if ((st = S->alloc(S->d_dinv_sqrt, (size_t)n * 4)) != GP_OK || (st = S->alloc(S->d_dinv, (size_t)n * 4)) != GP_OK ||
            (st = S->alloc(S->d_split, C.split->size() * sizeof(SplitRow))) != GP_OK ||
            (st = S->alloc(S->d_carry, (size_t)C.num_slots * wpad * 4)) != GP_OK ||
            (st = S->alloc(S->d_ctrl, kHopCtrlWords * sizeof(unsigned long long))) != GP_OK ||
            (st = S->alloc(S->d_slab[0], (size_t)n * w * es)) != GP_OK || (st = S->alloc(S->d_slab[1], (size_t)n * w * es)) != GP_OK)
            return fail_clean(st);
        for (int64_t i = 0; i < nbuf; ++i)
            if ((st = S->alloc(S->d_col[(size_t)i], (size_t)C.max_edges * 4)) != GP_OK ||
                (st = S->alloc(S->d_segs[(size_t)i], (size_t)C.max_segs * sizeof(Segment))) != GP_OK)
                return fail_clean(st);
        hipError_t e = hipMemsetAsync(S->d_ctrl, 0, kHopCtrlWords * sizeof(unsigned long long), S->cmp);
        // small vectors: pageable sources, so these copies are synchronous in effect
        if (e == hipSuccess) e = hipMemcpyAsync(S->d_dinv_sqrt, plan->dinv_sqrt.data(), (size_t)n * 4, hipMemcpyHostToDevice, S->cmp);
        if (e == hipSuccess) e = hipMemcpyAsync(S->d_dinv, plan->dinv.data(), (size_t)n * 4, hipMemcpyHostToDevice, S->cmp);
        if (e == hipSuccess && !C.split->empty())
            e = hipMemcpyAsync(S->d_split, C.split->data(), C.split->size() * sizeof(SplitRow), hipMemcpyHostToDevice, S->cmp);
        if (e == hipSuccess) e = hipStreamSynchronize(S->cmp);
        if (e != hipSuccess) return fail_clean(fail(GP_ERR_DEVICE, "setting up the streamed schedule: %s", hipGetErrorString(e)));
        S->blocks_stay = nbuf >= C.b;
        S->blocks_loaded = false;
    }
    // Ordinary host memory cannot be read or written by a kernel; it goes through the plan's
    // pinned staging ring.  Accepted where every transfer is one contiguous run, i.e. whole
    // rows of operands without row padding.
    if (pageable && (w < d || ldx != d || ldo != d))
        return fail(GP_ERR_UNSUPPORTED,
                    "operands in pageable host memory need contiguous rows (ldx = ldo = d) and an HBM budget that holds "
                    "whole rows (slab width %lld of %d columns); use pinned host memory",
                    (long long)w, d);
    if (pageable && !S->stager) {
        S->stager = new Stager();
        if ((st = S->stager->init(cur)) != GP_OK) {
            delete S->stager;
            S->stager = nullptr;
            return st;
        }
    }
    Stager* const stager = pageable ? S->stager : nullptr;
    const StreamSchedule& C = S->sched;
    const int32_t b = C.b;
    const bool blocks_stay = S->blocks_stay;
    S->used_b = b;
    S->used_c = (d + w - 1) / w;
    float* const d_carry = S->d_carry;
    char* const* d_slab = S->d_slab;

    const float* edge_w = agg == GP_AGG_SYM ? S->d_dinv_sqrt : nullptr;
    const float* row_scale = agg == GP_AGG_SYM ? S->d_dinv_sqrt : agg == GP_AGG_MEAN ? S->d_dinv : nullptr;
    const int64_t out_slab = n * ldo * es;  // bytes between two hop slabs in the host stack
    // a block that stays is sent once per plan, not once per call
    std::vector<char> blk_used((size_t)nbuf, (blocks_stay && S->blocks_loaded) ? 1 : 0);
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
        StreamedState* S;
        Stager* stager;
        ~Joiner()
        {
            // whatever way the call ends, nothing of it is still running afterwards
            (void)hipStreamSynchronize(S->in);
            (void)hipStreamSynchronize(S->cmp);
            (void)hipStreamSynchronize(S->out);
            if (stager) (void)stager->finish();
            for (auto& t : v)
                if (t.joinable()) t.join();
        }
    } joiner{copiers, S, stager};

    for (int64_t c0 = 0; c0 < d; c0 += w) {
        const int32_t wc = (int32_t)std::min<int64_t>(w, d - c0);
        // X[:, c0 : c0+wc] -> slab 0 (its previous content must have left first)
        if (out_used[0]) GP_HIP(hipStreamWaitEvent(S->cmp, S->out_done[0], 0));
        if ((st = move_rows(d_slab[0], w, (const char*)X + c0 * es, ldx, n, wc, dtype, hipMemcpyHostToDevice, S->cmp, stager)) !=
            GP_OK)
            return st;
        out_used[0] = false;  // nothing leaves from the slab that holds X

        for (int32_t k = 1; k <= K; ++k) {
            const int src = (k - 1) & 1, dst = k & 1;
            // the slab about to be overwritten may still be on its way to the host
            if (out_used[dst]) GP_HIP(hipStreamWaitEvent(S->cmp, S->out_done[dst], 0));
            int64_t rows_done = 0, split_done = 0;
            for (int32_t p = 0; p < b; ++p, ++blk_seq) {
                const int buf = blocks_stay ? p : (int)(blk_seq % nbuf);
                const int64_t e_lo = (*C.block_off)[(size_t)p], e_cnt = (*C.block_off)[(size_t)p + 1] - e_lo;
                const int64_t s_lo = (*C.seg_off)[(size_t)p], s_cnt = (*C.seg_off)[(size_t)p + 1] - s_lo;
                if (!(blocks_stay && blk_used[(size_t)buf])) {  // a block that stays is sent once
                    if (blk_used[(size_t)buf]) GP_HIP(hipStreamWaitEvent(S->in, S->blk_free[(size_t)buf], 0));
                    if (e_cnt)
                        GP_HIP(hipMemcpyAsync(S->d_col[(size_t)buf], plan->pinned_col + e_lo, (size_t)e_cnt * 4, hipMemcpyHostToDevice,
                                              S->in));
                    if (s_cnt)
                        GP_HIP(hipMemcpyAsync(S->d_segs[(size_t)buf], C.pinned_segs + s_lo, (size_t)s_cnt * sizeof(Segment),
                                              hipMemcpyHostToDevice, S->in));
                    GP_HIP(hipEventRecord(S->blk_ready[(size_t)buf], S->in));
                    GP_HIP(hipStreamWaitEvent(S->cmp, S->blk_ready[(size_t)buf], 0));
                }
                HopArgs a;
                a.segs = S->d_segs[(size_t)buf];
                a.num_segs = s_cnt;
                a.col = S->d_col[(size_t)buf];
                a.col_base = e_lo;
                a.edge_w = edge_w;
                a.row_scale = row_scale;
                a.xin = d_slab[src];
                a.ldin = w;
                a.xout = d_slab[dst];
                a.ldout = w;
                a.carry = d_carry;
                a.carry_ld = wpad;
                a.ctrl = S->d_ctrl;
                a.d = wc;
                a.dtype = dtype;
                a.column_slices = plan->opt.column_slices <= 8 ? plan->opt.column_slices : 0;
                a.persistent_blocks = plan->opt.persistent_blocks;
                a.column_tile = plan->opt.column_tile;
                if ((st = hop_passes(a, S->cmp)) != GP_OK) return st;
                GP_HIP(hipEventRecord(S->blk_free[(size_t)buf], S->cmp));
                blk_used[(size_t)buf] = 1;
                // Rows that no later block writes to are final now: complete the cut
                // ones among them and send the range home while the next blocks run.
                const int64_t rows_to = C.rows_final[(size_t)p], split_to = C.split_final[(size_t)p];
                if (split_to > split_done) {
                    FixupArgs f;
                    f.split = S->d_split + split_done;
                    f.num_split = split_to - split_done;
                    f.carry = d_carry;
                    f.carry_ld = wpad;
                    f.row_scale = row_scale;
                    f.xout = d_slab[dst];
                    f.ldout = w;
                    f.d = wc;
                    f.dtype = dtype;
                    f.column_tile = plan->opt.column_tile;
                    if ((st = fixup_passes(f, S->cmp)) != GP_OK) return st;
                    split_done = split_to;
                }
                // (small ranges are held back and leave with the next one)
                if (rows_to > rows_done && (rows_to - rows_done >= kMinRowsPerCopy || p == b - 1)) {
                    GP_HIP(hipEventRecord(S->hop_done, S->cmp));
                    GP_HIP(hipStreamWaitEvent(S->out, S->hop_done, 0));
                    if ((st = move_rows((char*)out + (int64_t)k * out_slab + (rows_done * ldo + c0) * es, ldo,
                                        d_slab[dst] + rows_done * w * es, w, rows_to - rows_done, wc, dtype,
                                        hipMemcpyDeviceToHost, S->out, stager)) != GP_OK)
                        return st;
                    rows_done = rows_to;
                }
            }
            if (blocks_stay) S->blocks_loaded = true;
            GP_HIP(hipEventRecord(S->out_done[dst], S->out));
            out_used[dst] = true;
        }
    }
    GP_HIP(hipStreamSynchronize(S->in));
    GP_HIP(hipStreamSynchronize(S->cmp));
    GP_HIP(hipStreamSynchronize(S->out));
    return stager ? stager->finish() : GP_OK;
}

}  // namespace gp

using namespace gp;

extern "C" gp_status gp_plan_streamed_shape(const gp_plan* plan, int64_t* edge_blocks, int64_t* column_blocks)
{
    if (!plan || !edge_blocks || !column_blocks) return fail(GP_ERR_INVALID_ARG, "NULL argument");
    std::lock_guard<std::mutex> lk(plan->mu);
    const StreamedState* S = (const StreamedState*)plan->streamed;
    *edge_blocks = S ? S->used_b : 0;
    *column_blocks = S ? S->used_c : 0;
    return GP_OK;
}
