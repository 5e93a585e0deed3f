// gp_propagate: the hop loop of Algorithm 1 (k = 1..K, every edge block, then
// the rows cut between blocks) for operands that live in HBM, and plan upload.
#include <algorithm>
#include <exception>
#include <functional>

#include "gp_internal.h"

namespace gp {

namespace {

template <class T>
gp_status upload(T*& dptr, const std::vector<T>& h, hipStream_t stream)
{
    if (dptr || h.empty()) return GP_OK;  // already there (the device planner leaves its results), or nothing to send
    GP_HIP(hipMalloc((void**)&dptr, h.size() * sizeof(T)));
    GP_HIP(hipMemcpyAsync(dptr, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice, stream));
    return GP_OK;
}

void release(DevicePlan& D)
{
    (void)hipFree(D.col);
    (void)hipFree(D.dinv_sqrt);
    (void)hipFree(D.dinv);
    (void)hipFree(D.segs);
    (void)hipFree(D.split);
    (void)hipFree(D.carry);
    (void)hipFree(D.edge_ws);
    (void)hipFree(D.ctrl);
    (void)hipFree(D.ping[0]);
    (void)hipFree(D.ping[1]);
    (void)hipFree(D.comb);
    for (XcdWork& w : D.work) (void)hipFree(w.recs);
    for (void* p : D.retired) (void)hipFree(p);
    (void)hipFree(D.split_col);
    (void)hipFree(D.split_edge_ws);
    (void)hipFree(D.split_cold);
    (void)hipFree(D.split_rows);
    for (void* q : {(void*)D.lds_members, (void*)D.lds_member_off, (void*)D.lds_group_off, (void*)D.lds_groups, (void*)D.lds_octets,
                    (void*)D.lds_ids, (void*)D.lds_list_of_set, (void*)D.lds_col, (void*)D.lds_cold, (void*)D.lds_planes,
                    (void*)D.lds_wave_cut, (void*)D.lds_packed})
        (void)hipFree(q);
    (void)hipFree(D.split_carry);
    D = DevicePlan();
}

// Uploads the plan once per plan (to the device that is current at that time)
// and (re)sizes the partial-row buffer for d columns.
gp_status ensure_device(const gp_plan* plan, int32_t d, bool want_edge_weights, hipStream_t stream)
{
    std::lock_guard<std::mutex> lk(plan->mu);
    DevicePlan& D = plan->dev;
    int cur = -1;
    GP_HIP(hipGetDevice(&cur));
    if (D.device >= 0 && D.device != cur)
        return fail(GP_ERR_INVALID_ARG, "plan lives on device %d but device %d is current", D.device, cur);
    if (D.device < 0 || !D.ctrl) {
        gp_status st;
        if ((st = upload(D.col, plan->col, stream)) != GP_OK || (st = upload(D.dinv_sqrt, plan->dinv_sqrt, stream)) != GP_OK ||
            (st = upload(D.dinv, plan->dinv, stream)) != GP_OK || (st = upload(D.segs, plan->segs, stream)) != GP_OK ||
            (st = upload(D.split, plan->split, stream)) != GP_OK) {
            release(D);
            return st;
        }
        if (hipMalloc((void**)&D.ctrl, kHopCtrlWords * sizeof(unsigned long long)) != hipSuccess ||
            hipMemsetAsync(D.ctrl, 0, kHopCtrlWords * sizeof(unsigned long long), stream) != hipSuccess) {
            release(D);
            return fail(GP_ERR_OOM_DEVICE, "cursor buffer of the hop kernel");
        }
        // pageable sources: the copies above are staged, but finish them before returning
        // so the host vectors may be touched freely afterwards
        GP_HIP(hipStreamSynchronize(stream));
        D.device = cur;
    }
    if (want_edge_weights && !D.edge_ws && plan->nnz > 0) {
        // one coalesced fp32 per non-zero instead of one random 4-byte gather per non-zero and hop
        GP_HIP(hipMalloc((void**)&D.edge_ws, (size_t)plan->nnz * sizeof(float)));
        gp_status st = launch_fill_edge_weights(D.col, D.dinv_sqrt, D.edge_ws, plan->nnz, stream);
        if (st != GP_OK) return st;
        GP_HIP(hipStreamSynchronize(stream));  // once per plan: later calls may come on other streams
    }
    const int64_t need_ld = ((int64_t)d + 3) / 4 * 4;
    if (plan->num_slots > 0 && need_ld > D.carry_ld) {
        // work enqueued earlier may still be using the old buffer: it is kept until the plan goes
        if (D.carry) D.retired.push_back(D.carry);
        D.carry = nullptr;
        D.carry_ld = 0;
        GP_HIP(hipMalloc((void**)&D.carry, (size_t)plan->num_slots * need_ld * sizeof(float)));
        D.carry_ld = need_ld;
    }
    return GP_OK;
}

// width of one kernel pass over the columns: everything at once unless the row is
// wider than the kernels hold; a pass is a multiple of 16 bytes so every pass keeps
// the alignment of the first
int64_t pass_width(int64_t tile, gp_dtype dtype, int32_t d, int64_t lda, int64_t ldb, const void* pa, const void* pb)
{
    const int es = dtype == GP_F32 ? 4 : 2;
    const int64_t unit = 16 / es;
    const int64_t cap = max_columns_per_pass(vector_width(dtype, d, lda, ldb, pa, pb));
    if (tile <= 0 || tile > cap) tile = d <= cap ? d : cap;
    if (tile < d) tile = std::max<int64_t>(unit, tile / unit * unit);
    return tile;
}

// Decides whether this plan's hops run from explicit per-XCD work lists and with which
// slice shape.  The lists pay when the rows of a cluster draw most of their sources
// from the cluster itself and one slice of a cluster's rows fits the share of an XCD's
// L2 that the streams beside it (column ids, written rows, sources outside the cluster)
// leave free.  A slice is at least 128 bytes (one cache line) wide.
constexpr double kL2Share = 0.75;
constexpr int64_t kLineBytes = 128;

int64_t l2_bytes_per_xcd()
{
    static const int64_t v = [] {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return (int64_t)4 << 20;
        const int64_t l2 = prop.l2CacheSize;
        return (l2 >= (1 << 20) && l2 <= (64 << 20)) ? l2 : (int64_t)4 << 20;
    }();
    return v;
}

}  // namespace

bool choose_cache_schedule(const gp_plan* plan, int32_t d, int es, int vec, int& num_slices, int& slice_elems)
{
    if (plan->opt.cache_schedule == 2 || plan->segs.empty()) return false;
    const bool forced = plan->opt.cache_schedule == 1;
    if (!plan->clusters.ready) cluster_rows(*plan, plan->clusters);
    const RowClusters& C = plan->clusters;
    if (!forced && (C.num < 2 || C.inside_fraction < 0.5)) return false;
    const int nvec = (d + vec - 1) / vec;
    const int64_t vec_bytes = (int64_t)vec * es;
    int S = 0;
    if (plan->opt.column_slices > 0) {
        S = (int)std::min<int64_t>(plan->opt.column_slices, nvec);
    } else {
        const double room = kL2Share * (double)l2_bytes_per_xcd();
        for (int s = 1; s <= 16 && s <= nvec; ++s) {
            const int64_t bytes = (int64_t)((nvec + s - 1) / s) * vec_bytes;
            if (s > 1 && bytes < kLineBytes) break;
            // a slice of a row that does not start on a line boundary touches one more line
            if (C.typical_rows * (double)(bytes + kLineBytes - vec_bytes) <= room) {
                S = s;
                break;
            }
        }
        if (S == 0) {
            if (!forced) return false;
            S = std::min(nvec, 8);
        }
    }
    const int slice_vecs = (nvec + S - 1) / S;
    num_slices = (nvec + slice_vecs - 1) / slice_vecs;
    slice_elems = slice_vecs * vec;
    return true;
}

namespace {

template <class T>
gp_status upload_now(T*& dptr, const std::vector<T>& h, hipStream_t stream)
{
    dptr = nullptr;
    if (h.empty()) return GP_OK;
    GP_HIP(hipMalloc((void**)&dptr, h.size() * sizeof(T)));
    hipError_t e = hipMemcpyAsync(dptr, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);  // pageable source: done before the vector goes away
    if (e != hipSuccess) {
        (void)hipFree(dptr);
        dptr = nullptr;
        return fail(GP_ERR_DEVICE, "upload failed: %s", hipGetErrorString(e));
    }
    return GP_OK;
}

// What this plan's split schedule calls hot (plan->mu held; decided once per plan, from the graph
// and the plan's options): its row clusters if it has them, else its most popular rows if
// they are the source of enough non-zeros to be worth a launch of their own, else nothing.
constexpr double kMinHubFraction = 0.15;
constexpr double kMinHubWork = 2e9;  // non-zeros x columns below which the pass's launches cost more than they save
void decide_hot_mode(const gp_plan* plan, int32_t d)
{
    if (plan->hot_mode != 0) return;
    plan->hot_mode = 3;
    if (plan->opt.cache_schedule == 2 || plan->segs.empty()) return;
    if (!plan->clusters.ready) cluster_rows(*plan, plan->clusters);
    const RowClusters& C = plan->clusters;
    // clusters count if a typical one could be kept close at all: its rows' narrowest slices (one line)
    // in the share of an L2 the schedule counts on
    const bool small_enough = C.typical_rows * (double)kLineBytes <= kL2Share * (double)l2_bytes_per_xcd();
    if (plan->opt.cache_schedule == 1 || (C.num >= 2 && C.inside_fraction >= 0.5 && small_enough)) {
        plan->hot_sets = hot_sets_from_clusters(C);
        plan->hot_mode = 1;
        return;
    }
    const bool forced = plan->opt.hub_pass == 1;
    if (plan->opt.hub_pass == 2 || plan->opt.lds_pass == 2 || plan->opt.split_records == 2) return;
    if (!forced && (double)plan->nnz * (double)d < kMinHubWork) return;
    // about 2048 work items (set x strip) per launch, sets of at least 1024 rows (measured on config 3: 10 / 20 / 40 /
    // 81 / 160 sets of its 25 strips give an LDS launch of 1.28 / 1.08 / 1.07 / 0.80 / 0.77 ms and a segment launch
    // of 6.66 / 6.75 / 6.77 / 6.83 / 6.86 - 7.03 ms: larger sets order more rows by their number of hot non-zeros)
    const int64_t strips = ((int64_t)d + 3) / 4;
    int64_t sets = plan->opt.hub_sets > 0 ? plan->opt.hub_sets : std::max<int64_t>(1, 2048 / strips);
    int64_t rows_per_set = std::max<int64_t>(plan->opt.hub_sets > 0 ? 64 : 1024, (plan->n + sets - 1) / sets);
    HotSets H = hot_sets_from_hubs(*plan, kLdsMaxMembers, rows_per_set);
    if (!forced && H.hot_fraction < kMinHubFraction) return;
    // ... but no more sets than have enough to read each (the hubs do not depend on the sets: same list)
    const int64_t reads = (int64_t)(1.5 * H.hot_fraction * (double)plan->nnz);
    if (plan->opt.hub_sets == 0 && reads / kLdsMinReadsPerSet < H.num_sets) {
        sets = std::max<int64_t>(1, reads / (2 * kLdsMinReadsPerSet));
        rows_per_set = std::max<int64_t>(1024, (plan->n + sets - 1) / sets);
        H = hot_sets_from_hubs(*plan, kLdsMaxMembers, rows_per_set);
    }
    plan->hot_sets = std::move(H);
    plan->hot_mode = 2;
}

// The split schedule on the device (plan->mu held): reordered column list, cold records,
// the rows that own partial rows, and a partial-row buffer wide enough for d columns.
gp_status ensure_split(const gp_plan* plan, int32_t d, bool want_edge_weights, hipStream_t stream)
{
    DevicePlan& D = plan->dev;
    gp_status st;
    if (!D.split_ready) {
        SplitSchedule sch;
        build_split_schedule(*plan, plan->hot_sets, sch);
        if (sch.num_slots > INT32_MAX) return fail(GP_ERR_OVERFLOW, "%lld partial rows exceed int32", (long long)sch.num_slots);
        if ((st = upload_now(D.split_col, sch.col, stream)) != GP_OK || (st = upload_now(D.split_cold, sch.cold, stream)) != GP_OK ||
            (st = upload_now(D.split_rows, sch.split, stream)) != GP_OK)
            return st;
        D.split_num_cold = (int64_t)sch.cold.size();
        D.split_num_rows = (int64_t)sch.split.size();
        D.split_num_slots = sch.num_slots;
        D.split_hot_host.swap(sch.hot);
        D.split_ready = true;
    }
    if (want_edge_weights && !D.split_edge_ws && plan->nnz > 0) {
        GP_HIP(hipMalloc((void**)&D.split_edge_ws, (size_t)plan->nnz * sizeof(float)));
        if ((st = launch_fill_edge_weights(D.split_col, D.dinv_sqrt, D.split_edge_ws, plan->nnz, stream)) != GP_OK) return st;
        GP_HIP(hipStreamSynchronize(stream));
    }
    const int64_t need_ld = ((int64_t)d + 3) / 4 * 4;
    if (D.split_num_slots > 0 && need_ld > D.split_carry_ld) {
        if (D.split_carry) D.retired.push_back(D.split_carry);
        D.split_carry = nullptr;
        D.split_carry_ld = 0;
        GP_HIP(hipMalloc((void**)&D.split_carry, (size_t)D.split_num_slots * need_ld * sizeof(float)));
        D.split_carry_ld = need_ld;
    }
    return GP_OK;
}

// The LDS pass's schedule on the device (plan->mu held), and planes for rows of d columns.
// D.lds_state says afterwards whether the pass applies to this plan (1) or not (2).
gp_status ensure_lds(const gp_plan* plan, int32_t d, hipStream_t stream)
{
    DevicePlan& D = plan->dev;
    gp_status st;
    if (plan->opt.lds_pass == 2) D.lds_state = 2;
    if (D.lds_state == 0) {
        // Padding of the groups is work without result: beyond a limit the per-XCD lists (clusters)
        // or plain gathers from memory (hubs) are the better schedule, unless the pass is forced.
        const bool forced = plan->opt.lds_pass == 1 || plan->opt.lds_pass == 3;
        const double limit = plan->hot_mode == 2 ? kLdsMaxCostHubs : kLdsMaxCostClusters;
        LdsSchedule L;
        if (build_lds_schedule(*plan, plan->hot_sets, forced ? kLdsForcedCost : limit, plan->opt.lds_pass == 1 ? 2 : plan->opt.lds_pass == 3 ? 1 : 0,
                               L)) {
            if ((st = upload_now(D.lds_col, L.col, stream)) != GP_OK || (st = upload_now(D.lds_cold, L.cold, stream)) != GP_OK ||
                (st = upload_now(D.lds_members, L.members, stream)) != GP_OK ||
                (st = upload_now(D.lds_member_off, L.member_off, stream)) != GP_OK ||
                (st = upload_now(D.lds_list_of_set, L.list_of_set, stream)) != GP_OK ||
                (st = upload_now(D.lds_group_off, L.group_off, stream)) != GP_OK ||
                (st = upload_now(D.lds_wave_cut, L.wave_cut, stream)) != GP_OK ||
                (st = upload_now(D.lds_groups, L.groups, stream)) != GP_OK || (st = upload_now(D.lds_ids, L.ids, stream)) != GP_OK)
                return st;
            D.lds_set_reads = L.set_reads;
            if ((st = prepare_hot_lds(L.max_members)) != GP_OK) return st;
            D.lds_max_members = L.max_members;
            D.lds_num_members = (int64_t)L.members.size();
            D.lds_num_sets = (int32_t)L.list_of_set.size();
            D.lds_state = 1;
        } else {
            D.lds_state = 2;
        }
    }
    const int64_t strips = ((int64_t)d + 3) / 4;
    if (D.lds_state == 1 && (int)strips != D.lds_octets_strips) {
        // the launch's work units for rows of this many strips
        std::vector<LdsOctet> octets;
        deal_lds_octets(D.lds_set_reads, (int)strips, octets, D.lds_octet_off);
        if (D.lds_octets) D.retired.push_back(D.lds_octets);
        D.lds_octets = nullptr;
        D.lds_octets_strips = 0;
        if ((st = upload_now(D.lds_octets, octets, stream)) != GP_OK) return st;
        D.lds_octets_strips = (int)strips;
    }
    if (D.lds_state == 1 && strips > D.lds_planes_strips) {
        if (D.lds_planes) D.retired.push_back(D.lds_planes);
        if (D.lds_packed) D.retired.push_back(D.lds_packed);
        D.lds_planes = D.lds_packed = nullptr;
        D.lds_planes_strips = 0;
        GP_HIP(hipMalloc((void**)&D.lds_planes, (size_t)((strips + 7) / 8) * plan->segs.size() * 32 * sizeof(float)));
        // lists that several sets stage (the hubs) are packed strip by strip once per hop
        if (plan->hot_mode == 2) GP_HIP(hipMalloc((void**)&D.lds_packed, (size_t)strips * (size_t)D.lds_num_members * 4 * sizeof(float)));
        D.lds_planes_strips = strips;
    }
    return GP_OK;
}

// Gives the launch explicit work lists if the plan's cache schedule applies to it
// (building and uploading them on first use of a slice shape).  *split comes back true
// when the lists hold the hot pieces of the split schedule: the caller then runs the cold
// records first and reads column ids, weights and partial rows from the split schedule.
gp_status attach_work_lists(const gp_plan* plan, HopArgs& a, hipStream_t stream, bool may_build = true, bool* split = nullptr,
                            bool* lds = nullptr)
{
    if (split) *split = false;
    if (lds) *lds = false;
    const int es = a.dtype == GP_F32 ? 4 : 2;
    const int vec = hop_vector_width(a);
    // several column passes: implicit lists (explicit ones are cut for the whole row)
    if (pass_width(a.column_tile, a.dtype, a.d, a.ldin, a.xout ? a.ldout : a.ldin, a.xin, a.xout ? a.xout : a.xin) < a.d)
        return GP_OK;
    std::lock_guard<std::mutex> lk(plan->mu);
    int S = 0, elems = 0;
    if (!may_build && plan->hot_mode == 0) return GP_OK;  // nothing built yet: implicit lists
    decide_hot_mode(plan, a.d);
    DevicePlan& D = plan->dev;
    // the hot non-zeros can come out of LDS where the segment kernel's vectors are whole strips of four columns:
    // fp32 rows, or bf16 rows of a multiple of four columns in vectors of 4 or 8; a caller that may not allocate
    // gets the pass if an earlier call has left everything it needs
    const int64_t strips = ((int64_t)a.d + 3) / 4;
    const bool all_there = D.lds_state == 1 && D.lds_octets_strips == (int)strips && D.lds_planes_strips >= strips;  // nothing to build
    const bool lds_call = lds && (may_build || all_there) && a.d >= 4 && plan->opt.lds_pass != 2 && plan->opt.split_records != 2 &&
                          (a.dtype == GP_F32 ? vec == 4 : (a.d % 4 == 0 && (vec == 4 || vec == 8)));
    // the LDS pass: wherever the plan's lists are short enough for it (the plan's clusters, or its hubs)
    if (lds_call && (plan->hot_mode == 1 || plan->hot_mode == 2)) {
        gp_status st = all_there ? GP_OK : ensure_lds(plan, a.d, stream);
        if (st != GP_OK) return st;
        if (D.lds_state == 1) {
            *lds = true;
            return GP_OK;
        }
    }
    // no clusters: nothing an L2 could be made to hold
    if (plan->hot_mode != 1 || !choose_cache_schedule(plan, a.d, es, vec, S, elems)) return GP_OK;
    // hot and cold pieces in phases of their own need buffers of their own: only where the caller may allocate
    // (not worth it when hardly anything leaves the clusters: every row then pays two partial rows for nothing)
    const bool want_split = split && may_build && plan->opt.split_records != 2 &&
                            (plan->opt.split_records == 1 || plan->clusters.inside_fraction < 0.98);
    if (want_split) {
        gp_status st = ensure_split(plan, a.d, a.edge_w != nullptr, stream);
        if (st != GP_OK) return st;
    }
    const XcdWork* found = nullptr;
    for (const XcdWork& w : D.work)
        if (w.num_slices == S && w.slice_elems == elems && w.split == want_split) found = &w;
    if (!found && !may_build) return GP_OK;
    if (!found) {
        std::vector<Segment> recs;
        XcdWork w;
        w.num_slices = S;
        w.slice_elems = elems;
        w.split = want_split;
        build_xcd_lists(*plan, want_split ? D.split_hot_host : plan->segs, plan->clusters, S, elems, a.d, recs, w.off);
        // a request to the cursor should be worth about 64 non-zeros of gathering
        const int64_t mean_len = std::max<int64_t>(1, plan->nnz / std::max<int64_t>(1, (int64_t)plan->segs.size()));
        w.chunk_records = (int)std::min<int64_t>(32, std::max<int64_t>(1, 64 / mean_len));
        GP_HIP(hipMalloc((void**)&w.recs, recs.size() * sizeof(Segment)));
        hipError_t e = hipMemcpyAsync(w.recs, recs.data(), recs.size() * sizeof(Segment), hipMemcpyHostToDevice, stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);  // pageable source: done before `recs` goes away
        if (e != hipSuccess) {
            (void)hipFree(w.recs);
            return fail(GP_ERR_DEVICE, "upload of the work lists failed: %s", hipGetErrorString(e));
        }
        D.work.push_back(w);
        found = &D.work.back();
    }
    a.segs = found->recs;
    a.num_segs = found->off[8];
    a.xcd_off = found->off;
    a.chunk_records = found->chunk_records;
    a.num_slices = found->num_slices;
    a.slice_elems = found->slice_elems;
    if (split) *split = found->split;
    return GP_OK;
}

}  // namespace

gp_status hop_passes(const HopArgs& a0, hipStream_t stream)
{
    const int es = a0.dtype == GP_F32 ? 4 : 2;
    const int64_t tile = pass_width(a0.column_tile, a0.dtype, a0.d, a0.ldin, a0.xout ? a0.ldout : a0.ldin, a0.xin, a0.xout ? a0.xout : a0.xin);
    for (int64_t c0 = 0; c0 < a0.d; c0 += tile) {
        HopArgs a = a0;
        a.d = (int32_t)std::min<int64_t>(tile, a0.d - c0);
        a.xin = (const char*)a0.xin + c0 * es;
        a.xout = (char*)a0.xout + c0 * es;
        a.carry = a0.carry ? a0.carry + c0 : nullptr;
        a.xout = a0.xout ? (char*)a0.xout + c0 * es : nullptr;
        a.comb = a0.comb ? a0.comb + c0 : nullptr;
        if (tile < a0.d && a0.xcd_off) return fail(GP_ERR_INVALID_ARG, "explicit work lists need a single column pass");
        profile_begin("gp_hop_segments", stream);
        gp_status st = launch_hop(a, stream);
        profile_end(stream);
        if (st != GP_OK) return st;
    }
    return GP_OK;
}

gp_status fixup_passes(const FixupArgs& f0, hipStream_t stream)
{
    const int es = f0.dtype == GP_F32 ? 4 : 2;
    const int64_t tile = f0.xout ? pass_width(f0.column_tile, f0.dtype, f0.d, f0.ldout, f0.ldout, f0.xout, f0.xout)
                                 : pass_width(f0.column_tile, GP_F32, f0.d, f0.ldc, f0.ldc, f0.comb, f0.comb);
    for (int64_t c0 = 0; c0 < f0.d; c0 += tile) {
        FixupArgs f = f0;
        f.d = (int32_t)std::min<int64_t>(tile, f0.d - c0);
        f.xout = (char*)f0.xout + c0 * es;
        f.carry = f0.carry + c0;
        f.xout = f0.xout ? (char*)f0.xout + c0 * es : nullptr;
        f.comb = f0.comb ? f0.comb + c0 : nullptr;
        profile_begin("gp_fixup_rows", stream);
        gp_status st = launch_fixup(f, stream);
        profile_end(stream);
        if (st != GP_OK) return st;
    }
    return GP_OK;
}

gp_status propagate_resident(const gp_plan* plan, const void* X, int64_t ldx, int32_t d, gp_dtype dtype, gp_agg agg,
                             int32_t K, void* out, int64_t ldo, hipStream_t stream)
{
    gp_status st = ensure_device(plan, d, agg == GP_AGG_SYM, stream);
    if (st != GP_OK) return st;
    const DevicePlan& D = plan->dev;
    return resident_hops(plan, X, ldx, d, dtype, agg, K, out, ldo, stream, D.carry, D.carry_ld, D.ctrl, true);
}

// One hop with the LDS pass: the non-zeros whose source is on a list first, out of LDS, into the
// planes; then the segment kernel over the other non-zeros, in the same order of segments, adding
// the plane entries and finishing every segment as the plan says (a = the hop's launch as it would
// be on implicit lists; its record list, column list and weights are replaced here).
gp_status lds_hop(const gp_plan* plan, HopArgs& a, gp_agg agg, hipStream_t stream)
{
    const DevicePlan& D = plan->dev;
    gp_status st;
    HotLdsArgs h;
    h.members = D.lds_members;
    h.member_off = D.lds_member_off;
    h.list_of_set = D.lds_list_of_set;
    h.group_off = D.lds_group_off;
    h.wave_cut = D.lds_wave_cut;
    h.groups = D.lds_groups;
    h.octets = D.lds_octets;
    h.octet_off = D.lds_octet_off;
    h.ids = D.lds_ids;
    h.num_sets = D.lds_num_sets;
    h.max_members = D.lds_max_members;
    h.src_scale = agg == GP_AGG_SYM ? D.dinv_sqrt : nullptr;
    h.xin = a.xin;
    h.dtype = a.dtype;
    h.ldin = a.ldin;
    h.planes = D.lds_planes;
    h.num_pos = (int64_t)plan->segs.size();
    // Strips of a position that lie together in the planes, P.  Both launches pay per line they touch: the
    // LDS kernel's store of a strip's sums of 64 positions touches 8 P lines, the segment kernel's record
    // strips / P.  With long segments (clusters) stores are rare and P = 8 serves the reader; with short
    // ones (hubs) the stores are what the LDS kernel waits for, and P = 2 .. 4 is the least in sum.
    const int64_t together = plan->opt.plane_strips > 0 ? plan->opt.plane_strips : plan->hot_mode == 2 ? 4 : 8;
    h.plane_log2 = together == 1 ? 0 : together == 2 ? 1 : together == 4 ? 2 : 3;
    h.packed = D.lds_packed;
    h.num_members = D.lds_num_members;
    h.d = a.d;
    h.ctrl = a.ctrl;
    if (h.packed) {
        profile_begin("gp_pack_strips", stream);
        st = launch_pack_strips(h, stream);
        profile_end(stream);
        if (st != GP_OK) return st;
    }
    profile_begin("gp_hop_cluster_lds", stream);
    st = launch_hot_lds(h, stream);
    profile_end(stream);
    if (st != GP_OK) return st;
    a.segs = D.lds_cold;
    a.col = D.lds_col;
    if (a.edge_w) {  // weights by column id: the per-edge array follows the plan's column order
        a.edge_w = D.dinv_sqrt;
        a.edge_w_per_edge = false;
    }
    a.planes = D.lds_planes;
    a.num_pos = h.num_pos;
    a.plane_log2 = h.plane_log2;
    return hop_passes(a, stream);
}

// The hop loop on a plan that is already on the device.  may_allocate = false: only what
// exists is used (work lists that have been built, else the implicit ones; for the sym
// operator the per-edge weight array if it exists, else the weights gathered by column id,
// which are the same numbers) and nothing is allocated.
gp_status resident_hops(const gp_plan* plan, const void* X, int64_t ldx, int32_t d, gp_dtype dtype, gp_agg agg, int32_t K,
                        void* out, int64_t ldo, hipStream_t stream, float* carry, int64_t carry_ld,
                        unsigned long long* ctrl, bool may_allocate)
{
    gp_status st = GP_OK;
    const DevicePlan& D = plan->dev;
    const int64_t n = plan->n;
    const int es = dtype == GP_F32 ? 4 : 2;
    char* base = (char*)out;
    const int64_t slab = n * ldo * es;

    // slot 0 = X
    if (X != out) {
        profile_begin("gp_copy_rows", stream);
        st = launch_copy_rows(X, ldx, out, ldo, n, d, dtype, stream);
        profile_end(stream);
        if (st != GP_OK) return st;
    }

    const bool per_edge = D.edge_ws != nullptr;
    const float* edge_w = agg == GP_AGG_SYM ? (per_edge ? D.edge_ws : D.dinv_sqrt) : nullptr;
    const float* row_scale = agg == GP_AGG_SYM ? D.dinv_sqrt : agg == GP_AGG_MEAN ? D.dinv : nullptr;

    for (int32_t k = 1; k <= K; ++k) {
        HopArgs a;
        a.segs = D.segs;
        a.num_segs = (int64_t)plan->segs.size();
        a.col = D.col;
        a.col_base = 0;
        a.edge_w = edge_w;
        a.edge_w_per_edge = per_edge;
        a.row_scale = row_scale;
        a.xin = base + (int64_t)(k - 1) * slab;
        a.ldin = ldo;
        a.xout = base + (int64_t)k * slab;
        a.ldout = ldo;
        a.carry = carry;
        a.carry_ld = carry_ld;
        a.ctrl = ctrl;
        a.d = d;
        a.dtype = dtype;
        a.column_slices = plan->opt.column_slices;
        a.persistent_blocks = plan->opt.persistent_blocks;
        a.column_tile = plan->opt.column_tile;
        bool split = false, lds = false;
        HopArgs cold = a;  // as it stands: implicit lists
        if ((st = attach_work_lists(plan, a, stream, may_allocate, &split, &lds)) != GP_OK) return st;
        if (split) {
            // Records that gather outside their row's cluster first, whole rows wide: nothing of
            // theirs is worth keeping in a cache, and run on their own they evict nothing that is.
            // Then the records that gather inside it, from the per-XCD lists.  Both kinds leave
            // partial rows; the fix-up below joins them.
            a.col = cold.col = D.split_col;
            if (a.edge_w) {
                a.edge_w = cold.edge_w = D.split_edge_ws;
                a.edge_w_per_edge = cold.edge_w_per_edge = true;
            }
            a.carry = cold.carry = D.split_carry;
            a.carry_ld = cold.carry_ld = D.split_carry_ld;
            cold.segs = D.split_cold;
            cold.num_segs = D.split_num_cold;
            if (cold.num_segs > 0 && (st = hop_passes(cold, stream)) != GP_OK) return st;
        }
        if (lds) {
            if ((st = lds_hop(plan, a, agg, stream)) != GP_OK) return st;
        } else if ((st = hop_passes(a, stream)) != GP_OK) {
            return st;
        }
        if (split ? D.split_num_rows > 0 : !plan->split.empty()) {
            FixupArgs f;
            f.split = split ? D.split_rows : D.split;
            f.num_split = split ? D.split_num_rows : (int64_t)plan->split.size();
            f.carry = split ? D.split_carry : carry;
            f.carry_ld = split ? D.split_carry_ld : carry_ld;
            f.row_scale = row_scale;
            f.xout = a.xout;
            f.ldout = ldo;
            f.d = d;
            f.dtype = dtype;
            f.column_tile = plan->opt.column_tile;
            if ((st = fixup_passes(f, stream)) != GP_OK) return st;
        }
    }
    return GP_OK;
}

// out = sum_k coeff[k] * A^^k X without the stack: hop k reads slab (k-1)&1 (X for k = 1),
// writes slab k&1 (nothing for k = K) and adds coeff[k] times its fp32 rows into the
// accumulator, which is `out` itself for fp32 and an fp32 scratch for bf16 storage.
gp_status propagate_combine(const gp_plan* plan, const void* X, int64_t ldx, int32_t d, gp_dtype dtype, gp_agg agg,
                            int32_t K, const float* coeff, void* out, int64_t ldo, hipStream_t stream)
{
    gp_status st = ensure_device(plan, d, agg == GP_AGG_SYM, stream);
    if (st != GP_OK) return st;
    DevicePlan& D = plan->dev;
    const int64_t n = plan->n;
    const int es = dtype == GP_F32 ? 4 : 2;
    const int64_t ldp = ((int64_t)d + 16 / es - 1) / (16 / es) * (16 / es);  // slab rows start on 16 bytes
    const int64_t ldc_scratch = ((int64_t)d + 3) / 4 * 4;
    {
        std::lock_guard<std::mutex> lk(plan->mu);
        const int64_t need = n * ldp * es;
        if (K >= 2 && need > D.ping_bytes) {
            if (D.ping[0]) D.retired.push_back(D.ping[0]);
            if (D.ping[1]) D.retired.push_back(D.ping[1]);
            D.ping[0] = D.ping[1] = nullptr;
            D.ping_bytes = 0;
            GP_HIP(hipMalloc(&D.ping[0], (size_t)need));
            GP_HIP(hipMalloc(&D.ping[1], (size_t)need));
            D.ping_bytes = need;
        }
        if (dtype == GP_BF16 && n * ldc_scratch > D.comb_elems) {
            if (D.comb) D.retired.push_back(D.comb);
            D.comb = nullptr;
            D.comb_elems = 0;
            GP_HIP(hipMalloc((void**)&D.comb, (size_t)(n * ldc_scratch) * sizeof(float)));
            D.comb_elems = n * ldc_scratch;
        }
    }
    float* comb = dtype == GP_F32 ? (float*)out : D.comb;
    const int64_t ldc = dtype == GP_F32 ? ldo : ldc_scratch;

    // k = 0 term
    profile_begin("gp_scale_convert", stream);
    st = launch_scale_convert(X, ldx, dtype, comb, ldc, GP_F32, n, d, coeff[0], stream);
    profile_end(stream);
    if (st != GP_OK) return st;

    const float* edge_w = agg == GP_AGG_SYM ? D.edge_ws : nullptr;
    const float* row_scale = agg == GP_AGG_SYM ? D.dinv_sqrt : agg == GP_AGG_MEAN ? D.dinv : nullptr;
    for (int32_t k = 1; k <= K; ++k) {
        HopArgs a;
        a.segs = D.segs;
        a.num_segs = (int64_t)plan->segs.size();
        a.col = D.col;
        a.col_base = 0;
        a.edge_w = edge_w;
        a.edge_w_per_edge = true;
        a.row_scale = row_scale;
        a.xin = k == 1 ? X : D.ping[(k - 1) & 1];
        a.ldin = k == 1 ? ldx : ldp;
        a.xout = k == K ? nullptr : D.ping[k & 1];
        a.ldout = ldp;
        a.carry = D.carry;
        a.carry_ld = D.carry_ld;
        a.ctrl = D.ctrl;
        a.d = d;
        a.dtype = dtype;
        a.column_slices = plan->opt.column_slices;
        a.persistent_blocks = plan->opt.persistent_blocks;
        a.column_tile = plan->opt.column_tile;
        a.comb = comb;
        a.ldc = ldc;
        a.gamma = coeff[k];
        bool lds = false;
        if ((st = attach_work_lists(plan, a, stream, true, nullptr, &lds)) != GP_OK) return st;
        if (lds) {
            if ((st = lds_hop(plan, a, agg, stream)) != GP_OK) return st;
        } else if ((st = hop_passes(a, stream)) != GP_OK) {
            return st;
        }
        if (!plan->split.empty()) {
            FixupArgs f;
            f.split = D.split;
            f.num_split = (int64_t)plan->split.size();
            f.carry = D.carry;
            f.carry_ld = D.carry_ld;
            f.row_scale = row_scale;
            f.xout = a.xout;
            f.ldout = ldp;
            f.d = d;
            f.dtype = dtype;
            f.column_tile = plan->opt.column_tile;
            f.comb = comb;
            f.ldc = ldc;
            f.gamma = coeff[k];
            if ((st = fixup_passes(f, stream)) != GP_OK) return st;
        }
    }
    if (dtype == GP_BF16) {
        profile_begin("gp_scale_convert", stream);
        st = launch_scale_convert(comb, ldc, GP_F32, out, ldo, GP_BF16, n, d, 1.0f, stream);
        profile_end(stream);
        if (st != GP_OK) return st;
    }
    return GP_OK;
}

}  // namespace gp

using namespace gp;

extern "C" gp_status gp_plan_row_clusters(const gp_plan* plan, int32_t* label, int32_t* num_clusters, double* inside_fraction,
                                          double* typical_rows)
{
    if (!plan) return fail(GP_ERR_INVALID_ARG, "plan is NULL");
    try {
        std::lock_guard<std::mutex> lk(plan->mu);
        if (!plan->clusters.ready) cluster_rows(*plan, plan->clusters);
        const RowClusters& C = plan->clusters;
        if (label) std::copy(C.label.begin(), C.label.end(), label);
        if (num_clusters) *num_clusters = C.num;
        if (inside_fraction) *inside_fraction = C.inside_fraction;
        if (typical_rows) *typical_rows = C.typical_rows;
    } catch (const std::exception& e) {
        return fail(GP_ERR_OOM_HOST, "gp_plan_row_clusters: %s", e.what());
    }
    return GP_OK;
}

extern "C" gp_status gp_plan_work_lists(const gp_plan* plan, int32_t d, gp_dtype dtype, int32_t vec, int32_t* num_slices,
                                        int32_t* slice_elems, int64_t* xcd_off, void* records, int64_t capacity)
{
    if (!plan || !num_slices || !slice_elems || !xcd_off) return fail(GP_ERR_INVALID_ARG, "NULL argument");
    if (d <= 0 || (dtype != GP_F32 && dtype != GP_BF16)) return fail(GP_ERR_INVALID_ARG, "bad d or dtype");
    const int es = dtype == GP_F32 ? 4 : 2;
    if (vec != 1 && vec != 2 && vec != 4 && !(vec == 8 && es == 2)) return fail(GP_ERR_INVALID_ARG, "vec = %d is no vector width", vec);
    try {
        std::lock_guard<std::mutex> lk(plan->mu);
        int S = 0, elems = 0;
        *num_slices = 0;
        *slice_elems = 0;
        for (int x = 0; x <= 8; ++x) xcd_off[x] = 0;
        if (!choose_cache_schedule(plan, d, es, vec, S, elems)) return GP_OK;  // implicit lists
        std::vector<Segment> recs;
        build_xcd_lists(*plan, plan->segs, plan->clusters, S, elems, d, recs, xcd_off);
        *num_slices = S;
        *slice_elems = elems;
        if (records) {
            if (capacity < (int64_t)recs.size())
                return fail(GP_ERR_INVALID_ARG, "records has room for %lld of %lld", (long long)capacity, (long long)recs.size());
            std::copy(recs.begin(), recs.end(), (Segment*)records);
        }
    } catch (const std::exception& e) {
        return fail(GP_ERR_OOM_HOST, "gp_plan_work_lists: %s", e.what());
    }
    return GP_OK;
}

extern "C" gp_status gp_plan_lds_schedule(const gp_plan* plan, int32_t d, int32_t order, gp_lds_view* v)
{
    if (!plan || !v) return fail(GP_ERR_INVALID_ARG, "NULL argument");
    if (order < 0 || order > 2) return fail(GP_ERR_INVALID_ARG, "order must be 0, 1 or 2");
    if (d < 4) return fail(GP_ERR_INVALID_ARG, "d = %d: the pass needs at least four columns", d);
    try {
        std::lock_guard<std::mutex> lk(plan->mu);
        v->num_groups = v->num_ids = v->num_members = v->num_positions = 0;
        v->num_sets = v->num_lists = v->conflict_free = v->hot_mode = 0;
        decide_hot_mode(plan, d);
        if (plan->hot_mode != 1 && plan->hot_mode != 2) return GP_OK;
        LdsSchedule L;
        const double limit = plan->hot_mode == 2 ? kLdsMaxCostHubs : kLdsMaxCostClusters;
        if (!build_lds_schedule(*plan, plan->hot_sets, order == 0 ? limit : kLdsForcedCost, order, L)) return GP_OK;
        v->hot_mode = plan->hot_mode;
        v->num_groups = (int64_t)L.groups.size() - 1;  // (without the sentinel)
        v->num_ids = (int64_t)L.ids.size();
        v->num_members = (int64_t)L.members.size();
        v->num_positions = (int64_t)L.cold.size();
        v->num_sets = (int32_t)L.list_of_set.size();
        v->num_lists = (int32_t)L.member_off.size() - 1;
        v->conflict_free = L.conflict_free ? 1 : 0;
        const bool per_group = v->group_set || v->group_id_off || v->group_steps || v->rec_pos;
        if ((per_group && v->group_capacity < v->num_groups) || (v->ids && v->id_capacity < v->num_ids) ||
            (v->list_of_set && v->set_capacity < v->num_sets) || (v->member_off && v->set_capacity < v->num_lists + 1) ||
            (v->members && v->member_capacity < v->num_members) ||
            ((v->rest || v->col) && v->position_capacity < std::max<int64_t>(v->num_positions, v->col ? plan->nnz : 0)))
            return fail(GP_ERR_INVALID_ARG, "an array is too small: %lld groups, %lld ids, %d sets, %d lists, %lld members, %lld positions",
                        (long long)v->num_groups, (long long)v->num_ids, v->num_sets, v->num_lists, (long long)v->num_members,
                        (long long)v->num_positions);
        for (int32_t c = 0; c < v->num_sets; ++c)
            for (int32_t g = L.group_off[(size_t)c]; g < L.group_off[(size_t)c + 1]; ++g) {
                if (v->group_set) v->group_set[g] = c;
                if (v->group_id_off) v->group_id_off[g] = L.groups[(size_t)g].id_off;
                if (v->group_steps) v->group_steps[g] = L.groups[(size_t)g].steps;
            }
        if (v->rec_pos)
            for (int64_t g = 0; g < v->num_groups; ++g)
                for (int l = 0; l < 64; ++l)
                    v->rec_pos[g * 64 + l] = l < L.groups[(size_t)g].count ? (int32_t)(L.groups[(size_t)g].first_pos + l) : -1;
        if (v->ids) std::copy(L.ids.begin(), L.ids.end(), v->ids);
        if (v->list_of_set) std::copy(L.list_of_set.begin(), L.list_of_set.end(), v->list_of_set);
        if (v->member_off) std::copy(L.member_off.begin(), L.member_off.end(), v->member_off);
        if (v->members) std::copy(L.members.begin(), L.members.end(), v->members);
        if (v->rest) std::copy(L.cold.begin(), L.cold.end(), (Segment*)v->rest);
        if (v->col) std::copy(L.col.begin(), L.col.end(), v->col);
    } catch (const std::exception& e) {
        return fail(GP_ERR_OOM_HOST, "gp_plan_lds_schedule: %s", e.what());
    }
    return GP_OK;
}

extern "C" void gp_plan_destroy(gp_plan* plan)
{
    if (!plan) return;
    if (plan->dev.device >= 0) {
        const int home = plan->dev.device;  // release() resets the record
        int cur = -1;
        if (hipGetDevice(&cur) == hipSuccess) {
            if (cur != home) (void)hipSetDevice(home);
            (void)hipDeviceSynchronize();
            release(plan->dev);
            if (cur != home && cur >= 0) (void)hipSetDevice(cur);
        }
    }
    release_pinned(plan);
    delete plan;
}

extern "C" gp_status gp_propagate_combine(const gp_plan* plan, const void* X, int64_t ldx, int32_t d, gp_dtype dtype,
                                          gp_agg agg, int32_t K, const float* coeff, void* out, int64_t ldo,
                                          void* hip_stream)
{
    if (!plan) return fail(GP_ERR_INVALID_ARG, "plan is NULL");
    if (!X || !out || !coeff) return fail(GP_ERR_INVALID_ARG, "X, out or coeff is NULL");
    if (d <= 0) return fail(GP_ERR_INVALID_ARG, "d = %d must be positive", d);
    if (K < 0) return fail(GP_ERR_INVALID_ARG, "K = %d is negative", K);
    if (ldx < d || ldo < d) return fail(GP_ERR_INVALID_ARG, "leading dimension smaller than d");
    if (dtype != GP_F32 && dtype != GP_BF16) return fail(GP_ERR_INVALID_ARG, "unknown dtype %d", (int)dtype);
    if (agg != GP_AGG_SYM && agg != GP_AGG_MEAN && agg != GP_AGG_SUM)
        return fail(GP_ERR_INVALID_ARG, "unknown aggregation %d", (int)agg);
    if (X == out) return fail(GP_ERR_INVALID_ARG, "X and out must not overlap");
    const int es = dtype == GP_F32 ? 4 : 2;
    if (((uintptr_t)X % es) || ((uintptr_t)out % es)) return fail(GP_ERR_INVALID_ARG, "X / out not aligned to the element size");
    hipPointerAttribute_t ax, ao;
    if (hipPointerGetAttributes(&ax, X) != hipSuccess || hipPointerGetAttributes(&ao, out) != hipSuccess) {
        (void)hipGetLastError();
        return fail(GP_ERR_INVALID_ARG, "X / out is not device memory");
    }
    if (ax.type != hipMemoryTypeDevice || ao.type != hipMemoryTypeDevice)
        return fail(GP_ERR_UNSUPPORTED, "gp_propagate_combine takes device-resident operands only");
    try {
        return propagate_combine(plan, X, ldx, d, dtype, agg, K, coeff, out, ldo, (hipStream_t)hip_stream);
    } catch (const std::exception& e) {
        return fail(GP_ERR_OOM_HOST, "gp_propagate_combine: %s", e.what());
    }
}

extern "C" gp_status gp_propagate(const gp_plan* plan, const void* X, int64_t ldx, int32_t d, gp_dtype dtype,
                                  gp_agg agg, int32_t K, void* out_stack, int64_t ldo, void* hip_stream)
{
    if (!plan) return fail(GP_ERR_INVALID_ARG, "plan is NULL");
    if (!X || !out_stack) return fail(GP_ERR_INVALID_ARG, "X or out_stack is NULL");
    if (d <= 0) return fail(GP_ERR_INVALID_ARG, "d = %d must be positive", d);
    if (K < 0) return fail(GP_ERR_INVALID_ARG, "K = %d is negative", K);
    if (ldx < d || ldo < d) return fail(GP_ERR_INVALID_ARG, "leading dimension smaller than d (ldx %lld, ldo %lld, d %d)",
                                        (long long)ldx, (long long)ldo, d);
    if (dtype != GP_F32 && dtype != GP_BF16) return fail(GP_ERR_INVALID_ARG, "unknown dtype %d", (int)dtype);
    if (agg != GP_AGG_SYM && agg != GP_AGG_MEAN && agg != GP_AGG_SUM)
        return fail(GP_ERR_INVALID_ARG, "unknown aggregation %d", (int)agg);
    if (X == out_stack && ldx != ldo) return fail(GP_ERR_INVALID_ARG, "X aliases slot 0 but ldx != ldo");
    const int es = dtype == GP_F32 ? 4 : 2;
    if (((uintptr_t)X % es) || ((uintptr_t)out_stack % es))
        return fail(GP_ERR_INVALID_ARG, "X / out_stack not aligned to the element size");

    // 0 = device memory, 1 = pinned host memory, 2 = ordinary (pageable) host memory, which the
    // runtime does not know about
    auto kind_of = [](const void* p) {
        hipPointerAttribute_t at;
        if (hipPointerGetAttributes(&at, p) != hipSuccess) {
            (void)hipGetLastError();
            return 2;
        }
        if (at.type == hipMemoryTypeDevice) return 0;
        if (at.type == hipMemoryTypeHost) return 1;
        return at.type == hipMemoryTypeUnregistered ? 2 : 3;
    };
    const int kx = kind_of(X), ko = kind_of(out_stack);
    try {  // nothing may leave the C boundary as an exception
        if (kx == 0 && ko == 0) return propagate_resident(plan, X, ldx, d, dtype, agg, K, out_stack, ldo, (hipStream_t)hip_stream);
        if ((kx == 1 || kx == 2) && (ko == 1 || ko == 2))
            return propagate_streamed(plan, X, ldx, d, dtype, agg, K, out_stack, ldo, kx == 2 || ko == 2);
    } catch (const std::exception& e) {
        return fail(GP_ERR_OOM_HOST, "gp_propagate: %s", e.what());
    }
    return fail(GP_ERR_INVALID_ARG, "X and out_stack must both be device memory or both be host memory");
}
