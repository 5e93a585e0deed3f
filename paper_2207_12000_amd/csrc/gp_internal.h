// Internal declarations shared by the library's translation units.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <functional>
#include <mutex>
#include <string>
#include <vector>

#include "gp.h"

namespace gp {

// ---- error text ---------------------------------------------------------
gp_status fail(gp_status s, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
#define GP_HIP(call)                                                                      \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess)                                                             \
            return gp::fail(e_ == hipErrorOutOfMemory ? GP_ERR_OOM_DEVICE : GP_ERR_DEVICE, \
                            "%s failed: %s", #call, hipGetErrorString(e_));               \
    } while (0)

// ---- options ------------------------------------------------------------
struct Options {
    int64_t segment_edges = 0;  // 0 = chosen per plan from the non-zero count
    int64_t column_tile = 0;
    int64_t column_slices = 0;
    int64_t persistent_blocks = 0;
    int64_t cache_schedule = 0;  // 0 = decided per plan, 1 = explicit per-XCD lists always, 2 = never
    int64_t split_records = 0;   // explicit lists: 0 / 1 = hot and cold pieces in phases of their own, 2 = whole records
    int64_t lc_tile_rows = 0;  // 0 = chosen per call from the batch size
    int64_t hbm_budget_bytes = 0;
    int64_t lds_pass = 0;        // hot pieces gathered from LDS where the clusters fit it: 0 = automatic, 1 = wherever possible
                                 // (conflict-free order), 2 = never, 3 = wherever possible (column-list order)
    int64_t device_plan_chunk = 0;  // GP_PLAN_ON_DEVICE: most candidate entries sorted at once, 0 = 2^31 - 1
};
Options& options();

int host_threads();
// Runs fn(t, nthreads) on nthreads host threads (t = 0 .. nthreads-1) and joins.
void parallel_run(int nthreads, const std::function<void(int, int)>& fn);

// ---- the schedule the kernels walk ----------------------------------------
// One run of consecutive non-zeros of one row, inside one edge block.
struct alignas(16) Segment {
    uint32_t start_lo;  // first non-zero (index into the sorted list), low 32 bits
    uint8_t start_hi;   // bits 32..39
    uint8_t slice;      // column slice the record is for (explicit per-XCD work lists; 0 in the plan's own list)
    uint16_t len;       // number of non-zeros, 0 for a row without any
    int32_t row;        // destination row
    int32_t slot;       // -1: the run is the whole row, result goes to the output row
                        // >=0: partial row, result goes to this row of the carry buffer
};
static_assert(sizeof(Segment) == 16, "Segment must be 16 bytes");

// A row that was cut (by a block boundary or by the segment length): its
// partial rows are carry slots [first_slot, first_slot + count) in list order.
struct SplitRow {
    int32_t row;
    int32_t count;
    int64_t first_slot;
};

// Row clusters of the cache schedule (gp_cluster.cpp).
struct RowClusters {
    bool ready = false;
    std::vector<int32_t> label;    // n: cluster of every row, clusters numbered 0 .. num-1
    int32_t num = 0;
    double inside_fraction = 0.0;  // share of the non-zeros whose source lies in the row's own cluster
    double typical_rows = 0.0;     // rows in the cluster of a typical non-zero (non-zero-weighted mean size)
};

// Explicit per-XCD work lists on the device, for one slice shape.
struct XcdWork {
    int num_slices = 0, slice_elems = 0, chunk_records = 1;
    bool split = false;       // the records are the hot pieces of the split schedule
    Segment* recs = nullptr;  // DEVICE
    int64_t off[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
};

struct LdsGroup;
struct DevicePlan {
    int device = -1;
    int32_t* col = nullptr;
    float* dinv_sqrt = nullptr;
    float* dinv = nullptr;
    Segment* segs = nullptr;
    SplitRow* split = nullptr;
    float* edge_ws = nullptr;   // nnz: dinv_sqrt[col[e]], built on first use of the sym operator
    float* carry = nullptr;     // num_slots x carry_ld fp32
    int64_t carry_ld = 0;
    unsigned long long* ctrl = nullptr;  // kHopCtrlWords words, zero between launches
    // scratch of gp_propagate_combine: two hop slabs and (bf16 storage) an fp32 accumulator
    void* ping[2] = {nullptr, nullptr};
    float* comb = nullptr;
    int64_t ping_bytes = 0, comb_elems = 0;
    std::vector<XcdWork> work;  // explicit work lists built so far (one per slice shape)
    // split schedule (hot / cold pieces of every segment), made on first use
    bool split_ready = false;
    int32_t* split_col = nullptr;     // reordered column list
    float* split_edge_ws = nullptr;   // per-edge weights in that order (sym operator)
    Segment* split_cold = nullptr;    // cold records, walked as an implicit list
    int64_t split_num_cold = 0;
    SplitRow* split_rows = nullptr;
    int64_t split_num_rows = 0, split_num_slots = 0;
    float* split_carry = nullptr;
    int64_t split_carry_ld = 0;
    std::vector<Segment> split_hot_host;  // hot records in plan order (source of the per-XCD lists)
    // LDS pass over the hot pieces: 0 = not looked at yet, 1 = ready, 2 = does not apply to this plan
    int lds_state = 0;
    int32_t *lds_members = nullptr, *lds_group_off = nullptr, *lds_rec_row = nullptr, *lds_rec_slot = nullptr;
    int64_t* lds_member_off = nullptr;
    LdsGroup* lds_groups = nullptr;
    uint16_t* lds_ids = nullptr;
    int32_t lds_max_members = 0;
    SplitRow* lds_fixup_rows = nullptr;
    int64_t lds_num_fixup_rows = 0;
    std::vector<void*> retired;  // buffers that were outgrown: freed with the plan, never while work may still use them
};

}  // namespace gp

struct gp_plan {
    int64_t n = 0, nnz = 0;
    uint32_t flags = 0;
    int32_t num_blocks = 0;
    std::vector<int64_t> block_off;
    std::vector<int32_t> block_row_lo, block_row_hi;
    std::vector<int64_t> rowptr;
    std::vector<int32_t> col;
    std::vector<int32_t> deg;
    std::vector<float> dinv_sqrt, dinv;

    // kernel schedule (library's own; not part of the checked plan)
    int64_t segment_edges = 0;
    std::vector<gp::Segment> segs;       // grouped by block, longest first inside a block
    std::vector<int64_t> seg_off;        // b+1: block p owns segs [seg_off[p], seg_off[p+1])
    std::vector<gp::SplitRow> split;     // ascending row
    int64_t num_slots = 0;

    gp::Options opt;  // the library options as they stood when the plan was made
    bool norms_on_device = false;  // GP_PLAN_ON_DEVICE: deg / dinv_sqrt / dinv came from the device

    mutable std::mutex mu;
    mutable gp::RowClusters clusters;  // made on first use (under mu)
    mutable gp::DevicePlan dev;
    // streamed schedule: pinned host mirror of col (made on first use) and the state kept
    // from one streamed call to the next (gp_stream.cpp owns both)
    mutable int32_t* pinned_col = nullptr;
    mutable void* streamed = nullptr;
};

namespace gp {

gp_status build_schedule(gp_plan* plan);
// segments, split rows and partial-row slots for the sorted list of `plan` cut at block_off
// (block p = [block_off[p], block_off[p+1])): the plan's own blocks, or another cut of the same list
gp_status cut_schedule(const gp_plan& plan, const std::vector<int64_t>& block_off, std::vector<Segment>& segs,
                       std::vector<int64_t>& seg_off, std::vector<SplitRow>& split, int64_t& num_slots);
void cluster_rows(const gp_plan& P, RowClusters& C);
void build_xcd_lists(const gp_plan& P, const std::vector<Segment>& segs, const RowClusters& C, int S, int slice_elems, int d,
                     std::vector<Segment>& recs, int64_t off[9]);
// The plan's segments cut into records that gather inside the row's cluster (hot) and records
// that gather outside it (cold), with a column list reordered to match (gp_cluster.cpp).
struct SplitSchedule {
    std::vector<int32_t> col;
    std::vector<Segment> hot, cold;
    std::vector<SplitRow> split;
    int64_t num_slots = 0;
};
void build_split_schedule(const gp_plan& P, const RowClusters& C, SplitSchedule& out);

// The hot pieces arranged for the LDS pass (gp_cluster.cpp builds it, gp_hot_lds.hip runs it): a
// cluster's source rows are staged in LDS one strip of four fp32 columns at a time, and
// its hot records, 64 to a group (one per lane, longest first), gather from there.
constexpr int kLdsBytesPerCu = 160 * 1024;
constexpr int kLdsMaxMembers = 10192;  // (rows rounded up to 16, + 16 zero rows) x 16 bytes and a few words must fit the LDS
struct LdsGroup {
    int64_t id_off;  // first of its steps x 64 local source indices; 8 consecutive steps of a lane lie together
    int32_t steps;   // multiple of 8; shorter records are padded with reads of zero rows
    int32_t pad;
};
struct LdsSchedule {
    std::vector<int32_t> members;     // rows of cluster c, ascending: members[member_off[c] .. member_off[c+1])
    std::vector<int64_t> member_off;  // num + 1
    std::vector<int32_t> group_off;   // num + 1: groups of cluster c
    std::vector<LdsGroup> groups;
    // 64 per group: where lane l's sum goes (row -1: no record).  slot >= 0: that partial row; -1: the
    // output row; <= -2: the output row, after adding partial row -2 - slot (written by the cold launch)
    std::vector<int32_t> rec_row, rec_slot;
    std::vector<SplitRow> fixup_rows;  // the cut rows this pass does not finish itself
    std::vector<uint16_t> ids;
    int32_t max_members = 0;  // largest cluster that has hot records
    int64_t hot_edges = 0;
    bool conflict_free = false;  // reads ordered so that the lanes of one LDS pass hit different banks
};
// Rows a strip occupies in LDS for a cluster of m rows: the rows, rounded up to 16, and 16 zero
// rows (one per bank group) that padding reads point at.
constexpr double kLdsMaxPadding = 0.3;  // padding reads the automatic choice accepts, as a share of the hot non-zeros
inline int64_t lds_rows(int64_t m) { return (m + 15) / 16 * 16 + 16; }
// false (and `out` unspecified) where the pass does not apply: a cluster with hot records is
// too large for the LDS, or padding would add more than `max_padding` of the hot non-zeros.
// order: 0 = conflict-free if its padding is acceptable, else the column list's; 1 = the
// column list's; 2 = conflict-free.
bool build_lds_schedule(const gp_plan& P, const RowClusters& C, const SplitSchedule& S, double max_padding, int order,
                        LdsSchedule& out);
struct HotLdsArgs {
    // DEVICE arrays of the schedule
    const int32_t* members;
    const int64_t* member_off;
    const int32_t* group_off;
    const LdsGroup* groups;
    const int32_t *rec_row, *rec_slot;
    const uint16_t* ids;
    int32_t num_clusters, max_members;
    const float* src_scale;  // DEVICE n weights applied to source rows, or nullptr
    const float* row_scale;  // DEVICE n scales applied to rows stored whole, or nullptr
    const float* xin;
    int64_t ldin;
    float* xout;
    int64_t ldout;
    float* carry;
    int64_t carry_ld;
    int32_t d;
    unsigned long long* ctrl;  // as HopArgs::ctrl
};
gp_status launch_hot_lds(const HotLdsArgs& a, hipStream_t stream);
// Slice shape of the explicit work lists for rows of d elements in vectors of `vec`
// (element size es), or false if this plan keeps the implicit lists.
bool choose_cache_schedule(const gp_plan* plan, int32_t d, int es, int vec, int& num_slices, int& slice_elems);
// fills plan->nnz, rowptr, col, deg from validated input pairs, on the current GPU
gp_status csr_on_device(const int32_t* src, const int32_t* dst, int64_t m, int64_t n, bool sym, bool loops, gp_plan* plan);
// fills block_row_lo / block_row_hi from rowptr and block_off, on the current GPU
gp_status block_rows_on_device(gp_plan* plan);

// resident schedule: everything already in HBM
gp_status propagate_resident(const gp_plan* plan, const void* X, int64_t ldx, int32_t d, gp_dtype dtype,
                             gp_agg agg, int32_t K, void* out, int64_t ldo, hipStream_t stream);
gp_status resident_hops(const gp_plan* plan, const void* X, int64_t ldx, int32_t d, gp_dtype dtype, gp_agg agg, int32_t K,
                        void* out, int64_t ldo, hipStream_t stream, float* carry, int64_t carry_ld,
                        unsigned long long* ctrl, bool may_allocate);
// streamed schedule: operands in pinned host memory
gp_status propagate_streamed(const gp_plan* plan, const void* X, int64_t ldx, int32_t d, gp_dtype dtype,
                             gp_agg agg, int32_t K, void* out, int64_t ldo, bool pageable);

// ---- kernel launchers (gp_kernels.hip) -------------------------------------
constexpr int kHopCtrlWords = 16;
struct HopArgs {
    const Segment* segs;    // DEVICE
    int64_t num_segs;
    const int32_t* col;     // DEVICE; entry e of the sorted list is col[e - col_base]
    int64_t col_base;
    const float* edge_w;    // DEVICE: nullptr (weight 1), or an n-vector gathered by column id,
                            // or (edge_w_per_edge) one weight per non-zero, indexed like col
    bool edge_w_per_edge = false;
    const float* row_scale; // DEVICE n-vector applied once per finished row, or nullptr
    const void* xin;        // DEVICE n x d, leading dimension ldin
    int64_t ldin;
    void* xout;             // DEVICE n x d, leading dimension ldout
    int64_t ldout;
    float* carry;           // DEVICE num_slots x carry_ld
    int64_t carry_ld;
    int32_t d;
    gp_dtype dtype;
    // DEVICE, kHopCtrlWords 64-bit words, zero between launches: the work cursors of the 8 XCDs
    // and the count of finished lane groups.  Launches that share it must not overlap in time.
    unsigned long long* ctrl = nullptr;
    // work lists.  xcd_off == nullptr: implicit lists over segs[0 .. num_segs), the slice count
    // chosen by launch_hop (column_slices: 1, 2, 4, 8 or 0 = automatic).  Otherwise HOST
    // array of 9 offsets: XCD x walks records [xcd_off[x], xcd_off[x+1]) of segs, each record
    // naming its slice; num_slices / slice_elems are then the caller's (slice_elems a
    // multiple of hop_vector_width()).
    const int64_t* xcd_off = nullptr;
    int chunk_records = 1;  // explicit lists: consecutive records handed out per request
    int num_slices = 1;
    int slice_elems = 0;
    int64_t column_slices = 0;
    int64_t persistent_blocks = 0;  // workgroups of the launch, 0 = as many as stay resident
    int64_t column_tile = 0;        // feature columns per kernel pass, 0 = automatic
    // optional running combination: comb[row] += gamma * result row (fp32, leading dimension ldc);
    // xout may then be nullptr (result row not stored)
    float* comb = nullptr;
    int64_t ldc = 0;
    float gamma = 0.0f;
};
gp_status launch_hop(const HopArgs& a, hipStream_t stream);
// widest vector (in elements) the operands of this launch are aligned for
int hop_vector_width(const HopArgs& a);

struct FixupArgs {
    const SplitRow* split;  // DEVICE
    int64_t num_split;
    const float* carry;
    int64_t carry_ld;
    const float* row_scale;
    void* xout;
    int64_t ldout;
    int32_t d;
    gp_dtype dtype;
    float* comb = nullptr;  // as in HopArgs
    int64_t ldc = 0;
    float gamma = 0.0f;
    int64_t column_tile = 0;
};
gp_status launch_fixup(const FixupArgs& a, hipStream_t stream);

gp_status launch_scale_convert(const void* src, int64_t lds, gp_dtype src_type, void* dst, int64_t ldd, gp_dtype dst_type,
                               int64_t n, int32_t d, float gamma, hipStream_t stream);
gp_status launch_zero_words(unsigned long long* p, int count, hipStream_t stream);
gp_status launch_fill_edge_weights(const int32_t* col, const float* by_col, float* w, int64_t nnz, hipStream_t stream);
// max_blocks > 0 caps the grid (copies over the host link need few workgroups and
// must leave the compute units to the kernels running beside them)
gp_status launch_copy_rows(const void* src, int64_t lds, void* dst, int64_t ldd, int64_t n, int32_t d,
                           gp_dtype dtype, hipStream_t stream, int max_blocks = 0);

void release_pinned(gp_plan* plan);

// all column passes of one hop kernel / of the fix-up, with the partial-row buffer
// offset pass by pass
gp_status hop_passes(const HopArgs& a, hipStream_t stream);
gp_status fixup_passes(const FixupArgs& f, hipStream_t stream);

// widest vector (in elements) every row start of both operands is aligned for
int vector_width(gp_dtype dtype, int32_t d, int64_t ld_a, int64_t ld_b, const void* pa, const void* pb);
// most feature columns one kernel pass covers with vectors of `vec` elements
int max_columns_per_pass(int vec);

// ---- profiling --------------------------------------------------------------
bool profiling_on();
void profile_begin(const char* name, hipStream_t stream);
void profile_end(hipStream_t stream);

}  // namespace gp
