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
    int64_t hub_pass = 0;        // graphs without row clusters: the most popular rows served from LDS: 0 = where it pays, 1 = always, 2 = never
    int64_t hub_sets = 0;        // hub pass: row sets the rows are cut into, 0 = automatic
    int64_t plane_strips = 0;    // LDS pass: strips of one position that lie together in the planes (1, 2, 4, 8), 0 = automatic
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

// Which non-zeros are "hot" (their source row is worth keeping close: in the L2 of the XCD
// that asks, or in LDS), and how the rows that own them are grouped into sets of work.
// Every set gathers its hot non-zeros from one list of rows.  Two ways to make them
// (gp_cluster.cpp): from row clusters (set = list = cluster: a row's hot non-zeros are those
// whose source is in the row's own cluster), or from the most popular rows (one list, the
// hubs, shared by all sets; sets are ranges of rows; hot = the source is a hub).
struct HotSets {
    int32_t num_sets = 0, num_lists = 0;
    std::vector<int32_t> set_of_row;   // n
    std::vector<int32_t> list_of_set;  // num_sets
    std::vector<int32_t> list_of_row;  // n: the list row j is on, -1 = none
    double hot_fraction = 0.0;         // share of the non-zeros that are hot
    // LDS pass: a segment with fewer hot non-zeros than this keeps them with its others.  A segment's sums
    // cross from one launch to the other through memory, a row's bytes written and read: about what two
    // gathers of popular rows cost the segment kernel.
    int32_t min_hot = 1;
    bool hot(int32_t row, int32_t src) const
    {
        const int32_t l = list_of_row[(size_t)src];
        return l >= 0 && l == list_of_set[(size_t)set_of_row[(size_t)row]];
    }
};

// Explicit per-XCD work lists on the device, for one slice shape.
struct XcdWork {
    int num_slices = 0, slice_elems = 0, chunk_records = 1;
    bool split = false;       // the records are the hot pieces of the split schedule
    Segment* recs = nullptr;  // DEVICE
    int64_t off[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
};

struct LdsGroup;
struct LdsOctet;
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
    int32_t *lds_members = nullptr, *lds_group_off = nullptr, *lds_list_of_set = nullptr, *lds_col = nullptr, *lds_wave_cut = nullptr;
    LdsOctet* lds_octets = nullptr;
    int64_t lds_octet_off[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
    std::vector<int64_t> lds_set_reads;  // per set: reads of its groups (octets are dealt per column count)
    int lds_octets_strips = 0;           // the strip count lds_octets was dealt for
    Segment* lds_cold = nullptr;    // the segments' other parts in position order
    float* lds_edge_ws = nullptr;   // per-edge weights in lds_col's order (sym operator)
    float* lds_planes = nullptr;
    float* lds_packed = nullptr;    // the lists' rows strip by strip (rewritten every hop)
    int64_t lds_num_members = 0;
    int64_t lds_planes_strips = 0;  // planes allocated
    int32_t lds_num_sets = 0;
    int64_t* lds_member_off = nullptr;
    LdsGroup* lds_groups = nullptr;
    uint16_t* lds_ids = nullptr;
    int32_t lds_max_members = 0;
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
    // what the split schedule calls hot: 0 = not decided yet, 1 = the row's own cluster, 2 = the hubs, 3 = nothing
    mutable int hot_mode = 0;
    mutable gp::HotSets hot_sets;
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
HotSets hot_sets_from_clusters(const RowClusters& C);
// the `hubs` most popular source rows; sets of about rows_per_set consecutive rows
HotSets hot_sets_from_hubs(const gp_plan& P, int32_t hubs, int64_t rows_per_set);

// The plan's segments cut into records that gather from hot rows and records that gather
// from the others (cold), with a column list reordered to match (gp_cluster.cpp).
struct SplitSchedule {
    std::vector<int32_t> col;
    std::vector<Segment> hot, cold;
    std::vector<SplitRow> split;
    int64_t num_slots = 0;
};
void build_split_schedule(const gp_plan& P, const HotSets& H, SplitSchedule& out);

// The hot non-zeros arranged for the LDS pass (gp_cluster.cpp builds it, gp_hot_lds.hip runs it):
// a list's rows are staged in LDS one strip of four fp32 columns at a time, and the hot
// parts of the segments of a set that gathers from it, 64 to a group (one per lane, longest
// first), are added up from there into planes: plane t holds, for every position (a
// segment's place in the pass's own order), the four sums of strip t.  The segment kernel
// then takes the segments' other non-zeros in position order and adds the plane entries.
constexpr int kLdsGroupCostSteps = 12;  // a group's end costs a wave about as much as this many steps (config 3, hubs: 487 -> 447 us with 8 .. 32)
constexpr int kWaveCuts = 16;  // runs a set's groups are cut into (one per wave of a 1024-thread workgroup, two per wave of a 512-thread one)
constexpr uint8_t kAddPlaneEntry = 0x80;  // in a record's slice byte (implicit lists): add the plane entry of the record's list position
constexpr int kLdsBytesPerCu = 160 * 1024;
constexpr int kLdsMaxMembers = 10192;  // (rows rounded up to 16, + 16 zero rows) x 16 bytes and a few words must fit the LDS
struct LdsGroup {
    int64_t id_off;     // first of its steps x 64 places; 8 consecutive steps of a lane lie together
    int64_t first_pos;  // lane l fills the plane entries of position first_pos + l, l < count
    int32_t steps;      // multiple of 8; shorter segments are padded with reads of zero rows
    int32_t count;      // lanes that have a segment (the others read zero rows only)
};
// One work unit of the pass: eight consecutive strips (an octet) of one set.
struct LdsOctet {
    int32_t set, octet;
};
struct LdsSchedule {
    std::vector<int32_t> col;         // the column list, every segment's hot non-zeros first
    std::vector<Segment> cold;        // every segment's other non-zeros, in position order; slice = kAddPlaneEntry where it has hot ones
    std::vector<int32_t> members;     // rows of list l, ascending: members[member_off[l] .. member_off[l+1])
    std::vector<int64_t> member_off;  // num_lists + 1
    std::vector<int32_t> list_of_set; // num_sets
    std::vector<int32_t> group_off;   // num_sets + 1: groups of set c
    std::vector<int32_t> wave_cut;    // kWaveCuts + 1 per set: its groups cut into runs of about equal cost (reads plus kLdsGroupCostSteps steps per group)
    std::vector<LdsGroup> groups;     // and a sentinel whose id_off is the length of ids
    std::vector<int64_t> set_reads;   // per set: reads of its groups, padding included
    std::vector<uint16_t> ids;
    int32_t max_members = 0;  // longest list that hot non-zeros gather from
    int64_t hot_edges = 0;
    bool conflict_free = false;  // reads ordered so that the lanes of one LDS pass hit different banks
};
// Rows a strip occupies in LDS for a cluster of m rows: the rows, rounded up to 16, and 16 zero
// rows (one per bank group) that padding reads point at.
// Measured on config 4 (4,660-row clusters, rows of 441 hot non-zeros): reads in column-list order
// come out of LDS at 46.7 TB/s, in conflict-free order at 89 TB/s, and the same rows out of the L2s
// (per-XCD lists) at 22.9 TB/s; rows that miss the L2s arrive at about 7 TB/s.
constexpr double kLdsConflictFreeGain = 1.9;
constexpr double kLdsMaxCostClusters = 1.8;  // reads (in column-list-order equivalents) per hot non-zero beyond which the L2 lists are as fast
constexpr double kLdsMaxCostHubs = 4.0;      // ... beyond which gathering the hubs from memory is as fast
constexpr double kLdsForcedCost = 64.0;      // the limit when the pass is forced: whatever the padding
constexpr int32_t kHubMinHot = 3;  // hubs: non-zeros on the list a segment needs for them to go through LDS (measured on config 3: 3 .. 5 is best)
constexpr int64_t kLdsMinReadsPerSet = 100000;  // reads a set must have on average for a strip's staging (~9 us per work item) to pay
inline int64_t lds_rows(int64_t m) { return (m + 15) / 16 * 16 + 16; }
// false (and `out` unspecified) where the pass does not apply: a list that hot records gather
// from is too long for the LDS, or the reads (padding included; a read of the conflict-free
// order counts 1 / kLdsConflictFreeGain) exceed max_cost per hot non-zero.
// order: 1 = the column list's; 0 / 2 = conflict-free as far as the same number of steps allows.
// gp_device_sort.hip: device-wide radix sort (ascending) and duplicate removal of at most 2^31 - 1 64-bit keys.
// low_bits / high_bits: how many bits of the key's low and high word can differ between keys (the others are
// equal in all keys, or zero).  `other` is a second buffer of `count` keys; *sorted comes back as the one of the
// two that holds the result.  scratch: device_sort_scratch_words(count) 32-bit words on the device.
// device_unique_keys writes the distinct keys of a sorted list to `out` (not the list itself) and leaves their
// number in a word of the scratch, *total (DEVICE).
size_t device_sort_scratch_words(int64_t count);
// exclusive prefix sums of a[0 .. N) in place (32-bit, DEVICE); sums: device_scan_scratch_words(N) words of scratch
size_t device_scan_scratch_words(int64_t N);
gp_status device_exclusive_scan(uint32_t* a, int64_t N, uint32_t* sums, hipStream_t stream);
gp_status device_sort_keys(uint64_t* keys, uint64_t* other, int64_t count, int low_bits, int high_bits, uint32_t* scratch,
                           hipStream_t stream, uint64_t** sorted);
gp_status device_unique_keys(const uint64_t* sorted, uint64_t* out, int64_t count, uint32_t* scratch, hipStream_t stream,
                             const uint32_t** total);
bool build_lds_schedule(const gp_plan& P, const HotSets& H, double max_cost, int order, LdsSchedule& out);
// The (set, octet) pairs of a launch over rows of `strips` strips, dealt to the 8 XCDs: set by set, every
// octet to the XCD with the least work so far (work = the set's reads times the octet's strips), so that the
// strips of a set run on all XCDs at about the same time, each XCD streaming the set's index list for a few
// octets at once.
void deal_lds_octets(const std::vector<int64_t>& set_reads, int strips, std::vector<LdsOctet>& octets, int64_t (&off)[9]);
struct HotLdsArgs {
    // DEVICE arrays of the schedule
    const int32_t* members;
    const int64_t* member_off;
    const int32_t* list_of_set;
    const int32_t* group_off;
    const int32_t* wave_cut;
    const LdsGroup* groups;
    const LdsOctet* octets;   // DEVICE
    const int64_t* octet_off; // HOST, 9 entries: XCD x takes octets [octet_off[x], octet_off[x+1])
    const uint16_t* ids;
    int32_t num_sets, max_members;
    const float* src_scale;  // DEVICE n weights applied to source rows, or nullptr
    const void* xin;         // DEVICE rows of `dtype` (bf16 rows: d a multiple of 4)
    gp_dtype dtype;
    int64_t ldin;
    float* planes;           // DEVICE ceil(d / 32) x num_pos x 32 floats; the four sums of strip t at position p lie at
                             // ((t >> plane_log2) * num_pos + p) * (4 << plane_log2) + (t & ((1 << plane_log2) - 1)) * 4
    int64_t num_pos;
    int plane_log2 = 3;      // 0 .. 3: 2^plane_log2 strips of a position lie together
    float* packed;           // DEVICE scratch, ceil(d / 4) x num_members x 4 floats: the lists' rows strip by strip;
                             // nullptr: strips are staged straight from xin
    int64_t num_members;     // rows on all lists together
    int32_t d;
    unsigned long long* ctrl;  // as HopArgs::ctrl
};
// Once per device and list length, before the first launch_hot_lds (not a stream operation: kept out of the
// launch so that a launch can be captured in a graph): clears the kernel for the LDS it will ask for.
gp_status prepare_hot_lds(int32_t max_members);
gp_status launch_pack_strips(const HotLdsArgs& a, hipStream_t stream);  // fills a.packed (where the lists are shared)
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
    // optional plane entries (vectors of 4 columns, or of 8 bf16 columns with d a multiple of 4; implicit lists): a
    // record whose slice byte is kAddPlaneEntry adds, to the four columns of strip t, planes[((t >> plane_log2) * num_pos + p)
    // * (4 << plane_log2) + (t & ((1 << plane_log2) - 1)) * 4 ..], p being its place in segs
    const float* planes = nullptr;
    int64_t num_pos = 0;
    int plane_log2 = 3;
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
