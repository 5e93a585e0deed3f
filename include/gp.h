/* gp.h -- C boundary of the K-hop graph feature precompute for MI355X (gfx950).
 *
 * The library computes the hop stack [X, A^ X, ..., A^^K X] that a
 * precomputation-based / linear-convolution GNN trains on (paper Section 3.2,
 * Algorithm 1 "Block-wise feature aggregation"; the k = 0 term is the one the
 * Appendix A model consumes), where A^ is a constant linear aggregation
 * operator over the graph's adjacency list:
 *
 *   GP_AGG_SYM   A^ = D~^-1/2 A~ D~^-1/2      (Eq. 1, the normalised adjacency;
 *                                             D~ = row sums of the listed 0/1 matrix)
 *   GP_AGG_MEAN  A^ = D^-1 A                   (row-normalised mean)
 *   GP_AGG_SUM   A^ = A                        (plain sum; diagonal as listed)
 *
 * The adjacency list is first decomposed into disjoint, balanced edge blocks
 * whose union is the whole list (Section 3.2, "Precomputation on GPU": the sets
 * E^(1..a) and the identity S = sum_l D~^-1/2 A~^(l) D~^-1/2); every hop is run
 * block by block and rows cut by a block boundary are completed by a fixed-order
 * sum of partial rows (Algorithm 1, the accumulation over j).
 *
 * All entry points are plain C.  Every pointer argument says whether it is a
 * HOST or a DEVICE pointer.  No call aborts or throws; each returns a gp_status
 * and leaves a message for gp_last_error().  One GPU; the current HIP device at
 * the time of the first gp_propagate on a plan is the plan's device.
 */
#ifndef GP_H
#define GP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gp_plan gp_plan; /* opaque; owned by the library */

typedef enum {
    GP_OK = 0,
    GP_ERR_INVALID_ARG = 1,  /* null pointer, negative size, ld < d, unknown enum/flag, device and host operands mixed */
    GP_ERR_INDEX_RANGE = 2,  /* a node id outside [0, n) */
    GP_ERR_OVERFLOW = 3,     /* a count does not fit the type the layout stores it in */
    GP_ERR_OOM_HOST = 4,
    GP_ERR_OOM_DEVICE = 5,
    GP_ERR_DEVICE = 6,       /* a HIP call failed, or no usable device */
    GP_ERR_UNSUPPORTED = 7
} gp_status;

typedef enum { GP_AGG_SYM = 0, GP_AGG_MEAN = 1, GP_AGG_SUM = 2 } gp_agg;
typedef enum { GP_F32 = 0, GP_BF16 = 1 } gp_dtype;

/* plan flags */
enum { GP_SYMMETRISE = 1u, GP_ADD_SELF_LOOPS = 2u, GP_PLAN_ON_DEVICE = 4u };

/* ---------------------------------------------------------------------------
 * gp_plan_blocks -- edge decomposition and normalisation vectors.
 * (Section 3.2: decomposition of the edge set into disjoint balanced sets;
 *  Eq. 1 / the block-sum identity for the degree vectors; Eq. 11 for the block
 *  count, which has one free parameter and is the smallest count within budget.)
 *
 *  src, dst  HOST, m int32 each.  Pair (src = j, dst = i) means "i aggregates
 *            from j": non-zero (row i, col j).  Read only during the call.
 *  m         number of input pairs, >= 0.
 *  n         number of nodes, 1 .. 2^31-1.
 *  block_budget_edges  largest number of non-zeros one block may hold, > 0.
 *  flags     GP_SYMMETRISE also inserts (row j, col i); GP_ADD_SELF_LOOPS
 *            inserts (i, i) for every i.  GP_PLAN_ON_DEVICE sorts and de-duplicates
 *            the non-zeros and computes the degree and normalisation vectors on the
 *            current GPU instead of on the host threads (same plan, bit for bit;
 *            needs a GPU).  The entries are sorted in row ranges of at most
 *            2^31 - 1 candidates each (option "device_plan_chunk" lowers that), so
 *            only a single row with more candidates than that is GP_ERR_UNSUPPORTED.
 *            The column list and the norm vectors then stay on that GPU, which is
 *            the plan's device from then on: the first gp_propagate sends only the
 *            kernel schedule.
 *  out_plan  HOST; receives the plan (NULL on error).  Free with gp_plan_destroy.
 *
 * The non-zeros form a SET: duplicate pairs collapse, input pairs with
 * src == dst are dropped (the diagonal is exactly the self-loop flag).  They
 * are listed in ascending (row, col) order; with nnz of them,
 * b = max(1, ceil(nnz / budget)) and block p is the contiguous range
 * [p*q + min(p,r), (p+1)*q + min(p+1,r)), q = nnz div b, r = nnz mod b, so
 * block sizes differ by at most one.  deg[i] = number of non-zeros in row i.
 * dinv_sqrt[i] = (float)(1/sqrt((double)deg)), dinv[i] = (float)(1/(double)deg),
 * both 0 where deg = 0.  Runs on the host only (no GPU needed) unless
 * GP_PLAN_ON_DEVICE is set.
 * Errors: INVALID_ARG, INDEX_RANGE, OVERFLOW, OOM_HOST.
 */
gp_status gp_plan_blocks(const int32_t *src, const int32_t *dst, int64_t m, int64_t n,
                         int64_t block_budget_edges, uint32_t flags, gp_plan **out_plan);

void gp_plan_destroy(gp_plan *plan); /* NULL is allowed; frees host and device memory of the plan */

/* Accessors.  Returned HOST pointers stay valid until gp_plan_destroy.  A NULL
 * plan gives 0 / NULL. */
int64_t gp_plan_num_nodes(const gp_plan *plan);
int64_t gp_plan_nnz(const gp_plan *plan);
int32_t gp_plan_num_blocks(const gp_plan *plan);
const int64_t *gp_plan_block_offsets(const gp_plan *plan); /* b+1: block p = [off[p], off[p+1]) */
const int32_t *gp_plan_block_row_lo(const gp_plan *plan);  /* b: row of the block's first non-zero (0 if empty) */
const int32_t *gp_plan_block_row_hi(const gp_plan *plan);  /* b: row of its last non-zero (-1 if empty) */
const int64_t *gp_plan_rowptr(const gp_plan *plan);        /* n+1 */
const int32_t *gp_plan_col(const gp_plan *plan);           /* nnz, ascending (row, col) */
const int32_t *gp_plan_degree(const gp_plan *plan);        /* n */
const float *gp_plan_dinv_sqrt(const gp_plan *plan);       /* n */
const float *gp_plan_dinv(const gp_plan *plan);            /* n */

/* Kernel schedule of the plan (library's own work decomposition, exposed so host
 * logic can be checked without a GPU).  Every block is cut into segments: runs
 * of consecutive non-zeros of one row, at most "segment_edges" long, never
 * crossing a block boundary; a row without non-zeros has one segment of length
 * 0.  A row made of one segment is written directly; a row cut into several has
 * consecutive partial-row slots, in list order, that are summed afterwards.
 * Segment record, 16 bytes: { uint32 start_lo; uint8 start_hi; uint8 slice; uint16 len;
 * int32 row; int32 slot (-1 = whole row) }, start = start_hi << 32 | start_lo (40 bits);
 * slice is 0 in this list and names a column slice in gp_plan_work_lists' records. */
int64_t gp_plan_num_segments(const gp_plan *plan);
const void *gp_plan_segments(const gp_plan *plan);            /* num_segments records, grouped by block */
const int64_t *gp_plan_segment_offsets(const gp_plan *plan);  /* b+1: block p owns [off[p], off[p+1]) */
int64_t gp_plan_num_partial_rows(const gp_plan *plan);        /* number of slots */
int64_t gp_plan_segment_edges(const gp_plan *plan);           /* the segment length limit this plan used */

/* Cache schedule of the device-resident hops (library's own; exposed so host logic
 * can be checked without a GPU).  The paper's decomposition is agnostic on nodes
 * (Section 3.2, Limitation paragraph); the order in which destination rows are
 * processed does not change the result, only how often a gathered feature row is still
 * in the cache of the part of the chip that asks for it.  Algorithm 1's two cuts --
 * column blocks and edge blocks -- are re-used here as that order.
 *
 * gp_plan_row_clusters: rows grouped by synchronous label propagation over the
 * non-zero pattern (every row takes the most frequent label among its sources, ties to
 * the smallest label, until few rows change; deterministic).  label: HOST, n ints or
 * NULL; clusters are numbered 0 .. *num_clusters-1.  *inside_fraction = share of the
 * non-zeros whose source lies in the row's own cluster; *typical_rows = rows in the
 * cluster of a typical non-zero.  Computed on first use and kept with the plan.
 *
 * gp_plan_work_lists: the explicit work lists a hop over rows of d elements of `dtype`,
 * gathered in vectors of `vec` elements, would walk: *num_slices column slices of
 * *slice_elems elements (the last one narrower), and for each of the GPU's 8 XCDs the
 * records [xcd_off[x], xcd_off[x+1]) -- the plan's segments, each with the column slice
 * it is for, listed cluster by cluster.  Every (segment, slice) pair appears exactly
 * once over the 8 lists.  *num_slices = 0 means this plan keeps the implicit lists
 * (XCD x takes slice x mod S of every segment): its rows do not gather mostly from
 * their own cluster, or no slice of at least 128 bytes makes a cluster's rows fit the
 * share of a 4 MB L2 the schedule counts on.  xcd_off: HOST, 9 entries.  records:
 * HOST, room for `capacity` 16-byte records, or NULL to get the counts only.
 * Errors: INVALID_ARG, OOM_HOST. */
/* gp_plan_lds_schedule: the schedule of the LDS pass (library's own; exposed so host logic
 * can be checked without a GPU).  Hops over fp32 rows, and over bf16 rows of a multiple of
 * four columns, take the non-zeros whose source row is on a short list of rows (the hot
 * ones) from the compute units' LDS: a workgroup stages four feature columns (as fp32, 16 bytes) of the list's rows, scaled by the operator's source weight,
 * and one lane per segment adds up the segment's hot sources from there, leaving the four
 * sums in a plane entry; the segment kernel then gathers the segments' other non-zeros from
 * memory, adds the plane entries and finishes every segment as the plan says (output row,
 * or partial-row slot).  Lists have at most 10192 rows.  Rows are grouped into sets; a set
 * gathers from one list.  hot_mode 1: the plan has row clusters (gp_plan_row_clusters) whose
 * typical size an L2 could hold, and sets = lists = clusters, a row's hot non-zeros being
 * those with the source in the row's own cluster.  hot_mode 2: it has none, but the 10192
 * rows that are most often a source account for at least 15 % of the non-zeros (and non-zeros
 * times d is at least 2e9: below that the pass's launches cost more than they save): they are
 * the one list, every set (a range of consecutive
 * rows; about 2048 / strips of them) gathers from it; a segment with fewer than three
 * sources on the list keeps them among its other non-zeros (handing a segment's sums from
 * one launch to the other costs about two gathers).
 * The pass takes the plan's segments in an order of its own: set by set, inside a set most
 * hot non-zeros first.  A segment's place in that order is its position p; rest[p] is the
 * segment's record (gp_plan_segments' format) reduced to its other non-zeros, which are
 * col[start .. start + len) of a column list that has every segment's hot non-zeros moved
 * to the front of the segment (both parts keep their order); its slice byte is 0x80 where
 * the segment has hot non-zeros that the pass takes.  64 consecutive positions of a set form a group; lane l of
 * group g fills the plane entries of position rec_pos[64 g + l] (-1: none: past the set's
 * end, or a segment without hot non-zeros).  Every lane of a group walks group_steps[g] (a
 * multiple of 8) reads; read t of lane l is ids[group_id_off[g] + (t / 8) * 512 + l * 8 +
 * t % 8]: the place of the source row on the set's list (list l = members[member_off[l] ..
 * member_off[l+1]), ascending), or, for padding, one of 16 zero rows that follow the list
 * from the next multiple of 16.  Every group walks as many steps as its longest segment
 * has reads, rounded up to 8.  order 2 (and order 0) arranges a group's reads inside those
 * steps so that the 16 lanes the LDS serves together -- lanes {0-3, 12-15, 20-27} and
 * {4-11, 16-19, 28-31} of each half of a wavefront on gfx950 -- read 16 different residues
 * of the place mod 16 at every step, i.e. do not collide on a bank, as far as that can be:
 * where a residue has more reads among the 16 segments than there are steps, the surplus
 * takes padding slots of its own segments and meets one other read there.  order 1 keeps
 * the column list's order (about 2.5 collisions per step).  With order 0 the pass applies
 * only where the reads (padding included; a read of order 2 counting 1 / 1.9)
 * stay below 1.8 per hot non-zero for clusters and 4 for hubs: beyond that the same rows
 * are as fast out of the L2s, or memory, and where a set has at least 100000 reads on
 * average (staging a strip costs the same whatever is read from it).  d (>= 4) is the column count the sets of
 * hot_mode 2 are sized for.
 * The call fills the counts of *view (num_groups = 0: the pass does not apply to this
 * plan) and every array of *view that is not NULL (HOST memory; capacities in elements,
 * set_capacity covering list_of_set and member_off, position_capacity covering rest and,
 * if asked for, col with its nnz entries).  What a plan calls hot is decided once, by this
 * call or by the first gp_propagate.
 * Errors: INVALID_ARG, OOM_HOST. */
typedef struct gp_lds_view {
    int64_t num_groups, num_ids, num_members, num_positions; /* out */
    int32_t num_sets, num_lists, conflict_free, hot_mode;    /* out */
    int64_t group_capacity, id_capacity, set_capacity, member_capacity, position_capacity; /* in */
    int32_t *group_set;      /* per group: its set */
    int64_t *group_id_off;   /* per group */
    int32_t *group_steps;    /* per group */
    int32_t *rec_pos;        /* 64 per group */
    uint16_t *ids;           /* num_ids */
    int32_t *list_of_set;    /* num_sets */
    int64_t *member_off;     /* num_lists + 1 */
    int32_t *members;        /* num_members */
    void *rest;              /* num_positions 16-byte records */
    int32_t *col;            /* nnz */
} gp_lds_view;
gp_status gp_plan_lds_schedule(const gp_plan *plan, int32_t d, int32_t order, gp_lds_view *view);
gp_status gp_plan_row_clusters(const gp_plan *plan, int32_t *label, int32_t *num_clusters,
                               double *inside_fraction, double *typical_rows);
gp_status gp_plan_work_lists(const gp_plan *plan, int32_t d, gp_dtype dtype, int32_t vec, int32_t *num_slices,
                             int32_t *slice_elems, int64_t *xcd_off, void *records, int64_t capacity);

/* ---------------------------------------------------------------------------
 * gp_propagate -- the hop stack (Algorithm 1's SX_list plus slot 0 = X).
 *
 *  plan      from gp_plan_blocks.
 *  X         n x d row-major, leading dimension ldx elements (ldx >= d), of
 *            `dtype`.  DEVICE pointer, or HOST pointer (then out_stack must be host
 *            memory too and the streamed schedule is used).  Host memory should be
 *            PINNED: the link then runs at its rate.  Ordinary (pageable) host
 *            memory is accepted when ldx = ldo = d and the HBM budget holds whole
 *            rows (GP_ERR_UNSUPPORTED otherwise): it moves through a ring of pinned
 *            buffers (512 MiB, kept with the plan) filled and emptied by host
 *            threads of the library.  It is the way to run operands larger than
 *            the pinned memory a machine grants.
 *  d         feature columns, >= 1.
 *  dtype     GP_F32, or GP_BF16 storage (accumulation is always fp32; a stored
 *            bf16 value is the fp32 accumulator rounded to nearest even).
 *  agg       the operator, see above.
 *  K         hops, >= 0 (0 writes slot 0 only).
 *  out_stack K+1 slabs of n x d, leading dimension ldo (>= d); slab k starts at
 *            element k*n*ldo and receives A^^k X.  Same memory kind as X.  X may
 *            be exactly slab 0 (then ldx must equal ldo and no copy is made);
 *            any other overlap is an error the library does not detect.
 *  hip_stream  a hipStream_t, or NULL for the default stream.
 *
 * Device-resident operands: the call enqueues all work on hip_stream and
 * returns; the caller synchronises.  Pinned-host operands: blocks and column
 * slabs are streamed through HBM on library-owned side streams and the call
 * returns after the last slab has reached out_stack (streams, events and staging
 * buffers are kept with the plan and reused by later calls of the same shape; edge
 * blocks that all fit the budget are sent once per plan).  The first call on a plan
 * uploads the plan to the current device and allocates scratch (partial-row
 * buffer); later calls with the same d reuse both.  Calls on ONE plan must not
 * overlap in time (they share that scratch); different plans are independent.
 * Results are deterministic: the same inputs and options give the same bits on every
 * call (how a row's partial sums are grouped depends on the schedule, so the streamed and
 * the resident schedule, or two settings of "split_records", "lds_pass" or "hub_pass", may differ
 * in the last bits).
 * Errors: INVALID_ARG, OOM_DEVICE, DEVICE, UNSUPPORTED.
 */
gp_status gp_propagate(const gp_plan *plan, const void *X, int64_t ldx, int32_t d, gp_dtype dtype,
                       gp_agg agg, int32_t K, void *out_stack, int64_t ldo, void *hip_stream);

/* gp_plan_streamed_shape -- the decomposition the last streamed gp_propagate on this
 * plan ran with (Section 3.2, "Optimal graph decomposition", Eq. 12): *edge_blocks = b,
 * *column_blocks = c; both 0 before any streamed call.  The library takes
 *     B_S = 4 nnz + 16 segments            (column ids and segment records, bytes)
 *     B_X = (2 n s + 4 partial_rows) d     (two column slabs and the partial rows; s = element bytes)
 *     B_GPU = HBM budget - (8 n + 16 partial_rows + 4096)
 * and the pair (b*, c*) = gp_solve_aggregation_blocks(B_S, B_X, B_GPU, 2, 1, ceil(d / (16/s))):
 * two edge-block buffers of B_S / b, column slabs of ceil(d / c) columns rounded up to whole
 * 16-byte vectors.  If the plan already has at least b* blocks they are used as they are
 * (and the slabs are made as wide as then fits, so c <= c*); otherwise the sorted list is
 * cut anew into b* balanced blocks -- the planner's rule, another count -- with segments
 * and partial rows of their own (one more block at a time, should the cut's own
 * book-keeping exceed the estimate), and c = c*, or the next c whose slab of whole
 * 16-byte column groups fits (Eq. 12 divides B_X evenly; a slab cannot). */
gp_status gp_plan_streamed_shape(const gp_plan *plan, int64_t *edge_blocks, int64_t *column_blocks);

/* ---------------------------------------------------------------------------
 * gp_propagate_noalloc -- gp_propagate for callers that cannot allocate: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and same kernels as gp_propagate on device-resident operands, and the same
 * bits in out_stack whenever both calls take the same schedule -- whole records (option
 * "split_records" = 2, or a graph without row clusters or popular rows worth a pass), or the
 * LDS pass with what an earlier gp_propagate on the plan has built for it; else a row's
 * partial sums are grouped differently and the two agree to rounding -- but the call makes
 * no allocation of any kind: the scratch
 * the kernels need (work cursors, partial rows of rows that were cut) is a fixed array
 * in device memory of 64 MiB + 256 bytes that each GPU the library is used on holds
 * until the process ends.
 *
 *  plan   must already be on the current device (the first gp_propagate on a plan
 *         uploads it); else GP_ERR_INVALID_ARG.  What earlier calls built is used (work
 *         lists, per-edge weights, the LDS pass's schedule and planes for rows of as many
 *         columns); what they did not build is done without (implicit lists, weights
 *         gathered by column id -- the same numbers).
 *  X, out_stack  DEVICE only (pinned-host operands: GP_ERR_INVALID_ARG).
 *
 * Limit: plan partial rows x round_up(d, 4) x 4 bytes <= gp_noalloc_partial_row_bytes()
 * (64 MiB), else GP_ERR_UNSUPPORTED with the sizes in gp_last_error().  All calls on one
 * GPU share that GPU's array: calls that overlap in time on one GPU race (also with
 * different plans or streams).  Enqueued on hip_stream; nothing in it is a memset, so the
 * call may be captured.  Errors: INVALID_ARG, UNSUPPORTED, DEVICE.
 */
gp_status gp_propagate_noalloc(const gp_plan *plan, const void *X, int64_t ldx, int32_t d, gp_dtype dtype,
                               gp_agg agg, int32_t K, void *out_stack, int64_t ldo, void *hip_stream);
int64_t gp_noalloc_partial_row_bytes(void);

/* ---------------------------------------------------------------------------
 * gp_propagate_combine -- a constant polynomial graph filter without the stack:
 *     out = sum_{k=0..K} coeff[k] * A^^k X.
 * (Appendix A, Eq. 13: the generalized-PageRank propagation sum_k gamma_k S^k H
 *  with constant gamma; with coeff[k] = alpha (1-alpha)^k for k < K and
 *  (1-alpha)^K for k = K it is the K-step Personalized-PageRank diffusion that the
 *  Limitation paragraph of Section 3.1 names as another precomputable filter.)
 *
 *  coeff  HOST, K+1 floats, read during the call.
 *  out    DEVICE, n x d of `dtype`, leading dimension ldo; must not overlap X.
 *  X      DEVICE (pinned-host operands: GP_ERR_UNSUPPORTED).
 * Hops are chained as in gp_propagate (each hop consumes the previous hop as
 * stored in `dtype`); every term is added in fp32 from the fp32 accumulator of
 * its hop, and bf16 output is rounded once at the end.  Two n x d slabs (and,
 * for bf16, an n x d fp32 accumulator) are allocated on first use and kept with
 * the plan.  Enqueued on hip_stream; deterministic.  Other arguments and errors
 * as gp_propagate.
 */
gp_status gp_propagate_combine(const gp_plan *plan, const void *X, int64_t ldx, int32_t d, gp_dtype dtype,
                               gp_agg agg, int32_t K, const float *coeff, void *out, int64_t ldo,
                               void *hip_stream);

/* ---------------------------------------------------------------------------
 * gp_lc_forward -- forward pass of an LC-version model over a mini-batch of the
 * hop stack (Appendix A, the LC version of GPRGNN:
 *     H[i] = sum_{k=0..K} gamma[k] * MLP(X_k[batch[i]]),
 *     MLP(Z) = relu(... relu(Z W_1) ... W_{T-1}) W_T,
 *  the T weight matrices shared by all hops, no bias terms; with gamma = e_K it is
 *  the single-branch H^LC of Section 3.1, the LC version of a GCN).  The softmax
 *  the paper puts on top is gp_lc_softmax.
 *
 *  stack   DEVICE, K+1 slabs of n x d as gp_propagate writes them: slab k starts at
 *          element k*n*ld, rows ld elements apart (ld >= d), of `dtype` (bf16 is
 *          widened exactly; all arithmetic is fp32 on the matrix cores).
 *  batch   DEVICE, B row numbers; NULL means rows 0 .. B-1 (then B <= n).  A row
 *          number outside [0, n) is not an error: that output row is computed
 *          from a row of zeros.
 *  gamma   HOST, K+1 floats, read during the call.  0 <= K <= 15.
 *  T       layers, 1 .. 8.  W: HOST array of T DEVICE pointers; W[t] is dense
 *          row-major in_t x width[t], in_0 = d, in_t = width[t-1].  width: HOST,
 *          T ints, each 1 .. 256 (others: GP_ERR_UNSUPPORTED).
 *  out     DEVICE, B x width[T-1] fp32, rows ldo floats apart; must not overlap
 *          the inputs.
 *
 * Enqueued on hip_stream; deterministic.  With K >= 1 the per-hop results pass
 * through a library-owned buffer per device (at most 256 MiB, grown on demand),
 * so calls on one device must not overlap in time.  Growing that buffer is the
 * only allocation: after a call with at least as many rows and output columns,
 * a call enqueues kernels only and may be captured in a HIP graph.
 * Errors: INVALID_ARG, UNSUPPORTED, OOM_DEVICE, DEVICE.
 */
gp_status gp_lc_forward(const void *stack, int64_t ld, gp_dtype dtype, int64_t n, int32_t d, int32_t K,
                        const int32_t *batch, int64_t B, const float *gamma, int32_t T,
                        const float *const *W, const int32_t *width, float *out, int64_t ldo,
                        void *hip_stream);

/* ---------------------------------------------------------------------------
 * gp_lc_forward_branches -- the general H^LC of Section 3.1 (the LC version of
 * JKNet): one branch per hop, of its own depth, combined by COMB:
 *     branch_k = relu(... relu(X_k[batch] W_1) ... W_{depth[k]-1}) W_{depth[k]},
 *     H        = COMB_k(gamma[k] * branch_k).
 * The paper's formula is depth[k] = k for k = 1..K (hop 0 left out) with COMB =
 * concatenation or max pooling; depth[k] = T for every k with GP_COMB_SUM is
 * gp_lc_forward.
 *
 *  depth   HOST, K+1 ints in 0 .. T; 0 leaves hop k out; at least one non-zero.
 *  comb    GP_COMB_SUM / GP_COMB_MAX: all branches must end in the same width
 *          (INVALID_ARG otherwise), out is B x that width;
 *          GP_COMB_CONCAT: out is B x (sum of the branches' widths), branches side
 *          by side in hop order.
 * Everything else as gp_lc_forward (concatenation writes the result directly and
 * needs no library buffer).
 */
typedef enum { GP_COMB_SUM = 0, GP_COMB_CONCAT = 1, GP_COMB_MAX = 2 } gp_comb;
gp_status gp_lc_forward_branches(const void *stack, int64_t ld, gp_dtype dtype, int64_t n, int32_t d, int32_t K,
                                 const int32_t *batch, int64_t B, const float *gamma, const int32_t *depth,
                                 gp_comb comb, int32_t T, const float *const *W, const int32_t *width,
                                 float *out, int64_t ldo, void *hip_stream);

/* gp_lc_softmax -- Y = softmax(H) row by row, in place (Section 3.1: the predicted
 * label matrix Y = softmax(H^LC)).  H: DEVICE, B x C fp32, rows ld floats apart
 * (ld >= C).  fp32 arithmetic, row maximum subtracted before exp.  Enqueued on
 * hip_stream.  Errors: INVALID_ARG, DEVICE. */
gp_status gp_lc_softmax(float *H, int64_t B, int32_t C, int64_t ld, void *hip_stream);

/* ---------------------------------------------------------------------------
 * Optimal graph decomposition (Section 3.2, Eq. 11 and Eq. 12): block counts
 * from byte volumes, the available GPU volume and the environment's coefficients
 * (all in the same unit, e.g. bytes or GB; coefficients are measured by watching
 * memory use on small graphs).  Host only.
 *
 * gp_solve_normalisation_blocks: the smallest natural a with
 *     (alpha_A*B_A + alpha_S*B_S) / a + alpha_D*B_D <= B_GPU.
 * gp_solve_aggregation_blocks: naturals (b, c), c <= max_c (a feature matrix has
 * only so many columns), minimising b*c subject to
 *     beta_S*B_S / b + beta_X*B_X / c <= B_GPU,
 * by exhaustive search; among equal products the pair with the smaller c wins
 * (the paper does not say; fewer column blocks means fewer re-sends of every
 * edge block).  Errors: INVALID_ARG (negative volume or coefficient, B_GPU <= 0,
 * max_c < 1, NULL output), UNSUPPORTED when no block count can satisfy the constraint (the
 * fixed term alone exceeds B_GPU, or max_c is too small).
 */
gp_status gp_solve_normalisation_blocks(double B_A, double B_S, double B_D, double B_GPU, double alpha_A,
                                        double alpha_S, double alpha_D, int64_t *a);
gp_status gp_solve_aggregation_blocks(double B_S, double B_X, double B_GPU, double beta_S, double beta_X,
                                      int64_t max_c, int64_t *b, int64_t *c);

/* ---------------------------------------------------------------------------
 * Library-wide knobs.  gp_set_option changes the process-wide defaults;
 * gp_plan_blocks copies them into the plan it makes, and every later call on that
 * plan uses the plan's copy ("lc_tile_rows" and the HBM budget, which belong to
 * calls without a plan or to the machine, are read when the call is made).
 */

/* Upper limit of HBM bytes the streamed schedule may use for its staging buffers
 * (the memory budget B_GPU of Eq. 12).  0 = choose from the device's free memory. */
gp_status gp_set_hbm_budget_bytes(int64_t bytes);

/* Named integer options; unknown names give INVALID_ARG.
 *   "segment_edges"   longest run of non-zeros one lane group walks before the row
 *                     is split into partial rows (8 .. 32768), or 0 (default):
 *                     chosen per plan as about nnz / 65536 within 64 .. 1024.  Read
 *                     by gp_plan_blocks.
 *   "column_tile"     feature columns per pass of the kernel, 0 = automatic.
 *   "persistent_blocks"  workgroups of the hop kernel (0 = as many as stay resident).
 *   "lc_tile_rows"       batch rows per work item of gp_lc_forward: 32 or 64 (0 = by batch size).
 *   "column_slices"   column slices one pass is divided into (1 .. 16; 0 = automatic).
 *                     Implicit work lists take 1, 2, 4 or 8 (anything else = automatic).
 *   "split_records"   explicit work lists: 0 / 1 = every record is cut into the non-zeros
 *                     whose source lies in the row's cluster and the others; the others are
 *                     gathered first, whole rows wide, in a launch of their own, and the two
 *                     partial rows are joined by the fix-up; 2 = whole records.
 *   "lds_pass"        0 = the non-zeros whose source is on a short list of rows are gathered from LDS
 *                     where gp_plan_lds_schedule has a schedule for the plan; 1 = the same, with
 *                     the conflict-free order whatever padding it costs; 3 = the same, with the
 *                     column list's order; 2 = never (per-XCD work lists through the L2s).
 *   "hub_pass"        plans without row clusters: 0 = the most popular rows are served from LDS
 *                     where they are the source of enough non-zeros (gp_plan_lds_schedule,
 *                     hot_mode 2), 1 = whenever the LDS pass applies, 2 = never.
 *   "hub_sets"        hot_mode 2: number of row sets the rows are cut into (1 .. 65536; 0 = about
 *                     2048 / strips, fewer where a set would have less than 100000 reads).
 *   "plane_strips"    LDS pass: how many strips' sums of one segment lie together in the buffer
 *                     the two launches of a hop share (1, 2, 4 or 8; 8 = one 128-byte line per
 *                     segment and eight strips: fewest lines touched by the launch that reads
 *                     them; 1 = a strip's sums of consecutive segments lie together: whole lines
 *                     for the launch that writes them).  0 = 8 with row clusters (long segments,
 *                     few stores), 4 with hubs (short segments: the stores weigh as much as the
 *                     reads).  The results do not depend on it.
 *   "device_plan_chunk"  GP_PLAN_ON_DEVICE: most candidate entries sorted at once
 *                     (1 .. 2^31 - 1; 0 = 2^31 - 1).  Read by gp_plan_blocks.
 *   "cache_schedule"  0 = explicit per-XCD work lists where the plan's row clusters
 *                     call for them (see gp_plan_work_lists), 1 = always, 2 = never.
 */
gp_status gp_set_option(const char *name, int64_t value);
int64_t gp_get_option(const char *name); /* -1 for an unknown name */

/* ---------------------------------------------------------------------------
 * Kernel timing for benchmarks: while enabled, every kernel launch made by
 * gp_propagate is bracketed by HIP events on the launch stream.
 * gp_profile_read synchronises those events and reports, for kernels whose name
 * starts with `prefix` ("" = all), the launch count and the summed duration.
 */
gp_status gp_profile_enable(int32_t on); /* also clears what was recorded */
gp_status gp_profile_read(const char *prefix, int64_t *launches, double *total_ms);

const char *gp_status_string(gp_status s);
const char *gp_last_error(void); /* thread-local text of the calling thread's last failure */

#ifdef __cplusplus
}
#endif
#endif /* GP_H */
