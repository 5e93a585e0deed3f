// Device side of gp_plan_blocks (flag GP_PLAN_ON_DEVICE): the non-zero set of the
// matrix being normalised, sorted and de-duplicated on the GPU, and the degree and
// normalisation vectors of Eq. 1 computed there.  The paper runs its adjacency
// normalisation block-wise on the GPU (Section 3.2, Section 4.2); here the
// normalisation needs no matrix at all, only the sorted set and its row counts, so the
// GPU's share is: count the candidate entries of every row, cut the rows into ranges
// whose candidates fit one sort, and per range emit one 64-bit key (row << 32 | col)
// per candidate, radix-sort the keys, drop duplicates, split them back into columns and
// find every row's first entry by binary search; then degrees, 1/sqrt(deg) and 1/deg
// (in fp64, narrowed once: the host planner's recipe) and the rows at the block
// boundaries.  Integers and correctly rounded operations only, so the result is the host
// planner's bit for bit.  The sort and the duplicate removal are gp_device_sort.hip's.
// The column list and the two norm vectors stay on the device for gp_propagate.
#include <hip/hip_runtime.h>

#include <cstring>

#include "gp_block_scan.h"
#include "gp_internal.h"

namespace gp {

namespace {

constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void gp_keys_to_columns(const uint64_t* __restrict__ keys, int64_t nnz,
                                                               int32_t* __restrict__ col)
{
    for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < nnz; e += (int64_t)gridDim.x * kThreads)
        col[e] = (int32_t)(keys[e] & 0xFFFFFFFFu);
}

// candidates of every row before duplicates collapse (cnt is preset to the self-loop count)
__global__ __launch_bounds__(kThreads) void gp_count_candidates(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                                                int64_t m, int sym, unsigned long long* __restrict__ cnt)
{
    for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < m; e += (int64_t)gridDim.x * kThreads) {
        const int32_t s = src[e], t = dst[e];
        if (s == t) continue;
        atomicAdd(cnt + t, 1ULL);
        if (sym) atomicAdd(cnt + s, 1ULL);
    }
}

__global__ __launch_bounds__(kThreads) void gp_fill_words(unsigned long long* __restrict__ p, int64_t count, unsigned long long v)
{
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < count; i += (int64_t)gridDim.x * kThreads) p[i] = v;
}

// Keys of the candidates whose row lies in [r0, r1).  Entry e of the edge list (e < m), or the self-loop of
// row r0 + (e - m), gives up to two keys.  Two passes over the entries, in tiles of kEmitTile consecutive ones:
// the first counts every tile's keys, an exclusive scan of the counts gives each tile its first slot, and the
// second writes the keys in entry order -- no cursor, no atomics, and the same order on every run.
constexpr int kEmitItems = 16;
constexpr int64_t kEmitTile = (int64_t)kThreads * kEmitItems;

__device__ inline int keys_of_entry(const int32_t* __restrict__ src, const int32_t* __restrict__ dst, int64_t m, int64_t span,
                                    int sym, int64_t r0, int64_t r1, int64_t e, uint64_t (&key)[2])
{
    if (e >= span) return 0;
    if (e >= m) {  // the self-loop of row r0 + (e - m)
        const uint64_t i = (uint64_t)(r0 + (e - m));
        key[0] = (i << 32) | i;
        return 1;
    }
    const uint32_t s = (uint32_t)src[e], t = (uint32_t)dst[e];
    if (s == t) return 0;
    int k = 0;
    if ((int64_t)t >= r0 && (int64_t)t < r1) key[k++] = ((uint64_t)t << 32) | s;
    if (sym && (int64_t)s >= r0 && (int64_t)s < r1) key[k++] = ((uint64_t)s << 32) | t;
    return k;
}

__global__ __launch_bounds__(kThreads) void gp_count_keys_range(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                                                int64_t m, int sym, int loops, int64_t r0, int64_t r1,
                                                                uint32_t* __restrict__ tile_count, int64_t tiles)
{
    __shared__ uint32_t ws[kScanWaves + 1];
    const int64_t span = m + (loops ? r1 - r0 : 0);
    const int64_t t0 = (int64_t)blockIdx.x * kEmitTile;
    uint32_t c = 0;
    uint64_t key[2];
    for (int j = 0; j < kEmitItems; ++j) c += (uint32_t)keys_of_entry(src, dst, m, span, sym, r0, r1, t0 + (int64_t)j * kThreads + threadIdx.x, key);
    uint32_t total;
    block_exclusive(c, ws, &total);
    if (threadIdx.x == 0) {
        tile_count[blockIdx.x] = total;
        if (blockIdx.x == 0) tile_count[tiles] = 0;  // the scan leaves the number of keys here
    }
}

__global__ __launch_bounds__(kThreads) void gp_emit_keys_range(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                                               int64_t m, int sym, int loops, int64_t r0, int64_t r1,
                                                               const uint32_t* __restrict__ tile_first, uint64_t* __restrict__ keys,
                                                               int64_t capacity)
{
    __shared__ uint32_t ws[kScanWaves + 1];
    const int64_t span = m + (loops ? r1 - r0 : 0);
    const int64_t t0 = (int64_t)blockIdx.x * kEmitTile;
    uint32_t run = tile_first[blockIdx.x];
    for (int j = 0; j < kEmitItems; ++j) {  // 256 consecutive entries per step, in order
        uint64_t key[2];
        const int c = keys_of_entry(src, dst, m, span, sym, r0, r1, t0 + (int64_t)j * kThreads + threadIdx.x, key);
        uint32_t total;
        const uint32_t at = run + block_exclusive((uint32_t)c, ws, &total);
        for (int k = 0; k < c; ++k)
            if ((int64_t)at + k < capacity) keys[at + k] = key[k];  // (the bound always holds: the buffer has one slot per candidate)
        run += total;
    }
}

// rowptr[i] = base + number of keys below (i << 32), i = r0 .. r1 (keys hold rows [r0, r1) only)
__global__ __launch_bounds__(kThreads) void gp_row_starts_range(const uint64_t* __restrict__ keys, int64_t count, int64_t r0,
                                                                int64_t r1, int64_t base, int64_t* __restrict__ rowptr)
{
    for (int64_t i = r0 + (int64_t)blockIdx.x * kThreads + threadIdx.x; i <= r1; i += (int64_t)gridDim.x * kThreads) {
        const uint64_t probe = (uint64_t)i << 32;
        int64_t lo = 0, hi = count;
        while (lo < hi) {
            const int64_t mid = lo + (hi - lo) / 2;
            if (keys[mid] < probe)
                lo = mid + 1;
            else
                hi = mid;
        }
        rowptr[i] = base + lo;
    }
}

// deg[i] = entries of row i; the norm vectors of Eq. 1: fp64 square root and division (both
// correctly rounded), narrowed once; 0 where the row is empty
__global__ __launch_bounds__(kThreads) void gp_degrees_and_norms(const int64_t* __restrict__ rowptr, int64_t n,
                                                                 int32_t* __restrict__ deg, float* __restrict__ dinv_sqrt,
                                                                 float* __restrict__ dinv)
{
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kThreads) {
        const int32_t g = (int32_t)(rowptr[i + 1] - rowptr[i]);
        deg[i] = g;
        dinv_sqrt[i] = g > 0 ? (float)(1.0 / sqrt((double)g)) : 0.0f;
        dinv[i] = g > 0 ? (float)(1.0 / (double)g) : 0.0f;
    }
}

// rows of the first and last entry of every block (0 and -1 for an empty block)
__global__ void gp_block_rows(const int64_t* __restrict__ rowptr, int64_t n, const int64_t* __restrict__ block_off, int32_t b,
                              int32_t* __restrict__ row_lo, int32_t* __restrict__ row_hi)
{
    const int32_t p = (int32_t)(blockIdx.x * blockDim.x + threadIdx.x);
    if (p >= b) return;
    const int64_t lo = block_off[p], hi = block_off[p + 1];
    int32_t rl = 0, rh = -1;
    if (hi > lo) {
        auto row_of = [&](int64_t e) {  // the i with rowptr[i] <= e < rowptr[i + 1]
            int64_t a = 0, z = n;       // invariant: rowptr[a] <= e, rowptr[z] > e
            while (z - a > 1) {
                const int64_t mid = a + (z - a) / 2;
                if (rowptr[mid] <= e)
                    a = mid;
                else
                    z = mid;
            }
            return (int32_t)a;
        };
        rl = row_of(lo);
        rh = row_of(hi - 1);
    }
    row_lo[p] = rl;
    row_hi[p] = rh;
}

inline unsigned grid_for(int64_t items) { return (unsigned)std::min<int64_t>((items + kThreads - 1) / kThreads, 256 * 32); }

struct DeviceBuffers {
    std::vector<void*> ptrs;
    ~DeviceBuffers()
    {
        for (void* p : ptrs) (void)hipFree(p);
    }
    template <class T>
    gp_status alloc(T*& p, size_t count)
    {
        p = nullptr;
        void* q = nullptr;
        GP_HIP(hipMalloc(&q, std::max<size_t>(count, 1) * sizeof(T)));
        ptrs.push_back(q);
        p = (T*)q;
        return GP_OK;
    }
};

}  // namespace

gp_status csr_on_device(const int32_t* src, const int32_t* dst, int64_t m, int64_t n, bool sym, bool loops, gp_plan* plan)
{
    hipStream_t stream = nullptr;
    DeviceBuffers B;
    int32_t *d_src, *d_dst;
    unsigned long long* d_cnt;
    int64_t* d_rowptr;
    gp_status st;
    if ((st = B.alloc(d_src, (size_t)m)) != GP_OK || (st = B.alloc(d_dst, (size_t)m)) != GP_OK ||
        (st = B.alloc(d_cnt, (size_t)n)) != GP_OK ||
        (st = B.alloc(d_rowptr, (size_t)n + 1)) != GP_OK)
        return st;
    // ---- candidates per row, and row ranges whose candidates fit one sort ------------
    hipLaunchKernelGGL(gp_fill_words, dim3(grid_for(n)), dim3(kThreads), 0, stream, d_cnt, n, loops ? 1ULL : 0ULL);
    GP_HIP(hipGetLastError());
    if (m) {
        GP_HIP(hipMemcpyAsync(d_src, src, (size_t)m * 4, hipMemcpyHostToDevice, stream));
        GP_HIP(hipMemcpyAsync(d_dst, dst, (size_t)m * 4, hipMemcpyHostToDevice, stream));
        hipLaunchKernelGGL(gp_count_candidates, dim3(grid_for(m)), dim3(kThreads), 0, stream, d_src, d_dst, m, sym ? 1 : 0, d_cnt);
        GP_HIP(hipGetLastError());
    }
    std::vector<unsigned long long> cnt((size_t)n);
    GP_HIP(hipMemcpyAsync(cnt.data(), d_cnt, (size_t)n * sizeof(unsigned long long), hipMemcpyDeviceToHost, stream));
    GP_HIP(hipStreamSynchronize(stream));
    int64_t limit = options().device_plan_chunk > 0 ? options().device_plan_chunk : (INT64_C(1) << 31) - 1;
    std::vector<int64_t> range_lo, range_cnt;  // row ranges [range_lo[k], range_lo[k+1]) and their candidate counts
    int64_t total = 0, largest = 0;
    {
        int64_t acc = 0;
        range_lo.push_back(0);
        for (int64_t i = 0; i < n; ++i) {
            const int64_t c = (int64_t)cnt[(size_t)i];
            if (c > (INT64_C(1) << 31) - 1)
                return fail(GP_ERR_UNSUPPORTED, "row %lld alone has %lld candidate entries: plan on the host", (long long)i, (long long)c);
            if (acc > 0 && acc + c > limit) {
                range_cnt.push_back(acc);
                range_lo.push_back(i);
                acc = 0;
            }
            acc += c;
            total += c;
        }
        range_cnt.push_back(acc);
        range_lo.push_back(n);
        for (int64_t c : range_cnt) largest = std::max(largest, c);
    }
    std::vector<unsigned long long>().swap(cnt);

    uint64_t *d_keys, *d_sorted;
    int32_t* d_col = nullptr;  // stays with the plan
    if ((st = B.alloc(d_keys, (size_t)largest)) != GP_OK || (st = B.alloc(d_sorted, (size_t)largest)) != GP_OK) return st;
    GP_HIP(hipMalloc((void**)&d_col, (size_t)std::max<int64_t>(total, 1) * sizeof(int32_t)));
    struct ColGuard {
        int32_t*& p;
        bool keep = false;
        ~ColGuard()
        {
            if (!keep) {
                (void)hipFree(p);
                p = nullptr;
            }
        }
    } col_guard{d_col};
    uint32_t *d_scratch, *d_emit;  // the sort's digit tables and the duplicate removal's tile counts; the key emission's tile counts
    if ((st = B.alloc(d_scratch, device_sort_scratch_words(largest))) != GP_OK) return st;
    {
        const int64_t most_tiles = (m + n + kEmitTile - 1) / kEmitTile + 1;  // (+ 1: the total)
        if ((st = B.alloc(d_emit, (size_t)most_tiles + device_scan_scratch_words(most_tiles))) != GP_OK) return st;
    }
    // bits in which keys can differ: a column is below n, a row of the range below its end
    auto bits_of = [](int64_t values) {
        int b = 0;
        while (b < 32 && (INT64_C(1) << b) < values) ++b;
        return b;
    };

    int64_t nnz = 0;
    for (size_t k = 0; k < range_cnt.size(); ++k) {
        const int64_t r0 = range_lo[k], r1 = range_lo[k + 1], cand = range_cnt[k];
        int64_t uniq = 0;
        uint64_t* d_distinct = d_keys;  // (no candidates: nothing is read from it)
        if (cand > 0) {
            const int64_t span = m + (loops ? r1 - r0 : 0), emit_tiles = (span + kEmitTile - 1) / kEmitTile;
            hipLaunchKernelGGL(gp_count_keys_range, dim3((unsigned)emit_tiles), dim3(kThreads), 0, stream, d_src, d_dst, m, sym ? 1 : 0,
                               loops ? 1 : 0, r0, r1, d_emit, emit_tiles);
            GP_HIP(hipGetLastError());
            if ((st = device_exclusive_scan(d_emit, emit_tiles + 1, d_emit + emit_tiles + 1, stream)) != GP_OK) return st;
            hipLaunchKernelGGL(gp_emit_keys_range, dim3((unsigned)emit_tiles), dim3(kThreads), 0, stream, d_src, d_dst, m, sym ? 1 : 0,
                               loops ? 1 : 0, r0, r1, d_emit, d_keys, cand);
            GP_HIP(hipGetLastError());
            uint64_t* sorted = nullptr;
            if ((st = device_sort_keys(d_keys, d_sorted, cand, bits_of(n), bits_of(r1), d_scratch, stream, &sorted)) != GP_OK) return st;
            // the distinct keys go into the buffer the sorted ones are not in
            d_distinct = sorted == d_keys ? d_sorted : d_keys;
            const uint32_t* d_total = nullptr;
            if ((st = device_unique_keys(sorted, d_distinct, cand, d_scratch, stream, &d_total)) != GP_OK) return st;
            uint32_t count = 0;
            GP_HIP(hipMemcpyAsync(&count, d_total, sizeof(uint32_t), hipMemcpyDeviceToHost, stream));
            GP_HIP(hipStreamSynchronize(stream));
            uniq = (int64_t)count;
            hipLaunchKernelGGL(gp_keys_to_columns, dim3(grid_for(uniq)), dim3(kThreads), 0, stream, d_distinct, uniq, d_col + nnz);
            GP_HIP(hipGetLastError());
        }
        // first entries of rows r0 .. r1 (row r1's start is written again, identically, by the next range)
        hipLaunchKernelGGL(gp_row_starts_range, dim3(grid_for(r1 - r0 + 1)), dim3(kThreads), 0, stream, d_distinct, uniq, r0, r1, nnz,
                           d_rowptr);
        GP_HIP(hipGetLastError());
        GP_HIP(hipStreamSynchronize(stream));  // d_keys is refilled by the next range
        nnz += uniq;
    }

    // ---- degrees and the normalisation vectors of Eq. 1 -------------------------------
    int32_t* d_deg;
    float *d_dinv_sqrt = nullptr, *d_dinv = nullptr;  // stay with the plan
    if ((st = B.alloc(d_deg, (size_t)n)) != GP_OK) return st;
    if (hipMalloc((void**)&d_dinv_sqrt, (size_t)n * sizeof(float)) != hipSuccess ||
        hipMalloc((void**)&d_dinv, (size_t)n * sizeof(float)) != hipSuccess) {
        (void)hipFree(d_dinv_sqrt);
        (void)hipFree(d_dinv);
        return fail(GP_ERR_OOM_DEVICE, "normalisation vectors on the device");
    }
    hipLaunchKernelGGL(gp_degrees_and_norms, dim3(grid_for(n)), dim3(kThreads), 0, stream, d_rowptr, n, d_deg, d_dinv_sqrt, d_dinv);

    plan->nnz = nnz;
    plan->rowptr.resize((size_t)n + 1);
    plan->col.resize((size_t)nnz);
    plan->deg.resize((size_t)n);
    plan->dinv_sqrt.resize((size_t)n);
    plan->dinv.resize((size_t)n);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(plan->rowptr.data(), d_rowptr, ((size_t)n + 1) * sizeof(int64_t), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess && nnz) e = hipMemcpyAsync(plan->col.data(), d_col, (size_t)nnz * sizeof(int32_t), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipMemcpyAsync(plan->deg.data(), d_deg, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipMemcpyAsync(plan->dinv_sqrt.data(), d_dinv_sqrt, (size_t)n * sizeof(float), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipMemcpyAsync(plan->dinv.data(), d_dinv, (size_t)n * sizeof(float), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) {
        (void)hipFree(d_dinv_sqrt);
        (void)hipFree(d_dinv);
        return fail(GP_ERR_DEVICE, "planning on the device: %s", hipGetErrorString(e));
    }
    // what gp_propagate needs of the plan is already where it will be used
    int cur = -1;
    GP_HIP(hipGetDevice(&cur));
    plan->dev.device = cur;
    plan->dev.col = nnz ? d_col : nullptr;
    col_guard.keep = nnz > 0;
    plan->dev.dinv_sqrt = d_dinv_sqrt;
    plan->dev.dinv = d_dinv;
    plan->norms_on_device = true;
    return GP_OK;
}

// rows at the block boundaries, found on the device from the row pointers
gp_status block_rows_on_device(gp_plan* plan)
{
    const int32_t b = plan->num_blocks;
    const int64_t n = plan->n;
    DeviceBuffers B;
    int64_t *d_rowptr, *d_off;
    int32_t *d_lo, *d_hi;
    gp_status st;
    if ((st = B.alloc(d_rowptr, (size_t)n + 1)) != GP_OK || (st = B.alloc(d_off, (size_t)b + 1)) != GP_OK ||
        (st = B.alloc(d_lo, (size_t)b)) != GP_OK || (st = B.alloc(d_hi, (size_t)b)) != GP_OK)
        return st;
    GP_HIP(hipMemcpy(d_rowptr, plan->rowptr.data(), ((size_t)n + 1) * sizeof(int64_t), hipMemcpyHostToDevice));
    GP_HIP(hipMemcpy(d_off, plan->block_off.data(), ((size_t)b + 1) * sizeof(int64_t), hipMemcpyHostToDevice));
    hipLaunchKernelGGL(gp_block_rows, dim3((unsigned)((b + kThreads - 1) / kThreads)), dim3(kThreads), 0, nullptr, d_rowptr, n, d_off, b,
                       d_lo, d_hi);
    GP_HIP(hipGetLastError());
    GP_HIP(hipMemcpy(plan->block_row_lo.data(), d_lo, (size_t)b * sizeof(int32_t), hipMemcpyDeviceToHost));
    GP_HIP(hipMemcpy(plan->block_row_hi.data(), d_hi, (size_t)b * sizeof(int32_t), hipMemcpyDeviceToHost));
    return GP_OK;
}

}  // namespace gp
