// Device side of gp_plan_blocks (flag GP_PLAN_ON_DEVICE): the non-zero set of the
// matrix being normalised, sorted and de-duplicated on the GPU.  The paper runs its
// adjacency normalisation block-wise on the GPU (Section 3.2, Section 4.2); here the
// normalisation needs no matrix at all, only the sorted set and its row counts, so
// the GPU's share is: emit one 64-bit key (row << 32 | col) per candidate entry,
// radix-sort the keys, drop duplicates, split them back into columns, and find
// every row's first entry by binary search.  Integers only, so the result is the
// host planner's bit for bit.  The sort and the duplicate removal are rocPRIM's
// device-wide primitives; the kernels around them are this file's.
#include <hip/hip_runtime.h>

#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_select.hpp>

#include "gp_internal.h"

namespace gp {

namespace {

constexpr int kThreads = 256;
constexpr uint64_t kNoKey = ~UINT64_C(0);  // sorts after every real key

// pair e -> key slots [e*per, e*per + per): (row = dst, col = src) and, when
// symmetrising, its mirror; a self pair leaves its slots empty.
__global__ __launch_bounds__(kThreads) void gp_emit_keys(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                                         int64_t m, int per, uint64_t* __restrict__ keys)
{
    for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < m; e += (int64_t)gridDim.x * kThreads) {
        const uint32_t s = (uint32_t)src[e], t = (uint32_t)dst[e];
        const bool self = s == t;
        keys[e * per] = self ? kNoKey : ((uint64_t)t << 32) | s;
        if (per == 2) keys[e * per + 1] = self ? kNoKey : ((uint64_t)s << 32) | t;
    }
}

__global__ __launch_bounds__(kThreads) void gp_emit_loop_keys(int64_t n, uint64_t* __restrict__ keys)
{
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kThreads)
        keys[i] = ((uint64_t)i << 32) | (uint64_t)i;
}

__global__ __launch_bounds__(kThreads) void gp_keys_to_columns(const uint64_t* __restrict__ keys, int64_t nnz,
                                                               int32_t* __restrict__ col)
{
    for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < nnz; e += (int64_t)gridDim.x * kThreads)
        col[e] = (int32_t)(keys[e] & 0xFFFFFFFFu);
}

// rowptr[i] = number of keys below (i << 32), i = 0 .. n
__global__ __launch_bounds__(kThreads) void gp_row_starts(const uint64_t* __restrict__ keys, int64_t nnz, int64_t n,
                                                          int64_t* __restrict__ rowptr)
{
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i <= n; i += (int64_t)gridDim.x * kThreads) {
        const uint64_t probe = (uint64_t)i << 32;
        int64_t lo = 0, hi = nnz;
        while (lo < hi) {
            const int64_t mid = lo + (hi - lo) / 2;
            if (keys[mid] < probe)
                lo = mid + 1;
            else
                hi = mid;
        }
        rowptr[i] = lo;
    }
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
    const int per = sym ? 2 : 1;
    const int64_t total = m * per + (loops ? n : 0);
    if (total >= (INT64_C(1) << 31))
        return fail(GP_ERR_UNSUPPORTED, "%lld candidate entries: planning on the device is limited to 2^31 - 1; plan on the host",
                    (long long)total);
    hipStream_t stream = nullptr;
    DeviceBuffers B;
    int32_t *d_src, *d_dst, *d_col;
    uint64_t *d_keys, *d_sorted, *d_unique;
    int64_t* d_rowptr;
    size_t* d_count;
    gp_status st;
    if ((st = B.alloc(d_src, (size_t)m)) != GP_OK || (st = B.alloc(d_dst, (size_t)m)) != GP_OK ||
        (st = B.alloc(d_keys, (size_t)total)) != GP_OK || (st = B.alloc(d_sorted, (size_t)total)) != GP_OK ||
        (st = B.alloc(d_count, 1)) != GP_OK || (st = B.alloc(d_rowptr, (size_t)n + 1)) != GP_OK)
        return st;
    if (m) {
        GP_HIP(hipMemcpyAsync(d_src, src, (size_t)m * 4, hipMemcpyHostToDevice, stream));
        GP_HIP(hipMemcpyAsync(d_dst, dst, (size_t)m * 4, hipMemcpyHostToDevice, stream));
        hipLaunchKernelGGL(gp_emit_keys, dim3(grid_for(m)), dim3(kThreads), 0, stream, d_src, d_dst, m, per, d_keys);
        GP_HIP(hipGetLastError());
    }
    if (loops) {
        hipLaunchKernelGGL(gp_emit_loop_keys, dim3(grid_for(n)), dim3(kThreads), 0, stream, n, d_keys + m * per);
        GP_HIP(hipGetLastError());
    }

    int64_t nnz = 0;
    if (total > 0) {
        // all 64 bits are sorted: empty slots are all ones and must end up last
        size_t tmp_bytes = 0;
        GP_HIP(rocprim::radix_sort_keys(nullptr, tmp_bytes, d_keys, d_sorted, (size_t)total, 0u, 64u, stream));
        char* d_tmp = nullptr;
        if ((st = B.alloc(d_tmp, tmp_bytes)) != GP_OK) return st;
        GP_HIP(rocprim::radix_sort_keys(d_tmp, tmp_bytes, d_keys, d_sorted, (size_t)total, 0u, 64u, stream));
        d_unique = d_keys;  // the unsorted keys are no longer needed
        size_t tmp2 = 0;
        GP_HIP(rocprim::unique(nullptr, tmp2, d_sorted, d_unique, d_count, (size_t)total, rocprim::equal_to<uint64_t>(), stream));
        char* d_tmp2 = d_tmp;
        if (tmp2 > tmp_bytes && (st = B.alloc(d_tmp2, tmp2)) != GP_OK) return st;
        GP_HIP(rocprim::unique(d_tmp2, tmp2, d_sorted, d_unique, d_count, (size_t)total, rocprim::equal_to<uint64_t>(), stream));
        size_t count = 0;
        uint64_t last = 0;
        GP_HIP(hipMemcpyAsync(&count, d_count, sizeof(size_t), hipMemcpyDeviceToHost, stream));
        GP_HIP(hipStreamSynchronize(stream));
        if (count > 0) {
            GP_HIP(hipMemcpy(&last, d_unique + (count - 1), sizeof(uint64_t), hipMemcpyDeviceToHost));
            if (last == kNoKey) --count;  // the one survivor of all empty slots
        }
        nnz = (int64_t)count;
    } else {
        d_unique = d_keys;
    }

    hipLaunchKernelGGL(gp_row_starts, dim3(grid_for(n + 1)), dim3(kThreads), 0, stream, d_unique, nnz, n, d_rowptr);
    GP_HIP(hipGetLastError());
    d_col = (int32_t*)d_sorted;  // reuse: the sorted keys with duplicates are done with
    if (nnz) {
        hipLaunchKernelGGL(gp_keys_to_columns, dim3(grid_for(nnz)), dim3(kThreads), 0, stream, d_unique, nnz, d_col);
        GP_HIP(hipGetLastError());
    }

    plan->nnz = nnz;
    plan->rowptr.resize((size_t)n + 1);
    plan->col.resize((size_t)nnz);
    plan->deg.resize((size_t)n);
    GP_HIP(hipMemcpyAsync(plan->rowptr.data(), d_rowptr, ((size_t)n + 1) * sizeof(int64_t), hipMemcpyDeviceToHost, stream));
    if (nnz) GP_HIP(hipMemcpyAsync(plan->col.data(), d_col, (size_t)nnz * sizeof(int32_t), hipMemcpyDeviceToHost, stream));
    GP_HIP(hipStreamSynchronize(stream));
    for (int64_t i = 0; i < n; ++i) plan->deg[i] = (int32_t)(plan->rowptr[i + 1] - plan->rowptr[i]);
    return GP_OK;
}

}  // namespace gp
