// Device-wide sort and duplicate removal of 64-bit keys, for planning on the GPU (the
// non-zero set of the matrix that Eq. 1 normalises, as keys row << 32 | column; Section
// 3.2's block-wise normalisation needs the set sorted and without duplicates).
//
// Sort: least-significant-digit radix sort, 8 bits per pass, only over the bit ranges that
// can differ between keys (the caller says how many low and high bits are in use).  A pass
// is three steps: (1) every workgroup counts the digits of its tile of 16384 consecutive
// keys into a table laid out digit-major, [digit][workgroup]; (2) an exclusive scan of that
// table as one flat array, which turns every entry into the place where the workgroup's
// first key of that digit goes; (3) every workgroup walks its tile again, 256 keys at a time
// in index order, ranks each key among the keys of the same digit before it (inside the
// wavefront by eight ballots, across the four wavefronts and across the steps by counters in
// LDS) and writes it to its place.  Equal digits keep their order, so the passes compose.
//
// Duplicate removal on the sorted keys: a key is kept if it differs from the one before it;
// tiles of 4096 keys count what they keep, an exclusive scan of the counts gives every tile's
// first output place (and, behind the last tile, the total), and a second walk writes the
// kept keys in order.
//
// The scan is this file's too: chunk sums, a one-workgroup scan of the sums, then every
// chunk scanned with its offset.  All counts fit 32 bits (at most 2^31 - 1 keys per call).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <utility>

#include "gp_block_scan.h"
#include "gp_internal.h"

namespace gp {

namespace {

constexpr int kThreads = kScanThreads;
constexpr int kWaves = kScanWaves;
constexpr int kSortItems = 64;                       // keys per thread of a sort tile
constexpr int64_t kSortTile = kThreads * kSortItems; // 16384
constexpr int kScanItems = 16;                       // entries per thread of a scan chunk / keys per thread of a unique tile
constexpr int64_t kScanChunk = kThreads * kScanItems;  // 4096

// ---- exclusive scan of a[0 .. N) in place --------------------------------------------------

__global__ __launch_bounds__(kThreads) void gp_scan_chunk_sums(const uint32_t* __restrict__ a, int64_t N, uint32_t* __restrict__ sums)
{
    __shared__ uint32_t ws[kWaves + 1];
    const int64_t c0 = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kScanItems;
    uint32_t s = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j)
        if (c0 + j < N) s += a[c0 + j];
    uint32_t total;
    block_exclusive(s, ws, &total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(kThreads) void gp_scan_sums(uint32_t* __restrict__ sums, int64_t P)
{
    __shared__ uint32_t ws[kWaves + 1];
    uint32_t carry = 0;
    for (int64_t p0 = 0; p0 < P; p0 += kThreads) {  // (the same trip count for every thread)
        const int64_t p = p0 + threadIdx.x;
        const uint32_t v = p < P ? sums[p] : 0;
        uint32_t total;
        const uint32_t ex = block_exclusive(v, ws, &total);
        if (p < P) sums[p] = carry + ex;
        carry += total;
    }
}

__global__ __launch_bounds__(kThreads) void gp_scan_chunks(uint32_t* __restrict__ a, int64_t N, const uint32_t* __restrict__ sums)
{
    __shared__ uint32_t ws[kWaves + 1];
    const int64_t c0 = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kScanItems;
    uint32_t v[kScanItems], s = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        v[j] = c0 + j < N ? a[c0 + j] : 0;
        s += v[j];
    }
    uint32_t total;
    uint32_t run = sums[blockIdx.x] + block_exclusive(s, ws, &total);
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        if (c0 + j < N) a[c0 + j] = run;
        run += v[j];
    }
}

}  // namespace

size_t device_scan_scratch_words(int64_t N) { return (size_t)((std::max<int64_t>(N, 1) + kScanChunk - 1) / kScanChunk + 1); }

gp_status device_exclusive_scan(uint32_t* a, int64_t N, uint32_t* sums, hipStream_t stream)
{
    if (N <= 0) return GP_OK;
    const int64_t P = (N + kScanChunk - 1) / kScanChunk;
    hipLaunchKernelGGL(gp_scan_chunk_sums, dim3((unsigned)P), dim3(kThreads), 0, stream, a, N, sums);
    hipLaunchKernelGGL(gp_scan_sums, dim3(1), dim3(kThreads), 0, stream, sums, P);
    hipLaunchKernelGGL(gp_scan_chunks, dim3((unsigned)P), dim3(kThreads), 0, stream, a, N, sums);
    GP_HIP(hipGetLastError());
    return GP_OK;
}

namespace {

// ---- one radix pass ---------------------------------------------------------------------

__global__ __launch_bounds__(kThreads) void gp_radix_count(const uint64_t* __restrict__ keys, int64_t count, int shift,
                                                           uint32_t* __restrict__ table)
{
    __shared__ uint32_t h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t t0 = (int64_t)blockIdx.x * kSortTile;
    for (int i = 0; i < kSortItems; ++i) {
        const int64_t e = t0 + (int64_t)i * kThreads + threadIdx.x;
        if (e < count) atomicAdd(&h[(unsigned)(keys[e] >> shift) & 0xFFu], 1u);
    }
    __syncthreads();
    table[(int64_t)threadIdx.x * gridDim.x + blockIdx.x] = h[threadIdx.x];
}

__global__ __launch_bounds__(kThreads) void gp_radix_scatter(const uint64_t* __restrict__ in, uint64_t* __restrict__ out, int64_t count,
                                                             int shift, const uint32_t* __restrict__ table)
{
    __shared__ uint32_t base[256];            // where the workgroup's next key of a digit goes
    __shared__ uint32_t in_wave[kWaves][256];  // keys of a digit per wavefront, this step
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    base[threadIdx.x] = table[(int64_t)threadIdx.x * gridDim.x + blockIdx.x];
#pragma unroll
    for (int w = 0; w < kWaves; ++w) in_wave[w][threadIdx.x] = 0;
    __syncthreads();
    const int64_t t0 = (int64_t)blockIdx.x * kSortTile;
    for (int i = 0; i < kSortItems; ++i) {
        if (t0 + (int64_t)i * kThreads >= count) break;  // (the same for every thread of the workgroup)
        const int64_t e = t0 + (int64_t)i * kThreads + threadIdx.x;
        const bool valid = e < count;
        const uint64_t key = valid ? in[e] : 0;
        const unsigned digit = (unsigned)(key >> shift) & 0xFFu;
        // the lanes of this wavefront that hold a key of the same digit
        unsigned long long peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = (digit >> b) & 1u;
            const unsigned long long with = __ballot(bit);
            peers &= bit ? with : ~with;
        }
        const int rank = __popcll(peers & ((1ull << lane) - 1ull));
        if (valid && rank == 0) in_wave[wave][digit] = (uint32_t)__popcll(peers);
        __syncthreads();
        if (valid) {
            uint32_t place = base[digit] + (uint32_t)rank;
            for (int w = 0; w < wave; ++w) place += in_wave[w][digit];
            if ((int64_t)place < count) out[place] = key;  // (always true; keeps a slip in the tables from writing elsewhere)
        }
        __syncthreads();
        {  // thread t closes digit t's step
            uint32_t s = 0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                s += in_wave[w][threadIdx.x];
                in_wave[w][threadIdx.x] = 0;
            }
            base[threadIdx.x] += s;
        }
        __syncthreads();
    }
}

// ---- duplicate removal --------------------------------------------------------------------

__device__ inline bool kept(const uint64_t* __restrict__ keys, int64_t e, int64_t count)
{
    return e < count && (e == 0 || keys[e] != keys[e - 1]);
}

__global__ __launch_bounds__(kThreads) void gp_unique_count(const uint64_t* __restrict__ keys, int64_t count,
                                                            uint32_t* __restrict__ tile_count, int64_t tiles)
{
    __shared__ uint32_t ws[kWaves + 1];
    const int64_t t0 = (int64_t)blockIdx.x * kScanChunk;
    uint32_t s = 0;
    for (int j = 0; j < kScanItems; ++j) s += kept(keys, t0 + (int64_t)j * kThreads + threadIdx.x, count) ? 1u : 0u;
    uint32_t total;
    block_exclusive(s, ws, &total);
    if (threadIdx.x == 0) {
        tile_count[blockIdx.x] = total;
        if (blockIdx.x == 0) tile_count[tiles] = 0;  // the scan leaves the total here
    }
}

__global__ __launch_bounds__(kThreads) void gp_unique_write(const uint64_t* __restrict__ keys, int64_t count,
                                                            const uint32_t* __restrict__ tile_first, uint64_t* __restrict__ out)
{
    __shared__ uint32_t ws[kWaves + 1];
    const int64_t t0 = (int64_t)blockIdx.x * kScanChunk;
    uint32_t run = tile_first[blockIdx.x];
    for (int j = 0; j < kScanItems; ++j) {  // 256 consecutive keys per step, in order
        const int64_t e = t0 + (int64_t)j * kThreads + threadIdx.x;
        const bool k = kept(keys, e, count);
        uint32_t total;
        const uint32_t ex = block_exclusive(k ? 1u : 0u, ws, &total);
        if (k && (int64_t)(run + ex) < count) out[run + ex] = keys[e];  // (the bound always holds)
        run += total;
    }
}

int passes_of(int bits) { return (bits + 7) / 8; }

}  // namespace

size_t device_sort_scratch_words(int64_t count)
{
    const int64_t sort_tiles = std::max<int64_t>(1, (count + kSortTile - 1) / kSortTile);
    const int64_t table = 256 * sort_tiles;
    const int64_t uniq_tiles = std::max<int64_t>(1, (count + kScanChunk - 1) / kScanChunk) + 1;
    const int64_t a = std::max(table, uniq_tiles);
    return (size_t)(a + (a + kScanChunk - 1) / kScanChunk + 1);
}

gp_status device_sort_keys(uint64_t* keys, uint64_t* other, int64_t count, int low_bits, int high_bits, uint32_t* scratch,
                           hipStream_t stream, uint64_t** sorted)
{
    *sorted = keys;
    if (count <= 1) return GP_OK;
    if (count > (INT64_C(1) << 31) - 1) return fail(GP_ERR_UNSUPPORTED, "device sort: %lld keys exceed 2^31 - 1", (long long)count);
    if (low_bits < 0 || low_bits > 32 || high_bits < 0 || high_bits > 32) return fail(GP_ERR_INVALID_ARG, "device sort: bit counts must be 0 .. 32");
    const int64_t tiles = (count + kSortTile - 1) / kSortTile;
    const int64_t table_len = 256 * tiles;
    uint32_t* table = scratch;
    uint32_t* sums = scratch + table_len;
    uint64_t *from = keys, *to = other;
    for (int half = 0; half < 2; ++half) {
        const int bits = half == 0 ? low_bits : high_bits;
        for (int p = 0; p < passes_of(bits); ++p) {
            const int shift = half * 32 + p * 8;
            hipLaunchKernelGGL(gp_radix_count, dim3((unsigned)tiles), dim3(kThreads), 0, stream, from, count, shift, table);
            GP_HIP(hipGetLastError());
            gp_status st = device_exclusive_scan(table, table_len, sums, stream);
            if (st != GP_OK) return st;
            hipLaunchKernelGGL(gp_radix_scatter, dim3((unsigned)tiles), dim3(kThreads), 0, stream, from, to, count, shift, table);
            GP_HIP(hipGetLastError());
            std::swap(from, to);
        }
    }
    *sorted = from;
    return GP_OK;
}

gp_status device_unique_keys(const uint64_t* sorted, uint64_t* out, int64_t count, uint32_t* scratch, hipStream_t stream,
                             const uint32_t** total)
{
    if (count < 0 || count > (INT64_C(1) << 31) - 1) return fail(GP_ERR_UNSUPPORTED, "device unique: %lld keys exceed 2^31 - 1", (long long)count);
    const int64_t tiles = std::max<int64_t>(1, (count + kScanChunk - 1) / kScanChunk);
    uint32_t* tile_count = scratch;
    uint32_t* sums = scratch + tiles + 1;
    hipLaunchKernelGGL(gp_unique_count, dim3((unsigned)tiles), dim3(kThreads), 0, stream, sorted, count, tile_count, tiles);
    GP_HIP(hipGetLastError());
    gp_status st = device_exclusive_scan(tile_count, tiles + 1, sums, stream);
    if (st != GP_OK) return st;
    hipLaunchKernelGGL(gp_unique_write, dim3((unsigned)tiles), dim3(kThreads), 0, stream, sorted, count, tile_count, out);
    GP_HIP(hipGetLastError());
    *total = tile_count + tiles;
    return GP_OK;
}

}  // namespace gp
