// Forward pass of an LC-version model over the hop stack (Appendix A: the LC version
// of GPRGNN; Section 3.1: the H^LC formula for the single-branch case):
//
//     H[batch] = sum_k gamma_k * MLP(X_k[batch]),   MLP(Z) = relu(..relu(Z W_1)..W_{T-1}) W_T.
//
// This is the one dense contraction on the path, so it runs on the matrix cores:
// fp32 MFMA (v_mfma_f32_32x32x2_f32), all layers of one hop fused in one kernel.
// A workgroup of four waves owns 64 batch rows (32 for very small batches) of one hop;
// the hops' results are summed afterwards in hop order.  The rows' features (later: the
// previous layer's activations) sit in LDS as the A operand; the weights are the B
// operand, read straight from L2 (all T matrices together are a few hundred KB and
// stay there) one 8-row chunk ahead of the MFMAs that use them; the layer output
// stays in accumulator registers until every wave is done with the LDS tile, then
// replaces it (ReLU applied on the way).  Nothing but the gathered rows and the
// per-hop B x C results touches HBM.
//
// Index freedom used: MFMA sums over k and yields 32 columns per tile, but which k
// and which column a lane supplies is the kernel's choice as long as A and B agree.
// Lane half hh of a wave takes k = 8c + 4hh + s for step s of chunk c (one 16-byte
// LDS read feeds four MFMA steps), and column j of a wave's tile t is output column
// base + NT*j + t, so the NT tiles of a wave need NT consecutive weights per lane
// (one vector load) and produce NT consecutive activations per lane (one vector
// LDS store).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <mutex>

#include "gp_internal.h"

namespace gp {

namespace {

constexpr int kLcThreads = 256;
constexpr int kPanel = 256;      // widest inner dimension staged in LDS at once
constexpr int kLd = kPanel + 4;  // LDS row stride in floats (16-byte aligned rows, banks staggered)
constexpr int kMaxLayers = 8;
constexpr int kMaxHops = 16;
constexpr int64_t kWorkspaceBytes = INT64_C(256) << 20;  // cap on the partial results of one piece

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef unsigned short v4u16 __attribute__((ext_vector_type(4)));

struct LcArgs {
    const void* stack;
    int64_t ld, slab;  // elements: row stride, distance between hop slabs
    int64_t n;
    int d;
    int hops;                 // branches in use: work item = tile * hops + branch
    int hop_of[kMaxHops];     // branch -> slab of the stack it reads
    int depth[kMaxHops];      // branch -> number of weight matrices it applies
    int out_off[kMaxHops];    // branch -> first output column when branches are written side by side
    int direct;               // 1: branches write the final result (side by side, or there is just one)
    const int32_t* batch;
    int64_t B;
    float gamma[kMaxHops];
    int T;
    const float* W[kMaxLayers];
    int width[kMaxLayers];
    int wvec[kMaxLayers];  // 1: W_t rows may be read with NT-wide vector loads
    int xvec;              // 1: stack rows may be read four elements at a time
    float* dst;            // the result (direct), else the partial results [branch][B][ldd]
    int64_t ldd;
};

__device__ __forceinline__ float widen(float v) { return v; }
__device__ __forceinline__ float widen(unsigned short v) { return __uint_as_float((unsigned)v << 16); }

__device__ __forceinline__ v4f load4(const float* p) { return *reinterpret_cast<const v4f*>(p); }
__device__ __forceinline__ v4f load4(const unsigned short* p)
{
    const v4u16 b = *reinterpret_cast<const v4u16*>(p);
    v4f r;
    r.x = widen(b.x), r.y = widen(b.y), r.z = widen(b.z), r.w = widen(b.w);
    return r;
}

// 64 x kin panel of the batch rows of one slab -> LDS, widened to fp32, zero beyond
// kin (up to the next multiple of 8), zero for rows past the batch or ids outside
// [0, n) (those rows are never stored).  Eight independent requests per thread are
// in flight before the first is written to LDS.
template <typename T, int TM>
__device__ __forceinline__ void lc_gather(float* __restrict__ tile, const T* __restrict__ slab, const LcArgs& a,
                                          int64_t row0, int p0, int kin, int tid)
{
    constexpr int U = 8;
    const unsigned nq = (unsigned)(((kin + 7) & ~7) >> 2);  // groups of four columns per row
    const unsigned total = TM * nq;
    for (unsigned base = 0; base < total; base += U * kLcThreads) {
        int64_t id[U];
        unsigned r[U], q[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned idx = base + u * kLcThreads + tid;
            r[u] = idx / nq, q[u] = idx - r[u] * nq;
            const int64_t br = row0 + r[u];
            id[u] = -1;
            if (idx < total && br < a.B) id[u] = a.batch ? (int64_t)a.batch[br] : br;
        }
        v4f v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            v[u] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
            if (id[u] >= 0 && id[u] < a.n) {
                const T* src = slab + id[u] * a.ld + p0 + 4 * q[u];
                const int c0 = 4 * (int)q[u];
                if (a.xvec && c0 + 4 <= kin) {
                    v[u] = load4(src);
                } else {
                    if (c0 + 0 < kin) v[u].x = widen(src[0]);
                    if (c0 + 1 < kin) v[u].y = widen(src[1]);
                    if (c0 + 2 < kin) v[u].z = widen(src[2]);
                    if (c0 + 3 < kin) v[u].w = widen(src[3]);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (base + u * kLcThreads + tid < total) *reinterpret_cast<v4f*>(tile + r[u] * kLd + 4 * q[u]) = v[u];
    }
}

// How the four waves of a workgroup split a layer with N output columns.
//   wide   (N > 64):  wave w owns columns [w*32*NT, (w+1)*32*NT), NT = ceil(N/128), of
//                     BOTH 32-row blocks: every weight is fetched by exactly one wave.
//   narrow (N <= 64): wave w owns row block w & 1 and columns [(w>>1)*32, +32): all four
//                     matrix cores stay busy on a 40- or 64-class output layer.
// A wave whose columns all lie beyond N sits the layer out.  Tile (r, t) of a wave is
// accumulator r*NT + t; column i of tile t is output column colbase + NT*i + t.
struct WaveMap {
    int rbw;      // row blocks this wave owns: 2 (wide) or 1 (narrow)
    int nt;       // 32-column tiles per row block: 1 or 2
    int rb0;      // first row block
    int colbase;  // first column
};
template <int RB>  // RB = 32-row blocks per work item: 2 (64 rows) or 1 (32 rows, all waves split the columns)
__device__ __forceinline__ WaveMap wave_map(int N, int wave)
{
    WaveMap m;
    if (RB == 1 || N > 64) {
        m.rbw = RB, m.nt = (N + 127) >> 7, m.rb0 = 0, m.colbase = wave * 32 * m.nt;
    } else {
        m.rbw = 1, m.nt = 1, m.rb0 = wave & 1, m.colbase = (wave >> 1) * 32;
    }
    return m;
}

// Weights of one full 8-row chunk for this lane: rows 4hh .. 4hh+3 of the chunk that
// starts at Wc (= W + 8c*N, the same for the whole wave), NT columns.  Loads are
// never predicated (a predicated load costs a branch): a lane whose columns lie
// beyond N reads column 0 instead (coff is clamped) and its products are discarded
// when the layer's output is stored.  roff = 4hh*N; vectors use coff[0] only.
template <int NT, bool VEC>
__device__ __forceinline__ void lc_load_b(const float* Wc, int N, int roff, const int (&coff)[NT], float (&b)[4][NT])
{
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const float* p = Wc + s * N;
        if constexpr (NT == 2 && VEC) {
            const v2f v = *reinterpret_cast<const v2f*>(p + (unsigned)(roff + coff[0]));
            b[s][0] = v.x, b[s][1] = v.y;
        } else {
#pragma unroll
            for (int t = 0; t < NT; ++t) b[s][t] = p[(unsigned)(roff + coff[t])];
        }
    }
}

// The last, partial chunk (rows_left < 8 rows): a row beyond the matrix is read as
// row 0 of the chunk and replaced by zero.
template <int NT>
__device__ __forceinline__ void lc_load_b_tail(const float* Wc, int N, int rows_left, int hh, const int (&coff)[NT],
                                               float (&b)[4][NT])
{
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int r = 4 * hh + s;
        const bool ok = r < rows_left;
        const int roff = ok ? r * N : 0;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const float v = Wc[roff + coff[t]];
            b[s][t] = ok ? v : 0.0f;
        }
    }
}

// nothing moves across: neither in the compiler's middle end (the memory clobber) nor
// in its instruction scheduler
__device__ __forceinline__ void lc_fence()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// the 4 * RBW * NT MFMAs of one chunk: step s multiplies k = 8c + 4hh + s
template <int RBW, int NT>
__device__ __forceinline__ void lc_mfma_chunk(const v4f (&av)[RBW], const float (&b)[4][NT], v16f (&acc)[4])
{
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int r = 0; r < RBW; ++r)
#pragma unroll
            for (int t = 0; t < NT; ++t)
                acc[r * NT + t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[r][s], b[s][t], acc[r * NT + t], 0, 0, 0);
}

// acc += tile(64 x kin) * W(kin x N) for this wave's share (see WaveMap).  Operands
// are requested one chunk before they are used, in two alternating register sets.  A
// request past the last full chunk repeats that chunk (harmless, in bounds) instead
// of being skipped, which keeps the loop free of predicated loads.
template <int RBW, int NT, bool VEC>
__device__ __forceinline__ void lc_layer(const float* tile, int kin, const float* W, int N, const WaveMap& m, int j, int hh,
                                         v16f (&acc)[4])
{
    const int colb = m.colbase + NT * j;
    const float* arow = tile + (m.rb0 * 32 + j) * kLd + 4 * hh;
    const int full = kin >> 3;
    const int roff = 4 * hh * N;
    int coff[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) coff[t] = colb + t < N ? colb + t : 0;
    if (full > 0) {
        auto load_a = [&](int c, v4f (&av)[RBW]) {
#pragma unroll
            for (int r = 0; r < RBW; ++r) av[r] = *reinterpret_cast<const v4f*>(arow + r * 32 * kLd + min(c, full - 1) * 8);
        };
        auto load_b = [&](int c, float (&b)[4][NT]) { lc_load_b<NT, VEC>(W + (int64_t)min(c, full - 1) * 8 * N, N, roff, coff, b); };
        float b0[4][NT], b1[4][NT];
        v4f a0[RBW], a1[RBW];
        // the fences keep each request group ahead of the MFMA group it is written
        // before; left alone, the compiler sinks the loads to their first use
        load_b(0, b0), load_a(0, a0);
        int c = 0;
        for (; c + 2 <= full; c += 2) {  // steady state: two chunks per trip, no exits inside
            load_b(c + 1, b1), load_a(c + 1, a1);
            lc_fence();
            lc_mfma_chunk<RBW, NT>(a0, b0, acc);
            lc_fence();
            load_b(c + 2, b0), load_a(c + 2, a0);
            lc_fence();
            lc_mfma_chunk<RBW, NT>(a1, b1, acc);
            lc_fence();
        }
        if (c < full) lc_mfma_chunk<RBW, NT>(a0, b0, acc);  // an odd last chunk is already here
    }
    if (kin & 7) {
        float bt[4][NT];
        v4f at[RBW];
        lc_load_b_tail<NT>(W + (int64_t)full * 8 * N, N, kin & 7, hh, coff, bt);
#pragma unroll
        for (int r = 0; r < RBW; ++r) at[r] = *reinterpret_cast<const v4f*>(arow + r * 32 * kLd + full * 8);  // zero beyond kin
        lc_mfma_chunk<RBW, NT>(at, bt, acc);
    }
}

template <int RB>
__device__ __forceinline__ void lc_layer_any(const float* tile, int kin, const float* W, int N, bool vec, int wave, int j,
                                             int hh, v16f (&acc)[4])
{
    const WaveMap m = wave_map<RB>(N, wave);
    if (m.colbase >= N) return;
    if (m.nt == 2) {
        if (vec)
            lc_layer<RB, 2, true>(tile, kin, W, N, m, j, hh, acc);
        else
            lc_layer<RB, 2, false>(tile, kin, W, N, m, j, hh, acc);
    } else if (RB == 2 && m.rbw == 2) {
        lc_layer<RB, 1, false>(tile, kin, W, N, m, j, hh, acc);
    } else {
        lc_layer<1, 1, false>(tile, kin, W, N, m, j, hh, acc);
    }
}

// accumulator element e of a 32x32 tile sits in row 8*(e/4) + 4*(lane/32) + e%4
__device__ __forceinline__ int acc_row(int e, int hh) { return 8 * (e >> 2) + 4 * hh + (e & 3); }

// tile <- relu(acc) for this wave's share of a layer of width Np; columns beyond Np
// (products of clamped loads) become zeros; acc <- 0
template <int RBW, int NT>
__device__ __forceinline__ void lc_store_relu(float* __restrict__ tile, int Np, const WaveMap& m, int j, int hh, v16f (&acc)[4])
{
    bool keep[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) keep[t] = m.colbase + NT * j + t < Np;
#pragma unroll
    for (int r = 0; r < RBW; ++r)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            float* p = tile + ((m.rb0 + r) * 32 + acc_row(e, hh)) * kLd + m.colbase + NT * j;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const float x = acc[r * NT + t][e];
                p[t] = (x < 0.0f || !keep[t]) ? 0.0f : x;  // NaN stays NaN
            }
        }
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = (v16f)(0.0f);
}

// Every column below the next multiple of 8 of Np must be written (the next layer
// reads that far): a wave that sat the layer out holds zeros and stores them too
// when its columns start below that bound.
template <int RB>
__device__ __forceinline__ void lc_store_relu_any(float* tile, int Np, int wave, int j, int hh, v16f (&acc)[4])
{
    const WaveMap m = wave_map<RB>(Np, wave);
    if (m.colbase >= ((Np + 7) & ~7)) return;
    if (m.nt == 2)
        lc_store_relu<RB, 2>(tile, Np, m, j, hh, acc);
    else if (RB == 2 && m.rbw == 2)
        lc_store_relu<RB, 1>(tile, Np, m, j, hh, acc);
    else
        lc_store_relu<1, 1>(tile, Np, m, j, hh, acc);
}

// One workgroup: 32*RB batch rows of one branch (hop k, the first depth_k layers); writes
// gamma_k * branch_k either to its slab of the partial results or, when branches are
// concatenated, to its columns of the result.
template <typename T, int RB>
__global__ __launch_bounds__(kLcThreads, 2) void gp_lc_mlp(const LcArgs a)
{
    constexpr int TM = 32 * RB;
    extern __shared__ __align__(16) float tile[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 31, hh = lane >> 5;
    const int br = (int)(blockIdx.x % (unsigned)a.hops);
    const int k = a.hop_of[br], layers = a.depth[br];
    const int64_t row0 = (int64_t)(blockIdx.x / (unsigned)a.hops) * TM;
    const int C = a.width[layers - 1];

    v16f acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = (v16f)(0.0f);

    const T* slab = static_cast<const T*>(a.stack) + (int64_t)k * a.slab;
    const int N1 = a.width[0];
    for (int p0 = 0; p0 < a.d; p0 += kPanel) {  // first layer, one panel of feature columns at a time
        const int kin = min(kPanel, a.d - p0);
        if (p0 > 0) __syncthreads();  // every wave is done with the previous panel (nothing is in the tile before the first)
        lc_gather<T, TM>(tile, slab, a, row0, p0, kin, tid);
        __syncthreads();
        lc_layer_any<RB>(tile, kin, a.W[0] + (int64_t)p0 * N1, N1, a.wvec[0] != 0, wave, j, hh, acc);
    }
    for (int t = 1; t < layers; ++t) {
        const int Np = a.width[t - 1], N = a.width[t];
        __syncthreads();  // every wave is done reading the tile
        lc_store_relu_any<RB>(tile, Np, wave, j, hh, acc);
        __syncthreads();
        lc_layer_any<RB>(tile, Np, a.W[t], N, a.wvec[t] != 0, wave, j, hh, acc);
    }

    const float g = a.gamma[k];
    float* dst = a.direct ? a.dst + a.out_off[br] : a.dst + (int64_t)br * a.B * a.ldd;
    const WaveMap m = wave_map<RB>(C, wave);
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        if (r >= m.rbw) break;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            if (t >= m.nt) break;
            const int col = m.colbase + m.nt * j + t;
            // (r, t) -> accumulator r*nt + t; nt is 1 or 2
            const v16f& v = m.nt == 1 ? acc[r] : acc[r * 2 + t];
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int64_t row = row0 + (m.rb0 + r) * 32 + acc_row(e, hh);
                if (row < a.B && col < C) dst[row * a.ldd + col] = g * v[e];
            }
        }
    }
}

// out[i][c] = sum (or maximum) over the branches, in branch order, of the partial results
__global__ __launch_bounds__(kLcThreads) void gp_lc_reduce(const float* __restrict__ part, int items, int take_max, int64_t B,
                                                           int C, float* __restrict__ out, int64_t ldo)
{
    const int64_t total = B * C;
    for (int64_t i = (int64_t)blockIdx.x * kLcThreads + threadIdx.x; i < total; i += (int64_t)gridDim.x * kLcThreads) {
        float s = part[i];
        for (int it = 1; it < items; ++it) {
            const float v = part[(int64_t)it * total + i];
            s = take_max ? (v > s || v != v ? v : s) : s + v;  // a NaN branch makes the maximum NaN
        }
        out[(i / C) * ldo + i % C] = s;
    }
}

// Y = softmax(H) row by row, in place: one wave per row, row maximum subtracted first
__global__ __launch_bounds__(kLcThreads) void gp_lc_softmax_rows(float* __restrict__ H, int64_t B, int C, int64_t ld)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * kLcThreads + threadIdx.x) >> 6;
    const int64_t waves = (int64_t)gridDim.x * (kLcThreads >> 6);
    for (int64_t r = wave; r < B; r += waves) {
        float* row = H + r * ld;
        float m = -INFINITY;
        for (int c = lane; c < C; c += 64) m = fmaxf(m, row[c]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
        float sum = 0.0f;
        for (int c = lane; c < C; c += 64) sum += expf(row[c] - m);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
        const float inv = 1.0f / sum;
        for (int c = lane; c < C; c += 64) row[c] = expf(row[c] - m) * inv;
    }
}

// partial results of the split schedule: one grow-only buffer per device
struct Workspace {
    float* p = nullptr;
    size_t bytes = 0;
};
std::mutex g_ws_mu;
Workspace g_ws[64];

gp_status workspace(size_t bytes, float** out)
{
    int dev = 0;
    GP_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return fail(GP_ERR_UNSUPPORTED, "device ordinal %d not supported", dev);
    std::lock_guard<std::mutex> lk(g_ws_mu);
    Workspace& w = g_ws[dev];
    if (w.bytes < bytes) {
        if (w.p) GP_HIP(hipFree(w.p));  // waits for the device: no earlier launch still uses it
        w.p = nullptr, w.bytes = 0;
        GP_HIP(hipMalloc((void**)&w.p, bytes));
        w.bytes = bytes;
    }
    *out = w.p;
    return GP_OK;
}

int compute_units()
{
    static int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
            n = 256;
        return n;
    }();
    return cus;
}

template <typename T, int RB>
gp_status launch_mlp(const LcArgs& a, unsigned grid, hipStream_t stream)
{
    constexpr size_t lds = (size_t)32 * RB * kLd * sizeof(float);
    // the kernel's LDS tile is above the 64 KB a kernel gets by default: raise the limit
    // once per device (the attribute belongs to the device's copy of the kernel)
    static std::atomic<uint64_t> done{0};
    int dev = 0;
    GP_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return fail(GP_ERR_UNSUPPORTED, "device ordinal %d not supported", dev);
    if (!(done.load(std::memory_order_acquire) >> dev & 1)) {
        GP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gp_lc_mlp<T, RB>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        done.fetch_or(UINT64_C(1) << dev, std::memory_order_release);
    }
    profile_begin("gp_lc_mlp", stream);
    hipLaunchKernelGGL((gp_lc_mlp<T, RB>), dim3(grid), dim3(kLcThreads), lds, stream, a);
    profile_end(stream);
    GP_HIP(hipGetLastError());
    return GP_OK;
}

}  // namespace

gp_status lc_forward(const void* stack, int64_t ld, gp_dtype dtype, int64_t n, int32_t d, int32_t K, const int32_t* batch,
                     int64_t B, const float* gamma, const int32_t* depth, gp_comb comb, int32_t T, const float* const* W,
                     const int32_t* width, float* out, int64_t ldo, hipStream_t stream)
{
    if (!stack || !gamma || !W || !width || !out) return fail(GP_ERR_INVALID_ARG, "NULL argument");
    if (dtype != GP_F32 && dtype != GP_BF16) return fail(GP_ERR_INVALID_ARG, "unknown dtype %d", (int)dtype);
    if (comb != GP_COMB_SUM && comb != GP_COMB_CONCAT && comb != GP_COMB_MAX)
        return fail(GP_ERR_INVALID_ARG, "unknown combination %d", (int)comb);
    if (n < 1 || d < 1 || ld < d) return fail(GP_ERR_INVALID_ARG, "need n >= 1, d >= 1, ld >= d");
    if (K < 0 || K + 1 > kMaxHops) return fail(GP_ERR_UNSUPPORTED, "K = %d: 0 .. %d hops supported", K, kMaxHops - 1);
    if (T < 1 || T > kMaxLayers) return fail(GP_ERR_UNSUPPORTED, "T = %d: 1 .. %d layers supported", T, kMaxLayers);
    if (B < 0 || (!batch && B > n)) return fail(GP_ERR_INVALID_ARG, "B = %lld out of range", (long long)B);
    for (int t = 0; t < T; ++t) {
        if (!W[t]) return fail(GP_ERR_INVALID_ARG, "W[%d] is NULL", t);
        if (width[t] < 1 || width[t] > kPanel)
            return fail(GP_ERR_UNSUPPORTED, "layer %d is %d wide: 1 .. %d supported", t + 1, width[t], kPanel);
    }

    LcArgs a{};
    a.stack = stack, a.ld = ld, a.slab = n * ld, a.n = n, a.d = d;
    a.batch = batch, a.B = B, a.T = T;
    // branches in use, their depths and where their columns go
    int C = 0, total_width = 0;
    for (int k = 0; k <= K; ++k) {
        const int dk = depth ? depth[k] : T;
        if (dk < 0 || dk > T) return fail(GP_ERR_INVALID_ARG, "depth[%d] = %d outside 0 .. T", k, dk);
        a.gamma[k] = gamma[k];
        if (dk == 0) continue;
        const int wk = width[dk - 1];
        if (comb != GP_COMB_CONCAT && a.hops > 0 && wk != C)
            return fail(GP_ERR_INVALID_ARG, "branches of widths %d and %d cannot be summed or maximised", C, wk);
        C = std::max(C, wk);
        a.hop_of[a.hops] = k, a.depth[a.hops] = dk, a.out_off[a.hops] = comb == GP_COMB_CONCAT ? total_width : 0;
        total_width += wk;
        ++a.hops;
    }
    if (a.hops == 0) return fail(GP_ERR_INVALID_ARG, "every hop is left out (all depths are 0)");
    const int out_width = comb == GP_COMB_CONCAT ? total_width : C;
    if (ldo < out_width) return fail(GP_ERR_INVALID_ARG, "ldo < output width %d", out_width);
    if (B == 0) return GP_OK;
    a.direct = comb == GP_COMB_CONCAT || a.hops == 1;
    for (int t = 0; t < T; ++t) {
        a.W[t] = W[t], a.width[t] = width[t];
        a.wvec[t] = width[t] > 128 && width[t] % 2 == 0 && (uintptr_t)W[t] % 8 == 0;  // two tiles per wave, pairs aligned
    }
    const size_t esz = dtype == GP_F32 ? 4 : 2;
    a.xvec = ld % 4 == 0 && (uintptr_t)stack % (4 * esz) == 0;

    // One workgroup per (row tile, branch), so that a mini-batch of a few thousand rows
    // still fills the chip; the branches' results are then combined in hop order.
    // Tiles are 64 rows; 32 rows when even those give no more than one workgroup per CU
    // (the call then lasts as long as one work item, and a 32-row item is the shorter
    // one: 37 against 56 us at the paper's model shape; from two items per CU on, 64-row
    // items win because each weight is fetched once per 64 rows).  Large batches go
    // through in pieces that keep the partial results within a fixed size.
    int tm = (int)options().lc_tile_rows;
    if (tm == 0) tm = ((B + 31) / 32) * a.hops <= (int64_t)compute_units() ? 32 : 64;
    const int64_t piece = a.direct ? B : std::max<int64_t>(64, kWorkspaceBytes / ((int64_t)a.hops * C * 4) / 64 * 64);
    float* part = nullptr;
    if (!a.direct) {
        gp_status st = workspace((size_t)a.hops * std::min(piece, B) * C * sizeof(float), &part);
        if (st != GP_OK) return st;
    }
    for (int64_t b0 = 0; b0 < B; b0 += piece) {
        LcArgs p = a;
        p.B = std::min(piece, B - b0);
        p.batch = batch ? batch + b0 : nullptr;
        if (!batch) p.stack = static_cast<const char*>(stack) + (size_t)b0 * ld * esz, p.n = n - b0;
        if (a.direct)
            p.dst = out + b0 * ldo, p.ldd = ldo;
        else
            p.dst = part, p.ldd = C;
        const int64_t grid = (p.B + tm - 1) / tm * a.hops;
        if (grid > 0x7fffffffLL) return fail(GP_ERR_UNSUPPORTED, "batch too large for one launch");
        gp_status st;
        if (tm == 64)
            st = dtype == GP_F32 ? launch_mlp<float, 2>(p, (unsigned)grid, stream)
                                 : launch_mlp<unsigned short, 2>(p, (unsigned)grid, stream);
        else
            st = dtype == GP_F32 ? launch_mlp<float, 1>(p, (unsigned)grid, stream)
                                 : launch_mlp<unsigned short, 1>(p, (unsigned)grid, stream);
        if (st != GP_OK) return st;
        if (!a.direct) {
            const unsigned rgrid = (unsigned)std::min<int64_t>((p.B * C + kLcThreads - 1) / kLcThreads, 256 * 8);
            profile_begin("gp_lc_reduce", stream);
            hipLaunchKernelGGL(gp_lc_reduce, dim3(rgrid), dim3(kLcThreads), 0, stream, part, a.hops, comb == GP_COMB_MAX ? 1 : 0,
                               p.B, C, out + b0 * ldo, ldo);
            profile_end(stream);
            GP_HIP(hipGetLastError());
        }
    }
    return GP_OK;
}

}  // namespace gp

extern "C" gp_status gp_lc_forward(const void* stack, int64_t ld, gp_dtype dtype, int64_t n, int32_t d, int32_t K,
                                   const int32_t* batch, int64_t B, const float* gamma, int32_t T, const float* const* W,
                                   const int32_t* width, float* out, int64_t ldo, void* hip_stream)
{
    try {
        return gp::lc_forward(stack, ld, dtype, n, d, K, batch, B, gamma, nullptr, GP_COMB_SUM, T, W, width, out, ldo,
                              (hipStream_t)hip_stream);
    } catch (const std::exception& e) {
        return gp::fail(GP_ERR_OOM_HOST, "gp_lc_forward: %s", e.what());
    }
}

extern "C" gp_status gp_lc_softmax(float* H, int64_t B, int32_t C, int64_t ld, void* hip_stream)
{
    using namespace gp;
    if (!H) return fail(GP_ERR_INVALID_ARG, "NULL argument");
    if (B < 0 || C < 1 || ld < C) return fail(GP_ERR_INVALID_ARG, "need B >= 0, C >= 1, ld >= C");
    if (B == 0) return GP_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    const unsigned grid = (unsigned)std::min<int64_t>((B + 3) / 4, 256 * 16);
    profile_begin("gp_lc_softmax_rows", stream);
    hipLaunchKernelGGL(gp_lc_softmax_rows, dim3(grid), dim3(kLcThreads), 0, stream, H, B, (int)C, ld);
    profile_end(stream);
    GP_HIP(hipGetLastError());
    return GP_OK;
}

extern "C" gp_status gp_lc_forward_branches(const void* stack, int64_t ld, gp_dtype dtype, int64_t n, int32_t d, int32_t K,
                                            const int32_t* batch, int64_t B, const float* gamma, const int32_t* depth,
                                            gp_comb comb, int32_t T, const float* const* W, const int32_t* width, float* out,
                                            int64_t ldo, void* hip_stream)
{
    try {
        if (!depth) return gp::fail(GP_ERR_INVALID_ARG, "NULL argument");
        return gp::lc_forward(stack, ld, dtype, n, d, K, batch, B, gamma, depth, comb, T, W, width, out, ldo,
                              (hipStream_t)hip_stream);
    } catch (const std::exception& e) {
        return gp::fail(GP_ERR_OOM_HOST, "gp_lc_forward_branches: %s", e.what());
    }
}
