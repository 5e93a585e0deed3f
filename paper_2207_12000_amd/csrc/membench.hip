// Stand-alone micro-benchmark (not part of libgp.so): streaming-read bandwidth and
// random row-gather bandwidth against the table's footprint, for 512-, 128- and
// 64-byte rows.  It measures the two ceilings the hop kernel lives between: rows
// served from the 4 MB per-XCD L2 and rows that miss it.
//   hipcc -O3 --offload-arch=gfx950 -o membench paper_2207_12000_amd/csrc/membench.hip && ./membench
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <cstdint>

#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)

__global__ __launch_bounds__(256) void stream_read(const float4* __restrict__ p, size_t n4, float* out)
{
    float4 acc = {0, 0, 0, 0};
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i + 3 * stride < n4; i += 4 * stride) {
        float4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
        acc.x += a.x + b.x + c.x + d.x; acc.y += a.y + b.y + c.y + d.y;
        acc.z += a.z + b.z + c.z + d.z; acc.w += a.w + b.w + c.w + d.w;
    }
    for (; i < n4; i += stride) { float4 a = p[i]; acc.x += a.x; acc.y += a.y; acc.z += a.z; acc.w += a.w; }
    if (acc.x + acc.y + acc.z + acc.w == 12345.678f) out[0] = 1.0f;
}

// each group of G lanes gathers rows of ROWB bytes (G*16 = ROWB); idx has `per` indices per group
template <int G, int U>
__global__ __launch_bounds__(256) void gather_rows(const float4* __restrict__ tab, const int* __restrict__ idx, int per,
                                                   float* out)
{
    const int lane = threadIdx.x % G;
    const size_t gid = ((size_t)blockIdx.x * 256 + threadIdx.x) / G;
    const int* my = idx + gid * per;
    float4 acc = {0, 0, 0, 0};
    for (int t = 0; t < per; t += U) {
        float4 x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = tab[(size_t)my[t + u] * G + lane];
#pragma unroll
        for (int u = 0; u < U; ++u) { acc.x += x[u].x; acc.y += x[u].y; acc.z += x[u].z; acc.w += x[u].w; }
    }
    if (acc.x + acc.y + acc.z + acc.w == 12345.678f) out[0] = 1.0f;
}

template <int G, int U>
double run_gather(const float4* tab, size_t rows, int per, size_t groups, int* d_idx, float* d_out)
{
    std::vector<int> h(groups * per);
    uint64_t s = 88172645463325252ull;
    for (auto& v : h) { s ^= s << 13; s ^= s >> 7; s ^= s << 17; v = (int)(s % rows); }
    CK(hipMemcpy(d_idx, h.data(), h.size() * 4, hipMemcpyHostToDevice));
    const int blocks = (int)(groups * G / 256);
    hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    for (int w = 0; w < 2; ++w) hipLaunchKernelGGL((gather_rows<G, U>), dim3(blocks), dim3(256), 0, 0, tab, d_idx, per, d_out);
    CK(hipEventRecord(a));
    const int reps = 5;
    for (int w = 0; w < reps; ++w) hipLaunchKernelGGL((gather_rows<G, U>), dim3(blocks), dim3(256), 0, 0, tab, d_idx, per, d_out);
    CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
    float ms; CK(hipEventElapsedTime(&ms, a, b));
    return (double)groups * per * G * 16 * reps / (ms * 1e-3) / 1e12;
}

int main()
{
    float* d_out; CK(hipMalloc(&d_out, 4));
    const size_t maxb = (size_t)4 << 30;
    float4* buf; CK(hipMalloc(&buf, maxb)); CK(hipMemset(buf, 0, maxb));
    hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    printf("stream read\n");
    for (size_t mb : {16, 32, 64, 128, 192, 256, 512, 1024, 4096}) {
        const size_t n4 = mb * (1 << 20) / 16;
        for (int blocks : {2048, 8192}) {
            for (int w = 0; w < 2; ++w) hipLaunchKernelGGL(stream_read, dim3(blocks), dim3(256), 0, 0, buf, n4, d_out);
            const int reps = mb <= 256 ? 20 : 5;
            CK(hipEventRecord(a));
            for (int w = 0; w < reps; ++w) hipLaunchKernelGGL(stream_read, dim3(blocks), dim3(256), 0, 0, buf, n4, d_out);
            CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
            float ms; CK(hipEventElapsedTime(&ms, a, b));
            printf("  %5zu MB blocks %5d : %.2f TB/s (%.1f us)\n", mb, blocks, (double)n4 * 16 * reps / (ms * 1e-3) / 1e12, ms * 1e3 / reps);
        }
    }
    const size_t groups = 1 << 18;  // groups, each `per` gathers
    const int per = 16;
    int* d_idx; CK(hipMalloc(&d_idx, groups * 8 * per * 4));
    printf("random row gather (uniform), TB/s of gathered bytes\n");
    for (size_t mb : {2, 8, 24, 64, 128, 512, 2048}) {
        const size_t bytes = mb << 20;
        printf("  table %5zu MB: 512B rows U4 %.2f  U8 %.2f  U16 %.2f | 128B rows U4 %.2f U8 %.2f | 64B rows U4 %.2f U8 %.2f\n", mb,
               run_gather<32, 4>(buf, bytes / 512, per, groups, d_idx, d_out),
               run_gather<32, 8>(buf, bytes / 512, per, groups, d_idx, d_out),
               run_gather<32, 16>(buf, bytes / 512, per, groups, d_idx, d_out),
               run_gather<8, 4>(buf, bytes / 128, per, groups * 4, d_idx, d_out),
               run_gather<8, 8>(buf, bytes / 128, per, groups * 4, d_idx, d_out),
               run_gather<4, 4>(buf, bytes / 64, per, groups * 8, d_idx, d_out),
               run_gather<4, 8>(buf, bytes / 64, per, groups * 8, d_idx, d_out));
    }
    return 0;
}
