// gp: the hot pieces of the split schedule gathered from LDS (gfx950).
//
// Where the non-zero pattern has row clusters small enough, a cluster's source rows fit
// the 160 KB of LDS a compute unit has, four fp32 columns (16 bytes) at a time.  A
// workgroup then stages one such column strip of one cluster, pre-multiplied by the
// source's weight (Eq. 2's D^-1/2 on the right of A), and every hot record of the cluster
// gathers from there: one lane per record, one 16-byte LDS read per non-zero, the local
// source indices (16 bits) streamed from a list that is laid out so that a wavefront
// reads whole lines.  Random 16-byte reads come out of LDS at about 43 TB/s over the
// chip against 23 TB/s out of the L2s, and out-of-cluster traffic cannot evict anything.
//
// Work item = (cluster, strip).  Eight consecutive strips (one 128-byte line of a source
// row) form an octet; octet o belongs to XCD o % 8, so that the lines a strip fill pulls
// in serve the other strips of the octet from the same L2.  The workgroups of an XCD
// take items from that XCD's cursor (ctrl[0..8)); ctrl[8] counts finished workgroups and
// the last one zeroes all nine words, as in the segment kernel.
//
// Results: a record's sum goes where the record says: a partial-row slot (the fix-up pass
// joins partial rows as for any other launch), or the output row scaled by row_scale,
// after adding the one partial row the launch before this one left for it, if any.
// Summation order per record is fixed by the schedule (eight interleaved chains), so
// runs repeat bit for bit.
#include "gp_internal.h"

namespace gp {
namespace {

typedef float v4f_a16 __attribute__((ext_vector_type(4)));
typedef float v4f_a4 __attribute__((ext_vector_type(4), aligned(4)));  // 16-byte access from a dword boundary
typedef unsigned v4u __attribute__((ext_vector_type(4)));

constexpr int kLanes = 64;
constexpr int kStepBlock = 8;  // steps of a lane that lie together in the id list
constexpr int kAhead = 4;      // index loads in flight per lane

// 16 x the low / high 16 bits of a word: the byte offset of an LDS row from its index, in one
// instruction (a shift whose operand is read as a zero-extended half word)
__device__ inline unsigned low_half_times_16(unsigned packed)
{
    unsigned r;
    const unsigned four = 4;
    asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0"
        : "=v"(r)
        : "v"(four), "v"(packed));
    return r;
}
__device__ inline unsigned high_half_times_16(unsigned packed)
{
    unsigned r;
    const unsigned four = 4;
    asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1"
        : "=v"(r)
        : "v"(four), "v"(packed));
    return r;
}
// The row at a byte offset of the LDS.  The kernel declares no static LDS, so its dynamic
// array starts at LDS address 0 (launch_hot_lds checks the kernel's static size) and the
// offset is the address: no add per read.
typedef const __attribute__((address_space(3))) v4f_a16 lds_v4f;
__device__ inline v4f_a16 lds_row(unsigned byte_offset) { return *reinterpret_cast<lds_v4f*>(byte_offset); }

__global__ __launch_bounds__(1024) void gp_hop_cluster_lds(
    const int32_t* __restrict__ members, const int64_t* __restrict__ member_off, const int32_t* __restrict__ group_off,
    const LdsGroup* __restrict__ groups, const int32_t* __restrict__ rec_row, const int32_t* __restrict__ rec_slot,
    const uint16_t* __restrict__ ids, int num_clusters, const float* __restrict__ src_scale,
    const float* __restrict__ row_scale, const float* __restrict__ xin, int64_t ldin, float* __restrict__ xout, int64_t ldout,
    float* __restrict__ carry, int64_t carry_ld, int d, unsigned long long* __restrict__ ctrl, int lds_rows_max)
{
    // LDS: the strip's rows from byte 0 (an index times 16 is then the address itself), and
    // after them the word through which a workgroup learns its next item
    extern __shared__ __align__(16) char lds_raw[];
    v4f_a16* lds = reinterpret_cast<v4f_a16*>(lds_raw);
    unsigned long long& next_item = *reinterpret_cast<unsigned long long*>(lds_raw + (size_t)lds_rows_max * 16);
    // ... and the count of the item's record groups handed out so far (a wave's first group is its own number)
    int& groups_taken = *reinterpret_cast<int*>(lds_raw + (size_t)lds_rows_max * 16 + 8);

    const int lane = threadIdx.x & (kLanes - 1);
    const int wave = threadIdx.x / kLanes, waves = blockDim.x / kLanes;
    const int xcd = blockIdx.x & 7;
    const int64_t wgs = gridDim.x >> 3;  // workgroups of this XCD
    const int nstrips = (d + 3) / 4;
    const int opc = (nstrips + 7) / 8;  // octets per cluster
    const int64_t octets = (int64_t)num_clusters * opc;
    const int64_t my_octets = octets > xcd ? (octets - xcd + 7) / 8 : 0;
    const int64_t items = my_octets * 8;

    int64_t item = blockIdx.x >> 3;
    while (item < items) {
        if (threadIdx.x == 0) {
            next_item = (unsigned long long)wgs + atomicAdd(ctrl + xcd, 1ULL);
            groups_taken = waves;
        }
        const int64_t octet = (item >> 3) * 8 + xcd;
        const int c = (int)(octet / opc);
        const int strip = (int)(octet % opc) * 8 + (int)(item & 7);
        const int g_lo = group_off[c], g_hi = group_off[c + 1];
        const bool valid = strip < nstrips && g_hi > g_lo;
        const int col0 = min(strip * 4, d - 4);  // the last strip moves back to end with the row
        int m = 0;
        if (valid) {
            const int64_t m_lo = member_off[c];
            m = (int)(member_off[c + 1] - m_lo);
            const int32_t* mem = members + m_lo;
            // stage the strip: the cluster's rows, then zero rows up to the 16 that padding reads point at
            const int rows = (m + 15) / 16 * 16 + 16;
            for (int i0 = 0; i0 < rows; i0 += 4 * (int)blockDim.x) {
                int row[4];
                v4f_a16 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = i0 + u * (int)blockDim.x + (int)threadIdx.x;
                    row[u] = i < m ? mem[i] : -1;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    v[u] = v4f_a16{0.0f, 0.0f, 0.0f, 0.0f};
                    if (row[u] >= 0) v[u] = *reinterpret_cast<const v4f_a4*>(xin + (int64_t)row[u] * ldin + col0);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = i0 + u * (int)blockDim.x + (int)threadIdx.x;
                    if (src_scale && row[u] >= 0) v[u] *= src_scale[row[u]];
                    if (i < rows) lds[i] = v[u];
                }
            }
        }
        __syncthreads();
        const int64_t following = (int64_t)next_item;
        if (valid) {
            // groups are listed longest first: handing them out one by one keeps the waves level to the end
            for (int g = g_lo + wave; g < g_hi;) {
                const LdsGroup G = groups[g];
                // A lane's indices come kStepBlock (8, one 16-byte load) at a time.  Two register
                // sets of kAhead such loads alternate: while one is worked through the other is in
                // flight, which covers the latency of the list (it streams from memory) with four
                // waves per SIMD.  Loads past the end re-read the last block (never used).
                const v4u* ip = reinterpret_cast<const v4u*>(ids + G.id_off) + lane;
                const int nb = G.steps / kStepBlock;
                v4f_a16 acc[kStepBlock];
#pragma unroll
                for (int u = 0; u < kStepBlock; ++u) acc[u] = v4f_a16{0.0f, 0.0f, 0.0f, 0.0f};
                if (nb > 0) {
                    auto fetch = [&](v4u(&q)[kAhead], int b0) {
#pragma unroll
                        for (int i = 0; i < kAhead; ++i) q[i] = ip[(int64_t)min(b0 + i, nb - 1) * kLanes];
                    };
                    auto work = [&](const v4u(&q)[kAhead], int b0) {
#pragma unroll
                        for (int i = 0; i < kAhead; ++i) {
                            if (b0 + i < nb) {  // the same for every lane of the group
                                v4f_a16 x[kStepBlock];
#pragma unroll
                                for (int u = 0; u < 4; ++u) {
                                    x[2 * u] = lds_row(low_half_times_16(q[i][u]));
                                    x[2 * u + 1] = lds_row(high_half_times_16(q[i][u]));
                                }
#pragma unroll
                                for (int u = 0; u < kStepBlock; ++u) acc[u] += x[u];
                            }
                        }
                    };
                    v4u qa[kAhead], qb[kAhead];
                    fetch(qa, 0);
                    for (int b = 0; b < nb; b += 2 * kAhead) {
                        fetch(qb, b + kAhead);
                        work(qa, b);
                        fetch(qa, b + 2 * kAhead);
                        work(qb, b + kAhead);
                    }
                }
                const v4f_a16 sum = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
                const int row = rec_row[(int64_t)g * kLanes + lane];
                if (row >= 0) {
                    const int slot = rec_slot[(int64_t)g * kLanes + lane];
                    if (slot < 0) {
                        // the whole row, or all of it but one partial row that an earlier launch left in its slot
                        v4f_a16 total = sum;
                        if (slot < -1) total += *reinterpret_cast<const v4f_a4*>(carry + (int64_t)(-2 - slot) * carry_ld + col0);
                        const float s = row_scale ? row_scale[row] : 1.0f;
                        *reinterpret_cast<v4f_a4*>(xout + (int64_t)row * ldout + col0) = total * s;
                    } else {
                        *reinterpret_cast<v4f_a4*>(carry + (int64_t)slot * carry_ld + col0) = sum;
                    }
                }
                int taken = 0;
                if (lane == 0) taken = atomicAdd(&groups_taken, 1);
                g = g_lo + __builtin_amdgcn_readfirstlane(taken);
            }
        }
        __syncthreads();  // every read of this strip is done before the next one is staged
        item = following;
    }
    if (threadIdx.x == 0) {
        if (atomicAdd(ctrl + 8, 1ULL) == (unsigned long long)gridDim.x - 1) {
            __threadfence();
#pragma unroll
            for (int i = 0; i < 9; ++i) atomicExch(ctrl + i, 0ULL);
        }
    }
}

}  // namespace

gp_status launch_hot_lds(const HotLdsArgs& a, hipStream_t stream)
{
    if (a.d < 4 || a.num_clusters <= 0 || !a.ctrl || !a.xin || !a.xout)
        return fail(GP_ERR_INVALID_ARG, "LDS pass: needs at least four fp32 columns, clusters and a cursor buffer");
    if (a.max_members < 0 || a.max_members > kLdsMaxMembers)
        return fail(GP_ERR_INVALID_ARG, "LDS pass: a cluster of %d rows does not fit the LDS", a.max_members);
    if (a.carry && a.carry_ld < a.d) return fail(GP_ERR_INVALID_ARG, "LDS pass: partial rows narrower than d");
    const size_t shm = (size_t)lds_rows(a.max_members) * 16 + 16;  // the rows, the item word and the group count
    // the kernel addresses its dynamic LDS from 0: true as long as it has no static LDS before it
    hipFuncAttributes attr;
    GP_HIP(hipFuncGetAttributes(&attr, (const void*)gp_hop_cluster_lds));
    if (attr.sharedSizeBytes != 0)
        return fail(GP_ERR_UNSUPPORTED, "LDS pass: the kernel was built with %zu bytes of static LDS", (size_t)attr.sharedSizeBytes);
    // beyond 64 KB of dynamic LDS a kernel has to be cleared for the size (a host-side setting, per device)
    GP_HIP(hipFuncSetAttribute((const void*)gp_hop_cluster_lds, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm));
    // two workgroups of 512 per compute unit where two strips fit its LDS, else one of 1024
    const bool two = shm <= (size_t)kLdsBytesPerCu / 2 - 64;
    const dim3 grid(8 * 32 * (two ? 2 : 1)), block(two ? 512 : 1024);
    hipLaunchKernelGGL(gp_hop_cluster_lds, grid, block, shm, stream, a.members, a.member_off, a.group_off, a.groups, a.rec_row,
                       a.rec_slot, a.ids, a.num_clusters, a.src_scale, a.row_scale, a.xin, a.ldin, a.xout, a.ldout, a.carry,
                       a.carry_ld, a.d, a.ctrl, (int)lds_rows(a.max_members));
    GP_HIP(hipGetLastError());
    return GP_OK;
}

}  // namespace gp
