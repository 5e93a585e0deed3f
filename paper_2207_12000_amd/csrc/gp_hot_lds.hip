// gp: the hot non-zeros of a hop gathered from LDS (gfx950).
//
// A short list of rows (at most 10,192) fits the 160 KB of LDS a compute unit has, four
// fp32 columns (16 bytes) at a time.  A list is a cluster of the non-zero pattern, served
// to the rows of that cluster, or the most popular rows of a graph without clusters,
// served to every set of rows.  A workgroup stages one such column strip of one list,
// pre-multiplied by the source's weight (Eq. 2's D^-1/2 on the right of A), and the hot
// part of every segment of the set -- the non-zeros whose source is on the list -- is
// added up from there: one lane per segment, one 16-byte LDS read per non-zero, the
// sources' places on the list (16 bits) streamed from an index list that is laid out so
// that a wavefront reads whole lines.  Random 16-byte reads come out of LDS at about
// 47 TB/s over the chip, conflict-free ones at about 90, against 23 TB/s out of the L2s.
//
// Work item = (set, strip).  Eight consecutive strips (one 128-byte line of a source row)
// form an octet, and the host deals every (set, octet) pair to one XCD (a list per XCD, set
// by set, each pair to the XCD with the least work so far), so that the lines a strip fill
// pulls in serve the other strips of the octet from the same L2 and all XCDs stream the same
// set's index list at about the same time.  The workgroups of an XCD take items from that
// XCD's cursor (ctrl[0..8)); ctrl[8] counts finished workgroups and the last one zeroes all
// nine words, as in the segment kernel.
//
// Results: for every position (a segment's place in the order this pass takes them: 64
// consecutive positions to a group, one per lane) and every strip, four sums -- a plane
// entry.  2^plane_log2 strips of a position lie together (eight: one 128-byte line per
// position and octet, which suits the segment kernel that reads them; fewer: a wavefront's
// store of 64 positions touches fewer lines, which suits this kernel where segments are
// short).  The segment kernel, which takes the segments' other non-zeros in the same
// order, adds them in.  Summation order per segment is fixed by the schedule (four
// interleaved chains), so runs repeat bit for bit.
#include "gp_internal.h"

namespace gp {
namespace {

typedef float v4f_a16 __attribute__((ext_vector_type(4)));
typedef float v4f_a4 __attribute__((ext_vector_type(4), aligned(4)));  // 16-byte access from a dword boundary
typedef unsigned v4u __attribute__((ext_vector_type(4)));

typedef unsigned short v4h_a2 __attribute__((ext_vector_type(4), aligned(2)));  // four bf16 from an element boundary

// four consecutive columns of a stored row as fp32: fp32 storage, or bf16 storage widened
__device__ inline v4f_a16 load_strip(const float* p) { return *reinterpret_cast<const v4f_a4*>(p); }
__device__ inline v4f_a16 load_strip(const uint16_t* p)
{
    const v4h_a2 h = *reinterpret_cast<const v4h_a2*>(p);
    v4f_a16 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = __uint_as_float((unsigned)h[i] << 16);
    return v;
}

constexpr int kLanes = 64;
constexpr int kStepBlock = 8;  // steps of a lane that lie together in the id list
constexpr int kAhead = 4;      // index loads in flight per lane
constexpr int kChains = 4;     // interleaved summation chains per lane and column

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

// The lists' rows strip by strip, one run of memory per (strip, list), each row times its
// source weight: packed[(t * num_members + i) * 4 ..] = w(row) * X[row][4 t .. 4 t + 4), row =
// members[i]; the last strip is moved back to end with the row.  A thread walks its row 16 bytes
// at a time (a line serves eight consecutive steps out of the caches) and a wavefront stores
// 64 consecutive entries, so that staging a strip later reads its 16 bytes per row once, not a
// line per row.
template <typename T>
__global__ __launch_bounds__(256) void gp_pack_strips(const int32_t* __restrict__ members, int64_t num_members,
                                                      const float* __restrict__ src_scale, const T* __restrict__ xin,
                                                      int64_t ldin, int d, float* __restrict__ packed)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= num_members) return;
    const int row = members[i];
    const float w = src_scale ? src_scale[row] : 1.0f;
    const T* src = xin + (int64_t)row * ldin;
    const int nstrips = (d + 3) / 4;
    for (int t0 = 0; t0 < nstrips; t0 += 8) {
        v4f_a16 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int t = min(t0 + u, nstrips - 1);
            v[u] = load_strip(src + min(t * 4, d - 4));
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (t0 + u < nstrips) *reinterpret_cast<v4f_a16*>(packed + ((int64_t)(t0 + u) * num_members + i) * 4) = v[u] * w;
    }
}

struct OctetLists {
    int64_t off[9];
};

template <typename T>
__global__ __launch_bounds__(1024) void gp_hop_cluster_lds(
    const int32_t* __restrict__ members, const int64_t* __restrict__ member_off, const int32_t* __restrict__ list_of_set,
    const int32_t* __restrict__ group_off, const int32_t* __restrict__ wave_cut,
    const LdsGroup* __restrict__ groups, const LdsOctet* __restrict__ octets, const OctetLists lists,
    const uint16_t* __restrict__ ids,
    const float* __restrict__ packed, int64_t num_members, const float* __restrict__ src_scale, const T* __restrict__ xin,
    int64_t ldin, float* __restrict__ planes, int64_t num_pos, int d, unsigned long long* __restrict__ ctrl, int lds_rows_max, int plane_log2)
{
    // LDS: the strip's rows from byte 0 (an index times 16 is then the address itself), and
    // after them the word through which a workgroup learns its next item
    extern __shared__ __align__(16) char lds_raw[];
    v4f_a16* lds = reinterpret_cast<v4f_a16*>(lds_raw);
    unsigned long long& next_item = *reinterpret_cast<unsigned long long*>(lds_raw + (size_t)lds_rows_max * 16);

    const int lane = threadIdx.x & (kLanes - 1);
    // (the same in every lane of a wave: said so, so that what is derived from it is scalar arithmetic and scalar loads)
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kLanes)), waves = blockDim.x / kLanes;
    const int xcd = blockIdx.x & 7;
    const int64_t wgs = gridDim.x >> 3;  // workgroups of this XCD
    const int nstrips = (d + 3) / 4;
    const LdsOctet* mine = octets + lists.off[xcd];
    const int64_t items = (lists.off[xcd + 1] - lists.off[xcd]) * 8;  // an octet = eight items, strip by strip

    int64_t item = blockIdx.x >> 3;
    while (item < items) {
        if (threadIdx.x == 0) next_item = (unsigned long long)wgs + atomicAdd(ctrl + xcd, 1ULL);
        const LdsOctet o = mine[item >> 3];
        const int c = o.set;
        const int strip = o.octet * 8 + (int)(item & 7);
        const int g_lo = group_off[c], g_hi = group_off[c + 1];
        const bool valid = strip < nstrips && g_hi > g_lo;
        int m = 0;
        if (valid) {
            const int list = list_of_set[c];
            const int64_t m_lo = member_off[list];
            m = (int)(member_off[list + 1] - m_lo);
            // stage the strip: the list's rows, then zero rows up to the 16 that padding reads point at.  The
            // rows come packed (one run of memory; lists that many sets share), or straight from the matrix,
            // 16 bytes of every row, times the row's source weight (a list that only this set stages).
            const int rows = (m + 15) / 16 * 16 + 16;
            const v4f_a16* src = reinterpret_cast<const v4f_a16*>(packed) + ((int64_t)strip * num_members + m_lo);
            const int32_t* mem = members + m_lo;
            const int col0 = min(strip * 4, d - 4);  // the last strip moves back to end with the row
            for (int i0 = 0; i0 < rows; i0 += 4 * (int)blockDim.x) {
                v4f_a16 v[4];
                if (packed) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int i = i0 + u * (int)blockDim.x + (int)threadIdx.x;
                        v[u] = i < m ? src[i] : v4f_a16{0.0f, 0.0f, 0.0f, 0.0f};
                    }
                } else {
                    int row[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int i = i0 + u * (int)blockDim.x + (int)threadIdx.x;
                        row[u] = i < m ? mem[i] : -1;
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        v[u] = v4f_a16{0.0f, 0.0f, 0.0f, 0.0f};
                        if (row[u] >= 0) v[u] = load_strip(xin + (int64_t)row[u] * ldin + col0);
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (src_scale && row[u] >= 0) v[u] *= src_scale[row[u]];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = i0 + u * (int)blockDim.x + (int)threadIdx.x;
                    if (i < rows) lds[i] = v[u];
                }
            }
        }
        __syncthreads();
        const int64_t following = (int64_t)next_item;
        if (valid) {
            // A wave takes a run of consecutive groups of the set; the host has cut the set's groups into 16
            // runs of about equal cost (wave_cut: reads, and a fixed cost per group).  The groups' indices lie one after the other
            // in the index list, so the run is one stream of blocks (8 reads of every lane = one 16-byte load per
            // lane), walked without a stop at the group boundaries.  Two register sets of kAhead blocks
            // alternate: while one is worked through the other is in flight, which covers the latency of the
            // list (it streams from memory) with four waves per SIMD.  Loads past the run's end re-read its
            // last block (never used).
            const int parts = kWaveCuts / waves;
            const int32_t* cut = wave_cut + (int64_t)c * (kWaveCuts + 1);
            int g = __builtin_amdgcn_readfirstlane(cut[wave * parts]);
            const int g_end = __builtin_amdgcn_readfirstlane(cut[(wave + 1) * parts]);
            if (g < g_end) {
                const int64_t k_end = groups[g_end].id_off >> 9;  // (the list of groups ends with a sentinel)
                int64_t k = groups[g].id_off >> 9;
                // The descriptors of the run's groups are read 64 at a time, one per lane, and handed out with
                // v_readlane: a scalar load per group would share its counter with the LDS reads, and every wait
                // for those would then also wait for a descriptor on its way from memory.
                int batch = g;  // group of lane 0's descriptor
                int d_steps = 0, d_count = 0;
                long long d_pos = 0;
                auto read_batch = [&](int g0) {
                    const LdsGroup G = groups[min(g0 + lane, g_end)];
                    d_steps = G.steps;
                    d_count = G.count;
                    d_pos = G.first_pos;
                    batch = g0;
                };
                auto blocks_of = [&](int gg) { return __builtin_amdgcn_readlane(d_steps, gg - batch) / kStepBlock; };
                // where this lane's sums of group gg go: the plane entry of (strip, position), 16 bytes; -1: nowhere
                auto entry_of = [&](int gg) -> int64_t {
                    const int count = __builtin_amdgcn_readlane(d_count, gg - batch);
                    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)d_pos, gg - batch);
                    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)((unsigned long long)d_pos >> 32), gg - batch);
                    const int64_t first = (int64_t)(((unsigned long long)hi << 32) | lo);
                    return lane < count ? ((((int64_t)(strip >> plane_log2) * num_pos + first + lane) << (2 + plane_log2)) +
                                           ((strip & ((1 << plane_log2) - 1)) << 2))
                                        : -1;
                };
                read_batch(g);
                int64_t k_group_end = k + blocks_of(g);
                int64_t entry = entry_of(g);
                const v4u* ip = reinterpret_cast<const v4u*>(ids) + lane;
                v4f_a16 acc[kChains];
#pragma unroll
                for (int u = 0; u < kChains; ++u) acc[u] = v4f_a16{0.0f, 0.0f, 0.0f, 0.0f};
                auto fetch = [&](v4u(&q)[kAhead], int64_t k0) {
#pragma unroll
                    for (int i = 0; i < kAhead; ++i) q[i] = ip[min(k0 + i, k_end - 1) * kLanes];
                };
                auto add_block = [&](const v4u& q) {
                    v4f_a16 x[kStepBlock];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        x[2 * u] = lds_row(low_half_times_16(q[u]));
                        x[2 * u + 1] = lds_row(high_half_times_16(q[u]));
                    }
#pragma unroll
                    for (int u = 0; u < kStepBlock; ++u) acc[u % kChains] += x[u];
                };
                auto work = [&](const v4u(&q)[kAhead], int64_t k0) {
                    if (k0 + kAhead < k_group_end) {  // no group ends in these blocks: straight through
#pragma unroll
                        for (int i = 0; i < kAhead; ++i) add_block(q[i]);
                        return;
                    }
                    // a group ends somewhere in these blocks (short segments: most of the time).  Two blocks of one
                    // group are still taken in one go, so that their sixteen reads overlap.
                    auto leave = [&]() {  // the group's last block is done: its sums leave, the next group begins
                        const v4f_a16 sum = (acc[0] + acc[1]) + (acc[2] + acc[3]);
                        if (entry >= 0) *reinterpret_cast<v4f_a16*>(planes + entry) = sum;
#pragma unroll
                        for (int u = 0; u < kChains; ++u) acc[u] = v4f_a16{0.0f, 0.0f, 0.0f, 0.0f};
                        ++g;
                        if (g < g_end) {
                            if (g - batch == kLanes) read_batch(g);
                            k_group_end += blocks_of(g);
                            entry = entry_of(g);
                        }
                    };
#pragma unroll
                    for (int i = 0; i < kAhead; i += 2) {
                        const bool has0 = k0 + i < k_end, has1 = k0 + i + 1 < k_end;  // the same for every lane of the wave
                        if (has1 && k0 + i + 1 != k_group_end) {  // both blocks belong to one group
                            add_block(q[i]);
                            add_block(q[i + 1]);
                            if (k0 + i + 2 == k_group_end) leave();
                        } else {
                            if (has0) {
                                add_block(q[i]);
                                if (k0 + i + 1 == k_group_end) leave();
                            }
                            if (has1) {
                                add_block(q[i + 1]);
                                if (k0 + i + 2 == k_group_end) leave();
                            }
                        }
                    }
                };
                v4u qa[kAhead], qb[kAhead];
                fetch(qa, k);
                for (; k < k_end; k += 2 * kAhead) {
                    fetch(qb, k + kAhead);
                    work(qa, k);
                    fetch(qa, k + 2 * kAhead);
                    work(qb, k + kAhead);
                }
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

gp_status prepare_hot_lds(int32_t max_members)
{
    if (max_members < 0 || max_members > kLdsMaxMembers) return fail(GP_ERR_INVALID_ARG, "LDS pass: a list of %d rows does not fit the LDS", max_members);
    const size_t shm = (size_t)lds_rows(max_members) * 16 + 16;
    for (const void* kernel : {(const void*)gp_hop_cluster_lds<float>, (const void*)gp_hop_cluster_lds<uint16_t>}) {
        // the kernel addresses its dynamic LDS from 0: true as long as it has no static LDS before it
        hipFuncAttributes attr;
        GP_HIP(hipFuncGetAttributes(&attr, kernel));
        if (attr.sharedSizeBytes != 0)
            return fail(GP_ERR_UNSUPPORTED, "LDS pass: the kernel was built with %zu bytes of static LDS", (size_t)attr.sharedSizeBytes);
        // beyond 64 KB of dynamic LDS a kernel has to be cleared for the size (a host-side setting, per device)
        GP_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm));
    }
    return GP_OK;
}

gp_status launch_pack_strips(const HotLdsArgs& a, hipStream_t stream)
{
    if (a.d < 4 || !a.xin || !a.packed || !a.members || a.num_members <= 0)
        return fail(GP_ERR_INVALID_ARG, "packing strips: needs at least four columns, lists and a buffer");
    const dim3 grid((unsigned)((a.num_members + 255) / 256)), block(256);
    if (a.dtype == GP_F32)
        hipLaunchKernelGGL(gp_pack_strips<float>, grid, block, 0, stream, a.members, a.num_members, a.src_scale, (const float*)a.xin, a.ldin,
                           a.d, a.packed);
    else
        hipLaunchKernelGGL(gp_pack_strips<uint16_t>, grid, block, 0, stream, a.members, a.num_members, a.src_scale, (const uint16_t*)a.xin,
                           a.ldin, a.d, a.packed);
    GP_HIP(hipGetLastError());
    return GP_OK;
}

gp_status launch_hot_lds(const HotLdsArgs& a, hipStream_t stream)
{
    if (a.d < 4 || a.num_sets <= 0 || !a.ctrl || !a.xin || !a.planes || a.num_pos <= 0 || a.num_members <= 0 || !a.octets || !a.octet_off)
        return fail(GP_ERR_INVALID_ARG, "LDS pass: needs at least four columns, record sets, lists, planes and a cursor buffer");
    if (a.plane_log2 < 0 || a.plane_log2 > 3) return fail(GP_ERR_INVALID_ARG, "LDS pass: 1, 2, 4 or 8 strips of a position lie together");
    if (a.dtype == GP_BF16 && a.d % 4 != 0) return fail(GP_ERR_INVALID_ARG, "LDS pass: bf16 rows need a multiple of four columns");
    if (a.max_members < 0 || a.max_members > kLdsMaxMembers)
        return fail(GP_ERR_INVALID_ARG, "LDS pass: a list of %d rows does not fit the LDS", a.max_members);
    const size_t shm = (size_t)lds_rows(a.max_members) * 16 + 16;  // the rows and the item word
    // two workgroups of 512 per compute unit where two strips fit its LDS, else one of 1024
    const bool two = shm <= (size_t)kLdsBytesPerCu / 2 - 64;
    const dim3 grid(8 * 32 * (two ? 2 : 1)), block(two ? 512 : 1024);
    OctetLists lists;
    for (int x = 0; x <= 8; ++x) lists.off[x] = a.octet_off[x];
    if (a.dtype == GP_F32)
        hipLaunchKernelGGL(gp_hop_cluster_lds<float>, grid, block, shm, stream, a.members, a.member_off, a.list_of_set, a.group_off,
                           a.wave_cut, a.groups, a.octets, lists, a.ids, a.packed, a.num_members, a.src_scale, (const float*)a.xin, a.ldin,
                           a.planes, a.num_pos, a.d, a.ctrl, (int)lds_rows(a.max_members), a.plane_log2);
    else
        hipLaunchKernelGGL(gp_hop_cluster_lds<uint16_t>, grid, block, shm, stream, a.members, a.member_off, a.list_of_set, a.group_off,
                           a.wave_cut, a.groups, a.octets, lists, a.ids, a.packed, a.num_members, a.src_scale, (const uint16_t*)a.xin,
                           a.ldin, a.planes, a.num_pos, a.d, a.ctrl, (int)lds_rows(a.max_members), a.plane_log2);
    GP_HIP(hipGetLastError());
    return GP_OK;
}

}  // namespace gp
