// HIP kernels for gfx950: the gather / scale / accumulate of one hop
// (Algorithm 1, the product S^(j) X^(i) and the accumulation over j), the
// fixed-order completion of rows that were cut, and the slot-0 copy.
//
// Work shape.  A wavefront (64 lanes) is divided into lane groups of G lanes.
// One group owns one record at a time: a segment (a run of at most a few hundred
// consecutive non-zeros of one destination row) and a column slice of it.  The
// lanes of a group span the slice's columns, each lane holding VPL vectors of VEC
// consecutive elements, so a gathered feature row is read by one coalesced
// 16-byte-per-lane load.  The group reads its column ids G at a time with one
// coalesced load (each lane a different id, plus that id's weight).  A group that
// is a whole wavefront lifts one id at a time into scalar registers and computes
// the row address there; narrower groups hand the ids round with in-group
// shuffles.  Eight rows are in flight per group, spread over four accumulators
// (also what keeps the fp32 sums short-chained).  No cross-lane reduction is
// needed: lanes own columns, not edges.
#include <hip/hip_runtime.h>

#include "gp_internal.h"

namespace gp {

namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;

// Vectors of N elements that need no more than 4-byte alignment: gfx950 loads and stores
// 8 and 16 bytes per lane from any dword boundary, so rows need not start on a multiple
// of the vector size (a row of 602 floats is 2408 bytes: every other row starts 8 bytes
// off a 16-byte boundary).
template <typename E, int N>
struct VecOf {
    typedef E type __attribute__((ext_vector_type(N), aligned(N * sizeof(E) < 4 ? N * sizeof(E) : 4)));
};
template <typename E>
struct VecOf<E, 1> {
    typedef E type;
};

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// round to nearest even; NaN stays NaN (quiet), infinities pass through
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Row<T, VEC>: one aligned VEC-element vector of a feature row, widened to fp32.
template <typename T, int VEC>
struct Row;

template <int VEC>
struct Row<float, VEC> {
    using V = typename VecOf<float, VEC>::type;
    __device__ static __forceinline__ V load_raw(const float* p) { return *reinterpret_cast<const V*>(p); }
    __device__ static __forceinline__ V zero_raw()
    {
        V z;
        if constexpr (VEC == 1) {
            z = 0.0f;
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) z[i] = 0.0f;
        }
        return z;
    }
    __device__ static __forceinline__ void widen(const V& t, float (&x)[VEC])
    {
        if constexpr (VEC == 1) {
            x[0] = t;
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) x[i] = t[i];
        }
    }
    __device__ static __forceinline__ void load(const float* p, float (&x)[VEC])
    {
        const V* q = reinterpret_cast<const V*>(p);
        const V t = *q;
        if constexpr (VEC == 1) {
            x[0] = t;
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) x[i] = t[i];
        }
    }
    __device__ static __forceinline__ void store(float* p, const float (&x)[VEC])
    {
        V t;
        if constexpr (VEC == 1) {
            t = x[0];
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) t[i] = x[i];
        }
        *reinterpret_cast<V*>(p) = t;
    }
    // finished output rows: nothing reads them again during this launch, so they are
    // stored with the streaming hint and leave the L2 to the gathered rows
    __device__ static __forceinline__ void store_stream(float* p, const float (&x)[VEC])
    {
        V t;
        if constexpr (VEC == 1) {
            t = x[0];
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) t[i] = x[i];
        }
        __builtin_nontemporal_store(t, reinterpret_cast<V*>(p));
    }
};

template <int VEC>
struct Row<uint16_t, VEC> {
    using V = typename VecOf<uint16_t, VEC>::type;
    __device__ static __forceinline__ V load_raw(const uint16_t* p) { return *reinterpret_cast<const V*>(p); }
    __device__ static __forceinline__ V zero_raw()
    {
        V z;
        if constexpr (VEC == 1) {
            z = 0;
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) z[i] = 0;
        }
        return z;
    }
    __device__ static __forceinline__ void widen(const V& t, float (&x)[VEC])
    {
        if constexpr (VEC == 1) {
            x[0] = bf16_to_f32(t);
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) x[i] = bf16_to_f32(t[i]);
        }
    }
    __device__ static __forceinline__ void load(const uint16_t* p, float (&x)[VEC])
    {
        const V* q = reinterpret_cast<const V*>(p);
        const V t = *q;
        if constexpr (VEC == 1) {
            x[0] = bf16_to_f32(t);
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) x[i] = bf16_to_f32(t[i]);
        }
    }
    __device__ static __forceinline__ void store(uint16_t* p, const float (&x)[VEC])
    {
        V t;
        if constexpr (VEC == 1) {
            t = f32_to_bf16(x[0]);
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) t[i] = f32_to_bf16(x[i]);
        }
        *reinterpret_cast<V*>(p) = t;
    }
    __device__ static __forceinline__ void store_stream(uint16_t* p, const float (&x)[VEC])
    {
        V t;
        if constexpr (VEC == 1) {
            t = f32_to_bf16(x[0]);
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) t[i] = f32_to_bf16(x[i]);
        }
        __builtin_nontemporal_store(t, reinterpret_cast<V*>(p));
    }
};

// ---------------------------------------------------------------------------
// one hop over a list of segments
// ---------------------------------------------------------------------------
typedef int v4i __attribute__((ext_vector_type(4)));

struct SegRegs {
    int64_t e0;  // first non-zero, relative to the column buffer
    int len, row, slot, slice;
};

__device__ __forceinline__ SegRegs unpack_segment(const v4i raw, int64_t col_base)
{
    SegRegs s;
    s.e0 = (((int64_t)((uint32_t)raw[1] & 0xFFu) << 32) | (int64_t)(uint32_t)raw[0]) - col_base;
    s.slice = (int)(((uint32_t)raw[1] >> 8) & 0xFFu);
    s.len = (int)((uint32_t)raw[1] >> 16);
    s.row = raw[2];
    s.slot = raw[3];
    return s;
}

// Lane groups are persistent.  Each of the 8 XCDs (workgroups are handed to them
// round-robin by id) walks a work list of its own: in the implicit form XCD x takes
// column slice x mod num_slices of every record, the XCDs that share a slice taking
// the records interleaved; in the explicit form the host has written one list per
// XCD (records [off[x], off[x+1]) of `segs`), each record naming its column slice, so
// that what an XCD's private L2 must hold at any time -- the source rows its current
// records draw from, one slice wide -- is the host's choice (Algorithm 1's cut into
// column blocks and edge blocks, used as a cache schedule).  Group q of an XCD takes
// positions q, q + stride, ... of that XCD's list.  The index stream is software
// pipelined in registers so that the only memory round trip a record waits for is
// its row gathers: the record two positions ahead and the first WIN column ids of the
// next one are requested while the current one is gathered.
// EDGE_W: 0 = every weight is 1; 1 = weight gathered from an n-vector by column id;
// 2 = weight read from a per-edge array laid out like the column list.
struct XcdLists {
    int64_t off[9];
    int explicit_lists;
};

// Implicit lists are walked in fixed shares: group q of an XCD takes positions q,
// q + groups, q + 2 groups, ...  Explicit lists are handed out in chunks of
// `chunk_records` consecutive positions from one cursor per XCD (ctrl[0..8)): with fixed
// shares the groups of an XCD drift apart (they do not run at the same speed) and the
// window of the list they work in -- what the L2 has to hold -- grows to many times the
// intended size.  Every group starts with the chunk of its own number and asks for the
// next one while it works; ctrl[8] counts the groups that are done and the last one puts
// all nine words back to zero, so the buffer is zero between launches.
template <typename T, int VEC, int G, int VPL, int EDGE_W>
__global__ __launch_bounds__(kThreads) void gp_hop_segments(const Segment* __restrict__ segs, int64_t num_segs,
                                                            const XcdLists lists, unsigned long long* __restrict__ ctrl,
                                                            int chunk_records, const int32_t* __restrict__ col,
                                                            int64_t col_base,
                                                            const float* __restrict__ edge_w,
                                                            const float* __restrict__ row_scale,
                                                            const T* __restrict__ xin, int64_t ldin,
                                                            T* __restrict__ xout, int64_t ldout,
                                                            float* __restrict__ carry, int64_t carry_ld, int d,
                                                            int num_slices, int slice_elems, float* __restrict__ comb,
                                                            int64_t ldc, float gamma, const float* __restrict__ planes,
                                                            int64_t num_pos, int run_log2, int plane_log2)
{
    constexpr int GPB = kThreads / G;
    constexpr int PF = G >= 32 ? 1 : 32 / G;  // column ids each lane prefetches per segment
    constexpr int WIN = PF * G;               // edges of a segment covered by the prefetch
    constexpr int U = VPL * VEC * (int)sizeof(T) <= 16 ? 8 : 4;  // row gathers in flight per group
    // interleaved fp32 accumulators per column (short summation chains); bf16 storage
    // tolerates longer chains and its 8-element vectors are register hungry
    constexpr int NACC = sizeof(T) == 2 ? 2 : 4;
    const int lane = threadIdx.x % G;
    const int xcd = blockIdx.x & 7;
    // This XCD's list: the record of position p < count is segs[place_of(p)].  Implicit lists: the
    // XCDs that share a slice take the records interleaved, in runs of 2^run_log2 consecutive records
    // (1 as a rule; 8 where records add plane entries: the entries of 8 consecutive records share their lines, which then
    // only one XCD asks for).
    int64_t base, count;
    int rstep, xcd_slice;
    if (lists.explicit_lists) {
        base = lists.off[xcd];
        count = lists.off[xcd + 1] - base;
        rstep = 1;
        xcd_slice = -1;  // every record names its slice
    } else {
        const int reps = 8 / num_slices;  // num_slices is 1, 2, 4 or 8 here
        base = xcd / num_slices;
        const int64_t run = (int64_t)1 << run_log2;
        const int64_t runs = (num_segs + run - 1) >> run_log2;                       // of all XCDs
        const int64_t mine = runs > base ? (runs - base + reps - 1) / reps : 0;      // of this one
        count = mine << run_log2;
        if (mine > 0 && base + (mine - 1) * reps == runs - 1) count -= runs * run - num_segs;  // the last run may be short
        rstep = reps;
        xcd_slice = xcd & (num_slices - 1);
    }
    const int64_t run_mask = ((int64_t)1 << run_log2) - 1;
    auto place_of = [&](int64_t p) -> int64_t {
        if (lists.explicit_lists) return base + p;
        return ((((p >> run_log2) * rstep) + base) << run_log2) + (p & run_mask);
    };
    // Positions of this group, in the order it visits them.  A chunk is chunk_records
    // consecutive positions; chunk numbers below `groups` are fixed (the group's own
    // number), later ones come from the XCD's cursor.  chunk_records == 0: fixed shares.
    const bool dynamic = chunk_records > 0;
    const int64_t csize = dynamic ? chunk_records : 1;
    const int64_t groups = (int64_t)(gridDim.x >> 3) * GPB;  // lane groups of this XCD
    auto take = [&]() -> int64_t {  // one atomic per group, result shared inside the group
        unsigned long long t = 0;
        if (lane == 0) t = atomicAdd(ctrl + xcd, 1ULL);
        const unsigned lo = __shfl((unsigned)t, 0, G), hi = __shfl((unsigned)(t >> 32), 0, G);
        return groups + (int64_t)(((unsigned long long)hi << 32) | lo);
    };
    int64_t chunk = (int64_t)(blockIdx.x >> 3) * GPB + threadIdx.x / G;
    int64_t pos = chunk * csize, pos_end = pos + csize;
    int64_t next_chunk = (dynamic && pos < count) ? take() : chunk + groups;
    auto advance = [&]() -> int64_t {  // the position after `pos`, or one past the end of the list
        if (pos >= count) return pos;
        if (++pos < pos_end) return pos;
        chunk = next_chunk;
        pos = chunk * csize;
        pos_end = pos + csize;
        next_chunk = (dynamic && pos < count) ? take() : chunk + groups;
        return pos;
    };

    const v4i* sp = reinterpret_cast<const v4i*>(segs);
    const v4i none = {0, 0, 0, -1};  // length 0: nothing to fetch
    int64_t t0 = pos, t1 = advance(), t2 = advance();
    SegRegs s0 = unpack_segment(t0 < count ? sp[place_of(t0)] : none, col_base);
    v4i raw1 = t1 < count ? sp[place_of(t1)] : none;
    int c0[PF];
    float w0[PF];
#pragma unroll
    for (int j = 0; j < PF; ++j) {
        const bool in = j * G + lane < s0.len;
        c0[j] = in ? col[s0.e0 + j * G + lane] : 0;
        w0[j] = (EDGE_W == 2 && in) ? edge_w[s0.e0 + j * G + lane] : 0.0f;
    }
    const int nvec = (d + VEC - 1) / VEC;
    const int slice_vecs = slice_elems / VEC;

    while (t0 < count) {
        // ---- requests for the segments to come -----------------------------------
        const int64_t t3 = advance();
        const SegRegs s1 = unpack_segment(raw1, col_base);
        const v4i raw2 = t2 < count ? sp[place_of(t2)] : none;
        int c1[PF];
        float w1[PF];
#pragma unroll
        for (int j = 0; j < PF; ++j) {
            const bool in = j * G + lane < s1.len;
            c1[j] = in ? col[s1.e0 + j * G + lane] : 0;
            w1[j] = (EDGE_W == 2 && in) ? edge_w[s1.e0 + j * G + lane] : 0.0f;
        }

        // ---- this segment ----------------------------------------------------------
        // A group that is a whole wavefront keeps the record in scalar registers.
        SegRegs r = s0;
        if constexpr (G == 64) {
            r.len = __builtin_amdgcn_readfirstlane(s0.len);
            r.row = __builtin_amdgcn_readfirstlane(s0.row);
            r.slot = __builtin_amdgcn_readfirstlane(s0.slot);
            r.slice = __builtin_amdgcn_readfirstlane(s0.slice);
            r.e0 = (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)((uint64_t)s0.e0 >> 32)) << 32) |
                             (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)s0.e0));
        }
        // This lane's vectors: vector j of a row covers columns [j*VEC, j*VEC + VEC), except
        // that the last vector of a row whose length is no multiple of VEC is moved back to
        // end with the row (its first `fresh` columns then repeat the vector before it: they
        // are computed twice, identically).  A lane past the slice's end is not live: it
        // follows the slice's first vector and stores nothing.
        const int slice = xcd_slice >= 0 ? xcd_slice : r.slice;
        const int vlo = slice * slice_vecs, vhi = min(nvec, vlo + slice_vecs);
        bool live[VPL];
        int coff[VPL], fresh[VPL];
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
            const int j = vlo + v * G + lane;
            live[v] = j < vhi;
            int c = (live[v] ? j : vlo) * VEC;
            fresh[v] = 0;
            if (c + VEC > d) {
                fresh[v] = c + VEC - d;
                c = d - VEC;
            }
            coff[v] = c;
        }
        float acc[NACC][VPL][VEC];
#pragma unroll
        for (int u = 0; u < NACC; ++u)
#pragma unroll
            for (int v = 0; v < VPL; ++v)
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[u][v][i] = 0.0f;

        const int len = r.len;
        if constexpr (G == 64) {
            // One row per load instruction: id and weight come out of the lane that holds them
            // into scalar registers and the row address is scalar arithmetic; lanes that are
            // not live take no part in the load.  Two sets of row registers alternate, so the
            // rows of the next US edges are on their way while the last US are added up, and
            // the ids of the next 64 edges are requested before the current 64 are gathered.
            using V = typename Row<T, VEC>::V;
            constexpr int US = VPL == 1 ? 8 : VPL == 2 ? 4 : 2;
            auto request = [&](V (&x)[US][VPL], float (&w)[US], int ids, float wts, int t, int cnt) {
                if (t + US <= cnt) {
#pragma unroll
                    for (int u = 0; u < US; ++u) {
                        const uint32_t c = (uint32_t)__builtin_amdgcn_readlane(ids, t + u);
                        w[u] = EDGE_W ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(wts), t + u)) : 1.0f;
                        const T* src = xin + (uint64_t)c * (uint64_t)ldin;
#pragma unroll
                        for (int v = 0; v < VPL; ++v)
                            x[u][v] = live[v] ? Row<T, VEC>::load_raw(src + coff[v]) : Row<T, VEC>::zero_raw();
                    }
                } else {
#pragma unroll
                    for (int u = 0; u < US; ++u) {
                        const bool on = t + u < cnt;  // the same for the whole wavefront
                        const uint32_t c = (uint32_t)__builtin_amdgcn_readlane(ids, on ? t + u : t);
                        w[u] = (EDGE_W && on) ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(wts), on ? t + u : t)) : 0.0f;
                        const T* src = xin + (uint64_t)c * (uint64_t)ldin;
#pragma unroll
                        for (int v = 0; v < VPL; ++v)
                            x[u][v] = (live[v] && (EDGE_W || on)) ? Row<T, VEC>::load_raw(src + coff[v]) : Row<T, VEC>::zero_raw();
                    }
                }
            };
            auto add_up = [&](const V (&x)[US][VPL], const float (&w)[US], int first_acc) {
#pragma unroll
                for (int u = 0; u < US; ++u)
#pragma unroll
                    for (int v = 0; v < VPL; ++v) {
                        float xf[VEC];
                        Row<T, VEC>::widen(x[u][v], xf);
                        float(&a)[VEC] = acc[(first_acc + u) % NACC][v];
#pragma unroll
                        for (int i = 0; i < VEC; ++i) a[i] = EDGE_W ? fmaf(w[u], xf[i], a[i]) : a[i] + xf[i];
                    }
            };
            int ids = c0[0];
            float wts = w0[0];
            if (EDGE_W == 1 && lane < len) wts = edge_w[ids];
            for (int base_e = 0; base_e < len; base_e += 64) {
                const int cnt = min(64, len - base_e);
                const int left = len - base_e - 64;  // edges past this batch
                int idn = 0;
                float wn = 0.0f;
                if (lane < left) {
                    idn = col[r.e0 + base_e + 64 + lane];
                    if (EDGE_W == 2) wn = edge_w[r.e0 + base_e + 64 + lane];
                }
                V xa[US][VPL], xb[US][VPL];
                float wa[US], wb[US];
                request(xa, wa, ids, wts, 0, cnt);
                for (int t = 0; t < cnt; t += 2 * US) {
                    const bool more = t + US < cnt;
                    if (more) request(xb, wb, ids, wts, t + US, cnt);
                    add_up(xa, wa, 0);
                    if (more) {
                        if (t + 2 * US < cnt) request(xa, wa, ids, wts, t + 2 * US, cnt);
                        add_up(xb, wb, US);
                    }
                }
                if (EDGE_W == 1 && lane < left) wn = edge_w[idn];
                ids = idn;
                wts = wn;
            }
        } else {
            // several lane groups per wavefront, each with a record of its own: ids and weights
            // are handed round inside the group
            auto gather_batch = [&](int ids, float wts, int cnt) {
                for (int t = 0; t < cnt; t += U) {
                    typename Row<T, VEC>::V x[U][VPL];  // rows stay in their stored form while in flight
                    float w[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        // lanes past cnt hold id 0 / weight 0; their rows are not read
                        const int c = __shfl(ids, t + u, G);
                        w[u] = EDGE_W ? __shfl(wts, t + u, G) : 1.0f;
                        const bool on = t + u < cnt;
                        const T* src = xin + (int64_t)c * ldin;
#pragma unroll
                        for (int v = 0; v < VPL; ++v) {
                            x[u][v] = (on && live[v]) ? Row<T, VEC>::load_raw(src + coff[v]) : Row<T, VEC>::zero_raw();
                        }
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u)
#pragma unroll
                        for (int v = 0; v < VPL; ++v) {
                            float xf[VEC];
                            Row<T, VEC>::widen(x[u][v], xf);
#pragma unroll
                            for (int i = 0; i < VEC; ++i)
                                acc[u % NACC][v][i] =
                                    EDGE_W ? fmaf(w[u], xf[i], acc[u % NACC][v][i]) : acc[u % NACC][v][i] + xf[i];
                        }
                }
            };
#pragma unroll
            for (int j = 0; j < PF; ++j) {
                const int cnt = min(G, len - j * G);
                if (cnt > 0) {
                    float wj = w0[j];
                    if (EDGE_W == 1 && lane < cnt) wj = edge_w[c0[j]];
                    gather_batch(c0[j], wj, cnt);
                }
            }
            for (int base_e = WIN; base_e < len; base_e += G) {  // the part of a long segment past the prefetch
                const int cnt = min(G, len - base_e);
                int id = 0;
                float wj = 0.0f;
                if (lane < cnt) {
                    id = col[r.e0 + base_e + lane];
                    if (EDGE_W == 1) wj = edge_w[id];
                    if (EDGE_W == 2) wj = edge_w[r.e0 + base_e + lane];
                }
                gather_batch(id, wj, cnt);
            }
        }

        const bool partial = r.slot >= 0;
        const float rs = (!partial && row_scale) ? row_scale[r.row] : 1.0f;
        // what an earlier launch has already added up for this record (the sums of its other non-zeros,
        // four columns to an entry, one plane per vector of the row) joins the sum here
        constexpr bool kCanAddPlanes = VEC == 4 || (VEC == 8 && sizeof(T) == 2);  // whole strips of four columns per vector
        bool planed = false;
        if constexpr (kCanAddPlanes) planed = planes != nullptr && (r.slice & kAddPlaneEntry) != 0;
        const int64_t place = place_of(t0);
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
            if (!live[v]) continue;
            float o[VEC];
            float before[VEC];
#pragma unroll
            for (int i = 0; i < VEC; ++i) before[i] = 0.0f;
            if constexpr (kCanAddPlanes) {
                if (planed) {  // 2^plane_log2 strips of a record lie together (eight: an octet, one 128-byte line)
                    // strip of the vector's first column (a last vector moved back ends with the row, as the last strip does)
                    const int t = (coff[v] + 3) >> 2;
#pragma unroll
                    for (int h = 0; h < VEC / 4; ++h) {  // (a vector of eight columns: two strips, maybe of two octets)
                        float part[4];
                        Row<float, 4>::load(planes + ((((int64_t)((t + h) >> plane_log2) * num_pos + place) << (2 + plane_log2)) +
                                                      (((t + h) & ((1 << plane_log2) - 1)) << 2)),
                                            part);
#pragma unroll
                        for (int i = 0; i < 4; ++i) before[h * 4 + i] = part[i];
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                float t = acc[0][v][i];
                if constexpr (NACC == 2) t += acc[1][v][i];
                if constexpr (NACC == 4) t = (t + acc[1][v][i]) + (acc[2][v][i] + acc[3][v][i]);
                o[i] = (t + before[i]) * rs;
            }
            if (partial) {
                Row<float, VEC>::store(carry + (int64_t)r.slot * carry_ld + coff[v], o);
            } else {
                if (xout) Row<T, VEC>::store_stream(xout + (int64_t)r.row * ldout + coff[v], o);
                if (comb) {  // running filter output: comb[row] += gamma * (A^^k X)[row], every column once
                    float* cp = comb + (int64_t)r.row * ldc + coff[v];
#pragma unroll
                    for (int i = 0; i < VEC; ++i)
                        if (i >= fresh[v]) cp[i] = fmaf(gamma, o[i], cp[i]);
                }
            }
        }

        s0 = s1;
        raw1 = raw2;
#pragma unroll
        for (int j = 0; j < PF; ++j) {
            c0[j] = c1[j];
            w0[j] = w1[j];
        }
        t0 = t1;
        t1 = t2;
        t2 = t3;
    }

    // every ticket this group asked for has been answered by now; the last group to get
    // here puts the cursors back to zero for the next launch
    if (dynamic && lane == 0) {
        const unsigned long long all_groups = (unsigned long long)gridDim.x * GPB;
        if (atomicAdd(ctrl + 8, 1ULL) == all_groups - 1) {
            __threadfence();
#pragma unroll
            for (int i = 0; i < 9; ++i) atomicExch(ctrl + i, 0ULL);
        }
    }
}

// a few 64-bit words put to zero (a fill kernel, so that a caller may capture it in a graph)
__global__ void gp_zero_words(unsigned long long* p, int count)
{
    if ((int)threadIdx.x < count) p[threadIdx.x] = 0ULL;
}

// per-edge weights for the sym operator: w[e] = dinv_sqrt[col[e]] (built once per plan)
__global__ __launch_bounds__(kThreads) void gp_fill_edge_weights(const int32_t* __restrict__ col,
                                                                 const float* __restrict__ by_col, float* __restrict__ w,
                                                                 int64_t nnz)
{
    for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < nnz; e += (int64_t)gridDim.x * kThreads)
        w[e] = by_col[col[e]];
}

// ---------------------------------------------------------------------------
// rows that were cut: add their partial rows in list order, scale, store
// ---------------------------------------------------------------------------
template <typename T, int VEC, int G, int VPL>
__global__ __launch_bounds__(kThreads) void gp_fixup_rows(const SplitRow* __restrict__ split, int64_t num_split,
                                                          const float* __restrict__ carry, int64_t carry_ld,
                                                          const float* __restrict__ row_scale, T* __restrict__ xout,
                                                          int64_t ldout, int d, float* __restrict__ comb, int64_t ldc,
                                                          float gamma)
{
    constexpr int GPB = kThreads / G;
    const int lane = threadIdx.x % G;
    const int64_t rid = (int64_t)blockIdx.x * GPB + threadIdx.x / G;
    if (rid >= num_split) return;
    const SplitRow sr = split[rid];
    const float rs = row_scale ? row_scale[sr.row] : 1.0f;
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
        int c0 = (v * G + lane) * VEC, fresh = 0;
        if (c0 >= d) continue;
        if (c0 + VEC > d) {  // last vector of a row whose length is no multiple of VEC: moved back to end with the row
            fresh = c0 + VEC - d;
            c0 = d - VEC;
        }
        float acc[kUnroll][VEC];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[u][i] = 0.0f;
        const float* p = carry + sr.first_slot * carry_ld + c0;
        for (int s = 0; s < sr.count; s += kUnroll) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                if (s + u < sr.count) {
                    float x[VEC];
                    Row<float, VEC>::load(p + (int64_t)(s + u) * carry_ld, x);
#pragma unroll
                    for (int i = 0; i < VEC; ++i) acc[u][i] += x[i];
                }
            }
        }
        float r[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) r[i] = ((acc[0][i] + acc[1][i]) + (acc[2][i] + acc[3][i])) * rs;
        if (xout) Row<T, VEC>::store_stream(xout + (int64_t)sr.row * ldout + c0, r);
        if (comb) {
            float* cp = comb + (int64_t)sr.row * ldc + c0;
#pragma unroll
            for (int i = 0; i < VEC; ++i)
                if (i >= fresh) cp[i] = fmaf(gamma, r[i], cp[i]);
        }
    }
}

// comb = gamma * X (fp32 accumulator of the filter output), or out = bf16(comb)
template <typename TI, typename TO>
__global__ __launch_bounds__(kThreads) void gp_scale_convert(const TI* __restrict__ src, int64_t lds, TO* __restrict__ dst,
                                                             int64_t ldd, int64_t n, int d, float gamma)
{
    const int64_t total = n * d;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (int64_t)gridDim.x * kThreads) {
        const int64_t r = i / d, c = i - r * d;
        float x[1];
        Row<TI, 1>::load(src + r * lds + c, x);
        x[0] *= gamma;
        Row<TO, 1>::store(dst + r * ldd + c, x);
    }
}

// ---------------------------------------------------------------------------
// slot 0: out[0] = X (the k = 0 term of the stack)
// ---------------------------------------------------------------------------
template <typename U>
__global__ __launch_bounds__(kThreads) void gp_copy_rows(const U* __restrict__ src, int64_t lds, U* __restrict__ dst,
                                                         int64_t ldd, int64_t n, int64_t w)
{
    // four independent elements per thread and trip: a small grid (the host-link copies
    // run on 16 workgroups beside the hop kernel) still keeps enough bytes in flight
    const int64_t total = n * w, step = (int64_t)gridDim.x * kThreads;
    int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    for (; i + 3 * step < total; i += 4 * step) {
        U v[4];
        int64_t o[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t e = i + u * step, r = e / w, c = e - r * w;
            v[u] = src[r * lds + c];
            o[u] = r * ldd + c;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) dst[o[u]] = v[u];
    }
    for (; i < total; i += step) {
        const int64_t r = i / w, c = i - r * w;
        dst[r * ldd + c] = src[r * lds + c];
    }
}

// ---- dispatch ---------------------------------------------------------------

}  // namespace

int vector_width(gp_dtype dtype, int32_t d, int64_t ld_a, int64_t ld_b, const void* pa, const void* pb)
{
    const int es = dtype == GP_F32 ? 4 : 2;
    int vec = 16 / es;  // 16 bytes per lane whenever rows are at least that long and start on dword boundaries
    while (vec > 1) {
        const int64_t need = std::min<int64_t>((int64_t)vec * es, 4);  // loads and stores want dword alignment at most
        const bool ok = vec <= d && (ld_a * es) % need == 0 && (ld_b * es) % need == 0 &&
                        ((uintptr_t)pa % need) == 0 && ((uintptr_t)pb % need) == 0;
        if (ok) break;
        vec /= 2;
    }
    return vec;
}

namespace {

template <typename T, int VEC, int G, int VPL>
gp_status launch_hop_t(const HopArgs& a, hipStream_t stream)
{
    constexpr int GPB = kThreads / G;
    XcdLists lists;
    int64_t longest = 0;  // records in the longest per-XCD list
    if (a.xcd_off) {
        for (int x = 0; x <= 8; ++x) lists.off[x] = a.xcd_off[x];
        for (int x = 0; x < 8; ++x) longest = std::max(longest, lists.off[x + 1] - lists.off[x]);
        lists.explicit_lists = 1;
    } else {
        for (int x = 0; x <= 8; ++x) lists.off[x] = 0;
        const int reps = 8 / a.num_slices;  // XCDs that share one slice
        longest = (a.num_segs + reps - 1) / reps;
        lists.explicit_lists = 0;
    }
    const int64_t chunks = (longest + GPB - 1) / GPB;  // workgroups per XCD that find work
    if (chunks == 0) return GP_OK;
    // explicit lists are handed out from cursors, in chunks of about 64 non-zeros
    const int chunk_records = a.xcd_off ? std::max(1, a.chunk_records) : 0;
    if (chunk_records && !a.ctrl) return fail(GP_ERR_INVALID_ARG, "hop launch without its cursor buffer");
    // persistent lane groups: as many workgroups as stay resident, fewer if the lists are short
    static const int resident = [] {
        int per_cu = 0, dev = 0;
        hipDeviceProp_t prop;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gp_hop_segments<T, VEC, G, VPL, 2>, kThreads, 0) !=
                hipSuccess ||
            hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess || per_cu <= 0)
            return 2048;
        return per_cu * prop.multiProcessorCount;
    }();
    int64_t persist = a.persistent_blocks > 0 ? a.persistent_blocks : resident;
    persist = (persist + 7) / 8 * 8;
    const int64_t blocks = std::min<int64_t>(persist, 8 * chunks);
    const dim3 grid((unsigned)blocks), block(kThreads);
    if (a.edge_w && a.edge_w_per_edge)
        hipLaunchKernelGGL((gp_hop_segments<T, VEC, G, VPL, 2>), grid, block, 0, stream, a.segs, a.num_segs, lists, a.ctrl, chunk_records, a.col,
                           a.col_base, a.edge_w, a.row_scale, (const T*)a.xin, a.ldin, (T*)a.xout, a.ldout, a.carry,
                           a.carry_ld, a.d, a.num_slices, a.slice_elems, a.comb, a.ldc, a.gamma, a.planes, a.num_pos, a.planes ? 3 : 0, a.plane_log2);
    else if (a.edge_w)
        hipLaunchKernelGGL((gp_hop_segments<T, VEC, G, VPL, 1>), grid, block, 0, stream, a.segs, a.num_segs, lists, a.ctrl, chunk_records, a.col,
                           a.col_base, a.edge_w, a.row_scale, (const T*)a.xin, a.ldin, (T*)a.xout, a.ldout, a.carry,
                           a.carry_ld, a.d, a.num_slices, a.slice_elems, a.comb, a.ldc, a.gamma, a.planes, a.num_pos, a.planes ? 3 : 0, a.plane_log2);
    else
        hipLaunchKernelGGL((gp_hop_segments<T, VEC, G, VPL, 0>), grid, block, 0, stream, a.segs, a.num_segs, lists, a.ctrl, chunk_records, a.col,
                           a.col_base, a.edge_w, a.row_scale, (const T*)a.xin, a.ldin, (T*)a.xout, a.ldout, a.carry,
                           a.carry_ld, a.d, a.num_slices, a.slice_elems, a.comb, a.ldc, a.gamma, a.planes, a.num_pos, a.planes ? 3 : 0, a.plane_log2);
    GP_HIP(hipGetLastError());
    return GP_OK;
}

template <typename T, int VEC, int G, int VPL>
gp_status launch_fixup_t(const FixupArgs& a, hipStream_t stream)
{
    constexpr int GPB = kThreads / G;
    const int64_t blocks = (a.num_split + GPB - 1) / GPB;
    if (blocks == 0) return GP_OK;
    if (blocks > INT32_MAX) return fail(GP_ERR_UNSUPPORTED, "%lld workgroups exceed the grid limit", (long long)blocks);
    hipLaunchKernelGGL((gp_fixup_rows<T, VEC, G, VPL>), dim3((unsigned)blocks), dim3(kThreads), 0, stream, a.split,
                       a.num_split, a.carry, a.carry_ld, a.row_scale, (T*)a.xout, a.ldout, a.d, a.comb, a.ldc, a.gamma);
    GP_HIP(hipGetLastError());
    return GP_OK;
}

// Shape of the lane groups for a row of `d` elements in vectors of `vec`:
// the smallest power-of-two group (8..64 lanes) that covers the row with one
// vector per lane, else 64 lanes with several vectors per lane (at most kMaxVpl).
constexpr int kMaxVpl = 8;
inline int max_vpl(int vec) { return std::min(kMaxVpl, 16 / vec); }
inline void group_shape(int32_t d, int vec, int& G, int& vpl)
{
    const int nvec = (d + vec - 1) / vec;
    G = 8;
    while (G < 64 && G < nvec) G *= 2;
    vpl = (nvec + G - 1) / G;
}

#define GP_SHAPE_CASES(FN, T, VEC)                                                  \
    if (G == 8 && vpl == 1) return FN<T, VEC, 8, 1>(a, stream);                     \
    if (G == 16 && vpl == 1) return FN<T, VEC, 16, 1>(a, stream);                   \
    if (G == 32 && vpl == 1) return FN<T, VEC, 32, 1>(a, stream);                   \
    if (G == 64 && vpl == 1) return FN<T, VEC, 64, 1>(a, stream);                   \
    if (G == 64 && vpl == 2) return FN<T, VEC, 64, 2>(a, stream);                   \
    if (G == 64 && vpl == 3) return FN<T, VEC, 64, 3>(a, stream);                   \
    if (G == 64 && vpl == 4) return FN<T, VEC, 64, 4>(a, stream);                   \
    if (G == 64 && vpl == 5) return FN<T, VEC, 64, 5>(a, stream);                   \
    if (G == 64 && vpl == 6) return FN<T, VEC, 64, 6>(a, stream);                   \
    if (G == 64 && vpl == 7) return FN<T, VEC, 64, 7>(a, stream);                   \
    if (G == 64 && vpl == 8) return FN<T, VEC, 64, 8>(a, stream);

#define GP_VEC_CASES(FN, T, MAXVEC)                                                 \
    if (vec == 1) { GP_SHAPE_CASES(FN, T, 1) }                                      \
    if (vec == 2) { GP_SHAPE_CASES(FN, T, 2) }                                      \
    if (vec == 4) { GP_SHAPE_CASES(FN, T, 4) }                                      \
    if (MAXVEC == 8 && vec == 8) { GP_SHAPE_CASES(FN, T, (MAXVEC == 8 ? 8 : 4)) }

}  // namespace

int max_columns_per_pass(int vec) { return 64 * max_vpl(vec) * vec; }

int hop_vector_width(const HopArgs& a)
{
    // carry rows are fp32 and 16-byte aligned by construction (carry_ld % 4 == 0)
    int vec = vector_width(a.dtype, a.d, a.ldin, a.xout ? a.ldout : a.ldin, a.xin, a.xout ? a.xout : a.xin);
    if (a.comb) vec = std::min(vec, vector_width(GP_F32, a.d, a.ldc, a.ldc, a.comb, a.comb));
    return vec;
}

// Column slices of the implicit work lists: each XCD's private L2 then sees only 1/S of
// every row and holds S times more distinct rows.  Measured on MI355X on graphs whose
// reuse comes from popular rows only: two slices pay for rows of 512 .. 1023 bytes (a slice
// is still >= 256 contiguous bytes); narrower slices lose more to the smaller requests and
// to the repeated per-record work than they gain in hits, and wider rows are best gathered whole.
int implicit_slices(const HopArgs& a, int vec)
{
    const int es = a.dtype == GP_F32 ? 4 : 2;
    const int nvec = (a.d + vec - 1) / vec;
    int S = (int)a.column_slices;
    if (S != 1 && S != 2 && S != 4 && S != 8) {
        const int64_t row_bytes = (int64_t)a.d * es;
        S = (row_bytes >= 512 && row_bytes < 1024) ? 2 : 1;
    }
    while (S > 1 && nvec < S) S /= 2;
    return S;
}

gp_status launch_hop(const HopArgs& a_in, hipStream_t stream)
{
    HopArgs a = a_in;
    const int vec = hop_vector_width(a);
    const int nvec = (a.d + vec - 1) / vec;
    if (a.xcd_off) {
        // explicit lists: the caller fixed the slices when it wrote the records
        if (a.num_slices < 1 || a.num_slices > 255 || a.slice_elems <= 0 || a.slice_elems % vec != 0 ||
            (int64_t)a.num_slices * a.slice_elems < a.d)
            return fail(GP_ERR_INVALID_ARG, "work lists do not fit the launch (slices %d x %d elements, d %d, vec %d)",
                        a.num_slices, a.slice_elems, a.d, vec);
    } else {
        a.num_slices = implicit_slices(a, vec);
        a.slice_elems = (nvec + a.num_slices - 1) / a.num_slices * vec;
    }
    if (a.planes && (a.plane_log2 < 0 || a.plane_log2 > 3))
        return fail(GP_ERR_INVALID_ARG, "plane entries: 1, 2, 4 or 8 strips of a record lie together");
    int G, vpl;
    group_shape(a.slice_elems, vec, G, vpl);
    if (vpl > max_vpl(vec)) return fail(GP_ERR_UNSUPPORTED, "d = %d needs column tiling (vec = %d)", a.d, vec);
    if (a.dtype == GP_F32) {
        GP_VEC_CASES(launch_hop_t, float, 4)
    } else {
        GP_VEC_CASES(launch_hop_t, uint16_t, 8)
    }
    return fail(GP_ERR_UNSUPPORTED, "no kernel for d = %d, vec = %d", a.d, vec);
}

gp_status launch_fixup(const FixupArgs& a, hipStream_t stream)
{
    // the fix-up reads fp32 carry rows and writes T rows: use the vector width both allow
    int vec = a.xout ? vector_width(a.dtype, a.d, a.ldout, a.ldout, a.xout, a.xout) : 4;
    if (a.comb) vec = std::min(vec, vector_width(GP_F32, a.d, a.ldc, a.ldc, a.comb, a.comb));
    if (vec > 4) vec = 4;
    while (vec > 1 && (a.carry_ld % vec != 0)) vec /= 2;
    int G, vpl;
    group_shape(a.d, vec, G, vpl);
    if (vpl > max_vpl(vec)) return fail(GP_ERR_UNSUPPORTED, "d = %d needs column tiling (vec = %d)", a.d, vec);
    if (a.dtype == GP_F32) {
        GP_VEC_CASES(launch_fixup_t, float, 4)
    } else {
        GP_VEC_CASES(launch_fixup_t, uint16_t, 4)
    }
    return fail(GP_ERR_UNSUPPORTED, "no fix-up kernel for d = %d, vec = %d", a.d, vec);
}

gp_status launch_scale_convert(const void* src, int64_t lds, gp_dtype src_type, void* dst, int64_t ldd, gp_dtype dst_type,
                               int64_t n, int32_t d, float gamma, hipStream_t stream)
{
    if (n == 0) return GP_OK;
    const int64_t blocks = std::min<int64_t>((n * d + kThreads - 1) / kThreads, 256 * 32);
    const dim3 grid((unsigned)blocks), block(kThreads);
    if (src_type == GP_F32 && dst_type == GP_F32)
        hipLaunchKernelGGL((gp_scale_convert<float, float>), grid, block, 0, stream, (const float*)src, lds, (float*)dst, ldd, n, d, gamma);
    else if (src_type == GP_BF16 && dst_type == GP_F32)
        hipLaunchKernelGGL((gp_scale_convert<uint16_t, float>), grid, block, 0, stream, (const uint16_t*)src, lds, (float*)dst, ldd, n, d, gamma);
    else if (src_type == GP_F32 && dst_type == GP_BF16)
        hipLaunchKernelGGL((gp_scale_convert<float, uint16_t>), grid, block, 0, stream, (const float*)src, lds, (uint16_t*)dst, ldd, n, d, gamma);
    else
        return fail(GP_ERR_UNSUPPORTED, "scale/convert between these types is not needed");
    GP_HIP(hipGetLastError());
    return GP_OK;
}

gp_status launch_zero_words(unsigned long long* p, int count, hipStream_t stream)
{
    if (count <= 0 || count > 64) return fail(GP_ERR_INVALID_ARG, "zero_words: count %d outside 1 .. 64", count);
    hipLaunchKernelGGL(gp_zero_words, dim3(1), dim3(64), 0, stream, p, count);
    GP_HIP(hipGetLastError());
    return GP_OK;
}

gp_status launch_fill_edge_weights(const int32_t* col, const float* by_col, float* w, int64_t nnz, hipStream_t stream)
{
    if (nnz == 0) return GP_OK;
    const int64_t blocks = std::min<int64_t>((nnz + kThreads - 1) / kThreads, 256 * 32);
    hipLaunchKernelGGL(gp_fill_edge_weights, dim3((unsigned)blocks), dim3(kThreads), 0, stream, col, by_col, w, nnz);
    GP_HIP(hipGetLastError());
    return GP_OK;
}

gp_status launch_copy_rows(const void* src, int64_t lds, void* dst, int64_t ldd, int64_t n, int32_t d, gp_dtype dtype,
                           hipStream_t stream, int max_blocks)
{
    if (n == 0) return GP_OK;
    const int es = dtype == GP_F32 ? 4 : 2;
    const int64_t row_bytes = (int64_t)d * es;
    // widest unit (16, 8, 4, 2 bytes) that divides the row, both strides and both bases
    int unit = 16;
    while (unit > es) {
        if (row_bytes % unit == 0 && (lds * es) % unit == 0 && (ldd * es) % unit == 0 && (uintptr_t)src % unit == 0 &&
            (uintptr_t)dst % unit == 0)
            break;
        unit /= 2;
    }
    const int64_t w = row_bytes / unit, total = n * w;
    const int64_t blocks = std::min<int64_t>((total + kThreads - 1) / kThreads, max_blocks > 0 ? max_blocks : 256 * 32);
    const dim3 grid((unsigned)blocks), block(kThreads);
    const int64_t s = lds * es / unit, t = ldd * es / unit;
    switch (unit) {
    case 16:
        hipLaunchKernelGGL(gp_copy_rows<uint4>, grid, block, 0, stream, (const uint4*)src, s, (uint4*)dst, t, n, w);
        break;
    case 8:
        hipLaunchKernelGGL(gp_copy_rows<uint2>, grid, block, 0, stream, (const uint2*)src, s, (uint2*)dst, t, n, w);
        break;
    case 4:
        hipLaunchKernelGGL(gp_copy_rows<uint32_t>, grid, block, 0, stream, (const uint32_t*)src, s, (uint32_t*)dst, t, n, w);
        break;
    default:
        hipLaunchKernelGGL(gp_copy_rows<uint16_t>, grid, block, 0, stream, (const uint16_t*)src, s, (uint16_t*)dst, t, n, w);
        break;
    }
    GP_HIP(hipGetLastError());
    return GP_OK;
}

}  // namespace gp
