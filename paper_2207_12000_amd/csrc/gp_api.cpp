// C boundary glue: error text, options, accessors, kernel-timing hooks.
#include <cstdio>
#include <cstring>
#include <functional>

#include "gp_internal.h"

namespace gp {

static thread_local char g_err[512] = "";

gp_status fail(gp_status s, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return s;
}

Options& options()
{
    static Options o;
    return o;
}

// ---- profiling ------------------------------------------------------------
namespace {
struct Timed {
    std::string name;
    hipEvent_t a, b;
};
std::mutex g_prof_mu;
bool g_prof_on = false;
std::vector<Timed> g_prof;
// the launch a thread is in the middle of bracketing: one per calling thread, so that
// threads (and the streams they launch on) do not pair up each other's events
thread_local hipEvent_t g_open = nullptr;
thread_local const char* g_open_name = "";

void clear_profile()
{
    for (auto& t : g_prof) {
        (void)hipEventDestroy(t.a);
        (void)hipEventDestroy(t.b);
    }
    g_prof.clear();
}
}  // namespace

bool profiling_on() { return g_prof_on; }

void profile_begin(const char* name, hipStream_t stream)
{
    if (!g_prof_on) return;
    if (g_open) (void)hipEventDestroy(g_open);  // a begin without its end: dropped
    if (hipEventCreate(&g_open) != hipSuccess) {
        g_open = nullptr;
        return;
    }
    g_open_name = name;
    (void)hipEventRecord(g_open, stream);
}

void profile_end(hipStream_t stream)
{
    if (!g_open) return;
    hipEvent_t b;
    if (!g_prof_on || hipEventCreate(&b) != hipSuccess) {
        (void)hipEventDestroy(g_open);
        g_open = nullptr;
        return;
    }
    (void)hipEventRecord(b, stream);
    {
        std::lock_guard<std::mutex> lk(g_prof_mu);
        g_prof.push_back(Timed{g_open_name, g_open, b});
    }
    g_open = nullptr;
}

}  // namespace gp

using namespace gp;

extern "C" {

const char* gp_status_string(gp_status s)
{
    switch (s) {
    case GP_OK: return "GP_OK";
    case GP_ERR_INVALID_ARG: return "GP_ERR_INVALID_ARG";
    case GP_ERR_INDEX_RANGE: return "GP_ERR_INDEX_RANGE";
    case GP_ERR_OVERFLOW: return "GP_ERR_OVERFLOW";
    case GP_ERR_OOM_HOST: return "GP_ERR_OOM_HOST";
    case GP_ERR_OOM_DEVICE: return "GP_ERR_OOM_DEVICE";
    case GP_ERR_DEVICE: return "GP_ERR_DEVICE";
    case GP_ERR_UNSUPPORTED: return "GP_ERR_UNSUPPORTED";
    }
    return "GP_ERR_UNKNOWN";
}

const char* gp_last_error(void) { return g_err; }

gp_status gp_set_hbm_budget_bytes(int64_t bytes)
{
    if (bytes < 0) return fail(GP_ERR_INVALID_ARG, "HBM budget %lld is negative", (long long)bytes);
    options().hbm_budget_bytes = bytes;
    return GP_OK;
}

gp_status gp_set_option(const char* name, int64_t value)
{
    if (!name) return fail(GP_ERR_INVALID_ARG, "option name is NULL");
    if (!strcmp(name, "segment_edges")) {
        if (value != 0 && (value < 8 || value > 32768))
            return fail(GP_ERR_INVALID_ARG, "segment_edges must be 0 (automatic) or 8 .. 32768");
        options().segment_edges = value;
        return GP_OK;
    }
    if (!strcmp(name, "column_tile")) {
        if (value < 0) return fail(GP_ERR_INVALID_ARG, "column_tile must be >= 0");
        options().column_tile = value;
        return GP_OK;
    }
    if (!strcmp(name, "column_slices")) {
        if (value < 0 || value > 16) return fail(GP_ERR_INVALID_ARG, "column_slices must be 0 (automatic) or 1 .. 16");
        options().column_slices = value;
        return GP_OK;
    }
    if (!strcmp(name, "cache_schedule")) {
        if (value < 0 || value > 2) return fail(GP_ERR_INVALID_ARG, "cache_schedule must be 0 (automatic), 1 (on) or 2 (off)");
        options().cache_schedule = value;
        return GP_OK;
    }
    if (!strcmp(name, "split_records")) {
        if (value < 0 || value > 2) return fail(GP_ERR_INVALID_ARG, "split_records must be 0 (automatic), 1 (on) or 2 (off)");
        options().split_records = value;
        return GP_OK;
    }
    if (!strcmp(name, "lds_pass")) {
        if (value < 0 || value > 3)
            return fail(GP_ERR_INVALID_ARG,
                        "lds_pass must be 0 (automatic), 1 (wherever possible), 2 (never) or 3 (wherever possible, reads in "
                        "column-list order)");
        options().lds_pass = value;
        return GP_OK;
    }
    if (!strcmp(name, "hub_pass")) {
        if (value < 0 || value > 2) return fail(GP_ERR_INVALID_ARG, "hub_pass must be 0 (where it pays), 1 (always) or 2 (never)");
        options().hub_pass = value;
        return GP_OK;
    }
    if (!strcmp(name, "hub_sets")) {
        if (value < 0 || value > 65536) return fail(GP_ERR_INVALID_ARG, "hub_sets must be 0 (automatic) or 1 .. 65536");
        options().hub_sets = value;
        return GP_OK;
    }
    if (!strcmp(name, "plane_strips")) {
        if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8)
            return fail(GP_ERR_INVALID_ARG, "plane_strips must be 0 (automatic), 1, 2, 4 or 8");
        options().plane_strips = value;
        return GP_OK;
    }
    if (!strcmp(name, "device_plan_chunk")) {
        if (value < 0 || value > (INT64_C(1) << 31) - 1) return fail(GP_ERR_INVALID_ARG, "device_plan_chunk must be 0 .. 2^31 - 1");
        options().device_plan_chunk = value;
        return GP_OK;
    }
    if (!strcmp(name, "persistent_blocks")) {
        if (value < 0 || value > (1 << 20)) return fail(GP_ERR_INVALID_ARG, "persistent_blocks must be 0 .. 2^20");
        options().persistent_blocks = value;
        return GP_OK;
    }
    if (!strcmp(name, "lc_tile_rows")) {
        if (value != 0 && value != 32 && value != 64) return fail(GP_ERR_INVALID_ARG, "lc_tile_rows must be 0, 32 or 64");
        options().lc_tile_rows = value;
        return GP_OK;
    }
    return fail(GP_ERR_INVALID_ARG, "unknown option '%s'", name);
}

int64_t gp_get_option(const char* name)
{
    if (!name) return -1;
    if (!strcmp(name, "segment_edges")) return options().segment_edges;
    if (!strcmp(name, "column_tile")) return options().column_tile;
    if (!strcmp(name, "column_slices")) return options().column_slices;
    if (!strcmp(name, "persistent_blocks")) return options().persistent_blocks;
    if (!strcmp(name, "cache_schedule")) return options().cache_schedule;
    if (!strcmp(name, "device_plan_chunk")) return options().device_plan_chunk;
    if (!strcmp(name, "split_records")) return options().split_records;
    if (!strcmp(name, "lds_pass")) return options().lds_pass;
    if (!strcmp(name, "hub_pass")) return options().hub_pass;
    if (!strcmp(name, "hub_sets")) return options().hub_sets;
    if (!strcmp(name, "plane_strips")) return options().plane_strips;
    if (!strcmp(name, "lc_tile_rows")) return options().lc_tile_rows;
    if (!strcmp(name, "hbm_budget_bytes")) return options().hbm_budget_bytes;
    return -1;
}

gp_status gp_profile_enable(int32_t on)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    clear_profile();
    g_prof_on = on != 0;
    return GP_OK;
}

gp_status gp_profile_read(const char* prefix, int64_t* launches, double* total_ms)
{
    if (!launches || !total_ms) return fail(GP_ERR_INVALID_ARG, "output pointer is NULL");
    std::lock_guard<std::mutex> lk(g_prof_mu);
    const size_t plen = prefix ? strlen(prefix) : 0;
    int64_t cnt = 0;
    double ms = 0.0;
    for (auto& t : g_prof) {
        if (plen && t.name.compare(0, plen, prefix) != 0) continue;
        GP_HIP(hipEventSynchronize(t.b));
        float e = 0.f;
        GP_HIP(hipEventElapsedTime(&e, t.a, t.b));
        ms += e;
        ++cnt;
    }
    *launches = cnt;
    *total_ms = ms;
    return GP_OK;
}

int64_t gp_plan_num_nodes(const gp_plan* p) { return p ? p->n : 0; }
int64_t gp_plan_nnz(const gp_plan* p) { return p ? p->nnz : 0; }
int32_t gp_plan_num_blocks(const gp_plan* p) { return p ? p->num_blocks : 0; }
const int64_t* gp_plan_block_offsets(const gp_plan* p) { return p ? p->block_off.data() : nullptr; }
const int32_t* gp_plan_block_row_lo(const gp_plan* p) { return p ? p->block_row_lo.data() : nullptr; }
const int32_t* gp_plan_block_row_hi(const gp_plan* p) { return p ? p->block_row_hi.data() : nullptr; }
const int64_t* gp_plan_rowptr(const gp_plan* p) { return p ? p->rowptr.data() : nullptr; }
const int32_t* gp_plan_col(const gp_plan* p) { return p ? p->col.data() : nullptr; }
const int32_t* gp_plan_degree(const gp_plan* p) { return p ? p->deg.data() : nullptr; }
const float* gp_plan_dinv_sqrt(const gp_plan* p) { return p ? p->dinv_sqrt.data() : nullptr; }
const float* gp_plan_dinv(const gp_plan* p) { return p ? p->dinv.data() : nullptr; }
int64_t gp_plan_num_segments(const gp_plan* p) { return p ? (int64_t)p->segs.size() : 0; }
const void* gp_plan_segments(const gp_plan* p) { return p ? p->segs.data() : nullptr; }
const int64_t* gp_plan_segment_offsets(const gp_plan* p) { return p ? p->seg_off.data() : nullptr; }
int64_t gp_plan_num_partial_rows(const gp_plan* p) { return p ? p->num_slots : 0; }
int64_t gp_plan_segment_edges(const gp_plan* p) { return p ? p->segment_edges : 0; }

}  // extern "C"
