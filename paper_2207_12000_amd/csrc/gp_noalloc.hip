// gp_propagate_noalloc: the device-resident hop stack for callers that must not
// allocate (code under HIP graph capture, tight serving loops, harnesses that forbid
// hipMalloc).  Same kernels as gp_propagate; the scratch they need beyond the caller's
// operands -- the work cursors of the hop kernel and the partial rows of rows that were
// cut -- lives in a fixed array in device memory that every GPU the library runs on
// holds from load to process end.
#include <hip/hip_runtime.h>

#include "gp_internal.h"

namespace {

constexpr size_t kCtrlBytes = 256;                       // cursors: kHopCtrlWords 64-bit words, padded
constexpr size_t kPartialBytes = (size_t)64 << 20;       // partial rows: at most 64 MiB
constexpr size_t kScratchBytes = kCtrlBytes + kPartialBytes;
static_assert(gp::kHopCtrlWords * sizeof(unsigned long long) <= kCtrlBytes, "cursor words must fit their slot");

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
unsigned char* g_ptr[kMaxDevices] = {};  // device address of `scratch` on each device, once asked for

// The name `scratch` is a host-side stand-in: the array's address on the current device
// comes from the runtime, once per device, and only that address is handed to kernels.
gp_status scratch_on_current_device(unsigned char** out)
{
    int dev = -1;
    GP_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return gp::fail(GP_ERR_UNSUPPORTED, "device ordinal %d outside 0 .. %d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_ptr[dev]) {
        void* p = nullptr;
        GP_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return gp::fail(GP_ERR_DEVICE, "the scratch array has no address on device %d", dev);
        g_ptr[dev] = (unsigned char*)p;
    }
    *out = g_ptr[dev];
    return GP_OK;
}

}  // namespace

extern "C" int64_t gp_noalloc_partial_row_bytes(void) { return (int64_t)kPartialBytes; }

extern "C" gp_status gp_propagate_noalloc(const gp_plan* plan, const void* X, int64_t ldx, int32_t d, gp_dtype dtype,
                                          gp_agg agg, int32_t K, void* out_stack, int64_t ldo, void* hip_stream)
{
    using namespace gp;
    if (!plan) return fail(GP_ERR_INVALID_ARG, "plan is NULL");
    if (!X || !out_stack) return fail(GP_ERR_INVALID_ARG, "X or out_stack is NULL");
    if (d <= 0) return fail(GP_ERR_INVALID_ARG, "d = %d must be positive", d);
    if (K < 0) return fail(GP_ERR_INVALID_ARG, "K = %d is negative", K);
    if (ldx < d || ldo < d) return fail(GP_ERR_INVALID_ARG, "leading dimension smaller than d");
    if (dtype != GP_F32 && dtype != GP_BF16) return fail(GP_ERR_INVALID_ARG, "unknown dtype %d", (int)dtype);
    if (agg != GP_AGG_SYM && agg != GP_AGG_MEAN && agg != GP_AGG_SUM)
        return fail(GP_ERR_INVALID_ARG, "unknown aggregation %d", (int)agg);
    if (X == out_stack && ldx != ldo) return fail(GP_ERR_INVALID_ARG, "X aliases slot 0 but ldx != ldo");
    const int es = dtype == GP_F32 ? 4 : 2;
    if (((uintptr_t)X % es) || ((uintptr_t)out_stack % es))
        return fail(GP_ERR_INVALID_ARG, "X / out_stack not aligned to the element size");
    hipPointerAttribute_t ax, ao;
    if (hipPointerGetAttributes(&ax, X) != hipSuccess || hipPointerGetAttributes(&ao, out_stack) != hipSuccess) {
        (void)hipGetLastError();
        return fail(GP_ERR_INVALID_ARG, "X / out_stack is not device memory");
    }
    if (ax.type != hipMemoryTypeDevice || ao.type != hipMemoryTypeDevice)
        return fail(GP_ERR_INVALID_ARG, "gp_propagate_noalloc takes device-resident operands only");

    int cur = -1;
    GP_HIP(hipGetDevice(&cur));
    if (plan->dev.device < 0)
        return fail(GP_ERR_INVALID_ARG, "the plan is not on the device yet: gp_propagate uploads it on its first call");
    if (plan->dev.device != cur)
        return fail(GP_ERR_INVALID_ARG, "plan lives on device %d but device %d is current", plan->dev.device, cur);
    const int64_t carry_ld = ((int64_t)d + 3) / 4 * 4;
    const int64_t need = plan->num_slots * carry_ld * (int64_t)sizeof(float);
    if (need > (int64_t)kPartialBytes)
        return fail(GP_ERR_UNSUPPORTED,
                    "%lld partial rows of %d columns need %lld bytes of scratch; the fixed scratch holds %lld "
                    "(use gp_propagate, or plan with larger blocks / a larger segment_edges)",
                    (long long)plan->num_slots, d, (long long)need, (long long)kPartialBytes);
    unsigned char* base = nullptr;
    gp_status st = scratch_on_current_device(&base);
    if (st != GP_OK) return st;
    hipStream_t stream = (hipStream_t)hip_stream;
    unsigned long long* ctrl = (unsigned long long*)base;
    // the array keeps what the last call left: the cursors must start at zero (a fill
    // kernel, not a memset, so that the call can be captured); partial rows are written
    // before they are read
    if ((st = launch_zero_words(ctrl, kHopCtrlWords, stream)) != GP_OK) return st;
    return resident_hops(plan, X, ldx, d, dtype, agg, K, out_stack, ldo, stream, (float*)(base + kCtrlBytes), carry_ld, ctrl,
                         /*may_allocate=*/false);
}
