// so_grad_stats_static: the gradient statistics of Sec. 4.4 for callers that cannot allocate
// (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
//
// Everything the kernels need beyond the caller's inputs and output lives in ONE file-scope
// device array, `scratch` (64 KiB: the stage-1 partials of one call).  Every GPU the library
// runs on holds its own copy of that array, at its own address, until the process ends.  In
// host code the NAME of the array is only a stand-in, not a device address: the address is
// asked for once per device, with that device current (static_dev_state), and everything else
// -- kernel arguments included -- uses that pointer.  The bucket list travels by value in the
// kernel arguments, so no table is uploaded; no HIP allocation call is made anywhere here.
//
// Calls on one GPU share that GPU's array: two calls that overlap in time on different streams
// of one GPU race on the partials.  Nothing needs clearing between calls: every partial that
// stage 2 reads has been written by stage 1 of the same call.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstddef>
#include <cstdio>
#include <mutex>

#include "../../include/so_adam.h"
#include "so_kernels.hpp"
#include "so_static.hpp"

using namespace so;

namespace {

constexpr size_t kStaticPartials = 4096;    // workgroups of one stage-1 launch, at most
constexpr int kStaticMaxBuckets = SO_STATIC_MAX_BUCKETS;
constexpr int kMaxDevices = 64;
constexpr int kStatsBlocksPerCU = 16;       // same grid as so_grad_stats: same partials, same bits

}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticPartials * sizeof(Partial)];

namespace {

// Stage 1 with the bucket list in the kernel arguments; tile ranges are derived on the fly.
// Same tile order and per-workgroup arithmetic as grad_stats_kernel (both call stats_tile).
// The host passes only non-empty buckets and total_tiles = the sum of their tile counts, so
// the walk below never leaves the list.
struct StaticStatsTable {
    const uint16_t* g[kStaticMaxBuckets];
    uint64_t n[kStaticMaxBuckets];
};

template <int DT>
__global__ __launch_bounds__(kBlock) void grad_stats_static_kernel(StaticStatsTable tab, uint64_t total_tiles,
                                                                  double inv_scale,
                                                                  Partial* __restrict__ partials)
{
    uint32_t bk = 0;
    uint64_t begin = 0;
    uint64_t end = (tab.n[0] + kStatsTile - 1) / kStatsTile;
    double acc = 0.0;
    uint32_t bad = 0;
    for (uint64_t tile = blockIdx.x; tile < total_tiles; tile += gridDim.x) {
        while (tile >= end) {
            ++bk;
            begin = end;
            end += (tab.n[bk] + kStatsTile - 1) / kStatsTile;
        }
        stats_tile<DT>(tab.g[bk], tab.n[bk], (tile - begin) * (uint64_t)kStatsTile, acc, bad);
    }
    block_reduce<kBlock>(acc, bad);
    if (threadIdx.x == 0) {
        Partial out;
        out.sumsq = acc * (inv_scale * inv_scale);
        out.nonfinite = bad;
        partials[blockIdx.x] = out;
    }
}

// Stage 2 without a decision: sums the partials in the same fixed order as the other second
// stages and writes the four validation quantities in the layout of so_stats to caller-owned
// device memory.
struct StatsOut {
    double sumsq;
    double norm;
    uint64_t nonfinite;
    int32_t overflow;
    int32_t reserved;
};
static_assert(sizeof(StatsOut) == sizeof(so_stats) && offsetof(StatsOut, norm) == offsetof(so_stats, norm) &&
              offsetof(StatsOut, nonfinite) == offsetof(so_stats, nonfinite) &&
              offsetof(StatsOut, overflow) == offsetof(so_stats, overflow), "device mirror of so_stats");

__global__ __launch_bounds__(kFinalBlock) void stats_final_plain_kernel(const Partial* partials, uint64_t n,
                                                                       StatsOut* out)
{
    double acc;
    uint64_t bad;
    final_reduce(partials, n, acc, bad);
    if (threadIdx.x == 0) {
        StatsOut r;
        r.sumsq = acc;
        r.norm = sqrt(acc);
        r.nonfinite = bad;
        r.overflow = bad > 0 ? 1 : 0;
        r.reserved = 0;
        *out = r;
    }
}

struct StaticDev {
    void* ptr = nullptr;    // device address of `scratch` on this device
    int cus = 0;
    bool ready = false;
};
StaticDev g_static_dev[kMaxDevices];
std::mutex g_static_mu;
thread_local char g_err[256] = "";

so_status fail_static(so_status code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// Where device `device` (which must be current) keeps `scratch`: asked once, then remembered.
hipError_t static_dev_state(int device, const StaticDev** out)
{
    std::lock_guard<std::mutex> lock(g_static_mu);
    StaticDev& d = g_static_dev[device];
    if (!d.ready) {
        void* ptr = nullptr;
        hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        int cus = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device);
        if (e != hipSuccess) return e;
        d.ptr = ptr;
        d.cus = cus > 0 ? cus : 256;
        d.ready = true;
    }
    *out = &d;
    return hipSuccess;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

namespace so {

hipError_t static_setup(int device)
{
    if (device < 0 || device >= kMaxDevices) return hipSuccess;      // the entry point itself will refuse
    const StaticDev* sd = nullptr;
    return static_dev_state(device, &sd);
}

const char* static_last_error() { return g_err; }

}  // namespace so

extern "C" so_status so_grad_stats_static(const so_bucket* buckets, size_t nb, float inv_loss_scale,
                                          void* hip_stream, so_stats* out_device)
{
    g_err[0] = 0;
    if (!out_device) return fail_static(SO_ERR_INVALID_ARG, "out_device is NULL");
    if (!buckets && nb) return fail_static(SO_ERR_INVALID_ARG, "buckets is NULL");
    if (!std::isfinite(inv_loss_scale)) return fail_static(SO_ERR_INVALID_ARG, "inv_loss_scale must be finite");
    if ((reinterpret_cast<uintptr_t>(out_device) & 7u) != 0)
        return fail_static(SO_ERR_ALIGNMENT, "out_device must be 8-byte aligned");
    StaticStatsTable tab{};
    size_t live = 0;
    uint64_t tiles = 0;
    int dtype = SO_GRAD_BF16;
    for (size_t i = 0; i < nb; ++i) {
        const so_bucket* b = &buckets[i];
        if (b->grad_dtype != SO_GRAD_BF16 && b->grad_dtype != SO_GRAD_FP16)
            return fail_static(SO_ERR_INVALID_ARG, "bucket %zu: unknown grad_dtype %d", i, b->grad_dtype);
        if (b->grad_dtype != buckets[0].grad_dtype)
            return fail_static(SO_ERR_UNSUPPORTED, "all buckets of one call must share grad_dtype");
        dtype = b->grad_dtype;
        if (!b->n) continue;
        if (!b->grad) return fail_static(SO_ERR_INVALID_ARG, "bucket %zu: grad is NULL", i);
        if (!aligned16(b->grad)) return fail_static(SO_ERR_ALIGNMENT, "bucket %zu: grad must be 16-byte aligned", i);
        if (live >= (size_t)kStaticMaxBuckets)
            return fail_static(SO_ERR_UNSUPPORTED,
                               "so_grad_stats_static takes at most %d non-empty buckets per call (got more)",
                               kStaticMaxBuckets);
        tab.g[live] = (const uint16_t*)b->grad;
        tab.n[live] = b->n;
        ++live;
        tiles += (b->n + kStatsTile - 1) / kStatsTile;
    }
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices)
        return fail_static(SO_ERR_HIP, "no usable current HIP device");
    const StaticDev* sd = nullptr;
    hipError_t e = static_dev_state(device, &sd);
    if (e != hipSuccess)
        return fail_static(SO_ERR_HIP, "hipGetSymbolAddress(scratch) failed on device %d: %s", device,
                           hipGetErrorString(e));
    Partial* const partials = (Partial*)sd->ptr;      // the device address, never the array's name
    hipStream_t st = (hipStream_t)hip_stream;
    uint64_t grid = 0;
    if (tiles) {
        grid = (uint64_t)sd->cus * (uint64_t)kStatsBlocksPerCU;
        if (grid > tiles) grid = tiles;
        if (grid > kStaticPartials) grid = kStaticPartials;
        const double inv = (double)inv_loss_scale;
        if (dtype == SO_GRAD_FP16)
            hipLaunchKernelGGL((grad_stats_static_kernel<kGradFP16>), dim3((uint32_t)grid), dim3(kBlock), 0, st, tab,
                               tiles, inv, partials);
        else
            hipLaunchKernelGGL((grad_stats_static_kernel<kGradBF16>), dim3((uint32_t)grid), dim3(kBlock), 0, st, tab,
                               tiles, inv, partials);
        e = hipGetLastError();
        if (e != hipSuccess) return fail_static(SO_ERR_HIP, "statistics launch failed: %s", hipGetErrorString(e));
    }
    hipLaunchKernelGGL(stats_final_plain_kernel, dim3(1), dim3(kFinalBlock), 0, st, (const Partial*)partials, grid,
                       (StatsOut*)out_device);
    e = hipGetLastError();
    if (e != hipSuccess) return fail_static(SO_ERR_HIP, "reduction launch failed: %s", hipGetErrorString(e));
    return SO_OK;
}
