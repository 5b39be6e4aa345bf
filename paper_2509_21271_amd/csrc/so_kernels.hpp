// Device code of the fused Adam(W) bucket step for gfx950 (MI355X).
//
// Everything here is element-wise streaming work bound by HBM bandwidth: 28 bytes per
// parameter per step (paper Sec. 4.6 describes the CPU counterpart, GraceAdam; Sec. 4.5 the
// 16-bit <-> fp32 casts that are fused into this kernel; Sec. 4.4 the gradient norm and
// NaN/Inf validation that the speculative variant produces as a by-product).  No matrix
// cores are involved.
//
// Shape of the step kernel, chosen by measurement on MI355X: ONE single-wavefront workgroup
// per 256 elements (64 threads, one 16-byte access per lane per fp32 array, 8 bytes per
// 16-bit array), launched as a plain grid so that the hardware hands tiles to compute units in
// address order, and inside a wavefront one memory instruction at a time (load p, wait, load
// m, wait, ... store v, wait, store q).  Occupancy (32 wavefronts per compute unit) supplies
// the parallelism.  The chip-wide effect is a narrow window that sweeps the arrays front to
// back, with reads and writes of one array arriving as dense bursts; persistent grid-stride
// loops with several loads in flight per lane reach 5.0-5.5 TB/s on this part, this shape
// 6.3-6.7 TB/s.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace so {

constexpr int kVec = 4;                            // elements per lane per access
constexpr int kStepBlock = 64;                     // threads per step workgroup (1 wavefront)
constexpr int kTile = kStepBlock * kVec;           // elements per step workgroup: 256

constexpr int kBlock = 256;                        // threads per workgroup of the other kernels
constexpr int kStatsVec = 8;                       // 16-bit elements per lane per access (16 B)
constexpr int kStatsUnroll = 4;
constexpr int kStatsSub = kBlock * kStatsVec;      // 2048
constexpr int kStatsTile = kStatsSub * kStatsUnroll;   // 8192

constexpr int kGradBF16 = 0;
constexpr int kGradFP16 = 1;

// Forms of the step kernel (Sec. 4.4): the ordinary in-place step; the speculative ping-pong
// step, which writes the other state set and produces the gradient statistics as a by-product;
// and the speculative save step, which updates in place, writes the old state out and produces
// the statistics too.
constexpr int kModeSync = 0;
constexpr int kModePingPong = 1;
constexpr int kModeSave = 2;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Scalars of one step of one bucket (its parameter group), all derived on the host in double
// and rounded once to fp32.
struct StepConsts {
    float b1;           // beta1
    float c1;           // 1 - beta1 (exact in fp32 for beta1 in [0.5, 1))
    float b2;           // beta2
    float c2;           // 1 - beta2
    float rsb2;         // 1 / sqrt(1 - beta2^t)
    float eps;
    float step_size;    // lr / (1 - beta1^t)
    float lr_wd;        // lr * weight_decay (decoupled), 0 otherwise
    float wd_l2;        // weight_decay when folded into the gradient, 0 otherwise
    uint32_t lp_fp16;   // working copy: 0 = bf16, 1 = IEEE fp16
};

// One bucket as the step kernel sees it.  In-place steps have *_in == *_out.
struct StepEntry {
    const uint16_t* g;
    const float* p_in;
    const float* m_in;
    const float* v_in;
    float* p_out;
    float* m_out;
    float* v_out;
    uint16_t* q_out;
    float* p_save;          // SAVE mode only: old p, m, v are written here
    float* m_save;
    float* v_save;
    uint64_t n;
    uint64_t tile_begin;    // global index of the bucket's first tile
    StepConsts c;
};

struct StatsEntry {
    const uint16_t* g;
    uint64_t n;
    uint64_t tile_begin;
    uint64_t tile_end;
};

// Per-workgroup partial of the gradient statistics.
struct Partial {
    double sumsq;
    uint64_t nonfinite;
};

// Result slot written by the second reduction stage; layout mirrored by the host runtime.
struct DevResult {
    double sumsq;
    double norm;
    uint64_t nonfinite;
    int32_t overflow;
    int32_t action;
    double clip;
    float grad_scale;
    float next_loss_scale;
};

// Launch-wide parameters of the step kernel.
struct StepParams {
    float s;            // gradient multiplier (clip / loss_scale)
    uint32_t pad0;
    uint32_t nb;              // entries in the bucket table
    uint32_t uniform_tiles;   // > 0: 2-D launch, every bucket has this many tiles (the last may have fewer)
    uint32_t bucket_offset;   // 2-D launch: table index of grid row 0
    uint32_t reserved;
    uint64_t tile_offset;     // 1-D launch: tile index of workgroup 0
    const DevResult* guard;   // optional: take s and the skip flag from the GPU-side result
    Partial* partials;        // STATS: one slot per workgroup of this launch
    const StepConsts* consts; // optional: step scalars kept on the GPU (device-side step count)
};

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ float fp16_lo(uint32_t w)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xFFFFu));
}
__device__ __forceinline__ float fp16_hi(uint32_t w)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16));
}

template <int DT>
__device__ __forceinline__ void decode4(u32x2 w, float (&g)[4])
{
    if (DT == kGradBF16) {
        g[0] = bf16_lo(w.x); g[1] = bf16_hi(w.x); g[2] = bf16_lo(w.y); g[3] = bf16_hi(w.y);
    } else {
        g[0] = fp16_lo(w.x); g[1] = fp16_hi(w.x); g[2] = fp16_lo(w.y); g[3] = fp16_hi(w.y);
    }
}

template <int DT>
__device__ __forceinline__ float decode1(uint16_t h)
{
    return DT == kGradBF16 ? __uint_as_float((uint32_t)h << 16)
                           : (float)__builtin_bit_cast(_Float16, h);
}

// fp32 -> bf16 bits, round to nearest even; NaN stays a quiet NaN.
__device__ __forceinline__ uint32_t bf16_rne(float x)
{
    uint32_t u = __float_as_uint(x);
    uint32_t r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    uint32_t nan = (u >> 16) | 0x0040u;
    return (x != x) ? nan : r;
}

// fp32 -> IEEE fp16 bits, round to nearest even (hardware conversion).
__device__ __forceinline__ uint32_t fp16_rne(float x)
{
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)x);
}
__device__ __forceinline__ uint32_t lp_round(float x, uint32_t lp_fp16)
{
    return lp_fp16 ? fp16_rne(x) : bf16_rne(x);
}

// The Adam(W) update of one element.  Operation order is fixed and every product/sum is a
// single IEEE fp32 operation (compiled with contraction off; fused operations are spelled
// fmaf).  The parameter is rounded once: p - (lr*wd*p + step_size * m/denom).
__device__ __forceinline__ void adam_update(float g, float& p, float& m, float& v,
                                            const StepConsts& k, float s)
{
    float gs = fmaf(k.wd_l2, p, g * s);
    m = fmaf(k.b1, m, k.c1 * gs);
    v = fmaf(k.b2, v, (k.c2 * gs) * gs);
    float denom = fmaf(sqrtf(v), k.rsb2, k.eps);
    float upd = fmaf(k.lr_wd, p, k.step_size * (m / denom));
    p = p - upd;
}

__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_down(x, o, 64);
    return x;
}
__device__ __forceinline__ uint32_t wave_sum(uint32_t x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_down(x, o, 64);
    return x;
}
__device__ __forceinline__ unsigned long long wave_sum(unsigned long long x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_down(x, o, 64);
    return x;
}

// Wavefront totals for the single-wavefront workgroups (step kernel, gather kernel), where the
// reduction sits at the end of every wavefront's life and its latency costs occupancy: data
// movement by DPP row shifts inside the vector ALU instead of round trips through the LDS
// crossbar.  Four shifted adds (by 1, 2, 4, 8 lanes; lanes shifted in from outside a row of 16
// read zero) leave each row's sum in its last lane; the four row sums are read out and added
// in a fixed order.  Every lane returns the total.  All 64 lanes must be active.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_shift(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
template <int CTRL>
__device__ __forceinline__ double dpp_shift(double v)
{
    const uint64_t u = (uint64_t)__double_as_longlong(v);
    const uint32_t lo = dpp_shift<CTRL>((uint32_t)u), hi = dpp_shift<CTRL>((uint32_t)(u >> 32));
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}
__device__ __forceinline__ uint32_t lane_value(uint32_t v, int lane)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, lane);
}
__device__ __forceinline__ double lane_value(double v, int lane)
{
    const uint64_t u = (uint64_t)__double_as_longlong(v);
    const uint32_t lo = lane_value((uint32_t)u, lane), hi = lane_value((uint32_t)(u >> 32), lane);
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}
template <typename T>
__device__ __forceinline__ T wave_total(T x)
{
    x += dpp_shift<0x111>(x);       // row_shr:1
    x += dpp_shift<0x112>(x);       // row_shr:2
    x += dpp_shift<0x114>(x);       // row_shr:4
    x += dpp_shift<0x118>(x);       // row_shr:8
    return (lane_value(x, 15) + lane_value(x, 31)) + (lane_value(x, 47) + lane_value(x, 63));
}

// Fixed-order workgroup reduction: wavefront shuffles, then an LDS pass over the per-
// wavefront sums.  Thread 0 ends up with the totals.
template <int THREADS>
__device__ __forceinline__ void block_reduce(double& acc, uint32_t& bad)
{
    __shared__ double sh_acc[THREADS / 64];
    __shared__ uint32_t sh_bad[THREADS / 64];
    acc = wave_sum(acc);
    bad = wave_sum(bad);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { sh_acc[wave] = acc; sh_bad[wave] = bad; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double a = sh_acc[0];
        uint32_t b = sh_bad[0];
#pragma unroll
        for (int w = 1; w < THREADS / 64; ++w) { a += sh_acc[w]; b += sh_bad[w]; }
        acc = a;
        bad = b;
    }
}

// All arrays live in device (global) memory.  Pointers that reach the kernel inside a table
// entry carry no address-space information, so say it explicitly: this selects global_load /
// global_store instead of the slower generic (flat) forms.  Streaming hint: nothing is reused.
#define SO_GLOBAL __attribute__((address_space(1)))
template <typename T>
__device__ __forceinline__ T ld_stream(const T* p)
{
    return __builtin_nontemporal_load((const SO_GLOBAL T*)p);
}
template <typename T>
__device__ __forceinline__ void st_stream(T* p, T v)
{
    __builtin_nontemporal_store(v, (SO_GLOBAL T*)p);
}
template <typename T>
__device__ __forceinline__ T ld_plain(const T* p) { return *(const SO_GLOBAL T*)p; }
template <typename T>
__device__ __forceinline__ void st_plain(T* p, T v) { *(SO_GLOBAL T*)p = v; }

// Buffer-descriptor accesses of the step kernel.  The cache-policy bits were chosen by
// measurement: loads "nt" (streaming); stores that go back to the addresses just read (the
// in-place step) "nt sc1" -- 3 % faster than "nt" alone and 10 % faster than default policy on
// MI355X -- and the stores of the ping-pong step, which writes the other state set, "sc1"
// alone, which is 4 % faster there than "nt sc1" (6.38 against 6.11 TB/s over 1.3 B elements).
// (The save-mode copies, the restore pass and the gather kernel also write elsewhere, but
// measured 0.5-2 % better with "nt sc1".)
constexpr int kLoadPolicy = 2;              // bit 0: sc0, bit 1: nt, bit 4: sc1
constexpr int kStorePolicy = 2 | 16;
constexpr int kStorePolicyElsewhere = 16;
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t tile_rsrc(const void* base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 buf_ld4(rsrc_t r, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, kLoadPolicy);
}
__device__ __forceinline__ u32x2 buf_ld2(rsrc_t r, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, kLoadPolicy);
}
template <int POLICY = kStorePolicy>
__device__ __forceinline__ void buf_st4(rsrc_t r, uint32_t off, u32x4 v)
{
    __builtin_amdgcn_raw_buffer_store_b128(v, r, off, 0, POLICY);
}
template <int POLICY = kStorePolicy>
__device__ __forceinline__ void buf_st2(rsrc_t r, uint32_t off, u32x2 v)
{
    __builtin_amdgcn_raw_buffer_store_b64(v, r, off, 0, POLICY);
}

// Wait until every load and store this wavefront has issued is complete, and keep the
// compiler from moving memory operations across this point.
__device__ __forceinline__ void phase_fence()
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

template <bool STATS>
__device__ __forceinline__ void stat_accum(float g, double& acc, uint32_t& bad)
{
    if (STATS) {
        bool fin = __builtin_isfinite(g);
        double gd = fin ? (double)g : 0.0;
        acc = fma(gd, gd, acc);
        bad += fin ? 0u : 1u;
    }
}

// One tile (256 elements) of one bucket.  FULL tiles need no bounds checks.
template <int DT, int MODE, bool FULL>
__device__ __forceinline__ void step_tile(const StepEntry& e, uint64_t base, const StepParams& k,
                                          float s, double& acc, uint32_t& bad)
{
    constexpr bool STATS = MODE != kModeSync, SAVE = MODE == kModeSave;
    constexpr int ST = MODE == kModePingPong ? kStorePolicyElsewhere : kStorePolicy;
    const uint64_t off = base + threadIdx.x * kVec;
    if (FULL) {
        // One memory instruction at a time per wavefront, one array after the other, through
        // buffer descriptors that cover exactly this tile (anything outside would be dropped
        // by the hardware range check).
        const uint32_t vo4 = threadIdx.x * 16u, vo2 = threadIdx.x * 8u;
        const rsrc_t r_p = tile_rsrc(e.p_in + base, kTile * 4), r_m = tile_rsrc(e.m_in + base, kTile * 4);
        const rsrc_t r_v = tile_rsrc(e.v_in + base, kTile * 4), r_g = tile_rsrc(e.g + base, kTile * 2);
        u32x4 p = buf_ld4(r_p, vo4);
        phase_fence();
        u32x4 m = buf_ld4(r_m, vo4);
        phase_fence();
        u32x4 v = buf_ld4(r_v, vo4);
        phase_fence();
        u32x2 gw = buf_ld2(r_g, vo2);
        if (SAVE) {
            buf_st4(tile_rsrc(e.p_save + base, kTile * 4), vo4, p);
            phase_fence();
            buf_st4(tile_rsrc(e.m_save + base, kTile * 4), vo4, m);
            phase_fence();
            buf_st4(tile_rsrc(e.v_save + base, kTile * 4), vo4, v);
            phase_fence();
        }
        float g[4];
        decode4<DT>(gw, g);
        float pp[4] = {__uint_as_float(p.x), __uint_as_float(p.y), __uint_as_float(p.z), __uint_as_float(p.w)};
        float mm[4] = {__uint_as_float(m.x), __uint_as_float(m.y), __uint_as_float(m.z), __uint_as_float(m.w)};
        float vv[4] = {__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
        uint32_t qb[4];
        if (STATS) {                    // as stat_accum8: one finiteness test on the lane's sum
            double t = acc;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double gd = (double)g[j];
                t = fma(gd, gd, t);
            }
            if (__builtin_isfinite(t)) {
                acc = t;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) stat_accum<true>(g[j], acc, bad);
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            adam_update(g[j], pp[j], mm[j], vv[j], e.c, s);
            qb[j] = lp_round(pp[j], e.c.lp_fp16);
        }
        buf_st4<ST>(tile_rsrc(e.p_out + base, kTile * 4), vo4,
                    u32x4{__float_as_uint(pp[0]), __float_as_uint(pp[1]), __float_as_uint(pp[2]), __float_as_uint(pp[3])});
        phase_fence();
        buf_st4<ST>(tile_rsrc(e.m_out + base, kTile * 4), vo4,
                    u32x4{__float_as_uint(mm[0]), __float_as_uint(mm[1]), __float_as_uint(mm[2]), __float_as_uint(mm[3])});
        phase_fence();
        buf_st4<ST>(tile_rsrc(e.v_out + base, kTile * 4), vo4,
                    u32x4{__float_as_uint(vv[0]), __float_as_uint(vv[1]), __float_as_uint(vv[2]), __float_as_uint(vv[3])});
        phase_fence();
        buf_st2<ST>(tile_rsrc(e.q_out + base, kTile * 2), vo2, u32x2{qb[0] | (qb[1] << 16), qb[2] | (qb[3] << 16)});
    } else {
#pragma unroll 1
        for (int j = 0; j < kVec; ++j) {
            const uint64_t i = off + j;
            if (i < e.n) {
                float g = decode1<DT>(ld_plain(e.g + i));
                float p = ld_plain(e.p_in + i), m = ld_plain(e.m_in + i), v = ld_plain(e.v_in + i);
                if (SAVE) {
                    st_plain(e.p_save + i, p); st_plain(e.m_save + i, m); st_plain(e.v_save + i, v);
                }
                stat_accum<STATS>(g, acc, bad);
                adam_update(g, p, m, v, e.c, s);
                st_plain(e.p_out + i, p); st_plain(e.m_out + i, m); st_plain(e.v_out + i, v);
                st_plain(e.q_out + i, (uint16_t)lp_round(p, e.c.lp_fp16));
            }
        }
    }
}

// The fused step, one workgroup per tile.  Three launch forms:
//   SINGLE            1-D grid over the tiles of one bucket passed by value (tile_offset + x);
//   table, uniform    2-D grid: y = bucket (bucket_offset + y), x = tile inside the bucket --
//                     all buckets have the same tile count except a shorter last one, whose
//                     surplus workgroups exit at once;
//   table, ragged     1-D grid over all tiles, bucket found by bisection on tile_begin.
// A guarded step first looks at the GPU-side validation result: on overflow every workgroup
// exits before touching memory (a skipped iteration costs only the launch).
template <int DT, int MODE, bool SINGLE>
__global__ __launch_bounds__(kStepBlock) void adam_step_kernel(StepParams k, StepEntry single,
                                                              const StepEntry* __restrict__ table)
{
    float s = k.s;
    if (k.guard != nullptr) {
        if (k.guard->overflow) return;
        s = k.guard->grad_scale;
    }
    StepEntry e;
    uint64_t local;                    // tile index inside the bucket
    uint32_t slot = blockIdx.x;        // where this workgroup's statistics partial goes
    if (SINGLE) {
        e = single;
        local = k.tile_offset + blockIdx.x;
    } else if (k.uniform_tiles != 0) {
        e = table[k.bucket_offset + blockIdx.y];
        local = blockIdx.x;
        slot = blockIdx.y * gridDim.x + blockIdx.x;
    } else {
        const uint64_t tile = k.tile_offset + blockIdx.x;
        uint32_t lo = 0, hi = k.nb - 1;
        while (lo < hi) {
            const uint32_t mid = (lo + hi + 1) >> 1;
            if (table[mid].tile_begin <= tile) lo = mid; else hi = mid - 1;
        }
        e = table[lo];
        local = tile - e.tile_begin;
    }
    if (k.consts != nullptr) {         // scalars of this step come from the GPU-side train state
        const uint32_t lp = e.c.lp_fp16;
        e.c = *k.consts;
        e.c.lp_fp16 = lp;
    }
    const uint64_t base = local * (uint64_t)kTile;
    double acc = 0.0;
    uint32_t bad = 0;
    if (base < e.n) {
        if (base + kTile <= e.n) step_tile<DT, MODE, true>(e, base, k, s, acc, bad);
        else                     step_tile<DT, MODE, false>(e, base, k, s, acc, bad);
    }
    if (MODE != kModeSync) {
        acc = wave_total(acc);
        if (__any(bad != 0)) bad = wave_total(bad);         // rare: skip the second reduction otherwise
        if (threadIdx.x == 0) {
            const double sd = (double)s;
            Partial out;
            out.sumsq = acc * (sd * sd);
            out.nonfinite = bad;
            k.partials[slot] = out;
        }
    }
}

// Statistics of the eight gradients packed in one 16-byte vector.  The sum of squares is
// first formed as if all eight were finite; an Inf or NaN among them makes exactly that sum
// non-finite (squares of finite 16-bit values are far inside the range of a double), and only
// then the eight are gone through one by one.
template <int DT>
__device__ __forceinline__ void stat_accum8(u32x4 w, double& acc, uint32_t& bad)
{
    float g[8];
    decode4<DT>(u32x2{w.x, w.y}, *(float(*)[4])&g[0]);
    decode4<DT>(u32x2{w.z, w.w}, *(float(*)[4])&g[4]);
    double t = acc;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const double gd = (double)g[j];
        t = fma(gd, gd, t);
    }
    if (__builtin_isfinite(t)) {          // the common case: all eight finite
        acc = t;
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) stat_accum<true>(g[j], acc, bad);
    }
}

// One 8192-element tile of the stage-1 statistics, all 256 threads of a workgroup: 16-byte
// loads of 8 gradients per lane, four in flight.
template <int DT>
__device__ __forceinline__ void stats_tile(const uint16_t* g, uint64_t n, uint64_t base, double& acc,
                                           uint32_t& bad)
{
    const uint32_t lane_off = threadIdx.x * kStatsVec;
    if (base + kStatsTile <= n) {
        u32x4 w[kStatsUnroll];
#pragma unroll
        for (int u = 0; u < kStatsUnroll; ++u)
            w[u] = ld_stream((const u32x4*)(g + base + (uint64_t)u * kStatsSub + lane_off));
#pragma unroll
        for (int u = 0; u < kStatsUnroll; ++u) stat_accum8<DT>(w[u], acc, bad);
    } else {
#pragma unroll 1
        for (int u = 0; u < kStatsUnroll; ++u) {
#pragma unroll 1
            for (int j = 0; j < kStatsVec; ++j) {
                const uint64_t i = base + (uint64_t)u * kStatsSub + lane_off + j;
                if (i < n) stat_accum<true>(decode1<DT>(ld_plain(g + i)), acc, bad);
            }
        }
    }
}

// Stage 1 of the standalone gradient statistics (Sec. 4.4: global norm and NaN/Inf check).
// Grid-stride over the tiles of all buckets, interleaved (workgroup b takes tiles b, b+G, ...);
// one partial per workgroup.
template <int DT>
__global__ __launch_bounds__(kBlock) void grad_stats_kernel(const StatsEntry* __restrict__ table,
                                                           uint64_t total_tiles, double inv_scale,
                                                           Partial* __restrict__ partials)
{
    StatsEntry e = table[0];
    uint32_t bk = 0;
    double acc = 0.0;
    uint32_t bad = 0;
    for (uint64_t tile = blockIdx.x; tile < total_tiles; tile += gridDim.x) {
        while (tile >= e.tile_end) { ++bk; e = table[bk]; }
        stats_tile<DT>(e.g, e.n, (tile - e.tile_begin) * (uint64_t)kStatsTile, acc, bad);
    }
    block_reduce<kBlock>(acc, bad);
    if (threadIdx.x == 0) {
        Partial out;
        out.sumsq = acc * (inv_scale * inv_scale);
        out.nonfinite = bad;
        partials[blockIdx.x] = out;
    }
}

constexpr int kFinalBlock = 1024;

__device__ __forceinline__ void final_reduce(const Partial* partials, uint64_t n, double& acc,
                                             uint64_t& bad)
{
    __shared__ double sh_acc[kFinalBlock / 64];
    __shared__ uint64_t sh_bad[kFinalBlock / 64];
    acc = 0.0;
    bad = 0;
    for (uint64_t i = threadIdx.x; i < n; i += kFinalBlock) {
        acc += partials[i].sumsq;
        bad += partials[i].nonfinite;
    }
    acc = wave_sum(acc);
    bad = wave_sum((unsigned long long)bad);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { sh_acc[wave] = acc; sh_bad[wave] = bad; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double a = sh_acc[0];
        uint64_t b = sh_bad[0];
        for (int w = 1; w < kFinalBlock / 64; ++w) { a += sh_acc[w]; b += sh_bad[w]; }
        acc = a;
        bad = b;
    }
}

// (The non-template kernels of this header are `static`: more than one source file of the
// library includes it.)
// Intermediate stage for long partial lists: workgroup b sums in[b*kReduceSpan ..
// (b+1)*kReduceSpan) in a fixed order into out[b].  in and out must not overlap.
constexpr uint64_t kReduceSpan = 4096;
static __global__ __launch_bounds__(kFinalBlock) void reduce_partials_kernel(const Partial* __restrict__ in,
                                                                     uint64_t n, Partial* __restrict__ out)
{
    const uint64_t lo = (uint64_t)blockIdx.x * kReduceSpan;
    const uint64_t len = n - lo < kReduceSpan ? n - lo : kReduceSpan;
    double acc;
    uint64_t bad;
    final_reduce(in + lo, len, acc, bad);
    if (threadIdx.x == 0) { out[blockIdx.x].sumsq = acc; out[blockIdx.x].nonfinite = bad; }
}

static __global__ void copy_partials_kernel(const Partial* __restrict__ in, uint64_t n, Partial* __restrict__ out)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = in[i];
}

// Stage 2: fixed-order sum of all partials, then the validation outcome of Sec. 4.4 computed
// on the GPU (clip coefficient, gradient multiplier, skip flag) so that a following guarded
// step needs no host round trip.
static __global__ __launch_bounds__(kFinalBlock) void stats_final_kernel(const Partial* partials,
                                                                 uint64_t n, double max_norm,
                                                                 double loss_scale,
                                                                 double min_loss_scale,
                                                                 DevResult* out)
{
    double acc;
    uint64_t bad;
    final_reduce(partials, n, acc, bad);
    if (threadIdx.x == 0) {
        DevResult r;
        r.sumsq = acc;
        r.norm = sqrt(acc);
        r.nonfinite = bad;
        r.overflow = bad > 0 ? 1 : 0;
        double clip = 1.0;
        if (max_norm > 0.0) {
            double c = max_norm / (r.norm + 1e-6);
            clip = c < 1.0 ? c : 1.0;
        }
        r.clip = clip;
        r.grad_scale = (float)(clip / loss_scale);
        double half = loss_scale * 0.5;
        r.next_loss_scale = (float)(r.overflow ? (half > min_loss_scale ? half : min_loss_scale)
                                               : loss_scale);
        r.action = r.overflow ? 1 : (clip < 1.0 ? 2 : 0);
        *out = r;
    }
}

// Train state kept on the GPU between iterations, so that a loop of iterations needs no host
// round trip: Adam's step count and the running powers of beta for the bias corrections, the
// loss scale and its growth counter, and the scalars of the step now in flight.
struct DevTrain {
    double b1t, b2t;        // beta1^t, beta2^t for the step count t below
    int64_t t;              // 1-based count of the step that is applied next
    float loss_scale;       // what the next iteration's gradients are scaled by
    uint32_t clean;         // iterations in a row without NaN/Inf since the last change of the scale
    StepConsts consts;      // scalars of the step now in flight (a snapshot: the step kernel reads
                            // nothing else of this struct, so t and the powers can move on at once)
};

// What so_train_reset fixes for the run.
struct TrainSetup {
    double b1, b2, lr, eps, wd;
    double max_norm, min_loss_scale, max_loss_scale;
    uint32_t growth_interval;
    int32_t adamw, bias_correction, reserved;
};

// Second reduction stage of an autonomous iteration (Sec. 4.4 validator, entirely on the GPU):
// reduces the partials of the raw (still loss-scaled) gradients, decides skip / clip, derives
// this step's scalars, and moves step count, beta powers and loss scale on to the next
// iteration.
static __global__ __launch_bounds__(kFinalBlock) void train_final_kernel(const Partial* partials, uint64_t n,
                                                                 TrainSetup su, DevResult* out,
                                                                 DevTrain* tr)
{
    double acc;
    uint64_t bad;
    final_reduce(partials, n, acc, bad);
    if (threadIdx.x == 0) {
        DevTrain st = *tr;
        const double scale = (double)st.loss_scale;
        const double inv = (double)(float)(1.0 / scale);      // the fp32 multiplier a host would pass
        DevResult r;
        r.sumsq = acc * (inv * inv);
        r.norm = sqrt(r.sumsq);
        r.nonfinite = bad;
        r.overflow = bad > 0 ? 1 : 0;
        double clip = 1.0;
        if (su.max_norm > 0.0) {
            const double c = su.max_norm / (r.norm + 1e-6);
            clip = c < 1.0 ? c : 1.0;
        }
        r.clip = clip;
        r.grad_scale = (float)(clip / scale);
        r.action = r.overflow ? 1 : (clip < 1.0 ? 2 : 0);
        if (r.overflow) {
            const double half = scale * 0.5;
            st.loss_scale = (float)(half > su.min_loss_scale ? half : su.min_loss_scale);
            st.clean = 0;
        } else {
            double bc1 = 1.0, bc2 = 1.0;
            if (su.bias_correction) { bc1 = 1.0 - st.b1t; bc2 = 1.0 - st.b2t; }
            StepConsts c;
            c.b1 = (float)su.b1;
            c.c1 = (float)(1.0 - su.b1);
            c.b2 = (float)su.b2;
            c.c2 = (float)(1.0 - su.b2);
            c.rsb2 = (float)(1.0 / sqrt(bc2));
            c.eps = (float)su.eps;
            c.step_size = (float)(su.lr / bc1);
            c.lr_wd = su.adamw ? (float)(su.lr * su.wd) : 0.f;
            c.wd_l2 = su.adamw ? 0.f : (float)su.wd;
            c.lp_fp16 = 0;
            st.consts = c;
            st.t += 1;                          // step t is on its way: the next one is t + 1
            st.b1t *= su.b1;
            st.b2t *= su.b2;
            st.clean += 1;
            if (su.growth_interval != 0 && st.clean >= su.growth_interval) {
                const double up = scale * 2.0;
                st.loss_scale = (float)(up < su.max_loss_scale ? up : su.max_loss_scale);
                st.clean = 0;
            }
        }
        r.next_loss_scale = st.loss_scale;
        *out = r;
        *tr = st;
    }
}

// Rollback of a SAVE-mode speculative step: copy the saved p, m, v back and re-derive the
// 16-bit working copy from the restored parameters (same rounding => same bits as before).
// Same shape as the step kernel: one single-wavefront workgroup per 256 elements, one memory
// instruction in flight at a time.
static __global__ __launch_bounds__(kStepBlock) void restore_kernel(const float* __restrict__ p_save,
                                                            const float* __restrict__ m_save,
                                                            const float* __restrict__ v_save,
                                                            float* __restrict__ p, float* __restrict__ m,
                                                            float* __restrict__ v,
                                                            uint16_t* __restrict__ q, uint64_t n,
                                                            uint32_t lp_fp16)
{
    const uint64_t base = (uint64_t)blockIdx.x * kTile;
    if (base + kTile <= n) {
        const uint32_t vo4 = threadIdx.x * 16u, vo2 = threadIdx.x * 8u;
        u32x4 x = buf_ld4(tile_rsrc(p_save + base, kTile * 4), vo4);
        phase_fence();
        buf_st4(tile_rsrc(p + base, kTile * 4), vo4, x);
        phase_fence();
        const float a0 = __uint_as_float(x.x), a1 = __uint_as_float(x.y), a2 = __uint_as_float(x.z),
                    a3 = __uint_as_float(x.w);
        buf_st2(tile_rsrc(q + base, kTile * 2), vo2,
                u32x2{lp_round(a0, lp_fp16) | (lp_round(a1, lp_fp16) << 16),
                      lp_round(a2, lp_fp16) | (lp_round(a3, lp_fp16) << 16)});
        phase_fence();
        x = buf_ld4(tile_rsrc(m_save + base, kTile * 4), vo4);
        phase_fence();
        buf_st4(tile_rsrc(m + base, kTile * 4), vo4, x);
        phase_fence();
        x = buf_ld4(tile_rsrc(v_save + base, kTile * 4), vo4);
        phase_fence();
        buf_st4(tile_rsrc(v + base, kTile * 4), vo4, x);
    } else {
#pragma unroll 1
        for (int j = 0; j < kVec; ++j) {
            const uint64_t i = base + threadIdx.x * kVec + j;
            if (i < n) {
                const float pp = ld_plain(p_save + i);
                st_plain(p + i, pp);
                st_plain(m + i, ld_plain(m_save + i));
                st_plain(v + i, ld_plain(v_save + i));
                st_plain(q + i, (uint16_t)lp_round(pp, lp_fp16));
            }
        }
    }
}

// 16-bit working copy from fp32 parameters (Sec. 4.5, the cast on the GPU side of the link):
// q[i] = the step's own rounding of p[i], so a copy made here and one left by a step that
// stored the same p hold the same bits.  6 bytes per parameter; shape of the step kernel.
static __global__ __launch_bounds__(kStepBlock) void cast_lp_kernel(const float* __restrict__ p,
                                                                    uint16_t* __restrict__ q, uint64_t n,
                                                                    uint32_t lp_fp16)
{
    const uint64_t base = (uint64_t)blockIdx.x * kTile;
    if (base + kTile <= n) {
        const u32x4 x = buf_ld4(tile_rsrc(p + base, kTile * 4), threadIdx.x * 16u);
        const float a0 = __uint_as_float(x.x), a1 = __uint_as_float(x.y), a2 = __uint_as_float(x.z),
                    a3 = __uint_as_float(x.w);
        buf_st2(tile_rsrc(q + base, kTile * 2), threadIdx.x * 8u,
                u32x2{lp_round(a0, lp_fp16) | (lp_round(a1, lp_fp16) << 16),
                      lp_round(a2, lp_fp16) | (lp_round(a3, lp_fp16) << 16)});
    } else {
#pragma unroll 1
        for (int j = 0; j < kVec; ++j) {
            const uint64_t i = base + threadIdx.x * kVec + j;
            if (i < n) st_plain(q + i, (uint16_t)lp_round(ld_plain(p + i), lp_fp16));
        }
    }
}

// Gather/scatter of tensor slices into flat buckets (bucket layout, Sec. 4.3).  One
// workgroup-strided element copy per slice chunk; T is the element container (2 or 4 bytes).
struct CopySlice {
    const void* src;
    void* dst;
    uint64_t len;           // elements
    uint64_t chunk_begin;   // global index of the slice's first chunk
    uint64_t chunk_end;
    uint64_t head;          // elements before dst reaches a 16-byte boundary; they form chunk 0 if > 0
};
constexpr int kCopyChunkBytes = 1024;        // bytes per workgroup of a plain copy: one 16-byte access per lane
constexpr int kStatsCopyChunkBytes = 2048;   // ... of a copy with statistics: two per lane, both in flight
constexpr int kDirShift = 8;            // one directory entry per 256 chunks

// Gather / scatter of tensor slices.  Same shape as the step kernel, for the same reason (a
// plain grid of single-wavefront workgroups, one 16-byte load and one store per lane, reaches
// 6.7 TB/s on this part where 256-thread workgroups looping over 32 KB chunks reach 5.4):
// workgroup c copies chunk c.  Which slice a chunk belongs to is found by bisection between
// two entries of a directory that names the slice of every 256th chunk, so the search rarely
// takes a step.
//
// Alignment.  The chunks of a slice are laid out from the first 16-byte boundary of its
// DESTINATION: the few elements before it (the slice's "head") are chunk 0, copied element by
// element, and every later chunk stores whole aligned 16-byte vectors.  If the source then
// sits at the same offset inside its 16-byte granule the loads are aligned too.  If not
// (tensors of odd sizes laid back to back), a lane reads the two aligned source granules that
// hold its 16 bytes and shifts them together (v_alignbyte); the granules read always contain at
// least one byte of the slice, so no access leaves the memory the slice lives in.
//
// SDT >= 0 (16-bit elements only): the elements are gradients of type SDT and the copy also
// produces stage 1 of the gradient statistics (Sec. 4.4) -- one partial per workgroup, i.e.
// per 1024 gradients -- so that gathering gradients into buckets (Sec. 4.3) and validating them
// cost one pass over the gradients instead of two.
// The 16 bytes that start `delta` (1..15) bytes into granule a and end in the next granule b.
__device__ __forceinline__ u32x4 funnel16(u32x4 a, u32x4 b, uint32_t delta)
{
    const uint32_t sh = delta & 3u;
    switch (delta >> 2) {
    case 0:
        return u32x4{__builtin_amdgcn_alignbyte(a.y, a.x, sh), __builtin_amdgcn_alignbyte(a.z, a.y, sh),
                     __builtin_amdgcn_alignbyte(a.w, a.z, sh), __builtin_amdgcn_alignbyte(b.x, a.w, sh)};
    case 1:
        return u32x4{__builtin_amdgcn_alignbyte(a.z, a.y, sh), __builtin_amdgcn_alignbyte(a.w, a.z, sh),
                     __builtin_amdgcn_alignbyte(b.x, a.w, sh), __builtin_amdgcn_alignbyte(b.y, b.x, sh)};
    case 2:
        return u32x4{__builtin_amdgcn_alignbyte(a.w, a.z, sh), __builtin_amdgcn_alignbyte(b.x, a.w, sh),
                     __builtin_amdgcn_alignbyte(b.y, b.x, sh), __builtin_amdgcn_alignbyte(b.z, b.y, sh)};
    default:
        return u32x4{__builtin_amdgcn_alignbyte(b.x, a.w, sh), __builtin_amdgcn_alignbyte(b.y, b.x, sh),
                     __builtin_amdgcn_alignbyte(b.z, b.y, sh), __builtin_amdgcn_alignbyte(b.w, b.z, sh)};
    }
}

template <typename T, int SDT>
__global__ __launch_bounds__(kStepBlock) void flatten_kernel(const CopySlice* __restrict__ slices,
                                                            uint32_t n_slices,
                                                            const uint32_t* __restrict__ dir,
                                                            uint32_t n_dir, uint64_t chunk_offset,
                                                            double inv_scale, Partial* __restrict__ partials)
{
    static_assert(SDT < 0 || sizeof(T) == 2, "statistics are defined for 16-bit gradients");
    // A copy with statistics ends every wavefront's life with a reduction; two vectors per
    // lane, both in flight, keep the memory pipes as busy as the plain copy's one.
    constexpr uint32_t kBytes = SDT >= 0 ? kStatsCopyChunkBytes : kCopyChunkBytes;
    constexpr uint32_t kElems = kBytes / sizeof(T);
    constexpr uint32_t kPer16 = 16 / sizeof(T);
    constexpr int VPL = kBytes / (16 * kStepBlock);        // 16-byte vectors per lane
    constexpr int DT = SDT < 0 ? 0 : SDT;
    const uint64_t c = chunk_offset + blockIdx.x;
    const uint64_t d = c >> kDirShift;
    uint32_t lo = dir[d];
    uint32_t hi = d + 1 < n_dir ? dir[d + 1] : n_slices - 1;
    while (lo < hi) {                   // last slice with chunk_begin <= c
        const uint32_t mid = (lo + hi + 1) >> 1;
        if (slices[mid].chunk_begin <= c) lo = mid; else hi = mid - 1;
    }
    const CopySlice sl = slices[lo];
    const uint64_t k = c - sl.chunk_begin;
    uint64_t start = 0;
    uint32_t cnt = (uint32_t)sl.head;
    if (sl.head == 0 || k != 0) {
        start = sl.head + (k - (sl.head ? 1u : 0u)) * (uint64_t)kElems;
        const uint64_t left = sl.len - start;
        cnt = left < kElems ? (uint32_t)left : kElems;
    }
    const T* src = (const T*)sl.src + start;
    T* dst = (T*)sl.dst + start;
    double acc = 0.0;
    uint32_t bad = 0;
    if (((uintptr_t)dst & 15u) == 0) {
        const uint32_t nvec = cnt / kPer16;
        const uint32_t delta = (uint32_t)((uintptr_t)src & 15u);      // same for the whole wavefront
        u32x4 x[VPL];
#pragma unroll
        for (int v = 0; v < VPL; ++v) x[v] = u32x4{0u, 0u, 0u, 0u};
        if (delta == 0) {
            const rsrc_t r = tile_rsrc(src, nvec * 16u);
#pragma unroll
            for (int v = 0; v < VPL; ++v) {
                const uint32_t idx = v * kStepBlock + threadIdx.x;
                if (idx < nvec) x[v] = buf_ld4(r, idx * 16u);
            }
        } else if (nvec != 0) {
            // the two aligned granules that hold a lane's 16 source bytes, shifted together
            const rsrc_t r = tile_rsrc((const char*)src - delta, (nvec + 1u) * 16u);
            u32x4 a[VPL], b[VPL];
#pragma unroll
            for (int v = 0; v < VPL; ++v) {
                const uint32_t idx = v * kStepBlock + threadIdx.x;
                a[v] = b[v] = u32x4{0u, 0u, 0u, 0u};
                if (idx < nvec) {
                    a[v] = buf_ld4(r, idx * 16u);
                    b[v] = buf_ld4(r, idx * 16u + 16u);
                }
            }
#pragma unroll
            for (int v = 0; v < VPL; ++v) x[v] = funnel16(a[v], b[v], delta);
        }
        phase_fence();
        {
            const rsrc_t w = tile_rsrc(dst, nvec * 16u);
#pragma unroll
            for (int v = 0; v < VPL; ++v) {
                const uint32_t idx = v * kStepBlock + threadIdx.x;
                if (idx < nvec) buf_st4(w, idx * 16u, x[v]);
            }
        }
        if (SDT >= 0) {                                        // lanes past nvec hold zeros
#pragma unroll
            for (int v = 0; v < VPL; ++v) stat_accum8<DT>(x[v], acc, bad);
        }
        const uint32_t i = nvec * kPer16 + threadIdx.x;        // fewer than 16 bytes are left
        if (i < cnt) {
            const T e = ld_plain(src + i);
            st_plain(dst + i, e);
            if (SDT >= 0) stat_accum<true>(decode1<DT>((uint16_t)e), acc, bad);
        }
    } else {                            // the head of a slice: fewer than 16 bytes
        for (uint32_t i = threadIdx.x; i < cnt; i += kStepBlock) {
            const T e = ld_plain(src + i);
            st_plain(dst + i, e);
            if (SDT >= 0) stat_accum<true>(decode1<DT>((uint16_t)e), acc, bad);
        }
    }
    if (SDT >= 0) {                     // the workgroup is one wavefront
        acc = wave_total(acc);
        if (__any(bad != 0)) bad = wave_total(bad);         // rare: skip the second reduction otherwise
        if (threadIdx.x == 0) {
            Partial out;
            out.sumsq = acc * (inv_scale * inv_scale);
            out.nonfinite = bad;
            partials[blockIdx.x] = out;
        }
    }
}

}  // namespace so
