// so_probe: a torch-free driver of the library for profilers.
//
// Allocates a resident multi-bucket state with hipMalloc (gradients set to a finite bf16
// byte pattern, state zero), runs the benchmark's whole-path step (gradient statistics +
// GPU-side validation + guarded fused step) a few times, then one plain copy of 2^28 fp32
// elements (flatten_kernel: exactly 1 GiB read and 1 GiB written) that serves as the
// known-size reference when reading rocprofv3's FETCH_SIZE / WRITE_SIZE counters, and one
// gather with fused gradient statistics over 2^28 gradients.
//
// usage: so_probe [n_buckets=81] [bucket_elems=100000000] [last_bucket_elems=30261248] [steps=2]
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

#include "so_adam.h"
#include "so_adam_aux.h"

#define HIP_OK(x)                                                                      \
    do {                                                                               \
        hipError_t e_ = (x);                                                           \
        if (e_ != hipSuccess) {                                                        \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                    \
            return 1;                                                                  \
        }                                                                              \
    } while (0)
#define SO_OKAY(x)                                                                     \
    do {                                                                               \
        so_status s_ = (x);                                                            \
        if (s_ != SO_OK) {                                                             \
            fprintf(stderr, "%s: status %d: %s\n", #x, (int)s_, so_last_error(ctx));   \
            return 1;                                                                  \
        }                                                                              \
    } while (0)

int main(int argc, char** argv)
{
    const size_t nb = argc > 1 ? strtoull(argv[1], nullptr, 10) : 81;
    const uint64_t bucket = argc > 2 ? strtoull(argv[2], nullptr, 10) : 100000000ull;
    const uint64_t last = argc > 3 ? strtoull(argv[3], nullptr, 10) : 30261248ull;
    const int steps = argc > 4 ? atoi(argv[4]) : 2;
    if (nb == 0 || bucket == 0 || last == 0 || last > bucket || (bucket % 8) != 0) {
        fprintf(stderr, "bad arguments\n");
        return 2;
    }
    const uint64_t total = (nb - 1) * bucket + last;
    float *p, *m, *v;
    uint16_t *g, *q;
    HIP_OK(hipMalloc((void**)&p, total * 4));
    HIP_OK(hipMalloc((void**)&m, total * 4));
    HIP_OK(hipMalloc((void**)&v, total * 4));
    HIP_OK(hipMalloc((void**)&g, total * 2));
    HIP_OK(hipMalloc((void**)&q, total * 2));
    HIP_OK(hipMemset(p, 0, total * 4));
    HIP_OK(hipMemset(m, 0, total * 4));
    HIP_OK(hipMemset(v, 0, total * 4));
    HIP_OK(hipMemset(g, 0x3A, total * 2));      // bf16 0x3A3A = 7.1e-4, finite
    HIP_OK(hipMemset(q, 0, total * 2));

    so_ctx* ctx = nullptr;
    if (so_create(&ctx, 0, nullptr) != SO_OK) { fprintf(stderr, "so_create failed\n"); return 1; }
    std::vector<so_bucket> b(nb);
    for (size_t i = 0; i < nb; ++i) {
        const uint64_t off = i * bucket;
        b[i] = so_bucket{};
        b[i].grad = g + off; b[i].param = p + off; b[i].exp_avg = m + off; b[i].exp_avg_sq = v + off;
        b[i].param_lp = q + off;
        b[i].n = (i + 1 == nb) ? last : bucket;
        b[i].grad_dtype = SO_GRAD_BF16;
    }
    so_hparams hp{1e-4f, 0.9f, 0.999f, 1e-8f, 0.01f, 1, 1};
    SO_OKAY(so_set_profiling(ctx, 1));
    for (int t = 1; t <= steps; ++t) {
        SO_OKAY(so_grad_stats_enqueue(ctx, b.data(), nb, 1.0f, 1.0f));
        SO_OKAY(so_adam_step_guarded(ctx, b.data(), nb, &hp, t));
    }
    std::vector<double> ms(steps);
    size_t got = 0;
    SO_OKAY(so_read_step_kernel_ms(ctx, ms.data(), ms.size(), &got));
    so_stats st;
    so_decision dec;
    SO_OKAY(so_grad_stats_fetch(ctx, &st, &dec));
    printf("params %llu buckets %zu norm %.6f clip %.6g\n", (unsigned long long)total, nb, st.norm, dec.clip);
    for (size_t i = 0; i < got; ++i)
        printf("step kernel %zu: %.3f ms  %.1f GB/s (28 B/param)\n", i, ms[i], 28.0 * total / (ms[i] * 1e6));

    // known-size reference copy: 2^28 fp32 elements
    const uint64_t ncal = 1ull << 28;
    float *src, *dst;
    HIP_OK(hipMalloc((void**)&src, ncal * 4));
    HIP_OK(hipMalloc((void**)&dst, ncal * 4));
    HIP_OK(hipMemset(src, 1, ncal * 4));
    HIP_OK(hipMemset(dst, 0, ncal * 4));
    so_slice sl{0, 0, 0, 0, ncal};
    void* tp[1] = {src};
    void* bp[1] = {dst};
    SO_OKAY(so_flatten(ctx, &sl, 1, tp, bp, 4, 0));
    printf("reference copy: flatten_kernel<unsigned int> moved %llu bytes each way\n", (unsigned long long)(ncal * 4));
    // the gather with fused gradient statistics over 2^28 of the 16-bit gradients (0.5 GiB each way)
    if (total >= ncal) {                        // g and q hold at least 2^28 elements
        void* gp[1] = {g};
        void* qp[1] = {q};
        SO_OKAY(so_flatten_grad_stats(ctx, &sl, 1, gp, qp, SO_GRAD_BF16, 1.0f, 1.0f));
        SO_OKAY(so_grad_stats_fetch(ctx, &st, &dec));
        printf("gather + statistics over %llu gradients: norm %.6f\n", (unsigned long long)ncal, st.norm);
    }
    so_destroy(ctx);
    return 0;
}
