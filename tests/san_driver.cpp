// Sanitizer driver (test infrastructure): built by tests/test_sanitizers.py with
//   -fsanitize=address,undefined -fno-sanitize-recover=all
// together with oracle/adam_oracle.c and the library's host-only source file, and run on the
// CPU.  Every buffer is a heap allocation of exactly the size a call is entitled to touch, so
// an access one element too far, an uninitialised count or a signed overflow aborts the run.
// Results are cross-checked only lightly here (the pins and host-logic tests do that); the
// point of this program is to drive every host-side code path under the sanitizers.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "so_adam.h"

extern "C" {
double orc_decode16(uint16_t bits, int dtype);
int orc_is_nonfinite16(uint16_t bits, int dtype);
uint16_t orc_f32_to_bf16(float x);
uint16_t orc_f32_to_fp16(float x);
void orc_grad_stats(const uint16_t* g, uint64_t n, int dtype, float inv_scale, double* sumsq, uint64_t* nonfinite);
void orc_adamw_step(const uint16_t* g, int dtype, float* p, float* m, float* v, uint16_t* q, uint64_t n, float lr,
                    float beta1, float beta2, float eps, float wd, int64_t t, float s, int adamw,
                    int bias_correction, int lp_fp16);
double orc_clip_coef(double norm, double max_norm);
}

#define CHECK(cond)                                                              \
    do {                                                                         \
        if (!(cond)) {                                                           \
            fprintf(stderr, "san_driver: check failed: %s (line %d)\n", #cond, __LINE__); \
            return 1;                                                            \
        }                                                                        \
    } while (0)

static uint32_t rng_state = 0x1234567u;
static uint32_t rnd()
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 17; rng_state ^= rng_state << 5;
    return rng_state;
}

template <typename T>
struct Exact {      // heap array of exactly n elements (n == 0: a one-byte block never dereferenced as T)
    T* p; size_t n;
    explicit Exact(size_t n_) : p((T*)malloc(n_ ? n_ * sizeof(T) : 1)), n(n_) {}
    ~Exact() { free(p); }
};

static int drive_oracle()
{
    // every 16-bit pattern through both decoders and the scan
    uint64_t bad_bf16 = 0, bad_fp16 = 0;
    for (uint32_t b = 0; b < 65536; ++b) {
        bad_bf16 += orc_is_nonfinite16((uint16_t)b, 0);
        bad_fp16 += orc_is_nonfinite16((uint16_t)b, 1);
        (void)orc_decode16((uint16_t)b, 0);
        (void)orc_decode16((uint16_t)b, 1);
    }
    CHECK(bad_bf16 == 2 * 128 && bad_fp16 == 2 * 1024);
    // both narrowings over a spread of fp32 patterns, including NaN, Inf, subnormals, max
    for (uint32_t i = 0; i < 2000000; ++i) {
        uint32_t u = (i < 65536) ? (i << 16) | (rnd() & 0xFFFFu) : rnd();
        float x;
        memcpy(&x, &u, 4);
        (void)orc_f32_to_bf16(x);
        (void)orc_f32_to_fp16(x);
    }
    const size_t sizes[] = {0, 1, 2, 7, 8, 9, 255, 1000, 4099};
    for (size_t n : sizes) {
        for (int dtype = 0; dtype < 2; ++dtype) {
            Exact<uint16_t> g(n), q(n);
            Exact<float> p(n), m(n), v(n);
            for (size_t i = 0; i < n; ++i) {
                g.p[i] = (uint16_t)(rnd() >> 7);                         // all exponents, NaN/Inf included
                p.p[i] = (float)((int)(rnd() % 2001) - 1000) * 1e-5f;
                m.p[i] = (float)((int)(rnd() % 2001) - 1000) * 1e-7f;
                v.p[i] = (float)(rnd() % 1000) * 1e-12f;
            }
            double sumsq = -1.0;
            uint64_t bad = ~0ull;
            orc_grad_stats(g.p, n, dtype, 0.5f, &sumsq, &bad);
            CHECK(sumsq >= 0.0 && bad <= n);
            for (int variant = 0; variant < 8; ++variant)
                orc_adamw_step(g.p, dtype, p.p, m.p, v.p, q.p, n, 1e-4f, 0.9f, 0.999f, 1e-8f, 0.01f,
                               1 + variant * 1000, 0.25f, variant & 1, (variant >> 1) & 1, (variant >> 2) & 1);
        }
    }
    CHECK(orc_clip_coef(0.5, 1.0) == 1.0 && orc_clip_coef(4.0, 0.0) == 1.0 && orc_clip_coef(4.0, 1.0) < 0.26);
    CHECK(std::isnan(orc_clip_coef(NAN, 1.0)) || orc_clip_coef(NAN, 1.0) == 1.0);
    return 0;
}

static int drive_layout()
{
    for (int round = 0; round < 300; ++round) {
        const size_t nt = rnd() % 9;
        Exact<uint64_t> numel(nt);
        uint64_t total = 0;
        for (size_t i = 0; i < nt; ++i) { numel.p[i] = rnd() % 50; total += numel.p[i]; }
        const uint64_t bucket = 1 + rnd() % 17;
        size_t ns = 12345;
        uint64_t nb = 12345;
        CHECK(so_layout_plan(nt ? numel.p : nullptr, nt, bucket, nullptr, 0, &ns, &nb) == SO_OK);
        CHECK(nb == (total + bucket - 1) / bucket);
        Exact<so_slice> out(ns);
        size_t ns2 = 0;
        CHECK(so_layout_plan(nt ? numel.p : nullptr, nt, bucket, out.p, ns, &ns2, &nb) == SO_OK && ns2 == ns);
        uint64_t flat = 0;
        for (size_t i = 0; i < ns; ++i) {
            const so_slice& s = out.p[i];
            CHECK(s.len > 0 && s.tensor < nt && s.tensor_offset + s.len <= numel.p[s.tensor]);
            CHECK(s.bucket_offset + s.len <= bucket && s.bucket * bucket + s.bucket_offset == flat);
            flat += s.len;
        }
        CHECK(flat == total);
        if (ns > 0) {       // a table one entry too short is refused, and never written past
            Exact<so_slice> small(ns - 1);
            CHECK(so_layout_plan(numel.p, nt, bucket, small.p, ns - 1, &ns2, &nb) == SO_ERR_INVALID_ARG);
        }
    }
    size_t ns;
    uint64_t nb;
    CHECK(so_layout_plan(nullptr, 0, 0, nullptr, 0, &ns, &nb) == SO_ERR_INVALID_ARG);
    CHECK(so_layout_plan(nullptr, 3, 4, nullptr, 0, &ns, &nb) == SO_ERR_INVALID_ARG);
    CHECK(so_layout_plan(nullptr, 0, 4, nullptr, 0, nullptr, &nb) == SO_ERR_INVALID_ARG);
    const uint64_t big[2] = {1ull << 62, 1ull << 62};         // sums stay below 2^64
    CHECK(so_layout_plan(big, 2, 1ull << 61, nullptr, 0, &ns, &nb) == SO_OK && ns == 4 && nb == 4);
    return 0;
}

static int drive_scalars()
{
    const double norms[] = {0.0, 1e-30, 0.999999, 1.0, 1.000001, 89.6, 1e30, INFINITY, NAN};
    const double maxn[] = {-1.0, 0.0, 1.0, 2.5};
    const double scales[] = {1.0, 1.5, 65536.0, 1e-3};
    for (double n : norms)
        for (double mx : maxn)
            for (double sc : scales)
                for (int ov = 0; ov < 2; ++ov) {
                    so_stats st{n * n, n, (uint64_t)ov * 3, ov, 0};
                    so_decision d;
                    memset(&d, 0xAB, sizeof(d));
                    CHECK(so_validate(&st, mx, sc, 1.0, &d) == SO_OK);
                    CHECK(d.action == (ov ? SO_ROLLBACK_SKIP : (d.clip < 1.0 ? SO_ROLLBACK_REDO : SO_COMMIT)));
                    CHECK(d.reserved == 0);
                }
    so_decision d;
    so_stats st{1.0, 1.0, 0, 0, 0};
    CHECK(so_validate(nullptr, 1.0, 1.0, 1.0, &d) == SO_ERR_INVALID_ARG);
    CHECK(so_validate(&st, 1.0, 1.0, 1.0, nullptr) == SO_ERR_INVALID_ARG);
    CHECK(so_validate(&st, 1.0, 0.0, 1.0, &d) == SO_ERR_INVALID_ARG);
    CHECK(so_validate(&st, 1.0, NAN, 1.0, &d) == SO_ERR_INVALID_ARG);

    float scale = 8.0f;
    uint32_t clean = 0;
    const int overflow[] = {0, 0, 0, 0, 1, 0, 1, 1, 1, 1, 0, 0};
    const float want[] = {8, 16, 16, 16, 8, 8, 4, 2, 1, 1, 1, 2};
    for (int i = 0; i < 12; ++i) {
        float next = -1.f;
        CHECK(so_loss_scale_next(scale, overflow[i], &clean, 2, 1.0f, 16.0f, &next) == SO_OK);
        CHECK(next == want[i]);
        scale = next;
    }
    clean = 0xFFFFFFFEu;                      // the counter may not wrap into an early growth
    float next = 0.f;
    CHECK(so_loss_scale_next(4.0f, 0, &clean, 0, 1.0f, 16.0f, &next) == SO_OK && next == 4.0f);
    CHECK(so_loss_scale_next(4.0f, 0, &clean, 0, 1.0f, 16.0f, &next) == SO_OK && next == 4.0f);
    CHECK(so_loss_scale_next(0.0f, 0, &clean, 2, 1.0f, 16.0f, &next) == SO_ERR_INVALID_ARG);
    CHECK(so_loss_scale_next(1.0f, 0, nullptr, 2, 1.0f, 16.0f, &next) == SO_ERR_INVALID_ARG);
    CHECK(so_loss_scale_next(1.0f, 0, &clean, 2, 2.0f, 1.0f, &next) == SO_ERR_INVALID_ARG);

    uint64_t n = 99;
    CHECK(so_plan_resident(41.9, 0.85, 42.1, 1.0, 0.85, 117, 117, &n) == SO_OK && n == 46);
    CHECK(so_plan_resident(1.0, 1.0, 1.0, 0.0, 0.0, 10, 7, &n) == SO_OK && n == 7);
    CHECK(so_plan_resident(0.0, 0.0, 0.0, 1.0, 1.0, 10, 10, &n) == SO_OK && n == 0);
    CHECK(so_plan_resident(1.0, 1.0, 1.0, 1.0, 1.0, 0, 10, &n) == SO_OK && n == 0);
    CHECK(so_plan_resident(NAN, 1.0, 1.0, 1.0, 1.0, 4, 4, &n) == SO_ERR_INVALID_ARG);
    CHECK(so_plan_resident(INFINITY, 1.0, 1.0, 1.0, 1.0, 4, 4, &n) == SO_ERR_INVALID_ARG);
    CHECK(so_plan_resident(1.0, 1.0, 1.0, 1.0, 1.0, 4, 4, nullptr) == SO_ERR_INVALID_ARG);
    so_arena_layout lay;
    const uint64_t ns[] = {0, 1, 524288, 524289, 8030261248ull, (1ull << 59)};
    for (uint64_t nn : ns) {
        memset(&lay, 0xCD, sizeof(lay));
        CHECK(so_arena_plan(nn, &lay) == SO_OK);
        CHECK(lay.param == 0 && lay.grad >= 4 * nn && lay.exp_avg >= lay.grad + 2 * nn &&
              lay.param_lp >= lay.exp_avg + 4 * nn && lay.exp_avg_sq >= lay.param_lp + 2 * nn &&
              lay.bytes >= lay.exp_avg_sq + 4 * nn && lay.bytes % (2u << 20) == 0);
    }
    CHECK(so_arena_plan(~0ull, &lay) == SO_ERR_INVALID_ARG);
    CHECK(so_arena_plan(1ull << 61, &lay) == SO_ERR_INVALID_ARG);
    CHECK(so_arena_plan(8, nullptr) == SO_ERR_INVALID_ARG);
    so_arena_alt alt;
    for (uint64_t nn : {1ull, 524289ull, 8030261248ull}) {
        CHECK(so_arena_plan(nn, &lay) == SO_OK);
        const uint64_t ws = 2 * lay.bytes + (40ull << 30);
        for (uint32_t index = 0; index < 64; ++index) {
            so_arena_layout c5, c9;
            memset(&c5, 0xCD, sizeof(c5)); memset(&c9, 0xCD, sizeof(c9)); memset(&alt, 0xCD, sizeof(alt));
            CHECK(so_arena_candidate(nn, ws, 99, index, &c5, nullptr) == SO_OK && c5.bytes <= ws);
            CHECK(so_arena_candidate(nn, ws, 99, index, &c9, &alt) == SO_OK && c9.bytes <= ws);
            CHECK(alt.param + 4 * nn <= ws && alt.param_lp + 2 * nn <= ws);
        }
        CHECK(so_arena_candidate(nn, lay.bytes / 2, 99, 1, &lay, nullptr) == SO_ERR_INVALID_ARG);
    }
    CHECK(so_arena_candidate(0, 1ull << 40, 1, 1, &lay, nullptr) == SO_ERR_INVALID_ARG);
    CHECK(so_arena_candidate(8, 1ull << 40, 1, 1, nullptr, nullptr) == SO_ERR_INVALID_ARG);
    CHECK(strstr(so_version(), "gfx950") != nullptr);
    return 0;
}

int main()
{
    if (drive_oracle() || drive_layout() || drive_scalars()) return 1;
    printf("sanitizer driver OK\n");
    return 0;
}
