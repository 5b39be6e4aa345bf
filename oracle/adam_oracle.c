/*
 * Reference oracle for the mixed-precision Adam(W) bucket step -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is a slow, scalar, double-precision statement of what the optimizer hot path
 * computes.  It exists so that tests, the smoke check and the benchmark's cpu_baseline leg
 * have something independent to compare the GPU library against.  It shares no code,
 * headers, tables or helpers with the GPU library and must never be linked into it.
 *
 * What it follows:
 *   - The optimizer is Adam with bias correction (Kingma & Ba, Algorithm 1) in its
 *     decoupled-weight-decay form (Loshchilov & Hutter, Algorithm 2), which are the two
 *     definitions the paper cites for its optimizer (Sec. 2.2 "model states", Sec. 4.6
 *     GraceAdam).  The paper itself prints no update equation.
 *   - The optimizer consumes 16-bit gradients and keeps fp32 master state; the updated
 *     parameters are cast back to a 16-bit working copy (Sec. 4.5, mixed-precision casts).
 *   - The global validation quantities are the L2 norm of all gradients and a NaN/Inf
 *     check over all gradients (Sec. 4.4, first paragraph).
 *
 * Arithmetic: every element is updated in double precision starting from the fp32-stored
 * state; each of m, v, p is rounded to fp32 exactly once, on store (C's double->float
 * conversion, round-to-nearest-even).  The 16-bit working copy is the round-to-nearest-even
 * bf16 of the stored fp32 parameter.  No blocking, no vector code, no reordering.
 *
 * Parity pins (tests/test_oracle_pins.py): step-1 closed form, constant-gradient
 * trajectory, pure weight decay, lr=0, exact-rational brute force on tiny buckets, a
 * hand-worked dyadic example (tests/golden), exhaustive 16-bit decode / non-finite / bf16
 * rounding checks against numpy, exactly representable norms, and an fp64 library AdamW.
 * tests/test_oracle_mutants.py plants mistakes in a copy of this file and checks that the
 * pins catch each of them.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define ORC_GRAD_BF16 0
#define ORC_GRAD_FP16 1

/* Decode one 16-bit floating-point bit pattern to double, field by field.
 * bf16: 1 sign, 8 exponent (bias 127), 7 fraction bits.
 * fp16: 1 sign, 5 exponent (bias 15), 10 fraction bits (IEEE 754 binary16). */
double orc_decode16(uint16_t bits, int dtype)
{
    int ebits = (dtype == ORC_GRAD_FP16) ? 5 : 8;
    int fbits = 15 - ebits;
    int bias = (1 << (ebits - 1)) - 1;
    int sign = (bits >> 15) & 1;
    int e = (bits >> fbits) & ((1 << ebits) - 1);
    int f = bits & ((1 << fbits) - 1);
    double mag;
    if (e == (1 << ebits) - 1) {
        mag = (f == 0) ? INFINITY : NAN;
    } else if (e == 0) {
        mag = ldexp((double)f, 1 - bias - fbits);           /* subnormal or zero */
    } else {
        mag = ldexp(1.0 + ldexp((double)f, -fbits), e - bias);
    }
    return sign ? -mag : mag;
}

/* 1 if the pattern is +-inf or NaN (Sec. 4.4: the global NaN/Inf check). */
int orc_is_nonfinite16(uint16_t bits, int dtype)
{
    return !isfinite(orc_decode16(bits, dtype));
}

/* Round an fp32 value to bf16, nearest, ties to the even 7-bit fraction.  NaN stays NaN
 * (quiet, sign kept); overflow past the largest finite bf16 goes to infinity, as IEEE
 * rounding prescribes. */
uint16_t orc_f32_to_bf16(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu) != 0u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t upper = u >> 16;
    uint32_t lower = u & 0xFFFFu;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u)))
        upper += 1u;
    return (uint16_t)upper;
}

/* Round an fp32 value to IEEE binary16 bits, nearest, ties to even: take the exact value,
 * find the spacing of binary16 numbers at its magnitude (2^-24 in the subnormal range,
 * 2^(e-10) for exponent e), divide, round the quotient to an integer with ties to even
 * (nearbyint under the default rounding mode), and re-encode.  Overflow past 65504 + half a
 * step gives infinity; NaN stays NaN. */
uint16_t orc_f32_to_fp16(float x)
{
    uint16_t sign = signbit(x) ? 0x8000u : 0u;
    if (isnan(x)) return (uint16_t)(sign | 0x7E00u);
    double a = fabs((double)x);
    if (isinf(a)) return (uint16_t)(sign | 0x7C00u);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);            /* a = f * 2^e, f in [0.5, 1)  ->  exponent of a is e - 1 */
    int ex = e - 1;
    if (ex < -14) ex = -14;        /* subnormal range shares the spacing of the smallest normal */
    double step = ldexp(1.0, ex - 10);
    double qd = nearbyint(a / step);            /* exact division by a power of two */
    /* qd in [0, 2048]; 2048 means the value rounded up into the next binade */
    long q = (long)qd;
    int be = ex + 15;              /* biased exponent if normal */
    if (q >= 2048) { q = 1024; be += 1; }
    uint16_t bits;
    if (q < 1024) bits = (uint16_t)q;                           /* subnormal (be == 1 here) */
    else bits = (uint16_t)((be << 10) | (q - 1024));
    if (be >= 31 && q >= 1024) bits = 0x7C00u;                  /* overflow */
    return (uint16_t)(sign | bits);
}

/* Gradient statistics of one bucket (Sec. 4.4): the count of non-finite gradient
 * elements and the sum of squares of the unscaled gradients g*inv_scale, accumulated in
 * double in index order.  Non-finite elements are counted but left out of the sum, so the
 * sum stays defined; callers ignore it whenever the count is non-zero. */
void orc_grad_stats(const uint16_t* g, uint64_t n, int dtype, float inv_scale,
                    double* sumsq, uint64_t* nonfinite)
{
    double acc = 0.0;
    uint64_t bad = 0;
    double s = (double)inv_scale;
    for (uint64_t i = 0; i < n; ++i) {
        double x = orc_decode16(g[i], dtype);
        if (!isfinite(x)) {
            ++bad;
        } else {
            double y = x * s;
            acc += y * y;
        }
    }
    *sumsq = acc;
    *nonfinite = bad;
}

/* beta^t by repeated multiplication in double (t >= 0). */
static double pow_int(double b, int64_t t)
{
    double r = 1.0;
    for (int64_t k = 0; k < t; ++k) r *= b;
    return r;
}

/*
 * One Adam(W) step over one bucket, in place.
 *
 *   g   16-bit gradients (dtype as above), n elements
 *   p,m,v  fp32 master parameter, first and second moment, n elements each, updated
 *   q   16-bit working copy of p (bit patterns; bf16, or binary16 if lp_fp16), n elements, written
 *   lr, beta1, beta2, eps, wd   hyper-parameters, given as fp32 and widened to double
 *   t   1-based count of applied steps (bias correction uses beta^t)
 *   s   multiplier applied to every gradient (clip coefficient / loss scale), fp32
 *   adamw            1: decoupled decay  p <- p - lr*wd*p - lr*mhat/(sqrt(vhat)+eps)
 *                    0: L2 decay folded into the gradient, g <- g*s + wd*p
 *   bias_correction  0 replaces both correction factors by 1
 *
 * Adam Algorithm 1: m <- b1 m + (1-b1) g ; v <- b2 v + (1-b2) g^2 ;
 * mhat = m/(1-b1^t) ; vhat = v/(1-b2^t) ; epsilon is added outside the square root.
 */
void orc_adamw_step(const uint16_t* g, int dtype, float* p, float* m, float* v, uint16_t* q,
                    uint64_t n, float lr_f, float beta1_f, float beta2_f, float eps_f,
                    float wd_f, int64_t t, float s_f, int adamw, int bias_correction, int lp_fp16)
{
    double lr = lr_f, b1 = beta1_f, b2 = beta2_f, eps = eps_f, wd = wd_f, s = s_f;
    double bc1 = 1.0, bc2 = 1.0;
    if (bias_correction) {
        bc1 = 1.0 - pow_int(b1, t);
        bc2 = 1.0 - pow_int(b2, t);
    }
    for (uint64_t i = 0; i < n; ++i) {
        double gi = orc_decode16(g[i], dtype) * s;
        double pi = p[i], mi = m[i], vi = v[i];
        if (!adamw) gi += wd * pi;
        double mn = b1 * mi + (1.0 - b1) * gi;
        double vn = b2 * vi + (1.0 - b2) * gi * gi;
        double mhat = mn / bc1;
        double vhat = vn / bc2;
        double pn = pi;
        if (adamw) pn -= lr * wd * pi;
        pn -= lr * mhat / (sqrt(vhat) + eps);
        m[i] = (float)mn;
        v[i] = (float)vn;
        p[i] = (float)pn;
        q[i] = lp_fp16 ? orc_f32_to_fp16(p[i]) : orc_f32_to_bf16(p[i]);
    }
}

/* 16-bit working copy of fp32 parameters (Sec. 4.5, the cast of mixed-precision training):
 * element by element the rounding that orc_adamw_step applies to the parameter it stores. */
void orc_cast_lp(const float* p, uint16_t* q, uint64_t n, int lp_fp16)
{
    for (uint64_t i = 0; i < n; ++i) q[i] = lp_fp16 ? orc_f32_to_fp16(p[i]) : orc_f32_to_bf16(p[i]);
}

/* Global-norm clipping coefficient (Sec. 4.4 cites norm clipping; the constant 1e-6 in the
 * denominator is this build's reading): min(1, max_norm / (norm + 1e-6)), in double.
 * max_norm <= 0 means "no clipping". */
double orc_clip_coef(double norm, double max_norm)
{
    if (!(max_norm > 0.0)) return 1.0;
    double c = max_norm / (norm + 1e-6);
    return c < 1.0 ? c : 1.0;
}
