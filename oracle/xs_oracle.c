/*
 * CPU oracle for the fused gradient-synchronisation step of CrossoverScheduler
 * (arXiv 2103.07974).  TEST INFRASTRUCTURE ONLY: tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it; no product code does, and it shares
 * no code, header, table or helper with the HIP library.
 *
 * The method is exact (a schedule plus a fusion, Sections 2.1-2.2: the result of
 * every task equals plain synchronous data-parallel SGD), so each function here
 * is the plain definition written as scalar loops, one tensor element at a time,
 * with no blocking, fusion or reordering:
 *
 *   layout / pack / unpack  - Section 2.1, tensor fusion: all gradient tensors of
 *                             one model are laid end to end in one buffer
 *                             (Algorithm 1, step "Fuse all gradient into one group").
 *   average                 - Algorithm 1, step "Receive averaged gradients":
 *                             the W workers' fused gradients are summed and
 *                             divided by W (data parallelism, Section 1).
 *   update                  - Algorithm 1, step "Model Update", x <- SGD(x, g).
 *                             The paper does not say which SGD; the reading taken
 *                             is the momentum form of the framework it used
 *                             (Section 3.1):  d = g + wd*x ; v = mu*v + d ;
 *                             x = x - lr*v  (no dampening, no Nesterov).
 *   loss scale / skip       - not in the paper; mixed-precision workload only:
 *                             gradients are multiplied by 1/loss_scale, and if any
 *                             valid gradient element of any worker is inf or NaN
 *                             the whole step is skipped and a flag is raised.
 *
 * Arithmetic: xo_reduce_sgd_f64 computes in IEEE double (the definition).
 * xo_reduce_sgd_f32 takes the same steps with every operation rounded to IEEE
 * single, replicas added left to right, no fused multiply-add (build with
 * -ffp-contract=off); it exists so that tests can also report the distance in
 * units in the last place from a single-precision evaluation.
 *
 * Parity pins (tests/test_oracle_*.py): pack->unpack identity and pure-Python
 * concatenation; identical replicas; exact integer sums; closed-form momentum
 * recurrences and a 2x2 matrix power; torch.optim.SGD in double; hand-derived
 * values in tests/golden/; a one-operation-at-a-time Python brute force.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#include <math.h>

#define XO_F32 0
#define XO_F16 1
#define XO_BF16 2   /* bfloat16: the upper half of an IEEE single */

/* ---- layout: Section 2.1 (tensor fusion) -------------------------------- */
/* offsets[0] = 0; offsets[t+1] = offsets[t] + numel[t] rounded up to a multiple
 * of align.  align = 1 is plain concatenation; offsets[T] is the bucket length. */
int xo_layout(const uint64_t *numel, uint32_t n_tensors, uint64_t align, uint64_t *offsets)
{
    if (align == 0) return -1;
    offsets[0] = 0;
    for (uint32_t t = 0; t < n_tensors; ++t) {
        uint64_t end = offsets[t] + numel[t];
        uint64_t rem = end % align;
        if (rem != 0) end += align - rem;
        offsets[t + 1] = end;
    }
    return 0;
}

/* ---- pack: Algorithm 1, "Fuse all gradient into one group" ---------------- */
/* Bit copy of each tensor, in list order, to bucket[offsets[t] ...]; every
 * bucket element not covered by a tensor (padding) becomes +0. */
int xo_pack(uint32_t elem_size, uint32_t n_tensors, const void *const *tensors,
            const uint64_t *numel, const uint64_t *offsets, void *bucket)
{
    unsigned char *b = (unsigned char *)bucket;
    memset(b, 0, (size_t)(offsets[n_tensors] * elem_size));
    for (uint32_t t = 0; t < n_tensors; ++t) {
        const unsigned char *src = (const unsigned char *)tensors[t];
        for (uint64_t k = 0; k < numel[t]; ++k)
            for (uint32_t c = 0; c < elem_size; ++c)
                b[(offsets[t] + k) * elem_size + c] = src[k * elem_size + c];
    }
    return 0;
}

/* ---- unpack: inverse of pack; padding is ignored -------------------------- */
int xo_unpack(uint32_t elem_size, uint32_t n_tensors, const void *bucket,
              const uint64_t *numel, const uint64_t *offsets, void *const *tensors)
{
    const unsigned char *b = (const unsigned char *)bucket;
    for (uint32_t t = 0; t < n_tensors; ++t) {
        unsigned char *dst = (unsigned char *)tensors[t];
        for (uint64_t k = 0; k < numel[t]; ++k)
            for (uint32_t c = 0; c < elem_size; ++c)
                dst[k * elem_size + c] = b[(offsets[t] + k) * elem_size + c];
    }
    return 0;
}

/* ---- IEEE binary16 -> double, exact -------------------------------------- */
static double half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)       v = ldexp((double)m, -24);               /* zero / subnormal */
    else if (e == 31) v = (m == 0) ? INFINITY : NAN;
    else              v = ldexp((double)(1024 + m), e - 25);
    return sign ? -v : v;
}

/* ---- bfloat16 -> double, exact: sign, 8 exponent bits, 7 fraction bits ------- */
static double bfloat_to_double(uint16_t b)
{
    int sign = (b >> 15) & 1;
    int e = (b >> 7) & 0xff;
    int m = b & 0x7f;
    double v;
    if (e == 0)        v = ldexp((double)m, -133);              /* zero / subnormal: m * 2^-7 * 2^-126 */
    else if (e == 255) v = (m == 0) ? INFINITY : NAN;
    else               v = ldexp((double)(128 + m), e - 134);   /* (1 + m/128) * 2^(e-127) */
    return sign ? -v : v;
}

static double load_grad(const void *p, int dtype, uint64_t j)
{
    if (dtype == XO_F16) return half_to_double(((const uint16_t *)p)[j]);
    if (dtype == XO_BF16) return bfloat_to_double(((const uint16_t *)p)[j]);
    return (double)((const float *)p)[j];
}

/* ---- overflow test on the valid elements of W packed buckets ------------- */
/* Returns 1 if any element inside a tensor's range (padding excluded) of any
 * replica is +-inf or NaN, else 0. */
int xo_any_nonfinite(const void *const *replicas, uint32_t W, int dtype, uint32_t n_tensors,
                     const uint64_t *numel, const uint64_t *offsets)
{
    for (uint32_t w = 0; w < W; ++w)
        for (uint32_t t = 0; t < n_tensors; ++t)
            for (uint64_t k = 0; k < numel[t]; ++k) {
                double g = load_grad(replicas[w], dtype, offsets[t] + k);
                if (!isfinite(g)) return 1;
            }
    return 0;
}

/* ---- average + update, double precision (the definition) ------------------ */
/* For every bucket element j:
 *   s     = g_0[j] + g_1[j] + ... + g_{W-1}[j]
 *   g_avg = s / W * inv_loss_scale
 *   d     = g_avg + wd * x[j];  v[j] = mu * v[j] + d;  x[j] = x[j] - lr * v[j]
 * x and v are double arrays updated in place. */
int xo_reduce_sgd_f64(const void *const *replicas, uint32_t W, int dtype, uint64_t n,
                      double *x, double *v, double lr, double mu, double wd,
                      double inv_loss_scale, int threads)
{
    if (W == 0) return -1;
    int64_t nn = (int64_t)n;
    #pragma omp parallel for num_threads(threads) if (threads > 1)
    for (int64_t j = 0; j < nn; ++j) {
        double s = 0.0;
        for (uint32_t w = 0; w < W; ++w) s += load_grad(replicas[w], dtype, (uint64_t)j);
        double g_avg = s / (double)W * inv_loss_scale;
        double d = g_avg + wd * x[j];
        v[j] = mu * v[j] + d;
        x[j] = x[j] - lr * v[j];
    }
    return 0;
}

/* ---- the same steps with every operation rounded to single ---------------- */
/* Replicas added left to right starting from g_0; the averaging and the loss
 * scale are one multiplication by the single-precision constant
 * inv_loss_scale * (1/W). */
int xo_reduce_sgd_f32(const void *const *replicas, uint32_t W, int dtype, uint64_t n,
                      float *x, float *v, float lr, float mu, float wd,
                      float inv_loss_scale, int threads)
{
    if (W == 0) return -1;
    int64_t nn = (int64_t)n;
    volatile float one_over_w = 1.0f / (float)W;
    const float c = inv_loss_scale * one_over_w;
    #pragma omp parallel for num_threads(threads) if (threads > 1)
    for (int64_t j = 0; j < nn; ++j) {
        float s = (float)load_grad(replicas[0], dtype, (uint64_t)j);
        for (uint32_t w = 1; w < W; ++w) {
            float g = (float)load_grad(replicas[w], dtype, (uint64_t)j);
            s = s + g;
        }
        float g_avg = s * c;
        float wx = wd * x[j];
        float d = g_avg + wx;
        float mv = mu * v[j];
        float vn = mv + d;
        float lv = lr * vn;
        v[j] = vn;
        x[j] = x[j] - lv;
    }
    return 0;
}

/* ---- half-precision copy of the updated parameters (mixed-precision workload) -------- */
/* Round each single-precision value to the nearest binary16 / bfloat16, ties to even,
 * written out on the value (frexp/ldexp/nearbyint), not on the bit pattern.  Overflow goes
 * to infinity, NaN stays NaN (quiet, sign kept), results below the smallest normal are
 * rounded on the subnormal grid. */
static uint16_t round_to_small_float(float xf, int exp_bits, int frac_bits)
{
    const int bias = (1 << (exp_bits - 1)) - 1;
    const int emax = bias;                 /* largest finite exponent */
    const int emin = 1 - bias;             /* smallest normal exponent */
    uint16_t sign = signbit(xf) ? (uint16_t)(1u << (exp_bits + frac_bits)) : 0;
    const uint16_t exp_all = (uint16_t)(((1u << exp_bits) - 1) << frac_bits);
    if (isnan(xf)) return (uint16_t)(sign | exp_all | (1u << (frac_bits - 1)));
    if (isinf(xf)) return (uint16_t)(sign | exp_all);
    double a = fabs((double)xf);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                    /* a = f * 2^e, f in [0.5, 1)  =>  a in [2^(e-1), 2^e) */
    int ex = e - 1;                        /* a = m * 2^ex, m in [1, 2) */
    if (ex < emin) ex = emin;              /* subnormal grid shares the smallest normal's spacing */
    double q = ldexp(a, frac_bits - ex);   /* in units of the last place */
    double r = nearbyint(q);               /* ties to even in the default rounding mode */
    if (r >= ldexp(1.0, frac_bits + 1)) { r = ldexp(r, -1); ex += 1; }   /* rounded up to 2.0 */
    if (ex > emax) return (uint16_t)(sign | exp_all);                     /* overflow */
    uint32_t ri = (uint32_t)r;
    if (ri < (1u << frac_bits)) return (uint16_t)(sign | ri);             /* subnormal or zero */
    return (uint16_t)(sign | (uint32_t)((ex + bias) << frac_bits) | (ri - (1u << frac_bits)));
}

int xo_round_params(const float *x, uint64_t n, int dtype, uint16_t *out)
{
    if (dtype != XO_F16 && dtype != XO_BF16) return -1;
    for (uint64_t j = 0; j < n; ++j)
        out[j] = (dtype == XO_F16) ? round_to_small_float(x[j], 5, 10)
                                   : round_to_small_float(x[j], 8, 7);
    return 0;
}
