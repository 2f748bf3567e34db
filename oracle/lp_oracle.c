/*
 * lp_oracle.c -- plain CPU definition of the low-precision forward pass.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement
 * of what the fixed-point layers of the paper compute.  It exists so that the
 * GPU library can be checked against it; nothing in the product path may call
 * it.  It shares no code, header, table or constant with the GPU library.
 *
 * What is implemented, and the passage of the paper each part follows:
 *
 *   orc_quantize   Qm.f fixed-point quantizer of the low-precision layers
 *                  (Sec. 2 "Low-precision add-on for Caffe": signed n-bit
 *                  value with m integer bits *including the sign* and f
 *                  fraction bits, parameters BD/AD; deterministic rounding;
 *                  Sec. 2.5 "Insights": values that do not fit saturate).
 *   orc_quantize_stochastic
 *                  the STOCHASTIC rounding_scheme (Sec. 2.4 "Deterministic vs.
 *                  Stochastic rounding"): one of the two
 *                  neighbouring grid points, up with probability equal to the
 *                  fractional part, so the expectation is the input.
 *   orc_range      layer-wise split of n bits into integer and fraction bits
 *                  from the dynamic range (Sec. 2.3 "Layer-wise quantization"):
 *                  fewest integer bits such that the share of values that can
 *                  no longer be represented stays below a threshold.
 *   orc_range_acc  the same rule applied to exact integer accumulators.
 *   orc_conv       LPConvolution forward on integer codes (Sec. 2), exact.
 *   orc_fc         LPInnerProduct forward on integer codes (Sec. 2), exact.
 *   orc_act        LPAct (+ ReLU) on exact accumulators: requantize to the
 *                  layer's output Qm.f (Sec. 2.1 workflow), count zeros
 *                  (sparsity = zeros / elements, Sec. 3.1).
 *   orc_act_stochastic
 *                  the same with the STOCHASTIC rounding_scheme (Sec. 2.4).
 *   orc_maxpool2x2 the 2x2/stride-2 pooling between VGG16 blocks (VGG16 is the
 *                  paper's benchmark network; "Pooling" column of Table 1).
 *
 * Conventions
 *   - A code q with format (n, m, f), n = m + f, stands for the real q * 2^-f
 *     and lies in [-2^(n-1), 2^(n-1) - 1].
 *   - Codes are held in int32_t, accumulators in int64_t, tensors in NCHW
 *     (activations) / [Cout][Cin][R][S] (weights) order.  Everything is a
 *     direct loop over the definition; there is no blocking or reordering.
 *   - Every function returns 0 on success, a negative number on bad arguments.
 *   - `threads` > 1 only spreads the outermost loop over OpenMP threads.
 *
 * Every function here is pinned by tests/test_oracle_*.py against
 * hand-worked values, closed forms, exact rational arithmetic, brute force and
 * library routines; none is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_ROUND_AWAY = 0, ORC_ROUND_EVEN = 1 };

static int fmt_ok(int n, int m, int f)
{
    return n >= 2 && n <= 16 && m >= 1 && m <= n && f >= 0 && n == m + f;
}

static int64_t code_min(int n) { return -((int64_t)1 << (n - 1)); }
static int64_t code_max(int n) { return ((int64_t)1 << (n - 1)) - 1; }

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------- quantize */

/* Sec. 2: value -> nearest multiple of 2^-f, saturated to the signed n-bit
 * range.  x * 2^f is exact in double for every float32 x, so the rounding acts
 * on the exact real.  NaN maps to code 0.  sat_count counts the inputs whose
 * rounded value had to be clipped; zero_count counts codes equal to 0. */
int orc_quantize(const float *x, int64_t count, int n, int m, int f, int mode,
                 int32_t *code, uint64_t *zero_count, uint64_t *sat_count)
{
    if (!fmt_ok(n, m, f) || count < 0 || (mode != ORC_ROUND_AWAY && mode != ORC_ROUND_EVEN))
        return -1;
    const double lo = (double)code_min(n), hi = (double)code_max(n);
    uint64_t zeros = 0, sats = 0;
    for (int64_t i = 0; i < count; ++i) {
        double t = ldexp((double)x[i], f);
        double r;
        if (isnan(t))
            r = 0.0;
        else if (mode == ORC_ROUND_AWAY)
            r = round(t);      /* halfway cases away from zero */
        else
            r = nearbyint(t);  /* halfway cases to even (default FP environment) */
        if (r < lo) { r = lo; ++sats; }
        if (r > hi) { r = hi; ++sats; }
        code[i] = (int32_t)r;
        zeros += (code[i] == 0);
    }
    if (zero_count) *zero_count = zeros;
    if (sat_count) *sat_count = sats;
    return 0;
}

/* Sec. 2.4: stochastic rounding.  u[i] in [0,1) is the random number drawn for
 * element i (passed in, so no generator lives here).  With t = x * 2^f the
 * result is floor(t) + 1 if u < t - floor(t), else floor(t); then saturate. */
int orc_quantize_stochastic(const float *x, const double *u, int64_t count, int n, int m, int f,
                            int32_t *code, uint64_t *zero_count, uint64_t *sat_count)
{
    if (!fmt_ok(n, m, f) || count < 0) return -1;
    const double lo = (double)code_min(n), hi = (double)code_max(n);
    uint64_t zeros = 0, sats = 0;
    for (int64_t i = 0; i < count; ++i) {
        double t = ldexp((double)x[i], f);
        double r;
        if (isnan(t)) {
            r = 0.0;
        } else {
            double fl = floor(t);
            double frac = t - fl; /* exact: t has at most 24 significant bits */
            r = (u[i] < frac) ? fl + 1.0 : fl;
        }
        if (r < lo) { r = lo; ++sats; }
        if (r > hi) { r = hi; ++sats; }
        code[i] = (int32_t)r;
        zeros += (code[i] == 0);
    }
    if (zero_count) *zero_count = zeros;
    if (sat_count) *sat_count = sats;
    return 0;
}

/* ------------------------------------------------------------------- range */

/* Sec. 2.3: with n fixed, a value is lost for m integer bits (sign included)
 * when its magnitude reaches 2^(m-1).  Returns through *m_out the smallest m
 * in [1, n] whose lost share is at most `threshold` (m = n if there is none).
 * lost[1..n] (optional, n+1 entries, entry 0 unused) receives the counts. */
int orc_range(const float *v, int64_t count, int n, double threshold, int *m_out, uint64_t *lost)
{
    if (n < 2 || n > 16 || count < 0 || !(threshold >= 0.0) || !m_out) return -1;
    int chosen = n;
    int found = 0;
    for (int m = 1; m <= n; ++m) {
        const double limit = ldexp(1.0, m - 1);
        uint64_t c = 0;
        for (int64_t i = 0; i < count; ++i)
            c += (fabs((double)v[i]) >= limit);
        if (lost) lost[m] = c;
        if (!found && (double)c <= threshold * (double)count) {
            chosen = m;
            found = 1;
        }
    }
    *m_out = chosen;
    return 0;
}

/* The same rule on exact accumulators that stand for acc * 2^-f_acc, after
 * ReLU when relu != 0 (negative values become 0 and are never lost). */
int orc_range_acc(const int64_t *acc, int64_t count, int f_acc, int relu, int n, double threshold,
                  int *m_out, uint64_t *lost)
{
    if (n < 2 || n > 16 || count < 0 || f_acc < 0 || f_acc > 40 || !(threshold >= 0.0) || !m_out)
        return -1;
    int chosen = n;
    int found = 0;
    for (int m = 1; m <= n; ++m) {
        const int64_t limit = (int64_t)1 << (m - 1 + f_acc);
        uint64_t c = 0;
        for (int64_t i = 0; i < count; ++i) {
            int64_t a = acc[i];
            if (relu && a < 0) a = 0;
            if (a >= limit || a <= -limit) ++c;
        }
        if (lost) lost[m] = c;
        if (!found && (double)c <= threshold * (double)count) {
            chosen = m;
            found = 1;
        }
    }
    *m_out = chosen;
    return 0;
}

/* -------------------------------------------------------------------- conv */

typedef struct {
    int N, Cin, H, W, Cout, R, S, stride, pad;
} orc_conv_shape;

static int conv_shape_ok(const orc_conv_shape *c)
{
    return c && c->N > 0 && c->Cin > 0 && c->H > 0 && c->W > 0 && c->Cout > 0 && c->R > 0 &&
           c->S > 0 && c->stride > 0 && c->pad >= 0 && c->H + 2 * c->pad >= c->R &&
           c->W + 2 * c->pad >= c->S;
}

int orc_conv_out_hw(const orc_conv_shape *c, int *Ho, int *Wo)
{
    if (!conv_shape_ok(c)) return -1;
    *Ho = (c->H + 2 * c->pad - c->R) / c->stride + 1;
    *Wo = (c->W + 2 * c->pad - c->S) / c->stride + 1;
    return 0;
}

/* One output of the cross-correlation (no kernel flip), zero outside the
 * image: sum over ci, r, s of X[n,ci,y*stride+r-pad,x*stride+s-pad] * W[co,ci,r,s]. */
static int64_t conv_one(const orc_conv_shape *c, const int32_t *x, const int32_t *w, int n, int co,
                        int y, int xo)
{
    int64_t acc = 0;
    for (int ci = 0; ci < c->Cin; ++ci)
        for (int r = 0; r < c->R; ++r) {
            const int iy = y * c->stride + r - c->pad;
            if (iy < 0 || iy >= c->H) continue;
            for (int s = 0; s < c->S; ++s) {
                const int ix = xo * c->stride + s - c->pad;
                if (ix < 0 || ix >= c->W) continue;
                const int64_t a = x[(((int64_t)n * c->Cin + ci) * c->H + iy) * c->W + ix];
                const int64_t b = w[(((int64_t)co * c->Cin + ci) * c->R + r) * c->S + s];
                acc += a * b;
            }
        }
    return acc;
}

/* bias code with fb fraction bits joins an accumulator with f_acc fraction
 * bits as bias * 2^(f_acc - fb); needs fb <= f_acc (Sec. 2.1: biases are
 * quantized blobs like the weights). */
static int bias_shift_ok(const int32_t *bias, int f_acc, int fb)
{
    return !bias || (fb >= 0 && fb <= f_acc && f_acc - fb < 40);
}

/* LPConvolution forward, Sec. 2.  acc is [N][Cout][Ho][Wo]; its fraction bits
 * are f_acc = fx + fw (the caller's bookkeeping; only f_acc - fb is used). */
int orc_conv(const orc_conv_shape *c, const int32_t *x, const int32_t *w, const int32_t *bias,
             int f_acc, int fb, int64_t *acc, int threads)
{
    int Ho, Wo;
    if (orc_conv_out_hw(c, &Ho, &Wo) || !x || !w || !acc || !bias_shift_ok(bias, f_acc, fb))
        return -1;
    const int64_t rows = (int64_t)c->N * c->Cout;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(threads > 1 ? threads : 1)
#endif
    for (int64_t row = 0; row < rows; ++row) {
        const int n = (int)(row / c->Cout), co = (int)(row % c->Cout);
        for (int y = 0; y < Ho; ++y)
            for (int xo = 0; xo < Wo; ++xo) {
                int64_t a = conv_one(c, x, w, n, co, y, xo);
                if (bias) a += (int64_t)bias[co] * ((int64_t)1 << (f_acc - fb));
                acc[(row * Ho + y) * Wo + xo] = a;
            }
    }
    (void)threads;
    return 0;
}

/* The same definition evaluated only at listed flat output indices
 * ((n*Cout + co)*Ho + y)*Wo + x, for spot checks at sizes where the whole
 * tensor would take too long. */
int orc_conv_sampled(const orc_conv_shape *c, const int32_t *x, const int32_t *w,
                     const int32_t *bias, int f_acc, int fb, const int64_t *flat_index,
                     int64_t count, int64_t *acc)
{
    int Ho, Wo;
    if (orc_conv_out_hw(c, &Ho, &Wo) || !x || !w || !acc || !flat_index ||
        !bias_shift_ok(bias, f_acc, fb))
        return -1;
    const int64_t total = (int64_t)c->N * c->Cout * Ho * Wo;
    for (int64_t i = 0; i < count; ++i) {
        int64_t t = flat_index[i];
        if (t < 0 || t >= total) return -2;
        const int xo = (int)(t % Wo); t /= Wo;
        const int y = (int)(t % Ho);  t /= Ho;
        const int co = (int)(t % c->Cout);
        const int n = (int)(t / c->Cout);
        int64_t a = conv_one(c, x, w, n, co, y, xo);
        if (bias) a += (int64_t)bias[co] * ((int64_t)1 << (f_acc - fb));
        acc[i] = a;
    }
    return 0;
}

/* ---------------------------------------------------------------------- fc */

/* LPInnerProduct forward, Sec. 2: acc[b][o] = sum_k X[b][k] * W[o][k] (+bias). */
int orc_fc(int M, int K, int Nout, const int32_t *x, const int32_t *w, const int32_t *bias,
           int f_acc, int fb, int64_t *acc, int threads)
{
    if (M <= 0 || K <= 0 || Nout <= 0 || !x || !w || !acc || !bias_shift_ok(bias, f_acc, fb))
        return -1;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(threads > 1 ? threads : 1)
#endif
    for (int b = 0; b < M; ++b)
        for (int o = 0; o < Nout; ++o) {
            int64_t a = 0;
            for (int k = 0; k < K; ++k)
                a += (int64_t)x[(int64_t)b * K + k] * (int64_t)w[(int64_t)o * K + k];
            if (bias) a += (int64_t)bias[o] * ((int64_t)1 << (f_acc - fb));
            acc[(int64_t)b * Nout + o] = a;
        }
    (void)threads;
    return 0;
}

/* --------------------------------------------------------------------- act */

/* LPAct followed by the activation function, Sec. 2.1.  The accumulator stands
 * for acc * 2^-f_acc; the output code has fo fraction bits, so the real value
 * is divided by 2^s, s = f_acc - fo, rounded to nearest and saturated to n
 * bits.  ReLU and this quantizer commute (it is monotone and maps 0 to 0), so
 * max(acc, 0) is taken first.  zero_count = number of output codes equal to 0
 * (Sec. 3.1: sparsity is zeros over elements).  sat_count (optional) = number
 * of elements whose rounded value lay outside the code range and was clipped:
 * the share of activations the layer's format loses (Sec. 2.3 keeps that
 * share under a user threshold when it places the point). */
int orc_act(const int64_t *acc, int64_t count, int f_acc, int n, int m, int fo, int relu, int mode,
            int32_t *code, uint64_t *zero_count, uint64_t *sat_count)
{
    if (!fmt_ok(n, m, fo) || count < 0 || f_acc < 0 || (mode != ORC_ROUND_AWAY && mode != ORC_ROUND_EVEN))
        return -1;
    const int s = f_acc - fo;
    if (s > 62 || s < -31) return -1;
    const int64_t lo = code_min(n), hi = code_max(n);
    const int64_t bound = (int64_t)1 << 62;
    uint64_t zeros = 0, sats = 0;
    for (int64_t i = 0; i < count; ++i) {
        int64_t v = acc[i];
        if (v >= bound || v <= -bound) return -2; /* outside the supported accumulator width */
        if (relu && v < 0) v = 0;
        int64_t r;
        if (s > 0) {
            const int64_t d = (int64_t)1 << s;
            if (mode == ORC_ROUND_AWAY) {
                const int64_t mag = v < 0 ? -v : v;
                const int64_t q = (mag + d / 2) / d; /* halfway cases go up in magnitude */
                r = v < 0 ? -q : q;
            } else {
                int64_t q = v / d, rem = v % d;  /* C division truncates toward zero ... */
                if (rem < 0) { q -= 1; rem += d; } /* ... turn it into floor division */
                if (2 * rem > d) q += 1;
                else if (2 * rem == d) q += (q & 1); /* halfway cases to the even neighbour */
                r = q;
            }
        } else {
            /* multiply by 2^-s >= 1; a magnitude already beyond the code range stays beyond */
            if (v > hi) r = hi + 1;
            else if (v < lo) r = lo - 1;
            else r = v * ((int64_t)1 << (-s));
        }
        if (r < lo) { r = lo; ++sats; }
        if (r > hi) { r = hi; ++sats; }
        code[i] = (int32_t)r;
        zeros += (r == 0);
    }
    if (zero_count) *zero_count = zeros;
    if (sat_count) *sat_count = sats;
    return 0;
}

/* LPAct with the STOCHASTIC rounding_scheme of Sec. 2.4, then as orc_act.  u[i]
 * in [0,1) is the random number drawn for element i (passed in).  With
 * t = max(acc,0) / 2^s the code is floor(t) + 1 if u < t - floor(t), else
 * floor(t); s <= 0 needs no rounding.  The comparison is exact: t - floor(t) is
 * rem / 2^s with an integer rem < 2^62, so u * 2^s (a power-of-two scaling) is
 * compared with rem in long double (64-bit significand, asserted below). */
int orc_act_stochastic(const int64_t *acc, const double *u, int64_t count, int f_acc, int n, int m,
                       int fo, int relu, int32_t *code, uint64_t *zero_count, uint64_t *sat_count)
{
    _Static_assert(__LDBL_MANT_DIG__ >= 64, "long double must hold a 62-bit integer exactly");
    if (!fmt_ok(n, m, fo) || count < 0 || f_acc < 0) return -1;
    const int s = f_acc - fo;
    if (s > 62 || s < -31) return -1;
    const int64_t lo = code_min(n), hi = code_max(n);
    const int64_t bound = (int64_t)1 << 62;
    uint64_t zeros = 0, sats = 0;
    for (int64_t i = 0; i < count; ++i) {
        int64_t v = acc[i];
        if (v >= bound || v <= -bound) return -2;
        if (!(u[i] >= 0.0 && u[i] < 1.0)) return -3;
        if (relu && v < 0) v = 0;
        int64_t r;
        if (s > 0) {
            const int64_t d = (int64_t)1 << s;
            int64_t q = v / d, rem = v % d;
            if (rem < 0) { q -= 1; rem += d; } /* floor division */
            if ((long double)ldexp(u[i], s) < (long double)rem) q += 1;
            r = q;
        } else {
            if (v > hi) r = hi + 1;
            else if (v < lo) r = lo - 1;
            else r = v * ((int64_t)1 << (-s));
        }
        if (r < lo) { r = lo; ++sats; }
        if (r > hi) { r = hi; ++sats; }
        code[i] = (int32_t)r;
        zeros += (r == 0);
    }
    if (zero_count) *zero_count = zeros;
    if (sat_count) *sat_count = sats;
    return 0;
}

/* ----------------------------------------------------------------- maxpool */

/* 2x2 max, stride 2, on codes in NCHW; H and W must be even. */
int orc_maxpool2x2(const int32_t *x, int N, int C, int H, int W, int32_t *y)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || (H & 1) || (W & 1) || !x || !y) return -1;
    const int Ho = H / 2, Wo = W / 2;
    for (int64_t p = 0; p < (int64_t)N * C; ++p)
        for (int i = 0; i < Ho; ++i)
            for (int j = 0; j < Wo; ++j) {
                const int32_t *q = x + (p * H + 2 * i) * W + 2 * j;
                int32_t best = q[0];
                if (q[1] > best) best = q[1];
                if (q[W] > best) best = q[W];
                if (q[W + 1] > best) best = q[W + 1];
                y[(p * Ho + i) * Wo + j] = best;
            }
    return 0;
}
