/*
 * CPU oracle for ActorQ 8-bit policy inference (arXiv 1910.01055).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the GPU
 * library is checked against.  It shares no code, header, table or constant
 * with the HIP path and must never be called from it.
 *
 * What it follows:
 *   - Sec. 3.2 "Post-Training Quantization": uniform affine quantization
 *     Q_n(W) = round(W / delta), delta spanning |min(W,0)| + |max(W,0)|,
 *     dequantization D(W_q, delta) = delta * W_q, per-channel quantization
 *     for convolutions, weights and activations at the same precision.
 *   - Sec. 3.1: actors run the quantized policy; the learner stays fp32
 *     (the fp64 forward below is that full-precision policy).
 * The paper gives no integer recipe (zero-point, accumulator, requantization);
 * the readings taken here are listed beside each function.
 *
 * Every loop is written in the order of the definition: batch row outermost,
 * then output feature, then the reduction index.  No blocking, no SIMD
 * intrinsics, no reordering.  OpenMP only splits the outermost (independent)
 * batch/row loop.
 *
 * Pin status: every function here is pinned by tests/test_oracle_pins.py
 * against closed forms, hand-exact cases, big-integer brute force or a
 * textbook library routine, except the int8-vs-fp32 action error, which is a
 * reported number only ("parity unpinned").
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_OK = 0, ORC_EINVAL = 1, ORC_ENONFINITE = 3, ORC_EOVERFLOW = 7 };

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of threads the batch-row loops may use from now on (a benchmark reports the oracle on one core
 * next to the oracle on all of them); returns the count in effect. */
int orc_set_num_threads(int n) {
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
    return omp_get_max_threads();
#else
    (void)n;
    return 1;
#endif
}

/* round-half-to-even of v (default FP environment), then clamp to [lo, hi] in
 * float before the conversion so that huge or NaN inputs are defined: values
 * not >= lo (NaN included) give lo. */
static int32_t rint_clamp(float v, int32_t lo, int32_t hi) {
    float r = rintf(v);
    if (!(r >= (float)lo)) return lo;
    if (r > (float)hi) return hi;
    return (int32_t)r;
}

/* ------------------------------------------------------------------------
 * Sec. 3.2, delta = (|min(W,0)| + |max(W,0)|) / 2^n.
 * Reading: affine with zero-point z = round(-lo / s); qdenom is 255 for the
 * default 2^n - 1 reading (error <= s/2 everywhere) or 256 for the literal
 * 2^n.  All arithmetic in fp32, IEEE division, round-half-even.
 * -------------------------------------------------------------------- */
/* n-bit form (Sec. 3.2 states Q_n for a general n; App. on quantization-aware training sweeps n below 8):
 * qdenom = 2^n - 1 or 2^n as above, codes and zero-point in [0, qmax] with qmax = 2^n - 1. */
int orc_qparams_asym_n(const float* w, int64_t n, float qdenom, int32_t qmax, float* scale, int32_t* zp) {
    float lo = 0.0f, hi = 0.0f; /* min(W,0), max(W,0): zero is always inside */
    for (int64_t i = 0; i < n; ++i) {
        if (!isfinite(w[i])) return ORC_ENONFINITE;
        if (w[i] < lo) lo = w[i];
        if (w[i] > hi) hi = w[i];
    }
    float s = (hi - lo) / qdenom;
    if (hi == lo) s = 1.0f;
    *scale = s;
    *zp = rint_clamp(-lo / s, 0, qmax);
    return ORC_OK;
}

int orc_qparams_asym(const float* w, int64_t n, float qdenom, float* scale, int32_t* zp) {
    return orc_qparams_asym_n(w, n, qdenom, 255, scale, zp);
}

/* q = clamp(round(W / s) + z, 0, qmax), unsigned codes (8-bit containers). */
void orc_quantize_asym_n(const float* w, int64_t n, float scale, int32_t zp, int32_t qmax, uint8_t* q) {
    for (int64_t i = 0; i < n; ++i)
        q[i] = (uint8_t)(rint_clamp(w[i] / scale, -zp, qmax - zp) + zp);
}

void orc_quantize_asym(const float* w, int64_t n, float scale, int32_t zp, uint8_t* q) {
    orc_quantize_asym_n(w, n, scale, zp, 255, q);
}

/* D(W_q, delta) = delta * (W_q - z) (Sec. 3.2 dequantization with the zero-point reading). */
void orc_dequantize_asym(const uint8_t* q, int64_t n, float scale, int32_t zp, float* w) {
    for (int64_t i = 0; i < n; ++i) w[i] = scale * (float)((int32_t)q[i] - zp);
}

/* Per-output-channel symmetric: each row n of W[rows][cols] gets
 * s[n] = max_k |W[n,k]| / 127 (all-zero row: s = 1), codes in [-127, 127]. */
/* n-bit form: s[n] = max|W| / qw, codes in [-qw, qw], qw = 2^(n-1) - 1 (127 for 8 bits). */
int orc_quantize_sym_rows_n(const float* w, int64_t rows, int64_t cols, int32_t qw, float* scales, int8_t* q) {
    for (int64_t r = 0; r < rows; ++r) {
        float m = 0.0f;
        for (int64_t c = 0; c < cols; ++c) {
            float v = w[r * cols + c];
            if (!isfinite(v)) return ORC_ENONFINITE;
            float a = fabsf(v);
            if (a > m) m = a;
        }
        float s = m / (float)qw;
        if (m == 0.0f) s = 1.0f;
        scales[r] = s;
        for (int64_t c = 0; c < cols; ++c)
            q[r * cols + c] = (int8_t)rint_clamp(w[r * cols + c] / s, -qw, qw);
    }
    return ORC_OK;
}

int orc_quantize_sym_rows(const float* w, int64_t rows, int64_t cols, float* scales, int8_t* q) {
    return orc_quantize_sym_rows_n(w, rows, cols, 127, scales, q);
}

void orc_dequantize_sym_rows(const int8_t* q, int64_t rows, int64_t cols, const float* scales, float* w) {
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) w[r * cols + c] = scales[r] * (float)q[r * cols + c];
}

/* ------------------------------------------------------------------------
 * Per-layer integer constants.  The paper is silent; reading:
 *   m[n]      = s_in * s_w[n]                       (one fp32 multiply)
 *   bias_q[n] = round(b[n] / (s_in * s_w[n]))       (fp64, saturated to int32)
 *   M[n]      = s_in * s_w[n] / s_out  (fp64) = f * 2^e, f in [0.5, 1)
 *   M0[n]     = round(f * 2^31) normalised into [2^30, 2^31), r[n] = 31 - e
 * s_out <= 0 means the layer is not requantized (last layer, LayerNorm layer);
 * then M0 and r are written as 0.
 * -------------------------------------------------------------------- */
int orc_layer_consts(float s_in, const float* s_w, float s_out, const float* bias, int64_t n_out,
                     float* m, int32_t* bias_q, int32_t* M0, int32_t* rshift) {
    for (int64_t n = 0; n < n_out; ++n) {
        m[n] = s_in * s_w[n];
        double sw = (double)s_in * (double)s_w[n];
        double bq = rint((double)bias[n] / sw);
        if (!(bq >= -2147483647.0)) bq = -2147483647.0;
        if (bq > 2147483647.0) bq = 2147483647.0;
        bias_q[n] = (int32_t)bq;
        if (s_out > 0.0f) {
            double M = sw / (double)s_out;
            int e;
            double f = frexp(M, &e);
            int64_t q = llround(f * 2147483648.0);
            if (q == 2147483648LL) { q = 1073741824LL; e += 1; }
            int32_t r = 31 - e;
            if (r < 1 || r > 62) return ORC_EINVAL;
            M0[n] = (int32_t)q;
            rshift[n] = r;
        } else {
            M0[n] = 0;
            rshift[n] = 0;
        }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------
 * Fully connected accumulator: the zero-point-corrected integer dot product
 *   acc[b,n] = bias_q[n] + sum_k (a[b,k] - z_a) * (w[n,k] - z_w[n])
 * a: unsigned 8-bit codes [B][K]; w: codes widened to int16 [N][K] (unsigned
 * 0..255 or signed -127..127).  Summed in int64 and required to fit int32.
 * -------------------------------------------------------------------- */
int orc_fc_acc(const uint8_t* a, int64_t B, int64_t K, int32_t z_a, const int16_t* w, int64_t N,
               const int32_t* z_w, const int32_t* bias_q, int32_t* acc) {
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t n = 0; n < N; ++n) {
            int64_t s = bias_q[n];
            for (int64_t k = 0; k < K; ++k)
                s += (int64_t)((int32_t)a[b * K + k] - z_a) * (int64_t)((int32_t)w[n * K + k] - z_w[n]);
            if (s > 2147483647LL || s < -2147483648LL) bad = 1;
            acc[b * N + n] = (int32_t)s;
        }
    }
    return bad ? ORC_EOVERFLOW : ORC_OK;
}

/* Direct VALID convolution, NHWC input a[B][H][W][C], weights w[Co][kh][kw][C],
 * output acc[B][OH][OW][Co], OH = (H - kh) / stride + 1.  Seven loops, as the
 * definition reads. */
int orc_conv_acc(const uint8_t* a, int64_t B, int64_t H, int64_t W, int64_t C, int32_t z_a,
                 const int16_t* w, int64_t Co, int64_t kh, int64_t kw, int64_t stride,
                 const int32_t* z_w, const int32_t* bias_q, int32_t* acc) {
    int64_t OH = (H - kh) / stride + 1, OW = (W - kw) / stride + 1;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t oy = 0; oy < OH; ++oy)
            for (int64_t ox = 0; ox < OW; ++ox)
                for (int64_t co = 0; co < Co; ++co) {
                    int64_t s = bias_q[co];
                    for (int64_t ky = 0; ky < kh; ++ky)
                        for (int64_t kx = 0; kx < kw; ++kx)
                            for (int64_t ci = 0; ci < C; ++ci) {
                                int32_t av = a[((b * H + oy * stride + ky) * W + ox * stride + kx) * C + ci];
                                int32_t wv = w[((co * kh + ky) * kw + kx) * C + ci];
                                s += (int64_t)(av - z_a) * (int64_t)(wv - z_w[co]);
                            }
                    if (s > 2147483647LL || s < -2147483648LL) bad = 1;
                    acc[((b * OH + oy) * OW + ox) * Co + co] = (int32_t)s;
                }
    return bad ? ORC_EOVERFLOW : ORC_OK;
}

/* Requantize a hidden layer: v = (acc * M0 + 2^(r-1)) >> r  (int64, arithmetic
 * shift, ties toward +inf), a' = clamp(v + z_out, relu ? z_out : 0, 255). */
void orc_requant(const int32_t* acc, int64_t rows, int64_t N, const int32_t* M0, const int32_t* rshift,
                 int32_t z_out, int32_t relu, uint8_t* out) {
    int64_t lo = relu ? z_out : 0;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < rows; ++b)
        for (int64_t n = 0; n < N; ++n) {
            int64_t p = (int64_t)acc[b * N + n] * (int64_t)M0[n] + ((int64_t)1 << (rshift[n] - 1));
            int64_t v = (p >> rshift[n]) + z_out; /* >> on a negative int64 is arithmetic with gcc */
            if (v < lo) v = lo;
            if (v > 255) v = 255;
            out[b * N + n] = (uint8_t)v;
        }
}

/* Dequantized layer output y[b,n] = (float)acc[b,n] * m[n]: two correctly
 * rounded fp32 operations, hence reproducible bit for bit. */
void orc_dequant_acc(const int32_t* acc, int64_t rows, int64_t N, const float* m, float* y) {
    for (int64_t b = 0; b < rows; ++b)
        for (int64_t n = 0; n < N; ++n) y[b * N + n] = (float)acc[b * N + n] * m[n];
}

/* LayerNorm over the N features of a row (biased variance, eps inside the
 * square root, gain and offset), then tanh; statistics in fp64 on the fp32
 * dequantized accumulators; t rounded to fp32; then requantized with the
 * activation's (s_out, z_out) in fp32 like any other activation. */
void orc_ln_tanh(const int32_t* acc, int64_t rows, int64_t N, const float* m, const float* gamma,
                 const float* beta, double eps, float s_out, int32_t z_out, float* t_out, uint8_t* codes) {
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < rows; ++b) {
        double mu = 0.0;
        for (int64_t n = 0; n < N; ++n) mu += (double)((float)acc[b * N + n] * m[n]);
        mu /= (double)N;
        double var = 0.0;
        for (int64_t n = 0; n < N; ++n) {
            double d = (double)((float)acc[b * N + n] * m[n]) - mu;
            var += d * d;
        }
        var /= (double)N;
        double inv = 1.0 / sqrt(var + eps);
        for (int64_t n = 0; n < N; ++n) {
            double x = (double)((float)acc[b * N + n] * m[n]);
            double y = (x - mu) * inv * (double)gamma[n] + (double)beta[n];
            float t = (float)tanh(y);
            t_out[b * N + n] = t;
            codes[b * N + n] = (uint8_t)(rint_clamp(t / s_out, -z_out, 255 - z_out) + z_out);
        }
    }
}

/* tanh of fp32 values evaluated in fp64 and rounded to fp32. */
void orc_tanh_f32(const float* y, int64_t n, float* t) {
    for (int64_t i = 0; i < n; ++i) t[i] = (float)tanh((double)y[i]);
}

/* Row-wise argmax, lowest index on ties. */
void orc_argmax_rows(const float* y, int64_t rows, int64_t N, int32_t* idx) {
    for (int64_t b = 0; b < rows; ++b) {
        int32_t best = 0;
        for (int64_t n = 1; n < N; ++n)
            if (y[b * N + n] > y[b * N + best]) best = (int32_t)n;
        idx[b] = best;
    }
}

/* ------------------------------------------------------------------------
 * Exploration on the actor (Sec. 4.1): Gaussian noise on the policy output
 * with a per-actor sigma (continuous control), epsilon-greedy on the argmax
 * action (discrete control; the paper names DQN, epsilon-greedy is that
 * algorithm's exploration rule).
 *
 * The random numbers come from the counter-based generator Philox4x32-10 as
 * defined by Salmon, Moraes, Dror and Shaw, "Parallel random numbers: as easy
 * as 1, 2, 3" (SC'11): ten rounds of
 *     (hi0, lo0) = M0 * c0      (32 x 32 -> 64 bit products)
 *     (hi1, lo1) = M1 * c2
 *     c <- (hi1 ^ c1 ^ k0,  lo1,  hi0 ^ c3 ^ k1,  lo0)
 * with the key advanced by the Weyl constants (W0, W1) before every round
 * but the first.  Readings taken here (the paper fixes none of this):
 *   key     = (seed low word, seed high word)
 *   counter = (batch row, block, step low word, step high word)
 *   Gaussian noise: block = feature index / 4; the four output words give two
 *     Box-Muller pairs, u1 = ((x >> 8) + 1) / 2^24 in (0, 1], u2 = (y >> 8) / 2^24
 *     in [0, 1); z_even = sqrt(-2 ln u1) cos(2 pi u2), z_odd = ... sin(2 pi u2);
 *     action' = action + sigma[row] * z, evaluated in fp64, rounded to fp32.
 *     No clipping (the paper states none).
 *   epsilon-greedy: block = 0xFFFFFFFF; u = (x0 >> 8) / 2^24 as fp32 (exact);
 *     if u < epsilon (fp32 compare) the action becomes floor(x1 * A / 2^32).
 * ---------------------------------------------------------------------- */
void orc_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0;
        c1 = n1;
        c2 = n2;
        c3 = n3;
    }
    out[0] = c0;
    out[1] = c1;
    out[2] = c2;
    out[3] = c3;
}

void orc_explore_gaussian(float* actions, int64_t rows, int64_t A, const float* sigma, uint64_t seed,
                          uint64_t step) {
    const double two_pi = 6.283185307179586476925286766559;
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    for (int64_t b = 0; b < rows; ++b) {
        for (int64_t n = 0; n < A; ++n) {
            const uint32_t ctr[4] = {(uint32_t)b, (uint32_t)(n / 4), (uint32_t)step, (uint32_t)(step >> 32)};
            uint32_t r[4];
            orc_philox4x32_10(ctr, key, r);
            const int j = (int)(n % 4), pair = j / 2;
            const double u1 = ((double)(r[2 * pair] >> 8) + 1.0) / 16777216.0;
            const double u2 = (double)(r[2 * pair + 1] >> 8) / 16777216.0;
            const double rad = sqrt(-2.0 * log(u1));
            const double z = (j % 2 == 0) ? rad * cos(two_pi * u2) : rad * sin(two_pi * u2);
            actions[b * A + n] = (float)((double)actions[b * A + n] + (double)sigma[b] * z);
        }
    }
}

void orc_explore_eps_greedy(int32_t* idx, int64_t rows, int64_t A, float epsilon, uint64_t seed, uint64_t step) {
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    for (int64_t b = 0; b < rows; ++b) {
        const uint32_t ctr[4] = {(uint32_t)b, 0xFFFFFFFFu, (uint32_t)step, (uint32_t)(step >> 32)};
        uint32_t r[4];
        orc_philox4x32_10(ctr, key, r);
        const float u = (float)(r[0] >> 8) * (1.0f / 16777216.0f);
        if (u < epsilon) idx[b] = (int32_t)(((uint64_t)r[1] * (uint64_t)A) >> 32);
    }
}

/* ------------------------------------------------------------------------
 * Full-precision policy (the learner's / the fp32 actor's network), evaluated
 * in fp64 from fp32 parameters: textbook affine layer, VALID convolution,
 * ReLU, LayerNorm and tanh.  Activations stay fp64 between layers.
 * -------------------------------------------------------------------- */
void orc_fc_f64(const double* x, int64_t B, int64_t K, const float* w, const float* bias, int64_t N, double* y) {
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t n = 0; n < N; ++n) {
            double s = (double)bias[n];
            for (int64_t k = 0; k < K; ++k) s += x[b * K + k] * (double)w[n * K + k];
            y[b * N + n] = s;
        }
}

void orc_conv_f64(const double* x, int64_t B, int64_t H, int64_t W, int64_t C, const float* w,
                  const float* bias, int64_t Co, int64_t kh, int64_t kw, int64_t stride, double* y) {
    int64_t OH = (H - kh) / stride + 1, OW = (W - kw) / stride + 1;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t oy = 0; oy < OH; ++oy)
            for (int64_t ox = 0; ox < OW; ++ox)
                for (int64_t co = 0; co < Co; ++co) {
                    double s = (double)bias[co];
                    for (int64_t ky = 0; ky < kh; ++ky)
                        for (int64_t kx = 0; kx < kw; ++kx)
                            for (int64_t ci = 0; ci < C; ++ci)
                                s += x[((b * H + oy * stride + ky) * W + ox * stride + kx) * C + ci] *
                                     (double)w[((co * kh + ky) * kw + kx) * C + ci];
                    y[((b * OH + oy) * OW + ox) * Co + co] = s;
                }
}

void orc_relu_f64(double* x, int64_t n) {
    for (int64_t i = 0; i < n; ++i)
        if (x[i] < 0.0) x[i] = 0.0;
}

void orc_tanh_f64(double* x, int64_t n) {
    for (int64_t i = 0; i < n; ++i) x[i] = tanh(x[i]);
}

void orc_layernorm_f64(double* x, int64_t rows, int64_t N, const float* gamma, const float* beta, double eps) {
    for (int64_t b = 0; b < rows; ++b) {
        double mu = 0.0;
        for (int64_t n = 0; n < N; ++n) mu += x[b * N + n];
        mu /= (double)N;
        double var = 0.0;
        for (int64_t n = 0; n < N; ++n) var += (x[b * N + n] - mu) * (x[b * N + n] - mu);
        var /= (double)N;
        double inv = 1.0 / sqrt(var + eps);
        for (int64_t n = 0; n < N; ++n) x[b * N + n] = (x[b * N + n] - mu) * inv * (double)gamma[n] + (double)beta[n];
    }
}

/* ------------------------------------------------------------------------
 * Half-precision actor (the paper's fp16 policies: Sec. 3.2 quantizes trained
 * policies "to fp16 and int8", Sec. 5 / App. runtime breakdown runs actors at
 * q = 16).  Reading: every tensor of the half-precision policy - parameters,
 * the observation, and the output of every operator (affine layer, LayerNorm,
 * tanh, action head) - is an IEEE binary16 value; an operator's arithmetic is
 * exact (fp64 here) and its result is rounded once, to nearest, ties to even.
 * The only new arithmetic is that rounding, written out from the format:
 * 1 sign, 5 exponent (bias 15), 10 fraction bits, gradual underflow below
 * 2^-14, overflow to infinity at and above 65520.
 * The rounded value is returned widened to fp32 (exactly representable).
 * -------------------------------------------------------------------- */
static double round_half_even_int(double v) {
    /* v >= 0, below 2^52: nearest integer, ties to the even one */
    double f = floor(v);
    double d = v - f;
    if (d > 0.5) return f + 1.0;
    if (d < 0.5) return f;
    return fmod(f, 2.0) == 0.0 ? f : f + 1.0;
}

static float round_binary16(double x) {
    if (isnan(x)) return NAN;
    double a = fabs(x);
    double r;
    if (a == 0.0) {
        r = 0.0;
    } else if (isinf(a)) {
        r = INFINITY;
    } else {
        int e;
        (void)frexp(a, &e); /* a = m * 2^e, m in [0.5, 1): a in [2^(e-1), 2^e) */
        int exp2 = e - 1;   /* floor(log2 a) */
        if (exp2 < -14) exp2 = -14; /* subnormal range shares the spacing of the lowest binade */
        double ulp = ldexp(1.0, exp2 - 10); /* spacing of binary16 values in this binade */
        r = round_half_even_int(a / ulp) * ulp; /* a / ulp < 2^11 + 1: exact in fp64 */
        if (r >= 65520.0) r = INFINITY; /* 65504 is the largest finite value; halfway to 2^16 rounds up */
    }
    return (float)(x < 0.0 || (x == 0.0 && signbit(x)) ? -r : r);
}

void orc_round_fp16(const double* x, int64_t n, float* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = round_binary16(x[i]);
}
