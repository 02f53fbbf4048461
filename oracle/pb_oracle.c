/*
 * pb_oracle.c -- plain CPU oracle for the PrecisionBatching hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  Slow, obviously-correct C written from the paper
 * (arXiv 2003.00822).  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the HIP product path never does and shares no
 * code, table or helper with it.
 *
 * Each function follows one step of the method and cites the passage it
 * restates.  Where the paper is silent or inconsistent the reading taken is
 * written next to the step.  Floating point is fp64 except where the paper
 * fixes fp32 (weights, activations, scales, outputs are fp32 arrays).
 *
 * Parity pins (tests marked "not gpu"): the printed 2x2 worked example of the
 * supplementary material, exhaustive two's-complement reconstruction, numpy
 * int64 brute-force products, one-hot / all-ones / INT32_MIN activation
 * vectors, exact rational dequantization, a library LSTM cell.
 * Parity unpinned (definitions by choice, the paper prints no values for them):
 *   - pbo_quantize: symmetric step d = max|W| / (2^(B-1)-1), round-half-even;
 *     only invariants are pinned.
 *   - pbo_quantize_mode: the three other quantizers of Section 3.3 (the
 *     printed range formula, the 1-bit +-1 code, the clipping search); the
 *     paper gives the formula of the first only, the scale of the second and
 *     the error measure and candidate set of the third are readings; only
 *     invariants are pinned.
 *   - pbo_fixed_point: saturation and NaN rule of the fp32 -> fixed cast.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* Section 3.3 (weight quantization): Q(W) = d * round(W / d), values on a
 * linearly spaced grid.  Reading: the grid is symmetric per tensor,
 * d = max|W| / (2^(B-1) - 1) for a B-bit two's-complement code (B counts the
 * sign layer), codes clamped to [-2^(B-1), 2^(B-1)-1]; "round" is
 * round-half-to-even in fp32; an all-zero matrix takes d = 1; for B = 1 the
 * divisor is 1 (codes {-1, 0}).  Returns the integer codes q = round(W/d)
 * and d; Q(W) = d * q. */
int pbo_quantize(const float *W, int64_t n, int bits, int32_t *q, float *d_out)
{
    if (bits < 1 || bits > 16 || n < 0) return -1;
    float M = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        float a = fabsf(W[i]);
        if (a > M) M = a;
    }
    int32_t qmax = (1 << (bits - 1)) - 1;
    int32_t qmin = -(1 << (bits - 1));
    float d = (M == 0.0f) ? 1.0f : M / (float)(qmax > 0 ? qmax : 1);
    for (int64_t i = 0; i < n; ++i) {
        float r = rintf(W[i] / d); /* default rounding mode: to nearest, ties to even */
        int32_t v;
        if (r != r) v = 0;
        else if (r >= (float)qmax) v = qmax;
        else if (r <= (float)qmin) v = qmin;
        else v = (int32_t)r;
        q[i] = v;
    }
    *d_out = d;
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Section 3.3, the other quantizers it describes.  All keep the grid linearly
 * spaced (Q(W) = d * q, q a B-bit two's-complement code), so the bitlayers and
 * scales follow from (q, d) exactly as for pbo_quantize.
 *
 * mode 1, "range": the printed formula, d = (max(W) - min(W)) / 2^n with
 *   n = B - 1 magnitude bits (PBatch-n stores n + 1 layers), q = round(W / d)
 *   clamped to the code range [-2^n, 2^n - 1]; d = 1 if max = min.
 * mode 2, "sign": "for quantizing to 1 bit ... exclude representing 0 and
 *   instead ... represent a positive and negative value": q = +1 for W >= 0,
 *   -1 otherwise (B = 2: sign layer + one magnitude layer).  The paper gives
 *   no scale; reading: d = mean|W| (the least-squares scale of a sign code).
 * mode 3, "clip": "optimize over a clipping threshold to find a quantized
 *   matrix with the smallest mean error versus the full precision weight
 *   matrix".  Reading: thresholds T_k = max|W| * k / 32, k = 1..32; for each,
 *   the symmetric quantizer with d_k = T_k / (2^(B-1) - 1) and clamping; the
 *   error is the mean of |W - d_k q|; the smallest wins, the larger threshold
 *   on a tie.
 * So that a parallel implementation can reproduce the sums bit for bit, the two
 * means are taken over values truncated to multiples of 2^(e-30), where
 * 2^e <= max|W| < 2^(e+1): integers below 2^31, summed exactly in 64 bits
 * (n <= 2^32 elements).  fp32 products and differences are rounded separately
 * (compiled without contraction). */
static uint64_t pbo_fix30(float a, int e) /* trunc(|a| * 2^(30-e)), a finite, |a| < 2^(e+1) */
{
    float t = truncf(ldexpf(fabsf(a), 30 - e));
    return (t != t) ? 0u : (uint64_t)t;
}

static int32_t pbo_round_clamp(float w, float d, int32_t qmin, int32_t qmax)
{
    float r = rintf(w / d);
    if (r != r) return 0;
    if (r >= (float)qmax) return qmax;
    if (r <= (float)qmin) return qmin;
    return (int32_t)r;
}

int pbo_quantize_mode(const float *W, int64_t n, int bits, int mode, int32_t *q, float *d_out)
{
    if (bits < 1 || bits > 16 || n < 1) return -1;
    if (mode == 0) return pbo_quantize(W, n, bits, q, d_out);
    float M = 0.0f, hi = -INFINITY, lo = INFINITY;
    for (int64_t i = 0; i < n; ++i) {
        float w = W[i];
        if (w != w) continue;
        if (fabsf(w) > M) M = fabsf(w);
        if (w > hi) hi = w;
        if (w < lo) lo = w;
    }
    int32_t qmax = (1 << (bits - 1)) - 1, qmin = -(1 << (bits - 1));
    int e = 0;
    if (M > 0.0f) (void)frexpf(M, &e), e -= 1; /* M = f * 2^(e+1), 0.5 <= f < 1  ->  2^e <= M */
    if (mode == 1) {
        float d = (hi > lo) ? (hi - lo) / (float)(1 << (bits - 1)) : 1.0f;
        for (int64_t i = 0; i < n; ++i) q[i] = pbo_round_clamp(W[i], d, qmin, qmax);
        *d_out = d;
        return 0;
    }
    if (mode == 2) {
        if (bits != 2) return -1;
        uint64_t S = 0;
        for (int64_t i = 0; i < n; ++i) {
            if (W[i] != W[i]) { q[i] = 1; continue; }
            S += pbo_fix30(W[i], e);
            q[i] = (W[i] >= 0.0f) ? 1 : -1;
        }
        *d_out = (float)(ldexp((double)S, e - 30) / (double)n);
        return 0;
    }
    if (mode == 3) {
        int32_t qm = qmax > 0 ? qmax : 1;
        if (M == 0.0f) {
            for (int64_t i = 0; i < n; ++i) q[i] = 0;
            *d_out = 1.0f;
            return 0;
        }
        int best = 32;
        uint64_t best_err = 0;
        for (int k = 32; k >= 1; --k) {
            float T = M * ((float)k * 0.03125f);
            float d = T / (float)qm;
            uint64_t E = 0;
            for (int64_t i = 0; i < n; ++i) {
                if (W[i] != W[i]) continue;
                float p = d * (float)pbo_round_clamp(W[i], d, qmin, qmax);
                E += pbo_fix30(W[i] - p, e);
            }
            if (k == 32 || E < best_err) { best = k; best_err = E; }
        }
        float d = (M * ((float)best * 0.03125f)) / (float)qm;
        for (int64_t i = 0; i < n; ++i) q[i] = pbo_round_clamp(W[i], d, qmin, qmax);
        *d_out = d;
        return 0;
    }
    return -1;
}

/* ------------------------------------------------------------------------ */
/* Section 3.2 (two's-complement extension), Algorithm 1 (bitlayers W^(b) and
 * scales S, first scale negated) and the printed example of the supplement:
 * the B-bit two's-complement image of each code is split into B bitlayers,
 * most significant (sign) layer first; layer i holds bit B-1-i and has the
 * integer scale s_0 = -2^(B-1), s_i = +2^(B-1-i).
 * layers: [bits][n] of 0/1 bytes; s: [bits]. */
int pbo_bitlayers(const int32_t *q, int64_t n, int bits, uint8_t *layers, int64_t *s)
{
    if (bits < 1 || bits > 16) return -1;
    for (int i = 0; i < bits; ++i) {
        int pos = bits - 1 - i;
        s[i] = (i == 0) ? -((int64_t)1 << pos) : ((int64_t)1 << pos);
        for (int64_t e = 0; e < n; ++e) {
            uint32_t u = (uint32_t)q[e];
            layers[(int64_t)i * n + e] = (uint8_t)((u >> pos) & 1u);
        }
    }
    return 0;
}

/* Algorithm 1, scales S: the step d of the grid is folded into the power-of-two
 * layer scale, scales[i] = d * s_i (exact in fp32 up to over/underflow). */
void pbo_scales(float d, int bits, float *scales)
{
    for (int i = 0; i < bits; ++i) {
        int pos = bits - 1 - i;
        float si = ldexpf(1.0f, pos);
        scales[i] = (i == 0) ? -(d * si) : d * si;
    }
}

/* ------------------------------------------------------------------------ */
/* Section 3.3 (activations: "a multiplication and a cast") and Algorithm 2,
 * x_q = Int(x * 2^f).  Reading: the product is taken in fp32 (exact, a power
 * of two), the cast truncates toward zero, values outside the k-bit
 * two's-complement range saturate, NaN maps to 0.  act_bits = k (32 on the
 * main path). */
int pbo_fixed_point(const float *x, int64_t n, int frac_bits, int act_bits, int32_t *xq)
{
    if (act_bits < 2 || act_bits > 32) return -1;
    double hi = ldexp(1.0, act_bits - 1) - 1.0; /*  2^(k-1) - 1 */
    double lo = -ldexp(1.0, act_bits - 1);      /* -2^(k-1)     */
    for (int64_t i = 0; i < n; ++i) {
        float p = x[i] * ldexpf(1.0f, frac_bits);
        double t;
        if (p != p) t = 0.0;
        else t = trunc((double)p);
        if (t > hi) t = hi;
        if (t < lo) t = lo;
        xq[i] = (int32_t)t;
    }
    return 0;
}

/* Section 3.2 (x as k bitlayers, first one negated), Algorithm 2 (plane
 * weights [-2^31, 2^30, ..., 2^0]) and the printed x^(b), S_x of the
 * supplement: plane j holds bit j of the k-bit two's-complement image of x_q;
 * its weight is c_j = 2^j, except the top plane, c_(k-1) = -2^(k-1).
 * planes: [k][n] of 0/1 bytes (index 0 = least significant); c: [k]. */
int pbo_planes(const int32_t *xq, int64_t n, int act_bits, uint8_t *planes, int64_t *c)
{
    if (act_bits < 2 || act_bits > 32) return -1;
    for (int j = 0; j < act_bits; ++j) {
        c[j] = (j == act_bits - 1) ? -((int64_t)1 << j) : ((int64_t)1 << j);
        for (int64_t e = 0; e < n; ++e)
            planes[(int64_t)j * n + e] = (uint8_t)(((uint32_t)xq[e] >> j) & 1u);
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Section 3.1, the batched product W^(b)_i [x^(b)_1 ... x^(b)_k]: every entry
 * is a sum of 1-bit products (Section 3.4: AND, then a population count).
 * layer: [R][C] 0/1, planes: [k][C] 0/1, P: [R][k]. */
void pbo_bit_products(const uint8_t *layer, const uint8_t *planes, int64_t R, int64_t C, int k, int64_t *P)
{
    for (int64_t r = 0; r < R; ++r)
        for (int j = 0; j < k; ++j) {
            int64_t cnt = 0;
            for (int64_t col = 0; col < C; ++col)
                cnt += (int64_t)(layer[r * C + col] & planes[(int64_t)j * C + col]);
            P[r * k + j] = cnt;
        }
}

/* Algorithm 2, the right-multiplication by the plane-weight vector:
 * A[r] = sum_j c_j * P[r][j]. */
void pbo_plane_weighting(const int64_t *P, const int64_t *c, int64_t R, int k, int64_t *A)
{
    for (int64_t r = 0; r < R; ++r) {
        int64_t a = 0;
        for (int j = 0; j < k; ++j) a += c[j] * P[r * k + j];
        A[r] = a;
    }
}

/* Algorithm 2, the loop over (bitlayer, scale) pairs, restricted to the first
 * m pairs (the number of bitlayers accumulated is the run-time knob of the
 * abstract and of Section 1): T[r] = sum_{i<m} s_i * A[i][r].
 * Reading: "first m" is in most-significant-first order, i.e. the sign layer
 * and the top m-1 magnitude layers. */
void pbo_accumulate(const int64_t *A, const int64_t *s, int m, int64_t R, int64_t *T)
{
    for (int64_t r = 0; r < R; ++r) {
        int64_t t = 0;
        for (int i = 0; i < m; ++i) t += s[i] * A[(int64_t)i * R + r];
        T[r] = t;
    }
}

/* Algorithm 2, z <- z + scale / 2^32 * (...): with d folded into the scales
 * the divisor left is the activations' 2^f.  y[r] = fp32( sum_{i<m}
 * scales[i] * A[i][r] * 2^-f ), the sum taken in fp64 in layer order. */
void pbo_dequant(const int64_t *A, const float *scales, int m, int64_t R, int frac_bits, float *y)
{
    for (int64_t r = 0; r < R; ++r) {
        double z = 0.0;
        for (int i = 0; i < m; ++i)
            z += (double)scales[i] * (double)A[(int64_t)i * R + r];
        y[r] = (float)ldexp(z, -frac_bits);
    }
}

/* ------------------------------------------------------------------------ */
/* Algorithm 2 end to end, one activation vector at a time, in the paper's
 * order: fixed point -> planes -> per bitlayer: 1-bit products, plane
 * weighting -> accumulation over the first m layers -> fp32.
 * layers: [B][R][C] 0/1 bytes; X: [N][C] fp32.
 * Outputs (any may be NULL): A [m][N][R], T [N][R], Y [N][R].
 * s (integer layer scales, [B]) is needed for T only. */
int pbo_matmul_bitserial(const uint8_t *layers, const float *scales, const int64_t *s, int bits, int bits_used,
                         int64_t R, int64_t C, const float *X, int64_t N, int frac_bits, int act_bits,
                         int64_t *A_out, int64_t *T_out, float *Y_out)
{
    if (bits_used < 1 || bits_used > bits) return -1;
    int k = act_bits, m = bits_used;
    int32_t *xq = (int32_t *)malloc(sizeof(int32_t) * (size_t)C);
    uint8_t *planes = (uint8_t *)malloc((size_t)k * (size_t)C);
    int64_t *c = (int64_t *)malloc(sizeof(int64_t) * (size_t)k);
    int64_t *P = (int64_t *)malloc(sizeof(int64_t) * (size_t)R * (size_t)k);
    int64_t *A = (int64_t *)malloc(sizeof(int64_t) * (size_t)m * (size_t)R);
    if (!xq || !planes || !c || !P || !A) { free(xq); free(planes); free(c); free(P); free(A); return -2; }
    for (int64_t n = 0; n < N; ++n) {
        pbo_fixed_point(X + n * C, C, frac_bits, act_bits, xq);
        pbo_planes(xq, C, act_bits, planes, c);
        for (int i = 0; i < m; ++i) {
            pbo_bit_products(layers + (int64_t)i * R * C, planes, R, C, k, P);
            pbo_plane_weighting(P, c, R, k, A + (int64_t)i * R);
        }
        if (A_out)
            for (int i = 0; i < m; ++i)
                memcpy(A_out + ((int64_t)i * N + n) * R, A + (int64_t)i * R, sizeof(int64_t) * (size_t)R);
        if (T_out && s) pbo_accumulate(A, s, m, R, T_out + n * R);
        if (Y_out) pbo_dequant(A, scales, m, R, frac_bits, Y_out + n * R);
    }
    free(xq); free(planes); free(c); free(P); free(A);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* The plain result the method reaches exactly (Section 3.1: the decomposition
 * is a rewriting of W x): per bitlayer, A_i[n][r] = sum_c bit_i[r][c] * x_q[n][c].
 * Written out as that definition, with no bit planes.  A: [m][N][R]. */
void pbo_layer_products_direct(const uint8_t *layers, int bits_used, int64_t R, int64_t C,
                               const int32_t *xq, int64_t N, int64_t *A)
{
    for (int i = 0; i < bits_used; ++i)
        for (int64_t n = 0; n < N; ++n)
            for (int64_t r = 0; r < R; ++r) {
                int64_t a = 0;
                const uint8_t *row = layers + ((int64_t)i * R + r) * C;
                for (int64_t col = 0; col < C; ++col)
                    if (row[col]) a += (int64_t)xq[n * C + col];
                A[((int64_t)i * N + n) * R + r] = a;
            }
}

/* ------------------------------------------------------------------------ */
/* Section 3.4, "packing the 0s and 1s into the bits of an integer array":
 * the same algorithm on packed words (AND + popcount).  Plain uint64 words,
 * bit (c mod 64) of word c/64, zero padding.  Used for large shapes and as
 * the timed CPU baseline; checked against the byte-per-bit functions above. */
int64_t pbo_words_per_row(int64_t C) { return (C + 63) / 64; }

void pbo_pack_words(const uint8_t *bits01, int64_t R, int64_t C, uint64_t *words)
{
    int64_t Cw = pbo_words_per_row(C);
    memset(words, 0, sizeof(uint64_t) * (size_t)R * (size_t)Cw);
    for (int64_t r = 0; r < R; ++r)
        for (int64_t col = 0; col < C; ++col)
            if (bits01[r * C + col]) words[r * Cw + col / 64] |= (uint64_t)1 << (col % 64);
}

/* layers_w: [B][R][Cw] packed weight bitlayers; X: [N][C]; rows [r0, r1) only.
 * A_out: [m][N][R] (only rows r0..r1-1 written); Y_out: [N][R] likewise. */
int pbo_matmul_words(const uint64_t *layers_w, const float *scales, int bits, int bits_used,
                     int64_t R, int64_t C, int64_t r0, int64_t r1, const float *X, int64_t N,
                     int frac_bits, int act_bits, int64_t *A_out, float *Y_out)
{
    if (bits_used < 1 || bits_used > bits) return -1;
    int k = act_bits, m = bits_used;
    int64_t Cw = pbo_words_per_row(C);
    int32_t *xq = (int32_t *)malloc(sizeof(int32_t) * (size_t)C);
    uint8_t *planes = (uint8_t *)malloc((size_t)k * (size_t)C);
    uint64_t *planes_w = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)k * (size_t)Cw);
    int64_t *c = (int64_t *)malloc(sizeof(int64_t) * (size_t)k);
    int64_t *Arow = (int64_t *)malloc(sizeof(int64_t) * (size_t)m);
    if (!xq || !planes || !planes_w || !c || !Arow) {
        free(xq); free(planes); free(planes_w); free(c); free(Arow);
        return -2;
    }
    for (int64_t n = 0; n < N; ++n) {
        pbo_fixed_point(X + n * C, C, frac_bits, act_bits, xq);
        pbo_planes(xq, C, act_bits, planes, c);
        pbo_pack_words(planes, k, C, planes_w); /* the bitwise transpose of Section 3.4 */
        for (int64_t r = r0; r < r1; ++r) {
            for (int i = 0; i < m; ++i) {
                const uint64_t *wrow = layers_w + ((int64_t)i * R + r) * Cw;
                int64_t a = 0;
                for (int j = 0; j < k; ++j) {
                    const uint64_t *prow = planes_w + (int64_t)j * Cw;
                    int64_t cnt = 0;
                    for (int64_t w = 0; w < Cw; ++w) cnt += __builtin_popcountll(wrow[w] & prow[w]);
                    a += c[j] * cnt;
                }
                Arow[i] = a;
                if (A_out) A_out[((int64_t)i * N + n) * R + r] = a;
            }
            if (Y_out) {
                double z = 0.0;
                for (int i = 0; i < m; ++i) z += (double)scales[i] * (double)Arow[i];
                Y_out[n * R + r] = (float)ldexp(z, -frac_bits);
            }
        }
    }
    free(xq); free(planes); free(planes_w); free(c); free(Arow);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* LSTM cell on top of the quantized product (Section 4.2/4.3: the LSTM's input
 * and hidden linear maps are replaced by the quantized product, the
 * nonlinearities stay in full precision).  The paper does not print the cell
 * equations; reading: the standard cell, gate order (i, f, g, o) along the
 * 4H rows of the fused gate matrix applied to [x_t ; h_(t-1)]:
 *   c' = sigmoid(f) * c + sigmoid(i) * tanh(g),  h' = sigmoid(o) * tanh(c').
 * gates: [N][4H] pre-activations without bias; bias: [4H] or NULL.
 * Computed in fp64, rounded to fp32. */
static double sigmoid_d(double v) { return 1.0 / (1.0 + exp(-v)); }

void pbo_lstm_pointwise(const float *gates, const float *bias, const float *c_prev, int64_t H, int64_t N,
                        float *h_out, float *c_out)
{
    for (int64_t n = 0; n < N; ++n)
        for (int64_t u = 0; u < H; ++u) {
            const float *g = gates + n * 4 * H;
            double gi = (double)g[u] + (bias ? (double)bias[u] : 0.0);
            double gf = (double)g[H + u] + (bias ? (double)bias[H + u] : 0.0);
            double gg = (double)g[2 * H + u] + (bias ? (double)bias[2 * H + u] : 0.0);
            double go = (double)g[3 * H + u] + (bias ? (double)bias[3 * H + u] : 0.0);
            double cn = sigmoid_d(gf) * (double)c_prev[n * H + u] + sigmoid_d(gi) * tanh(gg);
            double hn = sigmoid_d(go) * tanh(cn);
            c_out[n * H + u] = (float)cn;
            h_out[n * H + u] = (float)hn;
        }
}
