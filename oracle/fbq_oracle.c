/*
 * CPU oracle for the sub-branched weight-only-quantized linear layer of FBQuant.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 definition that the
 * GPU library is checked against.  It shares no code, header, table or helper with
 * the HIP path, and nothing in the product may call it: only tests, the smoke check
 * and the benchmark's cpu_baseline leg do.
 *
 * What it computes (paper notation on the left, this file's row-major arrays on the right;
 * N = output features, K = input features, g = group size along K, G = K/g, b = bits,
 * qmax = 2^b - 1, r = rank, M = tokens):
 *
 *   Sigma = B.A            (Sec. 4.2, low-rank sub-branch)     Sigma[n,k] = sum_j A[k,j] * B[j,n]
 *                          the paper's A is r x d_in and B is d_out x r; here A is [K,r] and
 *                          B is [r,N] (y = x.A.B), i.e. the transposes.
 *   Q(W - Sigma)           (Sec. 4.1, feedback: the sub-branch is subtracted before the
 *                          round-to-nearest linear quantizer; Alg. 1 forward line)
 *   W_F = Q(W - Sigma) + Sigma        (Sec. 4.1, definition of the reconstructed weight)
 *   Z' = Q(W - Sigma) X^T + B A X^T   (Alg. 1, "quantization output")   y = x.Wq^T + (x.A).B
 *
 * The paper fixes only "linear quantizer", "round-to-nearest", "scaling factor s" and "group
 * size 128".  The reading taken here (asymmetric min-max, real-valued fp16 zero):
 *   per row n and group of g consecutive k:  mn = min R, mx = max R  (R = W - Sigma)
 *   s = (mx - mn)/qmax (1 if the group is constant), stored as fp16 (RNE; smallest normal
 *   if it underflows); z = -mn/s16 stored as fp16; if fp16 rounding of s or z pushes an end of
 *   the range more than half a step outside [0, qmax], s16 is bumped to the next fp16 and z
 *   recomputed, so that no element is ever clamped by more than the rounding itself;
 *   q = clamp(round_half_even(R/s16 + z16), 0, qmax);   dequant  w_q = s16 * (q - z16).
 * With this reading |W - W_F| = s16*|u - q| <= s16/2 for every element (Sec. 4.1, the bound).
 *
 * Packed layout of the codes (uint32 words, rows contiguous, row stride K*b/32 words):
 *   b = 4: word k/8 holds code k%8 = i at bits [4i, 4i+4).
 *   b = 3: codes k/32 = u live in words 3u, 3u+1, 3u+2.  For j = k%32 < 30: word j/10,
 *          field i = j%10; fields 0..4 sit at bits [3i, 3i+3), fields 5..9 at bits
 *          [16+3(i-5), 16+3(i-5)+3).  Code 30 is spread over bit 15 of the three words
 *          (bit c of the code in word c); code 31 likewise over bit 31.
 *
 * Parity pins (tests/test_oracle_*.py): fp16 conversions against numpy for every bit pattern;
 * codes in range and arg-min by brute force over all 2^b candidates; pack/unpack round trips
 * and a bit-by-bit layout check with Python integers; dequantized values on the group grid;
 * the identity W - W_F = R - Q(R) and the s/2 bound, with the negative case (no feedback)
 * violating it; y against exact rational arithmetic on tiny layers, against a dense fp64 GEMM
 * of the materialised W_F, against numpy's textbook group-RTN GEMV when B = 0, and exactly
 * against integer arithmetic when s = 1, z = 0; the reconstruction step's loss against the trace
 * form, its gradients against the closed form of Sec. 4.2 and against central differences of the
 * loss with the quantized weight held fixed, the exact zero of dL/dA while B = 0, and the s/2 bound
 * after every update.  No function here is left unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define FBQO_OK 0
#define FBQO_BAD_ARG 1
#define FBQO_NO_MEM 2

/* ---------------------------------------------------------------- fp16 <-> fp64 */

/* IEEE binary16 bit pattern -> double, exact. */
double fbqo_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);                 /* zero and subnormals: m * 2^-24 */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m + 1024), e - 25);     /* (1 + m/1024) * 2^(e-15) */
    return sign ? -v : v;
}

/* double -> IEEE binary16 bit pattern, round to nearest, ties to even. */
uint16_t fbqo_double_to_half(double d)
{
    uint16_t sign = signbit(d) ? 0x8000u : 0u;
    double a = fabs(d);
    if (isnan(d)) return 0x7e00u;
    if (a >= 65520.0) return sign | 0x7c00u;       /* halfway between 65504 and 2^16 rounds to inf */
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                            /* a = f * 2^e, f in [0.5, 1) */
    int q = e - 11;                                /* spacing of fp16 values near a is 2^q ... */
    if (q < -24) q = -24;                          /* ... but never finer than the subnormal step */
    double scaled = ldexp(a, -q);                  /* exact: a power-of-two scaling */
    double rn = nearbyint(scaled);                 /* default rounding mode: ties to even */
    /* rn is an integer in [0, 2048]; value = rn * 2^q */
    if (rn == 0.0) return sign;
    int mant = (int)rn;
    if (mant == 2048) { mant = 1024; q += 1; }
    if (mant < 1024)                               /* subnormal (only possible when q == -24) */
        return sign | (uint16_t)mant;
    int ebits = q + 25;                            /* (1024+m) * 2^(ebits-25) */
    if (ebits >= 31) return sign | 0x7c00u;
    return sign | (uint16_t)(ebits << 10) | (uint16_t)(mant - 1024);
}

void fbqo_half_to_double_array(const uint16_t *h, double *out, long n)
{
    for (long i = 0; i < n; ++i) out[i] = fbqo_half_to_double(h[i]);
}

void fbqo_double_to_half_array(const double *d, uint16_t *out, long n)
{
    for (long i = 0; i < n; ++i) out[i] = fbqo_double_to_half(d[i]);
}

/* ---------------------------------------------------------------- sub-branch */

/* One row of Sigma = B.A (Sec. 4.2):  sigma_row[k] = sum_j A[k,j] * B[j,n]. */
static void sigma_row(int K, int N, int r, const uint16_t *A, const uint16_t *B, int n, double *out)
{
    for (int k = 0; k < K; ++k) {
        double acc = 0.0;
        for (int j = 0; j < r; ++j)
            acc += fbqo_half_to_double(A[(size_t)k * r + j]) * fbqo_half_to_double(B[(size_t)j * N + n]);
        out[k] = acc;
    }
}

/* Sigma [N,K] in full. */
int fbqo_sigma(int N, int K, int r, const uint16_t *A, const uint16_t *B, double *Sigma)
{
    if (N < 1 || K < 1 || r < 0 || !Sigma) return FBQO_BAD_ARG;
    if (r > 0 && (!A || !B)) return FBQO_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        sigma_row(K, N, r, A, B, n, Sigma + (size_t)n * K);
    return FBQO_OK;
}

/* ---------------------------------------------------------------- quantizer */

static int shape_ok(int N, int K, int bits, int group)
{
    if (N < 1 || K < 1 || group < 1) return 0;
    if (bits != 3 && bits != 4) return 0;
    if (K % group) return 0;
    return 1;
}

/* Packed rows hold whole words (b=4: 8 codes) or whole 3-word units (b=3: 32 codes). */
static int packable(int N, int K, int bits)
{
    if (!shape_ok(N, K, bits, K)) return 0;
    return K % (bits == 4 ? 8 : 32) == 0;
}

/* Scale and zero of one group from its min and max (see the header for the reading). */
static void group_params(double mn, double mx, int qmax, uint16_t *s16_out, uint16_t *z16_out)
{
    double s = (mx - mn) / (double)qmax;
    if (!(s > 0.0)) s = 1.0;
    uint16_t s16 = fbqo_double_to_half(s);
    if (s16 < 0x0400u) s16 = 0x0400u;              /* smallest positive normal fp16 */
    uint16_t z16;
    for (;;) {
        double sd = fbqo_half_to_double(s16);
        z16 = fbqo_double_to_half(-mn / sd);
        double zd = fbqo_half_to_double(z16);
        double ulo = mn / sd + zd, uhi = mx / sd + zd;
        if (ulo >= -0.5 && uhi <= (double)qmax + 0.5) break;
        if (s16 >= 0x7bffu) break;                 /* largest finite fp16: nothing left to widen */
        s16 += 1;                                  /* next representable fp16 above */
    }
    *s16_out = s16;
    *z16_out = z16;
}

/*
 * Feedback quantizer Q(W - Sigma) (Sec. 4.1; Alg. 1 forward).  With r == 0 this is the plain
 * group-wise round-to-nearest quantizer Q(W).  codes [N,K] in 0..qmax, scales/zeros [N,G] fp16.
 */
int fbqo_quantize(int N, int K, int r, int bits, int group, const uint16_t *W, const uint16_t *A,
                  const uint16_t *B, uint8_t *codes, uint16_t *scales, uint16_t *zeros)
{
    if (!shape_ok(N, K, bits, group) || r < 0 || !W || !codes || !scales || !zeros) return FBQO_BAD_ARG;
    if (r > 0 && (!A || !B)) return FBQO_BAD_ARG;
    const int qmax = (1 << bits) - 1;
    const int G = K / group;
    int failed = 0;
#pragma omp parallel
    {
        double *R = (double *)malloc(sizeof(double) * (size_t)K);
        if (!R) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (int n = 0; n < N; ++n) {
            if (!R) continue;
            sigma_row(K, N, r, A, B, n, R);                       /* R <- Sigma row */
            for (int k = 0; k < K; ++k)                            /* R <- W - Sigma */
                R[k] = fbqo_half_to_double(W[(size_t)n * K + k]) - R[k];
            for (int gi = 0; gi < G; ++gi) {
                const double *Rg = R + (size_t)gi * group;
                double mn = Rg[0], mx = Rg[0];
                for (int i = 1; i < group; ++i) {
                    if (Rg[i] < mn) mn = Rg[i];
                    if (Rg[i] > mx) mx = Rg[i];
                }
                uint16_t s16, z16;
                group_params(mn, mx, qmax, &s16, &z16);
                scales[(size_t)n * G + gi] = s16;
                zeros[(size_t)n * G + gi] = z16;
                double sd = fbqo_half_to_double(s16), zd = fbqo_half_to_double(z16);
                for (int i = 0; i < group; ++i) {
                    double u = Rg[i] / sd + zd;
                    double q = nearbyint(u);                       /* round to nearest, ties to even */
                    if (q < 0.0) q = 0.0;
                    if (q > (double)qmax) q = (double)qmax;
                    codes[(size_t)n * K + (size_t)gi * group + i] = (uint8_t)q;
                }
            }
        }
        free(R);
    }
    return failed ? FBQO_NO_MEM : FBQO_OK;
}

/* ---------------------------------------------------------------- packing */

static size_t row_words(int K, int bits) { return (size_t)K * bits / 32; }

/* Position of bit c (0 = LSB) of code k inside a packed row: word index and bit index. */
static void code_bit_position(int bits, int k, int c, size_t *word, int *bit)
{
    if (bits == 4) {
        *word = (size_t)(k / 8);
        *bit = 4 * (k % 8) + c;
        return;
    }
    int u = k / 32, j = k % 32;
    if (j < 30) {
        int i = j % 10;
        *word = (size_t)(3 * u + j / 10);
        *bit = (i < 5 ? 3 * i : 16 + 3 * (i - 5)) + c;
    } else {
        *word = (size_t)(3 * u + c);
        *bit = (j == 30) ? 15 : 31;
    }
}

static unsigned row_code(const uint32_t *row, int bits, int k)
{
    unsigned q = 0;
    for (int c = 0; c < bits; ++c) {
        size_t w; int bit;
        code_bit_position(bits, k, c, &w, &bit);
        q |= ((row[w] >> bit) & 1u) << c;
    }
    return q;
}

int fbqo_pack(int N, int K, int bits, const uint8_t *codes, uint32_t *words)
{
    if (!packable(N, K, bits) || !codes || !words) return FBQO_BAD_ARG;
    const size_t rw = row_words(K, bits);
    const unsigned qmax = (1u << bits) - 1u;
    memset(words, 0, sizeof(uint32_t) * rw * (size_t)N);
    for (int n = 0; n < N; ++n) {
        uint32_t *row = words + rw * (size_t)n;
        for (int k = 0; k < K; ++k) {
            unsigned q = codes[(size_t)n * K + k];
            if (q > qmax) return FBQO_BAD_ARG;
            for (int c = 0; c < bits; ++c) {
                size_t w; int bit;
                code_bit_position(bits, k, c, &w, &bit);
                row[w] |= ((q >> c) & 1u) << bit;
            }
        }
    }
    return FBQO_OK;
}

int fbqo_unpack(int N, int K, int bits, const uint32_t *words, uint8_t *codes)
{
    if (!packable(N, K, bits) || !codes || !words) return FBQO_BAD_ARG;
    const size_t rw = row_words(K, bits);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            codes[(size_t)n * K + k] = (uint8_t)row_code(words + rw * (size_t)n, bits, k);
    return FBQO_OK;
}

/* ---------------------------------------------------------------- dequantize / reconstruct */

/* One row of the main-path weight:  wq[k] = s16 * (q - z16)  (fp64, from the packed words). */
static void dequant_row(int K, int bits, int group, const uint32_t *row, const uint16_t *srow,
                        const uint16_t *zrow, double *wq)
{
    for (int k = 0; k < K; ++k) {
        double s = fbqo_half_to_double(srow[k / group]);
        double z = fbqo_half_to_double(zrow[k / group]);
        wq[k] = s * ((double)row_code(row, bits, k) - z);
    }
}

int fbqo_dequant(int N, int K, int bits, int group, const uint32_t *words, const uint16_t *scales,
                 const uint16_t *zeros, double *Wq)
{
    if (!shape_ok(N, K, bits, group) || !packable(N, K, bits) || !words || !scales || !zeros || !Wq)
        return FBQO_BAD_ARG;
    const size_t rw = row_words(K, bits);
    const int G = K / group;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        dequant_row(K, bits, group, words + rw * (size_t)n, scales + (size_t)n * G, zeros + (size_t)n * G,
                    Wq + (size_t)n * K);
    return FBQO_OK;
}

/* W_F = Q(W - Sigma) + Sigma (Sec. 4.1), [N,K] fp64. */
int fbqo_reconstruct(int N, int K, int r, int bits, int group, const uint32_t *words, const uint16_t *scales,
                     const uint16_t *zeros, const uint16_t *A, const uint16_t *B, double *WF)
{
    if (!shape_ok(N, K, bits, group) || !packable(N, K, bits) || r < 0 || !words || !scales || !zeros || !WF)
        return FBQO_BAD_ARG;
    if (r > 0 && (!A || !B)) return FBQO_BAD_ARG;
    const size_t rw = row_words(K, bits);
    const int G = K / group;
    int failed = 0;
#pragma omp parallel
    {
        double *sig = (double *)malloc(sizeof(double) * (size_t)K);
        if (!sig) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (int n = 0; n < N; ++n) {
            if (!sig) continue;
            double *out = WF + (size_t)n * K;
            dequant_row(K, bits, group, words + rw * (size_t)n, scales + (size_t)n * G, zeros + (size_t)n * G, out);
            sigma_row(K, N, r, A, B, n, sig);
            for (int k = 0; k < K; ++k) out[k] += sig[k];
        }
        free(sig);
    }
    return failed ? FBQO_NO_MEM : FBQO_OK;
}

/* ---------------------------------------------------------------- the layer */

/*
 * y = x.Wq^T + (x.A).B   (Alg. 1 "quantization output", transposed to row-major tokens):
 *   t[m,j] = sum_k x[m,k] * A[k,j]
 *   y[m,n] = sum_k x[m,k] * s16[n,k/g] * (q[n,k] - z16[n,k/g]) + sum_j t[m,j] * B[j,n]
 * Everything in fp64; the weight row is dequantized on the fly and never stored.
 */
int fbqo_linear(int M, int N, int K, int r, int bits, int group, const uint16_t *x, const uint32_t *words,
                const uint16_t *scales, const uint16_t *zeros, const uint16_t *A, const uint16_t *B, double *y)
{
    if (!shape_ok(N, K, bits, group) || !packable(N, K, bits) || M < 1 || r < 0 || !x || !words || !scales ||
        !zeros || !y)
        return FBQO_BAD_ARG;
    if (r > 0 && (!A || !B)) return FBQO_BAD_ARG;
    const size_t rw = row_words(K, bits);
    const int G = K / group;

    double *xd = (double *)malloc(sizeof(double) * (size_t)M * K);
    double *t = (double *)malloc(sizeof(double) * (size_t)M * (r > 0 ? r : 1));
    if (!xd || !t) { free(xd); free(t); return FBQO_NO_MEM; }
    fbqo_half_to_double_array(x, xd, (long)M * K);

    /* down-projection t = x.A */
    for (int m = 0; m < M; ++m)
        for (int j = 0; j < r; ++j) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += xd[(size_t)m * K + k] * fbqo_half_to_double(A[(size_t)k * r + j]);
            t[(size_t)m * r + j] = acc;
        }

    int failed = 0;
#pragma omp parallel
    {
        double *wq = (double *)malloc(sizeof(double) * (size_t)K);
        if (!wq) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (int n = 0; n < N; ++n) {
            if (!wq) continue;
            dequant_row(K, bits, group, words + rw * (size_t)n, scales + (size_t)n * G, zeros + (size_t)n * G, wq);
            for (int m = 0; m < M; ++m) {
                double acc = 0.0;
                for (int k = 0; k < K; ++k) acc += xd[(size_t)m * K + k] * wq[k];      /* main path */
                double up = 0.0;
                for (int j = 0; j < r; ++j)                                            /* up-projection */
                    up += t[(size_t)m * r + j] * fbqo_half_to_double(B[(size_t)j * N + n]);
                y[(size_t)m * N + n] = acc + up;
            }
        }
        free(wq);
    }
    free(xd);
    free(t);
    return failed ? FBQO_NO_MEM : FBQO_OK;
}

/* y = x.W^T for a materialised fp64 weight [N,K] (second, independent route to y via W_F). */
int fbqo_dense_linear(int M, int N, int K, const uint16_t *x, const double *Wd, double *y)
{
    if (M < 1 || N < 1 || K < 1 || !x || !Wd || !y) return FBQO_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += fbqo_half_to_double(x[(size_t)m * K + k]) * Wd[(size_t)n * K + k];
            y[(size_t)m * N + n] = acc;
        }
    return FBQO_OK;
}

/* ---------------------------------------------------------------- layer-wise reconstruction */

/*
 * One iteration of the loop body of Alg. 1 (Sec. 4.2) for one layer, on T calibration tokens X [T,K].
 * The steps are taken in the algorithm's order, and the gradient is obtained by differentiating
 * the forward pass as written there (not from the closed form -2.Delta_F.X^T.X, which the tests
 * use as a pin):
 *   Z  = W X^T                                   the fp16 layer's output                [N,T]
 *   Z' = Q(W - Sigma) X^T + B A X^T              quantized main path plus sub-branch    [N,T]
 *   L  = sum of squares of Z - Z'
 *   backward with W and Q(W - Sigma) held constant ("detached"): only the term B A X^T depends
 *   on A and B.  In this file's orientation (A [K,r], B [r,N], Z'^T = X Wq^T + (X A) B), with
 *   E = dL/dZ' = -2 (Z - Z') and S = X A:   dL/dB = S^T E^T,   dL/dA = X^T (E^T B^T).
 *   A <- A - lr dL/dA,  B <- B - lr dL/dB        plain gradient descent
 * Readings where the paper is silent:
 *   - the loss is the SQUARED Frobenius norm: the trace form the paper equates it with, and the
 *     gradient it prints, are those of the square;
 *   - "gradient descent" is the plain update above (no momentum, no adaptive scaling);
 *   - A and B are kept as real-valued masters (fp64 here); the forward pass uses their fp16
 *     roundings A16, B16 - the values a deployed layer would hold, so that the codes, scales and
 *     zeros written here together with A16, B16 are a consistent layer for the inference path -
 *     and the gradient with respect to a master is taken to be that with respect to its rounding.
 * Outputs describe the parameters BEFORE the update: codes/scales/zeros = Q(W - Sigma16), A16, B16,
 * loss, gradA [K,r], gradB [r,N].  A and B are updated in place.
 */
int fbqo_train_step(int N, int K, int r, int bits, int group, int T, const uint16_t *W, const uint16_t *X,
                    double *A, double *B, double lr, uint8_t *codes, uint16_t *scales, uint16_t *zeros,
                    uint16_t *A16, uint16_t *B16, double *gradA, double *gradB, double *loss)
{
    if (!shape_ok(N, K, bits, group) || r < 1 || T < 1) return FBQO_BAD_ARG;
    if (!W || !X || !A || !B || !codes || !scales || !zeros || !A16 || !B16 || !gradA || !gradB || !loss)
        return FBQO_BAD_ARG;
    const int G = K / group;
    fbqo_double_to_half_array(A, A16, (long)K * r);
    fbqo_double_to_half_array(B, B16, (long)r * N);
    int rc = fbqo_quantize(N, K, r, bits, group, W, A16, B16, codes, scales, zeros);
    if (rc != FBQO_OK) return rc;

    double *Xd = (double *)malloc((size_t)T * K * sizeof(double));
    double *S = (double *)malloc((size_t)T * r * sizeof(double));       /* S = X A16 */
    double *E = (double *)malloc((size_t)N * T * sizeof(double));       /* E = dL/dZ' */
    double *dS = (double *)malloc((size_t)T * r * sizeof(double));      /* dL/dS = E^T B16^T */
    double *row_loss = (double *)malloc((size_t)N * sizeof(double));
    if (!Xd || !S || !E || !dS || !row_loss) { free(Xd); free(S); free(E); free(dS); free(row_loss); return FBQO_NO_MEM; }
    fbqo_half_to_double_array(X, Xd, (long)T * K);
    for (int t = 0; t < T; ++t)
        for (int j = 0; j < r; ++j) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k) acc += Xd[(size_t)t * K + k] * fbqo_half_to_double(A16[(size_t)k * r + j]);
            S[(size_t)t * r + j] = acc;
        }

#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        double l = 0.0;
        for (int t = 0; t < T; ++t) {
            double z = 0.0, zq = 0.0, zs = 0.0;
            for (int k = 0; k < K; ++k) {
                const double s = fbqo_half_to_double(scales[(size_t)n * G + k / group]);
                const double zp = fbqo_half_to_double(zeros[(size_t)n * G + k / group]);
                const double wq = s * ((double)codes[(size_t)n * K + k] - zp);
                z += fbqo_half_to_double(W[(size_t)n * K + k]) * Xd[(size_t)t * K + k];   /* Z  = W X^T */
                zq += wq * Xd[(size_t)t * K + k];                                         /* Q(W - Sigma) X^T */
            }
            for (int j = 0; j < r; ++j) zs += fbqo_half_to_double(B16[(size_t)j * N + n]) * S[(size_t)t * r + j];
            const double e = z - (zq + zs);
            l += e * e;
            E[(size_t)n * T + t] = -2.0 * e;
        }
        row_loss[n] = l;
        for (int j = 0; j < r; ++j) {                                   /* dL/dB = S^T E^T */
            double acc = 0.0;
            for (int t = 0; t < T; ++t) acc += S[(size_t)t * r + j] * E[(size_t)n * T + t];
            gradB[(size_t)j * N + n] = acc;
        }
    }
    double total = 0.0;
    for (int n = 0; n < N; ++n) total += row_loss[n];
    *loss = total;

    for (int t = 0; t < T; ++t)
        for (int j = 0; j < r; ++j) {
            double acc = 0.0;
            for (int n = 0; n < N; ++n) acc += E[(size_t)n * T + t] * fbqo_half_to_double(B16[(size_t)j * N + n]);
            dS[(size_t)t * r + j] = acc;
        }
#pragma omp parallel for schedule(static)
    for (int k = 0; k < K; ++k)
        for (int j = 0; j < r; ++j) {                                   /* dL/dA = X^T dS */
            double acc = 0.0;
            for (int t = 0; t < T; ++t) acc += Xd[(size_t)t * K + k] * dS[(size_t)t * r + j];
            gradA[(size_t)k * r + j] = acc;
        }

    for (long i = 0; i < (long)K * r; ++i) A[i] -= lr * gradA[i];
    for (long i = 0; i < (long)r * N; ++i) B[i] -= lr * gradB[i];
    free(Xd); free(S); free(E); free(dS); free(row_loss);
    return FBQO_OK;
}

int fbqo_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
