/*
 * CPU oracle for the W6A16 linear layer of FP6-LLM (arXiv 2401.14112).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the slow, plain definition that the HIP
 * kernels are checked against.  Nothing in the product path may call it, and it
 * shares no code, header, table or constant with the HIP sources.
 *
 * What is defined here, and where the paper defines it:
 *   - the e3m2 value of a 6-bit code: Section 2.2, Eq. 1, with bias 3; the E=0
 *     binade is read as IEEE-style subnormals because that is what the bit-copy
 *     cast of Section 5.3, Eq. 3 (fp16 with E16 := Ex, times 2^(15-3)) yields;
 *     E=7 is an ordinary binade (largest magnitude 28, no inf/NaN).
 *   - the per-output-channel fp16 scale: Algorithm 1 (the "Scales" input) and
 *     Section 3 (coarse-grained quantization); the quantizer itself is not in the
 *     paper: round-to-nearest-even onto the e3m2 grid of W/scale with
 *     scale = fp16(rowmax|W| / 28).
 *   - the packed stream: Section 5.2 asks for an ahead-of-time re-layout so that
 *     the kernel reads aligned words; the layout stated in fp6o_pos() is this
 *     library's own (one 16-row x 256-k tile per 64-lane wave).
 *   - the linear layer: Section 6, C = A x B with A = [M,K] weights, B = [K,N]
 *     activations stored column-major (so X is [N][K]) and C column-major
 *     (Y is [N][M]).
 *
 * Everything is written as plain loops in double precision.  OpenMP only splits
 * independent output rows across host cores; it does not reorder any sum.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define FP6O_TILE_ROWS 16
#define FP6O_TILE_K 256
#define FP6O_TILE_BYTES 3072 /* 16 * 256 * 6 / 8 */

/* ------------------------------------------------------------------ fp16 -- */

/* IEEE binary16 bit pattern -> exact double. */
double fp6o_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 31;
    int f = h & 1023;
    double mag;
    if (e == 0)
        mag = ldexp((double)f, -24); /* subnormal: 0.f * 2^-14 */
    else if (e == 31)
        mag = (f == 0) ? INFINITY : NAN;
    else
        mag = ldexp((double)(1024 + f), e - 25); /* 1.f * 2^(e-15) */
    return sign ? -mag : mag;
}

/* double -> nearest binary16, ties to even, subnormals kept, sign of zero kept. */
uint16_t fp6o_double_to_half(double x)
{
    uint16_t sign = signbit(x) ? 0x8000u : 0u;
    double a = fabs(x);
    if (isnan(a))
        return (uint16_t)(sign | 0x7e00u);
    if (a >= 65520.0) /* midpoint between 65504 and 2^16 rounds to even = inf */
        return (uint16_t)(sign | 0x7c00u);
    if (a < ldexp(1.0, -14)) {
        /* grid spacing 2^-24; nearbyint() rounds to even in the default mode */
        double r = nearbyint(ldexp(a, 24));
        return (uint16_t)(sign | (uint16_t)r); /* r == 1024 is the first normal */
    }
    int ex;
    (void)frexp(a, &ex); /* a = m * 2^ex, m in [0.5, 1) */
    int e = ex - 1;      /* a in [2^e, 2^(e+1)) */
    double r = nearbyint(ldexp(a, 10 - e)); /* in [1024, 2048] */
    if (r == 2048.0) {
        r = 1024.0;
        e += 1;
    }
    return (uint16_t)(sign | (uint16_t)((e + 15) << 10) | (uint16_t)(r - 1024.0));
}

/* ---------------------------------------------------------------- decode -- */

/* Value of code c = s e2 e1 e0 m1 m0 (Eq. 1, bias = 2^(3-1)-1 = 3). */
double fp6o_decode(int code)
{
    int S = (code >> 5) & 1;
    int E = (code >> 2) & 7;
    int M = code & 3;
    double mag;
    if (E == 0)
        mag = ldexp(M / 4.0, 1 - 3); /* 0.M * 2^(1-bias) */
    else
        mag = ldexp(1.0 + M / 4.0, E - 3); /* 1.M * 2^(E-bias) */
    return S ? -mag : mag;
}

/* -------------------------------------------------------------- quantize -- */

/* fp16 nearest to amax/28 (ties to even), decided with exact arithmetic:
 * among the fp16 values around the quotient, the one minimising |28*h - amax|. */
uint16_t fp6o_scale_for_amax(uint16_t amax_bits)
{
    double a = fp6o_half_to_double((uint16_t)(amax_bits & 0x7fffu));
    uint16_t guess = fp6o_double_to_half(a / 28.0);
    int lo = guess > 0 ? guess - 1 : 0;
    int hi = guess + 1;
    int best = -1;
    double best_err = 0.0;
    for (int h = lo; h <= hi; ++h) {
        double err = fabs(28.0 * fp6o_half_to_double((uint16_t)h) - a); /* exact */
        if (best < 0 || err < best_err || (err == best_err && (h & 1) == 0 && (best & 1) == 1)) {
            best = h;
            best_err = err;
        }
    }
    return (uint16_t)best;
}

/* Code of one weight given the (already rounded) fp16 scale of its row:
 * sign bit copied, magnitude = grid point nearest to |w|/scale, ties to the even
 * code, anything beyond the grid saturates at 28.  |w| - decode(g)*scale is exact
 * in double (both are multiples of 2^-28 below 2^21), so the argmin is exact. */
int fp6o_quantize_one(uint16_t w_bits, uint16_t scale_bits)
{
    int sign = (w_bits >> 15) & 1;
    double a = fp6o_half_to_double((uint16_t)(w_bits & 0x7fffu));
    double s = fp6o_half_to_double((uint16_t)(scale_bits & 0x7fffu));
    if (s == 0.0)
        return sign << 5;
    int best = 0;
    double best_err = fabs(a - fp6o_decode(0) * s);
    for (int g = 1; g < 32; ++g) {
        double err = fabs(a - fp6o_decode(g) * s);
        if (err < best_err || (err == best_err && (g & 1) == 0)) {
            best = g;
            best_err = err;
        }
    }
    return (sign << 5) | best;
}

/* W fp16 [M][K] row-major -> codes [M][K] (one byte each) and scales fp16 [M].
 * Returns 0, or 1 if W holds an inf/NaN (outside the method's domain). */
int fp6o_quantize(const uint16_t *W, int64_t M, int64_t K, uint8_t *codes, uint16_t *scales)
{
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        uint16_t amax = 0;
        for (int64_t k = 0; k < K; ++k) {
            uint16_t mag = (uint16_t)(W[m * K + k] & 0x7fffu);
            if (mag >= 0x7c00u)
                bad |= 1;
            if (mag > amax) /* for finite non-negative fp16, bit order = value order */
                amax = mag;
        }
        uint16_t sc = fp6o_scale_for_amax(amax);
        scales[m] = sc;
        for (int64_t k = 0; k < K; ++k)
            codes[m * K + k] = (uint8_t)fp6o_quantize_one(W[m * K + k], sc);
    }
    return bad;
}

/* ---------------------------------------------------------------- layout -- */

int64_t fp6o_packed_bytes(int64_t M, int64_t K) { return M * K * 6 / 8; }

/*
 * Bit address, in the packed stream, of bit b of the code of weight (m, k);
 * b = 0..5 = m0, m1, e0, e1, e2, s.
 *
 * The matrix is cut into tiles of 16 rows x 256 columns, stored k-tile major
 * (the tiles of columns 0..255 for rows 0..15, 16..31, ..., then those of columns
 * 256..511, ...), 3072 bytes each: waves that work on neighbouring rows at the same
 * depth of the reduction read neighbouring memory.  A tile is three planes of 1024 bytes; a plane is 64 slots of 16 bytes, slot
 * = 16*q + r for row r of the tile and the q-th group of 8 columns inside each
 * run of 32 columns.  The slot (r, q) therefore owns 12 little-endian 32-bit
 * words, word d of them sitting in plane d/4 at byte 4*(d%4) of the slot.  Words
 * 0..5 are one dense 192-bit stream holding the 32 codes of runs 0..3, words
 * 6..11 another holding runs 4..7: inside a stream the code of (run, column j
 * of the group) has index i = 8*(run%4) + j and occupies bits 6i .. 6i+5, least
 * significant code bit first, bit n of the stream being bit n%32 of word n/32.
 */
uint64_t fp6o_pos(int64_t M, int64_t K, int64_t m, int64_t k, int b)
{
    int64_t row_tile = m / FP6O_TILE_ROWS;
    int r = (int)(m % FP6O_TILE_ROWS);
    int64_t k_tile = k / FP6O_TILE_K;
    int kk = (int)(k % FP6O_TILE_K);
    int run = kk / 32;      /* which run of 32 columns inside the tile */
    int q = (kk % 32) / 8;  /* which group of 8 inside the run */
    int j = kk % 8;         /* column inside the group */
    int slot = 16 * q + r;
    int stream = run / 4;               /* 0: runs 0..3, 1: runs 4..7 */
    int n = 6 * (8 * (run % 4) + j) + b; /* bit index inside the 192-bit stream */
    int d = 6 * stream + n / 32;        /* word of the slot, 0..11 */
    int plane = d / 4;
    uint64_t tile = (uint64_t)(k_tile * (M / FP6O_TILE_ROWS) + row_tile);
    uint64_t byte_addr = tile * FP6O_TILE_BYTES + (uint64_t)plane * 1024u + (uint64_t)slot * 16u
                         + (uint64_t)(d % 4) * 4u;
    return byte_addr * 8u + (uint64_t)(n % 32);
}

/* codes [M][K] -> packed stream (every bit of the stream is written). */
void fp6o_pack(const uint8_t *codes, int64_t M, int64_t K, uint8_t *packed)
{
    memset(packed, 0, (size_t)fp6o_packed_bytes(M, K));
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k)
            for (int b = 0; b < 6; ++b)
                if ((codes[m * K + k] >> b) & 1) {
                    uint64_t p = fp6o_pos(M, K, m, k, b);
                    packed[p >> 3] |= (uint8_t)(1u << (p & 7));
                }
}

/* packed stream -> codes [M][K]. */
void fp6o_unpack_codes(const uint8_t *packed, int64_t M, int64_t K, uint8_t *codes)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            int c = 0;
            for (int b = 0; b < 6; ++b) {
                uint64_t p = fp6o_pos(M, K, m, k, b);
                c |= ((packed[p >> 3] >> (p & 7)) & 1) << b;
            }
            codes[m * K + k] = (uint8_t)c;
        }
}

/* ------------------------------------------------------- the three calls -- */

/* fp16 W [M][K] -> packed codes + fp16 scales. */
int fp6o_quantize_pack(const uint16_t *W, int64_t M, int64_t K, uint8_t *packed, uint16_t *scales)
{
    uint8_t *codes = (uint8_t *)malloc((size_t)(M * K));
    if (!codes)
        return 2;
    int bad = fp6o_quantize(W, M, K, codes, scales);
    fp6o_pack(codes, M, K, packed);
    free(codes);
    return bad;
}

/* packed + scales -> fp16 [M][K]: nearest fp16 to decode(code)*scale.  The product
 * has at most 3+11 significant bits, so it is exact in double and rounded once. */
int fp6o_unpack(const uint8_t *packed, const uint16_t *scales, int64_t M, int64_t K, uint16_t *W)
{
    uint8_t *codes = (uint8_t *)malloc((size_t)(M * K));
    if (!codes)
        return 2;
    fp6o_unpack_codes(packed, M, K, codes);
    for (int64_t m = 0; m < M; ++m) {
        double s = fp6o_half_to_double(scales[m]);
        for (int64_t k = 0; k < K; ++k)
            W[m * K + k] = fp6o_double_to_half(fp6o_decode(codes[m * K + k]) * s);
    }
    free(codes);
    return 0;
}

/* Y[n][rows[i]] = scale * sum_k decode(code[row][k]) * X[n][k], k ascending, in
 * double, for the listed rows (rows == NULL: all M rows, i = m).  codes is [M][K],
 * X is fp16 [N][K], Y is double [N][nrows]. */
void fp6o_linear_codes(const uint8_t *codes, const uint16_t *scales, const uint16_t *X, int64_t M,
                       int64_t N, int64_t K, const int64_t *rows, int64_t nrows, double *Y)
{
    if (!rows)
        nrows = M;
    double *Xd = (double *)malloc((size_t)(N * K) * sizeof(double));
    for (int64_t i = 0; i < N * K; ++i)
        Xd[i] = fp6o_half_to_double(X[i]);
    double table[64];
    for (int c = 0; c < 64; ++c)
        table[c] = fp6o_decode(c);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        int64_t m = rows ? rows[i] : i;
        double s = fp6o_half_to_double(scales[m]);
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += table[codes[m * K + k]] * Xd[n * K + k];
            Y[n * nrows + i] = s * acc;
        }
    }
    free(Xd);
}

/* Same, starting from the packed stream (reads it through fp6o_pos). */
int fp6o_linear(const uint8_t *packed, const uint16_t *scales, const uint16_t *X, int64_t M,
                int64_t N, int64_t K, const int64_t *rows, int64_t nrows, double *Y)
{
    if (!rows)
        nrows = M;
    /* gather only the rows that are asked for */
    uint8_t *codes = (uint8_t *)malloc((size_t)(nrows * K));
    uint16_t *sc = (uint16_t *)malloc((size_t)nrows * sizeof(uint16_t));
    if (!codes || !sc) {
        free(codes);
        free(sc);
        return 2;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        int64_t m = rows ? rows[i] : i;
        sc[i] = scales[m];
        for (int64_t k = 0; k < K; ++k) {
            int c = 0;
            for (int b = 0; b < 6; ++b) {
                uint64_t p = fp6o_pos(M, K, m, k, b);
                c |= ((packed[p >> 3] >> (p & 7)) & 1) << b;
            }
            codes[i * K + k] = (uint8_t)c;
        }
    }
    fp6o_linear_codes(codes, sc, X, nrows, N, K, NULL, nrows, Y);
    free(codes);
    free(sc);
    return 0;
}

/* The linear layer followed by the element-wise steps that a decoder block
 * attaches to it (Section 7.3 runs whole LLaMA / OPT decoders: their projections
 * carry an optional bias, the feed-forward block multiplies silu(gate) by up, and
 * the last projection of each half of a block is added to the residual stream).
 * All in double, no intermediate rounding, in this order:
 *     z[n][m] = scale[m] * sum_k decode(code[m][k]) * X[n][k]      (fp6o_linear)
 *     z[n][m] += bias[m]                                            if bias
 *     gated:  y[n][i] = z[n][2i] / (1 + exp(-z[n][2i])) * z[n][2i+1]   (M/2 outputs)
 *     else:   y[n][m] = z[n][m]
 *     y[n][o] += residual[n][o]                                     if residual
 * bias is fp16 [M]; residual is fp16 [N][Mout], Mout = M/2 when gated, else M.
 * rows (NULL: all) lists OUTPUT rows o; Y is double [N][nrows]. */
int fpxo_linear_fused(int bits, int64_t group, const uint8_t *packed, const uint16_t *scales, const uint16_t *X,
                      int64_t M, int64_t N, int64_t K, const uint16_t *bias, const uint16_t *residual, int gated,
                      const int64_t *rows, int64_t nrows, double *Y);

int fp6o_linear_fused(const uint8_t *packed, const uint16_t *scales, const uint16_t *X, int64_t M,
                      int64_t N, int64_t K, const uint16_t *bias, const uint16_t *residual, int gated,
                      const int64_t *rows, int64_t nrows, double *Y)
{
    return fpxo_linear_fused(6, 0, packed, scales, X, M, N, K, bias, residual, gated, rows, nrows, Y);
}

/* Plain fp16-weight linear layer in double, for the W16A16 comparison kernel:
 * Y[n][m] = sum_k W[m][k] * X[n][k]. */
void fp6o_linear_f16(const uint16_t *W, const uint16_t *X, int64_t M, int64_t N, int64_t K,
                     const int64_t *rows, int64_t nrows, double *Y)
{
    if (!rows)
        nrows = M;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        int64_t m = rows ? rows[i] : i;
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += fp6o_half_to_double(W[m * K + k]) * fp6o_half_to_double(X[n * K + k]);
            Y[n * nrows + i] = acc;
        }
    }
}

/* ====================================================================== *
 * Group-wise scales (fine-grained quantization; Section 3 of the paper
 * contrasts it with the coarse-grained, one-scale-per-channel scheme that FP6
 * is used with, and Algorithm 1 multiplies the scales into the weights before
 * the matrix multiplication, which is what a scale per group of columns needs).
 * One fp16 scale per row and per group of `group` consecutive columns:
 * scales is [M][K/group]; inside its group every weight is quantized exactly as
 * in the per-row scheme (fp6o_scale_for_amax, fp6o_quantize_one).  The packed
 * stream is the 6-bit one (fp6o_pos).
 * ====================================================================== */

int fp6go_quantize(const uint16_t *W, int64_t M, int64_t K, int64_t group, uint8_t *codes, uint16_t *scales)
{
    int bad = 0;
    int64_t G = K / group;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t g = 0; g < G; ++g) {
            uint16_t amax = 0;
            for (int64_t k = g * group; k < (g + 1) * group; ++k) {
                uint16_t mag = (uint16_t)(W[m * K + k] & 0x7fffu);
                if (mag >= 0x7c00u)
                    bad |= 1;
                if (mag > amax)
                    amax = mag;
            }
            uint16_t sc = fp6o_scale_for_amax(amax);
            scales[m * G + g] = sc;
            for (int64_t k = g * group; k < (g + 1) * group; ++k)
                codes[m * K + k] = (uint8_t)fp6o_quantize_one(W[m * K + k], sc);
        }
    return bad;
}

int fp6go_quantize_pack(const uint16_t *W, int64_t M, int64_t K, int64_t group, uint8_t *packed, uint16_t *scales)
{
    uint8_t *codes = (uint8_t *)malloc((size_t)(M * K));
    if (!codes)
        return 2;
    int bad = fp6go_quantize(W, M, K, group, codes, scales);
    fp6o_pack(codes, M, K, packed);
    free(codes);
    return bad;
}

/* nearest fp16 to decode(code) * scale[m][k/group] (exact product, one rounding) */
int fp6go_unpack(const uint8_t *packed, const uint16_t *scales, int64_t M, int64_t K, int64_t group, uint16_t *W)
{
    uint8_t *codes = (uint8_t *)malloc((size_t)(M * K));
    if (!codes)
        return 2;
    int64_t G = K / group;
    fp6o_unpack_codes(packed, M, K, codes);
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k)
            W[m * K + k] = fp6o_double_to_half(fp6o_decode(codes[m * K + k]) * fp6o_half_to_double(scales[m * G + k / group]));
    free(codes);
    return 0;
}

/* Y[n][i] = sum_k scale[row][k/group] * decode(code[row][k]) * X[n][k], k ascending, in double. */
int fp6go_linear(const uint8_t *packed, const uint16_t *scales, const uint16_t *X, int64_t M, int64_t N,
                 int64_t K, int64_t group, const int64_t *rows, int64_t nrows, double *Y)
{
    if (!rows)
        nrows = M;
    int64_t G = K / group;
    double *Xd = (double *)malloc((size_t)(N * K) * sizeof(double));
    if (!Xd)
        return 2;
    for (int64_t i = 0; i < N * K; ++i)
        Xd[i] = fp6o_half_to_double(X[i]);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        int64_t m = rows ? rows[i] : i;
        double *wd = (double *)malloc((size_t)K * sizeof(double));
        for (int64_t k = 0; k < K; ++k) {
            int c = 0;
            for (int b = 0; b < 6; ++b) {
                uint64_t p = fp6o_pos(M, K, m, k, b);
                c |= ((packed[p >> 3] >> (p & 7)) & 1) << b;
            }
            wd[k] = fp6o_decode(c) * fp6o_half_to_double(scales[m * G + k / group]); /* exact */
        }
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += wd[k] * Xd[n * K + k];
            Y[n * nrows + i] = acc;
        }
        free(wd);
    }
    free(Xd);
    return 0;
}

/* ====================================================================== *
 * The 5-bit variant (W5A16).  The paper presents its scheme as independent of
 * the bit-width (Section 1: "6-bit, 5-bit, 3-bit, etc."; Section 5.2: the
 * pre-packing applies to any x; Section 5.3: the cast of Eq. 3 applies to any
 * bit-width).  FP5 is read as e2m2: code = s e1 e0 m1 m0, Eq. 1 with
 * bias = 2^(2-1)-1 = 1, the E = 0 binade subnormal (0.M * 2^(1-bias)) and E = 3
 * an ordinary binade, exactly as for e3m2: values 0 .25 .5 .75 | 1 1.25 1.5 1.75
 * | 2 2.5 3 3.5 | 4 5 6 7.  Quantizer: the same recipe with 7 in place of 28.
 * Everything below mirrors the 6-bit functions above, written out again.
 * ====================================================================== */

#define FP5O_TILE_BYTES 2560 /* 16 * 256 * 5 / 8 */

double fp5o_decode(int code)
{
    int S = (code >> 4) & 1;
    int E = (code >> 2) & 3;
    int M = code & 3;
    double mag;
    if (E == 0)
        mag = ldexp(M / 4.0, 1 - 1); /* 0.M * 2^(1-bias) */
    else
        mag = ldexp(1.0 + M / 4.0, E - 1); /* 1.M * 2^(E-bias) */
    return S ? -mag : mag;
}

/* fp16 nearest to amax/7 (ties to even), decided with exact arithmetic. */
uint16_t fp5o_scale_for_amax(uint16_t amax_bits)
{
    double a = fp6o_half_to_double((uint16_t)(amax_bits & 0x7fffu));
    uint16_t guess = fp6o_double_to_half(a / 7.0);
    int lo = guess > 0 ? guess - 1 : 0;
    int hi = guess + 1;
    int best = -1;
    double best_err = 0.0;
    for (int h = lo; h <= hi; ++h) {
        double err = fabs(7.0 * fp6o_half_to_double((uint16_t)h) - a); /* exact */
        if (best < 0 || err < best_err || (err == best_err && (h & 1) == 0 && (best & 1) == 1)) {
            best = h;
            best_err = err;
        }
    }
    return (uint16_t)best;
}

/* Sign bit copied, magnitude = grid point nearest to |w|/scale, ties to the even code,
 * beyond the grid saturates at 7; the differences are exact in double. */
int fp5o_quantize_one(uint16_t w_bits, uint16_t scale_bits)
{
    int sign = (w_bits >> 15) & 1;
    double a = fp6o_half_to_double((uint16_t)(w_bits & 0x7fffu));
    double s = fp6o_half_to_double((uint16_t)(scale_bits & 0x7fffu));
    if (s == 0.0)
        return sign << 4;
    int best = 0;
    double best_err = fabs(a - fp5o_decode(0) * s);
    for (int g = 1; g < 16; ++g) {
        double err = fabs(a - fp5o_decode(g) * s);
        if (err < best_err || (err == best_err && (g & 1) == 0)) {
            best = g;
            best_err = err;
        }
    }
    return (sign << 4) | best;
}

int fp5o_quantize(const uint16_t *W, int64_t M, int64_t K, uint8_t *codes, uint16_t *scales)
{
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        uint16_t amax = 0;
        for (int64_t k = 0; k < K; ++k) {
            uint16_t mag = (uint16_t)(W[m * K + k] & 0x7fffu);
            if (mag >= 0x7c00u)
                bad |= 1;
            if (mag > amax)
                amax = mag;
        }
        uint16_t sc = fp5o_scale_for_amax(amax);
        scales[m] = sc;
        for (int64_t k = 0; k < K; ++k)
            codes[m * K + k] = (uint8_t)fp5o_quantize_one(W[m * K + k], sc);
    }
    return bad;
}

int64_t fp5o_packed_bytes(int64_t M, int64_t K) { return M * K * 5 / 8; }

/*
 * Bit address, in the packed 5-bit stream, of bit b of the code of weight (m, k);
 * b = 0..4 = m0, m1, e0, e1, s.
 *
 * Tiles of 16 rows x 256 columns, k-tile major as in the 6-bit layout, 2560 bytes each.  A tile is two
 * planes of 1024 bytes (64 slots of 16 bytes) followed by one plane of 512 bytes
 * (64 slots of 8 bytes); slot = 16*q + r as in the 6-bit layout.  The slot owns
 * ten 32-bit words: words 0..3 in plane 0, 4..7 in plane 1, 8..9 in plane 2.
 * Words 0..4 (D0..D4) serve column runs 0..3, words 5..9 runs 4..7.  The 32 codes
 * of four runs, index i = 8*(run%4) + j, are placed so that shifts and masks on
 * whole words rebuild four codes at a time (Section 5.3): code i < 20 sits in
 * place in byte i%4 of D[i/4] as  s . . . e1 e0 m1 m0  (sign at bit 7, the rest at
 * bits 3..0, i.e. the top byte of the fp16 that Eq. 3 asks for); that leaves bits
 * 6, 5, 4 of all twenty bytes free, and the remaining twelve codes (i = 20..31,
 * byte lane i%4, group g = (i-20)/4) are spread over them:
 *   g = 0:  s -> D0.6   e1 -> D0.5   e0 -> D0.4   m1 -> D1.6   m0 -> D1.5
 *   g = 1:  s -> D1.4   e1 -> D2.6   e0 -> D2.5   m1 -> D2.4   m0 -> D3.6
 *   g = 2:  s -> D3.5   e1 -> D3.4   e0 -> D4.6   m1 -> D4.5   m0 -> D4.4
 * (Dn.x = bit x of the byte of lane i%4 in word Dn).
 */
uint64_t fp5o_pos(int64_t M, int64_t K, int64_t m, int64_t k, int b)
{
    static const int spread_word[3][5] = { /* indexed [g][b], b = m0 m1 e0 e1 s */
        {1, 1, 0, 0, 0}, {3, 2, 2, 2, 1}, {4, 4, 4, 3, 3}};
    static const int spread_bit[3][5] = {
        {5, 6, 4, 5, 6}, {6, 4, 5, 6, 4}, {4, 5, 6, 4, 5}};
    int64_t row_tile = m / FP6O_TILE_ROWS;
    int r = (int)(m % FP6O_TILE_ROWS);
    int64_t k_tile = k / FP6O_TILE_K;
    int kk = (int)(k % FP6O_TILE_K);
    int run = kk / 32;
    int q = (kk % 32) / 8;
    int j = kk % 8;
    int slot = 16 * q + r;
    int half = run / 4;           /* 0: words 0..4, 1: words 5..9 */
    int i = 8 * (run % 4) + j;    /* index among the 32 codes of the four runs */
    int lane_byte = i % 4;
    int word, bit;
    if (i < 20) {
        word = i / 4;
        bit = (b == 4) ? 7 : b;
    } else {
        int g = (i - 20) / 4;
        word = spread_word[g][b];
        bit = spread_bit[g][b];
    }
    int d = 5 * half + word;      /* word of the slot, 0..9 */
    uint64_t tile = (uint64_t)(k_tile * (M / FP6O_TILE_ROWS) + row_tile);
    uint64_t in_tile = d < 8 ? (uint64_t)(d / 4) * 1024u + (uint64_t)slot * 16u + (uint64_t)(d % 4) * 4u
                             : 2048u + (uint64_t)slot * 8u + (uint64_t)(d - 8) * 4u;
    return (tile * FP5O_TILE_BYTES + in_tile + (uint64_t)lane_byte) * 8u + (uint64_t)bit;
}

void fp5o_pack(const uint8_t *codes, int64_t M, int64_t K, uint8_t *packed)
{
    memset(packed, 0, (size_t)fp5o_packed_bytes(M, K));
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k)
            for (int b = 0; b < 5; ++b)
                if ((codes[m * K + k] >> b) & 1) {
                    uint64_t p = fp5o_pos(M, K, m, k, b);
                    packed[p >> 3] |= (uint8_t)(1u << (p & 7));
                }
}

void fp5o_unpack_codes(const uint8_t *packed, int64_t M, int64_t K, uint8_t *codes)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            int c = 0;
            for (int b = 0; b < 5; ++b) {
                uint64_t p = fp5o_pos(M, K, m, k, b);
                c |= ((packed[p >> 3] >> (p & 7)) & 1) << b;
            }
            codes[m * K + k] = (uint8_t)c;
        }
}

int fp5o_quantize_pack(const uint16_t *W, int64_t M, int64_t K, uint8_t *packed, uint16_t *scales)
{
    uint8_t *codes = (uint8_t *)malloc((size_t)(M * K));
    if (!codes)
        return 2;
    int bad = fp5o_quantize(W, M, K, codes, scales);
    fp5o_pack(codes, M, K, packed);
    free(codes);
    return bad;
}

/* nearest fp16 to decode(code)*scale: the product is exact in double, rounded once. */
int fp5o_unpack(const uint8_t *packed, const uint16_t *scales, int64_t M, int64_t K, uint16_t *W)
{
    uint8_t *codes = (uint8_t *)malloc((size_t)(M * K));
    if (!codes)
        return 2;
    fp5o_unpack_codes(packed, M, K, codes);
    for (int64_t m = 0; m < M; ++m) {
        double s = fp6o_half_to_double(scales[m]);
        for (int64_t k = 0; k < K; ++k)
            W[m * K + k] = fp6o_double_to_half(fp5o_decode(codes[m * K + k]) * s);
    }
    free(codes);
    return 0;
}

/* Y[n][i] = scale * sum_k decode(code[row][k]) * X[n][k], k ascending, in double. */
void fp5o_linear_codes(const uint8_t *codes, const uint16_t *scales, const uint16_t *X, int64_t M,
                       int64_t N, int64_t K, const int64_t *rows, int64_t nrows, double *Y)
{
    if (!rows)
        nrows = M;
    double *Xd = (double *)malloc((size_t)(N * K) * sizeof(double));
    for (int64_t i = 0; i < N * K; ++i)
        Xd[i] = fp6o_half_to_double(X[i]);
    double table[32];
    for (int c = 0; c < 32; ++c)
        table[c] = fp5o_decode(c);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        int64_t m = rows ? rows[i] : i;
        double s = fp6o_half_to_double(scales[m]);
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += table[codes[m * K + k]] * Xd[n * K + k];
            Y[n * nrows + i] = s * acc;
        }
    }
    free(Xd);
}

int fp5o_linear(const uint8_t *packed, const uint16_t *scales, const uint16_t *X, int64_t M,
                int64_t N, int64_t K, const int64_t *rows, int64_t nrows, double *Y)
{
    if (!rows)
        nrows = M;
    uint8_t *codes = (uint8_t *)malloc((size_t)(nrows * K));
    uint16_t *sc = (uint16_t *)malloc((size_t)nrows * sizeof(uint16_t));
    if (!codes || !sc) {
        free(codes);
        free(sc);
        return 2;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        int64_t m = rows ? rows[i] : i;
        sc[i] = scales[m];
        for (int64_t k = 0; k < K; ++k) {
            int c = 0;
            for (int b = 0; b < 5; ++b) {
                uint64_t p = fp5o_pos(M, K, m, k, b);
                c |= ((packed[p >> 3] >> (p & 7)) & 1) << b;
            }
            codes[i * K + k] = (uint8_t)c;
        }
    }
    fp5o_linear_codes(codes, sc, X, nrows, N, K, NULL, nrows, Y);
    free(codes);
    free(sc);
    return 0;
}

/* ====================================================================== *
 * The 4-bit variant (W4A16), same reasoning as the 5-bit one: FP4 is read as
 * e2m1, code = s e1 e0 m0, Eq. 1 with bias 2^(2-1)-1 = 1, subnormal E = 0
 * binade, no inf/NaN: values 0 .5 | 1 1.5 | 2 3 | 4 6.  Quantizer: the same
 * recipe with 6 in place of 28.
 * ====================================================================== */

#define FP4O_TILE_BYTES 2048 /* 16 * 256 * 4 / 8 */

double fp4o_decode(int code)
{
    int S = (code >> 3) & 1;
    int E = (code >> 1) & 3;
    int M = code & 1;
    double mag;
    if (E == 0)
        mag = ldexp(M / 2.0, 1 - 1); /* 0.M * 2^(1-bias) */
    else
        mag = ldexp(1.0 + M / 2.0, E - 1); /* 1.M * 2^(E-bias) */
    return S ? -mag : mag;
}

/* fp16 nearest to amax/6 (ties to even), decided with exact arithmetic. */
uint16_t fp4o_scale_for_amax(uint16_t amax_bits)
{
    double a = fp6o_half_to_double((uint16_t)(amax_bits & 0x7fffu));
    uint16_t guess = fp6o_double_to_half(a / 6.0);
    int lo = guess > 0 ? guess - 1 : 0;
    int hi = guess + 1;
    int best = -1;
    double best_err = 0.0;
    for (int h = lo; h <= hi; ++h) {
        double err = fabs(6.0 * fp6o_half_to_double((uint16_t)h) - a); /* exact */
        if (best < 0 || err < best_err || (err == best_err && (h & 1) == 0 && (best & 1) == 1)) {
            best = h;
            best_err = err;
        }
    }
    return (uint16_t)best;
}

int fp4o_quantize_one(uint16_t w_bits, uint16_t scale_bits)
{
    int sign = (w_bits >> 15) & 1;
    double a = fp6o_half_to_double((uint16_t)(w_bits & 0x7fffu));
    double s = fp6o_half_to_double((uint16_t)(scale_bits & 0x7fffu));
    if (s == 0.0)
        return sign << 3;
    int best = 0;
    double best_err = fabs(a - fp4o_decode(0) * s);
    for (int g = 1; g < 8; ++g) {
        double err = fabs(a - fp4o_decode(g) * s);
        if (err < best_err || (err == best_err && (g & 1) == 0)) {
            best = g;
            best_err = err;
        }
    }
    return (sign << 3) | best;
}

int fp4o_quantize(const uint16_t *W, int64_t M, int64_t K, uint8_t *codes, uint16_t *scales)
{
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        uint16_t amax = 0;
        for (int64_t k = 0; k < K; ++k) {
            uint16_t mag = (uint16_t)(W[m * K + k] & 0x7fffu);
            if (mag >= 0x7c00u)
                bad |= 1;
            if (mag > amax)
                amax = mag;
        }
        uint16_t sc = fp4o_scale_for_amax(amax);
        scales[m] = sc;
        for (int64_t k = 0; k < K; ++k)
            codes[m * K + k] = (uint8_t)fp4o_quantize_one(W[m * K + k], sc);
    }
    return bad;
}

int64_t fp4o_packed_bytes(int64_t M, int64_t K) { return M * K / 2; }

/*
 * Bit address of bit b (0..3 = m0, e0, e1, s) of the code of weight (m, k) in the packed
 * 4-bit stream.  Tiles of 16 rows x 256 columns, k-tile major, 2048 bytes each: two
 * planes of 1024 bytes, 64 slots of 16 bytes per plane, slot = 16*q + r as in the other
 * layouts.  The slot owns eight 32-bit words, word d in plane d/4 at byte 4*(d%4); word d
 * holds the eight codes of run d (columns 32*d + 8*q + j), code j in bits 4j .. 4j+3.
 */
uint64_t fp4o_pos(int64_t M, int64_t K, int64_t m, int64_t k, int b)
{
    int64_t row_tile = m / FP6O_TILE_ROWS;
    int r = (int)(m % FP6O_TILE_ROWS);
    int64_t k_tile = k / FP6O_TILE_K;
    int kk = (int)(k % FP6O_TILE_K);
    int run = kk / 32;
    int q = (kk % 32) / 8;
    int j = kk % 8;
    int slot = 16 * q + r;
    uint64_t tile = (uint64_t)(k_tile * (M / FP6O_TILE_ROWS) + row_tile);
    uint64_t byte_addr = tile * FP4O_TILE_BYTES + (uint64_t)(run / 4) * 1024u + (uint64_t)slot * 16u
                         + (uint64_t)(run % 4) * 4u;
    return byte_addr * 8u + (uint64_t)(4 * j + b);
}

void fp4o_pack(const uint8_t *codes, int64_t M, int64_t K, uint8_t *packed)
{
    memset(packed, 0, (size_t)fp4o_packed_bytes(M, K));
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k)
            for (int b = 0; b < 4; ++b)
                if ((codes[m * K + k] >> b) & 1) {
                    uint64_t p = fp4o_pos(M, K, m, k, b);
                    packed[p >> 3] |= (uint8_t)(1u << (p & 7));
                }
}

void fp4o_unpack_codes(const uint8_t *packed, int64_t M, int64_t K, uint8_t *codes)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            int c = 0;
            for (int b = 0; b < 4; ++b) {
                uint64_t p = fp4o_pos(M, K, m, k, b);
                c |= ((packed[p >> 3] >> (p & 7)) & 1) << b;
            }
            codes[m * K + k] = (uint8_t)c;
        }
}

int fp4o_quantize_pack(const uint16_t *W, int64_t M, int64_t K, uint8_t *packed, uint16_t *scales)
{
    uint8_t *codes = (uint8_t *)malloc((size_t)(M * K));
    if (!codes)
        return 2;
    int bad = fp4o_quantize(W, M, K, codes, scales);
    fp4o_pack(codes, M, K, packed);
    free(codes);
    return bad;
}

int fp4o_unpack(const uint8_t *packed, const uint16_t *scales, int64_t M, int64_t K, uint16_t *W)
{
    uint8_t *codes = (uint8_t *)malloc((size_t)(M * K));
    if (!codes)
        return 2;
    fp4o_unpack_codes(packed, M, K, codes);
    for (int64_t m = 0; m < M; ++m) {
        double s = fp6o_half_to_double(scales[m]);
        for (int64_t k = 0; k < K; ++k)
            W[m * K + k] = fp6o_double_to_half(fp4o_decode(codes[m * K + k]) * s);
    }
    free(codes);
    return 0;
}

void fp4o_linear_codes(const uint8_t *codes, const uint16_t *scales, const uint16_t *X, int64_t M,
                       int64_t N, int64_t K, const int64_t *rows, int64_t nrows, double *Y)
{
    if (!rows)
        nrows = M;
    double *Xd = (double *)malloc((size_t)(N * K) * sizeof(double));
    for (int64_t i = 0; i < N * K; ++i)
        Xd[i] = fp6o_half_to_double(X[i]);
    double table[16];
    for (int c = 0; c < 16; ++c)
        table[c] = fp4o_decode(c);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        int64_t m = rows ? rows[i] : i;
        double s = fp6o_half_to_double(scales[m]);
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += table[codes[m * K + k]] * Xd[n * K + k];
            Y[n * nrows + i] = s * acc;
        }
    }
    free(Xd);
}

int fp4o_linear(const uint8_t *packed, const uint16_t *scales, const uint16_t *X, int64_t M,
                int64_t N, int64_t K, const int64_t *rows, int64_t nrows, double *Y)
{
    if (!rows)
        nrows = M;
    uint8_t *codes = (uint8_t *)malloc((size_t)(nrows * K));
    uint16_t *sc = (uint16_t *)malloc((size_t)nrows * sizeof(uint16_t));
    if (!codes || !sc) {
        free(codes);
        free(sc);
        return 2;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        int64_t m = rows ? rows[i] : i;
        sc[i] = scales[m];
        for (int64_t k = 0; k < K; ++k) {
            int c = 0;
            for (int b = 0; b < 4; ++b) {
                uint64_t p = fp4o_pos(M, K, m, k, b);
                c |= ((packed[p >> 3] >> (p & 7)) & 1) << b;
            }
            codes[i * K + k] = (uint8_t)c;
        }
    }
    fp4o_linear_codes(codes, sc, X, nrows, N, K, NULL, nrows, Y);
    free(codes);
    free(sc);
    return 0;
}

/* ====================================================================== *
 * The 3-bit variant (W3A16; the paper lists 3-bit among the widths its scheme
 * supports, Section 1).  FP3 is read as e2m0, code = s e1 e0: Eq. 1 with bias
 * 2^(2-1)-1 = 1 and no mantissa bits, the E = 0 binade read as subnormals
 * 0.M * 2^(1-bias) = 0, no inf/NaN: values 0 | 1 | 2 | 4.  (The other 3-bit
 * split, e1m1 with bias 0, gives the uniform grid 0 1 2 3, i.e. a sign-magnitude
 * integer; e2m0 is the one with a floating-point character.)  Quantizer: the
 * same recipe with 4 in place of 28.
 * ====================================================================== */

#define FP3O_TILE_BYTES 3072 /* 16 * 512 * 3 / 8 */

double fp3o_decode(int code)
{
    int S = (code >> 2) & 1;
    int E = code & 3;
    double mag = E == 0 ? 0.0 : ldexp(1.0, E - 1); /* 0.M * 2^(1-bias) with no M; 1.M * 2^(E-bias) */
    return S ? -mag : mag;
}

/* fp16 nearest to amax/4 (ties to even), decided with exact arithmetic. */
uint16_t fp3o_scale_for_amax(uint16_t amax_bits)
{
    double a = fp6o_half_to_double((uint16_t)(amax_bits & 0x7fffu));
    uint16_t guess = fp6o_double_to_half(a / 4.0);
    int lo = guess > 0 ? guess - 1 : 0;
    int hi = guess + 1;
    int best = -1;
    double best_err = 0.0;
    for (int h = lo; h <= hi; ++h) {
        double err = fabs(4.0 * fp6o_half_to_double((uint16_t)h) - a); /* exact */
        if (best < 0 || err < best_err || (err == best_err && (h & 1) == 0 && (best & 1) == 1)) {
            best = h;
            best_err = err;
        }
    }
    return (uint16_t)best;
}

int fp3o_quantize_one(uint16_t w_bits, uint16_t scale_bits)
{
    int sign = (w_bits >> 15) & 1;
    double a = fp6o_half_to_double((uint16_t)(w_bits & 0x7fffu));
    double s = fp6o_half_to_double((uint16_t)(scale_bits & 0x7fffu));
    if (s == 0.0)
        return sign << 2;
    int best = 0;
    double best_err = fabs(a - fp3o_decode(0) * s);
    for (int g = 1; g < 4; ++g) {
        double err = fabs(a - fp3o_decode(g) * s);
        if (err < best_err || (err == best_err && (g & 1) == 0)) {
            best = g;
            best_err = err;
        }
    }
    return (sign << 2) | best;
}

int fp3o_quantize(const uint16_t *W, int64_t M, int64_t K, uint8_t *codes, uint16_t *scales)
{
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        uint16_t amax = 0;
        for (int64_t k = 0; k < K; ++k) {
            uint16_t mag = (uint16_t)(W[m * K + k] & 0x7fffu);
            if (mag >= 0x7c00u)
                bad |= 1;
            if (mag > amax)
                amax = mag;
        }
        uint16_t sc = fp3o_scale_for_amax(amax);
        scales[m] = sc;
        for (int64_t k = 0; k < K; ++k)
            codes[m * K + k] = (uint8_t)fp3o_quantize_one(W[m * K + k], sc);
    }
    return bad;
}

/* tiles of 16 rows x 512 columns; a matrix whose K is an odd multiple of 256 pads its last tile */
int64_t fp3o_packed_bytes(int64_t M, int64_t K) { return (K + 511) / 512 * (M / FP6O_TILE_ROWS) * FP3O_TILE_BYTES; }

/*
 * Bit address of bit b (0..2 = e0, e1, s) of the code of weight (m, k) in the packed
 * 3-bit stream.  Tiles of 16 rows x 512 columns, k-tile major, 3072 bytes each: three
 * planes of 1024 bytes (64 slots of 16 bytes, slot = 16*q + r as in the other layouts), so
 * that a lane fetches its share of a tile with three whole 128-bit loads.  The two halves of
 * a tile (256 columns each, half h = columns 256h .. 256h+255) are laid out alike: a half
 * gives the slot six 32-bit words, words 3g .. 3g+2 serving the runs 4g .. 4g+3 of the half
 * (g = 0, 1).  The reader wants, per run, a word of eight 4-bit fields "s e1 e0 0" (the
 * 4-bit code of the same value), field j = column 32*run + 8*q + j.  Runs 4g+i, i < 3, sit
 * in word 3g+i in exactly that form, which leaves bit 0 of every field free; the three bits
 * of run 4g+3 are spread over those free bits: its bit b+1 of field j is bit 4j of word
 * 3g+b.  (The ahead-of-time bit-level re-layout of Section 5.2 with a 3+1 split: the
 * reader needs one AND per in-place run and three AND/shift/OR for the spread one.)
 * Words 0..3 of half h fill the slot's 16 bytes of plane 2h (the first and the last plane);
 * words 4, 5 are words 2h, 2h+1 of the slot's 16 bytes of the middle plane.  A reader that
 * wants one half only fetches one 16-byte and one 8-byte piece; one that wants the tile
 * fetches three 16-byte pieces.  When K is an odd multiple of 256 the second half of the last
 * tile of every row tile is padding (zero bits).
 */
uint64_t fp3o_pos(int64_t M, int64_t K, int64_t m, int64_t k, int b)
{
    (void)K;
    int64_t row_tile = m / FP6O_TILE_ROWS;
    int r = (int)(m % FP6O_TILE_ROWS);
    int64_t k_tile = k / 512;
    int half = (int)(k % 512) / 256;
    int kk = (int)(k % 256);
    int run = kk / 32;
    int q = (kk % 32) / 8;
    int j = kk % 8;
    int slot = 16 * q + r;
    int g = run / 4, i = run % 4;
    int word = i < 3 ? 3 * g + i : 3 * g + b;
    int bit = i < 3 ? 4 * j + b + 1 : 4 * j;
    uint64_t tile = (uint64_t)(k_tile * (M / FP6O_TILE_ROWS) + row_tile);
    uint64_t byte_addr = tile * FP3O_TILE_BYTES + (uint64_t)slot * 16u
                         + (word < 4 ? (uint64_t)(2 * half) * 1024u + (uint64_t)word * 4u
                                     : 1024u + (uint64_t)(2 * half + word - 4) * 4u);
    return byte_addr * 8u + (uint64_t)bit;
}

void fp3o_pack(const uint8_t *codes, int64_t M, int64_t K, uint8_t *packed)
{
    memset(packed, 0, (size_t)fp3o_packed_bytes(M, K));
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k)
            for (int b = 0; b < 3; ++b)
                if ((codes[m * K + k] >> b) & 1) {
                    uint64_t p = fp3o_pos(M, K, m, k, b);
                    packed[p >> 3] |= (uint8_t)(1u << (p & 7));
                }
}

void fp3o_unpack_codes(const uint8_t *packed, int64_t M, int64_t K, uint8_t *codes)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            int c = 0;
            for (int b = 0; b < 3; ++b) {
                uint64_t p = fp3o_pos(M, K, m, k, b);
                c |= ((packed[p >> 3] >> (p & 7)) & 1) << b;
            }
            codes[m * K + k] = (uint8_t)c;
        }
}

int fp3o_quantize_pack(const uint16_t *W, int64_t M, int64_t K, uint8_t *packed, uint16_t *scales)
{
    uint8_t *codes = (uint8_t *)malloc((size_t)(M * K));
    if (!codes)
        return 2;
    int bad = fp3o_quantize(W, M, K, codes, scales);
    fp3o_pack(codes, M, K, packed);
    free(codes);
    return bad;
}

int fp3o_unpack(const uint8_t *packed, const uint16_t *scales, int64_t M, int64_t K, uint16_t *W)
{
    uint8_t *codes = (uint8_t *)malloc((size_t)(M * K));
    if (!codes)
        return 2;
    fp3o_unpack_codes(packed, M, K, codes);
    for (int64_t m = 0; m < M; ++m) {
        double s = fp6o_half_to_double(scales[m]);
        for (int64_t k = 0; k < K; ++k)
            W[m * K + k] = fp6o_double_to_half(fp3o_decode(codes[m * K + k]) * s);
    }
    free(codes);
    return 0;
}

void fp3o_linear_codes(const uint8_t *codes, const uint16_t *scales, const uint16_t *X, int64_t M,
                       int64_t N, int64_t K, const int64_t *rows, int64_t nrows, double *Y)
{
    if (!rows)
        nrows = M;
    double *Xd = (double *)malloc((size_t)(N * K) * sizeof(double));
    for (int64_t i = 0; i < N * K; ++i)
        Xd[i] = fp6o_half_to_double(X[i]);
    double table[8];
    for (int c = 0; c < 8; ++c)
        table[c] = fp3o_decode(c);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        int64_t m = rows ? rows[i] : i;
        double s = fp6o_half_to_double(scales[m]);
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += table[codes[m * K + k]] * Xd[n * K + k];
            Y[n * nrows + i] = s * acc;
        }
    }
    free(Xd);
}

int fp3o_linear(const uint8_t *packed, const uint16_t *scales, const uint16_t *X, int64_t M,
                int64_t N, int64_t K, const int64_t *rows, int64_t nrows, double *Y)
{
    if (!rows)
        nrows = M;
    uint8_t *codes = (uint8_t *)malloc((size_t)(nrows * K));
    uint16_t *sc = (uint16_t *)malloc((size_t)nrows * sizeof(uint16_t));
    if (!codes || !sc) {
        free(codes);
        free(sc);
        return 2;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        int64_t m = rows ? rows[i] : i;
        sc[i] = scales[m];
        for (int64_t k = 0; k < K; ++k) {
            int c = 0;
            for (int b = 0; b < 3; ++b) {
                uint64_t p = fp3o_pos(M, K, m, k, b);
                c |= ((packed[p >> 3] >> (p & 7)) & 1) << b;
            }
            codes[i * K + k] = (uint8_t)c;
        }
    }
    fp3o_linear_codes(codes, sc, X, nrows, N, K, NULL, nrows, Y);
    free(codes);
    free(sc);
    return 0;
}

/* The same steps after the linear layer of any of the formats of this file: bits = 6, 5, 4 or 3 selects
 * fp6o_linear, fp5o_linear, fp4o_linear or fp3o_linear; bits = 6 with group > 0 selects the group-wise
 * scales of fp6go_linear.  fp6o_linear_fused above is this function with bits = 6, group = 0. */
int fpxo_linear_fused(int bits, int64_t group, const uint8_t *packed, const uint16_t *scales, const uint16_t *X,
                      int64_t M, int64_t N, int64_t K, const uint16_t *bias, const uint16_t *residual, int gated,
                      const int64_t *rows, int64_t nrows, double *Y)
{
    if (bits < 3 || bits > 6 || (group > 0 && bits != 6))
        return 4;
    const int64_t Mout = gated ? M / 2 : M;
    if (gated && M % 2)
        return 3;
    if (!rows)
        nrows = Mout;
    const int64_t per = gated ? 2 : 1; /* weight rows behind one output row */
    int64_t *wrows = (int64_t *)malloc((size_t)(nrows * per) * sizeof(int64_t));
    double *Z = (double *)malloc((size_t)(N * nrows * per) * sizeof(double));
    if (!wrows || !Z) {
        free(wrows);
        free(Z);
        return 2;
    }
    for (int64_t i = 0; i < nrows; ++i) {
        int64_t o = rows ? rows[i] : i;
        for (int64_t j = 0; j < per; ++j)
            wrows[i * per + j] = o * per + j;
    }
    int rc;
    if (bits == 6 && group > 0)
        rc = fp6go_linear(packed, scales, X, M, N, K, group, wrows, nrows * per, Z);
    else if (bits == 6)
        rc = fp6o_linear(packed, scales, X, M, N, K, wrows, nrows * per, Z);
    else if (bits == 5)
        rc = fp5o_linear(packed, scales, X, M, N, K, wrows, nrows * per, Z);
    else if (bits == 4)
        rc = fp4o_linear(packed, scales, X, M, N, K, wrows, nrows * per, Z);
    else
        rc = fp3o_linear(packed, scales, X, M, N, K, wrows, nrows * per, Z);
    if (rc == 0) {
        for (int64_t n = 0; n < N; ++n)
            for (int64_t i = 0; i < nrows; ++i) {
                int64_t o = rows ? rows[i] : i;
                double z[2] = {0.0, 0.0};
                for (int64_t j = 0; j < per; ++j) {
                    z[j] = Z[n * nrows * per + i * per + j];
                    if (bias)
                        z[j] += fp6o_half_to_double(bias[o * per + j]);
                }
                double y = gated ? z[0] / (1.0 + exp(-z[0])) * z[1] : z[0];
                if (residual)
                    y += fp6o_half_to_double(residual[n * Mout + o]);
                Y[n * nrows + i] = y;
            }
    }
    free(wrows);
    free(Z);
    return rc;
}

#ifdef _OPENMP
#include <omp.h>
int fp6o_threads(void) { return omp_get_max_threads(); }
#else
int fp6o_threads(void) { return 1; }
#endif
