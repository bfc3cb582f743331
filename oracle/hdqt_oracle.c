/*
 * CPU oracle for Hadamard Domain Quantized Training (HDQT) matmuls.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
 * library is checked against.  It is compiled on its own (gcc, no headers
 * shared with the HIP sources) and nothing in the product path may call it.
 *
 * What it computes, step by step, in the paper's notation (Methodology
 * section: problem statement Z = X W, quantizer Q, Sylvester Hadamard H_k,
 * block-diagonal H, stochastic rounding, tiled low-bit accumulation):
 *
 *   1. orientation    pick the two operands and the contraction dimension D
 *   2. transform      y = x H along D, H = BlockDiag(H_k, .., H_k), order
 *                     n = 2^k, unnormalised +-1 entries (H H^T = n I)
 *   3. calibration    amax = max |y| over the tensor, alpha = 1/(clip*amax)
 *   4. quantizer Q    code = clamp(round(alpha * y * 2^(b-1))) as a b-bit
 *                     two's-complement integer; "round" is nearest-even or
 *                     stochastic (floor + Bernoulli(frac))
 *   5. tiled matmul   acc = sum over tiles t of sat_a(sum_{d in tile t}
 *                     qA[i,d] qB[j,d]), tiles of s along D, sat_a = clamp to
 *                     an a-bit signed accumulator
 *   6. dequantize     out = acc * scaleA * scaleB / n   (the 1/n undoes
 *                     H H^T = n I; the product needs no inverse transform)
 *
 * Precision.  The paper does not fix one.  Steps 2-4 decide integers (the
 * codes), so they are taken in binary32 -- the precision the GPU kernels
 * compute in -- with every rounding spelled out: the transform is the
 * balanced pairwise summation tree over the signed terms in natural index
 * order, the scale is one multiplication and one correctly rounded division,
 * the code is one multiplication and one rounding.  Build with
 * -ffp-contract=off so that no fused multiply-add replaces these.
 *
 *   5'. second reading of step 5 (orc_tiled_matmul_requant): every tile's
 *                     partial-sum tensor goes through Q with a bits and its own
 *                     max, and the tile results are added
 *   5''. input gradient of a convolution (orc_col2im_acc, an extension): the
 *                     accumulators of dX = G W^T folded back onto the layer's input
 *                     (the transpose of im2col) as exact integer sums, then step 6
 *   6''. input gradient behind a rectifier (orc_relu_mask, an extension): step 6's
 *                     values where the layer's input is positive, zero elsewhere
 *   6'. narrow output (orc_dequantize_bf16, an extension that is not in the
 *                     paper): step 6's binary32 value rounded to bfloat16,
 *                     nearest, ties to even; pinned by hand-built ties and a
 *                     library conversion
 *
 * Parity pins live in tests/ (H H^T = n I, scipy's Hadamard matrix, fp64
 * transform, grid inputs with known codes, hand-computed saturation cases,
 * exact int64 matmul when nothing saturates, an independent Philox engine).
 * The accuracy tables of the paper are "parity unpinned": they need its
 * datasets and training code.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_ROUND_NEAREST 0
#define ORC_ROUND_STOCHASTIC 1

#define ORC_FWD 0        /* Z[M,N]  = X[M,K] W[K,N]      contraction K */
#define ORC_BWD_INPUT 1  /* dX[M,K] = G[M,N] W[K,N]^T    contraction N */
#define ORC_BWD_WEIGHT 2 /* dW[K,N] = X[M,K]^T G[M,N]    contraction M */

/* ------------------------------------------------------------------ */
/* Hadamard matrices (Methodology: Sylvester form)                     */
/* ------------------------------------------------------------------ */

/* H_0 = [1]; H_k = [[H_{k-1}, H_{k-1}], [H_{k-1}, -H_{k-1}]].
 * Writes the n x n matrix (n = 2^k) of +1/-1 entries, row-major. */
void orc_hadamard_matrix(int k, int8_t *H)
{
    int64_t n = (int64_t)1 << k;
    H[0] = 1;
    for (int64_t m = 1; m < n; m *= 2) {
        /* the m x m matrix sits in the top-left corner with row pitch n */
        for (int64_t r = 0; r < m; ++r)
            for (int64_t c = 0; c < m; ++c) {
                int8_t h = H[r * n + c];
                H[r * n + (c + m)] = h;
                H[(r + m) * n + c] = h;
                H[(r + m) * n + (c + m)] = (int8_t)-h;
            }
    }
}

/* Block order (Methodology, block-diagonal H = BlockDiag(H_k, ..., H_k)): the
 * blocks must tile the contraction length exactly, so the order actually used
 * is the requested order n lowered to the largest power of two dividing D. */
int orc_n_eff(int64_t D, int n)
{
    int m = 1;
    while (m * 2 <= n && D % (m * 2) == 0)
        m *= 2;
    return m;
}

/* Balanced pairwise sum of term[lo..hi] (inclusive) in binary32. */
static float pairwise_sum(const float *term, int lo, int hi)
{
    if (lo == hi)
        return term[lo];
    int mid = lo + (hi - lo) / 2;
    float left = pairwise_sum(term, lo, mid);
    float right = pairwise_sum(term, mid + 1, hi);
    return left + right;
}

/* Blocked transform of T[rows, cols] (row-major) along `axis`
 * (1: along a row, D = cols; 0: along a column, D = rows) with blocks of
 * order n (n must divide D).  Y has T's shape and layout.
 * y[block*n + i] = sum_j H[i][j] * x[block*n + j], naive O(n^2). */
void orc_hadamard_transform(const float *T, int64_t rows, int64_t cols, int axis,
                            int n, float *Y)
{
    int k = 0;
    while (((int64_t)1 << k) < n)
        ++k;
    int8_t *H = (int8_t *)malloc((size_t)n * n);
    orc_hadamard_matrix(k, H);
    int64_t D = axis ? cols : rows;
    int64_t lines = axis ? rows : cols;
    int64_t step = axis ? 1 : cols;     /* distance between consecutive d */
    int64_t line_step = axis ? cols : 1;
#pragma omp parallel
    {
        float *term = (float *)malloc(sizeof(float) * (size_t)n);
#pragma omp for schedule(static)
        for (int64_t l = 0; l < lines; ++l) {
            const float *x = T + l * line_step;
            float *y = Y + l * line_step;
            for (int64_t blk = 0; blk < D / n; ++blk) {
                for (int i = 0; i < n; ++i) {
                    for (int j = 0; j < n; ++j) {
                        float v = x[(blk * n + j) * step];
                        term[j] = H[(int64_t)i * n + j] > 0 ? v : -v;
                    }
                    y[(blk * n + i) * step] = pairwise_sum(term, 0, n - 1);
                }
            }
        }
        free(term);
    }
    free(H);
}

/* Same transform with every sum taken left to right in binary64: used by the
 * tests to bound the binary32 tree's rounding error, never by the path. */
void orc_hadamard_transform_f64(const float *T, int64_t rows, int64_t cols, int axis,
                                int n, double *Y)
{
    int k = 0;
    while (((int64_t)1 << k) < n)
        ++k;
    int8_t *H = (int8_t *)malloc((size_t)n * n);
    orc_hadamard_matrix(k, H);
    int64_t D = axis ? cols : rows;
    int64_t lines = axis ? rows : cols;
    int64_t step = axis ? 1 : cols;
    int64_t line_step = axis ? cols : 1;
    for (int64_t l = 0; l < lines; ++l)
        for (int64_t blk = 0; blk < D / n; ++blk)
            for (int i = 0; i < n; ++i) {
                double sum = 0.0;
                for (int j = 0; j < n; ++j)
                    sum += (double)H[(int64_t)i * n + j] *
                           (double)T[l * line_step + (blk * n + j) * step];
                Y[l * line_step + (blk * n + i) * step] = sum;
            }
    free(H);
}

/* ------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11)                   */
/* ------------------------------------------------------------------ */

void orc_philox4x32_10(const uint32_t ctr_in[4], const uint32_t key_in[2], uint32_t out[4])
{
    const uint64_t MUL_A = 0xD2511F53u, MUL_B = 0xCD9E8D57u;
    const uint32_t WEYL_A = 0x9E3779B9u, WEYL_B = 0xBB67AE85u;
    uint32_t c0 = ctr_in[0], c1 = ctr_in[1], c2 = ctr_in[2], c3 = ctr_in[3];
    uint32_t k0 = key_in[0], k1 = key_in[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t pa = MUL_A * (uint64_t)c0;
        uint64_t pb = MUL_B * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)pb;
        uint32_t n2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)pa;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += WEYL_A;
        k1 += WEYL_B;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 16 random bits that element e (row-major linear index in the source
 * tensor) of tensor `tensor_id` draws under `seed`.  One Philox block serves
 * eight consecutive elements: counter = (e/8 low, e/8 high, tensor_id, 0),
 * key = (seed low, seed high); element e takes half-word (e mod 2) of output
 * word ((e/2) mod 4). */
uint32_t orc_sr_bits(uint64_t seed, uint32_t tensor_id, uint64_t e)
{
    uint64_t blk = e >> 3;
    uint32_t ctr[4] = {(uint32_t)blk, (uint32_t)(blk >> 32), tensor_id, 0u};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    uint32_t word = out[(e >> 1) & 3];
    return (word >> (16 * (e & 1))) & 0xFFFFu;
}

/* ------------------------------------------------------------------ */
/* Quantizer Q (Methodology: uniform integer quantization, max          */
/* calibration, stochastic rounding on selected tensors)               */
/* ------------------------------------------------------------------ */

/* Quantize T[rows, cols] along `axis` in the Hadamard domain.
 *   had_block  requested order n (1 = no transform); lowered by orc_n_eff
 *   b          code width, 2..8
 *   round_mode ORC_ROUND_*
 *   clip       factor on the maximum (1, or 0.975 in the paper's forward pass)
 * Outputs:
 *   codes      int8, contraction-major: codes[line * D + d] with
 *              line = row (axis 1) or column (axis 0)
 *   scale_out  the value of one code step, clip*amax / 2^(b-1)
 *   n_eff_out  block order used
 * Returns 0, or -1 on bad arguments. */
int orc_quantize(const float *T, int64_t rows, int64_t cols, int axis, int had_block,
                 int b, int round_mode, float clip, uint32_t tensor_id, uint64_t seed,
                 int8_t *codes, float *scale_out, int *n_eff_out)
{
    if (!T || !codes || rows <= 0 || cols <= 0 || b < 2 || b > 8 || had_block < 1 ||
        (had_block & (had_block - 1)) != 0 || !(clip > 0.0f) || clip > 1.0f)
        return -1;
    int64_t D = axis ? cols : rows;
    int64_t lines = axis ? rows : cols;
    int n = orc_n_eff(D, had_block);
    if (n_eff_out)
        *n_eff_out = n;

    int64_t total = rows * cols;
    float *Y = (float *)malloc(sizeof(float) * (size_t)total);
    orc_hadamard_transform(T, rows, cols, axis, n, Y);

    float amax = 0.0f;
    for (int64_t e = 0; e < total; ++e) {
        float m = fabsf(Y[e]);
        if (m > amax)
            amax = m;
    }
    float amax_clipped = clip * amax;
    float levels = (float)(1 << (b - 1)); /* 2^(b-1) */
    int qmin = -(1 << (b - 1)), qmax = (1 << (b - 1)) - 1;

    if (amax_clipped == 0.0f) {
        memset(codes, 0, (size_t)total);
        if (scale_out)
            *scale_out = 0.0f;
        free(Y);
        return 0;
    }
    float inv = levels / amax_clipped;   /* alpha * 2^(b-1), one rounded division */
    float scale = amax_clipped / levels; /* exact: division by a power of two */
    if (scale_out)
        *scale_out = scale;

#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            int64_t e = r * cols + c;
            float v = Y[e] * inv;
            float q;
            if (round_mode == ORC_ROUND_STOCHASTIC) {
                float fl = floorf(v);
                float frac = v - fl; /* exact */
                float u = (float)orc_sr_bits(seed, tensor_id, (uint64_t)e);
                q = fl + ((u < frac * 65536.0f) ? 1.0f : 0.0f);
            } else {
                q = rintf(v); /* round half to even */
            }
            if (q < (float)qmin)
                q = (float)qmin;
            if (q > (float)qmax)
                q = (float)qmax;
            int64_t line = axis ? r : c;
            int64_t d = axis ? c : r;
            codes[line * D + d] = (int8_t)q;
        }
    (void)lines;
    free(Y);
    return 0;
}

/* Exported code format: lines x D, contraction index contiguous.
 * b <= 4: two codes per byte, even index in bits 0-3, odd index in bits 4-7,
 * two's-complement nibbles, row pitch ceil(D/2) with a zero pad nibble when D
 * is odd.  b > 4: one int8 per code, pitch D. */
int64_t orc_packed_pitch(int64_t D, int b) { return b <= 4 ? (D + 1) / 2 : D; }

void orc_pack_codes(const int8_t *codes, int64_t lines, int64_t D, int b, uint8_t *packed)
{
    int64_t pitch = orc_packed_pitch(D, b);
    for (int64_t l = 0; l < lines; ++l) {
        if (b > 4) {
            memcpy(packed + l * pitch, codes + l * D, (size_t)D);
            continue;
        }
        for (int64_t j = 0; j < pitch; ++j) {
            uint8_t lo = (uint8_t)codes[l * D + 2 * j] & 0xF;
            uint8_t hi = (2 * j + 1 < D) ? ((uint8_t)codes[l * D + 2 * j + 1] & 0xF) : 0;
            packed[l * pitch + j] = (uint8_t)(lo | (hi << 4));
        }
    }
}

/* ------------------------------------------------------------------ */
/* Tiled integer matmul with a-bit accumulators                         */
/* ------------------------------------------------------------------ */

static int64_t saturate(int64_t p, int a)
{
    int64_t hi = ((int64_t)1 << (a - 1)) - 1;
    int64_t lo = -((int64_t)1 << (a - 1));
    return p > hi ? hi : (p < lo ? lo : p);
}

/* One output: tiles [t*s, min((t+1)*s, D)); the tile's sum is formed exactly,
 * then held in an a-bit accumulator (saturating once, on the finished sum);
 * tile results are added without further narrowing. */
static int32_t tiled_dot(const int8_t *qa, const int8_t *qb, int64_t D, int64_t s, int a)
{
    int64_t acc = 0;
    for (int64_t t0 = 0; t0 < D; t0 += s) {
        int64_t t1 = t0 + s < D ? t0 + s : D;
        int64_t part = 0;
        for (int64_t d = t0; d < t1; ++d)
            part += (int64_t)qa[d] * (int64_t)qb[d];
        acc += saturate(part, a);
    }
    return (int32_t)acc;
}

/* acc[i, j] for i < RA, j < RB from codes qA[RA, D], qB[RB, D]. */
void orc_tiled_matmul(const int8_t *qA, const int8_t *qB, int64_t RA, int64_t RB, int64_t D,
                      int64_t s, int a, int32_t *acc)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < RA; ++i)
        for (int64_t j = 0; j < RB; ++j)
            acc[i * RB + j] = tiled_dot(qA + i * D, qB + j * D, D, s, a);
}

/* Only the listed outputs: acc[p] for (ii[p], jj[p]), p < count. */
void orc_tiled_matmul_sampled(const int8_t *qA, const int8_t *qB, int64_t D, int64_t s, int a,
                              const int64_t *ii, const int64_t *jj, int64_t count,
                              int32_t *acc)
{
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < count; ++p)
        acc[p] = tiled_dot(qA + ii[p] * D, qB + jj[p] * D, D, s, a);
}

/* out = acc * (scaleA * scaleB) / n, three binary32 operations. */
float orc_dequant_factor(float scaleA, float scaleB, int n_eff)
{
    float prod = scaleA * scaleB;
    return prod * (1.0f / (float)n_eff); /* 1/n is a power of two: exact */
}

void orc_dequantize(const int32_t *acc, int64_t count, float scaleA, float scaleB, int n_eff,
                    float *out)
{
    float dq = orc_dequant_factor(scaleA, scaleB, n_eff);
    for (int64_t p = 0; p < count; ++p)
        out[p] = (float)acc[p] * dq;
}

/* Input gradient behind a rectifier (an engineering extension: a framework applies this
 * as a separate pass over dX).  When the layer's input is x = max(pre, 0), the gradient of
 * `pre` is the layer's input gradient where x is positive and zero elsewhere:
 *     masked[p] = x[p] > 0 ? dX[p] : +0
 * x has dX's shape (the im2col matrix for the matrix path, the activation for the folded
 * path).  Entries that are masked out are +0.0f whatever the sign of dX[p]. */
void orc_relu_mask(const float *dX, const float *x, int64_t count, float *masked)
{
    for (int64_t p = 0; p < count; ++p)
        masked[p] = x[p] > 0.0f ? dX[p] : 0.0f;
}

/* Narrow output (an engineering extension, not a step of the paper, whose layers hand
 * binary32 on): the dequantized binary32 value of step 6 rounded once more, to bfloat16
 * (1 sign, 8 exponent, 7 fraction bits: the upper half of a binary32), round to nearest,
 * ties to even.  Returned as the 16-bit pattern.  Finite inputs; a value beyond the
 * largest finite bfloat16 rounds to infinity, as IEEE rounding prescribes. */
uint16_t orc_bf16_bits(float x)
{
    uint32_t u;
    memcpy(&u, &x, sizeof u);
    uint32_t keep = u >> 16;      /* sign, exponent, 7 fraction bits */
    uint32_t rest = u & 0xFFFFu;  /* the 16 fraction bits that go */
    if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u)))
        keep += 1u; /* magnitude up by one unit; a carry into the exponent is the right result */
    return (uint16_t)keep;
}

void orc_dequantize_bf16(const int32_t *acc, int64_t count, float scaleA, float scaleB, int n_eff,
                         uint16_t *out)
{
    float dq = orc_dequant_factor(scaleA, scaleB, n_eff);
    for (int64_t p = 0; p < count; ++p)
        out[p] = orc_bf16_bits((float)acc[p] * dq);
}

/* Input gradient of a convolution layer (an engineering extension: the paper's layers
 * stop at the gradient of the im2col matrix and leave the fold to the framework).
 * The layer's input act[batch, C, H, W] enters the matmuls as X[M, K], M = batch*H*W,
 * K = C*kh*kw, with X[(b,y,x), c*kh*kw + ty*kw + tx] = act[b, c, y + ty - ph, x + tx - pw]
 * (zero outside the image; ph = (kh-1)/2, pw = (kw-1)/2; stride 1).  The gradient of act is
 * the transpose of that map applied to dX = G W^T:
 *     dAct[b,c,y,x] = sum over taps (ty,tx) of dX[(b, y - ty + ph, x - tx + pw), c*kh*kw + ty*kw + tx]
 * over the taps whose source pixel lies in the image.  Here the sum is taken on the
 * integer accumulators of step 5, which is exact, and step 6 is applied once to the sum:
 *     accAct = sum of acc[...]  (int32),   dAct = fl(float(accAct) * dq)
 * (dequantization is linear, so this is the fold of the dequantized dX up to rounding,
 * and it does not depend on the order of the sum). */
void orc_col2im_acc(const int32_t *acc, int64_t batch, int C, int H, int W, int kh, int kw,
                    int32_t *acc_act)
{
    const int ph = (kh - 1) / 2, pw = (kw - 1) / 2;
    const int64_t K = (int64_t)C * kh * kw;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < batch; ++b)
        for (int c = 0; c < C; ++c)
            for (int y = 0; y < H; ++y)
                for (int x = 0; x < W; ++x) {
                    int64_t sum = 0;
                    for (int ty = 0; ty < kh; ++ty)
                        for (int tx = 0; tx < kw; ++tx) {
                            const int yp = y - ty + ph, xp = x - tx + pw;
                            if (yp < 0 || yp >= H || xp < 0 || xp >= W)
                                continue;
                            const int64_t m = (b * H + yp) * W + xp;
                            sum += acc[m * K + ((int64_t)c * kh + ty) * kw + tx];
                        }
                    acc_act[((b * C + c) * H + y) * W + x] = (int32_t)sum;
                }
}

/* ------------------------------------------------------------------ */
/* Second reading of the low-bit accumulator: tiled quantization        */
/* ------------------------------------------------------------------ */

/* Methodology, "tiled quantization ... limiting computations to tiles of size s",
 * read through the paper's own emulation device, the quantizer Q: the partial-sum
 * tensor of every tile t,
 *     P_t[i,j] = sum_{d in tile t} qA[i,d] qB[j,d]        (exact integers),
 * is passed through Q with a bits and its own max calibration, and the tile
 * results are added:
 *     m_t      = max_{i,j} |P_t[i,j]|                      (over the whole tensor)
 *     inv_t    = fl(2^(a-1) / m_t)                         (binary32, correctly rounded)
 *     c_t[i,j] = clamp(RNE(fl(float(P_t[i,j]) * inv_t)), -2^(a-1), 2^(a-1) - 1)
 *     acc[i,j] = sum_t c_t[i,j] * m_t                      (exact; value = acc / 2^(a-1))
 * A tile whose partial sums are all zero contributes nothing.  Same conventions as
 * the operand quantizer above (scale by 2^(b-1), two's-complement clamp, nearest-even).
 * tile_max (nullable) receives m_t for every tile. */
void orc_tiled_matmul_requant(const int8_t *qA, const int8_t *qB, int64_t RA, int64_t RB,
                              int64_t D, int64_t s, int a, int64_t *acc, int32_t *tile_max)
{
    int32_t *P = (int32_t *)malloc((size_t)(RA * RB) * sizeof(int32_t));
    const int32_t qmax = (int32_t)(((int64_t)1 << (a - 1)) - 1), qmin = -qmax - 1;
    for (int64_t p = 0; p < RA * RB; ++p) acc[p] = 0;
    int64_t t = 0;
    for (int64_t t0 = 0; t0 < D; t0 += s, ++t) {
        int64_t t1 = t0 + s < D ? t0 + s : D;
        int32_t m = 0;
#pragma omp parallel for schedule(static) reduction(max : m)
        for (int64_t i = 0; i < RA; ++i)
            for (int64_t j = 0; j < RB; ++j) {
                int32_t sum = 0;
                for (int64_t d = t0; d < t1; ++d)
                    sum += (int32_t)qA[i * D + d] * (int32_t)qB[j * D + d];
                P[i * RB + j] = sum;
                int32_t mag = sum < 0 ? -sum : sum;
                if (mag > m) m = mag;
            }
        if (tile_max) tile_max[t] = m;
        if (m == 0) continue;
        /* a binary64 quotient of two integers below 2^31 rounds to binary32 without
         * double-rounding error only if both are binary32 values; m < 2^24 here */
        float inv = (float)((double)((int64_t)1 << (a - 1)) / (double)m);
#pragma omp parallel for schedule(static)
        for (int64_t p = 0; p < RA * RB; ++p) {
            float v = (float)P[p] * inv;
            float r = rintf(v); /* round half to even */
            int32_t c = r > (float)qmax ? qmax : (r < (float)qmin ? qmin : (int32_t)r);
            acc[p] += (int64_t)c * (int64_t)m;
        }
    }
    free(P);
}

/* value = acc * 2^-(a-1) * (scaleA * scaleB) / n: the factor is the three binary32
 * operations of orc_dequant_factor followed by an exact scaling by a power of two. */
float orc_requant_factor(float scaleA, float scaleB, int n_eff, int a)
{
    return ldexpf(orc_dequant_factor(scaleA, scaleB, n_eff), -(a - 1));
}

void orc_dequantize_requant(const int64_t *acc, int64_t count, float scaleA, float scaleB,
                            int n_eff, int a, float *out)
{
    float dq = orc_requant_factor(scaleA, scaleB, n_eff, a);
    for (int64_t p = 0; p < count; ++p)
        out[p] = (float)acc[p] * dq;
}

/* ------------------------------------------------------------------ */
/* The three matmuls of one training step                               */
/* ------------------------------------------------------------------ */

typedef struct {
    int b;              /* code width */
    int round_mode;     /* ORC_ROUND_* */
    float clip;         /* factor on the maximum */
    uint32_t tensor_id; /* random stream selector */
} orc_operand_t;

typedef struct {
    int had_block;  /* requested Hadamard order n */
    int acc_bits;   /* accumulator width a */
    int64_t s;      /* tile length along the contraction */
    uint64_t seed;  /* random seed */
    orc_operand_t A, B;
} orc_params_t;

/* kind selects operands (P, Q) and shapes:
 *   FWD:        P = X[M,K] axis 1, Q = W[K,N] axis 0, out Z[M,N],  D = K
 *   BWD_INPUT:  P = G[M,N] axis 1, Q = W[K,N] axis 1, out dX[M,K], D = N
 *   BWD_WEIGHT: P = X[M,K] axis 0, Q = G[M,N] axis 0, out dW[K,N], D = M
 * Optional outputs (may be NULL): acc_out int32 [RA*RB]; codesA int8 [RA*D];
 * codesB int8 [RB*D]; scales float[2]. */
int orc_gemm(int kind, const float *P, const float *Q, int64_t M, int64_t K, int64_t N,
             const orc_params_t *prm, float *out, int32_t *acc_out, int8_t *codesA,
             int8_t *codesB, float *scales)
{
    int64_t RA, RB, D, p_rows, p_cols, q_rows, q_cols;
    int p_axis, q_axis;
    switch (kind) {
    case ORC_FWD:
        RA = M; RB = N; D = K;
        p_rows = M; p_cols = K; p_axis = 1;
        q_rows = K; q_cols = N; q_axis = 0;
        break;
    case ORC_BWD_INPUT:
        RA = M; RB = K; D = N;
        p_rows = M; p_cols = N; p_axis = 1;
        q_rows = K; q_cols = N; q_axis = 1;
        break;
    case ORC_BWD_WEIGHT:
        RA = K; RB = N; D = M;
        p_rows = M; p_cols = K; p_axis = 0;
        q_rows = M; q_cols = N; q_axis = 0;
        break;
    default:
        return -1;
    }
    if (prm->acc_bits < 2 || prm->acc_bits > 32 || prm->s < 1)
        return -1;
    int8_t *qa = codesA ? codesA : (int8_t *)malloc((size_t)(RA * D));
    int8_t *qb = codesB ? codesB : (int8_t *)malloc((size_t)(RB * D));
    int32_t *acc = acc_out ? acc_out : (int32_t *)malloc(sizeof(int32_t) * (size_t)(RA * RB));
    float sa = 0.0f, sb = 0.0f;
    int na = 0, nb = 0;
    int rc = orc_quantize(P, p_rows, p_cols, p_axis, prm->had_block, prm->A.b, prm->A.round_mode,
                          prm->A.clip, prm->A.tensor_id, prm->seed, qa, &sa, &na);
    if (rc == 0)
        rc = orc_quantize(Q, q_rows, q_cols, q_axis, prm->had_block, prm->B.b,
                          prm->B.round_mode, prm->B.clip, prm->B.tensor_id, prm->seed, qb, &sb,
                          &nb);
    if (rc == 0) {
        /* both operands share D, hence the same block order */
        orc_tiled_matmul(qa, qb, RA, RB, D, prm->s, prm->acc_bits, acc);
        if (out)
            orc_dequantize(acc, RA * RB, sa, sb, na, out);
        if (scales) {
            scales[0] = sa;
            scales[1] = sb;
        }
    }
    if (!codesA) free(qa);
    if (!codesB) free(qb);
    if (!acc_out) free(acc);
    return rc;
}

/* Number of threads the OpenMP loops above use (for reporting timings). */
#ifdef _OPENMP
#include <omp.h>
int orc_num_threads(void) { return omp_get_max_threads(); }
#else
int orc_num_threads(void) { return 1; }
#endif
