/*
 * hdqt.h -- C ABI of the MI355X (gfx950) library for the matmuls of Hadamard
 * Domain Quantized Training (HDQT).
 *
 * The paper's problem statement (Methodology section) is Z = X W with
 * Z in R^{N x C}, X in R^{N x D}, W in R^{D x C}, needed in the forward and the
 * backward pass.  This header writes the three shapes as M (the paper's N,
 * batch x positions), K (the paper's D, fan-in) and N (the paper's C, output
 * features), to keep "N" unambiguous:
 *
 *   forward          Z [M,N] = X[M,K]   W[K,N]      contraction over K
 *   input gradient   dX[M,K] = G[M,N]   W[K,N]^T    contraction over N
 *   weight gradient  dW[K,N] = X[M,K]^T G[M,N]      contraction over M
 *
 * Each matmul runs, on the device, the steps the paper describes:
 *   - blocked Sylvester-Hadamard transform of both operands along the
 *     contraction dimension (H = BlockDiag(H_k,..,H_k), order n = 2^k,
 *     entries +-1, so H H^T = n I and the product needs no inverse transform);
 *   - the quantizer Q: max calibration over the transformed tensor, scaling
 *     into +-1, b-bit integer codes, rounding to nearest-even or stochastic;
 *   - the tiled integer matmul: the contraction is cut into tiles of length s,
 *     each tile's sum is held in an a-bit signed accumulator (it saturates),
 *     tile results are added in 32 bits;
 *   - dequantization: acc * scaleA * scaleB / n.
 *
 * Conventions for every entry point
 *   pointers    DEVICE memory owned by the caller unless a parameter says
 *               "host"; 16-byte aligned; dense row-major, no strides
 *   allocation  the library allocates nothing and keeps no state between
 *               calls; scratch comes from the caller's workspace
 *   ordering    all work is enqueued on `stream` (a hipStream_t passed as
 *               void*, NULL = the default stream) and the call returns without
 *               waiting; outputs are valid once the stream reaches that point
 *   errors      0 on success; a negative HDQT_E* code for argument errors,
 *               found on the host before anything is launched; HDQT_EHIP when
 *               a launch fails (hdqt_last_hip_error() gives the HIP code)
 *   inputs      must be finite and such that 2^(b-1)/max|.| is finite;
 *               otherwise the result is unspecified (no fault, no error)
 */
#ifndef HDQT_H
#define HDQT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HDQT_VERSION 1

/* ---- rounding inside Q (Methodology: nearest by default, stochastic on the
 *      tensors the ablation found sensitive) ---- */
typedef enum { HDQT_ROUND_NEAREST = 0, HDQT_ROUND_STOCHASTIC = 1 } hdqt_round_t;

typedef enum { HDQT_GEMM_FWD = 0, HDQT_GEMM_BWD_INPUT = 1, HDQT_GEMM_BWD_WEIGHT = 2 } hdqt_gemm_kind_t;

/* ---- error codes ---- */
#define HDQT_OK 0
#define HDQT_EINVAL_NULL (-1)     /* a required pointer is NULL */
#define HDQT_EINVAL_DIM (-2)      /* a dimension is <= 0 or above 4 194 240 (65535 * 64), or a
                                     tensor has 2^40 elements or more */
#define HDQT_EINVAL_HADAMARD (-3) /* had_block is not a power of two in [1, 256] */
#define HDQT_EINVAL_BITS (-4)     /* b outside [2, 8] */
#define HDQT_EINVAL_ACC (-5)      /* acc_bits outside [2, 32], or the sum of all tiles may leave int32 */
#define HDQT_EINVAL_TILE (-6)     /* s < 1, or one tile's exact sum may leave int32 */
#define HDQT_EINVAL_CLIP (-7)     /* clip outside (0, 1] */
#define HDQT_EINVAL_ROUND (-8)    /* unknown rounding mode */
#define HDQT_EINVAL_AXIS (-9)     /* axis not 0 or 1 / unknown gemm kind */
#define HDQT_EWORKSPACE (-10)     /* workspace NULL or smaller than required */
#define HDQT_EALIGN (-11)         /* a pointer is not 16-byte aligned */
#define HDQT_EHIP (-12)           /* a HIP call failed */
#define HDQT_EINVAL_GEOMETRY (-13) /* convolution geometry (or layer shape) outside what the
                                      activation-source kernels take: see hdqt_conv_t */
#define HDQT_ESCRATCH (-14)        /* hdqt_gemm_fwd_static: the shape needs more scratch than the
                                      library's fixed device array holds */

/* One quantized operand; names follow the paper's quantizer Q. */
typedef struct {
    int32_t b;          /* bit width of the integer codes, 2..8 (the paper's b)            */
    int32_t round;      /* hdqt_round_t                                                      */
    float clip;         /* factor on max|x| before scaling, in (0, 1]: 1, or 0.975 as in
                           the paper's forward pass for weights and activations            */
    uint32_t tensor_id; /* selects the random stream of this tensor (stochastic only)       */
} hdqt_operand_t;

typedef struct {
    int32_t had_block;  /* requested Hadamard order n = 2^k, 1..256; 1 = no transform.  The
                           order used is the largest power of two <= n dividing the
                           contraction length (see hdqt_n_eff)                             */
    int32_t acc_bits;   /* accumulator width a, 2..32; 32 never saturates                   */
    int64_t s;          /* tile length along the contraction, >= 1; s >= D is one tile      */
    uint64_t seed;      /* key of the stochastic-rounding generator                         */
    hdqt_operand_t A;   /* left operand of the product  (X, G, X for the three kinds)       */
    hdqt_operand_t B;   /* right operand of the product (W, W, G)                           */
} hdqt_params_t;

/* Where hdqt_gemm_* keeps its intermediates inside the caller's workspace
 * (byte offsets).  Lets a test read the codes and scales of a whole matmul. */
typedef struct {
    size_t scaleA;   /* float: value of one code step of operand A */
    size_t scaleB;   /* float */
    size_t codesA;   /* packed codes [RA, D] */
    size_t codesB;   /* packed codes [RB, D] */
    size_t acc;      /* int32 slices of a split contraction (see hdqt_gemm_codes) */
    size_t total;    /* bytes required */
    int64_t RA, RB, D;
    int32_t n_eff;
} hdqt_ws_layout_t;

/* Block order used for a contraction of length D when n is requested
 * (Methodology, H = BlockDiag(H_k, ..., H_k): the blocks must tile D exactly):
 * the largest power of two <= n that divides D.  Host function. */
int hdqt_n_eff(int64_t D, int had_block);

/* Row pitch in bytes of packed codes: ceil(D/2) for b <= 4, D for b > 4. */
int64_t hdqt_codes_pitch(int64_t D, int b);

/* Workspace bytes hdqt_quantize needs (a small constant). */
size_t hdqt_quantize_workspace_size(void);

/* Workspace bytes (and layout) one hdqt_gemm_* call needs.  Returns 0 and
 * fills *layout (if not NULL) on success, a negative code on bad arguments. */
int hdqt_workspace_layout(int gemm_kind, int64_t M, int64_t K, int64_t N,
                          const hdqt_params_t *params, hdqt_ws_layout_t *layout);
size_t hdqt_workspace_size(int gemm_kind, int64_t M, int64_t K, int64_t N,
                           const hdqt_params_t *params); /* 0 on bad arguments */

/*
 * Transform and quantize one tensor (Methodology: Hadamard domain + Q).
 *   T          fp32 [rows, cols], row-major (device)
 *   axis       contraction axis: 1 = along a row (D = cols), 0 = along a
 *              column (D = rows)
 *   had_block  requested Hadamard order
 *   op         width, rounding, clip, tensor_id (host pointer)
 *   seed       stochastic-rounding seed
 *   codes_out  packed codes, contraction-major: `lines` x D with the
 *              contraction index contiguous (lines = rows for axis 1, cols for
 *              axis 0, i.e. axis 0 writes the transpose).  b <= 4: byte j of a
 *              line holds code 2j in bits 0-3 and code 2j+1 in bits 4-7
 *              (two's complement nibbles), pitch ceil(D/2), zero pad nibble if
 *              D is odd; b > 4: one int8 per code, pitch D.  (device)
 *   scale_out  one float: the value of a code step, clip*max|y| / 2^(b-1)
 *              (0 for an all-zero tensor).  (device)
 * Stochastic rounding of element e (row-major index in T): floor(v) + [u < frac(v) 2^16]
 * with u the 16-bit half-word (e mod 2) of word ((e/2) mod 4) of the
 * Philox4x32-10 block with counter (e/8 low, e/8 high, tensor_id, 0) and key
 * (seed low, seed high).
 */
int hdqt_quantize(const float *T, int64_t rows, int64_t cols, int axis, int had_block,
                  const hdqt_operand_t *op, uint64_t seed, void *codes_out, float *scale_out,
                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same quantization along BOTH axes of one tensor, from one read of it per
 * pass.  A training step needs every activation and gradient tensor in two
 * Hadamard domains (X along K for the forward product and along M for the weight
 * gradient; G along N for the input gradient and along M for the weight
 * gradient); the passes over the source are what costs.  The outputs are
 * bit-identical to two hdqt_quantize calls with axis 1 and axis 0:
 *   codes_axis1 [rows, pitch(cols)], scale_axis1   contraction along a row
 *   codes_axis0 [cols, pitch(rows)], scale_axis0   contraction along a column
 * Workspace: hdqt_quantize_dual_workspace_size() bytes.  Shapes the fused
 * kernels do not cover (rows or cols not a multiple of 64, block order above
 * 64, codes wider than 4 bits) run as two single-axis quantizations.
 */
size_t hdqt_quantize_dual_workspace_size(void);
int hdqt_quantize_dual(const float *T, int64_t rows, int64_t cols, int had_block,
                       const hdqt_operand_t *op_axis1, const hdqt_operand_t *op_axis0,
                       uint64_t seed, void *codes_axis1, float *scale_axis1, void *codes_axis0,
                       float *scale_axis0, void *workspace, size_t workspace_bytes, void *stream);

/*
 * A convolution's input as the source of the matmuls (Experiments: the convolutions of
 * the paper's networks run as matmuls on the unfolded activation).  The activation
 * act[batch, channels, height, width] (fp32, row-major, device) stands for its im2col
 * matrix X[M, K], M = batch*height*width, K = channels*kh*kw: row (b, y, x), column
 * c*kh*kw + ty*kw + tx holds act[b, c, y + ty - (kh-1)/2, x + tx - (kw-1)/2], zero outside
 * the image (stride 1, output of the input's size).  The kernels read the activation,
 * kh*kw times smaller than X, and never need X in memory.
 * Taken: kh, kw odd (<= 15); width a power of two <= 64 with height*width a multiple of
 * 64, or width a multiple of 64; and what the two-axis kernels need of X (M and K
 * multiples of 64, block orders <= 64, both axes' codes of at most 4 bits or both of 5 to
 * 8).  Anything else:
 * HDQT_EINVAL_GEOMETRY, and the caller unfolds the activation itself.
 */
typedef struct {
    int64_t batch;
    int32_t channels, height, width;
    int32_t kh, kw;
} hdqt_conv_t;

/* hdqt_quantize_dual on the im2col matrix of `act`; outputs, workspace and errors as there. */
int hdqt_quantize_dual_im2col(const float *act, const hdqt_conv_t *geo, int had_block,
                              const hdqt_operand_t *op_axis1, const hdqt_operand_t *op_axis0,
                              uint64_t seed, void *codes_axis1, float *scale_axis1,
                              void *codes_axis0, float *scale_axis0, void *workspace,
                              size_t workspace_bytes, void *stream);

/*
 * The im2col matrix itself, for the layers the activation-source entry points refuse
 * (strides, K off a multiple of 64, tiny images): X[(b, yo, xo), c*kh*kw + ty*kw + tx] =
 * act[b, c, yo*stride + ty - pad_h, xo*stride + tx - pad_w], zero outside the image;
 * X is [batch*Ho*Wo, channels*kh*kw] with Ho = (height + 2*pad_h - kh)/stride + 1 and Wo
 * alike (fp32, device, 16-byte aligned).  Pure data movement, one launch.
 */
int hdqt_im2col(const float *act, int64_t batch, int channels, int height, int width, int kh,
                int kw, int stride, int pad_h, int pad_w, float *X, void *stream);

/*
 * Tiled integer matmul on packed codes (Methodology: tiles of size s, low-bit
 * accumulators) followed by dequantization:
 *   acc[i,j] = sum_t sat_a( sum_{d in tile t} qA[i,d] qB[j,d] )
 *   out[i,j] = (float)acc[i,j] * (scaleA * scaleB) * (1/n_eff)
 *   qA [RA, D], qB [RB, D]  packed codes as written by hdqt_quantize (device)
 *   bA, bB                  their code widths
 *   scaleA, scaleB          device pointers to one float each
 *   out     fp32 [RA, RB] (device, may be NULL if acc_out is given)
 *   acc_out int32 [RA, RB] (device, may be NULL)
 *   workspace: hdqt_gemm_codes_workspace_size(RA, RB, D, s) bytes of device memory
 *   (0 for most shapes, then NULL is fine).  Few output tiles with a long
 *   contraction are split over workgroups along the contraction; every part
 *   writes its totals (sums of whole clamped tiles, so the result is the same)
 *   to a slice of the workspace and a second pass adds the slices.
 */
size_t hdqt_gemm_codes_workspace_size(int64_t RA, int64_t RB, int64_t D, int64_t s);
int hdqt_gemm_codes(const void *qA, const void *qB, int bA, int bB, const float *scaleA,
                    const float *scaleB, int64_t RA, int64_t RB, int64_t D, int n_eff,
                    int acc_bits, int64_t s, float *out, int32_t *acc_out, void *workspace,
                    size_t workspace_bytes, void *stream);

/*
 * The same matmul with a narrow output (not a step of the paper, whose layers hand
 * fp32 on; it halves what the input gradient of a wide layer writes, which is the one
 * thing that bounds that matmul): out[i,j] is the fp32 value above rounded to
 * bfloat16 (nearest, ties to even) and stored as its 16-bit pattern.
 *   out     bfloat16 [RA, RB] (device, 16-byte aligned, may be NULL if acc_out is given)
 * Everything else, the workspace included, as for hdqt_gemm_codes.
 */
int hdqt_gemm_codes_bf16(const void *qA, const void *qB, int bA, int bB, const float *scaleA,
                         const float *scaleB, int64_t RA, int64_t RB, int64_t D, int n_eff,
                         int acc_bits, int64_t s, uint16_t *out, int32_t *acc_out,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * The second reading of "tiled quantization" (Methodology: tiles of size s reduce
 * the partial sums an a-bit accumulator has to hold): instead of a saturating
 * register, every tile's partial-sum tensor goes through the paper's quantizer Q
 * with a bits and its own max calibration, and the tile results are added:
 *   P_t[i,j] = sum_{d in tile t} qA[i,d] qB[j,d]           m_t = max_{i,j} |P_t[i,j]|
 *   c_t[i,j] = clamp(RNE(fl(float(P_t[i,j]) * fl(2^(a-1) / m_t))), -2^(a-1), 2^(a-1)-1)
 *   acc[i,j] = sum_t c_t[i,j] * m_t     (exact)      out = (float)acc * 2^-(a-1) * scaleA*scaleB / n_eff
 * Arguments as for hdqt_gemm_codes; acc_bits 2..24; acc_out (nullable) receives acc.
 * HDQT_EINVAL_TILE if a tile sum may not be exact in binary32 (s * 2^(bA+bB-2) >= 2^24),
 * HDQT_EINVAL_ACC if acc may leave int32.
 * Packed 4-bit codes on both sides, D a multiple of 8, s of 32, acc_bits <= 16 (and at most
 * 512 tiles per part of a split contraction): two passes through the matrix-core kernel,
 * the first keeping only the maxima m_t, the second quantizing every tile sum as it is
 * produced; no tile sum is stored, and the workspace holds the maxima and, for a split
 * contraction, one int32 slice of the output per part.  Everything else: an emulation that
 * materialises all tile sums (ceil(D/s) * RA*RB*4 bytes plus the maxima).
 * hdqt_gemm_codes_requant_workspace_size is the latter, an upper bound for every operand
 * width; hdqt_gemm_codes_requant_workspace_size_for is what the call with these widths
 * needs (0 for arguments the call would reject), and the call accepts either.
 * hdqt_gemm_requant is the same for one of the three matmuls of a step, from the fp32
 * tensors (P, Q = X, W / G, W / X, G for the three kinds).
 */
size_t hdqt_gemm_codes_requant_workspace_size(int64_t RA, int64_t RB, int64_t D, int64_t s);
size_t hdqt_gemm_codes_requant_workspace_size_for(int64_t RA, int64_t RB, int64_t D, int64_t s,
                                                  int bA, int bB, int acc_bits);
int hdqt_gemm_codes_requant(const void *qA, const void *qB, int bA, int bB, const float *scaleA,
                            const float *scaleB, int64_t RA, int64_t RB, int64_t D, int n_eff,
                            int acc_bits, int64_t s, float *out, int32_t *acc_out,
                            void *workspace, size_t workspace_bytes, void *stream);
size_t hdqt_gemm_requant_workspace_size(int gemm_kind, int64_t M, int64_t K, int64_t N,
                                        const hdqt_params_t *params);
int hdqt_gemm_requant(int gemm_kind, const float *P, const float *Q, float *out, int64_t M,
                      int64_t K, int64_t N, const hdqt_params_t *params, int32_t *acc_out,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * The three matmuls of a training step (Methodology, problem statement Z = X W "needed
 * in the forward and the backward pass": forward Z = X W, input gradient dX = G W^T,
 * weight gradient dW = X^T G; each with both operands in the Hadamard domain of its
 * contraction dimension, quantized by Q, multiplied in tiles of size s with a-bit
 * accumulators -- Experiments: 4-bit inputs, 8-bit accumulators, tile 32).  X, W, G, the
 * outputs: fp32 device tensors with the shapes at the top of this file.  `acc_out` (nullable)
 * receives the int32 accumulators of the output's shape.  `params` is a host
 * pointer.  Workspace: hdqt_workspace_size(kind, ...) bytes.
 */
int hdqt_gemm_fwd(const float *X, const float *W, float *Z, int64_t M, int64_t K, int64_t N,
                  const hdqt_params_t *params, int32_t *acc_out, void *workspace,
                  size_t workspace_bytes, void *stream);
int hdqt_gemm_bwd_input(const float *G, const float *W, float *dX, int64_t M, int64_t K,
                        int64_t N, const hdqt_params_t *params, int32_t *acc_out,
                        void *workspace, size_t workspace_bytes, void *stream);
int hdqt_gemm_bwd_weight(const float *X, const float *G, float *dW, int64_t M, int64_t K,
                         int64_t N, const hdqt_params_t *params, int32_t *acc_out,
                         void *workspace, size_t workspace_bytes, void *stream);
/* hdqt_gemm_bwd_input with dX narrowed to bfloat16 (see hdqt_gemm_codes_bf16); same
 * workspace, same errors. */
int hdqt_gemm_bwd_input_bf16(const float *G, const float *W, uint16_t *dX, int64_t M, int64_t K,
                             int64_t N, const hdqt_params_t *params, int32_t *acc_out,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * hdqt_gemm_fwd for callers that cannot allocate and have no workspace to hand over: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments without the workspace, same results bit for bit.  The calibration records and
 * the codes of both operands live in a fixed device array inside the library
 * (hdqt_gemm_fwd_static_max_bytes() = 8 MiB per GPU the library has run on, held until the
 * process ends); the call allocates nothing, on the host or the device (as long as the
 * optional profiling is off).
 *   HDQT_ESCRATCH   hdqt_workspace_size(HDQT_GEMM_FWD, M, K, N, params) exceeds the array
 *                   (nothing is launched); other errors as for hdqt_gemm_fwd
 * All calls on one GPU share that GPU's array: two calls whose work overlaps in time on the
 * same GPU (different streams or threads) race.  Calls on one stream, one after the other,
 * are fine: every call clears and rewrites what it reads.
 */
size_t hdqt_gemm_fwd_static_max_bytes(void);
int hdqt_gemm_fwd_static(const float *X, const float *W, float *Z, int64_t M, int64_t K, int64_t N,
                         const hdqt_params_t *params, int32_t *acc_out, void *stream);

/*
 * All three matmuls of one layer's training step in one call (Methodology: every
 * matmul of the forward and the backward pass is quantized in its own Hadamard
 * domain):
 *   Z  = hdqt_gemm_fwd(X, W; *fwd)
 *   dX = hdqt_gemm_bwd_input(G, W; *bwd_input)      skipped when dX is NULL
 *   dW = hdqt_gemm_bwd_weight(X, G; *bwd_weight)
 * with results bit-identical to those three calls.  What the call saves is memory
 * traffic: X and G are each needed along both of their axes, and here each is
 * read once per quantization pass for both (see hdqt_quantize_dual), so the
 * step reads X and G four times in total instead of eight.
 * X, W, G, Z, dX, dW: fp32 device tensors; the three params are host pointers
 * (bwd_input may be NULL when dX is); the operands' tensor_ids and the seeds
 * are taken from the params of the matmul each quantization belongs to.
 * Workspace: hdqt_layer_step_workspace_size(...) bytes (0 = invalid arguments),
 * device memory, 16-byte aligned, contents undefined on entry and on return.
 */
size_t hdqt_layer_step_workspace_size(int64_t M, int64_t K, int64_t N, const hdqt_params_t *fwd,
                                      const hdqt_params_t *bwd_input,
                                      const hdqt_params_t *bwd_weight);
int hdqt_layer_step(const float *X, const float *W, const float *G, float *Z, float *dX,
                    float *dW, int64_t M, int64_t K, int64_t N, const hdqt_params_t *fwd,
                    const hdqt_params_t *bwd_input, const hdqt_params_t *bwd_weight,
                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * hdqt_layer_step for a convolution layer: X is given as the activation (see hdqt_conv_t),
 * M and K follow from `geo`.  Z [M, N], dXcol [M, K] (the gradient of the im2col matrix:
 * folding it back onto the activation is the caller's) and dW [K, N] as for
 * hdqt_layer_step, bit for bit what that call returns on the unfolded activation.
 * dXcol and bwd_input are required.  Workspace: hdqt_conv_step_workspace_size(...) bytes,
 * 0 if the geometry is not taken (then hdqt_conv_step returns HDQT_EINVAL_GEOMETRY).
 */
size_t hdqt_conv_step_workspace_size(const hdqt_conv_t *geo, int64_t N, const hdqt_params_t *fwd,
                                     const hdqt_params_t *bwd_input,
                                     const hdqt_params_t *bwd_weight);
int hdqt_conv_step(const float *act, const hdqt_conv_t *geo, const float *W, const float *G,
                   float *Z, float *dXcol, float *dW, int64_t N, const hdqt_params_t *fwd,
                   const hdqt_params_t *bwd_input, const hdqt_params_t *bwd_weight,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * hdqt_layer_fwd for a convolution layer: Z and the saved codes of X along M from the
 * activation (see hdqt_conv_t); M = batch*height*width and K = channels*kh*kw follow from
 * `geo`.  bwd_weight and saved are required (both code sets come from the same kernels);
 * sizes from hdqt_layer_saved_size(M, K, ...) and hdqt_layer_fwd_workspace_size(M, K, N, ...).
 * hdqt_layer_bwd then runs as for any layer (its dX is the gradient of the im2col matrix).
 * HDQT_EINVAL_GEOMETRY if the geometry is not taken.
 */
int hdqt_conv_fwd(const float *act, const hdqt_conv_t *geo, const float *W, float *Z, int64_t N,
                  const hdqt_params_t *fwd, const hdqt_params_t *bwd_weight, void *saved,
                  size_t saved_bytes, void *workspace, size_t workspace_bytes, void *stream);

/*
 * hdqt_layer_bwd for a convolution layer, with the input gradient folded back onto the
 * activation inside the matmul: dAct[batch, channels, height, width] (fp32, device) instead
 * of the [M, K] gradient of the im2col matrix, which is never written.
 *   dAct[b,c,y,x] = float( sum over the window's taps (ty,tx) whose source pixel
 *                   (y - ty + (kh-1)/2, x - tx + (kw-1)/2) lies in the image of
 *                   acc[(b, that pixel), c*kh*kw + ty*kw + tx] ) * scaleG * scaleW / n_eff
 * with acc the integer accumulators of dX = G W^T: the taps are added as integers (exact,
 * order-free) and dequantized once.  dW as for hdqt_layer_bwd.  dAct, bwd_input and W are
 * required.  Workspace: hdqt_layer_bwd_workspace_size(M, K, N, ...) with M = batch*height*width,
 * K = channels*kh*kw.
 * Taken: 4-bit codes, s and N multiples of 32, ceil(N/s) * min(2^(acc_bits-1), 64 s) <= 32767
 * (the folded tile is kept as 16-bit integers); kh, kw odd; width a power
 * of two <= 128; height*width a power of two <= 128, or height*width = 256 with N <= 128
 * and a window of at most nine taps (a workgroup multiplies both halves of an image), or
 * 128/width >= kh image rows per strip.  Anything else: HDQT_EINVAL_GEOMETRY (before anything is launched), and the caller
 * takes hdqt_layer_bwd and folds its dX.
 */
int hdqt_conv_bwd(const float *G, const float *W, const void *saved, const hdqt_conv_t *geo,
                  float *dAct, float *dW, int64_t N, const hdqt_params_t *bwd_input,
                  const hdqt_params_t *bwd_weight, void *workspace, size_t workspace_bytes,
                  void *stream);

/*
 * The input gradient behind a rectifier (not a step of the paper, whose layers hand dX on; a
 * framework applies this as a pass of its own over dX).  When the layer's input is
 * x = max(pre, 0), the gradient of `pre` is dX where x > 0 and zero elsewhere; these variants
 * write that instead of dX, from inside the matmul's epilogue where the kernel has one
 * (otherwise in the pass that finishes a split contraction, or in one more pass):
 *     out[p] = x_mask[p] > 0 ? dX[p] : +0
 *   x_mask    fp32, the shape of the output it masks (device, 16-byte aligned): the layer's
 *             input X [M, K] for hdqt_gemm_bwd_input_masked and hdqt_layer_bwd_masked, the
 *             activation [batch, C, H, W] for hdqt_conv_bwd_masked (its folded gradient is
 *             what is masked)
 * Everything else -- the other arguments, the workspace, the errors, dW -- as for
 * hdqt_gemm_bwd_input, hdqt_layer_bwd and hdqt_conv_bwd; dX / dAct is required; acc_out
 * (hdqt_gemm_bwd_input_masked) receives the accumulators unmasked.
 */
int hdqt_gemm_bwd_input_masked(const float *G, const float *W, const float *x_mask, float *dX, int64_t M,
                               int64_t K, int64_t N, const hdqt_params_t *params, int32_t *acc_out,
                               void *workspace, size_t workspace_bytes, void *stream);
int hdqt_layer_bwd_masked(const float *G, const float *W, const void *saved, const float *x_mask,
                          float *dX, float *dW, int64_t M, int64_t K, int64_t N,
                          const hdqt_params_t *bwd_input, const hdqt_params_t *bwd_weight,
                          void *workspace, size_t workspace_bytes, void *stream);
int hdqt_conv_bwd_masked(const float *G, const float *W, const void *saved, const hdqt_conv_t *geo,
                         const float *act_mask, float *dAct, float *dW, int64_t N,
                         const hdqt_params_t *bwd_input, const hdqt_params_t *bwd_weight,
                         void *workspace, size_t workspace_bytes, void *stream);

/* The folded input gradient alone, on packed codes: qG [M, N] codes of G along N, qW [K, N]
 * codes of W along N (as hdqt_quantize writes them), their scales (device), the contraction
 * length N and its block order n_eff; dAct as for hdqt_conv_bwd.  No workspace. */
int hdqt_gemm_codes_fold(const void *qG, const void *qW, int bG, int bW, const float *scaleG,
                         const float *scaleW, const hdqt_conv_t *geo, int64_t N, int n_eff,
                         int acc_bits, int64_t s, float *dAct, void *stream);

/*
 * The same step as two calls, for training loops in which the gradient G arrives
 * long after the forward product (Methodology: the forward and the backward
 * matmuls of a layer):
 *   hdqt_layer_fwd  Z = hdqt_gemm_fwd(X, W; *fwd); when bwd_weight is not NULL, X is
 *                   also quantized along M with bwd_weight->A / had_block / seed,
 *                   from the same reads, and those codes and their scale are left
 *                   in `saved`: the activation is kept for the backward pass as b-bit
 *                   codes (hdqt_layer_saved_size bytes, 1/8 of fp32 X at b = 4)
 *                   instead of X itself.
 *   hdqt_layer_bwd  dW = hdqt_gemm_bwd_weight(X, G; *bwd_weight) with X taken from
 *                   `saved`, and, when dX is not NULL, dX = hdqt_gemm_bwd_input(G, W;
 *                   *bwd_input); G is read once per pass for both.
 * Results are bit-identical to the hdqt_gemm_* calls.  bwd_weight must be the same
 * in both calls.  saved: device memory, 16-byte aligned, written by hdqt_layer_fwd,
 * read by hdqt_layer_bwd, owned by the caller in between; its layout (a 256-byte
 * header holding the scale, then packed codes [K, pitch(M)]) is private to the
 * library.  Workspaces as for the other entry points (the *_workspace_size
 * functions return 0 for invalid arguments); params are host pointers.
 */
size_t hdqt_layer_saved_size(int64_t M, int64_t K, const hdqt_params_t *bwd_weight);
size_t hdqt_layer_fwd_workspace_size(int64_t M, int64_t K, int64_t N, const hdqt_params_t *fwd,
                                     const hdqt_params_t *bwd_weight);
int hdqt_layer_fwd(const float *X, const float *W, float *Z, int64_t M, int64_t K, int64_t N,
                   const hdqt_params_t *fwd, const hdqt_params_t *bwd_weight, void *saved,
                   size_t saved_bytes, void *workspace, size_t workspace_bytes, void *stream);
size_t hdqt_layer_bwd_workspace_size(int64_t M, int64_t K, int64_t N,
                                     const hdqt_params_t *bwd_input,
                                     const hdqt_params_t *bwd_weight);
int hdqt_layer_bwd(const float *G, const float *W, const void *saved, float *dX, float *dW,
                   int64_t M, int64_t K, int64_t N, const hdqt_params_t *bwd_input,
                   const hdqt_params_t *bwd_weight, void *workspace, size_t workspace_bytes,
                   void *stream);

/*
 * Optional per-kernel timing, for benchmarks.  While enabled, every kernel the
 * library launches is bracketed by two HIP events on its stream (this is the
 * only state the library keeps, and events are the only thing it creates).
 * hdqt_profile_collect waits for all recorded events, writes one row per
 * kernel that ran (name, number of launches, summed elapsed milliseconds) into
 * rows[0 .. max_rows) (host memory), clears the record and returns the number
 * of kernels that ran.  Not for use under graph capture.  The switch and the record are
 * process-wide: while it is on, launches from every thread and stream are recorded, and
 * one collect returns them all (thread-safe, but two threads' launches are not kept apart).
 */
typedef struct {
    char name[48];
    int64_t launches;
    double total_ms;
} hdqt_kernel_time_t;
int hdqt_profile_enable(int on);
int hdqt_profile_collect(hdqt_kernel_time_t *rows, int max_rows);

/*
 * Measurement aid for benchmarks (no step of the paper): the rate of the int8 matrix pipe and
 * the shader clock under that load, which on this chip depends on the operands' switching
 * activity.  256 * waves_per_simd workgroups of 4 waves (waves_per_simd in 1..4: that many
 * waves share every SIMD of the chip's 256 CUs) loop `iters` times over 16 independent
 * v_mfma_i32_32x32x32_i8 on the operand fragments in `fragments` (8 KiB, device: eight
 * fragments of 64 lanes x 16 int8), registers only.
 *   result   two int64 (device, 8-byte aligned): shader-clock cycles and wall-clock ticks
 *            (hipDeviceAttributeWallClockRate) that one wave spent in its loop, i.e. on
 *            16 * iters MFMAs (the launch's duration, timed by the caller, gives the rate)
 *   scratch  1 MiB of device memory the kernel may overwrite
 * HDQT_EINVAL_DIM for iters outside [1, 2^20] or waves_per_simd outside [1, 4].
 */
int hdqt_wall_clock_khz(void);      /* rate of those ticks on the current device, 0 if unknown (host) */
int hdqt_probe_matrix_clock(const void *fragments, int iters, int waves_per_simd, long long *result,
                            void *scratch, size_t scratch_bytes, void *stream);

/* Text for an error code (static string, host). */
const char *hdqt_strerror(int code);
/* HIP error code of the last HDQT_EHIP on this thread (0 if none). */
int hdqt_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* HDQT_H */
