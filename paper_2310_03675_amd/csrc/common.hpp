// Shared declarations of the HDQT device library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hdqt {

constexpr int kMaxHadamard = 256;   // largest supported block order
constexpr int kWave = 64;

// Per-operand calibration record in the workspace.  max|y| is reduced with
// integer atomicMax on the bit patterns (non-negative floats order like unsigned
// integers).  Atomics on one address are serialised, so the workgroups spread
// over 64 slots, each on its own 128-byte line; pass 2 reads one slot per lane
// and finishes the reduction inside the wave.  `scale` is the value of one
// code step, written by pass 2.
constexpr int kAmaxSlots = 64;
constexpr int kAmaxSlotStride = 32;     // dwords
struct QMeta {
    float scale;
    uint32_t pad[31];
    uint32_t amax[kAmaxSlots * kAmaxSlotStride];
};
constexpr int64_t kQMetaDwords = sizeof(QMeta) / 4;

// One quantize request, resolved by the host.
struct QuantArgs {
    const float* T;
    int64_t rows, cols;     // source tensor, row-major
    int axis;               // 1: contraction along a row, 0: along a column
    int log2n;              // log2 of the block order actually used
    int b;                  // code width
    int stochastic;         // 0 nearest-even, 1 stochastic
    float clip;
    uint32_t tensor_id;
    uint32_t seed_lo, seed_hi;
    QMeta* meta;            // device
    uint8_t* codes;         // device, packed, contraction-major
    float* scale_out;       // device, may alias &meta->scale, may be null
};

// One tensor quantized along both axes from one read ("row" = axis 1, along the
// columns; "col" = axis 0, along the rows).
struct DualArgs {
    const float* T;
    int64_t rows, cols;
    int log2n_row, log2n_col;
    int b_row, st_row;
    float clip_row;
    uint32_t tid_row;
    int b_col, st_col;
    float clip_col;
    uint32_t tid_col;
    uint32_t seed_row_lo, seed_row_hi;   // Philox key per axis
    uint32_t seed_col_lo, seed_col_hi;
    QMeta* meta_row;
    QMeta* meta_col;
    uint8_t* codes_row;     // [rows, cols/2]
    uint8_t* codes_col;     // [cols, rows/2]
    float* scale_row_out;   // may be null
    float* scale_col_out;
    int profile_tag;        // which tensor of the step this is (timing table only): 0 none, 1 X, 2 W, 3 G
    // Convolution source (conv != 0): T points at an activation [batch, C, H, W] and the
    // tensor that is quantized is its im2col matrix for a kh x kw window, stride 1, zero
    // padding (kh - 1) / 2 and (kw - 1) / 2: row = pixel (b, y, x), column c*kh*kw + ty*kw + tx
    // holds act[b, c, y + ty - ph, x + tx - pw].  rows = batch*H*W, cols = C*kh*kw.
    int conv;
    int cC, cH, cW, ckh, ckw;
    int pPH, pPW, pCN;      // the part of the activation a 64 x 64 tile reads: rows, row length, channels
};

struct GemmArgs {
    const uint8_t* qA;      // [RA, pitchA] packed codes
    const uint8_t* qB;      // [RB, pitchB]
    int64_t pitchA, pitchB;
    int bA, bB;
    int64_t RA, RB, D;
    int64_t s;              // tile length in codes
    int s_pad;              // tile length rounded up to the MFMA K granularity
    int64_t n_tiles;        // ceil(D / s)
    int acc_lo, acc_hi;     // accumulator range [-2^(a-1), 2^(a-1)-1]
    int acc_lo_scaled, acc_hi_scaled;   // the same bounds times 256 (set by the 4-bit fast path)
    int jA, jB, fin_shift;              // 16-bit saturation path: operand factors 2^jA, 2^jB; 16 - acc_bits
    const float* scaleA;    // device scalars
    const float* scaleB;
    float inv_n;            // 1 / n_eff (a power of two)
    float* out;             // [RA, RB] or null
    uint16_t* out_bf16;     // [RA, RB] bfloat16 patterns or null: the same values, narrowed (nearest even)
    const float* mask_src;  // null, or a tensor of the fp32 output's shape: the output is written
                            // where mask_src > 0 and +0 elsewhere (the rectifier's backward pass
                            // behind an input gradient); the integer outputs are not masked
    int32_t* acc_out;       // [RA, RB] or null
    int partial16;          // the slices hold 16-bit integers (a part's totals fit: parts of few tiles)
    int32_t* partial;       // [splits, RA, RB] when splits > 1: one slice per part of the contraction;
                            // second reading of the accumulator: [n_tiles, RA, RB], every tile's sums
    uint32_t* tile_max;     // second reading only: max |tile sum| per tile, zero beforehand
    int req_bits;           // second reading in the matrix-core kernel: a, and the clamp bounds
    float req_lo, req_hi;   // -2^(a-1) and 2^(a-1) - 1, each plus 1.5 * 2^23
    int stream_out;         // fp32 output too large to stay cached: written with streaming stores
    int profile_tag;        // which matmul of the step this is (timing table only): 0 none, 1 + kind
    int splits;             // workgroups sharing one output tile along the contraction
    int64_t tiles_per_split;
    // Fold (fold != 0): the product is the gradient of an im2col matrix, qA holds the codes of
    // G [batch*H*W pixels, D], qB those of W [C*kh*kw, D], and what is written is the gradient
    // of the activation, out[batch, C, H, W]: the accumulators of a pixel's kh*kw taps are
    // added up inside the workgroup (exact integers) and dequantized once.
    int fold;
    int fC, fH, fW, fkh, fkw;
    int64_t fbatch;
    int f_log2w, f_log2hw;  // W and (image mode) H*W are powers of two
    int f_imgs;             // images per 128-pixel row tile (H*W <= 128), else 0: strips of one image
    int f_rows_c;           // strip mode: image rows a row tile computes (128 / W), kh - 1 of them halo
    int f_rows_out;         // strip mode: image rows a row tile writes
    int f_strips;           // strip mode: row tiles per image
    int f_cg;               // channels per column tile: 128 / (kh*kw)
    int f_pair;             // images of 256 pixels, one stage per tile: a workgroup computes both
                            // 128-pixel halves of an image (grid.y = images) and folds them together
};
// fills the fold fields from the geometry; false if the fast kernel does not take it
bool gemm_fold_plan(GemmArgs* g, int64_t batch, int C, int H, int W, int kh, int kw);

// Unfolding of an activation [batch, C, H, W] into X [M = batch*Ho*Wo, K = C*kh*kw] (im2col.hip)
struct Im2colArgs {
    const float* act;
    float* X;
    int64_t M;
    int C, H, W, kh, kw, stride, ph, pw, Ho, Wo;
};
hipError_t launch_im2col(const Im2colArgs& a, hipStream_t stream);

// Launchers (host).  Each returns the hipError_t of its last launch.
hipError_t launch_quantize(const QuantArgs& q, hipStream_t stream);
hipError_t launch_gemm(const GemmArgs& g, hipStream_t stream);
// Second reading of the low-bit accumulator: every tile's partial sums to g.partial and their
// maxima to g.tile_max, then Q with acc_bits per tile and the sum over tiles (see gemm.hip).
hipError_t launch_gemm_requant(const GemmArgs& g, int acc_bits, hipStream_t stream);
// The same result without storing a tile sum, for the shapes the matrix-core kernel takes
// (gemm_requant_fast_eligible): pass 1 multiplies and keeps only g.tile_max, pass 2 multiplies
// again and quantizes every tile sum with its tile's maximum as it leaves the matrix core.
// With a split contraction pass 2 writes its parts' totals to g.partial ([splits, RA, RB]),
// which launch_reduce then adds; g.inv_n carries the factor 2^-(a-1) in that case and here.
bool gemm_requant_fast_eligible(const GemmArgs& g, int acc_bits);
hipError_t launch_gemm_requant_fast(const GemmArgs& g, int acc_bits, int pass, hipStream_t stream);
constexpr int kMaxDualBatch = 3;
// the two passes of the two-axis quantization, each for up to kMaxDualBatch tensors in one launch
hipError_t launch_dual_pass1(const DualArgs* qs, int n, hipStream_t stream);
hipError_t launch_dual_pass2(const DualArgs* qs, int n, hipStream_t stream);
bool dual_pass2_batchable(const DualArgs* qs, int n);
// fills the patch extents of a convolution source; false if the kernels do not take the geometry
bool dual_conv_plan(DualArgs* q);
// zero a[0, na) and b[0, nb) (b may be null) in one launch
hipError_t launch_zero2(uint32_t* a, int64_t na, uint32_t* b, int64_t nb, hipStream_t stream);
// sum the `splits` slices of `partial` ([splits, count]); the totals go to acc_out
// (nullable) and, dequantized, to out (nullable)
// out_bf16 (nullable): the dequantized totals narrowed to bfloat16
hipError_t launch_reduce(const int32_t* partial, int splits, int64_t count, const float* scaleA,
                         const float* scaleB, float inv_n, float* out, uint16_t* out_bf16,
                         int32_t* acc_out, hipStream_t stream, const float* mask_src = nullptr,
                         bool slices16 = false);
bool reduce_takes_slices16(int splits, int64_t count);
// out[e] = mask_src[e] > 0 ? out[e] : +0 (for the matmul paths that do not mask in their epilogue)
hipError_t launch_relu_mask(float* out, const float* mask_src, int64_t count, hipStream_t stream);
// whether the matrix-core kernel applies g.mask_src in its own epilogue
bool gemm_fast_masks(const GemmArgs& g);

// Optional per-kernel timing (off by default).  When enabled through the C ABI,
// every launch is bracketed by two HIP events on its stream.
enum KernelId {
    K_FILL = 0, K_ROW_ABSMAX, K_ROW_QUANT, K_COL_ABSMAX, K_COL_QUANT, K_PLAIN_ABSMAX,
    K_PLAIN_QUANT, K_GEMM_ALIGNED, K_GEMM_GENERIC, K_REDUCE, K_GEMM_I4, K_DUAL_ABSMAX, K_DUAL_QUANT,
    K_GEMM_I4_FWD, K_GEMM_I4_BWD_INPUT, K_GEMM_I4_BWD_WEIGHT,
    K_DUAL_ABSMAX_X, K_DUAL_ABSMAX_W, K_DUAL_ABSMAX_G, K_DUAL_QUANT_X, K_DUAL_QUANT_W, K_DUAL_QUANT_G,
    K_DUAL_ABSMAX_BATCH, K_DUAL_QUANT_BATCH, K_REQUANT_TILES, K_REQUANT_SUM, K_IM2COL, K_RELU_MASK,
    K_COUNT
};
bool quantize_fast_eligible(const QuantArgs& q);
hipError_t launch_quantize_fast(const QuantArgs& q, hipStream_t stream);
bool quantize_dual_eligible(const DualArgs& q);
hipError_t launch_quantize_dual(const DualArgs& q, hipStream_t stream);
bool gemm_fast_eligible(const GemmArgs& g);
hipError_t launch_gemm_fast(const GemmArgs& g, hipStream_t stream);
const char* kernel_name(int id);
bool profiling_enabled();
void profile_begin(int id, hipStream_t stream);
void profile_end(int id, hipStream_t stream);
struct ProfileScope {
    int id; hipStream_t stream; bool on;
    ProfileScope(int i, hipStream_t s) : id(i), stream(s), on(profiling_enabled()) { if (on) profile_begin(id, stream); }
    ~ProfileScope() { if (on) profile_end(id, stream); }
};

// ---- device helpers -------------------------------------------------------

// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies
// and a Weyl key schedule.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1, uint32_t out[4])
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Random 16 bits of element e: half-word (e & 1) of word ((e >> 1) & 3) of `blk`.
__device__ __forceinline__ uint32_t sr_halfword(const uint32_t blk[4], uint32_t e_low3)
{
    const uint32_t w = blk[(e_low3 >> 1) & 3];
    return (w >> (16 * (e_low3 & 1))) & 0xFFFFu;
}

// alpha * 2^(b-1): one correctly rounded division.  A binary64 quotient of two
// binary32 values rounds to binary32 without double-rounding error (53 >= 2*24+2).
// binary32 -> bfloat16 pattern, nearest, ties to even (finite values; a carry out of the
// fraction moves to the next binade or to infinity, which is the correctly rounded result)
__device__ __forceinline__ uint32_t bf16_bits(float x)
{
    const uint32_t u = __float_as_uint(x);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ float inverse_step(float amax_clipped, int b)
{
    const double levels = (double)(1 << (b - 1));
    return (float)(levels / (double)amax_clipped);
}

// Rounding step of Q.  v = y * inv; nearest-even, or floor + Bernoulli(frac)
// with a 16-bit threshold; then the clamp to the b-bit range.
__device__ __forceinline__ int quantize_value(float y, float inv, int qmin, int qmax,
                                              bool stochastic, uint32_t u16)
{
    const float v = y * inv;
    float q;
    if (stochastic) {
        const float fl = floorf(v);
        const float frac = v - fl;
        q = fl + (((float)u16 < frac * 65536.0f) ? 1.0f : 0.0f);
    } else {
        q = rintf(v);
    }
    q = fminf(fmaxf(q, (float)qmin), (float)qmax);
    return (int)q;
}


// ---- calibration helpers --------------------------------------------------

__device__ __forceinline__ float wave_max_shfl(float m)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, kWave));
    return m;
}

// One atomicMax per workgroup (256 threads), into the workgroup's slot, and only
// if it can raise the slot.  `smem` holds one float per wave.
__device__ __forceinline__ void block_atomic_max(float m, QMeta* meta, float* smem)
{
    m = wave_max_shfl(m);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) smem[wave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        float r = smem[0];
        for (int w = 1; w < (int)(blockDim.x >> 6); ++w) r = fmaxf(r, smem[w]);
        const uint32_t slot = (blockIdx.x + blockIdx.y * gridDim.x) % kAmaxSlots;
        uint32_t* target = &meta->amax[slot * kAmaxSlotStride];
        const uint32_t bits = __float_as_uint(r);
        if (bits > __hip_atomic_load(target, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
            atomicMax(target, bits);
    }
}

struct Scaling {
    float inv;      // alpha * 2^(b-1); 0 for an all-zero tensor (every code is then 0)
    float scale;    // value of one code step
};

// Must be reached by whole waves: lane l reads slot l.
__device__ __forceinline__ Scaling load_scaling(const QMeta* meta, float clip, int b)
{
    const float slot = __uint_as_float(meta->amax[(threadIdx.x & 63) * kAmaxSlotStride]);
    const float amax = wave_max_shfl(slot);
    const float amax_c = clip * amax;
    Scaling s;
    const bool zero = (amax_c == 0.0f);
    s.inv = zero ? 0.0f : inverse_step(amax_c, b);
    s.scale = zero ? 0.0f : amax_c / (float)(1 << (b - 1));
    return s;
}

__device__ __forceinline__ void publish_scale(const QuantArgs& q, const Scaling& s)
{
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
        q.meta->scale = s.scale;
        if (q.scale_out) *q.scale_out = s.scale;
    }
}

} // namespace hdqt
