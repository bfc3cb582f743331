// C ABI of the HDQT library: argument validation, workspace planning and the
// sequence of launches of each entry point.  See include/hdqt.h for the
// contract of every function.

#include "../../include/hdqt.h"
#include "common.hpp"

#include <limits.h>
#include <mutex>

namespace {

thread_local int g_last_hip_error = 0;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
inline bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

int check_operand(const hdqt_operand_t* op)
{
    if (!op) return HDQT_EINVAL_NULL;
    if (op->b < 2 || op->b > 8) return HDQT_EINVAL_BITS;
    if (op->round != HDQT_ROUND_NEAREST && op->round != HDQT_ROUND_STOCHASTIC)
        return HDQT_EINVAL_ROUND;
    if (!(op->clip > 0.0f) || op->clip > 1.0f) return HDQT_EINVAL_CLIP;
    return HDQT_OK;
}

int check_hadamard(int had_block)
{
    if (!is_pow2(had_block) || had_block > hdqt::kMaxHadamard) return HDQT_EINVAL_HADAMARD;
    return HDQT_OK;
}

// Per dimension: the kernels put up to one workgroup per 64 rows on the y axis of the
// grid, which holds 65535.
constexpr int64_t kMaxDim = (int64_t)65535 * 64 + 1;
constexpr int64_t kMaxElems = (int64_t)1 << 40;      // per tensor

int check_dims2(int64_t rows, int64_t cols)
{
    if (rows <= 0 || cols <= 0 || rows >= kMaxDim || cols >= kMaxDim) return HDQT_EINVAL_DIM;
    if (rows > kMaxElems / cols) return HDQT_EINVAL_DIM;
    return HDQT_OK;
}

// Range checks of the integer matmul: one tile's exact sum and the sum of all
// (clamped) tiles must both fit in 32 bits.
int check_accumulation(int64_t D, int64_t s, int acc_bits, int bA, int bB)
{
    if (s < 1) return HDQT_EINVAL_TILE;
    if (acc_bits < 2 || acc_bits > 32) return HDQT_EINVAL_ACC;
    const int64_t s_eff = s < D ? s : D;
    const int64_t max_prod = ((int64_t)1 << (bA - 1)) * ((int64_t)1 << (bB - 1));
    if (s_eff > (((int64_t)1 << 31) - 1) / max_prod) return HDQT_EINVAL_TILE;
    const int64_t tile_max = s_eff * max_prod;
    const int64_t acc_max = (int64_t)1 << (acc_bits - 1);
    const int64_t per_tile = tile_max < acc_max ? tile_max : acc_max;
    const int64_t n_tiles = (D + s_eff - 1) / s_eff;
    if (n_tiles > (((int64_t)1 << 31) - 1) / per_tile) return HDQT_EINVAL_ACC;
    return HDQT_OK;
}

struct Orientation {
    int64_t RA, RB, D;
    int64_t a_rows, a_cols, b_rows, b_cols;
    int a_axis, b_axis;
};

int orient(int kind, int64_t M, int64_t K, int64_t N, Orientation* o)
{
    switch (kind) {
    case HDQT_GEMM_FWD:          // A = X[M,K] along K, B = W[K,N] along K
        *o = {M, N, K, M, K, K, N, 1, 0};
        return HDQT_OK;
    case HDQT_GEMM_BWD_INPUT:    // A = G[M,N] along N, B = W[K,N] along N
        *o = {M, K, N, M, N, K, N, 1, 1};
        return HDQT_OK;
    case HDQT_GEMM_BWD_WEIGHT:   // A = X[M,K] along M, B = G[M,N] along M
        *o = {K, N, M, M, K, M, N, 0, 0};
        return HDQT_OK;
    default:
        return HDQT_EINVAL_AXIS;
    }
}

int check_gemm(int kind, int64_t M, int64_t K, int64_t N, const hdqt_params_t* p, Orientation* o)
{
    if (!p) return HDQT_EINVAL_NULL;
    int rc = orient(kind, M, K, N, o);
    if (rc) return rc;
    if (M <= 0 || K <= 0 || N <= 0 || M >= kMaxDim || K >= kMaxDim || N >= kMaxDim)
        return HDQT_EINVAL_DIM;
    if ((rc = check_dims2(M, K)) || (rc = check_dims2(K, N)) || (rc = check_dims2(M, N))) return rc;
    if ((rc = check_hadamard(p->had_block))) return rc;
    if ((rc = check_operand(&p->A)) || (rc = check_operand(&p->B))) return rc;
    return check_accumulation(o->D, p->s, p->acc_bits, p->A.b, p->B.b);
}

int log2i(int v)
{
    int k = 0;
    while ((1 << k) < v) ++k;
    return k;
}

int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return HDQT_EHIP;
}

// Parts the contraction is split into when the output has too few tiles to fill the chip.
// The matmul kernels keep two workgroups per CU resident (512 on the chip); every part
// writes an int32 slice of the output that a second pass reads back.  The number of parts is
// the one a simple cost model likes best: the multiplication at the rate the kernels reach
// on a full chip (0.8 POP/s on whole 128 x 128 tiles), slowed down in proportion when
// fewer than 512 workgroups exist, plus one more launch and the slices written and read at
// the 8 TB/s that data of this size gets from the caches.  (A weight gradient with nine
// output tiles takes all the parts it can get; a forward product that already has one
// workgroup per CU takes none; a 2048 x 4608 x 512 product with 64 tiles takes eight.)
int choose_splits(int64_t RA, int64_t RB, int64_t D, int64_t n_tiles)
{
    const int64_t blocks = ((RA + 127) / 128) * ((RB + 127) / 128);
    if (blocks >= 512 || n_tiles < 8) return 1;
    int64_t most = 512 / blocks;
    if (most > n_tiles / 4) most = n_tiles / 4;
    if (most > 1024) most = 1024;
    const double ops = 2.0 * 128.0 * 128.0 * (double)blocks * (double)D;      // what the tiles cost, padding included
    const double slice_us = 8.0 * (double)RA * (double)RB / 8.0e6;            // one slice, written and read
    double best_t = 0.0;
    int best = 1;
    for (int64_t c = 1; c <= most; ++c) {
        const double fill = (double)(blocks * c) / 512.0;
        double t = ops / (0.8e9 * (fill < 1.0 ? fill : 1.0));
        if (c > 1) t += 4.0 + slice_us * (double)c;
        if (c == 1 || t < best_t) { best_t = t; best = (int)c; }
    }
    return best;
}

constexpr size_t kMetaBytes = (sizeof(hdqt::QMeta) + 255) / 256 * 256;

int run_quantize(const float* T, int64_t rows, int64_t cols, int axis, int n_eff,
                 const hdqt_operand_t* op, uint64_t seed, hdqt::QMeta* meta, void* codes,
                 float* scale_out, hipStream_t stream)
{
    hdqt::QuantArgs q{};
    q.T = T; q.rows = rows; q.cols = cols; q.axis = axis;
    q.log2n = log2i(n_eff);
    q.b = op->b; q.stochastic = (op->round == HDQT_ROUND_STOCHASTIC);
    q.clip = op->clip; q.tensor_id = op->tensor_id;
    q.seed_lo = (uint32_t)seed; q.seed_hi = (uint32_t)(seed >> 32);
    q.meta = meta; q.codes = static_cast<uint8_t*>(codes); q.scale_out = scale_out;
    const hipError_t e = hdqt::launch_quantize(q, stream);
    return e == hipSuccess ? HDQT_OK : hip_fail(e);
}

hdqt::DualArgs make_dual_args(const float* T, int64_t rows, int64_t cols, int n1,
                              const hdqt_operand_t* op1, uint64_t seed1, int n0,
                              const hdqt_operand_t* op0, uint64_t seed0, hdqt::QMeta* meta1,
                              hdqt::QMeta* meta0, void* codes1, void* codes0, float* scale1_out,
                              float* scale0_out, int profile_tag)
{
    hdqt::DualArgs d{};
    d.profile_tag = profile_tag;
    d.T = T; d.rows = rows; d.cols = cols;
    d.log2n_row = log2i(n1); d.log2n_col = log2i(n0);
    d.b_row = op1->b; d.st_row = (op1->round == HDQT_ROUND_STOCHASTIC);
    d.clip_row = op1->clip; d.tid_row = op1->tensor_id;
    d.b_col = op0->b; d.st_col = (op0->round == HDQT_ROUND_STOCHASTIC);
    d.clip_col = op0->clip; d.tid_col = op0->tensor_id;
    d.seed_row_lo = (uint32_t)seed1; d.seed_row_hi = (uint32_t)(seed1 >> 32);
    d.seed_col_lo = (uint32_t)seed0; d.seed_col_hi = (uint32_t)(seed0 >> 32);
    d.meta_row = meta1; d.meta_col = meta0;
    d.codes_row = static_cast<uint8_t*>(codes1); d.codes_col = static_cast<uint8_t*>(codes0);
    d.scale_row_out = scale1_out; d.scale_col_out = scale0_out;
    return d;
}

// rows and columns of the im2col matrix; false if the geometry is not a valid one
bool conv_matrix_shape(const hdqt_conv_t* geo, int64_t* M, int64_t* K)
{
    if (!geo || geo->batch < 1 || geo->channels < 1 || geo->height < 1 || geo->width < 1 || geo->kh < 1 ||
        geo->kw < 1)
        return false;
    const int64_t hw = (int64_t)geo->height * geo->width;
    if (geo->batch > kMaxDim / hw) return false;
    *M = geo->batch * hw;
    *K = (int64_t)geo->channels * geo->kh * geo->kw;
    return *M < kMaxDim && *K < kMaxDim;
}

// Make `d` read its tensor from the activation `geo` describes; false if the two-axis
// kernels do not take that geometry.
bool set_conv_source(hdqt::DualArgs* d, const hdqt_conv_t* geo)
{
    d->conv = 1;
    d->cC = geo->channels; d->cH = geo->height; d->cW = geo->width;
    d->ckh = geo->kh; d->ckw = geo->kw;
    return hdqt::dual_conv_plan(d);
}

// Both quantizations of one tensor (axis 1 and axis 0): from a single read per
// pass when the fused kernel takes the shape, else one after the other.  Both
// calibration records must be zero.
int run_quantize_pair(const float* T, int64_t rows, int64_t cols, int n1, const hdqt_operand_t* op1,
                      uint64_t seed1, int n0, const hdqt_operand_t* op0, uint64_t seed0,
                      hdqt::QMeta* meta1, hdqt::QMeta* meta0, void* codes1, void* codes0,
                      float* scale1_out, float* scale0_out, hipStream_t stream, int profile_tag = 0)
{
    const hdqt::DualArgs d = make_dual_args(T, rows, cols, n1, op1, seed1, n0, op0, seed0, meta1, meta0,
                                            codes1, codes0, scale1_out, scale0_out, profile_tag);
    if (hdqt::quantize_dual_eligible(d)) {
        const hipError_t e = hdqt::launch_quantize_dual(d, stream);
        return e == hipSuccess ? HDQT_OK : hip_fail(e);
    }
    const int rc = run_quantize(T, rows, cols, 1, n1, op1, seed1, meta1, codes1, scale1_out, stream);
    if (rc) return rc;
    return run_quantize(T, rows, cols, 0, n0, op0, seed0, meta0, codes0, scale0_out, stream);
}

// Resolve tile length, accumulator range and the split of the contraction.
hdqt::GemmArgs plan_gemm(const void* qA, const void* qB, int bA, int bB, const float* scaleA,
                         const float* scaleB, int64_t RA, int64_t RB, int64_t D, int n_eff,
                         int acc_bits, int64_t s, float* out, int32_t* acc_out, int profile_tag = 0,
                         uint16_t* out_bf16 = nullptr, bool keep_tiles = false)
{
    hdqt::GemmArgs g{};
    g.profile_tag = profile_tag;
    g.qA = static_cast<const uint8_t*>(qA); g.qB = static_cast<const uint8_t*>(qB);
    g.pitchA = hdqt_codes_pitch(D, bA); g.pitchB = hdqt_codes_pitch(D, bB);
    g.bA = bA; g.bB = bB; g.RA = RA; g.RB = RB; g.D = D;
    g.s = s < D ? s : D;
    g.acc_lo = acc_bits >= 32 ? INT_MIN : -(1 << (acc_bits - 1));
    g.acc_hi = acc_bits >= 32 ? INT_MAX : (1 << (acc_bits - 1)) - 1;
    if (!keep_tiles) {
        // Tiles that cannot saturate need not be kept apart: while m * s products of the
        // largest magnitude, 2^(bA-1) * 2^(bB-1) each, fit the accumulator, the clamp of a
        // group of m tiles changes nothing and the sum over the group is the sum of its
        // tiles' sums.  Groups of 256 or 128 codes are whole stages of the matrix-core kernel
        // (16-bit accumulators with 4-bit inputs, 32-bit ones with any inputs).
        const int64_t max_prod = ((int64_t)1 << (bA - 1)) * ((int64_t)1 << (bB - 1));
        for (int64_t grp = 256; grp >= 128; grp /= 2)
            if (g.s < grp && grp % g.s == 0 && grp <= D && grp * max_prod <= (int64_t)g.acc_hi) {
                g.s = grp;
                break;
            }
    }
    // The parts of a split contraction are chosen from the tiles as they stand here; parts
    // begin on a stage of the matrix-core kernel (128 codes) when the tile length divides
    // one: every 16-byte load of a part then lies inside one 64-byte run of its row
    // (measured on the benchmark layer's weight gradient: 37 -> 40 tiles per part, 35.7 ->
    // 33.1 us), and a tile of 16 codes never starts in the middle of a 32-code step.
    const int64_t plan_tiles = (D + g.s - 1) / g.s;
    g.splits = choose_splits(RA, RB, D, plan_tiles);
    int64_t part_tiles = (plan_tiles + g.splits - 1) / g.splits;
    if (g.splits > 1 && g.s < 128 && 128 % g.s == 0) {
        const int64_t q = 128 / g.s;
        part_tiles = (part_tiles + q - 1) / q * q;
    }
    const int64_t part_codes = part_tiles * g.s;
    if (!keep_tiles) {
        // Tiles that cannot saturate at all: every clamp is the identity and the result is the
        // plain integer product, so the tiles may as well be longer (the kernels clamp at tile
        // ends: 2048 codes are 16 stages of the matrix-core kernel between two clamps) and the
        // accumulator 32 bits wide -- as long as the product itself, times the factor 256 the
        // packed-code kernel carries, stays inside int32, and a part of a split contraction
        // stays a whole number of tiles (fewer, longer parts would leave compute units idle:
        // the weight gradient of the 65536 x 1152 x 128 layer with 8-bit codes and 32-bit
        // accumulators fell from 52 parts to 8).
        const int64_t max_prod = ((int64_t)1 << (bA - 1)) * ((int64_t)1 << (bB - 1));
        const int64_t room = (bA <= 4 && bB <= 4) ? ((int64_t)1 << 22) : ((int64_t)1 << 31);
        if (g.s % 128 == 0 && g.s * max_prod <= (int64_t)g.acc_hi && D * max_prod < room) {
            while (g.s * 2 <= 2048 && g.s * 2 <= D && (g.splits == 1 || part_codes % (g.s * 2) == 0))
                g.s *= 2;
            g.acc_lo = INT_MIN;
            g.acc_hi = INT_MAX;
        }
    }
    g.s_pad = (int)((g.s + 15) / 16 * 16);
    g.n_tiles = (D + g.s - 1) / g.s;
    g.scaleA = scaleA; g.scaleB = scaleB;
    g.inv_n = 1.0f / (float)n_eff;
    g.out = out; g.acc_out = acc_out; g.out_bf16 = out_bf16;
    // An output larger than half the 256 MB memory-side cache cannot stay there until
    // someone reads it; written normally it would sit there dirty and be written back
    // in the middle of the next kernel's reads (measured: the pass over X that follows
    // the input gradient of the 65536 x 1152 layer takes 90 us instead of 53 us).
    const int64_t out_elem = out ? (int64_t)sizeof(float) : (int64_t)sizeof(uint16_t);
    g.stream_out = (RA * RB * out_elem >= ((int64_t)128 << 20)) ? 1 : 0;
    g.tiles_per_split = g.splits > 1 ? part_codes / g.s : g.n_tiles;
    g.splits = (int)((g.n_tiles + g.tiles_per_split - 1) / g.tiles_per_split);
    return g;
}

// Bytes of workspace the matmul needs: with a split contraction every part writes
// its totals to a slice of its own ([splits, RA, RB] int32), summed by a second pass.
size_t partial_bytes(int64_t RA, int64_t RB, int64_t D, int64_t s)
{
    const int64_t s_eff = s < D ? s : D;
    int splits = choose_splits(RA, RB, D, (D + s_eff - 1) / s_eff);
    // plan_gemm may merge tiles into groups of 128 or 256 codes; whatever it decides fits
    for (int64_t grp = 128; grp <= 256; grp *= 2)
        if (s_eff < grp && grp % s_eff == 0 && grp <= D) {
            const int alt = choose_splits(RA, RB, D, (D + grp - 1) / grp);
            if (alt > splits) splits = alt;
        }
    return splits > 1 ? (size_t)splits * (size_t)(RA * RB) * sizeof(int32_t) : 0;
}

int run_planned_gemm(hdqt::GemmArgs g, void* ws, size_t ws_bytes, hipStream_t stream)
{
    hipError_t e;
    if (g.splits > 1) {
        if (!ws || ws_bytes < (size_t)g.splits * (size_t)(g.RA * g.RB) * sizeof(int32_t))
            return HDQT_EWORKSPACE;
        g.partial = static_cast<int32_t*>(ws);
        // A part of few tiles has totals of 16 bits: slices of half the bytes (the matrix-core
        // kernel's packed-code instances write them, the many-slices pass reads them).
        const int64_t max_prod = ((int64_t)1 << (g.bA - 1)) * ((int64_t)1 << (g.bB - 1));
        const int64_t tile_sum = g.s * max_prod;
        const int64_t per_tile = tile_sum < (int64_t)g.acc_hi + 1 ? tile_sum : (int64_t)g.acc_hi + 1;
        g.partial16 = (hdqt::gemm_fast_eligible(g) && g.bA <= 4 && !g.fold &&
                       per_tile * g.tiles_per_split <= 32767 &&
                       hdqt::reduce_takes_slices16(g.splits, g.RA * g.RB)) ? 1 : 0;
        e = hdqt::launch_gemm(g, stream);
        if (e != hipSuccess) return hip_fail(e);
        e = hdqt::launch_reduce(g.partial, g.splits, g.RA * g.RB, g.scaleA, g.scaleB, g.inv_n, g.out,
                                g.out_bf16, g.acc_out, stream, g.mask_src, g.partial16 != 0);
        return e == hipSuccess ? HDQT_OK : hip_fail(e);
    }
    e = hdqt::launch_gemm(g, stream);
    if (e != hipSuccess) return hip_fail(e);
    // the rectifier's mask, where the matmul's own epilogue does not apply it
    if (g.mask_src && g.out && !hdqt::gemm_fast_masks(g)) {
        const int64_t count = g.fold ? g.fbatch * g.fC * g.fH * g.fW : g.RA * g.RB;
        e = hdqt::launch_relu_mask(g.out, g.mask_src, count, stream);
    }
    return e == hipSuccess ? HDQT_OK : hip_fail(e);
}

int run_gemm_codes(const void* qA, const void* qB, int bA, int bB, const float* scaleA,
                   const float* scaleB, int64_t RA, int64_t RB, int64_t D, int n_eff, int acc_bits,
                   int64_t s, float* out, uint16_t* out_bf16, int32_t* acc_out, void* workspace,
                   size_t workspace_bytes, void* stream)
{
    if (!qA || !qB || !scaleA || !scaleB || (!out && !out_bf16 && !acc_out)) return HDQT_EINVAL_NULL;
    if (RA <= 0 || RB <= 0 || D <= 0 || RA >= kMaxDim || RB >= kMaxDim || D >= kMaxDim)
        return HDQT_EINVAL_DIM;
    int rc;
    if ((rc = check_dims2(RA, D)) || (rc = check_dims2(RB, D)) || (rc = check_dims2(RA, RB)))
        return rc;
    if (bA < 2 || bA > 8 || bB < 2 || bB > 8) return HDQT_EINVAL_BITS;
    if (!is_pow2(n_eff) || n_eff > hdqt::kMaxHadamard || D % n_eff != 0)
        return HDQT_EINVAL_HADAMARD;
    if ((rc = check_accumulation(D, s, acc_bits, bA, bB))) return rc;
    if (misaligned(qA) || misaligned(qB) || misaligned(out) || misaligned(out_bf16) ||
        misaligned(acc_out) || misaligned(workspace))
        return HDQT_EALIGN;
    return run_planned_gemm(plan_gemm(qA, qB, bA, bB, scaleA, scaleB, RA, RB, D, n_eff, acc_bits, s,
                                      out, acc_out, 0, out_bf16),
                            workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

int run_gemm(int kind, const float* P, const float* Q, float* out, int64_t M, int64_t K, int64_t N,
             const hdqt_params_t* prm, int32_t* acc_out, void* ws, size_t ws_bytes, void* stream_v,
             uint16_t* out_bf16 = nullptr, const float* mask_src = nullptr)
{
    hdqt_ws_layout_t L;
    int rc = hdqt_workspace_layout(kind, M, K, N, prm, &L);
    if (rc) return rc;
    if (!P || !Q || (!out && !out_bf16 && !acc_out)) return HDQT_EINVAL_NULL;
    if (!ws || ws_bytes < L.total) return HDQT_EWORKSPACE;
    if (misaligned(P) || misaligned(Q) || misaligned(out) || misaligned(out_bf16) || misaligned(acc_out) ||
        misaligned(ws))
        return HDQT_EALIGN;
    Orientation o;
    orient(kind, M, K, N, &o);
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char* base = static_cast<char*>(ws);
    hdqt::QMeta* metaA = reinterpret_cast<hdqt::QMeta*>(base + L.scaleA);
    hdqt::QMeta* metaB = reinterpret_cast<hdqt::QMeta*>(base + L.scaleB);
    void* codesA = base + L.codesA;
    void* codesB = base + L.codesB;
    hdqt::GemmArgs g = plan_gemm(codesA, codesB, prm->A.b, prm->B.b, &metaA->scale, &metaB->scale,
                                 o.RA, o.RB, o.D, L.n_eff, prm->acc_bits, prm->s, out, acc_out, 1 + kind,
                                 out_bf16);
    if (mask_src && (misaligned(mask_src) || !out)) return out ? HDQT_EALIGN : HDQT_EINVAL_NULL;
    g.mask_src = mask_src;
    // one launch clears both calibration records (they are adjacent)
    hipError_t e = hdqt::launch_zero2(reinterpret_cast<uint32_t*>(metaA), (int64_t)(2 * kMetaBytes / 4),
                                      nullptr, 0, stream);
    if (e != hipSuccess) return hip_fail(e);
    rc = run_quantize(P, o.a_rows, o.a_cols, o.a_axis, L.n_eff, &prm->A, prm->seed, metaA, codesA,
                      nullptr, stream);
    if (rc) return rc;
    rc = run_quantize(Q, o.b_rows, o.b_cols, o.b_axis, L.n_eff, &prm->B, prm->seed, metaB, codesB,
                      nullptr, stream);
    if (rc) return rc;
    return run_planned_gemm(g, base + L.acc, L.total - L.acc, stream);
}


// Workspace of hdqt_layer_step.  Offsets in bytes; the calibration records are
// contiguous from offset 0, so one launch clears them all.
enum { T_X1, T_X0, T_W0, T_W1, T_G1, T_G0, T_COUNT };
struct StepLayout {
    size_t meta[T_COUNT];
    size_t codes[T_COUNT];
    size_t acc[3];           // per matmul: slices of a split contraction
    size_t acc_bytes[3];
    int splits[3];
    int n_eff[3];
    size_t zero_bytes;
    size_t total;
};

int plan_step(int64_t M, int64_t K, int64_t N, const hdqt_params_t* const prm[3], bool with_dx,
              StepLayout* L)
{
    Orientation o[3];
    for (int k = 0; k < 3; ++k) {
        if (k == HDQT_GEMM_BWD_INPUT && !with_dx) continue;
        const int rc = check_gemm(k, M, K, N, prm[k], &o[k]);
        if (rc) return rc;
    }
    size_t off = 0;
    for (int t = 0; t < T_COUNT; ++t) { L->meta[t] = off; off += kMetaBytes; }
    for (int k = 0; k < 3; ++k) {
        L->acc[k] = off;
        L->acc_bytes[k] = 0;
        L->splits[k] = 1;
        L->n_eff[k] = 1;
        if (k == HDQT_GEMM_BWD_INPUT && !with_dx) continue;
        L->n_eff[k] = hdqt_n_eff(o[k].D, prm[k]->had_block);
        const int64_t s = prm[k]->s < o[k].D ? prm[k]->s : o[k].D;
        L->splits[k] = choose_splits(o[k].RA, o[k].RB, o[k].D, (o[k].D + s - 1) / s);
    }
    L->zero_bytes = off;
    for (int k = 0; k < 3; ++k) {
        L->acc[k] = off;
        if (k == HDQT_GEMM_BWD_INPUT && !with_dx) continue;
        L->acc_bytes[k] = partial_bytes(o[k].RA, o[k].RB, o[k].D, prm[k]->s);
        off = align_up(off + L->acc_bytes[k], 256);
    }
    const hdqt_params_t *fwd = prm[0], *bwi = prm[1], *bww = prm[2];
    const size_t bytes[T_COUNT] = {
        (size_t)(M * hdqt_codes_pitch(K, fwd->A.b)),                 // X along K
        (size_t)(K * hdqt_codes_pitch(M, bww->A.b)),                 // X along M
        (size_t)(N * hdqt_codes_pitch(K, fwd->B.b)),                 // W along K
        with_dx ? (size_t)(K * hdqt_codes_pitch(N, bwi->B.b)) : 0,   // W along N
        with_dx ? (size_t)(M * hdqt_codes_pitch(N, bwi->A.b)) : 0,   // G along N
        (size_t)(N * hdqt_codes_pitch(M, bww->B.b)),                 // G along M
    };
    for (int t = 0; t < T_COUNT; ++t) {
        L->codes[t] = off;
        off = align_up(off + bytes[t], 256);
    }
    L->total = off;
    return HDQT_OK;
}


// ---- forward and backward halves of a layer's step, with X's codes along M handed over
constexpr size_t kSavedHeader = 256;     // the scale (one float) of the saved codes, then padding

struct FwdLayout {
    size_t metaX1, metaX0, metaW0;       // contiguous from offset 0
    size_t acc, acc_bytes;
    size_t codesX1, codesW0;
    size_t total;
    int n_fwd, n_bww;
};

int plan_fwd(int64_t M, int64_t K, int64_t N, const hdqt_params_t* fwd, const hdqt_params_t* bww,
             FwdLayout* L)
{
    Orientation o;
    int rc = check_gemm(HDQT_GEMM_FWD, M, K, N, fwd, &o);
    if (rc) return rc;
    L->n_fwd = hdqt_n_eff(K, fwd->had_block);
    L->n_bww = 1;
    if (bww) {
        Orientation ow;
        if ((rc = check_gemm(HDQT_GEMM_BWD_WEIGHT, M, K, N, bww, &ow))) return rc;
        L->n_bww = hdqt_n_eff(M, bww->had_block);
    }
    size_t off = 0;
    L->metaX1 = off; off += kMetaBytes;
    L->metaX0 = off; off += kMetaBytes;
    L->metaW0 = off; off += kMetaBytes;
    L->acc = off;
    L->acc_bytes = partial_bytes(M, N, K, fwd->s);
    off = align_up(off + L->acc_bytes, 256);
    L->codesX1 = off;
    off = align_up(off + (size_t)(M * hdqt_codes_pitch(K, fwd->A.b)), 256);
    L->codesW0 = off;
    off = align_up(off + (size_t)(N * hdqt_codes_pitch(K, fwd->B.b)), 256);
    L->total = off;
    return HDQT_OK;
}

struct BwdLayout {
    size_t metaG1, metaG0, metaW1;       // contiguous from offset 0
    size_t acc[2], acc_bytes[2];         // input gradient, weight gradient
    size_t codesG1, codesG0, codesW1;
    size_t total;
    int n_bwi, n_bww;
};

int plan_bwd(int64_t M, int64_t K, int64_t N, const hdqt_params_t* bwi, const hdqt_params_t* bww,
             BwdLayout* L)
{
    Orientation o;
    int rc = check_gemm(HDQT_GEMM_BWD_WEIGHT, M, K, N, bww, &o);
    if (rc) return rc;
    L->n_bww = hdqt_n_eff(M, bww->had_block);
    L->n_bwi = 1;
    if (bwi) {
        if ((rc = check_gemm(HDQT_GEMM_BWD_INPUT, M, K, N, bwi, &o))) return rc;
        L->n_bwi = hdqt_n_eff(N, bwi->had_block);
    }
    size_t off = 0;
    L->metaG1 = off; off += kMetaBytes;
    L->metaG0 = off; off += kMetaBytes;
    L->metaW1 = off; off += kMetaBytes;
    L->acc[0] = off;
    L->acc_bytes[0] = bwi ? partial_bytes(M, K, N, bwi->s) : 0;
    off = align_up(off + L->acc_bytes[0], 256);
    L->acc[1] = off;
    L->acc_bytes[1] = partial_bytes(K, N, M, bww->s);
    off = align_up(off + L->acc_bytes[1], 256);
    L->codesG1 = off;
    off = align_up(off + (bwi ? (size_t)(M * hdqt_codes_pitch(N, bwi->A.b)) : 0), 256);
    L->codesG0 = off;
    off = align_up(off + (size_t)(N * hdqt_codes_pitch(M, bww->B.b)), 256);
    L->codesW1 = off;
    off = align_up(off + (bwi ? (size_t)(K * hdqt_codes_pitch(N, bwi->B.b)) : 0), 256);
    L->total = off;
    return HDQT_OK;
}

// ---- second reading of the low-bit accumulator (tiled quantization of the partial sums)

int check_requant(int64_t RA, int64_t RB, int64_t D, int64_t s, int acc_bits, int bA, int bB)
{
    if (s < 1) return HDQT_EINVAL_TILE;
    if (acc_bits < 2 || acc_bits > 24) return HDQT_EINVAL_ACC;
    const int64_t s_eff = s < D ? s : D;
    const int64_t max_prod = ((int64_t)1 << (bA - 1)) * ((int64_t)1 << (bB - 1));
    // a tile sum must be exact in binary32 ...
    if (s_eff > (((int64_t)1 << 24) - 1) / max_prod) return HDQT_EINVAL_TILE;
    // ... and the sum over tiles of code * maximum must stay inside int32
    const int64_t n_tiles = (D + s_eff - 1) / s_eff;
    const int64_t per_tile = ((int64_t)1 << (acc_bits - 1)) * s_eff * max_prod;
    if (n_tiles > (((int64_t)1 << 31) - 1) / per_tile) return HDQT_EINVAL_ACC;
    (void)RA; (void)RB;
    return HDQT_OK;
}

// workspace of the emulation: the maxima and every tile's sums ([n_tiles, RA, RB] int32)
size_t requant_bytes(int64_t RA, int64_t RB, int64_t D, int64_t s)
{
    const int64_t s_eff = s < D ? s : D;
    const int64_t n_tiles = (D + s_eff - 1) / s_eff;
    return align_up((size_t)n_tiles * sizeof(uint32_t), 256) +
           (size_t)n_tiles * (size_t)(RA * RB) * sizeof(int32_t);
}

hdqt::GemmArgs plan_requant(const void* qA, const void* qB, int bA, int bB, const float* scaleA,
                            const float* scaleB, int64_t RA, int64_t RB, int64_t D, int n_eff, int64_t s,
                            float* out, int32_t* acc_out)
{
    // (the tiles are what this reading quantizes: they stay as given)
    return plan_gemm(qA, qB, bA, bB, scaleA, scaleB, RA, RB, D, n_eff, 32, s, out, acc_out, 0, nullptr, true);
}

// workspace of the path that will run: the two passes through the matrix-core kernel keep
// only the maxima (and, with a split contraction, one int32 slice per part)
size_t requant_bytes_for(int64_t RA, int64_t RB, int64_t D, int64_t s, int bA, int bB, int acc_bits)
{
    const hdqt::GemmArgs g = plan_requant(nullptr, nullptr, bA, bB, nullptr, nullptr, RA, RB, D, 1, s, nullptr, nullptr);
    if (!hdqt::gemm_requant_fast_eligible(g, acc_bits)) return requant_bytes(RA, RB, D, s);
    return align_up((size_t)g.n_tiles * sizeof(uint32_t), 256) +
           (g.splits > 1 ? (size_t)g.splits * (size_t)(RA * RB) * sizeof(int32_t) : 0);
}

int run_requant(const void* qA, const void* qB, int bA, int bB, const float* scaleA, const float* scaleB,
                int64_t RA, int64_t RB, int64_t D, int n_eff, int acc_bits, int64_t s, float* out,
                int32_t* acc_out, void* ws, size_t ws_bytes, hipStream_t stream)
{
    if (!ws || ws_bytes < requant_bytes_for(RA, RB, D, s, bA, bB, acc_bits)) return HDQT_EWORKSPACE;
    hdqt::GemmArgs g = plan_requant(qA, qB, bA, bB, scaleA, scaleB, RA, RB, D, n_eff, s, out, acc_out);
    char* base = static_cast<char*>(ws);
    g.tile_max = reinterpret_cast<uint32_t*>(base);
    g.partial = reinterpret_cast<int32_t*>(base + align_up((size_t)g.n_tiles * sizeof(uint32_t), 256));
    hipError_t e = hdqt::launch_zero2(g.tile_max, g.n_tiles, nullptr, 0, stream);
    if (e != hipSuccess) return hip_fail(e);
    if (hdqt::gemm_requant_fast_eligible(g, acc_bits)) {
        // value = acc * 2^-(a-1) * (scaleA * scaleB) / n_eff: both trailing factors are powers of two
        g.inv_n = g.inv_n * ldexpf(1.0f, -(acc_bits - 1));
        e = hdqt::launch_gemm_requant_fast(g, acc_bits, 1, stream);
        if (e != hipSuccess) return hip_fail(e);
        e = hdqt::launch_gemm_requant_fast(g, acc_bits, 2, stream);
        if (e != hipSuccess) return hip_fail(e);
        if (g.splits > 1)
            e = hdqt::launch_reduce(g.partial, g.splits, g.RA * g.RB, g.scaleA, g.scaleB, g.inv_n, g.out, nullptr,
                                    g.acc_out, stream);
        return e == hipSuccess ? HDQT_OK : hip_fail(e);
    }
    e = hdqt::launch_gemm_requant(g, acc_bits, stream);
    return e == hipSuccess ? HDQT_OK : hip_fail(e);
}

} // namespace

extern "C" {

int hdqt_n_eff(int64_t D, int had_block)
{
    if (D <= 0 || had_block < 1) return 1;
    int m = 1;
    while (m * 2 <= had_block && D % (m * 2) == 0) m *= 2;
    return m;
}

int64_t hdqt_codes_pitch(int64_t D, int b) { return b <= 4 ? (D + 1) / 2 : D; }

size_t hdqt_quantize_workspace_size(void) { return kMetaBytes; }

int hdqt_workspace_layout(int gemm_kind, int64_t M, int64_t K, int64_t N,
                          const hdqt_params_t* params, hdqt_ws_layout_t* layout)
{
    Orientation o;
    const int rc = check_gemm(gemm_kind, M, K, N, params, &o);
    if (rc) return rc;
    hdqt_ws_layout_t L;
    L.RA = o.RA; L.RB = o.RB; L.D = o.D;
    L.n_eff = hdqt_n_eff(o.D, params->had_block);
    size_t off = 0;
    // two calibration records, adjacent; `scale` is the first member of each
    L.scaleA = off;
    off += kMetaBytes;
    L.scaleB = off;
    off += kMetaBytes;
    L.codesA = off;
    off = align_up(off + (size_t)(o.RA * hdqt_codes_pitch(o.D, params->A.b)), 256);
    L.codesB = off;
    off = align_up(off + (size_t)(o.RB * hdqt_codes_pitch(o.D, params->B.b)), 256);
    L.acc = off;
    off = align_up(off + partial_bytes(o.RA, o.RB, o.D, params->s) + 256, 256);
    L.total = off;
    if (layout) *layout = L;
    return HDQT_OK;
}

size_t hdqt_workspace_size(int gemm_kind, int64_t M, int64_t K, int64_t N,
                           const hdqt_params_t* params)
{
    hdqt_ws_layout_t L;
    return hdqt_workspace_layout(gemm_kind, M, K, N, params, &L) == HDQT_OK ? L.total : 0;
}

int hdqt_quantize(const float* T, int64_t rows, int64_t cols, int axis, int had_block,
                  const hdqt_operand_t* op, uint64_t seed, void* codes_out, float* scale_out,
                  void* workspace, size_t workspace_bytes, void* stream)
{
    if (!T || !codes_out || !scale_out || !op) return HDQT_EINVAL_NULL;
    int rc = check_dims2(rows, cols);
    if (rc) return rc;
    if (axis != 0 && axis != 1) return HDQT_EINVAL_AXIS;
    if ((rc = check_hadamard(had_block))) return rc;
    if ((rc = check_operand(op))) return rc;
    if (!workspace || workspace_bytes < hdqt_quantize_workspace_size()) return HDQT_EWORKSPACE;
    if (misaligned(T) || misaligned(codes_out) || misaligned(workspace)) return HDQT_EALIGN;
    if ((reinterpret_cast<uintptr_t>(scale_out) & 3u) != 0) return HDQT_EALIGN;
    const int64_t D = axis ? cols : rows;
    const hipError_t e = hdqt::launch_zero2(static_cast<uint32_t*>(workspace), hdqt::kQMetaDwords,
                                            nullptr, 0, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return run_quantize(T, rows, cols, axis, hdqt_n_eff(D, had_block), op, seed,
                        static_cast<hdqt::QMeta*>(workspace), codes_out, scale_out,
                        static_cast<hipStream_t>(stream));
}

size_t hdqt_quantize_dual_workspace_size(void) { return 2 * kMetaBytes; }

int hdqt_quantize_dual(const float* T, int64_t rows, int64_t cols, int had_block,
                       const hdqt_operand_t* op_axis1, const hdqt_operand_t* op_axis0, uint64_t seed,
                       void* codes_axis1, float* scale_axis1, void* codes_axis0, float* scale_axis0,
                       void* workspace, size_t workspace_bytes, void* stream_v)
{
    if (!T || !op_axis1 || !op_axis0 || !codes_axis1 || !codes_axis0 || !scale_axis1 || !scale_axis0)
        return HDQT_EINVAL_NULL;
    int rc = check_dims2(rows, cols);
    if (rc) return rc;
    if ((rc = check_hadamard(had_block))) return rc;
    if ((rc = check_operand(op_axis1)) || (rc = check_operand(op_axis0))) return rc;
    if (!workspace || workspace_bytes < hdqt_quantize_dual_workspace_size()) return HDQT_EWORKSPACE;
    if (misaligned(T) || misaligned(codes_axis1) || misaligned(codes_axis0) || misaligned(workspace))
        return HDQT_EALIGN;
    if (((reinterpret_cast<uintptr_t>(scale_axis1) | reinterpret_cast<uintptr_t>(scale_axis0)) & 3u) != 0)
        return HDQT_EALIGN;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char* base = static_cast<char*>(workspace);
    hdqt::QMeta* meta1 = reinterpret_cast<hdqt::QMeta*>(base);
    hdqt::QMeta* meta0 = reinterpret_cast<hdqt::QMeta*>(base + kMetaBytes);
    const hipError_t e = hdqt::launch_zero2(reinterpret_cast<uint32_t*>(base),
                                            (int64_t)(2 * kMetaBytes / 4), nullptr, 0, stream);
    if (e != hipSuccess) return hip_fail(e);
    return run_quantize_pair(T, rows, cols, hdqt_n_eff(cols, had_block), op_axis1, seed,
                             hdqt_n_eff(rows, had_block), op_axis0, seed, meta1, meta0, codes_axis1,
                             codes_axis0, scale_axis1, scale_axis0, stream);
}

int hdqt_quantize_dual_im2col(const float* act, const hdqt_conv_t* geo, int had_block,
                              const hdqt_operand_t* op_axis1, const hdqt_operand_t* op_axis0,
                              uint64_t seed, void* codes_axis1, float* scale_axis1, void* codes_axis0,
                              float* scale_axis0, void* workspace, size_t workspace_bytes, void* stream_v)
{
    if (!act || !geo || !op_axis1 || !op_axis0 || !codes_axis1 || !codes_axis0 || !scale_axis1 ||
        !scale_axis0)
        return HDQT_EINVAL_NULL;
    int64_t rows, cols;
    if (!conv_matrix_shape(geo, &rows, &cols)) return HDQT_EINVAL_DIM;
    int rc;
    if ((rc = check_dims2(rows, cols)) || (rc = check_hadamard(had_block)) ||
        (rc = check_operand(op_axis1)) || (rc = check_operand(op_axis0)))
        return rc;
    if (!workspace || workspace_bytes < 2 * kMetaBytes) return HDQT_EWORKSPACE;
    if (misaligned(act) || misaligned(codes_axis1) || misaligned(codes_axis0) || misaligned(workspace))
        return HDQT_EALIGN;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char* base = static_cast<char*>(workspace);
    hdqt::QMeta* meta1 = reinterpret_cast<hdqt::QMeta*>(base);
    hdqt::QMeta* meta0 = reinterpret_cast<hdqt::QMeta*>(base + kMetaBytes);
    hdqt::DualArgs d = make_dual_args(act, rows, cols, hdqt_n_eff(cols, had_block), op_axis1, seed,
                                      hdqt_n_eff(rows, had_block), op_axis0, seed, meta1, meta0,
                                      codes_axis1, codes_axis0, scale_axis1, scale_axis0, 0);
    if (!set_conv_source(&d, geo) || !hdqt::quantize_dual_eligible(d)) return HDQT_EINVAL_GEOMETRY;
    hipError_t e = hdqt::launch_zero2(reinterpret_cast<uint32_t*>(base), (int64_t)(2 * kMetaBytes / 4),
                                      nullptr, 0, stream);
    if (e == hipSuccess) e = hdqt::launch_quantize_dual(d, stream);
    return e == hipSuccess ? HDQT_OK : hip_fail(e);
}

int hdqt_im2col(const float* act, int64_t batch, int channels, int height, int width, int kh, int kw,
                int stride, int pad_h, int pad_w, float* X, void* stream)
{
    if (!act || !X) return HDQT_EINVAL_NULL;
    if (batch < 1 || channels < 1 || height < 1 || width < 1 || kh < 1 || kw < 1 || stride < 1 || pad_h < 0 ||
        pad_w < 0 || kh > 255 || kw > 255 || height + 2 * pad_h < kh || width + 2 * pad_w < kw)
        return HDQT_EINVAL_DIM;
    const int Ho = (height + 2 * pad_h - kh) / stride + 1, Wo = (width + 2 * pad_w - kw) / stride + 1;
    const int64_t per_image = (int64_t)Ho * Wo, K = (int64_t)channels * kh * kw;
    if (batch > kMaxDim / per_image) return HDQT_EINVAL_DIM;
    const int64_t M = batch * per_image;
    int rc = check_dims2(M, K);
    if (rc) return rc;
    if ((int64_t)channels * height * width >= ((int64_t)1 << 31) || (M + 3) / 4 >= ((int64_t)1 << 31))
        return HDQT_EINVAL_DIM;
    if (misaligned(act) || misaligned(X)) return HDQT_EALIGN;
    hdqt::Im2colArgs a{act, X, M, channels, height, width, kh, kw, stride, pad_h, pad_w, Ho, Wo};
    const hipError_t e = hdqt::launch_im2col(a, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? HDQT_OK : hip_fail(e);
}

size_t hdqt_gemm_codes_workspace_size(int64_t RA, int64_t RB, int64_t D, int64_t s)
{
    if (RA <= 0 || RB <= 0 || D <= 0 || s < 1 || RA >= kMaxDim || RB >= kMaxDim || D >= kMaxDim) return 0;
    return partial_bytes(RA, RB, D, s);
}

int hdqt_gemm_codes(const void* qA, const void* qB, int bA, int bB, const float* scaleA,
                    const float* scaleB, int64_t RA, int64_t RB, int64_t D, int n_eff,
                    int acc_bits, int64_t s, float* out, int32_t* acc_out, void* workspace,
                    size_t workspace_bytes, void* stream)
{
    return run_gemm_codes(qA, qB, bA, bB, scaleA, scaleB, RA, RB, D, n_eff, acc_bits, s, out, nullptr,
                          acc_out, workspace, workspace_bytes, stream);
}

int hdqt_gemm_codes_bf16(const void* qA, const void* qB, int bA, int bB, const float* scaleA,
                         const float* scaleB, int64_t RA, int64_t RB, int64_t D, int n_eff,
                         int acc_bits, int64_t s, uint16_t* out, int32_t* acc_out, void* workspace,
                         size_t workspace_bytes, void* stream)
{
    return run_gemm_codes(qA, qB, bA, bB, scaleA, scaleB, RA, RB, D, n_eff, acc_bits, s, nullptr, out,
                          acc_out, workspace, workspace_bytes, stream);
}

size_t hdqt_gemm_codes_requant_workspace_size(int64_t RA, int64_t RB, int64_t D, int64_t s)
{
    if (RA <= 0 || RB <= 0 || D <= 0 || s < 1 || RA >= kMaxDim || RB >= kMaxDim || D >= kMaxDim) return 0;
    return requant_bytes(RA, RB, D, s);
}

size_t hdqt_gemm_codes_requant_workspace_size_for(int64_t RA, int64_t RB, int64_t D, int64_t s, int bA,
                                                  int bB, int acc_bits)
{
    if (RA <= 0 || RB <= 0 || D <= 0 || s < 1 || RA >= kMaxDim || RB >= kMaxDim || D >= kMaxDim) return 0;
    if (bA < 2 || bA > 8 || bB < 2 || bB > 8) return 0;
    if (check_requant(RA, RB, D, s, acc_bits, bA, bB)) return 0;
    return requant_bytes_for(RA, RB, D, s, bA, bB, acc_bits);
}

int hdqt_gemm_codes_requant(const void* qA, const void* qB, int bA, int bB, const float* scaleA,
                            const float* scaleB, int64_t RA, int64_t RB, int64_t D, int n_eff,
                            int acc_bits, int64_t s, float* out, int32_t* acc_out, void* workspace,
                            size_t workspace_bytes, void* stream)
{
    if (!qA || !qB || !scaleA || !scaleB || (!out && !acc_out)) return HDQT_EINVAL_NULL;
    if (RA <= 0 || RB <= 0 || D <= 0 || RA >= kMaxDim || RB >= kMaxDim || D >= kMaxDim)
        return HDQT_EINVAL_DIM;
    int rc;
    if ((rc = check_dims2(RA, D)) || (rc = check_dims2(RB, D)) || (rc = check_dims2(RA, RB))) return rc;
    if (bA < 2 || bA > 8 || bB < 2 || bB > 8) return HDQT_EINVAL_BITS;
    if (!is_pow2(n_eff) || n_eff > hdqt::kMaxHadamard || D % n_eff != 0) return HDQT_EINVAL_HADAMARD;
    if ((rc = check_requant(RA, RB, D, s, acc_bits, bA, bB))) return rc;
    if (misaligned(qA) || misaligned(qB) || misaligned(out) || misaligned(acc_out) || misaligned(workspace))
        return HDQT_EALIGN;
    return run_requant(qA, qB, bA, bB, scaleA, scaleB, RA, RB, D, n_eff, acc_bits, s, out, acc_out,
                       workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

size_t hdqt_gemm_requant_workspace_size(int gemm_kind, int64_t M, int64_t K, int64_t N,
                                        const hdqt_params_t* params)
{
    hdqt_ws_layout_t L;
    if (hdqt_workspace_layout(gemm_kind, M, K, N, params, &L) != HDQT_OK) return 0;
    if (check_requant(L.RA, L.RB, L.D, params->s, params->acc_bits, params->A.b, params->B.b)) return 0;
    return L.acc + requant_bytes_for(L.RA, L.RB, L.D, params->s, params->A.b, params->B.b, params->acc_bits);
}

int hdqt_gemm_requant(int gemm_kind, const float* P, const float* Q, float* out, int64_t M, int64_t K,
                      int64_t N, const hdqt_params_t* params, int32_t* acc_out, void* workspace,
                      size_t workspace_bytes, void* stream_v)
{
    hdqt_ws_layout_t L;
    int rc = hdqt_workspace_layout(gemm_kind, M, K, N, params, &L);
    if (rc) return rc;
    if ((rc = check_requant(L.RA, L.RB, L.D, params->s, params->acc_bits, params->A.b, params->B.b)))
        return rc;
    if (!P || !Q || (!out && !acc_out)) return HDQT_EINVAL_NULL;
    if (!workspace || workspace_bytes < L.acc + requant_bytes_for(L.RA, L.RB, L.D, params->s, params->A.b,
                                                                  params->B.b, params->acc_bits))
        return HDQT_EWORKSPACE;
    if (misaligned(P) || misaligned(Q) || misaligned(out) || misaligned(acc_out) || misaligned(workspace))
        return HDQT_EALIGN;
    Orientation o;
    orient(gemm_kind, M, K, N, &o);
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char* base = static_cast<char*>(workspace);
    hdqt::QMeta* metaA = reinterpret_cast<hdqt::QMeta*>(base + L.scaleA);
    hdqt::QMeta* metaB = reinterpret_cast<hdqt::QMeta*>(base + L.scaleB);
    hipError_t e = hdqt::launch_zero2(reinterpret_cast<uint32_t*>(metaA), (int64_t)(2 * kMetaBytes / 4),
                                      nullptr, 0, stream);
    if (e != hipSuccess) return hip_fail(e);
    rc = run_quantize(P, o.a_rows, o.a_cols, o.a_axis, L.n_eff, &params->A, params->seed, metaA,
                      base + L.codesA, nullptr, stream);
    if (rc) return rc;
    rc = run_quantize(Q, o.b_rows, o.b_cols, o.b_axis, L.n_eff, &params->B, params->seed, metaB,
                      base + L.codesB, nullptr, stream);
    if (rc) return rc;
    return run_requant(base + L.codesA, base + L.codesB, params->A.b, params->B.b, &metaA->scale,
                       &metaB->scale, L.RA, L.RB, L.D, L.n_eff, params->acc_bits, params->s, out, acc_out,
                       base + L.acc, workspace_bytes - L.acc, stream);
}

size_t hdqt_layer_step_workspace_size(int64_t M, int64_t K, int64_t N, const hdqt_params_t* fwd,
                                      const hdqt_params_t* bwd_input, const hdqt_params_t* bwd_weight)
{
    const hdqt_params_t* prm[3] = {fwd, bwd_input, bwd_weight};
    StepLayout L;
    return plan_step(M, K, N, prm, bwd_input != nullptr, &L) == HDQT_OK ? L.total : 0;
}

} // extern "C"

namespace {

// X is the [M, K] matrix, or, with `geo`, the activation whose im2col matrix it is.
int run_layer_step(const float* X, const hdqt_conv_t* geo, const float* W, const float* G, float* Z,
                   float* dX, float* dW, int64_t M, int64_t K, int64_t N, const hdqt_params_t* fwd,
                   const hdqt_params_t* bwd_input, const hdqt_params_t* bwd_weight, void* workspace,
                   size_t workspace_bytes, void* stream_v)
{
    if (!X || !W || !G || !Z || !dW || !fwd || !bwd_weight) return HDQT_EINVAL_NULL;
    const bool with_dx = dX != nullptr;
    if (with_dx && !bwd_input) return HDQT_EINVAL_NULL;
    const hdqt_params_t* prm[3] = {fwd, bwd_input, bwd_weight};
    StepLayout L;
    int rc = plan_step(M, K, N, prm, with_dx, &L);
    if (rc) return rc;
    if (!workspace || workspace_bytes < L.total) return HDQT_EWORKSPACE;
    if (misaligned(X) || misaligned(W) || misaligned(G) || misaligned(Z) || misaligned(dX) ||
        misaligned(dW) || misaligned(workspace))
        return HDQT_EALIGN;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char* base = static_cast<char*>(workspace);
    auto meta = [&](int t) { return reinterpret_cast<hdqt::QMeta*>(base + L.meta[t]); };
    auto codes = [&](int t) { return static_cast<void*>(base + L.codes[t]); };
    auto acc = [&](int k) { return static_cast<void*>(base + L.acc[k]); };

    const int nF = L.n_eff[HDQT_GEMM_FWD], nI = L.n_eff[HDQT_GEMM_BWD_INPUT],
              nW = L.n_eff[HDQT_GEMM_BWD_WEIGHT];
    // X along K (forward) and along M (weight gradient); W along N (input gradient) and
    // along K (forward); G along N (input gradient) and along M (weight gradient)
    bool g_done = false;
    hipError_t e;
    if (!with_dx) {
        if (geo) return HDQT_EINVAL_GEOMETRY;       // (hdqt_conv_step asks for dXcol)
        e = hdqt::launch_zero2(reinterpret_cast<uint32_t*>(base), (int64_t)(L.zero_bytes / 4), nullptr, 0,
                               stream);
        if (e != hipSuccess) return hip_fail(e);
    } else {
        hdqt::DualArgs dX3[3] = {
            make_dual_args(X, M, K, nF, &fwd->A, fwd->seed, nW, &bwd_weight->A, bwd_weight->seed,
                           meta(T_X1), meta(T_X0), codes(T_X1), codes(T_X0), nullptr, nullptr, 1),
            make_dual_args(W, K, N, nI, &bwd_input->B, bwd_input->seed, nF, &fwd->B, fwd->seed,
                           meta(T_W1), meta(T_W0), codes(T_W1), codes(T_W0), nullptr, nullptr, 2),
            make_dual_args(G, M, N, nI, &bwd_input->A, bwd_input->seed, nW, &bwd_weight->B,
                           bwd_weight->seed, meta(T_G1), meta(T_G0), codes(T_G1), codes(T_G0), nullptr,
                           nullptr, 3)};
        if (geo && !set_conv_source(&dX3[0], geo)) return HDQT_EINVAL_GEOMETRY;
        const hdqt::DualArgs &dx = dX3[0], &dw = dX3[1], &dg = dX3[2];
        const bool dual = hdqt::quantize_dual_eligible(dx) && hdqt::quantize_dual_eligible(dw) &&
                          hdqt::quantize_dual_eligible(dg);
        // an activation source is read by the two-axis kernels only (nothing is launched before
        // this is known)
        if (geo && !dual) return HDQT_EINVAL_GEOMETRY;
        e = hdqt::launch_zero2(reinterpret_cast<uint32_t*>(base), (int64_t)(L.zero_bytes / 4), nullptr, 0,
                               stream);
        if (e != hipSuccess) return hip_fail(e);
        if (dual) {
            // all three tensors take the two-axis kernels: one launch finds all six maxima,
            // and W's codes ride along with X's when the rounding modes agree
            e = hdqt::launch_dual_pass1(dX3, 3, stream);
            if (e != hipSuccess) return hip_fail(e);
            // G first: its tiles take longest (two random streams) and start while the chip fills
            const hdqt::DualArgs gxw[3] = {dg, dx, dw};
            if (hdqt::dual_pass2_batchable(gxw, 3)) {
                e = hdqt::launch_dual_pass2(gxw, 3, stream);
            } else {
                if (hdqt::dual_pass2_batchable(dX3, 2)) {
                    e = hdqt::launch_dual_pass2(dX3, 2, stream);
                } else {
                    e = hdqt::launch_dual_pass2(&dx, 1, stream);
                    if (e == hipSuccess) e = hdqt::launch_dual_pass2(&dw, 1, stream);
                }
                if (e == hipSuccess) e = hdqt::launch_dual_pass2(&dg, 1, stream);
            }
            if (e != hipSuccess) return hip_fail(e);
            g_done = true;
        }
    }
    if (!g_done) {
        rc = run_quantize_pair(X, M, K, nF, &fwd->A, fwd->seed, nW, &bwd_weight->A, bwd_weight->seed,
                               meta(T_X1), meta(T_X0), codes(T_X1), codes(T_X0), nullptr, nullptr, stream, 1);
        if (rc) return rc;
        if (with_dx)
            rc = run_quantize_pair(W, K, N, nI, &bwd_input->B, bwd_input->seed, nF, &fwd->B, fwd->seed,
                                   meta(T_W1), meta(T_W0), codes(T_W1), codes(T_W0), nullptr, nullptr, stream, 2);
        else
            rc = run_quantize(W, K, N, 0, nF, &fwd->B, fwd->seed, meta(T_W0), codes(T_W0), nullptr, stream);
        if (rc) return rc;
    }
    hdqt::GemmArgs g_fwd = plan_gemm(codes(T_X1), codes(T_W0), fwd->A.b, fwd->B.b, &meta(T_X1)->scale,
                                     &meta(T_W0)->scale, M, N, K, nF, fwd->acc_bits, fwd->s, Z, nullptr,
                                     1 + HDQT_GEMM_FWD);
    // Nobody can read Z before the two backward products of this call have run, and those move
    // several times the memory-side cache: from 16 MB on, Z is written with streaming stores
    // too.  (Measured on the 65536 x 1152 x 128 layer, Z = 33.5 MB: left in the cache as dirty
    // lines it is written back under the kernels that follow -- forward 30.1 -> 28.1 us, and
    // the next call's pass over X 66.6 -> 60.8 us.)  The forward call on its own keeps the
    // 128 MB mark: its caller reads Z next.
    if (M * N * (int64_t)sizeof(float) >= ((int64_t)16 << 20)) g_fwd.stream_out = 1;
    rc = run_planned_gemm(g_fwd, acc(HDQT_GEMM_FWD), L.acc_bytes[HDQT_GEMM_FWD], stream);
    if (rc) return rc;

    // ---- backward: G along N and along M.  The weight gradient goes first: its
    // operand, X's codes along M, was written by the forward part and is the older
    // data in the memory-side cache; the input gradient's large output comes last.
    if (g_done)
        rc = HDQT_OK;
    else if (with_dx)
        rc = run_quantize_pair(G, M, N, nI, &bwd_input->A, bwd_input->seed, nW, &bwd_weight->B,
                               bwd_weight->seed, meta(T_G1), meta(T_G0), codes(T_G1), codes(T_G0),
                               nullptr, nullptr, stream, 3);
    else
        rc = run_quantize(G, M, N, 0, nW, &bwd_weight->B, bwd_weight->seed, meta(T_G0), codes(T_G0),
                          nullptr, stream);
    if (rc) return rc;
    rc = run_planned_gemm(plan_gemm(codes(T_X0), codes(T_G0), bwd_weight->A.b, bwd_weight->B.b,
                                    &meta(T_X0)->scale, &meta(T_G0)->scale, K, N, M, nW,
                                    bwd_weight->acc_bits, bwd_weight->s, dW, nullptr,
                                    1 + HDQT_GEMM_BWD_WEIGHT),
                          acc(HDQT_GEMM_BWD_WEIGHT), L.acc_bytes[HDQT_GEMM_BWD_WEIGHT], stream);
    if (rc || !with_dx) return rc;
    return run_planned_gemm(plan_gemm(codes(T_G1), codes(T_W1), bwd_input->A.b, bwd_input->B.b,
                                      &meta(T_G1)->scale, &meta(T_W1)->scale, M, K, N, nI,
                                      bwd_input->acc_bits, bwd_input->s, dX, nullptr,
                                      1 + HDQT_GEMM_BWD_INPUT),
                            acc(HDQT_GEMM_BWD_INPUT), L.acc_bytes[HDQT_GEMM_BWD_INPUT], stream);
}

} // namespace

extern "C" {

int hdqt_layer_step(const float* X, const float* W, const float* G, float* Z, float* dX, float* dW,
                    int64_t M, int64_t K, int64_t N, const hdqt_params_t* fwd,
                    const hdqt_params_t* bwd_input, const hdqt_params_t* bwd_weight,
                    void* workspace, size_t workspace_bytes, void* stream)
{
    return run_layer_step(X, nullptr, W, G, Z, dX, dW, M, K, N, fwd, bwd_input, bwd_weight, workspace,
                          workspace_bytes, stream);
}

size_t hdqt_conv_step_workspace_size(const hdqt_conv_t* geo, int64_t N, const hdqt_params_t* fwd,
                                     const hdqt_params_t* bwd_input, const hdqt_params_t* bwd_weight)
{
    int64_t M, K;
    if (!conv_matrix_shape(geo, &M, &K) || !bwd_input) return 0;
    hdqt::DualArgs d{};
    d.rows = M; d.cols = K;
    if (!set_conv_source(&d, geo)) return 0;
    return hdqt_layer_step_workspace_size(M, K, N, fwd, bwd_input, bwd_weight);
}

int hdqt_conv_step(const float* act, const hdqt_conv_t* geo, const float* W, const float* G, float* Z,
                   float* dXcol, float* dW, int64_t N, const hdqt_params_t* fwd,
                   const hdqt_params_t* bwd_input, const hdqt_params_t* bwd_weight, void* workspace,
                   size_t workspace_bytes, void* stream)
{
    if (!geo || !dXcol || !bwd_input) return HDQT_EINVAL_NULL;
    int64_t M, K;
    if (!conv_matrix_shape(geo, &M, &K)) return HDQT_EINVAL_DIM;
    return run_layer_step(act, geo, W, G, Z, dXcol, dW, M, K, N, fwd, bwd_input, bwd_weight, workspace,
                          workspace_bytes, stream);
}

size_t hdqt_layer_saved_size(int64_t M, int64_t K, const hdqt_params_t* bwd_weight)
{
    if (!bwd_weight || check_dims2(M, K) || check_operand(&bwd_weight->A)) return 0;
    return kSavedHeader + align_up((size_t)(K * hdqt_codes_pitch(M, bwd_weight->A.b)), 256);
}

size_t hdqt_layer_fwd_workspace_size(int64_t M, int64_t K, int64_t N, const hdqt_params_t* fwd,
                                     const hdqt_params_t* bwd_weight)
{
    FwdLayout L;
    return plan_fwd(M, K, N, fwd, bwd_weight, &L) == HDQT_OK ? L.total : 0;
}

} // extern "C"

namespace {

// X is the [M, K] matrix, or, with `geo`, the activation whose im2col matrix it is.
int run_layer_fwd(const float* X, const hdqt_conv_t* geo, const float* W, float* Z, int64_t M, int64_t K,
                  int64_t N, const hdqt_params_t* fwd, const hdqt_params_t* bwd_weight, void* saved,
                  size_t saved_bytes, void* workspace, size_t workspace_bytes, void* stream_v)
{
    if (!X || !W || !Z || !fwd) return HDQT_EINVAL_NULL;
    if (bwd_weight && !saved) return HDQT_EINVAL_NULL;
    FwdLayout L;
    int rc = plan_fwd(M, K, N, fwd, bwd_weight, &L);
    if (rc) return rc;
    if (!workspace || workspace_bytes < L.total) return HDQT_EWORKSPACE;
    if (bwd_weight && saved_bytes < hdqt_layer_saved_size(M, K, bwd_weight)) return HDQT_EWORKSPACE;
    if (misaligned(X) || misaligned(W) || misaligned(Z) || misaligned(saved) || misaligned(workspace))
        return HDQT_EALIGN;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char* base = static_cast<char*>(workspace);
    char* sv = static_cast<char*>(saved);
    auto meta = [&](size_t off) { return reinterpret_cast<hdqt::QMeta*>(base + off); };
    hdqt::DualArgs dconv{};
    if (geo) {
        // an activation source is read by the two-axis kernels only: both code sets are made,
        // and nothing is launched before the geometry is known to be taken
        if (!bwd_weight) return HDQT_EINVAL_NULL;
        dconv = make_dual_args(X, M, K, L.n_fwd, &fwd->A, fwd->seed, L.n_bww, &bwd_weight->A,
                               bwd_weight->seed, meta(L.metaX1), meta(L.metaX0), base + L.codesX1,
                               sv + kSavedHeader, nullptr, reinterpret_cast<float*>(sv), 1);
        if (!set_conv_source(&dconv, geo) || !hdqt::quantize_dual_eligible(dconv))
            return HDQT_EINVAL_GEOMETRY;
    }
    hipError_t e = hdqt::launch_zero2(reinterpret_cast<uint32_t*>(base), (int64_t)(3 * kMetaBytes / 4),
                                      nullptr, 0, stream);
    if (e != hipSuccess) return hip_fail(e);
    if (geo) {
        e = hdqt::launch_quantize_dual(dconv, stream);
        rc = e == hipSuccess ? HDQT_OK : hip_fail(e);
    } else if (bwd_weight)
        rc = run_quantize_pair(X, M, K, L.n_fwd, &fwd->A, fwd->seed, L.n_bww, &bwd_weight->A,
                               bwd_weight->seed, meta(L.metaX1), meta(L.metaX0), base + L.codesX1,
                               sv + kSavedHeader, nullptr, reinterpret_cast<float*>(sv), stream, 1);
    else
        rc = run_quantize(X, M, K, 1, L.n_fwd, &fwd->A, fwd->seed, meta(L.metaX1), base + L.codesX1,
                          nullptr, stream);
    if (rc) return rc;
    rc = run_quantize(W, K, N, 0, L.n_fwd, &fwd->B, fwd->seed, meta(L.metaW0), base + L.codesW0, nullptr,
                      stream);
    if (rc) return rc;
    return run_planned_gemm(plan_gemm(base + L.codesX1, base + L.codesW0, fwd->A.b, fwd->B.b,
                                      &meta(L.metaX1)->scale, &meta(L.metaW0)->scale, M, N, K, L.n_fwd,
                                      fwd->acc_bits, fwd->s, Z, nullptr, 1 + HDQT_GEMM_FWD),
                            base + L.acc, L.acc_bytes, stream);
}

} // namespace

extern "C" {

int hdqt_layer_fwd(const float* X, const float* W, float* Z, int64_t M, int64_t K, int64_t N,
                   const hdqt_params_t* fwd, const hdqt_params_t* bwd_weight, void* saved,
                   size_t saved_bytes, void* workspace, size_t workspace_bytes, void* stream)
{
    return run_layer_fwd(X, nullptr, W, Z, M, K, N, fwd, bwd_weight, saved, saved_bytes, workspace,
                         workspace_bytes, stream);
}

int hdqt_conv_fwd(const float* act, const hdqt_conv_t* geo, const float* W, float* Z, int64_t N,
                  const hdqt_params_t* fwd, const hdqt_params_t* bwd_weight, void* saved,
                  size_t saved_bytes, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!geo) return HDQT_EINVAL_NULL;
    int64_t M, K;
    if (!conv_matrix_shape(geo, &M, &K)) return HDQT_EINVAL_DIM;
    return run_layer_fwd(act, geo, W, Z, M, K, N, fwd, bwd_weight, saved, saved_bytes, workspace,
                         workspace_bytes, stream);
}

size_t hdqt_layer_bwd_workspace_size(int64_t M, int64_t K, int64_t N, const hdqt_params_t* bwd_input,
                                     const hdqt_params_t* bwd_weight)
{
    BwdLayout L;
    return plan_bwd(M, K, N, bwd_input, bwd_weight, &L) == HDQT_OK ? L.total : 0;
}

} // extern "C"

namespace {

// dX is the gradient of the [M, K] matrix, or, with `geo`, of the activation it was unfolded from.
int run_layer_bwd(const float* G, const float* W, const void* saved, const hdqt_conv_t* geo, float* dX,
                  float* dW, int64_t M, int64_t K, int64_t N, const hdqt_params_t* bwd_input,
                  const hdqt_params_t* bwd_weight, void* workspace, size_t workspace_bytes,
                  void* stream_v, const float* mask_src = nullptr)
{
    if (!G || !saved || !dW || !bwd_weight) return HDQT_EINVAL_NULL;
    const bool with_dx = dX != nullptr;
    if (mask_src && !with_dx) return HDQT_EINVAL_NULL;
    if (misaligned(mask_src)) return HDQT_EALIGN;
    if (with_dx && (!bwd_input || !W)) return HDQT_EINVAL_NULL;
    BwdLayout L;
    int rc = plan_bwd(M, K, N, with_dx ? bwd_input : nullptr, bwd_weight, &L);
    if (rc) return rc;
    if (!workspace || workspace_bytes < L.total) return HDQT_EWORKSPACE;
    if (misaligned(G) || misaligned(W) || misaligned(saved) || misaligned(dX) || misaligned(dW) ||
        misaligned(workspace))
        return HDQT_EALIGN;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char* base = static_cast<char*>(workspace);
    const char* sv = static_cast<const char*>(saved);
    auto meta = [&](size_t off) { return reinterpret_cast<hdqt::QMeta*>(base + off); };
    hdqt::GemmArgs g_dx{};
    if (with_dx) {
        g_dx = plan_gemm(base + L.codesG1, base + L.codesW1, bwd_input->A.b, bwd_input->B.b,
                         &meta(L.metaG1)->scale, &meta(L.metaW1)->scale, M, K, N, L.n_bwi,
                         bwd_input->acc_bits, bwd_input->s, dX, nullptr, 1 + HDQT_GEMM_BWD_INPUT);
        // (nothing is launched before the geometry is known to be taken)
        if (geo && !hdqt::gemm_fold_plan(&g_dx, geo->batch, geo->channels, geo->height, geo->width, geo->kh,
                                         geo->kw))
            return HDQT_EINVAL_GEOMETRY;
        g_dx.mask_src = mask_src;
    } else if (geo) {
        return HDQT_EINVAL_NULL;
    }
    hipError_t e = hdqt::launch_zero2(reinterpret_cast<uint32_t*>(base), (int64_t)(3 * kMetaBytes / 4),
                                      nullptr, 0, stream);
    if (e != hipSuccess) return hip_fail(e);
    if (with_dx)
        rc = run_quantize_pair(G, M, N, L.n_bwi, &bwd_input->A, bwd_input->seed, L.n_bww, &bwd_weight->B,
                               bwd_weight->seed, meta(L.metaG1), meta(L.metaG0), base + L.codesG1,
                               base + L.codesG0, nullptr, nullptr, stream, 3);
    else
        rc = run_quantize(G, M, N, 0, L.n_bww, &bwd_weight->B, bwd_weight->seed, meta(L.metaG0),
                          base + L.codesG0, nullptr, stream);
    if (rc) return rc;
    rc = run_planned_gemm(plan_gemm(sv + kSavedHeader, base + L.codesG0, bwd_weight->A.b, bwd_weight->B.b,
                                    reinterpret_cast<const float*>(sv), &meta(L.metaG0)->scale, K, N, M,
                                    L.n_bww, bwd_weight->acc_bits, bwd_weight->s, dW, nullptr,
                                    1 + HDQT_GEMM_BWD_WEIGHT),
                          base + L.acc[1], L.acc_bytes[1], stream);
    if (rc || !with_dx) return rc;
    rc = run_quantize(W, K, N, 1, L.n_bwi, &bwd_input->B, bwd_input->seed, meta(L.metaW1),
                      base + L.codesW1, nullptr, stream);
    if (rc) return rc;
    return run_planned_gemm(g_dx, base + L.acc[0], L.acc_bytes[0], stream);
}

} // namespace

extern "C" {

int hdqt_layer_bwd(const float* G, const float* W, const void* saved, float* dX, float* dW, int64_t M,
                   int64_t K, int64_t N, const hdqt_params_t* bwd_input,
                   const hdqt_params_t* bwd_weight, void* workspace, size_t workspace_bytes,
                   void* stream)
{
    return run_layer_bwd(G, W, saved, nullptr, dX, dW, M, K, N, bwd_input, bwd_weight, workspace,
                         workspace_bytes, stream);
}

int hdqt_conv_bwd(const float* G, const float* W, const void* saved, const hdqt_conv_t* geo, float* dAct,
                  float* dW, int64_t N, const hdqt_params_t* bwd_input, const hdqt_params_t* bwd_weight,
                  void* workspace, size_t workspace_bytes, void* stream)
{
    if (!geo || !dAct) return HDQT_EINVAL_NULL;
    int64_t M, K;
    if (!conv_matrix_shape(geo, &M, &K)) return HDQT_EINVAL_DIM;
    return run_layer_bwd(G, W, saved, geo, dAct, dW, M, K, N, bwd_input, bwd_weight, workspace,
                         workspace_bytes, stream);
}

int hdqt_layer_bwd_masked(const float* G, const float* W, const void* saved, const float* x_mask,
                          float* dX, float* dW, int64_t M, int64_t K, int64_t N,
                          const hdqt_params_t* bwd_input, const hdqt_params_t* bwd_weight, void* workspace,
                          size_t workspace_bytes, void* stream)
{
    if (!x_mask || !dX) return HDQT_EINVAL_NULL;
    return run_layer_bwd(G, W, saved, nullptr, dX, dW, M, K, N, bwd_input, bwd_weight, workspace,
                         workspace_bytes, stream, x_mask);
}

int hdqt_conv_bwd_masked(const float* G, const float* W, const void* saved, const hdqt_conv_t* geo,
                         const float* act_mask, float* dAct, float* dW, int64_t N,
                         const hdqt_params_t* bwd_input, const hdqt_params_t* bwd_weight, void* workspace,
                         size_t workspace_bytes, void* stream)
{
    if (!geo || !dAct || !act_mask) return HDQT_EINVAL_NULL;
    int64_t M, K;
    if (!conv_matrix_shape(geo, &M, &K)) return HDQT_EINVAL_DIM;
    return run_layer_bwd(G, W, saved, geo, dAct, dW, M, K, N, bwd_input, bwd_weight, workspace,
                         workspace_bytes, stream, act_mask);
}

int hdqt_gemm_bwd_input_masked(const float* G, const float* W, const float* x_mask, float* dX, int64_t M,
                               int64_t K, int64_t N, const hdqt_params_t* params, int32_t* acc_out,
                               void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x_mask || !dX) return HDQT_EINVAL_NULL;
    return run_gemm(HDQT_GEMM_BWD_INPUT, G, W, dX, M, K, N, params, acc_out, workspace, workspace_bytes,
                    stream, nullptr, x_mask);
}

int hdqt_gemm_codes_fold(const void* qG, const void* qW, int bG, int bW, const float* scaleG,
                         const float* scaleW, const hdqt_conv_t* geo, int64_t N, int n_eff, int acc_bits,
                         int64_t s, float* dAct, void* stream)
{
    if (!qG || !qW || !scaleG || !scaleW || !geo || !dAct) return HDQT_EINVAL_NULL;
    int64_t M, K;
    if (!conv_matrix_shape(geo, &M, &K) || N <= 0 || N >= kMaxDim) return HDQT_EINVAL_DIM;
    int rc;
    if ((rc = check_dims2(M, N)) || (rc = check_dims2(K, N)) || (rc = check_dims2(M, K))) return rc;
    if (bG < 2 || bG > 8 || bW < 2 || bW > 8) return HDQT_EINVAL_BITS;
    if (!is_pow2(n_eff) || n_eff > hdqt::kMaxHadamard || N % n_eff != 0) return HDQT_EINVAL_HADAMARD;
    if ((rc = check_accumulation(N, s, acc_bits, bG, bW))) return rc;
    if (misaligned(qG) || misaligned(qW) || misaligned(dAct)) return HDQT_EALIGN;
    hdqt::GemmArgs g = plan_gemm(qG, qW, bG, bW, scaleG, scaleW, M, K, N, n_eff, acc_bits, s, dAct, nullptr,
                                 1 + HDQT_GEMM_BWD_INPUT);
    if (!hdqt::gemm_fold_plan(&g, geo->batch, geo->channels, geo->height, geo->width, geo->kh, geo->kw))
        return HDQT_EINVAL_GEOMETRY;
    return run_planned_gemm(g, nullptr, 0, static_cast<hipStream_t>(stream));
}


int hdqt_gemm_fwd(const float* X, const float* W, float* Z, int64_t M, int64_t K, int64_t N,
                  const hdqt_params_t* params, int32_t* acc_out, void* workspace,
                  size_t workspace_bytes, void* stream)
{
    return run_gemm(HDQT_GEMM_FWD, X, W, Z, M, K, N, params, acc_out, workspace, workspace_bytes,
                    stream);
}

int hdqt_gemm_bwd_input(const float* G, const float* W, float* dX, int64_t M, int64_t K, int64_t N,
                        const hdqt_params_t* params, int32_t* acc_out, void* workspace,
                        size_t workspace_bytes, void* stream)
{
    return run_gemm(HDQT_GEMM_BWD_INPUT, G, W, dX, M, K, N, params, acc_out, workspace,
                    workspace_bytes, stream);
}

int hdqt_gemm_bwd_input_bf16(const float* G, const float* W, uint16_t* dX, int64_t M, int64_t K,
                             int64_t N, const hdqt_params_t* params, int32_t* acc_out, void* workspace,
                             size_t workspace_bytes, void* stream)
{
    return run_gemm(HDQT_GEMM_BWD_INPUT, G, W, nullptr, M, K, N, params, acc_out, workspace,
                    workspace_bytes, stream, dX);
}

int hdqt_gemm_bwd_weight(const float* X, const float* G, float* dW, int64_t M, int64_t K,
                         int64_t N, const hdqt_params_t* params, int32_t* acc_out, void* workspace,
                         size_t workspace_bytes, void* stream)
{
    return run_gemm(HDQT_GEMM_BWD_WEIGHT, X, G, dW, M, K, N, params, acc_out, workspace,
                    workspace_bytes, stream);
}

// ---- hdqt_gemm_fwd without a workspace argument and without any allocation ----
//
// The calibration records and the codes of both operands, which hdqt_gemm_fwd keeps in the
// caller's workspace, live in a file-scope device array instead.  Every GPU the library runs
// on holds its own copy of the array at its own address: the address is asked for once per
// device (hipGetSymbolAddress with that device current) and only that pointer is ever handed
// to a kernel -- in host code the array's name is a stand-in, not a device address.
} // extern "C"

namespace {
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {nullptr};
std::mutex g_scratch_mu;

// device pointer of `scratch` on the current device; nullptr (and the HIP error recorded) on failure
void* static_scratch()
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        g_last_hip_error = (int)(e != hipSuccess ? e : hipErrorInvalidDevice);
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            g_last_hip_error = (int)(e != hipSuccess ? e : hipErrorInvalidSymbol);
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}
} // namespace

extern "C" {

size_t hdqt_gemm_fwd_static_max_bytes(void) { return kStaticScratchBytes; }

int hdqt_gemm_fwd_static(const float* X, const float* W, float* Z, int64_t M, int64_t K, int64_t N,
                         const hdqt_params_t* params, int32_t* acc_out, void* stream)
{
    hdqt_ws_layout_t L;
    const int rc = hdqt_workspace_layout(HDQT_GEMM_FWD, M, K, N, params, &L);
    if (rc) return rc;
    if (L.total > kStaticScratchBytes) return HDQT_ESCRATCH;
    void* ptr = static_scratch();
    if (!ptr) return HDQT_EHIP;
    // run_gemm clears the calibration records with a kernel before anything reads them, and
    // writes every code byte that the matmul reads: what an earlier call left behind in the
    // array is never seen.
    return run_gemm(HDQT_GEMM_FWD, X, W, Z, M, K, N, params, acc_out, ptr, kStaticScratchBytes, stream);
}

const char* hdqt_strerror(int code)
{
    switch (code) {
    case HDQT_OK: return "success";
    case HDQT_EINVAL_NULL: return "a required pointer is NULL";
    case HDQT_EINVAL_DIM: return "a dimension is not positive or is too large";
    case HDQT_EINVAL_HADAMARD: return "Hadamard block order must be a power of two in [1, 256]";
    case HDQT_EINVAL_BITS: return "code width b must be in [2, 8]";
    case HDQT_EINVAL_ACC: return "accumulator width must be in [2, 32] and the total must fit int32";
    case HDQT_EINVAL_TILE: return "tile length s must be >= 1 and a tile's sum must fit int32";
    case HDQT_EINVAL_CLIP: return "clip factor must be in (0, 1]";
    case HDQT_EINVAL_ROUND: return "unknown rounding mode";
    case HDQT_EINVAL_AXIS: return "axis must be 0 or 1 / unknown matmul kind";
    case HDQT_EWORKSPACE: return "workspace is NULL or too small";
    case HDQT_EALIGN: return "a pointer is not 16-byte aligned";
    case HDQT_EHIP: return "a HIP call failed (see hdqt_last_hip_error)";
    case HDQT_ESCRATCH: return "the shape needs more scratch than the library's fixed device array holds";
    case HDQT_EINVAL_GEOMETRY: return "convolution geometry or layer shape not taken by the activation-source kernels";
    default: return "unknown error code";
    }
}

int hdqt_last_hip_error(void) { return g_last_hip_error; }

} // extern "C"
