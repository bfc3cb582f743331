// C ABI of the HDQT library: argument validation, workspace planning and the
// sequence of launches of each entry point.  See include/hdqt.h for the
// contract of every function.

#include "../../include/hdqt.h"
#include "common.hpp"

#include <limits.h>

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

constexpr int64_t kMaxDim = (int64_t)1 << 31;        // per dimension
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

// how many workgroups share an output tile along the contraction
int choose_splits(int64_t RA, int64_t RB, int64_t n_tiles)
{
    const int64_t blocks = ((RA + 127) / 128) * ((RB + 127) / 128);
    if (blocks >= 512 || n_tiles < 8) return 1;
    int64_t want = (1024 + blocks - 1) / blocks;
    if (want > n_tiles / 4) want = n_tiles / 4;
    if (want > 1024) want = 1024;
    return want < 1 ? 1 : (int)want;
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

// Resolve tile length, accumulator range and the split of the contraction.
hdqt::GemmArgs plan_gemm(const void* qA, const void* qB, int bA, int bB, const float* scaleA,
                         const float* scaleB, int64_t RA, int64_t RB, int64_t D, int n_eff,
                         int acc_bits, int64_t s, float* out, int32_t* acc_out)
{
    hdqt::GemmArgs g{};
    g.qA = static_cast<const uint8_t*>(qA); g.qB = static_cast<const uint8_t*>(qB);
    g.pitchA = hdqt_codes_pitch(D, bA); g.pitchB = hdqt_codes_pitch(D, bB);
    g.bA = bA; g.bB = bB; g.RA = RA; g.RB = RB; g.D = D;
    g.s = s < D ? s : D;
    g.s_pad = (int)((g.s + 15) / 16 * 16);
    g.n_tiles = (D + g.s - 1) / g.s;
    g.acc_lo = acc_bits >= 32 ? INT_MIN : -(1 << (acc_bits - 1));
    g.acc_hi = acc_bits >= 32 ? INT_MAX : (1 << (acc_bits - 1)) - 1;
    g.scaleA = scaleA; g.scaleB = scaleB;
    g.inv_n = 1.0f / (float)n_eff;
    g.out = out; g.acc_out = acc_out;
    g.splits = choose_splits(RA, RB, g.n_tiles);
    g.tiles_per_split = (g.n_tiles + g.splits - 1) / g.splits;
    g.splits = (int)((g.n_tiles + g.tiles_per_split - 1) / g.tiles_per_split);
    return g;
}

// With a split contraction the workgroups add their partial totals into an
// int32 buffer (acc_out, or the workspace when the caller wants no accumulators)
// that must be zero beforehand; the dequantization is then a pass of its own.
int run_planned_gemm(hdqt::GemmArgs g, int32_t* acc_ws, bool target_is_zero, hipStream_t stream)
{
    hipError_t e;
    if (g.splits > 1) {
        int32_t* target = g.acc_out ? g.acc_out : acc_ws;
        if (!target) return HDQT_EWORKSPACE;
        g.acc_out = target;
        if (!target_is_zero) {
            e = hdqt::launch_zero2(reinterpret_cast<uint32_t*>(target), g.RA * g.RB, nullptr, 0, stream);
            if (e != hipSuccess) return hip_fail(e);
        }
        e = hdqt::launch_gemm(g, stream);
        if (e != hipSuccess) return hip_fail(e);
        if (g.out) {
            e = hdqt::launch_dequant(target, g.RA * g.RB, g.scaleA, g.scaleB, g.inv_n, g.out, stream);
            if (e != hipSuccess) return hip_fail(e);
        }
        return HDQT_OK;
    }
    e = hdqt::launch_gemm(g, stream);
    return e == hipSuccess ? HDQT_OK : hip_fail(e);
}

int run_gemm(int kind, const float* P, const float* Q, float* out, int64_t M, int64_t K, int64_t N,
             const hdqt_params_t* prm, int32_t* acc_out, void* ws, size_t ws_bytes, void* stream_v)
{
    hdqt_ws_layout_t L;
    int rc = hdqt_workspace_layout(kind, M, K, N, prm, &L);
    if (rc) return rc;
    if (!P || !Q || (!out && !acc_out)) return HDQT_EINVAL_NULL;
    if (!ws || ws_bytes < L.total) return HDQT_EWORKSPACE;
    if (misaligned(P) || misaligned(Q) || misaligned(out) || misaligned(acc_out) || misaligned(ws))
        return HDQT_EALIGN;
    Orientation o;
    orient(kind, M, K, N, &o);
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char* base = static_cast<char*>(ws);
    hdqt::QMeta* metaA = reinterpret_cast<hdqt::QMeta*>(base + L.scaleA);
    hdqt::QMeta* metaB = reinterpret_cast<hdqt::QMeta*>(base + L.scaleB);
    void* codesA = base + L.codesA;
    void* codesB = base + L.codesB;
    int32_t* acc_ws = reinterpret_cast<int32_t*>(base + L.acc);
    hdqt::GemmArgs g = plan_gemm(codesA, codesB, prm->A.b, prm->B.b, &metaA->scale, &metaB->scale,
                                 o.RA, o.RB, o.D, L.n_eff, prm->acc_bits, prm->s, out, acc_out);
    // one launch clears both calibration records (they are adjacent) and, when the
    // contraction is split, the accumulation target
    uint32_t* acc_target = g.splits > 1 ? reinterpret_cast<uint32_t*>(acc_out ? acc_out : acc_ws) : nullptr;
    hipError_t e = hdqt::launch_zero2(reinterpret_cast<uint32_t*>(metaA), (int64_t)(2 * kMetaBytes / 4),
                                      acc_target, acc_target ? o.RA * o.RB : 0, stream);
    if (e != hipSuccess) return hip_fail(e);
    rc = run_quantize(P, o.a_rows, o.a_cols, o.a_axis, L.n_eff, &prm->A, prm->seed, metaA, codesA,
                      nullptr, stream);
    if (rc) return rc;
    rc = run_quantize(Q, o.b_rows, o.b_cols, o.b_axis, L.n_eff, &prm->B, prm->seed, metaB, codesB,
                      nullptr, stream);
    if (rc) return rc;
    return run_planned_gemm(g, acc_ws, true, stream);
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
    off = align_up(off + (size_t)(o.RA * o.RB) * sizeof(int32_t), 256);
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

int hdqt_gemm_codes(const void* qA, const void* qB, int bA, int bB, const float* scaleA,
                    const float* scaleB, int64_t RA, int64_t RB, int64_t D, int n_eff,
                    int acc_bits, int64_t s, float* out, int32_t* acc_out, void* workspace,
                    size_t workspace_bytes, void* stream)
{
    if (!qA || !qB || !scaleA || !scaleB || (!out && !acc_out)) return HDQT_EINVAL_NULL;
    if (RA <= 0 || RB <= 0 || D <= 0 || RA >= kMaxDim || RB >= kMaxDim || D >= kMaxDim)
        return HDQT_EINVAL_DIM;
    int rc;
    if ((rc = check_dims2(RA, D)) || (rc = check_dims2(RB, D)) || (rc = check_dims2(RA, RB)))
        return rc;
    if (bA < 2 || bA > 8 || bB < 2 || bB > 8) return HDQT_EINVAL_BITS;
    if (!is_pow2(n_eff) || n_eff > hdqt::kMaxHadamard || D % n_eff != 0)
        return HDQT_EINVAL_HADAMARD;
    if ((rc = check_accumulation(D, s, acc_bits, bA, bB))) return rc;
    if (misaligned(qA) || misaligned(qB) || misaligned(out) || misaligned(acc_out) ||
        misaligned(workspace))
        return HDQT_EALIGN;
    int32_t* acc_ws = nullptr;
    if (workspace && workspace_bytes >= (size_t)(RA * RB) * sizeof(int32_t))
        acc_ws = static_cast<int32_t*>(workspace);
    return run_planned_gemm(plan_gemm(qA, qB, bA, bB, scaleA, scaleB, RA, RB, D, n_eff, acc_bits, s,
                                      out, acc_out),
                            acc_ws, false, static_cast<hipStream_t>(stream));
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

int hdqt_gemm_bwd_weight(const float* X, const float* G, float* dW, int64_t M, int64_t K,
                         int64_t N, const hdqt_params_t* params, int32_t* acc_out, void* workspace,
                         size_t workspace_bytes, void* stream)
{
    return run_gemm(HDQT_GEMM_BWD_WEIGHT, X, G, dW, M, K, N, params, acc_out, workspace,
                    workspace_bytes, stream);
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
    default: return "unknown error code";
    }
}

int hdqt_last_hip_error(void) { return g_last_hip_error; }

} // extern "C"
