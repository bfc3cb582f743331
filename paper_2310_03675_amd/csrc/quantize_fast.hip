// Hadamard-domain quantization, tuned kernels (gfx950).
//
// Same arithmetic as quantize.hip (butterfly strides 1, 2, 4, ... in that
// order; one multiplication, one rounding, one clamp per value), different
// machinery:
//   * cross-lane butterfly stages use DPP moves (lane xor 1, 2, 4, 8) and the
//     gfx950 lane-swap instructions (lane xor 16, 32) instead of LDS permutes;
//   * axis 1: two 8-element chunks per thread and iteration, so four 16-byte
//     loads are in flight per lane;
//   * axis 0: each wave owns a strip of 32 columns and walks down it in steps
//     of 64 rows (one Hadamard block of rows at most), prefetching the next
//     step; the four waves of a workgroup sit side by side, so a workgroup
//     reads 512 contiguous bytes of every row; the packed codes of up to 256
//     rows are gathered in LDS and leave as runs of 128 bytes per column.
//     Block orders 128 and 256 hold all 256 rows of the strip at once: the last one or
//     two butterfly stages pair the registers of different 64-row steps.
// Covers block orders up to 256 on both axes (axis 0: column counts that are multiples of
// 4); everything else stays with the generic kernels.

#include "common.hpp"
#include "lane_ops.hpp"

namespace hdqt {

namespace {

constexpr int kThreads = 256;
using namespace lanes;

// ---------------------------------------------------------------------------
// axis 1: the tensor is one flat array of 8-element chunks; a wave covers 512
// consecutive elements, so blocks of up to 512 never leave a wave (the library
// caps the order at 256).  Requires an even row length when b <= 4.
// ---------------------------------------------------------------------------

struct RowCtx {
    const QuantArgs* q;
    int64_t total;
    int log2n;
    float qminf, qmaxf, magic, inv;
    uint32_t flip1, flip2, flip4, flip8;
};

// One iteration of a workgroup: kRowUnroll chunks per thread, chunk index
// base + u*stride + thread.  GUARD = false: every chunk of the iteration lies
// wholly inside the tensor, loads and stores are unconditional.
template <int U>
struct RowRegs {
    float v[U][8];
};

template <int U, bool GUARD>
__device__ __forceinline__ void row_load(RowRegs<U>& r, const RowCtx& x, int64_t base, int64_t stride)
{
    const QuantArgs& q = *x.q;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t e0 = (base + u * stride + threadIdx.x) << 3;
        if (!GUARD || e0 + 8 <= x.total) {
            const float4 lo = *reinterpret_cast<const float4*>(q.T + e0);
            const float4 hi = *reinterpret_cast<const float4*>(q.T + e0 + 4);
            r.v[u][0] = lo.x; r.v[u][1] = lo.y; r.v[u][2] = lo.z; r.v[u][3] = lo.w;
            r.v[u][4] = hi.x; r.v[u][5] = hi.y; r.v[u][6] = hi.z; r.v[u][7] = hi.w;
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) r.v[u][i] = (e0 + i < x.total) ? q.T[e0 + i] : 0.0f;
        }
    }
}

// Transform and reduce / quantize the chunks loaded by row_load for `base`.
template <int U, bool QUANT, bool STOCH, bool GUARD>
__device__ __forceinline__ void row_compute(RowRegs<U>& r, const RowCtx& x, int64_t base, int64_t stride,
                                            float& amax)
{
    const QuantArgs& q = *x.q;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        float* v = r.v[u];
        butterfly8(v, x.log2n);
        if (x.log2n > 3) {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = stage_dpp<1>(v[i], x.flip1);
        }
        if (x.log2n > 4) {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = stage_dpp<2>(v[i], x.flip2);
        }
        if (x.log2n > 5) {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = stage_dpp<4>(v[i], x.flip4);
        }
        if (x.log2n > 6) {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = stage_dpp<8>(v[i], x.flip8);
        }
        if (x.log2n > 7) {
#pragma unroll
            for (int i = 0; i < 8; i += 2) stage_swap<false>(v[i], v[i + 1]);
        }
    }
    if (!QUANT) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(r.v[u][i]));
        return;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t c = base + u * stride + threadIdx.x;
        const int64_t e0 = c << 3;
        if (GUARD && e0 >= x.total) continue;
        uint32_t rnd[4] = {0, 0, 0, 0};
        if (STOCH)
            philox4x32_10((uint32_t)c, (uint32_t)(c >> 32), q.tensor_id, 0u, q.seed_lo, q.seed_hi, rnd);
        uint32_t cw[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
            cw[i] = code_word<STOCH>(r.v[u][i], x.inv, x.qminf, x.qmaxf, x.magic,
                                     sr_halfword(rnd, (uint32_t)i));
        const bool full = !GUARD || (e0 + 8 <= x.total);
        if (q.b <= 4) {
            const uint32_t w = pack_nibbles(cw);
            if (full) {
                reinterpret_cast<uint32_t*>(q.codes)[c] = w;
            } else {
                for (int i = 0; i < 8 && e0 + i < x.total; i += 2)
                    q.codes[(e0 + i) >> 1] = (uint8_t)(w >> (4 * i));
            }
        } else {
            const uint32_t w0 = pack_bytes(cw), w1 = pack_bytes(cw + 4);
            if (full) {
                reinterpret_cast<uint2*>(q.codes)[c] = make_uint2(w0, w1);
            } else {
                for (int i = 0; i < 8 && e0 + i < x.total; ++i)
                    q.codes[e0 + i] = (uint8_t)((i < 4 ? w0 : w1) >> (8 * (i & 3)));
            }
        }
    }
}

template <int U, bool QUANT, bool STOCH>
__global__ __launch_bounds__(kThreads) void fwht_row_fast_kernel(QuantArgs q)
{
    __shared__ float red[kThreads / kWave];
    const int lane = threadIdx.x & 63;
    RowCtx x;
    x.q = &q;
    x.total = q.rows * q.cols;
    x.log2n = q.log2n;
    x.qminf = (float)(-(1 << (q.b - 1)));
    x.qmaxf = (float)((1 << (q.b - 1)) - 1);
    x.magic = kMagic + (q.b <= 4 ? 8.0f : 128.0f);
    x.flip1 = (uint32_t)(lane & 1) << 31;
    x.flip2 = (uint32_t)(lane & 2) << 30;
    x.flip4 = (uint32_t)(lane & 4) << 29;
    x.flip8 = (uint32_t)(lane & 8) << 28;
    x.inv = 0.0f;
    const int64_t nchunks = (x.total + 7) >> 3;
    const int64_t nfull = x.total >> 3;
    // Iteration `it` of the tensor covers chunks [it*256*U, (it+1)*256*U): a contiguous
    // span per workgroup and iteration, chunk = it*256*U + u*256 + thread.
    // Pass 2 walks the iterations from the end of the tensor to the start: the part
    // pass 1 read last is the part most likely still held by the memory-side cache.
    const int64_t stride = kThreads;
    const int64_t per_iter = (int64_t)kThreads * U;
    const int64_t n_iter = (nchunks + per_iter - 1) / per_iter;
    auto base_of = [&](int64_t it) { return (QUANT ? (n_iter - 1 - it) : it) * per_iter; };
    auto guarded = [&](int64_t base) { return base + (U - 1) * stride + kThreads > nfull; };

    // software pipeline: the loads of the next iteration are issued before the
    // current one is transformed, so requests stay outstanding during the arithmetic
    int64_t it = blockIdx.x;
    RowRegs<U> cur, nxt;
    bool g_cur = false;
    if (it < n_iter) {
        g_cur = guarded(base_of(it));
        if (g_cur) row_load<U, true>(cur, x, base_of(it), stride);
        else row_load<U, false>(cur, x, base_of(it), stride);
    }
    if (QUANT) {
        const Scaling sc = load_scaling(q.meta, q.clip, q.b);
        publish_scale(q, sc);
        x.inv = sc.inv;
    }
    float amax = 0.0f;
    while (it < n_iter) {
        const int64_t it_next = it + gridDim.x;
        bool g_nxt = false;
        if (it_next < n_iter) {
            g_nxt = guarded(base_of(it_next));
            if (g_nxt) row_load<U, true>(nxt, x, base_of(it_next), stride);
            else row_load<U, false>(nxt, x, base_of(it_next), stride);
        }
        if (g_cur) row_compute<U, QUANT, STOCH, true>(cur, x, base_of(it), stride, amax);
        else row_compute<U, QUANT, STOCH, false>(cur, x, base_of(it), stride, amax);
        cur = nxt;
        g_cur = g_nxt;
        it = it_next;
    }
    if (!QUANT) block_atomic_max(amax, q.meta, red);
}

// ---------------------------------------------------------------------------
// axis 0: T[D, cols] -> codes[cols, D].  Wave w of a workgroup owns columns
// [32*wc, 32*wc+32) of the workgroup's strip and rows [64*SUBS*wr, +64*SUBS),
// (wc, wr) = (w % WC, w / WC).  Lane (rg, cg) = (lane / 8, lane % 8) holds rows
// 8*rg .. 8*rg+7 of columns 4*cg .. 4*cg+3 of the current 64-row step.
// Requires: block order <= 64, cols % 4 == 0, D even when b <= 4.
// ---------------------------------------------------------------------------
struct ColStep {
    float v[4][8];       // [column][row]
};

template <bool GUARD>
__device__ __forceinline__ void col_load(ColStep& s, const float* T, int64_t D, int64_t cols,
                                         int64_t row0, int64_t col0)
{
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
        if (!GUARD || (row0 + i < D && col0 < cols))
            x = *reinterpret_cast<const float4*>(T + (row0 + i) * cols + col0);
        s.v[0][i] = x.x; s.v[1][i] = x.y; s.v[2][i] = x.z; s.v[3][i] = x.w;
    }
}

__device__ __forceinline__ void col_transform(ColStep& s, int log2n, uint32_t flip8)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) butterfly8(s.v[j], log2n);
    if (log2n > 3) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 8; ++i) s.v[j][i] = stage_dpp<8>(s.v[j][i], flip8);
    }
    if (log2n > 4) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 8; i += 2) stage_swap<false>(s.v[j][i], s.v[j][i + 1]);
    }
    if (log2n > 5) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 8; i += 2) stage_swap<true>(s.v[j][i], s.v[j][i + 1]);
    }
}

// Quantize one 64-row step of the wave's strip (already transformed) and put its packed codes
// into the wave's LDS staging area: the step's 8 codes of a lane and column are one dword
// (b <= 4) or two.
template <bool STOCH, bool B4>
__device__ __forceinline__ void col_emit(const ColStep& cur, const QuantArgs& q, float inv, float qminf,
                                         float qmaxf, float magic, int64_t row0, int64_t col0, int sub,
                                         int rg, int cg, uint32_t* stage_w, int stage_pitch)
{
    const int64_t cols = q.cols;
    uint32_t cw[4][8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        // the lane's four elements of this row, e .. e+3 with e % 4 == 0, lie in
        // one Philox block: its words (e%8)/2 and (e%8)/2 + 1
        uint32_t w01[2] = {0u, 0u};
        if (STOCH) {
            const int64_t e = (row0 + i) * cols + col0;
            const uint64_t blk = (uint64_t)e >> 3;
            uint32_t rnd[4];
            philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), q.tensor_id, 0u, q.seed_lo,
                          q.seed_hi, rnd);
            const bool upper = (e & 4) != 0;
            w01[0] = upper ? rnd[2] : rnd[0];
            w01[1] = upper ? rnd[3] : rnd[1];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t u = (w01[j >> 1] >> (16 * (j & 1))) & 0xFFFFu;
            cw[j][i] = code_word<STOCH>(cur.v[j][i], inv, qminf, qmaxf, magic, u);
        }
    }
    // dword index inside the column's run: 8 codes are 1 (b <= 4) or 2 dwords
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        uint32_t* dst = stage_w + (cg * 4 + j) * stage_pitch;
        if (B4) {
            dst[sub * 8 + rg] = pack_nibbles(cw[j]);
        } else {
            dst[(sub * 8 + rg) * 2] = pack_bytes(cw[j]);
            dst[(sub * 8 + rg) * 2 + 1] = pack_bytes(cw[j] + 4);
        }
    }
}

// Block orders 128 and 256: the wave's 256 rows are loaded whole (the same lane holds the same
// row of every 64-row step, so strides 64 and 128 pair registers), each step is transformed
// up to stride 32 as above, and the last one or two stages run across the steps.  No
// prefetch inside the wave: 128 registers of loads are in flight from the start, and the
// other waves of the SIMD cover the arithmetic.
template <bool QUANT, bool STOCH, bool B4, bool GUARD>
__device__ __forceinline__ float col_strip_wide(const QuantArgs& q, float inv, int64_t tile_row0,
                                                int64_t col0, int lane, uint32_t* stage_w, int stage_pitch)
{
    const int64_t D = q.rows, cols = q.cols;
    const int cg = lane & 7, rg = lane >> 3;
    const float qminf = (float)(-(1 << (q.b - 1))), qmaxf = (float)((1 << (q.b - 1)) - 1);
    const float magic = kMagic + (B4 ? 8.0f : 128.0f);
    const uint32_t flip8 = (uint32_t)(lane & 8) << 28;
    float amax = 0.0f;

    ColStep st[4];
#pragma unroll
    for (int sub = 0; sub < 4; ++sub)
        col_load<GUARD>(st[sub], q.T, D, cols, tile_row0 + sub * 64 + rg * 8, col0);
#pragma unroll
    for (int sub = 0; sub < 4; ++sub) col_transform(st[sub], 6, flip8);
    const bool order256 = q.log2n > 7;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            // stride 64: steps (0, 1) and (2, 3); stride 128: steps (0, 2) and (1, 3)
            float a0 = st[0].v[j][i], a1 = st[1].v[j][i], a2 = st[2].v[j][i], a3 = st[3].v[j][i];
            const float s01 = a0 + a1, d01 = a0 - a1, s23 = a2 + a3, d23 = a2 - a3;
            a0 = s01; a1 = d01; a2 = s23; a3 = d23;
            if (order256) {
                const float s02 = a0 + a2, d02 = a0 - a2, s13 = a1 + a3, d13 = a1 - a3;
                a0 = s02; a2 = d02; a1 = s13; a3 = d13;
            }
            st[0].v[j][i] = a0; st[1].v[j][i] = a1; st[2].v[j][i] = a2; st[3].v[j][i] = a3;
        }
    if (!QUANT) {
#pragma unroll
        for (int sub = 0; sub < 4; ++sub)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(st[sub].v[j][i]));
    } else {
#pragma unroll
        for (int sub = 0; sub < 4; ++sub)
            col_emit<STOCH, B4>(st[sub], q, inv, qminf, qmaxf, magic, tile_row0 + sub * 64 + rg * 8, col0, sub, rg,
                                cg, stage_w, stage_pitch);
    }
    return amax;
}

// Load, transform and (QUANT) quantize the wave's strip; packed codes go to the
// wave's LDS staging area `stage_w` ([32 columns][pitch dwords]); returns max|y|.
template <bool QUANT, bool STOCH, bool B4, int SUBS, bool GUARD>
__device__ __forceinline__ float col_strip(const QuantArgs& q, float inv, int64_t tile_row0,
                                           int64_t col0, int lane, uint32_t* stage_w, int stage_pitch)
{
    const int64_t D = q.rows, cols = q.cols;
    const int cg = lane & 7, rg = lane >> 3;
    const int log2n = q.log2n;
    const float qminf = (float)(-(1 << (q.b - 1))), qmaxf = (float)((1 << (q.b - 1)) - 1);
    const float magic = kMagic + (B4 ? 8.0f : 128.0f);
    const uint32_t flip8 = (uint32_t)(lane & 8) << 28;
    float amax = 0.0f;

    ColStep cur, nxt;
    col_load<GUARD>(cur, q.T, D, cols, tile_row0 + rg * 8, col0);
#pragma unroll
    for (int sub = 0; sub < SUBS; ++sub) {
        const int64_t row0 = tile_row0 + sub * 64 + rg * 8;
        if (sub + 1 < SUBS) col_load<GUARD>(nxt, q.T, D, cols, row0 + 64, col0);
        col_transform(cur, log2n, flip8);
        if (!QUANT) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(cur.v[j][i]));
        } else {
            col_emit<STOCH, B4>(cur, q, inv, qminf, qmaxf, magic, row0, col0, sub, rg, cg, stage_w, stage_pitch);
        }
        if (sub + 1 < SUBS) cur = nxt;
    }
    return amax;
}

template <bool QUANT, bool STOCH, bool B4, int SUBS, bool WIDEN = false>
__global__ __launch_bounds__(kThreads) void fwht_col_fast_kernel(QuantArgs q, int WC)
{
    static_assert(!WIDEN || SUBS == 4, "block orders 128 and 256 span the strip's 256 rows");
    __shared__ float red[kThreads / kWave];
    constexpr int kDw = B4 ? 1 : 2;          // dwords per 8 codes
    constexpr int kPitch = SUBS * 8 * kDw + 1;
    __shared__ uint32_t stage[QUANT ? 4 : 1][QUANT ? 32 * kPitch : 1];

    const int64_t D = q.rows, cols = q.cols;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wc = wave % WC, wr = wave / WC;
    const int WR = 4 / WC;
    // pass 2 walks the tensor from its end to its start (see the axis-1 kernel)
    const int64_t by = QUANT ? (gridDim.y - 1 - blockIdx.y) : blockIdx.y;
    const int64_t bx = QUANT ? (gridDim.x - 1 - blockIdx.x) : blockIdx.x;
    const int64_t tile_row0 = (by * WR + wr) * (64 * SUBS);
    const int64_t strip_col0 = (bx * WC + wc) * 32;
    const int64_t col0 = strip_col0 + (lane & 7) * 4;

    float inv = 0.0f;
    if (QUANT) {
        const Scaling sc = load_scaling(q.meta, q.clip, q.b);
        publish_scale(q, sc);
        inv = sc.inv;
    }
    uint32_t* stage_w = QUANT ? stage[wave] : nullptr;
    float amax;
    const bool inside = tile_row0 + 64 * SUBS <= D && strip_col0 + 32 <= cols;
    if constexpr (WIDEN) {
        if (inside) amax = col_strip_wide<QUANT, STOCH, B4, false>(q, inv, tile_row0, col0, lane, stage_w, kPitch);
        else amax = col_strip_wide<QUANT, STOCH, B4, true>(q, inv, tile_row0, col0, lane, stage_w, kPitch);
    } else {
        if (inside) amax = col_strip<QUANT, STOCH, B4, SUBS, false>(q, inv, tile_row0, col0, lane, stage_w, kPitch);
        else amax = col_strip<QUANT, STOCH, B4, SUBS, true>(q, inv, tile_row0, col0, lane, stage_w, kPitch);
    }

    if (!QUANT) {
        block_atomic_max(amax, q.meta, red);
        return;
    }
    __syncthreads();

    // ---- store: 16-byte (b <= 4) or 32-byte (b > 4) units, 2*SUBS units per column
    const int64_t pitch = B4 ? (D >> 1) : D;
    constexpr int unit_bytes = B4 ? 16 : 32;
    constexpr int units = 2 * SUBS;
#pragma unroll
    for (int it = 0; it < SUBS; ++it) {
        const int idx = it * 64 + lane;
        const int col_l = idx / units, part = idx - col_l * units;
        const int64_t c = strip_col0 + col_l;
        if (c >= cols) continue;
        const int64_t byte0 = (B4 ? (tile_row0 >> 1) : tile_row0) + part * unit_bytes;
        const int64_t valid = pitch - byte0;
        if (valid <= 0) continue;
        uint8_t* dst = q.codes + c * pitch + byte0;
        const uint32_t* src = stage_w + col_l * kPitch + part * (unit_bytes / 4);
        if ((pitch & 15) == 0 && valid >= unit_bytes) {
            uint4* d4 = reinterpret_cast<uint4*>(dst);
            d4[0] = make_uint4(src[0], src[1], src[2], src[3]);
            if (unit_bytes == 32) d4[1] = make_uint4(src[4], src[5], src[6], src[7]);
        } else {
            for (int k = 0; k < unit_bytes && k < valid; ++k)
                dst[k] = (uint8_t)(src[k >> 2] >> (8 * (k & 3)));
        }
    }
}

int clamp_grid(int64_t blocks, int64_t cap)
{
    if (blocks < 1) blocks = 1;
    return (int)(blocks < cap ? blocks : cap);
}

template <int SUBS, bool STOCH, bool WIDEN = false>
hipError_t launch_col(const QuantArgs& q, hipStream_t stream)
{
    const int64_t D = q.rows;
    int WC = (int)((q.cols + 31) / 32);
    WC = WC >= 4 ? 4 : (WC >= 2 ? 2 : 1);
    const int WR = 4 / WC;
    const dim3 grid((unsigned)((q.cols + 32 * WC - 1) / (32 * WC)),
                    (unsigned)((D + 64 * SUBS * WR - 1) / (64 * SUBS * WR)));
    {
        ProfileScope ps(K_COL_ABSMAX, stream);
        hipLaunchKernelGGL((fwht_col_fast_kernel<false, false, true, SUBS, WIDEN>), grid, dim3(kThreads), 0,
                           stream, q, WC);
    }
    ProfileScope ps(K_COL_QUANT, stream);
    if (q.b <= 4)
        hipLaunchKernelGGL((fwht_col_fast_kernel<true, STOCH, true, SUBS, WIDEN>), grid, dim3(kThreads), 0,
                           stream, q, WC);
    else
        hipLaunchKernelGGL((fwht_col_fast_kernel<true, STOCH, false, SUBS, WIDEN>), grid, dim3(kThreads), 0,
                           stream, q, WC);
    return hipGetLastError();
}

template <int U>
hipError_t launch_row(const QuantArgs& q, int64_t nchunks, hipStream_t stream)
{
    const int64_t per_block = (int64_t)kThreads * U;
    const int grid = clamp_grid((nchunks + per_block - 1) / per_block, 1 << 16);
    {
        ProfileScope ps(K_ROW_ABSMAX, stream);
        hipLaunchKernelGGL((fwht_row_fast_kernel<U, false, false>), dim3(grid), dim3(kThreads), 0, stream, q);
    }
    ProfileScope ps(K_ROW_QUANT, stream);
    if (q.stochastic)
        hipLaunchKernelGGL((fwht_row_fast_kernel<U, true, true>), dim3(grid), dim3(kThreads), 0, stream, q);
    else
        hipLaunchKernelGGL((fwht_row_fast_kernel<U, true, false>), dim3(grid), dim3(kThreads), 0, stream, q);
    return hipGetLastError();
}

} // namespace

bool quantize_fast_eligible(const QuantArgs& q)
{
    const int64_t D = q.axis ? q.cols : q.rows;
    if (D & 1) return false;
    if (q.axis == 1) return q.log2n <= 8;
    return q.log2n <= 8 && (q.cols & 3) == 0;
}

// Pass 1 and pass 2 of one tensor (the calibration record must already be zero).
hipError_t launch_quantize_fast(const QuantArgs& q, hipStream_t stream)
{
    if (q.axis == 1) {
        const int64_t nchunks = (q.rows * q.cols + 7) >> 3;
        // four chunks per thread when that still leaves every CU several workgroups
        if (nchunks >= (int64_t)kThreads * 4 * 4096) return launch_row<4>(q, nchunks, stream);
        return launch_row<1>(q, nchunks, stream);
    }
    // block orders 128 and 256: strips of 256 rows, held whole
    if (q.log2n > 6) return q.stochastic ? launch_col<4, true, true>(q, stream) : launch_col<4, false, true>(q, stream);
    // long strips (256 rows per wave) when that still gives every CU several waves
    const int64_t waves_long = ((q.cols + 31) / 32) * ((q.rows + 255) / 256);
    if (waves_long >= 4096)
        return q.stochastic ? launch_col<4, true>(q, stream) : launch_col<4, false>(q, stream);
    return q.stochastic ? launch_col<1, true>(q, stream) : launch_col<1, false>(q, stream);
}

} // namespace hdqt
