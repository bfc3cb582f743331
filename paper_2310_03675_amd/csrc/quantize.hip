// Hadamard-domain quantization kernels (gfx950).
//
// Paper, Methodology section: y = x H along the contraction dimension with
// H = BlockDiag(H_k,..,H_k) in Sylvester form; Q(y) with alpha calibrated on
// the maximum of the tensor; nearest or stochastic rounding.
//
// This file holds the kernels for the shapes the tuned kernels (quantize_fast.hip,
// quantize_dual.hip) do not take -- odd contraction lengths, block orders 128 and
// 256 along axis 0, column counts that are not multiples of 4 -- and the fill kernel.
//
// Two passes over the source tensor, both HBM-bound:
//   pass 1  transform in registers, reduce max|y|, one atomicMax per workgroup
//   pass 2  transform again, scale, round, clamp, pack, store codes
// The transformed values never go to memory.
//
// The butterfly runs with strides 1, 2, 4, ..., n/2 in that order: this fixes
// the binary32 rounding to the balanced pairwise tree over the signed terms in
// natural index order.  A thread owns 8 consecutive contraction indices
// (strides 1, 2, 4 in registers); larger strides pair threads.

#include "common.hpp"

namespace hdqt {

namespace {

constexpr int kThreads = 256;

// strides 1, 2, 4 over eight register values, limited to strides < 2^log2n
__device__ __forceinline__ void butterfly8(float v[8], int log2n)
{
    if (log2n >= 1) {
#pragma unroll
        for (int i = 0; i < 8; i += 2) {
            const float a = v[i], c = v[i + 1];
            v[i] = a + c;
            v[i + 1] = a - c;
        }
    }
    if (log2n >= 2) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (!(i & 2)) {
                const float a = v[i], c = v[i + 2];
                v[i] = a + c;
                v[i + 2] = a - c;
            }
        }
    }
    if (log2n >= 3) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float a = v[i], c = v[i + 4];
            v[i] = a + c;
            v[i + 4] = a - c;
        }
    }
}

// one cross-lane stage: the lane whose `mask` bit is clear holds the lower half
__device__ __forceinline__ float pair_lanes(float own, int lane, int mask)
{
    const float other = __shfl_xor(own, mask, kWave);
    return (lane & mask) ? (other - own) : (own + other);
}

// ---------------------------------------------------------------------------
// Contraction along columns of the source (axis 0): T[D, cols] -> codes[cols, D].
// A workgroup owns 256 rows x 32 columns.  Thread (rg, cg) holds rows
// rg*8 .. rg*8+7 of columns cg*4 .. cg*4+3; strides 8, 16, 32 pair lanes of a
// wave, strides 64, 128 pair waves through LDS.  The packed codes are
// transposed through LDS so that each column's 256 codes leave as one run.
// Requires: D even when b <= 4.
// ---------------------------------------------------------------------------
constexpr int kColTileRows = 256;
constexpr int kColTileCols = 32;

template <bool QUANT>
__global__ __launch_bounds__(kThreads) void fwht_col_kernel(QuantArgs q)
{
    __shared__ float red[kThreads / kWave];
    __shared__ float xch[32 * kThreads];            // cross-wave exchange, value-major
    __shared__ uint32_t stage[kColTileCols][2 * 32 + 1];

    const int64_t D = q.rows, cols = q.cols;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int cg = tid & 7, rg = tid >> 3;
    const int64_t tile_row0 = (int64_t)blockIdx.y * kColTileRows;
    const int64_t tile_col0 = (int64_t)blockIdx.x * kColTileCols;
    const int64_t row0 = tile_row0 + rg * 8;
    const int64_t col0 = tile_col0 + cg * 4;
    const int log2n = q.log2n;
    const int qmin = -(1 << (q.b - 1)), qmax = (1 << (q.b - 1)) - 1;
    const bool vec = ((cols & 3) == 0);

    Scaling sc{};
    if (QUANT) {
        sc = load_scaling(q.meta, q.clip, q.b);
        publish_scale(q, sc);
    }

    float v[4][8];   // [column][row]
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int64_t r = row0 + i;
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r < D) {
            const float* p = q.T + r * cols + col0;
            if (vec) {
                if (col0 < cols) x = *reinterpret_cast<const float4*>(p);
            } else {
                if (col0 + 0 < cols) x.x = p[0];
                if (col0 + 1 < cols) x.y = p[1];
                if (col0 + 2 < cols) x.z = p[2];
                if (col0 + 3 < cols) x.w = p[3];
            }
        }
        v[0][i] = x.x; v[1][i] = x.y; v[2][i] = x.z; v[3][i] = x.w;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) butterfly8(v[j], log2n);
    // strides 8, 16, 32: partner thread = tid ^ 8, 16, 32 (same wave)
    for (int st = 3; st < log2n && st < 6; ++st) {
        const int mask = 8 << (st - 3);
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 8; ++i) v[j][i] = pair_lanes(v[j][i], lane, mask);
    }
    // strides 64, 128: partner thread = tid ^ 64, 128 (another wave)
    for (int st = 6; st < log2n; ++st) {
        const int mask = 64 << (st - 6);
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 8; ++i) xch[(j * 8 + i) * kThreads + tid] = v[j][i];
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float other = xch[(j * 8 + i) * kThreads + (tid ^ mask)];
                v[j][i] = (tid & mask) ? (other - v[j][i]) : (v[j][i] + other);
            }
    }

    if (!QUANT) {
        float amax = 0.0f;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(v[j][i]));
        block_atomic_max(amax, q.meta, red);
        return;
    }

    // ---- quantize: element e = r * cols + c draws from Philox block e >> 3 ----
    uint32_t packed[4][2];
#pragma unroll
    for (int j = 0; j < 4; ++j) packed[j][0] = packed[j][1] = 0u;
    uint32_t rnd[4] = {0, 0, 0, 0};
    int64_t cached_blk = -1;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t u = 0;
            if (q.stochastic) {
                const int64_t e = (row0 + i) * cols + (col0 + j);
                const int64_t blk = e >> 3;
                if (blk != cached_blk) {
                    philox4x32_10((uint32_t)blk, (uint32_t)((uint64_t)blk >> 32), q.tensor_id, 0u,
                                  q.seed_lo, q.seed_hi, rnd);
                    cached_blk = blk;
                }
                u = sr_halfword(rnd, (uint32_t)(e & 7));
            }
            const int code =
                quantize_value(v[j][i], sc.inv, qmin, qmax, q.stochastic != 0, u);
            if (q.b <= 4)
                packed[j][0] |= ((uint32_t)code & 0xFu) << (4 * i);
            else
                packed[j][i >> 2] |= ((uint32_t)code & 0xFFu) << (8 * (i & 3));
        }
    }

    // ---- transpose the packed codes through LDS and store column runs ----
    const int dw = (q.b <= 4) ? 1 : 2;           // dwords per (column, row group)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        stage[cg * 4 + j][rg * dw] = packed[j][0];
        if (dw == 2) stage[cg * 4 + j][rg * dw + 1] = packed[j][1];
    }
    __syncthreads();

    const int col_l = tid >> 3, part = tid & 7;
    const int64_t c = tile_col0 + col_l;
    if (c >= cols) return;
    const int64_t pitch = (q.b <= 4) ? (D >> 1) : D;
    const int run_bytes = (q.b <= 4) ? 128 : 256;            // bytes of this column in the tile
    const int part_bytes = run_bytes / 8;                    // 16 or 32
    const int64_t byte0 = ((q.b <= 4) ? (tile_row0 >> 1) : tile_row0) + part * part_bytes;
    const int64_t valid = pitch - byte0;                     // bytes of this part inside the line
    if (valid <= 0) return;
    uint8_t* dst = q.codes + c * pitch + byte0;
    const uint32_t* src = &stage[col_l][part * (part_bytes / 4)];
    if ((pitch & 15) == 0 && valid >= part_bytes) {
        uint4* d4 = reinterpret_cast<uint4*>(dst);
        d4[0] = make_uint4(src[0], src[1], src[2], src[3]);
        if (part_bytes == 32) d4[1] = make_uint4(src[4], src[5], src[6], src[7]);
    } else {
        for (int k = 0; k < part_bytes && k < valid; ++k)
            dst[k] = (uint8_t)(src[k >> 2] >> (8 * (k & 3)));
    }
}

// ---------------------------------------------------------------------------
// No transform and any shape (used when the contraction length is odd, where
// the block order is 1 and a line of codes ends in a pad nibble).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void absmax_plain_kernel(QuantArgs q)
{
    __shared__ float red[kThreads / kWave];
    const int64_t total = q.rows * q.cols;
    float amax = 0.0f;
    for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < total;
         e += (int64_t)gridDim.x * kThreads)
        amax = fmaxf(amax, fabsf(q.T[e]));
    block_atomic_max(amax, q.meta, red);
}

__global__ __launch_bounds__(kThreads) void quant_plain_kernel(QuantArgs q)
{
    const int64_t D = q.axis ? q.cols : q.rows;
    const int64_t lines = q.axis ? q.rows : q.cols;
    const int per_byte = (q.b <= 4) ? 2 : 1;
    const int64_t pitch = (q.b <= 4) ? ((D + 1) >> 1) : D;
    const int qmin = -(1 << (q.b - 1)), qmax = (1 << (q.b - 1)) - 1;
    const Scaling sc = load_scaling(q.meta, q.clip, q.b);
    publish_scale(q, sc);
    for (int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x; idx < lines * pitch;
         idx += (int64_t)gridDim.x * kThreads) {
        const int64_t line = idx / pitch, jb = idx - line * pitch;
        uint32_t byte = 0;
        for (int h = 0; h < per_byte; ++h) {
            const int64_t d = jb * per_byte + h;
            if (d >= D) break;
            const int64_t e = q.axis ? (line * q.cols + d) : (d * q.cols + line);
            uint32_t u = 0;
            if (q.stochastic) {
                uint32_t rnd[4];
                const uint64_t blk = (uint64_t)e >> 3;
                philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), q.tensor_id, 0u, q.seed_lo,
                              q.seed_hi, rnd);
                u = sr_halfword(rnd, (uint32_t)(e & 7));
            }
            const int code =
                quantize_value(q.T[e], sc.inv, qmin, qmax, q.stochastic != 0, u);
            byte |= (q.b <= 4) ? (((uint32_t)code & 0xFu) << (4 * h)) : ((uint32_t)code & 0xFFu);
        }
        q.codes[idx] = (uint8_t)byte;
    }
}

__global__ void zero2_kernel(uint32_t* a, int64_t na, uint32_t* b, int64_t nb)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < na + nb;
         i += (int64_t)gridDim.x * blockDim.x) {
        if (i < na) a[i] = 0u;
        else b[i - na] = 0u;
    }
}

int clamp_grid(int64_t blocks, int64_t cap)
{
    if (blocks < 1) blocks = 1;
    return (int)(blocks < cap ? blocks : cap);
}

} // namespace

hipError_t launch_zero2(uint32_t* a, int64_t na, uint32_t* b, int64_t nb, hipStream_t stream)
{
    if (!b) nb = 0;
    const int grid = clamp_grid((na + nb + 255) / 256, 2048);
    ProfileScope ps(K_FILL, stream);
    hipLaunchKernelGGL(zero2_kernel, dim3(grid), dim3(256), 0, stream, a, na, b, nb);
    return hipGetLastError();
}

// Pass 1 and pass 2 of one tensor.  The calibration record must be zero.
hipError_t launch_quantize(const QuantArgs& q, hipStream_t stream)
{
    const int64_t D = q.axis ? q.cols : q.rows;
    const int64_t total = q.rows * q.cols;
    if (quantize_fast_eligible(q)) return launch_quantize_fast(q, stream);

    if (D & 1) {   // odd contraction length: block order is 1
        const int grid1 = clamp_grid((total + kThreads - 1) / kThreads, 4096);
        {
            ProfileScope ps(K_PLAIN_ABSMAX, stream);
            hipLaunchKernelGGL(absmax_plain_kernel, dim3(grid1), dim3(kThreads), 0, stream, q);
        }
        const int64_t lines = q.axis ? q.rows : q.cols;
        const int64_t bytes = lines * ((q.b <= 4) ? ((D + 1) >> 1) : D);
        const int grid2 = clamp_grid((bytes + kThreads - 1) / kThreads, 4096);
        ProfileScope ps(K_PLAIN_QUANT, stream);
        hipLaunchKernelGGL(quant_plain_kernel, dim3(grid2), dim3(kThreads), 0, stream, q);
        return hipGetLastError();
    }
    // (axis 1 with an even row length is always taken by the tuned kernel: what is left
    // here is axis 0 with a block order above 64 or a column count that is not a
    // multiple of 4)
    const dim3 grid((unsigned)((q.cols + kColTileCols - 1) / kColTileCols),
                    (unsigned)((D + kColTileRows - 1) / kColTileRows));
    {
        ProfileScope ps(K_COL_ABSMAX, stream);
        hipLaunchKernelGGL(fwht_col_kernel<false>, grid, dim3(kThreads), 0, stream, q);
    }
    ProfileScope ps(K_COL_QUANT, stream);
    hipLaunchKernelGGL(fwht_col_kernel<true>, grid, dim3(kThreads), 0, stream, q);
    return hipGetLastError();
}

} // namespace hdqt
