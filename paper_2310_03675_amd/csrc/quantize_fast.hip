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
// Covers block orders up to 256 (axis 1) and 64 (axis 0); everything else
// stays with the generic kernels.

#include "common.hpp"

namespace hdqt {

namespace {

constexpr int kThreads = 256;
typedef unsigned v2u __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float as_f(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t as_u(float f) { return __float_as_uint(f); }

template <int CTRL>
__device__ __forceinline__ float dpp_move(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}

// value held by lane (lane ^ M), M in {1, 2, 4, 8}
template <int M>
__device__ __forceinline__ float lane_xor(float x)
{
    if (M == 1) return dpp_move<0xB1>(x);                      // quad_perm [1,0,3,2]
    if (M == 2) return dpp_move<0x4E>(x);                      // quad_perm [2,3,0,1]
    if (M == 4) return dpp_move<0x1B>(dpp_move<0x141>(x));     // half-row mirror, then quad reverse
    return dpp_move<0x128>(x);                                 // row rotate by 8
}

// Butterfly stage pairing lane and lane ^ M.  `flip` is 0x80000000 in the lane
// that holds the upper half (it computes other - own) and 0 in the other.
template <int M>
__device__ __forceinline__ float stage_dpp(float own, uint32_t flip)
{
    return lane_xor<M>(own) + as_f(as_u(own) ^ flip);
}

// Butterfly stage pairing lane and lane ^ 16 (W32 = false) or lane ^ 32 (true),
// on two values at once.  The swap brings, into one lane, the two halves of a
// pair (of `a` in the lower lanes, of `b` in the upper lanes); sum and
// difference are formed there and swapped back.
template <bool W32>
__device__ __forceinline__ void stage_swap(float& a, float& b)
{
    v2u r = W32 ? __builtin_amdgcn_permlane32_swap(as_u(a), as_u(b), false, false)
                : __builtin_amdgcn_permlane16_swap(as_u(a), as_u(b), false, false);
    const float lo = as_f(r[0]), hi = as_f(r[1]);
    const float s = lo + hi, d = lo - hi;
    r = W32 ? __builtin_amdgcn_permlane32_swap(as_u(s), as_u(d), false, false)
            : __builtin_amdgcn_permlane16_swap(as_u(s), as_u(d), false, false);
    a = as_f(r[0]);
    b = as_f(r[1]);
}

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
        for (int i = 0; i < 8; ++i)
            if (!(i & 2)) {
                const float a = v[i], c = v[i + 2];
                v[i] = a + c;
                v[i + 2] = a - c;
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

__device__ __forceinline__ float wave_max(float m)
{
    m = fmaxf(m, lane_xor<1>(m));
    m = fmaxf(m, lane_xor<2>(m));
    m = fmaxf(m, lane_xor<4>(m));
    m = fmaxf(m, lane_xor<8>(m));
    m = fmaxf(m, __shfl_xor(m, 16, kWave));
    m = fmaxf(m, __shfl_xor(m, 32, kWave));
    return m;
}

// One atomicMax per workgroup, and only if it can raise the current value: all
// workgroups target one word, and atomics on one address are serialised.
__device__ __forceinline__ void block_atomic_max(float m, uint32_t* target, float* smem)
{
    m = wave_max(m);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) smem[wave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        float r = smem[0];
        for (int w = 1; w < kThreads / kWave; ++w) r = fmaxf(r, smem[w]);
        const uint32_t bits = __float_as_uint(r);
        if (bits > __hip_atomic_load(target, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
            atomicMax(target, bits);
    }
}

struct Scaling {
    float inv, scale;
    bool zero;
};

__device__ __forceinline__ Scaling load_scaling(const QMeta* meta, float clip, int b)
{
    Scaling s;
    const float amax = __uint_as_float(meta->amax_bits);
    const float amax_c = clip * amax;
    s.zero = (amax_c == 0.0f);
    s.inv = s.zero ? 0.0f : inverse_step(amax_c, b);
    s.scale = s.zero ? 0.0f : amax_c / (float)(1 << (b - 1));
    return s;
}

__device__ __forceinline__ void publish_scale(const QuantArgs& q, const Scaling& s)
{
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
        q.meta->scale = s.scale;
        if (q.scale_out) *q.scale_out = s.scale;
    }
}

// ---------------------------------------------------------------------------
// axis 1: the tensor is one flat array of 8-element chunks; a wave covers 512
// consecutive elements, so blocks of up to 512 never leave a wave (the library
// caps the order at 256).  Requires an even row length when b <= 4.
// ---------------------------------------------------------------------------
constexpr int kRowUnroll = 2;

template <bool QUANT, bool STOCH>
__global__ __launch_bounds__(kThreads) void fwht_row_fast_kernel(QuantArgs q)
{
    __shared__ float red[kThreads / kWave];
    const int64_t total = q.rows * q.cols;
    const int64_t nchunks = (total + 7) >> 3;
    const int lane = threadIdx.x & 63;
    const int log2n = q.log2n;
    const int qmin = -(1 << (q.b - 1)), qmax = (1 << (q.b - 1)) - 1;
    const uint32_t flip1 = (uint32_t)(lane & 1) << 31, flip2 = (uint32_t)(lane & 2) << 30,
                   flip4 = (uint32_t)(lane & 4) << 29, flip8 = (uint32_t)(lane & 8) << 28;

    Scaling sc{};
    if (QUANT) {
        sc = load_scaling(q.meta, q.clip, q.b);
        publish_scale(q, sc);
    }
    float amax = 0.0f;
    const int64_t stride = (int64_t)gridDim.x * kThreads;

    for (int64_t base = (int64_t)blockIdx.x * kThreads; base < nchunks; base += stride * kRowUnroll) {
        float v[kRowUnroll][8];
        int64_t cidx[kRowUnroll];
#pragma unroll
        for (int u = 0; u < kRowUnroll; ++u) {
            const int64_t c = base + u * stride + threadIdx.x;
            cidx[u] = c;
            const int64_t e0 = c << 3;
            if (e0 + 8 <= total) {
                const float4 lo = *reinterpret_cast<const float4*>(q.T + e0);
                const float4 hi = *reinterpret_cast<const float4*>(q.T + e0 + 4);
                v[u][0] = lo.x; v[u][1] = lo.y; v[u][2] = lo.z; v[u][3] = lo.w;
                v[u][4] = hi.x; v[u][5] = hi.y; v[u][6] = hi.z; v[u][7] = hi.w;
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) v[u][i] = (e0 + i < total) ? q.T[e0 + i] : 0.0f;
            }
        }
#pragma unroll
        for (int u = 0; u < kRowUnroll; ++u) {
            butterfly8(v[u], log2n);
            if (log2n > 3) {
#pragma unroll
                for (int i = 0; i < 8; ++i) v[u][i] = stage_dpp<1>(v[u][i], flip1);
            }
            if (log2n > 4) {
#pragma unroll
                for (int i = 0; i < 8; ++i) v[u][i] = stage_dpp<2>(v[u][i], flip2);
            }
            if (log2n > 5) {
#pragma unroll
                for (int i = 0; i < 8; ++i) v[u][i] = stage_dpp<4>(v[u][i], flip4);
            }
            if (log2n > 6) {
#pragma unroll
                for (int i = 0; i < 8; ++i) v[u][i] = stage_dpp<8>(v[u][i], flip8);
            }
            if (log2n > 7) {
#pragma unroll
                for (int i = 0; i < 8; i += 2) stage_swap<false>(v[u][i], v[u][i + 1]);
            }
        }
        if (!QUANT) {
#pragma unroll
            for (int u = 0; u < kRowUnroll; ++u)
#pragma unroll
                for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(v[u][i]));
            continue;
        }
#pragma unroll
        for (int u = 0; u < kRowUnroll; ++u) {
            const int64_t c = cidx[u];
            const int64_t e0 = c << 3;
            if (e0 >= total) continue;
            uint32_t rnd[4] = {0, 0, 0, 0};
            if (STOCH)
                philox4x32_10((uint32_t)c, (uint32_t)(c >> 32), q.tensor_id, 0u, q.seed_lo,
                              q.seed_hi, rnd);
            int code[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                code[i] = quantize_value(v[u][i], sc.inv, qmin, qmax, STOCH,
                                         sr_halfword(rnd, (uint32_t)i));
            const bool full = (e0 + 8 <= total);
            if (q.b <= 4) {
                uint32_t w = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) w |= ((uint32_t)code[i] & 0xFu) << (4 * i);
                if (full) {
                    reinterpret_cast<uint32_t*>(q.codes)[c] = w;
                } else {
                    for (int i = 0; i < 8 && e0 + i < total; i += 2)
                        q.codes[(e0 + i) >> 1] = (uint8_t)(w >> (4 * i));
                }
            } else {
                uint32_t w0 = 0, w1 = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    w0 |= ((uint32_t)code[i] & 0xFFu) << (8 * i);
                    w1 |= ((uint32_t)code[i + 4] & 0xFFu) << (8 * i);
                }
                if (full) {
                    reinterpret_cast<uint2*>(q.codes)[c] = make_uint2(w0, w1);
                } else {
                    for (int i = 0; i < 8 && e0 + i < total; ++i) q.codes[e0 + i] = (uint8_t)code[i];
                }
            }
        }
    }
    if (!QUANT) block_atomic_max(amax, &q.meta->amax_bits, red);
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

__device__ __forceinline__ void col_load(ColStep& s, const float* T, int64_t D, int64_t cols,
                                         int64_t row0, int64_t col0)
{
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row0 + i < D && col0 < cols)
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

template <bool QUANT, bool STOCH, int SUBS>
__global__ __launch_bounds__(kThreads) void fwht_col_fast_kernel(QuantArgs q, int WC)
{
    __shared__ float red[kThreads / kWave];
    __shared__ uint32_t stage[QUANT ? 4 : 1][32][QUANT ? (SUBS * 16 + 1) : 1];

    const int64_t D = q.rows, cols = q.cols;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int cg = lane & 7, rg = lane >> 3;
    const int wc = wave % WC, wr = wave / WC;
    const int WR = 4 / WC;
    const int64_t tile_row0 = ((int64_t)blockIdx.y * WR + wr) * (64 * SUBS);
    const int64_t strip_col0 = ((int64_t)blockIdx.x * WC + wc) * 32;
    const int64_t col0 = strip_col0 + cg * 4;
    const int log2n = q.log2n;
    const int qmin = -(1 << (q.b - 1)), qmax = (1 << (q.b - 1)) - 1;
    const uint32_t flip8 = (uint32_t)(lane & 8) << 28;

    Scaling sc{};
    if (QUANT) {
        sc = load_scaling(q.meta, q.clip, q.b);
        publish_scale(q, sc);
    }
    float amax = 0.0f;

    ColStep cur, nxt;
    col_load(cur, q.T, D, cols, tile_row0 + rg * 8, col0);
#pragma unroll
    for (int sub = 0; sub < SUBS; ++sub) {
        const int64_t row0 = tile_row0 + sub * 64 + rg * 8;
        if (sub + 1 < SUBS) col_load(nxt, q.T, D, cols, row0 + 64, col0);
        col_transform(cur, log2n, flip8);
        if (!QUANT) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(cur.v[j][i]));
        } else {
            uint32_t packed[4][2];
#pragma unroll
            for (int j = 0; j < 4; ++j) packed[j][0] = packed[j][1] = 0u;
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
                    const int code = quantize_value(cur.v[j][i], sc.inv, qmin, qmax, STOCH, u);
                    if (q.b <= 4)
                        packed[j][0] |= ((uint32_t)code & 0xFu) << (4 * i);
                    else
                        packed[j][i >> 2] |= ((uint32_t)code & 0xFFu) << (8 * (i & 3));
                }
            }
            // dword index inside the column's run: 8 codes are 1 (b <= 4) or 2 dwords
            if (q.b <= 4) {
#pragma unroll
                for (int j = 0; j < 4; ++j) stage[wave][cg * 4 + j][sub * 8 + rg] = packed[j][0];
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    stage[wave][cg * 4 + j][(sub * 8 + rg) * 2] = packed[j][0];
                    stage[wave][cg * 4 + j][(sub * 8 + rg) * 2 + 1] = packed[j][1];
                }
            }
        }
        if (sub + 1 < SUBS) cur = nxt;
    }

    if (!QUANT) {
        block_atomic_max(amax, &q.meta->amax_bits, red);
        return;
    }
    __syncthreads();

    // ---- store: 16-byte (b <= 4) or 32-byte (b > 4) units, 2*SUBS units per column
    const int64_t pitch = (q.b <= 4) ? (D >> 1) : D;
    const int unit_bytes = (q.b <= 4) ? 16 : 32;
    const int units = 2 * SUBS;
#pragma unroll
    for (int it = 0; it < SUBS; ++it) {
        const int idx = it * 64 + lane;
        const int col_l = idx / units, part = idx - col_l * units;
        const int64_t c = strip_col0 + col_l;
        if (c >= cols) continue;
        const int64_t byte0 = ((q.b <= 4) ? (tile_row0 >> 1) : tile_row0) + part * unit_bytes;
        const int64_t valid = pitch - byte0;
        if (valid <= 0) continue;
        uint8_t* dst = q.codes + c * pitch + byte0;
        const uint32_t* src = &stage[wave][col_l][part * (unit_bytes / 4)];
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

template <int SUBS, bool STOCH>
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
        hipLaunchKernelGGL((fwht_col_fast_kernel<false, false, SUBS>), grid, dim3(kThreads), 0, stream, q, WC);
    }
    ProfileScope ps(K_COL_QUANT, stream);
    hipLaunchKernelGGL((fwht_col_fast_kernel<true, STOCH, SUBS>), grid, dim3(kThreads), 0, stream, q, WC);
    return hipGetLastError();
}

} // namespace

bool quantize_fast_eligible(const QuantArgs& q)
{
    const int64_t D = q.axis ? q.cols : q.rows;
    if (D & 1) return false;
    if (q.axis == 1) return q.log2n <= 8;
    return q.log2n <= 6 && (q.cols & 3) == 0;
}

// Pass 1 and pass 2 of one tensor (the calibration record must already be zero).
hipError_t launch_quantize_fast(const QuantArgs& q, hipStream_t stream)
{
    if (q.axis == 1) {
        const int64_t nchunks = (q.rows * q.cols + 7) >> 3;
        const int64_t per_block = (int64_t)kThreads * kRowUnroll;
        const int grid = clamp_grid((nchunks + per_block - 1) / per_block, 256 * 8);
        {
            ProfileScope ps(K_ROW_ABSMAX, stream);
            hipLaunchKernelGGL((fwht_row_fast_kernel<false, false>), dim3(grid), dim3(kThreads), 0, stream, q);
        }
        ProfileScope ps(K_ROW_QUANT, stream);
        if (q.stochastic)
            hipLaunchKernelGGL((fwht_row_fast_kernel<true, true>), dim3(grid), dim3(kThreads), 0, stream, q);
        else
            hipLaunchKernelGGL((fwht_row_fast_kernel<true, false>), dim3(grid), dim3(kThreads), 0, stream, q);
        return hipGetLastError();
    }
    // long strips (256 rows per wave) when that still gives every CU several waves
    const int64_t waves_long = ((q.cols + 31) / 32) * ((q.rows + 255) / 256);
    if (waves_long >= 4096)
        return q.stochastic ? launch_col<4, true>(q, stream) : launch_col<4, false>(q, stream);
    return q.stochastic ? launch_col<1, true>(q, stream) : launch_col<1, false>(q, stream);
}

} // namespace hdqt
