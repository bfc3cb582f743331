// Tiled integer matmul with a-bit accumulators on the int8 MFMA units (gfx950).
//
// Paper, Methodology section: the contraction is cut into tiles of size s and
// each tile's partial sum is kept in a low-bit accumulator; Experiments: 8-bit
// accumulators, tile 32.  Here:
//   acc[i,j] = sum_t clamp( sum_{d in tile t} qA[i,d] qB[j,d], -2^(a-1), 2^(a-1)-1 )
//   out[i,j] = float(acc[i,j]) * (scaleA*scaleB) * (1/n)
//
// Both operands are contraction-major packed codes.  A workgroup (4 waves)
// owns a 128 x 128 output tile; each wave a 64 x 64 quarter as 2 x 2 MFMA
// blocks of 32 x 32.  Codes are unpacked to int8 on their way into LDS.  Every
// tile of the contraction is padded (with zeros, in LDS only) to a multiple of
// the MFMA depth, so an MFMA never mixes two tiles; after a tile's last MFMA
// the 32-bit tile sums are clamped and added to the running totals.

#include "common.hpp"

namespace hdqt {

namespace {

typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int BM = 128, BN = 128;
constexpr int KC = 64;          // virtual contraction positions per LDS stage
constexpr int KG = 16;          // contraction depth of one MFMA
constexpr int LDP = KC + 16;    // LDS row pitch in bytes

__device__ __forceinline__ int wave_max_int(int v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = max(v, __shfl_xor(v, off, kWave));
    return v;
}

__device__ __forceinline__ int sext_nibble(uint32_t nib)
{
    return ((int)(nib << 28)) >> 28;
}

// code d of a line (generic, any width)
__device__ __forceinline__ int fetch_code(const uint8_t* line, int64_t d, int b)
{
    if (b <= 4) {
        const uint32_t byte = line[d >> 1];
        return sext_nibble((d & 1) ? (byte >> 4) : (byte & 0xFu));
    }
    return (int)(int8_t)line[d];
}

// Fill rows [row0, row0+128) x virtual positions [kv0, kv0+KC) of one operand.
// ALIGNED: s and D are multiples of 16, so virtual position == code index and
// 16 codes are 8 (b <= 4) or 16 (b > 4) aligned bytes.
template <bool ALIGNED>
__device__ __forceinline__ void load_operand(uint8_t (*lds)[LDP], const uint8_t* q, int64_t pitch,
                                             int b, int64_t R, int64_t D, int64_t row0,
                                             int64_t kv0, int64_t kv_end, int64_t s, int s_pad)
{
    const int tid = threadIdx.x;
    if (ALIGNED) {
#pragma unroll
        for (int it = 0; it < (BM * KC / 16) / kThreads; ++it) {
            const int idx = tid + it * kThreads;
            const int r = idx >> 2, ch = idx & 3;
            const int64_t row = row0 + r;
            const int64_t d = kv0 + ch * 16;
            uint32_t o[4] = {0u, 0u, 0u, 0u};
            if (row < R && d < kv_end && d < D) {
                if (b <= 4) {
                    const uint2 w = *reinterpret_cast<const uint2*>(q + row * pitch + (d >> 1));
                    const uint32_t ww[2] = {w.x, w.y};
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
#pragma unroll
                        for (int k = 0; k < 8; ++k) {
                            const int c = sext_nibble((ww[h] >> (4 * k)) & 0xFu);
                            o[h * 2 + (k >> 2)] |= ((uint32_t)c & 0xFFu) << (8 * (k & 3));
                        }
                    }
                } else {
                    const uint4 w = *reinterpret_cast<const uint4*>(q + row * pitch + d);
                    o[0] = w.x; o[1] = w.y; o[2] = w.z; o[3] = w.w;
                }
            }
            *reinterpret_cast<uint4*>(&lds[r][ch * 16]) = make_uint4(o[0], o[1], o[2], o[3]);
        }
    } else {
        // 32 consecutive virtual positions of one row per thread
        const int r = tid >> 1, half = tid & 1;
        const int64_t row = row0 + r;
        const int64_t p0 = kv0 + half * 32;
        int64_t tile = p0 / s_pad;
        int off = (int)(p0 - tile * s_pad);
        const uint8_t* line = q + row * pitch;
        for (int i = 0; i < 32; i += 4) {
            uint32_t w = 0;
            for (int k = 0; k < 4; ++k) {
                const int64_t d = tile * s + off;
                int c = 0;
                if (row < R && off < s && d < D && (p0 + i + k) < kv_end) c = fetch_code(line, d, b);
                w |= ((uint32_t)c & 0xFFu) << (8 * k);
                if (++off == s_pad) { off = 0; ++tile; }
            }
            *reinterpret_cast<uint32_t*>(&lds[r][half * 32 + i]) = w;
        }
    }
}

// REQUANT (second reading of the accumulator, Methodology: tiled quantization): instead of
// clamping and adding, every finished tile's sums are written to g.partial[t] and their
// largest magnitude is folded into g.tile_max[t]; requant_sum_kernel does the rest.
template <bool ALIGNED, bool REQUANT>
__global__ __launch_bounds__(kThreads) void gemm_tiled_kernel(GemmArgs g)
{
    __shared__ __attribute__((aligned(16))) uint8_t As[BM][LDP];
    __shared__ __attribute__((aligned(16))) uint8_t Bs[BN][LDP];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t row0 = (int64_t)blockIdx.y * BM;     // rows of A -> output rows
    const int64_t col0 = (int64_t)blockIdx.x * BN;     // rows of B -> output columns

    // contraction range of this workgroup, in tiles and in virtual positions
    const int64_t t_begin = (int64_t)blockIdx.z * g.tiles_per_split;
    int64_t t_end = t_begin + g.tiles_per_split;
    if (t_end > g.n_tiles) t_end = g.n_tiles;
    const int64_t kv_begin = t_begin * g.s_pad, kv_end = t_end * g.s_pad;
    const int steps_per_tile = g.s_pad / KG;

    v16i part[2][2], total[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) { part[a][c][r] = 0; total[a][c][r] = 0; }

    int step_in_tile = 0;
    for (int64_t kv0 = kv_begin; kv0 < kv_end; kv0 += KC) {
        __syncthreads();
        load_operand<ALIGNED>(As, g.qA, g.pitchA, g.bA, g.RA, g.D, row0, kv0, kv_end, g.s, g.s_pad);
        load_operand<ALIGNED>(Bs, g.qB, g.pitchB, g.bB, g.RB, g.D, col0, kv0, kv_end, g.s, g.s_pad);
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < KC / KG; ++ks) {
            if (kv0 + ks * KG >= kv_end) break;
            long fa[2], fb[2];
#pragma unroll
            for (int a = 0; a < 2; ++a)
                fa[a] = *reinterpret_cast<const long*>(
                    &As[wm * 64 + a * 32 + (lane & 31)][ks * KG + (lane >> 5) * 8]);
#pragma unroll
            for (int c = 0; c < 2; ++c)
                fb[c] = *reinterpret_cast<const long*>(
                    &Bs[wn * 64 + c * 32 + (lane & 31)][ks * KG + (lane >> 5) * 8]);
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int c = 0; c < 2; ++c)
                    part[a][c] = __builtin_amdgcn_mfma_i32_32x32x16_i8(fa[a], fb[c], part[a][c], 0, 0, 0);
            if (REQUANT && step_in_tile + 1 == steps_per_tile) {
                step_in_tile = 0;
                const int64_t t = (kv0 + ks * KG) / g.s_pad;
                int32_t* slice = g.partial + t * g.RA * g.RB;
                int m = 0;
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        const int64_t j = col0 + wn * 64 + c * 32 + (lane & 31);
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int64_t i = row0 + wm * 64 + a * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                            const int pv = part[a][c][r];
                            part[a][c][r] = 0;
                            if (i < g.RA && j < g.RB) {
                                slice[i * g.RB + j] = pv;
                                m = max(m, pv < 0 ? -pv : pv);
                            }
                        }
                    }
                m = wave_max_int(m);
                if (lane == 0 && (uint32_t)m > __hip_atomic_load(&g.tile_max[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
                    atomicMax(&g.tile_max[t], (uint32_t)m);
            } else if (++step_in_tile == steps_per_tile) {
                step_in_tile = 0;
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int c = 0; c < 2; ++c)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            int p = part[a][c][r];
                            p = p < g.acc_lo ? g.acc_lo : (p > g.acc_hi ? g.acc_hi : p);
                            total[a][c][r] += p;
                            part[a][c][r] = 0;
                        }
            }
        }
    }

    if (REQUANT) return;
    // ---- store.  32x32 block: lane holds column (lane & 31); register r is
    // row 8*(r/4) + 4*(lane/32) + (r%4).
    const float dq = (g.scaleA[0] * g.scaleB[0]) * g.inv_n;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int64_t j = col0 + wn * 64 + c * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t i = row0 + wm * 64 + a * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (i < g.RA && j < g.RB) {
                    const int v = total[a][c][r];
                    if (g.splits > 1) {
                        g.partial[((int64_t)blockIdx.z * g.RA + i) * g.RB + j] = v;
                    } else {
                        if (g.acc_out) g.acc_out[i * g.RB + j] = v;
                        if (g.out) g.out[i * g.RB + j] = (float)v * dq;
                        if (g.out_bf16) g.out_bf16[i * g.RB + j] = (uint16_t)bf16_bits((float)v * dq);
                    }
                }
            }
        }
}

// Totals of a split contraction: element e of the output is the sum of element e of
// every slice.  VEC = 4: count is a multiple of 4, so every slice is 16-byte aligned.
template <int VEC>
__global__ __launch_bounds__(256) void reduce_kernel(const int32_t* partial, int splits, int64_t count,
                                                     const float* scaleA, const float* scaleB,
                                                     float inv_n, float* out, uint16_t* out_bf16,
                                                     int32_t* acc_out, const float* mask_src)
{
    const float dq = (scaleA[0] * scaleB[0]) * inv_n;
    for (int64_t e = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * VEC; e < count;
         e += (int64_t)gridDim.x * blockDim.x * VEC) {
        int t[4] = {0, 0, 0, 0};
        const int32_t* src = partial + e;
#pragma unroll 4
        for (int z = 0; z < splits; ++z, src += count) {
            if (VEC == 4) {
                const int4 v = *reinterpret_cast<const int4*>(src);
                t[0] += v.x; t[1] += v.y; t[2] += v.z; t[3] += v.w;
            } else {
                t[0] += src[0];
            }
        }
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            if (acc_out) acc_out[e + k] = t[k];
            if (out) out[e + k] = (mask_src && !(mask_src[e + k] > 0.0f)) ? 0.0f : (float)t[k] * dq;
            if (out_bf16) out_bf16[e + k] = (uint16_t)bf16_bits((float)t[k] * dq);
        }
    }
}

// The same for many slices: sixteen threads share an element (a group of VEC), each adds up
// every sixteenth slice, and the first of them adds the sixteen sums from LDS.  A thread of
// the kernel above walks all slices one after the other, which is latency, not bandwidth,
// once there are more than a few dozen.
template <int VEC, bool S16 = false>
__global__ __launch_bounds__(256) void reduce_many_kernel(const int32_t* partial, int splits, int64_t count,
                                                          const float* scaleA, const float* scaleB,
                                                          float inv_n, float* out, uint16_t* out_bf16,
                                                          int32_t* acc_out, const float* mask_src)
{
    constexpr int SG = 16, EPB = 256 / SG;      // slice groups, elements per block
    __shared__ int red[SG][EPB][4];
    const int el = threadIdx.x % EPB, sg = threadIdx.x / EPB;
    const int64_t e = ((int64_t)blockIdx.x * EPB + el) * VEC;
    int t[4] = {0, 0, 0, 0};
    if (e < count) {
        if constexpr (S16) {
            // slices of 16-bit integers (VEC = 4: four of them are one 8-byte load)
            const int16_t* src = reinterpret_cast<const int16_t*>(partial) + (int64_t)sg * count + e;
#pragma unroll 4
            for (int z = sg; z < splits; z += SG, src += (int64_t)SG * count) {
                const short4 v = *reinterpret_cast<const short4*>(src);
                t[0] += v.x; t[1] += v.y; t[2] += v.z; t[3] += v.w;
            }
        } else {
            const int32_t* src = partial + (int64_t)sg * count + e;
#pragma unroll 4
            for (int z = sg; z < splits; z += SG, src += (int64_t)SG * count) {
                if (VEC == 4) {
                    const int4 v = *reinterpret_cast<const int4*>(src);
                    t[0] += v.x; t[1] += v.y; t[2] += v.z; t[3] += v.w;
                } else {
                    t[0] += src[0];
                }
            }
        }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) red[sg][el][k] = t[k];
    __syncthreads();
    if (sg != 0 || e >= count) return;
    const float dq = (scaleA[0] * scaleB[0]) * inv_n;
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        int sum = 0;
#pragma unroll
        for (int j = 0; j < SG; ++j) sum += red[j][el][k];
        if (acc_out) acc_out[e + k] = sum;
        if (out) out[e + k] = (mask_src && !(mask_src[e + k] > 0.0f)) ? 0.0f : (float)sum * dq;
        if (out_bf16) out_bf16[e + k] = (uint16_t)bf16_bits((float)sum * dq);
    }
}

// Second reading, second step: Q with `a` bits on every tile's partial sums, with the
// tile's own maximum, and the sum over tiles.  Per element e and tile t:
//   inv_t = fl(2^(a-1) / m_t),  c = clamp(RNE(fl(float(P_t[e]) * inv_t))),  acc += c * m_t
// (exact integers); value = acc * 2^-(a-1), dequantized like any other total.
constexpr int kTileChunk = 2048;
__global__ __launch_bounds__(256) void requant_sum_kernel(const int32_t* partial, const uint32_t* tile_max,
                                                          int64_t n_tiles, int64_t count, int a,
                                                          const float* scaleA, const float* scaleB,
                                                          float inv_n, float pow2, float* out,
                                                          int32_t* acc_out)
{
    __shared__ float inv_s[kTileChunk];
    __shared__ int m_s[kTileChunk];
    const float qmax = (float)((1 << (a - 1)) - 1), qmin = -(float)(1 << (a - 1));
    const float dq = ((scaleA[0] * scaleB[0]) * inv_n) * pow2;     // pow2 = 2^-(a-1): exact scaling
    const int64_t per_block = (int64_t)blockDim.x;
    const int64_t rounds = (count + per_block * gridDim.x - 1) / (per_block * gridDim.x);
    // every thread of a block walks the same tiles, so the chunk tables are filled once per round
    for (int64_t round = 0; round < rounds; ++round) {
        const int64_t e = (round * gridDim.x + blockIdx.x) * per_block + threadIdx.x;
        int acc = 0;
        for (int64_t t0 = 0; t0 < n_tiles; t0 += kTileChunk) {
            const int chunk = (int)(n_tiles - t0 < kTileChunk ? n_tiles - t0 : kTileChunk);
            __syncthreads();
            for (int k = threadIdx.x; k < chunk; k += blockDim.x) {
                const uint32_t m = tile_max[t0 + k];
                m_s[k] = (int)m;
                // binary64 quotient of two binary32-exact integers, rounded once more to binary32
                inv_s[k] = m ? (float)((double)(1 << (a - 1)) / (double)m) : 0.0f;
            }
            __syncthreads();
            if (e < count) {
                const int32_t* src = partial + t0 * count + e;
                for (int k = 0; k < chunk; ++k, src += count) {
                    const float v = (float)src[0] * inv_s[k];
                    const float r = fminf(fmaxf(rintf(v), qmin), qmax);
                    acc += (int)r * m_s[k];
                }
            }
        }
        if (e < count) {
            if (acc_out) acc_out[e] = acc;
            if (out) out[e] = (float)acc * dq;
        }
    }
}

__global__ __launch_bounds__(256) void relu_mask_kernel(float* out, const float* mask_src, int64_t count)
{
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += (int64_t)gridDim.x * blockDim.x)
        if (!(mask_src[e] > 0.0f)) out[e] = 0.0f;
}

} // namespace

hipError_t launch_relu_mask(float* out, const float* mask_src, int64_t count, hipStream_t stream)
{
    int64_t blocks = (count + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    ProfileScope ps(K_RELU_MASK, stream);
    hipLaunchKernelGGL(relu_mask_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, out, mask_src, count);
    return hipGetLastError();
}

// 16-bit slices are read by the many-slices kernel only, four elements per 8-byte load
bool reduce_takes_slices16(int splits, int64_t count)
{
    return splits >= 32 && count % 4 == 0 && (count / 4 + 15) / 16 < ((int64_t)1 << 31);
}

hipError_t launch_reduce(const int32_t* partial, int splits, int64_t count, const float* scaleA,
                         const float* scaleB, float inv_n, float* out, uint16_t* out_bf16,
                         int32_t* acc_out, hipStream_t stream, const float* mask_src, bool slices16)
{
    const bool vec = (count % 4 == 0);
    const int64_t groups = vec ? count / 4 : count;
    if (slices16 && !reduce_takes_slices16(splits, count)) return hipErrorInvalidValue;
    if (splits >= 32 && (groups + 15) / 16 < ((int64_t)1 << 31)) {
        ProfileScope ps(K_REDUCE, stream);
        const dim3 grid((unsigned)((groups + 15) / 16));
        if (slices16)
            hipLaunchKernelGGL((reduce_many_kernel<4, true>), grid, dim3(256), 0, stream, partial, splits, count,
                               scaleA, scaleB, inv_n, out, out_bf16, acc_out, mask_src);
        else if (vec)
            hipLaunchKernelGGL(reduce_many_kernel<4>, grid, dim3(256), 0, stream, partial, splits, count, scaleA,
                               scaleB, inv_n, out, out_bf16, acc_out, mask_src);
        else
            hipLaunchKernelGGL(reduce_many_kernel<1>, grid, dim3(256), 0, stream, partial, splits, count, scaleA,
                               scaleB, inv_n, out, out_bf16, acc_out, mask_src);
        return hipGetLastError();
    }
    int64_t blocks = ((vec ? count / 4 : count) + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    ProfileScope ps(K_REDUCE, stream);
    if (vec)
        hipLaunchKernelGGL(reduce_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, stream, partial, splits,
                           count, scaleA, scaleB, inv_n, out, out_bf16, acc_out, mask_src);
    else
        hipLaunchKernelGGL(reduce_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, stream, partial, splits,
                           count, scaleA, scaleB, inv_n, out, out_bf16, acc_out, mask_src);
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs& g, hipStream_t stream)
{
    if (gemm_fast_eligible(g)) return launch_gemm_fast(g, stream);
    const dim3 grid((unsigned)((g.RB + BN - 1) / BN), (unsigned)((g.RA + BM - 1) / BM),
                    (unsigned)g.splits);
    const bool aligned = (g.s % 16 == 0) && (g.D % 16 == 0) && (g.s_pad == g.s);
    ProfileScope ps(aligned ? K_GEMM_ALIGNED : K_GEMM_GENERIC, stream);
    if (aligned)
        hipLaunchKernelGGL((gemm_tiled_kernel<true, false>), grid, dim3(kThreads), 0, stream, g);
    else
        hipLaunchKernelGGL((gemm_tiled_kernel<false, false>), grid, dim3(kThreads), 0, stream, g);
    return hipGetLastError();
}

hipError_t launch_gemm_requant(const GemmArgs& g_in, int acc_bits, hipStream_t stream)
{
    GemmArgs g = g_in;
    const int64_t blocks = ((g.RB + BN - 1) / BN) * ((g.RA + BM - 1) / BM);
    // the tiles are independent: spread them over enough workgroups to fill the chip
    int64_t parts = (1024 + blocks - 1) / blocks;
    if (parts > g.n_tiles) parts = g.n_tiles;
    if (parts > 65535) parts = 65535;
    g.tiles_per_split = (g.n_tiles + parts - 1) / parts;
    g.splits = (int)((g.n_tiles + g.tiles_per_split - 1) / g.tiles_per_split);
    const dim3 grid((unsigned)((g.RB + BN - 1) / BN), (unsigned)((g.RA + BM - 1) / BM), (unsigned)g.splits);
    const bool aligned = (g.s % 16 == 0) && (g.D % 16 == 0) && (g.s_pad == g.s);
    {
        ProfileScope ps(K_REQUANT_TILES, stream);
        if (aligned)
            hipLaunchKernelGGL((gemm_tiled_kernel<true, true>), grid, dim3(kThreads), 0, stream, g);
        else
            hipLaunchKernelGGL((gemm_tiled_kernel<false, true>), grid, dim3(kThreads), 0, stream, g);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t count = g.RA * g.RB;
    int64_t nb = (count + 255) / 256;
    if (nb > 8192) nb = 8192;
    ProfileScope ps(K_REQUANT_SUM, stream);
    hipLaunchKernelGGL(requant_sum_kernel, dim3((unsigned)nb), dim3(256), 0, stream, g.partial, g.tile_max,
                       g.n_tiles, count, acc_bits, g.scaleA, g.scaleB, g.inv_n,
                       ldexpf(1.0f, -(acc_bits - 1)), g.out, g.acc_out);
    return hipGetLastError();
}

} // namespace hdqt
