// Hadamard-domain quantization of one tensor along BOTH axes from one read
// (gfx950).
//
// A training step needs every activation and gradient tensor quantized twice:
// along its rows for one matmul and along its columns for another (X along K
// for the forward product and along M for the weight gradient; G along N for
// the input gradient and along M for the weight gradient).  The two results
// are the paper's quantizer Q applied in two Hadamard domains; they share
// nothing but the source, and the source is what costs: the kernels are
// HBM-bound.  Here pass 1 computes both maxima and pass 2 both code sets from a
// single read of the tensor each.  The results are bit-identical to two
// single-axis quantizations.
//
// A wave holds a tile of 64 rows x 64 columns in registers, 64 values per lane:
// lane (rg, cg) = (lane / 8, lane % 8) has rows 8*rg + i (i < 8) of columns
// 32*h + 4*cg + j (h < 2, j < 4).  Both transforms run on that one layout:
//   along the columns of a row (axis 1): strides 1, 2 pair registers (j),
//     strides 4, 8, 16 pair lanes (lane xor 1, 2, 4), stride 32 pairs registers (h);
//   along the rows of a column (axis 0): strides 1, 2, 4 pair registers (i),
//     strides 8, 16, 32 pair lanes (lane xor 8, 16, 32).
// The stages that pair lanes through DPP are single multiply-adds that leave the
// upper lane's result negated (see stage_fma8); the sign a lane has accumulated,
// (-1)^popcount(lane & 7) after axis 1 and (-1)^(lane bit 3) after axis 0, is
// folded into the reciprocal step the lane quantizes with.
// The axis-1 transform is done row by row on copies (eight values at a time),
// the axis-0 transform then in place.  No LDS is involved.
// Requires rows and cols multiples of 64 and block orders up to 64.  Codes of up to
// 4 bits are packed two per byte; the WIDE instances write codes of 5 to 8 bits, one
// per byte (both axes of a tensor, and all tensors of a launch, on the same side).

#include "common.hpp"
#include "lane_ops.hpp"

namespace hdqt {

namespace {

using namespace lanes;

constexpr int kThreads = 256;
constexpr int kTile = 64;

struct Tile {
    float v[2][4][8];        // [h][j][i]
};

struct DualCtx {
    const DualArgs* q;
    int cg, rg;
    int log2n_row, log2n_col;      // block orders; compile-time 6 in the kernel instances for n = 64
    float c1, c2, c4, c8;          // -1 where the lane bit is set, else +1
    float inv_row, inv_col;        // reciprocal steps, times the lane's accumulated sign
    float qmin_row, qmax_row, qmin_col, qmax_col;
};

__device__ __forceinline__ void tile_load(Tile& t, const DualArgs& q, const DualCtx& x, int64_t row0,
                                          int64_t col0)
{
    // a uniform address per (i, h) plus one 32-bit offset per lane (cols < 2^26: quantize_dual_eligible):
    // one 64-bit vector addition per row of the tile is all that is left of the address arithmetic
    // (buffer loads with scalar offsets take that out too, 21 instructions of 1711, and change no time)
    const float* base = q.T + row0 * q.cols + col0;
    const uint32_t lo = (uint32_t)(x.rg * 8) * (uint32_t)q.cols + (uint32_t)(x.cg * 4);
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const float4 a = *reinterpret_cast<const float4*>(&(base + i * q.cols + 32 * h)[lo]);
            t.v[h][0][i] = a.x; t.v[h][1][i] = a.y; t.v[h][2][i] = a.z; t.v[h][3][i] = a.w;
        }
}

// The same tile when the source is an activation and the tensor its im2col matrix.
// The 64 rows of a tile are 64 consecutive pixels of one image (whole image rows when
// W <= 64, a 64-pixel run of one row otherwise), its 64 columns a run of (channel, tap)
// pairs: everything the tile reads lies in a patch of pCN channels x pPH rows x pPW
// pixels, zero border included.  The wave copies the patch into its own piece of LDS
// with coalesced reads, then gathers its 64 x 64 values from there: an element's patch
// address is (row part of its pixel) + (column part of its channel and tap).
// The activation is read from HBM about once per pass instead of kh*kw times.
constexpr int kPatchUnroll = 32;

__device__ __forceinline__ void tile_load_conv(Tile& t, const DualArgs& q, const DualCtx& x,
                                               int64_t row0, int64_t col0, float* patch, int lane)
{
    const int W = q.cW, H = q.cH, C = q.cC, kw = q.ckw, khw = q.ckh * q.ckw;
    const int ph = (q.ckh - 1) / 2, pw = (kw - 1) / 2;
    const int PH = q.pPH, PW = q.pPW, CN = q.pCN;
    int* coltab = reinterpret_cast<int*>(patch + ((CN * PH * PW + 3) & ~3));      // 64 column parts

    // where the tile lies (the same in every lane)
    const uint32_t m0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)row0);
    const uint32_t k0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)col0);
    const uint32_t HW = (uint32_t)(H * W);
    const uint32_t b = m0 / HW, rem = m0 - b * HW;
    const int y_first = (int)(rem / (uint32_t)W), x_first = (int)(rem - (uint32_t)y_first * (uint32_t)W);
    const int c_lo = (int)(k0 / (uint32_t)khw);

    // ---- patch: row q = (channel c_lo + q / PH, image row y_first - ph + q % PH).  Rows of up
    // to 32 words go two per step (32 lanes each).  What costs here is the number of load
    // round trips, not the instructions: kPatchUnroll steps issue their loads together
    // (every address is clamped into the activation, so no load is conditional), then store.
    // (One row per step with scalar row arithmetic halves the vector instructions and is
    // 35 % slower: twice the round trips.)
    const bool two = PW <= 32;
    const int lpr = two ? 32 : 64, rpi = two ? 2 : 1;
    const int lrow = two ? (lane >> 5) : 0, lx = lane & (lpr - 1);
    const int rows_total = CN * PH;
    const int steps = (rows_total + rpi - 1) / rpi;
    const float* img = q.T + (int64_t)b * C * H * W;
    for (int ch = 0; ch * lpr < PW; ++ch) {
        const int pxx = ch * lpr + lx;
        const int gx = x_first - pw + pxx;
        const bool col_ok = pxx < PW && gx >= 0 && gx < W;
        const int gxc = gx < 0 ? 0 : (gx >= W ? W - 1 : gx);
        int c_rel = 0, pyy = lrow;
        while (pyy >= PH) { pyy -= PH; ++c_rel; }
        for (int it0 = 0; it0 < steps; it0 += kPatchUnroll) {
            float v[kPatchUnroll];
            bool keep[kPatchUnroll];
#pragma unroll
            for (int u = 0; u < kPatchUnroll; ++u) {
                const int gy = y_first - ph + pyy, c = c_lo + c_rel;
                const int gyc = gy < 0 ? 0 : (gy >= H ? H - 1 : gy);
                const int cc = c >= C ? C - 1 : c;
                v[u] = img[(cc * H + gyc) * W + gxc];
                keep[u] = col_ok && gy >= 0 && gy < H && c < C;
                pyy += rpi;
                while (pyy >= PH) { pyy -= PH; ++c_rel; }
            }
#pragma unroll
            for (int u = 0; u < kPatchUnroll; ++u) {
                const int qrow = (it0 + u) * rpi + lrow;
                if (pxx < PW && qrow < rows_total) patch[qrow * PW + pxx] = keep[u] ? v[u] : 0.0f;
            }
        }
    }
    // ---- column parts of the tile's 64 columns, one per lane
    {
        const uint32_t k = k0 + (uint32_t)lane;
        const uint32_t c = k / (uint32_t)khw, tap = k - c * (uint32_t)khw;
        const uint32_t ty = tap / (uint32_t)kw, tx = tap - ty * (uint32_t)kw;
        coltab[lane] = ((int)c - c_lo) * PH * PW + (int)ty * PW + (int)tx;
    }
    // LDS operations of one wave are carried out in order; the fence keeps the compiler
    // from moving the reads below above the writes of other lanes
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- gather: pixel 8*rg + i of the tile is (image row off / Wt, position off % Wt),
    // Wt = min(W, 64), a power of two.  With Wt >= 8 the lane's eight pixels are neighbours
    // in one image row: eight consecutive patch words per column.
    const int wt_shift = (W >= 64) ? 6 : (31 - __builtin_clz((unsigned)W));
    if (wt_shift >= 3) {
        const int off = x.rg * 8;
        const float* base = patch + (off >> wt_shift) * PW + (off & ((1 << wt_shift) - 1));
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int4 cp = *reinterpret_cast<const int4*>(coltab + 32 * h + 4 * x.cg);
            const float* p0 = base + cp.x;
            const float* p1 = base + cp.y;
            const float* p2 = base + cp.z;
            const float* p3 = base + cp.w;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                t.v[h][0][i] = p0[i];
                t.v[h][1][i] = p1[i];
                t.v[h][2][i] = p2[i];
                t.v[h][3][i] = p3[i];
            }
        }
    } else {
        int rowpart[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int off = x.rg * 8 + i;
            rowpart[i] = (off >> wt_shift) * PW + (off & ((1 << wt_shift) - 1));
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int4 cp = *reinterpret_cast<const int4*>(coltab + 32 * h + 4 * x.cg);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                t.v[h][0][i] = patch[rowpart[i] + cp.x];
                t.v[h][1][i] = patch[rowpart[i] + cp.y];
                t.v[h][2][i] = patch[rowpart[i] + cp.z];
                t.v[h][3][i] = patch[rowpart[i] + cp.w];
            }
        }
    }
}

// Random bits of stochastic rounding for the lane's elements of one tile row: four
// consecutive elements at h = 0 (index e, e % 4 == 0) and four at h = 1 (index
// e + 32).  Each group lies in one Philox block (block e/8, words (e%8)/2 and
// (e%8)/2 + 1), and lanes cg and cg ^ 1 need the same two blocks, the even lane the
// lower words, the odd lane the upper ones.  So the even lane computes the block of
// h = 0, the odd lane that of h = 1, and they trade the halves the other needs:
// one Philox call per lane and row instead of two.
__device__ __forceinline__ void random_words(int64_t e, bool odd, uint32_t tensor_id, uint32_t k0,
                                             uint32_t k1, uint32_t w_h0[2], uint32_t w_h1[2])
{
    const uint64_t blk = ((uint64_t)e >> 3) + (odd ? 4u : 0u);
    uint32_t r[4];
    philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), tensor_id, 0u, k0, k1, r);
    const uint32_t send0 = odd ? r[0] : r[2], send1 = odd ? r[1] : r[3];
    const uint32_t recv0 = __float_as_uint(lane_xor<1>(__uint_as_float(send0)));
    const uint32_t recv1 = __float_as_uint(lane_xor<1>(__uint_as_float(send1)));
    w_h0[0] = odd ? recv0 : r[0];
    w_h0[1] = odd ? recv1 : r[1];
    w_h1[0] = odd ? r[2] : recv0;
    w_h1[1] = odd ? r[3] : recv1;
}

// Axis 1 for the lane's row 8*rg + i of the tile: transform, then absmax (pass
// 1) or codes (pass 2).
template <bool QUANT, bool STOCH, bool WIDE>
__device__ __forceinline__ void row_line(const Tile& t, int i, const DualCtx& x, int64_t row0,
                                         int64_t col0, float& amax)
{
    const DualArgs& q = *x.q;
    const int log2n = x.log2n_row;
    float w[8];              // index 4*h + j
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int j = 0; j < 4; ++j) w[4 * h + j] = t.v[h][j][i];
    if (log2n >= 1) {
#pragma unroll
        for (int k = 0; k < 8; k += 2) {
            const float a = w[k], c = w[k + 1];
            w[k] = a + c;
            w[k + 1] = a - c;
        }
    }
    if (log2n >= 2) {
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (!(k & 2)) {
                const float a = w[k], c = w[k + 2];
                w[k] = a + c;
                w[k + 2] = a - c;
            }
    }
    if (log2n >= 3) {
        stage_fma8<1>(w, x.c1);
    }
    if (log2n >= 4) {
        stage_fma8<2>(w, x.c2);
    }
    if (log2n >= 5) {
        stage_fma8<4>(w, x.c4);
    }
    if (!QUANT) {
        // max(|a + c|, |a - c|) = |a| + |c|, also after rounding: the last stage of
        // pass 1 needs no differences
        if (log2n >= 6) {
#pragma unroll
            for (int k = 0; k < 4; ++k) amax = fmaxf(amax, fabsf(w[k]) + fabsf(w[k + 4]));
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) amax = fmaxf(amax, fabsf(w[k]));
        }
        return;
    }
    if (log2n >= 6) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float a = w[k], c = w[k + 4];
            w[k] = a + c;
            w[k + 4] = a - c;
        }
    }
    const int64_t row = row0 + x.rg * 8 + i;
    const float magic = kMagic + (WIDE ? 128.0f : 8.0f);
    uint32_t both = 0;       // the lane's eight codes: low half h = 0, high half h = 1
    uint32_t rnd[2][2] = {{0u, 0u}, {0u, 0u}};
    if (STOCH)
        random_words(row * q.cols + col0 + x.cg * 4, (x.cg & 1) != 0, q.tid_row, q.seed_row_lo,
                     q.seed_row_hi, rnd[0], rnd[1]);
    if constexpr (WIDE) {
        // one byte per code: the lane's four codes of each half are a dword.  Lanes cg and
        // cg ^ 1 trade one of them: the even lane ends up with columns 4cg .. 4cg+7, the odd
        // one with columns 32+4(cg-1) .. 32+4cg+3, eight bytes per lane and store.
        uint32_t word[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint32_t cw[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t u = (rnd[h][j >> 1] >> (16 * (j & 1))) & 0xFFFFu;
                cw[j] = code_word<STOCH>(w[4 * h + j], x.inv_row, x.qmin_row, x.qmax_row, magic, u);
            }
            word[h] = pack_bytes(cw);
        }
        const bool odd = (x.cg & 1) != 0;
        const uint32_t other = __float_as_uint(lane_xor<1>(__uint_as_float(odd ? word[0] : word[1])));
        const uint2 pair = odd ? make_uint2(other, word[1]) : make_uint2(word[0], other);
        const int byte_off = odd ? 32 + 4 * (x.cg - 1) : 4 * x.cg;
        *reinterpret_cast<uint2*>(q.codes_row + row * q.cols + col0 + byte_off) = pair;
        return;
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const uint32_t* w01 = rnd[h];
        // 0x4B400000 << 4j has no bits in the low 16: the low half of the sum is the
        // four offset nibbles
        uint32_t acc = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t u = (w01[j >> 1] >> (16 * (j & 1))) & 0xFFFFu;
            acc += code_word<STOCH>(w[4 * h + j], x.inv_row, x.qmin_row, x.qmax_row, magic, u) << (4 * j);
        }
        both |= (acc & 0xFFFFu) << (16 * h);
    }
    both ^= 0x88888888u;
    // Lanes cg and cg ^ 1 trade halves: the even one ends up with columns
    // 4cg .. 4cg+7 (bytes 2cg .. 2cg+3 of the row's 32), the odd one with columns
    // 32+4(cg-1) .. 32+4cg+3 (bytes 16+2(cg-1) ..).
    const uint32_t other = __float_as_uint(lane_xor<1>(__uint_as_float(both)));
    const bool odd = (x.cg & 1) != 0;
    const uint32_t word = __builtin_amdgcn_perm(other, both, odd ? 0x03020706u : 0x05040100u);
    const int byte_off = odd ? 16 + 2 * (x.cg - 1) : 2 * x.cg;
    // (uniform address of the tile's row i, 32-bit offset of the lane's row group and bytes)
    const uint32_t lo = (uint32_t)(x.rg * 8) * (uint32_t)(q.cols >> 1) + (uint32_t)byte_off;
    *reinterpret_cast<uint32_t*>(&(q.codes_row + (row0 + i) * (q.cols >> 1) + (col0 >> 1))[lo]) = word;
}

// Axis 0 on the whole tile, in place.  The two lanes of a swap stage carry the
// same sign (it depends on lane bit 3 only), so those stages need no care.
// MAX_ONLY (pass 1, block order 64): the last stage is replaced by |lo| + |hi| of
// the swapped-in pairs, returned as a running maximum; the tile is then spent.
template <bool MAX_ONLY>
__device__ __forceinline__ float col_transform(Tile& t, int log2n, float c8)
{
    float m = 0.0f;
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float* v = t.v[h][j];
            butterfly8(v, log2n);
            if (log2n > 3) stage_fma8<8>(v, c8);
            if (log2n > 4) {
#pragma unroll
                for (int i = 0; i < 8; i += 2) stage_swap<false>(v[i], v[i + 1]);
            }
            if (MAX_ONLY) {
#pragma unroll
                for (int i = 0; i < 8; i += 2) {
                    const v2u r = __builtin_amdgcn_permlane32_swap(as_u(v[i]), as_u(v[i + 1]), false, false);
                    m = fmaxf(m, fabsf(as_f(r[0])) + fabsf(as_f(r[1])));
                }
            } else if (log2n > 5) {
#pragma unroll
                for (int i = 0; i < 8; i += 2) stage_swap<true>(v[i], v[i + 1]);
            }
        }
    return m;
}

template <bool STOCH, bool WIDE>
__device__ __forceinline__ void col_codes(const Tile& t, const DualCtx& x, int64_t row0, int64_t col0)
{
    const DualArgs& q = *x.q;
    const float magic = kMagic + (WIDE ? 128.0f : 8.0f);
    const int64_t pitch = WIDE ? q.rows : q.rows >> 1;
    uint32_t cw[2][4][8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint32_t rnd[2][2] = {{0u, 0u}, {0u, 0u}};
        if (STOCH)
            random_words((row0 + x.rg * 8 + i) * q.cols + col0 + x.cg * 4, (x.cg & 1) != 0, q.tid_col,
                         q.seed_col_lo, q.seed_col_hi, rnd[0], rnd[1]);
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t u = (rnd[h][j >> 1] >> (16 * (j & 1))) & 0xFFFFu;
                cw[h][j][i] = code_word<STOCH>(t.v[h][j][i], x.inv_col, x.qmin_col, x.qmax_col, magic, u);
            }
    }
    // column 32h + 4cg + j, rows 8rg .. 8rg+7: one dword (two with a byte per code); the
    // eight rg lanes of a column write 32 (64) consecutive bytes
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (WIDE) {
                uint8_t* dst = q.codes_col + (col0 + 32 * h + x.cg * 4 + j) * pitch + row0 + x.rg * 8;
                *reinterpret_cast<uint2*>(dst) = make_uint2(pack_bytes(cw[h][j]), pack_bytes(cw[h][j] + 4));
            } else {
                const uint32_t lo = (uint32_t)(x.cg * 4) * (uint32_t)pitch + (uint32_t)(x.rg * 4);
                uint8_t* dst = &(q.codes_col + (col0 + 32 * h + j) * pitch + (row0 >> 1))[lo];
                *reinterpret_cast<uint32_t*>(dst) = pack_nibbles(cw[h][j]);
            }
        }
}

// One atomicMax per workgroup and record (see block_atomic_max in common.hpp).
__device__ __forceinline__ void block_atomic_max2(float m_row, float m_col, QMeta* meta_row,
                                                  QMeta* meta_col, float (*smem)[2], uint32_t block_id)
{
    m_row = wave_max(m_row);
    m_col = wave_max(m_col);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { smem[wave][0] = m_row; smem[wave][1] = m_col; }
    __syncthreads();
    if (threadIdx.x < 2) {
        const int which = threadIdx.x;
        float r = smem[0][which];
        for (int w = 1; w < kThreads / kWave; ++w) r = fmaxf(r, smem[w][which]);
        QMeta* meta = which ? meta_col : meta_row;
        const uint32_t slot = block_id % kAmaxSlots;
        uint32_t* target = &meta->amax[slot * kAmaxSlotStride];
        const uint32_t bits = __float_as_uint(r);
        if (bits > __hip_atomic_load(target, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
            atomicMax(target, bits);
    }
}

// ---- the two phases of a tile, shared by the two-launch and the one-launch kernels

template <bool N64>
__device__ __forceinline__ void dual_setup(DualCtx& x, const DualArgs& q, int lane)
{
    x.q = &q;
    // with the block orders known at compile time the stage conditions, the branches around
    // them and the register copies at their joins disappear (about a tenth of the kernel)
    x.log2n_row = N64 ? 6 : q.log2n_row;
    x.log2n_col = N64 ? 6 : q.log2n_col;
    x.cg = lane & 7;
    x.rg = lane >> 3;
    x.c1 = (lane & 1) ? -1.0f : 1.0f;
    x.c2 = (lane & 2) ? -1.0f : 1.0f;
    x.c4 = (lane & 4) ? -1.0f : 1.0f;
    x.c8 = (lane & 8) ? -1.0f : 1.0f;
    x.inv_row = x.inv_col = 0.0f;
    x.qmin_row = (float)(-(1 << (q.b_row - 1)));
    x.qmax_row = (float)((1 << (q.b_row - 1)) - 1);
    x.qmin_col = (float)(-(1 << (q.b_col - 1)));
    x.qmax_col = (float)((1 << (q.b_col - 1)) - 1);
}

// reciprocal steps (with the lane's accumulated signs) from the two scalings;
// one thread of the grid publishes the scales
__device__ __forceinline__ void dual_set_scaling(DualCtx& x, const DualArgs& q, const Scaling& s_row,
                                                 const Scaling& s_col, bool publisher)
{
    // signs accumulated by the stage_fma8 stages that actually run
    float sg_row = 1.0f;
    if (x.log2n_row >= 3) sg_row *= x.c1;
    if (x.log2n_row >= 4) sg_row *= x.c2;
    if (x.log2n_row >= 5) sg_row *= x.c4;
    x.inv_row = s_row.inv * sg_row;
    x.inv_col = x.log2n_col > 3 ? s_col.inv * x.c8 : s_col.inv;
    if (publisher && threadIdx.x == 0) {
        q.meta_row->scale = s_row.scale;
        q.meta_col->scale = s_col.scale;
        if (q.scale_row_out) *q.scale_row_out = s_row.scale;
        if (q.scale_col_out) *q.scale_col_out = s_col.scale;
    }
}

// both maxima of a tile; `t` is spent afterwards
__device__ __forceinline__ void dual_absmax(Tile& t, const DualCtx& x, int64_t row0, int64_t col0,
                                            float& amax_row, float& amax_col)
{
#pragma unroll
    for (int i = 0; i < 8; ++i) row_line<false, false, false>(t, i, x, row0, col0, amax_row);
    if (x.log2n_col > 5) {
        amax_col = fmaxf(amax_col, col_transform<true>(t, x.log2n_col, x.c8));
    } else {
        col_transform<false>(t, x.log2n_col, x.c8);
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < 8; ++i) amax_col = fmaxf(amax_col, fabsf(t.v[h][j][i]));
    }
}

// both code sets of a tile; `t` is spent afterwards
template <bool ST_ROW, bool ST_COL, bool WIDE>
__device__ __forceinline__ void dual_codes(Tile& t, const DualCtx& x, int64_t row0, int64_t col0)
{
    float unused = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) row_line<true, ST_ROW, WIDE>(t, i, x, row0, col0, unused);
    col_transform<false>(t, x.log2n_col, x.c8);
    col_codes<ST_COL, WIDE>(t, x, row0, col0);
}

// One launch covers up to kMaxBatch tensors: the workgroups of tensor k are
// [first[k], first[k+1]) of a one-dimensional grid, numbered along its columns first.
// Small tensors (a layer's weights) ride along with a large one instead of paying
// for a launch of their own.
struct DualBatch {
    DualArgs t[kMaxDualBatch];
    int n;
    int first[kMaxDualBatch + 1];
    int gx[kMaxDualBatch];       // workgroups along the columns
    int WC[kMaxDualBatch];       // waves side by side in a workgroup (1, 2 or 4)
    int lds_per_wave;            // floats of LDS per wave (convolution sources), a multiple of 4
    int spread;                  // pass 2: every spread-th workgroup of the grid is one of tensor 0 (0: off)
};

// Workgroup number -> number in the tensor-after-tensor order.  With `spread`, the workgroups of
// tensor 0 (the stochastically rounded one of a per-tensor launch: twice the vector
// instructions per tile, a tenth of the bytes) stand at every spread-th place of the grid
// instead of in front of it, so that they run beside the memory-bound tiles of the others,
// not before them.
__device__ __forceinline__ int batch_order(const DualBatch& b)
{
    const int bid = (int)blockIdx.x;
    if (!b.spread) return bid;
    const int c0 = b.first[1], slot = bid / b.spread;
    if (bid - slot * b.spread == 0 && slot < c0) return slot;
    const int before = slot + 1 < c0 ? slot + 1 : c0;      // tensor 0's workgroups at or before this place
    return bid - before + c0;
}

// Wave w of a workgroup owns the tile at columns [64*wc, 64*wc + 64) of the
// workgroup's strip and rows [64*wr, 64*wr + 64), (wc, wr) = (w % WC, w / WC).
// One tile per wave and no register prefetch: what hides the memory latency is
// the number of resident waves, and a second tile in registers halves it
// (measured: 67 us against 85 us for pass 1 of a 65536 x 1152 tensor).
//
// ROUND selects the rounding of pass 2: bit 0 = stochastic along the rows, bit 1 =
// along the columns; kRoundPerTensor = every tensor of the launch is either nearest on
// both axes or stochastic on both, told by its own flags (a layer's X and W next to
// its G), so that the short, arithmetic-heavy stochastic tensor shares a launch with
// the long, memory-bound ones instead of running after them on a half-empty chip.
constexpr int kRoundPerTensor = 4;
constexpr int kRoundWide = 8;        // added to ROUND: codes of 5 to 8 bits, one per byte

template <bool QUANT, int ROUND, bool N64, bool CONV>
__device__ __forceinline__ void dual_block(const DualBatch& b, int k, int vb, float (*red)[2], float* lds)
{
    const DualArgs& q = b.t[k];
    const int count = b.first[k + 1] - b.first[k];
    // pass 2 walks a tensor from its end to its start: it begins with what pass 1
    // read last, which is most likely still in the memory-side cache
    int local = vb - b.first[k];
    if (QUANT) local = count - 1 - local;
    const int gx = b.gx[k], WC = b.WC[k];
    const int64_t by = local / gx, bx = local - (local / gx) * gx;

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int wc = wave % WC, wr = wave / WC, WR = 4 / WC;
    const int64_t col0 = (bx * WC + wc) * kTile;
    const int64_t row0 = (by * WR + wr) * kTile;
    // rows % 64 == cols % 64 == 0: a tile is entirely inside the tensor or entirely outside
    const bool live = col0 < q.cols && row0 < q.rows;

    DualCtx x;
    dual_setup<N64>(x, q, lane);
    Tile t;
    if (live) {
        if (CONV && q.conv) tile_load_conv(t, q, x, row0, col0, lds + wave * b.lds_per_wave, lane);
        else tile_load(t, q, x, row0, col0);
    }
    if (QUANT) {
        const Scaling s_row = load_scaling(q.meta_row, q.clip_row, q.b_row);
        const Scaling s_col = load_scaling(q.meta_col, q.clip_col, q.b_col);
        dual_set_scaling(x, q, s_row, s_col, local == 0);
        if (live) dual_codes<(ROUND & 1) != 0, (ROUND & 2) != 0, (ROUND & kRoundWide) != 0>(t, x, row0, col0);
    } else {
        float amax_row = 0.0f, amax_col = 0.0f;
        if (live) dual_absmax(t, x, row0, col0, amax_row, amax_col);
        block_atomic_max2(amax_row, amax_col, q.meta_row, q.meta_col, red, (uint32_t)local);
    }
}

template <bool QUANT, int ROUND, bool N64, bool CONV>
__global__ __launch_bounds__(kThreads) void fwht_dual_kernel(DualBatch b)
{
    __shared__ float red[kThreads / kWave][2];
    extern __shared__ __attribute__((aligned(16))) float lds[];      // CONV: one patch per wave

    const int vb = QUANT ? batch_order(b) : (int)blockIdx.x;
    int k = 0;
    while (k + 1 < b.n && vb >= b.first[k + 1]) ++k;
    if constexpr ((ROUND & 7) == kRoundPerTensor) {
        // two complete bodies, chosen per workgroup: sharing anything between them
        // (one load, one setup) lets the compiler keep both paths' registers alive
        if (b.t[k].st_row) dual_block<QUANT, 3 | (ROUND & kRoundWide), N64, CONV>(b, k, vb, red, lds);
        else dual_block<QUANT, ROUND & kRoundWide, N64, CONV>(b, k, vb, red, lds);
    } else {
        dual_block<QUANT, ROUND, N64, CONV>(b, k, vb, red, lds);
    }
}

bool all_order_64(const DualArgs* qs, int n)
{
    for (int k = 0; k < n; ++k)
        if (qs[k].log2n_row != 6 || qs[k].log2n_col != 6) return false;
    return true;
}

bool make_batch(const DualArgs* qs, int n, DualBatch* b)
{
    if (n < 1 || n > kMaxDualBatch) return false;
    b->n = n;
    int64_t total = 0;
    int lds = 0;
    for (int k = 0; k < n; ++k) {
        const DualArgs& q = qs[k];
        const int64_t strips = q.cols / kTile;
        const int WC = (strips % 4 == 0) ? 4 : (strips % 2 == 0) ? 2 : 1;
        const int64_t tall = (int64_t)kTile * (4 / WC);
        const int64_t gx = strips / WC, gy = (q.rows + tall - 1) / tall;
        b->t[k] = q;
        if (q.conv) {
            const int need = ((q.pCN * q.pPH * q.pPW + 3) & ~3) + kTile;
            if (need > lds) lds = need;
        }
        b->first[k] = (int)total;
        b->gx[k] = (int)gx;
        b->WC[k] = WC;
        total += gx * gy;
        if (total >= ((int64_t)1 << 31)) return false;
    }
    b->first[n] = (int)total;
    b->lds_per_wave = lds;
    b->spread = 0;
    return true;
}

} // namespace

// Geometries the im2col source takes: odd windows, and tiles of 64 pixels that are whole
// image rows (W a power of two up to 64, H*W a multiple of 64) or lie inside one row
// (W a multiple of 64); the patch of a tile must fit the wave's share of LDS.
constexpr int kMaxPatchFloats = 3008;      // 12 KB per wave with the column table

bool dual_conv_plan(DualArgs* q)
{
    const int W = q->cW, H = q->cH, kh = q->ckh, kw = q->ckw;
    if (q->cC < 1 || H < 1 || W < 1 || kh < 1 || kw < 1 || kh % 2 == 0 || kw % 2 == 0) return false;
    if (kh > 15 || kw > 15) return false;
    const bool row_run = (W % kTile == 0);
    const bool whole_rows = (W < kTile) && (kTile % W == 0) && (((int64_t)H * W) % kTile == 0);
    if (!row_run && !whole_rows) return false;
    // one image is indexed with 32 bits
    if ((int64_t)q->cC * H * W >= ((int64_t)1 << 31) || q->rows >= ((int64_t)1 << 31) || q->cols >= ((int64_t)1 << 31))
        return false;
    if (q->rows % ((int64_t)H * W) != 0 || q->cols != (int64_t)q->cC * kh * kw) return false;
    q->pPH = (row_run ? 1 : kTile / W) + kh - 1;
    q->pPW = (row_run ? kTile : W) + kw - 1;
    q->pCN = (kTile - 1) / (kh * kw) + 2;
    return q->pCN * q->pPH * q->pPW <= kMaxPatchFloats;
}

bool quantize_dual_eligible(const DualArgs& q)
{
    if (q.cols >= ((int64_t)1 << 26) || q.rows >= ((int64_t)1 << 26)) return false;      // 32-bit lane offsets
    return (q.rows % kTile == 0) && (q.cols % kTile == 0) && q.log2n_row <= 6 && q.log2n_col <= 6 &&
           q.b_row <= 8 && q.b_col <= 8 && (q.b_row <= 4) == (q.b_col <= 4) &&
           (q.rows / kTile) * (q.cols / kTile) < ((int64_t)1 << 30);
}

// Pass 1 (both maxima) of n tensors in one launch; their calibration records must be zero.
hipError_t launch_dual_pass1(const DualArgs* qs, int n, hipStream_t stream)
{
    DualBatch b;
    if (!make_batch(qs, n, &b)) return hipErrorInvalidValue;
    const int id = n > 1 ? K_DUAL_ABSMAX_BATCH
                         : (qs[0].profile_tag ? K_DUAL_ABSMAX_X + (qs[0].profile_tag - 1) : K_DUAL_ABSMAX);
    ProfileScope ps(id, stream);
    const dim3 grid((unsigned)b.first[n]), block(kThreads);
    const size_t lds = (size_t)(kThreads / kWave) * b.lds_per_wave * sizeof(float);
    const bool n64 = all_order_64(qs, n);
    if (lds) {      // a convolution source among the tensors
        if (n64) hipLaunchKernelGGL((fwht_dual_kernel<false, 0, true, true>), grid, block, lds, stream, b);
        else hipLaunchKernelGGL((fwht_dual_kernel<false, 0, false, true>), grid, block, lds, stream, b);
    } else if (n64) {
        hipLaunchKernelGGL((fwht_dual_kernel<false, 0, true, false>), grid, block, 0, stream, b);
    } else {
        hipLaunchKernelGGL((fwht_dual_kernel<false, 0, false, false>), grid, block, 0, stream, b);
    }
    return hipGetLastError();
}

// Whether the tensors can share a pass-2 launch: same rounding modes everywhere, or each
// tensor nearest on both axes or stochastic on both; and all of them with packed 4-bit
// codes or all with a byte per code.
bool dual_pass2_batchable(const DualArgs* qs, int n)
{
    bool same = true, paired = true;
    for (int k = 0; k < n; ++k) {
        if ((qs[k].b_row <= 4) != (qs[0].b_row <= 4)) return false;
        if (qs[k].st_row != qs[0].st_row || qs[k].st_col != qs[0].st_col) same = false;
        if (qs[k].st_row != qs[k].st_col) paired = false;
    }
    return same || paired;
}

// Pass 2 (both code sets) of n tensors in one launch (see dual_pass2_batchable).
hipError_t launch_dual_pass2(const DualArgs* qs, int n, hipStream_t stream)
{
    DualBatch b;
    if (!make_batch(qs, n, &b) || !dual_pass2_batchable(qs, n)) return hipErrorInvalidValue;
    bool same = true;
    for (int k = 1; k < n; ++k)
        if (qs[k].st_row != qs[0].st_row || qs[k].st_col != qs[0].st_col) same = false;
    const int id = n > 1 ? K_DUAL_QUANT_BATCH
                         : (qs[0].profile_tag ? K_DUAL_QUANT_X + (qs[0].profile_tag - 1) : K_DUAL_QUANT);
    ProfileScope ps(id, stream);
    const dim3 grid((unsigned)b.first[n]), block(kThreads);
    const bool n64 = all_order_64(qs, n);
    const size_t lds = (size_t)(kThreads / kWave) * b.lds_per_wave * sizeof(float);
#define HDQT_LAUNCH_PASS2(ROUND)                                                                     \
    do {                                                                                            \
        if (lds && n64) hipLaunchKernelGGL((fwht_dual_kernel<true, ROUND, true, true>), grid, block, lds, stream, b); \
        else if (lds) hipLaunchKernelGGL((fwht_dual_kernel<true, ROUND, false, true>), grid, block, lds, stream, b); \
        else if (n64) hipLaunchKernelGGL((fwht_dual_kernel<true, ROUND, true, false>), grid, block, 0, stream, b); \
        else hipLaunchKernelGGL((fwht_dual_kernel<true, ROUND, false, false>), grid, block, 0, stream, b); \
    } while (0)
    const int mode = !same ? kRoundPerTensor : (qs[0].st_row ? 1 : 0) | (qs[0].st_col ? 2 : 0);
    // A stochastic tensor in front of nearest ones: its workgroups among theirs (see batch_order),
    // over the first three quarters of the grid (a heavy workgroup among the last ones is the
    // kernel's tail: spread over the whole grid the launch took 102 us instead of 95.6) and at
    // an odd distance: workgroups go to the eight XCDs in turn, and at a distance of 8 (6) every
    // heavy one lands on the same XCD (on four of them): 122 (100) us.  At 7: 93.4 us.
    if (mode == kRoundPerTensor && qs[0].st_row && b.first[1] > 0) {
        bool rest_nearest = true;
        for (int k = 1; k < n; ++k) rest_nearest = rest_nearest && !qs[k].st_row;
        int64_t q = (int64_t)b.first[n] * 3 / (4 * (int64_t)b.first[1]);
        if (q % 2 == 0) --q;
        if (rest_nearest && q >= 3 && q < ((int64_t)1 << 30)) b.spread = (int)q;
    }
    if (qs[0].b_row > 4) {
        switch (mode) {
        case kRoundPerTensor: HDQT_LAUNCH_PASS2(kRoundPerTensor | kRoundWide); break;
        case 3: HDQT_LAUNCH_PASS2(3 | kRoundWide); break;
        case 1: HDQT_LAUNCH_PASS2(1 | kRoundWide); break;
        case 2: HDQT_LAUNCH_PASS2(2 | kRoundWide); break;
        default: HDQT_LAUNCH_PASS2(0 | kRoundWide); break;
        }
    } else {
        switch (mode) {
        case kRoundPerTensor: HDQT_LAUNCH_PASS2(kRoundPerTensor); break;
        case 3: HDQT_LAUNCH_PASS2(3); break;
        case 1: HDQT_LAUNCH_PASS2(1); break;
        case 2: HDQT_LAUNCH_PASS2(2); break;
        default: HDQT_LAUNCH_PASS2(0); break;
        }
    }
#undef HDQT_LAUNCH_PASS2
    return hipGetLastError();
}

// Pass 1 and pass 2 of one tensor.  (A one-launch variant for small tensors -- tile
// kept in registers across a grid-wide barrier -- was built and measured: correct,
// but the cooperative launch it needs for a guaranteed co-resident grid costs about
// 25 us more than an ordinary launch on this stack, more than the launch it saves.)
hipError_t launch_quantize_dual(const DualArgs& q, hipStream_t stream)
{
    const hipError_t e = launch_dual_pass1(&q, 1, stream);
    return e != hipSuccess ? e : launch_dual_pass2(&q, 1, stream);
}

} // namespace hdqt
