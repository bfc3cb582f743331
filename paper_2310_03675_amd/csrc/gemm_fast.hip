// Fast path of the tiled integer matmul (gfx950).
//
// Same result as the generic kernel (tiles of size s along the contraction,
// each tile's sum clamped to the a-bit accumulator range, 32-bit total), for
//   both operands packed 4-bit, or both with a byte per code (the WIDE instances: the
//   bytes go to LDS as they are, nothing is scaled, generic clamp only);
//   s a multiple of 32 (or 16), D a multiple of 8 (packed) or 4 (bytes): rows of whole dwords;
//   a row that ends inside a 32-code unit is padded with zeros on its way to LDS.
//
// What differs from the generic kernel:
//   * v_mfma_i32_32x32x32_i8: one MFMA consumes 32 contraction positions.
//   * eight waves per 128 x 128 workgroup tile, each 64 rows x 32 columns: 106-124
//     VGPRs, so four waves share a SIMD and fill each other's MFMA / LDS / barrier
//     latencies (four waves of 64 x 64 need 168-198 VGPRs: two per SIMD).
//   * Nibble unpack without sign extension: a code in the high nibble of a
//     byte IS 16*code as int8, so (w << 4) & 0xF0F0F0F0 and w & 0xF0F0F0F0 give
//     the even and the odd codes of a dword, each scaled by 16.  Both operands
//     use the same order of positions inside a 32-group, so the dot product is
//     unchanged; it arrives scaled by 256.
//   * 8-bit accumulators (the paper's setting), s = 32 or 64: saturating the
//     scaled tile sum to int16 (v_cvt_pk_i16_i32, two sums per instruction)
//     leaves exactly clamp(sum, -128, 127) in the high byte of each half, and
//     v_dot4c_i32_i8 with the byte selector (0,1,0,1) adds the two high bytes
//     to the running total: one VALU instruction per tile sum.  The two sums
//     of a pair are two consecutive tiles of the same output element.
//   * the same setting with tiles of 32, plain output, at most 255 tiles per part: the
//     kernel first asks whether a tile can saturate at all (EPI_CERT8_S32, below) and
//     adds the ones that cannot straight onto the totals in the matrix core.
//   * any other accumulator width or tile length: v_med3_i32 against bounds
//     scaled by 256, add, and one exact shift at the end.
//   * LDS holds int8, double-buffered, and the global loads run two stages
//     (one in the s = 64 instance) ahead of the multiplication, across
//     output-tile boundaries.

#include "common.hpp"

#include <type_traits>

namespace hdqt {

namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef short v2s __attribute__((ext_vector_type(2)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));

constexpr int kWaves = 8;             // waves per workgroup: 8 measured 3-7 % faster than 4 on the layer
                                      // shapes and on 4096^3 (see the kernel)
constexpr int BM = 128, BN = 128;
constexpr int KS_LONG = 128;          // codes per LDS stage: 4 MFMA steps.  (Stages of 64 codes leave
                                      // room for three workgroups per CU instead of two; measured
                                      // slower on all three layer shapes.)
constexpr int KSTEP = 32;             // codes per MFMA
constexpr int kScaleShift = 8;        // both operands carry a factor 16

enum Epilogue { EPI_GENERIC = 0, EPI_SAT8_S32 = 1, EPI_SAT8_S64 = 2, EPI_STAGES = 3, EPI_SAT16_S32 = 4,
                EPI_SAT16_S64 = 5, EPI_SAT8_S16 = 6, EPI_SAT16_S16 = 7, EPI_CLAMP_S16 = 8,
                EPI_REQ_MAX = 9, EPI_REQ_SUM = 10, EPI_REQ_MAX_S32 = 11, EPI_REQ_SUM_S32 = 12,
                EPI_CERT8_S32 = 13, EPI_CERT16_S32 = 14 };
// EPI_CERT8_S32: 8-bit accumulators, tiles of 32 packed 4-bit codes, as EPI_SAT8_S32 -- but a
// tile whose sums provably stay inside the accumulator is not clamped at all.  The proof is
// the Cauchy-Schwarz bound: |sum_k a_k b_k| <= sqrt(sum a_k^2 * sum b_k^2), so with nA the largest
// sum of squares over the wave's rows of A in this tile and nB the same over its columns of B,
// nA * nB <= 127^2 means that no clamp of the tile can act, and the matrix core adds the tile
// straight onto the totals (no vector instruction at all).  The sums of squares cost four
// v_dot8_i32_i4 per 16-byte unit on its way to LDS, a few lane operations and a 512-byte table.
// The totals therefore carry the factor 256 of the unpacking throughout.  Tiles that fail the
// test are saturated to int16 as before and added with v_dot2_i32_i16, i.e. still times 256;
// a sum that saturates upwards adds 32767 where 127 * 256 = 32512 is meant, 255 too many, so
// that a total is 256 * (T + p) - p with T the true total and p <= 255 the number of its
// tiles that saturated upwards (hence at most 255 tiles per part): p = -total mod 256 and
// T = (total + p) / 256 - p, taken once at the end of an output tile.
// Quantizer output of heavy-tailed tensors (activations, most gradients) has small codes and
// passes nearly everywhere; codes that fill their range fail, and then this is EPI_SAT8_S32
// plus the test.
// EPI_CERT16_S32: the same test in front of EPI_SAT16_S32 (packed 4-bit codes, accumulators of
// 9 to 12 bits: wider ones cannot saturate on tiles of 32 at all).  The bound is the
// accumulator's own, (2^(a-1) - 1)^2, which nearly every tile of nearly any data meets; the
// operands go to LDS scaled as for EPI_SAT16, the clamped tiles are added with their low bits
// cleared as there, so the totals are exact multiples of 2^(16-a) and need no correction.
// EPI_REQ_MAX / EPI_REQ_SUM: the second reading of the low-bit accumulator (Methodology, tiled
// quantization: every tile's partial-sum tensor through Q with a bits and its own maximum) as
// two passes over the same product, neither of which stores a tile sum.  The first keeps, per
// tile of the contraction, the largest magnitude over the whole output (registers -> wave ->
// a table in LDS -> one atomic per workgroup and tile into g.tile_max); the second repeats the
// multiplication and, with m_t known, quantizes each tile sum where it leaves the matrix core:
//     c = clamp(RNE(fl(float(P) * fl(2^(a-1) / m_t)))),   total += c * m_t.
// Five vector instructions per tile sum: conversion, multiplication, the addition of 1.5 * 2^23
// (whose rounding is the round-to-nearest-even, and whose low mantissa bits are then 2^22 + c),
// the clamp against bounds carrying the same offset, and a 24-bit multiply-add with m_t; the
// offsets' contribution, 2^22 * sum of m_t, is subtracted once per output element (modulo
// 2^32, like every step; the true total fits, which the caller has checked).
// The _S32 instances are those for tiles of one 32-code step (no running tile sum to keep).
constexpr int kReqTable = 512;         // tiles of one part of the contraction (table entries in LDS)
constexpr float kReqMagic = 12582912.0f;   // 1.5 * 2^23
// EPI_CLAMP_S16: tiles of 16 codes with the compare-select clamp, for the accumulator widths
// neither conversion trick covers (fewer bits than bA + bB).
// The _S16 instances (tiles of 16 codes) split every 32-code step into two
// v_mfma_i32_32x32x16_i8: the 16-byte LDS fragment of a lane already holds, in its low and
// high halves, what that instruction wants from the lane for the first and the second tile
// of the step (packed codes: even positions first, then odd ones; byte codes: the loader
// stores the 8-byte quarters of a step in the order 0, 2, 1, 3).
// EPI_SAT16: accumulators of a bits, bA + bB <= a <= 16, tiles of 32 or 64.  The operands go to
// LDS scaled by 2^jA and 2^jB, jA + jB = 16 - a (a code of b bits times 2^(8-b) still fits a
// byte), so a tile's sum arrives times 2^(16-a) and saturating it to int16 is the a-bit clamp,
// still times 2^(16-a) once the low 16 - a bits are cleared (32767 is not a multiple);
// v_dot2c_i32_i16 adds the two halves of a pair to the total, and one exact shift at the
// end takes the factor out.  (EPI_SAT8 is the case a = 8 with 4-bit
// operands, whose unpacking gives the factor 256 for free.)
// EPI_STAGES: the generic clamp for tiles that are whole stages (s a multiple of KS_LONG): the
// tile ends are tested once per stage, so nothing branches between the MFMAs of a stage and
// the fragment loads of its four steps can run ahead of them.

template <int UNITS_A, int UNITS_B>
struct Staged {
    uint4 a[UNITS_A], b[UNITS_B];     // (row, k-step) units per operand per thread
};

// Operands are read through buffer descriptors that cover exactly their bytes: a unit that
// lies outside (a row beyond the last one, a position beyond the part's end, a halo row of
// the fold) is given an offset beyond the descriptor's range and comes back as zeros from
// the hardware's range check.  No branch surrounds the load, so the compiler can count the
// loads in flight: with the load inside an `if` it waited for all of them at the top of
// every stage, the ones just issued for the stage after next included.
typedef unsigned int u4v __attribute__((ext_vector_type(4)));
constexpr uint32_t kOutside = 0x80000000u;      // operands are smaller than 2 GiB (gemm_fast_eligible)

__device__ __forceinline__ __amdgpu_buffer_rsrc_t operand_rsrc(const uint8_t* q, int64_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(q), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ uint4 load_unit(__amdgpu_buffer_rsrc_t rs, int64_t pitch, int64_t R, int64_t row,
                                           int64_t k, int64_t k_end)
{
    const bool ok = row >= 0 && row < R && k < k_end;
    const uint32_t off = ok ? (uint32_t)(row * pitch + (k >> 1)) : kOutside;
    return __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0));
}

// a byte per code: the 32 codes of a unit are two of these, at byte offsets k and k + 16
__device__ __forceinline__ uint4 load_unit_wide(__amdgpu_buffer_rsrc_t rs, int64_t pitch, int64_t R, int64_t row,
                                                int64_t k, int64_t k_end, int half)
{
    const bool ok = row >= 0 && row < R && k < k_end;
    const uint32_t off = ok ? (uint32_t)(row * pitch + k + 16 * half) : kOutside;
    return __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0));
}

__device__ __forceinline__ void store_unit(uint8_t* lds_row_k, const uint4& w)
{
    const uint32_t m = 0xF0F0F0F0u;
    const uint4 even = make_uint4((w.x << 4) & m, (w.y << 4) & m, (w.z << 4) & m, (w.w << 4) & m);
    const uint4 odd = make_uint4(w.x & m, w.y & m, w.z & m, w.w & m);
    *reinterpret_cast<uint4*>(lds_row_k) = even;
    *reinterpret_cast<uint4*>(lds_row_k + 16) = odd;
}

// A unit that straddles the end of a row (D no multiple of 32) was loaded with the first codes
// of the next row behind its own: dword j holds `per_dword` codes starting at first + j *
// per_dword of the unit and is kept only where that lies below `valid`, the number of the
// unit's codes inside the row (a multiple of per_dword, see gemm_fast_eligible).
__device__ __forceinline__ void mask_tail(uint4& w, int valid, int per_dword, int first)
{
    w.x = first < valid ? w.x : 0u;
    w.y = first + per_dword < valid ? w.y : 0u;
    w.z = first + 2 * per_dword < valid ? w.z : 0u;
    w.w = first + 3 * per_dword < valid ? w.w : 0u;
}

// total += 256 * (clamp(p0/256, -128, 127) + clamp(p1/256, -128, 127)), plus 255 for each of the
// two that saturates upwards (see EPI_CERT8_S32)
__device__ __forceinline__ int add_sat8_pair_scaled(int total, int p0, int p1)
{
    const v2s pk = __builtin_amdgcn_cvt_pk_i16(p0, p1);
    const v2s ones = {1, 1};
    return __builtin_amdgcn_sdot2(pk, ones, total, false);
}

// sum of the squares of the 32 signed 4-bit codes of a unit
__device__ __forceinline__ int unit_norm(const uint4& w)
{
    int n = __builtin_amdgcn_sdot8((int)w.x, (int)w.x, 0, false);
    n = __builtin_amdgcn_sdot8((int)w.y, (int)w.y, n, false);
    n = __builtin_amdgcn_sdot8((int)w.z, (int)w.z, n, false);
    return __builtin_amdgcn_sdot8((int)w.w, (int)w.w, n, false);
}

// max(x, x of the lane SHR places below in the same row of 16 lanes; 0 where there is none)
template <int SHR>
__device__ __forceinline__ int max_row_shr(int x)
{
    const int below = __builtin_amdgcn_update_dpp(0, x, 0x110 + SHR, 0xF, 0xF, true);
    return x > below ? x : below;
}

// total += clamp(p0/256, -128, 127) + clamp(p1/256, -128, 127)
__device__ __forceinline__ int add_sat8_pair(int total, int p0, int p1)
{
    const v2s pk = __builtin_amdgcn_cvt_pk_i16(p0, p1);
    return __builtin_amdgcn_sdot4(__builtin_bit_cast(int, pk), 0x01000100, total, false);
}

// total += floor_f(clamp(p0, -32768, 32767)) + floor_f(clamp(p1, -32768, 32767)), floor_f =
// down to a multiple of the factor 2^need the sums carry (`low_clear` has the low `need` bits
// of both halves clear): a sum that saturates upwards becomes 32767, which is
// (2^(a-1) - 1) * 2^need plus a remainder that must not add up over the tiles.
__device__ __forceinline__ int add_sat16_pair(int total, int p0, int p1, uint32_t low_clear)
{
    const v2s pk = __builtin_amdgcn_cvt_pk_i16(p0, p1);
    const v2s ones = {1, 1};
    return __builtin_amdgcn_sdot2(__builtin_bit_cast(v2s, __builtin_bit_cast(uint32_t, pk) & low_clear), ones,
                                  total, false);
}

// Four bytes, each holding code * 16 (a nibble in its high half), to code * 2^j, j < 4:
// a shift right by k = 4 - j inside every byte, then sign extension from bit 7 - k.  Bit 7
// is set before the subtraction so that no byte borrows from its neighbour, and cleared
// (or, for a negative code, set) by the last exclusive or.
__device__ __forceinline__ uint32_t rescale_bytes(uint32_t hi_form, int k, uint32_t keep, uint32_t sign)
{
    const uint32_t t = (hi_form >> k) & keep;
    return (((t ^ sign) | 0x80808080u) - sign) ^ 0x80808080u;
}

// 32 packed 4-bit codes -> LDS as bytes code * 2^j (even codes first, then odd ones)
__device__ __forceinline__ void store_unit_scaled(uint8_t* lds_row_k, const uint4& w, int j)
{
    const uint32_t m = 0xF0F0F0F0u;
    uint4 even = make_uint4((w.x << 4) & m, (w.y << 4) & m, (w.z << 4) & m, (w.w << 4) & m);
    uint4 odd = make_uint4(w.x & m, w.y & m, w.z & m, w.w & m);
    if (j < 4) {
        const int k = 4 - j;
        const uint32_t keep = (0xFFu >> k) * 0x01010101u, sign = (0x80u >> k) * 0x01010101u;
        even = make_uint4(rescale_bytes(even.x, k, keep, sign), rescale_bytes(even.y, k, keep, sign),
                          rescale_bytes(even.z, k, keep, sign), rescale_bytes(even.w, k, keep, sign));
        odd = make_uint4(rescale_bytes(odd.x, k, keep, sign), rescale_bytes(odd.y, k, keep, sign),
                         rescale_bytes(odd.z, k, keep, sign), rescale_bytes(odd.w, k, keep, sign));
    }
    *reinterpret_cast<uint4*>(lds_row_k) = even;
    *reinterpret_cast<uint4*>(lds_row_k + 16) = odd;
}

// 16 codes, a byte each, times 2^j (the caller guarantees that they still fit)
__device__ __forceinline__ uint4 scale_bytes(const uint4& w, int j)
{
    const uint32_t keep = ((0xFFu << j) & 0xFFu) * 0x01010101u;
    return make_uint4((w.x << j) & keep, (w.y << j) & keep, (w.z << j) & keep, (w.w << j) & keep);
}

// clamp(v, lo, hi), lo <= hi.  Plain C++ on purpose: written as inline assembly (one
// v_med3_i32) the compiler does not see that the instruction reads an MFMA result and leaves
// out the wait states the hardware needs between the two (found as a lost tile sum in the
// first element of a block).
__device__ __forceinline__ int clamp3(int v, int lo, int hi)
{
    const int t = v < lo ? lo : v;
    return t > hi ? hi : t;
}

// Work of a workgroup: the output tiles (blockIdx.y, ct), ct = blockIdx.z,
// blockIdx.z + gridDim.z, ..., each over the part [k_begin, k_end) of the
// contraction that blockIdx.x selects, as one stream of stages of KS codes.
// The part index is the fastest-varying block coordinate: the workgroups that
// share an output tile run together and between them read whole rows of the
// operands, which keeps the DRAM pages they touch open.
// The stream is software-pipelined across tile boundaries: the global loads run
// one stage ahead of the multiplication, LDS holds two stages, and a tile's
// output stores are issued while the next tile's first stage is already in
// flight.  With gridDim.z = 1 a workgroup walks along a
// whole row strip of the output, which is how short contractions (one or two
// stages per tile) keep loads, MFMAs and stores overlapped.
// NARROW: workgroup tile of 128 rows x 64 columns instead of 128 x 128, the eight waves four
// high and two wide with one 32 x 32 block each, for outputs of at most 64 columns, which
// would leave half of every 128-column tile -- half the MFMAs and half the tile sums -- to
// nothing.
// MASK (plain fp32 output only): g.mask_src, a tensor of the output's shape, is read at the end
// of a tile (all of a wave's values in flight together) and the output is written where it is
// positive, +0 elsewhere.  An instance of its own: the 32 values cost registers.  (The fold
// epilogue masks with a run-time test: it reads one value per output element anyway.)
template <int EPI, int KS, bool STREAM, int WAVES, bool BF16, bool FOLD, bool WIDE = false, bool NARROW = false,
          bool MASK = false, bool PAIR = false>
__global__ __launch_bounds__(64 * WAVES, WAVES == 8 ? (MASK ? 3 : 4) : 2) void gemm_i4_kernel(GemmArgs g)
{
    static_assert(!PAIR || FOLD, "pair mode is a way of folding");
    static_assert(!MASK || (!BF16 && !FOLD && !WIDE && !NARROW), "masked output: plain packed instances only");
    static_assert(!NARROW || (WAVES == 8 && !BF16 && !FOLD && !WIDE), "narrow tiles: plain packed instances only");
    constexpr int TM = BM, TN = NARROW ? 64 : BN;   // the workgroup's tile
    // ROWWIDE (streamed outputs, i.e. at least 128 MB): a wave is one block high and two wide
    // instead of two high and one wide, so that its two stores of a row are neighbours (256
    // bytes; streaming stores of 256-byte pieces reach 5.0 TB/s where 128-byte pieces reach
    // 4.6).  Same fragment reads per MFMA.  The benchmark layer's input gradient inside the
    // step: 73.3 -> 70.6 us; its bfloat16 variant 57.7 -> 55.4 us.
    constexpr bool ROWWIDE = STREAM && !NARROW && !FOLD && WAVES == 8;
    constexpr int RS = (NARROW || ROWWIDE) ? 1 : 2; // 32-row MFMA blocks per wave
    constexpr int WROWS = 32 * RS;
    constexpr bool kSat16 = (EPI == EPI_SAT16_S32 || EPI == EPI_SAT16_S64 || EPI == EPI_SAT16_S16);
    constexpr bool kSat8 = (EPI == EPI_SAT8_S32 || EPI == EPI_SAT8_S64 || EPI == EPI_SAT8_S16);
    constexpr bool kPairs16 = (EPI == EPI_SAT8_S16 || EPI == EPI_SAT16_S16 || EPI == EPI_CLAMP_S16);      // pairs of 16-code tiles
    constexpr bool kPairs32 = (EPI == EPI_SAT8_S32 || EPI == EPI_SAT16_S32);      // pairs of 32-code tiles
    constexpr bool kPairs64 = (EPI == EPI_SAT8_S64 || EPI == EPI_SAT16_S64);      // pairs of 64-code tiles
    static_assert(!WIDE || !kSat8, "the 8-bit clamp trick needs the factor 256 of the nibble unpack");
    constexpr int SHIFT = WIDE ? 0 : kScaleShift;      // factor the totals carry, as a shift
    // factor left in a finished total, as a shift: none after the 8-bit trick
    constexpr bool kReqMax = (EPI == EPI_REQ_MAX || EPI == EPI_REQ_MAX_S32);
    constexpr bool kReqSum = (EPI == EPI_REQ_SUM || EPI == EPI_REQ_SUM_S32), kReq = kReqMax || kReqSum;
    constexpr bool kReqS32 = (EPI == EPI_REQ_MAX_S32 || EPI == EPI_REQ_SUM_S32);
    static_assert(!kReq || (!BF16 && !FOLD && !WIDE && !NARROW && !MASK), "second reading: plain packed instances only");
    constexpr bool kCert16 = (EPI == EPI_CERT16_S32);
    constexpr bool kCert = (EPI == EPI_CERT8_S32) || kCert16;
    static_assert(!kCert || (WAVES == 8 && KS == KS_LONG && !BF16 && !FOLD && !WIDE && !MASK), "certified tiles: plain packed instances only");
    const int fin_shift = (kSat16 || kCert16) ? g.fin_shift : ((kSat8 || kReq || kCert) ? 0 : SHIFT);
    const uint32_t low_clear = (kSat16 || kCert16) ? (0xFFFFu & (0xFFFFu << g.fin_shift)) * 0x00010001u : 0u;
    constexpr int REGS = WIDE ? 2 : 1;                 // 16-byte registers per unit in flight
    // WAVES = 4: each wave a 64 x 64 quarter (2 x 2 MFMA blocks).  WAVES = 8: each wave
    // 64 rows x 32 columns (2 x 1 MFMA blocks): half the accumulators per wave, so four
    // waves fit a SIMD instead of two, at 1.5 LDS fragment reads per MFMA instead of 1.
    constexpr int NTHREADS = 64 * WAVES;
    constexpr int WN = (NARROW || ROWWIDE) ? 2 : WAVES / 2;      // waves side by side
    constexpr int CS = NARROW ? 1 : 4 / WN;         // 32-column MFMA blocks per wave: 2 or 1
    constexpr int HS = RS > CS ? RS : CS;
    constexpr int WCOLS = 32 * CS;
    constexpr int NSTEP = KS / KSTEP;
    constexpr int LDP = KS + 16;          // LDS row pitch in bytes (int8 codes)
    constexpr int UNITS = TM * NSTEP / NTHREADS;    // 16-byte units of A per thread
    constexpr int UNITS_B = UNITS;                  // of B (narrow: only the threads of rows < TN)
    static_assert(!kPairs64 || KS == KS_LONG, "a pair of 64-code tiles is one long stage");
    __shared__ __attribute__((aligned(16))) uint8_t As[2][TM][LDP];
    __shared__ __attribute__((aligned(16))) uint8_t Bs[2][TN][LDP];
    // second reading: per tile of this part, the running maximum (times 256) in the first pass,
    // m_t and fl(2^(a-1) / m_t) / 256 in the second
    // certified tiles: per stage buffer and operand, the largest sum of squares over the 16 rows
    // each wave loaded, for each of the stage's four tiles
    __shared__ int cert_n[kCert ? 2 : 1][2][kCert ? WAVES : 1][4];
    bool cert_clamped = false;        // (wave-uniform) some tile of the current output tile went through the clamp
    // Codes that fill their range pass the test nowhere, and a workgroup that finds this out stops
    // testing: when any wave's first stage holds a tile that has to be clamped, every wave takes
    // the clamp for every tile from the third stage on, without sums of squares, table or flags.
    // cert_off is written during the first stage's multiplication and read after the barriers of
    // later stages, i.e. after every wave has left the first stage: the same value in all waves.
    __shared__ int cert_off;
    bool cert_plain = false;          // (workgroup-uniform) the test has been given up
    int cert_stage = 0;               // 0: the first stage of this workgroup, 1: a later one
    if constexpr (kCert) {
        if (threadIdx.x == 0) cert_off = 0;   // (ordered before the first write by the barrier of the first stage)
    }
    __shared__ int req_m[kReq ? kReqTable : 1];
    __shared__ float req_inv[kReqSum ? kReqTable : 1];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int64_t row0 = (int64_t)blockIdx.y * TM;
    // fold: a column tile is f_cg whole channels (f_cg * kh * kw <= 128 columns)
    const int col_stride = FOLD ? g.f_cg * g.fkh * g.fkw : TN;
    const int n_ct = FOLD ? (g.fC + g.f_cg - 1) / g.f_cg : (int)((g.RB + TN - 1) / TN);
    // fold, strip mode: row tile = f_rows_c image rows of one image starting (kh-1)/2 rows above
    // the rows it writes; rows outside the image are zero
    const int f_ph = FOLD ? (g.fkh - 1) / 2 : 0, f_pw = FOLD ? (g.fkw - 1) / 2 : 0;
    const int f_img = (FOLD && !g.f_imgs) ? (int)blockIdx.y / g.f_strips : 0;
    const int f_y0 = (FOLD && !g.f_imgs) ? ((int)blockIdx.y % g.f_strips) * g.f_rows_out - f_ph : 0;
    // fold, pair mode: row tiles 2 blockIdx.y and 2 blockIdx.y + 1 are the two halves of image
    // blockIdx.y; the load stream and the multiply stream each know which half they are at
    constexpr bool f_pair = PAIR;     // (an instance of its own: where a pixel's accumulators lie is then a compile-time choice)
    int f_half = 0, c_half = 0;
    auto a_row = [&](int r) -> int64_t {          // source row of qA for row r of the tile, -1: zero
        if (f_pair) return ((int64_t)blockIdx.y * 2 + f_half) * TM + r;
        if (!FOLD || g.f_imgs) return row0 + r;
        const int yy = f_y0 + (r >> g.f_log2w);
        if (yy < 0 || yy >= g.fH) return -1;
        return ((int64_t)f_img * g.fH + yy) * g.fW + (r & (g.fW - 1));
    };

    const int64_t t_begin = (int64_t)blockIdx.x * g.tiles_per_split;
    int64_t t_end = t_begin + g.tiles_per_split;
    if (t_end > g.n_tiles) t_end = g.n_tiles;
    const int64_t k_begin = t_begin * g.s;
    int64_t k_end = t_end * g.s;
    if (k_end > g.D) k_end = g.D;
    if (k_begin >= k_end) return;         // not reached: every part has at least one tile
    const int steps_per_tile = (int)(g.s / KSTEP);
    const int lo = g.acc_lo_scaled, hi = g.acc_hi_scaled;
    if constexpr (kReq) {
        // (ordered before the first use by the barrier of the first stage)
        const int n_local = (int)(t_end - t_begin);      // <= kReqTable (gemm_requant_fast_eligible)
        for (int i = tid; i < kReqTable; i += NTHREADS) {
            if constexpr (kReqMax) req_m[i] = 0;
            else {
                const uint32_t m = i < n_local ? g.tile_max[t_begin + i] : 0u;
                req_m[i] = (int)m;
                // binary64 quotient of two binary32-exact integers, rounded once more to binary32;
                // the factor 2^-8 (exact) takes out the 256 the tile sums carry
                req_inv[i] = m ? (float)((double)(1 << (g.req_bits - 1)) / (double)m) * 0.00390625f : 0.0f;
            }
        }
    }

    // loader mapping: unit u = tid + NTHREADS*i -> row u / NSTEP, k-step u % NSTEP
    const int lrow = tid / NSTEP, lks = tid % NSTEP;
    constexpr int ROWS_PER_PASS = NTHREADS / NSTEP;

    v16i total[RS][CS];
    v16i part[RS][CS];                // EPI_GENERIC only
#pragma unroll
    for (int a = 0; a < RS; ++a)
#pragma unroll
        for (int c = 0; c < CS; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) { total[a][c][r] = 0; part[a][c][r] = 0; }
    const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    const float dq = (g.scaleA[0] * g.scaleB[0]) * g.inv_n;

    const __amdgpu_buffer_rsrc_t rsA = operand_rsrc(g.qA, g.RA * g.pitchA), rsB = operand_rsrc(g.qB, g.RB * g.pitchB);

    // ---- the load stream: position of the next stage to fetch
    int f_ct = blockIdx.z;
    int64_t f_k = k_begin;
    auto fetch_next = [&](Staged<UNITS * REGS, UNITS_B * REGS>& st) {
        // (past the end of the stream the loads are still issued, with offsets outside the
        // operands: the number of loads in flight then does not depend on the path taken, and
        // the wait at the top of a stage can leave the newer stage's loads in flight)
        const int64_t ke = f_ct < n_ct ? k_end : 0;
        const int64_t col0 = (int64_t)f_ct * col_stride;
#pragma unroll
        for (int i = 0; i < UNITS; ++i) {
            const int r = lrow + ROWS_PER_PASS * i;
            if constexpr (WIDE) {
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    st.a[2 * i + hf] = load_unit_wide(rsA, g.pitchA, g.RA, a_row(r), f_k + lks * KSTEP, ke, hf);
                    st.b[2 * i + hf] = load_unit_wide(rsB, g.pitchB, g.RB, col0 + r, f_k + lks * KSTEP, ke, hf);
                }
            } else {
                st.a[i] = load_unit(rsA, g.pitchA, g.RA, a_row(r), f_k + lks * KSTEP, ke);
                // (narrow: the threads of rows 64 .. 127 of the pass have no unit of B: row -1)
                if (i < UNITS_B)
                    st.b[i] = load_unit(rsB, g.pitchB, g.RB, (!NARROW || r < TN) ? col0 + r : -1,
                                        f_k + lks * KSTEP, ke);
            }
        }
        f_k += KS;
        if (f_k >= k_end) {
            f_k = k_begin;
            if (f_pair && f_half == 0) f_half = 1;      // the image's other half, same column tile
            else { f_half = 0; f_ct += gridDim.z; }
        }
    };
    auto frag = [&](const uint8_t(*lds)[LDP], int base_row, int ks) -> v4i {
        return *reinterpret_cast<const v4i*>(&lds[base_row + (lane & 31)][ks * KSTEP + (lane >> 5) * 16]);
    };

    // ---- the multiply stream
    const int lane_row = wm * WROWS + 4 * (lane >> 5), lane_col = wn * WCOLS + (lane & 31);
    const uint32_t lane_off = (uint32_t)lane_row * (uint32_t)g.RB + (uint32_t)lane_col;
    int c_ct = blockIdx.z;
    int64_t c_k = k_begin;
    int step_in_tile = 0;

    // MASK: the values of g.mask_src at the wave's output positions of tile `ct`, requested a
    // whole tile ahead of the epilogue that tests them (read there, right before the stores,
    // their latency stood in front of every tile: 245 us instead of 71 us for the benchmark
    // layer's input gradient)
    float mk[MASK ? RS : 1][MASK ? CS : 1][MASK ? 16 : 1];
    auto prefetch_mask = [&](const int ct) {
        if (ct >= n_ct) return;
        const int64_t col0 = (int64_t)ct * TN;
        const float* mb = g.mask_src + row0 * g.RB + col0;
        const bool interior = (row0 + TM <= g.RA) && (col0 + TN <= g.RB);
#pragma unroll
        for (int a = 0; a < (MASK ? RS : 1); ++a)
#pragma unroll
            for (int c = 0; c < (MASK ? CS : 1); ++c)
#pragma unroll
                for (int r = 0; r < (MASK ? 16 : 1); ++r) {
                    const int rr = a * 32 + 8 * (r >> 2) + (r & 3);
                    const int64_t uo = (int64_t)rr * g.RB + c * 32;
                    const bool ok = interior || ((row0 + lane_row + rr < g.RA) && (col0 + lane_col + c * 32 < g.RB));
                    mk[a][c][r] = ok ? __builtin_nontemporal_load(&(mb + uo)[lane_off]) : 0.0f;
                }
    };

    // ---- second reading: what happens to a finished tile's sums (p, times 256)
    int req_tile = 0;                 // index of the tile inside this part
    uint32_t req_corr = 0;            // second pass: sum of m_t over the tiles so far
    auto req_finish = [&](v16i (&p)[RS][CS]) {
        if constexpr (kReqMax) {
            int mx = 0, mn = 0;
#pragma unroll
            for (int a = 0; a < RS; ++a)
#pragma unroll
                for (int c = 0; c < CS; ++c)
#pragma unroll
                    for (int r = 0; r < 16; r += 2) {
                        mx = max(max(mx, p[a][c][r]), p[a][c][r + 1]);
                        mn = min(min(mn, p[a][c][r]), p[a][c][r + 1]);
                    }
            int v = max(mx, -mn);      // >= 0: lanes the data-parallel moves fill with 0 change nothing
            v = max(v, __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true));      // quad_perm [1,0,3,2]
            v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true));      // quad_perm [2,3,0,1]
            v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true));     // row_half_mirror
            v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, true));     // row_mirror
            const int w = max(max(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
                              max(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
            if (lane == 0) atomicMax(&req_m[req_tile], w);
        } else if constexpr (kReqSum) {
            const uint32_t m = (uint32_t)__builtin_amdgcn_readfirstlane(req_m[req_tile]);
            const float inv = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(req_inv[req_tile])));
            req_corr += m;
#pragma unroll
            for (int a = 0; a < RS; ++a)
#pragma unroll
                for (int c = 0; c < CS; ++c)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float v = (float)p[a][c][r] * inv;
                        const float u = __builtin_amdgcn_fmed3f(v + kReqMagic, g.req_lo, g.req_hi);
                        total[a][c][r] += (int)__umul24(__float_as_uint(u), m);
                    }
        }
        ++req_tile;
    };

    // One stage: registers -> LDS buffer `buf`, barrier, refill the registers with
    // the next stage, multiply; at the end of a tile, write it out.
    // Whole stages only: positions at or beyond k_end are zero in LDS and add nothing.
    // One barrier per stage is enough: buffer `buf` was last read two stages ago,
    // and every wave has passed the previous stage's barrier since.
    // `gave_up` (a std::true_type / false_type; only EPI_CERT8_S32 has both): the stage as the
    // workgroup runs it once the test of its tiles has been given up -- EPI_SAT8_S32's loop
    // with totals that carry the factor 256.  A body of its own, in a loop of its own: there
    // the totals are single registers again, and the clamps of one pair overlap the MFMAs of
    // the next as in EPI_SAT8_S32 (as a branch inside the testing stage the same code either
    // spilled 30 registers or, cut into pairs by the flags' branches, ran 9 % slower).
    auto stage = [&](Staged<UNITS * REGS, UNITS_B * REGS>& st, const int buf, auto gave_up) {
        constexpr bool kGaveUp = decltype(gave_up)::value;
        constexpr bool kTest = kCert && !kGaveUp;
        if (g.D & (KSTEP - 1)) {
            // rows that end inside a 32-code unit: the thread's units of this stage all start at
            // the same position of their rows
            const int64_t valid = g.D - (c_k + lks * KSTEP);
            if (valid < KSTEP) {
#pragma unroll
                for (int i = 0; i < UNITS * REGS; ++i) {
                    mask_tail(st.a[i], (int)valid, WIDE ? 4 : 8, WIDE ? 16 * (i & 1) : 0);
                    if (i < UNITS_B * REGS) mask_tail(st.b[i], (int)valid, WIDE ? 4 : 8, WIDE ? 16 * (i & 1) : 0);
                }
            }
        }
        if (kTest && !cert_plain) {
            // lane l of the wave holds tile l % 4 of row 16 * wave + l / 4 of both operands.
            // One swap of the wave's halves and one of its odd and even rows bring the largest
            // over lane bits 4 and 5 of A into the lower half and of B into the upper half; two
            // shifted maxima inside the rows finish in lanes 12 .. 15 (A) and 44 .. 47 (B).
            static_assert(!kCert || UNITS == 1, "one unit per thread and operand");
            const int na = unit_norm(st.a[0]), nb = unit_norm(st.b[0]);
            typedef unsigned v2u __attribute__((ext_vector_type(2)));
            v2u sw = __builtin_amdgcn_permlane32_swap((unsigned)na, (unsigned)nb, false, false);
            int m = (int)(sw[0] > sw[1] ? sw[0] : sw[1]);
            sw = __builtin_amdgcn_permlane16_swap((unsigned)m, (unsigned)m, false, false);
            m = (int)(sw[0] > sw[1] ? sw[0] : sw[1]);
            m = max_row_shr<4>(m);
            m = max_row_shr<8>(m);
            if ((lane & 28) == 12) cert_n[buf][lane >> 5][wave][lane & 3] = m;
        }
#pragma unroll
        for (int i = 0; i < UNITS; ++i) {
            const int r = lrow + ROWS_PER_PASS * i;
            if constexpr (WIDE && kPairs16) {
                // quarters 0, 2 | 1, 3 of the step: a lane's fragment then holds its share of
                // the first 16 positions in its low half and of the second 16 in its high half
                const uint4 a0 = scale_bytes(st.a[2 * i], g.jA), a1 = scale_bytes(st.a[2 * i + 1], g.jA);
                const uint4 b0 = scale_bytes(st.b[2 * i], g.jB), b1 = scale_bytes(st.b[2 * i + 1], g.jB);
                *reinterpret_cast<uint4*>(&As[buf][r][lks * KSTEP]) = make_uint4(a0.x, a0.y, a1.x, a1.y);
                *reinterpret_cast<uint4*>(&As[buf][r][lks * KSTEP + 16]) = make_uint4(a0.z, a0.w, a1.z, a1.w);
                *reinterpret_cast<uint4*>(&Bs[buf][r][lks * KSTEP]) = make_uint4(b0.x, b0.y, b1.x, b1.y);
                *reinterpret_cast<uint4*>(&Bs[buf][r][lks * KSTEP + 16]) = make_uint4(b0.z, b0.w, b1.z, b1.w);
            } else if constexpr (WIDE) {
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    *reinterpret_cast<uint4*>(&As[buf][r][lks * KSTEP + 16 * hf]) =
                        kSat16 ? scale_bytes(st.a[2 * i + hf], g.jA) : st.a[2 * i + hf];
                    *reinterpret_cast<uint4*>(&Bs[buf][r][lks * KSTEP + 16 * hf]) =
                        kSat16 ? scale_bytes(st.b[2 * i + hf], g.jB) : st.b[2 * i + hf];
                }
            } else if constexpr (kSat16 || kCert16) {
                store_unit_scaled(&As[buf][r][lks * KSTEP], st.a[i], g.jA);
                if (i < UNITS_B && (!NARROW || r < TN)) store_unit_scaled(&Bs[buf][r][lks * KSTEP], st.b[i], g.jB);
            } else {
                store_unit(&As[buf][r][lks * KSTEP], st.a[i]);
                if (i < UNITS_B && (!NARROW || r < TN)) store_unit(&Bs[buf][r][lks * KSTEP], st.b[i]);
            }
        }
        __syncthreads();
        fetch_next(st);
        // cert_ok: the pair's tiles go straight onto the totals; cert_no: through the clamp.  Two
        // flags whose relation the compiler cannot see: written as if / else, the two ways of
        // updating the totals (whole register tuples by the matrix core, single registers by the
        // clamp) meet in a join that copies all 32 of them on both sides; as two independent
        // conditional blocks each updates them in place.
        int cert_ok[NSTEP / 2] = {}, cert_no[NSTEP / 2] = {};
        v4i cert_fa[2][RS], cert_fb[2][CS];
        if constexpr (kTest) {
#pragma unroll
            for (int pr = 0; pr < NSTEP / 2; ++pr) cert_no[pr] = 1;
        }
        if (kTest && cert_plain) {
            // (a stage in the testing body after the test was given up: every flag stays down)
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int h = 0; h < HS; ++h) {
                    if (h < RS) cert_fa[q][h] = frag(As[buf], wm * WROWS + h * 32, q);
                    if (h < CS) cert_fb[q][h] = frag(Bs[buf], wn * WCOLS + h * 32, q);
                }
        }
        if (kTest && !cert_plain) {
            // lanes 0 .. 15: the loader waves of this wave's rows of A, lanes 16 .. 31: of its
            // columns of B (waves repeat where there are fewer than four), tile l % 4
            const int j = (lane >> 2) & 3, op = (lane >> 4) & 1;
            constexpr int LA = WROWS / 16, LB = WCOLS / 16;
            const int lw = op ? wn * LB + j % LB : wm * LA + j % LA;
            int m = cert_n[buf][op][lw][lane & 3];
            const int off = cert_stage ? cert_off : 0;
            // (the first pair's fragments set out while the flags are worked out)
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int h = 0; h < HS; ++h) {
                    if (h < RS) cert_fa[q][h] = frag(As[buf], wm * WROWS + h * 32, q);
                    if (h < CS) cert_fb[q][h] = frag(Bs[buf], wn * WCOLS + h * 32, q);
                }
            m = max_row_shr<4>(m);
            m = max_row_shr<8>(m);
            const int limit = kCert16 ? g.acc_hi * g.acc_hi : 127 * 127;      // (a <= 12: no overflow)
            int any_no = 0;
#pragma unroll
            for (int pr = 0; pr < NSTEP / 2; ++pr) {
                const int a0 = __builtin_amdgcn_readlane(m, 12 + 2 * pr), a1 = __builtin_amdgcn_readlane(m, 13 + 2 * pr);
                const int b0 = __builtin_amdgcn_readlane(m, 28 + 2 * pr), b1 = __builtin_amdgcn_readlane(m, 29 + 2 * pr);
                // (sums of squares of 32 codes: at most 2048 each)
                cert_ok[pr] = __builtin_amdgcn_readfirstlane((a0 * b0 <= limit && a1 * b1 <= limit) ? 1 : 0);
                asm volatile("s_xor_b32 %0, %1, 1" : "=s"(cert_no[pr]) : "s"(cert_ok[pr]) : "scc");
                any_no |= cert_no[pr];
            }
            if (cert_stage == 0) {
                if (any_no && lane == 0) cert_off = 1;
                cert_stage = 1;
            } else if (__builtin_amdgcn_readfirstlane(off)) {
                cert_plain = true;
            }
        }
        // Tiles of 16 and 32 codes: the waves that are multiplying and clamping go first
        // (measured on 4096^3 with tiles of 32: 156 -> 146 us; nothing for tiles of 64, and
        // the whole-stage loop loses 5 %, so it is left alone)
        if constexpr (kPairs32 || kPairs16) __builtin_amdgcn_s_setprio(1);
        if (kCert && (kGaveUp || cert_plain)) __builtin_amdgcn_s_setprio(1);

        if constexpr (kPairs16) {
            // two tiles per step
#pragma unroll
            for (int ks = 0; ks < NSTEP; ++ks) {
                v4i fa[RS], fb[CS];
#pragma unroll
                for (int h = 0; h < HS; ++h) {
                    if (h < RS) fa[h] = frag(As[buf], wm * WROWS + h * 32, ks);
                    if (h < CS) fb[h] = frag(Bs[buf], wn * WCOLS + h * 32, ks);
                }
                auto half = [](const v4i& f, int hi) -> long {
                    const v2i p = hi ? v2i{f.z, f.w} : v2i{f.x, f.y};
                    return __builtin_bit_cast(long, p);
                };
#pragma unroll
                for (int a = 0; a < RS; ++a)
#pragma unroll
                    for (int c = 0; c < CS; ++c) {
                        const v16i p0 = __builtin_amdgcn_mfma_i32_32x32x16_i8(half(fa[a], 0), half(fb[c], 0), zero, 0, 0, 0);
                        const v16i p1 = __builtin_amdgcn_mfma_i32_32x32x16_i8(half(fa[a], 1), half(fb[c], 1), zero, 0, 0, 0);
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            if constexpr (EPI == EPI_CLAMP_S16)
                                total[a][c][r] += clamp3(p0[r], lo, hi) + clamp3(p1[r], lo, hi);
                            else
                                total[a][c][r] = kSat16 ? add_sat16_pair(total[a][c][r], p0[r], p1[r], low_clear)
                                                        : add_sat8_pair(total[a][c][r], p0[r], p1[r]);
                        }
                    }
            }
        } else if (kCert && kGaveUp) {
            cert_clamped = true;
#pragma unroll
            for (int pr = 0; pr < NSTEP / 2; ++pr) {
                v4i fa[2][RS], fb[2][CS];
#pragma unroll
                for (int q = 0; q < 2; ++q)
#pragma unroll
                    for (int h = 0; h < HS; ++h) {
                        if (h < RS) fa[q][h] = frag(As[buf], wm * WROWS + h * 32, pr * 2 + q);
                        if (h < CS) fb[q][h] = frag(Bs[buf], wn * WCOLS + h * 32, pr * 2 + q);
                    }
#pragma unroll
                for (int a = 0; a < RS; ++a)
#pragma unroll
                    for (int c = 0; c < CS; ++c) {
                        const v16i p0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[0][a], fb[0][c], zero, 0, 0, 0);
                        const v16i p1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[1][a], fb[1][c], zero, 0, 0, 0);
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            total[a][c][r] = kCert16 ? add_sat16_pair(total[a][c][r], p0[r], p1[r], low_clear)
                                                     : add_sat8_pair_scaled(total[a][c][r], p0[r], p1[r]);
                    }
            }
        } else if (kCert) {
            // two tiles per half stage, straight onto the totals where the test allows it
#pragma unroll
            for (int pr = 0; pr < NSTEP / 2; ++pr) {
                v4i fa[2][RS], fb[2][CS];
#pragma unroll
                for (int q = 0; q < 2; ++q)
#pragma unroll
                    for (int h = 0; h < HS; ++h) {
                        if (h < RS) fa[q][h] = pr ? frag(As[buf], wm * WROWS + h * 32, pr * 2 + q) : cert_fa[q][h];
                        if (h < CS) fb[q][h] = pr ? frag(Bs[buf], wn * WCOLS + h * 32, pr * 2 + q) : cert_fb[q][h];
                    }
                if (cert_ok[pr]) {
#pragma unroll
                    for (int q = 0; q < 2; ++q)
#pragma unroll
                        for (int a = 0; a < RS; ++a)
#pragma unroll
                            for (int c = 0; c < CS; ++c)
                                total[a][c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[q][a], fb[q][c], total[a][c], 0, 0, 0);
                }
                if (cert_no[pr]) {
                    cert_clamped = true;
#pragma unroll
                    for (int a = 0; a < RS; ++a)
#pragma unroll
                        for (int c = 0; c < CS; ++c) {
                            const v16i p0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[0][a], fb[0][c], zero, 0, 0, 0);
                            const v16i p1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[1][a], fb[1][c], zero, 0, 0, 0);
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                total[a][c][r] = kCert16 ? add_sat16_pair(total[a][c][r], p0[r], p1[r], low_clear)
                                                         : add_sat8_pair_scaled(total[a][c][r], p0[r], p1[r]);
                        }
                }
            }
        } else if (kPairs32 || kPairs64) {
            // two tiles per half stage (s = 32) or per stage (s = 64)
#pragma unroll
            for (int pr = 0; pr < (kPairs32 ? NSTEP / 2 : 1); ++pr) {
                constexpr int SPT = kPairs32 ? 1 : 2;      // steps per tile
                v4i fa[2 * SPT][RS], fb[2 * SPT][CS];
#pragma unroll
                for (int q = 0; q < 2 * SPT; ++q)
#pragma unroll
                    for (int h = 0; h < HS; ++h) {
                        if (h < RS) fa[q][h] = frag(As[buf], wm * WROWS + h * 32, pr * 2 * SPT + q);
                        if (h < CS) fb[q][h] = frag(Bs[buf], wn * WCOLS + h * 32, pr * 2 * SPT + q);
                    }
#pragma unroll
                for (int a = 0; a < RS; ++a)
#pragma unroll
                    for (int c = 0; c < CS; ++c) {
                        v16i p0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[0][a], fb[0][c], zero, 0, 0, 0);
                        if (SPT == 2)
                            p0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[1][a], fb[1][c], p0, 0, 0, 0);
                        v16i p1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[SPT][a], fb[SPT][c], zero, 0, 0, 0);
                        if (SPT == 2)
                            p1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[SPT + 1][a], fb[SPT + 1][c], p1, 0, 0, 0);
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            total[a][c][r] = kSat16 ? add_sat16_pair(total[a][c][r], p0[r], p1[r], low_clear)
                                                    : add_sat8_pair(total[a][c][r], p0[r], p1[r]);
                    }
            }
        } else if (kReq) {
#pragma unroll
            for (int ks = 0; ks < NSTEP; ++ks) {
                v4i fa[RS], fb[CS];
#pragma unroll
                for (int h = 0; h < HS; ++h) {
                    if (h < RS) fa[h] = frag(As[buf], wm * WROWS + h * 32, ks);
                    if (h < CS) fb[h] = frag(Bs[buf], wn * WCOLS + h * 32, ks);
                }
                // (positions at or beyond k_end are zero in LDS: such a step lies beyond the
                // part's last tile and must not be counted as one)
                const bool inside = c_k + ks * KSTEP < k_end;
                if constexpr (kReqS32) {
                    // every step is a tile: the matrix core starts from zero each time
                    v16i p[RS][CS];
#pragma unroll
                    for (int a = 0; a < RS; ++a)
#pragma unroll
                        for (int c = 0; c < CS; ++c)
                            p[a][c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[a], fb[c], zero, 0, 0, 0);
                    if (inside) req_finish(p);
                } else {
                    if (step_in_tile == 0) {
#pragma unroll
                        for (int a = 0; a < RS; ++a)
#pragma unroll
                            for (int c = 0; c < CS; ++c)
                                part[a][c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[a], fb[c], zero, 0, 0, 0);
                    } else {
#pragma unroll
                        for (int a = 0; a < RS; ++a)
#pragma unroll
                            for (int c = 0; c < CS; ++c)
                                part[a][c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[a], fb[c], part[a][c], 0, 0, 0);
                    }
                    if (inside && ++step_in_tile == steps_per_tile) {
                        step_in_tile = 0;
                        req_finish(part);
                    }
                }
            }
        } else if (EPI == EPI_STAGES) {
            v4i fa[NSTEP][RS], fb[NSTEP][CS];
#pragma unroll
            for (int ks = 0; ks < NSTEP; ++ks)
#pragma unroll
                for (int h = 0; h < HS; ++h) {
                    if (h < RS) fa[ks][h] = frag(As[buf], wm * WROWS + h * 32, ks);
                    if (h < CS) fb[ks][h] = frag(Bs[buf], wn * WCOLS + h * 32, ks);
                }
#pragma unroll
            for (int ks = 0; ks < NSTEP; ++ks)
#pragma unroll
                for (int a = 0; a < RS; ++a)
#pragma unroll
                    for (int c = 0; c < CS; ++c)
                        part[a][c] =
                            __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[ks][a], fb[ks][c], part[a][c], 0, 0, 0);
            // issue order: the fragments of step ks + 1 are requested before the MFMAs of step ks
            // (left alone, the scheduler puts every read right in front of its use to save
            // registers, and each MFMA pair then waits a whole LDS round trip)
            constexpr int kReads = RS + CS, kMfmas = RS * CS;
            __builtin_amdgcn_sched_group_barrier(0x100, 2 * kReads, 0);
#pragma unroll
            for (int ks = 0; ks < NSTEP; ++ks) {
                __builtin_amdgcn_sched_group_barrier(0x008, kMfmas, 0);
                if (ks + 2 < NSTEP) __builtin_amdgcn_sched_group_barrier(0x100, kReads, 0);
            }
            step_in_tile += NSTEP;
            if (step_in_tile >= steps_per_tile) {
                step_in_tile = 0;
#pragma unroll
                for (int a = 0; a < RS; ++a)
#pragma unroll
                    for (int c = 0; c < CS; ++c)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            total[a][c][r] += clamp3(part[a][c][r], lo, hi);
                            part[a][c][r] = 0;
                        }
            }
        } else {
#pragma unroll
            for (int ks = 0; ks < NSTEP; ++ks) {
                v4i fa[RS], fb[CS];
#pragma unroll
                for (int h = 0; h < HS; ++h) {
                    if (h < RS) fa[h] = frag(As[buf], wm * WROWS + h * 32, ks);
                    if (h < CS) fb[h] = frag(Bs[buf], wn * WCOLS + h * 32, ks);
                }
#pragma unroll
                for (int a = 0; a < RS; ++a)
#pragma unroll
                    for (int c = 0; c < CS; ++c)
                        part[a][c] =
                            __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[a], fb[c], part[a][c], 0, 0, 0);
                if (++step_in_tile == steps_per_tile) {
                    step_in_tile = 0;
#pragma unroll
                    for (int a = 0; a < RS; ++a)
#pragma unroll
                        for (int c = 0; c < CS; ++c)
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                total[a][c][r] += clamp3(part[a][c][r], lo, hi);
                                part[a][c][r] = 0;
                            }
                }
            }
        }

        if constexpr (kPairs32 || kPairs16) __builtin_amdgcn_s_setprio(0);
        if (kCert && (kGaveUp || cert_plain)) __builtin_amdgcn_s_setprio(0);
        c_k += KS;
        if (c_k < k_end) return;

        // ---- end of the output tile (row0, c_ct)
        if ((EPI == EPI_GENERIC || EPI == EPI_STAGES) && step_in_tile != 0) {
            // a short last tile (D not a multiple of s) ends without reaching steps_per_tile
            step_in_tile = 0;
#pragma unroll
            for (int a = 0; a < RS; ++a)
#pragma unroll
                for (int c = 0; c < CS; ++c)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        total[a][c][r] += clamp3(part[a][c][r], lo, hi);
                        part[a][c][r] = 0;
                    }
        }
        if constexpr (kCert && !kCert16) {
            if (cert_clamped) {
                cert_clamped = false;
#pragma unroll
                for (int a = 0; a < RS; ++a)
#pragma unroll
                    for (int c = 0; c < CS; ++c)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int t = total[a][c][r], p = -t & 255;
                            total[a][c][r] = ((t + p) >> kScaleShift) - p;
                        }
            } else {
#pragma unroll
                for (int a = 0; a < RS; ++a)
#pragma unroll
                    for (int c = 0; c < CS; ++c)
#pragma unroll
                        for (int r = 0; r < 16; ++r) total[a][c][r] >>= kScaleShift;
            }
        }
        if constexpr (kReq) {
            if (step_in_tile != 0) {      // a short last tile (D not a multiple of s)
                step_in_tile = 0;
                req_finish(part);
            }
            req_tile = 0;
            if constexpr (kReqMax) {      // the first pass writes nothing but the maxima, at the very end
                c_k = k_begin;
                c_ct += gridDim.z;
                return;
            }
            // the second pass: take out the offsets 2^22 * m_t that came along with the codes
            const uint32_t corr = req_corr << 22;
            req_corr = 0;
#pragma unroll
            for (int a = 0; a < RS; ++a)
#pragma unroll
                for (int c = 0; c < CS; ++c)
#pragma unroll
                    for (int r = 0; r < 16; ++r) total[a][c][r] = (int)((uint32_t)total[a][c][r] - corr);
        }
        if constexpr (PAIR) {
            // ---- fold, pair mode (images of 256 pixels, one stage per tile): half 0 multiplied out
            // of buffer 0 and half 1 out of buffer 1, so the image's 256 pixel rows of accumulators
            // (int16) lie in four quarters of 64 -- As[0], Bs[0] (half 0, written while half 1
            // still needs the buffers 1), As[1], Bs[1] (half 1) -- and are folded after the second
            // half.  Offsets in int16 from the start of As.
            constexpr int AP = 130;      // pitch in int16 (65 dwords: neighbouring pixels, neighbouring banks)
            constexpr int kQuarter = 64 * AP;
            static_assert(sizeof(As[0]) >= ((size_t)kQuarter + BN) * sizeof(int16_t) &&
                          sizeof(Bs[0]) >= (size_t)kQuarter * sizeof(int16_t), "a quarter must fit one stage buffer");
            int16_t* accP = reinterpret_cast<int16_t*>(&As[0][0][0]);
            const int dB = (int)((reinterpret_cast<uintptr_t>(&Bs[0][0][0]) - reinterpret_cast<uintptr_t>(&As[0][0][0])) / 2);
            constexpr int dBuf = (int)(sizeof(As[0]) / 2);
            auto quarter = [&](int qi) { return (qi & 1) * dB + (qi >> 1) * dBuf; };
            __syncthreads();             // every wave is done reading this half's operands
            {
                // (a wave's 64 rows are one quarter: wm = 0, 1; rr + 4 * (lane >> 5) < 64)
                int16_t* dst = accP + quarter(2 * c_half + wm) + (4 * (lane >> 5)) * AP + lane_col;
#pragma unroll
                for (int a = 0; a < RS; ++a)
#pragma unroll
                    for (int c = 0; c < CS; ++c)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int rr = a * 32 + 8 * (r >> 2) + (r & 3);
                            dst[rr * AP + c * 32] = (int16_t)(total[a][c][r] >> fin_shift);
                            total[a][c][r] = 0;
                        }
            }
            c_k = k_begin;
            if (c_half == 0) {
                // the words read for taps outside the image, behind the first quarter
                if (tid < BN) accP[kQuarter + tid] = 0;
                c_half = 1;              // (the barrier of the next stage orders these writes)
                return;
            }
            c_half = 0;
            __syncthreads();
            const int W = g.fW, H = g.fH, kw = g.fkw, khw = g.fkh * g.fkw;
            const int q = tid & 255;                         // pixel of the image
            const int ry = q >> g.f_log2w, x = q & (W - 1);
            int off[9];
            int ty = 0, tx = 0;
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                const int ryp = ry - ty + f_ph, xp = x - tx + f_pw;
                const bool ok = t < khw && ryp >= 0 && ryp < H && xp >= 0 && xp < W;
                const int p = (ryp << g.f_log2w) + xp;
                off[t] = ok ? quarter(p >> 6) + (p & 63) * AP + t : kQuarter;
                if (++tx == kw) { tx = 0; ++ty; }
            }
            const int cbase = c_ct * g.f_cg;
            // the thread's channels: c0, c0 + 2, ... below c_end; their outputs lie a whole image apart
            const int c0 = tid >> 8, c_end = min(g.f_cg, g.fC - cbase);
            const int64_t o0 = ((int64_t)blockIdx.y * g.fC + cbase + c0) * (H * W) + q;
            const int64_t o_step = (int64_t)(NTHREADS / 256) * (H * W);
            float* po = g.out + o0;
            const float* pm = g.mask_src ? g.mask_src + o0 : nullptr;
            const int16_t* col = accP + c0 * khw;
            for (int c = c0; c < c_end; c += NTHREADS / 256) {
                int sum = 0;
#pragma unroll
                for (int t = 0; t < 9; ++t) sum += col[off[t]];
                float f = (float)sum * dq;
                if (pm) { f = pm[0] > 0.0f ? f : 0.0f; pm += o_step; }
                po[0] = f;
                po += o_step;
                col += (NTHREADS / 256) * khw;
            }
            __syncthreads();             // the next stage overwrites the buffers the sums were read from
            c_ct += gridDim.z;
            return;
        }
        if constexpr (FOLD) {
            // ---- fold: the tile's accumulators go to LDS (int16: at most 255 tiles of +-128),
            // then every thread adds up the kh*kw taps of its pixels and channels.  Both operand
            // buffers are free here: the stages still to come are in registers.
            constexpr int AP = 130;      // pitch in int16 (65 dwords: neighbouring pixels, neighbouring banks)
            static_assert(sizeof(As) >= ((size_t)BM * AP + BN) * sizeof(int16_t), "accumulator tile must fit the A buffers");
            int16_t* accT = reinterpret_cast<int16_t*>(&As[0][0][0]);
            __syncthreads();             // every wave is done reading this stage's operands
#pragma unroll
            for (int a = 0; a < RS; ++a)
#pragma unroll
                for (int c = 0; c < CS; ++c)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int rr = a * 32 + 8 * (r >> 2) + (r & 3);
                        const int v = total[a][c][r] >> fin_shift;
                        total[a][c][r] = 0;
                        accT[(lane_row + rr) * AP + lane_col + c * 32] = (int16_t)v;
                    }
            // the word behind the tile, read for taps outside the image; c * khw + BM * AP stays
            // inside the A buffers for every channel of a column tile
            if (tid < BN) accT[BM * AP + tid] = 0;
            __syncthreads();
            const int W = g.fW, H = g.fH, kw = g.fkw, khw = g.fkh * g.fkw;
            const int q = tid & (BM - 1);                 // pixel of the tile
            int il = 0, ry, rows_part, y;
            int64_t b;
            bool out_ok;
            const int x = q & (W - 1);
            if (g.f_imgs) {                               // whole images: q = (image, row, position)
                il = q >> g.f_log2hw;
                ry = (q & ((1 << g.f_log2hw) - 1)) >> g.f_log2w;
                rows_part = H;
                b = (int64_t)blockIdx.y * g.f_imgs + il;
                y = ry;
                out_ok = b < g.fbatch;
            } else {                                      // a strip of one image, halo rows first and last
                ry = q >> g.f_log2w;
                rows_part = g.f_rows_c;
                b = f_img;
                y = f_y0 + ry;
                out_ok = ry >= f_ph && ry < f_ph + g.f_rows_out && y < H;
            }
            const int cbase = c_ct * g.f_cg;
            const int16_t* img_part = accT + (il << g.f_log2hw) * AP;      // (il = 0 in strip mode)
            if (khw <= 9) {
                // up to nine taps: where each one reads, worked out once for the pixel (a tap whose
                // source pixel lies outside reads the zero word behind the tile), then three
                // instructions per tap and channel
                int off[9];
                int ty = 0, tx = 0;
#pragma unroll
                for (int t = 0; t < 9; ++t) {
                    const int ryp = ry - ty + f_ph, xp = x - tx + f_pw;
                    const bool ok = t < khw && ryp >= 0 && ryp < rows_part && xp >= 0 && xp < W;
                    off[t] = ok ? ((il << g.f_log2hw) + (ryp << g.f_log2w) + xp) * AP + t : BM * AP;
                    if (++tx == kw) { tx = 0; ++ty; }
                }
                for (int c = tid / BM; c < g.f_cg; c += NTHREADS / BM) {
                    if (!out_ok || cbase + c >= g.fC) continue;
                    const int16_t* col = accT + c * khw;
                    int sum = 0;
#pragma unroll
                    for (int t = 0; t < 9; ++t) sum += col[off[t]];
                    const int64_t o = (((int64_t)b * g.fC + cbase + c) * H + y) * W + x;
                    g.out[o] = (g.mask_src && !(g.mask_src[o] > 0.0f)) ? 0.0f : (float)sum * dq;
                }
            } else {
                for (int c = tid / BM; c < g.f_cg; c += NTHREADS / BM) {
                    if (!out_ok || cbase + c >= g.fC) continue;
                    int sum = 0;
                    for (int ty = 0; ty < g.fkh; ++ty) {
                        const int ryp = ry - ty + f_ph;
                        if (ryp < 0 || ryp >= rows_part) continue;
                        for (int tx = 0; tx < kw; ++tx) {
                            const int xp = x - tx + f_pw;
                            if (xp < 0 || xp >= W) continue;
                            sum += img_part[((ryp << g.f_log2w) + xp) * AP + c * khw + ty * kw + tx];
                        }
                    }
                    const int64_t o = (((int64_t)b * g.fC + cbase + c) * H + y) * W + x;
                    g.out[o] = (g.mask_src && !(g.mask_src[o] > 0.0f)) ? 0.0f : (float)sum * dq;
                }
            }
            __syncthreads();             // the next stage overwrites the buffers the sums were read from
            c_k = k_begin;
            c_ct += gridDim.z;
            return;
        }
        // Element (a, c, r) of the lane lies at tile_off + (32a + 8(r/4) + r%4) RB + 32c
        // (uniform) + lane_off (per lane, 32 bits: RB <= 2^21 on this path).
        const int64_t col0 = (int64_t)c_ct * TN;
        const int64_t tile_off = row0 * g.RB + col0;
        const bool interior = (row0 + TM <= g.RA) && (col0 + TN <= g.RB);
        float* ob = (g.splits == 1 && g.out) ? g.out + tile_off : nullptr;
        // (the narrow output has kernel instances of its own: its epilogue costs the others registers)
        uint16_t* hb = (BF16 && g.splits == 1 && g.out_bf16) ? g.out_bf16 + tile_off : nullptr;
        // bfloat16 output of an interior tile with an even row length: lanes l and l ^ 1 hold
        // neighbouring columns and trade their values, so that every lane stores one dword
        const bool pair_bf16 = hb && interior && (g.RB % 2 == 0);
        const bool slice16 = g.splits > 1 && g.partial16;
        int32_t* ab = slice16 ? nullptr
                              : (g.splits > 1 ? g.partial + (int64_t)blockIdx.x * g.RA * g.RB + tile_off
                                              : (g.acc_out ? g.acc_out + tile_off : nullptr));
        int16_t* ab16 = slice16 ? reinterpret_cast<int16_t*>(g.partial) + (int64_t)blockIdx.x * g.RA * g.RB + tile_off
                                : nullptr;
        if constexpr (BF16) if (pair_bf16) {
            const bool odd = lane & 1;
            auto value = [&](int t) -> float {
                return (float)(t >> fin_shift) * dq;
            };
            // quad_perm [1,0,3,2]: the value of lane ^ 1
            auto neighbour = [](float f) -> float {
                return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(f), 0xB1, 0xF, 0xF, true));
            };
            // two binary32 values -> two bfloat16 in one dword (v_cvt_pk_bf16_f32: nearest even)
            auto pack = [](float lo, float hi) -> uint32_t {
                const f2 v = {lo, hi};
                return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf2));
            };
#pragma unroll
            for (int a = 0; a < RS; ++a) {
                if constexpr (CS == 2) {
                    // 64 columns per wave: the even lanes store the pairs of the left 32-column
                    // block, the odd lanes those of the right one, so the 32 lanes that share a
                    // row write its whole 128-byte line with one instruction
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float f0 = value(total[a][0][r]), f1 = value(total[a][CS - 1][r]);
                        const float n0 = neighbour(f0), n1 = neighbour(f1);
                        const uint32_t word = pack(odd ? n1 : f0, odd ? f1 : n0);
                        const int rr = a * 32 + 8 * (r >> 2) + (r & 3);
                        const uint32_t off = lane_off + (odd ? 31u : 0u);
                        uint32_t* dst = reinterpret_cast<uint32_t*>(hb + (int64_t)rr * g.RB + off);
                        if (STREAM) __builtin_nontemporal_store(word, dst);
                        else *dst = word;
                    }
                } else {
                    // 32 columns per wave: the even lane stores both columns of row r, the odd
                    // lane both columns of row r + 1 (r even): 64-byte pieces of four rows
#pragma unroll
                    for (int r = 0; r < 16; r += 2) {
                        const float f0 = value(total[a][0][r]), f1 = value(total[a][0][r + 1]);
                        const float n0 = neighbour(f0), n1 = neighbour(f1);
                        const uint32_t word = pack(odd ? n1 : f0, odd ? f1 : n0);
                        const int rr = a * 32 + 8 * (r >> 2) + (r & 3);
                        const uint32_t off = lane_off + (odd ? (uint32_t)g.RB - 1u : 0u);
                        uint32_t* dst = reinterpret_cast<uint32_t*>(hb + (int64_t)rr * g.RB + off);
                        if (STREAM) __builtin_nontemporal_store(word, dst);
                        else *dst = word;
                    }
                }
            }
        }
        // The common case on a path of its own -- fp32 output only, a tile inside the output:
        // nothing is tested per element, so the 32 stores of a wave are one run of
        // conversions and stores (with the tests, each store sat in an exec-masked block of
        // its own behind its own branches).
        const bool plain_out = !MASK && interior && ob && !ab && !ab16 && !(BF16 && hb);
        if (plain_out) {
#pragma unroll
            for (int a = 0; a < RS; ++a)
#pragma unroll
                for (int c = 0; c < CS; ++c)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int rr = a * 32 + 8 * (r >> 2) + (r & 3);
                        const int64_t uo = (int64_t)rr * g.RB + c * 32;
                        const float f = (float)(total[a][c][r] >> fin_shift) * dq;
                        total[a][c][r] = 0;
                        if (STREAM) __builtin_nontemporal_store(f, &(ob + uo)[lane_off]);
                        else (ob + uo)[lane_off] = f;
                    }
        }
        // the same for the 16-bit slices of a split contraction (measured on the benchmark
        // layer's weight gradient: 25.4 -> 23.2 us; a third block for 32-bit slices made every
        // kernel a little slower and nothing faster)
        const bool plain_slices = interior && ab16 && !ob && !ab && !(BF16 && hb);
        if (plain_slices) {
#pragma unroll
            for (int a = 0; a < RS; ++a)
#pragma unroll
                for (int c = 0; c < CS; ++c)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int rr = a * 32 + 8 * (r >> 2) + (r & 3);
                        const int64_t uo = (int64_t)rr * g.RB + c * 32;
                        (ab16 + uo)[lane_off] = (int16_t)(total[a][c][r] >> fin_shift);
                        total[a][c][r] = 0;
                    }
        }
        if (!plain_out && !plain_slices) {
#pragma unroll
        for (int a = 0; a < RS; ++a)
#pragma unroll
            for (int c = 0; c < CS; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int rr = a * 32 + 8 * (r >> 2) + (r & 3);
                    const int64_t uo = (int64_t)rr * g.RB + c * 32;
                    const int v = total[a][c][r] >> fin_shift;
                    total[a][c][r] = 0;
                    bool ok = interior;
                    if (!interior)
                        ok = (row0 + lane_row + rr < g.RA) && (col0 + lane_col + c * 32 < g.RB);
                    if (BF16 && hb && !pair_bf16 && ok) (hb + uo)[lane_off] = (uint16_t)bf16_bits((float)v * dq);
                    if (ok) {
                        if (ab) (ab + uo)[lane_off] = v;
                        if (ab16) (ab16 + uo)[lane_off] = (int16_t)v;
                        if (ob) {
                            // (a template flag, not a run-time branch: merging the two stores
                            // would drop the streaming hint)
                            float f = (float)v * dq;
                            if constexpr (MASK) f = mk[a][c][r] > 0.0f ? f : 0.0f;
                            if (STREAM) __builtin_nontemporal_store(f, &(ob + uo)[lane_off]);
                            else (ob + uo)[lane_off] = f;
                        }
                    }
                }
        }
        // the next tile's mask values set out now: a tile's worth of time to arrive
        if constexpr (MASK) prefetch_mask(c_ct + (int)gridDim.z);
        c_k = k_begin;
        c_ct += gridDim.z;
    };
    if constexpr (MASK) prefetch_mask(c_ct);

    // The global loads run two stages ahead of the multiplication where the registers allow
    // it (one stage of 128 codes is 8 MFMAs per wave, about 0.5 us of matrix time per SIMD,
    // less than a trip to L2 under load), one stage ahead in the s = 64 instance, which has
    // no eight registers to spare at four waves per SIMD.
    // (the fold epilogue needs the registers; with a byte per code a stage in flight is twice as many)
    constexpr bool kDeep = !kPairs64 && !FOLD && !WIDE;
    // EPI_CERT8_S32 has the loop of its given-up stages (see `stage`) in the instances for
    // outputs that stay in the caches.  Those for streamed outputs go on in the testing stage
    // with every flag down: with the second loop compiled in, their testing stage came out 14 %
    // slower (the forward product of the 65536 x 1152 x 128 layer: 25.7 against 22.6 us), and
    // the one given-up case measured there, that layer's input gradient, is 10 % faster with
    // its clamps cut into pairs (67.4 against 75.6 us: it is bound by its stores).
    constexpr bool kTwoLoops = kCert && !STREAM;
    if constexpr (kDeep) {
        Staged<UNITS * REGS, UNITS_B * REGS> st0, st1;
        fetch_next(st0);
        fetch_next(st1);
        while (c_ct < n_ct) {       // stage() advances c_ct at the end of a tile
            stage(st0, 0, std::false_type{});
            if (c_ct >= n_ct) break;
            stage(st1, 1, std::false_type{});
            if (kTwoLoops && cert_plain) break;      // (left where the buffers are back in step)
        }
        if constexpr (kTwoLoops) {
            while (c_ct < n_ct) {
                stage(st0, 0, std::true_type{});
                if (c_ct >= n_ct) break;
                stage(st1, 1, std::true_type{});
            }
        }
    } else {
        Staged<UNITS * REGS, UNITS_B * REGS> st;
        fetch_next(st);
        int buf = 0;
        while (c_ct < n_ct) {
            stage(st, buf, std::false_type{});
            buf ^= 1;
        }
    }
    if constexpr (kReqMax) {
        // this workgroup's maxima (every output tile it walked) into the tensor's
        __syncthreads();
        for (int i = tid; i < (int)(t_end - t_begin); i += NTHREADS) {
            const uint32_t m = (uint32_t)req_m[i] >> kScaleShift;
            if (m) atomicMax(&g.tile_max[t_begin + i], m);
        }
    }
}

bool sat8_path(const GemmArgs& g) { return g.acc_hi == 127 && (g.s == 16 || g.s == 32 || g.s == 64); }

// Saturation through the int16 conversion (EPI_SAT16): accumulators of bA + bB to 16 bits,
// tiles of 32 or 64 codes.  Fills in the operand factors when `plan` is given.
bool sat16_path(const GemmArgs& g, GemmArgs* plan = nullptr)
{
    if ((g.s != 16 && g.s != 32 && g.s != 64) || g.fold || g.out_bf16 || g.acc_hi > 32767) return false;
    if ((g.bA > 4) != (g.bB > 4)) return false;
    if (g.bA <= 4 && sat8_path(g)) return false;      // has its own, cheaper instances
    int a = 1;
    while (((int64_t)1 << (a - 1)) - 1 < g.acc_hi) ++a;
    // a code of b bits times 2^(8 - b) still fits a byte; packed codes are unpacked as 4-bit ones
    const int capA = g.bA > 4 ? 8 - g.bA : 4, capB = g.bB > 4 ? 8 - g.bB : 4;
    const int need = 16 - a;
    if (need > capA + capB) return false;
    if (g.tiles_per_split >= 65536) return false;     // totals carry the factor 2^need: |.| <= tiles * 2^15
    if (plan) {
        plan->jA = need < capA ? need : capA;
        plan->jB = need - plan->jA;
        plan->fin_shift = need;
    }
    return true;
}

} // namespace

// Geometries the fold epilogue takes: W a power of two up to 128; either whole images per
// 128-pixel row tile (H*W a power of two up to 128) or strips of 128 / W image rows of which
// kh - 1 are halo (recomputed by the neighbouring strips); odd windows of at most 128 taps.
bool gemm_fold_plan(GemmArgs* g, int64_t batch, int C, int H, int W, int kh, int kw)
{
    auto pow2 = [](int v) { return v > 0 && (v & (v - 1)) == 0; };
    auto log2i = [](int v) { int l = 0; while ((1 << l) < v) ++l; return l; };
    if (batch < 1 || C < 1 || H < 1 || W < 1 || kh < 1 || kw < 1 || kh % 2 == 0 || kw % 2 == 0) return false;
    if (!pow2(W) || W > BM || kh * kw > BN || kh > 15 || kw > 15) return false;
    if (g->RA != batch * (int64_t)H * W || g->RB != (int64_t)C * kh * kw || g->D % KSTEP != 0) return false;
    g->splits = 1;                        // short contractions; the fold needs whole totals
    g->tiles_per_split = g->n_tiles;
    if (batch * (int64_t)C * H * W >= ((int64_t)1 << 40)) return false;
    g->fold = 1;
    g->fbatch = batch; g->fC = C; g->fH = H; g->fW = W; g->fkh = kh; g->fkw = kw;
    g->f_log2w = log2i(W);
    g->f_cg = BN / (kh * kw);
    const int64_t hw = (int64_t)H * W;
    if (hw <= BM) {
        if (!pow2((int)hw)) return false;
        g->f_imgs = BM / (int)hw;
        g->f_log2hw = log2i((int)hw);
        g->f_rows_c = H; g->f_rows_out = H; g->f_strips = 1;
    } else if (hw == 2 * BM && kh * kw <= 9 && kh * kw > 1 && g->D <= KS_LONG && batch <= 65535) {
        // an image is two row tiles and a tile one stage: both halves in one workgroup, no halo
        g->f_pair = 1;
        g->f_imgs = 0;
        g->f_log2hw = 8;
        g->f_rows_c = H; g->f_rows_out = H; g->f_strips = 1;
    } else {
        g->f_imgs = 0;
        g->f_log2hw = 7;                  // unused: one image part per tile
        g->f_rows_c = BM / W;
        g->f_rows_out = g->f_rows_c - (kh - 1);
        if (g->f_rows_out < 1) return false;
        g->f_strips = (H + g->f_rows_out - 1) / g->f_rows_out;
        if (batch * g->f_strips > 65535) return false;      // grid.y
    }
    if (g->f_imgs && (batch + g->f_imgs - 1) / g->f_imgs > 65535) return false;
    // int16 accumulator tile: |total| <= tiles * min(2^(a-1), what a tile's products can add up to)
    const int64_t tile_sum = g->s * (((int64_t)1 << (g->bA - 1)) * ((int64_t)1 << (g->bB - 1)));
    const int64_t per_tile = tile_sum < (int64_t)g->acc_hi + 1 ? tile_sum : (int64_t)g->acc_hi + 1;
    if (per_tile > 32767 || per_tile * g->n_tiles > 32767) return false;
    return gemm_fast_eligible(*g);
}

bool gemm_fast_eligible(const GemmArgs& g)
{
    if ((g.bA > 4) != (g.bB > 4)) return false;      // packed or bytes, the same on both sides
    // rows of whole dwords (the 16-byte loads then start on one); a row may end inside a 32-code
    // unit, whose remainder the kernel clears
    if (g.D % (g.bA > 4 ? 4 : 8) != 0) return false;
    if (g.RB > ((int64_t)1 << 21)) return false;     // 32-bit offsets inside an output tile
    // 32-bit offsets into the operands, with room for the "outside" offset
    if ((g.RA + 256) * g.pitchA >= ((int64_t)1 << 31) || (g.RB + 256) * g.pitchB >= ((int64_t)1 << 31)) return false;
    if (g.s == 16) {
        // two tiles per 32-code step: saturating epilogues only, parts that start on a step
        if (g.fold || g.out_bf16 || (g.splits > 1 && g.tiles_per_split % 2 != 0)) return false;
        if (sat16_path(g) || (g.bA <= 4 && sat8_path(g))) return true;
        // compare-select clamp: totals (times 256 with packed codes) must stay inside int32
        const int64_t max_prod = ((int64_t)1 << (g.bA - 1)) * ((int64_t)1 << (g.bB - 1));
        const int64_t tile_max = 16 * max_prod, acc_max = (int64_t)g.acc_hi + 1;
        const int64_t per_tile = tile_max < acc_max ? tile_max : acc_max;
        return per_tile * g.tiles_per_split < ((int64_t)1 << (g.bA > 4 ? 31 : 22));
    }
    if (g.s % KSTEP != 0) return false;
    if (sat16_path(g)) return true;
    if (g.bA > 4) {
        // a byte per code: nothing is scaled; a tile's sum (|code| <= 128 on both sides) and
        // a part's total must stay inside int32
        if (g.fold || g.out_bf16) return false;
        const int64_t tile_max = g.s << 14, acc_max = (int64_t)g.acc_hi + 1;
        const int64_t per_tile = tile_max < acc_max ? tile_max : acc_max;
        if (g.s >= ((int64_t)1 << 16)) return false;
        return per_tile * g.tiles_per_split < ((int64_t)1 << 31);
    }
    if (sat8_path(g)) return true;      // unscaled int32 total: covered by the API's range check
    // generic epilogue: totals carry a factor 256 and must stay inside int32
    const int64_t tile_max = g.s * 64;                            // |code| <= 8 on both sides
    const int64_t acc_max = (int64_t)g.acc_hi + 1;
    const int64_t per_tile = tile_max < acc_max ? tile_max : acc_max;
    if (tile_max >= ((int64_t)1 << 22)) return false;
    return per_tile * g.tiles_per_split < ((int64_t)1 << 22);
}

// Whether the kernel applies g.mask_src itself: the fold epilogue, and the instances of the
// packed-code epilogues HDQT_LAUNCH_I4 covers with a whole, unsplit output.  Everything else
// is masked by a pass of its own after the matmul (or by the pass that adds a split
// contraction's slices).
bool gemm_fast_masks(const GemmArgs& g)
{
    if (!g.mask_src || !g.out || !gemm_fast_eligible(g)) return false;
    if (g.fold) return true;
    if (g.splits > 1 || g.out_bf16 || g.bA > 4 || g.s == 16) return false;
    return !sat16_path(g);
}

// Outputs of at most 64 columns take the 128 x 64 workgroup tile where such instances exist
// (packed codes, fp32 / int32 output, the epilogues of the paper's settings).
static bool narrow_tiles(const GemmArgs& g)
{
    if (g.RB > 64 || g.fold || g.out_bf16 || g.bA > 4 || g.s == 16 || g.mask_src) return false;
    return !sat16_path(g);
}

// Tiles of 32 packed codes with 8-bit accumulators take the instances that test whether a tile
// can saturate at all (EPI_CERT8_S32) where the plain fp32 / int32 output is asked for, a
// part has at most 255 tiles (the count of upward saturations must fit the totals' low byte)
// and at least five stages: the test costs a quarter of a clamped stage and can only be given
// up from the third stage on, so on short contractions (an input gradient over 64 to 512
// output channels) it loses 5 to 10 % where it fails and gains little where it holds.  The
// 128 x 64 tile has no such instance either (half the clamps per wave to save, the same test
// to pay: 4 % slower on the 262144 x 576 x 64 layer).
// One more case, by measurement alone: a streamed output that a workgroup walks across for
// eight column tiles or more (the input gradient of the 65536 x 1152 x 128 layer: one stage
// per tile, codes that fail the test, so the workgroups give it up at their second tile) runs
// 5 % faster in these instances' given-up state than in EPI_SAT8_S32 -- 68 against 72 us, in
// six interleaved runs; with fewer column tiles (576 or 320 columns) it is 5 to 7 % slower.
static bool cert_tiles(const GemmArgs& g, int64_t n_ct)
{
    if (g.fold || g.out_bf16 || g.bA > 4 || g.bB > 4 || g.mask_src) return false;
    if (g.acc_hi != 127 || g.s != 32 || g.tiles_per_split > 255) return false;
    if (g.tiles_per_split * g.s > 4 * KS_LONG) return true;
    return g.stream_out && n_ct >= 8 && g.D >= KS_LONG;
}

// The same test in front of the int16-saturation instances (EPI_CERT16_S32): packed codes, at
// least five stages per part, accumulators narrow enough for the squared bound to fit 32 bits.
static bool cert16_tiles(const GemmArgs& g)
{
    if (g.bA > 4 || g.bB > 4 || g.mask_src || g.s != 32 || g.acc_hi > 2047) return false;
    return g.tiles_per_split * g.s > 4 * KS_LONG;
}

// Second reading of the accumulator in this kernel: packed 4-bit codes on both sides, tiles that
// are whole 32-code steps, accumulators of at most 16 bits (the rounding by addition needs
// |value| < 2^22), at most kReqTable tiles per part, tile sums times 256 inside int32.
bool gemm_requant_fast_eligible(const GemmArgs& g, int acc_bits)
{
    if (g.bA > 4 || g.bB > 4 || g.fold || g.out_bf16 || g.mask_src) return false;
    if (g.D % 8 != 0 || g.s % KSTEP != 0) return false;
    if (acc_bits < 2 || acc_bits > 16) return false;
    if (g.RB > ((int64_t)1 << 21)) return false;
    if ((g.RA + 256) * g.pitchA >= ((int64_t)1 << 31) || (g.RB + 256) * g.pitchB >= ((int64_t)1 << 31)) return false;
    if (g.tiles_per_split > kReqTable) return false;
    return g.s * 64 < ((int64_t)1 << 22);
}

hipError_t launch_gemm_requant_fast(const GemmArgs& g_in, int acc_bits, int pass, hipStream_t stream)
{
    GemmArgs g = g_in;
    g.req_bits = acc_bits;
    g.req_lo = kReqMagic - (float)(1 << (acc_bits - 1));
    g.req_hi = kReqMagic + (float)((1 << (acc_bits - 1)) - 1);
    const int64_t n_ct = (g.RB + BN - 1) / BN, n_rt = (g.RA + BM - 1) / BM;
    const int64_t stages = (g.tiles_per_split * g.s + KS_LONG - 1) / KS_LONG;
    int64_t gx = n_ct;
    if (stages <= 2) {
        gx = (512 + n_rt * g.splits - 1) / (n_rt * g.splits);
        if (gx > n_ct) gx = n_ct;
        if (gx < 1) gx = 1;
    }
    const dim3 grid((unsigned)g.splits, (unsigned)n_rt, (unsigned)gx), block(64 * kWaves);
    ProfileScope ps(pass == 1 ? K_REQUANT_TILES : K_REQUANT_SUM, stream);
#define HDQT_LAUNCH_REQ(EPI, STREAM) \
    hipLaunchKernelGGL((gemm_i4_kernel<EPI, KS_LONG, STREAM, kWaves, false, false>), grid, block, 0, stream, g)
    const bool s32 = g.s == KSTEP;
    if (pass == 1) {
        if (s32) HDQT_LAUNCH_REQ(EPI_REQ_MAX_S32, false);
        else HDQT_LAUNCH_REQ(EPI_REQ_MAX, false);
    } else if (g.stream_out) {
        if (s32) HDQT_LAUNCH_REQ(EPI_REQ_SUM_S32, true);
        else HDQT_LAUNCH_REQ(EPI_REQ_SUM, true);
    } else {
        if (s32) HDQT_LAUNCH_REQ(EPI_REQ_SUM_S32, false);
        else HDQT_LAUNCH_REQ(EPI_REQ_SUM, false);
    }
#undef HDQT_LAUNCH_REQ
    return hipGetLastError();
}

hipError_t launch_gemm_fast(const GemmArgs& g_in, hipStream_t stream)
{
    GemmArgs g = g_in;
    const bool wide = g.bA > 4;
    const int64_t lo = (int64_t)g.acc_lo * (wide ? 1 : 256), hi = (int64_t)g.acc_hi * (wide ? 1 : 256);
    g.acc_lo_scaled = lo < INT32_MIN ? INT32_MIN : (int)lo;
    g.acc_hi_scaled = hi > INT32_MAX ? INT32_MAX : (int)hi;
    // Short contractions (at most two stages per output tile): a workgroup walks along
    // its row strip of the output as long as that leaves about two workgroups per CU.
    const bool narrow = narrow_tiles(g);
    int64_t n_ct = (g.RB + BN - 1) / BN, n_rt = (g.RA + BM - 1) / BM;
    if (narrow) n_ct = (g.RB + 63) / 64;
    if (g.fold) {
        n_ct = (g.fC + g.f_cg - 1) / g.f_cg;
        n_rt = g.f_imgs ? (g.fbatch + g.f_imgs - 1) / g.f_imgs : g.fbatch * g.f_strips;      // (pair mode: images)
    }
    const bool s32 = sat8_path(g) && g.s == 32;
    const bool sat16 = sat16_path(g, &g);
    const bool masked = gemm_fast_masks(g) && !g.fold;
    const int64_t KS = KS_LONG;
    const int64_t stages = (g.tiles_per_split * g.s + KS - 1) / KS;
    int64_t gx = n_ct;
    if (stages <= 2) {
        gx = (512 + n_rt * g.splits - 1) / (n_rt * g.splits);
        if (gx > n_ct) gx = n_ct;
        if (gx < 1) gx = 1;
    }
    const dim3 grid((unsigned)g.splits, (unsigned)n_rt, (unsigned)gx);
    ProfileScope ps(g.profile_tag ? K_GEMM_I4_FWD + (g.profile_tag - 1) : K_GEMM_I4, stream);
#define HDQT_LAUNCH_I4(EPI)                                                                          \
    do {                                                                                             \
        const dim3 block(64 * kWaves);                                                               \
        if (masked) {                                                                                \
            if (g.stream_out) hipLaunchKernelGGL((gemm_i4_kernel<EPI, KS_LONG, true, kWaves, false, false, false, false, true>), grid, block, 0, stream, g); \
            else hipLaunchKernelGGL((gemm_i4_kernel<EPI, KS_LONG, false, kWaves, false, false, false, false, true>), grid, block, 0, stream, g); \
        } else if (g.fold && g.f_pair)                                                               \
            hipLaunchKernelGGL((gemm_i4_kernel<EPI, KS_LONG, false, kWaves, false, true, false, false, false, true>), grid, block, 0, stream, g); \
        else if (g.fold)                                                                             \
            hipLaunchKernelGGL((gemm_i4_kernel<EPI, KS_LONG, false, kWaves, false, true>), grid, block, 0, stream, g); \
        else if (narrow) {                                                                           \
            if (g.stream_out) hipLaunchKernelGGL((gemm_i4_kernel<EPI, KS_LONG, true, kWaves, false, false, false, true>), grid, block, 0, stream, g); \
            else hipLaunchKernelGGL((gemm_i4_kernel<EPI, KS_LONG, false, kWaves, false, false, false, true>), grid, block, 0, stream, g); \
        } else if (g.out_bf16) {                                                                     \
            if (g.stream_out) hipLaunchKernelGGL((gemm_i4_kernel<EPI, KS_LONG, true, kWaves, true, false>), grid, block, 0, stream, g); \
            else hipLaunchKernelGGL((gemm_i4_kernel<EPI, KS_LONG, false, kWaves, true, false>), grid, block, 0, stream, g); \
        } else if (g.stream_out)                                                                     \
            hipLaunchKernelGGL((gemm_i4_kernel<EPI, KS_LONG, true, kWaves, false, false>), grid, block, 0, stream, g); \
        else                                                                                         \
            hipLaunchKernelGGL((gemm_i4_kernel<EPI, KS_LONG, false, kWaves, false, false>), grid, block, 0, stream, g); \
    } while (0)
#define HDQT_LAUNCH_SAT16(EPI, WIDE)                                                                  \
    do {                                                                                             \
        const dim3 block(64 * kWaves);                                                               \
        if (g.stream_out) hipLaunchKernelGGL((gemm_i4_kernel<EPI, KS_LONG, true, kWaves, false, false, WIDE>), grid, block, 0, stream, g); \
        else hipLaunchKernelGGL((gemm_i4_kernel<EPI, KS_LONG, false, kWaves, false, false, WIDE>), grid, block, 0, stream, g); \
    } while (0)
    if (g.s == 16) {
        if (sat16 && wide) HDQT_LAUNCH_SAT16(EPI_SAT16_S16, true);
        else if (sat16) HDQT_LAUNCH_SAT16(EPI_SAT16_S16, false);
        else if (!wide && sat8_path(g)) HDQT_LAUNCH_SAT16(EPI_SAT8_S16, false);
        else if (wide) HDQT_LAUNCH_SAT16(EPI_CLAMP_S16, true);
        else HDQT_LAUNCH_SAT16(EPI_CLAMP_S16, false);
    } else if (sat16) {
        if (wide && g.s == 32) HDQT_LAUNCH_SAT16(EPI_SAT16_S32, true);
        else if (wide) HDQT_LAUNCH_SAT16(EPI_SAT16_S64, true);
        else if (g.s == 32 && cert16_tiles(g)) HDQT_LAUNCH_SAT16(EPI_CERT16_S32, false);
        else if (g.s == 32) HDQT_LAUNCH_SAT16(EPI_SAT16_S32, false);
        else HDQT_LAUNCH_SAT16(EPI_SAT16_S64, false);
    } else if (wide) {
        const dim3 block(64 * kWaves);
        if (g.s % KS_LONG == 0) {
            if (g.stream_out) hipLaunchKernelGGL((gemm_i4_kernel<EPI_STAGES, KS_LONG, true, kWaves, false, false, true>), grid, block, 0, stream, g);
            else hipLaunchKernelGGL((gemm_i4_kernel<EPI_STAGES, KS_LONG, false, kWaves, false, false, true>), grid, block, 0, stream, g);
        } else {
            if (g.stream_out) hipLaunchKernelGGL((gemm_i4_kernel<EPI_GENERIC, KS_LONG, true, kWaves, false, false, true>), grid, block, 0, stream, g);
            else hipLaunchKernelGGL((gemm_i4_kernel<EPI_GENERIC, KS_LONG, false, kWaves, false, false, true>), grid, block, 0, stream, g);
        }
    } else if (s32 && !masked && !narrow && cert_tiles(g, n_ct)) {
        const dim3 block(64 * kWaves);
        if (g.stream_out)
            hipLaunchKernelGGL((gemm_i4_kernel<EPI_CERT8_S32, KS_LONG, true, kWaves, false, false>), grid, block, 0, stream, g);
        else
            hipLaunchKernelGGL((gemm_i4_kernel<EPI_CERT8_S32, KS_LONG, false, kWaves, false, false>), grid, block, 0, stream, g);
    } else if (s32) HDQT_LAUNCH_I4(EPI_SAT8_S32);
    else if (sat8_path(g)) HDQT_LAUNCH_I4(EPI_SAT8_S64);
    else if (g.s % KS_LONG == 0) HDQT_LAUNCH_I4(EPI_STAGES);
    else HDQT_LAUNCH_I4(EPI_GENERIC);
#undef HDQT_LAUNCH_I4
#undef HDQT_LAUNCH_SAT16
    return hipGetLastError();
}

} // namespace hdqt
