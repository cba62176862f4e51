// Weight-streaming GEMMs of the bf16 verification layer on the gfx950 matrix cores, with the
// layer's element-wise work fused in, and the packer that lays weights out in streaming order.
//
//   Y[m][n] = sum_k X[m][k] * W[n][k],   X = up to 64 activation rows (float32), W = [N, K] bf16.
//
// The work is memory bound: every weight byte is needed exactly once per step, the
// activations are small and cache resident.  Design points:
//   * W is cut into fragments that are exactly one operand of v_mfma_f32_32x32x16_bf16 - 32
//     weight rows x 16 k-values, lane l holding the 8 consecutive k-values (l / 32) * 8 .. + 7
//     of row l % 32 - and the fragments of one 32-row tile are stored one after the other
//     along K.  A wavefront reads a tile as one contiguous stream, 1 KiB per load
//     instruction, straight into operand registers, through a ring of four 8 KiB pieces whose
//     loads are issued unconditionally so that the wait before every MFMA is exact.
//   * activations stay float32 in memory; when a workgroup stages its K slice of X into LDS
//     (once, in fragment order) each value is split into hi + lo bf16 parts and both are
//     multiplied, so the product is accurate to ~2^-17 instead of 2^-9 at no cost in HBM
//     bytes.  This keeps a 32-layer pass inside the 2e-2 bar.  With X resident, the main loop
//     has no barrier: each of the four waves only streams weights, reads X fragments from LDS
//     and issues MFMAs.
//   * work unit = (group of 32-row tiles, K slice), one per workgroup, one workgroup per CU.
//     The hardware deals workgroups to the eight XCDs round robin (workgroup i runs on XCD
//     i % 8; the grid's x dimension is the XCD), so all slices of a tile run on one XCD and
//     their partial tiles (16-bit fixed point with a per-tile scale: they are HBM traffic, the
//     kernel is bound by its total traffic) meet in that XCD's L2: writer = plain stores, wait
//     for completion, then an atomic on the group's arrival counter; once all slices have
//     arrived (a short, bounded wait) every wave invalidates its L1 and takes an equal share of
//     the group's output: it adds the partials in slice order (bit-reproducible) and runs the
//     epilogue (gemm_reduce_phase; one load round trip, which is what that phase costs).  This is the
//     synchronisation the compiler itself emits between CUs that share an L2; the device-wide
//     release (an L2 write-back per workgroup) measured 2x slower end to end.  The placement
//     is checked, not assumed: every arrival adds to the 4-bit field of the XCD it really ran
//     on (read from the XCC_ID register); arrivals spread over several fields, or a wait that
//     ran out, raise a sticky flag in the workspace (SV_WS_STATUS) - results are then suspect.
//   * epilogues are tile local: weight rows are permuted at pack time so that a RoPE pair
//     (j, j + 64) and a SwiGLU pair (gate, up) sit 16 lanes apart in the same tile.
//   * RMSNorm is folded in: staging multiplies by the gain and sums x^2 over its K slice;
//     the slices of one group cover K exactly once, so the last wave has the full row sums
//     and scales the output rows by 1/sqrt(mean + eps).
#ifndef SV_GEMM_MFMA_H
#define SV_GEMM_MFMA_H

#include <type_traits>

#include "sv_internal.h"

namespace sv {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kFragRows = 32;    // weight rows per fragment and per tile (MFMA N)
constexpr int kFragK = 16;       // k-values per fragment (MFMA K)
constexpr int kBlkK = 128;       // granularity of K slices (8 fragments)
constexpr int kChunkBlks = 4;    // K blocks of X resident in LDS at a time (512 k-values = 2 pieces)
constexpr int kPieceFrags = 8;   // fragments per ring slot: 128 k-values, 8 KiB per wave
constexpr int kRing = 4;         // ring slots: 32 KiB of weights in flight per wave
constexpr int kTileFloats = kMTile * kFragRows;   // one partial tile, [64][32] values
constexpr int kTileVec4 = kTileFloats / 8;        // .. as stored: scaled int16 pairs, [4][64 lanes] uint4 = 4 KiB
constexpr int kXcds = 8;
constexpr int kCntStride = 32;     // 32-bit words per group's counters: a 128-byte line of its own
constexpr int kRedBatch = 3;       // reduction work items whose loads are in flight together

enum { PRO_PLAIN = 0, PRO_GAIN = 1 };
enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_OUT = 3 };
enum { PACK_PLAIN = 0, PACK_PAIR16_HEAD = 1, PACK_PAIR16_GU = 2 };

// Packer: src [rows, K] bf16 row-major -> fragment order, with a row permutation:
//   PACK_PLAIN        dst row = off + n
//   PACK_PAIR16_HEAD  heads of 128 rows; row d of a head goes to 32*((d%64)/16) + 16*(d/64) + d%16
//                     (a tile holds 16 rows j and their rotary partners j + 64)
//   PACK_PAIR16_GU    dst row = 32*(n/16) + off + n%16   (off = 0 gate, 16 up)
// One thread moves one 16-byte chunk (8 k-values); chunk (n, kc) lands at uint4 index
// ((n/32) * (K/16) + kc/2) * 64 + (n%32) + 32 * (kc%2).
__global__ void pack_rows_mfma(const uint4* __restrict__ src, uint4* __restrict__ dst, int rows,
                               int K, int mode, int off) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int chunks_per_row = K / 8;
  if (i >= (size_t)rows * chunks_per_row) return;
  const int n_src = (int)(i / chunks_per_row), kc = (int)(i % chunks_per_row);
  int n;
  if (mode == PACK_PAIR16_HEAD) {
    const int d = n_src % 128;
    n = off + (n_src - d) + 32 * ((d % 64) / 16) + 16 * (d / 64) + d % 16;
  } else if (mode == PACK_PAIR16_GU) {
    n = 32 * (n_src / 16) + off + n_src % 16;
  } else {
    n = off + n_src;
  }
  const size_t frag = (size_t)(n / kFragRows) * (K / kFragK) + (kc >> 1);
  dst[frag * 64 + (n % kFragRows) + 32 * (kc & 1)] = src[i];
}

// 8-bit weights (E4M3 codes, one float32 scale per row): the same tiles and row permutations,
// but one 16-byte load of a lane now carries two k-steps - the lane's 8 codes of k-step 2j, then
// its 8 codes of k-step 2j + 1 - so a tile is (K / 32) x 64 uint4 and a piece of 128 k-values is
// four loads.  One thread moves 8 codes: piece (n, kc8) of a source row lands in the uint2 at
// (((n/32) * (K/32) + kc8/4) * 64 + n%32 + 32 * (kc8%2)) * 2 + (kc8/2)%2.
__device__ inline int packed_row(int n_src, int mode, int off) {
  if (mode == PACK_PAIR16_HEAD) {
    const int d = n_src % 128;
    return off + (n_src - d) + 32 * ((d % 64) / 16) + 16 * (d / 64) + d % 16;
  }
  if (mode == PACK_PAIR16_GU) return 32 * (n_src / 16) + off + n_src % 16;
  return off + n_src;
}
__global__ void pack_rows_mfma_w8(const uint2* __restrict__ src, uint2* __restrict__ dst, int rows,
                                  int K, int mode, int off) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int per_row = K / 8;
  if (i >= (size_t)rows * per_row) return;
  const int n = packed_row((int)(i / per_row), mode, off), kc8 = (int)(i % per_row);
  const size_t load = (size_t)(n / kFragRows) * (K / 32) + (kc8 >> 2);
  dst[(load * 64 + (n % kFragRows) + 32 * (kc8 & 1)) * 2 + ((kc8 >> 1) & 1)] = src[i];
}
// int4 codes: `src` holds a row's K codes two per byte (even k in the low nibble), i.e. 8 codes
// per 32-bit word in k order.  A 16-byte load of the packed form carries a lane's 8 codes of four
// consecutive k-steps: word s of lane (n % 32) + 32 * (k-half) is k-step s of the load.
__global__ void pack_rows_mfma_w4(const uint32_t* __restrict__ src, uint32_t* __restrict__ dst, int rows,
                                  int K, int mode, int off) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int per_row = K / 8;
  if (i >= (size_t)rows * per_row) return;
  const int n = packed_row((int)(i / per_row), mode, off), kc8 = (int)(i % per_row);
  const size_t load = (size_t)(n / kFragRows) * (K / 64) + (kc8 >> 3);
  dst[(load * 64 + (n % kFragRows) + 32 * (kc8 & 1)) * 4 + ((kc8 >> 1) & 3)] = src[i];
}
__global__ void pack_row_scales(const float* __restrict__ src, float* __restrict__ dst, int rows,
                                int mode, int off) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < rows) dst[packed_row(i, mode, off)] = src[i];
}

struct GemmArgs {
  const float* X;        // [M, K] float32 activations
  const float* gain;     // [K] RMSNorm gain (PRO_GAIN) or unused
  const uint4* Wp;       // packed weights, N rows (bf16 fragments, or E4M3 codes: see pack_rows_mfma_w8)
  const float* wscale;   // 8-bit weights: [N] scale of each packed row; unused otherwise
  int M, N, K;
  int S;                 // K slices: 1 or even, at most 8
  int gpx;               // tile groups per XCD (units per XCD = gpx * S)
  // quotients the host works out once (the kernels do no integer division on their way to the
  // first load): tiles per group and remainder, 128-k pieces per slice and remainder,
  // ceil(2^16 / S) for unit -> (group, slice)
  int tq, trem, pq, prem;
  unsigned inv_S;
  int n_xcd;             // XCDs of the device (8 on MI355X; 1 for a single-XCD partition)
  // Scratch of the split-K reduction.  Every address belongs to one XCD - regions are indexed
  // [row tile][XCD][..] - so whatever one product leaves in an XCD's write-back L2 can never
  // meet another XCD's use of the same address by a later product of the same launch.
  int ucap;              // units per XCD the regions are laid out for (>= gpx * S)
  int tstride;           // partial tiles per XCD the regions are laid out for (>= gpx * (tq + 1) * S)
  uint4* part16;         // [m_tiles][n_xcd][tstride] partial tiles ([tile of the XCD][S]), kTileVec4 uint4 each (scaled int16)
  float* pscale;         // [m_tiles][n_xcd][tstride] inverse scale of each partial tile
  float* sumsq;          // [m_tiles][n_xcd][ucap][64] row sums of x^2 over each unit's K slice (RMSNorm, row scales of the partial tiles)
  unsigned* group_cnt;   // [m_tiles][n_xcd][ucap][kCntStride]: arrival (4 bits per XCD) and departure counters of a group in the first two words, zero between products
  int* status;           // sticky: != 0 once slices of one tile were seen on different XCDs
  float eps;
  const float* x_res;    // EPI_RESID: residual input [M, N]
  float* x_io;           // EPI_RESID: x_io [M, N] = x_res + Y (may alias x_res);  EPI_OUT: x_io [M, N] = Y
  float* act;            // EPI_SWIGLU: act [M, N/2] = silu(gate) * up
  float* q_out;          // EPI_QKV: [M, nh*128] float32, rotated
  bf16_t* kc;            // EPI_QKV: caches [B][nh][cap][128]
  bf16_t* vc;
  const int32_t* depth;
  const int32_t* prefix_len;
  int p_max, cap, T, nh;
  float theta;
};

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// Two floats -> packed bf16 (round to nearest even; one v_cvt_pk_bf16_f32 on gfx950).
__device__ inline uint32_t pack_bf16x2(float a, float b) {
  const f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ inline float bf16_lo_f32(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ inline float bf16_hi_f32(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// ---- partial tiles in transit: 16-bit fixed point with one power-of-two scale per tile -----
// A split-K partial tile is written once and read once; its bytes are HBM traffic on top of the
// weights (the L2 does not hold them until the reduction).  Stored as int16 pairs, scaled by a
// power of two that brings the tile's largest magnitude into [2^13, 2^14), they cost half the
// bytes of float32, cannot overflow whatever the activations, and carry an absolute error of at
// most 2^-14 of the tile maximum (what matters downstream is the error against the size of the
// row, not of the single element; fp16 with its 11-bit mantissa measured 6 times worse there).
//  - Rows of different size.  Where the activations are the raw residual stream (PRO_GAIN: the
//    normalisation is applied after the reduction), every row is first divided by a power of two
//    close to the norm of its activations over the slice - half the exponent of the row's sum of
//    squares, which the staging pass has anyway.  What is left of a row is bounded by the norm
//    of the weight rows alone, so rows of very different size that share a tile (episodes at
//    different scales, an outlier token) keep the same relative precision.  The other two
//    products take normalised quantities (attention output, SwiGLU output) and skip this.
//  - Infinities and NaNs.  A tile whose maximum is not finite takes a slower path: the scale
//    comes from its finite elements, every other element is stored as the code -32768 (never
//    produced otherwise) and the tile's inverse scale is stored negative; the reader turns the
//    code back into NaN.  So a NaN stays in the elements it reaches by the arithmetic of the
//    model, as with float32 partial sums (an infinity comes back as NaN).
// Register r (0..31: the two accumulators of a wave, see the layout at the tile store) goes to
// half r % 2 of dword r / 2 of the lane; dwords 4q..4q+3 form the lane's uint4 of store q.

// |v| as an integer that orders like the magnitude, NaN above infinity above all numbers
__device__ inline unsigned mag_bits(float v) { return __float_as_uint(v) & 0x7fffffffu; }
// maximum over the wave, in all-VALU data-parallel-primitive steps (a butterfly of lane
// permutes through LDS costs several hundred cycles of latency per tile): a running maximum
// inside each row of 16 lanes, then the row results handed on to the last lane, which is read.
// Lanes a step has no source for take the 0 given as the old value.
__device__ inline unsigned wave_max_u32(unsigned v) {
  auto step = [&](auto ctrl, auto rows) {
    const unsigned o = (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, decltype(ctrl)::value, decltype(rows)::value, 0xf, false);
    v = v > o ? v : o;
  };
  typedef std::integral_constant<int, 0xf> all_rows;
  step(std::integral_constant<int, 0x111>{}, all_rows{});                          // row_shr:1
  step(std::integral_constant<int, 0x112>{}, all_rows{});                          // row_shr:2
  step(std::integral_constant<int, 0x114>{}, all_rows{});                          // row_shr:4
  step(std::integral_constant<int, 0x118>{}, all_rows{});                          // row_shr:8: lane 15 of a row has the row's maximum
  step(std::integral_constant<int, 0x142>{}, std::integral_constant<int, 0xa>{});  // row_bcast:15 into rows 1 and 3
  step(std::integral_constant<int, 0x143>{}, std::integral_constant<int, 0xc>{});  // row_bcast:31 into rows 2 and 3
  return (unsigned)__builtin_amdgcn_readlane((int)v, 63);
}
constexpr unsigned kInfBits = 0x7f800000u;
__device__ inline unsigned finite_mag_bits(float v) {
  const unsigned m = mag_bits(v);
  return m < kInfBits ? m : 0u;
}
// scale = 2^(13 - e) for a finite tile maximum in [2^e, 2^(e+1)), inv = 1 / scale (exponents
// clamped so that both stay normal numbers)
__device__ inline void partial_tile_scale(unsigned max_bits, float& scale, float& inv) {
  const unsigned eb = max_bits >> 23;
  unsigned se = 267u - eb;                 // >= 13 for every finite maximum
  se = se > 240u ? 240u : se;
  scale = __uint_as_float(se << 23);
  inv = __uint_as_float((254u - se) << 23);
}
// two values -> int16 pair, round to nearest even: adding 1.5 * 2^23 leaves the rounded integer
// in the low mantissa bits (|a * scale| < 2^14 here)
__device__ inline unsigned pack_q16x2(float a, float b, float scale) {
  const unsigned ua = __float_as_uint(fmaf(a, scale, 12582912.0f));
  const unsigned ub = __float_as_uint(fmaf(b, scale, 12582912.0f));
  return __builtin_amdgcn_perm(ub, ua, 0x05040100u);     // low halves of ua (bits 15:0) and ub (bits 31:16)
}
// h = floor(exponent(ssq) / 2), -64 .. 64: the row is stored times 2^-h and read back times 2^h
__device__ inline int row_half_exp(float ssq) { return ((int)((__float_as_uint(ssq) >> 23) & 255u) - 127) >> 1; }
__device__ inline float row_scale(float ssq) { return __uint_as_float((unsigned)(127 - row_half_exp(ssq)) << 23); }
// the reader keeps h + 64 of four slices in the bytes of one word
__device__ inline unsigned row_exp_bytes(float s0, float s1, float s2, float s3) {
  return (unsigned)(row_half_exp(s0) + 64) | (unsigned)(row_half_exp(s1) + 64) << 8 |
         (unsigned)(row_half_exp(s2) + 64) << 16 | (unsigned)(row_half_exp(s3) + 64) << 24;
}
__device__ inline float row_scale_inv(unsigned bytes, int i) {
  return __uint_as_float((63u + ((bytes >> (8 * i)) & 255u)) << 23);
}
// the same for a tile with non-finite elements: those become the code 0x8000
__device__ inline unsigned pack_q16x2_coded(float a, float b, float scale) {
  const unsigned ua = mag_bits(a) < kInfBits ? __float_as_uint(fmaf(a, scale, 12582912.0f)) & 0xffffu : 0x8000u;
  const unsigned ub = mag_bits(b) < kInfBits ? __float_as_uint(fmaf(b, scale, 12582912.0f)) & 0xffffu : 0x8000u;
  return ua | (ub << 16);
}
__device__ inline float q16_lo(unsigned d) { return (float)((int)(d << 16) >> 16); }
__device__ inline float q16_hi(unsigned d) { return (float)((int)d >> 16); }

// Value of the lane 16 places away (lane ^ 16) without a trip through LDS: the gfx950 row swap
// returns {rows 0,0,2,2} and {rows 1,1,3,3} of its operand (rows of 16 lanes).
__device__ inline float lane_xor16(float v, int lane) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float((lane & 16) ? r[0] : r[1]);
}
// 16 per-lane partial sums (one per row) -> row totals over the 64 lanes, by halving: after the
// exchanges over the lane distances 32, 16, 8, 4 every lane holds one row's sum over a group of
// lanes, two more steps finish it; lane l ends with the total of row index
// 8 * bit5(l) + 4 * bit4(l) + 2 * bit3(l) + bit2(l).  All exchanges stay in the vector ALU:
// half and row swaps (gfx950), row rotation, half-row mirror + quad reversal, quad permutes.
template <int CTRL>
__device__ inline float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ inline float row_sums_butterfly(const float (&ssq)[16], int lane) {
  float v8[8], v4[4], v2[2], v1;
  const bool h8 = lane & 8, h4 = lane & 4;
#pragma unroll
  for (int i = 0; i < 8; ++i) {        // lanes 0..31 keep rows i, lanes 32..63 rows i + 8
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(ssq[i]), __float_as_uint(ssq[i + 8]), false, false);
    v8[i] = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {        // rows of 16 lanes: even ones keep value i, odd ones i + 4
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v8[i]), __float_as_uint(v8[i + 4]), false, false);
    v4[i] = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const float mine = h8 ? v4[i + 2] : v4[i], other = h8 ? v4[i] : v4[i + 2];
    v2[i] = mine + dpp_f32<0x128>(other);                               // row_ror:8 = lane ^ 8
  }
  {
    const float mine = h4 ? v2[1] : v2[0], other = h4 ? v2[0] : v2[1];
    v1 = mine + dpp_f32<0x1B>(dpp_f32<0x141>(other));                   // half-row mirror, quads reversed = lane ^ 4
  }
  v1 += dpp_f32<0x4E>(v1);                                              // lane ^ 2
  v1 += dpp_f32<0xB1>(v1);                                              // lane ^ 1
  return v1;
}

// x * sigmoid(x) with the hardware exponential and reciprocal (1 ulp each)
__device__ inline float silu_fast(float x) {
  return x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}

// One 16-byte load of E4M3 codes -> the two bf16 operand fragments it carries (exact: every
// E4M3 value is a bf16 value).  Hardware conversion to float32 pairs, then the pack-convert.
typedef float f32x2v_t __attribute__((ext_vector_type(2)));
__device__ inline void w8_to_frags(const u32x4_t raw, bf16x8_t& f0, bf16x8_t& f1) {
  u32x4_t a, b;
#pragma unroll
  for (int d = 0; d < 2; ++d) {
    const f32x2v_t lo0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)raw[d], false);
    const f32x2v_t hi0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)raw[d], true);
    a[2 * d] = pack_bf16x2(lo0[0], lo0[1]);
    a[2 * d + 1] = pack_bf16x2(hi0[0], hi0[1]);
    const f32x2v_t lo1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)raw[2 + d], false);
    const f32x2v_t hi1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)raw[2 + d], true);
    b[2 * d] = pack_bf16x2(lo1[0], lo1[1]);
    b[2 * d + 1] = pack_bf16x2(hi1[0], hi1[1]);
  }
  f0 = __builtin_bit_cast(bf16x8_t, a);
  f1 = __builtin_bit_cast(bf16x8_t, b);
}

// One 16-byte load of int4 codes (a lane's 8 codes of four consecutive k-steps, one 32-bit word
// per k-step, code i of a word in bits 4i .. 4i+3) -> four bf16 operand fragments.  A code c
// stands for the integer c - 8 (-8 .. 7): the code with its top bit flipped is that integer in
// 4-bit two's complement, which a signed bit-field extract widens; integer -> float32 ->
// bf16 is exact for these values.
__device__ inline void w4_to_frags(const u32x4_t raw, bf16x8_t (&f)[4]) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const int w = (int)(raw[d] ^ 0x88888888u);
    u32x4_t o;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      // (the builtin's result type is unsigned: the cast to int comes first)
      const float lo = (float)(int)__builtin_amdgcn_sbfe(w, 8 * j, 4);
      const float hi = (float)(int)__builtin_amdgcn_sbfe(w, 8 * j + 4, 4);
      o[j] = pack_bf16x2(lo, hi);
    }
    f[d] = __builtin_bit_cast(bf16x8_t, o);
  }
}

// 16-byte load of four floats from global memory
__device__ inline float4 ldg_f4(const __attribute__((address_space(1))) float* p) {
  const f32x4_t v = *(const __attribute__((address_space(1))) f32x4_t*)p;
  return make_float4(v[0], v[1], v[2], v[3]);
}

// XCD (accelerator complex die) this wave runs on: bits 3:0 of the XCC_ID hardware register.
__device__ inline int xcd_actual(int n_xcd) {
  return (int)(__builtin_amdgcn_s_getreg((4 - 1) << 11 | 0 << 6 | 20) & 0xf) % n_xcd;
}

// Position of element (row l % 32, k-half l / 32) inside the 64-slot fragment of k-step s.
// The XOR spreads the slots that one staging store instruction touches over all LDS banks;
// readers apply the same permutation, which keeps their 16-lane groups conflict free.
__device__ inline int frag_slot(int l, int s) { return ((l & 31) ^ (((s & 7) << 1) | (l >> 5))) | (l & 32); }

// Second half of gemm_stream_bf16: group barrier, then every wave of every slice reduces its
// share of the group's tiles and applies the epilogue.  `a` is the kernel-argument segment read
// through a pointer the compiler cannot trace back to the kernel's own copy, and every index is
// derived again from it: nothing of this phase stays live in scalar registers across the main
// loop, where spilled scalars cost stalls between the matrix instructions.
typedef const __attribute__((address_space(4))) GemmArgs* gemm_args_ptr_t;
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
template <int PRO, int EPI, int WF>
__device__ __forceinline__ void gemm_reduce_phase(gemm_args_ptr_t ap, int* s_pos, int* s_crow,
                                                  int tid, int lane, int wave, int xcd, int u, int mt) {
  GemmArgs a;                                // one batch of scalar loads; registers from here on
  {
    static_assert(sizeof(GemmArgs) % 4 == 0, "copied word by word");
    const __attribute__((address_space(4))) unsigned* src = (const __attribute__((address_space(4))) unsigned*)ap;
    unsigned* dst = reinterpret_cast<unsigned*>(&a);
#pragma unroll
    for (unsigned i = 0; i < sizeof(GemmArgs) / 4; ++i) dst[i] = src[i];
  }
  // pointers read from memory are generic to the compiler: name their address space, or every
  // access becomes a flat one
#define SV_GLOBAL(T, p) ((__attribute__((address_space(1))) T*)(p))
  const auto part16 = SV_GLOBAL(const uint4, a.part16);
  const auto pscale = SV_GLOBAL(const float, a.pscale);
  const auto sumsq = SV_GLOBAL(const float, a.sumsq);
  const auto wscale = SV_GLOBAL(const float, a.wscale);
  const auto status = SV_GLOBAL(int, a.status);
  const auto x_io = SV_GLOBAL(float, a.x_io);
  const auto x_res = SV_GLOBAL(const float, a.x_res);
  const auto act = SV_GLOBAL(float, a.act);
  const auto q_out = SV_GLOBAL(float, a.q_out);
  const auto kc = SV_GLOBAL(unsigned short, a.kc);
  const auto vc = SV_GLOBAL(unsigned short, a.vc);
  const auto depth = SV_GLOBAL(const int32_t, a.depth);
  const auto prefix_len = SV_GLOBAL(const int32_t, a.prefix_len);
  const int m0 = mt * kMTile;
  const int K = a.K, S = a.S;
  const int ug = (int)(((unsigned)u * a.inv_S) >> 16);   // u / S
  const int g = xcd * a.gpx + ug, sp = u - ug * S;
  const int tq = a.tq, trem = a.trem;
  const int t_begin = g * tq + min(g, trem);
  const int t_count = tq + (g < trem ? 1 : 0);
  const int rbase = 4 * (lane >> 5);

  // ---- group barrier, then every wave of every slice reduces its share ----
  // Arrival = add 1 to the 4-bit field of the XCD this workgroup really runs on; all S
  // arrivals in one field means the slices shared an L2, as planned.  The workgroups of a
  // group are dispatched within 64 consecutive workgroup ids, so they are resident together
  // and the wait below is short; it is bounded all the same (status bit 2 on give-up).
  __builtin_amdgcn_s_waitcnt(0);           // this wave's partial tiles are in L2
  __syncthreads();
  // (one line per group: arrivals and polls of different groups do not queue behind each other)
  const size_t xbase = (size_t)mt * a.n_xcd + xcd;       // this XCD's share of the scratch regions
  const int t0x = xcd * a.gpx * tq + min(xcd * a.gpx, trem);   // first tile of this XCD
  const auto gcnt = SV_GLOBAL(unsigned, a.group_cnt) + (xbase * a.ucap + ug) * kCntStride;
#undef SV_GLOBAL
  if (EPI == EPI_QKV && tid >= 64 && tid < 64 + kMTile) {
    // rotary position and cache row of each row of the m tile, by the second wave while the
    // first one waits for the group (ordered before their use by the barrier below)
    const int r = tid - 64;
    const int m = min(m0 + r, a.M - 1);
    const int b = m / a.T, t = m - b * a.T;
    int P = prefix_len[b];
    P = P < 0 ? 0 : (P > a.p_max ? a.p_max : P);
    s_pos[r] = P + depth[m];
    s_crow[r] = b * a.nh * a.cap + P + t;    // + head * cap, times 128, in the epilogue
  }
  if (tid == 0) {
    const unsigned field = 4u * (unsigned)xcd_actual(a.n_xcd);
    // the value the add returns is the first look at the counter: the last slice to arrive -
    // the one the group's finish time hangs on - goes on without a second round trip
    unsigned v = __hip_atomic_fetch_add(gcnt, 1u << field, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + (1u << field);
    unsigned n = 0;
    for (int spin = 0; spin < (1 << 16); ++spin) {
      n = 0;
#pragma unroll
      for (int x = 0; x < kXcds; ++x) n += (v >> (4 * x)) & 15u;
      if (n >= (unsigned)S) break;
      __builtin_amdgcn_s_sleep(8);           // ~0.25 us: polls are device-scope round trips, keep them few
      v = __hip_atomic_load(gcnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // not from L1
    }
    int bad = 0;
    if (n < (unsigned)S) bad |= 2;                                  // gave up waiting
    else if (v != ((unsigned)S << field)) bad |= 1;                 // slices on several XCDs
    if (bad) __hip_atomic_fetch_or(status, bad, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  asm volatile("buffer_inv sc0" ::: "memory");                      // drop stale L1 lines (the L2 is shared)
  // Row sums of all slices -> 1 / rms: every wave keeps the value of row `lane` and fetches
  // the rows it needs with a lane read.  The loads are only issued here; they are consumed
  // behind the first batch of partial-tile loads, so the two round trips overlap.
  float ss8[8];
  if (PRO == PRO_GAIN) {
#pragma unroll
    for (int s2 = 0; s2 < 8; ++s2)
      ss8[s2] = sumsq[(xbase * a.ucap + ug * S + min(s2, S - 1)) * kMTile + lane];
  }
  float rstd_lane = 1.0f;
  unsigned rexp_lo = 0, rexp_hi = 0;       // row `lane`: h + 64 of slices 0..3 / 4..7
  bool have_rstd = false;

  // Work item = one quad of one tile: the 8 rows x 32 columns that register quad `qd` of the
  // partial-tile layout holds (rows 8*(qd%4) + 4*(lane/32) + 0..3, +32 for qd >= 4).  The 4 * S
  // waves of the group's slices share the items so that a wave keeps its quad (S is 1 or
  // even): wave number wk = slice + S * wave takes quad wk % 8 of the tiles wk / 8,
  // wk / 8 + S / 2, ..; with S = 1 there are four waves, each takes two quads in turn.  What
  // depends on the rows only - 1 / rms and the row scales of the eight slices - is then
  // fetched once per quad: rinv[s][j] = 2^h of slice s and row row0 + j.
  const int ln = lane & 31;
  const int wk = sp + S * wave;
  const int t_step = S > 1 ? S >> 1 : 1;
  for (int qd = wk & 7; qd < 8; qd += 4 * S) {
    const int row0 = 8 * (qd & 3) + rbase + 32 * (qd >> 2);
    float rinv[8][4], rstd4[4];
    bool have_rows = false;
    for (int tl0 = wk >> 3; tl0 < t_count; tl0 += t_step * kRedBatch) {
      u32x2_t part[kRedBatch][8];
      float pinv[kRedBatch][8];
      float xres[kRedBatch][4];
      float wsc[kRedBatch];                                           // 8-bit weights: scale of this lane's weight row
#pragma unroll
      for (int bi = 0; bi < kRedBatch; ++bi) {                        // all loads of the batch first
        const int tl = tl0 + t_step * bi;
        if (tl >= t_count) break;
        const int tile = t_begin + tl;
        // registers 4qd .. 4qd+3 of the tile = dwords 2qd, 2qd+1 = half of the uint4 of store qd/2
        const size_t pidx = xbase * a.tstride + (size_t)(tile - t0x) * S;
        const auto pb = (const __attribute__((address_space(1))) u32x2_t*)(part16 + pidx * kTileVec4 + (qd >> 1) * 64 + lane) + (qd & 1);
#pragma unroll
        for (int s2 = 0; s2 < 8; ++s2) part[bi][s2] = pb[(size_t)min(s2, S - 1) * (kTileVec4 * 2)];
        if (S == 8) {
          // the eight scales of the tile in two loads instead of eight (the load queue holds 63
          // requests; batches of three items measured fastest, larger ones slower)
          typedef float f32x4a_t __attribute__((ext_vector_type(4)));
          const auto pv = (const __attribute__((address_space(1))) f32x4a_t*)(pscale + pidx);
          const f32x4a_t p0 = pv[0], p1 = pv[1];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            pinv[bi][e] = p0[e];
            pinv[bi][4 + e] = p1[e];
          }
        } else {
#pragma unroll
          for (int s2 = 0; s2 < 8; ++s2) pinv[bi][s2] = s2 < S ? pscale[pidx + min(s2, S - 1)] : 0.f;
        }
        if (EPI == EPI_RESID) {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            xres[bi][j] = x_res[(size_t)min(m0 + row0 + j, a.M - 1) * a.N + tile * 32 + ln];
        }
        if (WF) wsc[bi] = wscale[tile * 32 + ln];
      }
      // The phase is bound by the round trips of these loads, not by arithmetic: keep the whole
      // batch in flight together (left alone, the compiler sinks loads towards their uses).
      asm volatile("" ::: "memory");
      if (PRO == PRO_GAIN && !have_rstd) {
        // the row sums were requested before the batch; their first use must not move ahead of
        // the batch's loads, or the two round trips happen one after the other
#pragma unroll
        for (int s2 = 0; s2 < 8; ++s2) asm volatile("" : "+v"(ss8[s2]));
        float t = 0.f;
#pragma unroll
        for (int s2 = 0; s2 < 8; ++s2) t += s2 < S ? ss8[s2] : 0.f;
        rstd_lane = 1.0f / sqrtf(t / (float)K + a.eps);
        rexp_lo = row_exp_bytes(ss8[0], ss8[1], ss8[2], ss8[3]);
        rexp_hi = row_exp_bytes(ss8[4], ss8[5], ss8[6], ss8[7]);
        have_rstd = true;
      }
      if (PRO == PRO_GAIN && !have_rows) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const unsigned elo = (unsigned)__shfl((int)rexp_lo, row0 + j, kWave);
          const unsigned ehi = (unsigned)__shfl((int)rexp_hi, row0 + j, kWave);
#pragma unroll
          for (int s2 = 0; s2 < 8; ++s2) rinv[s2][j] = row_scale_inv(s2 < 4 ? elo : ehi, s2 & 3);
          rstd4[j] = __shfl(rstd_lane, row0 + j, kWave);
        }
        have_rows = true;
      }
#pragma unroll
      for (int bi = 0; bi < kRedBatch; ++bi) {
        const int tl = tl0 + t_step * bi;
        if (tl >= t_count) break;
        const int tile = t_begin + tl;
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        int any_flag = 0;                                             // sign bits of the inverse scales
#pragma unroll
        for (int s2 = 0; s2 < 8; ++s2) {                              // fixed slice order
          const unsigned d0 = part[bi][s2].x, d1 = part[bi][s2].y;
          const float w = fabsf(pinv[bi][s2]);                        // 0 beyond the last slice
          any_flag |= __float_as_int(pinv[bi][s2]);
          const float q[4] = {q16_lo(d0), q16_hi(d0), q16_lo(d1), q16_hi(d1)};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            // tile scale first, row scale second: neither product can overflow on its own
            if (PRO == PRO_GAIN)
              v[j] = fmaf(w * q[j], rinv[s2][j], v[j]);
            else
              v[j] += w * q[j];
          }
        }
        if (any_flag < 0) {                  // rare: a tile with non-finite elements among the eight
          const float nan = __uint_as_float(0x7fc00000u);
#pragma unroll
          for (int s2 = 0; s2 < 8; ++s2) {
            if (__float_as_int(pinv[bi][s2]) >= 0) continue;
            const unsigned d0 = part[bi][s2].x, d1 = part[bi][s2].y;
            if ((d0 & 0xffffu) == 0x8000u) v[0] = nan;
            if ((d0 >> 16) == 0x8000u) v[1] = nan;
            if ((d1 & 0xffffu) == 0x8000u) v[2] = nan;
            if ((d1 >> 16) == 0x8000u) v[3] = nan;
          }
        }
        if (PRO == PRO_GAIN) {
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] *= rstd4[j];
        }
        if (WF) {
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] *= wsc[bi];
        }
        if (EPI == EPI_RESID) {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (m0 + row0 + j < a.M)
              x_io[(size_t)(m0 + row0 + j) * a.N + tile * 32 + ln] = xres[bi][j] + v[j];
        }
        if (EPI == EPI_OUT) {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (m0 + row0 + j < a.M)
              x_io[(size_t)(m0 + row0 + j) * a.N + tile * 32 + ln] = v[j];
        }
        if (EPI == EPI_SWIGLU) {             // lanes 0..15 gate, 16..31 up of the same column
          const int F = a.N / 2;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float up = lane_xor16(v[j], lane);
            if (ln < 16 && m0 + row0 + j < a.M)
              act[(size_t)(m0 + row0 + j) * F + tile * 16 + ln] = silu_fast(v[j]) * up;
          }
        }
        if (EPI == EPI_QKV) {
          const int tiles_per_mat = a.nh * 4;  // 128 rows per head = 4 tiles
          const int which = tile / tiles_per_mat;                  // 0 q, 1 k, 2 v
          const int head = (tile % tiles_per_mat) / 4, uq = tile % 4;
          const int jr = 16 * uq + (ln & 15);                      // rotary pair index, 0..63
          const int dcol = jr + 64 * (ln >> 4);                    // column inside the head
          // angle in turns = position * theta^(-2j/128) / (2 pi)
          const float turn_freq = exp2f(-(float)jr * (1.0f / 64.0f) * log2f(a.theta)) * 0.15915494309189535f;
          const float sgn = (ln & 16) ? 1.0f : -1.0f;
          const int D = a.nh * 128;
          const auto cache = which == 1 ? kc : vc;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int ml = row0 + j;
            float val = v[j];
            const float partner = lane_xor16(val, lane);
            if (which != 2) {
              float turns = (float)s_pos[ml] * turn_freq;
              turns -= floorf(turns);        // reduced to [0, 1) before the hardware sin / cos
              val = val * __builtin_amdgcn_cosf(turns) + sgn * partner * __builtin_amdgcn_sinf(turns);
            }
            if (m0 + ml < a.M) {
              if (which == 0)
                q_out[(size_t)(m0 + ml) * D + head * 128 + dcol] = val;
              else
                cache[((size_t)s_crow[ml] + (size_t)head * a.cap) * 128 + dcol] = f32_to_bf16(val).bits;
            }
          }
        }
      }
    }
  }
  // the last workgroup to get here clears the group's two words for the next launch
  if (tid == 0 &&
      __hip_atomic_fetch_add(gcnt + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (unsigned)(S - 1)) {
    gcnt[0] = 0;
    gcnt[1] = 0;
  }
}

// LDS of one workgroup of the streaming GEMM (156 416 bytes; one workgroup per CU).
constexpr int kGemmXsVec = 32 * 2 * 2 * 64;      // X chunk: [32 k-steps][2 m-halves][hi, lo][64 slots] x 16 bytes = 128 KiB
constexpr int kGemmHeadVec = 3 * 8 * 64;         // single-chunk form: accumulators of tiles shared by two waves
constexpr size_t kGemmLdsBytes = (size_t)(kGemmXsVec + kGemmHeadVec) * 16 + 3 * kMTile * 4;
struct GemmLds {
  uint4* xs;            // X chunk
  uint4* s_head;        // accumulators handed between waves (single-chunk form)
  int* s_pos;           // EPI_QKV: rotary position of each row of the m tile
  int* s_crow;          // EPI_QKV: cache row (b * nh * cap + P + t) of each row
  float* s_rowscale;    // 2^-h of each row for this slice's partial tiles
};
__device__ __forceinline__ GemmLds carve_gemm_lds(uint4* base) {
  GemmLds l;
  l.xs = base;
  l.s_head = base + kGemmXsVec;
  l.s_pos = reinterpret_cast<int*>(base + kGemmXsVec + kGemmHeadVec);
  l.s_crow = l.s_pos + kMTile;
  l.s_rowscale = reinterpret_cast<float*>(l.s_crow + kMTile);
  return l;
}
constexpr size_t kGemmLdsAlloc = kGemmLdsBytes;

// One workgroup of the streaming GEMM: unit u of XCD xcd, row tile mt.  Launch shape of the
// stand-alone kernel: grid = (n_xcd, gpx * S, m_tiles), block = 256, 1 workgroup per CU (LDS).
// K must be a multiple of 256: slices are made of pieces of 16 fragments (2 K blocks), a chunk
// of X in LDS holds up to two pieces.
// MULTI: a K slice may span several LDS chunks (the host knows from its plan); the single-chunk
// form carries no re-staging code and nothing of it in registers through the main loop.
// WF (weight format): 0 = bf16 fragments as they are; 1 = E4M3 codes (four loads per piece), 2 =
// int4 codes (two loads per piece), both converted to bf16 fragments in registers, the row scales
// applied in the reduction.
// KEEP: the weights are read again, shortly afterwards, by the workgroups that multiply the
// same tiles with the other row tiles (more than 64 rows): the loads are ordinary ones, which the
// XCD's L2 keeps, instead of the non-temporal ones of the single-row-tile case.
template <int PRO, int EPI, bool MULTI, int WF, bool KEEP>
__device__ __forceinline__ void gemm_stream_body(gemm_args_ptr_t ap, const int xcd, const int u,
                                                 const int mt, const GemmLds lds) {
  const __attribute__((address_space(4))) GemmArgs& a = *ap;
  constexpr int kLoads = kPieceFrags >> WF;   // 16-byte loads per piece and lane: 8 (bf16), 4 (E4M3), 2 (int4)
  uint4* const xs = lds.xs;
  int* const s_pos = lds.s_pos;
  int* const s_crow = lds.s_crow;
  float* const s_rowscale = lds.s_rowscale;
  uint4* const s_head = lds.s_head;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: bookkeeping stays in scalar registers
  const int m0 = mt * kMTile;
  const int K = a.K, S = a.S;
  // (workgroups are dealt to the XCDs in turn: xcd = linear workgroup index modulo n_xcd; u =
  // unit inside that XCD's share)

  {
    const int ug = (int)(((unsigned)u * a.inv_S) >> 16);   // u / S
    const int g = xcd * a.gpx + ug;          // tile group (contiguous tiles), K slice
    const int sp = u - ug * S;
    const int tq = a.tq, trem = a.trem;
    const int t_begin = g * tq + min(g, trem);
    const int t_count = tq + (g < trem ? 1 : 0);
    const int pq = a.pq, prem = a.prem;
    const int p_begin = sp * pq + min(sp, prem);         // first piece (128 k-values) of the slice
    const int np = pq + (sp < prem ? 1 : 0);             // pieces in the slice
    const int n_chunks = (np + 3) >> 2;                  // LDS chunks of 4 pieces
    // Which pieces a wave multiplies.  MULTI: whole tiles wave, wave+4, .. (at most one, see the
    // host's plan).  Single-chunk form: the group's t_count * np pieces, tile after tile, are cut
    // into four equal consecutive runs, one per wave - with 21 or 22 tiles in a group whole
    // tiles would give waves of 5 and of 6 tiles, and the launch waits for the longest.  A tile
    // that straddles a cut is summed from the two waves' accumulators at the end (fewer than
    // four tiles: whole tiles, so that no tile is shared by more than two waves).
    const int my_tiles = t_count > wave ? (t_count - wave + 3) / 4 : 0;
    int b0 = 0, b1 = 0;                                  // this wave's run of pieces [b0, b1)
    if (!MULTI) {
      const int P = t_count * np;
      if (t_count >= 4) {
        b0 = (wave * P) >> 2;
        b1 = ((wave + 1) * P) >> 2;
      } else {
        b0 = min(wave, t_count) * np;
        b1 = min(wave + 1, t_count) * np;
      }
    }
    // first tile and first piece of the run (np <= 4 here; no division)
    const int ft = MULTI ? wave : (np == 4 ? b0 >> 2 : np == 3 ? (b0 * 21846) >> 16 : np == 2 ? b0 >> 1 : b0);
    const int cj0 = MULTI ? 0 : b0 - ft * np;
    const int n_run = MULTI ? my_tiles * np : b1 - b0;
    const size_t xbase = (size_t)mt * a.n_xcd + xcd;     // this XCD's share of the scratch regions
    const size_t unit_id = xbase * a.ucap + u;
    const int t0x = xcd * a.gpx * tq + min(xcd * a.gpx, trem);   // first tile of this XCD
    const size_t tile_stride = (size_t)(K / (kFragK << WF)) * 64;   // uint4 per tile
    typedef const __attribute__((address_space(1))) u32x4_t* wptr_t;
    const wptr_t wbase = (wptr_t)a.Wp + (size_t)(t_begin + ft) * tile_stride +
                         (size_t)(p_begin + cj0) * (kLoads * 64);

    // Ring of weight pieces.  Every step of the main loop issues exactly kPieceFrags loads into
    // the slot it has just consumed - a cache-resident dummy address once nothing is left - so
    // the number of younger loads behind any slot is a compile-time constant and the wait
    // before each MFMA is exact (a conditional load would force a full drain instead).
    u32x4_t ring[kRing][kLoads];
    // next piece to load: a running pointer (piece after piece, then a jump to this wave's next
    // tile), so that issuing costs a handful of scalar instructions
    wptr_t ip = n_run > 0 ? wbase : (wptr_t)a.Wp;
    const size_t tile_jump = (MULTI ? 4 : 1) * tile_stride - (size_t)np * (kLoads * 64);
    int ij = cj0, to_issue = n_run;
    auto issue = [&](u32x4_t* buf) {
#pragma unroll
      for (int f = 0; f < kLoads; ++f)        // streamed once: do not keep it in the caches
        buf[f] = KEEP ? ip[(unsigned)lane + f * 64u] : __builtin_nontemporal_load(ip + ((unsigned)lane + f * 64u));
      if (to_issue > 0) {
        ip += kLoads * 64;
        if (++ij == np) {
          ij = 0;
          ip += tile_jump;
        }
        if (--to_issue == 0) ip = (wptr_t)a.Wp;
      }
    };

    float ssq[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) ssq[r] = 0.f;

    // Staging chunk c of this slice, in two halves: wave w handles rows w, w+4, .. ; lane = 8-wide
    // k chunk.  x_load issues all 32 loads of the lane's 16 rows (and the gain), x_convert splits
    // the values into hi + lo bf16 and writes them to LDS in fragment order.
    auto x_load = [&](int c, float4 (&xa)[16], float4 (&xb)[16], float4& g0, float4& g1) {
      const int nkc = min(4, np - 4 * c) * 16;     // 8-wide chunks per row in this K chunk
      const int k = (p_begin + 4 * c) * kBlkK + (lane < nkc ? lane : 0) * 8;
      g0 = g1 = make_float4(1.f, 1.f, 1.f, 1.f);
      if (PRO == PRO_GAIN) {
        const auto gp = (const __attribute__((address_space(1))) float*)a.gain + k;
        g0 = ldg_f4(gp);
        g1 = ldg_f4(gp + 4);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wave + 4 * r;
        const auto p = (const __attribute__((address_space(1))) float*)a.X + (size_t)min(m, a.M - 1) * K + k;
        xa[r] = ldg_f4(p);
        xb[r] = ldg_f4(p + 4);
      }
    };
    // `before_row(r)` runs ahead of row r's conversion (the first chunk slips the ring's loads in)
    auto x_convert = [&](int c, const float4 (&xa)[16], const float4 (&xb)[16], const float4& g0,
                         const float4& g1, auto before_row) {
      const int nkc = min(4, np - 4 * c) * 16;
      const bool on = lane < nkc;
      const int s = lane >> 1;                     // k-step inside the chunk
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        before_row(r);
        // (rows beyond M repeat row M - 1: they cost nothing extra and are never written out)
        const int ml = wave + 4 * r;
        float v[8] = {xa[r].x, xa[r].y, xa[r].z, xa[r].w, xb[r].x, xb[r].y, xb[r].z, xb[r].w};
        if (PRO == PRO_GAIN) {
          float t = 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e) t += v[e] * v[e];
          ssq[r] += on ? t : 0.f;
          v[0] *= g0.x; v[1] *= g0.y; v[2] *= g0.z; v[3] *= g0.w;
          v[4] *= g1.x; v[5] *= g1.y; v[6] *= g1.z; v[7] *= g1.w;
        }
        uint4 hi4, lo4;
        hi4.x = pack_bf16x2(v[0], v[1]); hi4.y = pack_bf16x2(v[2], v[3]);
        hi4.z = pack_bf16x2(v[4], v[5]); hi4.w = pack_bf16x2(v[6], v[7]);
        lo4.x = pack_bf16x2(v[0] - bf16_lo_f32(hi4.x), v[1] - bf16_hi_f32(hi4.x));
        lo4.y = pack_bf16x2(v[2] - bf16_lo_f32(hi4.y), v[3] - bf16_hi_f32(hi4.y));
        lo4.z = pack_bf16x2(v[4] - bf16_lo_f32(hi4.z), v[5] - bf16_hi_f32(hi4.z));
        lo4.w = pack_bf16x2(v[6] - bf16_lo_f32(hi4.w), v[7] - bf16_hi_f32(hi4.w));
        const int slot = frag_slot((ml & 31) | ((lane & 1) << 5), s);
        const int base = ((s * 2 + (ml >> 5)) * 2) * 64 + slot;
        if (on) {
          xs[base] = hi4;
          xs[base + 64] = lo4;
        }
      }
    };
    // Row sums of x^2 over this K slice, published once the whole slice has been staged and
    // completed (waitcnt) before the barrier that precedes any tile arrival of this workgroup.
    auto publish_ssq = [&]() {
      const float v1 = row_sums_butterfly(ssq, lane);
      // row index held by this lane: bit 3 from lane bit 5, bit 2 from bit 4, bit 1 from bit 3,
      // bit 0 from bit 2
      const int r = ((lane >> 5) & 1) * 8 + ((lane >> 4) & 1) * 4 + ((lane >> 3) & 1) * 2 + ((lane >> 2) & 1);
      // (inline assembly for the same reason as the partial-tile stores below)
      if ((lane & 3) == 0) {
        asm volatile("global_store_dword %0, %1, off" ::"v"(a.sumsq + unit_id * kMTile + wave + 4 * r), "v"(v1) : "memory");
        s_rowscale[wave + 4 * r] = row_scale(v1);   // (an infinite or NaN sum: any scale will do, the values are not finite either)
      }
    };
    {
      // Chunk 0.  Only the ring's first piece is requested right behind the X loads, the others
      // while the rows are converted: a thousand waves asking for their whole ring at once put
      // 32 MB of weight requests in front of each other's X rows, and the X round trip - which
      // nothing can overlap - grows with the queue.  Spread over the conversion the same loads
      // still arrive before the main loop wants them (measured: 3.5 us per layer).
      float4 xa[16], xb[16], g0, g1;
      x_load(0, xa, xb, g0, g1);
      issue(ring[0]);
      x_convert(0, xa, xb, g0, g1, [&](int r) {
        static_assert(kRing == 4, "one slot every fourth row");
        if (r == 4) issue(ring[1]);
        if (r == 8) issue(ring[2]);
        if (r == 12) issue(ring[3]);
      });
    }
    if (PRO == PRO_GAIN && n_chunks == 1) publish_ssq();
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // X chunk 0 is in LDS; weight loads stay in flight

    f32x16_t acc0 = {}, acc1 = {};
    const int rbase = 4 * (lane >> 5);
    // row scales of this lane's 32 accumulator rows: known from here on in the single-chunk
    // form (kept in registers: a tile's end is on the critical path), read at the tile's end
    // in the other, where the row sums are complete only with the last chunk
    float4 rsa[4], rsb[4];
    if (PRO == PRO_GAIN && !MULTI) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        rsa[i] = *reinterpret_cast<const float4*>(&s_rowscale[8 * i + rbase]);
        rsb[i] = *reinterpret_cast<const float4*>(&s_rowscale[32 + 8 * i + rbase]);
      }
    }
    int ct = 0, cj = cj0;                                // piece being consumed: tile count, piece
    int steps_left = n_run;                              // single-chunk form: every wave walks its own run
    bool fresh = true;                                   // the accumulators hold nothing of the current tile yet
    bool head_pending = cj0 > 0;                         // the run starts inside a tile: its sum goes to the wave before
    // partial tile of this wave's current tile and this slice (data, inverse scale)
    const size_t pidx0 = xbase * a.tstride + (size_t)(t_begin + ft - t0x) * S + sp;
    const uint4* pt = a.part16 + pidx0 * kTileVec4 + lane;
    const float* ps = a.pscale + pidx0;

    // A finished tile goes out (called at the tile's last piece, or after the loop for a tile
    // shared with the next wave).
    auto finish_tile = [&]() {
      // Tile finished.  The partial tile goes out in register order as scaled int16 pairs
      // (each store instruction writes 1 KiB contiguous); the reducer reads it back with
      // the same lane -> register mapping.  Register r of lane l is row
      // 8*(r/4) + 4*(l/32) + r%4 (+32 for acc1), column l % 32 of the [64][32] tile.
      // The stores are issued from inline assembly on purpose: the compiler's wait-count
      // bookkeeping then sees loads only and keeps its waits exact; a store it knew of would
      // turn every later wait into a drain of the whole ring.  Unseen stores can only make
      // its waits longer, never too short; their own completion is awaited explicitly
      // before the arrival below.
      float t0[16], t1[16];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float4 ra = make_float4(1.f, 1.f, 1.f, 1.f), rb = ra;
        if (PRO == PRO_GAIN) {                     // rows brought to a common size
          ra = MULTI ? *reinterpret_cast<const float4*>(&s_rowscale[8 * i + rbase]) : rsa[i];
          rb = MULTI ? *reinterpret_cast<const float4*>(&s_rowscale[32 + 8 * i + rbase]) : rsb[i];
        }
        t0[4 * i] = acc0[4 * i] * ra.x;         t1[4 * i] = acc1[4 * i] * rb.x;
        t0[4 * i + 1] = acc0[4 * i + 1] * ra.y; t1[4 * i + 1] = acc1[4 * i + 1] * rb.y;
        t0[4 * i + 2] = acc0[4 * i + 2] * ra.z; t1[4 * i + 2] = acc1[4 * i + 2] * rb.z;
        t0[4 * i + 3] = acc0[4 * i + 3] * ra.w; t1[4 * i + 3] = acc1[4 * i + 3] * rb.w;
      }
      unsigned tmax = 0u;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const unsigned m0_ = mag_bits(t0[r]), m1_ = mag_bits(t1[r]);
        const unsigned mm = m0_ > m1_ ? m0_ : m1_;
        tmax = tmax > mm ? tmax : mm;
      }
      unsigned wmax = wave_max_u32(tmax);
      const bool clean = wmax < kInfBits;
      if (!clean) {                                // rare: the maximum of the finite elements
        tmax = 0u;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const unsigned m0_ = finite_mag_bits(t0[r]), m1_ = finite_mag_bits(t1[r]);
          const unsigned mm = m0_ > m1_ ? m0_ : m1_;
          tmax = tmax > mm ? tmax : mm;
        }
        wmax = wave_max_u32(tmax);
      }
      float psc, pinv;
      partial_tile_scale(wmax, psc, pinv);
      u32x4_t dq[4];
      if (clean) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = 8 * (q & 1) + 2 * e;     // register inside acc0 (q < 2) or acc1
            dq[q][e] = q < 2 ? pack_q16x2(t0[r], t0[r + 1], psc) : pack_q16x2(t1[r], t1[r + 1], psc);
          }
      } else {
        pinv = -pinv;                              // tells the reader to look for the code
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = 8 * (q & 1) + 2 * e;
            dq[q][e] = q < 2 ? pack_q16x2_coded(t0[r], t0[r + 1], psc) : pack_q16x2_coded(t1[r], t1[r + 1], psc);
          }
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const u32x4_t d = dq[q];
        // s_nop: a store of more than 64 bits reads its data registers a few cycles after
        // issue; the compiler cannot see that this is a store, so the wait states are explicit
        asm volatile("global_store_dwordx4 %0, %1, off\n\ts_nop 3" ::"v"(pt + q * 64), "v"(d) : "memory");
      }
      if (lane == 0) asm volatile("global_store_dword %0, %1, off" ::"v"(ps), "v"(pinv) : "memory");
    };

    // One step: the piece in `buf` (piece cj of this wave's current tile) is multiplied and the
    // slot is refilled.  The loop is compute bound at one wave per SIMD, so the bookkeeping
    // between the MFMA blocks is kept to a few scalar instructions: a tile's first product takes
    // a zero addend instead of cleared accumulators, finished tiles are stored straight from the
    // accumulator registers.
    auto step = [&](u32x4_t* buf) {
      if (MULTI || steps_left > 0) {
        --steps_left;
        const int jq = cj & 3;
        if (!MULTI || ct < my_tiles) {
          const uint4* xf = xs + (size_t)(jq * kPieceFrags * 4) * 64;
          // One basic block per piece: 32 LDS reads and 32 MFMAs.  The schedule is pinned so
          // that the four X operands of fragment f + 1 are read while the MFMAs of fragment f
          // run (left to itself the scheduler reads each operand right before its use, and the
          // matrix pipe waits for LDS every time).  k-step inside the chunk: jq * 8 + f; its
          // low 3 bits are those of f.
          auto piece_block = [&](auto first_of_tile) {
            constexpr bool kFirst = decltype(first_of_tile)::value;
            bf16x8_t wf[kPieceFrags];                    // the piece's eight weight fragments
#pragma unroll
            for (int l = 0; l < kLoads; ++l) {
              if (WF == 2) {
                bf16x8_t f4[4];
                w4_to_frags(buf[l], f4);
                wf[4 * l] = f4[0]; wf[4 * l + 1] = f4[1]; wf[4 * l + 2] = f4[2]; wf[4 * l + 3] = f4[3];
              } else if (WF == 1) {
                w8_to_frags(buf[l], wf[2 * l], wf[2 * l + 1]);
              } else {
                wf[l] = __builtin_bit_cast(bf16x8_t, buf[l]);
              }
            }
#pragma unroll
            for (int f = 0; f < kPieceFrags; ++f) {
              const uint4* xp = xf + (size_t)(f * 4) * 64 + frag_slot(lane, f);
              const bf16x8_t w = wf[f];
              const bf16x8_t x0h = __builtin_bit_cast(bf16x8_t, xp[0]);
              const bf16x8_t x0l = __builtin_bit_cast(bf16x8_t, xp[64]);
              const bf16x8_t x1h = __builtin_bit_cast(bf16x8_t, xp[128]);
              const bf16x8_t x1l = __builtin_bit_cast(bf16x8_t, xp[192]);
              if (kFirst && f == 0) {                    // a tile's first product: zero addend
                const f32x16_t zero = {};
                acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x0h, w, zero, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1h, w, zero, 0, 0, 0);
              } else {
                acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x0h, w, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1h, w, acc1, 0, 0, 0);
              }
              acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x0l, w, acc0, 0, 0, 0);
              acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1l, w, acc1, 0, 0, 0);
            }
            if (WF == 1) __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);   // conversion of fragment 0
            if (WF == 2) __builtin_amdgcn_sched_group_barrier(0x002, 21, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);       // LDS reads of fragment 0
#pragma unroll
            for (int f = 0; f < kPieceFrags - 1; ++f) {
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA of fragment f
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read of fragment f + 1
                if (WF == 1) __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);   // a quarter of fragment f + 1's conversion
                if (WF == 2) __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
              }
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
          };
          if (MULTI ? cj == 0 : fresh) piece_block(std::true_type{}); else piece_block(std::false_type{});
          fresh = false;
          if (cj == np - 1) {
            if (!MULTI && head_pending) {
              // the tile's first pieces belong to the wave before this one: it adds these sums
              // to its own after the loop and stores the tile
              head_pending = false;
              uint4* h = s_head + (size_t)(wave - 1) * 8 * 64 + lane;
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const f32x4_t lo4 = {acc0[4 * q], acc0[4 * q + 1], acc0[4 * q + 2], acc0[4 * q + 3]};
                const f32x4_t hi4 = {acc1[4 * q], acc1[4 * q + 1], acc1[4 * q + 2], acc1[4 * q + 3]};
                h[q * 64] = __builtin_bit_cast(uint4, lo4);
                h[(4 + q) * 64] = __builtin_bit_cast(uint4, hi4);
              }
            } else {
              finish_tile();
            }
            fresh = true;
            ps += (MULTI ? 4 : 1) * S;
            pt += (size_t)(MULTI ? 4 : 1) * S * kTileVec4;   // this wave's next tile
          }
        }
        if (++cj == np) {
          cj = 0;
          ++ct;
        }
      }
      issue(buf);
    };
    if (MULTI) {
      // A slice of several LDS chunks: a group has at most four tiles here, one per wave, whose
      // accumulators carry over from chunk to chunk, and all four waves walk the chunks together
      // (also a wave without a tile: re-staging needs them all).  The X rows of the next chunk
      // are requested before the four pieces of the current one are multiplied, so that their
      // round trip runs under the matrix work; every load keeps a fixed place in the order of
      // issue, and the waits stay exact.  The barriers order LDS traffic only.
      for (int c = 0; c < n_chunks; ++c) {
        const int cn = min(c + 1, n_chunks - 1);         // (the last round re-reads its own rows, unused)
        float4 xa[16], xb[16], g0, g1;
        x_load(cn, xa, xb, g0, g1);
#pragma unroll
        for (int sl = 0; sl < kRing; ++sl) step(ring[sl]);
        if (c + 1 < n_chunks) {
          asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // chunk c has been read by all
          x_convert(cn, xa, xb, g0, g1, [](int) {});
          if (PRO == PRO_GAIN && cn == n_chunks - 1) publish_ssq();
          asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        }
      }
    } else {
      while (steps_left > 0) {
#pragma unroll
        for (int sl = 0; sl < kRing; ++sl) step(ring[sl]);
      }
      // tiles shared by two waves: every wave has left the loop, the sums of the later pieces
      // are in LDS
      asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
      if (cj != 0) {                                     // the run ended inside a tile
        const uint4* h = s_head + (size_t)wave * 8 * 64 + lane;   // written by wave + 1
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4_t lo4 = __builtin_bit_cast(f32x4_t, h[q * 64]);
          const f32x4_t hi4 = __builtin_bit_cast(f32x4_t, h[(4 + q) * 64]);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc0[4 * q + e] += lo4[e];
            acc1[4 * q + e] += hi4[e];
          }
        }
        finish_tile();
      }
    }

    // ---- second half: group barrier, reduction, epilogue (arguments read afresh) ----
    gemm_args_ptr_t ap2 = ap;
    asm volatile("" : "+s"(ap2));
    gemm_reduce_phase<PRO, EPI, WF>(ap2, s_pos, s_crow, tid, lane, wave, xcd, u, mt);
  }
}

// One product per launch, block = 256.
//  - up to 64 rows (ROWS = false): grid = (n_xcd, gpx * S); y = unit.
//  - more rows (ROWS = true): grid = (n_xcd, gpx * m_tiles * S); y = (group * m_tiles + row tile)
//    * S + slice.  The S slices of one (group, row tile) follow each other - they meet at the
//    group barrier and must be resident together - and the row tiles of one group follow each
//    other on the same XCD: they stream the same weights at about the same time, so that all but
//    the first find them in that XCD's L2 and the matrix leaves HBM about once per launch however
//    many rows there are.
template <int PRO, int EPI, bool MULTI, int WF, bool ROWS>
__global__ __launch_bounds__(256, 1) void gemm_stream_bf16(const GemmArgs a) {
  __shared__ uint4 lds_raw[(kGemmLdsAlloc + 15) / 16];
  gemm_args_ptr_t ap = (gemm_args_ptr_t)__builtin_amdgcn_kernarg_segment_ptr();
  int u = blockIdx.y, mt = 0;
  if (ROWS) {
    const int m_tiles = (a.M + kMTile - 1) / kMTile;
    const int sp = (int)blockIdx.y % a.S, gm = (int)blockIdx.y / a.S;
    mt = gm % m_tiles;
    u = (gm / m_tiles) * a.S + sp;
  }
  gemm_stream_body<PRO, EPI, MULTI, WF, ROWS>(ap, blockIdx.x, u, mt, carve_gemm_lds(lds_raw));
}

}  // namespace sv
#endif
