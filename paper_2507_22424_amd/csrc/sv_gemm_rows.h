// The layer's products for MANY rows (several episodes verified together: hundreds of tree
// rows) on the gfx950 matrix cores.
//
// With up to 128 rows the products are bound by the bytes of the weights and
// gemm_stream_bf16 streams them once past activations that wait in LDS.  With hundreds of rows
// the same products are bound by the matrix cores, and what has to be kept small is the traffic
// per matrix instruction: every workgroup owns a 128-row x 256-column (or 384-column) block of
// the output, keeps it in accumulator registers and walks the whole K range; both operands
// arrive already cut into matrix-core fragments (1 KiB = 32 rows x 16 k-values, lane-major), so
// a fragment travels from memory into LDS with one direct-to-LDS load instruction per wave and
// from LDS into operand registers with one 16-byte read per lane, without any shuffling:
//   * weights: the packed layout of gemm_stream_bf16 as it is (same row permutations, so the
//     RoPE / SwiGLU epilogues stay tile local);
//   * activations: split_rows_kernel turns the float32 rows into hi + lo bf16 fragments once per
//     product (RMSNorm applied on the way), so that the error of a product stays at float32
//     rounding level as in the streaming kernel.
// A ring of k-steps lives in LDS (256 columns: four k-steps of 16 KiB = 8 activation + 8 weight
// fragments, two workgroups per CU; 384 columns: six k-steps of 20 KiB, one workgroup per CU);
// the loads of a k-step are issued ring depth - 1 steps ahead, each wave waits for its own loads
// with an exact count and one barrier per k-step publishes them; operands of the next k-step
// are read while the matrix instructions of the current one run.
// Workgroups are numbered so that an XCD works on four neighbouring column blocks times all row
// blocks at a time: whatever two of them share is fetched into that XCD's L2 once.
// A product whose output blocks alone would leave the chip short of workgroups (N = hidden, or
// few rows) splits K across up to 16 workgroups per block; their float32 partial blocks are added
// in fixed order by a reduction kernel that carries the product's epilogue (residual, SwiGLU,
// RoPE + K/V append).
#ifndef SV_GEMM_ROWS_H
#define SV_GEMM_ROWS_H

#include "sv_gemm_mfma.h"

namespace sv {

constexpr int kRowsTM = 128;        // rows of a workgroup's output block
constexpr int kRowsTN = 256;        // columns (384 where that makes the workgroups of a product a whole number of rounds of the chip)
constexpr int kRowsMaxKsplit = 16;  // K split of a product whose output blocks alone would leave the chip short of workgroups
constexpr int kRowsMinTiles = 1;    // more 64-row tiles than this: the products run on gemm_rows_kernel

struct RowsArgs {
  const uint4* Xs;       // activations as fragments: [M_pad / 32][K / 16][hi, lo][64 lanes]
  const uint4* Wp;       // packed weights: [N / 32][K / 16][64 lanes]
  int M, N, K;
  int m_tiles, n_tiles;  // blocks of kRowsTM rows / kRowsTN columns
  int n_xcd;
  int ksplit;            // workgroups that share one output block along K (1 .. kRowsMaxKsplit)
  float* part;           // ksplit > 1: [ksplit][m_tiles * kRowsTM][N] float32 partial sums
  // epilogues (ksplit == 1), as in gemm_stream_bf16
  float* act;            // EPI_SWIGLU: [M, N/2]
  float* q_out;          // EPI_QKV
  bf16_t* kc;
  bf16_t* vc;
  const int32_t* depth;
  const int32_t* prefix_len;
  int p_max, cap, T, nh;
  float theta;
};

// 1 / sqrt(mean(x^2) + eps) of every row.  grid = rows, block = 256.
__global__ __launch_bounds__(256) void rows_rstd_kernel(const float* __restrict__ x, int K, float eps,
                                                        float* __restrict__ rstd) {
  __shared__ float red[4];
  const float* xr = x + (size_t)blockIdx.x * K;
  float ss = 0.f;
  for (int i = threadIdx.x * 4; i < K; i += 1024) {
    const float4 v = *reinterpret_cast<const float4*>(xr + i);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = block_sum_256(ss, red);
  if (threadIdx.x == 0) rstd[blockIdx.x] = 1.0f / sqrtf(ss / (float)K + eps);
}

// float32 rows -> hi + lo bf16 fragments.  GAIN: every value is first multiplied by gain[k] *
// rstd[row] (RMSNorm).  Rows beyond M become zeros.  grid = (M_pad / 32, K / 256), block = 256:
// a workgroup converts 32 rows x 256 k-values; one thread handles 8 consecutive k-values of a
// row at a time, which are the 16 bytes one lane holds of a fragment.
template <bool GAIN>
__global__ __launch_bounds__(256) void split_rows_kernel(const float* __restrict__ x,
                                                         const float* __restrict__ gain,
                                                         const float* __restrict__ rstd, int M, int K,
                                                         uint4* __restrict__ Xs) {
  const int mb = blockIdx.x, kc = blockIdx.y;
  const int nks = K / kFragK;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int c = it * 256 + threadIdx.x;
    const int r = c >> 5, kq = c & 31;                  // row inside the block, 8-wide k chunk inside the 256
    const int row = mb * 32 + r, k = kc * 256 + kq * 8;
    float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (row < M) {
      const float4 a0 = *reinterpret_cast<const float4*>(x + (size_t)row * K + k);
      const float4 a1 = *reinterpret_cast<const float4*>(x + (size_t)row * K + k + 4);
      v[0] = a0.x; v[1] = a0.y; v[2] = a0.z; v[3] = a0.w; v[4] = a1.x; v[5] = a1.y; v[6] = a1.z; v[7] = a1.w;
      if (GAIN) {
        const float rs = rstd[row];
        const float4 g0 = *reinterpret_cast<const float4*>(gain + k);
        const float4 g1 = *reinterpret_cast<const float4*>(gain + k + 4);
        v[0] *= g0.x * rs; v[1] *= g0.y * rs; v[2] *= g0.z * rs; v[3] *= g0.w * rs;
        v[4] *= g1.x * rs; v[5] *= g1.y * rs; v[6] *= g1.z * rs; v[7] *= g1.w * rs;
      }
    }
    uint4 hi4, lo4;
    hi4.x = pack_bf16x2(v[0], v[1]); hi4.y = pack_bf16x2(v[2], v[3]);
    hi4.z = pack_bf16x2(v[4], v[5]); hi4.w = pack_bf16x2(v[6], v[7]);
    lo4.x = pack_bf16x2(v[0] - bf16_lo_f32(hi4.x), v[1] - bf16_hi_f32(hi4.x));
    lo4.y = pack_bf16x2(v[2] - bf16_lo_f32(hi4.y), v[3] - bf16_hi_f32(hi4.y));
    lo4.z = pack_bf16x2(v[4] - bf16_lo_f32(hi4.z), v[5] - bf16_hi_f32(hi4.z));
    lo4.w = pack_bf16x2(v[6] - bf16_lo_f32(hi4.w), v[7] - bf16_hi_f32(hi4.w));
    const int ks = (k / kFragK), lane = r + 32 * (kq & 1);
    uint4* dst = Xs + (((size_t)mb * nks + ks) * 2) * 64 + lane;
    dst[0] = hi4;
    dst[64] = lo4;
  }
}

// x_io[m][n] = x_res[m][n] + part[0][m][n] + part[1][m][n] + ..  (fixed order).  One thread = 4 columns.
__global__ __launch_bounds__(256) void rows_reduce_resid_kernel(const float* __restrict__ part, int ksplit,
                                                                size_t plane, const float* x_res,
                                                                float* x_io, size_t n_vec4) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n_vec4) return;
  float4 s = reinterpret_cast<const float4*>(x_res)[i];
  for (int z = 0; z < ksplit; ++z) {
    const float4 p = reinterpret_cast<const float4*>(part + (size_t)z * plane)[i];
    s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
  }
  reinterpret_cast<float4*>(x_io)[i] = s;
}

// The other two epilogues for products whose K range is split (few rows: the column blocks
// alone would leave most of the chip idle).  Both add the ksplit partial blocks in fixed order
// and then do what the fused epilogue of the unsplit kernel does, with the same arithmetic.
// Columns are in the packed order of the weights: tile = 32 columns, lanes 0..15 and 16..31 of a
// tile hold the two partners of a pair (gate / up of one output column; the rotary pair
// (j, j + 64) of a head).

// act[m][tile * 16 + j] = silu(gate) * up.  One thread = 4 output columns.
__global__ __launch_bounds__(256) void rows_reduce_swiglu_kernel(const float* __restrict__ part, int ksplit,
                                                                 size_t plane, int M, int N,
                                                                 float* __restrict__ act) {
  const int F = N / 2;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;   // (row, tile, quarter)
  const size_t per_row = (size_t)(N / 32) * 4;
  if (i >= (size_t)M * per_row) return;
  const int m = (int)(i / per_row);
  const int rem = (int)(i - (size_t)m * per_row);
  const int tile = rem >> 2, j4 = (rem & 3) * 4;
  float4 g = make_float4(0.f, 0.f, 0.f, 0.f), u = g;
  for (int z = 0; z < ksplit; ++z) {
    const float* p = part + (size_t)z * plane + (size_t)m * N + tile * 32 + j4;
    const float4 pg = *reinterpret_cast<const float4*>(p);
    const float4 pu = *reinterpret_cast<const float4*>(p + 16);
    g.x += pg.x; g.y += pg.y; g.z += pg.z; g.w += pg.w;
    u.x += pu.x; u.y += pu.y; u.z += pu.z; u.w += pu.w;
  }
  const float4 o = make_float4(silu_fast(g.x) * u.x, silu_fast(g.y) * u.y, silu_fast(g.z) * u.z,
                               silu_fast(g.w) * u.w);
  *reinterpret_cast<float4*>(act + (size_t)m * F + tile * 16 + j4) = o;
}

// q/k/v: RoPE at position prefix + depth on q and k, q written as float32, k and v appended to the
// bf16 cache.  One thread = one pair of partner columns of one row.
__global__ __launch_bounds__(256) void rows_reduce_qkv_kernel(const float* __restrict__ part, int ksplit,
                                                              size_t plane, const RowsArgs a) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;   // (row, tile, j)
  const size_t per_row = (size_t)(a.N / 32) * 16;
  if (i >= (size_t)a.M * per_row) return;
  const int m = (int)(i / per_row);
  const int rem = (int)(i - (size_t)m * per_row);
  const int tile = rem >> 4, j = rem & 15;
  float v0 = 0.f, v1 = 0.f;
  for (int z = 0; z < ksplit; ++z) {
    const float* p = part + (size_t)z * plane + (size_t)m * a.N + tile * 32 + j;
    v0 += p[0];
    v1 += p[16];
  }
  const int b = m / a.T, t = m - b * a.T;
  int P = a.prefix_len[b];
  P = P < 0 ? 0 : (P > a.p_max ? a.p_max : P);
  const int tiles_per_mat = a.nh * 4;
  const int which = tile / tiles_per_mat;
  const int head = (tile % tiles_per_mat) / 4, uq = tile % 4;
  const int jr = 16 * uq + j;
  float o0 = v0, o1 = v1;
  if (which != 2) {
    const float turn_freq = exp2f(-(float)jr * (1.0f / 64.0f) * log2f(a.theta)) * 0.15915494309189535f;
    float turns = (float)(P + a.depth[m]) * turn_freq;
    turns -= floorf(turns);
    const float c = __builtin_amdgcn_cosf(turns), s = __builtin_amdgcn_sinf(turns);
    o0 = v0 * c - v1 * s;
    o1 = v1 * c + v0 * s;
  }
  const int D = a.nh * 128;
  if (which == 0) {
    float* q = a.q_out + (size_t)m * D + head * 128 + jr;
    q[0] = o0;
    q[64] = o1;
  } else {
    bf16_t* cache = which == 1 ? a.kc : a.vc;
    bf16_t* dst = cache + ((size_t)b * a.nh * a.cap + (size_t)head * a.cap + P + t) * 128 + jr;
    dst[0] = f32_to_bf16(o0);
    dst[64] = f32_to_bf16(o1);
  }
}

// grid = (n_xcd, ceil(n_tiles / n_xcd) * m_tiles, ksplit), block = 256 (waves 2 x 2: rows wm * 64,
// columns wn * 32 * NTW of the block).  NTW = weight tiles (32 columns) per wave: 4 gives blocks
// of 256 columns, 6 blocks of 384 (for the q/k/v product of the 7B shape: 32 column blocks x 8 row
// blocks = 256 workgroups, one full round of the chip instead of one and a half).
// DEEP: eight k-steps in LDS and one workgroup per CU instead of four k-steps and two workgroups:
// for a single block of rows, where every weight byte comes from HBM and is used once, the loads
// in flight per workgroup are what sets its pace.
template <int EPI, bool SPLIT, int NTW, bool DEEP = false>
__global__ __launch_bounds__(256, (NTW == 4 && !DEEP) ? 2 : 1) void gemm_rows_kernel(const RowsArgs a) {
  constexpr int kFr = 8 + 2 * NTW;                 // fragments per k-step: 4 row blocks x (hi, lo), 2 * NTW weight tiles
  constexpr int kLw = kFr / 4;                     // direct-to-LDS loads per wave and k-step
  constexpr int kR = NTW == 6 ? 6 : (DEEP ? 8 : 4);   // k-steps resident in LDS (120 / 128 / 64 KiB)
  static_assert(kFr % 4 == 0 && (NTW == 4 || NTW == 6), "fragment loads are dealt evenly to the four waves");
  __shared__ uint4 ring[kR][kFr][64];
  __shared__ int s_pos[kRowsTM], s_crow[kRowsTM];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int seq = blockIdx.y;
  const int mt = seq % a.m_tiles, nt = (int)blockIdx.x + a.n_xcd * (seq / a.m_tiles);
  if (nt >= a.n_tiles) return;
  const int nks_all = a.K / kFragK;
  const int nks = nks_all / a.ksplit, ks0 = (int)blockIdx.z * nks;
  const int m0 = mt * kRowsTM;

  if (EPI == EPI_QKV && tid < kRowsTM) {
    const int m = min(m0 + tid, a.M - 1);
    const int b = m / a.T, t = m - b * a.T;
    int P = a.prefix_len[b];
    P = P < 0 ? 0 : (P > a.p_max ? a.p_max : P);
    s_pos[tid] = P + a.depth[m];
    s_crow[tid] = b * a.nh * a.cap + P + t;
  }

  // this wave's fragment loads per k-step: fragment f = kLw * wave + i; f < 8 is an activation
  // fragment (row block f / 2, hi or lo), the others are the weight tiles f - 8
  typedef const __attribute__((address_space(1))) uint4* gptr_t;
  gptr_t src[kLw];
  unsigned step[kLw];                                        // uint4 from one k-step to the next
#pragma unroll
  for (int i = 0; i < kLw; ++i) {
    const int f = kLw * wave + i;
    if (f < 8) {
      src[i] = (gptr_t)a.Xs + ((((size_t)(mt * 4 + (f >> 1)) * nks_all + ks0) * 2 + (f & 1)) * 64 + lane);
      step[i] = 128;
    } else {
      src[i] = (gptr_t)a.Wp + (((size_t)(nt * 2 * NTW + (f - 8)) * nks_all + ks0) * 64 + lane);
      step[i] = 64;
    }
  }
  // k-step j of this workgroup -> ring slot j % kR.  Past the last k-step the loads repeat it
  // (into a slot nobody reads any more): the number of loads in flight stays fixed and the
  // waits below are exact.
  auto issue = [&](int j) {
    const int jc = j < nks ? j : nks - 1;
    const int slot = j % kR;
    // Direct-to-LDS loads (lane l's 16 bytes land at the LDS address in M0 + 16 l), written as
    // inline assembly: the compiler, when it sees such a load, waits for ALL outstanding loads
    // before the next LDS read that might touch the same array, which would drain the ring at
    // every k-step; the waits that are really needed are the explicit ones below.
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) void*)&ring[slot][kLw * wave][0];
#pragma unroll
    for (int i = 0; i < kLw; ++i) {
      gptr_t g = src[i] + (size_t)jc * step[i];
      asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds0 + 1024u * i), "v"(g) : "memory");
    }
  };

  f32x16_t acc[2][NTW];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < NTW; ++j) acc[i][j] = f32x16_t{};

  struct Ops {
    bf16x8_t ah[2], al[2], b[NTW];
  };
  auto read_ops = [&](int j, Ops& o) {
    const int slot = j % kR;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      o.ah[i] = __builtin_bit_cast(bf16x8_t, ring[slot][2 * (2 * wm + i)][lane]);
      o.al[i] = __builtin_bit_cast(bf16x8_t, ring[slot][2 * (2 * wm + i) + 1][lane]);
    }
#pragma unroll
    for (int jn = 0; jn < NTW; ++jn) o.b[jn] = __builtin_bit_cast(bf16x8_t, ring[slot][8 + NTW * wn + jn][lane]);
  };
  // the two products (hi and lo half of the activations) of row block i with weight tiles [j0, j1)
  auto multiply = [&](const Ops& o, int i, int j0, int j1) {
#pragma unroll
    for (int jn = j0; jn < j1; ++jn) {
      acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(o.ah[i], o.b[jn], acc[i][jn], 0, 0, 0);
      acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(o.al[i], o.b[jn], acc[i][jn], 0, 0, 0);
    }
  };

#pragma unroll
  for (int j = 0; j < kR - 1; ++j) issue(j);
  // k-step 0 complete: own loads (kR - 2 younger k-steps may still be in flight), then everybody's
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((kR - 2) * kLw) : "memory");
  Ops o0, o1;
  read_ops(0, o0);
  // One iteration = k-step ks, in an order that is pinned (the scheduler may not move anything
  // across the fences): a first few products; then wait for k-step ks + 1 (own loads: kR - 3
  // younger k-steps may be in flight; then the barrier, which also tells that every wave has read
  // k-step ks - 1, whose slot is refilled next), refill, start the LDS reads of the operands of
  // k-step ks + 1; then the other products, which run while those reads return.  Left to itself
  // the scheduler moves each read down to just before its first use and the matrix cores then
  // wait for LDS at every k-step.
  auto iteration = [&](int ks, const Ops& cur, Ops& nxt) {
    multiply(cur, 0, 0, 2);
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((kR - 3) * kLw) : "memory");
    issue(ks + kR - 1);
    read_ops(ks + 1, nxt);
    __builtin_amdgcn_sched_barrier(0);
    multiply(cur, 0, 2, NTW);
    multiply(cur, 1, 0, NTW);
    __builtin_amdgcn_sched_barrier(0);
  };
  for (int ks = 0; ks < nks; ks += 2) {          // nks is even (K is a multiple of 256)
    iteration(ks, o0, o1);
    iteration(ks + 1, o1, o0);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // nothing of the ring is in flight when the wave ends

  // ---- output: register r of lane l of block (i, jn) is row 8*(r/4) + 4*(l/32) + r%4, column l%32 ----
  // The accumulator registers of a lane go through LDS (the ring is free now), one row block of
  // the wave at a time (at most 24 KiB per wave), and come back four at a time inside a loop, so
  // that the epilogue is a short piece of code run many times instead of 40 KiB of straight-line
  // code fetched for a single pass.
  const int ln = lane & 31, rbase = 4 * (lane >> 5);
  f32x4_t* stage = reinterpret_cast<f32x4_t*>(&ring[0][0][0]) + (size_t)wave * (NTW * 4 * 64) + lane;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // the ring (i = 0) / the first half (i = 1) has been read by all
#pragma unroll
    for (int jn = 0; jn < NTW; ++jn)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        stage[(jn * 4 + q) * 64] = f32x4_t{acc[i][jn][4 * q], acc[i][jn][4 * q + 1], acc[i][jn][4 * q + 2], acc[i][jn][4 * q + 3]};
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // (own data only)
#pragma unroll 1
    for (int item = 0; item < NTW * 4; ++item) {
      const int jn = item >> 2, q = item & 3;
      const int tile = nt * 2 * NTW + wn * NTW + jn;       // 32-row weight tile = 32 output columns
      const int ml0 = wm * 64 + i * 32 + 8 * q + rbase;    // row inside the block of the first value
      const f32x4_t vv = stage[item * 64];
      float v[4] = {vv[0], vv[1], vv[2], vv[3]};
      if (SPLIT) {
        float* dst = a.part + ((size_t)blockIdx.z * a.m_tiles * kRowsTM + m0 + ml0) * a.N + tile * 32 + ln;
#pragma unroll
        for (int j = 0; j < 4; ++j) dst[(size_t)j * a.N] = v[j];
      } else if (EPI == EPI_SWIGLU) {                      // lanes 0..15 gate, 16..31 up of the same column
        const int F = a.N / 2;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float up = lane_xor16(v[j], lane);
          if (ln < 16 && m0 + ml0 + j < a.M)
            a.act[(size_t)(m0 + ml0 + j) * F + tile * 16 + ln] = silu_fast(v[j]) * up;
        }
      } else if (EPI == EPI_QKV) {
        const int tiles_per_mat = a.nh * 4;
        const int which = tile / tiles_per_mat;
        const int head = (tile % tiles_per_mat) / 4, uq = tile % 4;
        const int jr = 16 * uq + (ln & 15);
        const int dcol = jr + 64 * (ln >> 4);
        const float turn_freq = exp2f(-(float)jr * (1.0f / 64.0f) * log2f(a.theta)) * 0.15915494309189535f;
        const float sgn = (ln & 16) ? 1.0f : -1.0f;
        const int D = a.nh * 128;
        bf16_t* cache = which == 1 ? a.kc : a.vc;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int ml = ml0 + j;
          float val = v[j];
          const float partner = lane_xor16(val, lane);
          if (which != 2) {
            float turns = (float)s_pos[ml] * turn_freq;
            turns -= floorf(turns);
            val = val * __builtin_amdgcn_cosf(turns) + sgn * partner * __builtin_amdgcn_sinf(turns);
          }
          if (m0 + ml < a.M) {
            if (which == 0)
              a.q_out[(size_t)(m0 + ml) * D + head * 128 + dcol] = val;
            else
              cache[((size_t)s_crow[ml] + (size_t)head * a.cap) * 128 + dcol] = f32_to_bf16(val);
          }
        }
      }
    }
  }
}

}  // namespace sv
#endif
