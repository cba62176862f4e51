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
//     along K.  A wavefront reads its tile as one contiguous stream, 1 KiB per load
//     instruction, straight into operand registers, one 128-wide K block ahead of the math.
//   * activations stay float32 in memory; while staging a K block into LDS (in fragment
//     order) each value is split into hi + lo bf16 parts and both are multiplied, so the
//     product is accurate to ~2^-17 instead of 2^-9 at no cost in HBM bytes (the matrix cores
//     idle most of the time on this path).  This keeps a 32-layer pass inside the 2e-2 bar.
//   * a workgroup owns 128 weight rows x one K slice.  Slices of the same rows are placed on
//     the same XCD (workgroup id modulo 8) so their partial tiles meet in that XCD's L2; the
//     workgroup that finishes last adds the partials in slice order (bit-reproducible) and
//     runs the epilogue: RMSNorm scale + RoPE + KV append, residual add, or SwiGLU.
//   * RMSNorm is folded in: the prologue multiplies by the gain and sums x^2 over its K
//     slice; the slices of one row group cover K exactly once, so the last workgroup has the
//     full row sums and scales the output rows by 1/sqrt(mean + eps).
#ifndef SV_GEMM_MFMA_H
#define SV_GEMM_MFMA_H

#include "sv_internal.h"

namespace sv {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kFragRows = 32;    // weight rows per fragment (MFMA N)
constexpr int kFragK = 16;       // k-values per fragment (MFMA K)
constexpr int kBlkK = 128;       // k-values staged per LDS block (8 fragments)
constexpr int kWgRows = 128;     // weight rows per workgroup (4 waves x 32)
constexpr int kTileFloats = kMTile * kWgRows;   // one partial tile, [64][128] float32

enum { PRO_PLAIN = 0, PRO_GAIN = 1 };
enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2 };

// Packer: src [rows, K] bf16 row-major -> fragment order.  Source row n goes to destination
// row  (n / group) * dst_stride + dst_off + n % group  (group = rows: plain placement behind
// dst_off rows; group = 64, dst_stride = 128: gate / up interleaved per 128-row tile).
// One thread moves one 16-byte chunk (8 k-values); chunk (n, kc) lands at uint4 index
// ((n/32) * (K/16) + kc/2) * 64 + (n%32) + 32 * (kc%2).
__global__ void pack_rows_mfma(const uint4* __restrict__ src, uint4* __restrict__ dst, int rows,
                               int K, int group, int dst_stride, int dst_off) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int chunks_per_row = K / 8;
  if (i >= (size_t)rows * chunks_per_row) return;
  const int n_src = (int)(i / chunks_per_row), kc = (int)(i % chunks_per_row);
  const int n = (n_src / group) * dst_stride + dst_off + n_src % group;
  const size_t frag = (size_t)(n / kFragRows) * (K / kFragK) + (kc >> 1);
  dst[frag * 64 + (n % kFragRows) + 32 * (kc & 1)] = src[i];
}

struct GemmArgs {
  const float* X;        // [M, K] float32 activations
  const float* gain;     // [K] RMSNorm gain (PRO_GAIN) or unused
  const uint4* Wp;       // packed weights, N rows
  int M, N, K, S;        // rows of X, weight rows, reduction length, K slices
  float* part;           // [m_tiles][G][S][64][128] partial tiles (S > 1)
  float* sumsq;          // [m_tiles][G][S][64] partial row sums of x^2 (PRO_GAIN)
  int* counters;         // [m_tiles][G] arrival counters, zero before and after the launch
  float eps;
  // EPI_RESID: x_io [M, N] += Y
  float* x_io;
  // EPI_SWIGLU: act [M, N/2] = silu(gate) * up; tile rows 0..63 = gate, 64..127 = up
  float* act;
  // EPI_QKV: N = 3 * nh * 128; tile = one head of q, k or v
  float* q_out;          // [M, nh*128] float32, rotated
  bf16_t* kc;            // caches [B][nh][cap][128]
  bf16_t* vc;
  const int32_t* depth;
  const int32_t* prefix_len;
  int p_max, cap, T, nh;
  float theta;
};

__device__ inline uint32_t pack_bf16x2(float a, float b) {
  return (uint32_t)f32_to_bf16(a).bits | ((uint32_t)f32_to_bf16(b).bits << 16);
}

// grid = (8 * ceil(G / 8) * S, m_tiles), block = 256.  Workgroup w serves row group
// g = w % 8 + 8 * ((w / 8) / S) and K slice (w / 8) % S: all slices of a group share w % 8.
template <int PRO, int EPI>
__global__ __launch_bounds__(256, 2) void gemm_fused_bf16(const GemmArgs a) {
  __shared__ uint4 lds[2 * 2048];          // 2 buffers x [8 k-steps][2 m-halves][hi, lo][64 lanes]
  __shared__ float s_rstd[kMTile];
  __shared__ int s_last;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int G = a.N / kWgRows, S = a.S;
  const int slot = blockIdx.x >> 3;
  const int g = (blockIdx.x & 7) + 8 * (slot / S);
  const int sp = slot % S;
  if (g >= G) return;
  const int mt = blockIdx.y, m0 = mt * kMTile;
  const int K = a.K;
  const int nblk = K / kBlkK;
  const int qn = nblk / S, rem = nblk % S;
  const int blk_begin = sp * qn + min(sp, rem);
  const int nb = qn + (sp < rem ? 1 : 0);
  const int ntile = g * 4 + wave;
  const uint4* wp = a.Wp + ((size_t)ntile * (K / kFragK) + (size_t)blk_begin * 8) * 64 + lane;

  f32x16_t acc0 = {}, acc1 = {};
  uint4 wreg[8], wnext[8];
  float4 xa[4], xb[4];                      // 4 chunks of 8 floats per thread
  float ssq[4] = {0.f, 0.f, 0.f, 0.f};
  const int kc = tid & 15;                  // this thread's 8-wide chunk inside a K block
  const int mrow = tid >> 4;                // rows mrow, mrow + 16, mrow + 32, mrow + 48

  auto load_x = [&](int blk) {
    const int k = (blk_begin + blk) * kBlkK + kc * 8;
    float4 g0 = make_float4(1.f, 1.f, 1.f, 1.f), g1 = g0;
    if (PRO == PRO_GAIN) {
      g0 = *reinterpret_cast<const float4*>(a.gain + k);
      g1 = *reinterpret_cast<const float4*>(a.gain + k + 4);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = m0 + mrow + 16 * i;
      if (m < a.M) {
        const float* p = a.X + (size_t)m * K + k;
        xa[i] = *reinterpret_cast<const float4*>(p);
        xb[i] = *reinterpret_cast<const float4*>(p + 4);
      } else {
        xa[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        xb[i] = xa[i];
      }
      if (PRO == PRO_GAIN) {
        ssq[i] += xa[i].x * xa[i].x + xa[i].y * xa[i].y + xa[i].z * xa[i].z + xa[i].w * xa[i].w +
                  xb[i].x * xb[i].x + xb[i].y * xb[i].y + xb[i].z * xb[i].z + xb[i].w * xb[i].w;
        xa[i].x *= g0.x; xa[i].y *= g0.y; xa[i].z *= g0.z; xa[i].w *= g0.w;
        xb[i].x *= g1.x; xb[i].y *= g1.y; xb[i].z *= g1.z; xb[i].w *= g1.w;
      }
    }
  };
  // hi = bf16(v), lo = bf16(v - hi); fragment slot of chunk (m, kc):
  // [k-step kc/2][m-half m/32][hi|lo][lane (m%32) + 32*(kc%2)]
  auto store_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = mrow + 16 * i;
      const float v[8] = {xa[i].x, xa[i].y, xa[i].z, xa[i].w, xb[i].x, xb[i].y, xb[i].z, xb[i].w};
      float r[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) r[e] = v[e] - to_f32(f32_to_bf16(v[e]));
      const uint4 hi = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]),
                                  pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
      const uint4 lo = make_uint4(pack_bf16x2(r[0], r[1]), pack_bf16x2(r[2], r[3]),
                                  pack_bf16x2(r[4], r[5]), pack_bf16x2(r[6], r[7]));
      const int base = buf * 2048 + (((kc >> 1) * 2 + (m >> 5)) * 2) * 64 + (m & 31) + 32 * (kc & 1);
      lds[base] = hi;
      lds[base + 64] = lo;
    }
  };

  if (nb > 0) {
#pragma unroll
    for (int s = 0; s < 8; ++s) wreg[s] = wp[(size_t)s * 64];
    load_x(0);
    store_x(0);
  }
  for (int blk = 0; blk < nb; ++blk) {
    const int cur = blk & 1;
    const bool more = blk + 1 < nb;
    if (more) {
#pragma unroll
      for (int s = 0; s < 8; ++s) wnext[s] = wp[((size_t)(blk + 1) * 8 + s) * 64];
      load_x(blk + 1);
    }
    __syncthreads();
    const uint4* xs = lds + cur * 2048;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const bf16x8_t w = __builtin_bit_cast(bf16x8_t, wreg[s]);
      const bf16x8_t x0h = __builtin_bit_cast(bf16x8_t, xs[((s * 2 + 0) * 2 + 0) * 64 + lane]);
      const bf16x8_t x0l = __builtin_bit_cast(bf16x8_t, xs[((s * 2 + 0) * 2 + 1) * 64 + lane]);
      const bf16x8_t x1h = __builtin_bit_cast(bf16x8_t, xs[((s * 2 + 1) * 2 + 0) * 64 + lane]);
      const bf16x8_t x1l = __builtin_bit_cast(bf16x8_t, xs[((s * 2 + 1) * 2 + 1) * 64 + lane]);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x0h, w, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1h, w, acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x0l, w, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1l, w, acc1, 0, 0, 0);
    }
    if (more) {
      store_x(cur ^ 1);
#pragma unroll
      for (int s = 0; s < 8; ++s) wreg[s] = wnext[s];
    }
  }

  // Accumulator register r of lane l holds row 8 * (r / 4) + 4 * (l / 32) + r % 4 (acc1: + 32)
  // and column wave * 32 + l % 32 of the workgroup's [64][128] tile.
  const int col = wave * 32 + (lane & 31);
  const int rbase = 4 * (lane >> 5);
  const size_t unit = (size_t)mt * G + g;

  if (PRO == PRO_GAIN) {                    // row sums of x^2 over this K slice
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float v = ssq[i];
      v += __shfl_xor(v, 8, kWave);
      v += __shfl_xor(v, 4, kWave);
      v += __shfl_xor(v, 2, kWave);
      v += __shfl_xor(v, 1, kWave);
      if (kc == 0) a.sumsq[(unit * S + sp) * kMTile + mrow + 16 * i] = v;
    }
  }
  if (S > 1) {
    float* pt = a.part + (unit * S + sp) * kTileFloats + col;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = 8 * (r >> 2) + rbase + (r & 3);
      pt[m * kWgRows] = acc0[r];
      pt[(m + 32) * kWgRows] = acc1[r];
    }
  }
  if (S > 1 || PRO == PRO_GAIN) {
    __threadfence();                        // release: partial tile and row sums are visible ...
    __syncthreads();
    if (tid == 0) {
      int last = 1;
      if (S > 1) {
        const int old = atomicAdd(a.counters + unit, 1);   // ... before the arrival is counted
        last = old == S - 1;
        if (last) a.counters[unit] = 0;     // left clean for the next launch
      }
      s_last = last;
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();                        // acquire: see the other slices' results
  }
  if (S > 1) {                              // fixed slice order, own slice from registers
    f32x16_t t0 = {}, t1 = {};
    for (int s2 = 0; s2 < S; ++s2) {
      if (s2 == sp) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          t0[r] += acc0[r];
          t1[r] += acc1[r];
        }
      } else {
        const float* pt = a.part + (unit * S + s2) * kTileFloats + col;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = 8 * (r >> 2) + rbase + (r & 3);
          t0[r] += pt[m * kWgRows];
          t1[r] += pt[(m + 32) * kWgRows];
        }
      }
    }
    acc0 = t0;
    acc1 = t1;
  }
  if (PRO == PRO_GAIN) {
    if (tid < kMTile) {
      float t = 0.f;
      for (int s2 = 0; s2 < S; ++s2) t += a.sumsq[(unit * S + s2) * kMTile + tid];
      s_rstd[tid] = 1.0f / sqrtf(t / (float)K + a.eps);
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = 8 * (r >> 2) + rbase + (r & 3);
      acc0[r] *= s_rstd[m];
      acc1[r] *= s_rstd[m + 32];
    }
  }

  if (EPI == EPI_RESID) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + 8 * (r >> 2) + rbase + (r & 3);
      if (m < a.M) a.x_io[(size_t)m * a.N + g * kWgRows + col] += acc0[r];
      if (m + 32 < a.M) a.x_io[(size_t)(m + 32) * a.N + g * kWgRows + col] += acc1[r];
    }
    return;
  }

  // The other epilogues pair columns held by different waves: go through LDS (the staging
  // buffers are free now; every wave passed the last barrier of the main loop).
  float* tile = reinterpret_cast<float*>(lds);            // [64][129]
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int m = 8 * (r >> 2) + rbase + (r & 3);
    tile[m * 129 + col] = acc0[r];
    tile[(m + 32) * 129 + col] = acc1[r];
  }
  __syncthreads();
  const int j = tid & 63;

  if (EPI == EPI_SWIGLU) {
    const int F = a.N / 2;
#pragma unroll 4
    for (int i = 0; i < 16; ++i) {
      const int ml = (tid >> 6) + 4 * i, m = m0 + ml;
      if (m >= a.M) continue;
      const float gt = tile[ml * 129 + j], up = tile[ml * 129 + 64 + j];
      a.act[(size_t)m * F + g * 64 + j] = gt / (1.0f + expf(-gt)) * up;
    }
    return;
  }

  if (EPI == EPI_QKV) {
    const int D = a.nh * 128;
    const int which = (g * kWgRows) / D;                  // 0 q, 1 k, 2 v
    const int head = ((g * kWgRows) % D) / 128;
    const float inv_freq = exp2f(-(float)j * (1.0f / 64.0f) * log2f(a.theta));
#pragma unroll 2
    for (int i = 0; i < 16; ++i) {
      const int ml = (tid >> 6) + 4 * i, m = m0 + ml;
      if (m >= a.M) continue;
      const int b = m / a.T, t = m - b * a.T;
      int P = a.prefix_len[b];
      P = P < 0 ? 0 : (P > a.p_max ? a.p_max : P);
      const float v0 = tile[ml * 129 + j], v1 = tile[ml * 129 + 64 + j];
      const size_t crow = (((size_t)b * a.nh + head) * a.cap + (size_t)(P + t)) * 128;
      if (which == 2) {
        a.vc[crow + j] = f32_to_bf16(v0);
        a.vc[crow + 64 + j] = f32_to_bf16(v1);
      } else {
        float sn, cs;
        sincosf((float)(P + a.depth[m]) * inv_freq, &sn, &cs);
        const float r0 = v0 * cs - v1 * sn, r1 = v1 * cs + v0 * sn;
        if (which == 0) {
          a.q_out[(size_t)m * D + head * 128 + j] = r0;
          a.q_out[(size_t)m * D + head * 128 + 64 + j] = r1;
        } else {
          a.kc[crow + j] = f32_to_bf16(r0);
          a.kc[crow + 64 + j] = f32_to_bf16(r1);
        }
      }
    }
  }
}

}  // namespace sv
#endif
