// Weight-streaming GEMM for few activation rows (bf16 in, float32 accumulate) on the gfx950
// matrix cores, and the packer that lays weights out in the order it streams them.
//
//   Y[m][n] = sum_k X[m][k] * W[n][k],  M <= 64 rows per workgroup pass, W = [N, K].
//
// The work is memory bound: every weight byte is needed exactly once per step while the
// activations (64 x K bf16) are small and stay in cache.  So W is cut into fragments that
// are exactly one operand of v_mfma_f32_32x32x16_bf16 - 32 weight rows x 16 k-values, lane l
// holding the 8 consecutive k-values (l / 32) * 8 .. + 7 of row l % 32 - and the fragments of
// one 32-row tile are stored one after the other along K.  A wavefront then reads its tile
// as one contiguous stream, 1 KiB per load instruction, straight into operand registers.
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

// Packer: src [rows, K] bf16 row-major  ->  fragment order, placed `row_off` rows into a
// destination matrix of the same K.  One thread moves one 16-byte chunk (8 k-values).
// Chunk (n, kc) lands at uint4 index ((n/32) * (K/16) + kc/2) * 64 + (n%32) + 32 * (kc%2).
__global__ void pack_rows_mfma(const uint4* __restrict__ src, uint4* __restrict__ dst, int rows,
                               int K, int row_off) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int chunks_per_row = K / 8;
  if (i >= (size_t)rows * chunks_per_row) return;
  const int n_src = (int)(i / chunks_per_row), kc = (int)(i % chunks_per_row);
  const int n = n_src + row_off;
  const size_t frag = (size_t)(n / kFragRows) * (K / kFragK) + (kc >> 1);
  dst[frag * 64 + (n % kFragRows) + 32 * (kc & 1)] = src[i];
}

// grid = (N / 128, n_split, m_tiles), block = 256.
// Wave w of workgroup x owns weight rows (4x + w) * 32 .. + 31 and the K-slice of split y.
// Activations of the current 128-wide K block sit in LDS in fragment order (filled by all
// four waves, double buffered); weight fragments go global -> registers, one K block ahead.
// Output: Yp[split][m_tile * 64 + m][n] float32 (plane stride `plane`), every element written.
__global__ __launch_bounds__(256) void gemm_skinny_bf16(const bf16_t* __restrict__ X, int M,
                                                        const uint4* __restrict__ Wp,
                                                        float* __restrict__ Yp, size_t plane,
                                                        int N, int K) {
  __shared__ uint4 xs[2][8 * 2 * 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m0 = blockIdx.z * kMTile;
  const int nblk = K / kBlkK;
  const int S = gridDim.y, sp = blockIdx.y;
  const int q = nblk / S, rem = nblk % S;
  const int blk_begin = sp * q + min(sp, rem);
  const int nb = q + (sp < rem ? 1 : 0);
  const int ntile = blockIdx.x * 4 + wave;
  const uint4* wp = Wp + ((size_t)ntile * (K / kFragK) + (size_t)blk_begin * 8) * 64 + lane;

  f32x16_t acc0 = {}, acc1 = {};
  uint4 wreg[8], wnext[8], xreg[4];

  auto load_x = [&](int blk) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = tid + 256 * i;           // 1024 chunks: row c / 16, chunk c % 16
      const int m = m0 + (c >> 4);
      const int k = (blk_begin + blk) * kBlkK + (c & 15) * 8;
      xreg[i] = m < M ? *reinterpret_cast<const uint4*>(X + (size_t)m * K + k)
                      : make_uint4(0u, 0u, 0u, 0u);
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = tid + 256 * i;
      const int m = c >> 4, kc = c & 15;
      xs[buf][((kc >> 1) * 2 + (m >> 5)) * 64 + (m & 31) + 32 * (kc & 1)] = xreg[i];
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
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const bf16x8_t w = __builtin_bit_cast(bf16x8_t, wreg[s]);
      const bf16x8_t x0 = __builtin_bit_cast(bf16x8_t, xs[cur][(s * 2 + 0) * 64 + lane]);
      const bf16x8_t x1 = __builtin_bit_cast(bf16x8_t, xs[cur][(s * 2 + 1) * 64 + lane]);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x0, w, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1, w, acc1, 0, 0, 0);
    }
    if (more) {
      store_x(cur ^ 1);
#pragma unroll
      for (int s = 0; s < 8; ++s) wreg[s] = wnext[s];
    }
  }

  // accumulator register r of lane l holds row 8 * (r / 4) + 4 * (l / 32) + r % 4 and
  // column l % 32 of the 32 x 32 tile (rows = activations, columns = weight rows)
  float* yp = Yp + (size_t)sp * plane + (size_t)m0 * N + (size_t)ntile * 32 + (lane & 31);
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int m = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
    yp[(size_t)m * N] = acc0[r];
    yp[(size_t)(m + 32) * N] = acc1[r];
  }
}

}  // namespace sv
#endif
