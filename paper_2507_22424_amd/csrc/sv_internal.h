// Internal helpers shared by the kernels of libspecvla_verify (gfx950 only).
#ifndef SV_INTERNAL_H
#define SV_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "specvla_verify.h"

namespace sv {

constexpr int kWave = 64;           // CDNA wavefront
constexpr int kMTile = 64;          // rows of activations one GEMM workgroup covers
constexpr size_t kAlign = 256;      // alignment of every region inside packed blobs / workspace

// bfloat16 stored as its 16 bits; converted by hand so that rounding is explicit
// (round to nearest, ties to even; NaN stays NaN).
struct bf16_t {
  uint16_t bits;
};

__host__ __device__ inline float to_f32(bf16_t v) {
  union { uint32_t u; float f; } c;
  c.u = (uint32_t)v.bits << 16;
  return c.f;
}
__host__ __device__ inline float to_f32(float v) { return v; }

__host__ __device__ inline bf16_t f32_to_bf16(float f) {
  union { uint32_t u; float f; } c;
  c.f = f;
  uint32_t u = c.u;
  bf16_t r;
  if ((u & 0x7fffffffu) > 0x7f800000u) {
    r.bits = (uint16_t)((u >> 16) | 0x0040u);
  } else {
    u += 0x7fffu + ((u >> 16) & 1u);
    r.bits = (uint16_t)(u >> 16);
  }
  return r;
}

template <typename T> struct Cvt;
template <> struct Cvt<float> {
  __device__ static inline float from(float f) { return f; }
};
template <> struct Cvt<bf16_t> {
  __device__ static inline bf16_t from(float f) { return f32_to_bf16(f); }
};

__host__ __device__ inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Sum over the 64 lanes of a wavefront; every lane gets the total.
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// Sum over a workgroup of 256 threads (4 waves); every thread gets the total.
// `scratch` must hold 4 floats of LDS and may be reused after the call returns.
__device__ inline float block_sum_256(float v, float* scratch) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
  __syncthreads();
  return scratch[0] + scratch[1] + scratch[2] + scratch[3];
}

// Where the pieces of a packed layer live (bytes from the start of the blob).
struct PackedLayout {
  size_t g1, g2, wqkv, wo, wgu, wd, total;
  size_t sqkv, so, sgu, sd;      // SV_BF16_W8 / SV_BF16_W4: float32 row scales in packed row order
};

inline PackedLayout packed_layout(const sv_model_cfg& c) {
  // half bytes per matrix element: float32 8, bf16 4, E4M3 2, int4 1
  const size_t eh = c.dtype == SV_F32 ? 8 : (c.dtype == SV_BF16_W8 ? 2 : (c.dtype == SV_BF16_W4 ? 1 : 4));
  const size_t H = c.hidden, D = (size_t)c.n_heads * c.head_dim, F = c.mlp_dim;
  PackedLayout L;
  size_t o = 0;
  L.g1 = o;   o = align_up(o + H * 4, kAlign);
  L.g2 = o;   o = align_up(o + H * 4, kAlign);
  L.wqkv = o; o = align_up(o + 3 * D * H * eh / 2, kAlign);
  L.wo = o;   o = align_up(o + H * D * eh / 2, kAlign);
  L.wgu = o;  o = align_up(o + 2 * F * H * eh / 2, kAlign);
  L.wd = o;   o = align_up(o + H * F * eh / 2, kAlign);
  L.sqkv = L.so = L.sgu = L.sd = 0;
  if (c.dtype == SV_BF16_W8 || c.dtype == SV_BF16_W4) {
    L.sqkv = o; o = align_up(o + 3 * D * 4, kAlign);
    L.so = o;   o = align_up(o + H * 4, kAlign);
    L.sgu = o;  o = align_up(o + 2 * F * 4, kAlign);
    L.sd = o;   o = align_up(o + H * 4, kAlign);
  }
  L.total = o;
  return L;
}

// Device scratch of one call (bytes from the start of the workspace).  Activations are
// float32 for both storage types.
struct WorkspaceLayout {
  size_t counters, sumsq, part, xhat, q, attn, act, head_z, head_logits, total;
  size_t counter_bytes, part_bytes;
  // packed head (bf16, scored rows a multiple of 32): its own counters, row sums, partial tiles
  size_t head_cnt, head_cnt_bytes, head_sumsq, head_part, head_part_bytes;
  // many rows (matrix-core bound products): activation fragments, 1 / rms, split-K partial blocks
  size_t rows_xs, rows_rstd, rows_part;
  size_t att_part;               // split tree attention: per split, query and head the unnormalised output, maximum, sum
  int rows_pad;
  int m_pad, m_tiles;
  int ucap, tstride, head_ucap, head_tstride;   // per-XCD extents of the split-K scratch regions (units, partial tiles)
};

}  // namespace sv
#endif
