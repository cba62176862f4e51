// Shape-generic kernels of the verification layer: norms, the split-K epilogues (RoPE + KV
// append, residual + norm, SwiGLU), a plain FMA GEMM for float32 models and the LM-head
// slice, the per-node argmax and the weight packers.
#ifndef SV_KERNELS_H
#define SV_KERNELS_H

#include "sv_internal.h"

namespace sv {

// ---------------------------------------------------------------------------------------
// RMSNorm of float32 rows: out[m] = x[m] / sqrt(mean(x[m]^2) + eps) * gain.
// grid = rows, block = 256.
// ---------------------------------------------------------------------------------------
template <typename TO>
__global__ __launch_bounds__(256) void rmsnorm_rows(const float* __restrict__ x,
                                                    const float* __restrict__ gain,
                                                    TO* __restrict__ out, int H, float eps) {
  __shared__ float red[4];
  const size_t row = blockIdx.x;
  const float* xr = x + row * H;
  float ss = 0.f;
  for (int i = threadIdx.x; i < H; i += 256) {
    const float v = xr[i];
    ss += v * v;
  }
  ss = block_sum_256(ss, red);
  const float rstd = 1.0f / sqrtf(ss / (float)H + eps);
  for (int i = threadIdx.x; i < H; i += 256) out[row * H + i] = Cvt<TO>::from(xr[i] * rstd * gain[i]);
}

// Same norm with the gain given in the model's storage type (final norm before the LM head).
template <typename TG, typename TO>
__global__ __launch_bounds__(256) void rmsnorm_rows_tg(const float* __restrict__ x,
                                                       const TG* __restrict__ gain,
                                                       TO* __restrict__ out, int H, float eps) {
  __shared__ float red[4];
  const size_t row = blockIdx.x;
  const float* xr = x + row * H;
  float ss = 0.f;
  for (int i = threadIdx.x; i < H; i += 256) {
    const float v = xr[i];
    ss += v * v;
  }
  ss = block_sum_256(ss, red);
  const float rstd = 1.0f / sqrtf(ss / (float)H + eps);
  for (int i = threadIdx.x; i < H; i += 256)
    out[row * H + i] = Cvt<TO>::from(xr[i] * rstd * to_f32(gain[i]));
}

// ---------------------------------------------------------------------------------------
// Plain FMA GEMM, any sizes: Y[m][n] = sum_k X[m][k] * W[n][k]   (W stored [N, K]).
// 64x64 output tile per workgroup of 16x16 threads, 4x4 outputs per thread, K in steps of 16.
// Serves float32 models (where 1e-5 parity rules out reduced-precision matrix cores) and the
// 256-row LM-head slice.  blockIdx.z cuts K into gridDim.z slices written to separate
// planes of Y (plane stride y_plane floats) that the epilogue kernels add in fixed order.
// ---------------------------------------------------------------------------------------
template <typename TX, typename TW>
__global__ __launch_bounds__(256) void gemm_nt_fma(const TX* __restrict__ X, int ldx,
                                                   const TW* __restrict__ W, int ldw,
                                                   float* __restrict__ Y, int ldy,
                                                   size_t y_plane, int M, int N, int K) {
  __shared__ float Xs[16][68];
  __shared__ float Ws[16][68];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int nz = gridDim.z, z = blockIdx.z;
  const int ksteps = ceil_div(K, 16);
  const int per = ceil_div(ksteps, nz);
  const int kbeg = z * per * 16;
  const int kend = min(K, (z + 1) * per * 16);
  float acc[4][4] = {};
  const int lrow = threadIdx.x >> 2;        // 0..63
  const int lk = (threadIdx.x & 3) * 4;     // 0,4,8,12
  for (int k0 = kbeg; k0 < kend; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k = k0 + lk + i;
      const int m = m0 + lrow, n = n0 + lrow;
      Xs[lk + i][lrow] = (m < M && k < kend) ? to_f32(X[(size_t)m * ldx + k]) : 0.f;
      Ws[lk + i][lrow] = (n < N && k < kend) ? to_f32(W[(size_t)n * ldw + k]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = Xs[k][ty * 4 + i];
        b[i] = Ws[k][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  float* Yz = Y + (size_t)z * y_plane;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n < N) Yz[(size_t)m * ldy + n] = acc[i][j];
    }
  }
}

// ---------------------------------------------------------------------------------------
// Epilogue of the fused q/k/v projection: adds the K-slices, rotates q and k (rotate-half
// pairing, angle = position * theta^(-2j/d), position = prefix_len[b] + depth[node]), writes
// q as float32 and appends k, v to the cache rows prefix_len[b] + node.
// part: [S][m_pad][3*D] float32.  grid = M rows, block = 256.
// The angle is evaluated in double so that float32 models keep 1e-5 parity at positions in
// the thousands.
// ---------------------------------------------------------------------------------------
template <typename TKV>
__global__ __launch_bounds__(256) void qkv_rope_append(
    const float* __restrict__ part, int S, size_t plane, int T, int nh, int d,
    const int32_t* __restrict__ depth, const int32_t* __restrict__ prefix_len, int p_max,
    int cap, float theta, float* __restrict__ q_out, TKV* __restrict__ kc,
    TKV* __restrict__ vc) {
  const int m = blockIdx.x;
  const int b = m / T, t = m - b * T;
  const int D = nh * d, half = d >> 1;
  int P = prefix_len[b];
  P = P < 0 ? 0 : (P > p_max ? p_max : P);
  const int pos = P + depth[m];
  const float* row = part + (size_t)m * 3 * D;
  int last_j = -1;
  float cs = 1.f, sn = 0.f;
  for (int idx = threadIdx.x; idx < nh * half; idx += 256) {
    const int h = idx / half, j = idx - h * half;
    if (j != last_j) {
      const double inv = pow((double)theta, -2.0 * (double)j / (double)d);
      double s_, c_;
      sincos((double)pos * inv, &s_, &c_);
      cs = (float)c_;
      sn = (float)s_;
      last_j = j;
    }
    const int c0 = h * d + j, c1 = c0 + half;
    float q0 = 0.f, q1 = 0.f, k0 = 0.f, k1 = 0.f, v0 = 0.f, v1 = 0.f;
    for (int s = 0; s < S; ++s) {
      const float* r = row + (size_t)s * plane;
      q0 += r[c0];
      q1 += r[c1];
      k0 += r[D + c0];
      k1 += r[D + c1];
      v0 += r[2 * D + c0];
      v1 += r[2 * D + c1];
    }
    q_out[(size_t)m * D + c0] = q0 * cs - q1 * sn;
    q_out[(size_t)m * D + c1] = q1 * cs + q0 * sn;
    const size_t crow = (((size_t)b * nh + h) * cap + (size_t)(P + t)) * d;
    kc[crow + j] = Cvt<TKV>::from(k0 * cs - k1 * sn);
    kc[crow + j + half] = Cvt<TKV>::from(k1 * cs + k0 * sn);
    vc[crow + j] = Cvt<TKV>::from(v0);
    vc[crow + j + half] = Cvt<TKV>::from(v1);
  }
}

// ---------------------------------------------------------------------------------------
// Tree attention, one wavefront per (query node, head): the node attends to every prefix
// key and to the tree nodes whose bit is set in its ancestor mask; online softmax in
// float32.  Lanes split the head dimension (d <= 128: elements lane and lane + 64).
// grid = (ceil(M / 4), nh), block = 256.
// ---------------------------------------------------------------------------------------
template <typename TKV, typename TO>
__global__ __launch_bounds__(256) void tree_attention_rowwise(
    const float* __restrict__ q, const TKV* __restrict__ kc, const TKV* __restrict__ vc,
    const int32_t* __restrict__ prefix_len, int p_max, const uint64_t* __restrict__ anc,
    int n_words, int T, int nh, int d, int cap, TO* __restrict__ out, int M) {
  const int lane = threadIdx.x & 63;
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int h = blockIdx.y;
  if (m >= M) return;                       // whole wave leaves together; no barriers below
  const int b = m / T;
  const int D = nh * d;
  int P = prefix_len[b];
  P = P < 0 ? 0 : (P > p_max ? p_max : P);
  const bool has0 = lane < d, has1 = lane + 64 < d;
  const float scale = 1.0f / sqrtf((float)d);
  const float q0 = has0 ? q[(size_t)m * D + h * d + lane] * scale : 0.f;
  const float q1 = has1 ? q[(size_t)m * D + h * d + lane + 64] * scale : 0.f;
  const TKV* kb = kc + ((size_t)b * nh + h) * cap * d;
  const TKV* vb = vc + ((size_t)b * nh + h) * cap * d;
  float mx = -INFINITY, l = 0.f, a0 = 0.f, a1 = 0.f;

  auto visit = [&](int key_row) {
    const TKV* kr = kb + (size_t)key_row * d;
    const TKV* vr = vb + (size_t)key_row * d;
    float s = (has0 ? q0 * to_f32(kr[lane]) : 0.f) + (has1 ? q1 * to_f32(kr[lane + 64]) : 0.f);
    s = wave_sum(s);
    const float mn = fmaxf(mx, s);
    const float corr = expf(mx - mn);       // exp(-inf) = 0 on the first key
    const float p = expf(s - mn);
    l = l * corr + p;
    a0 = a0 * corr + (has0 ? p * to_f32(vr[lane]) : 0.f);
    a1 = a1 * corr + (has1 ? p * to_f32(vr[lane + 64]) : 0.f);
    mx = mn;
  };

  for (int j = 0; j < P; ++j) visit(j);
  for (int w = 0; w < n_words; ++w) {
    uint64_t bits = anc[(size_t)m * n_words + w];
    const int valid = T - w * 64;             // bits at or above T name no node: ignore them
    if (valid < 64) bits &= valid > 0 ? ((1ull << valid) - 1ull) : 0ull;
    while (bits) {
      const int j = __ffsll((unsigned long long)bits) - 1;
      bits &= bits - 1;
      visit(P + w * 64 + j);
    }
  }
  const float inv = 1.0f / l;
  if (has0) out[(size_t)m * D + h * d + lane] = Cvt<TO>::from(a0 * inv);
  if (has1) out[(size_t)m * D + h * d + lane + 64] = Cvt<TO>::from(a1 * inv);
}

// ---------------------------------------------------------------------------------------
// Epilogue of the output / down projections: x[m] += sum of the K-slices (fixed order), and,
// when `gain` is given, the RMSNorm of the updated row for the GEMM that follows.
// part: [S][m_pad][H].  grid = M rows, block = 256.
// ---------------------------------------------------------------------------------------
template <typename TO>
__global__ __launch_bounds__(256) void residual_rmsnorm(const float* __restrict__ part, int S,
                                                        size_t plane, float* __restrict__ x,
                                                        const float* __restrict__ gain,
                                                        TO* __restrict__ xhat, int H, float eps) {
  __shared__ float red[4];
  const size_t row = blockIdx.x;
  float* xr = x + row * H;
  float ss = 0.f;
  for (int i = threadIdx.x; i < H; i += 256) {
    float v = xr[i];
    for (int s = 0; s < S; ++s) v += part[(size_t)s * plane + row * H + i];
    xr[i] = v;
    ss += v * v;
  }
  if (gain == nullptr) return;
  ss = block_sum_256(ss, red);
  const float rstd = 1.0f / sqrtf(ss / (float)H + eps);
  for (int i = threadIdx.x; i < H; i += 256)
    xhat[row * H + i] = Cvt<TO>::from(xr[i] * rstd * gain[i]);   // own writes, same thread
}

// ---------------------------------------------------------------------------------------
// Epilogue of the fused gate/up projection: act = silu(gate) * up with
// gate = columns [0, F), up = columns [F, 2F) of part [S][m_pad][2F].
// grid = (ceil(F / 256), M), block = 256.
// ---------------------------------------------------------------------------------------
template <typename TO>
__global__ __launch_bounds__(256) void swiglu_rows(const float* __restrict__ part, int S,
                                                   size_t plane, TO* __restrict__ act, int F) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  const size_t m = blockIdx.y;
  if (n >= F) return;
  float g = 0.f, u = 0.f;
  for (int s = 0; s < S; ++s) {
    const float* r = part + (size_t)s * plane + m * 2 * F;
    g += r[n];
    u += r[F + n];
  }
  act[m * F + n] = Cvt<TO>::from(g / (1.0f + expf(-g)) * u);
}

// ---------------------------------------------------------------------------------------
// Greedy choice per row: index of the largest logit, the lowest index on exact ties
// (NaN never wins).  The logits arrive as `planes` K-slices of the head GEMM, [planes][rows][n]
// with plane stride `plane`; they are added in plane order, the sums are written to
// `logits_out` ([rows][n], may be NULL) and scanned.  One wavefront per row.
// grid = rows, block = 64.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void argmax_rows(const float* __restrict__ parts, int planes,
                                                  size_t plane, float* __restrict__ logits_out,
                                                  int n, int token_lo, int32_t* __restrict__ out) {
  const size_t row = blockIdx.x;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int i = threadIdx.x; i < n; i += 64) {
    float v = 0.f;
    for (int p0 = 0; p0 < planes; p0 += 16) {          // 16 plane loads in flight, added in order
      float pv[16];
#pragma unroll
      for (int p = 0; p < 16; ++p)
        pv[p] = p0 + p < planes ? parts[(size_t)(p0 + p) * plane + row * n + i] : 0.f;
#pragma unroll
      for (int p = 0; p < 16; ++p) v += p0 + p < planes ? pv[p] : 0.f;
    }
    if (logits_out) logits_out[row * n + i] = v;
    if (v > best || (v == best && i < bi)) {
      best = v;
      bi = i;
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float ov = __shfl_xor(best, off, kWave);
    const int oi = __shfl_xor(bi, off, kWave);
    if (ov > best || (ov == best && oi < bi)) {
      best = ov;
      bi = oi;
    }
  }
  if (threadIdx.x == 0) out[row] = token_lo + (bi == 0x7fffffff ? 0 : bi);
}

// The same decision over finished logits (one plane, e.g. of the streaming head): 256 threads
// per row, four loads in flight per thread; the lowest index wins exact ties.
__global__ __launch_bounds__(256) void argmax_rows_wide(const float* __restrict__ logits,
                                                        float* __restrict__ logits_out, int n,
                                                        int token_lo, int32_t* __restrict__ out) {
  __shared__ float s_best[4];
  __shared__ int s_bi[4];
  const size_t row = blockIdx.x;
  const float* src = logits + row * n;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int i0 = threadIdx.x; i0 < n; i0 += 4 * 256) {
    float v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = i0 + 256 * u < n ? src[i0 + 256 * u] : -INFINITY;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + 256 * u;
      if (i >= n) continue;
      if (logits_out) logits_out[row * n + i] = v[u];
      if (v[u] > best || (v[u] == best && i < bi)) {
        best = v[u];
        bi = i;
      }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float ov = __shfl_xor(best, off, kWave);
    const int oi = __shfl_xor(bi, off, kWave);
    if (ov > best || (ov == best && oi < bi)) {
      best = ov;
      bi = oi;
    }
  }
  if ((threadIdx.x & 63) == 0) {
    s_best[threadIdx.x >> 6] = best;
    s_bi[threadIdx.x >> 6] = bi;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w)
      if (s_best[w] > best || (s_best[w] == best && s_bi[w] < bi)) {
        best = s_best[w];
        bi = s_bi[w];
      }
    out[row] = token_lo + (bi == 0x7fffffff ? 0 : bi);
  }
}

// ---------------------------------------------------------------------------------------
// Measurement aid: reads a buffer once the way the GEMM streams weights (non-temporal 16-byte
// loads, 1 KiB per wave and instruction, 8 KiB per wave in flight) and discards the data.
// grid = any, block = 256.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4_t* __restrict__ p, size_t n_vec,
                                                          u32x4_t* __restrict__ sink) {
  typedef const __attribute__((address_space(1))) u32x4_t* gptr_t;
  const gptr_t g = (gptr_t)p;
  const size_t lane = threadIdx.x & 63;
  const size_t n_waves = (size_t)gridDim.x * 4;
  u32x4_t acc = {0u, 0u, 0u, 0u};
  for (size_t blk = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6); blk * 512 < n_vec; blk += n_waves) {
    u32x4_t v[8];
#pragma unroll
    for (int f = 0; f < 8; ++f) {
      const size_t i = blk * 512 + f * 64 + lane;
      v[f] = __builtin_nontemporal_load(g + (i < n_vec ? i : n_vec - 1));
    }
#pragma unroll
    for (int f = 0; f < 8; ++f) acc ^= v[f];
  }
  if (acc[0] == 0x9e3779b9u && acc[1] == 0x7f4a7c15u && acc[2] == 0xf39cc060u) *sink = acc;   // keeps the loads
}

// ---------------------------------------------------------------------------------------
// Packers (load time).  pack_gain widens a gain vector to float32; pack_rows_plain copies
// a [rows, K] matrix behind `row_off` rows of the destination.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ void pack_gain(const T* __restrict__ src, float* __restrict__ dst, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = to_f32(src[i]);
}

template <typename T>
__global__ void pack_rows_plain(const T* __restrict__ src, T* __restrict__ dst, size_t n_elems,
                                size_t dst_off) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_elems) dst[dst_off + i] = src[i];
}

}  // namespace sv
#endif
