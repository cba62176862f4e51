// Tree attention of the bf16 verification layer on the gfx950 matrix cores.
//
// Node i of a draft tree attends to every prefix key and to the tree nodes on its own root
// path (its ancestor-or-self bitmask) - the keys an ordinary causal decode of that path would
// see (the paper verifies all paths of the tree in one pass, Sec. 4.1).
//
// One workgroup = one (episode, head, block of 16 query nodes); its four waves split the key
// range into 32-key tiles (flash-decoding inside the workgroup: no cross-workgroup traffic)
// and merge their partial (max, sum, output) through LDS at the end.  Everything is computed
// transposed, S^T = K Q^T and O^T = V^T P^T with v_mfma_f32_16x16x32_bf16, so that
//   * a K tile is a matrix-core operand as it sits in the cache (16 B per lane, no staging),
//   * a lane owns one query column: the online-softmax state and the rescale are per lane,
//   * the probabilities come out of the first product in exactly the register layout the
//     second one wants (the rows of the two 16-key sub-tiles are ordered so that k-slot
//     (g, e) of lane group g is key 8g + e of the tile);
//   * only V passes through LDS: stored as loaded (row = key), read back as the V^T operand
//     with the transposing LDS read of gfx950 (ds_read_b64_tr_b16) - no register shuffles.
// Queries and probabilities are split into hi + lo bf16 parts so that, with the exact bf16
// keys and values, the result carries float32-level rounding only.
#ifndef SV_ATTENTION_H
#define SV_ATTENTION_H

#include "sv_gemm_mfma.h"
#include "sv_internal.h"

namespace sv {

constexpr int kAttQ = 16;        // queries per workgroup
constexpr int kAttKeys = 32;     // keys per tile
constexpr int kAttSplitFill = 256;   // split the keys of a task while there are fewer workgroups than this
constexpr int kVtPitch = 72;     // LDS per wave = 128 * kVtPitch bytes (V tile in the loop, merge buffer after it)
// V tile in LDS: 288 bytes per key row (a row starts 8 banks after the one before), and rows
// 8..15 of every 16 hold their two 128-byte halves swapped: the 32 lanes that read together
// (keys 8g .. 8g+3 or +4 .. +7 of two lane groups, 32 bytes each) then hit 64 different banks.
constexpr int kVPitch = 288;
constexpr int kMergePitch = kAttQ + 1;   // floats per d row of the merge buffer (odd: the readers' rows fall on different banks)
static_assert(kAttKeys * kVPitch <= 128 * kVtPitch && 128 * kMergePitch * 4 <= 128 * kVtPitch,
              "V tile and merge rows must fit the wave's LDS share");
typedef short i16x4_t __attribute__((ext_vector_type(4)));
constexpr float kNegBig = -1.0e30f;

// 16-byte load from global memory (also when the compiler cannot tell where the pointer points)
__device__ inline uint4 ld_global_u4(const void* p) {
  const u32x4_t v = *(const __attribute__((address_space(1))) u32x4_t*)p;
  return make_uint4(v[0], v[1], v[2], v[3]);
}

__device__ inline bf16x8_t pack8_hi(const float* v) {
  const uint4 u = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]),
                             pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
  return __builtin_bit_cast(bf16x8_t, u);
}
__device__ inline void split8(const float* v, bf16x8_t& hi, bf16x8_t& lo) {
  uint4 h, l;
  h.x = pack_bf16x2(v[0], v[1]); h.y = pack_bf16x2(v[2], v[3]);
  h.z = pack_bf16x2(v[4], v[5]); h.w = pack_bf16x2(v[6], v[7]);
  l.x = pack_bf16x2(v[0] - bf16_lo_f32(h.x), v[1] - bf16_hi_f32(h.x));
  l.y = pack_bf16x2(v[2] - bf16_lo_f32(h.y), v[3] - bf16_hi_f32(h.y));
  l.z = pack_bf16x2(v[4] - bf16_lo_f32(h.z), v[5] - bf16_hi_f32(h.z));
  l.w = pack_bf16x2(v[6] - bf16_lo_f32(h.w), v[7] - bf16_hi_f32(h.w));
  hi = __builtin_bit_cast(bf16x8_t, h);
  lo = __builtin_bit_cast(bf16x8_t, l);
}

// Work of one workgroup of NW waves: query block bx = (episode, block of 16 nodes), head by.
// lds_raw: NW * 128 * kVtPitch bytes; s_m, s_l: [NW][16] floats; sync(): barrier of the waves
// that run this body (called twice).
// head_dim = 128.
// q: float32 [M, nh*128] (rotated);  kc, vc: bf16 [B][nh][cap][128];  out: float32 [M, nh*128].
// Long prefixes: the key tiles can be dealt to n_split workgroups (split = which of them this
// is); each then leaves, per query, its unnormalised output, running maximum and sum in
// `part` ([n_split][M][nh][kAttPartStride] floats) and attention_merge_kernel combines them in
// split order.  With n_split = 1 the result goes straight to `out`.
constexpr int kAttPartStride = 132;   // 128 outputs, maximum, sum, padding
template <int NW, typename Sync>
__device__ inline void tree_attention_body(
    const float* __restrict__ q, const bf16_t* __restrict__ kc, const bf16_t* __restrict__ vc,
    const int32_t* __restrict__ prefix_len, int p_max, const uint64_t* __restrict__ anc,
    int n_words, int T, int nh, int cap, float* __restrict__ out, int bx, int by,
    unsigned char* lds_raw, float (*s_m)[kAttQ], float (*s_l)[kAttQ], int tid, Sync sync,
    int split = 0, int n_split = 1, float* __restrict__ part = nullptr, int M_total = 0) {
  const int lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, c = lane & 15;      // lane group (0..3), column = query
  const int qblocks = (T + kAttQ - 1) / kAttQ;
  const int b = bx / qblocks, qb = bx % qblocks;
  const int h = by;
  const int D = nh * 128;
  int P = prefix_len[b];
  P = P < 0 ? 0 : (P > p_max ? p_max : P);
  const int nkeys = P + T;
  const int ntiles_all = (nkeys + kAttKeys - 1) / kAttKeys;
  // this workgroup's run of key tiles [t_first, ntiles)
  const int t_first = (int)(((long long)ntiles_all * split) / n_split);
  const int ntiles = (int)(((long long)ntiles_all * (split + 1)) / n_split);
  const int tq = min(qb * kAttQ + c, T - 1);   // this lane's query node (clamped in the tail)
  const size_t mrow = (size_t)b * T + tq;
  const bf16_t* kbase = kc + ((size_t)b * nh + h) * cap * 128;
  const bf16_t* vbase = vc + ((size_t)b * nh + h) * cap * 128;
  unsigned char* vt = lds_raw + wave * 128 * kVtPitch;

  // Q^T operand: lane = (query c, d-slice 32*ks + 8*g .. + 7), pre-scaled by 1/sqrt(128)
  bf16x8_t qh[4], ql[4];
  {
    const float scale = 0.08838834764831845f;
    const float* qp = q + mrow * D + h * 128 + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const float4 a0 = *reinterpret_cast<const float4*>(qp + 32 * ks);
      const float4 a1 = *reinterpret_cast<const float4*>(qp + 32 * ks + 4);
      const float v[8] = {a0.x * scale, a0.y * scale, a0.z * scale, a0.w * scale,
                          a1.x * scale, a1.y * scale, a1.z * scale, a1.w * scale};
      split8(v, qh[ks], ql[ks]);
    }
  }
  unsigned long long mask0 = anc[mrow * n_words], mask1 = n_words > 1 ? anc[mrow * n_words + 1] : 0ull;

  // K operand of tile t: [2 sub-tiles][4 k-steps]: lane = (key c of the sub-tile, d-slice)
  // V rows of tile t: lane loads V[key 4*i + g][8c .. 8c+7] for i = 0..7
  uint4 kreg[8], vreg[8];
  auto load_tile = [&](int t) {
    const int key0 = t * kAttKeys;
#pragma unroll
    for (int st = 0; st < 2; ++st) {
      // row c of sub-tile st is key 8 * (c / 4) + 4 * st + c % 4 of the tile: a lane then holds
      // the scores of keys 8g .. 8g+7, the order in which the second product takes them
      const int key = min(key0 + 8 * (c >> 2) + 4 * st + (c & 3), nkeys - 1);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
        kreg[st * 4 + ks] = ld_global_u4(kbase + (size_t)key * 128 + 32 * ks + 8 * g);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int key = min(key0 + 4 * i + g, nkeys - 1);
      vreg[i] = ld_global_u4(vbase + (size_t)key * 128 + 8 * c);
    }
  };

  f32x4_t o[8];
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) o[dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  float m_run = kNegBig, l_run = 0.f;

  int t = t_first + wave;
  if (t < ntiles) load_tile(t);
  for (; t < ntiles; t += NW) {
    // ---- S^T = K Q^T for the two 16-key sub-tiles ----
    f32x4_t s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const bf16x8_t k0 = __builtin_bit_cast(bf16x8_t, kreg[ks]);
      const bf16x8_t k1 = __builtin_bit_cast(bf16x8_t, kreg[4 + ks]);
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, qh[ks], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, qh[ks], s1, 0, 0, 0);
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, ql[ks], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, ql[ks], s1, 0, 0, 0);
    }
    // ---- V tile -> LDS as loaded: row = key, the lane's 8 elements of key 4i + g ----
#pragma unroll
    for (int i = 0; i < 8; ++i)
      *reinterpret_cast<uint4*>(vt + (4 * i + g) * kVPitch + ((16 * c) ^ (((4 * i + g) & 8) << 4))) = vreg[i];
    // prefetch the next tile of this wave while the rest of this one is computed
    const int tn = t + NW;
    const int key0 = t * kAttKeys;
    if (tn < ntiles) load_tile(tn);

    // ---- mask + online softmax (per lane: query column c) ----
    float p[8];
    float tile_max = kNegBig;
    if (key0 + kAttKeys <= P) {              // a tile of prefix keys only: every key is visible
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        p[e] = e < 4 ? s0[e & 3] : s1[e & 3];
        tile_max = fmaxf(tile_max, p[e]);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int kidx = key0 + 8 * g + e;
        const int tn_ = kidx - P;
        bool vis = kidx < P;
        if (tn_ >= 0 && tn_ < T) vis = ((tn_ < 64 ? mask0 >> tn_ : mask1 >> (tn_ - 64)) & 1ull) != 0;
        const float sv_ = e < 4 ? s0[e & 3] : s1[e & 3];
        p[e] = vis ? sv_ : kNegBig;
        tile_max = fmaxf(tile_max, p[e]);
      }
    }
    tile_max = fmaxf(tile_max, __shfl_xor(tile_max, 16, kWave));
    tile_max = fmaxf(tile_max, __shfl_xor(tile_max, 32, kWave));
    const float m_new = fmaxf(m_run, tile_max);
    // the running maximum moves in the first tiles and rarely afterwards: the rescaling of the
    // 32 output registers is skipped when no query of the wave needs it
    const bool rescale = __builtin_amdgcn_ballot_w64(m_new != m_run) != 0;
    const float corr = __expf(m_run - m_new);
    float psum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      p[e] = p[e] > 0.5f * kNegBig ? __expf(p[e] - m_new) : 0.f;
      psum += p[e];
    }
    psum += __shfl_xor(psum, 16, kWave);
    psum += __shfl_xor(psum, 32, kWave);
    l_run = (rescale ? l_run * corr : l_run) + psum;
    m_run = m_new;
    bf16x8_t ph, pl;
    split8(p, ph, pl);

    // ---- O^T = O^T * corr + V^T P^T ----
    // V^T operand by the LDS transpose read of gfx950: the 16 lanes of a group address 4 key
    // rows x 16 d columns (lane s: row s / 4, columns 4 * (s % 4) ..+3) and lane s receives
    // column s of the four rows.  Two reads give the lane V[keys 8g .. 8g+7][d = 16 dt + c].
    __builtin_amdgcn_s_waitcnt(0xc07f);      // lgkmcnt(0): this wave's V stores have landed
    typedef __attribute__((address_space(3))) i16x4_t* lds_v4_t;
    const unsigned char* vrow = vt + (8 * g + (c >> 2)) * kVPitch + 8 * (c & 3);
    const int half_swap = 128 * (g & 1);     // rows 8 .. 15 of each 16: halves swapped
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
      const unsigned char* vcol = vrow + 32 * dt + (dt < 4 ? half_swap : -half_swap);
      const i16x4_t va = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_t)vcol);
      const i16x4_t vb = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_t)(vcol + 4 * kVPitch));
      const uint2 va2 = __builtin_bit_cast(uint2, va), vb2 = __builtin_bit_cast(uint2, vb);
      const bf16x8_t v8 = __builtin_bit_cast(bf16x8_t, make_uint4(va2.x, va2.y, vb2.x, vb2.y));
      f32x4_t acc = o[dt];
      if (rescale) {
        acc[0] *= corr; acc[1] *= corr; acc[2] *= corr; acc[3] *= corr;
      }
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v8, ph, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v8, pl, acc, 0, 0, 0);
      o[dt] = acc;
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);      // V reads done before the next tile overwrites them
  }

  // ---- merge the waves ----
  sync();
  float* om = reinterpret_cast<float*>(lds_raw);          // [NW waves][128 d][kMergePitch] float32 (16 q used)
  if (g == 0) {
    s_m[wave][c] = m_run;
    s_l[wave][c] = l_run;
  }
#pragma unroll
  for (int dt = 0; dt < 8; ++dt)
#pragma unroll
    for (int r = 0; r < 4; ++r) om[(wave * 128 + 16 * dt + 4 * g + r) * kMergePitch + c] = o[dt][r];
  sync();
  // the first four waves finish d rows 32w .. 32w+31: lane -> (d = 32w + lane % 32, queries
  // (lane / 32) * 8 .. + 7)
  if (wave < 4) {
    const int d = 32 * wave + (lane & 31);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int qq = (lane >> 5) * 8 + i;
      float m_all = s_m[0][qq];
#pragma unroll
      for (int w = 1; w < NW; ++w) m_all = fmaxf(m_all, s_m[w][qq]);
      float num = 0.f, den = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const float sc = __expf(s_m[w][qq] - m_all);
        num += sc * om[(w * 128 + d) * kMergePitch + qq];
        den += sc * s_l[w][qq];
      }
      const int tnode = qb * kAttQ + qq;
      if (tnode < T) {
        if (n_split > 1) {
          float* dst = part + (((size_t)split * M_total + (size_t)b * T + tnode) * nh + h) * kAttPartStride;
          dst[d] = num;
          if (d == 0) {
            dst[128] = m_all;
            dst[129] = den;
          }
        } else {
          out[((size_t)b * T + tnode) * D + h * 128 + d] = num / den;
        }
      }
    }
  }
}

// grid = (B * ceil(T / 16), n_heads, n_split), block = 64 * NW (NW waves split the keys; at 340
// keys the kernel is latency bound and 8 waves measured slower than 4).
template <int NW>
__global__ __launch_bounds__(64 * NW) void tree_attention_mfma(
    const float* __restrict__ q, const bf16_t* __restrict__ kc, const bf16_t* __restrict__ vc,
    const int32_t* __restrict__ prefix_len, int p_max, const uint64_t* __restrict__ anc,
    int n_words, int T, int nh, int cap, float* __restrict__ out, float* __restrict__ part,
    int M_total) {
  // per wave: transposed V tile [128 d][32 keys] with padded rows; reused for the merge
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[NW * 128 * kVtPitch];
  __shared__ float s_m[NW][kAttQ], s_l[NW][kAttQ];
  // Workgroups are dealt to the XCDs in turn (linear index modulo 8), and each XCD has its own
  // L2: the tasks are renumbered so that an XCD gets a contiguous run of (head, query tile)
  // pairs - the query tiles of one head then read that head's K/V through one L2 instead of
  // fetching it from HBM once per XCD.
  // (the splits of one task follow each other on the same XCD)
  const unsigned ns = gridDim.z;
  const unsigned total = gridDim.x * gridDim.y * ns;
  const unsigned lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
  const unsigned item = (total & 7u) ? lin : (lin & 7u) * (total >> 3) + (lin >> 3);
  const unsigned task = item / ns, split = item - task * ns;
  const unsigned head = task / gridDim.x;
  tree_attention_body<NW>(q, kc, vc, prefix_len, p_max, anc, n_words, T, nh, cap, out,
                                 (int)(task - head * gridDim.x), (int)head, lds_raw, s_m, s_l,
                                 (int)threadIdx.x, [] { __syncthreads(); }, (int)split, (int)ns, part,
                                 M_total);
}

// out[m][h*128 + d] = sum_s e^(m_s - m) num_s[d] / sum_s e^(m_s - m) den_s, m = max_s m_s, the
// splits taken in order.  grid = (M, n_heads), block = 128 (thread = d).
__global__ __launch_bounds__(128) void attention_merge_kernel(const float* __restrict__ part, int n_split,
                                                              int M, int nh, float* __restrict__ out) {
  const int m = blockIdx.x, h = blockIdx.y, d = threadIdx.x;
  float m_all = kNegBig;
  for (int s = 0; s < n_split; ++s)
    m_all = fmaxf(m_all, part[(((size_t)s * M + m) * nh + h) * kAttPartStride + 128]);
  float num = 0.f, den = 0.f;
  for (int s = 0; s < n_split; ++s) {
    const float* p = part + (((size_t)s * M + m) * nh + h) * kAttPartStride;
    const float sc = __expf(p[128] - m_all);
    num += sc * p[d];
    den += sc * p[129];
  }
  out[(size_t)m * nh * 128 + h * 128 + d] = num / den;
}

}  // namespace sv
#endif
