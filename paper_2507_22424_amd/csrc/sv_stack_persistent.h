// The bf16 verification pass of a stack of layers as ONE persistent launch (up to 64 activation
// rows: one draft tree, or a few small ones).
//
// Why: with one launch per projection every phase of a layer pays launch ramp, activation
// staging, the wait for the slowest workgroup and the split-K reduction with the HBM pipe idle,
// and those fixed costs are as large as the streaming itself.  The weights do not depend on the
// activations, so here the weight stream never stops: one workgroup per CU stays resident for
// the whole stack and is split into two roles,
//   * waves 0-3 ("stream"): nothing but a ring of weight loads (kRingSlots x 8 KiB per wave,
//     issued unconditionally in a fixed rotation so that the wait counts are exact), the MFMAs
//     on the piece that has arrived, and the hand-over of finished tiles through LDS.  They issue
//     no other vector-memory instruction: loads return in order per wave, so anything queued
//     behind the ring would wait for the whole ring.  While a phase boundary is being worked
//     on, the ring keeps filling with the next phase's weights;
//   * waves 4-7 ("helper"): everything else - staging the activations of the next phase into
//     LDS (hi + lo bf16 split, RMSNorm gain and row sums), writing partial tiles, the group
//     barrier, the split-K reduction with its epilogue (RoPE + KV append, residual, SwiGLU),
//     tree attention, and the device-wide barrier between phases.
// The two roles meet only at workgroup barriers; both derive the barrier sequence from the
// same geometry (phase_geom), and a phase a workgroup has no work in has no barriers.
//
// Memory ordering.  The L2 caches of the eight XCDs are not coherent with each other inside a
// launch.  (a) Partial tiles, row sums and everything else that is produced and consumed by the
// slices of one tile group stay on one XCD, at addresses that only this XCD ever touches during
// the launch (per-XCD regions), ordered by the group's arrival counter as in gemm_stream_bf16.
// (b) Activations that cross XCDs (x, q, K/V rows of the tree, attention output, MLP
// activations) are written with device-scope (write-through) stores, each wave waits for its
// stores, the workgroups meet at a device-wide barrier built from device-scope atomics, and
// readers start with a device-scope acquire (invalidates stale lines).  All waits are bounded;
// a wait that runs out raises the sticky status word and later waits are skipped.
#ifndef SV_STACK_PERSISTENT_H
#define SV_STACK_PERSISTENT_H

#include "sv_attention.h"
#include "sv_gemm_mfma.h"
#include "sv_internal.h"

namespace sv {

constexpr int kStackCntStride = 16;  // 64-bit words between the arrival words of two groups (128 bytes)
constexpr int kStackMaxLayers = 32;   // layers per launch (pointer table in the kernel arguments)
constexpr int kRingSlots = 4;         // weight pieces in flight per stream wave
constexpr int kRingFrags = 8;         // fragments per piece: 128 k-values, 8 KiB per wave
constexpr int kUnitsPerXcd = 32;      // workgroups per XCD (one per CU)
constexpr int kSpinLimit = 1 << 16;
constexpr int kTsPerLayer = 16;       // timeline slots per (workgroup, layer)

struct PhasePlan {
  int N, K, S, gpx;
};

struct StackLayer {
  const unsigned char* packed;
  bf16_t* kc;
  bf16_t* vc;
};

// Launch description.  It lives in device memory (written by write_stack_args before the
// persistent launch) so that the kernel can index it freely.
struct StackArgs {
  StackLayer L[kStackMaxLayers];
  int n_layers;
  unsigned off_g1, off_g2;                 // byte offsets inside a packed layer
  size_t off_wqkv, off_wo, off_wgu, off_wd;
  PhasePlan plan[4];                       // qkv, o, gate/up, down
  int M, T, nh, n_xcd;
  float eps, theta;
  size_t part_xcd_tiles;                   // partial tiles (tile x slice) per XCD region
  int gmax;                                // row length of group_cnt
  int n_words, p_max, cap;
};

// Device buffers of a launch.  They are passed as separate kernel arguments (pointer arguments
// are known to be global memory; pointers read from memory are not).
struct StackBufs {
  float* x_io;                             // [M, H] residual stream, in/out
  float* q;                                // [M, nh*128]
  float* attn;                             // [M, nh*128]
  float* act;                              // [M, F]
  uint4* part16;                           // [n_xcd][part_xcd_tiles] partial tiles (kTileVec4 uint4 each)
  float* pscale;                           // [n_xcd][part_xcd_tiles] their inverse scales
  float* sumsq;                            // [n_xcd][32][64] row sums of x^2 per unit
  unsigned long long* group_cnt;           // [n_layers * 4][gmax] arrival words, kStackCntStride apart, zero at launch
  unsigned* grid_cnt;                      // [n_xcd] words 64 apart, zero at launch
  unsigned* wg_cnt;                        // [grid] words 32 apart (a line each), zero at launch
  unsigned* wg_flag;                       // [grid] words 32 apart, zero at launch
  int* status;
  const int32_t* depth;
  const int32_t* prefix_len;
  const uint64_t* anc;
  long long* ts;                           // optional [grid][n_layers][kTsPerLayer] clock samples
};

// Work of one workgroup (XCD xcd, unit u of that XCD) in one GEMM phase.
struct PhaseGeom {
  int g, gl, sp;                 // tile group, its index inside the XCD, K slice
  int t_begin, t_count, t_max;   // tiles of the group; t_max = most tiles any group has
  int p_begin, np;               // pieces (128 k-values) of the slice
  int rounds, n_chunks;          // tiles per wave (rounded up); LDS chunks (4 pieces) per slice
  bool active;
};

__host__ __device__ inline PhaseGeom phase_geom(const PhasePlan& p, int n_xcd, int xcd, int u) {
  PhaseGeom r;
  const int n_tiles = p.N / kFragRows, G = n_xcd * p.gpx, npieces = p.K / kBlkK;
  r.gl = u / p.S;
  r.sp = u % p.S;
  r.g = xcd * p.gpx + r.gl;
  const int tq = n_tiles / G, trem = n_tiles % G;
  r.t_max = tq + (trem ? 1 : 0);
  r.t_begin = r.g * tq + (r.g < trem ? r.g : trem);
  r.t_count = tq + (r.g < trem ? 1 : 0);
  const int pq = npieces / p.S, prem = npieces % p.S;
  r.p_begin = r.sp * pq + (r.sp < prem ? r.sp : prem);
  r.np = pq + (r.sp < prem ? 1 : 0);
  r.active = u < p.gpx * p.S && r.t_count > 0 && r.np > 0;
  if (!r.active) {
    r.t_count = 0;
    r.np = 0;
  }
  r.rounds = (r.t_count + 3) / 4;
  r.n_chunks = (r.np + 3) / 4;
  return r;
}

// Pointers read from the launch description in memory are generic to the compiler; telling it
// that they are neither LDS nor scratch lets it use global (not flat) instructions, which do
// not tie the vector-memory and LDS wait counters together.
template <typename T>
__device__ inline T* as_global(T* p) {
  return (T*)(__attribute__((address_space(1))) T*)p;
}

__device__ inline PhasePlan phase_plan(const StackArgs& a, int ph) { return a.plan[ph]; }

__device__ inline const uint4* phase_weights(const StackArgs& a, int layer, int ph) {
  const unsigned char* base = as_global(a.L[layer].packed);
  const size_t off = ph == 0 ? a.off_wqkv : ph == 1 ? a.off_wo : ph == 2 ? a.off_wgu : a.off_wd;
  return reinterpret_cast<const uint4*>(base + off);
}

// Barrier of all eight waves; LDS traffic of this wave is complete, vector-memory loads in
// flight are not waited for.
__device__ inline void wg_bar() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Attention work items are dealt round robin to the workgroups; every wave of every workgroup
// passes two barriers per pass.
__device__ inline int attention_passes(const StackArgs& a) {
  const int tasks = (a.M / a.T) * ((a.T + kAttQ - 1) / kAttQ) * a.nh;
  return (tasks + (int)gridDim.x - 1) / (int)gridDim.x;
}

// Walks the weight pieces of one stream wave in consumption order: layers, phases, rounds
// (tile wave + 4*round of the group), pieces of the slice.  Rounds in which this wave has no
// tile are walked as well (nothing is loaded or multiplied, the barriers still happen).
struct PieceCursor {
  int layer, ph, r, j;
  int np, rounds, my_tiles;
  bool multi, done;
  const uint4* wbase;
  size_t tile_stride4;

  __device__ inline bool load_phase(const StackArgs& a, int xcd, int u, int wave) {
    const PhasePlan p = phase_plan(a, ph);
    const PhaseGeom gm = phase_geom(p, a.n_xcd, xcd, u);
    np = gm.np;
    rounds = gm.rounds;
    multi = gm.n_chunks > 1;
    my_tiles = gm.t_count > wave ? (gm.t_count - wave + 3) / 4 : 0;
    const size_t tile_stride = (size_t)(p.K / kFragK) * 64;
    tile_stride4 = 4 * tile_stride;
    wbase = phase_weights(a, layer, ph) + (size_t)(gm.t_begin + wave) * tile_stride +
            (size_t)gm.p_begin * (kRingFrags * 64);
    r = 0;
    j = 0;
    return gm.active;
  }
  __device__ inline bool valid() const { return !done && r < my_tiles; }
  __device__ inline const uint4* ptr() const {
    return wbase + (size_t)r * tile_stride4 + (size_t)j * (kRingFrags * 64);
  }
  // Moves to the first phase at or after (layer, ph) in which this workgroup has work.
  // `between(ph)` runs once for every phase that is left behind (active or not).
  template <typename F>
  __device__ inline void seek(const StackArgs& a, int xcd, int u, int wave, F between) {
    while (layer < a.n_layers) {
      if (load_phase(a, xcd, u, wave)) return;
      between(ph);
      if (++ph == 4) {
        ph = 0;
        ++layer;
      }
    }
    done = true;
  }
  template <typename F>
  __device__ inline void advance(const StackArgs& a, int xcd, int u, int wave, F between) {
    if (done) return;
    if (++j < np) return;
    j = 0;
    if (++r < rounds) return;
    between(ph);
    if (++ph == 4) {
      ph = 0;
      ++layer;
    }
    seek(a, xcd, u, wave, between);
  }
};

// ---- stream role -------------------------------------------------------------------------------

__device__ inline void stream_role(const StackArgs& a, const uint4* xs, float4* tb, int wave, int lane,
                                   int xcd, int u) {
  const int att_bars = 2 * attention_passes(a);
  auto none = [](int) {};
  auto leave_phase = [&](int ph) {           // barriers of the attention stage, after the qkv phase
    if (ph == 0)
      for (int i = 0; i < att_bars; ++i) wg_bar();
  };
  PieceCursor ci, cc;                        // issue runs kRingSlots pieces ahead of consume
  ci.layer = ci.ph = 0; ci.done = false;
  cc.layer = cc.ph = 0; cc.done = false;
  ci.seek(a, xcd, u, wave, none);
  cc.seek(a, xcd, u, wave, leave_phase);

  // every step issues exactly kRingFrags loads (a harmless, cache-resident address when there is
  // nothing left to fetch), so the compiler's wait counts for slot s are exact
  const uint4* const idle_src = phase_weights(a, 0, 0);
  u32x4_t ring[kRingSlots][kRingFrags];
  auto issue = [&](u32x4_t* b) {
    const uint4* p = ci.valid() ? ci.ptr() : idle_src;
#pragma unroll
    for (int f = 0; f < kRingFrags; ++f)
      b[f] = __builtin_nontemporal_load((const __attribute__((address_space(1))) u32x4_t*)p + ((unsigned)lane + f * 64u));
    ci.advance(a, xcd, u, wave, none);
  };
#pragma unroll
  for (int s = 0; s < kRingSlots; ++s) issue(ring[s]);

  f32x16_t acc0 = {}, acc1 = {};
  float4* my_tb = tb + wave * (kTileFloats / 4);
  auto step = [&](u32x4_t* b) {
    if (!cc.done) {
      const int jq = cc.j & 3;
      if (jq == 0 && (cc.multi || cc.r == 0)) wg_bar();              // X chunk is staged
      if (cc.r < cc.my_tiles) {
        const uint4* xf = xs + (size_t)(jq * kRingFrags * 4) * 64;
#pragma unroll
        for (int f = 0; f < kRingFrags; ++f) {
          const uint4* xp = xf + (size_t)(f * 4) * 64 + frag_slot(lane, f);
          const bf16x8_t w = __builtin_bit_cast(bf16x8_t, b[f]);
          const bf16x8_t x0h = __builtin_bit_cast(bf16x8_t, xp[0]);
          const bf16x8_t x0l = __builtin_bit_cast(bf16x8_t, xp[64]);
          const bf16x8_t x1h = __builtin_bit_cast(bf16x8_t, xp[128]);
          const bf16x8_t x1l = __builtin_bit_cast(bf16x8_t, xp[192]);
          acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x0h, w, acc0, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1h, w, acc1, 0, 0, 0);
          acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x0l, w, acc0, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1l, w, acc1, 0, 0, 0);
        }
      }
      if (cc.j == cc.np - 1) {
        // tile finished: hand it to helper wave `wave` in register order [8 quads][64 lanes][4]
        if (cc.r > 0) wg_bar();                                      // helpers have read the previous tile
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
          my_tb[qd * 64 + lane] = make_float4(acc0[4 * qd], acc0[4 * qd + 1], acc0[4 * qd + 2], acc0[4 * qd + 3]);
          my_tb[(qd + 4) * 64 + lane] = make_float4(acc1[4 * qd], acc1[4 * qd + 1], acc1[4 * qd + 2], acc1[4 * qd + 3]);
        }
        wg_bar();                                                    // tile is in LDS
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          acc0[r] = 0.f;
          acc1[r] = 0.f;
        }
      } else if (cc.multi && jq == 3) {
        wg_bar();                                                    // chunk consumed, may be overwritten
      }
      cc.advance(a, xcd, u, wave, leave_phase);
    }
    issue(b);
  };
  while (!cc.done) {
#pragma unroll
    for (int s = 0; s < kRingSlots; ++s) step(ring[s]);
  }
}

// ---- helper role -------------------------------------------------------------------------------

struct SyncCtx {
  unsigned* wg_cnt;
  unsigned* wg_flag;
  unsigned* grid_cnt;
  int* status;
  int n_xcd, xcd;
  unsigned seq;
  bool dead;
};

// device-scope (write-through) stores to global memory
__device__ inline void st_dev(float* p, float v) {
  __hip_atomic_store((__attribute__((address_space(1))) float*)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_dev(unsigned* p, unsigned v) {
  __hip_atomic_store((__attribute__((address_space(1))) unsigned*)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float4 ld_global_f4(const float* p) {
  const f32x4_t v = *(const __attribute__((address_space(1))) f32x4_t*)p;
  return make_float4(v[0], v[1], v[2], v[3]);
}

// Device-wide barrier of the helper waves.  Every helper wave has waited for its own stores;
// the last of the four to get here arrives for the workgroup at its XCD's counter; helper wave
// 0 watches the counters and passes the news on through the workgroup's flag word.
__device__ inline void grid_sync(SyncCtx& s, int hw, int lane) {
  __builtin_amdgcn_s_waitcnt(0);
  ++s.seq;
  if (lane == 0) {
    const unsigned old = __hip_atomic_fetch_add(s.wg_cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((old & 3u) == 3u)
      __hip_atomic_fetch_add(s.grid_cnt + 64 * s.xcd, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (!s.dead) {
    bool ok = false;
    if (hw == 0) {
      const unsigned target = (unsigned)kUnitsPerXcd * s.seq;
      for (int spin = 0; spin < kSpinLimit && !ok; ++spin) {
        const unsigned v = lane < s.n_xcd ? __hip_atomic_load(s.grid_cnt + 64 * lane, __ATOMIC_RELAXED,
                                                              __HIP_MEMORY_SCOPE_AGENT)
                                          : target;
        ok = __all(v >= target);
        if (!ok) __builtin_amdgcn_s_sleep(8);   // device-scope polls are round trips to the memory side: keep them few
      }
      if (lane == 0) {
        if (!ok) atomicOr(s.status, 4);
        __hip_atomic_store(s.wg_flag, ok ? s.seq : 0x80000000u, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_WORKGROUP);
      }
    } else {
      for (int spin = 0; spin < kSpinLimit && !ok; ++spin) {
        const unsigned v = __hip_atomic_load(s.wg_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (v & 0x80000000u) break;
        ok = v >= s.seq;
        if (!ok) __builtin_amdgcn_s_sleep(2);
      }
    }
    if (!ok) s.dead = true;
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

__device__ inline void stamp(const StackArgs& a, const StackBufs& d, int layer, int hw, int lane, int slot) {
  if (d.ts && hw == 0 && lane == 0)
    d.ts[((size_t)blockIdx.x * a.n_layers + layer) * kTsPerLayer + slot] = wall_clock64();
}

// One GEMM phase as the helper waves see it.  X: activations of this phase [M, K].
template <int PRO, int EPI>
__device__ inline void helper_gemm_phase(const StackArgs& a, const StackBufs& d, int layer, int ph,
                                         const PhaseGeom& gm,
                                         const float* __restrict__ X, const float* __restrict__ gain,
                                         uint4* xs, const float4* tb, int hw, int lane, int xcd, int u,
                                         SyncCtx& sc) {
  const PhasePlan p = phase_plan(a, ph);
  const int K = p.K, S = p.S, N = p.N, M = a.M;
  const int np = gm.np;

  float ssq[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) ssq[r] = 0.f;

  // Stage chunk c (up to 4 pieces = 512 k-values) of this slice: helper wave w converts rows
  // w, w+4, ..; lane = 8-wide k chunk.
  auto stage = [&](int c) {
    const int nkc = min(4, np - 4 * c) * 16;
    const bool on = lane < nkc;
    const int k = (gm.p_begin + 4 * c) * kBlkK + (on ? lane : 0) * 8;
    float4 g0 = make_float4(1.f, 1.f, 1.f, 1.f), g1 = g0;
    if (PRO == PRO_GAIN) {
      g0 = ld_global_f4(gain + k);
      g1 = ld_global_f4(gain + k + 4);
    }
    const int s = lane >> 1;
    float4 xa[16], xb[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = hw + 4 * r;
      const float* src = X + (size_t)min(m, M - 1) * K + k;
      xa[r] = *reinterpret_cast<const float4*>(src);
      xb[r] = *reinterpret_cast<const float4*>(src + 4);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int ml = hw + 4 * r;
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
  // Row sums of x^2 over this K slice (16 per lane -> one per row with a halving butterfly;
  // lane l ends with the total of row index (l >> 2) & 15 of this wave's rows).
  float* my_ssq = d.sumsq + ((size_t)xcd * kUnitsPerXcd + u) * kMTile;
  auto publish_ssq = [&]() {
    const float v1 = row_sums_butterfly(ssq, lane);
    const int r = ((lane >> 5) & 1) * 8 + ((lane >> 4) & 1) * 4 + ((lane >> 3) & 1) * 2 + ((lane >> 2) & 1);
    if ((lane & 3) == 0) my_ssq[hw + 4 * r] = v1;
    __builtin_amdgcn_s_waitcnt(0);     // in L2 before the barrier behind which flush_tile reads all rows
  };

  // partial tile of (local tile tl, slice s) of this group, stored as in gemm_stream_bf16
  // (scaled int16 pairs + one inverse scale); the regions belong to this XCD
  uint4* part_x = d.part16 + (size_t)xcd * a.part_xcd_tiles * kTileVec4;
  float* pscale_x = d.pscale + (size_t)xcd * a.part_xcd_tiles;
  auto part_index = [&](int tl, int s) { return ((size_t)gm.gl * gm.t_max + tl) * S + s; };
  // takes stream wave hw's finished tile out of LDS and writes it as this slice's partial tile
  auto flush_tile = [&](int r) {
    const int tl = hw + 4 * r;
    float4 t[8];                                       // t[qd] = registers 4qd .. 4qd+3 of the tile
#pragma unroll
    for (int qd = 0; qd < 8; ++qd) t[qd] = tb[hw * (kTileFloats / 4) + qd * 64 + lane];
    if (PRO == PRO_GAIN) {
#pragma unroll
      for (int qd = 0; qd < 8; ++qd) {                 // rows brought to a common size, as in gemm_stream_bf16
        const float4 sq = *reinterpret_cast<const float4*>(my_ssq + 8 * (qd & 3) + 4 * (lane >> 5) + 32 * (qd >> 2));
        t[qd].x *= row_scale(sq.x); t[qd].y *= row_scale(sq.y);
        t[qd].z *= row_scale(sq.z); t[qd].w *= row_scale(sq.w);
      }
    }
    unsigned tmax = 0u;
#pragma unroll
    for (int qd = 0; qd < 8; ++qd) {
      const unsigned ma = mag_bits(t[qd].x), mb = mag_bits(t[qd].y), mc = mag_bits(t[qd].z), md = mag_bits(t[qd].w);
      const unsigned m1 = ma > mb ? ma : mb, m2 = mc > md ? mc : md, m3 = m1 > m2 ? m1 : m2;
      tmax = tmax > m3 ? tmax : m3;
    }
    unsigned wmax = wave_max_u32(tmax);
    const bool clean = wmax < kInfBits;
    if (!clean) {                                      // rare: the maximum of the finite elements
      tmax = 0u;
#pragma unroll
      for (int qd = 0; qd < 8; ++qd) {
        const unsigned ma = finite_mag_bits(t[qd].x), mb = finite_mag_bits(t[qd].y);
        const unsigned mc = finite_mag_bits(t[qd].z), md = finite_mag_bits(t[qd].w);
        const unsigned m1 = ma > mb ? ma : mb, m2 = mc > md ? mc : md, m3 = m1 > m2 ? m1 : m2;
        tmax = tmax > m3 ? tmax : m3;
      }
      wmax = wave_max_u32(tmax);
    }
    float psc, pinv;
    partial_tile_scale(wmax, psc, pinv);
    if (!clean) pinv = -pinv;
    if (tl < gm.t_count) {
      const size_t idx = part_index(tl, gm.sp);
      uint4* dst = part_x + idx * kTileVec4 + lane;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 lo = t[2 * q], hi = t[2 * q + 1];
        if (clean)
          dst[q * 64] = make_uint4(pack_q16x2(lo.x, lo.y, psc), pack_q16x2(lo.z, lo.w, psc),
                                   pack_q16x2(hi.x, hi.y, psc), pack_q16x2(hi.z, hi.w, psc));
        else
          dst[q * 64] = make_uint4(pack_q16x2_coded(lo.x, lo.y, psc), pack_q16x2_coded(lo.z, lo.w, psc),
                                   pack_q16x2_coded(hi.x, hi.y, psc), pack_q16x2_coded(hi.z, hi.w, psc));
      }
      if (lane == 0) pscale_x[idx] = pinv;
    }
  };

  stage(0);
  if (PRO == PRO_GAIN && gm.n_chunks == 1) publish_ssq();
  wg_bar();                                                          // X chunk 0 is staged
  stamp(a, d, layer, hw, lane, 3 * ph + 0);
  if (gm.n_chunks == 1) {
    for (int r = 0; r < gm.rounds; ++r) {
      wg_bar();                                                      // tiles of round r are in LDS
      flush_tile(r);
      if (r < gm.rounds - 1) wg_bar();                               // LDS tile buffers are free again
    }
  } else {
    for (int c = 1; c < gm.n_chunks; ++c) {
      wg_bar();                                                      // chunk c-1 consumed
      stage(c);
      if (PRO == PRO_GAIN && c == gm.n_chunks - 1) publish_ssq();
      wg_bar();                                                      // chunk c staged
    }
    wg_bar();
    flush_tile(0);
  }
  stamp(a, d, layer, hw, lane, 3 * ph + 1);

  // ---- group barrier: all 4*S helper waves of the group's slices have written their tiles ----
  __builtin_amdgcn_s_waitcnt(0);
  // (a 128-byte line per group: arrivals and polls of different groups must not share one)
  unsigned long long* gcnt = d.group_cnt + ((size_t)(layer * 4 + ph) * a.gmax + gm.g) * kStackCntStride;
  {
    const unsigned field = 8u * (unsigned)xcd_actual(a.n_xcd);
    if (lane == 0)
      __hip_atomic_fetch_add(gcnt, 1ull << field, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (!sc.dead) {
      unsigned long long v = 0;
      unsigned n = 0;
      for (int spin = 0; spin < kSpinLimit; ++spin) {
        v = __hip_atomic_load(gcnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        n = 0;
#pragma unroll
        for (int x = 0; x < kXcds; ++x) n += (unsigned)(v >> (8 * x)) & 255u;
        if (n >= 4u * (unsigned)S) break;
        __builtin_amdgcn_s_sleep(8);
      }
      int bad = 0;
      if (n < 4u * (unsigned)S) bad |= 2;
      else if (v != ((unsigned long long)(4 * S) << field)) bad |= 1;
      if (bad && lane == 0) atomicOr(d.status, bad);
      if (bad & 2) sc.dead = true;
    }
  }
  asm volatile("buffer_inv sc0" ::: "memory");

  // per-row values kept one per lane (lane = row), fetched with a lane read where needed
  float rstd_lane = 1.0f;
  unsigned rexp_lo = 0, rexp_hi = 0;         // row `lane`: h + 64 of slices 0..3 / 4..7
  if (PRO == PRO_GAIN) {
    const float* ss = d.sumsq + ((size_t)xcd * kUnitsPerXcd + gm.gl * S) * kMTile + lane;
    float ss8[8];
#pragma unroll
    for (int s2 = 0; s2 < 8; ++s2) ss8[s2] = ss[(size_t)min(s2, S - 1) * kMTile];
    float t = 0.f;
#pragma unroll
    for (int s2 = 0; s2 < 8; ++s2) t += s2 < S ? ss8[s2] : 0.f;
    rstd_lane = 1.0f / sqrtf(t / (float)K + a.eps);
    rexp_lo = row_exp_bytes(ss8[0], ss8[1], ss8[2], ss8[3]);
    rexp_hi = row_exp_bytes(ss8[4], ss8[5], ss8[6], ss8[7]);
  }
  int pos_lane = 0, crow_lane = 0;
  if (EPI == EPI_QKV) {
    const int m = min(lane, M - 1);
    const int b = m / a.T, t = m - b * a.T;
    int P = d.prefix_len[b];
    P = P < 0 ? 0 : (P > a.p_max ? a.p_max : P);
    pos_lane = P + d.depth[m];
    crow_lane = b * a.nh * a.cap + P + t;
  }

  // Work item = one quad (8 rows x 32 columns) of one tile; item i -> slice i % S, helper wave
  // (i / S) % 4, as in gemm_stream_bf16.
  const int ln = lane & 31;
  const int rbase = 4 * (lane >> 5);
  const int n_items = gm.t_count * 8;
  constexpr int kBatch = 4;
  int cur_qd = -1;
  float rinv[8][4], rstd4[4];
  for (int it0 = gm.sp + S * hw; it0 < n_items; it0 += 4 * S * kBatch) {
    uint2 part[kBatch][8];
    float pinv[kBatch][8];
    float xres[kBatch][4];
#pragma unroll
    for (int bi = 0; bi < kBatch; ++bi) {
      const int it = it0 + 4 * S * bi;
      if (it >= n_items) break;
      const int tl = it >> 3, qd = it & 7;
      const int row0 = 8 * (qd & 3) + rbase + 32 * (qd >> 2);
      const size_t idx = part_index(tl, 0);
      const uint2* pb = reinterpret_cast<const uint2*>(part_x + idx * kTileVec4 + (qd >> 1) * 64 + lane) + (qd & 1);
#pragma unroll
      for (int s2 = 0; s2 < 8; ++s2) {
        const int sl = min(s2, S - 1);
        part[bi][s2] = pb[(size_t)sl * (kTileVec4 * 2)];
        pinv[bi][s2] = s2 < S ? pscale_x[idx + sl] : 0.f;
      }
      if (EPI == EPI_RESID) {
        const int tile = gm.t_begin + tl;
#pragma unroll
        for (int j = 0; j < 4; ++j) xres[bi][j] = d.x_io[(size_t)min(row0 + j, M - 1) * N + tile * 32 + ln];
      }
    }
#pragma unroll
    for (int bi = 0; bi < kBatch; ++bi) {
      const int it = it0 + 4 * S * bi;
      if (it >= n_items) break;
      const int tl = it >> 3, qd = it & 7;
      const int tile = gm.t_begin + tl;
      const int row0 = 8 * (qd & 3) + rbase + 32 * (qd >> 2);
      float v[4] = {0.f, 0.f, 0.f, 0.f};
      if (PRO == PRO_GAIN && qd != cur_qd) {                         // as in gemm_stream_bf16
        cur_qd = qd;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const unsigned elo = (unsigned)__shfl((int)rexp_lo, row0 + j, kWave);
          const unsigned ehi = (unsigned)__shfl((int)rexp_hi, row0 + j, kWave);
#pragma unroll
          for (int s2 = 0; s2 < 8; ++s2) rinv[s2][j] = row_scale_inv(s2 < 4 ? elo : ehi, s2 & 3);
          rstd4[j] = __shfl(rstd_lane, row0 + j, kWave);
        }
      }
      int any_flag = 0;
#pragma unroll
      for (int s2 = 0; s2 < 8; ++s2) {                               // fixed slice order
        const unsigned d0 = part[bi][s2].x, d1 = part[bi][s2].y;
        const float w = fabsf(pinv[bi][s2]);                         // 0 beyond the last slice
        any_flag |= __float_as_int(pinv[bi][s2]);
        const float q[4] = {q16_lo(d0), q16_hi(d0), q16_lo(d1), q16_hi(d1)};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (PRO == PRO_GAIN)
            v[j] = fmaf(w * q[j], rinv[s2][j], v[j]);
          else
            v[j] += w * q[j];
        }
      }
      if (any_flag < 0) {                    // rare: a tile with non-finite elements among the eight
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
      if (EPI == EPI_RESID) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (row0 + j < M) st_dev(d.x_io + (size_t)(row0 + j) * N + tile * 32 + ln, xres[bi][j] + v[j]);
      }
      if (EPI == EPI_SWIGLU) {                                       // lanes 0..15 gate, 16..31 up
        const int F = N / 2;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float up = lane_xor16(v[j], lane);
          if (ln < 16 && row0 + j < M)
            st_dev(d.act + (size_t)(row0 + j) * F + tile * 16 + ln, silu_fast(v[j]) * up);
        }
      }
      if (EPI == EPI_QKV) {
        const int tiles_per_mat = a.nh * 4;
        const int which = tile / tiles_per_mat;                      // 0 q, 1 k, 2 v
        const int head = (tile % tiles_per_mat) / 4, uq = tile % 4;
        const int jr = 16 * uq + (ln & 15);
        const int dcol = jr + 64 * (ln >> 4);
        const float turn_freq = exp2f(-(float)jr * (1.0f / 64.0f) * log2f(a.theta)) * 0.15915494309189535f;
        const float sgn = (ln & 16) ? 1.0f : -1.0f;
        const int D = a.nh * 128;
        bf16_t* cache = which == 1 ? a.L[layer].kc : a.L[layer].vc;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int ml = row0 + j;
          float val = v[j];
          const float partner = lane_xor16(val, lane);
          const int pos = __shfl(pos_lane, ml, kWave);
          const int crow = __shfl(crow_lane, ml, kWave);
          if (which != 2) {
            float turns = (float)pos * turn_freq;
            turns -= floorf(turns);
            val = val * __builtin_amdgcn_cosf(turns) + sgn * partner * __builtin_amdgcn_sinf(turns);
          }
          // two neighbouring columns share one 32-bit device-scope store
          const unsigned mine = f32_to_bf16(val).bits;
          const unsigned other = (unsigned)__shfl_xor((int)mine, 1, kWave);
          if (ml < M) {
            if (which == 0)
              st_dev(d.q + (size_t)ml * D + head * 128 + dcol, val);
            else if (!(ln & 1))
              st_dev(reinterpret_cast<unsigned*>(cache + ((size_t)crow + (size_t)head * a.cap) * 128 + dcol),
                     mine | (other << 16));
          }
        }
      }
    }
  }
  stamp(a, d, layer, hw, lane, 3 * ph + 2);
}

// block = 64: copies the launch description word by word
__global__ void write_stack_args(const StackArgs src, StackArgs* dst) {
  static_assert(sizeof(StackArgs) % 4 == 0 && sizeof(StackArgs) <= 4000, "fits the kernel arguments");
  const unsigned* s = reinterpret_cast<const unsigned*>(&src);
  unsigned* d = reinterpret_cast<unsigned*>(dst);
  for (unsigned i = threadIdx.x; i < sizeof(StackArgs) / 4; i += 64) d[i] = s[i];
}

// grid = n_xcd * 32 workgroups (all resident: one per CU), block = 512.
__global__ __launch_bounds__(512) void verify_stack_persistent(const StackArgs* __restrict__ ap,
                                                              const StackBufs d) {
  const StackArgs& a = *ap;
  __shared__ uint4 xs[32 * 2 * 2 * 64];                 // X chunk, 128 KiB (attention scratch between phases)
  __shared__ float4 tb[4 * (kTileFloats / 4)];          // finished tiles of the four stream waves, 32 KiB
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps the bookkeeping in scalar registers
  const int xcd = blockIdx.x % a.n_xcd, u = blockIdx.x / a.n_xcd;

  if (wave < 4) {
    stream_role(a, xs, tb, wave, lane, xcd, u);
    return;
  }

  const int hw = wave - 4, htid = tid - 256;
  SyncCtx sc;
  sc.wg_cnt = d.wg_cnt + 32 * blockIdx.x;
  sc.wg_flag = d.wg_flag + 32 * blockIdx.x;
  sc.grid_cnt = d.grid_cnt;
  sc.status = d.status;
  sc.n_xcd = a.n_xcd;
  sc.xcd = xcd;
  sc.seq = 0;
  sc.dead = false;
  const int D = a.nh * 128;
  const int qblocks = (a.T + kAttQ - 1) / kAttQ;
  const int att_tasks = (a.M / a.T) * qblocks * a.nh;
  const int att_passes = attention_passes(a);
  unsigned char* att_lds = reinterpret_cast<unsigned char*>(xs);
  float(*s_m)[kAttQ] = reinterpret_cast<float(*)[kAttQ]>(att_lds + 4 * 128 * kVtPitch);
  float(*s_l)[kAttQ] = s_m + 4;

  for (int layer = 0; layer < a.n_layers; ++layer) {
    const unsigned char* pk = a.L[layer].packed;
    const float* g1 = reinterpret_cast<const float*>(pk + a.off_g1);
    const float* g2 = reinterpret_cast<const float*>(pk + a.off_g2);
    for (int ph = 0; ph < 4; ++ph) {
      const PhaseGeom gm = phase_geom(phase_plan(a, ph), a.n_xcd, xcd, u);
      if (gm.active) {
        if (ph == 0)
          helper_gemm_phase<PRO_GAIN, EPI_QKV>(a, d, layer, ph, gm, d.x_io, g1, xs, tb, hw, lane, xcd, u, sc);
        else if (ph == 1)
          helper_gemm_phase<PRO_PLAIN, EPI_RESID>(a, d, layer, ph, gm, d.attn, nullptr, xs, tb, hw, lane, xcd, u, sc);
        else if (ph == 2)
          helper_gemm_phase<PRO_GAIN, EPI_SWIGLU>(a, d, layer, ph, gm, d.x_io, g2, xs, tb, hw, lane, xcd, u, sc);
        else
          helper_gemm_phase<PRO_PLAIN, EPI_RESID>(a, d, layer, ph, gm, d.act, nullptr, xs, tb, hw, lane, xcd, u, sc);
      }
      grid_sync(sc, hw, lane);
      if (ph == 0) {
        stamp(a, d, layer, hw, lane, 12);
        for (int pass = 0; pass < att_passes; ++pass) {
          const int task = pass * (int)gridDim.x + (int)blockIdx.x;
          if (task < att_tasks) {
            tree_attention_body<4, true>(d.q, a.L[layer].kc, a.L[layer].vc, d.prefix_len, a.p_max, d.anc,
                                         a.n_words, a.T, a.nh, a.cap, d.attn, task / a.nh, task % a.nh,
                                         att_lds, s_m, s_l, htid, [] { wg_bar(); });
          } else {
            wg_bar();
            wg_bar();
          }
        }
        stamp(a, d, layer, hw, lane, 13);
        grid_sync(sc, hw, lane);
        stamp(a, d, layer, hw, lane, 14);
      }
    }
  }
  (void)D;
}

}  // namespace sv
#endif
