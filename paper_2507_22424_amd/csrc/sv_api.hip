// C-ABI entry points of libspecvla_verify: argument checks, launch planning, launches.
// No allocation, no global state, no synchronisation.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>

#include "specvla_verify.h"
#include "specvla_verify_aux.h"
#include "sv_accept.h"
#include "sv_attention.h"
#include "sv_gemm_mfma.h"
#include "sv_gemm_rows.h"
#include "sv_internal.h"
#include "sv_kernels.h"
#include "sv_tree_build.h"

namespace sv {

static int check_cfg(const sv_model_cfg* c) {
  if (!c) return SV_ERR_NULL;
  if (c->dtype != SV_F32 && c->dtype != SV_BF16 && c->dtype != SV_BF16_W8 && c->dtype != SV_BF16_W4)
    return SV_ERR_DTYPE;
  if (c->hidden < 1 || c->n_heads < 1 || c->head_dim < 2 || c->mlp_dim < 1 || c->vocab < 1)
    return SV_ERR_SHAPE;
  if ((c->head_dim & 1) || c->head_dim > 128) return SV_ERR_SHAPE;
  if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) return SV_ERR_SHAPE;
  if (c->dtype != SV_F32) {
    if (c->hidden % 256 || c->head_dim != 128 || c->n_heads % 2 || c->mlp_dim % 256)
      return SV_ERR_SHAPE;
  }
  return SV_OK;
}

// Shape of the work split of one streaming GEMM (bf16 path): K slices and tile groups per XCD.
// A slice should be about one LDS chunk (4 K blocks); slices longer than a chunk need at most
// one tile per wave (4 per group) because the accumulators then stay in registers.
struct GemmPlan {
  int S, gpx;
  bool multi;                                // a K slice spans more than one LDS chunk
};

static GemmPlan plan_gemm(int n_rows, int k, int n_xcd) {
  const int npair = k / (2 * kBlkK);         // pieces of 256 k-values
  const int tiles_per_xcd = ceil_div(n_rows / kFragRows, n_xcd);
  GemmPlan p;
  p.S = npair / 2;                           // about one LDS chunk (2 pieces) per slice
  if (p.S > 8) p.S = 8;
  if (p.S < 1) p.S = 1;
  if (p.S > 1) p.S &= ~1;                    // the reduction deals quads to waves for S = 1 or even
  p.gpx = 32 / p.S;                          // aim at 32 units per XCD (one per CU)
  if (p.gpx > tiles_per_xcd) p.gpx = tiles_per_xcd;
  if (p.gpx < 1) p.gpx = 1;
  // a slice that spans several LDS chunks keeps its accumulators in registers: one tile per wave
  const int chunks = ceil_div(ceil_div(2 * npair, p.S), 4);     // LDS chunks of the longest slice
  if (chunks > 1 && ceil_div(tiles_per_xcd, p.gpx) > 4) p.gpx = ceil_div(tiles_per_xcd, 4);
  p.multi = chunks > 1;
  return p;
}

// Fills the work split of one product into its argument block.
static GemmPlan fill_plan(GemmArgs& a, int N, int K, int n_xcd) {
  const GemmPlan p = plan_gemm(N, K, n_xcd);
  a.N = N; a.K = K; a.S = p.S; a.gpx = p.gpx; a.n_xcd = n_xcd;
  const int n_tiles = N / kFragRows, G = n_xcd * p.gpx, npieces = K / kBlkK;
  a.tq = n_tiles / G; a.trem = n_tiles % G;
  a.pq = npieces / p.S; a.prem = npieces % p.S;
  a.inv_S = (65536u + p.S - 1) / p.S;      // exact for the unit numbers that occur (< 4096)
  return p;
}

// Per-XCD extent of the split-K scratch regions for a product of N rows over K: units (gpx * S)
// and partial tiles (gpx * (tiles per group, rounded up) * S), the largest over the XCD counts a
// device can have.
static void scratch_extent(int N, int K, int* ucap, int* tstride) {
  for (int n_xcd = 1; n_xcd <= kXcds; n_xcd *= 2) {
    GemmArgs a;
    const GemmPlan p = fill_plan(a, N, K, n_xcd);
    const int u = p.gpx * p.S, t = p.gpx * (a.tq + 1) * p.S;
    if (u > *ucap) *ucap = u;
    if (t > *tstride) *tstride = t;
  }
}

// Workgroups that share the keys of one (episode, head, 16 queries) task of the tree attention:
// more than one where the tasks alone would leave the chip short of waves (long prefix, one
// episode), at least 8 key tiles each.
static int attention_splits(int n_tasks, int n_keys) {
  int s = 1;
  while (s < 8 && n_tasks * s < kAttSplitFill && (n_keys / kAttKeys) / (2 * s) >= 8) s *= 2;
  return s;
}

// Launch shape of one many-row product: columns per output block and workgroups per block
// along K.  K is split (by powers of two, an even number of at least 8 k-steps each) while the
// output blocks alone would fill less than about two thirds of the CUs.
struct RowsPlan {
  int tn, ksplit;
};
static RowsPlan rows_plan(int m_tiles, int N, int K, int n_xcd, bool may_widen) {
  RowsPlan p;
  p.tn = kRowsTN;
  p.ksplit = 1;
  const int cus = n_xcd * 32, nks = K / kFragK;
  const int blocks = (N / kRowsTN) * m_tiles;
  while (blocks * p.ksplit * 3 < cus * 2 && p.ksplit < kRowsMaxKsplit) {
    const int s2 = p.ksplit * 2;
    if (nks % s2 || (nks / s2) % 2 || nks / s2 < 8) break;
    p.ksplit = s2;
  }
  // 384-column blocks where they give a whole number of rounds of the chip and 256-column blocks
  // do not (q/k/v of the 7B shape with 8 row blocks: 256 workgroups instead of 384)
  if (may_widen && p.ksplit == 1 && N % 384 == 0 && ((N / 384) * m_tiles) % cus == 0 && blocks % cus != 0)
    p.tn = 384;
  return p;
}
// bytes of float32 partial blocks the split products of a layer need at most (any XCD count)
static size_t rows_part_bytes(int rows_pad, int H, int D, int F) {
  size_t need = 0;
  const int dims[4][2] = {{3 * D, H}, {H, D}, {2 * F, H}, {H, F}};
  for (int n_xcd = 1; n_xcd <= kXcds; n_xcd *= 2)
    for (int i = 0; i < 4; ++i) {
      const RowsPlan p = rows_plan(rows_pad / kRowsTM, dims[i][0], dims[i][1], n_xcd, i == 0);
      const size_t b = p.ksplit > 1 ? (size_t)p.ksplit * rows_pad * dims[i][0] * 4 : 0;
      if (b > need) need = b;
    }
  return need;
}

static int device_xcds() {
  static int cached[64] = {0};               // hardware facts only; a race rewrites the same value
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 1;
  if (cached[dev] == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 32;
    int x = cus / 32;
    cached[dev] = x < 1 ? 1 : (x > kXcds ? kXcds : x);
  }
  return cached[dev];
}

static WorkspaceLayout workspace_layout(const sv_model_cfg& c, int m_rows, int n_scored) {
  const size_t H = c.hidden, D = (size_t)c.n_heads * c.head_dim, F = c.mlp_dim;
  WorkspaceLayout L;
  L.m_tiles = ceil_div(m_rows, kMTile);
  L.m_pad = L.m_tiles * kMTile;
  const size_t mp = L.m_pad, mt = L.m_tiles;
  size_t n_max = 3 * D;
  if (2 * F > n_max) n_max = 2 * F;
  if (H > n_max) n_max = H;
  size_t o = 0;
  if (c.dtype != SV_F32) {
    // sized for the worst split over the XCD counts a device can have
    const int D_ = (int)D, H_ = (int)H, F_ = (int)F;
    L.ucap = 1; L.tstride = 1;
    scratch_extent(3 * D_, H_, &L.ucap, &L.tstride);
    scratch_extent(H_, D_, &L.ucap, &L.tstride);
    scratch_extent(2 * F_, H_, &L.ucap, &L.tstride);
    scratch_extent(H_, F_, &L.ucap, &L.tstride);
    L.counter_bytes = align_up((mt * kXcds * L.ucap * kCntStride + 64) * sizeof(int), kAlign);   // group counters + status word
    L.counters = o; o += L.counter_bytes;
    L.sumsq = o;    o = align_up(o + mt * kXcds * L.ucap * kMTile * 4, kAlign);
    // partial tiles: 16-bit data (4 KiB each) in the first half of the region, one scale each behind it
    L.part_bytes = align_up(mt * kXcds * L.tstride * (size_t)kTileFloats * 4, 2 * kAlign);
    L.part = o;     o += L.part_bytes;
    L.xhat = o;
  } else {
    L.counter_bytes = 0;
    L.ucap = L.tstride = 0;
    L.counters = L.sumsq = o;
    L.part_bytes = align_up(mp * n_max * 4, kAlign);
    L.part = o;     o += L.part_bytes;
    L.xhat = o;     o = align_up(o + mp * H * 4, kAlign);
  }
  L.q = o;           o = align_up(o + mp * D * 4, kAlign);
  L.attn = o;        o = align_up(o + mp * D * 4, kAlign);
  L.act = o;         o = align_up(o + mp * F * 4, kAlign);
  // many rows (bf16 weights, more than two row tiles): activation fragments of one product,
  // 1 / rms of the rows, float32 partial blocks of the products that split K
  L.rows_xs = L.rows_rstd = L.rows_part = 0;
  L.rows_pad = 0;
  if (c.dtype == SV_BF16 && mt > kRowsMinTiles) {
    size_t k_max = H > D ? H : D;
    if (F > k_max) k_max = F;
    L.rows_pad = ceil_div(m_rows, kRowsTM) * kRowsTM;
    L.rows_xs = o;   o = align_up(o + (size_t)L.rows_pad * k_max * 4, kAlign);
    L.rows_rstd = o; o = align_up(o + (size_t)L.rows_pad * 4, kAlign);
    L.rows_part = o; o = align_up(o + rows_part_bytes(L.rows_pad, (int)H, (int)(c.n_heads * c.head_dim), (int)F), kAlign);
  }
  // partial results of the tree attention when the keys of a task are split (bf16 models)
  L.att_part = 0;
  if (c.dtype != SV_F32) {
    L.att_part = o;
    o = align_up(o + (size_t)8 * mp * c.n_heads * kAttPartStride * 4, kAlign);
  }
  L.head_z = o;      o = align_up(o + mp * H * 4, kAlign);
  L.head_logits = o; o = align_up(o + mp * (size_t)(n_scored > 0 ? n_scored : 0) * 4 * 16, kAlign);   // up to 16 K-slice planes
  // (the regions above do not move with n_scored: a layer call finds them without knowing it)
  L.head_cnt = L.head_cnt_bytes = L.head_sumsq = L.head_part = L.head_part_bytes = 0;
  L.head_ucap = L.head_tstride = 0;
  if (c.dtype != SV_F32 && n_scored > 0 && n_scored % kFragRows == 0) {
    L.head_ucap = 1; L.head_tstride = 1;
    scratch_extent(n_scored, (int)H, &L.head_ucap, &L.head_tstride);
    L.head_cnt_bytes = align_up(mt * kXcds * L.head_ucap * kCntStride * sizeof(int), kAlign);
    L.head_cnt = o;   o += L.head_cnt_bytes;
    L.head_sumsq = o; o = align_up(o + mt * kXcds * L.head_ucap * kMTile * 4, kAlign);
    L.head_part_bytes = align_up(mt * kXcds * L.head_tstride * (size_t)kTileFloats * 4, 2 * kAlign);
    L.head_part = o;  o += L.head_part_bytes;
  }
  L.total = o;
  return L;
}

// Packed head: float32 gain, then the scored rows in fragment order.
struct HeadLayout {
  size_t gain, w, total;
};
static HeadLayout head_layout(const sv_model_cfg& c, int n) {
  HeadLayout L;
  L.gain = 0;
  L.w = align_up((size_t)c.hidden * 4, kAlign);
  L.total = L.w + align_up((size_t)n * c.hidden * 2, kAlign);
  return L;
}
static int check_packed_head(const sv_model_cfg* cfg, int vocab_lo, int vocab_hi) {
  const int rc = check_cfg(cfg);
  if (rc != SV_OK) return rc;
  if (cfg->dtype == SV_F32) return SV_ERR_DTYPE;
  if (vocab_lo < 0 || vocab_lo >= vocab_hi || vocab_hi > cfg->vocab ||
      (vocab_hi - vocab_lo) % kFragRows)
    return SV_ERR_SHAPE;
  return SV_OK;
}

// K slices of the LM-head GEMM (it has few output tiles, so the reduction is spread out).
static int head_planes(int hidden) {
  int p = hidden / 256;
  return p < 1 ? 1 : (p > 16 ? 16 : p);
}

static inline int launch_status() { return hipGetLastError() == hipSuccess ? SV_OK : SV_ERR_LAUNCH; }

__global__ void zero_ints(int* p, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// ---- float32 models: plain kernels, one launch per step of the layer ----------------------

static int verify_layer_f32(const sv_model_cfg& c, const char* packed, float* x,
                            const sv_kv_view& kv, const sv_tree& tree, int B, char* ws,
                            hipStream_t st, hipEvent_t* ev) {
  const int T_ = tree.n_nodes, M = B * T_;
  auto mark = [&](int i) {
    if (ev) (void)hipEventRecord(ev[i], st);
  };
  const int H = c.hidden, D = c.n_heads * c.head_dim, F = c.mlp_dim;
  const PackedLayout pl = packed_layout(c);
  const WorkspaceLayout wl = workspace_layout(c, M, 0);
  const float* g1 = (const float*)(packed + pl.g1);
  const float* g2 = (const float*)(packed + pl.g2);
  float* xhat = (float*)(ws + wl.xhat);
  float* q = (float*)(ws + wl.q);
  float* attn = (float*)(ws + wl.attn);
  float* act = (float*)(ws + wl.act);
  float* part = (float*)(ws + wl.part);
  auto gemm = [&](const float* X, size_t w_off, int N, int K) {
    dim3 grid(ceil_div(N, 64), ceil_div(M, 64), 1);
    gemm_nt_fma<float, float><<<grid, 256, 0, st>>>(X, K, (const float*)(packed + w_off), K, part,
                                                    N, 0, M, N, K);
  };
  rmsnorm_rows<float><<<M, 256, 0, st>>>(x, g1, xhat, H, c.rms_eps);
  mark(0);
  gemm(xhat, pl.wqkv, 3 * D, H);
  mark(1);
  qkv_rope_append<float><<<M, 256, 0, st>>>(part, 1, 0, T_, c.n_heads, c.head_dim, tree.depth,
                                            kv.prefix_len, kv.prefix_len_max, kv.capacity,
                                            c.rope_theta, q, (float*)kv.k, (float*)kv.v);
  mark(2);
  tree_attention_rowwise<float, float><<<dim3(ceil_div(M, 4), c.n_heads), 256, 0, st>>>(
      q, (const float*)kv.k, (const float*)kv.v, kv.prefix_len, kv.prefix_len_max, tree.anc_mask,
      tree.n_words, T_, c.n_heads, c.head_dim, kv.capacity, attn, M);
  mark(3);
  gemm(attn, pl.wo, H, D);
  mark(4);
  residual_rmsnorm<float><<<M, 256, 0, st>>>(part, 1, 0, x, g2, xhat, H, c.rms_eps);
  mark(5);
  gemm(xhat, pl.wgu, 2 * F, H);
  mark(6);
  swiglu_rows<float><<<dim3(ceil_div(F, 256), M), 256, 0, st>>>(part, 1, 0, act, F);
  mark(7);
  gemm(act, pl.wd, H, F);
  mark(8);
  residual_rmsnorm<float><<<M, 256, 0, st>>>(part, 1, 0, x, nullptr, (float*)nullptr, H,
                                             c.rms_eps);
  return launch_status();
}

// ---- bf16 models: five launches per layer ---------------------------------------------------

static int verify_layer_bf16(const sv_model_cfg& c, const char* packed, float* x,
                             const sv_kv_view& kv, const sv_tree& tree, int B, char* ws,
                             hipStream_t st, hipEvent_t* ev) {
  const int T_ = tree.n_nodes, M = B * T_;
  auto mark = [&](int i) {
    if (ev) (void)hipEventRecord(ev[i], st);
  };
  const int H = c.hidden, D = c.n_heads * c.head_dim, F = c.mlp_dim;
  const PackedLayout pl = packed_layout(c);
  const WorkspaceLayout wl = workspace_layout(c, M, 0);
  const int n_xcd = device_xcds();
  size_t n_max = 3 * (size_t)D;
  if (2 * (size_t)F > n_max) n_max = 2 * (size_t)F;
  if ((size_t)H > n_max) n_max = H;
  unsigned* counters = (unsigned*)(ws + wl.counters);
  GemmArgs a;
  memset(&a, 0, sizeof(a));
  a.M = M;
  a.n_xcd = n_xcd;
  // partial tiles: packed data in the first half of the region, one inverse scale per tile behind it
  a.part16 = (uint4*)(ws + wl.part);
  a.pscale = (float*)(ws + wl.part + wl.part_bytes / 2);
  a.sumsq = (float*)(ws + wl.sumsq);
  a.group_cnt = counters;
  a.status = (int*)(ws + wl.counters + wl.counter_bytes) - 1;   // last word of the counter region
  a.eps = c.rms_eps;
  float* q = (float*)(ws + wl.q);
  float* attn = (float*)(ws + wl.attn);
  float* act = (float*)(ws + wl.act);
  dim3 grid(n_xcd, 1, 1);                    // workgroup (x, y) -> XCD x, unit (and row tile) y
  const bool rows = wl.m_tiles > 1;
  bool multi = false;
  a.ucap = wl.ucap; a.tstride = wl.tstride;
  auto shape = [&](int N, int K) {
    const GemmPlan p = fill_plan(a, N, K, n_xcd);
    grid.y = p.gpx * p.S * wl.m_tiles;
    multi = p.multi;
  };
  // the kernel form for the shape just planned: single- or multi-chunk K slices
#define SV_LAUNCH_GEMM2(PRO, EPI, WF, ROWS)                                             \
  do {                                                                                 \
    if (multi) gemm_stream_bf16<PRO, EPI, true, WF, ROWS><<<grid, 256, 0, st>>>(a);    \
    else gemm_stream_bf16<PRO, EPI, false, WF, ROWS><<<grid, 256, 0, st>>>(a);         \
  } while (0)
#define SV_LAUNCH_GEMM(PRO, EPI)                                                       \
  do {                                                                                 \
    if (wf == 2 && rows) SV_LAUNCH_GEMM2(PRO, EPI, 2, true);                           \
    else if (wf == 2) SV_LAUNCH_GEMM2(PRO, EPI, 2, false);                             \
    else if (wf == 1 && rows) SV_LAUNCH_GEMM2(PRO, EPI, 1, true);                      \
    else if (wf == 1) SV_LAUNCH_GEMM2(PRO, EPI, 1, false);                             \
    else if (rows) SV_LAUNCH_GEMM2(PRO, EPI, 0, true);                                 \
    else SV_LAUNCH_GEMM2(PRO, EPI, 0, false);                                          \
  } while (0)

  const int wf = c.dtype == SV_BF16_W8 ? 1 : (c.dtype == SV_BF16_W4 ? 2 : 0);   // weight format of the kernels
  const bool w8 = wf != 0;                                                        // row scales present
  a.X = x; a.gain = (const float*)(packed + pl.g1); a.Wp = (const uint4*)(packed + pl.wqkv);
  a.wscale = w8 ? (const float*)(packed + pl.sqkv) : nullptr;
  shape(3 * D, H);
  a.q_out = q; a.kc = (bf16_t*)kv.k; a.vc = (bf16_t*)kv.v; a.depth = tree.depth;
  a.prefix_len = kv.prefix_len; a.p_max = kv.prefix_len_max; a.cap = kv.capacity; a.T = T_;
  a.nh = c.n_heads; a.theta = c.rope_theta;
  mark(0);
  SV_LAUNCH_GEMM(PRO_GAIN, EPI_QKV);
  mark(1);
  mark(2);
  {
    const int ns = attention_splits(B * ceil_div(T_, kAttQ) * c.n_heads, kv.prefix_len_max + T_);
    float* apart = (float*)(ws + wl.att_part);
    tree_attention_mfma<4><<<dim3(B * ceil_div(T_, kAttQ), c.n_heads, ns), 256, 0, st>>>(
        q, (const bf16_t*)kv.k, (const bf16_t*)kv.v, kv.prefix_len, kv.prefix_len_max,
        tree.anc_mask, tree.n_words, T_, c.n_heads, kv.capacity, attn, apart, M);
    if (ns > 1) attention_merge_kernel<<<dim3(M, c.n_heads), 128, 0, st>>>(apart, ns, M, c.n_heads, attn);
  }
  mark(3);
  a.X = attn; a.gain = nullptr; a.Wp = (const uint4*)(packed + pl.wo);
  a.wscale = w8 ? (const float*)(packed + pl.so) : nullptr;
  shape(H, D);
  a.x_res = x; a.x_io = x;
  SV_LAUNCH_GEMM(PRO_PLAIN, EPI_RESID);
  mark(4);
  a.X = x; a.gain = (const float*)(packed + pl.g2); a.Wp = (const uint4*)(packed + pl.wgu);
  a.wscale = w8 ? (const float*)(packed + pl.sgu) : nullptr;
  shape(2 * F, H);
  a.act = act;
  mark(5);
  SV_LAUNCH_GEMM(PRO_GAIN, EPI_SWIGLU);
  mark(6);
  a.X = act; a.gain = nullptr; a.Wp = (const uint4*)(packed + pl.wd);
  a.wscale = w8 ? (const float*)(packed + pl.sd) : nullptr;
  shape(H, F);
  a.x_res = x; a.x_io = x;
  mark(7);
  SV_LAUNCH_GEMM(PRO_PLAIN, EPI_RESID);
  mark(8);
#undef SV_LAUNCH_GEMM
#undef SV_LAUNCH_GEMM2
  return launch_status();
}

// ---- bf16 models, many rows: products bound by the matrix cores (sv_gemm_rows.h) -----------

static int verify_layer_rows(const sv_model_cfg& c, const char* packed, float* x,
                             const sv_kv_view& kv, const sv_tree& tree, int B, char* ws,
                             hipStream_t st, hipEvent_t* ev) {
  const int T_ = tree.n_nodes, M = B * T_;
  auto mark = [&](int i) {
    if (ev) (void)hipEventRecord(ev[i], st);
  };
  const int H = c.hidden, D = c.n_heads * c.head_dim, F = c.mlp_dim;
  const PackedLayout pl = packed_layout(c);
  const WorkspaceLayout wl = workspace_layout(c, M, 0);
  const int n_xcd = device_xcds();
  uint4* xs = (uint4*)(ws + wl.rows_xs);
  float* rstd = (float*)(ws + wl.rows_rstd);
  float* part = (float*)(ws + wl.rows_part);
  float* q = (float*)(ws + wl.q);
  float* attn = (float*)(ws + wl.attn);
  float* act = (float*)(ws + wl.act);
  RowsArgs a;
  memset(&a, 0, sizeof(a));
  a.Xs = xs; a.M = M; a.m_tiles = wl.rows_pad / kRowsTM; a.n_xcd = n_xcd; a.part = part;
  a.q_out = q; a.kc = (bf16_t*)kv.k; a.vc = (bf16_t*)kv.v; a.depth = tree.depth;
  a.prefix_len = kv.prefix_len; a.p_max = kv.prefix_len_max; a.cap = kv.capacity; a.T = T_;
  a.nh = c.n_heads; a.theta = c.rope_theta; a.act = act;
  const int mb = wl.rows_pad / 32;
  auto split = [&](const float* src, const float* gain, int K) {
    if (gain) {
      rows_rstd_kernel<<<M, 256, 0, st>>>(src, K, c.rms_eps, rstd);
      split_rows_kernel<true><<<dim3(mb, K / 256), 256, 0, st>>>(src, gain, rstd, M, K, xs);
    } else {
      split_rows_kernel<false><<<dim3(mb, K / 256), 256, 0, st>>>(src, nullptr, nullptr, M, K, xs);
    }
  };
  const size_t plane = (size_t)wl.rows_pad;       // rows of one partial block
  // One product: the unsplit kernel with its fused epilogue, or the K-split kernel followed by the
  // reduction that carries the same epilogue.
  auto product = [&](int epi, size_t w_off, int N, int K) {
    const RowsPlan p = rows_plan(a.m_tiles, N, K, n_xcd, epi == EPI_QKV);
    a.Wp = (const uint4*)(packed + w_off); a.N = N; a.K = K; a.n_tiles = N / p.tn; a.ksplit = p.ksplit;
    const dim3 grid(n_xcd, ceil_div(a.n_tiles, n_xcd) * a.m_tiles, p.ksplit);
    if (p.ksplit == 1 && epi == EPI_QKV) {
      if (p.tn == 384) gemm_rows_kernel<EPI_QKV, false, 6><<<grid, 256, 0, st>>>(a);
      else gemm_rows_kernel<EPI_QKV, false, 4><<<grid, 256, 0, st>>>(a);
      return;
    }
    if (p.ksplit == 1 && epi == EPI_SWIGLU) {
      gemm_rows_kernel<EPI_SWIGLU, false, 4><<<grid, 256, 0, st>>>(a);
      return;
    }
    if (a.m_tiles == 1) gemm_rows_kernel<EPI_RESID, true, 4, true><<<grid, 256, 0, st>>>(a);
    else gemm_rows_kernel<EPI_RESID, true, 4><<<grid, 256, 0, st>>>(a);
    if (epi == EPI_RESID) {
      const size_t n4 = (size_t)M * N / 4;
      rows_reduce_resid_kernel<<<(unsigned)((n4 + 255) / 256), 256, 0, st>>>(part, p.ksplit, plane * N, x, x, n4);
    } else if (epi == EPI_SWIGLU) {
      const size_t n = (size_t)M * (N / 32) * 4;
      rows_reduce_swiglu_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(part, p.ksplit, plane * N, M, N, act);
    } else {
      const size_t n = (size_t)M * (N / 32) * 16;
      rows_reduce_qkv_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(part, p.ksplit, plane * N, a);
    }
  };
  mark(0);
  split(x, (const float*)(packed + pl.g1), H);
  product(EPI_QKV, pl.wqkv, 3 * D, H);
  mark(1);
  mark(2);
  {
    const int ns = attention_splits(B * ceil_div(T_, kAttQ) * c.n_heads, kv.prefix_len_max + T_);
    float* apart = (float*)(ws + wl.att_part);
    tree_attention_mfma<4><<<dim3(B * ceil_div(T_, kAttQ), c.n_heads, ns), 256, 0, st>>>(
        q, (const bf16_t*)kv.k, (const bf16_t*)kv.v, kv.prefix_len, kv.prefix_len_max,
        tree.anc_mask, tree.n_words, T_, c.n_heads, kv.capacity, attn, apart, M);
    if (ns > 1) attention_merge_kernel<<<dim3(M, c.n_heads), 128, 0, st>>>(apart, ns, M, c.n_heads, attn);
  }
  mark(3);
  split(attn, nullptr, D);
  product(EPI_RESID, pl.wo, H, D);
  mark(4);
  mark(5);
  split(x, (const float*)(packed + pl.g2), H);
  product(EPI_SWIGLU, pl.wgu, 2 * F, H);
  mark(6);
  mark(7);
  split(act, nullptr, F);
  product(EPI_RESID, pl.wd, H, F);
  mark(8);
  return launch_status();
}

template <typename T>
static int pack_layer_t(const sv_model_cfg& c, const sv_layer_weights& w, char* packed,
                        hipStream_t st) {
  const PackedLayout pl = packed_layout(c);
  const int H = c.hidden, D = c.n_heads * c.head_dim, F = c.mlp_dim;
  pack_gain<T><<<ceil_div(H, 256), 256, 0, st>>>((const T*)w.g1, (float*)(packed + pl.g1), H);
  pack_gain<T><<<ceil_div(H, 256), 256, 0, st>>>((const T*)w.g2, (float*)(packed + pl.g2), H);
  // float32: q|k|v and gate|up stacked, row-major.  bf16: fragment order with the row
  // permutations of the tile-local epilogues (rotary pairs / gate-up pairs 16 lanes apart).
  struct Piece {
    const void* src; size_t dst; int rows, k;
    int plain_off;                 // float32: first destination row
    int mode, off;                 // bf16: see pack_rows_mfma
  };
  const Piece pieces[] = {
      {w.wq, pl.wqkv, D, H, 0, PACK_PAIR16_HEAD, 0},
      {w.wk, pl.wqkv, D, H, D, PACK_PAIR16_HEAD, D},
      {w.wv, pl.wqkv, D, H, 2 * D, PACK_PAIR16_HEAD, 2 * D},
      {w.wo, pl.wo, H, D, 0, PACK_PLAIN, 0},
      {w.wg, pl.wgu, F, H, 0, PACK_PAIR16_GU, 0},
      {w.wu, pl.wgu, F, H, F, PACK_PAIR16_GU, 16},
      {w.wd, pl.wd, H, F, 0, PACK_PLAIN, 0}};
  for (const Piece& p : pieces) {
    if (c.dtype == SV_F32) {
      const size_t n = (size_t)p.rows * p.k;
      pack_rows_plain<float><<<(unsigned)((n + 255) / 256), 256, 0, st>>>(
          (const float*)p.src, (float*)(packed + p.dst), n, (size_t)p.plain_off * p.k);
    } else {
      const size_t chunks = (size_t)p.rows * (p.k / 8);
      pack_rows_mfma<<<(unsigned)((chunks + 255) / 256), 256, 0, st>>>(
          (const uint4*)p.src, (uint4*)(packed + p.dst), p.rows, p.k, p.mode, p.off);
    }
  }
  return launch_status();
}

// z: [n_rows, H] float32 normalised rows; parts: [planes][m_pad * n] float32 logit planes.
template <typename T>
static int head_t(const sv_model_cfg& c, const T* g_final, const T* w_lm, const float* x,
                  int n_rows, int lo, int hi, int32_t* out_token, float* out_logits, float* z,
                  float* parts, hipStream_t st) {
  const int H = c.hidden, n = hi - lo;
  const int planes = head_planes(H);
  const size_t plane = (size_t)ceil_div(n_rows, kMTile) * kMTile * n;
  rmsnorm_rows_tg<T, float><<<n_rows, 256, 0, st>>>(x, g_final, z, H, c.rms_eps);
  dim3 grid(ceil_div(n, 64), ceil_div(n_rows, 64), planes);   // K cut into `planes` slices
  gemm_nt_fma<float, T><<<grid, 256, 0, st>>>(z, H, w_lm + (size_t)lo * H, H, parts, n, plane,
                                              n_rows, n, H);
  argmax_rows<<<n_rows, 64, 0, st>>>(parts, planes, plane, out_logits, n, lo, out_token);
  return launch_status();
}

// Scratch of sv_action_head_argmax_noalloc: the normalised rows and the logit planes of one call,
// in device memory that belongs to the library image (one copy per GPU, for the life of the
// process).  Host code never uses the array's name as an address: scratch_address() asks the
// runtime where the current device's copy lives, once per device.
constexpr int kNoallocMaxRows = 64, kNoallocMaxScored = 256, kNoallocMaxHidden = 8192;
constexpr size_t kNoallocZBytes = (size_t)kNoallocMaxRows * kNoallocMaxHidden * 4;
constexpr size_t kNoallocScratchBytes = kNoallocZBytes + (size_t)16 * kMTile * kNoallocMaxScored * 4;
static __device__ __align__(256) unsigned char scratch[kNoallocScratchBytes];

static int scratch_address(unsigned char** out) {
  static void* per_device[64] = {nullptr};
  static std::mutex lock;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return SV_ERR_LAUNCH;
  std::lock_guard<std::mutex> guard(lock);
  if (!per_device[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SV_ERR_LAUNCH;
    per_device[dev] = p;
  }
  *out = (unsigned char*)per_device[dev];
  return SV_OK;
}

// Head on the streaming kernel: RMSNorm gain in the staging pass, 1 / rms after the reduction,
// logits to the workspace, then the row argmax.
static int head_packed(const sv_model_cfg& c, const char* packed, const float* x, int n_rows,
                       int lo, int hi, int32_t* out_token, float* out_logits, char* ws,
                       hipStream_t st) {
  const int n = hi - lo, H = c.hidden;
  const WorkspaceLayout wl = workspace_layout(c, n_rows, n);
  const HeadLayout hl = head_layout(c, n);
  const int n_xcd = device_xcds();
  float* logits = (float*)(ws + wl.head_logits);
  GemmArgs a;
  memset(&a, 0, sizeof(a));
  const GemmPlan p = fill_plan(a, n, H, n_xcd);
  a.X = x; a.gain = (const float*)(packed + hl.gain); a.Wp = (const uint4*)(packed + hl.w);
  a.M = n_rows; a.ucap = wl.head_ucap; a.tstride = wl.head_tstride;
  a.part16 = (uint4*)(ws + wl.head_part);
  a.pscale = (float*)(ws + wl.head_part + wl.head_part_bytes / 2);
  a.sumsq = (float*)(ws + wl.head_sumsq);
  a.group_cnt = (unsigned*)(ws + wl.head_cnt);
  a.status = (int*)(ws + wl.counters + wl.counter_bytes) - 1;   // the layers' status word
  a.eps = c.rms_eps;
  a.x_io = logits;
  const dim3 grid(n_xcd, p.gpx * p.S * wl.m_tiles);
  if (wl.m_tiles > 1) {
    if (p.multi) gemm_stream_bf16<PRO_GAIN, EPI_OUT, true, false, true><<<grid, 256, 0, st>>>(a);
    else gemm_stream_bf16<PRO_GAIN, EPI_OUT, false, false, true><<<grid, 256, 0, st>>>(a);
  } else {
    if (p.multi) gemm_stream_bf16<PRO_GAIN, EPI_OUT, true, false, false><<<grid, 256, 0, st>>>(a);
    else gemm_stream_bf16<PRO_GAIN, EPI_OUT, false, false, false><<<grid, 256, 0, st>>>(a);
  }
  argmax_rows_wide<<<n_rows, 256, 0, st>>>(logits, out_logits, n, lo, out_token);
  return launch_status();
}

}  // namespace sv

using namespace sv;

extern "C" {

const char* sv_version(void) { return "libspecvla_verify 0.1 (gfx950)"; }

const char* sv_strerror(int status) {
  switch (status) {
    case SV_OK: return "ok";
    case SV_ERR_NULL: return "a required pointer is NULL";
    case SV_ERR_SHAPE: return "unsupported size";
    case SV_ERR_TREE: return "parent array is not a valid draft tree (or too deep)";
    case SV_ERR_TOKEN: return "inconsistent action range or threshold";
    case SV_ERR_WORKSPACE: return "workspace or packed buffer too small or misaligned";
    case SV_ERR_DTYPE: return "unknown dtype";
    case SV_ERR_LAUNCH: return "HIP launch error";
    default: return "unknown status";
  }
}

int sv_tree_build_masks(const int32_t* parent, int B, int T, int d_cap, int32_t* depth,
                        uint64_t* anc_mask) {
  if (!parent || !depth || !anc_mask) return SV_ERR_NULL;
  if (B < 1 || T < 1 || T > SV_MAX_TREE_NODES || d_cap < 0 || d_cap > SV_MAX_DEPTH)
    return SV_ERR_SHAPE;
  const int W = (T + 63) / 64;
  for (int b = 0; b < B; ++b) {
    const int32_t* par = parent + (size_t)b * T;
    int32_t* dep = depth + (size_t)b * T;
    uint64_t* anc = anc_mask + (size_t)b * T * W;
    if (par[0] != -1) return SV_ERR_TREE;
    dep[0] = 0;
    for (int w = 0; w < W; ++w) anc[w] = 0;
    anc[0] = 1;
    for (int i = 1; i < T; ++i) {
      const int p = par[i];
      if (p < 0 || p >= i) return SV_ERR_TREE;
      dep[i] = dep[p] + 1;
      if (dep[i] > d_cap) return SV_ERR_TREE;
      for (int w = 0; w < W; ++w) anc[(size_t)i * W + w] = anc[(size_t)p * W + w];
      anc[(size_t)i * W + (i >> 6)] |= 1ull << (i & 63);
    }
  }
  return SV_OK;
}

int sv_packed_layer_bytes(const sv_model_cfg* cfg, size_t* bytes) {
  if (!bytes) return SV_ERR_NULL;
  const int rc = check_cfg(cfg);
  if (rc != SV_OK) return rc;
  *bytes = packed_layout(*cfg).total;
  return SV_OK;
}

int sv_pack_layer(const sv_model_cfg* cfg, const sv_layer_weights* raw, void* packed,
                  size_t packed_bytes, void* stream) {
  const int rc = check_cfg(cfg);
  if (rc != SV_OK) return rc;
  if (!raw || !packed || !raw->g1 || !raw->wq || !raw->wk || !raw->wv || !raw->wo || !raw->g2 ||
      !raw->wg || !raw->wu || !raw->wd)
    return SV_ERR_NULL;
  if (packed_bytes < packed_layout(*cfg).total || ((uintptr_t)packed % kAlign))
    return SV_ERR_WORKSPACE;
  if (cfg->dtype == SV_BF16_W8 || cfg->dtype == SV_BF16_W4) return SV_ERR_DTYPE;   // sv_pack_layer_w8 / _w4 take the scales
  if (cfg->dtype == SV_F32) return pack_layer_t<float>(*cfg, *raw, (char*)packed, (hipStream_t)stream);
  return pack_layer_t<bf16_t>(*cfg, *raw, (char*)packed, (hipStream_t)stream);
}

static int pack_layer_codes(const sv_model_cfg* cfg, const sv_layer_weights* raw,
                            const sv_layer_scales* sc, void* packed_v, size_t packed_bytes,
                            void* stream, int dtype) {
  const int rc = check_cfg(cfg);
  if (rc != SV_OK) return rc;
  if (cfg->dtype != dtype) return SV_ERR_DTYPE;
  if (!raw || !sc || !packed_v || !raw->g1 || !raw->wq || !raw->wk || !raw->wv || !raw->wo ||
      !raw->g2 || !raw->wg || !raw->wu || !raw->wd || !sc->sq || !sc->sk || !sc->sv || !sc->so ||
      !sc->sg || !sc->su || !sc->sd)
    return SV_ERR_NULL;
  const sv_model_cfg& c = *cfg;
  const PackedLayout pl = packed_layout(c);
  if (packed_bytes < pl.total || ((uintptr_t)packed_v % kAlign)) return SV_ERR_WORKSPACE;
  char* packed = (char*)packed_v;
  hipStream_t st = (hipStream_t)stream;
  const int H = c.hidden, D = c.n_heads * c.head_dim, F = c.mlp_dim;
  pack_gain<bf16_t><<<ceil_div(H, 256), 256, 0, st>>>((const bf16_t*)raw->g1, (float*)(packed + pl.g1), H);
  pack_gain<bf16_t><<<ceil_div(H, 256), 256, 0, st>>>((const bf16_t*)raw->g2, (float*)(packed + pl.g2), H);
  struct Piece {
    const void* src; const float* scale; size_t dst, sdst; int rows, k, mode, off;
  };
  const Piece pieces[] = {
      {raw->wq, sc->sq, pl.wqkv, pl.sqkv, D, H, PACK_PAIR16_HEAD, 0},
      {raw->wk, sc->sk, pl.wqkv, pl.sqkv, D, H, PACK_PAIR16_HEAD, D},
      {raw->wv, sc->sv, pl.wqkv, pl.sqkv, D, H, PACK_PAIR16_HEAD, 2 * D},
      {raw->wo, sc->so, pl.wo, pl.so, H, D, PACK_PLAIN, 0},
      {raw->wg, sc->sg, pl.wgu, pl.sgu, F, H, PACK_PAIR16_GU, 0},
      {raw->wu, sc->su, pl.wgu, pl.sgu, F, H, PACK_PAIR16_GU, 16},
      {raw->wd, sc->sd, pl.wd, pl.sd, H, F, PACK_PLAIN, 0}};
  for (const Piece& p : pieces) {
    const size_t n8 = (size_t)p.rows * (p.k / 8);
    if (dtype == SV_BF16_W4)
      pack_rows_mfma_w4<<<(unsigned)((n8 + 255) / 256), 256, 0, st>>>(
          (const uint32_t*)p.src, (uint32_t*)(packed + p.dst), p.rows, p.k, p.mode, p.off);
    else
      pack_rows_mfma_w8<<<(unsigned)((n8 + 255) / 256), 256, 0, st>>>(
          (const uint2*)p.src, (uint2*)(packed + p.dst), p.rows, p.k, p.mode, p.off);
    pack_row_scales<<<ceil_div(p.rows, 256), 256, 0, st>>>(p.scale, (float*)(packed + p.sdst), p.rows,
                                                           p.mode, p.off);
  }
  return launch_status();
}

int sv_pack_layer_w8(const sv_model_cfg* cfg, const sv_layer_weights* raw,
                     const sv_layer_scales* sc, void* packed_v, size_t packed_bytes,
                     void* stream) {
  return pack_layer_codes(cfg, raw, sc, packed_v, packed_bytes, stream, SV_BF16_W8);
}

int sv_pack_layer_w4(const sv_model_cfg* cfg, const sv_layer_weights* raw,
                     const sv_layer_scales* sc, void* packed_v, size_t packed_bytes,
                     void* stream) {
  return pack_layer_codes(cfg, raw, sc, packed_v, packed_bytes, stream, SV_BF16_W4);
}

int sv_workspace_bytes(const sv_model_cfg* cfg, int B, int T, int n_scored, size_t* bytes) {
  if (!bytes) return SV_ERR_NULL;
  const int rc = check_cfg(cfg);
  if (rc != SV_OK) return rc;
  if (B < 1 || T < 1 || T > SV_MAX_TREE_NODES || n_scored < 0 || n_scored > cfg->vocab ||
      (long long)B * T > (1 << 15))
    return SV_ERR_SHAPE;
  *bytes = workspace_layout(*cfg, B * T, n_scored).total;
  return SV_OK;
}

int sv_workspace_init(const sv_model_cfg* cfg, int B, int T, int n_scored, void* workspace,
                      size_t ws_bytes, void* stream) {
  size_t total;
  const int rc = sv_workspace_bytes(cfg, B, T, n_scored, &total);
  if (rc != SV_OK) return rc;
  if (!workspace) return SV_ERR_NULL;
  if (((uintptr_t)workspace % kAlign) || ws_bytes < total) return SV_ERR_WORKSPACE;
  const WorkspaceLayout wl = workspace_layout(*cfg, B * T, n_scored);
  const size_t n = wl.counter_bytes / sizeof(int);
  if (n > 0)
    zero_ints<<<(unsigned)((n + 255) / 256), 256, 0, (hipStream_t)stream>>>(
        (int*)((char*)workspace + wl.counters), n);
  const size_t nh = wl.head_cnt_bytes / sizeof(int);
  if (nh > 0)
    zero_ints<<<(unsigned)((nh + 255) / 256), 256, 0, (hipStream_t)stream>>>(
        (int*)((char*)workspace + wl.head_cnt), nh);
  return launch_status();
}

int sv_workspace_region(const sv_model_cfg* cfg, int B, int T, int n_scored, int which,
                        size_t* offset, size_t* bytes) {
  if (!offset || !bytes) return SV_ERR_NULL;
  size_t total;
  const int rc = sv_workspace_bytes(cfg, B, T, n_scored, &total);
  if (rc != SV_OK) return rc;
  const WorkspaceLayout wl = workspace_layout(*cfg, B * T, n_scored);
  const size_t D = (size_t)cfg->n_heads * cfg->head_dim, M = (size_t)B * T;
  if (which == SV_WS_ATTN_OUT) {
    *offset = wl.attn;
    *bytes = M * D * 4;
  } else if (which == SV_WS_Q) {
    *offset = wl.q;
    *bytes = M * D * 4;
  } else if (which == SV_WS_STATUS) {
    *offset = wl.counters + (wl.counter_bytes ? wl.counter_bytes - 4 : 0);
    *bytes = wl.counter_bytes ? 4 : 0;
  } else {
    return SV_ERR_SHAPE;
  }
  return SV_OK;
}

static int verify_layer_checked(const sv_model_cfg* cfg, const void* packed, float* x,
                                const sv_kv_view* kv, const sv_tree* tree, int B,
                                void* workspace, size_t ws_bytes, void* stream,
                                hipEvent_t* ev) {
  const int rc = check_cfg(cfg);
  if (rc != SV_OK) return rc;
  if (!packed || !x || !kv || !tree || !workspace || !kv->k || !kv->v || !kv->prefix_len ||
      !tree->parent || !tree->depth || !tree->anc_mask)
    return SV_ERR_NULL;
  const int T = tree->n_nodes;
  if (B < 1 || T < 1 || T > SV_MAX_TREE_NODES || tree->n_words != (T + 63) / 64 ||
      (long long)B * T > (1 << 15))
    return SV_ERR_SHAPE;
  if (kv->prefix_len_max < 0 || (long long)kv->capacity < (long long)kv->prefix_len_max + T)
    return SV_ERR_SHAPE;
  if ((long long)B * cfg->n_heads * kv->capacity >= (1ll << 31)) return SV_ERR_SHAPE;   // cache rows are indexed in 32 bits
  if (((uintptr_t)workspace % kAlign) || ((uintptr_t)packed % kAlign) ||
      ws_bytes < workspace_layout(*cfg, B * T, 0).total)
    return SV_ERR_WORKSPACE;
  if (cfg->dtype == SV_F32)
    return verify_layer_f32(*cfg, (const char*)packed, x, *kv, *tree, B, (char*)workspace,
                            (hipStream_t)stream, ev);
  if (cfg->dtype == SV_BF16 && ceil_div(B * T, kMTile) > kRowsMinTiles)
    return verify_layer_rows(*cfg, (const char*)packed, x, *kv, *tree, B, (char*)workspace,
                             (hipStream_t)stream, ev);
  return verify_layer_bf16(*cfg, (const char*)packed, x, *kv, *tree, B, (char*)workspace,
                           (hipStream_t)stream, ev);
}

int sv_verify_layer(const sv_model_cfg* cfg, const void* packed, float* x, const sv_kv_view* kv,
                    const sv_tree* tree, int B, void* workspace, size_t ws_bytes, void* stream) {
  return verify_layer_checked(cfg, packed, x, kv, tree, B, workspace, ws_bytes, stream, nullptr);
}

int sv_verify_layer_timed(const sv_model_cfg* cfg, const void* packed, float* x,
                          const sv_kv_view* kv, const sv_tree* tree, int B, void* workspace,
                          size_t ws_bytes, void* stream, void* const* events) {
  if (!events) return SV_ERR_NULL;
  hipEvent_t ev[SV_N_TIMING_EVENTS];
  for (int i = 0; i < SV_N_TIMING_EVENTS; ++i) {
    if (!events[i]) return SV_ERR_NULL;
    ev[i] = (hipEvent_t)events[i];
  }
  return verify_layer_checked(cfg, packed, x, kv, tree, B, workspace, ws_bytes, stream, ev);
}

static int verify_stack_args(const sv_model_cfg* cfg, int n_layers, const void* const* packed,
                             float* x, const sv_kv_view* kv, const sv_tree* tree, int B,
                             void* workspace, size_t ws_bytes) {
  const int rc = check_cfg(cfg);
  if (rc != SV_OK) return rc;
  if (!packed || !x || !kv || !tree || !workspace || !tree->parent || !tree->depth || !tree->anc_mask)
    return SV_ERR_NULL;
  if (n_layers < 1) return SV_ERR_SHAPE;
  const int T = tree->n_nodes;
  if (B < 1 || T < 1 || T > SV_MAX_TREE_NODES || tree->n_words != (T + 63) / 64 ||
      (long long)B * T > (1 << 15))
    return SV_ERR_SHAPE;
  for (int l = 0; l < n_layers; ++l) {
    if (!packed[l] || !kv[l].k || !kv[l].v || !kv[l].prefix_len) return SV_ERR_NULL;
    if ((uintptr_t)packed[l] % kAlign) return SV_ERR_WORKSPACE;
    if (kv[l].prefix_len_max < 0 || (long long)kv[l].capacity < (long long)kv[l].prefix_len_max + T)
      return SV_ERR_SHAPE;
    if ((long long)B * cfg->n_heads * kv[l].capacity >= (1ll << 31)) return SV_ERR_SHAPE;
  }
  if (((uintptr_t)workspace % kAlign) || ws_bytes < workspace_layout(*cfg, B * T, 0).total)
    return SV_ERR_WORKSPACE;
  return SV_OK;
}

int sv_verify_stack(const sv_model_cfg* cfg, int n_layers, const void* const* packed, float* x,
                    const sv_kv_view* kv, const sv_tree* tree, int B, void* workspace,
                    size_t ws_bytes, void* stream) {
  const int rc = verify_stack_args(cfg, n_layers, packed, x, kv, tree, B, workspace, ws_bytes);
  if (rc != SV_OK) return rc;
  for (int l = 0; l < n_layers; ++l) {
    const int r2 = verify_layer_checked(cfg, packed[l], x, kv + l, tree, B, workspace, ws_bytes,
                                        stream, nullptr);
    if (r2 != SV_OK) return r2;
  }
  return SV_OK;
}

int sv_action_head_argmax(const sv_model_cfg* cfg, const void* g_final, const void* w_lm,
                          const float* x, int n_rows, int vocab_lo, int vocab_hi,
                          int32_t* out_token, float* out_logits, void* workspace,
                          size_t ws_bytes, void* stream) {
  const int rc = check_cfg(cfg);
  if (rc != SV_OK) return rc;
  if (!g_final || !w_lm || !x || !out_token || !workspace) return SV_ERR_NULL;
  if (n_rows < 1 || n_rows > (1 << 15) || vocab_lo < 0 || vocab_lo >= vocab_hi ||
      vocab_hi > cfg->vocab)
    return SV_ERR_SHAPE;
  if (((uintptr_t)workspace % kAlign) ||
      ws_bytes < workspace_layout(*cfg, n_rows, vocab_hi - vocab_lo).total)
    return SV_ERR_WORKSPACE;
  const WorkspaceLayout wl = workspace_layout(*cfg, n_rows, vocab_hi - vocab_lo);
  float* z = (float*)((char*)workspace + wl.head_z);
  float* parts = (float*)((char*)workspace + wl.head_logits);
  if (cfg->dtype == SV_F32)
    return head_t<float>(*cfg, (const float*)g_final, (const float*)w_lm, x, n_rows, vocab_lo,
                         vocab_hi, out_token, out_logits, z, parts, (hipStream_t)stream);
  return head_t<bf16_t>(*cfg, (const bf16_t*)g_final, (const bf16_t*)w_lm, x, n_rows, vocab_lo,
                        vocab_hi, out_token, out_logits, z, parts, (hipStream_t)stream);
}

int sv_action_head_argmax_noalloc(const sv_model_cfg* cfg, const void* g_final, const void* w_lm,
                                  const float* x, int n_rows, int vocab_lo, int vocab_hi,
                                  int32_t* out_token, float* out_logits, void* stream) {
  const int rc = check_cfg(cfg);
  if (rc != SV_OK) return rc;
  if (!g_final || !w_lm || !x || !out_token) return SV_ERR_NULL;
  if (n_rows < 1 || vocab_lo < 0 || vocab_lo >= vocab_hi || vocab_hi > cfg->vocab) return SV_ERR_SHAPE;
  if (n_rows > kNoallocMaxRows || vocab_hi - vocab_lo > kNoallocMaxScored || cfg->hidden > kNoallocMaxHidden)
    return SV_ERR_WORKSPACE;                  // beyond what the built-in scratch holds
  unsigned char* base = nullptr;
  const int rs = scratch_address(&base);
  if (rs != SV_OK) return rs;
  float* z = (float*)base;
  float* parts = (float*)(base + kNoallocZBytes);
  if (cfg->dtype == SV_F32)
    return head_t<float>(*cfg, (const float*)g_final, (const float*)w_lm, x, n_rows, vocab_lo,
                         vocab_hi, out_token, out_logits, z, parts, (hipStream_t)stream);
  return head_t<bf16_t>(*cfg, (const bf16_t*)g_final, (const bf16_t*)w_lm, x, n_rows, vocab_lo,
                        vocab_hi, out_token, out_logits, z, parts, (hipStream_t)stream);
}

int sv_packed_head_bytes(const sv_model_cfg* cfg, int vocab_lo, int vocab_hi, size_t* bytes) {
  if (!bytes) return SV_ERR_NULL;
  const int rc = check_packed_head(cfg, vocab_lo, vocab_hi);
  if (rc != SV_OK) return rc;
  *bytes = head_layout(*cfg, vocab_hi - vocab_lo).total;
  return SV_OK;
}

int sv_pack_head(const sv_model_cfg* cfg, const void* g_final, const void* w_lm, int vocab_lo,
                 int vocab_hi, void* packed_v, size_t packed_bytes, void* stream) {
  const int rc = check_packed_head(cfg, vocab_lo, vocab_hi);
  if (rc != SV_OK) return rc;
  if (!g_final || !w_lm || !packed_v) return SV_ERR_NULL;
  const int n = vocab_hi - vocab_lo, H = cfg->hidden;
  const HeadLayout hl = head_layout(*cfg, n);
  if (packed_bytes < hl.total || ((uintptr_t)packed_v % kAlign)) return SV_ERR_WORKSPACE;
  char* packed = (char*)packed_v;
  hipStream_t st = (hipStream_t)stream;
  pack_gain<bf16_t><<<ceil_div(H, 256), 256, 0, st>>>((const bf16_t*)g_final, (float*)(packed + hl.gain), H);
  const size_t n8 = (size_t)n * (H / 8);
  pack_rows_mfma<<<(unsigned)((n8 + 255) / 256), 256, 0, st>>>(
      (const uint4*)((const bf16_t*)w_lm + (size_t)vocab_lo * H), (uint4*)(packed + hl.w), n, H,
      PACK_PLAIN, 0);
  return launch_status();
}

int sv_action_head_argmax_packed(const sv_model_cfg* cfg, const void* packed_head, const float* x,
                                 int n_rows, int vocab_lo, int vocab_hi, int32_t* out_token,
                                 float* out_logits, void* workspace, size_t ws_bytes,
                                 void* stream) {
  const int rc = check_packed_head(cfg, vocab_lo, vocab_hi);
  if (rc != SV_OK) return rc;
  if (!packed_head || !x || !out_token || !workspace) return SV_ERR_NULL;
  if (n_rows < 1 || n_rows > (1 << 15)) return SV_ERR_SHAPE;
  if (((uintptr_t)workspace % kAlign) || ((uintptr_t)packed_head % kAlign) ||
      ws_bytes < workspace_layout(*cfg, n_rows, vocab_hi - vocab_lo).total)
    return SV_ERR_WORKSPACE;
  return head_packed(*cfg, (const char*)packed_head, x, n_rows, vocab_lo, vocab_hi, out_token,
                     out_logits, (char*)workspace, (hipStream_t)stream);
}

int sv_stream_read(const void* ptr, size_t bytes, void* sink, void* stream) {
  if (!ptr || !sink) return SV_ERR_NULL;
  if (bytes < 16 || (bytes % 16) || ((uintptr_t)ptr % 16) || ((uintptr_t)sink % 16)) return SV_ERR_SHAPE;
  const size_t n_vec = bytes / 16;
  size_t blocks = (n_vec + 2047) / 2048;               // 8 KiB per wave and round
  if (blocks > 2048) blocks = 2048;                    // 8 workgroups per CU walk the buffer
  stream_read_kernel<<<(unsigned)blocks, 256, 0, (hipStream_t)stream>>>((const u32x4_t*)ptr, n_vec,
                                                                       (u32x4_t*)sink);
  return launch_status();
}

int sv_relaxed_accept(const sv_tree* tree, const int32_t* draft_token,
                      const int32_t* target_token, int action_lo, int n_bins, int r, int B,
                      int d_cap, uint8_t* accept_mask, int32_t* accepted_len,
                      int32_t* best_node, int32_t* path, int32_t* out_tokens, void* stream) {
  if (!tree || !tree->parent || !tree->depth || !tree->anc_mask || !draft_token ||
      !target_token || !accept_mask || !accepted_len || !best_node || !path || !out_tokens)
    return SV_ERR_NULL;
  const int T = tree->n_nodes;
  if (B < 1 || B > (1 << 15) || T < 1 || T > SV_MAX_TREE_NODES ||
      tree->n_words != (T + 63) / 64 || d_cap < 0 || d_cap > SV_MAX_DEPTH)
    return SV_ERR_SHAPE;
  if (n_bins < 1 || r < 0 || action_lo < 0) return SV_ERR_TOKEN;
  relaxed_accept_kernel<<<B, 128, 0, (hipStream_t)stream>>>(
      tree->parent, tree->depth, tree->anc_mask, T, tree->n_words, draft_token, target_token,
      action_lo, n_bins, r, d_cap, accept_mask, accepted_len, best_node, path, out_tokens);
  return launch_status();
}

int sv_tree_build_device(const int32_t* cand_parent, const float* cand_logp,
                         const int32_t* cand_token, int n_cand, const int32_t* root_token, int B,
                         int T, int d_cap, int32_t* parent, int32_t* depth, uint64_t* anc_mask,
                         int32_t* draft_token, int32_t* status, void* stream) {
  if (!cand_parent || !cand_logp || !cand_token || !root_token || !parent || !depth || !anc_mask ||
      !draft_token || !status)
    return SV_ERR_NULL;
  if (B < 1 || B > (1 << 15) || T < 1 || T > SV_MAX_TREE_NODES || n_cand < T - 1 ||
      n_cand > kMaxCandidates || d_cap < 0 || d_cap > SV_MAX_DEPTH)
    return SV_ERR_SHAPE;
  tree_build_kernel<<<B, 256, 0, (hipStream_t)stream>>>(cand_parent, cand_logp, cand_token, n_cand,
                                                        root_token, T, (T + 63) / 64, d_cap, parent,
                                                        depth, anc_mask, draft_token, status);
  return launch_status();
}

int sv_commit_path(const sv_model_cfg* cfg, const sv_kv_view* kv, int T, const int32_t* path,
                   const int32_t* accepted_len, int B, int d_cap, void* stream) {
  const int rc = check_cfg(cfg);
  if (rc != SV_OK) return rc;
  if (!kv || !kv->k || !kv->v || !kv->prefix_len || !path || !accepted_len) return SV_ERR_NULL;
  if (B < 1 || B > (1 << 15) || T < 1 || T > SV_MAX_TREE_NODES || d_cap < 0 || d_cap > SV_MAX_DEPTH)
    return SV_ERR_SHAPE;
  if (kv->prefix_len_max < 0 || (long long)kv->capacity < (long long)kv->prefix_len_max + T)
    return SV_ERR_SHAPE;
  const dim3 grid(B, cfg->n_heads);
  if (cfg->dtype == SV_F32)
    commit_path_kernel<float><<<grid, 128, 0, (hipStream_t)stream>>>(
        (float*)kv->k, (float*)kv->v, kv->prefix_len, kv->prefix_len_max, kv->capacity, T,
        cfg->n_heads, cfg->head_dim, path, accepted_len, d_cap);
  else
    commit_path_kernel<bf16_t><<<grid, 128, 0, (hipStream_t)stream>>>(
        (bf16_t*)kv->k, (bf16_t*)kv->v, kv->prefix_len, kv->prefix_len_max, kv->capacity, T,
        cfg->n_heads, cfg->head_dim, path, accepted_len, d_cap);
  return launch_status();
}

int sv_advance_prefix(int32_t* prefix_len, const int32_t* accepted_len, int B, int d_cap,
                      void* stream) {
  if (!prefix_len || !accepted_len) return SV_ERR_NULL;
  if (B < 1 || B > (1 << 15) || d_cap < 0 || d_cap > SV_MAX_DEPTH) return SV_ERR_SHAPE;
  advance_prefix_kernel<<<(B + 63) / 64, 64, 0, (hipStream_t)stream>>>(prefix_len, accepted_len, B,
                                                                       d_cap);
  return launch_status();
}

}  // extern "C"
