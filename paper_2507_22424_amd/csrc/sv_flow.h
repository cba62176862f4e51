// The whole verifier stack (bf16 models, up to 64 tree rows) as ONE launch whose workgroups are
// dealt out product after product, layer after layer.
//
// A verification pass is a chain of dependent products (q/k/v -> attention -> output -> gate/up
// -> down, times the number of layers), each of which needs every output of the one before it.
// Launched one by one, every link of the chain pays the drain of one launch, the start of the
// next and the first round trip of its weight loads with the memory system idle.  Here the grid
// is (XCD, all units of all products in order): the hardware hands a compute unit to the next
// workgroup in line as soon as the one before it leaves, so a workgroup of the following product
// is already requesting its first weight pieces while the slower workgroups of the current one
// still finish.  Order is kept by counters: a workgroup waits (bounded) until every workgroup of
// the product before its own has reported in; producers write their outputs through to memory
// before they report, and no buffer is written twice inside one launch (each layer has its own
// activation buffers), so a reader can use ordinary cached loads: its L2 cannot hold an older
// copy.  Workgroups are dispatched in index order, so whatever a workgroup waits for was
// dispatched before it: the chain cannot lock up, and every wait is bounded all the same (a
// wait that runs out raises the sticky status word).
#ifndef SV_FLOW_H
#define SV_FLOW_H

#include "sv_attention.h"
#include "sv_gemm_mfma.h"

namespace sv {

constexpr int kFlowMaxLayers = 32;      // layers of one launch (deeper stacks: several launches)
constexpr int kFlowCntStride = 32;      // 32-bit words per completion counter: a line of its own
constexpr int kFlowSpin = 1 << 16;      // polls before a wait gives up (about 16 ms)

struct FlowAtt {
  const float* q;
  const bf16_t* kc;
  const bf16_t* vc;
  const int32_t* prefix_len;
  const uint64_t* anc;
  float* out;
  int p_max, n_words, T, nh, cap;
  int gx;                    // query blocks of all episodes (tasks per head)
  int total, per_xcd;        // tasks = gx * heads, dealt to the XCDs in contiguous runs
  const unsigned* wait_cnt;
  unsigned wait_val;
  unsigned* done_cnt;
  int* status;
};

struct FlowLayer {
  GemmArgs g[4];             // q/k/v, output, gate/up, down
  FlowAtt att;
};

// What the set-up kernel needs to write the table: the four products and the attention as they
// are for every layer, and what differs from layer to layer.
struct FlowSetup {
  GemmArgs g[4];
  FlowAtt att;
  const unsigned char* packed[kFlowMaxLayers];
  bf16_t* kc[kFlowMaxLayers];
  bf16_t* vc[kFlowMaxLayers];
  size_t off_g1, off_g2, off_wqkv, off_wo, off_wgu, off_wd, off_sqkv, off_so, off_sgu, off_sd;
  int w8;
  int n_layers;
  float* x;                  // caller's residual stream: input of layer 0, output of the last layer
  float* acts;               // per layer: q, attn, x1, act, x2 (float32), `act_stride` floats apart
  size_t act_stride, off_q, off_attn, off_x1, off_act, off_x2;
  unsigned* done;            // [layers][5] completion counters, kFlowCntStride words apart
  unsigned n_wg[5];          // workgroups that report per product
  FlowLayer* table;
};

__global__ void flow_setup_kernel(const FlowSetup s) {
  const int l = blockIdx.x * blockDim.x + threadIdx.x;
  if (l >= s.n_layers) return;
  FlowLayer L;
  for (int i = 0; i < 4; ++i) L.g[i] = s.g[i];
  L.att = s.att;
  const unsigned char* pk = s.packed[l];
  float* base = s.acts + (size_t)l * s.act_stride;
  float* xin = l == 0 ? s.x : s.acts + (size_t)(l - 1) * s.act_stride + s.off_x2;
  float* xout = l == s.n_layers - 1 ? s.x : base + s.off_x2;
  unsigned* done = s.done + (size_t)l * 5 * kFlowCntStride;
  // q/k/v
  L.g[0].X = xin; L.g[0].gain = (const float*)(pk + s.off_g1); L.g[0].Wp = (const uint4*)(pk + s.off_wqkv);
  L.g[0].wscale = s.w8 ? (const float*)(pk + s.off_sqkv) : nullptr;
  L.g[0].q_out = base + s.off_q; L.g[0].kc = s.kc[l]; L.g[0].vc = s.vc[l];
  L.g[0].wait_cnt = l == 0 ? nullptr : done - kFlowCntStride;      // down product of the layer before
  L.g[0].wait_val = l == 0 ? 0u : s.n_wg[4];
  L.g[0].done_cnt = done;
  // attention
  L.att.q = base + s.off_q; L.att.kc = s.kc[l]; L.att.vc = s.vc[l]; L.att.out = base + s.off_attn;
  L.att.wait_cnt = done; L.att.wait_val = s.n_wg[0]; L.att.done_cnt = done + kFlowCntStride;
  // output projection
  L.g[1].X = base + s.off_attn; L.g[1].Wp = (const uint4*)(pk + s.off_wo);
  L.g[1].wscale = s.w8 ? (const float*)(pk + s.off_so) : nullptr;
  L.g[1].x_res = xin; L.g[1].x_io = base + s.off_x1;
  L.g[1].wait_cnt = done + kFlowCntStride; L.g[1].wait_val = s.n_wg[1]; L.g[1].done_cnt = done + 2 * kFlowCntStride;
  // gate/up
  L.g[2].X = base + s.off_x1; L.g[2].gain = (const float*)(pk + s.off_g2); L.g[2].Wp = (const uint4*)(pk + s.off_wgu);
  L.g[2].wscale = s.w8 ? (const float*)(pk + s.off_sgu) : nullptr;
  L.g[2].act = base + s.off_act;
  L.g[2].wait_cnt = done + 2 * kFlowCntStride; L.g[2].wait_val = s.n_wg[2]; L.g[2].done_cnt = done + 3 * kFlowCntStride;
  // down
  L.g[3].X = base + s.off_act; L.g[3].Wp = (const uint4*)(pk + s.off_wd);
  L.g[3].wscale = s.w8 ? (const float*)(pk + s.off_sd) : nullptr;
  L.g[3].x_res = base + s.off_x1; L.g[3].x_io = xout;
  L.g[3].wait_cnt = done + 3 * kFlowCntStride; L.g[3].wait_val = s.n_wg[3]; L.g[3].done_cnt = done + 4 * kFlowCntStride;
  s.table[l] = L;
  for (int i = 0; i < 5; ++i) done[i * kFlowCntStride] = 0u;
}

struct FlowPlan {
  const FlowLayer* table;
  int n_layers;
  int ustart[6];             // first unit (per XCD) of q/k/v, attention, output, gate/up, down; units per layer
  int multi[4];              // a K slice of product i spans several LDS chunks
  long long* ts;             // measurement aid, or NULL: kFlowStamps device-clock stamps per workgroup
};
constexpr int kFlowStamps = 8;

constexpr size_t kFlowAttLds = 4 * 128 * kVtPitch + 2 * 4 * kAttQ * 4;
constexpr size_t kFlowLdsBytes = kGemmLdsAlloc > kFlowAttLds ? kGemmLdsAlloc : kFlowAttLds;

// grid = (n_xcd, units per layer * layers), block = 256.
template <bool W8>
__global__ __launch_bounds__(256, 1) void verify_flow_kernel(const FlowPlan p) {
  __shared__ uint4 lds_raw[(kFlowLdsBytes + 15) / 16];
  const int xcd = blockIdx.x;
  const int per_layer = p.ustart[5];
  const int layer = (int)blockIdx.y / per_layer;
  const int r = (int)blockIdx.y - layer * per_layer;
  const FlowLayer* L = p.table + layer;
  long long* ts = p.ts ? p.ts + ((size_t)blockIdx.y * gridDim.x + xcd) * kFlowStamps : nullptr;
  if (r >= p.ustart[1] && r < p.ustart[2]) {
    // ---- tree attention ----
    typedef const __attribute__((address_space(4))) FlowAtt* att_ptr_t;
    const __attribute__((address_space(4))) FlowAtt& A = *(att_ptr_t)(uintptr_t)&L->att;
    const int task = xcd * A.per_xcd + (r - p.ustart[1]);
    if (task >= A.total) return;
    const int tid = threadIdx.x;
    if (ts && tid == 0) ts[0] = wall_clock64();
    if (tid == 0) {
      const auto wc = (const __attribute__((address_space(1))) unsigned*)A.wait_cnt;
      int spin = 0;
      while (__hip_atomic_load(wc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < A.wait_val) {
        if (++spin > kFlowSpin) {
          __hip_atomic_fetch_or((__attribute__((address_space(1))) int*)A.status, 4, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          break;
        }
        __builtin_amdgcn_s_sleep(8);
      }
    }
    __syncthreads();
    if (ts && tid == 0) ts[1] = wall_clock64();
    const int head = task / A.gx;
#define SV_G(T, ptr) ((T*)(__attribute__((address_space(1))) T*)(ptr))
    unsigned char* lds = reinterpret_cast<unsigned char*>(lds_raw);
    float(*s_m)[kAttQ] = reinterpret_cast<float(*)[kAttQ]>(lds + 4 * 128 * kVtPitch);
    float(*s_l)[kAttQ] = s_m + 4;
    tree_attention_body<4, true>(SV_G(const float, A.q), SV_G(const bf16_t, A.kc), SV_G(const bf16_t, A.vc),
                                 SV_G(const int32_t, A.prefix_len), A.p_max, SV_G(const uint64_t, A.anc),
                                 A.n_words, A.T, A.nh, A.cap, SV_G(float, A.out), task - head * A.gx, head,
                                 lds, s_m, s_l, tid, [] { __syncthreads(); });
#undef SV_G
    if (ts && tid == 0) ts[2] = ts[3] = wall_clock64();
    __builtin_amdgcn_s_waitcnt(0);         // this wave's output rows are in memory
    __syncthreads();
    if (tid == 0) {
      __hip_atomic_fetch_add((__attribute__((address_space(1))) unsigned*)A.done_cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (ts) ts[4] = wall_clock64();
    }
    return;
  }
  const GemmLds lds = carve_gemm_lds(lds_raw);
  if (r < p.ustart[1]) {
    gemm_args_ptr_t ap = (gemm_args_ptr_t)(uintptr_t)&L->g[0];
    if (p.multi[0]) gemm_stream_body<PRO_GAIN, EPI_QKV, true, W8, true>(ap, xcd, r, 0, lds, ts);
    else gemm_stream_body<PRO_GAIN, EPI_QKV, false, W8, true>(ap, xcd, r, 0, lds, ts);
  } else if (r < p.ustart[3]) {
    gemm_args_ptr_t ap = (gemm_args_ptr_t)(uintptr_t)&L->g[1];
    if (p.multi[1]) gemm_stream_body<PRO_PLAIN, EPI_RESID, true, W8, true>(ap, xcd, r - p.ustart[2], 0, lds, ts);
    else gemm_stream_body<PRO_PLAIN, EPI_RESID, false, W8, true>(ap, xcd, r - p.ustart[2], 0, lds, ts);
  } else if (r < p.ustart[4]) {
    gemm_args_ptr_t ap = (gemm_args_ptr_t)(uintptr_t)&L->g[2];
    if (p.multi[2]) gemm_stream_body<PRO_GAIN, EPI_SWIGLU, true, W8, true>(ap, xcd, r - p.ustart[3], 0, lds, ts);
    else gemm_stream_body<PRO_GAIN, EPI_SWIGLU, false, W8, true>(ap, xcd, r - p.ustart[3], 0, lds, ts);
  } else {
    gemm_args_ptr_t ap = (gemm_args_ptr_t)(uintptr_t)&L->g[3];
    if (p.multi[3]) gemm_stream_body<PRO_PLAIN, EPI_RESID, true, W8, true>(ap, xcd, r - p.ustart[4], 0, lds, ts);
    else gemm_stream_body<PRO_PLAIN, EPI_RESID, false, W8, true>(ap, xcd, r - p.ustart[4], 0, lds, ts);
  }
}

}  // namespace sv
#endif
