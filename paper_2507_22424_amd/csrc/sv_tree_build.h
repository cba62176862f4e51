// Draft tree from the recorded top-K predictions of the draft model, built on the device.
//
// Sec. 4.1: the top-K predictions of the drafter are recorded and form a tree with several
// paths (the dynamic draft tree strategy the paper adopts; Sec. 5.1: top 8, at most 50 nodes).
// This is the final selection of that strategy: every candidate's score is the joint
// log-probability of its path (float32, accumulated from the root down, one addition per
// edge), the n_nodes - 1 best candidates are kept (lower candidate index wins ties, so a
// parent is never dropped before its child), and the kept nodes are numbered breadth first
// behind the root.  Output = exactly the arrays the verification calls take (parent, depth,
// ancestor-or-self bitmask, draft tokens), so a step needs no host round trip for its tree.
//
// One workgroup per episode; candidates <= 1024, kept in LDS; ranks by counting (n^2 / 256
// comparisons per thread: 264 candidates of the paper's setting = 272 per thread).
#ifndef SV_TREE_BUILD_H
#define SV_TREE_BUILD_H

#include "sv_internal.h"

namespace sv {

constexpr int kMaxCandidates = 1024;

// status[b]: 0 ok; bit 0 = a candidate's parent index is not an earlier candidate;
// bit 1 = a kept candidate is deeper than d_cap; bit 2 = a kept candidate's parent was not kept
// (log-probabilities above zero).  A flagged episode gets a root-only chain
// (every node a child of the root) so that later calls stay in bounds.
__global__ __launch_bounds__(256) void tree_build_kernel(
    const int32_t* __restrict__ cand_parent, const float* __restrict__ cand_logp,
    const int32_t* __restrict__ cand_token, int n_cand, const int32_t* __restrict__ root_token,
    int T, int n_words, int d_cap, int32_t* __restrict__ parent, int32_t* __restrict__ depth,
    uint64_t* __restrict__ anc_mask, int32_t* __restrict__ draft_token, int32_t* __restrict__ status) {
  __shared__ float s_score[kMaxCandidates];
  __shared__ int s_par[kMaxCandidates];
  __shared__ short s_depth[kMaxCandidates];
  __shared__ short s_node[kMaxCandidates];     // node index of a kept candidate, -1 otherwise
  __shared__ int s_bad;
  const int b = blockIdx.x, tid = threadIdx.x;
  const int32_t* cp = cand_parent + (size_t)b * n_cand;
  const float* lp = cand_logp + (size_t)b * n_cand;
  const int n_keep = T - 1;
  if (tid == 0) s_bad = 0;
  for (int c = tid; c < n_cand; c += 256) {
    const int p = cp[c];
    s_par[c] = p;
    if (p < -1 || p >= c) atomicOr(&s_bad, 1);
  }
  __syncthreads();
  if (s_bad == 0) {
    // score and depth of candidate c: walk up to the root, then add the log-probabilities
    // from the root down (the order of the sequential definition)
    for (int c = tid; c < n_cand; c += 256) {
      int path[SV_MAX_DEPTH + 1];
      int len = 0, node = c;
      while (node >= 0 && len <= SV_MAX_DEPTH) {
        path[len++] = node;
        node = s_par[node];
      }
      if (node >= 0) {                 // deeper than any tree this library takes
        s_depth[c] = (short)(SV_MAX_DEPTH + 1);
        s_score[c] = -__builtin_inff();
      } else {
        float sc = 0.f;
        for (int i = len - 1; i >= 0; --i) sc = sc + lp[path[i]];
        s_depth[c] = (short)len;
        s_score[c] = sc == sc ? sc : -__builtin_inff();   // NaN sorts last: the order stays total

      }
    }
    __syncthreads();
    // rank among all candidates: higher score first, lower index first on ties
    for (int c = tid; c < n_cand; c += 256) {
      const float sc = s_score[c];
      int rank = 0;
      for (int j = 0; j < n_cand; ++j) {
        const float sj = s_score[j];
        rank += (sj > sc || (sj == sc && j < c)) ? 1 : 0;
      }
      s_node[c] = rank < n_keep ? (short)0 : (short)-1;
      if (rank < n_keep && s_depth[c] > d_cap) atomicOr(&s_bad, 2);
    }
    __syncthreads();
    // log-probabilities above zero can rank a child before its parent: not a tree
    for (int c = tid; c < n_cand; c += 256)
      if (s_node[c] >= 0 && s_par[c] >= 0 && s_node[s_par[c]] < 0) atomicOr(&s_bad, 4);
    __syncthreads();
  }
  int32_t* par_o = parent + (size_t)b * T;
  int32_t* dep_o = depth + (size_t)b * T;
  int32_t* tok_o = draft_token + (size_t)b * T;
  uint64_t* anc_o = anc_mask + (size_t)b * T * n_words;
  if (s_bad != 0) {
    for (int i = tid; i < T; i += 256) {
      par_o[i] = i == 0 ? -1 : 0;
      dep_o[i] = i == 0 ? 0 : 1;
      tok_o[i] = root_token[b];
      for (int w = 0; w < n_words; ++w) anc_o[(size_t)i * n_words + w] = 0;
      anc_o[(size_t)i * n_words + (i >> 6)] |= 1ull << (i & 63);
      anc_o[(size_t)i * n_words] |= 1ull;
    }
    if (tid == 0) status[b] = s_bad;
    return;
  }
  // breadth-first number of a kept candidate: 1 + kept candidates before it in (depth, index)
  for (int c = tid; c < n_cand; c += 256) {
    if (s_node[c] < 0) continue;
    const int dc = s_depth[c];
    int before = 0;
    for (int j = 0; j < n_cand; ++j) {
      const int dj = s_depth[j];
      before += (s_node[j] >= 0 && (dj < dc || (dj == dc && j < c))) ? 1 : 0;
    }
    // s_node of kept candidates is only tested for >= 0 by the other threads, so writing the
    // final (>= 1) number here does not disturb their counts
    s_node[c] = (short)(1 + before);
  }
  __syncthreads();
  if (tid == 0) {
    par_o[0] = -1;
    dep_o[0] = 0;
    tok_o[0] = root_token[b];
    for (int w = 0; w < n_words; ++w) anc_o[w] = 0;
    anc_o[0] = 1ull;
    status[b] = 0;
  }
  const int32_t* tk = cand_token + (size_t)b * n_cand;
  for (int c = tid; c < n_cand; c += 256) {
    const int i = s_node[c];
    if (i < 1) continue;
    const int p = s_par[c];
    par_o[i] = p < 0 ? 0 : s_node[p];
    dep_o[i] = s_depth[c];
    tok_o[i] = tk[c];
    uint64_t m[2] = {1ull, 0ull};                      // the root
    for (int node = c; node >= 0; node = s_par[node]) {
      const int ni = s_node[node];
      m[ni >> 6] |= 1ull << (ni & 63);
    }
    for (int w = 0; w < n_words; ++w) anc_o[(size_t)i * n_words + w] = m[w];
  }
}

}  // namespace sv
#endif
