// Relaxed acceptance and longest accepted path: integer only, one workgroup per episode.
#ifndef SV_ACCEPT_H
#define SV_ACCEPT_H

#include "sv_internal.h"

namespace sv {

// Thread c owns tree node c (T <= 128 = block size).
//  1. own test: |bin(draft[c]) - bin(target[parent[c]])| <= r, both inside the action range;
//     the root passes by definition.  The results are gathered into a bitmask by ballot.
//  2. a node is accepted when no node on its root path failed: its ancestor-or-self mask
//     ANDed with the complement of the pass mask is empty (this is the scan of Alg. 1 that
//     stops at the first rejection, evaluated for all paths at once).
//  3. best = accepted node of greatest depth, lowest index among equals, found with an
//     integer max over the key (depth << 8 | 255 - c).
//  4. the nodes of best's ancestor mask write themselves into path[depth] and their draft
//     token into out_tokens[depth - 1]; the verifier's token of best closes the list.
__global__ __launch_bounds__(128) void relaxed_accept_kernel(
    const int32_t* __restrict__ parent, const int32_t* __restrict__ depth,
    const uint64_t* __restrict__ anc, int T, int n_words, const int32_t* __restrict__ draft,
    const int32_t* __restrict__ target, int action_lo, int n_bins, int r, int d_cap,
    uint8_t* __restrict__ accept_mask, int32_t* __restrict__ accepted_len,
    int32_t* __restrict__ best_node, int32_t* __restrict__ path,
    int32_t* __restrict__ out_tokens) {
  __shared__ unsigned long long pass_bits[2];
  __shared__ int best_key;
  const int b = blockIdx.x;
  const int c = threadIdx.x;
  const size_t base = (size_t)b * T;
  if (c == 0) best_key = 0;
  for (int i = c; i <= d_cap; i += 128) {
    path[(size_t)b * (d_cap + 1) + i] = -1;
    out_tokens[(size_t)b * (d_cap + 1) + i] = -1;
  }

  bool pass = false;
  int dep = 0;
  if (c < T) {
    dep = depth[base + c];
    if (c == 0) {
      pass = true;
      dep = 0;
    } else {
      int p = parent[base + c];
      p = p < 0 ? 0 : (p >= T ? T - 1 : p);
      const long long bd = (long long)draft[base + c] - action_lo;
      const long long bt = (long long)target[base + p] - action_lo;
      const long long diff = bd > bt ? bd - bt : bt - bd;
      pass = bd >= 0 && bd < n_bins && bt >= 0 && bt < n_bins && diff <= r &&
             dep >= 0 && dep <= d_cap;
    }
  }
  const unsigned long long ballot = __ballot(pass);
  if ((c & 63) == 0) pass_bits[c >> 6] = ballot;
  __syncthreads();

  bool acc = false;
  if (c < T) {
    unsigned long long blocked = 0;
    for (int w = 0; w < n_words; ++w) blocked |= anc[(base + c) * n_words + w] & ~pass_bits[w];
    acc = blocked == 0;
    accept_mask[base + c] = acc ? 1 : 0;
    if (acc) atomicMax(&best_key, (dep << 8) | (255 - c));
  }
  __syncthreads();
  const int key = best_key;                 // the root always contributes key 255
  const int best = 255 - (key & 255);
  const int len = key >> 8;
  if (c < T) {
    const unsigned long long word = anc[(base + best) * n_words + (c >> 6)];
    if (((word >> (c & 63)) & 1ull) && dep >= 0 && dep <= d_cap) {
      path[(size_t)b * (d_cap + 1) + dep] = c;
      if (c > 0 && dep >= 1) out_tokens[(size_t)b * (d_cap + 1) + dep - 1] = draft[base + c];
    }
  }
  if (c == 0) {
    accepted_len[b] = len;
    best_node[b] = best;
    out_tokens[(size_t)b * (d_cap + 1) + len] = target[base + best];
  }
}

// Commit of the accepted path (the step of Alg. 1 between two verification passes): the K/V
// rows of the accepted nodes, appended at cache rows P + node, move to rows P + depth, so that
// the cache again holds one contiguous prefix; the root (depth 0) already sits at row P.
// Moves run in increasing depth with a barrier in between: node index >= depth, so a row is
// read before a later move overwrites it.  grid = (B, n_heads), block = 128.
template <typename TKV>
__global__ __launch_bounds__(128) void commit_path_kernel(
    TKV* __restrict__ kc, TKV* __restrict__ vc, const int32_t* __restrict__ prefix_len, int p_max,
    int cap, int T, int nh, int d, const int32_t* __restrict__ path,
    const int32_t* __restrict__ accepted_len, int d_cap) {
  const int b = blockIdx.x, h = blockIdx.y;
  int P = prefix_len[b];
  P = P < 0 ? 0 : (P > p_max ? p_max : P);
  int len = accepted_len[b];
  len = len < 0 ? 0 : (len > d_cap ? d_cap : len);
  TKV* kb = kc + ((size_t)b * nh + h) * cap * d;
  TKV* vb = vc + ((size_t)b * nh + h) * cap * d;
  for (int i = 1; i <= len; ++i) {
    const int node = path[(size_t)b * (d_cap + 1) + i];
    if (node > i && node < T) {              // node == i: already in place
      for (int e = threadIdx.x; e < d; e += 128) {
        kb[(size_t)(P + i) * d + e] = kb[(size_t)(P + node) * d + e];
        vb[(size_t)(P + i) * d + e] = vb[(size_t)(P + node) * d + e];
      }
    }
    __syncthreads();
  }
}

// prefix_len[b] += accepted_len[b] + 1 (the root and the accepted draft tokens are now prefix).
__global__ void advance_prefix_kernel(int32_t* __restrict__ prefix_len,
                                      const int32_t* __restrict__ accepted_len, int B, int d_cap) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  int len = accepted_len[b];
  len = len < 0 ? 0 : (len > d_cap ? d_cap : len);
  prefix_len[b] += len + 1;
}

}  // namespace sv
#endif
