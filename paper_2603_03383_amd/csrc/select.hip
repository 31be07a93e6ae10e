// Selection kernels: per-row argmax, per-row top-k, candidate -> tree-node gather, and greedy
// longest-prefix acceptance over the static retrieve table (Section 3.2, "Zero-Copy Retrieval
// Strategy": the best path is chosen on the device and its tokens are gathered through the table).
// All orderings are total (value descending, then index ascending), so results do not depend on the
// reduction order.
#include "kernels.h"

namespace mdz {

struct Best {
  float v;
  int i;
};
// a precedes b in (value descending, index ascending) order
__device__ inline bool precedes(float av, int ai, float bv, int bi) { return av > bv || (av == bv && ai < bi); }

__device__ inline Best wave_best(Best a) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(a.v, o, 64);
    int oi = __shfl_xor(a.i, o, 64);
    if (precedes(ov, oi, a.v, a.i)) {
      a.v = ov;
      a.i = oi;
    }
  }
  return a;
}

// blockDim.x == 256; result valid in every thread
__device__ inline Best block_best_256(Best a, Best* smem4) {
  a = wave_best(a);
  if ((threadIdx.x & 63) == 0) smem4[threadIdx.x >> 6] = a;
  __syncthreads();
  Best r = smem4[0];
#pragma unroll
  for (int w = 1; w < 4; ++w)
    if (precedes(smem4[w].v, smem4[w].i, r.v, r.i)) r = smem4[w];
  __syncthreads();
  return r;
}

constexpr int kNoIndex = 0x7FFFFFFF;

// One block per row. Pass p selects the best element that strictly follows the previous pick.
__global__ void __launch_bounds__(256) topk_kernel(const float* __restrict__ logits, int V, int64_t ld, int k,
                                                   int32_t* __restrict__ out, int64_t out_ld) {
  __shared__ Best red[4];
  const float* row = logits + (int64_t)blockIdx.x * ld;
  float pv = INFINITY;
  int pi = -1;
  for (int p = 0; p < k; ++p) {
    Best b{-INFINITY, kNoIndex};
    for (int i = threadIdx.x; i < V; i += 256) {
      float v = row[i];
      bool after_prev = (p == 0) || precedes(pv, pi, v, i);
      if (after_prev && precedes(v, i, b.v, b.i)) {
        b.v = v;
        b.i = i;
      }
    }
    b = block_best_256(b, red);
    if (threadIdx.x == 0) out[(int64_t)blockIdx.x * out_ld + p] = b.i == kNoIndex ? -1 : b.i;
    pv = b.v;
    pi = b.i;
  }
}

int launch_topk(const float* logits, int rows, int V, int64_t ld, int k, int32_t* out, int64_t out_ld,
                hipStream_t st) {
  ProfScope prof_(PROF_SELECT, st);
  if (rows == 0 || k == 0) return MDZ_OK;
  topk_kernel<<<rows, 256, 0, st>>>(logits, V, ld, k, out, out_ld);
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

int launch_argmax(const float* logits, int rows, int V, int64_t ld, int32_t* out, hipStream_t st) {
  return launch_topk(logits, rows, V, ld, 1, out, 1, st);
}

__global__ void scatter_i32_kernel(const int32_t* __restrict__ src, int32_t* __restrict__ dst, int n,
                                   int64_t dst_stride) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i * dst_stride] = src[i];
}

int launch_scatter_i32(const int32_t* src, int32_t* dst, int n, int64_t dst_stride, hipStream_t st) {
  ProfScope prof_(PROF_SELECT, st);
  if (n == 0) return MDZ_OK;
  scatter_i32_kernel<<<(n + 63) / 64, 64, 0, st>>>(src, dst, n, dst_stride);
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

__global__ void tree_tokens_kernel(int tree, const int32_t* __restrict__ cand_flat, int32_t* __restrict__ tree_tokens,
                                   int B) {
  const TreeTables& t = c_trees[tree];
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= B * t.T) return;
  int b = idx / t.T, n = idx % t.T;
  tree_tokens[idx] = cand_flat[b * t.n_cand + t.cand_slot[n]];
}

int launch_tree_tokens(int tree, const int32_t* cand_flat, int32_t* tree_tokens, int B, hipStream_t st) {
  ProfScope prof_(PROF_SELECT, st);
  const TreeTables* t = host_tree(tree);
  int total = B * t->T;
  if (total == 0) return MDZ_OK;
  tree_tokens_kernel<<<(total + 255) / 256, 256, 0, st>>>(tree, cand_flat, tree_tokens, B);
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

// One wave per sequence; lane p evaluates path p of the retrieve table (n_paths <= 64).  The winner
// is the longest match, ties to the lowest path index; lane 0 writes the fixed-shape outputs.
__global__ void __launch_bounds__(64) accept_kernel(int tree, const int32_t* __restrict__ tree_tokens,
                                                    const int32_t* __restrict__ node_argmax,
                                                    int32_t* __restrict__ accept_len, int32_t* __restrict__ best_path,
                                                    int32_t* __restrict__ acc_nodes, int32_t* __restrict__ acc_tokens,
                                                    int32_t* __restrict__ next_root, int32_t* __restrict__ last_node) {
  const TreeTables& t = c_trees[tree];
  int b = blockIdx.x;
  int p = threadIdx.x;
  const int32_t* tok = tree_tokens + b * t.T;
  const int32_t* am = node_argmax + b * t.T;
  int len = 0;
  if (p < t.n_paths) {
    for (int c = 0; c <= t.K; ++c) {
      int n = t.retrieve[p][c];
      if (n < 0) break;
      if (n != 0 && tok[n] != am[t.parent[n]]) break;
      ++len;
    }
  }
  // key: longer first, then lower path index
  int key = len * 64 + (63 - p);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) key = max(key, __shfl_xor(key, o, 64));
  int A = key / 64, best = 63 - key % 64;
  if (p == 0) {
    accept_len[b] = A;
    best_path[b] = best;
    int last = 0;
    for (int c = 0; c <= t.K; ++c) {
      int n = c < A ? t.retrieve[best][c] : -1;
      acc_nodes[b * (t.K + 1) + c] = n;
      acc_tokens[b * (t.K + 1) + c] = n >= 0 ? tok[n] : -1;
      if (n >= 0) last = n;
    }
    last_node[b] = last;
    next_root[b] = am[last];
  }
}

int launch_accept(int tree, const int32_t* tree_tokens, const int32_t* node_argmax, int B, int32_t* accept_len,
                  int32_t* best_path, int32_t* acc_nodes, int32_t* acc_tokens, int32_t* next_root,
                  int32_t* last_node, hipStream_t st) {
  ProfScope prof_(PROF_ACCEPT, st);
  if (B == 0) return MDZ_OK;
  accept_kernel<<<B, 64, 0, st>>>(tree, tree_tokens, node_argmax, accept_len, best_path, acc_nodes, acc_tokens,
                                  next_root, last_node);
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

}  // namespace mdz
