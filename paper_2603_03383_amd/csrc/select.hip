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

// ---- two-stage variant for long rows: stage 1 finds the top-k of each of n_chunks column chunks (elements
// held in registers; n_chunks = 64, or more for rows longer than 131072), stage 2 merges the n_chunks*k candidates.  The top-k of the union of per-chunk top-k
// lists is the global top-k, and the order is total, so the result equals the single-stage kernel's.
constexpr int kSelChunks = 64;      // chunks per row, at least
constexpr int kSelMaxChunks = 256;  // and at most: rows of up to 524288 columns
constexpr int kSelPerThread = 8;    // stage 1 covers chunks of up to 256*8 = 2048 columns
static int sel_chunks(int V) {
  const int need = (V + 256 * kSelPerThread - 1) / (256 * kSelPerThread);
  return need > kSelChunks ? need : kSelChunks;
}

__global__ void __launch_bounds__(256) topk_stage1_kernel(const float* __restrict__ logits, int V, int64_t ld, int k,
                                                          float* __restrict__ cand_v, int32_t* __restrict__ cand_i) {
  __shared__ Best red[4];
  const int chunk = blockIdx.x, row = blockIdx.y, n_chunks = gridDim.x;
  const int per = (V + n_chunks - 1) / n_chunks;
  const int c0 = chunk * per, c1 = min(c0 + per, V);
  const float* src = logits + (int64_t)row * ld;
  float v[kSelPerThread];
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) {
    int i = c0 + threadIdx.x + j * 256;
    v[j] = i < c1 ? src[i] : -INFINITY;
  }
  float pv = INFINITY;
  int pi = -1;
  for (int p = 0; p < k; ++p) {
    Best b{-INFINITY, kNoIndex};
#pragma unroll
    for (int j = 0; j < kSelPerThread; ++j) {
      int i = c0 + threadIdx.x + j * 256;
      bool ok = i < c1 && (p == 0 || precedes(pv, pi, v[j], i));
      if (ok && precedes(v[j], i, b.v, b.i)) {
        b.v = v[j];
        b.i = i;
      }
    }
    b = block_best_256(b, red);
    if (threadIdx.x == 0) {
      int64_t o = ((int64_t)row * n_chunks + chunk) * k + p;
      cand_v[o] = b.v;
      cand_i[o] = b.i;
    }
    pv = b.v;
    pi = b.i;
  }
}

__global__ void __launch_bounds__(256) topk_stage2_kernel(const float* __restrict__ cand_v,
                                                          const int32_t* __restrict__ cand_i, int k, int n_chunks,
                                                          int32_t* __restrict__ out, int64_t out_ld) {
  __shared__ Best red[4];
  const int row = blockIdx.x;
  const int n = n_chunks * k;
  const float* cv = cand_v + (int64_t)row * n;
  const int32_t* ci = cand_i + (int64_t)row * n;
  float pv = INFINITY;
  int pi = -1;
  for (int p = 0; p < k; ++p) {
    Best b{-INFINITY, kNoIndex};
    for (int j = threadIdx.x; j < n; j += 256) {
      float v = cv[j];
      int i = ci[j];
      bool ok = i != kNoIndex && (p == 0 || precedes(pv, pi, v, i));
      if (ok && precedes(v, i, b.v, b.i)) {
        b.v = v;
        b.i = i;
      }
    }
    b = block_best_256(b, red);
    if (threadIdx.x == 0) out[(int64_t)row * out_ld + p] = b.i == kNoIndex ? -1 : b.i;
    pv = b.v;
    pi = b.i;
  }
}

// (sized for the largest chunk count, so it does not depend on the row length)
int64_t topk_scratch_bytes(int rows, int k) { return (int64_t)rows * kSelMaxChunks * k * 8; }

int launch_topk(const float* logits, int rows, int V, int64_t ld, int k, int32_t* out, int64_t out_ld, void* scratch,
                int64_t scratch_bytes, hipStream_t st) {
  ProfScope prof_(PROF_SELECT, st);
  if (rows == 0 || k == 0) return MDZ_OK;
  const int n_chunks = sel_chunks(V);
  if (V >= 8192 && n_chunks <= kSelMaxChunks && scratch && scratch_bytes >= topk_scratch_bytes(rows, k)) {
    float* cv = (float*)scratch;
    int32_t* ci = (int32_t*)(cv + (int64_t)rows * n_chunks * k);
    topk_stage1_kernel<<<dim3(n_chunks, rows), 256, 0, st>>>(logits, V, ld, k, cv, ci);
    MDZ_LAUNCH_CHECK();
    topk_stage2_kernel<<<rows, 256, 0, st>>>(cv, ci, k, n_chunks, out, out_ld);
  } else {
    topk_kernel<<<rows, 256, 0, st>>>(logits, V, ld, k, out, out_ld);
  }
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

// ---- all heads of all sequences in one pair of launches --------------------------------------------------------
// Row (b, j) of logits [B][K+1][V]: j = 0 is the base LM head (its argmax is the root candidate unless the caller
// gave root tokens), j = 1..K Medusa head j with its own top-k size caps[j-1].  The picks go straight to their
// segment of cand_flat [B][n_cand] = [root | head 1 | .. | head K].  Same two stages and the same total order as
// above, so the result equals per-head launches; it replaces 2 (K + 1) launches of ~10 us each by 2.
constexpr int kHeadsMaxK = 16;  // largest per-head top-k the stage-1 buffer is laid out for
__device__ inline int heads_row_k(const TreeTables& t, int j, bool have_root) { return j == 0 ? (have_root ? 0 : 1) : t.caps[j - 1]; }

__global__ void __launch_bounds__(256) heads_topk_stage1_kernel(int tree, const float* __restrict__ logits, int V,
                                                                bool have_root, float* __restrict__ cand_v,
                                                                int32_t* __restrict__ cand_i) {
  __shared__ Best red[4];
  const TreeTables& t = c_trees[tree];
  const int chunk = blockIdx.x, row = blockIdx.y, n_chunks = gridDim.x;
  const int k = heads_row_k(t, row % (t.K + 1), have_root);
  if (k == 0) return;
  const int per = (V + n_chunks - 1) / n_chunks;
  const int c0 = chunk * per, c1 = min(c0 + per, V);
  const float* src = logits + (int64_t)row * V;
  float v[kSelPerThread];
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) {
    int i = c0 + threadIdx.x + j * 256;
    v[j] = i < c1 ? src[i] : -INFINITY;
  }
  float pv = INFINITY;
  int pi = -1;
  for (int p = 0; p < k; ++p) {
    Best b{-INFINITY, kNoIndex};
#pragma unroll
    for (int j = 0; j < kSelPerThread; ++j) {
      int i = c0 + threadIdx.x + j * 256;
      bool ok = i < c1 && (p == 0 || precedes(pv, pi, v[j], i));
      if (ok && precedes(v[j], i, b.v, b.i)) {
        b.v = v[j];
        b.i = i;
      }
    }
    b = block_best_256(b, red);
    if (threadIdx.x == 0) {
      int64_t o = ((int64_t)row * n_chunks + chunk) * kHeadsMaxK + p;
      cand_v[o] = b.v;
      cand_i[o] = b.i;
    }
    pv = b.v;
    pi = b.i;
  }
}

__global__ void __launch_bounds__(256) heads_topk_stage2_kernel(int tree, const float* __restrict__ cand_v,
                                                                const int32_t* __restrict__ cand_i, int n_chunks,
                                                                const int32_t* __restrict__ root_token,
                                                                int32_t* __restrict__ cand_flat) {
  __shared__ Best red[4];
  const TreeTables& t = c_trees[tree];
  const int row = blockIdx.x, b = row / (t.K + 1), j = row % (t.K + 1);
  int seg = 0;  // start of row j's segment in the flat candidate buffer
  for (int i = 1; i <= j; ++i) seg += i == 1 ? 1 : t.caps[i - 2];
  int32_t* out = cand_flat + (int64_t)b * t.n_cand + seg;
  const int k = heads_row_k(t, j, root_token != nullptr);
  if (k == 0) {
    if (threadIdx.x == 0) out[0] = root_token[b];
    return;
  }
  const float* cv = cand_v + (int64_t)row * n_chunks * kHeadsMaxK;
  const int32_t* ci = cand_i + (int64_t)row * n_chunks * kHeadsMaxK;
  const int n = n_chunks * k;
  float pv = INFINITY;
  int pi = -1;
  for (int p = 0; p < k; ++p) {
    Best bst{-INFINITY, kNoIndex};
    for (int e = threadIdx.x; e < n; e += 256) {
      const int at = (e / k) * kHeadsMaxK + e % k;
      float v = cv[at];
      int i = ci[at];
      bool ok = i != kNoIndex && (p == 0 || precedes(pv, pi, v, i));
      if (ok && precedes(v, i, bst.v, bst.i)) {
        bst.v = v;
        bst.i = i;
      }
    }
    bst = block_best_256(bst, red);
    if (threadIdx.x == 0) out[p] = bst.i == kNoIndex ? -1 : bst.i;
    pv = bst.v;
    pi = bst.i;
  }
}

// true if launch_heads_select can serve this shape with this much scratch (else the caller selects head by head)
bool heads_select_supported(int tree, int B, int V, int64_t scratch_bytes) {
  const TreeTables* t = host_tree(tree);
  int kmax = 1;
  for (int k = 0; k < t->K; ++k) kmax = t->caps[k] > kmax ? t->caps[k] : kmax;
  const int n_chunks = sel_chunks(V);
  return V >= 8192 && n_chunks <= kSelMaxChunks && kmax <= kHeadsMaxK &&
         scratch_bytes >= (int64_t)B * (t->K + 1) * n_chunks * kHeadsMaxK * 8;
}

int launch_heads_select(int tree, const float* logits, int B, int V, const int32_t* root_token, int32_t* cand_flat,
                        void* scratch, hipStream_t st) {
  ProfScope prof_(PROF_SELECT, st);
  const TreeTables* t = host_tree(tree);
  const int rows = B * (t->K + 1);
  if (rows == 0) return MDZ_OK;
  const int n_chunks = sel_chunks(V);
  float* cv = (float*)scratch;
  int32_t* ci = (int32_t*)(cv + (int64_t)rows * n_chunks * kHeadsMaxK);
  heads_topk_stage1_kernel<<<dim3(n_chunks, rows), 256, 0, st>>>(tree, logits, V, root_token != nullptr, cv, ci);
  MDZ_LAUNCH_CHECK();
  heads_topk_stage2_kernel<<<rows, 256, 0, st>>>(tree, cv, ci, n_chunks, root_token, cand_flat);
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

int launch_argmax(const float* logits, int rows, int V, int64_t ld, int32_t* out, void* scratch, int64_t scratch_bytes,
                  hipStream_t st) {
  return launch_topk(logits, rows, V, ld, 1, out, 1, scratch, scratch_bytes, st);
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
