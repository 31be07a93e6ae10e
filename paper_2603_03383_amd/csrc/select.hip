// Selection kernels: per-row argmax, per-row top-k, candidate -> tree-node gather, and greedy
// longest-prefix acceptance over the static retrieve table (Section 3.2, "Zero-Copy Retrieval
// Strategy": the best path is chosen on the device and its tokens are gathered through the table).
// All orderings are total (value descending, then index ascending), so results do not depend on the
// reduction order.
#include "kernels.h"

namespace mdz {

typedef ArgCand Best;

// Best of the wave's 64 candidates, in every lane.  Within a row of 16 lanes the exchange runs on data-parallel
// primitives (lane ^ 1, lane ^ 2 by quad permutation, then the mirrored lane of the half row and of the row: four
// steps after which a row agrees); the four row results are read as scalars and combined.  (Twelve LDS-crossbar
// permutes per call, as __shfl_xor compiles to, made the k sequential picks of a top-k cost microseconds.)
__device__ inline Best wave_best(Best a) {
  auto take = [&](float ov, int oi) {
    if (precedes(ov, oi, a.v, a.i)) a.v = ov, a.i = oi;
  };
#define MDZ_DPP_STEP(CTRL)                                                                                      \
  take(__int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(a.v), CTRL, 0xF, 0xF, false)),             \
       __builtin_amdgcn_update_dpp(0, a.i, CTRL, 0xF, 0xF, false))
  MDZ_DPP_STEP(0xB1);   // quad_perm [1,0,3,2]
  MDZ_DPP_STEP(0x4E);   // quad_perm [2,3,0,1]
  MDZ_DPP_STEP(0x141);  // row_half_mirror
  MDZ_DPP_STEP(0x140);  // row_mirror
#undef MDZ_DPP_STEP
  Best r{__int_as_float(__builtin_amdgcn_readlane(__float_as_int(a.v), 0)), __builtin_amdgcn_readlane(a.i, 0)};
#pragma unroll
  for (int row = 1; row < 4; ++row) {
    const float ov = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(a.v), 16 * row));
    const int oi = __builtin_amdgcn_readlane(a.i, 16 * row);
    if (precedes(ov, oi, r.v, r.i)) r = Best{ov, oi};
  }
  return r;
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

// One workgroup per row: the best of the row's candidates (pairs left by the LM-head GEMM's argmax epilogue, one per
// workgroup and wave; index kNoIndex = empty).
__global__ void __launch_bounds__(256) argmax_merge_kernel(const ArgCand* __restrict__ cand, int n_cand,
                                                           int32_t* __restrict__ out) {
  __shared__ Best smem4[4];
  const int row = blockIdx.x;
  Best b{-INFINITY, kNoIndex};
  for (int c = threadIdx.x; c < n_cand; c += 256) {
    const Best h = cand[(int64_t)row * n_cand + c];
    if (h.i != kNoIndex && precedes(h.v, h.i, b.v, b.i)) b = h;
  }
  b = block_best_256(b, smem4);
  if (threadIdx.x == 0) out[row] = b.i == kNoIndex ? -1 : b.i;
}

int launch_argmax_merge(const ArgCand* cand, int rows, int n_cand, int32_t* out, hipStream_t st) {
  ProfScope prof_(PROF_SELECT, st);
  if (rows == 0) return MDZ_OK;
  argmax_merge_kernel<<<rows, 256, 0, st>>>(cand, n_cand, out);
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

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

// ---- two-stage variant for long rows ----------------------------------------------------------------------------
// Stage 1: every wave takes one chunk of 512 columns (8 per lane, in registers) and extracts its top-k, in order, with
// wave-level exchanges alone (no LDS, no barriers).  Stage 2: one wave per row merges the chunk lists (see below).
// The top-k of a union of top-k lists is the global top-k and the order is total (value descending, index
// ascending), so the result equals the single-stage kernel's.
// Rows come in two flavours: uniform (every row the same k, picks to out + row * out_ld) and heads (row (b, j) of
// logits [B][K+1][V]: j = 0 the base LM head, whose argmax is the root candidate unless the caller gave root
// tokens, j = 1..K Medusa head j with its own k = caps[j-1]; picks go straight to the row's segment of
// cand_flat [B][n_cand] = [root | head 1 | .. | head K]: one pair of launches for all heads of all sequences).
constexpr int kSelWaveCols = 512;   // columns per stage-1 chunk
constexpr int kSelMaxChunks = 512;  // rows of up to 262144 columns
constexpr int kSelMaxK = 16;        // candidates per chunk list (the lists are laid out for this many)
static int sel_chunks(int V) { return (V + kSelWaveCols - 1) / kSelWaveCols; }

struct SelRows {
  int tree;        // >= 0: heads flavour over this tree; -1: uniform
  int k;           // uniform: picks per row
  int64_t ld;      // uniform: row stride of the logits (heads: V)
  int64_t out_ld;  // uniform: row stride of the output
  bool have_root;  // heads: the caller supplies the root candidates
};
__device__ inline int sel_row_k(const SelRows& rs, int row) {
  if (rs.tree < 0) return rs.k;
  const TreeTables& t = c_trees[rs.tree];
  const int j = row % (t.K + 1);
  return j == 0 ? (rs.have_root ? 0 : 1) : t.caps[j - 1];
}

__global__ void __launch_bounds__(256) topk_stage1_kernel(SelRows rs, const float* __restrict__ logits, int V, int n_chunks,
                                                          float* __restrict__ cand_v, int32_t* __restrict__ cand_i) {
  const int lane = threadIdx.x & 63, chunk = blockIdx.x * 4 + (threadIdx.x >> 6), row = blockIdx.y;
  const int k = sel_row_k(rs, row);
  if (chunk >= n_chunks || k == 0) return;
  const int c0 = chunk * kSelWaveCols;
  const float* src = logits + (int64_t)row * (rs.tree < 0 ? rs.ld : (int64_t)V);
  float v[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int i = c0 + lane + j * 64;
    v[j] = i < V ? src[i] : -INFINITY;
  }
  const int64_t o = ((int64_t)row * n_chunks + chunk) * kSelMaxK;
  float pv = INFINITY;
  int pi = -1;
  for (int p = 0; p < k; ++p) {
    Best b{-INFINITY, kNoIndex};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int i = c0 + lane + j * 64;
      const bool ok = i < V && (p == 0 || precedes(pv, pi, v[j], i));
      if (ok && precedes(v[j], i, b.v, b.i)) b = Best{v[j], i};
    }
    b = wave_best(b);
    if (lane == 0) cand_v[o + p] = b.v, cand_i[o + p] = b.i;
    pv = b.v;
    pi = b.i;
  }
}

// One wave per row.  Every chunk list is already in order, so the row's next pick is the best of the lists' current
// heads: the lists are staged in LDS, every lane owns up to 8 of them (512 lists at most), offers the best of its
// heads, the wave picks, and the lane that owned the pick advances that list.
__global__ void __launch_bounds__(64) topk_stage2_kernel(SelRows rs, const float* __restrict__ cand_v,
                                                         const int32_t* __restrict__ cand_i, int n_chunks,
                                                         const int32_t* __restrict__ root_token, int32_t* __restrict__ out) {
  extern __shared__ __attribute__((aligned(8))) uint8_t sel_lds[];  // [n_chunks][k] values, then indices
  const int lane = threadIdx.x, row = blockIdx.x;
  const int k = sel_row_k(rs, row);
  int32_t* dst;
  if (rs.tree < 0) {
    dst = out + (int64_t)row * rs.out_ld;
  } else {
    const TreeTables& t = c_trees[rs.tree];
    const int b = row / (t.K + 1), j = row % (t.K + 1);
    int seg = 0;  // start of row j's segment in the flat candidate buffer
    for (int i = 1; i <= j; ++i) seg += i == 1 ? 1 : t.caps[i - 2];
    dst = out + (int64_t)b * t.n_cand + seg;
    if (k == 0) {
      if (lane == 0) dst[0] = root_token[b];
      return;
    }
  }
  float* lv = reinterpret_cast<float*>(sel_lds);
  int* li = reinterpret_cast<int*>(sel_lds) + n_chunks * k;
  const float* cv = cand_v + (int64_t)row * n_chunks * kSelMaxK;
  const int32_t* ci = cand_i + (int64_t)row * n_chunks * kSelMaxK;
  for (int c = lane; c < n_chunks; c += 64)
    for (int q = 0; q < k; ++q) lv[c * k + q] = cv[c * kSelMaxK + q], li[c * k + q] = ci[c * kSelMaxK + q];
  __syncthreads();
  int pos[kSelMaxChunks / 64];  // next entry of the lane's lists lane, lane + 64, ...
#pragma unroll
  for (int j = 0; j < kSelMaxChunks / 64; ++j) pos[j] = 0;
  for (int p = 0; p < k; ++p) {
    Best b{-INFINITY, kNoIndex};
#pragma unroll
    for (int j = 0; j < kSelMaxChunks / 64; ++j) {
      const int c = lane + 64 * j;
      if (c < n_chunks && pos[j] < k) {
        const Best h{lv[c * k + pos[j]], li[c * k + pos[j]]};
        if (h.i != kNoIndex && precedes(h.v, h.i, b.v, b.i)) b = h;
      }
    }
    const Best w = wave_best(b);
    if (lane == 0) dst[p] = w.i == kNoIndex ? -1 : w.i;
    if (w.i != kNoIndex && w.i == b.i) {  // column ids are unique: this lane owns the pick; advance its list
#pragma unroll
      for (int j = 0; j < kSelMaxChunks / 64; ++j) {
        const int c = lane + 64 * j;
        if (c < n_chunks && pos[j] < k && li[c * k + pos[j]] == w.i) ++pos[j];
      }
    }
  }
}

// bytes of candidate lists for `rows` rows (sized for the largest chunk count, so independent of the row length)
int64_t topk_scratch_bytes(int rows) { return (int64_t)rows * kSelMaxChunks * kSelMaxK * 8; }

static bool two_stage_ok(int rows, int V, int k, const void* scratch, int64_t scratch_bytes) {
  return V >= 8192 && sel_chunks(V) <= kSelMaxChunks && k <= kSelMaxK && scratch &&
         scratch_bytes >= (int64_t)rows * sel_chunks(V) * kSelMaxK * 8;
}

static int launch_two_stage(const SelRows& rs, const float* logits, int rows, int V, const int32_t* root_token,
                            int32_t* out, void* scratch, hipStream_t st) {
  const int n_chunks = sel_chunks(V);
  float* cv = (float*)scratch;
  int32_t* ci = (int32_t*)(cv + (int64_t)rows * n_chunks * kSelMaxK);
  topk_stage1_kernel<<<dim3((n_chunks + 3) / 4, rows), 256, 0, st>>>(rs, logits, V, n_chunks, cv, ci);
  MDZ_LAUNCH_CHECK();
  const int kmax = rs.tree < 0 ? rs.k : kSelMaxK;
  topk_stage2_kernel<<<rows, 64, (size_t)n_chunks * kmax * 8, st>>>(rs, cv, ci, n_chunks, root_token, out);
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

int launch_topk(const float* logits, int rows, int V, int64_t ld, int k, int32_t* out, int64_t out_ld, void* scratch,
                int64_t scratch_bytes, hipStream_t st) {
  ProfScope prof_(PROF_SELECT, st);
  if (rows == 0 || k == 0) return MDZ_OK;
  if (two_stage_ok(rows, V, k, scratch, scratch_bytes))
    return launch_two_stage(SelRows{-1, k, ld, out_ld, false}, logits, rows, V, nullptr, out, scratch, st);
  topk_kernel<<<rows, 256, 0, st>>>(logits, V, ld, k, out, out_ld);
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

// true if launch_heads_select can serve this shape with this much scratch (else the caller selects head by head)
bool heads_select_supported(int tree, int B, int V, const void* scratch, int64_t scratch_bytes) {
  const TreeTables* t = host_tree(tree);
  int kmax = 1;
  for (int k = 0; k < t->K; ++k) kmax = t->caps[k] > kmax ? t->caps[k] : kmax;
  return two_stage_ok(B * (t->K + 1), V, kmax, scratch, scratch_bytes);
}

int launch_heads_select(int tree, const float* logits, int B, int V, const int32_t* root_token, int32_t* cand_flat,
                        void* scratch, hipStream_t st) {
  ProfScope prof_(PROF_SELECT, st);
  const TreeTables* t = host_tree(tree);
  const int rows = B * (t->K + 1);
  if (rows == 0) return MDZ_OK;
  return launch_two_stage(SelRows{tree, 0, 0, 0, root_token != nullptr}, logits, rows, V, root_token, cand_flat, scratch, st);
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
