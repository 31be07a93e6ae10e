// Internal launch interface between the C-ABI layer (medusa_api.hip) and the kernel files.
// Every function enqueues on `st` and returns an mdz_status.  All pointers are device pointers.
#pragma once
#include "common.h"
#include "profile.h"

namespace mdz {

// Output of a GEMM: partial-sum slots, each [M][ld] fp32, `stride` elements apart.  The consumer adds slots
// 0..count-1 in that fixed order (results do not depend on scheduling).  count is `n` for every column when
// split_grid == 0.  Otherwise the GEMM cut its U = bands * n_stages (band, K-stage) units, numbered band-major,
// into split_grid equal contiguous ranges, range w = [floor(w*U/G), floor((w+1)*U/G)), and every range that
// touches a band wrote one slot of it: the count of a band follows from that arithmetic alone, so consumers
// need no table (and no dependent memory read) to know it.
struct Partials {
  const float* p;
  int n;  // slot count when split_grid == 0, else an upper bound
  int64_t stride;
  int64_t ld;
  int band_cols;             // columns per band
  int n_stages;              // K-stages per band
  uint32_t split_units;      // U
  uint32_t split_grid;       // G (0: every column has n slots)
  // owner of unit u: the range w with floor(w*U/G) <= u < floor((w+1)*U/G); U * G < 2^31 (checked by the GEMM)
  __host__ __device__ static inline uint32_t owner(uint32_t u, uint32_t U, uint32_t G) { return ((u + 1) * G - 1) / U; }
  __host__ __device__ inline int count(int col) const {
    if (split_grid == 0) return n;
    const uint32_t band = (uint32_t)col / (uint32_t)band_cols;
    return (int)(owner((band + 1) * n_stages - 1, split_units, split_grid) -
                 owner(band * n_stages, split_units, split_grid)) + 1;
  }
};
inline Partials single_slot(const float* p, int64_t stride, int64_t ld) { return Partials{p, p ? 1 : 0, stride, ld, 1, 1, 0, 0}; }

// ---- layout movers (layout.hip) ------------------------------------------------------------------
// to_f16: the source is bf16 and the packed copy holds the same values as binary16
int launch_pack_weight(int dtype, const void* src, int64_t n_rows, int64_t k, void* dst, int64_t dst_rows,
                       int64_t tile_offset, int64_t tile_stride, hipStream_t st, bool to_f16 = false);
int launch_kv_copy(int dtype, const KvGeom& g, void* kc, void* vc, int layer, int seq, int pos0, int n,
                   void* k_rows, void* v_rows, bool to_cache, hipStream_t st);
// status (nullable): device word that receives MDZ_STATUS_SEQ_RANGE when a length arrives out of range
int launch_kv_compact(int dtype, const KvGeom& g, void* kc, void* vc, int tree, const int32_t* acc_nodes,
                      const int32_t* accept_len, int32_t* seq_len, int32_t* kv_src_slots, int B,
                      int max_prefix, int32_t* status, hipStream_t st);
// zero fill by a kernel (bytes: any count; p 4-byte aligned)
int launch_fill_zero(void* p, int64_t bytes, hipStream_t st);

// ---- elementwise / small kernels (elementwise.hip) -------------------------------------------------
int launch_embed(int dtype, const void* embed, const int32_t* tokens, float* x, int rows, int d, int vocab,
                 hipStream_t st);
// x[r] += sum of partials (skipped if part.p == NULL); then xn[r] = x[r] * rsqrt(mean(x[r]^2) + eps) * g rounded
// to the storage dtype (skipped if xn == NULL); out_dtype >= 0 names another type for xn (binary16 beside bf16 gains)
int launch_residual_rmsnorm(int dtype, float* x, const Partials& part, const void* g, void* xn, int rows, int d,
                            float eps, hipStream_t st, int out_dtype = -1);
// the first norm of a verify pass (no residual update: xn = RMSNorm(x; g)) and the pass's RoPE table in ONE launch:
// cos/sin of (S_b + depth[n]) * base^(-2i/hd), evaluated in double: cs [B*T][hd/2][2] fp32; status (nullable)
// receives MDZ_STATUS_SEQ_RANGE when a length arrives out of range
int launch_first_norm_and_rope_table(int dtype, float* x, const void* g, void* xn, int rows, int d, float eps, int tree,
                                     const int32_t* seq_len, int B, int max_prefix, int head_dim, float rope_base, float* cs,
                                     int32_t* status, hipStream_t st);
// rotates q and k of qkv [B*T][3d] fp32 (given as partials); q -> q_out [B*T][d] storage dtype; k,v -> cache
// slots S_b + n
int launch_rope_kvwrite(int dtype, int tree, const Partials& qkv, const float* cs, void* q_out, const KvGeom& g,
                        void* kc, void* vc, int layer, const int32_t* seq_len, int B, int max_prefix,
                        hipStream_t st);
// u[m][f] = SiLU(gate) * up from the tile-interleaved gate/up GEMM output gu [M][2F] fp32
int launch_swiglu(int dtype, const Partials& gu, void* u, int M, int F, hipStream_t st);
// gathers row src_row[b] of hidden [B][Tsrc][d] into h [B][d] (same dtype)
int launch_gather_rows(int dtype, const void* hidden, const int32_t* src_row, int B, int Tsrc, int d, void* h,
                       hipStream_t st);
// z = h + SiLU(pre + b1) -> storage dtype
// z[k] = h + SiLU(sums of head k + bias of head k) for all n_heads Medusa heads in one launch: the partial sums of
// head k start part_head_stride floats after those of head k - 1 (same slot layout), or, part_head_stride < 0, are
// columns k*d .. of the [B][n_heads*d] output of one GEMM over the stacked matrices; z [n_heads][B][d]
struct HeadBiases {
  const void* p[MDZ_MAX_HEADS];
};
int launch_head_residual(int dtype, const void* h, const Partials& pre, int64_t part_head_stride, const HeadBiases& b1s,
                         int n_heads, void* z, int B, int d, hipStream_t st);
// storage-dtype copy of fp32 rows (hidden_out)
int launch_store_rows(int dtype, const float* src, void* dst, int64_t n, hipStream_t st);

// ---- selection kernels (select.hip) -----------------------------------------------------------------
// a (value, column) candidate of a row; index kNoIndex marks an empty one
struct ArgCand {
  float v;
  int i;
};
constexpr int kNoIndex = 0x7FFFFFFF;
// a precedes b in the selection order: value descending, then index ascending (total on non-NaN values)
__device__ inline bool precedes(float av, int ai, float bv, int bi) { return av > bv || (av == bv && ai < bi); }
// out[r] = index of the best of cand[r][0..n_cand) in that order (-1 if all are empty)
int launch_argmax_merge(const ArgCand* cand, int rows, int n_cand, int32_t* out, hipStream_t st);
// out[r] = argmax_v logits[r][v], ties -> lowest v
// (scratch: topk_scratch_bytes(rows) bytes enable the two-stage kernels for long rows; may be NULL)
int launch_argmax(const float* logits, int rows, int V, int64_t ld, int32_t* out, void* scratch, int64_t scratch_bytes,
                  hipStream_t st);
int64_t topk_scratch_bytes(int rows);
// out[r][0..k) = indices of the k largest of logits[r][:], descending, ties -> lower index
int launch_topk(const float* logits, int rows, int V, int64_t ld, int k, int32_t* out, int64_t out_ld, void* scratch,
                int64_t scratch_bytes, hipStream_t st);
// Candidate selection of all heads at once from logits [B][K+1][V] (row 0 of a sequence: the base LM head, used
// only when root_token is NULL): fills cand_flat [B][n_cand].  Needs heads_select_supported().
bool heads_select_supported(int tree, int B, int V, const void* scratch, int64_t scratch_bytes);
int launch_heads_select(int tree, const float* logits, int B, int V, const int32_t* root_token, int32_t* cand_flat,
                        void* scratch, hipStream_t st);
// dst[i * dst_stride] = src[i]
int launch_scatter_i32(const int32_t* src, int32_t* dst, int n, int64_t dst_stride, hipStream_t st);
int launch_tree_tokens(int tree, const int32_t* cand_flat, int32_t* tree_tokens, int B, hipStream_t st);
int launch_accept(int tree, const int32_t* tree_tokens, const int32_t* node_argmax, int B, int32_t* accept_len,
                  int32_t* best_path, int32_t* acc_nodes, int32_t* acc_tokens, int32_t* next_root,
                  int32_t* last_node, hipStream_t st);

// ---- GEMM: sum_k X[m][k] * W[n][k], W packed, X storage dtype [M][K] ------------------------------
// Writes at most max_split partial sums into `out` (partial s at out + s*M*ld, leading dimension ld) and
// describes them in *res.  max_split == 1 yields the finished product in out.
int launch_gemm(int dtype, const void* X, const void* Wp, float* out, int M, int N, int K, int64_t ld,
                int max_split, Partials* res, hipStream_t st);

// ---- tree-masked attention --------------------------------------------------------------------------
// q [B*T][d] storage dtype (rotated); att_out [B*T][d] storage dtype
int launch_tree_attention(int dtype, int tree, const void* q, const KvGeom& g, const void* kc, const void* vc,
                          int layer, const int32_t* seq_len, int B, int max_prefix, void* att_out, void* scratch,
                          int64_t scratch_bytes, hipStream_t st);
int64_t tree_attention_scratch_bytes(int dtype, int tree, const KvGeom& g, int B, int max_prefix);

}  // namespace mdz
