/*
 * libmedusa_hip — static-tree Medusa verification for a pre-norm decoder on MI355X (gfx950).
 *
 * C ABI.  Every entry point only ENQUEUES work on the caller's HIP stream (passed as void*, NULL =
 * the default stream): no call allocates device memory, synchronises, or copies to the host, so a
 * decode loop can be chained without the host seeing any result (the point of the paper's Section
 * 3.2 "Zero-Copy Retrieval Strategy").  Unless a parameter says HOST, every pointer is a DEVICE
 * pointer owned by the caller and must stay valid until the stream reaches the enqueued work.
 * Descriptor structs are HOST structs read during the call.
 *
 * Return value: mdz_status (0 = ok, negative = error).  On an error nothing has been enqueued and
 * medusa_last_error() describes the failure.  No exceptions, no aborts.
 *
 * Storage dtype (mdz_model_desc.dtype): the element type of weights, embeddings, norm gains, the
 * KV cache and the `hidden` tensors at the boundary: bf16, fp16 (IEEE binary16, the precision the
 * paper infers in: Section 4.1) or fp32.  bf16 and fp16 share every layout and kernel.  The residual
 * stream and all logits are fp32 in every mode.  Token ids, lengths and indices are int32.
 *
 * Static trees (Section 3.2, "Tensorization of Tree Topology"): the candidate tree is fixed at
 * compile time.  Node 0 is the root (the base model's own next token, depth 0); depth k holds
 * candidates of Medusa head k (Section 3.1: head k predicts position t+k+1).  A node is a tuple of
 * per-head candidate ranks; nodes are ordered by depth, then lexicographically.  For each tree the
 * library holds: parent[T], depth[T], cand_slot[T] (index into the flat candidate buffer
 * [root | top-k of head 1 | ... | top-k of head K]), anc_mask[T] (bit j of anc_mask[i] set iff node
 * j is i or an ancestor of i: the paper's [T,T] visibility matrix, one 64-bit word per row) and
 * retrieve[n_paths][K+1] (node indices root->leaf per leaf, leaves ascending, padded with -1: the
 * paper's retrieve table).
 */
#ifndef MEDUSA_H
#define MEDUSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MDZ_OK = 0,
  MDZ_EINVAL = -1,       /* null pointer, negative size, bad enum */
  MDZ_ESHAPE = -2,       /* sizes inconsistent with each other or with the tree */
  MDZ_EUNSUPPORTED = -3, /* valid but not built (e.g. a head_dim the kernels do not cover) */
  MDZ_EWORKSPACE = -4,   /* workspace smaller than medusa_workspace_bytes() */
  MDZ_EHIP = -5          /* a HIP runtime call failed (message holds hipGetErrorString) */
} mdz_status;

/* Compiled-in static trees.  MDZ_TREE_1 is the root alone (T = 1, K = 0): every entry point then computes one
 * ordinary autoregressive decode step, the baseline of the paper's Overhead and Speedup metrics (Section 4.1). */
typedef enum { MDZ_TREE_15 = 0, MDZ_TREE_64 = 1, MDZ_TREE_1 = 2, MDZ_TREE_64_K5 = 3 /* 64 nodes, five heads */ } mdz_tree_id;
typedef enum { MDZ_BF16 = 0, MDZ_FP32 = 1, MDZ_FP16 = 2 /* IEEE binary16: same layouts and kernels as bf16 */ } mdz_dtype;

/* Cache rows as stored.  MDZ_KV_FP8E4M3: the KV compression the paper points to for long sequences (Sections 4.2
 * and 5; the paper fixes no format): a row (one slot of one key/value head) is head_dim OCP FP8 E4M3 codes plus one
 * fp32 scale = max|row| / 448 (1 for a zero row); code = the E4M3 value nearest to x / scale, ties to even, decided in
 * fp32 on the fp32 value of the row (K after RoPE); attention reads value(code) * scale.  Half the bytes per slot
 * (132 instead of 256 per head and matrix at head_dim 128); `dtype` still names the type of rows at the boundary
 * (medusa_kv_write quantises, medusa_kv_read returns value(code) * scale rounded to dtype). */
typedef enum { MDZ_KV_PLAIN = 0, MDZ_KV_FP8E4M3 = 1 } mdz_kv_quant;

#define MDZ_MAX_HEADS 8

/* HOST struct: the decoder's shape. d == n_heads * head_dim (no bias).  n_kv_heads: key/value heads of
 * grouped-query attention (Table 1 of the paper: 32 query heads, 8 key/value heads); it must divide n_heads, query
 * head h reads key/value head h / (n_heads / n_kv_heads); 0 means n_heads (plain multi-head attention).
 * ffn_f16 = 1 (bf16 models): the two matrix products of every layer's feed-forward block take IEEE binary16
 * operands.  The layer's wgateup and wdown must then be packed with medusa_pack_weight_bf16_as_f16 (the same values:
 * a bf16 number of magnitude in [2^-14, 65504] is a binary16 number), and the block's two activations (the
 * normalised input, the SwiGLU output) are rounded to 11 significant bits instead of 8, which are the two largest
 * terms of a deep bf16 stack's rounding error.  What the layer computes (Section 3.2: the ordinary decoder layer on
 * the tree's rows) is unchanged; every other buffer, the gains, the cache and the other matrices stay bf16.  An
 * activation beyond 65504 in magnitude would overflow: this is an option for models whose feed-forward activations
 * are known to stay inside that range, off by default. */
typedef struct {
  int32_t d, n_heads, head_dim, ffn, vocab, n_layers;
  int32_t dtype; /* mdz_dtype */
  int32_t tree;  /* mdz_tree_id: fixes T, K and the per-head top-k sizes */
  float rms_eps;
  float rope_base;
  int32_t n_kv_heads;
  int32_t ffn_f16; /* 0 or 1; 1 is allowed for MDZ_BF16 only (see below) */
} mdz_model_desc;

/* HOST struct of device pointers: one decoder layer.  Matrices are in the library's PACKED layout
 * (see medusa_pack_weight): wqkv = rows of Wq, Wk, Wv stacked
 * ([d + 2 * n_kv_heads * head_dim, d]: 3d for multi-head attention); wgateup = Wgate and Wup with
 * their row tiles interleaved (tile 2j = gate tile j, tile 2j+1 = up tile j; [2*ffn, d]).
 * g_attn, g_ffn: RMSNorm gains [d], storage dtype. */
typedef struct {
  const void* wqkv;
  const void* wo;      /* [d, d] */
  const void* wgateup; /* [2*ffn, d] */
  const void* wdown;   /* [d, ffn] */
  const void* g_attn;
  const void* g_ffn;
} mdz_layer_weights;

/* HOST struct.  layers: HOST array of n_layers entries.  embed: [vocab, d] ROW-MAJOR storage dtype
 * (it is gathered, not multiplied).  lm_head: packed [vocab, d].  Medusa head k (0-based here):
 * head_w1[k] packed [d, d], head_b1[k] bias [d] storage dtype or NULL, head_lm[k] packed [vocab, d].
 * head_b1 itself may be NULL (no head has a bias).  If the packed head_w1 matrices lie back to back in memory
 * (head_w1[k] == head_w1[0] + k * medusa_packed_bytes(dtype, d, d)) the heads' first layers run as one launch. */
typedef struct {
  const mdz_layer_weights* layers;
  const void* embed;
  const void* lm_head;
  const void* g_final;
  int32_t n_medusa;
  const void* const* head_w1; /* HOST array [n_medusa] */
  const void* const* head_b1; /* HOST array [n_medusa] or NULL */
  const void* const* head_lm; /* HOST array [n_medusa] */
} mdz_weights;

/* Bits the kernels OR into mdz_kv_desc.status (a device word the caller clears and reads when it chooses). */
#define MDZ_STATUS_SEQ_RANGE 1 /* a seq_len[b] outside [0, max_prefix] reached a kernel and was clamped */

/* HOST struct: the KV cache.  k and v are two device allocations of medusa_kv_bytes() bytes each whose
 * internal layout belongs to the library (tiled for the attention kernels); fill and inspect them with
 * medusa_kv_write / medusa_kv_read.  Call medusa_kv_init once after allocating them: the attention kernels load
 * whole blocks of 32 slots and need the slots beyond a sequence's length to hold finite values.
 * cap = slots per sequence; a verify pass with prefix length S writes slots S..S+T-1, so S + T <= cap is required.
 * status (nullable): one int32 in device memory.  Lengths live on the device (a chained loop advances them without
 * the host), so a length outside [0, max_prefix] cannot be rejected by the call: every kernel clamps it (no access
 * leaves the cache) and tree_verify_layer / tree_verify_step / kv_compact OR MDZ_STATUS_SEQ_RANGE into *status. */
typedef struct {
  void* k;
  void* v;
  int32_t n_layers, batch, n_heads, head_dim, cap; /* n_heads: key/value heads (the heads the cache holds) */
  int32_t dtype; /* mdz_dtype */
  int32_t quant; /* mdz_kv_quant; MDZ_KV_FP8E4M3 needs a 16-bit dtype, head_dim 128 and a tree of 64 nodes or 1 node (with
                    the 1-node tree also a number of query heads that is a multiple of 4); anything else: MDZ_EUNSUPPORTED */
  int32_t* status; /* device, nullable */
} mdz_kv_desc;

/* ---- introspection (all HOST out-pointers) ------------------------------------------------- */

/* Sizes of a compiled-in tree: T nodes, K heads, n_paths leaves, n_cand = 1 + sum of top-k sizes.
 * topk (nullable) receives K entries (array of at least MDZ_MAX_HEADS ints). */
int medusa_tree_info(int tree, int32_t* T, int32_t* K, int32_t* n_paths, int32_t* n_cand, int32_t* topk);

/* Copies the compiled-in tables to HOST buffers (any may be NULL): parent[T], depth[T], cand_slot[T],
 * anc_mask[T], retrieve[n_paths*(K+1)].  Lets a caller audit exactly what the kernels use. */
int medusa_tree_tables(int tree, int32_t* parent, int32_t* depth, int32_t* cand_slot, uint64_t* anc_mask,
                       int32_t* retrieve);

/* Never NULL; thread-local; valid until the next failing call on this thread. */
const char* medusa_last_error(void);

/* ---- weight packing (one-time, outside any timed region) ------------------------------------ */

/* Rows per packed tile for a dtype (32 for bf16 and fp16, 16 for fp32). */
int medusa_pack_tile_rows(int dtype);

/* Bytes of a packed [n_rows, k] matrix (bf16: n_rows rounded up to 128 and k to 256; fp32: n_rows to 16). */
int64_t medusa_packed_bytes(int dtype, int64_t n_rows, int64_t k);

/* Re-tiles a ROW-MAJOR [n_rows, k] matrix `src` (row r = output feature r, contiguous over input
 * features: y = W x) into the streaming order of the GEMM kernels, same element type, same bytes.
 * Source row tile j (rows j*R .. j*R+R-1, R = medusa_pack_tile_rows) lands at tile index
 * tile_offset + j*tile_stride of `dst`, a packed matrix of dst_rows rows in total, so several matrices
 * can be stacked (wqkv: offsets 0, d/R, (d + kv width)/R, stride 1) or interleaved (wgateup: offsets 0 and 1,
 * stride 2).  n_rows must be a multiple of R unless tile_stride == 1 and this is the last matrix. */
int medusa_pack_weight(int dtype, const void* src, int64_t n_rows, int64_t k, void* dst, int64_t dst_rows,
                       int64_t tile_offset, int64_t tile_stride, void* stream);

/* The same re-tiling of a ROW-MAJOR bf16 matrix, with every element converted to IEEE binary16 on the way (exact
 * for magnitudes in [2^-14, 65504], round-to-nearest-even into binary16's subnormals below, infinity above): the
 * form of wgateup and wdown that a model with ffn_f16 = 1 takes.  Same sizes and bytes as the bf16 packing. */
int medusa_pack_weight_bf16_as_f16(const void* src, int64_t n_rows, int64_t k, void* dst, int64_t dst_rows,
                                   int64_t tile_offset, int64_t tile_stride, void* stream);

/* ---- KV cache ------------------------------------------------------------------------------- */

/* Bytes of EACH of desc->k and desc->v (negative = mdz_status). */
int64_t medusa_kv_bytes(const mdz_kv_desc* desc);

/* Enqueues a fill of desc->k and desc->v (and of *desc->status, if given) with zeros: a kernel, not a memset, so
 * the call may sit inside a captured graph. */
int medusa_kv_init(const mdz_kv_desc* desc, void* stream);

/* Copies n rows starting at slot pos0 of sequence `seq`, layer `layer`, between the cache and plain
 * buffers k_rows / v_rows laid out [n_heads][n][head_dim] in the storage dtype.  write: buffers ->
 * cache; read: cache -> buffers.  Requires 0 <= pos0, pos0 + n <= cap. */
int medusa_kv_write(const mdz_kv_desc* desc, int layer, int seq, int pos0, int n, const void* k_rows,
                    const void* v_rows, void* stream);
int medusa_kv_read(const mdz_kv_desc* desc, int layer, int seq, int pos0, int n, void* k_rows, void* v_rows,
                   void* stream);

/* ---- workspace ------------------------------------------------------------------------------ */

/* Bytes of scratch any of the calls below may need for batch B and prefix lengths <= max_prefix.
 * The caller allocates it once; calls on different streams need different workspaces. */
int64_t medusa_workspace_bytes(const mdz_model_desc* model, int B, int max_prefix);

/* ---- the hot path --------------------------------------------------------------------------- */

/* Section 3.1 (Medusa heads).  For each sequence b the input row is hidden[b][src_row[b]] (src_row NULL
 * => row 0), the post-final-norm hidden state the base LM head reads.  Head k = 1..K:
 * z = h + SiLU(W1_k h + b1_k); logits_k = Wlm_k z; candidates = the topk_k largest, descending,
 * ties -> lower id.  The root candidate is root_token[b] if root_token != NULL, else the argmax of the
 * base LM head on h.  Outputs: cand_flat [B, n_cand] = [root | head 1 | .. | head K]; tree_tokens [B, T]
 * with tree_tokens[n] = cand_flat[cand_slot[n]]; head_logits_opt (nullable) [B, K+1, vocab] fp32
 * (row 0 = base head, written only when it was computed).
 * hidden: [B, Tsrc, d] storage dtype. */
int medusa_heads(const mdz_model_desc* model, const mdz_weights* w, const void* hidden, const int32_t* src_row,
                 const int32_t* root_token, int B, int Tsrc, int32_t* cand_flat, int32_t* tree_tokens,
                 float* head_logits_opt, void* ws, int64_t ws_bytes, void* stream);

/* Section 3.2 (single-pass tree verification), one decoder layer `layer` over x [B*T, d] fp32 (in/out,
 * the residual stream).  For sequence b with prefix length S = seq_len[b] (clamped to [0, max_prefix]):
 * RMSNorm -> q,k,v -> RoPE at position S + depth[n] (rotate-half pairing, angle pos*base^(-2i/hd)) ->
 * k,v of node n stored to cache slot S + n -> node i attends to slots [0,S) and S+j for every j in
 * anc_mask[i], scale 1/sqrt(head_dim) -> output projection + residual -> RMSNorm ->
 * Wdown(SiLU(Wgate x) * Wup x) + residual.  seq_len: [B] device.  max_prefix + T <= kv->cap. */
int tree_verify_layer(const mdz_model_desc* model, const mdz_layer_weights* lw, int layer, float* x_inout,
                      const mdz_kv_desc* kv, const int32_t* seq_len, int B, int max_prefix, void* ws,
                      int64_t ws_bytes, void* stream);

/* For callers that cannot allocate device memory or carry a workspace (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): tree_verify_layer with the library's own scratch, a fixed buffer of
 * tree_verify_layer_static_scratch_bytes() bytes that is part of the loaded code object (one per GPU, held until the
 * process ends).  Same arguments, same kernels and bit-identical results as tree_verify_layer; the call allocates and
 * frees nothing (its first call on a device looks up the buffer's address).  A shape whose scratch need exceeds the
 * buffer (about 64 tree rows x 7B-class widths at prefixes up to 16K fits; batches do not) is refused with
 * MDZ_EWORKSPACE and nothing is enqueued.  Every call on a GPU shares that GPU's buffer: calls whose execution can
 * overlap on one GPU (different streams) race; calls on one stream are safe. */
int64_t tree_verify_layer_static_scratch_bytes(void);
int tree_verify_layer_static(const mdz_model_desc* model, const mdz_layer_weights* lw, int layer, float* x_inout,
                             const mdz_kv_desc* kv, const int32_t* seq_len, int B, int max_prefix, void* stream);

/* Section 3.2, the whole pass: embedding gather of tree_tokens [B, T] -> every layer as above -> final
 * RMSNorm -> LM head -> per-node argmax (ties -> lowest id).  Outputs: node_argmax [B, T];
 * hidden_out (nullable) [B, T, d] storage dtype = the post-final-norm hidden (what medusa_heads reads);
 * logits_opt (nullable) [B, T, vocab] fp32.  With logits_opt NULL the logits are not materialised where the shape
 * allows it (16-bit storage, B * T <= 64): the LM-head kernel keeps each row's best column itself; node_argmax is the
 * same either way, bit for bit (the selection order is total: value descending, then lowest id). */
int tree_verify_step(const mdz_model_desc* model, const mdz_weights* w, const int32_t* tree_tokens,
                     const mdz_kv_desc* kv, const int32_t* seq_len, int B, int max_prefix, int32_t* node_argmax,
                     void* hidden_out, float* logits_opt, void* ws, int64_t ws_bytes, void* stream);

/* Section 3.2 (zero-copy retrieval), greedy exact-match criterion.  Node n > 0 matches iff
 * tree_tokens[n] == node_argmax[parent[n]]; the root always matches.  For every row of the retrieve
 * table count the leading matching nodes; best_path = the longest (ties -> lowest row index),
 * accept_len A in [1, K+1].  acc_nodes / acc_tokens [B, K+1] = first A nodes of that row and their
 * tokens, -1 padded; last_node = acc_nodes[A-1]; next_root = node_argmax[last_node]. */
int accept_longest_prefix(int tree, const int32_t* tree_tokens, const int32_t* node_argmax, int B,
                          int32_t* accept_len, int32_t* best_path, int32_t* acc_nodes, int32_t* acc_tokens,
                          int32_t* next_root, int32_t* last_node, void* stream);

/* Section 3.2 (node -> KV position mapping).  For each sequence b with S = seq_len_inout[b] (clamped as
 * above) and A = accept_len[b]: in every layer, for K and V, cache row S + j <- row S + acc_nodes[b][j]
 * for j < A (in place, on the device, no staging buffer); kv_src_slots [B, K+1] = S + acc_nodes (-1
 * padded); seq_len_inout[b] = S + A. */
int kv_compact(const mdz_kv_desc* kv, int tree, const int32_t* acc_nodes, const int32_t* accept_len,
               int32_t* seq_len_inout, int32_t* kv_src_slots, int B, int max_prefix, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MEDUSA_H */
