// C-ABI layer of libmedusa_hip: argument checking, workspace carving and the order of kernel launches.
// Every step of the path runs in the kernels; this file only sequences them on the caller's stream.
#include <stdarg.h>
#include <string.h>

#include <atomic>

#include "kernels.h"

namespace mdz {

static thread_local char g_err[512] = "";

int num_cus() {
  static std::once_flag once;
  static int n = 256;
  std::call_once(once, []() {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
      n = prop.multiProcessorCount;
    else
      (void)hipGetLastError();  // no device: host-only callers keep the MI355X count
  });
  return n;
}

static std::atomic<int> g_force_unfused_rope{0};  // set only through medusa_test_force_unfused_rope

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int launch_gemm_generic(int dtype, const void* X, const void* Wp, float* Y, int M, int N, int K, int64_t ldy,
                        bool accumulate, hipStream_t st);
int launch_attention_generic(int dtype, int tree, const void* q, const KvGeom& g, const void* kc, const void* vc,
                             int layer, const int32_t* seq_len, int B, int max_prefix, void* att_out,
                             hipStream_t st);

bool gemm_mfma_supported(int dtype, int M, int N, int K);
int gemm_mfma_slots(int M, int N, int K, int max_split);
void gemm_mfma_describe(int M, int N, int K, int max_split, Partials* res, int* grid);
int launch_gemm_mfma(int dtype, const void* X, const void* Wp, float* P, int M, int N, int K, int64_t ldp,
                     int64_t part_stride, int max_split, Partials* res, hipStream_t st);

bool gemm_large_supported(int dtype, int M, int N, int K);
int gemm_large_slots(int M, int N, int K);
int launch_gemm_large(int dtype, const void* X, const void* Wp, float* P, int M, int N, int K, int64_t ldp,
                      int64_t part_stride, Partials* res, hipStream_t st);

bool gemm_mfma_swiglu_supported(int dtype, int M, int N, int K);
int launch_gemm_mfma_swiglu(int dtype, const void* X, const void* Wp, void* U, int M, int N, int K, hipStream_t st);
bool gemm_mfma_argmax_supported(int dtype, int M, int N, int K);
int gemm_mfma_argmax_cands(int M, int N, int K);
int launch_gemm_mfma_argmax(int dtype, const void* X, const void* Wp, int M, int N, int K, ArgCand* cand, hipStream_t st);
bool gemm_large_swiglu_supported(int dtype, int M, int N, int K);
int launch_gemm_large_swiglu(int dtype, const void* X, const void* Wp, void* U, int M, int N, int K, hipStream_t st);

int launch_gemm(int dtype, const void* X, const void* Wp, float* out, int M, int N, int K, int64_t ld, int max_split,
                Partials* res, hipStream_t st) {
  *res = single_slot(out, (int64_t)M * ld, ld);
  // several sequences at once: the MFMA-bound kernel (it splits K only when the caller's consumer reduces slots)
  if (gemm_large_supported(dtype, M, N, K) && (max_split > 1 || gemm_large_slots(M, N, K) == 1))
    return launch_gemm_large(dtype, X, Wp, out, M, N, K, ld, res->stride, res, st);
  const int rows_per_launch = M <= 64 ? M : 64;
  if (gemm_mfma_supported(dtype, rows_per_launch, N, K) && (M <= 64 || M % 64 == 0)) {
    // More than 64 rows (several sequences): one launch per block of 64 rows.  Every launch uses the same plan, so
    // the slot counts are identical; the first launch streams the matrix from HBM, the following ones mostly from
    // the memory-side cache.
    for (int m0 = 0; m0 < M; m0 += rows_per_launch) {
      int rc = launch_gemm_mfma(dtype, (const char*)X + (int64_t)m0 * K * 2, Wp, out + (int64_t)m0 * ld, rows_per_launch, N,
                                K, ld, res->stride, max_split, res, st);
      if (rc) return rc;
    }
    return MDZ_OK;
  }
  return launch_gemm_generic(dtype, X, Wp, out, M, N, K, ld, false, st);
}

// split-K is only worth its partial-sum traffic for skinny problems
static int max_split_for(int rows) { return (rows <= 64 || rows % 64 == 0) ? 12 : 1; }
// fp32 elements of partial-sum workspace a [rows, N] = [rows, K] x [N, K] GEMM needs
static int64_t gemm_part_elems(int dtype, int rows, int N, int K) {
  if (gemm_large_supported(dtype, rows, N, K)) return (int64_t)gemm_large_slots(rows, N, K) * rows * N;
  const int per = rows <= 64 ? rows : 64;
  const int slots = (gemm_mfma_supported(dtype, per, N, K) && (rows <= 64 || rows % 64 == 0))
                        ? gemm_mfma_slots(per, N, K, max_split_for(rows))
                        : 1;
  return (int64_t)slots * rows * N;
}

bool attn_mfma_supported(int dtype, int tree, const KvGeom& g);
int64_t attn_mfma_scratch_bytes(int B, int n_heads, int max_prefix);
int launch_attention_mfma(int dtype, int tree, const void* q, const Partials* qkv, const float* cs, const KvGeom& g, void* kc,
                          void* vc, int layer, const int32_t* seq_len, int B, int max_prefix, void* att_out,
                          void* scratch, int64_t scratch_bytes, hipStream_t st);

bool attn_decode_supported(int dtype, int tree, const KvGeom& g);
int64_t attn_decode_scratch_bytes(int B, int n_heads, int max_prefix);
int launch_attention_decode(int dtype, const void* q, const KvGeom& g, const void* kc, const void* vc, int layer,
                            const int32_t* seq_len, int B, int max_prefix, void* att_out, void* scratch,
                            int64_t scratch_bytes, hipStream_t st);

int64_t tree_attention_scratch_bytes(int dtype, int tree, const KvGeom& g, int B, int max_prefix) {
  if (attn_decode_supported(dtype, tree, g)) return attn_decode_scratch_bytes(B, q_heads(g), max_prefix);
  return attn_mfma_supported(dtype, tree, g) ? attn_mfma_scratch_bytes(B, q_heads(g), max_prefix) : 0;
}

int launch_tree_attention(int dtype, int tree, const void* q, const KvGeom& g, const void* kc, const void* vc,
                          int layer, const int32_t* seq_len, int B, int max_prefix, void* att_out, void* scratch,
                          int64_t scratch_bytes, hipStream_t st) {
  if (attn_decode_supported(dtype, tree, g))
    return launch_attention_decode(dtype, q, g, kc, vc, layer, seq_len, B, max_prefix, att_out, scratch, scratch_bytes, st);
  if (attn_mfma_supported(dtype, tree, g))
    return launch_attention_mfma(dtype, tree, q, nullptr, nullptr, g, (void*)kc, (void*)vc, layer, seq_len, B, max_prefix,
                                 att_out, scratch, scratch_bytes, st);
  return launch_attention_generic(dtype, tree, q, g, kc, vc, layer, seq_len, B, max_prefix, att_out, st);
}

// QKV partial sums -> RoPE -> cache rows -> attention.  One fused kernel where the MFMA attention applies (the
// partial sums must then come in 128-column bands so that a head's columns share one slot count).
int launch_rope_attention(int dtype, int tree, const Partials& qkv, const float* cs, void* q_scratch, const KvGeom& g,
                          void* kc, void* vc, int layer, const int32_t* seq_len, int B, int max_prefix, void* att_out,
                          void* scratch, int64_t scratch_bytes, hipStream_t st) {
  const bool unfused = g_force_unfused_rope.load(std::memory_order_relaxed) != 0;
  if (!unfused && attn_mfma_supported(dtype, tree, g) && qkv.stride % 4 == 0 && qkv.ld % 4 == 0 &&
      (qkv.split_grid == 0 || qkv.band_cols % 128 == 0))
    return launch_attention_mfma(dtype, tree, nullptr, &qkv, cs, g, kc, vc, layer, seq_len, B, max_prefix, att_out, scratch,
                                 scratch_bytes, st);
  int rc = launch_rope_kvwrite(dtype, tree, qkv, cs, q_scratch, g, kc, vc, layer, seq_len, B, max_prefix, st);
  if (rc) return rc;
  return launch_tree_attention(dtype, tree, q_scratch, g, kc, vc, layer, seq_len, B, max_prefix, att_out, scratch,
                               scratch_bytes, st);
}

// ---- workspace ------------------------------------------------------------------------------------
// key/value heads of a model (0 in the descriptor: as many as query heads) and the width of its K (or V) projection
static int kv_heads(const mdz_model_desc& m) { return m.n_kv_heads > 0 ? m.n_kv_heads : m.n_heads; }
static int kv_width(const mdz_model_desc& m) { return kv_heads(m) * m.head_dim; }
// operand type of the feed-forward block's two products
static int ffn_dtype(const mdz_model_desc& m) { return m.ffn_f16 ? (int)MDZ_FP16 : m.dtype; }

struct Workspace {
  int64_t rope_cs, x, xn, part, q, att, u, logits, h, z, hlogits, sel, sel_bytes, attn_scratch, total;
};

static int64_t align256(int64_t v) { return (v + 255) & ~int64_t(255); }

// layer_only: what tree_verify_layer touches (no logits, no head buffers, no selection lists)
static Workspace carve(const mdz_model_desc& m, int B, int max_prefix, bool layer_only = false) {
  const TreeTables* t = host_tree(m.tree);
  const int64_t es = elem_bytes(m.dtype);
  const int64_t rows = (int64_t)B * t->T;
  Workspace w{};
  int64_t off = 0;
  auto take = [&](int64_t bytes) {
    int64_t o = off;
    off = align256(off + bytes);
    return o;
  };
  w.rope_cs = take(rows * (m.head_dim / 2) * 2 * 4);
  w.x = take(rows * m.d * 4);
  w.xn = take(rows * m.d * es);
  {
    int64_t layer_part = 0;
    const int shapes[4][2] = {{m.d + 2 * kv_width(m), m.d}, {m.d, m.d}, {2 * m.ffn, m.d}, {m.d, m.ffn}};
    for (auto& sh : shapes) {
      int64_t e = gemm_part_elems(m.dtype, (int)rows, sh[0], sh[1]) * 4;
      layer_part = e > layer_part ? e : layer_part;
    }
    // every head's first-layer sums at once: from separate GEMMs, or from one GEMM over the stacked matrices
    int64_t head_part = layer_only ? 0 : gemm_part_elems(m.dtype, B, m.d, m.d) * 4 * (t->K > 0 ? t->K : 1);
    if (!layer_only && t->K > 1) {
      const int64_t stacked = gemm_part_elems(m.dtype, B, t->K * m.d, m.d) * 4;
      head_part = stacked > head_part ? stacked : head_part;
    }
    w.part = take(layer_part > head_part ? layer_part : head_part);
  }
  w.q = take(rows * m.d * es);
  w.att = take(rows * m.d * es);
  w.u = take(rows * m.ffn * es);
  if (!layer_only) {
    w.logits = take(rows * (int64_t)m.vocab * 4);
    w.h = take((int64_t)B * m.d * es);
    w.z = take((int64_t)B * m.d * es * (t->K > 0 ? t->K : 1));
    w.hlogits = take((int64_t)B * (t->K + 1) * m.vocab * 4);
    // candidate lists of the selection kernels: the verify step's rows, or the heads' B * (K + 1) rows
    const int64_t head_rows = (int64_t)B * (t->K + 1);
    w.sel_bytes = topk_scratch_bytes((int)(rows > head_rows ? rows : head_rows));
    w.sel = take(w.sel_bytes);
  }
  KvGeom g{m.n_layers, B, kv_heads(m), m.head_dim, max_prefix + t->T, (is_16bit(m.dtype) && m.head_dim % 32 == 0) ? 1 : 0,
           m.n_heads / kv_heads(m), 0};
  w.attn_scratch = take(tree_attention_scratch_bytes(m.dtype, m.tree, g, B, max_prefix));
  w.total = off;
  return w;
}

static int check_model(const mdz_model_desc* m) {
  MDZ_REQUIRE(m != nullptr, MDZ_EINVAL, "model descriptor is NULL");
  MDZ_REQUIRE(dtype_ok(m->dtype), MDZ_EINVAL, "bad dtype %d", m->dtype);
  MDZ_REQUIRE(host_tree(m->tree) != nullptr, MDZ_EINVAL, "bad tree id %d", m->tree);
  MDZ_REQUIRE(m->d > 0 && m->n_heads > 0 && m->head_dim > 0 && m->ffn > 0 && m->vocab > 0 && m->n_layers > 0,
              MDZ_EINVAL, "model sizes must be positive");
  MDZ_REQUIRE(m->n_kv_heads >= 0 && m->n_heads % kv_heads(*m) == 0, MDZ_ESHAPE,
              "n_kv_heads %d does not divide n_heads %d", m->n_kv_heads, m->n_heads);
  MDZ_REQUIRE(m->d == m->n_heads * m->head_dim, MDZ_ESHAPE, "d %d != n_heads %d * head_dim %d", m->d, m->n_heads,
              m->head_dim);
  MDZ_REQUIRE(m->head_dim % 2 == 0, MDZ_ESHAPE, "head_dim %d must be even (rotary pairs)", m->head_dim);
  const int R = is_16bit(m->dtype) ? kTileRowsBf16 : kTileRowsF32;
  MDZ_REQUIRE(m->ffn % R == 0 && m->d % R == 0, MDZ_ESHAPE, "d %d and ffn %d must be multiples of the tile height %d",
              m->d, m->ffn, R);
  MDZ_REQUIRE(!is_16bit(m->dtype) || (m->d % kKStepBf16 == 0 && m->ffn % kKStepBf16 == 0), MDZ_ESHAPE,
              "bf16 / fp16: d and ffn must be multiples of %d", kKStepBf16);
  MDZ_REQUIRE(m->rms_eps >= 0.f && m->rope_base > 1.f, MDZ_EINVAL, "bad rms_eps / rope_base");
  MDZ_REQUIRE(m->ffn_f16 == 0 || (m->ffn_f16 == 1 && m->dtype == MDZ_BF16), MDZ_EINVAL,
              "ffn_f16 is 0 or 1 and applies to bf16 models only (ffn_f16 %d, dtype %d)", m->ffn_f16, m->dtype);
  return MDZ_OK;
}

static int check_kv_quant(const mdz_kv_desc* kv) {
  MDZ_REQUIRE(kv->quant == MDZ_KV_PLAIN || kv->quant == MDZ_KV_FP8E4M3, MDZ_EINVAL, "bad kv quant %d", kv->quant);
  MDZ_REQUIRE(kv->quant == MDZ_KV_PLAIN || (is_16bit(kv->dtype) && kv->head_dim == 128), MDZ_EUNSUPPORTED,
              "8-bit kv rows need bf16 or fp16 at the boundary and head_dim 128 (dtype %d, head_dim %d)", kv->dtype,
              kv->head_dim);
  return MDZ_OK;
}

static int check_kv(const mdz_model_desc* m, const mdz_kv_desc* kv, int B, int max_prefix) {
  MDZ_REQUIRE(kv != nullptr && kv->k != nullptr && kv->v != nullptr, MDZ_EINVAL, "kv descriptor or its buffers NULL");
  MDZ_REQUIRE(dtype_ok(kv->dtype), MDZ_EINVAL, "bad kv dtype %d", kv->dtype);
  MDZ_REQUIRE(kv->n_layers > 0 && kv->batch > 0 && kv->n_heads > 0 && kv->head_dim > 0 && kv->cap > 0, MDZ_EINVAL,
              "kv sizes must be positive");
  int rc = check_kv_quant(kv);
  if (rc) return rc;
  if (m) {
    MDZ_REQUIRE(kv->quant == MDZ_KV_PLAIN || host_tree(m->tree)->T == 64 || host_tree(m->tree)->T == 1, MDZ_EUNSUPPORTED,
                "8-bit kv rows need a tree of 64 nodes or 1 node");
    MDZ_REQUIRE(kv->dtype == m->dtype && kv->n_heads == kv_heads(*m) && kv->head_dim == m->head_dim &&
                    kv->n_layers >= m->n_layers,
                MDZ_ESHAPE, "kv cache (L%d H%d hd%d dtype%d) does not match the model (L%d H%d hd%d dtype%d)",
                kv->n_layers, kv->n_heads, kv->head_dim, kv->dtype, m->n_layers, kv_heads(*m), m->head_dim, m->dtype);
  }
  MDZ_REQUIRE(B >= 0 && B <= kv->batch, MDZ_ESHAPE, "B %d exceeds kv batch %d", B, kv->batch);
  MDZ_REQUIRE(max_prefix >= 0, MDZ_EINVAL, "max_prefix %d < 0", max_prefix);
  return MDZ_OK;
}

// group: query heads per key/value head (1 where only the cache itself is touched)
static KvGeom geom(const mdz_kv_desc* kv, int group = 1) {
  return KvGeom{kv->n_layers, kv->batch, kv->n_heads, kv->head_dim, kv->cap,
                (is_16bit(kv->dtype) && kv->head_dim % 32 == 0) ? 1 : 0, group, kv->quant == MDZ_KV_FP8E4M3 ? 1 : 0};
}

// One decoder layer over rows = B*T rows of x.  On entry ws.xn holds RMSNorm(x; g_attn of this layer).  The
// layer's last residual update is fused with the NEXT norm: x += down-projection partials, then
// xn_next = RMSNorm(x; g_next) is written to xn_next (NULL: residual update only).
static int run_layer(const mdz_model_desc& m, const mdz_layer_weights& lw, int layer, float* x, const mdz_kv_desc* kv,
                     const int32_t* seq_len, int B, int max_prefix, char* ws, const Workspace& w, const void* g_next,
                     void* xn_next, hipStream_t st) {
  const TreeTables* t = host_tree(m.tree);
  const int rows = B * t->T;
  const int ms = max_split_for(rows);
  const KvGeom g = geom(kv, m.n_heads / kv_heads(m));
  int rc;
  float* cs = (float*)(ws + w.rope_cs);
  void* xn = ws + w.xn;
  float* part = (float*)(ws + w.part);
  void* q = ws + w.q;
  void* att = ws + w.att;
  void* u = ws + w.u;
  Partials pr;
  const int qkv_cols = m.d + 2 * kv_width(m);
  // operand type of the feed-forward block: binary16 for a bf16 model that asks for it (wgateup and wdown are then
  // packed as binary16 and the block's two activations are rounded to binary16), else the storage type
  const int fdt = ffn_dtype(m);
  if ((rc = launch_gemm(m.dtype, xn, lw.wqkv, part, rows, qkv_cols, m.d, qkv_cols, ms, &pr, st))) return rc;
  if ((rc = launch_rope_attention(m.dtype, m.tree, pr, cs, q, g, kv->k, kv->v, layer, seq_len, B, max_prefix, att,
                                  ws + w.attn_scratch, w.total - w.attn_scratch, st)))
    return rc;
  if ((rc = launch_gemm(m.dtype, att, lw.wo, part, rows, m.d, m.d, m.d, ms, &pr, st))) return rc;
  if ((rc = launch_residual_rmsnorm(m.dtype, x, pr, lw.g_ffn, xn, rows, m.d, m.rms_eps, st, fdt))) return rc;
  // SwiGLU in the GEMM's epilogue where a workgroup ends up with whole gate/up column pairs
  if (gemm_large_swiglu_supported(fdt, rows, 2 * m.ffn, m.d)) {
    if ((rc = launch_gemm_large_swiglu(fdt, xn, lw.wgateup, u, rows, 2 * m.ffn, m.d, st))) return rc;
  } else if (rows <= 64 && gemm_mfma_swiglu_supported(fdt, rows, 2 * m.ffn, m.d)) {
    if ((rc = launch_gemm_mfma_swiglu(fdt, xn, lw.wgateup, u, rows, 2 * m.ffn, m.d, st))) return rc;
  } else {
    if ((rc = launch_gemm(fdt, xn, lw.wgateup, part, rows, 2 * m.ffn, m.d, 2 * m.ffn, ms, &pr, st))) return rc;
    if ((rc = launch_swiglu(fdt, pr, u, rows, m.ffn, st))) return rc;
  }
  if ((rc = launch_gemm(fdt, u, lw.wdown, part, rows, m.d, m.ffn, m.d, ms, &pr, st))) return rc;
  return launch_residual_rmsnorm(m.dtype, x, pr, g_next, xn_next, rows, m.d, m.rms_eps, st);
}

// ---- static scratch for the entry point that may not allocate ---------------------------------------
// Device memory that belongs to the loaded code object: one copy per GPU the library runs on, held until the process
// ends.  In host code the array's name is only a handle for hipGetSymbolAddress; kernels get the address that call
// returns for the current device.
constexpr int64_t kStaticScratchBytes = 48ll << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices] = {};

// address of `scratch` on the current device (looked up on the first call per device)
static int static_scratch(void** out) {
  int dev = -1;
  MDZ_HIP(hipGetDevice(&dev));
  MDZ_REQUIRE(dev >= 0 && dev < kMaxDevices, MDZ_EUNSUPPORTED, "device ordinal %d beyond the %d the library tracks", dev,
              kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    MDZ_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    MDZ_REQUIRE(p != nullptr, MDZ_EHIP, "hipGetSymbolAddress returned no address for the static scratch");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MDZ_OK;
}

static int check_layer_weights(const mdz_layer_weights* lw) {
  MDZ_REQUIRE(lw && lw->wqkv && lw->wo && lw->wgateup && lw->wdown && lw->g_attn && lw->g_ffn, MDZ_EINVAL,
              "layer weights: NULL pointer");
  return MDZ_OK;
}

}  // namespace mdz

using namespace mdz;

extern "C" {
#pragma GCC visibility push(default)

const char* medusa_last_error(void) { return g_err; }

int medusa_tree_info(int tree, int32_t* T, int32_t* K, int32_t* n_paths, int32_t* n_cand, int32_t* topk) {
  const TreeTables* t = host_tree(tree);
  MDZ_REQUIRE(t != nullptr, MDZ_EINVAL, "bad tree id %d", tree);
  if (T) *T = t->T;
  if (K) *K = t->K;
  if (n_paths) *n_paths = t->n_paths;
  if (n_cand) *n_cand = t->n_cand;
  if (topk)
    for (int k = 0; k < t->K; ++k) topk[k] = t->caps[k];
  return MDZ_OK;
}

int medusa_tree_tables(int tree, int32_t* parent, int32_t* depth, int32_t* cand_slot, uint64_t* anc_mask,
                       int32_t* retrieve) {
  const TreeTables* t = host_tree(tree);
  MDZ_REQUIRE(t != nullptr, MDZ_EINVAL, "bad tree id %d", tree);
  for (int n = 0; n < t->T; ++n) {
    if (parent) parent[n] = t->parent[n];
    if (depth) depth[n] = t->depth[n];
    if (cand_slot) cand_slot[n] = t->cand_slot[n];
    if (anc_mask) anc_mask[n] = t->anc_mask[n];
  }
  if (retrieve)
    for (int p = 0; p < t->n_paths; ++p)
      for (int c = 0; c <= t->K; ++c) retrieve[p * (t->K + 1) + c] = t->retrieve[p][c];
  return MDZ_OK;
}

int medusa_pack_tile_rows(int dtype) {
  MDZ_REQUIRE(dtype_ok(dtype), MDZ_EINVAL, "bad dtype %d", dtype);
  return is_16bit(dtype) ? kTileRowsBf16 : kTileRowsF32;
}

int medusa_gemm_plan(int dtype, int M, int N, int K, int max_split, int32_t* grid, int32_t* band_cols, int32_t* n_stages,
                     int32_t* max_slots) {
  MDZ_REQUIRE(gemm_mfma_supported(dtype, M, N, K), MDZ_EUNSUPPORTED, "gemm plan: [%d,%d] x [%d,%d] is not a streaming-GEMM shape",
              M, K, N, K);
  Partials pr = single_slot(nullptr, 0, 0);
  int g = 0;
  gemm_mfma_describe(M, N, K, max_split, &pr, &g);
  if (grid) *grid = g;
  if (band_cols) *band_cols = pr.band_cols;
  if (n_stages) *n_stages = pr.n_stages;
  if (max_slots) *max_slots = pr.n;
  return MDZ_OK;
}

int medusa_gemm_slot_count(int dtype, int M, int N, int K, int max_split, int col) {
  MDZ_REQUIRE(gemm_mfma_supported(dtype, M, N, K) && col >= 0 && col < N, MDZ_EINVAL, "gemm slot count: bad arguments");
  Partials pr = single_slot(nullptr, 0, 0);
  gemm_mfma_describe(M, N, K, max_split, &pr, nullptr);
  return pr.count(col);
}

int64_t medusa_packed_bytes(int dtype, int64_t n_rows, int64_t k) {
  MDZ_REQUIRE(dtype_ok(dtype), MDZ_EINVAL, "bad dtype %d", dtype);
  MDZ_REQUIRE(n_rows > 0 && k > 0, MDZ_EINVAL, "packed_bytes: sizes must be positive");
  if (is_16bit(dtype)) return Packed<bf16_t>::padded_rows(n_rows) * Packed<bf16_t>::padded_k(k) * 2;
  return round_up(n_rows, kTileRowsF32) * k * 4;
}

int medusa_pack_weight(int dtype, const void* src, int64_t n_rows, int64_t k, void* dst, int64_t dst_rows,
                       int64_t tile_offset, int64_t tile_stride, void* stream) {
  MDZ_REQUIRE(dtype_ok(dtype), MDZ_EINVAL, "bad dtype %d", dtype);
  MDZ_REQUIRE(src && dst, MDZ_EINVAL, "pack: NULL pointer");
  MDZ_REQUIRE(n_rows > 0 && k > 0 && dst_rows >= n_rows, MDZ_EINVAL, "pack: bad sizes");
  return launch_pack_weight(dtype, src, n_rows, k, dst, dst_rows, tile_offset, tile_stride, (hipStream_t)stream);
}

int medusa_pack_weight_bf16_as_f16(const void* src, int64_t n_rows, int64_t k, void* dst, int64_t dst_rows,
                                   int64_t tile_offset, int64_t tile_stride, void* stream) {
  MDZ_REQUIRE(src && dst, MDZ_EINVAL, "pack: NULL pointer");
  MDZ_REQUIRE(n_rows > 0 && k > 0 && dst_rows >= n_rows, MDZ_EINVAL, "pack: bad sizes");
  return launch_pack_weight(MDZ_BF16, src, n_rows, k, dst, dst_rows, tile_offset, tile_stride, (hipStream_t)stream,
                            true);
}

int64_t medusa_kv_bytes(const mdz_kv_desc* kv) {
  MDZ_REQUIRE(kv != nullptr, MDZ_EINVAL, "kv descriptor NULL");
  MDZ_REQUIRE(dtype_ok(kv->dtype), MDZ_EINVAL, "bad kv dtype %d", kv->dtype);
  MDZ_REQUIRE(kv->n_layers > 0 && kv->batch > 0 && kv->n_heads > 0 && kv->head_dim > 0 && kv->cap > 0, MDZ_EINVAL,
              "kv sizes must be positive");
  int rc = check_kv_quant(kv);
  if (rc) return rc;
  if (kv->quant) return kv8_bytes(geom(kv));
  return kv_elems(geom(kv)) * elem_bytes(kv->dtype);
}

int medusa_kv_init(const mdz_kv_desc* kv, void* stream) {
  int rc = check_kv(nullptr, kv, 0, 0);
  if (rc) return rc;
  const int64_t bytes = medusa_kv_bytes(kv);
  if (bytes < 0) return (int)bytes;
  if ((rc = launch_fill_zero(kv->k, bytes, (hipStream_t)stream))) return rc;
  if ((rc = launch_fill_zero(kv->v, bytes, (hipStream_t)stream))) return rc;
  if (kv->status) return launch_fill_zero(kv->status, 4, (hipStream_t)stream);
  return MDZ_OK;
}

int medusa_test_force_unfused_rope(int on) { return g_force_unfused_rope.exchange(on ? 1 : 0); }

static int kv_rw(const mdz_kv_desc* kv, int layer, int seq, int pos0, int n, void* k_rows, void* v_rows, bool to_cache,
                 void* stream) {
  int rc = check_kv(nullptr, kv, 0, 0);
  if (rc) return rc;
  MDZ_REQUIRE(layer >= 0 && layer < kv->n_layers && seq >= 0 && seq < kv->batch, MDZ_EINVAL,
              "kv copy: layer %d / seq %d out of range", layer, seq);
  MDZ_REQUIRE(pos0 >= 0 && n >= 0 && pos0 + n <= kv->cap, MDZ_ESHAPE, "kv copy: rows [%d,%d) exceed cap %d", pos0,
              pos0 + n, kv->cap);
  MDZ_REQUIRE(k_rows || v_rows, MDZ_EINVAL, "kv copy: both row buffers NULL");
  return launch_kv_copy(kv->dtype, geom(kv), kv->k, kv->v, layer, seq, pos0, n, k_rows, v_rows, to_cache,
                        (hipStream_t)stream);
}

int medusa_kv_write(const mdz_kv_desc* kv, int layer, int seq, int pos0, int n, const void* k_rows, const void* v_rows,
                    void* stream) {
  return kv_rw(kv, layer, seq, pos0, n, (void*)k_rows, (void*)v_rows, true, stream);
}

int medusa_kv_read(const mdz_kv_desc* kv, int layer, int seq, int pos0, int n, void* k_rows, void* v_rows,
                   void* stream) {
  return kv_rw(kv, layer, seq, pos0, n, k_rows, v_rows, false, stream);
}

int64_t medusa_workspace_bytes(const mdz_model_desc* model, int B, int max_prefix) {
  int rc = check_model(model);
  if (rc) return rc;
  MDZ_REQUIRE(B >= 0 && max_prefix >= 0, MDZ_EINVAL, "workspace: negative B or max_prefix");
  return carve(*model, B, max_prefix).total;
}

int medusa_heads(const mdz_model_desc* model, const mdz_weights* w, const void* hidden, const int32_t* src_row,
                 const int32_t* root_token, int B, int Tsrc, int32_t* cand_flat, int32_t* tree_tokens,
                 float* head_logits_opt, void* ws, int64_t ws_bytes, void* stream) {
  int rc = check_model(model);
  if (rc) return rc;
  const mdz_model_desc& m = *model;
  const TreeTables* t = host_tree(m.tree);
  MDZ_REQUIRE(w && hidden && cand_flat && tree_tokens && ws, MDZ_EINVAL, "medusa_heads: NULL pointer");
  MDZ_REQUIRE(B >= 0 && Tsrc >= 1, MDZ_EINVAL, "medusa_heads: B %d, Tsrc %d", B, Tsrc);
  MDZ_REQUIRE(w->n_medusa == t->K, MDZ_ESHAPE, "medusa_heads: %d heads given, the tree has depth %d", w->n_medusa,
              t->K);
  MDZ_REQUIRE(t->K == 0 || (w->head_w1 && w->head_lm), MDZ_EINVAL, "medusa_heads: head weight arrays NULL");
  for (int k = 0; k < t->K; ++k)
    MDZ_REQUIRE(w->head_w1[k] && w->head_lm[k], MDZ_EINVAL, "medusa_heads: head %d weights NULL", k);
  MDZ_REQUIRE(root_token || w->lm_head, MDZ_EINVAL, "medusa_heads: need root_token or the base lm_head");
  const Workspace L = carve(m, B, 0);
  MDZ_REQUIRE(ws_bytes >= L.total, MDZ_EWORKSPACE, "medusa_heads: workspace %lld < %lld bytes", (long long)ws_bytes,
              (long long)L.total);
  if (B == 0) return MDZ_OK;
  hipStream_t st = (hipStream_t)stream;
  char* wsb = (char*)ws;
  void* h = wsb + L.h;
  float* part = (float*)(wsb + L.part);
  void* z = wsb + L.z;
  Partials pr;
  const int64_t V = m.vocab;
  const int64_t ld = (int64_t)(t->K + 1) * V;  // row stride of the [B][K+1][V] logits
  float* hl = head_logits_opt ? head_logits_opt : (float*)(wsb + L.hlogits);
  if ((rc = launch_gather_rows(m.dtype, hidden, src_row, B, Tsrc, m.d, h, st))) return rc;
  // the heads' candidates are selected in one pair of launches after the last GEMM where the shape allows it
  const bool batched = heads_select_supported(m.tree, B, m.vocab, wsb + L.sel, L.sel_bytes);
  // slot 0: root token
  if (root_token) {
    if (!batched && (rc = launch_scatter_i32(root_token, cand_flat, B, t->n_cand, st))) return rc;
  } else {
    if ((rc = launch_gemm(m.dtype, h, w->lm_head, hl, B, m.vocab, m.d, ld, 1, &pr, st))) return rc;
    if (!batched && (rc = launch_topk(hl, B, m.vocab, ld, 1, cand_flat, t->n_cand, wsb + L.sel, L.sel_bytes, st))) return rc;
  }
  // the K first-layer GEMMs (each into its own partial-sum region), one launch for the K residual blocks, then the
  // K vocabulary projections back to back
  const int64_t head_part = gemm_part_elems(m.dtype, B, m.d, m.d);
  const int64_t zrow = (int64_t)B * m.d * elem_bytes(m.dtype);
  HeadBiases b1s{};
  for (int k = 0; k < t->K; ++k) b1s.p[k] = w->head_b1 ? w->head_b1[k] : nullptr;
  // The packed layout puts a matrix's 128-row bands one after the other, so first-layer matrices that lie back to
  // back in memory ARE the packed [K*d, d] stack of them: one launch then serves all heads (they read the same h).
  bool stacked = t->K > 1 && m.d % 128 == 0 && (int64_t)B * t->K * m.d < ((int64_t)1 << 31) / 16;
  const int64_t w1_bytes = medusa_packed_bytes(m.dtype, m.d, m.d);
  for (int k = 1; k < t->K && stacked; ++k)
    stacked = (const char*)w->head_w1[k] == (const char*)w->head_w1[0] + k * w1_bytes;
  if (stacked) {
    const int n_all = t->K * m.d;
    if ((rc = launch_gemm(m.dtype, h, w->head_w1[0], part, B, n_all, m.d, n_all, max_split_for(B), &pr, st))) return rc;
    if ((rc = launch_head_residual(m.dtype, h, pr, -1, b1s, t->K, z, B, m.d, st))) return rc;
  } else {
    for (int k = 0; k < t->K; ++k)
      if ((rc = launch_gemm(m.dtype, h, w->head_w1[k], part + k * head_part, B, m.d, m.d, m.d, max_split_for(B), &pr, st)))
        return rc;
    pr.p = part;
    if ((rc = launch_head_residual(m.dtype, h, pr, head_part, b1s, t->K, z, B, m.d, st))) return rc;
  }
  int seg = 1;
  for (int k = 0; k < t->K; ++k) {
    float* lk = hl + (int64_t)(k + 1) * V;
    if ((rc = launch_gemm(m.dtype, (char*)z + k * zrow, w->head_lm[k], lk, B, m.vocab, m.d, ld, 1, &pr, st))) return rc;
    if (!batched &&
        (rc = launch_topk(lk, B, m.vocab, ld, t->caps[k], cand_flat + seg, t->n_cand, wsb + L.sel, L.sel_bytes, st)))
      return rc;
    seg += t->caps[k];
  }
  if (batched && (rc = launch_heads_select(m.tree, hl, B, m.vocab, root_token, cand_flat, wsb + L.sel, st))) return rc;
  return launch_tree_tokens(m.tree, cand_flat, tree_tokens, B, st);
}

// shared by the two layer entry points: argument checks, then the launches over workspace `ws` carved as `L`
static int verify_layer_checked(const mdz_model_desc* model, const mdz_layer_weights* lw, int layer, float* x_inout,
                                const mdz_kv_desc* kv, const int32_t* seq_len, int B, int max_prefix) {
  int rc = check_model(model);
  if (rc) return rc;
  if ((rc = check_layer_weights(lw))) return rc;
  if ((rc = check_kv(model, kv, B, max_prefix))) return rc;
  const TreeTables* t = host_tree(model->tree);
  MDZ_REQUIRE(x_inout && seq_len, MDZ_EINVAL, "tree_verify_layer: NULL pointer");
  MDZ_REQUIRE(layer >= 0 && layer < kv->n_layers, MDZ_EINVAL, "tree_verify_layer: layer %d outside the cache's %d",
              layer, kv->n_layers);
  MDZ_REQUIRE(max_prefix + t->T <= kv->cap, MDZ_ESHAPE, "max_prefix %d + T %d exceeds kv cap %d", max_prefix, t->T,
              kv->cap);
  return MDZ_OK;
}

static int verify_layer_run(const mdz_model_desc* model, const mdz_layer_weights* lw, int layer, float* x_inout,
                            const mdz_kv_desc* kv, const int32_t* seq_len, int B, int max_prefix, char* ws,
                            const Workspace& L, hipStream_t st) {
  int rc;
  const TreeTables* t = host_tree(model->tree);
  const int rows = B * t->T;
  if ((rc = launch_first_norm_and_rope_table(model->dtype, x_inout, lw->g_attn, ws + L.xn, rows, model->d, model->rms_eps,
                                             model->tree, seq_len, B, max_prefix, model->head_dim, model->rope_base,
                                             (float*)(ws + L.rope_cs), kv->status, st)))
    return rc;
  return run_layer(*model, *lw, layer, x_inout, kv, seq_len, B, max_prefix, ws, L, nullptr, nullptr, st);
}

int tree_verify_layer(const mdz_model_desc* model, const mdz_layer_weights* lw, int layer, float* x_inout,
                      const mdz_kv_desc* kv, const int32_t* seq_len, int B, int max_prefix, void* ws, int64_t ws_bytes,
                      void* stream) {
  int rc = verify_layer_checked(model, lw, layer, x_inout, kv, seq_len, B, max_prefix);
  if (rc) return rc;
  MDZ_REQUIRE(ws, MDZ_EINVAL, "tree_verify_layer: NULL workspace");
  const Workspace L = carve(*model, B, max_prefix);
  MDZ_REQUIRE(ws_bytes >= L.total, MDZ_EWORKSPACE, "tree_verify_layer: workspace %lld < %lld bytes",
              (long long)ws_bytes, (long long)L.total);
  if (B == 0) return MDZ_OK;
  return verify_layer_run(model, lw, layer, x_inout, kv, seq_len, B, max_prefix, (char*)ws, L, (hipStream_t)stream);
}

int64_t tree_verify_layer_static_scratch_bytes(void) { return kStaticScratchBytes; }

int tree_verify_layer_static(const mdz_model_desc* model, const mdz_layer_weights* lw, int layer, float* x_inout,
                             const mdz_kv_desc* kv, const int32_t* seq_len, int B, int max_prefix, void* stream) {
  int rc = verify_layer_checked(model, lw, layer, x_inout, kv, seq_len, B, max_prefix);
  if (rc) return rc;
  const Workspace L = carve(*model, B, max_prefix, /*layer_only=*/true);
  MDZ_REQUIRE(L.total <= kStaticScratchBytes, MDZ_EWORKSPACE,
              "tree_verify_layer_static: this shape (B %d, max_prefix %d) needs %lld bytes of scratch, the built-in buffer "
              "holds %lld; use tree_verify_layer with a caller workspace",
              B, max_prefix, (long long)L.total, (long long)kStaticScratchBytes);
  if (B == 0) return MDZ_OK;
  void* ws = nullptr;
  if ((rc = static_scratch(&ws))) return rc;
  // every byte of the scratch a kernel reads was written earlier in the same call, so nothing needs clearing
  return verify_layer_run(model, lw, layer, x_inout, kv, seq_len, B, max_prefix, (char*)ws, L, (hipStream_t)stream);
}

int tree_verify_step(const mdz_model_desc* model, const mdz_weights* w, const int32_t* tree_tokens,
                     const mdz_kv_desc* kv, const int32_t* seq_len, int B, int max_prefix, int32_t* node_argmax,
                     void* hidden_out, float* logits_opt, void* ws, int64_t ws_bytes, void* stream) {
  int rc = check_model(model);
  if (rc) return rc;
  const mdz_model_desc& m = *model;
  MDZ_REQUIRE(w && w->layers && w->embed && w->lm_head && w->g_final, MDZ_EINVAL, "tree_verify_step: NULL weights");
  for (int l = 0; l < m.n_layers; ++l)
    if ((rc = check_layer_weights(&w->layers[l]))) return rc;
  if ((rc = check_kv(model, kv, B, max_prefix))) return rc;
  const TreeTables* t = host_tree(m.tree);
  MDZ_REQUIRE(tree_tokens && seq_len && node_argmax && ws, MDZ_EINVAL, "tree_verify_step: NULL pointer");
  MDZ_REQUIRE(max_prefix + t->T <= kv->cap, MDZ_ESHAPE, "max_prefix %d + T %d exceeds kv cap %d", max_prefix, t->T,
              kv->cap);
  const Workspace L = carve(m, B, max_prefix);
  MDZ_REQUIRE(ws_bytes >= L.total, MDZ_EWORKSPACE, "tree_verify_step: workspace %lld < %lld bytes",
              (long long)ws_bytes, (long long)L.total);
  if (B == 0) return MDZ_OK;
  hipStream_t st = (hipStream_t)stream;
  char* wsb = (char*)ws;
  const int rows = B * t->T;
  float* x = (float*)(wsb + L.x);
  if ((rc = launch_embed(m.dtype, w->embed, tree_tokens, x, rows, m.d, m.vocab, st))) return rc;
  void* xn = wsb + L.xn;
  void* hid = hidden_out ? hidden_out : xn;
  if ((rc = launch_first_norm_and_rope_table(m.dtype, x, w->layers[0].g_attn, xn, rows, m.d, m.rms_eps, m.tree, seq_len, B,
                                             max_prefix, m.head_dim, m.rope_base, (float*)(wsb + L.rope_cs), kv->status, st)))
    return rc;
  for (int l = 0; l < m.n_layers; ++l) {
    const bool last = l + 1 == m.n_layers;
    if ((rc = run_layer(m, w->layers[l], l, x, kv, seq_len, B, max_prefix, wsb, L,
                        last ? w->g_final : w->layers[l + 1].g_attn, last ? hid : xn, st)))
      return rc;
  }
  // No logits asked for: the LM head keeps each row's best column in its epilogue and a small merge finishes the
  // argmax, so the [rows, vocab] fp32 logits are neither written nor read back.
  if (!logits_opt && gemm_mfma_argmax_supported(m.dtype, rows, m.vocab, m.d)) {
    const int n_cand = gemm_mfma_argmax_cands(rows, m.vocab, m.d);
    if ((int64_t)rows * n_cand * (int64_t)sizeof(ArgCand) <= L.sel_bytes) {
      ArgCand* cand = (ArgCand*)(wsb + L.sel);
      if ((rc = launch_gemm_mfma_argmax(m.dtype, hid, w->lm_head, rows, m.vocab, m.d, cand, st))) return rc;
      return launch_argmax_merge(cand, rows, n_cand, node_argmax, st);
    }
  }
  float* logits = logits_opt ? logits_opt : (float*)(wsb + L.logits);
  Partials pr;
  if ((rc = launch_gemm(m.dtype, hid, w->lm_head, logits, rows, m.vocab, m.d, m.vocab, 1, &pr, st))) return rc;
  return launch_argmax(logits, rows, m.vocab, m.vocab, node_argmax, wsb + L.sel, L.sel_bytes, st);
}

int accept_longest_prefix(int tree, const int32_t* tree_tokens, const int32_t* node_argmax, int B,
                          int32_t* accept_len, int32_t* best_path, int32_t* acc_nodes, int32_t* acc_tokens,
                          int32_t* next_root, int32_t* last_node, void* stream) {
  MDZ_REQUIRE(host_tree(tree) != nullptr, MDZ_EINVAL, "bad tree id %d", tree);
  MDZ_REQUIRE(B >= 0, MDZ_EINVAL, "accept: B %d < 0", B);
  MDZ_REQUIRE(tree_tokens && node_argmax && accept_len && best_path && acc_nodes && acc_tokens && next_root &&
                  last_node,
              MDZ_EINVAL, "accept_longest_prefix: NULL pointer");
  return launch_accept(tree, tree_tokens, node_argmax, B, accept_len, best_path, acc_nodes, acc_tokens, next_root,
                       last_node, (hipStream_t)stream);
}

int kv_compact(const mdz_kv_desc* kv, int tree, const int32_t* acc_nodes, const int32_t* accept_len,
               int32_t* seq_len_inout, int32_t* kv_src_slots, int B, int max_prefix, void* stream) {
  const TreeTables* t = host_tree(tree);
  MDZ_REQUIRE(t != nullptr, MDZ_EINVAL, "bad tree id %d", tree);
  int rc = check_kv(nullptr, kv, B, max_prefix);
  if (rc) return rc;
  MDZ_REQUIRE(acc_nodes && accept_len && seq_len_inout && kv_src_slots, MDZ_EINVAL, "kv_compact: NULL pointer");
  MDZ_REQUIRE(max_prefix + t->T <= kv->cap, MDZ_ESHAPE, "max_prefix %d + T %d exceeds kv cap %d", max_prefix, t->T,
              kv->cap);
  return launch_kv_compact(kv->dtype, geom(kv), kv->k, kv->v, tree, acc_nodes, accept_len, seq_len_inout, kv_src_slots,
                           B, max_prefix, kv->status, (hipStream_t)stream);
}

#pragma GCC visibility pop
}  // extern "C"
