// Layout movers: weight packing, KV cache import/export, KV compaction (Section 3.2: the accepted
// nodes' cache rows become the next rows of the sequence, moved on the device through an index
// table, never through the host).
#include "kernels.h"

namespace mdz {

template <typename T, typename TD = T>
__global__ void pack_weight_kernel(const T* __restrict__ src, int64_t n_rows, int64_t k, TD* __restrict__ dst,
                                   int64_t kp, int64_t tile_offset, int64_t tile_stride, int64_t n_rows_pad) {
  constexpr int R = Packed<T>::kTileRows;
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_rows_pad * kp) return;
  int64_t n = idx / kp, kk = idx % kp;
  int64_t dst_row = (tile_offset + (n / R) * tile_stride) * R + n % R;
  T v = (n < n_rows && kk < k) ? src[n * k + kk] : from_float<T>(0.f);
  if constexpr (std::is_same<T, TD>::value)
    dst[Packed<T>::index(dst_row, kk, kp)] = v;
  else  // every bf16 value inside binary16's normal range is a binary16 value: the copy is exact there
    dst[Packed<T>::index(dst_row, kk, kp)] = from_float<TD>(to_float(v));
}

int launch_pack_weight(int dtype, const void* src, int64_t n_rows, int64_t k, void* dst, int64_t dst_rows,
                       int64_t tile_offset, int64_t tile_stride, hipStream_t st, bool to_f16) {
  ProfScope prof_(PROF_MISC, st);
  MDZ_REQUIRE(!to_f16 || dtype == MDZ_BF16, MDZ_EINVAL, "pack: only a bf16 matrix is repacked as binary16");
  const int R = is_16bit(dtype) ? kTileRowsBf16 : kTileRowsF32;
  const int64_t kp = is_16bit(dtype) ? Packed<bf16_t>::padded_k(k) : k;
  const int64_t n_pad = round_up(n_rows, R);
  const int64_t n_tiles = n_pad / R;
  MDZ_REQUIRE(tile_stride >= 1 && tile_offset >= 0, MDZ_EINVAL, "pack: bad tile offset/stride");
  MDZ_REQUIRE((tile_offset + (n_tiles - 1) * tile_stride + 1) * R <= round_up(dst_rows, R), MDZ_ESHAPE,
              "pack: tiles of a [%lld,%lld] matrix at offset %lld stride %lld exceed dst_rows %lld",
              (long long)n_rows, (long long)k, (long long)tile_offset, (long long)tile_stride,
              (long long)dst_rows);
  MDZ_REQUIRE(n_rows % R == 0 || tile_stride == 1, MDZ_ESHAPE,
              "pack: n_rows %lld is not a multiple of the tile height %d and tiles are interleaved",
              (long long)n_rows, R);
  const int64_t total = n_pad * kp;
  const int threads = 256;
  const int64_t blocks = (total + threads - 1) / threads;
  if (to_f16)
    pack_weight_kernel<bf16_t, f16_t><<<dim3((unsigned)blocks), threads, 0, st>>>(
        (const bf16_t*)src, n_rows, k, (f16_t*)dst, kp, tile_offset, tile_stride, n_pad);
  else if (is_16bit(dtype))  // bf16 and fp16 move as the same 16-bit words
    pack_weight_kernel<bf16_t><<<dim3((unsigned)blocks), threads, 0, st>>>(
        (const bf16_t*)src, n_rows, k, (bf16_t*)dst, kp, tile_offset, tile_stride, n_pad);
  else
    pack_weight_kernel<float><<<dim3((unsigned)blocks), threads, 0, st>>>((const float*)src, n_rows, k, (float*)dst,
                                                                          kp, tile_offset, tile_stride, n_pad);
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

// rows buffers are [n_heads][n][head_dim]
template <typename T>
__global__ void kv_copy_kernel(KvGeom g, T* kc, T* vc, int layer, int seq, int pos0, int n, T* k_rows, T* v_rows,
                               bool to_cache) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t total = (int64_t)g.n_heads * n * g.head_dim;
  if (idx >= total) return;
  int i = idx % g.head_dim;
  int r = (idx / g.head_dim) % n;
  int h = idx / ((int64_t)g.head_dim * n);
  int64_t ki = k_index(g, layer, seq, h, pos0 + r, i);
  int64_t vi = v_index(g, layer, seq, h, pos0 + r, i);
  if (to_cache) {
    if (k_rows) kc[ki] = k_rows[idx];
    if (v_rows) vc[vi] = v_rows[idx];
  } else {
    if (k_rows) k_rows[idx] = kc[ki];
    if (v_rows) v_rows[idx] = vc[vi];
  }
}

int launch_kv8_copy(int dtype, const KvGeom& g, void* kc, void* vc, int layer, int seq, int pos0, int n, void* k_rows,
                    void* v_rows, bool to_cache, hipStream_t st);
int launch_kv8_compact_rows(const KvGeom& g, void* kc, void* vc, int tree, const int32_t* acc_nodes,
                            const int32_t* accept_len, const int32_t* seq_len, int B, int max_prefix, hipStream_t st);

int launch_kv_copy(int dtype, const KvGeom& g, void* kc, void* vc, int layer, int seq, int pos0, int n,
                   void* k_rows, void* v_rows, bool to_cache, hipStream_t st) {
  if (g.quant) return launch_kv8_copy(dtype, g, kc, vc, layer, seq, pos0, n, k_rows, v_rows, to_cache, st);
  ProfScope prof_(PROF_MISC, st);
  if (n == 0) return MDZ_OK;
  int64_t total = (int64_t)g.n_heads * n * g.head_dim;
  int threads = 256;
  unsigned blocks = (unsigned)((total + threads - 1) / threads);
  if (is_16bit(dtype))  // bf16 and fp16 move as the same 16-bit words
    kv_copy_kernel<bf16_t><<<blocks, threads, 0, st>>>(g, (bf16_t*)kc, (bf16_t*)vc, layer, seq, pos0, n,
                                                       (bf16_t*)k_rows, (bf16_t*)v_rows, to_cache);
  else
    kv_copy_kernel<float><<<blocks, threads, 0, st>>>(g, (float*)kc, (float*)vc, layer, seq, pos0, n,
                                                      (float*)k_rows, (float*)v_rows, to_cache);
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

// One thread owns one (layer, head, feature) column of one sequence, for K and for V, and performs the
// row moves j = 1..A-1 in order.  Source slots never lie below their destination (node_j >= j) and a
// slot is read (as source of move j') before a later move j > j' overwrites it, so the in-place forward
// order is safe; columns are independent of each other.
template <typename T>
__global__ void kv_compact_kernel(KvGeom g, T* kc, T* vc, int tree, const int32_t* __restrict__ acc_nodes,
                                  const int32_t* __restrict__ accept_len, const int32_t* __restrict__ seq_len,
                                  int max_prefix) {
  const TreeTables& t = c_trees[tree];
  int b = blockIdx.y;
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t cols = (int64_t)g.n_layers * g.n_heads * g.head_dim;
  if (idx >= cols) return;
  int i = idx % g.head_dim;
  int h = (idx / g.head_dim) % g.n_heads;
  int l = idx / ((int64_t)g.head_dim * g.n_heads);
  int S = min(max(seq_len[b], 0), max_prefix);
  int A = min(max(accept_len[b], 0), t.K + 1);
  for (int j = 1; j < A; ++j) {
    int node = acc_nodes[b * (t.K + 1) + j];
    if (node < 0 || node >= t.T) break;
    if (node == j) continue;
    kc[k_index(g, l, b, h, S + j, i)] = kc[k_index(g, l, b, h, S + node, i)];
    vc[v_index(g, l, b, h, S + j, i)] = vc[v_index(g, l, b, h, S + node, i)];
  }
}

__global__ void kv_compact_finish_kernel(int tree, const int32_t* __restrict__ acc_nodes,
                                         const int32_t* __restrict__ accept_len, int32_t* seq_len,
                                         int32_t* kv_src_slots, int B, int max_prefix, int32_t* status) {
  const TreeTables& t = c_trees[tree];
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  if (status && (seq_len[b] < 0 || seq_len[b] > max_prefix)) atomicOr(status, MDZ_STATUS_SEQ_RANGE);
  int S = min(max(seq_len[b], 0), max_prefix);
  int A = min(max(accept_len[b], 0), t.K + 1);
  for (int j = 0; j <= t.K; ++j) {
    int node = acc_nodes[b * (t.K + 1) + j];
    kv_src_slots[b * (t.K + 1) + j] = (j < A && node >= 0) ? S + node : -1;
  }
  seq_len[b] = S + A;
}

__global__ void __launch_bounds__(256) fill_zero_kernel(uint32_t* __restrict__ p, int64_t n_words) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x * 4;
  for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4; i < n_words; i += stride) {
    if (i + 4 <= n_words && (reinterpret_cast<uintptr_t>(p) & 15) == 0)
      *reinterpret_cast<u32x4_t*>(p + i) = u32x4_t{0, 0, 0, 0};
    else
      for (int64_t j = i; j < n_words && j < i + 4; ++j) p[j] = 0;
  }
}

int launch_fill_zero(void* p, int64_t bytes, hipStream_t st) {
  MDZ_REQUIRE(p && bytes >= 0 && bytes % 4 == 0 && (reinterpret_cast<uintptr_t>(p) & 3) == 0, MDZ_EINVAL,
              "fill: needs a 4-byte aligned range");
  if (bytes == 0) return MDZ_OK;
  const int64_t words = bytes / 4;
  int64_t blocks = (words / 4 + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  if (blocks < 1) blocks = 1;
  fill_zero_kernel<<<(unsigned)blocks, 256, 0, st>>>((uint32_t*)p, words);
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

int launch_kv_compact(int dtype, const KvGeom& g, void* kc, void* vc, int tree, const int32_t* acc_nodes,
                      const int32_t* accept_len, int32_t* seq_len, int32_t* kv_src_slots, int B, int max_prefix,
                      int32_t* status, hipStream_t st) {
  ProfScope prof_(PROF_COMPACT, st);
  if (B == 0) return MDZ_OK;
  int64_t cols = (int64_t)g.n_layers * g.n_heads * g.head_dim;
  int threads = 256;
  dim3 grid((unsigned)((cols + threads - 1) / threads), B);
  if (g.quant) {
    int rc = launch_kv8_compact_rows(g, kc, vc, tree, acc_nodes, accept_len, seq_len, B, max_prefix, st);
    if (rc) return rc;
  } else if (is_16bit(dtype))  // bf16 and fp16 move as the same 16-bit words
    kv_compact_kernel<bf16_t><<<grid, threads, 0, st>>>(g, (bf16_t*)kc, (bf16_t*)vc, tree, acc_nodes, accept_len,
                                                        seq_len, max_prefix);
  else
    kv_compact_kernel<float><<<grid, threads, 0, st>>>(g, (float*)kc, (float*)vc, tree, acc_nodes, accept_len,
                                                       seq_len, max_prefix);
  MDZ_LAUNCH_CHECK();
  kv_compact_finish_kernel<<<(B + 63) / 64, 64, 0, st>>>(tree, acc_nodes, accept_len, seq_len, kv_src_slots, B,
                                                         max_prefix, status);
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

}  // namespace mdz
