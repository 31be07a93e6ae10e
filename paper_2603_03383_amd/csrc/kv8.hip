// 8-bit KV cache rows (layout and format in common.h): the boundary movers (quantise rows into the cache,
// return rows as value(code) * scale) and the compaction of accepted rows.  The attention kernels and the
// RoPE + KV-write kernels read and write the same layout in place.
#include "kernels.h"

namespace mdz {

namespace {
constexpr int kHD = 128;

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
}  // namespace

// One workgroup of 128 threads per (head, row): thread i owns feature i.  rows buffers are [n_heads][n][128].
template <typename E>
__global__ void __launch_bounds__(kHD) kv8_write_kernel(KvGeom g, uint8_t* kc, uint8_t* vc, int layer, int seq, int pos0,
                                                         int n, const E* __restrict__ k_rows, const E* __restrict__ v_rows) {
  __shared__ float red[2][2];
  const int r = blockIdx.x, h = blockIdx.y, i = threadIdx.x;
  const int pos = pos0 + r;
  const int64_t src = ((int64_t)h * n + r) * kHD + i;
  const int64_t base = kv8_head_base(g, layer, seq, h);
  const float kx = k_rows ? to_float(k_rows[src]) : 0.f, vx = v_rows ? to_float(v_rows[src]) : 0.f;
  const float km = wave_max(fabsf(kx)), vm = wave_max(fabsf(vx));
  if ((i & 63) == 0) red[0][i >> 6] = km, red[1][i >> 6] = vm;
  __syncthreads();
  const float ks = kv8_scale_of(fmaxf(red[0][0], red[0][1])), vs = kv8_scale_of(fmaxf(red[1][0], red[1][1]));
  if (k_rows) {
    kc[base + kv8_k_code(pos, i)] = (uint8_t)(kv8_pack4(kx, 0.f, 0.f, 0.f, ks) & 0xFFu);
    if (i == 0) *reinterpret_cast<float*>(kc + base + kv8_scale(pos)) = ks;
  }
  if (v_rows) {
    vc[base + kv8_v_code(pos, i)] = (uint8_t)(kv8_pack4(vx, 0.f, 0.f, 0.f, vs) & 0xFFu);
    if (i == 0) *reinterpret_cast<float*>(vc + base + kv8_scale(pos)) = vs;
  }
}

template <typename E>
__global__ void __launch_bounds__(kHD) kv8_read_kernel(KvGeom g, const uint8_t* kc, const uint8_t* vc, int layer, int seq,
                                                        int pos0, int n, E* __restrict__ k_rows, E* __restrict__ v_rows) {
  const int r = blockIdx.x, h = blockIdx.y, i = threadIdx.x;
  const int pos = pos0 + r;
  const int64_t dst = ((int64_t)h * n + r) * kHD + i;
  const int64_t base = kv8_head_base(g, layer, seq, h);
  auto value = [](uint8_t code) { return __builtin_amdgcn_cvt_pk_f32_fp8((uint32_t)code, false)[0]; };
  // The product is rounded to fp32 first, then to E.  The empty asm makes the fp32 product opaque: without it the
  // compiler folds the multiply into a mixed-precision instruction that rounds once, straight to fp16.
  auto row_value = [&](const uint8_t* c, int64_t code_at) {
    float p = value(c[base + code_at]) * *reinterpret_cast<const float*>(c + base + kv8_scale(pos));
    asm volatile("" : "+v"(p));
    return from_float<E>(p);
  };
  if (k_rows) k_rows[dst] = row_value(kc, kv8_k_code(pos, i));
  if (v_rows) v_rows[dst] = row_value(vc, kv8_v_code(pos, i));
}

int launch_kv8_copy(int dtype, const KvGeom& g, void* kc, void* vc, int layer, int seq, int pos0, int n, void* k_rows,
                    void* v_rows, bool to_cache, hipStream_t st) {
  ProfScope prof_(PROF_MISC, st);
  if (n == 0) return MDZ_OK;
  dim3 grid(n, g.n_heads);
  if (to_cache)
    MDZ_WITH_ELEM16(dtype, (kv8_write_kernel<E><<<grid, kHD, 0, st>>>(g, (uint8_t*)kc, (uint8_t*)vc, layer, seq, pos0, n,
                                                                      (const E*)k_rows, (const E*)v_rows)));
  else
    MDZ_WITH_ELEM16(dtype, (kv8_read_kernel<E><<<grid, kHD, 0, st>>>(g, (const uint8_t*)kc, (const uint8_t*)vc, layer, seq,
                                                                     pos0, n, (E*)k_rows, (E*)v_rows)));
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

// Row moves of the accepted path, as in kv_compact_kernel: one thread owns one (layer, head, column) of one sequence
// and performs the moves j = 1..A-1 in order; column 128 is the row's scale.  Codes and scales move untouched.
__global__ void kv8_compact_kernel(KvGeom g, uint8_t* kc, uint8_t* vc, int tree, const int32_t* __restrict__ acc_nodes,
                                   const int32_t* __restrict__ accept_len, const int32_t* __restrict__ seq_len,
                                   int max_prefix) {
  const TreeTables& t = c_trees[tree];
  const int b = blockIdx.y;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t cols = (int64_t)g.n_layers * g.n_heads * (kHD + 1);
  if (idx >= cols) return;
  const int i = idx % (kHD + 1);
  const int h = (idx / (kHD + 1)) % g.n_heads;
  const int l = idx / ((int64_t)(kHD + 1) * g.n_heads);
  const int64_t base = kv8_head_base(g, l, b, h);
  const int S = min(max(seq_len[b], 0), max_prefix);
  const int A = min(max(accept_len[b], 0), t.K + 1);
  for (int j = 1; j < A; ++j) {
    const int node = acc_nodes[b * (t.K + 1) + j];
    if (node < 0 || node >= t.T) break;
    if (node == j) continue;
    if (i < kHD) {
      kc[base + kv8_k_code(S + j, i)] = kc[base + kv8_k_code(S + node, i)];
      vc[base + kv8_v_code(S + j, i)] = vc[base + kv8_v_code(S + node, i)];
    } else {
      *reinterpret_cast<float*>(kc + base + kv8_scale(S + j)) = *reinterpret_cast<const float*>(kc + base + kv8_scale(S + node));
      *reinterpret_cast<float*>(vc + base + kv8_scale(S + j)) = *reinterpret_cast<const float*>(vc + base + kv8_scale(S + node));
    }
  }
}

int launch_kv8_compact_rows(const KvGeom& g, void* kc, void* vc, int tree, const int32_t* acc_nodes,
                            const int32_t* accept_len, const int32_t* seq_len, int B, int max_prefix, hipStream_t st) {
  const int64_t cols = (int64_t)g.n_layers * g.n_heads * (kHD + 1);
  const int threads = 256;
  dim3 grid((unsigned)((cols + threads - 1) / threads), B);
  kv8_compact_kernel<<<grid, threads, 0, st>>>(g, (uint8_t*)kc, (uint8_t*)vc, tree, acc_nodes, accept_len, seq_len,
                                               max_prefix);
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

}  // namespace mdz
