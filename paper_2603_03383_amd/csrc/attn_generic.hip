// Portable tree-masked attention (Section 3.2: every tree node attends to the whole prefix and to the
// tree slots its row of the static visibility matrix allows).  One workgroup per (node, head); keys are
// processed in chunks with a running max / sum, so any prefix length fits.  Used for fp32 storage and
// for head sizes the MFMA kernel does not cover.
#include "kernels.h"

namespace mdz {

constexpr int kAttnChunk = 1024;

__device__ inline float wave_max_f(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ inline float wave_sum_f(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <typename T>
__global__ void __launch_bounds__(256) attn_generic_kernel(int tree, const T* __restrict__ q, KvGeom g,
                                                           const T* __restrict__ kc, const T* __restrict__ vc,
                                                           int layer, const int32_t* __restrict__ seq_len,
                                                           int max_prefix, T* __restrict__ att_out) {
  const TreeTables& t = c_trees[tree];
  __shared__ float qs[256];
  __shared__ float p[kAttnChunk];
  __shared__ float red[4];
  const int row = blockIdx.x, h = blockIdx.y;
  const int b = row / t.T, i = row % t.T;
  const int hd = g.head_dim, d = q_heads(g) * hd;
  const int hk = h / g.group;  // the key/value head this query head reads
  const int S = min(max(seq_len[b], 0), max_prefix);
  const int n_slots = S + t.T;
  const uint64_t mask = t.anc_mask[i];
  const float scale = 1.0f / sqrtf((float)hd);
  const int tid = threadIdx.x;
  if (tid < hd) qs[tid] = to_float(q[(int64_t)row * d + h * hd + tid]) * scale;
  __syncthreads();
  float m_run = -INFINITY, l_run = 0.f, acc = 0.f;
  for (int c0 = 0; c0 < n_slots; c0 += kAttnChunk) {
    const int c1 = min(c0 + kAttnChunk, n_slots);
    float lm = -INFINITY;
    for (int j = c0 + tid; j < c1; j += 256) {
      bool vis = j < S || ((mask >> (j - S)) & 1ull);
      float s = -INFINITY;
      if (vis) {
        s = 0.f;
        for (int e = 0; e < hd; ++e) s += qs[e] * to_float(kc[k_index(g, layer, b, hk, j, e)]);
      }
      p[j - c0] = s;
      lm = fmaxf(lm, s);
    }
    lm = wave_max_f(lm);
    if ((tid & 63) == 0) red[tid >> 6] = lm;
    __syncthreads();
    float cm = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float m_new = fmaxf(m_run, cm);
    float ls = 0.f;
    if (m_new > -INFINITY) {
      for (int j = c0 + tid; j < c1; j += 256) {
        float s = p[j - c0];
        float e = s > -INFINITY ? expf(s - m_new) : 0.f;
        p[j - c0] = e;
        ls += e;
      }
    } else {
      for (int j = c0 + tid; j < c1; j += 256) p[j - c0] = 0.f;
    }
    ls = wave_sum_f(ls);
    if ((tid & 63) == 0) red[tid >> 6] = ls;
    __syncthreads();
    float csum = red[0] + red[1] + red[2] + red[3];
    float old_scale = m_run > -INFINITY ? expf(m_run - m_new) : 0.f;
    l_run = l_run * old_scale + csum;
    if (tid < hd) {
      float a = acc * old_scale;
      for (int j = c0; j < c1; ++j) a += p[j - c0] * to_float(vc[v_index(g, layer, b, hk, j, tid)]);
      acc = a;
    }
    m_run = m_new;
    __syncthreads();
  }
  if (tid < hd) att_out[(int64_t)row * d + h * hd + tid] = from_float<T>(acc / l_run);
}

int launch_attention_generic(int dtype, int tree, const void* q, const KvGeom& g, const void* kc, const void* vc,
                             int layer, const int32_t* seq_len, int B, int max_prefix, void* att_out,
                             hipStream_t st) {
  ProfScope prof_(PROF_ATTN, st);
  const TreeTables* t = host_tree(tree);
  if (B == 0) return MDZ_OK;
  MDZ_REQUIRE(g.head_dim <= 256, MDZ_EUNSUPPORTED, "attention: head_dim %d > 256", g.head_dim);
  dim3 grid(B * t->T, q_heads(g));
  MDZ_WITH_ELEM(dtype, (attn_generic_kernel<E><<<grid, 256, 0, st>>>(tree, (const E*)q, g, (const E*)kc, (const E*)vc, layer,
                                                                     seq_len, max_prefix, (E*)att_out)));
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

}  // namespace mdz
