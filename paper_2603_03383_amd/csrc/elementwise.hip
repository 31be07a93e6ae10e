// Small row-wise kernels around the GEMMs: embedding gather, RMSNorm, RoPE + KV write, SwiGLU, the
// Medusa head residual (Section 3.1: z = h + SiLU(W1 h)).
#include "kernels.h"

namespace mdz {

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// blockDim.x == 256
__device__ inline float block_sum_256(float v, float* smem4) {
  v = wave_sum(v);
  int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) smem4[w] = v;
  __syncthreads();
  float r = smem4[0] + smem4[1] + smem4[2] + smem4[3];
  __syncthreads();
  return r;
}

template <typename T>
struct alignas(sizeof(T) * 4) Quad {
  T v[4];
};

template <typename T>
__global__ void embed_kernel(const T* __restrict__ embed, const int32_t* __restrict__ tokens, float* __restrict__ x,
                             int d, int vocab) {
  int r = blockIdx.x;
  int tok = tokens[r];
  tok = min(max(tok, 0), vocab - 1);
  const T* src = embed + (int64_t)tok * d;
  if (d % 4 == 0 && (reinterpret_cast<uintptr_t>(embed) | reinterpret_cast<uintptr_t>(x)) % 16 == 0) {  // four elements per thread
    for (int i = threadIdx.x * 4; i < d; i += blockDim.x * 4) {
      const Quad<T> q = *reinterpret_cast<const Quad<T>*>(src + i);
      *reinterpret_cast<float4*>(x + (int64_t)r * d + i) = float4{to_float(q.v[0]), to_float(q.v[1]), to_float(q.v[2]), to_float(q.v[3])};
    }
    return;
  }
  for (int i = threadIdx.x; i < d; i += blockDim.x) x[(int64_t)r * d + i] = to_float(src[i]);
}

int launch_embed(int dtype, const void* embed, const int32_t* tokens, float* x, int rows, int d, int vocab,
                 hipStream_t st) {
  ProfScope prof_(PROF_EMBED, st);
  if (rows == 0) return MDZ_OK;
  MDZ_WITH_ELEM(dtype, (embed_kernel<E><<<rows, 1024, 0, st>>>((const E*)embed, tokens, x, d, vocab)));
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

// RoPE table entry idx = (row, i): cos/sin of (S_b + depth[n]) * base^(-2i/hd), the angle evaluated in double so that
// long prefixes keep full fp32 accuracy.  This opens every verify pass: it also reports a length the pass has to clamp.
__device__ inline void rope_table_entry(int idx, int tree, const int32_t* __restrict__ seq_len, int B, int max_prefix, int half,
                                        double log2_base, float* __restrict__ cs, int32_t* status) {
  const TreeTables& t = c_trees[tree];
  if (idx >= B * t.T * half) return;
  int i = idx % half;
  int n = (idx / half) % t.T;
  int b = idx / (half * t.T);
  if (status && i == 0 && n == 0 && (seq_len[b] < 0 || seq_len[b] > max_prefix)) atomicOr(status, MDZ_STATUS_SEQ_RANGE);
  int S = min(max(seq_len[b], 0), max_prefix);
  double pos = (double)(S + t.depth[n]);
  double ang = pos * exp2(-(double)i / (double)half * log2_base);
  cs[2 * idx] = (float)cos(ang);
  cs[2 * idx + 1] = (float)sin(ang);
}

// The RoPE table of a verify pass, computed by extra workgroups of the pass's first norm launch (the two are
// independent; a launch of its own would cost more than the table takes).  n_blocks == 0: no table in this launch.
struct RopeJob {
  const int32_t* seq_len;
  float* cs;
  int32_t* status;
  int tree, B, max_prefix, half, n_blocks;
  double log2_base;
};

// x[r] += sum_s P[s][r] (fixed order s = 0..n_part-1), then xn[r] = x[r] * rsqrt(mean(x[r]^2) + eps) * g.
// Either half is optional: P == nullptr skips the residual update, xn == nullptr skips the norm.
// Workgroups beyond the rows (gridDim.x = rows + rope.n_blocks) fill the RoPE table.
template <typename T, typename TO = T>
__global__ void __launch_bounds__(256) residual_rmsnorm_kernel(float* __restrict__ x, Partials part,
                                                               const T* __restrict__ g, TO* __restrict__ xn, int d,
                                                               float eps, int rows, RopeJob rope) {
  if ((int)blockIdx.x >= rows) {
    rope_table_entry((blockIdx.x - rows) * 256 + threadIdx.x, rope.tree, rope.seq_len, rope.B, rope.max_prefix, rope.half,
                     rope.log2_base, rope.cs, rope.status);
    return;
  }
  const float* P = part.p;
  const int64_t part_stride = part.stride, ldp = part.ld;
  __shared__ float red[4];
  int r = blockIdx.x;
  float* xr = x + (int64_t)r * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) {
    float v = xr[i];
    if (P) {
      const int n_part = part.count(i);
      for (int s = 0; s < n_part; ++s) v += P[(int64_t)s * part_stride + (int64_t)r * ldp + i];
      xr[i] = v;
    }
    ss += v * v;
  }
  if (!xn) return;
  ss = block_sum_256(ss, red);
  float rs = 1.0f / sqrtf(ss / (float)d + eps);
  for (int i = threadIdx.x; i < d; i += 256) xn[(int64_t)r * d + i] = from_float<TO>(xr[i] * rs * to_float(g[i]));
}

// Fast path for d == 4 * blockDim (d = 4096 with 1024 threads): every thread owns one float4 of the row, all
// partial loads are issued at once, and the row never leaves registers between the two halves.
template <typename T, typename TO = T>
__global__ void __launch_bounds__(1024) residual_rmsnorm_vec4_kernel(float* __restrict__ x, Partials part,
                                                                     const T* __restrict__ g, TO* __restrict__ xn,
                                                                     int d, float eps, int rows, RopeJob rope) {
  if ((int)blockIdx.x >= rows) {
    rope_table_entry((blockIdx.x - rows) * 1024 + threadIdx.x, rope.tree, rope.seq_len, rope.B, rope.max_prefix, rope.half,
                     rope.log2_base, rope.cs, rope.status);
    return;
  }
  const float* P = part.p;
  const int64_t part_stride = part.stride, ldp = part.ld;
  __shared__ float red[16];
  const int r = blockIdx.x, i = threadIdx.x * 4;
  float4 v = *reinterpret_cast<const float4*>(x + (int64_t)r * d + i);
  if (P) {
    const int n_part = part.count(i);  // band widths are multiples of 32, so one count covers the float4
    // the first twelve slots (the most the streaming GEMM makes) are requested together, then added in slot order
    constexpr int kTogether = 12;
    const float* src = P + (int64_t)r * ldp + i;
    float4 p[kTogether];
#pragma unroll
    for (int s = 0; s < kTogether; ++s)
      if (s < n_part) p[s] = *reinterpret_cast<const float4*>(src + (int64_t)s * part_stride);
#pragma unroll
    for (int s = 0; s < kTogether; ++s)
      if (s < n_part) v.x += p[s].x, v.y += p[s].y, v.z += p[s].z, v.w += p[s].w;
    for (int s = kTogether; s < n_part; ++s) {
      const float4 q = *reinterpret_cast<const float4*>(src + (int64_t)s * part_stride);
      v.x += q.x, v.y += q.y, v.z += q.z, v.w += q.w;
    }
    *reinterpret_cast<float4*>(x + (int64_t)r * d + i) = v;
  }
  if (!xn) return;
  float ss = wave_sum(v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < 16; ++w) tot += red[w];
  const float rs = 1.0f / sqrtf(tot / (float)d + eps);
  const Quad<T> gi = *reinterpret_cast<const Quad<T>*>(g + i);  // gains and output: one 8- or 16-byte access each
  Quad<TO> o;
  o.v[0] = from_float<TO>(v.x * rs * to_float(gi.v[0]));
  o.v[1] = from_float<TO>(v.y * rs * to_float(gi.v[1]));
  o.v[2] = from_float<TO>(v.z * rs * to_float(gi.v[2]));
  o.v[3] = from_float<TO>(v.w * rs * to_float(gi.v[3]));
  *reinterpret_cast<Quad<TO>*>(xn + (int64_t)r * d + i) = o;
}

// out_dtype: element type of xn.  It differs from dtype (the gains' type) in one case only: a bf16 model whose
// feed-forward block takes binary16 operands.
static int launch_norm_with_rope(int dtype, int out_dtype, float* x, const Partials& part, const void* g, void* xn,
                                 int rows, int d, float eps, RopeJob rope, hipStream_t st) {
  if (rows == 0) return MDZ_OK;
  const int entries = rope.n_blocks ? rope.B * host_tree(rope.tree)->T * rope.half : 0;
  if (out_dtype != dtype) {
    MDZ_REQUIRE(dtype == MDZ_BF16 && out_dtype == MDZ_FP16 && rope.n_blocks == 0, MDZ_EINVAL,
                "norm: only bf16 gains with binary16 output may differ in type");
    if (d == 4096 && part.ld % 4 == 0 && part.stride % 4 == 0 && ((uintptr_t)g | (uintptr_t)xn) % 16 == 0)
      launch_timed(PROF_NORM, residual_rmsnorm_vec4_kernel<bf16_t, f16_t>, rows, 1024, 0, st, x, part, (const bf16_t*)g, (f16_t*)xn, d,
                   eps, rows, rope);
    else
      launch_timed(PROF_NORM, residual_rmsnorm_kernel<bf16_t, f16_t>, rows, 256, 0, st, x, part, (const bf16_t*)g, (f16_t*)xn, d, eps,
                   rows, rope);
    MDZ_LAUNCH_CHECK();
    return MDZ_OK;
  }
  if (d == 4096 && part.ld % 4 == 0 && part.stride % 4 == 0 && ((uintptr_t)g | (uintptr_t)xn) % 16 == 0) {
    rope.n_blocks = (entries + 1023) / 1024;
    MDZ_WITH_ELEM(dtype, (launch_timed(PROF_NORM, residual_rmsnorm_vec4_kernel<E>, rows + rope.n_blocks, 1024, 0, st, x, part,
                                       (const E*)g, (E*)xn, d, eps, rows, rope)));
  } else {
    rope.n_blocks = (entries + 255) / 256;
    MDZ_WITH_ELEM(dtype, (launch_timed(PROF_NORM, residual_rmsnorm_kernel<E>, rows + rope.n_blocks, 256, 0, st, x, part,
                                       (const E*)g, (E*)xn, d, eps, rows, rope)));
  }
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

int launch_residual_rmsnorm(int dtype, float* x, const Partials& part, const void* g, void* xn, int rows, int d,
                            float eps, hipStream_t st, int out_dtype) {
  return launch_norm_with_rope(dtype, out_dtype < 0 ? dtype : out_dtype, x, part, g, xn, rows, d, eps, RopeJob{}, st);
}

int launch_first_norm_and_rope_table(int dtype, float* x, const void* g, void* xn, int rows, int d, float eps, int tree,
                                     const int32_t* seq_len, int B, int max_prefix, int head_dim, float rope_base, float* cs,
                                     int32_t* status, hipStream_t st) {
  RopeJob rope{seq_len, cs, status, tree, B, max_prefix, head_dim / 2, 1, log2((double)rope_base)};
  return launch_norm_with_rope(dtype, dtype, x, single_slot(nullptr, 0, 0), g, xn, rows, d, eps, rope, st);
}

// grid (B*T, query heads), block = head_dim/2 threads... generalised: threads stride over i < half.  The QKV GEMM
// output has the query heads' columns first, then the key heads', then the value heads'; the first query head of a
// group also rotates and stores its group's key row and stores its value row.
template <typename T>
__global__ void rope_kvwrite_kernel(int tree, Partials part, const float* __restrict__ cs,
                                    T* __restrict__ q_out, KvGeom g, T* __restrict__ kc, T* __restrict__ vc, int layer,
                                    const int32_t* __restrict__ seq_len, int max_prefix) {
  const TreeTables& t = c_trees[tree];
  int row = blockIdx.x;  // b*T + n
  int h = blockIdx.y;
  int b = row / t.T, n = row % t.T;
  int hd = g.head_dim, half = hd / 2, dq = q_heads(g) * hd, dkv = g.n_heads * hd;
  int S = min(max(seq_len[b], 0), max_prefix);
  int slot = S + n;
  const float* qr = part.p + (int64_t)row * part.ld;
  auto rd = [&](int col) {  // fixed-order sum of the partial-sum slots of one column
    const int n_part = part.count(col);
    float v = 0.f;
    for (int p = 0; p < n_part; ++p) v += qr[(int64_t)p * part.stride + col];
    return v;
  };
  const bool leader = h % g.group == 0;
  const int hk = h / g.group;
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    float c = cs[((int64_t)row * half + i) * 2], s = cs[((int64_t)row * half + i) * 2 + 1];
    float qa = rd(h * hd + i), qb = rd(h * hd + i + half);
    q_out[(int64_t)row * dq + h * hd + i] = from_float<T>(qa * c - qb * s);
    q_out[(int64_t)row * dq + h * hd + i + half] = from_float<T>(qb * c + qa * s);
    if (leader) {
      float ka = rd(dq + hk * hd + i), kb = rd(dq + hk * hd + i + half);
      float va = rd(dq + dkv + hk * hd + i), vb = rd(dq + dkv + hk * hd + i + half);
      kc[k_index(g, layer, b, hk, slot, i)] = from_float<T>(ka * c - kb * s);
      kc[k_index(g, layer, b, hk, slot, i + half)] = from_float<T>(kb * c + ka * s);
      vc[v_index(g, layer, b, hk, slot, i)] = from_float<T>(va);
      vc[v_index(g, layer, b, hk, slot, i + half)] = from_float<T>(vb);
    }
  }
}

// bf16 or fp16 / head_dim 128 / tiled cache: one thread per (head, matrix, 4 rotary pairs), all partial-sum slots of its
// two float4 in flight at once.  grid (rows, query heads / 4), 192 threads; the key / value threads of a query head
// that does not lead its group have nothing to do.
constexpr int kMaxSlots = 8;
template <typename E>
__device__ inline uint2 pack4(float a, float b, float c, float d) {
  return uint2{Elem16<E>::pack2(a, b), Elem16<E>::pack2(c, d)};
}
// Q8: the cache holds 8-bit rows (common.h); the 16 threads of a (head, matrix) row agree on the row's scale first.
template <typename E, bool Q8>
__global__ void __launch_bounds__(192) rope_kvwrite_vec_kernel(int tree, Partials part, const float* __restrict__ cs,
                                                               E* __restrict__ q_out, KvGeom g, E* __restrict__ kc,
                                                               E* __restrict__ vc, int layer,
                                                               const int32_t* __restrict__ seq_len, int max_prefix) {
  const TreeTables& t = c_trees[tree];
  const int row = blockIdx.x, h = blockIdx.y * 4 + threadIdx.x / 48, w = threadIdx.x % 48;
  const int which = w / 16, i = (w % 16) * 4;  // matrix (q,k,v) and first of 4 features; partner at i + 64
  const int b = row / t.T, n = row % t.T;
  const int dq = q_heads(g) * 128, dkv = g.n_heads * 128;
  const int S = min(max(seq_len[b], 0), max_prefix);
  const int slot = S + n;
  const int hk = h / g.group;
  if (which != 0 && h % g.group != 0) return;
  const int col = (which == 0 ? h * 128 : which == 1 ? dq + hk * 128 : dq + dkv + hk * 128) + i;
  const float* src = part.p + (int64_t)row * part.ld + col;
  const int n_part = part.count(col);
  float4 lo[kMaxSlots], hi[kMaxSlots];
#pragma unroll
  for (int p = 0; p < kMaxSlots; ++p)
    if (p < n_part) {
      lo[p] = *reinterpret_cast<const float4*>(src + (int64_t)p * part.stride);
      hi[p] = *reinterpret_cast<const float4*>(src + (int64_t)p * part.stride + 64);
    }
  const float4 c01 = *reinterpret_cast<const float4*>(cs + ((int64_t)row * 64 + i) * 2);      // c0 s0 c1 s1
  const float4 c23 = *reinterpret_cast<const float4*>(cs + ((int64_t)row * 64 + i) * 2 + 4);  // c2 s2 c3 s3
  float4 a = {0.f, 0.f, 0.f, 0.f}, bq = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int p = 0; p < kMaxSlots; ++p)
    if (p < n_part) {
      a.x += lo[p].x, a.y += lo[p].y, a.z += lo[p].z, a.w += lo[p].w;
      bq.x += hi[p].x, bq.y += hi[p].y, bq.z += hi[p].z, bq.w += hi[p].w;
    }
  if (which == 2) {
    const float va[4] = {a.x, a.y, a.z, a.w}, vb[4] = {bq.x, bq.y, bq.z, bq.w};
    if constexpr (Q8) {
      float am = fmaxf(fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))),
                       fmaxf(fmaxf(fabsf(bq.x), fabsf(bq.y)), fmaxf(fabsf(bq.z), fabsf(bq.w))));
#pragma unroll
      for (int o = 1; o < 16; o <<= 1) am = fmaxf(am, __shfl_xor(am, o, 64));
      const float vs = kv8_scale_of(am);
      uint8_t* v8 = reinterpret_cast<uint8_t*>(vc) + kv8_head_base(g, layer, b, hk);
      const uint32_t wl = kv8_pack4(a.x, a.y, a.z, a.w, vs), wh = kv8_pack4(bq.x, bq.y, bq.z, bq.w, vs);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v8[kv8_v_code(slot, i + e)] = (uint8_t)(wl >> (8 * e));
        v8[kv8_v_code(slot, i + 64 + e)] = (uint8_t)(wh >> (8 * e));
      }
      if (w % 16 == 0) *reinterpret_cast<float*>(v8 + kv8_scale(slot)) = vs;
      return;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      vc[v_index(g, layer, b, hk, slot, i + e)] = from_float<E>(va[e]);
      vc[v_index(g, layer, b, hk, slot, i + 64 + e)] = from_float<E>(vb[e]);
    }
    return;
  }
  if constexpr (Q8) {
    if (which == 1) {  // rotated key row -> codes: 4 consecutive features of one key are 4 contiguous bytes
      const float r0 = a.x * c01.x - bq.x * c01.y, r1 = a.y * c01.z - bq.y * c01.w, r2 = a.z * c23.x - bq.z * c23.y,
                  r3 = a.w * c23.z - bq.w * c23.w;
      const float t0 = bq.x * c01.x + a.x * c01.y, t1 = bq.y * c01.z + a.y * c01.w, t2 = bq.z * c23.x + a.z * c23.y,
                  t3 = bq.w * c23.z + a.w * c23.w;
      float am = fmaxf(fmaxf(fmaxf(fabsf(r0), fabsf(r1)), fmaxf(fabsf(r2), fabsf(r3))),
                       fmaxf(fmaxf(fabsf(t0), fabsf(t1)), fmaxf(fabsf(t2), fabsf(t3))));
#pragma unroll
      for (int o = 1; o < 16; o <<= 1) am = fmaxf(am, __shfl_xor(am, o, 64));
      const float ks = kv8_scale_of(am);
      uint8_t* k8 = reinterpret_cast<uint8_t*>(kc) + kv8_head_base(g, layer, b, hk);
      *reinterpret_cast<uint32_t*>(k8 + kv8_k_code(slot, i)) = kv8_pack4(r0, r1, r2, r3, ks);
      *reinterpret_cast<uint32_t*>(k8 + kv8_k_code(slot, i + 64)) = kv8_pack4(t0, t1, t2, t3, ks);
      if (w % 16 == 0) *reinterpret_cast<float*>(k8 + kv8_scale(slot)) = ks;
      return;
    }
  }
  const uint2 rlo = pack4<E>(a.x * c01.x - bq.x * c01.y, a.y * c01.z - bq.y * c01.w, a.z * c23.x - bq.z * c23.y,
                             a.w * c23.z - bq.w * c23.w);
  const uint2 rhi = pack4<E>(bq.x * c01.x + a.x * c01.y, bq.y * c01.z + a.y * c01.w, bq.z * c23.x + a.z * c23.y,
                             bq.w * c23.z + a.w * c23.w);
  if (which == 0) {
    E* qo = q_out + (int64_t)row * dq + h * 128 + i;
    *reinterpret_cast<uint2*>(qo) = rlo;
    *reinterpret_cast<uint2*>(qo + 64) = rhi;
  } else {  // 4 consecutive features of one key are 8 contiguous bytes of the tiled K layout
    *reinterpret_cast<uint2*>(kc + k_index(g, layer, b, hk, slot, i)) = rlo;
    *reinterpret_cast<uint2*>(kc + k_index(g, layer, b, hk, slot, i + 64)) = rhi;
  }
}

int launch_rope_kvwrite(int dtype, int tree, const Partials& qkv, const float* cs, void* q_out, const KvGeom& g,
                        void* kc, void* vc, int layer, const int32_t* seq_len, int B, int max_prefix,
                        hipStream_t st) {
  ProfScope prof_(PROF_ROPE, st);
  const TreeTables* t = host_tree(tree);
  if (B == 0) return MDZ_OK;
  dim3 grid(B * t->T, q_heads(g));
  int threads = g.head_dim / 2 <= 64 ? 64 : 128;
  if (is_16bit(dtype) && g.tiled && g.head_dim == 128 && q_heads(g) % 4 == 0 && qkv.n <= kMaxSlots &&
      qkv.stride % 4 == 0 && (qkv.split_grid == 0 || qkv.band_cols % 128 == 0)) {
    if (g.quant)
      MDZ_WITH_ELEM16(dtype, (rope_kvwrite_vec_kernel<E, true><<<dim3(B * t->T, q_heads(g) / 4), 192, 0, st>>>(
                                 tree, qkv, cs, (E*)q_out, g, (E*)kc, (E*)vc, layer, seq_len, max_prefix)));
    else
      MDZ_WITH_ELEM16(dtype, (rope_kvwrite_vec_kernel<E, false><<<dim3(B * t->T, q_heads(g) / 4), 192, 0, st>>>(
                                 tree, qkv, cs, (E*)q_out, g, (E*)kc, (E*)vc, layer, seq_len, max_prefix)));
  } else if (g.quant) {
    MDZ_FAIL(MDZ_EUNSUPPORTED, "8-bit kv rows: the QKV output does not fit the vectorised RoPE kernel (slots %d, stride %lld)",
             qkv.n, (long long)qkv.stride);
  } else {
    MDZ_WITH_ELEM(dtype, (rope_kvwrite_kernel<E><<<grid, threads, 0, st>>>(tree, qkv, cs, (E*)q_out, g, (E*)kc, (E*)vc, layer,
                                                                           seq_len, max_prefix)));
  }
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

__device__ inline float silu_f(float v) { return v / (1.0f + expf(-v)); }

// gate feature f sits at column (2*(f/R))*R + f%R of gu, up at (2*(f/R)+1)*R + f%R (R = tile rows)
template <typename T>
__global__ void swiglu_kernel(Partials part, T* __restrict__ u, int M, int F) {
  const float* gu = part.p;
  constexpr int R = Packed<T>::kTileRows;
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)M * F) return;
  int f = idx % F;
  int64_t m = idx / F;
  int64_t col = (int64_t)(2 * (f / R)) * R + f % R;
  float gv = 0.f, uv = 0.f;
  const int ng = part.count((int)col), nu = part.count((int)col + R);
  for (int p = 0; p < ng; ++p) gv += gu[(int64_t)p * part.stride + m * 2 * F + col];
  for (int p = 0; p < nu; ++p) uv += gu[(int64_t)p * part.stride + m * 2 * F + col + R];
  u[idx] = from_float<T>(silu_f(gv) * uv);
}

// bf16 / fp16: one thread per 4 features, gate and up float4 of every slot in flight at once
template <typename E>
__global__ void __launch_bounds__(256) swiglu_vec_kernel(Partials part, E* __restrict__ u, int M, int F) {
  const int64_t idx = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (idx >= (int64_t)M * F) return;
  const int f = (int)(idx % F);
  const int64_t m = idx / F;
  const int64_t col = (int64_t)(2 * (f / 32)) * 32 + f % 32;
  const float* src = part.p + m * 2 * F + col;
  const int n_part = part.count((int)col);
  float4 gt[kMaxSlots], up[kMaxSlots];
#pragma unroll
  for (int p = 0; p < kMaxSlots; ++p)
    if (p < n_part) {
      gt[p] = *reinterpret_cast<const float4*>(src + (int64_t)p * part.stride);
      up[p] = *reinterpret_cast<const float4*>(src + (int64_t)p * part.stride + 32);
    }
  float4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int p = 0; p < kMaxSlots; ++p)
    if (p < n_part) {
      a.x += gt[p].x, a.y += gt[p].y, a.z += gt[p].z, a.w += gt[p].w;
      b.x += up[p].x, b.y += up[p].y, b.z += up[p].z, b.w += up[p].w;
    }
  *reinterpret_cast<uint2*>(u + idx) = pack4<E>(silu_f(a.x) * b.x, silu_f(a.y) * b.y, silu_f(a.z) * b.z, silu_f(a.w) * b.w);
}

int launch_swiglu(int dtype, const Partials& gu, void* u, int M, int F, hipStream_t st) {
  ProfScope prof_(PROF_SWIGLU, st);
  int64_t total = (int64_t)M * F;
  if (total == 0) return MDZ_OK;
  unsigned blocks = (unsigned)((total + 255) / 256);
  // gate and up tiles of a pair lie in the same band (band widths are multiples of 64), so one count serves both
  if (is_16bit(dtype) && F % 32 == 0 && gu.n <= kMaxSlots && gu.stride % 4 == 0 && (gu.split_grid == 0 || gu.band_cols % 64 == 0))
    MDZ_WITH_ELEM16(dtype, (swiglu_vec_kernel<E><<<(unsigned)((total / 4 + 255) / 256), 256, 0, st>>>(gu, (E*)u, M, F)));
  else
    MDZ_WITH_ELEM(dtype, (swiglu_kernel<E><<<blocks, 256, 0, st>>>(gu, (E*)u, M, F)));
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

template <typename T>
__global__ void gather_rows_kernel(const T* __restrict__ hidden, const int32_t* __restrict__ src_row, int Tsrc, int d,
                                   T* __restrict__ h) {
  int b = blockIdx.x;
  int r = src_row ? min(max(src_row[b], 0), Tsrc - 1) : 0;
  const T* src = hidden + ((int64_t)b * Tsrc + r) * d;
  if (d % 4 == 0 && (reinterpret_cast<uintptr_t>(hidden) | reinterpret_cast<uintptr_t>(h)) % 16 == 0) {  // four elements per thread
    for (int i = threadIdx.x * 4; i < d; i += blockDim.x * 4)
      *reinterpret_cast<Quad<T>*>(h + (int64_t)b * d + i) = *reinterpret_cast<const Quad<T>*>(src + i);
    return;
  }
  for (int i = threadIdx.x; i < d; i += blockDim.x) h[(int64_t)b * d + i] = src[i];
}

int launch_gather_rows(int dtype, const void* hidden, const int32_t* src_row, int B, int Tsrc, int d, void* h,
                       hipStream_t st) {
  ProfScope prof_(PROF_MISC, st);
  if (B == 0) return MDZ_OK;
  MDZ_WITH_ELEM(dtype, (gather_rows_kernel<E><<<B, 1024, 0, st>>>((const E*)hidden, src_row, Tsrc, d, (E*)h)));
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

// blockIdx.y = head, its z rows n elements.  part_head_stride >= 0: the heads' first-layer products came from separate
// GEMMs, head k's partial sums [B][d] start k * part_head_stride floats into the region.  part_head_stride < 0: they
// came from ONE GEMM over the heads' stacked matrices: head k's pre-activations are columns k*d .. k*d+d-1 of [B][K*d].
template <typename T>
__global__ void head_residual_kernel(const T* __restrict__ h, Partials part, int64_t part_head_stride, HeadBiases b1s,
                                     T* __restrict__ z, int64_t n, int d) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n) return;
  const int k = blockIdx.y;
  const int j = (int)(idx % d);
  const T* b1 = reinterpret_cast<const T*>(b1s.p[k]);
  const bool stacked = part_head_stride < 0;
  const int col = stacked ? k * d + j : j;
  const float* pp = stacked ? part.p + (idx / d) * part.ld + col : part.p + k * part_head_stride + idx;
  float p = 0.f;
  const int n_part = part.count(col);
  for (int s = 0; s < n_part; ++s) p += pp[(int64_t)s * part.stride];
  p += b1 ? to_float(b1[j]) : 0.f;
  z[k * n + idx] = from_float<T>(to_float(h[idx]) + silu_f(p));
}

int launch_head_residual(int dtype, const void* h, const Partials& pre, int64_t part_head_stride, const HeadBiases& b1s,
                         int n_heads, void* z, int B, int d, hipStream_t st) {
  ProfScope prof_(PROF_MISC, st);
  int64_t n = (int64_t)B * d;
  if (n == 0 || n_heads == 0) return MDZ_OK;
  dim3 blocks((unsigned)((n + 255) / 256), n_heads);
  MDZ_WITH_ELEM(dtype, (head_residual_kernel<E><<<blocks, 256, 0, st>>>((const E*)h, pre, part_head_stride, b1s, (E*)z, n, d)));
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

template <typename T>
__global__ void store_rows_kernel(const float* __restrict__ src, T* __restrict__ dst, int64_t n) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < n) dst[idx] = from_float<T>(src[idx]);
}

int launch_store_rows(int dtype, const float* src, void* dst, int64_t n, hipStream_t st) {
  ProfScope prof_(PROF_MISC, st);
  if (n == 0) return MDZ_OK;
  unsigned blocks = (unsigned)((n + 255) / 256);
  MDZ_WITH_ELEM(dtype, (store_rows_kernel<E><<<blocks, 256, 0, st>>>(src, (E*)dst, n)));
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

}  // namespace mdz
