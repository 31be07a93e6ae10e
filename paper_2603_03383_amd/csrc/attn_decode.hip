// Single-query attention over the tiled 16-bit (bf16 or fp16) KV cache: the degenerate tree of one node, i.e. one ordinary
// autoregressive decode step (Section 4.1: the Time_AR that the paper's Overhead and Speedup are measured
// against).  The node sees the prefix and itself, so the mask is "slot <= S".
//
// One workgroup = 4 waves handles one (sequence, head, key-split); a wave walks 32-key blocks of the tiled cache
// (common.h) with the same contiguous 16-byte-per-lane loads as the tree kernel.  There is one query, so the
// products are plain FMAs: in a K unit lane l holds 8 features of key l % 32, and the two half-waves hold the two
// halves of every 16-feature step, so a score is a 64-term sum per lane plus one exchange with lane ^ 32.  In a V
// unit lane l holds feature 32t + l % 32 for 8 keys; their probabilities come from the lanes that own those keys.
// Waves merge through LDS, key-splits through a second small kernel, both in a fixed order.
// Q8 = true: 8-bit rows (common.h): a block is 4 K units + 4 V units + 2 x 32 scales; a lane's 16 bytes of K unit j are
// its 8 features of k-steps 2j and 2j+1, its 16 bytes of V unit t the 8 keys of s2 = 0 and of s2 = 1; the score of key
// k is multiplied by the key's K scale and its probability by the key's V scale, in fp32.
#include "kernels.h"

namespace mdz {

typedef u32x4_t u32x4;

namespace {
constexpr int kHD = 128;

__device__ inline float fast_exp2_attn(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ inline float half_max(float v) {  // max over the 32 lanes of a half-wave (both halves hold the same set)
#pragma unroll
  for (int o = 16; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ inline float half_sum(float v) {
#pragma unroll
  for (int o = 16; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ inline void unpack8_fp8(u32x4 v, int half, float (&f)[8]) {  // the 8 codes in words 2*half, 2*half+1
  const uint32_t w0 = half ? v.z : v.x, w1 = half ? v.w : v.y;
  const auto a = __builtin_amdgcn_cvt_pk_f32_fp8(w0, false), b = __builtin_amdgcn_cvt_pk_f32_fp8(w0, true);
  const auto c = __builtin_amdgcn_cvt_pk_f32_fp8(w1, false), d = __builtin_amdgcn_cvt_pk_f32_fp8(w1, true);
  f[0] = a[0], f[1] = a[1], f[2] = b[0], f[3] = b[1], f[4] = c[0], f[5] = c[1], f[6] = d[0], f[7] = d[1];
}
template <typename E>
__device__ inline void unpack8(u32x4 v, float (&f)[8]) {
  f[0] = Elem16<E>::lo(v.x), f[1] = Elem16<E>::hi(v.x);
  f[2] = Elem16<E>::lo(v.y), f[3] = Elem16<E>::hi(v.y);
  f[4] = Elem16<E>::lo(v.z), f[5] = Elem16<E>::hi(v.z);
  f[6] = Elem16<E>::lo(v.w), f[7] = Elem16<E>::hi(v.w);
  // Keeps the conversions as instructions of their own.  For fp16 the compiler otherwise folds them into
  // mixed-precision FMAs (v_fma_mix_f32), which made this kernel three times slower than its bf16 twin.
#pragma unroll
  for (int i = 0; i < 8; ++i) asm volatile("" : "+v"(f[i]));
}
}  // namespace

template <typename E, bool Q8>
__global__ void __launch_bounds__(256)
    attn_decode_kernel(const E* __restrict__ q, KvGeom g, const E* __restrict__ kc, const E* __restrict__ vc,
                       int layer, const int32_t* __restrict__ seq_len, int max_prefix, E* __restrict__ att_out,
                       float* __restrict__ part_o, float* __restrict__ part_ml) {
  __shared__ float o_lds[4][kHD];
  __shared__ float ml_lds[4][2];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int key = lane & 31, half = lane >> 5;
  const int split = blockIdx.x, n_splits = gridDim.x, h = blockIdx.y, b = blockIdx.z;
  const int d = q_heads(g) * kHD;
  const int S = min(max(seq_len[b], 0), max_prefix);
  const int n_slots = S + 1;  // the prefix and the node itself
  const int nb = (n_slots + 31) >> 5;
  const int blk_begin = (int)((int64_t)split * nb / n_splits), blk_end = (int)((int64_t)(split + 1) * nb / n_splits);

  // the lane's 64 query features: 16*ks + 8*half + e, pre-scaled by log2(e) / sqrt(head_dim)
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)kHD);
  float qf[8][8];
  const u32x4* qp = reinterpret_cast<const u32x4*>(q + (int64_t)b * d + h * kHD);
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    unpack8<E>(qp[2 * ks + half], qf[ks]);
#pragma unroll
    for (int e = 0; e < 8; ++e) qf[ks][e] *= scale_log2;
  }

  // query head h reads key/value head h / group.  16-bit rows: unit i of block blk at kp[blk*512 + i*64]; 8-bit
  // rows: at kp[blk*264 + i*64], the scale of key `key` at ksc[blk*1056 + key]
  constexpr int kBlkPieces = Q8 ? kKv8BlockBytes / 16 : 512;
  const u32x4* kp;
  const u32x4* vp;
  const float* ksc = nullptr;
  const float* vsc = nullptr;
  if constexpr (Q8) {
    const int64_t hb = kv8_head_base(g, layer, b, h / g.group);
    const uint8_t* k0 = reinterpret_cast<const uint8_t*>(kc) + hb;
    const uint8_t* v0 = reinterpret_cast<const uint8_t*>(vc) + hb;
    kp = reinterpret_cast<const u32x4*>(k0) + lane, vp = reinterpret_cast<const u32x4*>(v0) + lane;
    ksc = reinterpret_cast<const float*>(k0 + 4096) + key, vsc = reinterpret_cast<const float*>(v0 + 4096) + key;
  } else {
    const int64_t head_base = kv_head_base(g, layer, b, h / g.group);
    kp = reinterpret_cast<const u32x4*>(kc + head_base) + lane;
    vp = reinterpret_cast<const u32x4*>(vc + head_base) + lane;
  }

  float m_run = -INFINITY, l_run = 0.f;
  float o[4] = {0.f, 0.f, 0.f, 0.f};  // feature 32t + key, over the keys this half-wave owns
  for (int blk = blk_begin + wave; blk < blk_end; blk += 4) {
    constexpr int kUnits = Q8 ? 4 : 8;
    u32x4 kd[kUnits], vd[kUnits];
#pragma unroll
    for (int i = 0; i < kUnits; ++i) kd[i] = kp[(int64_t)blk * kBlkPieces + i * 64];
#pragma unroll
    for (int i = 0; i < kUnits; ++i) vd[i] = vp[(int64_t)blk * kBlkPieces + i * 64];
    float k_scale = 1.f, v_scale = 1.f;
    if constexpr (Q8) k_scale = ksc[(int64_t)blk * (kKv8BlockBytes / 4)], v_scale = vsc[(int64_t)blk * (kKv8BlockBytes / 4)];
    float s = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      float kf[8];
      if constexpr (Q8)
        unpack8_fp8(kd[ks >> 1], ks & 1, kf);
      else
        unpack8<E>(kd[ks], kf);
#pragma unroll
      for (int e = 0; e < 8; ++e) s += qf[ks][e] * kf[e];
    }
    s += __shfl_xor(s, 32, 64);  // both half-waves now hold the score of key `key`
    s *= k_scale;
    s = (blk * 32 + key < n_slots) ? s : -INFINITY;
    const float m_new = fmaxf(m_run, half_max(s));  // finite: a block in range holds at least one visible slot
    const float p = fast_exp2_attn(s - m_new);
    const float alpha = fast_exp2_attn(m_run - m_new);
    l_run = l_run * alpha + half_sum(p);
    m_run = m_new;
#pragma unroll
    for (int t = 0; t < 4; ++t) o[t] *= alpha;
    // V unit (2t + s2): feature 32t + key, keys 16*s2 + 8*(e/4) + 4*half + e%4; the probability of key k lives in lane k
    const float pv = Q8 ? (blk * 32 + key < n_slots ? p * v_scale : 0.f) : p;  // the key's V scale rides on its probability
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      float pe[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) pe[e] = __shfl(pv, 16 * s2 + 8 * (e >> 2) + 4 * half + (e & 3), 64);
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        float vf[8];
        if constexpr (Q8)
          unpack8_fp8(vd[t], s2, vf);
        else
          unpack8<E>(vd[2 * t + s2], vf);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[t] += pe[e] * vf[e];
      }
    }
  }
#pragma unroll
  for (int t = 0; t < 4; ++t) o[t] += __shfl_xor(o[t], 32, 64);  // the two half-waves own disjoint keys

  // ---- merge the four waves (fixed order), then store or hand the partial result to the combine kernel
  if (half == 0) {
#pragma unroll
    for (int t = 0; t < 4; ++t) o_lds[wave][32 * t + key] = o[t];
    if (key == 0) ml_lds[wave][0] = m_run, ml_lds[wave][1] = l_run;
  }
  __syncthreads();
  if (threadIdx.x < kHD) {
    const int f = threadIdx.x;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, ml_lds[w][0]);
    const float M_safe = M == -INFINITY ? 0.f : M;
    float L = 0.f, acc = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float wt = fast_exp2_attn(ml_lds[w][0] - M_safe);
      L += wt * ml_lds[w][1];
      acc += wt * o_lds[w][f];
    }
    if (n_splits == 1) {
      att_out[(int64_t)b * d + h * kHD + f] = from_float<E>(acc / L);
    } else {
      const int64_t pidx = (int64_t)(b * q_heads(g) + h) * n_splits + split;
      part_o[pidx * kHD + f] = acc;
      if (f == 0) part_ml[pidx * 2] = M, part_ml[pidx * 2 + 1] = L;
    }
  }
}

template <typename E>
__global__ void __launch_bounds__(128)
    attn_decode_combine_kernel(int n_heads, int n_splits, const float* __restrict__ part_o, const float* __restrict__ part_ml,
                               E* __restrict__ att_out) {
  const int h = blockIdx.x, b = blockIdx.y, f = threadIdx.x;
  const int64_t p0 = (int64_t)(b * n_heads + h) * n_splits;
  float M = -INFINITY;
  for (int s = 0; s < n_splits; ++s) M = fmaxf(M, part_ml[(p0 + s) * 2]);
  float L = 0.f, acc = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const float w = fast_exp2_attn(part_ml[(p0 + s) * 2] - M);
    L += w * part_ml[(p0 + s) * 2 + 1];
    acc += w * part_o[(p0 + s) * kHD + f];
  }
  att_out[((int64_t)b * n_heads + h) * kHD + f] = from_float<E>(acc / L);
}

bool attn_decode_supported(int dtype, int tree, const KvGeom& g) {
  return is_16bit(dtype) && g.tiled && g.head_dim == kHD && host_tree(tree)->T == 1;
}

static int decode_splits(int B, int n_heads, int max_prefix) {
  const int nb = (max_prefix + 1 + 31) / 32;
  int by_len = nb / 4;                                     // >= one block per wave
  int by_fill = (512 + B * n_heads - 1) / (B * n_heads);   // aim at ~512 workgroups
  int s = by_len < by_fill ? by_len : by_fill;
  return s > 32 ? 32 : s < 1 ? 1 : s;
}

int64_t attn_decode_scratch_bytes(int B, int n_heads, int max_prefix) {
  const int s = decode_splits(B, n_heads, max_prefix);
  return s == 1 ? 0 : (int64_t)B * n_heads * s * (kHD + 2) * 4;
}

template <typename E, bool Q8>
static int launch_attention_decode_t(const void* q, const KvGeom& g, const void* kc, const void* vc, int layer,
                                     const int32_t* seq_len, int B, int max_prefix, void* att_out, void* scratch,
                                     int64_t scratch_bytes, hipStream_t st) {
  ProfScope prof_(PROF_ATTN, st);
  if (B == 0) return MDZ_OK;
  const int nq = q_heads(g);
  const int splits = decode_splits(B, nq, max_prefix);
  MDZ_REQUIRE(scratch_bytes >= attn_decode_scratch_bytes(B, nq, max_prefix), MDZ_EWORKSPACE,
              "decode attention: scratch too small");
  float* part_o = (float*)scratch;
  float* part_ml = part_o + (int64_t)B * nq * splits * kHD;
  attn_decode_kernel<E, Q8><<<dim3(splits, nq, B), 256, 0, st>>>((const E*)q, g, (const E*)kc, (const E*)vc, layer, seq_len,
                                                             max_prefix, (E*)att_out, part_o, part_ml);
  MDZ_LAUNCH_CHECK();
  if (splits > 1) {
    attn_decode_combine_kernel<E><<<dim3(nq, B), 128, 0, st>>>(nq, splits, part_o, part_ml, (E*)att_out);
    MDZ_LAUNCH_CHECK();
  }
  return MDZ_OK;
}

int launch_attention_decode(int dtype, const void* q, const KvGeom& g, const void* kc, const void* vc, int layer,
                            const int32_t* seq_len, int B, int max_prefix, void* att_out, void* scratch,
                            int64_t scratch_bytes, hipStream_t st) {
  if (g.quant)
    MDZ_WITH_ELEM16(dtype, return (launch_attention_decode_t<E, true>(q, g, kc, vc, layer, seq_len, B, max_prefix, att_out,
                                                                      scratch, scratch_bytes, st)));
  MDZ_WITH_ELEM16(dtype, return (launch_attention_decode_t<E, false>(q, g, kc, vc, layer, seq_len, B, max_prefix, att_out,
                                                                     scratch, scratch_bytes, st)));
}

}  // namespace mdz
