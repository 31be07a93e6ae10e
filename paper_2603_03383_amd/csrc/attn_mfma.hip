// Tree-masked attention for 16-bit storage (bf16 or fp16, element type E), 64-node tree, head_dim 128, on gfx950 MFMA
// (Section 3.2: all T candidates attend in one pass; node i sees the whole prefix plus the tree slots
// its row of the static visibility matrix allows).
//
// One workgroup = 4 waves handles one (sequence, head, key-split).  All 64 queries ride along every
// key, so K and V are read from HBM exactly once per head.  A wave walks 32-key blocks of the tiled
// cache (common.h): each 1 KiB unit is loaded with one contiguous 16-byte-per-lane load and used
// directly as an MFMA A operand.  Scores are computed transposed (keys x queries), which leaves every
// lane with 16 keys of ONE query: the running max / sum need a single exchange with lane+32, and the
// probabilities are packed to the storage type in place as the B operand of the second MFMA (out^T = V^T P^T).
// The tree mask is one 64-bit word per query (a compile-time table) tested only in blocks that reach
// past the prefix.  Waves merge through LDS, key-splits through a small second kernel, both in a fixed
// order, so results are deterministic.
// Q8 = true: the cache holds 8-bit rows (E4M3 codes + one fp32 scale per row, common.h).  A block is then 4 K units,
// 4 V units and 2 x 32 scales; codes convert exactly to the 16-bit element type in registers (two k-steps per 16-byte
// load), the K scales multiply the scores and the V scales the probabilities, both in fp32, so the MFMAs are the same.
// Key-splits: when the kernel starts from the QKV partial sums, the last split owns every block that holds a
// tree slot (it is the one that has to produce those K / V rows first) and the other splits share the blocks
// that hold prefix keys only, which need nothing but Q: the long dependent chain (reduce K and V, write them,
// read them back) then covers three blocks at most instead of an even share of the prefix.
#include "kernels.h"

namespace mdz {

typedef f32x16_t f32x16;
typedef u32x4_t u32x4;

constexpr int kHD = 128;         // head_dim
constexpr int kTQ = 64;          // queries (tree nodes)
constexpr int kQRow = kHD * 2 + 16;  // bytes per staged Q row
constexpr float kLazyLog2 = 8.f;  // see the key loop: how far a block's maximum may exceed the running reference

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// 8 E4M3 codes (words 2*half, 2*half+1 of v) -> 8 elements
template <typename E>
__device__ inline u32x4 fp8x8_to_elem(u32x4 v, int half) {
  const uint32_t w0 = half ? v.z : v.x, w1 = half ? v.w : v.y;
  return u32x4{Elem16<E>::from_fp8x2(w0, false), Elem16<E>::from_fp8x2(w0, true), Elem16<E>::from_fp8x2(w1, false),
               Elem16<E>::from_fp8x2(w1, true)};
}

template <typename E>
__device__ inline u32x4 pack8(const float* v) {
  return u32x4{Elem16<E>::pack2(v[0], v[1]), Elem16<E>::pack2(v[2], v[3]), Elem16<E>::pack2(v[4], v[5]),
               Elem16<E>::pack2(v[6], v[7])};
}

// NM head-matrices (q, or q k v, of head h) of the QKV GEMM output for the prologue below: thread (row = t/4,
// seg = t%4) sums the partial-sum slots (in order) of features [16*seg, 16*seg+16) and their rotary partners
// [64 + 16*seg, ...) of each matrix: lo[m][16], hi[m][16].  The loads of one slot of all NM matrices are issued
// together (8 float4 per matrix in flight per thread); matrix m starts at column cols[m].
template <int NM>
__device__ inline void qkv_gather(const Partials& part, int64_t row, const int (&cols)[NM], int seg, float (&lo)[NM][16],
                                  float (&hi)[NM][16]) {
  int n_part[NM], n_max = 0;
#pragma unroll
  for (int m = 0; m < NM; ++m) {
    n_part[m] = part.count(cols[m]);
    n_max = n_part[m] > n_max ? n_part[m] : n_max;
#pragma unroll
    for (int i = 0; i < 16; ++i) lo[m][i] = hi[m][i] = 0.f;
  }
  const float* src = part.p + row * part.ld + 16 * seg;
  for (int p = 0; p < n_max; ++p) {
    float4 a[NM][4], b[NM][4];
    const float* sp = src + (int64_t)p * part.stride;
#pragma unroll
    for (int m = 0; m < NM; ++m)
      if (p < n_part[m]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          a[m][i] = *reinterpret_cast<const float4*>(sp + cols[m] + 4 * i);
          b[m][i] = *reinterpret_cast<const float4*>(sp + cols[m] + 64 + 4 * i);
        }
      }
#pragma unroll
    for (int m = 0; m < NM; ++m)
      if (p < n_part[m]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          lo[m][4 * i] += a[m][i].x, lo[m][4 * i + 1] += a[m][i].y, lo[m][4 * i + 2] += a[m][i].z, lo[m][4 * i + 3] += a[m][i].w;
          hi[m][4 * i] += b[m][i].x, hi[m][4 * i + 1] += b[m][i].y, hi[m][4 * i + 2] += b[m][i].z, hi[m][4 * i + 3] += b[m][i].w;
        }
      }
  }
}

__device__ inline void rope16(const float* cs_row, int seg, float (&lo)[16], float (&hi)[16]) {
  const float* c = cs_row + 32 * seg;  // [i][cos, sin] for i = 16*seg ..
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    float cv = c[2 * i], sv = c[2 * i + 1];
    float a = lo[i], b = hi[i];
    lo[i] = a * cv - b * sv;
    hi[i] = b * cv + a * sv;
  }
}

// qkv.p == NULL: q holds the rotated queries and the cache already holds the tree rows (separate RoPE kernel).
// qkv.p != NULL: the kernel starts from the QKV GEMM's partial sums: it reduces them, rotates q and k (RoPE,
// cos/sin table cs [row][64][2]), keeps q in LDS, and — if its key range reaches the tree slots — writes the 64
// tree rows of K and V of its head into the cache before reading them back like any other key.  Workgroups of
// the same head that both reach the tree slots write identical values.
// NU = 2: a workgroup carries all 64 queries (two groups of 32).  NU = 1: it carries 32 of them, the two halves of a
// (sequence, head, split) being two workgroups (blockIdx.z = 2 * sequence + half): half the accumulators, so two
// workgroups share a CU and twice as many loads are in flight per CU, at the price of K and V passing through the
// CU twice (the second time from L2: the halves are a multiple of 8 workgroups apart, i.e. on one XCD).
template <typename E, bool Q8, int NU>
__global__ void __launch_bounds__(256, NU == 1 ? 2 : 1)
    attn_tree_mfma_kernel(int tree, const E* __restrict__ q, const Partials qkv, const float* __restrict__ cs,
                          KvGeom g, E* __restrict__ kc, E* __restrict__ vc, int layer,
                          const int32_t* __restrict__ seq_len, int max_prefix, E* __restrict__ att_out,
                          float* __restrict__ part_o, float* __restrict__ part_ml) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  MDZ_STAMP(0);
  const TreeTables& t = c_trees[tree];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int qi = lane & 31, gh = lane >> 5;
  constexpr int kQW = 32 * NU;          // queries of this workgroup
  constexpr int kOPadN = kQW + 2;       // LDS row stride of the merge buffer (floats): conflict-free writes and reads
  const int split = blockIdx.x, n_splits = gridDim.x, h = blockIdx.y;
  const int b = NU == 2 ? blockIdx.z : blockIdx.z >> 1;
  const int q0 = NU == 2 ? 0 : (blockIdx.z & 1) * 32;  // first query of this workgroup
  const int hk = h / g.group;  // the key/value head that query head h reads (grouped-query attention)
  const int d = q_heads(g) * kHD, dkv = g.n_heads * kHD;
  const int S = min(max(seq_len[b], 0), max_prefix);
  const int n_slots = S + kTQ;
  const int nb = (n_slots + 31) >> 5;
  int blk_begin, blk_end;
  if (qkv.p != nullptr && n_splits > 1) {  // last split: every block with a tree slot; the others: prefix-only blocks
    const int pb = S >> 5, ps = n_splits - 1;
    blk_begin = split == ps ? pb : (int)((int64_t)split * pb / ps);
    blk_end = split == ps ? nb : (int)((int64_t)(split + 1) * pb / ps);
  } else {
    blk_begin = (int)((int64_t)split * nb / n_splits);
    blk_end = (int)((int64_t)(split + 1) * nb / n_splits);
  }

  // 16-bit rows: block blk, unit i at kp[blk*512 + i*64].  8-bit rows: a block is 264 16-byte pieces: unit i at
  // kp[blk*264 + i*64], the four scales of keys 8j + 4gh .. +3 at ks_p[blk*264 + 2j]
  constexpr int kBlkPieces = Q8 ? kKv8BlockBytes / 16 : 512;
  const u32x4* kp;
  const u32x4* vp;
  const u32x4* ks_p = nullptr;
  const u32x4* vs_p = nullptr;
  if constexpr (Q8) {
    const int64_t hb = kv8_head_base(g, layer, b, hk);
    const u32x4* k0 = reinterpret_cast<const u32x4*>(reinterpret_cast<const uint8_t*>(kc) + hb);
    const u32x4* v0 = reinterpret_cast<const u32x4*>(reinterpret_cast<const uint8_t*>(vc) + hb);
    kp = k0 + lane, vp = v0 + lane;
    ks_p = k0 + 256 + gh, vs_p = v0 + 256 + gh;
  } else {
    const int64_t head_base = kv_head_base(g, layer, b, hk);
    kp = reinterpret_cast<const u32x4*>(kc + head_base) + lane;
    vp = reinterpret_cast<const u32x4*>(vc + head_base) + lane;
  }

  // K and V are both double buffered one block ahead of the block being multiplied, and every load is
  // unconditional (past the wave's last block it repeats that block and the result is not used): the wait counters
  // are in-order, so a wave then keeps a whole block (16 KiB of 16-bit rows) in flight while it works on the
  // previous one, which is what the HBM latency asks for at one wave per SIMD.
  u32x4 kb[2][8], vb[2][8];
  auto load_kv = [&](int blk, u32x4 (&kd)[8], u32x4 (&vd)[8]) {  // 8-bit rows: [0..3] codes, [4..7] the lane's 16 scales
#pragma unroll
    for (int i = 0; i < 8; ++i)
      kd[i] = (Q8 && i >= 4) ? ks_p[(int64_t)blk * kBlkPieces + 2 * (i - 4)] : kp[(int64_t)blk * kBlkPieces + i * 64];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      vd[i] = (Q8 && i >= 4) ? vs_p[(int64_t)blk * kBlkPieces + 2 * (i - 4)] : vp[(int64_t)blk * kBlkPieces + i * 64];
  };
  // this wave's blocks: blk_begin + wave, + 4, ... ; two per trip so that the buffers alternate statically
  const int n_mine = blk_begin + wave < blk_end ? (blk_end - blk_begin - wave + 3) >> 2 : 0;
  const int first = blk_begin + wave, last = first + 4 * (n_mine - 1);
  // A first block that lies wholly in the prefix depends on nothing this kernel computes: it is requested before the
  // prologue below, whose own loads then wait no longer than this one takes.  (A block with tree slots is written
  // by the prologue first.)
  // (not for 8-bit rows with 64 queries: that variant has no registers to hold the block through the prologue)
  const bool preloaded = !(Q8 && NU == 2) && n_mine > 0 && (first + 1) * 32 <= S;
  if (preloaded) load_kv(first, kb[0], vb[0]);

  // Q tile of this head -> LDS (rows padded by 16 B: the 16 B-per-lane operand reads below are bank-conflict
  // free).  The region is reused by the wave merge after the key loop.
  uint8_t* q_lds = reinterpret_cast<uint8_t*>(lds);
  if (qkv.p == nullptr) {
#pragma unroll
    for (int i = 0; i < 2 * NU; ++i) {
      int idx = threadIdx.x + i * 256;
      int row = idx >> 4, col = idx & 15;
      *reinterpret_cast<u32x4*>(q_lds + row * kQRow + col * 16) =
          *reinterpret_cast<const u32x4*>(q + (int64_t)(b * kTQ + q0 + row) * d + h * kHD + col * 8);
    }
  } else {
    // thread (row = t/4, seg = t%4): features [16 seg, +16) and their rotary partners of one row.  K / V rows: tree
    // node `row` (all 64, by all threads); Q rows: query q0 + row (the first 32 NU rows of threads).
    const int row = threadIdx.x >> 2, seg = threadIdx.x & 3;
    const int64_t grow_kv = (int64_t)b * kTQ + row, grow_q = (int64_t)b * kTQ + q0 + row;
    const float* cs_kv = cs + grow_kv * kHD;  // 64 pairs x 2
    auto stage_q = [&](float (&lo)[16], float (&hi)[16]) {
      uint8_t* qrow = q_lds + row * kQRow;
      rope16(cs + grow_q * kHD, seg, lo, hi);
      *reinterpret_cast<u32x4*>(qrow + 32 * seg) = pack8<E>(lo);
      *reinterpret_cast<u32x4*>(qrow + 32 * seg + 16) = pack8<E>(lo + 8);
      *reinterpret_cast<u32x4*>(qrow + 128 + 32 * seg) = pack8<E>(hi);
      *reinterpret_cast<u32x4*>(qrow + 128 + 32 * seg + 16) = pack8<E>(hi + 8);
    };
    // rotates the key row and writes the node's K and V rows into the cache
    auto write_kv = [&](float (&klo)[16], float (&khi)[16], float (&vlo)[16], float (&vhi)[16]) {
      const int slot = S + row;
      rope16(cs_kv, seg, klo, khi);
      if constexpr (Q8) {
        // row scales: the largest magnitude over the 4 threads (seg) of the row, then codes of this thread's 2 x 16 features
        float am[2] = {0.f, 0.f};
#pragma unroll
        for (int m = 0; m < 2; ++m) {
#pragma unroll
          for (int i = 0; i < 16; ++i) am[m] = fmaxf(am[m], fmaxf(fabsf((m == 0 ? klo : vlo)[i]), fabsf((m == 0 ? khi : vhi)[i])));
          am[m] = fmaxf(am[m], __shfl_xor(am[m], 1, 64));
          am[m] = fmaxf(am[m], __shfl_xor(am[m], 2, 64));
        }
        const float ks = kv8_scale_of(am[0]), vs = kv8_scale_of(am[1]);
        uint8_t* k8 = reinterpret_cast<uint8_t*>(kc) + kv8_head_base(g, layer, b, hk);
        uint8_t* v8 = reinterpret_cast<uint8_t*>(vc) + kv8_head_base(g, layer, b, hk);
        // 8 consecutive features of one key are 8 contiguous bytes of the 8-bit K layout
#pragma unroll
        for (int gh2 = 0; gh2 < 2; ++gh2) {
          const float* a = klo + 8 * gh2;
          const float* c = khi + 8 * gh2;
          *reinterpret_cast<uint2*>(k8 + kv8_k_code(slot, 16 * seg + 8 * gh2)) =
              uint2{kv8_pack4(a[0], a[1], a[2], a[3], ks), kv8_pack4(a[4], a[5], a[6], a[7], ks)};
          *reinterpret_cast<uint2*>(k8 + kv8_k_code(slot, 64 + 16 * seg + 8 * gh2)) =
              uint2{kv8_pack4(c[0], c[1], c[2], c[3], ks), kv8_pack4(c[4], c[5], c[6], c[7], ks)};
        }
#pragma unroll
        for (int i = 0; i < 16; i += 4) {
          const uint32_t wl = kv8_pack4(vlo[i], vlo[i + 1], vlo[i + 2], vlo[i + 3], vs);
          const uint32_t wh = kv8_pack4(vhi[i], vhi[i + 1], vhi[i + 2], vhi[i + 3], vs);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v8[kv8_v_code(slot, 16 * seg + i + e)] = (uint8_t)(wl >> (8 * e));
            v8[kv8_v_code(slot, 64 + 16 * seg + i + e)] = (uint8_t)(wh >> (8 * e));
          }
        }
        if (seg == 0) {
          *reinterpret_cast<float*>(k8 + kv8_scale(slot)) = ks;
          *reinterpret_cast<float*>(v8 + kv8_scale(slot)) = vs;
        }
      } else {
        // 8 consecutive features of one key are 16 contiguous bytes of the tiled K layout
        *reinterpret_cast<u32x4*>(kc + k_index(g, layer, b, hk, slot, 16 * seg)) = pack8<E>(klo);
        *reinterpret_cast<u32x4*>(kc + k_index(g, layer, b, hk, slot, 16 * seg + 8)) = pack8<E>(klo + 8);
        *reinterpret_cast<u32x4*>(kc + k_index(g, layer, b, hk, slot, 64 + 16 * seg)) = pack8<E>(khi);
        *reinterpret_cast<u32x4*>(kc + k_index(g, layer, b, hk, slot, 64 + 16 * seg + 8)) = pack8<E>(khi + 8);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          vc[v_index(g, layer, b, hk, slot, 16 * seg + i)] = from_float<E>(vlo[i]);
          vc[v_index(g, layer, b, hk, slot, 64 + 16 * seg + i)] = from_float<E>(vhi[i]);
        }
      }
    };
    if (blk_end * 32 > S && blk_begin < blk_end) {  // this range reaches the tree slots: produce their K / V rows
      // (workgroups of one key/value head that reach the tree slots all write them: identical values, no ordering needed)
      if constexpr (NU == 2) {
        float lo[3][16], hi[3][16];
        const int cols[3] = {h * kHD, d + hk * kHD, d + dkv + hk * kHD};  // columns of q, k, v in the QKV output
        qkv_gather<3>(qkv, grow_kv, cols, seg, lo, hi);
        stage_q(lo[0], hi[0]);
        write_kv(lo[1], hi[1], lo[2], hi[2]);
      } else {
        float lo[2][16], hi[2][16];
        const int cols[2] = {d + hk * kHD, d + dkv + hk * kHD};
        qkv_gather<2>(qkv, grow_kv, cols, seg, lo, hi);
        write_kv(lo[0], hi[0], lo[1], hi[1]);
        if (row < kQW) {
          float ql[1][16], qh[1][16];
          const int qcols[1] = {h * kHD};
          qkv_gather<1>(qkv, grow_q, qcols, seg, ql, qh);
          stage_q(ql[0], qh[0]);
        }
      }
    } else if (row < kQW) {
      float lo[1][16], hi[1][16];
      const int cols[1] = {h * kHD};
      qkv_gather<1>(qkv, grow_q, cols, seg, lo, hi);
      stage_q(lo[0], hi[0]);
    }
  }
  MDZ_STAMP(1);
  __syncthreads();  // Q tile complete; the tree rows written above are complete (stores drain before a barrier)
  MDZ_STAMP(2);
  // B operand of scores^T: lane holds query 32u + qi, features 16ks + 8gh .. +7
  const uint8_t* qfrag = q_lds + qi * kQRow + gh * 16;
  uint64_t mq[NU];
#pragma unroll
  for (int u = 0; u < NU; ++u) mq[u] = t.anc_mask[q0 + 32 * u + qi];
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)kHD);

  float m_run[NU], l_run[NU];
#pragma unroll
  for (int u = 0; u < NU; ++u) m_run[u] = -INFINITY, l_run[u] = 0.f;
  f32x16 o[4][NU];
#pragma unroll
  for (int tt = 0; tt < 4; ++tt)
#pragma unroll
    for (int u = 0; u < NU; ++u)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[tt][u][r] = 0.f;

  auto process = [&](int blk, const u32x4 (&kd)[8], const u32x4 (&vd)[8]) {
    // Compiler barrier: keeps the (loop-invariant) Q operand reads inside the loop, i.e. in LDS rather
    // than in 64 registers per lane that this kernel does not have to spare.
    asm volatile("" ::: "memory");
    f32x16 sc[NU];
#pragma unroll
    for (int u = 0; u < NU; ++u)
#pragma unroll
      for (int r = 0; r < 16; ++r) sc[u][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const u32x4 ka = Q8 ? fp8x8_to_elem<E>(kd[ks >> 1], ks & 1) : kd[ks];
#pragma unroll
      for (int u = 0; u < NU; ++u) {
        const u32x4 qv = *reinterpret_cast<const u32x4*>(qfrag + u * 32 * kQRow + ks * 32);
        sc[u] = Elem16<E>::mfma(ka, qv, sc[u]);
      }
    }
    // Visibility of this block's 32 keys for the lane's query, as one 32-bit word: prefix keys are
    // visible, a tree key S+j is visible iff bit j of the query's ancestor mask is set, keys beyond the
    // tree are not.  rel0 (wave-uniform) = offset of the block's first key from the tree's first slot.
    const int rel0 = blk * 32 - S;
    const bool need_mask = rel0 + 32 > 0;  // wave-uniform: the block reaches past the prefix
    float alpha[NU];
    u32x4 pf[NU][2];
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      float bmax = -INFINITY;
      // register r is key 8*(r/4) + 4*gh + r%4 of the block; its scale is component r%4 of scale piece r/4
      if (need_mask) {  // wave-uniform branch: only the (at most three) blocks that hold tree slots pay for the mask
        const uint32_t pre = rel0 >= 0 ? 0u : (0xFFFFFFFFu >> (32 + rel0));          // keys below S (rel0 in [-31,-1])
        const uint64_t tr = rel0 >= 0 ? (mq[u] >> rel0) : (mq[u] << (-rel0));        // rel0 in [-31, 63]
        const uint32_t vis = (pre | (uint32_t)tr) >> (4 * gh);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float s = sc[u][r] * (Q8 ? __uint_as_float(kd[4 + (r >> 2)][r & 3]) * scale_log2 : scale_log2);
          s = ((vis >> (8 * (r >> 2) + (r & 3))) & 1u) ? s : -INFINITY;
          sc[u][r] = s;
          bmax = fmaxf(bmax, s);
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float s = sc[u][r] * (Q8 ? __uint_as_float(kd[4 + (r >> 2)][r & 3]) * scale_log2 : scale_log2);
          sc[u][r] = s;
          bmax = fmaxf(bmax, s);
        }
      }
      bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
      // The running reference m_run only has to keep exp2(s - m_run) in range, it need not be the maximum: it is
      // moved (and the accumulators rescaled: 128 registers through the vector ALU) only when a block's maximum
      // exceeds it by more than 2^kLazyLog2, so probabilities stay below 2^kLazyLog2 and, in a long prefix, almost
      // no block rescales.  o, l and m stay consistent, so the merges below need no change.
      const float m_new = bmax > m_run[u] + kLazyLog2 ? bmax : m_run[u];
      const float m_safe = m_new == -INFINITY ? 0.f : m_new;
      alpha[u] = m_new == m_run[u] ? 1.f : fast_exp2(m_run[u] - m_safe);
      float sum = 0.f;
      uint32_t pk[8];
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        float p0 = fast_exp2(sc[u][r] - m_safe), p1 = fast_exp2(sc[u][r + 1] - m_safe);
        sum += p0 + p1;
        if constexpr (Q8) p0 *= __uint_as_float(vd[4 + (r >> 2)][r & 3]), p1 *= __uint_as_float(vd[4 + (r >> 2)][(r & 3) + 1]);
        pk[r >> 1] = Elem16<E>::pack2(p0, p1);
      }
      l_run[u] = l_run[u] * alpha[u] + sum;
      m_run[u] = m_new;
      pf[u][0] = u32x4{pk[0], pk[1], pk[2], pk[3]};
      pf[u][1] = u32x4{pk[4], pk[5], pk[6], pk[7]};
    }
    if (__any(alpha[0] != 1.f || alpha[NU - 1] != 1.f)) {
#pragma unroll
      for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int u = 0; u < NU; ++u)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[tt][u][r] *= alpha[u];
    }
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const u32x4 va = Q8 ? fp8x8_to_elem<E>(vd[tt], s2) : vd[tt * 2 + s2];
#pragma unroll
        for (int u = 0; u < NU; ++u) o[tt][u] = Elem16<E>::mfma(va, pf[u][s2], o[tt][u]);
      }
  };

  if (n_mine > 0) {
    if (!preloaded) load_kv(first, kb[0], vb[0]);
    for (int it = 0; it < n_mine; it += 2) {
      const int blk = first + 4 * it;
      load_kv(min(blk + 4, last), kb[1], vb[1]);
      __builtin_amdgcn_sched_barrier(0);
      process(blk, kb[0], vb[0]);
      __builtin_amdgcn_sched_barrier(0);
      load_kv(min(blk + 8, last), kb[0], vb[0]);
      __builtin_amdgcn_sched_barrier(0);
      if (it + 1 < n_mine) process(blk + 4, kb[1], vb[1]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  MDZ_STAMP(3);
  // ---- merge the four waves through LDS (fixed order) ------------------------------------------
  __syncthreads();  // every wave is done reading the Q tile that the merge buffer overlays
  float* o_lds = lds;                             // [4][kHD][kOPadN]
  float* m_lds = lds + 4 * kHD * kOPadN;          // [4][kQW]
  float* l_lds = m_lds + 4 * kQW;                 // [4][kQW]
#pragma unroll
  for (int u = 0; u < NU; ++u) {
    float l_tot = l_run[u] + __shfl_xor(l_run[u], 32, 64);
    if (gh == 0) {
      m_lds[wave * kQW + 32 * u + qi] = m_run[u];
      l_lds[wave * kQW + 32 * u + qi] = l_tot;
    }
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int hd = 32 * tt + 8 * (r >> 2) + 4 * gh + (r & 3);
        o_lds[(wave * kHD + hd) * kOPadN + 32 * u + qi] = o[tt][u][r];
      }
  }
  __syncthreads();
  // kTPQ threads per query; thread (qq = t / kTPQ, s = t % kTPQ) merges features 16*jj + kEW*s + e (jj < 8, e < kEW)
  constexpr int kTPQ = 256 / kQW, kEW = 16 / kTPQ;
  const int qq = threadIdx.x / kTPQ, s4 = (threadIdx.x % kTPQ) * kEW;
  float mw[4], M = -INFINITY;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    mw[w] = m_lds[w * kQW + qq];
    M = fmaxf(M, mw[w]);
  }
  const float M_safe = M == -INFINITY ? 0.f : M;
  float L = 0.f, wt[4];
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    wt[w] = fast_exp2(mw[w] - M_safe);
    L += wt[w] * l_lds[w * kQW + qq];
  }
  float acc[8 * kEW];
#pragma unroll
  for (int j = 0; j < 8 * kEW; ++j) {
    const int f = 16 * (j / kEW) + s4 + (j % kEW);
    float a = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) a += wt[w] * o_lds[(w * kHD + f) * kOPadN + qq];
    acc[j] = a;
  }
  const int q_out = q0 + qq;  // the query's row among the 64 of its sequence
  if (n_splits == 1) {
    const float inv = 1.0f / L;
    E* dst = att_out + (int64_t)(b * kTQ + q_out) * d + h * kHD + s4;
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
      if constexpr (kEW == 4)
        *reinterpret_cast<uint2*>(dst + 16 * jj) = uint2{Elem16<E>::pack2(acc[4 * jj] * inv, acc[4 * jj + 1] * inv),
                                                         Elem16<E>::pack2(acc[4 * jj + 2] * inv, acc[4 * jj + 3] * inv)};
      else
        *reinterpret_cast<uint32_t*>(dst + 16 * jj) = Elem16<E>::pack2(acc[2 * jj] * inv, acc[2 * jj + 1] * inv);
    }
  } else {
    const int64_t pidx = ((int64_t)(b * q_heads(g) + h) * n_splits + split);
    float* po = part_o + (pidx * kTQ + q_out) * kHD + s4;
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
      if constexpr (kEW == 4)
        *reinterpret_cast<float4*>(po + 16 * jj) = float4{acc[4 * jj], acc[4 * jj + 1], acc[4 * jj + 2], acc[4 * jj + 3]};
      else
        *reinterpret_cast<float2*>(po + 16 * jj) = float2{acc[2 * jj], acc[2 * jj + 1]};
    }
    if (threadIdx.x % kTPQ == 0) {
      part_ml[(pidx * 2 + 0) * kTQ + q_out] = M;
      part_ml[(pidx * 2 + 1) * kTQ + q_out] = L;
    }
  }
  MDZ_STAMP(4);
}

// Merges the key-splits of 16 queries of one (sequence, head): fixed order, exact same weighting rule as above.
// Thread (q = t/16, c = t%16) owns features 8c .. 8c+7 of query 16*blockIdx.z + q.
template <typename E>
__global__ void __launch_bounds__(256)
    attn_combine_kernel(int n_heads, int n_splits, const float* __restrict__ part_o, const float* __restrict__ part_ml,
                        E* __restrict__ att_out) {
  const int h = blockIdx.x, b = blockIdx.y;
  const int d = n_heads * kHD;
  const int qq = blockIdx.z * 16 + (threadIdx.x >> 4), f0 = (threadIdx.x & 15) * 8;
  const int64_t p0 = (int64_t)(b * n_heads + h) * n_splits;
  float M = -INFINITY;
  float L = 0.f;
  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;
  // Splits are taken eight at a time: the loads of a group are all requested before the first is used, so a merge of
  // many splits costs one memory round trip per eight, not one per split.  The weights refer to the running maximum
  // of the groups seen so far (the sums are rescaled when a later group raises it), in a fixed order.
  constexpr int kTogether = 8;
  for (int s0 = 0; s0 < n_splits; s0 += kTogether) {
    float ms[kTogether], ls[kTogether];
    float4 v0[kTogether], v1[kTogether];
#pragma unroll
    for (int s = 0; s < kTogether; ++s)
      if (s0 + s < n_splits) {
        ms[s] = part_ml[((p0 + s0 + s) * 2 + 0) * kTQ + qq];
        ls[s] = part_ml[((p0 + s0 + s) * 2 + 1) * kTQ + qq];
        const float4* po = reinterpret_cast<const float4*>(part_o + ((p0 + s0 + s) * kTQ + qq) * kHD + f0);
        v0[s] = po[0], v1[s] = po[1];
      }
    float Mg = M;
#pragma unroll
    for (int s = 0; s < kTogether; ++s)
      if (s0 + s < n_splits) Mg = fmaxf(Mg, ms[s]);
    if (Mg != M) {  // (first group: M = -inf and the sums are zero)
      const float r = M == -INFINITY ? 0.f : fast_exp2(M - Mg);
      L *= r;
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] *= r;
      M = Mg;
    }
#pragma unroll
    for (int s = 0; s < kTogether; ++s)
      if (s0 + s < n_splits) {
        const float w = fast_exp2(ms[s] - M);
        L += w * ls[s];
        acc[0] += w * v0[s].x, acc[1] += w * v0[s].y, acc[2] += w * v0[s].z, acc[3] += w * v0[s].w;
        acc[4] += w * v1[s].x, acc[5] += w * v1[s].y, acc[6] += w * v1[s].z, acc[7] += w * v1[s].w;
      }
  }
  const float inv = 1.0f / L;
  uint32_t pk[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) pk[j] = Elem16<E>::pack2(acc[2 * j] * inv, acc[2 * j + 1] * inv);
  *reinterpret_cast<u32x4*>(att_out + (int64_t)(b * kTQ + qq) * d + h * kHD + f0) = u32x4{pk[0], pk[1], pk[2], pk[3]};
}

bool attn_mfma_supported(int dtype, int tree, const KvGeom& g) {
  return is_16bit(dtype) && g.tiled && g.head_dim == kHD && host_tree(tree)->T == kTQ;
}

// Key-splits per (sequence, head).  fused: the kernel starts from the QKV partial sums, so one split is the tree
// split and the rest share the prefix: at most as many as keep every workgroup resident at once (one per CU: the
// merge buffer takes most of a CU's LDS).  Every further split costs about a microsecond per layer (its reduce of
// the Q partial sums, its share of the merge) and saves the blocks it takes off the others, so the best count grows
// with the square root of the prefix: measured best 1 / 3 / 5 / 8 splits at prefixes 128 / 1K / 4K / 16K.
static int attn_splits(int B, int n_heads, int max_prefix, bool fused) {
#ifdef MDZ_DEV_KNOBS
  static const char* env = getenv("MDZ_ATTN_SPLITS");  // development builds only
  if (env && atoi(env) > 0) return atoi(env) > 32 ? 32 : atoi(env);
#endif
  const int pairs = B * n_heads;
  if (fused) {
    int ps = num_cus() / pairs - 1;
    const int by_len = (int)sqrtf((float)(max_prefix >> 5) / 8.0f);
    if (ps > by_len) ps = by_len;
    if (ps > 31) ps = 31;
    return ps >= 1 ? ps + 1 : 1;
  }
  int nb = (max_prefix + kTQ + 31) / 32;
  int by_len = nb / 8;                        // >= 2 blocks per wave
  int by_fill = (512 + pairs - 1) / pairs;    // aim at ~512 workgroups
  int s = by_len < by_fill ? by_len : by_fill;
  if (s > 32) s = 32;
  if (s < 1) s = 1;
  return s;
}

int64_t attn_mfma_scratch_bytes(int B, int n_heads, int max_prefix) {
  int s = attn_splits(B, n_heads, max_prefix, true), s2 = attn_splits(B, n_heads, max_prefix, false);
  s = s > s2 ? s : s2;
  return s == 1 ? 0 : (int64_t)B * n_heads * s * (kTQ * kHD + 2 * kTQ) * 4;
}

template <typename E, bool Q8, int NU>
static int launch_attention_mfma_t(int tree, const void* q, const Partials* qkv, const float* cs, const KvGeom& g, void* kc,
                                   void* vc, int layer, const int32_t* seq_len, int B, int max_prefix, void* att_out,
                                   void* scratch, int64_t scratch_bytes, hipStream_t st) {
  if (B == 0) return MDZ_OK;
  // the merge buffer [4][128][32 NU + 2] + [4][2][32 NU] floats overlays the staged Q tile
  constexpr int lds_bytes = 4 * kHD * (32 * NU + 2) * 4 + 4 * 2 * 32 * NU * 4;
  static_assert(lds_bytes >= 32 * NU * kQRow && lds_bytes * (3 - NU) <= 160 * 1024, "LDS budget of the tree kernel");
  MDZ_SET_LDS_ONCE((attn_tree_mfma_kernel<E, Q8, NU>), lds_bytes);
  const int nq = q_heads(g);
  const int splits = attn_splits(B, nq, max_prefix, qkv != nullptr);
  MDZ_REQUIRE(scratch_bytes >= attn_mfma_scratch_bytes(B, nq, max_prefix), MDZ_EWORKSPACE,
              "attention: scratch too small");
  float* part_o = (float*)scratch;
  float* part_ml = part_o + (int64_t)B * nq * splits * kTQ * kHD;
  dim3 grid(splits, nq, B * (3 - NU));  // NU = 1: blockIdx.z = 2 * sequence + half
  const Partials none = single_slot(nullptr, 0, 0);
  launch_timed(PROF_ATTN, attn_tree_mfma_kernel<E, Q8, NU>, grid, 256, lds_bytes, st, tree, (const E*)q, qkv ? *qkv : none, cs, g,
               (E*)kc, (E*)vc, layer, seq_len, max_prefix, (E*)att_out, part_o, part_ml);
  MDZ_LAUNCH_CHECK();
  if (splits > 1) {
    launch_timed(PROF_ATTN, attn_combine_kernel<E>, dim3(nq, B, kTQ / 16), 256, 0, st, nq, splits, part_o, part_ml, (E*)att_out);
    MDZ_LAUNCH_CHECK();
  }
  return MDZ_OK;
}

int launch_attention_mfma(int dtype, int tree, const void* q, const Partials* qkv, const float* cs, const KvGeom& g,
                          void* kc, void* vc, int layer, const int32_t* seq_len, int B, int max_prefix, void* att_out,
                          void* scratch, int64_t scratch_bytes, hipStream_t st) {
  // 32 queries per workgroup (two workgroups per CU) where the kernel's time is its fixed chain and the machine has
  // room for twice the workgroups; 64 where K and V are long enough that passing them through the CUs twice costs
  // more (measured crossover: between 3K and 4K keys for 16-bit rows, between 12K and 16K for 8-bit rows).
  bool halves = B * q_heads(g) <= num_cus() && max_prefix < (g.quant ? 14336 : 3584);
#ifdef MDZ_DEV_KNOBS
  static const char* env = getenv("MDZ_ATTN_HALVES");  // development builds only: 1 = 32 queries per workgroup, 0 = 64
  if (env) halves = atoi(env) != 0;
#endif
#define MDZ_ATTN_CASE(Q8, NU)                                                                                          \
  MDZ_WITH_ELEM16(dtype, return (launch_attention_mfma_t<E, Q8, NU>(tree, q, qkv, cs, g, kc, vc, layer, seq_len, B,    \
                                                                    max_prefix, att_out, scratch, scratch_bytes, st)))
  if (g.quant) {
    if (halves) MDZ_ATTN_CASE(true, 1);
    MDZ_ATTN_CASE(true, 2);
  }
  if (halves) MDZ_ATTN_CASE(false, 1);
  MDZ_ATTN_CASE(false, 2);
#undef MDZ_ATTN_CASE
}

}  // namespace mdz
