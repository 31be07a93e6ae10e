// GEMM for many rows (several sequences verified together: M = B * T >= 128): sum_k X[m][k] * W[n][k], bf16 or fp16
// in (element type E), fp32 out.  At M = 1024 the layer GEMMs are bound by the matrix cores, not by the weight stream (1024 flop per
// weight byte against a machine balance of ~312), so this kernel is built around operand reuse:
//   * a workgroup (4 waves) owns a 128-row x 256-column output tile; a wave owns two 32-column tiles and all 128
//     rows: 8 accumulator tiles of 32 x 32 (128 accumulator registers; 256 rows would use the whole accumulator
//     file and the compiler then spills inside the loop);
//   * W arrives in the packed order (common.h): a wave-level load is one contiguous 1 KiB block that already is the
//     B operand of v_mfma_f32_32x32x16_bf16; one 64-feature stage per tile is double buffered in registers (a ring
//     of four stages was measured slower: the kernel is bound by the CU's request rate, not by latency);
//   * X (128 rows x 64 features per stage, L2 resident) is staged through LDS, double buffered, rows padded by 16 B
//     so the 16-byte-per-lane A-operand reads are bank-conflict free; every A operand read from LDS feeds two
//     MFMAs, which keeps the LDS pipe (128 B/clk) below the matrix pipe;
//   * narrow matrices are split along K into numbered partial-sum slots so that every CU has a tile (the consumer
//     adds the slots in order: deterministic, no float atomics);
//   * SWIGLU: for the gate/up matrix (gate and up tiles alternate in the packed order, so a wave's two tiles are the
//     gate and the up columns of the same 32 features) an unsplit launch writes SiLU(gate) * up as E straight from
//     the accumulators instead of 2 F fp32 sums per row for a second kernel to read back.
#include "kernels.h"

namespace mdz {

typedef f32x16_t f32x16;
typedef u32x4_t u32x4;

namespace {
constexpr int kBM = 128;                 // rows per workgroup
constexpr int kNT = 2;                   // 32-column tiles per wave
constexpr int kBN = 4 * kNT * 32;        // columns per workgroup
constexpr int kCK = 64;                  // features per stage
constexpr int kKS = kCK / 16;            // MFMA k-steps per stage
constexpr int kLRow = kCK * 2 + 16;      // bytes per staged X row
constexpr int kXL = kBM * (kCK / 8) / 256;  // 16-byte X loads per thread per stage
constexpr int kLdsBytes = 2 * kBM * kLRow;
}  // namespace

__device__ inline float silu_large(float v) { return v / (1.0f + expf(-v)); }

template <typename E, bool SWIGLU>
__global__ void __launch_bounds__(256)
    gemm_large_kernel(const E* __restrict__ X, int M, int K, const E* __restrict__ Wp, int n_tiles,
                      float* __restrict__ P, int ldp, int64_t part_stride, int stages_per_split, int nb_n, int nb_m,
                      E* __restrict__ U) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
  uint8_t(*lds)[kBM * kLRow] = reinterpret_cast<uint8_t(*)[kBM * kLRow]>(lds_raw);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Column blocks are dealt to XCDs the same
  // way and an XCD walks its column blocks with the row blocks innermost, so the workgroups that re-read one block
  // of W run on one XCD at about the same time and share it through that L2.
  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  const int bn = (seq / nb_m) * 8 + xcd, bm = seq % nb_m;
  if (bn >= nb_n) return;
  const int m0 = bm * kBM;
  const int n_stages = K / kCK;
  const int s_lo = blockIdx.z * stages_per_split, s_hi = min(s_lo + stages_per_split, n_stages);
  const int nst256 = (K + kStageFeatures - 1) / kStageFeatures;

  f32x16 acc[kNT][kBM / 32];
#pragma unroll
  for (int nt = 0; nt < kNT; ++nt)
#pragma unroll
    for (int mt = 0; mt < kBM / 32; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[nt][mt][r] = 0.f;

  // tiles beyond n_tiles re-read tile 0 and rows beyond M re-read row M-1; neither is stored
  const u32x4* wp[kNT];
#pragma unroll
  for (int nt = 0; nt < kNT; ++nt) {
    int tile = (bn * 4 + wave) * kNT + nt;
    tile = tile < n_tiles ? tile : 0;
    // packed order [band of 4 tiles][stage of 256 features][tile in band][16 k-steps][lane]
    wp[nt] = reinterpret_cast<const u32x4*>(Wp) + ((int64_t)(tile >> 2) * nst256 * kBandTiles + (tile & 3)) * 16 * 64 + lane;
  }
  u32x4 xr[kXL];
  u32x4 wb[2][kNT][kKS];
  auto load_x = [&](int s) {
#pragma unroll
    for (int i = 0; i < kXL; ++i) {
      const int idx = threadIdx.x + i * 256;
      const int row = idx / (kCK / 8), col = idx % (kCK / 8);
      const int rr = min(m0 + row, M - 1);
      xr[i] = *reinterpret_cast<const u32x4*>(X + (int64_t)rr * K + (int64_t)s * kCK + col * 8);
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < kXL; ++i) {
      const int idx = threadIdx.x + i * 256;
      const int row = idx / (kCK / 8), col = idx % (kCK / 8);
      *reinterpret_cast<u32x4*>(&lds[buf][row * kLRow + col * 16]) = xr[i];
    }
  };
  auto load_w = [&](int s, u32x4 (&dst)[kNT][kKS]) {
    // stage s covers k-steps [s * kKS, (s + 1) * kKS) of the matrix; the layout groups 16 k-steps per 256 features
    const int ks0 = s * kKS;
    const int64_t off = ((int64_t)(ks0 >> 4) * kBandTiles * 16 + (ks0 & 15)) * 64;
#pragma unroll
    for (int nt = 0; nt < kNT; ++nt)
#pragma unroll
      for (int ks = 0; ks < kKS; ++ks) dst[nt][ks] = wp[nt][off + ks * 64];
  };
  auto compute = [&](int buf, const u32x4 (&wv)[kNT][kKS]) {
    const uint8_t* base = &lds[buf][(lane & 31) * kLRow + (lane >> 5) * 16];
    u32x4 a[2][kBM / 32];
#pragma unroll
    for (int mt = 0; mt < kBM / 32; ++mt) a[0][mt] = *reinterpret_cast<const u32x4*>(base + mt * 32 * kLRow);
#pragma unroll
    for (int ks = 0; ks < kKS; ++ks) {
      // the A operands of the next k-step are read from LDS while this k-step's MFMAs run; sched_barrier keeps that
      // order (the compiler's own interleaving was measured 20 % slower)
      if (ks + 1 < kKS) {
#pragma unroll
        for (int mt = 0; mt < kBM / 32; ++mt)
          a[(ks + 1) & 1][mt] = *reinterpret_cast<const u32x4*>(base + mt * 32 * kLRow + (ks + 1) * 32);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int mt = 0; mt < kBM / 32; ++mt)
#pragma unroll
        for (int nt = 0; nt < kNT; ++nt)
          acc[nt][mt] = Elem16<E>::mfma(a[ks & 1][mt], wv[nt][ks], acc[nt][mt]);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  if (s_lo < s_hi) {
    load_x(s_lo);
    load_w(s_lo, wb[0]);
    store_x(0);
    __syncthreads();
    int s = s_lo;
    for (; s + 2 < s_hi; s += 2) {  // two stages per trip: the register and LDS buffers alternate statically
      load_x(s + 1);
      load_w(s + 1, wb[1]);
      compute(0, wb[0]);
      store_x(1);
      __syncthreads();
      load_x(s + 2);
      load_w(s + 2, wb[0]);
      compute(1, wb[1]);
      store_x(0);
      __syncthreads();
    }
    if (s + 1 < s_hi) {
      load_x(s + 1);
      load_w(s + 1, wb[1]);
      compute(0, wb[0]);
      store_x(1);
      __syncthreads();
      compute(1, wb[1]);
    } else {
      compute(0, wb[0]);
    }
  }

  // D layout of the 32x32 MFMA: lane holds column (lane % 32); register r is row 8*(r/4) + 4*(lane/32) + r%4.
  const int col = lane & 31, rbase = (lane >> 5) * 4;
  if constexpr (SWIGLU) {
    // tiles (2j, 2j + 1) of this wave = gate and up of features 32j .. 32j + 31; U is [M][n_tiles * 16]
    const int j = bn * 4 + wave;
    if (2 * j + 1 < n_tiles) {
      const int F = n_tiles * 16;
      E* urow = U + j * 32 + col;
#pragma unroll
      for (int mt = 0; mt < kBM / 32; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = m0 + mt * 32 + 8 * (r >> 2) + rbase + (r & 3);
          if (m < M) urow[(int64_t)m * F] = from_float<E>(silu_large(acc[0][mt][r]) * acc[1][mt][r]);
        }
    }
    return;
  }
  float* out = P + (int64_t)blockIdx.z * part_stride;
  int pitch = ldp;
  asm volatile("" : "+s"(pitch));  // keeps the row offsets out of registers until they are needed
#pragma unroll
  for (int nt = 0; nt < kNT; ++nt) {
    const int tile = (bn * 4 + wave) * kNT + nt;
    if (tile < n_tiles) {
      const int n = tile * 32 + col;
#pragma unroll
      for (int mt = 0; mt < kBM / 32; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = m0 + mt * 32 + 8 * (r >> 2) + rbase + (r & 3);
          if (m < M) out[m * pitch + n] = acc[nt][mt][r];
        }
    }
  }
}

namespace {
struct LargePlan {
  int nb_n, nb_m, ksplit, stages_per_split;
};
LargePlan plan_large(int M, int N, int K) {
  LargePlan p;
  p.nb_n = (N + kBN - 1) / kBN;
  p.nb_m = (M + kBM - 1) / kBM;
  const int n_stages = K / kCK;
  int want = (num_cus() + p.nb_n * p.nb_m - 1) / (p.nb_n * p.nb_m);  // enough workgroups for every CU
  if (want > 8) want = 8;
  if (want > n_stages) want = n_stages;
  if (want < 1) want = 1;
  p.stages_per_split = (n_stages + want - 1) / want;
  p.ksplit = (n_stages + p.stages_per_split - 1) / p.stages_per_split;
  return p;
}
}  // namespace

bool gemm_large_supported(int dtype, int M, int N, int K) {
  return is_16bit(dtype) && M >= 128 && N % 32 == 0 && K % kCK == 0 && K >= kCK && (int64_t)M * N < (int64_t)1 << 31;
}

// partial-sum slots launch_gemm_large will write for this problem (sizes the slot workspace)
int gemm_large_slots(int M, int N, int K) { return plan_large(M, N, K).ksplit; }

template <typename E, bool SWIGLU>
static int launch_gemm_large_t(const void* X, const void* Wp, float* P, int M, int N, int K, int64_t ldp,
                               int64_t part_stride, Partials* res, void* U, hipStream_t st) {
  const LargePlan p = plan_large(M, N, K);
  MDZ_REQUIRE((int64_t)M * ldp < (int64_t)1 << 31, MDZ_ESHAPE, "gemm: output of %d rows with pitch %lld is too large", M,
              (long long)ldp);
  MDZ_SET_LDS_ONCE((gemm_large_kernel<E, SWIGLU>), kLdsBytes);
  MDZ_REQUIRE(!SWIGLU || (p.ksplit == 1 && N % 64 == 0 && U), MDZ_EUNSUPPORTED, "gemm: fused SwiGLU needs an unsplit launch");
  res->n = p.ksplit;
  res->split_grid = 0;
  res->band_cols = kBN;
  res->n_stages = 1;
  res->split_units = 0;
  const int groups = (p.nb_n + 7) / 8;  // column blocks per XCD
  launch_timed(PROF_GEMM_LARGE, gemm_large_kernel<E, SWIGLU>, dim3(8 * groups * p.nb_m, 1, p.ksplit), 256, kLdsBytes, st,
               (const E*)X, M, K, (const E*)Wp, N / 32, P, (int)ldp, part_stride, p.stages_per_split, p.nb_n, p.nb_m,
               (E*)U);
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

int launch_gemm_large(int dtype, const void* X, const void* Wp, float* P, int M, int N, int K, int64_t ldp,
                      int64_t part_stride, Partials* res, hipStream_t st) {
  MDZ_WITH_ELEM16(dtype, return (launch_gemm_large_t<E, false>(X, Wp, P, M, N, K, ldp, part_stride, res, nullptr, st)));
}

// gate/up GEMM with the SwiGLU applied in the epilogue: U [M][N / 2] of the storage type.  Only where the large kernel
// runs unsplit (gemm_large_swiglu_supported); P is not written.
bool gemm_large_swiglu_supported(int dtype, int M, int N, int K) {
  return gemm_large_supported(dtype, M, N, K) && N % 64 == 0 && plan_large(M, N, K).ksplit == 1;
}

int launch_gemm_large_swiglu(int dtype, const void* X, const void* Wp, void* U, int M, int N, int K, hipStream_t st) {
  Partials unused;
  MDZ_WITH_ELEM16(dtype, return (launch_gemm_large_t<E, true>(X, Wp, nullptr, M, N, K, N, 0, &unused, U, st)));
}

}  // namespace mdz
