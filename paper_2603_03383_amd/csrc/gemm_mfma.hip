// Weight-streaming skinny GEMM for bf16 storage on gfx950: sum_k X[m][k] * W[n][k] for M <= 64 rows (the T
// tree nodes of one sequence, or up to 32 batch rows for the Medusa heads).  This kernel moves >95 % of a
// verify step's bytes (the decoder weights), so it is built around the HBM stream:
//   * W arrives in the packed order (common.h): every wave-level load is one contiguous 1 KiB block
//     (16 B per lane) that already is the B operand of v_mfma_f32_32x32x16_bf16 — no LDS, no shuffles.
//   * A wave owns NT tiles of 32 output columns and keeps one whole K-stage (CK input features, 8 or 16
//     k-steps) of W in flight in registers while it multiplies the previous stage (double buffering; the
//     loop body is branch-free so the hardware wait counters let the prefetch overlap the MFMAs).
//   * X (<= 64 x K bf16, L2 resident) is staged per K-stage through LDS, shared by the WPB waves of a
//     workgroup, rows padded by 16 B so the 16 B-per-lane operand reads are bank-conflict free.
//   * Work decomposition is flat and persistent: the (column band, K-stage) units are numbered band-major
//     and cut into gridDim.x equal contiguous ranges, one per workgroup, so every CU streams the same
//     number of bytes whatever the matrix shape (a per-CU stream is latency bound at ~50 GB/s, so balance
//     decides the kernel's duration).  A range that ends inside a band leaves a partial sum; partial sums go
//     to numbered slots of a workspace and the consumer adds slots 0..count-1 in that fixed order, so the
//     result is deterministic (no floating-point atomics).
#include "kernels.h"

namespace mdz {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// owner of flat unit u when U units are cut into G ranges [floor(w*U/G), floor((w+1)*U/G))
__host__ __device__ inline int64_t range_owner(int64_t u, int64_t U, int64_t G) { return ((u + 1) * G - 1) / U; }

template <int WPB, int NT, int MT, int CK>
__global__ void __launch_bounds__(WPB * 64)
    gemm_mfma_kernel(const bf16_t* __restrict__ X, int M, int K, const bf16_t* __restrict__ Wp, int n_tiles,
                     int n_stages, float* __restrict__ P, int64_t ldp, int64_t part_stride,
                     int32_t* __restrict__ counts, int whole_bands) {
  constexpr int ROWS = MT * 32;
  constexpr int KS = CK / 16;                       // MFMA k-steps per stage
  constexpr int LROW = CK * 2 + 16;                 // bytes per staged X row (16 B pad)
  constexpr int XL = ROWS * (CK / 8) / (WPB * 64);  // 16-byte X loads per thread per stage
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];  // 2 stages of ROWS x LROW bytes
  uint8_t(*lds)[ROWS * LROW] = reinterpret_cast<uint8_t(*)[ROWS * LROW]>(lds_raw);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t G = gridDim.x, w = blockIdx.x;
  const int bands = (n_tiles + WPB * NT - 1) / (WPB * NT);
  const int64_t U = (int64_t)bands * n_stages;
  int u_lo, u_hi;  // flat unit range of this workgroup (U < 2^31: checked on the host)
  if (whole_bands) {
    u_lo = (int)(w * bands / G) * n_stages;
    u_hi = (int)((w + 1) * bands / G) * n_stages;
  } else {
    u_lo = (int)(w * U / G);
    u_hi = (int)((w + 1) * U / G);
  }
  if (u_lo >= u_hi) return;
  const int nst256 = (K + kStageFeatures - 1) / kStageFeatures;  // stages of the packed layout

  f32x16 acc[NT][MT];
  auto zero_acc = [&]() {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[nt][mt][r] = 0.f;
  };
  zero_acc();

  u32x4 xr[XL];
  u32x4 wb[2][NT][KS];

  // X rows beyond M re-read row M-1: an output row depends only on its own X row, and rows >= M are never
  // stored.  Tiles beyond n_tiles re-read tile 0 and are never stored.  Both keep the loads branch-free.
  // (band, stage) of the unit being loaded next / multiplied next, advanced incrementally (no divisions)
  int lb = u_lo / n_stages, lc = u_lo % n_stages;
  int cb = lb, cc = lc;
  auto load_x = [&]() {
    const int c = lc;
#pragma unroll
    for (int i = 0; i < XL; ++i) {
      int idx = threadIdx.x + i * (WPB * 64);
      int row = idx / (CK / 8), col = idx % (CK / 8);
      int rr = row < M ? row : M - 1;
      xr[i] = *reinterpret_cast<const u32x4*>(X + (int64_t)rr * K + (int64_t)c * CK + col * 8);
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < XL; ++i) {
      int idx = threadIdx.x + i * (WPB * 64);
      int row = idx / (CK / 8), col = idx % (CK / 8);
      *reinterpret_cast<u32x4*>(&lds[buf][row * LROW + col * 16]) = xr[i];
    }
  };
  auto load_w = [&](u32x4 (&dst)[NT][KS]) {  // also advances the load cursor
    const int b = lb, c = lc;
    if (++lc == n_stages) {
      lc = 0;
      ++lb;
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      int tile = (b * WPB + wave) * NT + nt;
      tile = tile < n_tiles ? tile : 0;
      // packed order [band of 4 tiles][stage of 256 features][tile in band][16 k-steps][lane]
      const int st = CK == 256 ? c : (c >> 1), kin0 = CK == 256 ? 0 : (c & 1) * 8;
      const int64_t unit = (((int64_t)(tile >> 2) * nst256 + st) * kBandTiles + (tile & 3)) * 16 + kin0;
      const u32x4* p = reinterpret_cast<const u32x4*>(Wp) + unit * 64 + lane;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) dst[nt][ks] = p[ks * 64];
    }
  };
  auto compute = [&](int buf, const u32x4 (&wv)[NT][KS]) {
    const uint8_t* base = &lds[buf][(lane & 31) * LROW + (lane >> 5) * 16];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      bf16x8 a[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) a[mt] = *reinterpret_cast<const bf16x8*>(base + mt * 32 * LROW + ks * 32);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        bf16x8 b = __builtin_bit_cast(bf16x8, wv[nt][ks]);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mt], b, acc[nt][mt], 0, 0, 0);
      }
    }
  };
  // Ends the current band segment after unit u: write the accumulators as partial-sum slot
  // (this workgroup's rank among the band's writers) and clear them.
  // D layout of the 32x32 MFMA: lane holds column (lane % 32); register r is row 8*(r/4) + 4*(lane/32) + r%4.
  auto flush = [&]() {
    const int b = cb;
    int slot = 0;
    if (!whole_bands) {
      const int64_t first_owner = range_owner((int64_t)b * n_stages, U, G);
      slot = (int)(w - first_owner);
      if (counts && threadIdx.x == 0 && slot == 0)
        counts[b] = (int)(range_owner((int64_t)(b + 1) * n_stages - 1, U, G) - first_owner + 1);
    } else if (counts && threadIdx.x == 0) {
      counts[b] = 1;
    }
    float* out = P + (int64_t)slot * part_stride;
    const int col = lane & 31, rbase = (lane >> 5) * 4;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int tile = (b * WPB + wave) * NT + nt;
      if (tile < n_tiles) {
        const int n = tile * 32 + col;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            int m = mt * 32 + 8 * (r >> 2) + rbase + (r & 3);
            if (m < M) out[(int64_t)m * ldp + n] = acc[nt][mt][r];
          }
      }
    }
    zero_acc();
  };
  // after multiplying a unit: flush if it was the band's last stage, then advance the compute cursor
  auto finish_unit = [&](bool last_of_range) {
    if (cc + 1 == n_stages || last_of_range) flush();
    if (++cc == n_stages) {
      cc = 0;
      ++cb;
    }
  };

  int u = u_lo;
  load_x();
  load_w(wb[0]);
  store_x(0);
  __syncthreads();
  // Steady state: two units per trip.  sched_barrier pins the order "issue the next unit's loads, then
  // multiply the current unit", so a whole stage of W per wave is in flight during the MFMAs.
  for (; u + 2 < u_hi; u += 2) {
    load_x();
    load_w(wb[1]);
    __builtin_amdgcn_sched_barrier(0);
    compute(0, wb[0]);
    __builtin_amdgcn_sched_barrier(0);
    finish_unit(false);
    store_x(1);
    __syncthreads();
    load_x();
    load_w(wb[0]);
    __builtin_amdgcn_sched_barrier(0);
    compute(1, wb[1]);
    __builtin_amdgcn_sched_barrier(0);
    finish_unit(false);
    store_x(0);
    __syncthreads();
  }
  if (u + 1 < u_hi) {  // two units left
    load_x();
    load_w(wb[1]);
    __builtin_amdgcn_sched_barrier(0);
    compute(0, wb[0]);
    __builtin_amdgcn_sched_barrier(0);
    finish_unit(false);
    store_x(1);
    __syncthreads();
    compute(1, wb[1]);
    finish_unit(true);
  } else {  // one unit left
    compute(0, wb[0]);
    finish_unit(true);
  }
}

struct GemmPlan {
  int wpb, nt, mt, ck, grid, whole;
};

constexpr int kNumCU = 256;

static GemmPlan plan_gemm(int M, int N, int K, int max_split) {
  GemmPlan p;
  const int n_tiles = N / 32;
  p.mt = M <= 32 ? 1 : 2;
  p.ck = K % 256 == 0 ? 256 : 128;
  p.whole = max_split <= 1;
  p.nt = 1;
  p.wpb = (!p.whole && n_tiles <= 128) ? 2 : 4;
  p.grid = kNumCU;
  static const char* env = getenv("MDZ_GEMM_PLAN");  // development knob: "wpb,nt,grid,ck" (0 = keep default)
  if (env) {
    int a = 0, b = 0, c = 0, d = 0;
    if (sscanf(env, "%d,%d,%d,%d", &a, &b, &c, &d) == 4) {
      if (a == 2 || a == 4) p.wpb = a;
      if (b == 1 || b == 2) p.nt = b;
      if (c > 0) p.grid = c;
      if ((d == 128 || d == 256) && K % d == 0) p.ck = d;
    }
  }
  if (p.nt == 2) p.ck = 128;  // two tiles per wave only fit the register file with the short stage
  const int bands = (n_tiles + p.wpb * p.nt - 1) / (p.wpb * p.nt);
  const int n_stages = K / p.ck;
  const int64_t U = (int64_t)bands * n_stages;
  if (p.whole) {
    if (p.grid > bands) p.grid = bands;
  } else {
    if (p.grid > U) p.grid = (int)U;
    // a band may be shared by at most max_split writers: ceil(n_stages / floor(U/grid)) + 1 <= max_split
    while (p.grid > 1) {
      int64_t per = U / p.grid;
      int64_t writers = (n_stages + per - 1) / per + 1;
      if (writers <= max_split) break;
      p.grid = p.grid * 3 / 4;
    }
  }
  if (p.grid < 1) p.grid = 1;
  return p;
}

bool gemm_mfma_supported(int dtype, int M, int N, int K) {
  return dtype == MDZ_BF16 && M >= 1 && M <= 64 && N % 32 == 0 && K % 128 == 0 && K >= 128;
}

int gemm_mfma_band_cols(int M, int N, int K, int max_split) {
  GemmPlan p = plan_gemm(M, N, K, max_split);
  return p.wpb * p.nt * 32;
}

// Writes partial sums into slots of P (slot s at P + s*part_stride, each [M][ldp] fp32).  counts[band] receives
// the number of slots written for each band of `*band_cols` columns (1 everywhere when max_split <= 1).
int launch_gemm_mfma(const void* X, const void* Wp, float* P, int M, int N, int K, int64_t ldp, int64_t part_stride,
                     int max_split, int32_t* counts, int* band_cols, hipStream_t st) {
  GemmPlan p = plan_gemm(M, N, K, max_split);
  ProfScope prof_(p.mt == 2 ? (p.wpb == 4 ? PROF_GEMM_W64 : PROF_GEMM_N64) : (p.wpb == 4 ? PROF_GEMM_W32 : PROF_GEMM_N32),
                  st);
  const int n_tiles = N / 32, n_stages = K / p.ck;
  *band_cols = p.wpb * p.nt * 32;
  const bf16_t* x = (const bf16_t*)X;
  const bf16_t* w = (const bf16_t*)Wp;
#define MDZ_GEMM_CASE(WPB, NT, MT, CK)                                                                       \
  if (p.wpb == WPB && p.nt == NT && p.mt == MT && p.ck == CK) {                                              \
    constexpr int lds_bytes = 2 * MT * 32 * (CK * 2 + 16);                                                   \
    static bool attr_set = false;                                                                            \
    if (!attr_set) {                                                                                         \
      MDZ_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_mfma_kernel<WPB, NT, MT, CK>),          \
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));                   \
      attr_set = true;                                                                                       \
    }                                                                                                        \
    gemm_mfma_kernel<WPB, NT, MT, CK><<<p.grid, WPB * 64, lds_bytes, st>>>(x, M, K, w, n_tiles, n_stages, P, \
                                                                           ldp, part_stride, counts, p.whole); \
  } else
  MDZ_GEMM_CASE(4, 1, 2, 256)
  MDZ_GEMM_CASE(2, 1, 2, 256)
  MDZ_GEMM_CASE(4, 1, 1, 256)
  MDZ_GEMM_CASE(2, 1, 1, 256)
  MDZ_GEMM_CASE(4, 1, 2, 128)
  MDZ_GEMM_CASE(2, 1, 2, 128)
  MDZ_GEMM_CASE(4, 2, 2, 128)
  MDZ_GEMM_CASE(4, 1, 1, 128)
  MDZ_GEMM_CASE(2, 1, 1, 128)
  MDZ_GEMM_CASE(4, 2, 1, 128) {
    MDZ_FAIL(MDZ_EUNSUPPORTED, "gemm: no kernel for plan %d,%d,%d,%d", p.wpb, p.nt, p.mt, p.ck);
  }
#undef MDZ_GEMM_CASE
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

}  // namespace mdz
