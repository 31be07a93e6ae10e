// Weight-streaming skinny GEMM for 16-bit storage (bf16 or fp16, element type E) on gfx950: sum_k X[m][k] * W[n][k] for M <= 64 rows (the T
// tree nodes of one sequence, or up to 32 batch rows for the Medusa heads).  This kernel moves >95 % of a
// verify step's bytes (the decoder weights), so it is built around the HBM stream:
//   * W arrives in the packed order (common.h): every wave-level load is one contiguous 1 KiB block
//     (16 B per lane) that already is the B operand of v_mfma_f32_32x32x16_bf16 / _f16 — no LDS, no shuffles.
//   * A wave owns NT tiles of 32 output columns and moves W through a ring of four half K-stages in
//     registers: three half stages (CK/2 input features each) stay in flight while it multiplies the
//     fourth, and every load is unconditional so the hardware wait counters let the prefetch overlap
//     the MFMAs (a CU then keeps ~100 KB in flight, what the HBM latency asks for).
//   * X (<= 64 x K bf16, L2 resident) is staged per K-stage through LDS, shared by the WPB waves of a
//     workgroup, rows padded by 16 B so the 16 B-per-lane operand reads are bank-conflict free.
//   * Work decomposition is flat and persistent: the (column band, K-stage) units are numbered band-major
//     and cut into gridDim.x equal contiguous ranges, one per workgroup, so every CU streams the same
//     number of bytes whatever the matrix shape (a per-CU stream is latency bound at ~50 GB/s, so balance
//     decides the kernel's duration).  The grid is one workgroup per CU, or a little fewer when that makes
//     the ranges line up with the bands (plan_gemm).  A range that ends inside a band leaves a partial sum; partial sums go
//     to numbered slots of a workspace and the consumer adds slots 0..count-1 in that fixed order, so the
//     result is deterministic (no floating-point atomics).
//   * SWIGLU (the gate/up matrix, whose gate and up tiles alternate in the packed order, run with whole bands per
//     workgroup): waves 0/2 hold the gate columns and waves 1/3 the up columns of the same 32 features; at the end of
//     a band the up sums cross to their partner through LDS and SiLU(gate) * up is written as E, so neither the
//     fp32 sums nor a second kernel are needed.
//   * ARGMAX (the LM head of a verify pass, whole bands per workgroup, when the caller wants no logits): at the end
//     of a band a wave turns its 64 x 32 sums through LDS so that lane m holds row m, scans the 32 columns and keeps
//     the row's best (value, column) so far in two registers; at the end of its range it writes one candidate per
//     row.  A small kernel merges the workgroups' candidates; the fp32 logits never exist in memory.
#include "kernels.h"

namespace mdz {

typedef f32x16_t f32x16;
typedef u32x4_t u32x4;

__device__ inline float silu_mfma(float v) { return v / (1.0f + expf(-v)); }

template <int WPB, int NT, int MT, int CK, typename E, bool SWIGLU = false, bool ARGMAX = false>
__global__ void __launch_bounds__(WPB * 64)
    gemm_mfma_kernel(const E* __restrict__ X, int M, int K, const E* __restrict__ Wp, int n_tiles,
                     int n_stages, float* __restrict__ P, int64_t ldp, int64_t part_stride, int whole_bands,
                     E* __restrict__ Uout = nullptr, ArgCand* __restrict__ cand = nullptr) {
  static_assert(!SWIGLU || (WPB == 4 && NT == 1), "the SwiGLU epilogue pairs waves 0/1 and 2/3");
  static_assert(!ARGMAX || (NT == 1 && !SWIGLU), "the argmax epilogue scans one tile per wave");
  constexpr int ROWS = MT * 32;
  constexpr int KH = CK / 32;                       // MFMA k-steps per half stage
  constexpr int LROW = CK * 2 + 16;                 // bytes per staged X row (16 B pad)
  constexpr int XL = ROWS * (CK / 8) / (WPB * 64);  // 16-byte X loads per thread per stage
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];  // 2 stages of ROWS x LROW bytes
  uint8_t(*lds)[ROWS * LROW] = reinterpret_cast<uint8_t(*)[ROWS * LROW]>(lds_raw);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t G = gridDim.x, w = blockIdx.x;
  const uint32_t bands = (n_tiles + WPB * NT - 1) / (WPB * NT);
  const uint32_t U = bands * n_stages;
  int u_lo, u_hi;  // flat unit range of this workgroup (U * G < 2^31: checked on the host)
  if (whole_bands) {
    u_lo = (int)(w * bands / G) * n_stages;
    u_hi = (int)((w + 1) * bands / G) * n_stages;
  } else {
    u_lo = (int)(w * U / G);
    u_hi = (int)((w + 1) * U / G);
  }
  // ARGMAX: the best (value, column) of row (lane % ROWS) over the tiles this wave has finished; written as
  // candidate [row][workgroup * WPB + wave] when the range ends (also by a workgroup with an empty range)
  float best_v = -INFINITY;
  int best_i = kNoIndex;
  auto write_cand = [&]() {
    if constexpr (ARGMAX) {
      if (lane < ROWS && lane < M) cand[(int64_t)lane * (G * WPB) + w * WPB + wave] = ArgCand{best_v, best_i};
    }
  };
  MDZ_STAMP(0);
  if (u_lo >= u_hi) {
    write_cand();
    return;
  }
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
  u32x4 wb[4][NT][KH];  // ring of four half stages of W

  // X rows beyond M re-read row M-1: an output row depends only on its own X row, and rows >= M are never
  // stored.  Tiles beyond n_tiles re-read tile 0 and are never stored.  Loads past the end of the range re-read
  // the range's last half stage / last unit (a cache hit) and are never multiplied.  All of this keeps every
  // load unconditional, so the hardware's in-order wait counters let three half stages stay in flight.
  // Cursors, advanced incrementally (no divisions): W load (band, stage, half), X load (stage), compute (band, stage).
  int lb = u_lo / n_stages, lc = u_lo % n_stages, lh = 0, l_left = 2 * (u_hi - u_lo) - 1;  // advances left
  int xc = lc, x_left = u_hi - u_lo - 1;
  int cb = lb, cc = lc;
  auto load_x = [&]() {  // loads the X columns of the stage under the X cursor, then advances it
    const int c = xc;
    const int adv = x_left > 0;
    x_left -= adv;
    xc = (xc + adv == n_stages) ? 0 : xc + adv;
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
  auto load_w = [&](u32x4 (&dst)[NT][KH]) {  // loads the half stage under the W cursor, then advances it
    const int b = lb, c = lc, hf = lh;
    const int adv = l_left > 0;
    l_left -= adv;
    const int carry = lh & adv;  // the second half of a stage is followed by the next stage
    lh ^= adv;
    const int wrap = carry & (lc + 1 == n_stages);
    lc = wrap ? 0 : lc + carry;
    lb += wrap;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      int tile = (b * WPB + wave) * NT + nt;
      tile = tile < n_tiles ? tile : 0;
      // packed order [band of 4 tiles][stage of 256 features][tile in band][16 k-steps][lane]
      const int st = CK == 256 ? c : (c >> 1), kin0 = (CK == 256 ? 0 : (c & 1) * 8) + hf * KH;
      const int64_t unit = (((int64_t)(tile >> 2) * nst256 + st) * kBandTiles + (tile & 3)) * 16 + kin0;
      const u32x4* p = reinterpret_cast<const u32x4*>(Wp) + unit * 64 + lane;
#pragma unroll
      for (int ks = 0; ks < KH; ++ks) dst[nt][ks] = p[ks * 64];
    }
  };
  auto compute = [&](int buf, int hf, const u32x4 (&wv)[NT][KH]) {
    const uint8_t* base = &lds[buf][(lane & 31) * LROW + (lane >> 5) * 16 + hf * KH * 32];
#pragma unroll
    for (int ks = 0; ks < KH; ++ks) {
      u32x4 a[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) a[mt] = *reinterpret_cast<const u32x4*>(base + mt * 32 * LROW + ks * 32);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = Elem16<E>::mfma(a[mt], wv[nt][ks], acc[nt][mt]);
      }
    }
  };
  // Ends the current band segment: write the accumulators as partial-sum slot (this workgroup's rank among
  // the band's writers) and clear them.
  // D layout of the 32x32 MFMA: lane holds column (lane % 32); register r is row 8*(r/4) + 4*(lane/32) + r%4.
  auto flush = [&]() {
    const int b = cb;
    if constexpr (SWIGLU) {
      // exchange buffer behind the two X stages: [pair][row][33] floats
      float* xch = reinterpret_cast<float*>(lds_raw + 2 * ROWS * LROW) + (wave >> 1) * ROWS * 33;
      const int col = lane & 31, rbase = (lane >> 5) * 4;
      if (wave & 1) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int r = 0; r < 16; ++r) xch[(mt * 32 + 8 * (r >> 2) + rbase + (r & 3)) * 33 + col] = acc[0][mt][r];
      }
      __syncthreads();
      const int tile = b * WPB + wave;  // even waves: a gate tile; its features are 16 * tile .. + 31
      if (!(wave & 1) && tile + 1 < n_tiles) {
        int F = n_tiles * 16;  // (M * F < 2^31: checked on the host; opaque so that the row offsets are not hoisted)
        asm volatile("" : "+s"(F));
        E* urow = Uout + tile * 16 + col;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int m = mt * 32 + 8 * (r >> 2) + rbase + (r & 3);
            if (m < M) urow[m * F] = from_float<E>(silu_mfma(acc[0][mt][r]) * xch[m * 33 + col]);
          }
      }
      __syncthreads();
      zero_acc();
      return;
    }
    if constexpr (ARGMAX) {
      // the wave's own turn buffer behind the two X stages: [row][33] floats (no other wave touches it: no barrier)
      float* turn = reinterpret_cast<float*>(lds_raw + 2 * ROWS * LROW) + wave * ROWS * 33;
      const int col = lane & 31, rbase = (lane >> 5) * 4;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) turn[(mt * 32 + 8 * (r >> 2) + rbase + (r & 3)) * 33 + col] = acc[0][mt][r];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      const int tile = b * WPB + wave;
      if (tile < n_tiles) {
        const float* rp = turn + (lane % ROWS) * 33;
#pragma unroll
        for (int c = 0; c < 32; ++c) {
          const float v = rp[c];
          if (precedes(v, tile * 32 + c, best_v, best_i)) best_v = v, best_i = tile * 32 + c;
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      zero_acc();
      return;
    }
    // slot = this workgroup's rank among the ranges that touch the band (see Partials::count)
    const int slot = whole_bands ? 0 : (int)(w - Partials::owner((uint32_t)b * n_stages, U, G));
    float* out = P + (int64_t)slot * part_stride;
    const int col = lane & 31, rbase = (lane >> 5) * 4;
    // 32-bit element offsets (the host checks M * ldp < 2^31).  The empty asm makes the row pitch opaque here,
    // so the 32 row offsets are recomputed per flush (one multiply-add each) instead of being hoisted out of
    // the stream loop, where they would hold 64 registers for the whole kernel.
    int pitch = (int)ldp;
    asm volatile("" : "+s"(pitch));
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
            if (m < M) out[m * pitch + n] = acc[nt][mt][r];
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

  // X (an L2 hit) is requested first: the wait counters are in-order, so staging it then waits for nothing
  // that comes from HBM, and the first barrier passes while the first W half stages are still in flight.
  load_x();
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_barrier();  // all four waves' X requests enter the CU's memory pipeline ahead of any W request
  __builtin_amdgcn_sched_barrier(0);
  load_w(wb[0]);
  load_w(wb[1]);
  load_w(wb[2]);
  __builtin_amdgcn_sched_barrier(0);
  store_x(0);
  __syncthreads();
  MDZ_STAMP(1);
  // Steady state: two units (four half stages) per trip.  Before a half stage is multiplied the half stage
  // three ahead of it is requested, so three half stages of W per wave are in flight during the MFMAs;
  // sched_barrier pins that order.  The X columns of the next unit are requested at the start of a unit and
  // staged into the other LDS buffer after the unit's MFMAs.
  for (int u = u_lo; u < u_hi; u += 2) {
    load_x();
    load_w(wb[3]);
    __builtin_amdgcn_sched_barrier(0);
    compute(0, 0, wb[0]);
    __builtin_amdgcn_sched_barrier(0);
    if (u == u_lo) MDZ_STAMP(2);
    load_w(wb[0]);
    __builtin_amdgcn_sched_barrier(0);
    compute(0, 1, wb[1]);
    __builtin_amdgcn_sched_barrier(0);
    finish_unit(u + 1 == u_hi);
    store_x(1);
    __syncthreads();
    // second unit of the trip; past the end of the range its loads repeat the last ones and nothing is multiplied
    const bool live = u + 1 < u_hi;
    load_x();
    load_w(wb[1]);
    __builtin_amdgcn_sched_barrier(0);
    if (live) compute(1, 0, wb[2]);
    __builtin_amdgcn_sched_barrier(0);
    load_w(wb[2]);
    __builtin_amdgcn_sched_barrier(0);
    if (live) {
      compute(1, 1, wb[3]);
      finish_unit(u + 2 == u_hi);
    }
    __builtin_amdgcn_sched_barrier(0);
    store_x(0);
    __syncthreads();
  }
  MDZ_STAMP(3);
  write_cand();
}

struct GemmPlan {
  int wpb, nt, mt, ck, grid, whole;
  int slots;  // most partial-sum slots any band receives
};

static GemmPlan plan_gemm(int M, int N, int K, int max_split) {
  GemmPlan p;
  const int n_tiles = N / 32;
  p.mt = M <= 32 ? 1 : 2;
  // Stages of 128 features: the ring then holds 12 KiB per wave, the first product starts after 48 KiB per CU
  // instead of 96, and ranges are cut twice as finely; measured faster than 256 on every decoder shape.  Four
  // waves per workgroup share one staged X tile (X : W request bytes = 1 : 2; two waves would make it 1 : 1).
  p.ck = 128;
  p.whole = max_split <= 1;
  p.nt = 1;
  p.wpb = 4;
  const int kNumCU = num_cus();
  p.grid = kNumCU;
  bool forced = false;
#ifdef MDZ_DEV_KNOBS
  static const char* env = getenv("MDZ_GEMM_PLAN");  // development builds only: "wpb,nt,grid,ck" (0 = keep default)
  if (env) {
    int a = 0, b = 0, c = 0, d = 0;
    if (sscanf(env, "%d,%d,%d,%d", &a, &b, &c, &d) == 4) {
      if (a == 2 || a == 4) p.wpb = a;
      if (c > 0) p.grid = c;
      if ((d == 128 || d == 256) && K % d == 0) p.ck = d;
      forced = true;
    }
  }
#endif
  const int bands = (n_tiles + p.wpb * p.nt - 1) / (p.wpb * p.nt);
  const int n_stages = K / p.ck;
  const int64_t U = (int64_t)bands * n_stages;
  p.slots = 1;
  // A grid a little under one workgroup per CU whose equal ranges line up with the column bands (a range is a whole
  // number of bands, or a band a whole number of ranges) leaves no range that straddles a band: fewer partial-sum
  // slots for the consumer to add and no flush in mid-stream.
  if (!p.whole && !forced) {
    for (int gsz = kNumCU; gsz >= kNumCU * 3 / 4; --gsz) {
      if (U % gsz) continue;
      const int64_t u = U / gsz;
      if (n_stages % u == 0 || u % n_stages == 0) {
        p.grid = gsz;
        break;
      }
    }
  }
  if (p.whole) {
    if (p.grid > bands) p.grid = bands;
  } else {
    if (p.grid > U) p.grid = (int)U;
    // the most ranges that touch one band (exact, by the ownership rule of Partials) must fit max_split slots
    auto most_writers = [&](int grid) {
      uint32_t most = 0;
      for (int b = 0; b < bands; ++b) {
        uint32_t n = Partials::owner((uint32_t)(b + 1) * n_stages - 1, (uint32_t)U, grid) -
                     Partials::owner((uint32_t)b * n_stages, (uint32_t)U, grid) + 1;
        most = n > most ? n : most;
      }
      return (int)most;
    };
    while (p.grid > 1 && (U * p.grid >= (int64_t)1 << 31 || (p.slots = most_writers(p.grid)) > max_split)) p.grid = p.grid * 7 / 8;
    if (p.grid <= 1) p.slots = 1;
  }
  if (p.grid < 1) p.grid = 1;
  return p;
}

// most partial-sum slots per band that launch_gemm_mfma will use for this problem (sizes the slot workspace)
int gemm_mfma_slots(int M, int N, int K, int max_split) { return plan_gemm(M, N, K, max_split).slots; }

bool gemm_mfma_supported(int dtype, int M, int N, int K) {
  return is_16bit(dtype) && M >= 1 && M <= 64 && N % 32 == 0 && K % 128 == 0 && K >= 128;
}

// The decomposition launch_gemm_mfma will use, as the consumers see it (no GPU work): fills the slot-count fields of
// *res and, if grid is given, the number of workgroups.
void gemm_mfma_describe(int M, int N, int K, int max_split, Partials* res, int* grid) {
  const GemmPlan p = plan_gemm(M, N, K, max_split);
  const int n_tiles = N / 32, n_stages = K / p.ck;
  const int bands = (n_tiles + p.wpb * p.nt - 1) / (p.wpb * p.nt);
  res->band_cols = p.wpb * p.nt * 32;
  res->n_stages = n_stages;
  res->split_units = (uint32_t)bands * n_stages;
  res->split_grid = p.whole ? 0 : (uint32_t)p.grid;
  res->n = p.slots;
  if (grid) *grid = p.grid;
}

// Writes partial sums into slots of P (slot s at P + s*part_stride, each [M][ldp] fp32) and fills the fields of
// *res that describe how many slots each band of columns received (one everywhere when max_split <= 1).
template <typename E>
static int launch_gemm_mfma_t(const void* X, const void* Wp, float* P, int M, int N, int K, int64_t ldp, int64_t part_stride,
                              int max_split, Partials* res, hipStream_t st) {
  GemmPlan p = plan_gemm(M, N, K, max_split);
  const int tag = p.mt == 2 ? (p.wpb == 4 ? PROF_GEMM_W64 : PROF_GEMM_N64) : (p.wpb == 4 ? PROF_GEMM_W32 : PROF_GEMM_N32);
  const int n_tiles = N / 32, n_stages = K / p.ck;
  MDZ_REQUIRE((int64_t)M * ldp < (int64_t)1 << 31, MDZ_ESHAPE, "gemm: output of %d rows with pitch %lld is too large", M,
              (long long)ldp);
  const int bands = (n_tiles + p.wpb * p.nt - 1) / (p.wpb * p.nt);
  MDZ_REQUIRE((int64_t)bands * n_stages * p.grid < (int64_t)1 << 31, MDZ_ESHAPE, "gemm: %d x %d units on %d workgroups overflow",
              bands, n_stages, p.grid);
  gemm_mfma_describe(M, N, K, max_split, res, nullptr);
  const E* x = (const E*)X;
  const E* w = (const E*)Wp;
#define MDZ_GEMM_CASE(WPB, NT, MT, CK)                                                                       \
  if (p.wpb == WPB && p.nt == NT && p.mt == MT && p.ck == CK) {                                              \
    constexpr int lds_bytes = 2 * MT * 32 * (CK * 2 + 16);                                                   \
    MDZ_SET_LDS_ONCE((gemm_mfma_kernel<WPB, NT, MT, CK, E>), lds_bytes);                                     \
    launch_timed(tag, gemm_mfma_kernel<WPB, NT, MT, CK, E>, p.grid, WPB * 64, lds_bytes, st, x, M, K, w, n_tiles, \
                 n_stages, P, ldp, part_stride, p.whole, nullptr, nullptr);                                       \
  } else
  MDZ_GEMM_CASE(4, 1, 2, 128)
  MDZ_GEMM_CASE(4, 1, 1, 128)
  MDZ_GEMM_CASE(2, 1, 2, 128)
  MDZ_GEMM_CASE(2, 1, 1, 128)
  MDZ_GEMM_CASE(4, 1, 2, 256)
  MDZ_GEMM_CASE(4, 1, 1, 256) {
    MDZ_FAIL(MDZ_EUNSUPPORTED, "gemm: no kernel for plan %d,%d,%d,%d", p.wpb, p.nt, p.mt, p.ck);
  }
#undef MDZ_GEMM_CASE
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

// The gate/up GEMM with the SwiGLU in its epilogue: U [M][N / 2] of the storage type.  Whole bands per workgroup, so
// it is taken only where the bands nearly fill the chip (or fill it a whole number of times).
bool gemm_mfma_swiglu_supported(int dtype, int M, int N, int K) {
  if (!gemm_mfma_supported(dtype, M, N, K) || N % 128 != 0) return false;
  const int bands = N / 128, kNumCU = num_cus();
  return (bands >= kNumCU * 5 / 8 && bands <= kNumCU) || (bands > kNumCU && bands % kNumCU == 0);
}

template <typename E>
static int launch_gemm_mfma_swiglu_t(const void* X, const void* Wp, void* U, int M, int N, int K, hipStream_t st) {
  const int tag = M <= 32 ? PROF_GEMM_W32 : PROF_GEMM_W64;
  const int n_tiles = N / 32, n_stages = K / 128, bands = N / 128, kNumCU = num_cus();
  const int grid = bands < kNumCU ? bands : kNumCU;
  MDZ_REQUIRE((int64_t)bands * n_stages * grid < (int64_t)1 << 31 && (int64_t)M * N < (int64_t)1 << 31, MDZ_ESHAPE,
              "gemm: %d x %d units overflow", bands, n_stages);
#define MDZ_SWIGLU_CASE(MT)                                                                                         \
  {                                                                                                                  \
    constexpr int lds_bytes = 2 * MT * 32 * (128 * 2 + 16) + 2 * MT * 32 * 33 * 4;                                   \
    MDZ_SET_LDS_ONCE((gemm_mfma_kernel<4, 1, MT, 128, E, true>), lds_bytes);                                         \
    launch_timed(tag, gemm_mfma_kernel<4, 1, MT, 128, E, true>, grid, 256, lds_bytes, st, (const E*)X, M, K,         \
                 (const E*)Wp, n_tiles, n_stages, nullptr, 0, 0, 1, (E*)U, nullptr);                                  \
  }
  if (M <= 32) MDZ_SWIGLU_CASE(1) else MDZ_SWIGLU_CASE(2)
#undef MDZ_SWIGLU_CASE
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

// The LM head of a verify pass when only the per-row argmax is wanted: no logits are written.  cand receives
// M x gemm_mfma_argmax_cands(...) candidates (one per workgroup and wave); launch_argmax_merge picks each row's best.
bool gemm_mfma_argmax_supported(int dtype, int M, int N, int K) {
  return gemm_mfma_supported(dtype, M, N, K) && N / 128 >= num_cus() / 2;  // enough bands to fill the chip unsplit
}
int gemm_mfma_argmax_cands(int M, int N, int K) { return plan_gemm(M, N, K, 1).grid * 4; }

template <typename E>
static int launch_gemm_mfma_argmax_t(const void* X, const void* Wp, int M, int N, int K, ArgCand* cand, hipStream_t st) {
  const GemmPlan p = plan_gemm(M, N, K, 1);
  const int tag = p.mt == 2 ? PROF_GEMM_W64 : PROF_GEMM_W32;
  const int n_tiles = N / 32, n_stages = K / 128, bands = (n_tiles + 3) / 4;
  MDZ_REQUIRE(p.wpb == 4 && p.nt == 1 && p.ck == 128 && p.whole, MDZ_EUNSUPPORTED, "gemm: no argmax kernel for plan %d,%d,%d",
              p.wpb, p.nt, p.ck);
  MDZ_REQUIRE((int64_t)bands * n_stages * p.grid < (int64_t)1 << 31, MDZ_ESHAPE, "gemm: %d x %d units overflow", bands,
              n_stages);
#define MDZ_ARGMAX_CASE(MT)                                                                                    \
  {                                                                                                             \
    constexpr int lds_bytes = 2 * MT * 32 * (128 * 2 + 16) + 4 * MT * 32 * 33 * 4;                              \
    MDZ_SET_LDS_ONCE((gemm_mfma_kernel<4, 1, MT, 128, E, false, true>), lds_bytes);                             \
    launch_timed(tag, gemm_mfma_kernel<4, 1, MT, 128, E, false, true>, p.grid, 256, lds_bytes, st, (const E*)X, \
                 M, K, (const E*)Wp, n_tiles, n_stages, nullptr, 0, 0, 1, nullptr, cand);                       \
  }
  if (p.mt == 1) MDZ_ARGMAX_CASE(1) else MDZ_ARGMAX_CASE(2)
#undef MDZ_ARGMAX_CASE
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

int launch_gemm_mfma_argmax(int dtype, const void* X, const void* Wp, int M, int N, int K, ArgCand* cand, hipStream_t st) {
  MDZ_WITH_ELEM16(dtype, return launch_gemm_mfma_argmax_t<E>(X, Wp, M, N, K, cand, st));
}

int launch_gemm_mfma_swiglu(int dtype, const void* X, const void* Wp, void* U, int M, int N, int K, hipStream_t st) {
  MDZ_WITH_ELEM16(dtype, return launch_gemm_mfma_swiglu_t<E>(X, Wp, U, M, N, K, st));
}

int launch_gemm_mfma(int dtype, const void* X, const void* Wp, float* P, int M, int N, int K, int64_t ldp,
                     int64_t part_stride, int max_split, Partials* res, hipStream_t st) {
  MDZ_WITH_ELEM16(dtype, return launch_gemm_mfma_t<E>(X, Wp, P, M, N, K, ldp, part_stride, max_split, res, st));
}

}  // namespace mdz
