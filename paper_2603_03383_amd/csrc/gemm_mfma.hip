// Weight-streaming skinny GEMM for bf16 storage on gfx950: P[s][m][n] = sum over K-slice s of
// X[m][k] * W[n][k], M <= 64 rows (the T tree nodes of one sequence, or up to 32 batch rows for the
// Medusa heads).  This is the kernel that moves >95 % of a verify step's bytes (the decoder weights),
// so it is built around the HBM stream:
//   * W arrives in the packed order (common.h): every wave-level load is one contiguous 1 KiB block
//     (16 B per lane) that already is the B operand of v_mfma_f32_32x32x16_bf16 — no LDS, no shuffles.
//   * A wave owns NT tiles of 32 output columns and keeps one whole K-chunk (8 k-steps) of W in flight
//     in registers while it multiplies the previous chunk (software double buffering).
//   * X (<= 64 x K bf16, L2 resident) is staged per K-chunk through LDS, shared by the WPB waves of a
//     workgroup, rows padded by 16 B so the 16 B-per-lane operand reads are bank-conflict free.
//   * Split-K over blockIdx.y gives >= 256 workgroups for every matrix of the decoder; partial sums go
//     to a workspace and are added in a fixed order by the consumer kernel, so results are
//     deterministic (no floating-point atomics).
#include "kernels.h"

namespace mdz {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kChunkK = 128;                  // input features per pipeline stage
constexpr int kChunkSteps = kChunkK / 16;     // MFMA k-steps per stage
constexpr int kLdsRow = kChunkK * 2 + 16;     // bytes per staged X row (16 B pad)

template <int WPB, int NT, int MT>
__global__ void __launch_bounds__(WPB * 64)
    gemm_mfma_kernel(const bf16_t* __restrict__ X, int M, int K, const bf16_t* __restrict__ Wp, int n_tiles,
                     int n_chunks, float* __restrict__ P, int64_t ldp, int64_t part_stride) {
  constexpr int ROWS = MT * 32;
  constexpr int XL = ROWS * 16 / (WPB * 64);  // 16-byte X loads per thread per chunk
  __shared__ __attribute__((aligned(16))) uint8_t lds[2][ROWS * kLdsRow];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int S_k = gridDim.y, s = blockIdx.y;
  const int c_begin = (int)((int64_t)s * n_chunks / S_k), c_end = (int)((int64_t)(s + 1) * n_chunks / S_k);
  const int tile0 = (blockIdx.x * WPB + wave) * NT;
  const int64_t tile_elems = (int64_t)(K >> 4) * 512;  // bf16 elements of one packed 32-row tile

  const u32x4* wp[NT];
  bool live[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    live[nt] = tile0 + nt < n_tiles;
    int t = live[nt] ? tile0 + nt : 0;
    wp[nt] = reinterpret_cast<const u32x4*>(Wp + t * tile_elems) + lane;  // + (chunk*8 + ks) * 64
  }

  f32x16 acc[NT][MT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[nt][mt][r] = 0.f;

  u32x4 xr[XL];
  u32x4 wb[2][NT][kChunkSteps];

  auto load_x = [&](int c) {
#pragma unroll
    for (int i = 0; i < XL; ++i) {
      int idx = threadIdx.x + i * (WPB * 64);
      int row = idx >> 4, col = idx & 15;
      // branch-free and wait-free: tile rows beyond M re-read row M-1.  An output row depends only on its own
      // X row, and rows >= M are never stored, so their contents do not matter.
      int rr = row < M ? row : M - 1;
      xr[i] = *reinterpret_cast<const u32x4*>(X + (int64_t)rr * K + (int64_t)c * kChunkK + col * 8);
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < XL; ++i) {
      int idx = threadIdx.x + i * (WPB * 64);
      int row = idx >> 4, col = idx & 15;
      *reinterpret_cast<u32x4*>(&lds[buf][row * kLdsRow + col * 16]) = xr[i];
    }
  };
  auto load_w = [&](int c, u32x4 (&dst)[NT][kChunkSteps]) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int ks = 0; ks < kChunkSteps; ++ks)
        dst[nt][ks] = wp[nt][((int64_t)c * kChunkSteps + ks) * 64];  // dead tiles alias tile 0; never stored
  };
  auto compute = [&](int buf, const u32x4 (&w)[NT][kChunkSteps]) {
    const uint8_t* base = &lds[buf][(lane & 31) * kLdsRow + (lane >> 5) * 16];
#pragma unroll
    for (int ks = 0; ks < kChunkSteps; ++ks) {
      bf16x8 a[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        a[mt] = *reinterpret_cast<const bf16x8*>(base + mt * 32 * kLdsRow + ks * 32);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        bf16x8 b = __builtin_bit_cast(bf16x8, w[nt][ks]);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mt], b, acc[nt][mt], 0, 0, 0);
      }
    }
  };

  if (c_begin < c_end) {
    load_x(c_begin);
    load_w(c_begin, wb[0]);
    store_x(0);
    __syncthreads();
    int c = c_begin;
    // steady state: two chunks per trip, no branches inside, so the prefetch of chunk c+1 stays in flight
    // while chunk c is multiplied
    // sched_barrier: the loads must be ISSUED before the MFMAs of the previous chunk, not sunk below them
    for (; c + 2 < c_end; c += 2) {
      load_x(c + 1);
      load_w(c + 1, wb[1]);
      __builtin_amdgcn_sched_barrier(0);
      compute(0, wb[0]);
      __builtin_amdgcn_sched_barrier(0);
      store_x(1);
      __syncthreads();
      load_x(c + 2);
      load_w(c + 2, wb[0]);
      __builtin_amdgcn_sched_barrier(0);
      compute(1, wb[1]);
      __builtin_amdgcn_sched_barrier(0);
      store_x(0);
      __syncthreads();
    }
    if (c + 1 < c_end) {  // two chunks left
      load_x(c + 1);
      load_w(c + 1, wb[1]);
      __builtin_amdgcn_sched_barrier(0);
      compute(0, wb[0]);
      __builtin_amdgcn_sched_barrier(0);
      store_x(1);
      __syncthreads();
      compute(1, wb[1]);
    } else {  // one chunk left
      compute(0, wb[0]);
    }
  }

  // D layout of the 32x32 MFMA: lane holds column (lane % 32); register r is row 8*(r/4) + 4*(lane/32) + r%4.
  float* out = P + (int64_t)s * part_stride;
  const int col = lane & 31, rbase = (lane >> 5) * 4;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    if (!live[nt]) continue;
    const int n = (tile0 + nt) * 32 + col;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int m = mt * 32 + 8 * (r >> 2) + rbase + (r & 3);
        if (m < M) out[(int64_t)m * ldp + n] = acc[nt][mt][r];
      }
  }
}

struct GemmPlan {
  int wpb, nt, mt, split;
};

static GemmPlan plan_gemm(int M, int n_tiles, int n_chunks, int max_split) {
  GemmPlan p;
  p.mt = M <= 32 ? 1 : 2;
  if (n_tiles >= 2048) {
    p.wpb = 4;
    p.nt = 2;
  } else if (n_tiles > 256) {
    p.wpb = 4;
    p.nt = 1;
  } else {
    p.wpb = 2;
    p.nt = 1;
  }
  static const char* env = getenv("MDZ_GEMM_PLAN");  // development knob: "wpb,nt,split" (split 0 = auto)
  int force_split = 0;
  if (env) {
    int a = 0, b = 0, c = 0;
    if (sscanf(env, "%d,%d,%d", &a, &b, &c) == 3 && (a == 2 || a == 4) && (b == 1 || b == 2)) {
      p.wpb = a;
      p.nt = b;
      force_split = c;
    }
  }
  int groups = (n_tiles + p.wpb * p.nt - 1) / (p.wpb * p.nt);
  int split = force_split > 0 ? force_split : (256 + groups - 1) / groups;
  if (split > max_split) split = max_split;
  if (split > n_chunks) split = n_chunks;
  if (split < 1) split = 1;
  p.split = split;
  return p;
}

bool gemm_mfma_supported(int dtype, int M, int N, int K) {
  return dtype == MDZ_BF16 && M >= 1 && M <= 64 && N % 32 == 0 && K % kChunkK == 0 && K >= kChunkK;
}

// Writes n_part partial sums (each [M][N] fp32 with leading dimension ldp, part_stride elements apart).
int launch_gemm_mfma(const void* X, const void* Wp, float* P, int M, int N, int K, int64_t ldp, int64_t part_stride,
                     int max_split, int* n_part, hipStream_t st) {
  ProfScope prof_(PROF_GEMM, st);
  const int n_tiles = N / 32, n_chunks = K / kChunkK;
  GemmPlan p = plan_gemm(M, n_tiles, n_chunks, max_split);
  *n_part = p.split;
  dim3 grid((n_tiles + p.wpb * p.nt - 1) / (p.wpb * p.nt), p.split);
  const bf16_t* x = (const bf16_t*)X;
  const bf16_t* w = (const bf16_t*)Wp;
#define MDZ_GEMM_CASE(WPB, NT, MT)                                                                        \
  if (p.wpb == WPB && p.nt == NT && p.mt == MT) {                                                         \
    gemm_mfma_kernel<WPB, NT, MT><<<grid, WPB * 64, 0, st>>>(x, M, K, w, n_tiles, n_chunks, P, ldp, part_stride); \
  } else
  MDZ_GEMM_CASE(4, 2, 2)
  MDZ_GEMM_CASE(4, 1, 2)
  MDZ_GEMM_CASE(2, 1, 2)
  MDZ_GEMM_CASE(2, 2, 2)
  MDZ_GEMM_CASE(4, 2, 1)
  MDZ_GEMM_CASE(4, 1, 1)
  MDZ_GEMM_CASE(2, 1, 1)
  MDZ_GEMM_CASE(2, 2, 1) { MDZ_FAIL(MDZ_EUNSUPPORTED, "gemm: no kernel for plan %d,%d,%d", p.wpb, p.nt, p.mt); }
#undef MDZ_GEMM_CASE
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

}  // namespace mdz
