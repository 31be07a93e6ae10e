// Measurement probe (not part of the library): how fast can a many-row GEMM (M = 1024, the 16-sequence batch) run
// on this GPU with the largest output tile the register file allows?  One workgroup per 256 x 256 tile, four waves
// of 128 x 128 (all 256 accumulator registers), both operands brought into a four-stage LDS ring by
// global_load_lds (16 B per lane; X gathered from row-major as 16 rows x 64 B per instruction, W straight from the
// packed layout), XCD-aware tile order.  Three runs per shape: the loop without the loads (LDS reads + MFMAs), the
// loads alone, and both.  Timing only: inputs are zero, the sums are written once.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("err %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} }while(0)
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 v8 __attribute__((ext_vector_type(8)));
#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))
__device__ inline f32x16 mfma(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8, a), __builtin_bit_cast(v8, b), c, 0, 0, 0);
}
constexpr int NS = 4;                 // ring stages
constexpr int KC = 32;                // features per stage (2 k-steps)
constexpr int STAGE = 32768;          // bytes per stage: A 16 KiB + B 16 KiB

// X row-major [M][K] bf16; Wp packed [band][stage256][tile in band][16 k-steps][64 lanes][16 B]
template <int MODE>  // 0: full, 1: no DMA (LDS reads + MFMA only), 2: DMA only (no LDS reads / MFMA)
__global__ void __launch_bounds__(256) xl_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ Wp, float* __restrict__ out,
                                                 int K, int nb_m, int nb_n) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // workgroups are dealt round-robin to the 8 XCDs: the row blocks that share a column block stay on one XCD
  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  const int bn = (seq / nb_m) * 8 + xcd, bm = seq % nb_m;
  if (bn >= nb_n) return;
  const int n_stages = K / KC, nst256 = K / 256;
  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  // DMA sources of this wave: 4 A blocks (16 rows x 64 B each) and 4 W units (1 KiB each) per stage
  const uint8_t* a_src[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int blk = wave * 4 + q;  // 16-row block of the 256-row tile
    a_src[q] = reinterpret_cast<const uint8_t*>(X) + ((size_t)(bm * 256 + blk * 16 + (lane & 15)) * K) * 2 + (lane >> 4) * 16;
  }
  auto issue = [&](int s, int buf) {
    if (MODE == 1) return;
    uint8_t* base = lds + buf * STAGE;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      __builtin_amdgcn_global_load_lds(GLB_PTR(a_src[q] + (size_t)s * KC * 2), LDS_PTR(base + (wave * 4 + q) * 1024), 16, 0, 0);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int u = wave * 4 + q;           // unit = tile * 2 + ks within the stage
      const int tile = bn * 8 + (u >> 1), ksg = s * 2 + (u & 1);
      const size_t unit = (((size_t)(tile >> 2) * nst256 + (ksg >> 4)) * 4 + (tile & 3)) * 16 + (ksg & 15);
      __builtin_amdgcn_global_load_lds(GLB_PTR(reinterpret_cast<const uint8_t*>(Wp) + unit * 1024 + lane * 16),
                                       LDS_PTR(base + 16384 + u * 1024), 16, 0, 0);
    }
  };
  const int wm = wave >> 1, wn = wave & 1;
  // operand read offsets inside a stage
  const int row = lane & 31, half = lane >> 5;
  const int a_off = (wm * 8 + (row >> 4)) * 1024 + (row & 15) * 16;   // + t*2048 + (2*ks + half)*256
  const int b_off = 16384 + (wn * 8) * 1024 + lane * 16;              // + (j*2 + ks)*1024
  for (int s = 0; s < NS - 1; ++s) issue(s, s);
  for (int s = 0; s < n_stages; ++s) {
    // stage s has landed once at most the two younger stages' loads (8 per stage per wave) are outstanding
    if (MODE != 1) {
      if (s + 2 < n_stages) __builtin_amdgcn_s_waitcnt(0x4F70);        // vmcnt(16)
      else if (s + 1 < n_stages) __builtin_amdgcn_s_waitcnt(0x0F78);   // vmcnt(8)
      else __builtin_amdgcn_s_waitcnt(0x0F70);                         // vmcnt(0)
    }
    __syncthreads();
    if (s + NS - 1 < n_stages) issue(s + NS - 1, (s + NS - 1) % NS);
    if (MODE == 2) continue;
    const uint8_t* base = lds + (s % NS) * STAGE;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      u32x4 a[4], b[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) a[t] = *reinterpret_cast<const u32x4*>(base + a_off + t * 2048 + (2 * ks + half) * 256);
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = *reinterpret_cast<const u32x4*>(base + b_off + (j * 2 + ks) * 1024);
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[t][j] = mfma(a[t], b[j], acc[t][j]);
    }
  }
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) t += acc[i][j][r];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = t;
}

template <int MODE>
static void run(const char* name, const uint16_t* X, const uint16_t* W, float* out, int M, int N, int K) {
  const int nb_m = M / 256, nb_n = N / 256;
  CK(hipFuncSetAttribute(reinterpret_cast<const void*>(xl_kernel<MODE>), hipFuncAttributeMaxDynamicSharedMemorySize, NS * STAGE));
  hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
  for (int r = 0; r < 3; ++r) xl_kernel<MODE><<<(nb_n + 7) / 8 * 8 * nb_m, 256, NS * STAGE>>>(X, W, out, K, nb_m, nb_n);
  CK(hipEventRecord(a));
  const int reps = 20;
  for (int r = 0; r < reps; ++r) xl_kernel<MODE><<<(nb_n + 7) / 8 * 8 * nb_m, 256, NS * STAGE>>>(X, W, out, K, nb_m, nb_n);
  CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
  float ms; CK(hipEventElapsedTime(&ms, a, b));
  double fl = 2.0 * M * N * K * reps;
  printf("| %-24s | %d x %d x %d | %d | %8.1f | %7.1f | %5.1f |\n", name, M, N, K, nb_m * nb_n, ms * 1e3 / reps, fl / (ms * 1e-3) / 1e12,
         MODE == 1 ? 0.0 : (double)nb_m * nb_n * (K / KC) * STAGE / (ms * 1e-3 / reps) / 1e9 / 256);
}

int main() {
  const int M = 1024, K = 4096;
  uint16_t *X, *W; float* out;
  CK(hipMalloc(&X, (size_t)M * 11008 * 2)); CK(hipMemset(X, 0, (size_t)M * 11008 * 2));
  CK(hipMalloc(&W, (size_t)131072 * 4096 * 2)); CK(hipMemset(W, 0, (size_t)131072 * 4096 * 2));
  CK(hipMalloc(&out, 1 << 24));
  printf("| run | M x N x K | workgroups | us per launch | TFLOP/s (equivalent) | GB/s fetched per CU |\n|---|---|---|---|---|---|\n");
  for (int N : {16384, 12288, 22016 / 256 * 256, 128000}) {
    run<1>("LDS reads + MFMA only", X, W, out, M, N, K);
    run<2>("loads only", X, W, out, M, N, K);
    run<0>("loads + LDS reads + MFMA", X, W, out, M, N, K);
  }
  return 0;
}
