// Measurement probe (not part of the library): where the time of one launch of the two hot kernels goes, workgroup
// by workgroup.
//
// The library's own sources of the weight-streaming GEMM and of the tree attention are compiled here with
// -DMDZ_STAMPS, which turns the MDZ_STAMP(i) marks in them into wall-clock stamps (thread 0 of every workgroup, 100 MHz
// counter).  The probe launches the kernels through the library's own launch functions at the decoder's shapes and
// prints, per stamp, the minimum / mean / maximum over the workgroups, measured from the first workgroup's entry:
//
//   GEMM       0 entry   1 first X stage in LDS, three half stages of W requested   2 first products done
//              3 last unit multiplied and written (the workgroup's stream has ended)
//   attention  0 entry   1 prologue issued (queries staged; tree rows of K / V produced, by the last key-split)
//              2 after the barrier that follows it   3 key blocks done   4 waves merged, partial result written
//
// Weights rotate through 6 GB so that no launch finds its matrix in the memory-side cache; the operands are zeros
// (the kernels' timing does not depend on values), the outputs are not looked at.
//
// Build: hipcc --offload-arch=gfx950 -O3 -std=c++17 -DMDZ_STAMPS -I include -I paper_2603_03383_amd/csrc
//        -Xclang -target-feature -Xclang -packed-fp32-ops paper_2603_03383_amd/probes/stamps_probe.hip
// (paper_2603_03383_amd/build.py: build_probes).
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>

#include "../csrc/gemm_mfma.hip"
#include "../csrc/attn_mfma.hip"

namespace mdz {
// what the two sources expect from the rest of the library
void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vprintf(fmt, ap);
  va_end(ap);
  printf("\n");
}
bool prof_enabled() { return false; }
void prof_record(int, hipStream_t, bool) {}
bool prof_kernel_events(int, hipEvent_t*, hipEvent_t*) { return false; }
int num_cus() {
  hipDeviceProp_t p;
  return hipGetDeviceProperties(&p, 0) == hipSuccess ? p.multiProcessorCount : 256;
}
}  // namespace mdz

#define CK(x)                                                                    \
  do {                                                                           \
    hipError_t e_ = (x);                                                         \
    if (e_ != hipSuccess) {                                                      \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);     \
      exit(1);                                                                   \
    }                                                                            \
  } while (0)

using namespace mdz;

constexpr int kMaxWg = 4096;
static unsigned long long g_host[8 * kMaxWg];

static void clear_stamps() {
  void* p;
  CK(hipGetSymbolAddress(&p, HIP_SYMBOL(mdz::mdz_stamps)));
  CK(hipMemset(p, 0, sizeof(g_host)));
}
static void fetch_stamps() { CK(hipMemcpyFromSymbol(g_host, HIP_SYMBOL(mdz::mdz_stamps), sizeof(g_host))); }

// min / mean / max of stamp k over the workgroups selected by pick(i), in us after the earliest entry
template <typename Pick>
static void stats(int n_wg, int k, Pick pick, double t0, double* mn, double* av, double* mx) {
  *mn = 1e30, *mx = 0, *av = 0;
  int n = 0;
  for (int i = 0; i < n_wg; ++i) {
    if (!g_host[8 * i] || !g_host[8 * i + k] || !pick(i)) continue;
    const double t = ((double)g_host[8 * i + k] - t0) / 100.0;
    *mn = t < *mn ? t : *mn, *mx = t > *mx ? t : *mx, *av += t, ++n;
  }
  *av = n ? *av / n : 0;
}
static double first_entry(int n_wg, int* live) {
  double t0 = 1e30;
  *live = 0;
  for (int i = 0; i < n_wg; ++i)
    if (g_host[8 * i]) {
      ++*live;
      t0 = (double)g_host[8 * i] < t0 ? (double)g_host[8 * i] : t0;
    }
  return t0;
}

int main() {
  const int M = 64;
  // ---- GEMM ---------------------------------------------------------------------------------------------
  struct Shape {
    const char* name;
    int N, K, max_split;
  } shapes[] = {{"QKV", 12288, 4096, 12}, {"O", 4096, 4096, 12}, {"gate/up (sums)", 22016, 4096, 12}, {"down", 4096, 11008, 12},
                {"LM head", 128000, 4096, 1}};
  const size_t wbytes = (size_t)6 << 30;
  bf16_t *W, *X;
  float* P;
  CK(hipMalloc(&W, wbytes));
  CK(hipMemset(W, 0, wbytes));
  CK(hipMalloc(&X, (size_t)M * 11008 * 2));
  CK(hipMemset(X, 0, (size_t)M * 11008 * 2));
  CK(hipMalloc(&P, (size_t)12 * M * 22016 * 4 > (size_t)M * 128000 * 4 ? (size_t)12 * M * 22016 * 4 : (size_t)M * 128000 * 4));
  hipEvent_t ea, eb;
  CK(hipEventCreate(&ea));
  CK(hipEventCreate(&eb));
  printf("GEMM, M = 64 rows (us after the first workgroup's entry; min / mean / max over the workgroups; last of 8 launches)\n");
  printf("| shape | MB | workgroups | X staged | first products | stream ends | launch by events |\n|---|---|---|---|---|---|---|\n");
  for (auto& s : shapes) {
    const size_t mat = (size_t)s.N * s.K * 2;
    const int nrot = (int)(wbytes / mat) > 16 ? 16 : (int)(wbytes / mat);
    float ms = 0;
    for (int r = 0; r < 8; ++r) {
      clear_stamps();
      Partials res;
      CK(hipEventRecord(ea));
      const int rc = launch_gemm_mfma(MDZ_BF16, X, (const char*)W + (size_t)(r % nrot) * mat, P, M, s.N, s.K, s.N, (int64_t)M * s.N,
                                      s.max_split, &res, 0);
      CK(hipEventRecord(eb));
      CK(hipEventSynchronize(eb));
      if (rc) return 1;
      CK(hipEventElapsedTime(&ms, ea, eb));
    }
    fetch_stamps();
    int live;
    const double t0 = first_entry(kMaxWg, &live);
    double a[4][3];
    for (int k = 1; k < 4; ++k) stats(kMaxWg, k, [](int) { return true; }, t0, &a[k][0], &a[k][1], &a[k][2]);
    printf("| %s | %.1f | %d | %.1f / %.1f / %.1f | %.1f / %.1f / %.1f | %.1f / %.1f / %.1f | %.1f |\n", s.name, mat / 1e6, live, a[1][0],
           a[1][1], a[1][2], a[2][0], a[2][1], a[2][2], a[3][0], a[3][1], a[3][2], ms * 1e3);
  }
  CK(hipFree(W));
  CK(hipFree(P));

  // ---- tree attention from the QKV partial sums (32 heads, 64-node tree, one sequence) ---------------------------
  const int H = 32, D = 4096, T = 64, prefixes[] = {128, 1024, 2048, 4096, 8192, 16384};
  printf("\ntree attention, 32 heads, one sequence (us after the first workgroup's entry; mean over the workgroups of a kind; last of 8 launches)\n");
  printf("| prefix | key-splits x workgroups per split | kind of split | prologue issued | after its barrier | key blocks done | end (min / mean / max) | both kernels by events |\n|---|---|---|---|---|---|---|---|\n");
  for (int S : prefixes) {
    KvGeom g{1, 1, H, 128, S + T, 1, 1, 0};
    const size_t kvb = (size_t)kv_head_base(g, 1, 0, 0) * 2;
    bf16_t *kc, *vc, *att;
    float *part, *cs;
    int32_t* seq;
    void* scratch;
    CK(hipMalloc(&kc, kvb));
    CK(hipMalloc(&vc, kvb));
    CK(hipMemset(kc, 0, kvb));
    CK(hipMemset(vc, 0, kvb));
    const size_t pb = (size_t)2 * T * 3 * D * 4;
    CK(hipMalloc(&part, pb));
    CK(hipMemset(part, 0, pb));
    CK(hipMalloc(&cs, (size_t)T * 64 * 2 * 4));
    CK(hipMemset(cs, 0, (size_t)T * 64 * 2 * 4));
    CK(hipMalloc(&seq, 4));
    CK(hipMemcpy(seq, &S, 4, hipMemcpyHostToDevice));
    CK(hipMalloc(&att, (size_t)T * D * 2));
    const int64_t sb = attn_mfma_scratch_bytes(1, H, S);
    CK(hipMalloc(&scratch, sb > 0 ? sb : 256));
    // the QKV launch's own plan: 96 bands x 32 stages on 192 workgroups, two partial-sum slots per band
    Partials qkv{part, 2, (int64_t)T * 3 * D, 3 * D, 128, 32, 96 * 32, 192};
    float ms = 0;
    for (int r = 0; r < 8; ++r) {
      clear_stamps();
      CK(hipEventRecord(ea));
      const int rc = launch_attention_mfma(MDZ_BF16, MDZ_TREE_64, nullptr, &qkv, cs, g, kc, vc, 0, seq, 1, S, att, scratch, sb, 0);
      CK(hipEventRecord(eb));
      CK(hipEventSynchronize(eb));
      if (rc) return 1;
      CK(hipEventElapsedTime(&ms, ea, eb));
    }
    fetch_stamps();
    int live;
    const double t0 = first_entry(kMaxWg, &live);
    const int per_pair = live / H;                       // workgroups per head: splits x (1 or 2 query halves)
    const int halves = S < 3584 ? 2 : 1;                 // (the launcher's own rule)
    const int splits = per_pair / halves;
    for (int kind = 0; kind < (splits > 1 ? 2 : 1); ++kind) {
      // grid (splits, heads, halves): linear index = split + splits * (head + heads * half); the last split is the tree's
      auto pick = [&](int i) { return splits == 1 || ((i % splits == splits - 1) == (kind == 1)); };
      double a[5][3];
      for (int k = 1; k < 5; ++k) stats(kMaxWg, k, pick, t0, &a[k][0], &a[k][1], &a[k][2]);
      printf("| %d | %d x %d | %s | %.1f | %.1f | %.1f | %.1f / %.1f / %.1f | %.1f |\n", S, splits, H * halves,
             splits == 1 ? "single" : kind ? "tree blocks" : "prefix blocks", a[1][1], a[2][1], a[3][1], a[4][0], a[4][1], a[4][2],
             ms * 1e3);
    }
    CK(hipFree(kc));
    CK(hipFree(vc));
    CK(hipFree(part));
    CK(hipFree(cs));
    CK(hipFree(seq));
    CK(hipFree(att));
    CK(hipFree(scratch));
  }
  return 0;
}
