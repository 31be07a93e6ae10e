// Optional per-kernel timing with HIP events recorded on the caller's stream around each launch.
// Off by default (a single predictable branch per launch).  medusa_profile_begin creates the event
// pool, so no hot-path call ever creates an event.  Process-global: meant for a benchmark's own thread.
#pragma once
#include <hip/hip_runtime.h>

namespace mdz {

enum ProfTag {
  PROF_GEMM = 0,     // portable GEMM
  PROF_GEMM_W64,     // gemm_mfma_kernel<4,1,2,*>: 128-column bands, 64 rows (every layer GEMM and the LM head)
  PROF_GEMM_N64,     // gemm_mfma_kernel<2,1,2,*>: 64-column bands, 64 rows (development plans only)
  PROF_GEMM_W32,     // gemm_mfma_kernel<4,1,1,*>: <= 32 rows (Medusa heads, autoregressive step)
  PROF_GEMM_N32,     // gemm_mfma_kernel<2,1,1,*>: <= 32 rows (development plans only)
  PROF_GEMM_LARGE,   // gemm_large_kernel: >= 128 rows (several sequences)
  PROF_ATTN,         // tree-masked attention (+ its combine pass)
  PROF_NORM,         // RMSNorm
  PROF_ROPE,         // RoPE table, RoPE + KV write
  PROF_SWIGLU,
  PROF_EMBED,
  PROF_SELECT,       // argmax / top-k / candidate gather
  PROF_ACCEPT,
  PROF_COMPACT,
  PROF_MISC,
  PROF_NUM_TAGS
};

const char* prof_tag_name(int tag);
bool prof_enabled();
void prof_record(int tag, hipStream_t st, bool start);

struct ProfScope {
  int tag;
  hipStream_t st;
  bool on;
  ProfScope(int tag_, hipStream_t st_) : tag(tag_), st(st_), on(prof_enabled()) {
    if (on) prof_record(tag, st, true);
  }
  ~ProfScope() {
    if (on) prof_record(tag, st, false);
  }
};

}  // namespace mdz
