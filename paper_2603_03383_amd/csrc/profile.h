// Optional per-kernel timing.  Two forms: ProfScope records HIP events on the caller's stream around whatever is
// launched inside the scope (the event packets between kernels add 1-2 us per scope), and launch_timed launches
// ONE kernel whose own start and end timestamps the dispatch records into an event pair (hipExtLaunchKernelGGL: no
// packets between kernels, the duration a kernel trace shows).  Off by default (a single predictable branch per
// launch).  medusa_profile_begin creates the event pool, so no hot-path call ever creates an event.
// Process-global: meant for a benchmark's own thread.
#pragma once
#include <hip/hip_ext.h>
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
// hands out the next event pair of the pool for one kernel's own timestamps; false if the pool is full
bool prof_kernel_events(int tag, hipEvent_t* start, hipEvent_t* stop);

// kernel<<<grid, block, lds, st>>>(args...), timed by the dispatch itself while the profile is recording
template <typename... KArgs, typename... Args>
inline void launch_timed(int tag, void (*kernel)(KArgs...), dim3 grid, dim3 block, unsigned lds, hipStream_t st,
                         Args... args) {
  hipEvent_t e0, e1;
  if (prof_enabled() && prof_kernel_events(tag, &e0, &e1))
    hipExtLaunchKernelGGL(kernel, grid, block, lds, st, e0, e1, 0, static_cast<KArgs>(args)...);
  else
    hipLaunchKernelGGL(kernel, grid, block, lds, st, static_cast<KArgs>(args)...);
}

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
