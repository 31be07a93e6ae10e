// Measurement probe (not part of the library): what does it cost to hand data from one kernel to the next on this
// GPU, and can a device-side flag beat the in-order queue?
//
// A chain  small -> big -> small -> big ...  in which every kernel needs its predecessor's output.  `small` stands
// for the latency-bound kernels of a decoder layer (256 workgroups, every thread adds 9 float4 and writes one);
// `big` stands for a weight-streaming GEMM (256 workgroups, every wave reads a contiguous range with 16-byte loads,
// PRE KiB per wave requested BEFORE it looks at its predecessor's output).
//
//   stream order   one stream; the queue's own kernel boundary is the only synchronisation
//   counter        kernels alternate between two streams (so kernel n+1 becomes resident while kernel n runs and
//                  can request its first weights early) and wait on a device word that the predecessor's last
//                  workgroup publishes: one arrival counter, or per-XCD counters feeding one; with agent-scope
//                  fences around ordinary loads/stores, or without fences and the exchanged data moved by
//                  agent-scope (cache-bypassing) loads and stores
//   flags          as above, but every workgroup publishes a word of its own and the waiter reads all of them
//   write-value    no device-side arrival counting: hipStreamWriteValue32 after each kernel publishes completion
//
// Every wait is bounded (a kernel that gives up sets an error word and carries on), so the probe always terminates.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct alignas(256) Line { uint32_t v; uint32_t pad[63]; };
struct Sync {
  Line progress;           // sequence number of the last kernel that has completed
  Line err;
  Line done[4];            // arrival counters, slot = sequence number % 4
  Line sub[4][8];          // per-XCD arrival counters of the two-level variant
  uint32_t flags[4][256];  // per-workgroup words of the flag variant
  unsigned long long ts[64];
};
enum Variant { STREAM_ORDER = 0, COUNTER_FENCED, TWO_LEVEL_FENCED, FLAGS_FENCED, FLAGS_NOFENCE, TWO_LEVEL_NOFENCE, WRITE_VALUE, N_VARIANTS };
__constant__ int c_variant;
__device__ inline bool nofence() { return c_variant == FLAGS_NOFENCE || c_variant == TWO_LEVEL_NOFENCE; }
__device__ inline bool queue_signals() { return c_variant == STREAM_ORDER || c_variant == WRITE_VALUE; }
__device__ inline bool per_wg_flags() { return c_variant == FLAGS_FENCED || c_variant == FLAGS_NOFENCE; }
__device__ inline bool two_level() { return c_variant == TWO_LEVEL_FENCED || c_variant == TWO_LEVEL_NOFENCE; }

constexpr uint32_t kMaxSpins = 400000;  // bounded wait: ~0.2 s

__device__ inline void wait_for(Sync* s, uint32_t target, int n_prev) {
  if (c_variant == STREAM_ORDER) return;
  if (per_wg_flags()) {
    if (threadIdx.x < 64) {  // wave 0 reads every flag word of the predecessor
      uint32_t spins = 0;
      const uint32_t* f = s->flags[target & 3];
      for (;;) {
        bool ok = true;
        for (int i = threadIdx.x; i < n_prev; i += 64)
          ok &= (int32_t)(__hip_atomic_load(&f[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) >= 0;
        if (__ballot(ok) == ~0ull) break;
        __builtin_amdgcn_s_sleep(8);
        if (++spins > kMaxSpins) { if (threadIdx.x == 0) atomicOr(&s->err.v, 1u); break; }
      }
    }
  } else if (threadIdx.x == 0) {
    uint32_t spins = 0;
    while ((int32_t)(__hip_atomic_load(&s->progress.v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
      __builtin_amdgcn_s_sleep(8);
      if (++spins > kMaxSpins) { atomicOr(&s->err.v, 1u); break; }
    }
  }
  __syncthreads();
  if (!nofence() && c_variant != WRITE_VALUE) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

__device__ inline void signal_done(Sync* s, uint32_t q, int stamp) {
  if (queue_signals()) { if (stamp >= 0 && blockIdx.x == 0 && threadIdx.x == 0) s->ts[stamp] = wall_clock64(); return; }
  if (nofence()) __builtin_amdgcn_s_waitcnt(0);  // this thread's write-through stores are acknowledged
  __syncthreads();
  if (threadIdx.x == 0) {
    if (!nofence()) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    if (per_wg_flags()) {
      __hip_atomic_store(&s->flags[q & 3][blockIdx.x], q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (stamp >= 0 && blockIdx.x == 0) s->ts[stamp] = wall_clock64();
      return;
    }
    bool last;
    if (two_level()) {
      const uint32_t x = blockIdx.x & 7, n_sub = (gridDim.x + 7 - x) / 8;
      last = false;
      if (__hip_atomic_fetch_add(&s->sub[q & 3][x].v, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == n_sub - 1) {
        __hip_atomic_store(&s->sub[q & 3][x].v, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t groups = gridDim.x < 8 ? gridDim.x : 8;
        last = __hip_atomic_fetch_add(&s->done[q & 3].v, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == groups - 1;
      }
    } else {
      last = __hip_atomic_fetch_add(&s->done[q & 3].v, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == gridDim.x - 1;
    }
    if (last) {
      __hip_atomic_store(&s->done[q & 3].v, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (!nofence()) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      __hip_atomic_store(&s->progress.v, q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (stamp >= 0) s->ts[stamp] = wall_clock64();
    }
  }
}

// exchanged data: ordinary accesses, or agent-scope (cache-bypassing) ones in the fence-free variants
__device__ inline f32x4 ld4(const f32x4* p) {
  if (!nofence()) return *p;
  const float* f = reinterpret_cast<const float*>(p);
  f32x4 r;
  r.x = __hip_atomic_load(f + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  r.y = __hip_atomic_load(f + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  r.z = __hip_atomic_load(f + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  r.w = __hip_atomic_load(f + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return r;
}
__device__ inline void st4(f32x4* p, f32x4 v) {
  if (!nofence()) { *p = v; return; }
  float* f = reinterpret_cast<float*>(p);
  __hip_atomic_store(f + 0, v.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(f + 1, v.y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(f + 2, v.z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(f + 3, v.w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int NS>
__global__ void __launch_bounds__(256) small_kernel(const f32x4* __restrict__ in, f32x4* __restrict__ out, Sync* s, uint32_t q, int stamp) {
  wait_for(s, q - 1, 256);
  if (stamp >= 0 && blockIdx.x == 0 && threadIdx.x == 0) s->ts[stamp + 1] = wall_clock64();
  const int i = blockIdx.x * 256 + threadIdx.x;
  f32x4 v[NS];
#pragma unroll
  for (int k = 0; k < NS; ++k) v[k] = ld4(&in[(size_t)k * 65536 + i]);
  f32x4 a = v[0];
#pragma unroll
  for (int k = 1; k < NS; ++k) a += v[k];
  st4(&out[i], a);
  if (stamp >= 0 && blockIdx.x == 0 && threadIdx.x == 0) s->ts[stamp + 2] = wall_clock64();
  signal_done(s, q, stamp);
}

template <int PRE>
__global__ void __launch_bounds__(256) big_kernel(const u32x4* __restrict__ w, size_t units_per_wave, const f32x4* __restrict__ x,
                                                  f32x4* __restrict__ y, Sync* s, uint32_t q, int stamp) {
  const int wave = (blockIdx.x * 256 + threadIdx.x) >> 6, lane = threadIdx.x & 63;
  const u32x4* p = w + (size_t)wave * units_per_wave * 64 + lane;
  u32x4 pre[PRE];
#pragma unroll
  for (int u = 0; u < PRE; ++u) pre[u] = p[(size_t)u * 64];
  if (stamp >= 0 && blockIdx.x == 0 && threadIdx.x == 0) s->ts[stamp] = wall_clock64();
  wait_for(s, q - 1, 256);
  if (stamp >= 0 && blockIdx.x == 0 && threadIdx.x == 0) s->ts[stamp + 1] = wall_clock64();
  f32x4 xv = ld4(&x[(blockIdx.x * 256 + threadIdx.x) & 65535]);  // the predecessor's output
  u32x4 acc = {0, 0, 0, 0};
#pragma unroll
  for (int u = 0; u < PRE; ++u) { acc.x ^= pre[u].x; acc.y ^= pre[u].y; acc.z ^= pre[u].z; acc.w ^= pre[u].w; }
  for (size_t i = PRE; i + 12 <= units_per_wave; i += 12) {
    u32x4 v[12];
#pragma unroll
    for (int u = 0; u < 12; ++u) v[u] = p[(i + u) * 64];
#pragma unroll
    for (int u = 0; u < 12; ++u) { acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w; }
  }
  f32x4 r = xv;
  r.x += __uint_as_float((acc.x ^ acc.y ^ acc.z ^ acc.w) & 0x3FFFFFu);
  if (lane < 16) st4(&y[((size_t)wave * 16 + lane) & 65535], r);
  signal_done(s, q, stamp >= 0 ? stamp + 2 : -1);
}

static uint32_t g_q = 0;
static int g_variant = 0;

template <int PRE>
static void run(const char* name, bool two_streams, const u32x4* pool, size_t pool_bytes, size_t big_bytes, f32x4* slots, f32x4* xa,
                Sync* sync, hipStream_t* st, int pairs) {
  size_t units_per_wave = big_bytes / 1024 / 1024;  // 1024 waves, 1 KiB units
  units_per_wave = PRE + (units_per_wave - PRE) / 12 * 12;
  const size_t nrot = pool_bytes / (units_per_wave * 1024 * 1024);
  hipEvent_t e0, e1, ej;
  CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1)); CK(hipEventCreateWithFlags(&ej, hipEventDisableTiming));
  uint32_t& q = g_q;
  double best = 1e30;
  static Sync h;
  for (int rep = 0; rep < 3; ++rep) {
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0, st[0]));
    if (two_streams) { CK(hipEventRecord(ej, st[0])); CK(hipStreamWaitEvent(st[1], ej, 0)); }
    for (int i = 0; i < pairs; ++i) {
      const u32x4* wp = pool + (size_t)((i + rep * pairs) % nrot) * units_per_wave * 64 * 1024;  // never the same weights twice in a row
      const int stamp = (rep == 2 && i == pairs / 2) ? 0 : -1;
      ++q;
      small_kernel<9><<<256, 256, 0, two_streams ? st[q & 1] : st[0]>>>(slots, xa, sync, q, stamp >= 0 ? 8 : -1);
      if (g_variant == WRITE_VALUE) CK(hipStreamWriteValue32(two_streams ? st[q & 1] : st[0], &sync->progress.v, q, 0));
      ++q;
      big_kernel<PRE><<<256, 256, 0, two_streams ? st[q & 1] : st[0]>>>(wp, units_per_wave, xa, slots, sync, q, stamp);
      if (g_variant == WRITE_VALUE) CK(hipStreamWriteValue32(two_streams ? st[q & 1] : st[0], &sync->progress.v, q, 0));
    }
    if (two_streams) { CK(hipEventRecord(ej, st[1])); CK(hipStreamWaitEvent(st[0], ej, 0)); }
    CK(hipEventRecord(e1, st[0]));
    CK(hipDeviceSynchronize());
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    CK(hipMemcpy(&h, sync, sizeof(Sync), hipMemcpyDeviceToHost));
    if (h.err.v) { printf("%s: a bounded wait gave up; stopping\n", name); exit(3); }
    if (ms * 1e3 / pairs < best) best = ms * 1e3 / pairs;
  }
  printf("| %-34s | %-11s | %2d | %6.1f | %7.2f | %5.2f | %5.2f | %5.2f | %5.2f |\n", name, two_streams ? "two streams" : "one stream", PRE,
         units_per_wave * 1024.0 * 1024 / 1e6, best, (double)((long long)h.ts[10] - (long long)h.ts[9]) / 100.0,
         (double)((long long)h.ts[8] - (long long)h.ts[10]) / 100.0, (double)((long long)h.ts[1] - (long long)h.ts[8]) / 100.0,
         (double)((long long)h.ts[2] - (long long)h.ts[1]) / 100.0);
}

int main() {
  const size_t pool_bytes = (size_t)6 << 30;
  u32x4* pool; CK(hipMalloc(&pool, pool_bytes)); CK(hipMemset(pool, 1, pool_bytes));
  f32x4 *slots, *xa; CK(hipMalloc(&slots, 9 * 65536 * 16)); CK(hipMalloc(&xa, 65536 * 16));
  CK(hipMemset(slots, 0, 9 * 65536 * 16)); CK(hipMemset(xa, 0, 65536 * 16));
  Sync* sync; CK(hipMalloc(&sync, sizeof(Sync)));
  hipStream_t st[2];
  CK(hipStreamCreateWithFlags(&st[0], hipStreamNonBlocking)); CK(hipStreamCreateWithFlags(&st[1], hipStreamNonBlocking));
  const int pairs = 32;
  const char* vn[N_VARIANTS] = {"stream order (kernel boundary)", "one counter, fences", "per-XCD counters, fences", "per-workgroup flags, fences",
                                "per-workgroup flags, no fences", "per-XCD counters, no fences", "hipStreamWriteValue32"};
  printf("us: best of 3 chains of %d (small, big) pairs, per pair; small/big columns: one pair in mid-chain, wall clock of workgroup 0\n", pairs);
  printf("| handoff | streams | KiB per wave requested before the wait | big MB | us per pair | small: start -> loaded | small: loaded -> signalled | small signalled -> big starts computing | big: start -> done |\n|---|---|---|---|---|---|---|---|---|\n");
  for (size_t mb : {34, 100, 180}) {
    const size_t bytes = mb << 20;
    for (int v = 0; v < N_VARIANTS; ++v) {
      CK(hipMemcpyToSymbol(HIP_SYMBOL(c_variant), &v, sizeof(int)));
      g_variant = v;
      {  // everything up to the current sequence number counts as completed
        static Sync h0;
        memset(&h0, 0, sizeof h0);
        h0.progress.v = g_q;
        for (int a = 0; a < 4; ++a) for (int b = 0; b < 256; ++b) h0.flags[a][b] = g_q;
        CK(hipMemcpy(sync, &h0, sizeof(Sync), hipMemcpyHostToDevice));
      }
      CK(hipDeviceSynchronize());
      run<12>(vn[v], false, pool, pool_bytes, bytes, slots, xa, sync, st, pairs);
      if (v == STREAM_ORDER) continue;
      run<12>(vn[v], true, pool, pool_bytes, bytes, slots, xa, sync, st, pairs);
      run<24>(vn[v], true, pool, pool_bytes, bytes, slots, xa, sync, st, pairs);
    }
  }
  return 0;
}
