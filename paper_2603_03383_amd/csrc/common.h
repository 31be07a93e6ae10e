// Shared host/device helpers of libmedusa_hip: status handling, element types, the packed weight
// layout and the KV cache layout.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/medusa.h"
#include "tree_tables.h"

namespace mdz {

// ---- error reporting ---------------------------------------------------------------------------
void set_error(const char* fmt, ...);
#define MDZ_FAIL(code, ...)      \
  do {                           \
    ::mdz::set_error(__VA_ARGS__); \
    return (code);               \
  } while (0)
#define MDZ_REQUIRE(cond, code, ...) \
  do {                               \
    if (!(cond)) MDZ_FAIL(code, __VA_ARGS__); \
  } while (0)
#define MDZ_HIP(expr)                                                              \
  do {                                                                             \
    hipError_t e_ = (expr);                                                        \
    if (e_ != hipSuccess) MDZ_FAIL(MDZ_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)
#define MDZ_LAUNCH_CHECK() MDZ_HIP(hipGetLastError())

// ---- element types -----------------------------------------------------------------------------
struct bf16_t {
  uint16_t bits;
};

__host__ __device__ inline float bf16_to_float(bf16_t v) {
  union {
    uint32_t u;
    float f;
  } c;
  c.u = uint32_t(v.bits) << 16;
  return c.f;
}
// round to nearest, ties to even (finite inputs)
__host__ __device__ inline bf16_t float_to_bf16(float f) {
  union {
    uint32_t u;
    float f;
  } c;
  c.f = f;
  uint32_t u = c.u + 0x7FFFu + ((c.u >> 16) & 1u);
  return bf16_t{uint16_t(u >> 16)};
}

__host__ __device__ inline float to_float(float v) { return v; }
__host__ __device__ inline float to_float(bf16_t v) { return bf16_to_float(v); }
template <typename T>
__host__ __device__ inline T from_float(float f);
template <>
__host__ __device__ inline float from_float<float>(float f) {
  return f;
}
template <>
__host__ __device__ inline bf16_t from_float<bf16_t>(float f) {
  return float_to_bf16(f);
}

inline int elem_bytes(int dtype) { return dtype == MDZ_BF16 ? 2 : 4; }

// ---- packed weight layout ----------------------------------------------------------------------
// bf16: tiles of 32 rows.  A tile is a sequence of k-steps of 16 input features; one k-step is a
// 1 KiB block = 64 lanes x 8 bf16: lane l holds row (l % 32), features 16*ks + 8*(l / 32) .. +7.
// This is the B-operand order of the 32x32x16 bf16 MFMA, so a wave streams a tile with fully
// coalesced 16-byte-per-lane loads and no shuffling.
// fp32: tiles of 16 rows, plain row-major inside the matrix (the tile only matters for stacking).
constexpr int kTileRowsBf16 = 32;
constexpr int kTileRowsF32 = 16;
constexpr int kKStepBf16 = 16;

__host__ __device__ inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

template <typename T>
struct Packed;
template <>
struct Packed<bf16_t> {
  static constexpr int kTileRows = kTileRowsBf16;
  // element (row n, feature k) of a packed matrix with kp = padded feature count
  __host__ __device__ static inline int64_t index(int64_t n, int64_t k, int64_t kp) {
    int64_t tile = n >> 5, r = n & 31, ks = k >> 4, kk = k & 15;
    return (tile * (kp >> 4) + ks) * 512 + (r + 32 * (kk >> 3)) * 8 + (kk & 7);
  }
  __host__ __device__ static inline int64_t padded_k(int64_t k) { return round_up(k, kKStepBf16); }
};
template <>
struct Packed<float> {
  static constexpr int kTileRows = kTileRowsF32;
  __host__ __device__ static inline int64_t index(int64_t n, int64_t k, int64_t kp) { return n * kp + k; }
  __host__ __device__ static inline int64_t padded_k(int64_t k) { return k; }
};

// ---- KV cache layout ---------------------------------------------------------------------------
// The library owns this layout; callers go through medusa_kv_write / medusa_kv_read.
struct KvGeom {
  int n_layers, batch, n_heads, head_dim, cap;
};
// K element (layer l, sequence b, head h, slot pos, feature i)
__host__ __device__ inline int64_t k_index(const KvGeom& g, int l, int b, int h, int pos, int i) {
  return ((((int64_t)l * g.batch + b) * g.n_heads + h) * g.cap + pos) * g.head_dim + i;
}
__host__ __device__ inline int64_t v_index(const KvGeom& g, int l, int b, int h, int pos, int i) {
  return ((((int64_t)l * g.batch + b) * g.n_heads + h) * g.cap + pos) * g.head_dim + i;
}
inline int64_t kv_elems(const KvGeom& g) {
  return (int64_t)g.n_layers * g.batch * g.n_heads * g.cap * g.head_dim;
}

// ---- device copies of the trees -----------------------------------------------------------------
static __constant__ TreeTables c_trees[kNumTrees] = {kTree15, kTree64};

}  // namespace mdz
