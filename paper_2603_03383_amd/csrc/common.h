// Shared host/device helpers of libmedusa_hip: status handling, element types, the packed weight
// layout and the KV cache layout.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include <mutex>

#include "../../include/medusa.h"
#include "../../include/medusa_bench.h"
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

// Wall-clock stamps per workgroup, compiled in only by the timing probe (probes/stamps_probe.hip, -DMDZ_STAMPS):
// stamp i of workgroup w (its linear index in the grid) goes to mdz_stamps[8 w + i], in units of 10 ns.  In the
// library build the macro is empty.
#ifdef MDZ_STAMPS
__device__ unsigned long long mdz_stamps[8 * 4096];
#define MDZ_STAMP(i)                                                                                             \
  do {                                                                                                           \
    if (threadIdx.x == 0)                                                                                        \
      mdz_stamps[(blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z)) * 8 + (i)] = wall_clock64();  \
  } while (0)
#else
#define MDZ_STAMP(i) ((void)0)
#endif

// ---- device facts --------------------------------------------------------------------------------
// Compute units of the current device (read once; 256 when no device can be asked: host-only plan introspection).
int num_cus();

// Sets a kernel's dynamic-LDS limit once per device, from whichever thread gets there first (calls on different
// streams may come from different threads; a function attribute belongs to the device the code object is loaded on).
constexpr int kMaxDevices = 64;
#define MDZ_SET_LDS_ONCE(kernel_expr, bytes)                                                                   \
  do {                                                                                                         \
    static std::once_flag once_[::mdz::kMaxDevices];                                                           \
    static hipError_t once_err_[::mdz::kMaxDevices];                                                           \
    int dev_ = 0;                                                                                              \
    if (hipGetDevice(&dev_) != hipSuccess || dev_ < 0 || dev_ >= ::mdz::kMaxDevices) dev_ = 0;                 \
    std::call_once(once_[dev_], [&]() {                                                                        \
      once_err_[dev_] = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel_expr),                        \
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (bytes));              \
    });                                                                                                        \
    if (once_err_[dev_] != hipSuccess)                                                                         \
      MDZ_FAIL(MDZ_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(once_err_[dev_]));                      \
  } while (0)

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

// IEEE binary16 (the paper's inference precision, Section 4.1)
struct f16_t {
  uint16_t bits;
};
__host__ __device__ inline float to_float(f16_t v) { return (float)__builtin_bit_cast(_Float16, v.bits); }
template <>
__host__ __device__ inline f16_t from_float<f16_t>(float f) {
  return f16_t{__builtin_bit_cast(uint16_t, (_Float16)f)};  // round to nearest even
}

inline bool is_16bit(int dtype) { return dtype == MDZ_BF16 || dtype == MDZ_FP16; }
inline bool dtype_ok(int dtype) { return dtype == MDZ_BF16 || dtype == MDZ_FP32 || dtype == MDZ_FP16; }
inline int elem_bytes(int dtype) { return is_16bit(dtype) ? 2 : 4; }

// The two 16-bit storage types share every layout (packed weights, tiled KV cache) and every kernel; a kernel
// template takes the element type E and gets from Elem16<E> the packing of two floats into one 32-bit word, its
// inverse, and the 32x32x16 MFMA that consumes 8 elements per lane.
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
template <typename E>
struct Elem16;
template <>
struct Elem16<bf16_t> {
  __device__ static inline uint32_t pack2(float a, float b) {  // round to nearest even: one v_cvt_pk_bf16_f32
    typedef float f2 __attribute__((ext_vector_type(2)));
    typedef __bf16 v2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{a, b}, v2));
  }
  __device__ static inline float lo(uint32_t w) { return __uint_as_float(w << 16); }
  __device__ static inline float hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
  __device__ static inline uint32_t from_fp8x2(uint32_t src, bool hi_word) {  // two E4M3 codes -> two elements (exact)
    typedef __bf16 v2 __attribute__((ext_vector_type(2)));
    return hi_word ? __builtin_bit_cast(uint32_t, (v2)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(src, 1.0f, true))
                   : __builtin_bit_cast(uint32_t, (v2)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(src, 1.0f, false));
  }
  __device__ static inline f32x16_t mfma(u32x4_t a, u32x4_t b, f32x16_t c) {
    typedef __bf16 v8 __attribute__((ext_vector_type(8)));
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8, a), __builtin_bit_cast(v8, b), c, 0, 0, 0);
  }
};
template <>
struct Elem16<f16_t> {
  typedef _Float16 h2 __attribute__((ext_vector_type(2)));
  __device__ static inline uint32_t pack2(float a, float b) {
    return __builtin_bit_cast(uint32_t, h2{(_Float16)a, (_Float16)b});
  }
  __device__ static inline float lo(uint32_t w) { return (float)__builtin_bit_cast(h2, w).x; }
  __device__ static inline float hi(uint32_t w) { return (float)__builtin_bit_cast(h2, w).y; }
  __device__ static inline uint32_t from_fp8x2(uint32_t src, bool hi_word) {
    return hi_word ? __builtin_bit_cast(uint32_t, (h2)__builtin_amdgcn_cvt_scalef32_pk_f16_fp8(src, 1.0f, true))
                   : __builtin_bit_cast(uint32_t, (h2)__builtin_amdgcn_cvt_scalef32_pk_f16_fp8(src, 1.0f, false));
  }
  __device__ static inline f32x16_t mfma(u32x4_t a, u32x4_t b, f32x16_t c) {
    typedef _Float16 v8 __attribute__((ext_vector_type(8)));
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8, a), __builtin_bit_cast(v8, b), c, 0, 0, 0);
  }
};
// runs `body` with E bound to the element type of any storage dtype
#define MDZ_WITH_ELEM(dtype, body)    \
  do {                                \
    if ((dtype) == MDZ_BF16) {        \
      using E = ::mdz::bf16_t;        \
      body;                           \
    } else if ((dtype) == MDZ_FP16) { \
      using E = ::mdz::f16_t;         \
      body;                           \
    } else {                          \
      using E = float;                \
      body;                           \
    }                                 \
  } while (0)
// runs `body` with E bound to the element type of a 16-bit dtype
#define MDZ_WITH_ELEM16(dtype, body) \
  do {                               \
    if ((dtype) == MDZ_BF16) {       \
      using E = ::mdz::bf16_t;       \
      body;                          \
    } else {                         \
      using E = ::mdz::f16_t;        \
      body;                          \
    }                                \
  } while (0)

// ---- packed weight layout ----------------------------------------------------------------------
// 16-bit types (bf16, fp16; written as bf16 below): rows are grouped in tiles of 32 and tiles in bands of 4 (128 output columns); input features in
// k-steps of 16 and k-steps in stages of 16 (256 features).  Memory order: [band][stage][tile in band][k-step
// in stage][lane][8 bf16], where one k-step of one tile is a 1 KiB block of 64 lanes x 8 bf16: lane l holds row
// (l % 32), features 16*ks + 8*(l / 32) .. +7 — the B-operand order of the 32x32x16 bf16 MFMA.  So a wave loads
// a k-step with one fully coalesced 16-byte-per-lane instruction and no shuffling, the four waves of a workgroup
// read one contiguous 64 KiB block per stage, and successive stages of a band are contiguous: every workgroup
// streams linear memory.  Rows are padded to 128 and features to 256 (zero filled where the kernels read them).
// fp32: tiles of 16 rows, plain row-major inside the matrix (the tile only matters for stacking).
constexpr int kTileRowsBf16 = 32;
constexpr int kTileRowsF32 = 16;
constexpr int kKStepBf16 = 16;
constexpr int kBandTiles = 4;      // tiles per band of the bf16 layout
constexpr int kStageFeatures = 256;  // features per stage of the bf16 layout

__host__ __device__ inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

template <typename T>
struct Packed;
template <>
struct Packed<bf16_t> {
  static constexpr int kTileRows = kTileRowsBf16;
  // element (row n, feature k) of a packed matrix with kp = padded feature count (multiple of 256)
  __host__ __device__ static inline int64_t index(int64_t n, int64_t k, int64_t kp) {
    int64_t tile = n >> 5, r = n & 31, band = tile >> 2, tin = tile & 3;
    int64_t ks = k >> 4, kk = k & 15, st = ks >> 4, kin = ks & 15;
    int64_t unit = ((band * (kp >> 8) + st) * kBandTiles + tin) * 16 + kin;  // 1 KiB units
    return unit * 512 + (r + 32 * (kk >> 3)) * 8 + (kk & 7);
  }
  __host__ __device__ static inline int64_t padded_k(int64_t k) { return round_up(k, kStageFeatures); }
  __host__ __device__ static inline int64_t padded_rows(int64_t n) { return round_up(n, kTileRowsBf16 * kBandTiles); }
};
template <>
struct Packed<f16_t> : Packed<bf16_t> {};
template <>
struct Packed<float> {
  static constexpr int kTileRows = kTileRowsF32;
  __host__ __device__ static inline int64_t index(int64_t n, int64_t k, int64_t kp) { return n * kp + k; }
  __host__ __device__ static inline int64_t padded_k(int64_t k) { return k; }
  __host__ __device__ static inline int64_t padded_rows(int64_t n) { return round_up(n, kTileRowsF32); }
};

// ---- KV cache layout ---------------------------------------------------------------------------
// The library owns this layout; callers go through medusa_kv_write / medusa_kv_read.
// fp32: plain [layer][seq][head][slot][feature] for K and V.
// bf16 / fp16: per (layer, seq, head) the slots are grouped in blocks of 32; a block is a sequence of 1 KiB
// units of 64 lanes x 8 bf16, each unit being one MFMA A operand of the attention kernel, so a wave
// streams K and V with contiguous 16-byte-per-lane loads and no transposition:
//   K block (scores^T = K Q^T, rows = keys, contraction over features): unit ks holds for lane l
//     key (l % 32), features 16*ks + 8*(l / 32) .. +7.
//   V block (out^T = V^T P^T, rows = features, contraction over keys): unit (2*t + s2) holds for lane l
//     feature 32*t + (l % 32) and the 8 keys 16*s2 + 8*(e / 4) + 4*(l / 32) + (e % 4), e = 0..7 — the
//     order in which the score MFMA leaves its 16 keys per lane, so probabilities feed the second MFMA
//     straight from registers.
struct KvGeom {
  int n_layers, batch, n_heads, head_dim, cap;  // n_heads: key/value heads (the heads the cache holds)
  int tiled;  // 1: bf16 block layout above (head_dim % 32 == 0); 0: plain
  int group;  // query heads per key/value head (grouped-query attention; 1: plain multi-head attention)
  int quant;  // 1: 8-bit rows (E4M3 codes + one fp32 scale per row, layout below); needs tiled and head_dim 128
};
__host__ __device__ inline int q_heads(const KvGeom& g) { return g.n_heads * g.group; }
__host__ __device__ inline int kv_cap_pad(const KvGeom& g) { return g.tiled ? (g.cap + 31) & ~31 : g.cap; }
__host__ __device__ inline int64_t kv_head_base(const KvGeom& g, int l, int b, int h) {
  return (((int64_t)l * g.batch + b) * g.n_heads + h) * (int64_t)kv_cap_pad(g) * g.head_dim;
}
// K element (layer l, sequence b, head h, slot pos, feature i)
__host__ __device__ inline int64_t k_index(const KvGeom& g, int l, int b, int h, int pos, int i) {
  int64_t base = kv_head_base(g, l, b, h);
  if (!g.tiled) return base + (int64_t)pos * g.head_dim + i;
  int blk = pos >> 5, key = pos & 31, ks = i >> 4, kh = (i >> 3) & 1, e = i & 7;
  return base + (int64_t)blk * 32 * g.head_dim + ks * 512 + (key + 32 * kh) * 8 + e;
}
__host__ __device__ inline int64_t v_index(const KvGeom& g, int l, int b, int h, int pos, int i) {
  int64_t base = kv_head_base(g, l, b, h);
  if (!g.tiled) return base + (int64_t)pos * g.head_dim + i;
  int blk = pos >> 5, kk = pos & 31;
  int s2 = kk >> 4, ehi = (kk >> 3) & 1, kh = (kk >> 2) & 1, elo = kk & 3;
  int t = i >> 5, row = i & 31;
  return base + (int64_t)blk * 32 * g.head_dim + (t * 2 + s2) * 512 + (row + 32 * kh) * 8 + (ehi * 4 + elo);
}
inline int64_t kv_elems(const KvGeom& g) {
  return (int64_t)g.n_layers * g.batch * g.n_heads * kv_cap_pad(g) * g.head_dim;
}

// ---- 8-bit KV cache layout (MDZ_KV_FP8E4M3, head_dim 128) -----------------------------------------
// The KV compression the paper points to for long sequences (Sections 4.2 and 5).  A row (one slot of one
// key/value head) is 128 OCP FP8 E4M3 codes and one fp32 scale: scale = max|row| / 448 (1 for a zero row),
// code = nearest E4M3 value of x / scale (ties to even, decided in fp32), value read back = value(code) * scale.
// Per (layer, seq, head) the slots are grouped in blocks of 32; a block is 4 units of 1 KiB (64 lanes x 16 B)
// followed by the 32 scales, 4224 B in all, so a wave streams a block as one contiguous piece:
//   K unit j: lane l holds key (l % 32) and the 16 features 32j + 16p + 8(l / 32) + e, byte 8p + e (p < 2, e < 8):
//     the 8 bytes of one p convert to the A operand of k-step 2j + p of the 16-bit layout above.
//   V unit t: lane l holds feature 32t + (l % 32) and 16 keys, byte 8 s2 + e for key 16 s2 + 8(e / 4) + 4(l / 32) + e % 4:
//     the 8 bytes of one s2 convert to the A operand of unit (2t + s2) of the 16-bit layout.
constexpr int kKv8BlockBytes = 32 * 128 + 32 * 4;
constexpr float kE4M3Max = 448.0f;
__host__ __device__ inline int64_t kv8_head_base(const KvGeom& g, int l, int b, int h) {  // bytes
  return (((int64_t)l * g.batch + b) * g.n_heads + h) * (int64_t)(kv_cap_pad(g) >> 5) * kKv8BlockBytes;
}
__host__ __device__ inline int64_t kv8_k_code(int pos, int i) {  // byte offset inside the head's region
  const int blk = pos >> 5, key = pos & 31, j = i >> 5, p = (i >> 4) & 1, gh = (i >> 3) & 1, e = i & 7;
  return (int64_t)blk * kKv8BlockBytes + j * 1024 + (key + 32 * gh) * 16 + p * 8 + e;
}
__host__ __device__ inline int64_t kv8_v_code(int pos, int i) {
  const int blk = pos >> 5, kk = pos & 31, s2 = kk >> 4, ehi = (kk >> 3) & 1, kh = (kk >> 2) & 1, elo = kk & 3;
  const int t = i >> 5, row = i & 31;
  return (int64_t)blk * kKv8BlockBytes + t * 1024 + (row + 32 * kh) * 16 + s2 * 8 + ehi * 4 + elo;
}
__host__ __device__ inline int64_t kv8_scale(int pos) {  // byte offset of the slot's scale
  return (int64_t)(pos >> 5) * kKv8BlockBytes + 4096 + (pos & 31) * 4;
}
inline int64_t kv8_bytes(const KvGeom& g) {
  return (int64_t)g.n_layers * g.batch * g.n_heads * (kv_cap_pad(g) >> 5) * kKv8BlockBytes;
}
#if defined(__HIPCC__)
// quantiser shared by every kernel that writes 8-bit rows: scale of a row from its largest magnitude, and four
// values -> four codes (IEEE fp32 division, clamp, the hardware's round-to-nearest-even E4M3 conversion)
__device__ inline float kv8_scale_of(float amax) { return amax > 0.f ? amax / kE4M3Max : 1.0f; }
__device__ inline uint32_t kv8_pack4(float a, float b, float c, float d, float s) {
  auto q = [&](float v) { return fminf(fmaxf(v / s, -kE4M3Max), kE4M3Max); };
  int w = __builtin_amdgcn_cvt_pk_fp8_f32(q(a), q(b), 0, false);
  w = __builtin_amdgcn_cvt_pk_fp8_f32(q(c), q(d), w, true);
  return (uint32_t)w;
}
#endif

// ---- device copies of the trees -----------------------------------------------------------------
static __constant__ TreeTables c_trees[kNumTrees] = {kTree15, kTree64, kTree1, kTree64K5};

}  // namespace mdz
