// Shared device/host helpers of libcdf (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "cdf.h"

namespace cdf {

constexpr int kWave = 64;

// ---- host-side error text -------------------------------------------------
void set_error(const char* fmt, ...);

#define CDF_FAIL(code, ...)      \
  do {                           \
    cdf::set_error(__VA_ARGS__); \
    return (code);               \
  } while (0)

#define CDF_REQUIRE(cond, ...) \
  do {                         \
    if (!(cond)) CDF_FAIL(CDF_ERR_INVALID_ARG, __VA_ARGS__); \
  } while (0)

#define CDF_LAUNCH_CHECK(name)                                                        \
  do {                                                                                \
    hipError_t e__ = hipGetLastError();                                               \
    if (e__ != hipSuccess) CDF_FAIL(CDF_ERR_HIP, "%s: %s", name, hipGetErrorString(e__)); \
  } while (0)

// ---- optional per-kernel timing (host side, HIP events on the launch stream) ----
enum KernelId {
  K_FILTER = 0, K_SCAN, K_COMPACT, K_QUANTIZE, K_DEQUANTIZE, K_SPMM_PLAN, K_SPMM, K_SPMM_FIXUP,
  K_GEMM_FWD, K_GEMM_DW, K_GEMM_DW_REDUCE, K_GEMM_DM, K_SPMM_SLICED, K_RELU_MASK, K_TEST_ENCODE, K_GATHER_CODES, K_SPMM_XFORM,
  K_COUNT
};
void prof_begin(int id, hipStream_t st);
void prof_end(int id, hipStream_t st);
struct ProfScope {
  int id;
  hipStream_t st;
  ProfScope(int i, hipStream_t s) : id(i), st(s) { prof_begin(id, st); }
  ~ProfScope() { prof_end(id, st); }
};

// Rows per block of the cache test, of its scan / compaction, and of the one-pass test + message
// build (16 rows per wavefront): the per-block counts of all of them have this granularity.
constexpr int kRowsPerBlock = 64;

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline size_t elem_bytes(cdf_dtype dt) { return dt == CDF_BF16 ? 2 : 4; }

// Per-block counts and their exclusive offsets share one workspace area: counts first, offsets
// `scan_stride` ints later (a multiple of 4, so that both start on the same 16-byte phase).
inline int64_t scan_stride(int64_t nblocks) { return (nblocks + 1 + 3) / 4 * 4; }

// Elements per lane-vector for rows of `dim` elements spaced `ld` apart starting at p0 / p1:
// 4, 2 or 1, the widest for which every row start and every vector is naturally aligned.
inline int pick_epv(int32_t dim, int64_t ld, size_t esz, const void* p0, const void* p1 = nullptr,
                    const void* p2 = nullptr) {
  for (int epv = 4; epv > 1; epv >>= 1) {
    size_t vb = esz * epv;
    if (dim % epv == 0 && ld % epv == 0 && aligned(p0, vb) && (!p1 || aligned(p1, vb)) &&
        (!p2 || aligned(p2, vb)))
      return epv;
  }
  return 1;
}

inline int log2_ceil(int v) {
  int l = 0;
  while ((1 << l) < v) ++l;
  return l;
}

// ---- device helpers --------------------------------------------------------
typedef uint16_t bf16_t;  // bf16 storage: upper half of an IEEE fp32

__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }

// fp32 -> bf16, round to nearest, ties to even; NaN stays a quiet NaN.
__device__ __forceinline__ uint16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

template <typename T, int EPV>
struct VecIO;

template <>
struct VecIO<float, 4> {
  static __device__ __forceinline__ void load(const float* p, float (&v)[4]) {
    float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  static __device__ __forceinline__ void store(float* p, const float (&v)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <>
struct VecIO<float, 2> {
  static __device__ __forceinline__ void load(const float* p, float (&v)[2]) {
    float2 t = *reinterpret_cast<const float2*>(p);
    v[0] = t.x; v[1] = t.y;
  }
  static __device__ __forceinline__ void store(float* p, const float (&v)[2]) {
    *reinterpret_cast<float2*>(p) = make_float2(v[0], v[1]);
  }
};
template <>
struct VecIO<float, 1> {
  static __device__ __forceinline__ void load(const float* p, float (&v)[1]) { v[0] = *p; }
  static __device__ __forceinline__ void store(float* p, const float (&v)[1]) { *p = v[0]; }
};
template <>
struct VecIO<bf16_t, 8> {
  static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[8]) {
    uint4 t = *reinterpret_cast<const uint4*>(p);
    v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
    v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
    v[4] = __uint_as_float(t.z << 16); v[5] = __uint_as_float(t.z & 0xffff0000u);
    v[6] = __uint_as_float(t.w << 16); v[7] = __uint_as_float(t.w & 0xffff0000u);
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[8]) {
    uint4 t;
    t.x = f2bf(v[0]) | (static_cast<uint32_t>(f2bf(v[1])) << 16);
    t.y = f2bf(v[2]) | (static_cast<uint32_t>(f2bf(v[3])) << 16);
    t.z = f2bf(v[4]) | (static_cast<uint32_t>(f2bf(v[5])) << 16);
    t.w = f2bf(v[6]) | (static_cast<uint32_t>(f2bf(v[7])) << 16);
    *reinterpret_cast<uint4*>(p) = t;
  }
};
template <>
struct VecIO<bf16_t, 4> {
  static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[4]) {
    uint2 t = *reinterpret_cast<const uint2*>(p);
    v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
    v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[4]) {
    uint2 t;
    t.x = f2bf(v[0]) | (static_cast<uint32_t>(f2bf(v[1])) << 16);
    t.y = f2bf(v[2]) | (static_cast<uint32_t>(f2bf(v[3])) << 16);
    *reinterpret_cast<uint2*>(p) = t;
  }
};
template <>
struct VecIO<bf16_t, 2> {
  static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[2]) {
    uint32_t t = *reinterpret_cast<const uint32_t*>(p);
    v[0] = __uint_as_float(t << 16); v[1] = __uint_as_float(t & 0xffff0000u);
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[2]) {
    *reinterpret_cast<uint32_t*>(p) = f2bf(v[0]) | (static_cast<uint32_t>(f2bf(v[1])) << 16);
  }
};
template <>
struct VecIO<bf16_t, 1> {
  static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[1]) { v[0] = bf2f(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[1]) { *p = f2bf(v[0]); }
};

// Butterfly reductions over the lanes of a group of `g` lanes (g a power of two <= 64),
// strides 1, 2, ..., g/2: every lane of the group ends with the same value.
__device__ __forceinline__ float group_sum(float x, int g) {
  for (int off = 1; off < g; off <<= 1) x = x + __shfl_xor(x, off, kWave);
  return x;
}
__device__ __forceinline__ float group_max(float x, int g) {
  for (int off = 1; off < g; off <<= 1) x = fmaxf(x, __shfl_xor(x, off, kWave));
  return x;
}
__device__ __forceinline__ float group_min(float x, int g) {
  for (int off = 1; off < g; off <<= 1) x = fminf(x, __shfl_xor(x, off, kWave));
  return x;
}

}  // namespace cdf
