// Shared device/host helpers of the SAAP HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

#include "saap.h"

namespace saap {

typedef uint16_t bf16_t;  // storage type of a bfloat16 element

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

constexpr int kD = SAAP_HEAD_DIM;      // features per head
constexpr float kNegBig = -3.0e38f;    // finite stand-in for "no score yet"
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// ---- host side ---------------------------------------------------------------------------

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Launch-shape overrides for tuning sweeps.  Only builds with -DSAAP_TUNING_BUILD read the
// environment; the shipped library has no hidden inputs and always takes the default.
inline int env_int(const char* name, int dflt) {
#ifdef SAAP_TUNING_BUILD
  const char* v = getenv(name);
  return (v && *v) ? atoi(v) : dflt;
#else
  (void)name;
  return dflt;
#endif
}

// Compute units of the current device; 256 (MI355X) when the query fails.
int device_cus();

// Every entry point starts with begin_call(): an error that an earlier, unrelated HIP call of the process left
// behind is dropped, so that launch_status() reports this call's launches only.
inline void begin_call() { (void)hipGetLastError(); }
inline int32_t launch_status() { return hipGetLastError() == hipSuccess ? SAAP_OK : SAAP_HIP_ERROR; }

// ---- device side -------------------------------------------------------------------------

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// float -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Data-parallel-primitive lane exchanges (no LDS traffic).
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}
constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7-i inside each 8 lanes
constexpr int kDppMirror = 0x140;      // lane i <-> 15-i inside each 16 lanes

// Sum over each aligned group of 16 lanes; every lane of the group gets the total.
__device__ __forceinline__ float sum16(float x) {
  x += dpp_mov<kDppXor1>(x);
  x += dpp_mov<kDppXor2>(x);
  x += dpp_mov<kDppHalfMirror>(x);
  x += dpp_mov<kDppMirror>(x);
  return x;
}

// Maximum / sum over the 64 lanes, in every lane: four register-move steps inside the rows of 16 lanes, then the
// four row results are read as scalars (no LDS crossbar).  All 64 lanes must be active.
__device__ __forceinline__ float wave_max(float x) {
  x = fmaxf(x, dpp_mov<kDppXor1>(x));
  x = fmaxf(x, dpp_mov<kDppXor2>(x));
  x = fmaxf(x, dpp_mov<kDppHalfMirror>(x));
  x = fmaxf(x, dpp_mov<kDppMirror>(x));
  const int b = __float_as_int(x);
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(b, 0)), r1 = __int_as_float(__builtin_amdgcn_readlane(b, 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(b, 32)), r3 = __int_as_float(__builtin_amdgcn_readlane(b, 48));
  return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}
__device__ __forceinline__ float wave_sum(float x) {
  x = sum16(x);
  const int b = __float_as_int(x);
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(b, 0)), r1 = __int_as_float(__builtin_amdgcn_readlane(b, 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(b, 32)), r3 = __int_as_float(__builtin_amdgcn_readlane(b, 48));
  return (r0 + r1) + (r2 + r3);
}

// ---- wave-wide scans and reductions on DPP (no LDS crossbar round trips) ------------------------
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ unsigned dpp_u32(unsigned x) {
  return (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, ROW_MASK, 0xf, true);
}
// Inclusive prefix sum over the 64 lanes (lane order).
__device__ __forceinline__ unsigned wave_prefix_sum(unsigned x) {
  x += dpp_u32<0x111>(x);          // row_shr:1 (lanes shifted in from outside the row read 0)
  x += dpp_u32<0x112>(x);          // row_shr:2
  x += dpp_u32<0x114>(x);          // row_shr:4
  x += dpp_u32<0x118>(x);          // row_shr:8
  x += dpp_u32<0x142, 0xa>(x);     // row_bcast:15 into rows 1 and 3
  x += dpp_u32<0x143, 0xc>(x);     // row_bcast:31 into rows 2 and 3
  return x;
}
// Bitwise AND / OR over the 64 lanes; every lane gets the result.
__device__ __forceinline__ unsigned wave_and(unsigned x) {
  x &= dpp_u32<kDppXor1>(x);
  x &= dpp_u32<kDppXor2>(x);
  x &= dpp_u32<kDppHalfMirror>(x);
  x &= dpp_u32<kDppMirror>(x);
  return (unsigned)__builtin_amdgcn_readlane((int)x, 0) & (unsigned)__builtin_amdgcn_readlane((int)x, 16) &
         (unsigned)__builtin_amdgcn_readlane((int)x, 32) & (unsigned)__builtin_amdgcn_readlane((int)x, 48);
}
__device__ __forceinline__ unsigned wave_or(unsigned x) {
  x |= dpp_u32<kDppXor1>(x);
  x |= dpp_u32<kDppXor2>(x);
  x |= dpp_u32<kDppHalfMirror>(x);
  x |= dpp_u32<kDppMirror>(x);
  return (unsigned)__builtin_amdgcn_readlane((int)x, 0) | (unsigned)__builtin_amdgcn_readlane((int)x, 16) |
         (unsigned)__builtin_amdgcn_readlane((int)x, 32) | (unsigned)__builtin_amdgcn_readlane((int)x, 48);
}

// Exchanges across the four 16-lane rows of a wave with the gfx950 row-swap instructions:
// combines a value with the one held by the same lane of the other three rows.
template <typename F>
__device__ __forceinline__ float across_rows(float x, F op) {
  const unsigned u = __float_as_uint(x);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);   // {own, row ^ 1} in some order
  x = op(__uint_as_float(a[0]), __uint_as_float(a[1]));
  const unsigned v = __float_as_uint(x);
  const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);   // {own, lane ^ 32}
  return op(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float sum_rows(float x) { return across_rows(x, [](float a, float b) { return a + b; }); }
__device__ __forceinline__ float max_rows(float x) { return across_rows(x, [](float a, float b) { return fmaxf(a, b); }); }

// 16 or 8 bytes read once and not again soon (the K/V rows of a decode step): the load carries the
// non-temporal hint, so that the stream does not push the data that IS reused between launches (the
// classifier's weights) out of the caches.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 stream_load16(const void* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void stream_store16(void* p, const uint4& v) {
  u32x4_t w;
  w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  __builtin_nontemporal_store(w, reinterpret_cast<u32x4_t*>(p));
}
__device__ __forceinline__ uint2 stream_load8(const void* p) {
  const u32x2_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(p));
  return make_uint2(v[0], v[1]);
}

// Eight consecutive elements of a row, as loaded by one lane.
template <typename T> struct Vec8;
template <> struct Vec8<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float* p) {
    a = *reinterpret_cast<const float4*>(p);
    b = *reinterpret_cast<const float4*>(p + 4);
  }
  __device__ __forceinline__ void load_stream(const float* p) {
    const uint4 u = stream_load16(p), w = stream_load16(p + 4);
    a = make_float4(__uint_as_float(u.x), __uint_as_float(u.y), __uint_as_float(u.z), __uint_as_float(u.w));
    b = make_float4(__uint_as_float(w.x), __uint_as_float(w.y), __uint_as_float(w.z), __uint_as_float(w.w));
  }
  __device__ __forceinline__ void to_float(float* o) const {
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
  }
  static __device__ __forceinline__ float widen(float v) { return v; }
  static __device__ __forceinline__ float narrow(float v) { return v; }
  __device__ __forceinline__ float dot(const Vec8<float>& q) const {
    float s = a.x * q.a.x;
    s = fmaf(a.y, q.a.y, s); s = fmaf(a.z, q.a.z, s); s = fmaf(a.w, q.a.w, s);
    s = fmaf(b.x, q.b.x, s); s = fmaf(b.y, q.b.y, s); s = fmaf(b.z, q.b.z, s); s = fmaf(b.w, q.b.w, s);
    return s;
  }
};
template <> struct Vec8<bf16_t> {
  uint4 r;
  __device__ __forceinline__ void load(const bf16_t* p) { r = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void load_stream(const bf16_t* p) { r = stream_load16(p); }
  __device__ __forceinline__ void to_float(float* o) const {
    o[0] = bf16_lo(r.x); o[1] = bf16_hi(r.x); o[2] = bf16_lo(r.y); o[3] = bf16_hi(r.y);
    o[4] = bf16_lo(r.z); o[5] = bf16_hi(r.z); o[6] = bf16_lo(r.w); o[7] = bf16_hi(r.w);
  }
  static __device__ __forceinline__ float widen(bf16_t v) { return __uint_as_float((uint32_t)v << 16); }
  static __device__ __forceinline__ bf16_t narrow(float v) { return (bf16_t)f32_to_bf16_bits(v); }   // round to nearest even
  // Products of two bf16 numbers are exact in fp32; v_dot2_f32_bf16 adds two of them per step.
  __device__ __forceinline__ float dot(const Vec8<bf16_t>& q) const {
    float s = 0.f;
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, r.x), __builtin_bit_cast(bf16x2_t, q.r.x), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, r.y), __builtin_bit_cast(bf16x2_t, q.r.y), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, r.z), __builtin_bit_cast(bf16x2_t, q.r.z), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, r.w), __builtin_bit_cast(bf16x2_t, q.r.w), s, false);
    return s;
  }
};

// Eight features stored as OCP FP8 E4M3 codes (one byte each); queries against such rows are bf16.
typedef uint8_t fp8_t;
template <> struct Vec8<fp8_t> {
  uint2 r;
  __device__ __forceinline__ void load(const fp8_t* p) { r = *reinterpret_cast<const uint2*>(p); }
  __device__ __forceinline__ void load_stream(const fp8_t* p) { r = stream_load8(p); }
  __device__ __forceinline__ void to_float(float* o) const {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t a = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.x, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.x, true);
    const f32x2_t c = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.y, false), d = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.y, true);
    o[0] = a[0]; o[1] = a[1]; o[2] = b[0]; o[3] = b[1]; o[4] = c[0]; o[5] = c[1]; o[6] = d[0]; o[7] = d[1];
  }
  // The same eight values as bf16 (exact: an E4M3 value has 4 significant bits), so that the
  // dot product with a bf16 query runs on v_dot2_f32_bf16.
  __device__ __forceinline__ Vec8<bf16_t> as_bf16() const {
    float f[8];
    to_float(f);
    Vec8<bf16_t> w;
    // upper halves of two floats packed into one word
    w.r.x = __builtin_amdgcn_perm(__float_as_uint(f[1]), __float_as_uint(f[0]), 0x07060302u);
    w.r.y = __builtin_amdgcn_perm(__float_as_uint(f[3]), __float_as_uint(f[2]), 0x07060302u);
    w.r.z = __builtin_amdgcn_perm(__float_as_uint(f[5]), __float_as_uint(f[4]), 0x07060302u);
    w.r.w = __builtin_amdgcn_perm(__float_as_uint(f[7]), __float_as_uint(f[6]), 0x07060302u);
    return w;
  }
};
// Type of the query rows and of the key operand of the dot product for a cache stored as T.
template <typename T> struct DotType { typedef T type; };
template <> struct DotType<fp8_t> { typedef bf16_t type; };
template <typename T> __device__ __forceinline__ Vec8<T> dot_operand(const Vec8<T>& k) { return k; }
__device__ __forceinline__ Vec8<bf16_t> dot_operand(const Vec8<fp8_t>& k) { return k.as_bf16(); }

// Order-preserving map float -> uint32 (larger float, larger key); -0 and +0 must be
// canonicalised by the caller.
__device__ __forceinline__ uint32_t float_order_key(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

}  // namespace saap

// Debug builds (-DSAAP_TRACE_BUILD) stamp the 100 MHz wall clock at marked points of a kernel:
// thread 0 of every workgroup writes slot i of its 16-slot record.  The buffer address comes from
// the environment variable SAAP_TRACE_PTR (hex).  Release builds compile the marks away.
#ifdef SAAP_TRACE_BUILD
static __device__ unsigned long long* saap_trace_buf;
#define SAAP_TRACE(i)                                                                              \
  do {                                                                                             \
    if (saap_trace_buf && threadIdx.x == 0)                                                        \
      saap_trace_buf[((size_t)blockIdx.x + (size_t)gridDim.x * (blockIdx.y + (size_t)gridDim.y * blockIdx.z)) * 16 + (i)] = wall_clock64(); \
  } while (0)
#define SAAP_TRACE_VALUE(i, v)                                                                     \
  do {                                                                                             \
    if (saap_trace_buf)                                                                            \
      saap_trace_buf[((size_t)blockIdx.x + (size_t)gridDim.x * (blockIdx.y + (size_t)gridDim.y * blockIdx.z)) * 16 + (i)] = (unsigned long long)(v); \
  } while (0)
/* the same stamp taken by lane 0 of whichever wave runs the code */                               \
#define SAAP_TRACE_WAVE(i)                                                                         \
  do {                                                                                             \
    if (saap_trace_buf && (threadIdx.x & 63) == 0)                                                 \
      saap_trace_buf[((size_t)blockIdx.x + (size_t)gridDim.x * (blockIdx.y + (size_t)gridDim.y * blockIdx.z)) * 16 + (i)] = wall_clock64(); \
  } while (0)
static inline void saap_trace_arm() {
  const char* tp = getenv("SAAP_TRACE_PTR");
  unsigned long long* ptr = tp ? reinterpret_cast<unsigned long long*>(strtoull(tp, nullptr, 16)) : nullptr;
  (void)hipMemcpyToSymbol(HIP_SYMBOL(saap_trace_buf), &ptr, sizeof(ptr));
}
#else
#define SAAP_TRACE(i) do { } while (0)
#define SAAP_TRACE_VALUE(i, v) do { } while (0)
#define SAAP_TRACE_WAVE(i) do { } while (0)
static inline void saap_trace_arm() {}
#endif
