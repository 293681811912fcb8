// quantize_kv: 8-bit storage of a bucket-sorted K/V cache.  The paper names compression of the
// cached vectors as complementary to the partition (Section 2, related work on vector
// compression) without fixing a format; this build uses OCP FP8 E4M3 (bias 7, largest finite
// value 448) with one power-of-two scale per (sequence, KV head) and tensor, which halves the
// bytes the decode attention reads per key.
//   scale = 2^e, e the smallest integer with max|x| <= 448 * 2^e (1 for an all-zero unit)
//   code  = round-to-nearest-even of x / scale (the chip's v_cvt_pk_fp8_f32)
// Three launches for K and V together: per-unit maxima (atomic max on the bit pattern, which
// orders non-negative floats), the conversion, and clearing the maxima again.
#include "common.h"

namespace saap {
namespace {

constexpr int kQThreads = 256;
constexpr int kQSlices = 64;      // workgroups per (tensor, unit) in both passes
constexpr int kQUnroll = 4;       // 16-byte (bf16) loads a thread has in flight

template <typename T>
__global__ void __launch_bounds__(kQThreads)
absmax_kernel(const T* __restrict__ K, const T* __restrict__ V, unsigned* __restrict__ amax_bits, size_t pieces,
              int units) {
  const int unit = blockIdx.y, tensor = blockIdx.z;
  const T* x = (tensor ? V : K) + (size_t)unit * pieces * 8;
  float m = 0.f;
  // four loads in flight per thread (a piece past the end reads the last one again: the maximum does not change)
  const size_t step = (size_t)kQSlices * kQThreads;
  for (size_t i = (size_t)blockIdx.x * kQThreads + threadIdx.x; i < pieces; i += kQUnroll * step) {
    Vec8<T> v[kQUnroll];
#pragma unroll
    for (int u = 0; u < kQUnroll; ++u) v[u].load_stream(x + min(i + u * step, pieces - 1) * 8);
#pragma unroll
    for (int u = 0; u < kQUnroll; ++u) {
      float f[8];
      v[u].to_float(f);
#pragma unroll
      for (int e = 0; e < 8; ++e) m = fmaxf(m, fabsf(f[e]));
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
  if ((threadIdx.x & 63) == 0) atomicMax(&amax_bits[tensor * units + unit], __float_as_uint(m));
}

// 2^e with the smallest e such that amax <= 448 * 2^e; 448 = 0.875 * 2^9
__device__ __forceinline__ int unit_exponent(float amax) {
  int ex;
  const float f = frexpf(amax, &ex);
  const int e = f <= 0.875f ? ex - 9 : ex - 8;
  return min(max(e, -100), 100);
}

template <typename T>
__global__ void __launch_bounds__(kQThreads)
quantize_kernel(const T* __restrict__ K, const T* __restrict__ V, uint8_t* __restrict__ K8, uint8_t* __restrict__ V8,
                const unsigned* __restrict__ amax_bits, float* __restrict__ kscale, float* __restrict__ vscale,
                size_t pieces, int units) {
  const int unit = blockIdx.y, tensor = blockIdx.z;
  const T* x = (tensor ? V : K) + (size_t)unit * pieces * 8;
  uint2* y = reinterpret_cast<uint2*>((tensor ? V8 : K8) + (size_t)unit * pieces * 8);
  const float amax = __uint_as_float(amax_bits[tensor * units + unit]);
  const int e = amax > 0.f ? unit_exponent(amax) : 0;
  const float inv = ldexpf(1.f, -e);
  if (blockIdx.x == 0 && threadIdx.x == 0) (tensor ? vscale : kscale)[unit] = ldexpf(1.f, e);
  const size_t step = (size_t)kQSlices * kQThreads;
  for (size_t i = (size_t)blockIdx.x * kQThreads + threadIdx.x; i < pieces; i += kQUnroll * step) {
    Vec8<T> v[kQUnroll];
#pragma unroll
    for (int u = 0; u < kQUnroll; ++u) v[u].load_stream(x + min(i + u * step, pieces - 1) * 8);
#pragma unroll
    for (int u = 0; u < kQUnroll; ++u) {
      float f[8];
      v[u].to_float(f);
      int lo = 0, hi = 0;
      lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[0] * inv, f[1] * inv, lo, false);
      lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[2] * inv, f[3] * inv, lo, true);
      hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[4] * inv, f[5] * inv, hi, false);
      hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[6] * inv, f[7] * inv, hi, true);
      if (i + u * step < pieces) y[i + u * step] = make_uint2((unsigned)lo, (unsigned)hi);
    }
  }
}

__global__ void clear_words_kernel(unsigned* w, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) w[i] = 0u;
}

}  // namespace
}  // namespace saap

using namespace saap;

extern "C" int32_t saap_quantize_kv(const void* Ksorted, const void* Vsorted, uint8_t* K8, uint8_t* V8, float* kscale,
                                    float* vscale, int32_t S, int32_t Hkv, int32_t Ncap, int32_t d, int32_t dtype,
                                    void* ws, size_t ws_bytes, void* stream) {
  begin_call();
  if (!Ksorted || !Vsorted || !K8 || !V8 || !kscale || !vscale || !ws) return SAAP_INVALID_ARG;
  if (!aligned16(Ksorted) || !aligned16(Vsorted) || !aligned16(K8) || !aligned16(V8) || !aligned16(ws))
    return SAAP_INVALID_ARG;
  if (S <= 0 || Hkv <= 0 || Ncap <= 0) return SAAP_INVALID_ARG;
  if (dtype != SAAP_F32 && dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  if (d != kD) return SAAP_UNSUPPORTED;
  const long long units = (long long)S * Hkv;
  if (units > 65535 || 2 * units * sizeof(unsigned) > SAAP_WS_HEADER_BYTES) return SAAP_UNSUPPORTED;
  if (ws_bytes < SAAP_WS_HEADER_BYTES) return SAAP_WORKSPACE_TOO_SMALL;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  unsigned* amax_bits = reinterpret_cast<unsigned*>(ws);   // header words [2 * units], zero on entry and on exit
  const size_t pieces = (size_t)Ncap * kD / 8;
  const dim3 grid(kQSlices, (unsigned)units, 2);
  if (dtype == SAAP_BF16) {
    hipLaunchKernelGGL(absmax_kernel<bf16_t>, grid, dim3(kQThreads), 0, hs, static_cast<const bf16_t*>(Ksorted),
                       static_cast<const bf16_t*>(Vsorted), amax_bits, pieces, (int)units);
    hipLaunchKernelGGL(quantize_kernel<bf16_t>, grid, dim3(kQThreads), 0, hs, static_cast<const bf16_t*>(Ksorted),
                       static_cast<const bf16_t*>(Vsorted), K8, V8, amax_bits, kscale, vscale, pieces, (int)units);
  } else {
    hipLaunchKernelGGL(absmax_kernel<float>, grid, dim3(kQThreads), 0, hs, static_cast<const float*>(Ksorted),
                       static_cast<const float*>(Vsorted), amax_bits, pieces, (int)units);
    hipLaunchKernelGGL(quantize_kernel<float>, grid, dim3(kQThreads), 0, hs, static_cast<const float*>(Ksorted),
                       static_cast<const float*>(Vsorted), K8, V8, amax_bits, kscale, vscale, pieces, (int)units);
  }
  hipLaunchKernelGGL(clear_words_kernel, dim3((unsigned)((2 * units + 255) / 256)), dim3(256), 0, hs, amax_bits,
                     (int)(2 * units));
  return launch_status();
}
