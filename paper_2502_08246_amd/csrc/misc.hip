// Host-side utilities of the C ABI: workspace sizing, status strings, device query, and the
// fill kernel that zeroes the workspace header.
#include "common.h"

namespace saap {

size_t attn_workspace_bytes(long long units, int G);
size_t planned_workspace_bytes(long long units, int G);
size_t prefill_workspace_bytes(long long S, int Tq, int Hq, int Hkv, int nprobe);
size_t assign_workspace_bytes(long long rows);
size_t build_workspace_bytes(long long units, int N, int B);
size_t push_workspace_bytes(long long units, int B);
size_t classify_workspace_bytes(long long rows, int hidden);
size_t mass_workspace_bytes(long long units, int G, int B);
size_t mass_batch_workspace_bytes(long long units, long long R, int B);
size_t train_workspace_bytes(long long Hw, long long R, int d, int hidden, int B);

int device_cus() {
  // asked on every call: the caller may have switched devices since the last one
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) == hipSuccess &&
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
    return cus;
  return 256;
}

namespace {
__global__ void zero_words_kernel(uint32_t* p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}
// Reads `n` 16-byte words once (grid-stride, four non-temporal loads in flight per lane) and folds them into
// one word per workgroup: the streaming-read ceiling of the device for the benchmark report.
__global__ void __launch_bounds__(512) stream_read_kernel(const uint4* __restrict__ src, size_t n, uint32_t* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t acc = 0u;
  for (; i + 3 * stride < n; i += 4 * stride) {
    const uint4 a = stream_load16(src + i), b = stream_load16(src + i + stride), c = stream_load16(src + i + 2 * stride),
                d = stream_load16(src + i + 3 * stride);
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < n; i += stride) {
    const uint4 a = src[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o);
  if ((threadIdx.x & 63) == 0) atomicXor(&sink[blockIdx.x], acc);
}
// `iters` rounds of eight independent v_mfma_f32_32x32x16_bf16 per wave on operands read once from `ops` (16 bytes
// per lane and operand, the lane's offset wrapped to the buffer): what the matrix pipes sustain on THESE operand
// values with nothing else in the way (no LDS, no global traffic inside the loop).
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 probe_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float probe_f32x16;
__global__ void __launch_bounds__(256) mfma_rate_kernel(const uint4* __restrict__ ops, size_t n16, int iters, float* __restrict__ sink) {
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  union { uint4 u; probe_bf16x8 v; } a[2], b[2];
  a[0].u = ops[(4 * t) % n16]; a[1].u = ops[(4 * t + 1) % n16];
  b[0].u = ops[(4 * t + 2) % n16]; b[1].u = ops[(4 * t + 3) % n16];
  probe_f32x16 acc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[c][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c & 1].v, b[(c >> 1) & 1].v, acc[c], 0, 0, 0);
  }
  float r = 0.f;
#pragma unroll
  for (int c = 0; c < 8; ++c)
#pragma unroll
    for (int e = 0; e < 16; ++e) r += acc[c][e];
  if (r == 12345.678f) sink[0] = r;      // keeps the loop alive; practically never taken
}
}  // namespace

}  // namespace saap

using namespace saap;

extern "C" int32_t saap_stream_read_probe(const void* src, size_t bytes, void* sink, size_t sink_bytes, void* stream) {
  begin_call();
  if (!src || !sink || !aligned16(src) || !aligned16(sink) || bytes < 16) return SAAP_INVALID_ARG;
  // one workgroup of eight waves per compute unit: the shape that read fastest in a sweep of 128-512 threads
  // and 1-16 workgroups per compute unit (7.1 TB/s; 5.7-6.5 with more waves per compute unit)
  const unsigned grid = (unsigned)(device_cus() * env_int("SAAP_PROBE_WGS_PER_CU", 1));
  if (sink_bytes < (size_t)grid * sizeof(uint32_t)) return SAAP_WORKSPACE_TOO_SMALL;
  hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3((unsigned)env_int("SAAP_PROBE_THREADS", 512)), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint4*>(src), bytes / 16, static_cast<uint32_t*>(sink));
  return launch_status();
}

extern "C" int32_t saap_mfma_rate_probe(const void* operands, size_t bytes, int32_t iters, int32_t wgs_per_cu, void* sink,
                                        double* flop_out, void* stream) {
  begin_call();
  if (!operands || !sink || !aligned16(operands) || bytes < 64 || iters <= 0 || iters > (1 << 24) || wgs_per_cu <= 0 ||
      wgs_per_cu > 8)
    return SAAP_INVALID_ARG;
  const unsigned grid = (unsigned)(device_cus() * wgs_per_cu);
  if (flop_out) *flop_out = (double)grid * 4.0 * iters * 8.0 * (2.0 * 32 * 32 * 16);
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint4*>(operands), bytes / 16, (int)iters, static_cast<float*>(sink));
  return launch_status();
}

extern "C" size_t saap_workspace_bytes(int32_t op, const saap_shape* sh) {
  if (!sh) return 0;
  const long long S = sh->S, Hq = sh->Hq, Hkv = sh->Hkv;
  switch (op) {
    case SAAP_OP_SPARSE_DECODE_ATTENTION: {
      if (S <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv) return 0;
      const bool indep = sh->mode == SAAP_INDEPENDENT;
      return attn_workspace_bytes(indep ? S * Hq : S * Hkv, indep ? 1 : (int)(Hq / Hkv));
    }
    case SAAP_OP_PLANNED_DECODE_ATTENTION: {
      if (S <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv) return 0;
      const bool indep = sh->mode == SAAP_INDEPENDENT;
      return planned_workspace_bytes(indep ? S * Hq : S * Hkv, indep ? 1 : (int)(Hq / Hkv));
    }
    case SAAP_OP_PREFILL_SPARSE_ATTENTION:
      if (S <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv || sh->N <= 0 || sh->nprobe < 0) return 0;
      return prefill_workspace_bytes(S, sh->N, (int)Hq, (int)Hkv, sh->nprobe);
    case SAAP_OP_DENSE_DECODE_ATTENTION:
      if (S <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv) return 0;
      return attn_workspace_bytes(S * Hkv, (int)(Hq / Hkv));
    case SAAP_OP_ASSIGN_KEYS:
      if (S <= 0 || Hkv <= 0 || sh->N <= 0) return 0;
      return assign_workspace_bytes(S * Hkv * (long long)sh->N);
    case SAAP_OP_BUILD_BUCKET_INDEX:
      if (S <= 0 || Hkv <= 0 || sh->N <= 0 || sh->B <= 0) return 0;
      return build_workspace_bytes(S * Hkv, sh->N, sh->B);
    case SAAP_OP_CLASSIFY_QUERIES:
      if (S <= 0 || Hq <= 0 || sh->hidden < 0) return 0;
      return classify_workspace_bytes(S * Hq, sh->hidden);
    case SAAP_OP_WINDOW_PUSH:
    case SAAP_OP_APPEND_KEYS:
      if (S <= 0 || Hkv <= 0 || sh->B <= 0) return 0;
      return push_workspace_bytes(S * Hkv, sh->B);
    case SAAP_OP_SELECT_BUCKETS:
      return SAAP_WS_HEADER_BYTES;
    case SAAP_OP_QUERY_MODEL_LOSS_GRADS:
      if (Hkv <= 0 || sh->N <= 0 || sh->d <= 0 || sh->hidden <= 0 || sh->B <= 0) return 0;
      return train_workspace_bytes(Hkv, sh->N, sh->d, sh->hidden, sh->B);
    case SAAP_OP_BUCKET_ATTENTION_MASS_BATCH:
      if (S <= 0 || Hkv <= 0 || sh->N <= 0 || sh->B <= 0) return 0;
      return mass_batch_workspace_bytes(S * Hkv, sh->N, sh->B);
    case SAAP_OP_BUCKET_ATTENTION_MASS:
      if (S <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv || sh->B <= 0) return 0;
      return mass_workspace_bytes(S * Hkv, (int)(Hq / Hkv), sh->B);
    default:
      return 0;
  }
}

extern "C" int32_t saap_workspace_reset(void* ws, size_t ws_bytes, void* stream) {
  begin_call();
  if (!ws || !aligned16(ws) || ws_bytes < SAAP_WS_HEADER_BYTES) return SAAP_INVALID_ARG;
  const size_t n = SAAP_WS_HEADER_BYTES / sizeof(uint32_t);
  hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<uint32_t*>(ws), n);
  return launch_status();
}

extern "C" const char* saap_status_string(int32_t status) {
  switch (status) {
    case SAAP_OK: return "ok";
    case SAAP_INVALID_ARG: return "invalid argument";
    case SAAP_UNSUPPORTED: return "unsupported dtype, head size, group size or size limit";
    case SAAP_WORKSPACE_TOO_SMALL: return "workspace too small";
    case SAAP_BUCKET_FULL: return "bucket full";
    case SAAP_HIP_ERROR: return "HIP runtime error";
    default: return "unknown status";
  }
}

extern "C" int32_t saap_device_compute_units(void) {
  begin_call();
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return -1;
  return prop.multiProcessorCount;
}
