// select_buckets: the nprobe highest-scoring buckets per KV head (Section 4; Section 5
// "Batched queries" of arXiv 2502.08246: the classifier outputs of the G heads that share a
// KV head are summed and one top-nprobe list is taken).
//
// One workgroup per list.  Every bucket becomes a 64-bit key
//     (order-preserving image of the fp32 score) << 32 | (0xFFFFFFFF - bucket id)
// so keys are unique and "larger key" means (higher score, then lower id).  The keys are
// sorted in LDS with a bitonic network and the first nprobe ids are written out, which is
// exactly the (score descending, id ascending) order of the definition and is deterministic.
#include "common.h"

namespace saap {
namespace {

__global__ void __launch_bounds__(1024)
select_kernel(const float* __restrict__ scores, int32_t* __restrict__ selected, int Hq, int Hkv, int B,
              int nprobe, int independent, int n_pow2) {
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned long long* keys = reinterpret_cast<unsigned long long*>(smem);
  const int unit = blockIdx.x;
  const int G = Hq / Hkv;
  const int heads = independent ? 1 : G;
  // first score row of the list: (s, hq) for independent lists, (s, h*G) for group lists
  const size_t row0 = independent ? (size_t)unit : (size_t)unit * G;
  const float* sc = scores + row0 * B;

  for (int b = threadIdx.x; b < n_pow2; b += blockDim.x) {
    unsigned long long key = 0ull;   // padding sorts below every finite score
    if (b < B) {
      float g = sc[b];
      for (int i = 1; i < heads; ++i) g = g + sc[(size_t)i * B + b];   // fp32, head order
      g = g + 0.0f;                                                    // -0 -> +0
      key = ((unsigned long long)float_order_key(g) << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)b);
    }
    keys[b] = key;
  }
  __syncthreads();

  for (int k = 2; k <= n_pow2; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int i = threadIdx.x; i < n_pow2; i += blockDim.x) {
        const int x = i ^ j;
        if (x > i) {
          const unsigned long long a = keys[i], c = keys[x];
          const bool descending = (i & k) == 0;
          if (descending ? (a < c) : (a > c)) {
            keys[i] = c;
            keys[x] = a;
          }
        }
      }
      __syncthreads();
    }
  }

  for (int j = threadIdx.x; j < nprobe; j += blockDim.x)
    selected[(size_t)unit * nprobe + j] = (int32_t)(0xFFFFFFFFu - (unsigned)(keys[j] & 0xFFFFFFFFull));
}

}  // namespace
}  // namespace saap

using namespace saap;

extern "C" int32_t saap_select_buckets(const float* scores, int32_t* selected, int32_t S, int32_t Hq,
                                       int32_t Hkv, int32_t B, int32_t nprobe, int32_t mode, void* ws,
                                       size_t ws_bytes, void* stream) {
  (void)ws;
  (void)ws_bytes;
  if (!scores || !aligned16(scores)) return SAAP_INVALID_ARG;
  if (S <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || B <= 0) return SAAP_INVALID_ARG;
  if (mode != SAAP_GROUP_SUM && mode != SAAP_INDEPENDENT) return SAAP_INVALID_ARG;
  if (nprobe < 0 || nprobe > B) return SAAP_INVALID_ARG;
  if (B > SAAP_MAX_BUCKETS) return SAAP_UNSUPPORTED;
  if (nprobe == 0) return SAAP_OK;
  if (!selected || !aligned16(selected)) return SAAP_INVALID_ARG;
  int n_pow2 = 2;
  while (n_pow2 < B) n_pow2 <<= 1;
  int threads = n_pow2 / 2;
  if (threads < 64) threads = 64;
  if (threads > 1024) threads = 1024;
  const long long units = mode == SAAP_INDEPENDENT ? (long long)S * Hq : (long long)S * Hkv;
  const size_t lds = (size_t)n_pow2 * sizeof(unsigned long long);
  if (lds > 48 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return SAAP_HIP_ERROR;
  }
  hipLaunchKernelGGL(select_kernel, dim3((unsigned)units), dim3((unsigned)threads), lds,
                     static_cast<hipStream_t>(stream), scores, selected, Hq, Hkv, B, nprobe,
                     mode == SAAP_INDEPENDENT ? 1 : 0, n_pow2);
  return launch_status();
}
