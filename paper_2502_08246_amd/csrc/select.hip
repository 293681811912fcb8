// select_buckets: the nprobe highest-scoring buckets per KV head (Section 4; Section 5
// "Batched queries" of arXiv 2502.08246: the classifier outputs of the G heads that share a
// KV head are summed and one top-nprobe list is taken).
//
// One workgroup per list.  Every bucket becomes a 64-bit key
//     (order-preserving image of the fp32 score) << 32 | (0xFFFFFFFF - bucket id)
// so keys are unique and "larger key" means (higher score, then lower id).
//   * radix kernel (nprobe well below B): a most-significant-digit radix select over the 32-bit
//     score images (four passes of 8 bits, LDS histogram + one-wave scan) finds the score of the
//     nprobe-th bucket; buckets above it, and the lowest-id buckets equal to it, are compacted
//     and only those nprobe keys are put in order (by counting larger keys for lists up to
//     1024, by a bitonic network beyond).
//   * sort kernel (nprobe close to B): all keys are sorted in LDS with a bitonic network.
// Both give exactly the (score descending, id ascending) order of the definition.
#include "select_body.h"

namespace saap {
namespace {

__global__ void __launch_bounds__(1024)
select_kernel(const float* __restrict__ scores, int32_t* __restrict__ selected, int Hq, int Hkv, int B,
              int nprobe, int independent, int n_pow2, PlanOut po) {
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
      const float g = group_score(sc, heads, B, b);
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
  if (po.off) {
    // the ordered ids replace the sorted keys in LDS; lengths and first rows come from memory (this
    // kernel serves lists that take most of the buckets, where the attention dwarfs the selection)
    int* ids = reinterpret_cast<int*>(keys + n_pow2);
    for (int j = threadIdx.x; j < nprobe; j += blockDim.x) ids[j] = (int)(0xFFFFFFFFu - (unsigned)(keys[j] & 0xFFFFFFFFull));
    __syncthreads();
    const int kvu = independent ? (unit / Hq) * Hkv + (unit % Hq) / G : unit;
    emit_plan(ids, po.len + (size_t)kvu * po.runs, po.off + (size_t)kvu * (po.runs + 1), nprobe, po.resident,
              po.plan + (size_t)unit * po.ps);
  }
}


// max / sum over the 64 lanes of a wave on DPP and row swaps (no LDS crossbar); every lane gets it
template <int EPT, bool LOGITS>
__global__ void __launch_bounds__(1024)
select_radix_kernel(const float* __restrict__ scores, float* __restrict__ probs, int32_t* __restrict__ selected,
                    int Hq, int Hkv, int B, int nprobe, int independent, int n_sort, int cap, PlanOut po) {
  extern __shared__ __align__(16) unsigned char smem[];
  select_radix_body<EPT, LOGITS, false>(smem, (int)blockIdx.x, scores, probs, selected, Hq, Hkv, B, nprobe, independent,
                                        n_sort, cap, po);
}

}  // namespace
}  // namespace saap

using namespace saap;

// Shared body: `logits` false selects from `scores` as given; true applies the row softmax first
// (and writes the probabilities to `probs` if it is not null).
static int32_t select_impl(const float* scores, bool logits, float* probs, int32_t* selected, int32_t S,
                           int32_t Hq, int32_t Hkv, int32_t B, int32_t nprobe, int32_t mode, void* stream,
                           PlanOut po = PlanOut{}) {
  if (!scores || !aligned16(scores) || !aligned16(probs)) return SAAP_INVALID_ARG;
  if (S <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || B <= 0) return SAAP_INVALID_ARG;
  if (mode != SAAP_GROUP_SUM && mode != SAAP_INDEPENDENT) return SAAP_INVALID_ARG;
  if (nprobe < 0 || nprobe > B) return SAAP_INVALID_ARG;
  if (B > SAAP_MAX_BUCKETS) return SAAP_UNSUPPORTED;
  if (logits && mode == SAAP_GROUP_SUM) {
    const int G = Hq / Hkv;
    if (G != 1 && G != 2 && G != 4 && G != 8) return SAAP_UNSUPPORTED;
  }
  if (nprobe == 0)
    return po.off ? saap_build_visit_plan(nullptr, po.off, po.len, 0, mode, po.resident, po.plan, S, Hq, Hkv, po.runs, stream)
                  : SAAP_OK;
  if (!selected || !aligned16(selected)) return SAAP_INVALID_ARG;
  int n_pow2 = 2;
  while (n_pow2 < B) n_pow2 <<= 1;
  int n_sort = 2;
  while (n_sort < nprobe) n_sort <<= 1;
  const long long units = mode == SAAP_INDEPENDENT ? (long long)S * Hq : (long long)S * Hkv;
  const int indep = mode == SAAP_INDEPENDENT ? 1 : 0;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  if (logits && !(n_sort < n_pow2)) return SAAP_UNSUPPORTED;     // the fused softmax lives in the radix kernel
  if (n_sort < n_pow2 && (logits || env_int("SAAP_SELECT_FULL_SORT", 0) == 0)) {
    // radix select + sort of the selected keys only
    // elements per thread: 2 up to 1024 buckets, 4 up to 4096 (measured: 512 threads are best at 1024
    // and at 2048 buckets; more waves with loads in flight pull the score rows in faster, up to the
    // point where the barriers of a larger workgroup cost more), then 8
    int ept = env_int("SAAP_SELECT_EPT", 0);
    if (ept != 1 && ept != 2 && ept != 4 && ept != 8) ept = B <= 1024 ? 2 : B <= 4096 ? 4 : 8;
    while (ept < 8 && (long long)ept * 1024 < B) ept *= 2;
    int threads = (B + ept - 1) / ept;
    threads = (threads + 63) / 64 * 64;
    if (threads > 1024) threads = 1024;
    const SelectGeometry geo = select_geometry(B, nprobe, po.off != nullptr, po.runs);
    const int cap = geo.cap;
    const size_t lds = geo.lds;
    po.lds_off = geo.plan_off;
    const bool big_lds = lds > 48 * 1024;
    saap_trace_arm();
    const dim3 grid((unsigned)units), block((unsigned)threads);
#define SAAP_SELECT_LAUNCH(E, L)                                                                             \
  do {                                                                                                       \
    auto kern = select_radix_kernel<E, L>;                                                                   \
    if (big_lds && hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                  \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)  \
      return SAAP_HIP_ERROR;                                                                                 \
    hipLaunchKernelGGL(kern, grid, block, lds, hs, scores, probs, selected, Hq, Hkv, B, nprobe, indep, n_sort, cap, po); \
  } while (0)
#define SAAP_SELECT_CASE(E)                                                                                  \
  case E:                                                                                                    \
    if (logits)                                                                                              \
      SAAP_SELECT_LAUNCH(E, true);                                                                           \
    else                                                                                                     \
      SAAP_SELECT_LAUNCH(E, false);                                                                          \
    break
    switch (ept) {
      SAAP_SELECT_CASE(1);
      SAAP_SELECT_CASE(2);
      SAAP_SELECT_CASE(4);
      default: SAAP_SELECT_CASE(8);
    }
#undef SAAP_SELECT_CASE
#undef SAAP_SELECT_LAUNCH
    return launch_status();
  }
  int threads = n_pow2 / 2;
  if (threads < 64) threads = 64;
  if (threads > 1024) threads = 1024;
  const size_t lds = (size_t)n_pow2 * sizeof(unsigned long long) + (po.off ? (size_t)nprobe * sizeof(int) : 0);
  if (lds > 48 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return SAAP_HIP_ERROR;
  }
  hipLaunchKernelGGL(select_kernel, dim3((unsigned)units), dim3((unsigned)threads), lds, hs, scores, selected, Hq,
                     Hkv, B, nprobe, indep, n_pow2, po);
  return launch_status();
}

extern "C" int32_t saap_select_buckets(const float* scores, int32_t* selected, int32_t S, int32_t Hq,
                                       int32_t Hkv, int32_t B, int32_t nprobe, int32_t mode, void* ws,
                                       size_t ws_bytes, void* stream) {
  begin_call();
  (void)ws;
  (void)ws_bytes;
  return select_impl(scores, false, nullptr, selected, S, Hq, Hkv, B, nprobe, mode, stream);
}

extern "C" int32_t saap_select_buckets_from_logits(const float* logits, float* probs, int32_t* selected,
                                                   int32_t S, int32_t Hq, int32_t Hkv, int32_t B,
                                                   int32_t nprobe, int32_t mode, void* ws, size_t ws_bytes,
                                                   void* stream) {
  begin_call();
  (void)ws;
  (void)ws_bytes;
  if (!logits) return SAAP_INVALID_ARG;
  return select_impl(logits, true, probs, selected, S, Hq, Hkv, B, nprobe, mode, stream);
}

extern "C" int32_t saap_select_buckets_planned(const float* scores, int32_t input_kind, float* probs,
                                               const int32_t* off, const int32_t* len, int32_t resident_run,
                                               int32_t* selected, int32_t* plan, int32_t S, int32_t Hq,
                                               int32_t Hkv, int32_t B, int32_t nprobe, int32_t mode, void* ws,
                                               size_t ws_bytes, void* stream) {
  begin_call();
  (void)ws;
  (void)ws_bytes;
  if (!off || !len || !plan || !aligned16(plan)) return SAAP_INVALID_ARG;
  if (input_kind != SAAP_PROBS && input_kind != SAAP_LOGITS) return SAAP_INVALID_ARG;
  if (resident_run != -1 && resident_run != B) return SAAP_INVALID_ARG;
  if (nprobe + (resident_run >= 0 ? 1 : 0) > SAAP_MAX_BUCKETS) return SAAP_UNSUPPORTED;
  PlanOut po{};
  po.off = off; po.len = len; po.plan = plan;
  po.runs = B + (resident_run >= 0 ? 1 : 0);
  po.resident = resident_run;
  po.ps = (2 * (nprobe + (resident_run >= 0 ? 1 : 0)) + 2 + 3) & ~3;
  return select_impl(scores, input_kind == SAAP_LOGITS, input_kind == SAAP_LOGITS ? probs : nullptr, selected, S, Hq,
                     Hkv, B, nprobe, mode, stream, po);
}
