// bucket_attention_mass: the share of a query's softmax attention that falls into each bucket,
//   mass[b] = sum over the member keys n of bucket b of softmax_n(scale * <q, k_n>)
// with the softmax taken over ALL keys of the (sequence, KV head).  This is the row of A * H_k
// that the query model f_q is trained towards (Section 4 "Learning the query assignment", Eq. 1
// of arXiv 2502.08246); summed over a selection it is the attention mass the selection captures.
//
// Two kernels over the bucket-sorted cache (only K is read, 256 bytes per bf16 key):
//   * partial: a wave takes whole buckets (contiguous runs of rows); 16 lanes read one row with
//     one 16-byte load each, eight rows per group in flight; per bucket and head it keeps the
//     maximum m of t = log2(e) * scale * <q,k> and s = sum 2^(t - m), and writes (m, s);
//   * normalise: per query head, M = max_b m_b, L = sum_b s_b 2^(m_b - M), mass_b = s_b 2^(m_b - M) / L.
#include "common.h"

namespace saap {
namespace {

constexpr int kMassThreads = 256;
constexpr int kInFlight = 8;      // rows a 16-lane group has in flight

template <typename T, int G>
__global__ void __launch_bounds__(kMassThreads)
mass_partial_kernel(const T* __restrict__ q, const T* __restrict__ K, const int32_t* __restrict__ off,
                    const int32_t* __restrict__ len, float2* __restrict__ part, long long rows, int B,
                    float scale_log2) {
  const int unit = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane & 15, grp = lane >> 4;
  Vec8<T> qv[G];
#pragma unroll
  for (int g = 0; g < G; ++g) qv[g].load(q + ((size_t)unit * G + g) * kD + sub * 8);
  const T* Kb = K + (size_t)unit * rows * kD + sub * 8;
  const int n_waves = gridDim.x * (kMassThreads / 64);
  for (int b = blockIdx.x * (kMassThreads / 64) + wave; b < B; b += n_waves) {
    const int first = off[(size_t)unit * (B + 1) + b], n = len[(size_t)unit * B + b];
    float m[G], s[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      m[g] = kNegBig;
      s[g] = 0.f;
    }
    for (int r0 = grp; r0 < n; r0 += 4 * kInFlight) {      // rows r0, r0+4, ... of this 16-lane group
      Vec8<T> kv[kInFlight];
#pragma unroll
      for (int u = 0; u < kInFlight; ++u) kv[u].load(Kb + (size_t)(first + min(r0 + 4 * u, n - 1)) * kD);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float t[kInFlight];
        float bm = -INFINITY;
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
          const float d = sum16(kv[u].dot(qv[g])) * scale_log2;
          t[u] = r0 + 4 * u < n ? d : -INFINITY;
          bm = fmaxf(bm, t[u]);                           // finite: row r0 is real
        }
        const float mn = fmaxf(m[g], bm);
        float acc = s[g] * fast_exp2(m[g] - mn);
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) acc += fast_exp2(t[u] - mn);
        s[g] = acc;
        m[g] = mn;
      }
    }
    // the four groups of the wave
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float M = max_rows(m[g]);
      const float S = sum_rows(s[g] * fast_exp2(m[g] - M));
      if (lane == 0) part[((size_t)unit * B + b) * G + g] = make_float2(M, S);
    }
  }
}

template <int G>
__global__ void __launch_bounds__(256)
mass_normalise_kernel(const float2* __restrict__ part, float* __restrict__ mass, float* __restrict__ lse, int B) {
  __shared__ float s_red[4];
  const int row = blockIdx.x, unit = row / G, g = row % G, tid = threadIdx.x;
  const float2* pu = part + (size_t)unit * B * G + g;
  float M = kNegBig;
  for (int b = tid; b < B; b += 256) M = fmaxf(M, pu[(size_t)b * G].x);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
  if ((tid & 63) == 0) s_red[tid >> 6] = M;
  __syncthreads();
  M = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
  __syncthreads();
  float L = 0.f;
  for (int b = tid; b < B; b += 256) {
    const float2 p = pu[(size_t)b * G];
    L = fmaf(p.y, fast_exp2(p.x - M), L);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) L += __shfl_xor(L, o);
  if ((tid & 63) == 0) s_red[tid >> 6] = L;
  __syncthreads();
  L = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
  const float inv = L > 0.f ? 1.0f / L : 0.f;
  for (int b = tid; b < B; b += 256) {
    const float2 p = pu[(size_t)b * G];
    mass[(size_t)row * B + b] = p.y * fast_exp2(p.x - M) * inv;
  }
  if (tid == 0 && lse) lse[row] = L > 0.f ? (M + __log2f(L)) * kLn2 : -INFINITY;
}

template <typename T, int G>
void launch_mass(const void* q, const void* K, const int32_t* off, const int32_t* len, float2* part, float* mass,
                 float* lse, long long units, long long rows, int B, float scale_log2, hipStream_t hs) {
  const int cus = device_cus();
  // enough workgroups per unit to fill the chip a few times, never more waves than buckets
  long long per_unit = ((long long)cus * 8 + units - 1) / units;
  const long long by_buckets = (B + kMassThreads / 64 - 1) / (kMassThreads / 64);
  if (per_unit > by_buckets) per_unit = by_buckets;
  hipLaunchKernelGGL((mass_partial_kernel<T, G>), dim3((unsigned)per_unit, (unsigned)units), dim3(kMassThreads), 0, hs,
                     static_cast<const T*>(q), static_cast<const T*>(K), off, len, part, rows, B, scale_log2);
  hipLaunchKernelGGL(mass_normalise_kernel<G>, dim3((unsigned)(units * G)), dim3(256), 0, hs, part, mass, lse, B);
}

}  // namespace

size_t mass_workspace_bytes(long long units, int G, int B) {
  return (size_t)SAAP_WS_HEADER_BYTES + (size_t)units * B * G * sizeof(float2);
}

}  // namespace saap

using namespace saap;

extern "C" int32_t saap_bucket_attention_mass(const void* q, const void* Ksorted, const int32_t* off,
                                              const int32_t* len, float scale, float* mass, float* lse, int32_t S,
                                              int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t B, int32_t d,
                                              int32_t dtype, void* ws, size_t ws_bytes, void* stream) {
  if (!q || !Ksorted || !off || !len || !mass || !ws) return SAAP_INVALID_ARG;
  if (!aligned16(q) || !aligned16(Ksorted) || !aligned16(ws)) return SAAP_INVALID_ARG;
  if (S <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || Ncap <= 0 || B <= 0) return SAAP_INVALID_ARG;
  if (dtype != SAAP_F32 && dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  if (d != kD) return SAAP_UNSUPPORTED;
  const int G = Hq / Hkv;
  if (G != 1 && G != 2 && G != 4 && G != 8) return SAAP_UNSUPPORTED;
  const long long units = (long long)S * Hkv;
  if (units > 65535) return SAAP_UNSUPPORTED;
  if (ws_bytes < mass_workspace_bytes(units, G, B)) return SAAP_WORKSPACE_TOO_SMALL;
  float2* part = reinterpret_cast<float2*>(static_cast<char*>(ws) + SAAP_WS_HEADER_BYTES);
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const float sl2 = scale * kLog2e;
#define SAAP_CASE(TT, GG) launch_mass<TT, GG>(q, Ksorted, off, len, part, mass, lse, units, Ncap, B, sl2, hs); break
  if (dtype == SAAP_BF16) {
    switch (G) {
      case 1: SAAP_CASE(bf16_t, 1);
      case 2: SAAP_CASE(bf16_t, 2);
      case 4: SAAP_CASE(bf16_t, 4);
      case 8: SAAP_CASE(bf16_t, 8);
    }
  } else {
    switch (G) {
      case 1: SAAP_CASE(float, 1);
      case 2: SAAP_CASE(float, 2);
      case 4: SAAP_CASE(float, 4);
      case 8: SAAP_CASE(float, 8);
    }
  }
#undef SAAP_CASE
  return launch_status();
}
