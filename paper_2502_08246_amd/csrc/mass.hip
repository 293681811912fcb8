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

// ---- many queries per KV head (a training batch): scores on the matrix cores -----------------------
// 128 queries per workgroup sit in registers as the B operand of v_mfma_f32_32x32x16_bf16 (32 per
// wave, one lane per query and half of the key rows); the keys of a bucket stream through LDS in
// tiles of 32 as the A operand (padded rows, whole-row loads), so that one lane sees 16 scores of
// its query per tile and keeps the bucket's running maximum and sum for it.  A workgroup takes
// every n_slices-th bucket.  part[(unit*B + b)*R + q] = (m, s).
constexpr int kMassPitch = 136;      // bf16 elements per LDS row (272 bytes: conflict-free b128 reads)
constexpr int kMassQueries = 128;    // queries per workgroup

__global__ void __launch_bounds__(256)
mass_mfma_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ K, const int32_t* __restrict__ off,
                 const int32_t* __restrict__ len, float2* __restrict__ part, long long rows, int B, int R,
                 float scale_log2) {
  typedef __attribute__((ext_vector_type(16))) float f32x16_t;
  __shared__ __align__(16) bf16_t s_k[32 * kMassPitch];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int unit = blockIdx.z;
  const int qi = blockIdx.y * kMassQueries + wave * 32 + col;
  // B operand: lane holds features 16*step + 8*half .. +7 of query `col` (idle columns repeat the last query)
  bf16x8_t xb[8];
  {
    const bf16_t* qr = q + ((size_t)unit * R + min(qi, R - 1)) * kD + half * 8;
#pragma unroll
    for (int st = 0; st < 8; ++st) xb[st] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(qr + st * 16));
  }
  const bf16_t* Ku = K + (size_t)unit * rows * kD;
  for (int b = blockIdx.x; b < B; b += gridDim.x) {
    const int first = off[(size_t)unit * (B + 1) + b], n = len[(size_t)unit * B + b];
    float m = kNegBig, s = 0.f;
    for (int t0 = 0; t0 < n; t0 += 32) {
      __syncthreads();                                   // the previous tile has been read
      // 32 rows x 16 pieces of 16 bytes, two per thread; rows past the bucket repeat its last key
      uint4 piece[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int pi = tid + 256 * i, r = pi >> 4, pc = pi & 15;
        piece[i] = *reinterpret_cast<const uint4*>(Ku + (size_t)(first + min(t0 + r, n - 1)) * kD + pc * 8);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int pi = tid + 256 * i, r = pi >> 4, pc = pi & 15;
        *reinterpret_cast<uint4*>(&s_k[r * kMassPitch + pc * 8]) = piece[i];
      }
      __syncthreads();
      f32x16_t acc = {0};
#pragma unroll
      for (int st = 0; st < 8; ++st) {
        const bf16x8_t a = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(&s_k[col * kMassPitch + st * 16 + half * 8]));
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, xb[st], acc, 0, 0, 0);
      }
      // register r of this lane: key t0 + 8*(r/4) + 4*half + r%4 against query `col`
      float t[16], bm = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = t0 + 8 * (r / 4) + 4 * half + (r % 4);
        t[r] = key < n ? acc[r] * scale_log2 : -INFINITY;
        bm = fmaxf(bm, t[r]);
      }
      const float mn = fmaxf(m, bm);                     // may stay at the stand-in when this half holds no real key
      float add = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) add += fast_exp2(t[r] - mn);
      s = s * fast_exp2(m - mn) + add;
      m = mn;
    }
    // lanes l and l+32 hold the same query
    const float mo = __shfl_xor(m, 32), so = __shfl_xor(s, 32);
    const float M = fmaxf(m, mo);
    const float S = s * fast_exp2(m - M) + so * fast_exp2(mo - M);
    if (half == 0 && qi < R) part[((size_t)unit * B + b) * R + qi] = make_float2(M, S);
  }
}

// mass[(unit*R + q)*B + b] = s_b 2^(m_b - M) / L for 32 queries per workgroup: thread (query, bucket group).
__global__ void __launch_bounds__(256)
mass_normalise_batch_kernel(const float2* __restrict__ part, float* __restrict__ mass, float* __restrict__ lse, int B,
                            int R) {
  __shared__ float s_red[8][32];
  __shared__ float s_tile[32][33];
  const int tid = threadIdx.x, ql = tid & 31, bg = tid >> 5;
  const int unit = blockIdx.y, q0 = blockIdx.x * 32;
  const int qi = min(q0 + ql, R - 1);
  const float2* pu = part + (size_t)unit * B * R + qi;
  float M = kNegBig;
  for (int b = bg; b < B; b += 8) M = fmaxf(M, pu[(size_t)b * R].x);
  s_red[bg][ql] = M;
  __syncthreads();
#pragma unroll
  for (int g = 0; g < 8; ++g) M = fmaxf(M, s_red[g][ql]);
  __syncthreads();
  float L = 0.f;
  for (int b = bg; b < B; b += 8) {
    const float2 p = pu[(size_t)b * R];
    L = fmaf(p.y, fast_exp2(p.x - M), L);
  }
  s_red[bg][ql] = L;
  __syncthreads();
  L = 0.f;
#pragma unroll
  for (int g = 0; g < 8; ++g) L += s_red[g][ql];           // fixed order
  const float inv = L > 0.f ? 1.0f / L : 0.f;
  if (bg == 0 && q0 + ql < R && lse) lse[(size_t)unit * R + q0 + ql] = L > 0.f ? (M + __log2f(L)) * kLn2 : -INFINITY;
  // tiles of 32 queries x 32 buckets go through LDS so that the rows of `mass` are written in whole lines
  for (int bt = 0; bt < B; bt += 32) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int bb = bg * 4 + i, b = bt + bb;
      float v = 0.f;
      if (b < B) {
        const float2 p = pu[(size_t)b * R];
        v = p.y * fast_exp2(p.x - M) * inv;
      }
      s_tile[ql][bb] = v;
    }
    __syncthreads();
    const int row = tid >> 3, seg = tid & 7;
    if (q0 + row < R) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int b = bt + seg * 4 + i;
        if (b < B) mass[((size_t)unit * R + q0 + row) * B + b] = s_tile[row][seg * 4 + i];
      }
    }
  }
}

}  // namespace

size_t mass_batch_workspace_bytes(long long units, long long R, int B) {
  return (size_t)SAAP_WS_HEADER_BYTES + (size_t)units * R * B * sizeof(float2);
}

size_t mass_workspace_bytes(long long units, int G, int B) {
  return (size_t)SAAP_WS_HEADER_BYTES + (size_t)units * B * G * sizeof(float2);
}

}  // namespace saap

using namespace saap;

extern "C" int32_t saap_bucket_attention_mass(const void* q, const void* Ksorted, const int32_t* off,
                                              const int32_t* len, float scale, float* mass, float* lse, int32_t S,
                                              int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t B, int32_t d,
                                              int32_t dtype, void* ws, size_t ws_bytes, void* stream) {
  begin_call();
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

extern "C" int32_t saap_bucket_attention_mass_batch(const void* q, const void* Ksorted, const int32_t* off,
                                                    const int32_t* len, float scale, float* mass, float* lse,
                                                    int32_t S, int32_t Hkv, int32_t R, int32_t Ncap, int32_t B,
                                                    int32_t d, int32_t dtype, void* ws, size_t ws_bytes,
                                                    void* stream) {
  begin_call();
  if (!q || !Ksorted || !off || !len || !mass || !ws) return SAAP_INVALID_ARG;
  if (!aligned16(q) || !aligned16(Ksorted) || !aligned16(mass) || !aligned16(ws)) return SAAP_INVALID_ARG;
  if (S <= 0 || Hkv <= 0 || R <= 0 || Ncap <= 0 || B <= 0) return SAAP_INVALID_ARG;
  if (dtype != SAAP_F32 && dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  if (d != kD || dtype != SAAP_BF16) return SAAP_UNSUPPORTED;
  const long long units = (long long)S * Hkv;
  if (units > 65535 || (R + kMassQueries - 1) / kMassQueries > 65535) return SAAP_UNSUPPORTED;
  if (ws_bytes < mass_batch_workspace_bytes(units, R, B)) return SAAP_WORKSPACE_TOO_SMALL;
  float2* part = reinterpret_cast<float2*>(static_cast<char*>(ws) + SAAP_WS_HEADER_BYTES);
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const int qblocks = (R + kMassQueries - 1) / kMassQueries;
  // bucket slices: enough workgroups to fill the chip a few times, never more than buckets
  long long slices = ((long long)device_cus() * 4 + units * qblocks - 1) / (units * qblocks);
  if (slices > B) slices = B;
  if (slices < 1) slices = 1;
  hipLaunchKernelGGL(mass_mfma_kernel, dim3((unsigned)slices, (unsigned)qblocks, (unsigned)units), dim3(256), 0, hs,
                     static_cast<const bf16_t*>(q), static_cast<const bf16_t*>(Ksorted), off, len, part, (long long)Ncap,
                     B, R, scale * kLog2e);
  hipLaunchKernelGGL(mass_normalise_batch_kernel, dim3((unsigned)((R + 31) / 32), (unsigned)units), dim3(256), 0, hs, part,
                     mass, lse, B, R);
  return launch_status();
}
