// build_bucket_index and append_keys: the CSR index of Appendix F (tensors Off, Idx) of
// arXiv 2502.08246 plus the bucket-sorted copy of K and V, and the slot append used during
// generation.
//
// The sort is a stable counting sort, deterministic by construction (no atomics decide an
// order):
//   1. hist      every workgroup counts the bucket ids of its slice of positions
//   2. colscan   per bucket, exclusive scan of the slice counts over slices -> len, slice bases
//   3. offscan   per (sequence, head), exclusive scan of (len + slack) over buckets -> off
//   4. scatter   one wavefront per slice walks its positions in order, 64 at a time; the rank of
//                a position among equal ids inside the 64 comes from ballots, the running
//                position of every bucket is kept in LDS -> idx
//   5. permute   rows of K and V are copied to their slot, 16 bytes per lane, whole rows
#include "common.h"

namespace saap {
namespace {

constexpr int kSlice = 2048;   // positions per slice (one histogram / one scatter wave each)

__global__ void __launch_bounds__(256)
hist_kernel(const int32_t* __restrict__ ids, int32_t* __restrict__ slice_hist, int N, int B, int n_slices) {
  extern __shared__ int s_cnt[];
  const int slice = blockIdx.x, unit = blockIdx.y;
  for (int b = threadIdx.x; b < B; b += blockDim.x) s_cnt[b] = 0;
  __syncthreads();
  const int n0 = slice * kSlice, n1 = min(n0 + kSlice, N);
  const int32_t* idu = ids + (size_t)unit * N;
  int mine[kSlice / 256];
#pragma unroll
  for (int k = 0; k < kSlice / 256; ++k) {
    const int n = n0 + threadIdx.x + k * 256;
    mine[k] = n < n1 ? idu[n] : -1;
  }
#pragma unroll
  for (int k = 0; k < kSlice / 256; ++k)
    if (mine[k] >= 0 && mine[k] < B) atomicAdd(&s_cnt[mine[k]], 1);
  __syncthreads();
  int32_t* out = slice_hist + ((size_t)unit * n_slices + slice) * B;
  for (int b = threadIdx.x; b < B; b += blockDim.x) out[b] = s_cnt[b];
}

// One thread per (unit, bucket): counts of the slices -> exclusive bases, total -> len.
__global__ void __launch_bounds__(256)
colscan_kernel(int32_t* __restrict__ slice_hist, int32_t* __restrict__ len, int B, int n_slices) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x, unit = blockIdx.y;
  if (b >= B) return;
  int32_t* col = slice_hist + (size_t)unit * n_slices * B + b;
  int run = 0;
  int s = 0;
  for (; s + 8 <= n_slices; s += 8) {
    int c[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) c[i] = col[(size_t)(s + i) * B];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      col[(size_t)(s + i) * B] = run;
      run += c[i];
    }
  }
  for (; s < n_slices; ++s) {
    const int c = col[(size_t)s * B];
    col[(size_t)s * B] = run;
    run += c;
  }
  len[(size_t)unit * B + b] = run;
}

// One workgroup per unit: off[0] = 0, off[b+1] = off[b] + len[b] + slack.
__global__ void __launch_bounds__(1024)
offscan_kernel(const int32_t* __restrict__ len, int32_t* __restrict__ off, int B, int slack) {
  __shared__ int s_wsum[16];
  const int unit = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = (B + blockDim.x - 1) / blockDim.x;
  const int b0 = tid * per, b1 = min(b0 + per, B);
  const int32_t* l = len + (size_t)unit * B;
  int32_t* o = off + (size_t)unit * (B + 1);
  int mine = 0;
  for (int b = b0; b < b1; ++b) mine += l[b] + slack;
  const int incl = (int)wave_prefix_sum((unsigned)mine);
  if (lane == 63) s_wsum[wave] = incl;
  __syncthreads();
  int run = incl - mine;
  for (int w = 0; w < wave; ++w) run += s_wsum[w];
  if (tid == 0) o[0] = 0;
  for (int b = b0; b < b1; ++b) {
    run += l[b] + slack;
    o[b + 1] = run;
  }
}

__global__ void __launch_bounds__(256) fill_i32_kernel(int32_t* p, size_t n, int32_t v) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// One wavefront per slice.  s_next[b] = slot of the next member of bucket b.
__global__ void __launch_bounds__(64)
scatter_kernel(const int32_t* __restrict__ ids, const int32_t* __restrict__ slice_base,
               const int32_t* __restrict__ off, int32_t* __restrict__ idx, int N, int Ncap, int B,
               int n_slices, int id_bits) {
  extern __shared__ int s_next[];
  const int slice = blockIdx.x, unit = blockIdx.y, lane = threadIdx.x;
  const int32_t* base = slice_base + ((size_t)unit * n_slices + slice) * B;
  const int32_t* o = off + (size_t)unit * (B + 1);
  for (int b = lane; b < B; b += 64) s_next[b] = o[b] + base[b];
  __syncthreads();
  const int n0 = slice * kSlice, n1 = min(n0 + kSlice, N);
  const int32_t* idu = ids + (size_t)unit * N;
  int32_t* ix = idx + (size_t)unit * Ncap;
  const unsigned long long below = (1ull << lane) - 1ull;
  int mine[kSlice / 64];       // the wave's ids, loaded up front
#pragma unroll
  for (int k = 0; k < kSlice / 64; ++k) {
    const int n = n0 + k * 64 + lane;
    mine[k] = n < n1 ? idu[n] : -1;
  }
#pragma unroll
  for (int k = 0; k < kSlice / 64; ++k) {
    const int c = n0 + k * 64;
    if (c >= n1) break;
    const int n = c + lane;
    const int b = mine[k];
    const bool ok = b >= 0 && b < B;
    unsigned long long eq = __ballot(ok);
    for (int i = 0; i < id_bits; ++i) {
      const bool bit = (b >> i) & 1;
      const unsigned long long m = __ballot(bit);
      eq &= bit ? m : ~m;
    }
    if (ok) {
      const int rank = __popcll(eq & below);
      const int cnt = __popcll(eq);
      const int slot = s_next[b];
      ix[slot + rank] = n;
      if (rank == cnt - 1) s_next[b] = slot + cnt;
    }
    __syncthreads();   // one wave: orders the LDS update before the next 64 positions
  }
}

// Copy rows into their slots: out[slot] = in[idx[slot]] for member slots.
template <int CHUNKS /* 16-byte pieces per row */>
__global__ void __launch_bounds__(256)
permute_kernel(const uint4* __restrict__ K, const uint4* __restrict__ V, const int32_t* __restrict__ idx,
               uint4* __restrict__ Ks, uint4* __restrict__ Vs, int N, int Ncap, long long total_slots) {
  constexpr int kRowsPerThread = 4;
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const int piece = (int)(t % CHUNKS);
  const long long group = t / CHUNKS;               // handles slots group*4 .. group*4+3
  int src[kRowsPerThread];
  long long slot[kRowsPerThread];
#pragma unroll
  for (int r = 0; r < kRowsPerThread; ++r) {
    slot[r] = group * kRowsPerThread + r;
    src[r] = slot[r] < total_slots ? idx[slot[r]] : -1;
  }
  uint4 kv[kRowsPerThread], vv[kRowsPerThread];
#pragma unroll
  for (int r = 0; r < kRowsPerThread; ++r) {
    if (src[r] >= 0) {
      const long long unit = slot[r] / Ncap;
      const size_t in = ((size_t)unit * N + src[r]) * CHUNKS + piece;
      kv[r] = K[in];
      vv[r] = V[in];
    }
  }
#pragma unroll
  for (int r = 0; r < kRowsPerThread; ++r) {
    if (src[r] >= 0) {
      Ks[(size_t)slot[r] * CHUNKS + piece] = kv[r];
      Vs[(size_t)slot[r] * CHUNKS + piece] = vv[r];
    }
  }
}

// ---- append ------------------------------------------------------------------------------

template <typename T> __device__ __forceinline__ double to_f64(T v);
template <> __device__ __forceinline__ double to_f64<float>(float v) { return (double)v; }
template <> __device__ __forceinline__ double to_f64<bf16_t>(bf16_t v) {
  return (double)__uint_as_float((uint32_t)v << 16);
}

// One workgroup per (sequence, KV head): score the new key against every centroid in double
// precision (in-order sum of exact products), pick the best bucket (lowest id on ties), and
// store the key in the bucket's first free slot.
template <typename T>
__global__ void __launch_bounds__(256)
append_kernel(const T* __restrict__ x_new, const T* __restrict__ k_new, const T* __restrict__ v_new,
              const int32_t* __restrict__ pos_new, const T* __restrict__ cent, const float* __restrict__ bias,
              const int32_t* __restrict__ off, int32_t* __restrict__ len, int32_t* __restrict__ idx,
              T* __restrict__ Ks, T* __restrict__ Vs, int32_t* __restrict__ new_ids,
              int32_t* __restrict__ overflow, int Hkv, int Ncap, int B) {
  __shared__ double s_x[kD];
  __shared__ double s_best[256];
  __shared__ int s_id[256];
  __shared__ int s_slot;
  const int unit = blockIdx.x, h = unit % Hkv, tid = threadIdx.x;
  if (tid < kD) s_x[tid] = to_f64<T>(x_new[(size_t)unit * kD + tid]);
  __syncthreads();
  double best = 0.0;
  int best_id = -1;
  for (int b = tid; b < B; b += blockDim.x) {
    const T* c = cent + ((size_t)h * B + b) * kD;
    double t = 0.0;
    for (int j = 0; j < kD; ++j) t = fma(s_x[j], to_f64<T>(c[j]), t);
    if (bias) t += (double)bias[(size_t)h * B + b];
    if (best_id < 0 || t > best) {
      best = t;
      best_id = b;
    }
  }
  s_best[tid] = best;
  s_id[tid] = best_id;
  __syncthreads();
  for (int s = blockDim.x >> 1; s > 0; s >>= 1) {
    if (tid < s) {
      const int oid = s_id[tid + s];
      const double ob = s_best[tid + s];
      const int mid = s_id[tid];
      if (oid >= 0 && (mid < 0 || ob > s_best[tid] || (ob == s_best[tid] && oid < mid))) {
        s_best[tid] = ob;
        s_id[tid] = oid;
      }
    }
    __syncthreads();
  }
  const int b = s_id[0];
  if (tid == 0) {
    new_ids[unit] = b;
    const int32_t* o = off + (size_t)unit * (B + 1);
    const int cur = len[(size_t)unit * B + b];
    int slot = -1;
    if (o[b] + cur < o[b + 1]) {
      slot = o[b] + cur;
      len[(size_t)unit * B + b] = cur + 1;
      idx[(size_t)unit * Ncap + slot] = pos_new ? pos_new[unit / Hkv] : -2;
    } else {
      *overflow = 1;
    }
    s_slot = slot;
  }
  __syncthreads();
  const int slot = s_slot;
  if (slot >= 0 && tid < kD) {
    Ks[((size_t)unit * Ncap + slot) * kD + tid] = k_new[(size_t)unit * kD + tid];
    Vs[((size_t)unit * Ncap + slot) * kD + tid] = v_new[(size_t)unit * kD + tid];
  }
}

}  // namespace

size_t build_workspace_bytes(long long units, int N, int B) {
  const long long n_slices = (N + kSlice - 1) / kSlice;
  return (size_t)SAAP_WS_HEADER_BYTES + (size_t)units * n_slices * B * sizeof(int32_t);
}

}  // namespace saap

using namespace saap;

extern "C" int32_t saap_build_bucket_index(const int32_t* bucket_ids, const void* K, const void* V,
                                           int32_t* off, int32_t* len, int32_t* idx, void* Ksorted,
                                           void* Vsorted, int32_t S, int32_t Hkv, int32_t N, int32_t Ncap,
                                           int32_t B, int32_t d, int32_t dtype, int32_t slack, void* ws,
                                           size_t ws_bytes, void* stream) {
  if (!bucket_ids || !K || !V || !off || !len || !idx || !Ksorted || !Vsorted || !ws) return SAAP_INVALID_ARG;
  const void* ptrs[] = {bucket_ids, K, V, off, len, idx, Ksorted, Vsorted, ws};
  for (const void* p : ptrs)
    if (!aligned16(p)) return SAAP_INVALID_ARG;
  if (S <= 0 || Hkv <= 0 || N <= 0 || B <= 0 || slack < 0) return SAAP_INVALID_ARG;
  if (dtype != SAAP_F32 && dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  if ((long long)Ncap != (long long)N + (long long)B * slack) return SAAP_INVALID_ARG;
  if (d != kD || B > SAAP_MAX_BUCKETS) return SAAP_UNSUPPORTED;
  const long long units = (long long)S * Hkv;
  if (units > 65535) return SAAP_UNSUPPORTED;
  if (ws_bytes < build_workspace_bytes(units, N, B)) return SAAP_WORKSPACE_TOO_SMALL;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const int n_slices = (N + kSlice - 1) / kSlice;
  int32_t* slice_hist = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + SAAP_WS_HEADER_BYTES);
  int id_bits = 1;
  while ((1 << id_bits) < B) ++id_bits;

  hipLaunchKernelGGL(hist_kernel, dim3(n_slices, (unsigned)units), dim3(256), (size_t)B * sizeof(int), hs,
                     bucket_ids, slice_hist, N, B, n_slices);
  hipLaunchKernelGGL(colscan_kernel, dim3((B + 255) / 256, (unsigned)units), dim3(256), 0, hs, slice_hist, len,
                     B, n_slices);
  hipLaunchKernelGGL(offscan_kernel, dim3((unsigned)units), dim3(1024), 0, hs, len, off, B, slack);
  const size_t n_idx = (size_t)units * Ncap;
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n_idx + 255) / 256)), dim3(256), 0, hs, idx, n_idx, -1);
  hipLaunchKernelGGL(scatter_kernel, dim3(n_slices, (unsigned)units), dim3(64), (size_t)B * sizeof(int), hs,
                     bucket_ids, slice_hist, off, idx, N, Ncap, B, n_slices, id_bits);
  const long long total_slots = units * Ncap;
  if (dtype == SAAP_BF16) {
    const long long threads = (total_slots + 3) / 4 * 16;
    hipLaunchKernelGGL(permute_kernel<16>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, hs,
                       static_cast<const uint4*>(K), static_cast<const uint4*>(V), idx,
                       static_cast<uint4*>(Ksorted), static_cast<uint4*>(Vsorted), N, Ncap, total_slots);
  } else {
    const long long threads = (total_slots + 3) / 4 * 32;
    hipLaunchKernelGGL(permute_kernel<32>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, hs,
                       static_cast<const uint4*>(K), static_cast<const uint4*>(V), idx,
                       static_cast<uint4*>(Ksorted), static_cast<uint4*>(Vsorted), N, Ncap, total_slots);
  }
  return launch_status();
}

extern "C" int32_t saap_append_keys(const void* x_new, const void* k_new, const void* v_new,
                                    const int32_t* pos_new, const void* centroids, const float* bias,
                                    const int32_t* off, int32_t* len, int32_t* idx, void* Ksorted,
                                    void* Vsorted, int32_t* new_bucket_ids, int32_t* overflow_flag, int32_t S,
                                    int32_t Hkv, int32_t Ncap, int32_t B, int32_t d, int32_t dtype,
                                    void* stream) {
  if (!x_new || !k_new || !v_new || !centroids || !off || !len || !idx || !Ksorted || !Vsorted ||
      !new_bucket_ids || !overflow_flag)
    return SAAP_INVALID_ARG;
  if (S <= 0 || Hkv <= 0 || Ncap <= 0 || B <= 0) return SAAP_INVALID_ARG;
  if (dtype != SAAP_F32 && dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  if (d != kD) return SAAP_UNSUPPORTED;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const unsigned units = (unsigned)((long long)S * Hkv);
  if (dtype == SAAP_BF16)
    hipLaunchKernelGGL(append_kernel<bf16_t>, dim3(units), dim3(256), 0, hs,
                       static_cast<const bf16_t*>(x_new), static_cast<const bf16_t*>(k_new),
                       static_cast<const bf16_t*>(v_new), pos_new, static_cast<const bf16_t*>(centroids), bias,
                       off, len, idx, static_cast<bf16_t*>(Ksorted), static_cast<bf16_t*>(Vsorted),
                       new_bucket_ids, overflow_flag, Hkv, Ncap, B);
  else
    hipLaunchKernelGGL(append_kernel<float>, dim3(units), dim3(256), 0, hs, static_cast<const float*>(x_new),
                       static_cast<const float*>(k_new), static_cast<const float*>(v_new), pos_new,
                       static_cast<const float*>(centroids), bias, off, len, idx,
                       static_cast<float*>(Ksorted), static_cast<float*>(Vsorted), new_bucket_ids,
                       overflow_flag, Hkv, Ncap, B);
  return launch_status();
}
