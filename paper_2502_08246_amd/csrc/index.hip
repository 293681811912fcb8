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
//
// With a resident block (attention sink + recent keys, Section 3 "Per-head attention span")
// only the positions [lo, hi) go through steps 1-4; the resident positions are placed by
// their slot rule into one more run behind the B buckets, and window_push moves one key per
// decode step from that run into its bucket.
#include "common.h"

namespace saap {
namespace {

constexpr int kSlice = 2048;   // positions per slice (one histogram / one scatter wave each)

__global__ void __launch_bounds__(256)
hist_kernel(const int32_t* __restrict__ ids, int32_t* __restrict__ slice_hist, int N, int B, int n_slices,
            int lo, int hi) {
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
    mine[k] = n < n1 && n >= lo && n < hi ? idu[n] : -1;
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
colscan_kernel(int32_t* __restrict__ slice_hist, int32_t* __restrict__ len, int B, int n_slices, int lstride) {
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
  len[(size_t)unit * lstride + b] = run;
}

// One workgroup per unit: off[0] = 0, off[b+1] = off[b] + len[b] + slack.  With a resident
// block (W >= 0) len has B+1 and off B+2 entries per unit: len[B] = n_res, off[B+1] = off[B] + W.
__global__ void __launch_bounds__(1024)
offscan_kernel(int32_t* __restrict__ len, int32_t* __restrict__ off, int B, int slack, int W, int n_res) {
  __shared__ int s_wsum[16];
  const int unit = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = (B + blockDim.x - 1) / blockDim.x;
  const int b0 = tid * per, b1 = min(b0 + per, B);
  const int lstride = W >= 0 ? B + 1 : B;
  int32_t* l = len + (size_t)unit * lstride;
  int32_t* o = off + (size_t)unit * (lstride + 1);
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
    if (W >= 0 && b == B - 1) {
      o[B + 1] = run + W;
      l[B] = n_res;
    }
  }
}

// Resident keys of a unit: position -> slot of the resident run, ids kept for the later move.
__global__ void __launch_bounds__(256)
resident_kernel(const int32_t* __restrict__ ids, const int32_t* __restrict__ off, int32_t* __restrict__ idx,
                int32_t* __restrict__ res_ids, int N, int Ncap, int B, int n_sink, int n_recent, int n_res) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x, unit = blockIdx.y;
  const int W = n_sink + n_recent;
  if (j >= W) return;
  int32_t* rid = res_ids + (size_t)unit * W;
  if (j >= n_res) {              // slot r(p) = p while the block is not full: slots n_res.. are empty
    rid[j] = -1;
    return;
  }
  // j-th resident position in ascending order
  const int p = (N <= W || j < n_sink) ? j : N - n_recent + (j - n_sink);
  const int r = p < n_sink ? p : n_sink + (p - n_sink) % n_recent;
  const int base = off[(size_t)unit * (B + 2) + B];
  idx[(size_t)unit * Ncap + base + r] = p;
  rid[r] = ids[(size_t)unit * N + p];
}

__global__ void __launch_bounds__(256) fill_i32_kernel(int32_t* p, size_t n, int32_t v) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// One wavefront per slice.  s_next[b] = slot of the next member of bucket b.
__global__ void __launch_bounds__(64)
scatter_kernel(const int32_t* __restrict__ ids, const int32_t* __restrict__ slice_base,
               const int32_t* __restrict__ off, int32_t* __restrict__ idx, int N, int Ncap, int B,
               int n_slices, int id_bits, int lo, int hi, int ostride) {
  extern __shared__ int s_next[];
  const int slice = blockIdx.x, unit = blockIdx.y, lane = threadIdx.x;
  const int32_t* base = slice_base + ((size_t)unit * n_slices + slice) * B;
  const int32_t* o = off + (size_t)unit * ostride;
  // eight pairs of loads in flight per lane: one at a time the 2 * B / 64 dependent round trips took as long as
  // the scatter itself
  for (int b0 = 0; b0 < B; b0 += 64 * 8) {
    int ov[8], bv[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int b = min(b0 + u * 64 + lane, B - 1);
      ov[u] = o[b];
      bv[u] = base[b];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int b = b0 + u * 64 + lane;
      if (b < B) s_next[b] = ov[u] + bv[u];
    }
  }
  __syncthreads();
  const int n0 = slice * kSlice, n1 = min(n0 + kSlice, N);
  const int32_t* idu = ids + (size_t)unit * N;
  int32_t* ix = idx + (size_t)unit * Ncap;
  const unsigned long long below = (1ull << lane) - 1ull;
  int mine[kSlice / 64];       // the wave's ids, loaded up front
#pragma unroll
  for (int k = 0; k < kSlice / 64; ++k) {
    const int n = n0 + k * 64 + lane;
    mine[k] = n < n1 && n >= lo && n < hi ? idu[n] : -1;
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
    // one wave: its LDS accesses execute in order, so the update is seen by the next 64 positions.  No barrier:
    // a barrier also waits for the index store above, one memory round trip per 64 positions
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
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
      kv[r] = stream_load16(K + in);
      vv[r] = stream_load16(V + in);
    }
  }
#pragma unroll
  for (int r = 0; r < kRowsPerThread; ++r) {
    if (src[r] >= 0) {
      stream_store16(Ks + (size_t)slot[r] * CHUNKS + piece, kv[r]);
      stream_store16(Vs + (size_t)slot[r] * CHUNKS + piece, vv[r]);
    }
  }
}

// ---- append ------------------------------------------------------------------------------

template <typename T> __device__ __forceinline__ double to_f64(T v);
template <> __device__ __forceinline__ double to_f64<float>(float v) { return (double)v; }
template <> __device__ __forceinline__ double to_f64<bf16_t>(bf16_t v) {
  return (double)__uint_as_float((uint32_t)v << 16);
}

constexpr int kPushSlab = 64;         // centroids per workgroup (one wave) of window_push_kernel

// Eight bf16 elements (one 16-byte piece of a row) -> double.
__device__ __forceinline__ void widen8(const uint4& u, double* o) {
  o[0] = (double)bf16_lo(u.x); o[1] = (double)bf16_hi(u.x); o[2] = (double)bf16_lo(u.y); o[3] = (double)bf16_hi(u.y);
  o[4] = (double)bf16_lo(u.z); o[5] = (double)bf16_hi(u.z); o[6] = (double)bf16_lo(u.w); o[7] = (double)bf16_hi(u.w);
}

// Score of one centroid row against the key in s_x: the in-order double-precision sum of the
// exact products.  All 16-byte loads of the row (of half a row for fp32) are issued before the
// dependent chain of 128 fused multiply-adds starts.
template <typename T>
__device__ __forceinline__ double score_row(const T* __restrict__ c, const double* __restrict__ s_x);
template <>
__device__ __forceinline__ double score_row<bf16_t>(const bf16_t* __restrict__ c, const double* __restrict__ s_x) {
  uint4 u[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) u[i] = reinterpret_cast<const uint4*>(c)[i];
  double t = 0.0;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    double w[8];
    widen8(u[i], w);
#pragma unroll
    for (int j = 0; j < 8; ++j) t = fma(s_x[i * 8 + j], w[j], t);
  }
  return t;
}
template <>
__device__ __forceinline__ double score_row<float>(const float* __restrict__ c, const double* __restrict__ s_x) {
  double t = 0.0;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    float4 u[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) u[i] = reinterpret_cast<const float4*>(c)[half * 16 + i];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int j = (half * 16 + i) * 4;
      t = fma(s_x[j + 0], (double)u[i].x, t);
      t = fma(s_x[j + 1], (double)u[i].y, t);
      t = fma(s_x[j + 2], (double)u[i].z, t);
      t = fma(s_x[j + 3], (double)u[i].w, t);
    }
  }
  return t;
}

// (score, id) candidates: o beats m if it exists and is larger, or equal with the lower id.
__device__ __forceinline__ void take_better(double& best, int& best_id, double ob, int oid) {
  if (oid >= 0 && (best_id < 0 || ob > best || (ob == best && oid < best_id))) {
    best = ob;
    best_id = oid;
  }
}
// Best candidate of the wave, in every lane.  Inside the rows of 16 lanes the partners' candidates come over the
// data-parallel primitives (three register moves per step), between the rows over the row-swap instructions: no
// step goes through the LDS crossbar.  All 64 lanes must be active.
template <int CTRL>
__device__ __forceinline__ void take_better_dpp(double& best, int& best_id) {
  const unsigned long long u = (unsigned long long)__double_as_longlong(best);
  const unsigned long long lo = dpp_u32<CTRL>((unsigned)u), hi = dpp_u32<CTRL>((unsigned)(u >> 32));
  const int oid = (int)dpp_u32<CTRL>((unsigned)best_id);
  take_better(best, best_id, __longlong_as_double((long long)((hi << 32) | lo)), oid);
}
__device__ __forceinline__ void wave_best(double& best, int& best_id) {
  take_better_dpp<kDppXor1>(best, best_id);
  take_better_dpp<kDppXor2>(best, best_id);
  take_better_dpp<kDppHalfMirror>(best, best_id);
  take_better_dpp<kDppMirror>(best, best_id);
  // between the rows: the row-swap instructions hand every lane its own candidate and that of the same lane one
  // row (then two rows) away, in an order that is the same for the three words
  {
    const unsigned long long u = (unsigned long long)__double_as_longlong(best);
    const auto lo = __builtin_amdgcn_permlane16_swap((unsigned)u, (unsigned)u, false, false);
    const auto hi = __builtin_amdgcn_permlane16_swap((unsigned)(u >> 32), (unsigned)(u >> 32), false, false);
    const auto id = __builtin_amdgcn_permlane16_swap((unsigned)best_id, (unsigned)best_id, false, false);
    best = __longlong_as_double((long long)(((unsigned long long)hi[0] << 32) | lo[0]));
    best_id = (int)id[0];
    take_better(best, best_id, __longlong_as_double((long long)(((unsigned long long)hi[1] << 32) | lo[1])), (int)id[1]);
  }
  {
    const unsigned long long u = (unsigned long long)__double_as_longlong(best);
    const auto lo = __builtin_amdgcn_permlane32_swap((unsigned)u, (unsigned)u, false, false);
    const auto hi = __builtin_amdgcn_permlane32_swap((unsigned)(u >> 32), (unsigned)(u >> 32), false, false);
    const auto id = __builtin_amdgcn_permlane32_swap((unsigned)best_id, (unsigned)best_id, false, false);
    best = __longlong_as_double((long long)(((unsigned long long)hi[0] << 32) | lo[0]));
    best_id = (int)id[0];
    take_better(best, best_id, __longlong_as_double((long long)(((unsigned long long)hi[1] << 32) | lo[1])), (int)id[1]);
  }
}

// Best candidate of one slab of centroids, as exchanged between the workgroups of a unit.
struct PushPartial {
  double score;
  int id;
  int pad;
};

// window_push: P = ceil(B / 64) one-wave workgroups per (sequence, KV head), each scoring a slab of
// 64 centroids (one per lane); the last to arrive picks the bucket and does the bookkeeping.
// Which key is displaced and where it goes does not depend on the new key's bucket: every
// workgroup reads that state up front (the loads overlap the scoring), slab 0 copies the displaced
// row to its bucket, and the last workgroup, which runs after all of these reads, writes the new
// row and the updated counts.
// C: element type of the cache.  C = T stores the new rows as they are; C = fp8_t (an 8-bit cache,
// T = bf16) stores x / scale of the (sequence, head) rounded to E4M3, saturated at +-448.
template <typename C, typename T>
__device__ __forceinline__ C to_cache(T v, float inv_scale) {
  if constexpr (sizeof(C) == sizeof(T)) {
    return v;
  } else {
    const float f = fminf(fmaxf(Vec8<T>::widen(v) * inv_scale, -448.f), 448.f);
    return (C)(__builtin_amdgcn_cvt_pk_fp8_f32(f, f, 0, false) & 0xff);
  }
}

template <typename T, typename C = T>
__global__ void __launch_bounds__(64)
window_push_kernel(const T* __restrict__ x_new, const T* __restrict__ k_new, const T* __restrict__ v_new,
                   const int32_t* __restrict__ pos_new, const T* __restrict__ cent, const float* __restrict__ bias,
                   const int32_t* __restrict__ off, int32_t* __restrict__ len, int32_t* __restrict__ idx,
                   C* __restrict__ Ks, C* __restrict__ Vs, const float* __restrict__ kscale,
                   const float* __restrict__ vscale, int32_t* __restrict__ res_ids,
                   int32_t* __restrict__ new_ids, int32_t* __restrict__ overflow, PushPartial* __restrict__ part,
                   unsigned* __restrict__ counters, int Hkv, int Ncap, int B, int runs, int n_sink, int n_recent,
                   int P, int cpl /* centroids per lane: a workgroup scores 64 * cpl */) {
  // runs = B + 1: index with a resident run.  runs = B: plain index (append_keys): W = 0, every key
  // goes straight into its bucket, res_ids is not touched and pos_new may be null (idx gets -2).
  __shared__ double s_x[kD];
  const int slab = blockIdx.x, unit = blockIdx.y, h = unit % Hkv, lane = threadIdx.x;
  SAAP_TRACE(0);
  const int W = n_sink + n_recent;
  const int32_t* o = off + (size_t)unit * (runs + 1);
  int32_t* l = len + (size_t)unit * runs;
  int32_t* ix = idx + (size_t)unit * Ncap;
  int32_t* rid = res_ids + (size_t)unit * W;
  C* Ku = Ks + (size_t)unit * Ncap * kD;
  C* Vu = Vs + (size_t)unit * Ncap * kD;
  const float k_inv = kscale ? 1.0f / kscale[unit] : 1.f, v_inv = vscale ? 1.0f / vscale[unit] : 1.f;   // powers of two

  // ---- the new key, and what can be decided without its bucket (same values in every lane) ----
  const T x0 = x_new[(size_t)unit * kD + lane], x1 = x_new[(size_t)unit * kD + 64 + lane];
  const T k0 = k_new[(size_t)unit * kD + lane], k1 = k_new[(size_t)unit * kD + 64 + lane];
  const T v0 = v_new[(size_t)unit * kD + lane], v1 = v_new[(size_t)unit * kD + 64 + lane];
  const int pos = pos_new ? pos_new[unit / Hkv] : 0x7fffffff;
  const int res_base = o[B];
  // -1: refused   0: slot of a run that is still filling   1: ring slot, a key is displaced   2: no ring
  const int kind = pos < 0 ? -1 : pos < W ? 0 : n_recent > 0 ? 1 : 2;
  int slot = -1, dst = -1, e = -1, cur = 0, moved_pos = -1;
  bool refused = kind < 0;
  if (kind == 0) {
    slot = res_base + pos;                     // r(pos) = pos while the run is not full
  } else if (kind == 1) {
    const int r = n_sink + (pos - n_sink) % n_recent;
    e = rid[r];
    // e outside [0,B) means the caller broke the protocol (pushes out of order, foreign state):
    // refuse like a full bucket instead of indexing with it
    const bool ok = e >= 0 && e < B;
    cur = ok ? l[e] : 0;
    if (ok && o[e] + cur < o[e + 1]) {
      slot = res_base + r;
      dst = o[e] + cur;
      moved_pos = ix[slot];
    } else {
      refused = true;
    }
  }
  if (slab == 0 && dst >= 0) {                 // the displaced row: ring slot -> its bucket
    Ku[(size_t)dst * kD + lane] = Ku[(size_t)slot * kD + lane];
    Ku[(size_t)dst * kD + 64 + lane] = Ku[(size_t)slot * kD + 64 + lane];
    Vu[(size_t)dst * kD + lane] = Vu[(size_t)slot * kD + lane];
    Vu[(size_t)dst * kD + 64 + lane] = Vu[(size_t)slot * kD + 64 + lane];
  }

  // ---- this slab's best centroid ----
  s_x[lane] = to_f64<T>(x0);
  s_x[64 + lane] = to_f64<T>(x1);
  __syncthreads();
  SAAP_TRACE(1);
  double best = 0.0;
  int best_id = -1;
  for (int c = 0; c < cpl; ++c) {                // ascending ids per lane: ties keep the lowest
    const int bc = (slab * cpl + c) * kPushSlab + lane;
    if (bc < B) {
      double t = score_row<T>(cent + ((size_t)h * B + bc) * kD, s_x);
      if (bias) t += (double)bias[(size_t)h * B + bc];
      take_better(best, best_id, t, bc);
    }
  }
  SAAP_TRACE(2);
  wave_best(best, best_id);
  SAAP_TRACE(3);
  if (P > 1) {
    if (lane == 0) {
      PushPartial* mine = part + (size_t)unit * P + slab;
      __hip_atomic_store(&mine->score, best, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(&mine->id, best_id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // every load above has returned and every store has been acknowledged before the arrival counts
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    unsigned old = 0;
    if (lane == 0) old = __hip_atomic_fetch_add(&counters[unit], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = (unsigned)__shfl((int)old, 0);
    SAAP_TRACE(4);
    if (old != (unsigned)(P - 1)) return;
    // every partial was stored through to the device's coherent level and acknowledged before its arrival was
    // counted: loads of the same scope see it, and no cache has to be invalidated for them
    best = 0.0;
    best_id = -1;
    for (int i = lane; i < P; i += 64) {       // ascending slabs per lane
      PushPartial* q = part + (size_t)unit * P + i;
      const double qs = __hip_atomic_load(&q->score, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const int qi = __hip_atomic_load(&q->id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      take_better(best, best_id, qs, qi);
    }
    wave_best(best, best_id);
    SAAP_TRACE(5);
    if (lane == 0) __hip_atomic_store(&counters[unit], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }

  // ---- bookkeeping, by the one workgroup that knows the bucket ----
  const int b = best_id;
  if (kind == 2) {                             // no ring: the new key goes straight into its bucket
    const int c2 = l[b];
    if (o[b] + c2 < o[b + 1]) slot = o[b] + c2; else refused = true;
    cur = c2;
  }
  if (lane == 0) {
    new_ids[unit] = b;
    if (refused) {
      *overflow = 1;
    } else {
      if (kind == 0) {
        l[B] += 1;
        rid[pos] = b;
      } else if (kind == 1) {
        l[e] = cur + 1;
        ix[dst] = moved_pos;
        rid[slot - res_base] = b;
      } else {
        l[b] = cur + 1;
      }
      ix[slot] = pos_new ? pos : -2;
    }
  }
  if (!refused) {
    Ku[(size_t)slot * kD + lane] = to_cache<C, T>(k0, k_inv);
    Ku[(size_t)slot * kD + 64 + lane] = to_cache<C, T>(k1, k_inv);
    Vu[(size_t)slot * kD + lane] = to_cache<C, T>(v0, v_inv);
    Vu[(size_t)slot * kD + 64 + lane] = to_cache<C, T>(v1, v_inv);
  }
  SAAP_TRACE(6);
}

// ---- recompact: fresh slack behind every bucket without assigning the keys again ---------------
// One workgroup per unit: new offsets from the current lengths.  `runs` = B, or B + 1 with a
// resident run, which keeps its fixed number of slots.
__global__ void __launch_bounds__(1024)
reoffset_kernel(const int32_t* __restrict__ len, const int32_t* __restrict__ off, int32_t* __restrict__ off_new,
                int runs, int B, int slack, int Ncap_new, int32_t* __restrict__ overflow) {
  __shared__ int s_wsum[16];
  const int unit = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = (B + blockDim.x - 1) / blockDim.x;
  const int b0 = tid * per, b1 = min(b0 + per, B);
  const int32_t* l = len + (size_t)unit * runs;
  const int32_t* o = off + (size_t)unit * (runs + 1);
  int32_t* on = off_new + (size_t)unit * (runs + 1);
  int mine = 0;
  for (int b = b0; b < b1; ++b) mine += l[b] + slack;
  const int incl = (int)wave_prefix_sum((unsigned)mine);
  if (lane == 63) s_wsum[wave] = incl;
  __syncthreads();
  int run = incl - mine;
  for (int w = 0; w < wave; ++w) run += s_wsum[w];
  if (tid == 0) on[0] = 0;
  for (int b = b0; b < b1; ++b) {
    run += l[b] + slack;
    on[b + 1] = run;
    if (b == B - 1) {
      int end = run;
      if (runs > B) {
        end += o[B + 1] - o[B];
        on[B + 1] = end;
      }
      if (end > Ncap_new) *overflow = 1;
    }
  }
}

// One workgroup per (run, unit): the run's member slots move to their place in the new cache.
template <int CHUNKS /* 16-byte pieces per row */>
__global__ void __launch_bounds__(256)
recopy_kernel(const int32_t* __restrict__ off, const int32_t* __restrict__ len, const int32_t* __restrict__ off_new,
              const int32_t* __restrict__ idx, int32_t* __restrict__ idx_new, const uint4* __restrict__ Ks,
              const uint4* __restrict__ Vs, uint4* __restrict__ Kn, uint4* __restrict__ Vn, int runs, int Ncap,
              int Ncap_new, const int32_t* __restrict__ overflow) {
  if (*overflow) return;                       // the new cache is too small: nothing is moved
  const int b = blockIdx.x, unit = blockIdx.y, tid = threadIdx.x;
  const int first = off[(size_t)unit * (runs + 1) + b], dst = off_new[(size_t)unit * (runs + 1) + b];
  // a resident run is a ring: every slot up to its length moves, whatever position it holds
  const int n = len[(size_t)unit * runs + b];
  for (int r = tid; r < n; r += 256) idx_new[(size_t)unit * Ncap_new + dst + r] = idx[(size_t)unit * Ncap + first + r];
  constexpr int kRowsPerPass = 256 / CHUNKS;
  const int piece = tid % CHUNKS;
  for (int r = tid / CHUNKS; r < n; r += kRowsPerPass) {
    const size_t src = ((size_t)unit * Ncap + first + r) * CHUNKS + piece;
    const size_t out = ((size_t)unit * Ncap_new + dst + r) * CHUNKS + piece;
    stream_store16(Kn + out, stream_load16(Ks + src));
    stream_store16(Vn + out, stream_load16(Vs + src));
  }
}

}  // namespace

size_t push_workspace_bytes(long long units, int B) {
  const long long P = (B + kPushSlab - 1) / kPushSlab;       // the most workgroups per unit any plan uses
  return (size_t)SAAP_WS_HEADER_BYTES + (size_t)units * P * sizeof(PushPartial);
}

// Centroids per lane of the scoring workgroups: one when few units leave the device empty, more
// when there are enough units to fill it anyway (about two workgroups per compute unit in all).
static int push_centroids_per_lane(long long units, int B) {
  const long long slabs = (B + kPushSlab - 1) / kPushSlab;
  long long want = 2LL * device_cus() / units;                // workgroups per unit
  if (want < 1) want = 1;
  long long cpl = (slabs + want - 1) / want;
  if (cpl < 1) cpl = 1;
  if (cpl > 8) cpl = 8;
  return (int)cpl;
}

size_t build_workspace_bytes(long long units, int N, int B) {
  const long long n_slices = (N + kSlice - 1) / kSlice;
  return (size_t)SAAP_WS_HEADER_BYTES + (size_t)units * n_slices * B * sizeof(int32_t);
}

}  // namespace saap

using namespace saap;

// Shared body of the two build calls.  res_ids == nullptr: plain index (B runs); otherwise the
// index with a resident run of W = n_sink + n_recent slots behind the B buckets.
static int32_t build_index(const int32_t* bucket_ids, const void* K, const void* V, int32_t* off, int32_t* len,
                           int32_t* idx, void* Ksorted, void* Vsorted, int32_t* res_ids, int32_t S, int32_t Hkv,
                           int32_t N, int32_t Ncap, int32_t B, int32_t d, int32_t dtype, int32_t slack,
                           int32_t n_sink, int32_t n_recent, void* ws, size_t ws_bytes, void* stream) {
  const bool windowed = res_ids != nullptr;
  if (!bucket_ids || !K || !V || !off || !len || !idx || !Ksorted || !Vsorted || !ws) return SAAP_INVALID_ARG;
  const void* ptrs[] = {bucket_ids, K, V, off, len, idx, Ksorted, Vsorted, ws, res_ids};
  for (const void* p : ptrs)
    if (!aligned16(p)) return SAAP_INVALID_ARG;
  if (S <= 0 || Hkv <= 0 || N <= 0 || B <= 0 || slack < 0 || n_sink < 0 || n_recent < 0) return SAAP_INVALID_ARG;
  if (dtype != SAAP_F32 && dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  const long long W = (long long)n_sink + n_recent;
  if (W > 0x3fffffff) return SAAP_INVALID_ARG;
  const long long n_res = windowed ? (N < W ? N : W) : 0;
  if ((long long)Ncap != (long long)N - n_res + (long long)B * slack + (windowed ? W : 0)) return SAAP_INVALID_ARG;
  if (d != kD || B > SAAP_MAX_BUCKETS) return SAAP_UNSUPPORTED;
  const long long units = (long long)S * Hkv;
  if (units > 65535) return SAAP_UNSUPPORTED;
  if (ws_bytes < build_workspace_bytes(units, N, B)) return SAAP_WORKSPACE_TOO_SMALL;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const int n_slices = (N + kSlice - 1) / kSlice;
  int32_t* slice_hist = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + SAAP_WS_HEADER_BYTES);
  int id_bits = 1;
  while ((1 << id_bits) < B) ++id_bits;
  // positions [lo, hi) go into the buckets
  const int lo = windowed ? (N <= W ? 0 : n_sink) : 0;
  const int hi = windowed ? (N <= W ? 0 : N - n_recent) : N;
  const int lstride = windowed ? B + 1 : B;

  hipLaunchKernelGGL(hist_kernel, dim3(n_slices, (unsigned)units), dim3(256), (size_t)B * sizeof(int), hs,
                     bucket_ids, slice_hist, N, B, n_slices, lo, hi);
  hipLaunchKernelGGL(colscan_kernel, dim3((B + 255) / 256, (unsigned)units), dim3(256), 0, hs, slice_hist, len,
                     B, n_slices, lstride);
  hipLaunchKernelGGL(offscan_kernel, dim3((unsigned)units), dim3(1024), 0, hs, len, off, B, slack,
                     windowed ? (int)W : -1, (int)n_res);
  const size_t n_idx = (size_t)units * Ncap;
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n_idx + 255) / 256)), dim3(256), 0, hs, idx, n_idx, -1);
  hipLaunchKernelGGL(scatter_kernel, dim3(n_slices, (unsigned)units), dim3(64), (size_t)B * sizeof(int), hs,
                     bucket_ids, slice_hist, off, idx, N, Ncap, B, n_slices, id_bits, lo, hi, lstride + 1);
  if (windowed && W > 0)
    hipLaunchKernelGGL(resident_kernel, dim3((unsigned)((W + 255) / 256), (unsigned)units), dim3(256), 0, hs,
                       bucket_ids, off, idx, res_ids, N, Ncap, B, n_sink, n_recent, (int)n_res);
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

extern "C" int32_t saap_build_bucket_index(const int32_t* bucket_ids, const void* K, const void* V,
                                           int32_t* off, int32_t* len, int32_t* idx, void* Ksorted,
                                           void* Vsorted, int32_t S, int32_t Hkv, int32_t N, int32_t Ncap,
                                           int32_t B, int32_t d, int32_t dtype, int32_t slack, void* ws,
                                           size_t ws_bytes, void* stream) {
  begin_call();
  return build_index(bucket_ids, K, V, off, len, idx, Ksorted, Vsorted, nullptr, S, Hkv, N, Ncap, B, d, dtype, slack,
                     0, 0, ws, ws_bytes, stream);
}

extern "C" int32_t saap_build_windowed_index(const int32_t* bucket_ids, const void* K, const void* V,
                                             int32_t* off, int32_t* len, int32_t* idx, void* Ksorted,
                                             void* Vsorted, int32_t* resident_ids, int32_t S, int32_t Hkv,
                                             int32_t N, int32_t Ncap, int32_t B, int32_t d, int32_t dtype,
                                             int32_t slack, int32_t n_sink, int32_t n_recent, void* ws,
                                             size_t ws_bytes, void* stream) {
  begin_call();
  if (!resident_ids) return SAAP_INVALID_ARG;
  return build_index(bucket_ids, K, V, off, len, idx, Ksorted, Vsorted, resident_ids, S, Hkv, N, Ncap, B, d, dtype,
                     slack, n_sink, n_recent, ws, ws_bytes, stream);
}

extern "C" int32_t saap_window_push(const void* x_new, const void* k_new, const void* v_new,
                                    const int32_t* pos_new, const void* centroids, const float* bias,
                                    const int32_t* off, int32_t* len, int32_t* idx, void* Ksorted,
                                    void* Vsorted, int32_t* resident_ids, int32_t* new_bucket_ids,
                                    int32_t* overflow_flag, int32_t S, int32_t Hkv, int32_t Ncap, int32_t B,
                                    int32_t d, int32_t dtype, int32_t n_sink, int32_t n_recent, void* ws,
                                    size_t ws_bytes, void* stream) {
  begin_call();
  if (!x_new || !k_new || !v_new || !pos_new || !centroids || !off || !len || !idx || !Ksorted || !Vsorted ||
      !resident_ids || !new_bucket_ids || !overflow_flag || !ws)
    return SAAP_INVALID_ARG;
  if (!aligned16(centroids) || !aligned16(ws)) return SAAP_INVALID_ARG;
  if (S <= 0 || Hkv <= 0 || Ncap <= 0 || B <= 0 || n_sink < 0 || n_recent < 0) return SAAP_INVALID_ARG;
  if ((long long)n_sink + n_recent > Ncap) return SAAP_INVALID_ARG;
  if (dtype != SAAP_F32 && dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  if (d != kD || B > SAAP_MAX_BUCKETS) return SAAP_UNSUPPORTED;
  const long long units = (long long)S * Hkv;
  if (units > 65535 || units * sizeof(unsigned) > SAAP_WS_HEADER_BYTES) return SAAP_UNSUPPORTED;
  if (ws_bytes < push_workspace_bytes(units, B)) return SAAP_WORKSPACE_TOO_SMALL;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const int cpl = push_centroids_per_lane(units, B);
  const int P = (B + kPushSlab * cpl - 1) / (kPushSlab * cpl);
  unsigned* counters = static_cast<unsigned*>(ws);
  PushPartial* part = reinterpret_cast<PushPartial*>(static_cast<char*>(ws) + SAAP_WS_HEADER_BYTES);
  const dim3 grid((unsigned)P, (unsigned)units);
  if (dtype == SAAP_BF16)
    hipLaunchKernelGGL(window_push_kernel<bf16_t>, grid, dim3(64), 0, hs, static_cast<const bf16_t*>(x_new),
                       static_cast<const bf16_t*>(k_new), static_cast<const bf16_t*>(v_new), pos_new,
                       static_cast<const bf16_t*>(centroids), bias, off, len, idx, static_cast<bf16_t*>(Ksorted),
                       static_cast<bf16_t*>(Vsorted), nullptr, nullptr, resident_ids, new_bucket_ids, overflow_flag, part, counters,
                       Hkv, Ncap, B, B + 1, n_sink, n_recent, P, cpl);
  else
    hipLaunchKernelGGL(window_push_kernel<float>, grid, dim3(64), 0, hs, static_cast<const float*>(x_new),
                       static_cast<const float*>(k_new), static_cast<const float*>(v_new), pos_new,
                       static_cast<const float*>(centroids), bias, off, len, idx, static_cast<float*>(Ksorted),
                       static_cast<float*>(Vsorted), nullptr, nullptr, resident_ids, new_bucket_ids, overflow_flag, part, counters,
                       Hkv, Ncap, B, B + 1, n_sink, n_recent, P, cpl);
  return launch_status();
}

extern "C" int32_t saap_append_keys(const void* x_new, const void* k_new, const void* v_new,
                                    const int32_t* pos_new, const void* centroids, const float* bias,
                                    const int32_t* off, int32_t* len, int32_t* idx, void* Ksorted,
                                    void* Vsorted, int32_t* new_bucket_ids, int32_t* overflow_flag, int32_t S,
                                    int32_t Hkv, int32_t Ncap, int32_t B, int32_t d, int32_t dtype, void* ws,
                                    size_t ws_bytes, void* stream) {
  begin_call();
  saap_trace_arm();
  if (!x_new || !k_new || !v_new || !centroids || !off || !len || !idx || !Ksorted || !Vsorted ||
      !new_bucket_ids || !overflow_flag || !ws)
    return SAAP_INVALID_ARG;
  if (!aligned16(centroids) || !aligned16(ws)) return SAAP_INVALID_ARG;
  if (S <= 0 || Hkv <= 0 || Ncap <= 0 || B <= 0) return SAAP_INVALID_ARG;
  if (dtype != SAAP_F32 && dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  if (d != kD || B > SAAP_MAX_BUCKETS) return SAAP_UNSUPPORTED;
  const long long units = (long long)S * Hkv;
  if (units > 65535 || units * sizeof(unsigned) > SAAP_WS_HEADER_BYTES) return SAAP_UNSUPPORTED;
  if (ws_bytes < push_workspace_bytes(units, B)) return SAAP_WORKSPACE_TOO_SMALL;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const int cpl = push_centroids_per_lane(units, B);
  const int P = (B + kPushSlab * cpl - 1) / (kPushSlab * cpl);
  unsigned* counters = static_cast<unsigned*>(ws);
  PushPartial* part = reinterpret_cast<PushPartial*>(static_cast<char*>(ws) + SAAP_WS_HEADER_BYTES);
  const dim3 grid((unsigned)P, (unsigned)units);
  int32_t* no_resident = nullptr;
  // the push kernel on a plain index: no resident run, the key goes straight into its bucket
  if (dtype == SAAP_BF16)
    hipLaunchKernelGGL(window_push_kernel<bf16_t>, grid, dim3(64), 0, hs, static_cast<const bf16_t*>(x_new),
                       static_cast<const bf16_t*>(k_new), static_cast<const bf16_t*>(v_new), pos_new,
                       static_cast<const bf16_t*>(centroids), bias, off, len, idx, static_cast<bf16_t*>(Ksorted),
                       static_cast<bf16_t*>(Vsorted), nullptr, nullptr, no_resident, new_bucket_ids, overflow_flag, part, counters, Hkv,
                       Ncap, B, B, 0, 0, P, cpl);
  else
    hipLaunchKernelGGL(window_push_kernel<float>, grid, dim3(64), 0, hs, static_cast<const float*>(x_new),
                       static_cast<const float*>(k_new), static_cast<const float*>(v_new), pos_new,
                       static_cast<const float*>(centroids), bias, off, len, idx, static_cast<float*>(Ksorted),
                       static_cast<float*>(Vsorted), nullptr, nullptr, no_resident, new_bucket_ids, overflow_flag, part, counters, Hkv,
                       Ncap, B, B, 0, 0, P, cpl);
  return launch_status();
}

// The push kernel on an 8-bit cache (bf16 features and new rows, E4M3 rows in the cache).
// res_ids == nullptr: plain index (append), else the index with a resident run.
static int32_t push_fp8(const void* x_new, const void* k_new, const void* v_new, const int32_t* pos_new,
                        const void* centroids, const float* bias, const int32_t* off, int32_t* len, int32_t* idx,
                        uint8_t* K8, uint8_t* V8, const float* kscale, const float* vscale, int32_t* res_ids,
                        int32_t* new_bucket_ids, int32_t* overflow_flag, int32_t S, int32_t Hkv, int32_t Ncap,
                        int32_t B, int32_t d, int32_t n_sink, int32_t n_recent, void* ws, size_t ws_bytes,
                        void* stream) {
  if (!x_new || !k_new || !v_new || !centroids || !off || !len || !idx || !K8 || !V8 || !kscale || !vscale ||
      !new_bucket_ids || !overflow_flag || !ws)
    return SAAP_INVALID_ARG;
  if (!aligned16(centroids) || !aligned16(ws)) return SAAP_INVALID_ARG;
  if (S <= 0 || Hkv <= 0 || Ncap <= 0 || B <= 0 || n_sink < 0 || n_recent < 0) return SAAP_INVALID_ARG;
  if (res_ids && (!pos_new || (long long)n_sink + n_recent > Ncap)) return SAAP_INVALID_ARG;
  if (d != kD || B > SAAP_MAX_BUCKETS) return SAAP_UNSUPPORTED;
  const long long units = (long long)S * Hkv;
  if (units > 65535 || units * sizeof(unsigned) > SAAP_WS_HEADER_BYTES) return SAAP_UNSUPPORTED;
  if (ws_bytes < push_workspace_bytes(units, B)) return SAAP_WORKSPACE_TOO_SMALL;
  const int cpl = push_centroids_per_lane(units, B);
  const int P = (B + kPushSlab * cpl - 1) / (kPushSlab * cpl);
  unsigned* counters = static_cast<unsigned*>(ws);
  PushPartial* part = reinterpret_cast<PushPartial*>(static_cast<char*>(ws) + SAAP_WS_HEADER_BYTES);
  hipLaunchKernelGGL((window_push_kernel<bf16_t, fp8_t>), dim3((unsigned)P, (unsigned)units), dim3(64), 0,
                     static_cast<hipStream_t>(stream), static_cast<const bf16_t*>(x_new),
                     static_cast<const bf16_t*>(k_new), static_cast<const bf16_t*>(v_new), pos_new,
                     static_cast<const bf16_t*>(centroids), bias, off, len, idx, K8, V8, kscale, vscale, res_ids,
                     new_bucket_ids, overflow_flag, part, counters, Hkv, Ncap, B, res_ids ? B + 1 : B, n_sink, n_recent,
                     P, cpl);
  return launch_status();
}

extern "C" int32_t saap_append_keys_fp8(const void* x_new, const void* k_new, const void* v_new,
                                        const int32_t* pos_new, const void* centroids, const float* bias,
                                        const int32_t* off, int32_t* len, int32_t* idx, uint8_t* K8, uint8_t* V8,
                                        const float* kscale, const float* vscale, int32_t* new_bucket_ids,
                                        int32_t* overflow_flag, int32_t S, int32_t Hkv, int32_t Ncap, int32_t B,
                                        int32_t d, void* ws, size_t ws_bytes, void* stream) {
  begin_call();
  return push_fp8(x_new, k_new, v_new, pos_new, centroids, bias, off, len, idx, K8, V8, kscale, vscale, nullptr,
                  new_bucket_ids, overflow_flag, S, Hkv, Ncap, B, d, 0, 0, ws, ws_bytes, stream);
}

extern "C" int32_t saap_window_push_fp8(const void* x_new, const void* k_new, const void* v_new,
                                        const int32_t* pos_new, const void* centroids, const float* bias,
                                        const int32_t* off, int32_t* len, int32_t* idx, uint8_t* K8, uint8_t* V8,
                                        const float* kscale, const float* vscale, int32_t* resident_ids,
                                        int32_t* new_bucket_ids, int32_t* overflow_flag, int32_t S, int32_t Hkv,
                                        int32_t Ncap, int32_t B, int32_t d, int32_t n_sink, int32_t n_recent,
                                        void* ws, size_t ws_bytes, void* stream) {
  begin_call();
  if (!resident_ids) return SAAP_INVALID_ARG;
  return push_fp8(x_new, k_new, v_new, pos_new, centroids, bias, off, len, idx, K8, V8, kscale, vscale, resident_ids,
                  new_bucket_ids, overflow_flag, S, Hkv, Ncap, B, d, n_sink, n_recent, ws, ws_bytes, stream);
}

extern "C" int32_t saap_recompact_index(const int32_t* off, const int32_t* len, const int32_t* idx,
                                        const void* Ksorted, const void* Vsorted, int32_t* off_new,
                                        int32_t* idx_new, void* Ksorted_new, void* Vsorted_new,
                                        int32_t* overflow_flag, int32_t S, int32_t Hkv, int32_t Ncap,
                                        int32_t Ncap_new, int32_t B, int32_t resident, int32_t d, int32_t dtype,
                                        int32_t slack_new, void* stream) {
  begin_call();
  if (!off || !len || !idx || !Ksorted || !Vsorted || !off_new || !idx_new || !Ksorted_new || !Vsorted_new ||
      !overflow_flag)
    return SAAP_INVALID_ARG;
  const void* ptrs[] = {idx, Ksorted, Vsorted, idx_new, Ksorted_new, Vsorted_new};
  for (const void* p : ptrs)
    if (!aligned16(p)) return SAAP_INVALID_ARG;
  if (S <= 0 || Hkv <= 0 || Ncap <= 0 || Ncap_new <= 0 || B <= 0 || slack_new < 0) return SAAP_INVALID_ARG;
  if (resident != 0 && resident != 1) return SAAP_INVALID_ARG;
  if (Ksorted == Ksorted_new || Vsorted == Vsorted_new || idx == idx_new || off == off_new) return SAAP_INVALID_ARG;
  if (dtype != SAAP_F32 && dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  if (d != kD || B > SAAP_MAX_BUCKETS) return SAAP_UNSUPPORTED;
  const long long units = (long long)S * Hkv;
  if (units > 65535) return SAAP_UNSUPPORTED;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const int runs = B + resident;
  hipLaunchKernelGGL(reoffset_kernel, dim3((unsigned)units), dim3(1024), 0, hs, len, off, off_new, runs, B, slack_new,
                     Ncap_new, overflow_flag);
  const size_t n_idx = (size_t)units * Ncap_new;
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n_idx + 255) / 256)), dim3(256), 0, hs, idx_new, n_idx, -1);
  const dim3 grid((unsigned)runs, (unsigned)units);
  if (dtype == SAAP_BF16)
    hipLaunchKernelGGL(recopy_kernel<16>, grid, dim3(256), 0, hs, off, len, off_new, idx, idx_new,
                       static_cast<const uint4*>(Ksorted), static_cast<const uint4*>(Vsorted),
                       static_cast<uint4*>(Ksorted_new), static_cast<uint4*>(Vsorted_new), runs, Ncap, Ncap_new,
                       overflow_flag);
  else
    hipLaunchKernelGGL(recopy_kernel<32>, grid, dim3(256), 0, hs, off, len, off_new, idx, idx_new,
                       static_cast<const uint4*>(Ksorted), static_cast<const uint4*>(Vsorted),
                       static_cast<uint4*>(Ksorted_new), static_cast<uint4*>(Vsorted_new), runs, Ncap, Ncap_new,
                       overflow_flag);
  return launch_status();
}
