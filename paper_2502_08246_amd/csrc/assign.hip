// assign_keys: nearest-centroid assignment of keys at prefill (Section 2, indexing step, and
// Section 4 of arXiv 2502.08246): bucket = argmax_b <x, c_b> + bias_b.
//
// The result is DEFINED on double-precision scores (in-order sum of exact products, lowest id
// on ties).  Two kernels produce exactly that:
//   * mfma kernel (bf16 inputs): scores on the matrix cores, fp32 accumulation.  A workgroup
//     holds 256 keys in registers as the B operand of v_mfma_f32_32x32x16_bf16 and streams the
//     centroids through LDS in tiles of 32 as the A operand, so one lane owns one key and its 16
//     accumulator registers are 16 different centroids.  Per key the lane tracks the best and
//     second-best score; the low 4 bits of a score carry the accumulator register number, so
//     the running argmax costs 2.5 vector instructions per score (tag; max3 and med3 + max per pair).
//   * re-scoring kernel: a key whose best two fp32 scores are closer than the accumulation error
//     bound is scored again, 32 such keys of a head at a time: one more matrix-core pass (two
//     beyond 1024 buckets) finds every centroid within the bound of the key's maximum, and only
//     those (typically two) are scored in double precision.
//   * fp32 inputs: a plain double-precision kernel scores every key against every centroid.
// No score matrix is ever written to memory.
#include "common.h"

namespace saap {
namespace {

constexpr int kRowsPerWg = 256;   // keys per workgroup of the mfma kernel (4 waves x 64)
constexpr int kCentTile = 32;     // centroids per matrix tile
constexpr int kSlab = 64;         // centroids per LDS slab (two matrix tiles)
constexpr int kPitch = 136;       // bf16 elements per LDS row (272 bytes: conflict-free b128 reads)

// max_b |c_b| per KV head (fp32, rounded up a little).  16 lanes per centroid row.
constexpr int kNormThreads = 1024;
__global__ void __launch_bounds__(kNormThreads)
cent_norm_kernel(const bf16_t* __restrict__ cent, float* __restrict__ cmax, int B) {
  __shared__ float s_m[kNormThreads / 64];
  const int h = blockIdx.x, tid = threadIdx.x, piece = tid & 15, sub = tid >> 4;
  const bf16_t* cu = cent + (size_t)h * B * kD;
  float mx = 0.f;
  for (int b0 = 0; b0 < B; b0 += kNormThreads / 16 * 4) {
    Vec8<bf16_t> v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u].load(cu + (size_t)min(b0 + u * (kNormThreads / 16) + sub, B - 1) * kD + piece * 8);
#pragma unroll
    for (int u = 0; u < 4; ++u) mx = fmaxf(mx, sum16(v[u].dot(v[u])));
  }
  mx = max_rows(mx);
  if ((tid & 63) == 0) s_m[tid >> 6] = mx;
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < kNormThreads / 64; ++w) mx = fmaxf(mx, s_m[w]);
    cmax[h] = sqrtf(mx) * 1.0001f;
  }
}

template <bool HAS_BIAS>
__global__ void __launch_bounds__(256, 2)
assign_mfma_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ cent, const float* __restrict__ bias,
                   const float* __restrict__ cmax, int32_t* __restrict__ ids, int32_t* __restrict__ flagged,
                   unsigned* __restrict__ n_flagged, size_t list_cap, int Hkv, int N, int B, float tol) {
  __shared__ __align__(16) bf16_t s_c[2][kSlab * kPitch];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int unit = blockIdx.y, h = unit % Hkv;
  const int col = lane & 31, half = lane >> 5;
  const bf16_t* cu = cent + (size_t)h * B * kD;

  // B operand: two tiles of 32 keys per wave; lane holds features 16*step + 8*half .. +7 of key `col`.
  const int row_base = blockIdx.x * kRowsPerWg + wave * 64;
  bf16x8_t xb[2][8];
  float xnorm2[2];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    const int r = min(row_base + rt * 32 + col, N - 1);
    const bf16_t* xr = x + ((size_t)unit * N + r) * kD + half * 8;
    float s = 0.f;
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      const uint4 raw = *reinterpret_cast<const uint4*>(xr + st * 16);
      xb[rt][st] = __builtin_bit_cast(bf16x8_t, raw);
      const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        s = fmaf(bf16_lo(w[i]), bf16_lo(w[i]), s);
        s = fmaf(bf16_hi(w[i]), bf16_hi(w[i]), s);
      }
    }
    s += __shfl_xor(s, 32);
    xnorm2[rt] = s;
  }

  // Centroids stream through LDS in slabs of kSlab = 64 (two matrix tiles of 32), double
  // buffered: a slab is 1024 pieces of 16 bytes, four per thread, fetched into registers one
  // slab ahead (a slab's worth of matrix work covers the L2 latency) and stored mid-way through
  // the compute of the slab before.
  const int n_slabs = (B + kSlab - 1) / kSlab;
  // The staging registers must stay registers: fetch and stash run unconditionally (the last
  // pass fetches the last slab again and stores it into the idle buffer), which keeps them out of
  // control flow; behind a branch the compiler parked them in scratch memory and waited for every
  // load right after issuing it.
  typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;
  u32x4_t stage[kSlab / 16];
  auto fetch = [&](int t) {
#pragma unroll
    for (int i = 0; i < kSlab / 16; ++i) {
      const int piece = tid + i * 256, r = piece >> 4, pc = piece & 15;
      int b = t * kSlab + r;
      if (b >= B) b = 0;   // padding repeats centroid 0; a padded winner is re-scored (id >= B below)
      stage[i] = *reinterpret_cast<const u32x4_t*>(cu + (size_t)b * kD + pc * 8);
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int i = 0; i < kSlab / 16; ++i) {
      const int piece = tid + i * 256, r = piece >> 4, pc = piece & 15;
      *reinterpret_cast<u32x4_t*>(&s_c[buf][r * kPitch + pc * 8]) = stage[i];
    }
  };
  fetch(0);
  stash(0);
  fetch(min(1, n_slabs - 1));
  __syncthreads();

  const uint32_t keep = 0xFFFFFFF0u;
  float best[2], second[2];
  int best_tile[2];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    best[rt] = -INFINITY;
    second[rt] = -INFINITY;
    best_tile[rt] = 0;
  }

  typedef __attribute__((ext_vector_type(16))) float f32x16_t;
  // A operand of k-step `st` of matrix tile `sub` of the slab in `buf`
  auto a_frag = [&](int buf, int sub, int st) {
    const uint4 raw = *reinterpret_cast<const uint4*>(&s_c[buf][(sub * kCentTile + col) * kPitch + st * 16 + half * 8]);
    return __builtin_bit_cast(bf16x8_t, raw);
  };
  // running best / second best over accumulator registers r, r+1 of both key tiles; register r
  // of this lane is centroid 8*(r/4) + 4*half + r%4 of matrix tile `tile` (global tile number).
  // Two scores per step: with s <= b the second largest of {b, s, x, y} is max(s, med3(b, x, y)),
  // the largest max3(b, x, y): 2.5 vector instructions per score with the tag, not 3.
  auto track_pair = [&](const f32x16_t& c0, const f32x16_t& c1, int tile, int r) {
    float p0[2], p1[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      float s0 = c0[r + u], s1 = c1[r + u];
      if (HAS_BIAS) {
        const int b = tile * kCentTile + 8 * ((r + u) / 4) + 4 * half + ((r + u) % 4);
        const float bv = bias[(size_t)h * B + (b < B ? b : 0)];
        s0 += bv;
        s1 += bv;
      }
      p0[u] = __uint_as_float((__float_as_uint(s0) & keep) | (uint32_t)(r + u));
      p1[u] = __uint_as_float((__float_as_uint(s1) & keep) | (uint32_t)(r + u));
    }
    second[0] = fmaxf(second[0], __builtin_amdgcn_fmed3f(best[0], p0[0], p0[1]));
    best[0] = fmaxf(fmaxf(best[0], p0[0]), p0[1]);
    second[1] = fmaxf(second[1], __builtin_amdgcn_fmed3f(best[1], p1[0], p1[1]));
    best[1] = fmaxf(fmaxf(best[1], p1[0]), p1[1]);
  };
  // Software pipeline over matrix tiles: while the matrix cores work on tile (buf, sub) into
  // n0/n1, the vector pipe ranks the finished scores o0/o1 of the tile before.  One k-step (two
  // matrix instructions, 2 x 8 passes) is paired with one register pair of ranking (ten vector
  // instructions) between scheduling fences; left alone the compiler issues all sixteen matrix
  // instructions first and the two pipes run one after the other.
  auto step = [&](int buf, int sub, f32x16_t& n0, f32x16_t& n1, const f32x16_t& o0, const f32x16_t& o1,
                  int tile_old, bool has_new, bool has_old) {
    const float old0 = best[0], old1 = best[1];
    bf16x8_t a = a_frag(buf, sub, 0);
    if (has_new) {
      n0 = (f32x16_t){0};
      n1 = (f32x16_t){0};
    }
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      __builtin_amdgcn_sched_barrier(0);
      if (has_new) {
        const bf16x8_t a_next = a_frag(buf, sub, min(st + 1, 7));
        n0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, xb[0][st], n0, 0, 0, 0);
        n1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, xb[1][st], n1, 0, 0, 0);
        a = a_next;
      }
      if (has_old) track_pair(o0, o1, tile_old, 2 * st);
    }
    __builtin_amdgcn_sched_barrier(0);
    if (has_old) {
      best_tile[0] = best[0] != old0 ? tile_old : best_tile[0];
      best_tile[1] = best[1] != old1 ? tile_old : best_tile[1];
    }
  };

  f32x16_t a0, a1, b0 = {0}, b1 = {0};   // b0, b1: not read by the first step
  step(0, 0, a0, a1, b0, b1, 0, true, false);
  for (int t = 0; t < n_slabs - 1; ++t) {
    const int buf = t & 1;
    step(buf, 1, b0, b1, a0, a1, t * 2 + 0, true, true);
    stash(buf ^ 1);
    fetch(min(t + 2, n_slabs - 1));
    __syncthreads();
    step(buf ^ 1, 0, a0, a1, b0, b1, t * 2 + 1, true, true);
  }
  step((n_slabs - 1) & 1, 1, b0, b1, a0, a1, (n_slabs - 1) * 2 + 0, true, true);
  step(0, 0, a0, a1, b0, b1, (n_slabs - 1) * 2 + 1, false, true);

  // lanes l and l+32 own the same key: merge their candidates, lower id on equal packed scores
  const float tol_c = tol * cmax[h];
  __shared__ unsigned s_listed, s_list_base;
  if (tid == 0) s_listed = 0u;
  __syncthreads();
  bool listed[2];
  unsigned slot[2];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    const int r = (int)(__float_as_uint(best[rt]) & 15u);
    int id = best_tile[rt] * kCentTile + 8 * (r / 4) + 4 * half + (r % 4);
    const float ob = __shfl_xor(best[rt], 32);
    const float os = __shfl_xor(second[rt], 32);
    const int oid = __shfl_xor(id, 32);
    const float mb = best[rt], ms = second[rt];
    float nb, ns;
    if (ob > mb || (ob == mb && oid < id)) {
      nb = ob;
      ns = fmaxf(mb, os);
      id = oid;
    } else {
      nb = mb;
      ns = fmaxf(ob, ms);
    }
    const int row = row_base + rt * 32 + col;
    listed[rt] = false;
    if (half == 0 && row < N) {
      const size_t g = (size_t)unit * N + row;
      ids[g] = id;
      // error bound of the fp32 accumulation plus the 4 mantissa bits used for the register tag
      const float thr = tol_c * sqrtf(xnorm2[rt]) + 5e-6f * fabsf(nb);
      if (!(nb - ns > thr) || id >= B) {
        listed[rt] = true;
        slot[rt] = atomicAdd(&s_listed, 1u);
      }
    }
  }
  // one list per KV head (the re-scoring shares centroid loads between keys of a head); the
  // workgroup's keys are added in one piece, with one global counter update
  __syncthreads();
  if (tid == 0 && s_listed) s_list_base = atomicAdd(n_flagged + h, s_listed);
  __syncthreads();
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
    if (listed[rt])   // global row index fits in 31 bits: checked on the host
      flagged[(size_t)h * list_cap + s_list_base + slot[rt]] = (int32_t)((size_t)unit * N + row_base + rt * 32 + col);
}

// fp32 inputs: double-precision scoring of every key against every centroid (in-order sum,
// lowest id on ties).  One workgroup per key, grid-stride.
__global__ void __launch_bounds__(256)
assign_exact_f32_kernel(const float* __restrict__ x, const float* __restrict__ cent, const float* __restrict__ bias,
                        int32_t* __restrict__ ids, long long n_rows, int Hkv, int N, int B) {
  __shared__ double s_x[kD];
  __shared__ double s_best[256];
  __shared__ int s_id[256];
  const int tid = threadIdx.x;
  for (long long g = blockIdx.x; g < n_rows; g += gridDim.x) {
    const int h = (int)((g / N) % Hkv);
    __syncthreads();
    if (tid < kD) s_x[tid] = (double)x[(size_t)g * kD + tid];
    __syncthreads();
    double best = 0.0;
    int best_id = -1;
    for (int b = tid; b < B; b += blockDim.x) {
      const float* c = cent + ((size_t)h * B + b) * kD;
      double t = 0.0;
      for (int j = 0; j < kD; ++j) t = fma(s_x[j], (double)c[j], t);
      if (bias) t += (double)bias[(size_t)h * B + b];
      if (best_id < 0 || t > best) {
        best = t;
        best_id = b;
      }
    }
    s_best[tid] = best;
    s_id[tid] = best_id;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
      if (tid < s) {
        const int oid = s_id[tid + s], mid = s_id[tid];
        const double ob = s_best[tid + s];
        if (oid >= 0 && (mid < 0 || ob > s_best[tid] || (ob == s_best[tid] && oid < mid))) {
          s_best[tid] = ob;
          s_id[tid] = oid;
        }
      }
      __syncthreads();
    }
    if (tid == 0) ids[g] = s_id[0];
  }
}

// Re-scoring of the listed keys (bf16).  The keys are listed per KV head; a workgroup takes 32
// consecutive entries of one head's list as the B operand of the matrix instruction (every wave
// holds the same 32 keys) and its eight waves share out the centroid tiles, so a centroid row is
// read once for 32 keys.
//   pass 1: fp32 scores of all centroids on the matrix cores, running maximum per key; a wave keeps
//           the scores of its first kKeepTiles tiles in registers (all of them up to 1024 buckets)
//           and has the loads of those tiles in flight together;
//   pass 2: every centroid whose score is within the error bound of the key's maximum goes into a
//           candidate list in LDS: from the kept scores, and for further tiles from the same
//           instructions run again (same results bit for bit).  Any centroid that can be the
//           double-precision argmax is among them, because both fp32 scores carry at most half the
//           bound as error; a score that does not compare (NaN) counts as a candidate;
//   pass 3: the candidates (typically two per key) in double precision, in order, one per thread;
//           the largest per key, lowest id on ties, through LDS atomics (maximum of the scores in
//           an order-preserving integer form, then minimum of the ids that reach it).
// If the list overflows (degenerate keys, e.g. all scores equal) the group's keys are scored
// against every centroid in double precision instead.
// Grid: (Hkv, workgroups per head), the head fastest, so that the few workgroups that find a group
// of keys are the first to be dispatched.  counters[h] = length of head h's list, counters[Hkv] =
// workgroups that have finished.
constexpr int kGroupKeys = 32;
constexpr int kCandCap = 2048;
constexpr int kRescoreThreads = 512, kRescoreWaves = kRescoreThreads / 64;
constexpr int kKeepTiles = 4;      // matrix tiles per wave whose scores stay in registers between the passes

// double-precision score of centroid row c against key row xr (in order), rows of 16-byte pieces
__device__ __forceinline__ double score_bf16_f64(const uint4* __restrict__ xr, const uint4* __restrict__ c) {
  // The loads and conversions stay inside the (rarely taken) candidate path: hoisted out of a
  // caller's loop the key's 128 doubles would hold 256 registers for the whole kernel.
  asm volatile("" ::: "memory");
  double t = 0.0;
#pragma unroll
  for (int hh = 0; hh < 2; ++hh) {   // half a row of each in flight, then that half of the chain
    uint4 xw[kD / 16], cw[kD / 16];
#pragma unroll
    for (int j = 0; j < kD / 16; ++j) {
      xw[j] = xr[hh * (kD / 16) + j];
      cw[j] = c[hh * (kD / 16) + j];
    }
#pragma unroll
    for (int j = 0; j < kD / 16; ++j) {
      const uint32_t w[4] = {cw[j].x, cw[j].y, cw[j].z, cw[j].w}, v[4] = {xw[j].x, xw[j].y, xw[j].z, xw[j].w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        t = fma((double)bf16_lo(v[k]), (double)bf16_lo(w[k]), t);
        t = fma((double)bf16_hi(v[k]), (double)bf16_hi(w[k]), t);
      }
    }
  }
  return t;
}

__device__ __forceinline__ bool better(double s, int id, double best, int best_id) {
  return id >= 0 && (best_id < 0 || s > best || (s == best && id < best_id));
}

// Doubles as unsigned integers in the same order (no NaNs; -0 is turned into +0 first).
__device__ __forceinline__ unsigned long long ordered_bits(double v) {
  const unsigned long long u = (unsigned long long)__double_as_longlong(v + 0.0);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

__global__ void __launch_bounds__(kRescoreThreads)
assign_rescore_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ cent,
                      const float* __restrict__ bias, const float* __restrict__ cmax,
                      int32_t* __restrict__ ids, const int32_t* __restrict__ rows,
                      unsigned* __restrict__ counters, unsigned* __restrict__ stat, size_t list_cap, int Hkv,
                      int B, float tol) {
  typedef __attribute__((ext_vector_type(16))) float f32x16_t;
  __shared__ float s_max[kRescoreWaves][kGroupKeys];
  __shared__ float s_lim[kGroupKeys];
  __shared__ int s_key[kGroupKeys];        // global row of each key of the group
  __shared__ unsigned s_ncand;
  __shared__ int s_cand[kCandCap];         // key << 24 | centroid
  __shared__ unsigned long long s_cscore[kCandCap];   // ordered_bits of the candidate's score
  __shared__ unsigned long long s_kbest[kGroupKeys];
  __shared__ int s_kid[kGroupKeys];
  __shared__ double s_wbest[kRescoreWaves];
  __shared__ int s_wid[kRescoreWaves];
  __shared__ int s_flag;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int h = blockIdx.x;
  const unsigned n_rows = counters[h];
  const unsigned n_groups = (n_rows + kGroupKeys - 1) / kGroupKeys;
  rows += (size_t)h * list_cap;
  const bf16_t* cu = cent + (size_t)h * B * kD;
  const float* bu = bias ? bias + (size_t)h * B : nullptr;
  const int n_tiles = (B + kCentTile - 1) / kCentTile;

  SAAP_TRACE(0);
  for (unsigned grp = blockIdx.y; grp < n_groups; grp += gridDim.y) {
    const unsigned first = grp * kGroupKeys;
    const int n_here = (int)min((unsigned)kGroupKeys, n_rows - first);
    // B operand: lane holds features 16*step + 8*half .. +7 of key `col` (idle columns repeat the last key)
    const int gk = rows[first + min(col, n_here - 1)];
    const bf16_t* xr = x + (size_t)gk * kD + half * 8;
    bf16x8_t xb[8];
    float xnorm2 = 0.f;
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      Vec8<bf16_t> v;
      v.load(xr + st * 16);
      xb[st] = __builtin_bit_cast(bf16x8_t, v.r);
      xnorm2 += v.dot(v);
    }
    xnorm2 += __shfl_xor(xnorm2, 32);
    SAAP_TRACE(1);
    if (tid < kGroupKeys) {
      s_key[tid] = gk;
      s_kbest[tid] = 0ull;
      s_kid[tid] = 0x7fffffff;
    }
    if (tid == 0) s_ncand = 0u;

    // scores of centroid tile t for the 32 keys: register r of this lane is centroid
    // 32*t + 8*(r/4) + 4*half + r%4 against key `col`
    auto tile_load = [&](int t, bf16x8_t (&a)[8]) {
      const bf16_t* cr = cu + (size_t)min(t * kCentTile + col, B - 1) * kD + half * 8;
#pragma unroll
      for (int st = 0; st < 8; ++st) a[st] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(cr + st * 16));
    };
    auto tile_product = [&](const bf16x8_t (&a)[8]) {
      f32x16_t acc = {0};
#pragma unroll
      for (int st = 0; st < 8; ++st) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[st], xb[st], acc, 0, 0, 0);
      return acc;
    };
    auto centroid_of = [&](int t, int r) { return t * kCentTile + 8 * (r / 4) + 4 * half + (r % 4); };
    // the scores that are compared: matrix product plus the centroid's bias (one fp32 addition)
    auto add_bias = [&](f32x16_t& acc, int t) {
      if (bu) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] += bu[min(centroid_of(t, r), B - 1)];
      }
    };
    auto tile_scores = [&](int t) {
      bf16x8_t a[8];
      tile_load(t, a);
      f32x16_t acc = tile_product(a);
      add_bias(acc, t);
      return acc;
    };
    auto tile_max = [&](const f32x16_t& acc, int t, float mx) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (centroid_of(t, r) < B) mx = fmaxf(mx, acc[r]);
      return mx;
    };
    auto tile_candidates = [&](const f32x16_t& acc, int t, float lim) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int b = centroid_of(t, r);
        if (b < B && col < n_here && !(acc[r] < lim)) {
          const unsigned i = atomicAdd(&s_ncand, 1u);
          if (i < (unsigned)kCandCap) s_cand[i] = (col << 24) | b;
        }
      }
    };

    // the wave's first kKeepTiles tiles: every load goes out before the first product (tiles past
    // the end repeat the last one and are ignored below)
    f32x16_t kept[kKeepTiles];
    // the tile numbers are made opaque per group: as loop invariants the compiler computes every address of
    // every tile (centroid rows, biases) ahead of the loop and spills them
    int wave_t = wave;
    asm volatile("" : "+v"(wave_t));
    {
      bf16x8_t a[kKeepTiles][8];
#pragma unroll
      for (int k = 0; k < kKeepTiles; ++k) tile_load(min(wave_t + k * kRescoreWaves, n_tiles - 1), a[k]);
      __builtin_amdgcn_sched_barrier(0);     // left alone the compiler keeps three or four loads in flight
#pragma unroll
      for (int k = 0; k < kKeepTiles; ++k) kept[k] = tile_product(a[k]);
    }
#pragma unroll
    for (int k = 0; k < kKeepTiles; ++k) add_bias(kept[k], min(wave_t + k * kRescoreWaves, n_tiles - 1));
    float mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < kKeepTiles; ++k) {
      const int t = wave_t + k * kRescoreWaves;
      if (t < n_tiles) mx = tile_max(kept[k], t, mx);
    }
    for (int t = wave_t + kKeepTiles * kRescoreWaves; t < n_tiles; t += kRescoreWaves) mx = tile_max(tile_scores(t), t, mx);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    if (half == 0) s_max[wave][col] = mx;
    __syncthreads();
    SAAP_TRACE(2);
    if (tid < kGroupKeys) {
      float m = s_max[0][tid];
      for (int w = 1; w < kRescoreWaves; ++w) m = fmaxf(m, s_max[w][tid]);
      // two fp32 scores are compared: the same bound as for the first matrix pass
      s_lim[tid] = m - (tol * cmax[h] * sqrtf(xnorm2) + 5e-6f * fabsf(m));
    }
    __syncthreads();
    const float lim = s_lim[col];
#pragma unroll
    for (int k = 0; k < kKeepTiles; ++k) {
      const int t = wave_t + k * kRescoreWaves;
      if (t < n_tiles) tile_candidates(kept[k], t, lim);
    }
    for (int t = wave_t + kKeepTiles * kRescoreWaves; t < n_tiles; t += kRescoreWaves) tile_candidates(tile_scores(t), t, lim);
    __syncthreads();
    SAAP_TRACE(3);
    const unsigned n_cand = s_ncand;
    if (tid == 0) SAAP_TRACE_VALUE(7, n_cand);
    if (n_cand <= (unsigned)kCandCap) {
      for (unsigned i = tid; i < n_cand; i += kRescoreThreads) {
        const int key = s_cand[i] >> 24, b = s_cand[i] & 0xffffff;
        double t = score_bf16_f64(reinterpret_cast<const uint4*>(x + (size_t)s_key[key] * kD),
                                  reinterpret_cast<const uint4*>(cu + (size_t)b * kD));
        if (bu) t += (double)bu[b];
        const unsigned long long o = ordered_bits(t);
        s_cscore[i] = o;
        atomicMax(&s_kbest[key], o);
      }
      __syncthreads();
      SAAP_TRACE(4);
      for (unsigned i = tid; i < n_cand; i += kRescoreThreads) {
        const int key = s_cand[i] >> 24, b = s_cand[i] & 0xffffff;
        if (s_cscore[i] == s_kbest[key]) atomicMin(&s_kid[key], b);
      }
      __syncthreads();
      // every key has a candidate (its fp32 maximum is within the bound of itself)
      if (tid < n_here) ids[s_key[tid]] = s_kid[tid];
      SAAP_TRACE(5);
    } else {
      // too many candidates: every key of the group against every centroid in double precision
      for (int key = 0; key < n_here; ++key) {
        const uint4* xk = reinterpret_cast<const uint4*>(x + (size_t)s_key[key] * kD);
        double best = 0.0;
        int best_id = -1;
        for (int b = tid; b < B; b += kRescoreThreads) {
          double t = score_bf16_f64(xk, reinterpret_cast<const uint4*>(cu + (size_t)b * kD));
          if (bu) t += (double)bu[b];
          if (better(t, b, best, best_id)) {
            best = t;
            best_id = b;
          }
        }
        for (int o = 1; o < 64; o <<= 1) {
          const double ob = __shfl_xor(best, o);
          const int oid = __shfl_xor(best_id, o);
          if (better(ob, oid, best, best_id)) {
            best = ob;
            best_id = oid;
          }
        }
        if (lane == 0) {
          s_wbest[wave] = best;
          s_wid[wave] = best_id;
        }
        __syncthreads();
        if (tid == 0) {
          for (int w = 1; w < kRescoreWaves; ++w)
            if (better(s_wbest[w], s_wid[w], best, best_id)) {
              best = s_wbest[w];
              best_id = s_wid[w];
            }
          ids[s_key[key]] = best_id;
        }
        __syncthreads();
      }
    }
    __syncthreads();
  }
  // Every workgroup has read its list length by now; the last one to leave keeps the total for
  // diagnostics and leaves all counters zero for the next call.
  __syncthreads();
  if (tid == 0) s_flag = atomicAdd(counters + Hkv, 1u) == gridDim.x * gridDim.y - 1 ? 1 : 0;
  __syncthreads();
  if (s_flag) {
    unsigned total = 0;
    for (int i = tid; i < Hkv; i += kRescoreThreads) {
      total += __hip_atomic_load(counters + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      counters[i] = 0u;
    }
    if (tid == 0) {
      *stat = 0u;
      counters[Hkv] = 0u;
    }
    __syncthreads();
    if (total) atomicAdd(stat, total);
  }
  SAAP_TRACE(6);
}

}  // namespace

// header | cmax[<=4095 floats] + 1 word: keys re-scored by the last call (16 KiB) | flagged row list [rows] int32
size_t assign_workspace_bytes(long long rows) {
  return (size_t)SAAP_WS_HEADER_BYTES + 16384 + (size_t)rows * sizeof(int32_t);
}

}  // namespace saap

using namespace saap;

extern "C" int32_t saap_assign_keys(const void* x, const void* centroids, const float* bias,
                                    int32_t* bucket_ids, int32_t S, int32_t Hkv, int32_t N, int32_t B,
                                    int32_t d, int32_t dtype, void* ws, size_t ws_bytes, void* stream) {
  begin_call();
  saap_trace_arm();
  if (!x || !centroids || !bucket_ids || !ws) return SAAP_INVALID_ARG;
  if (!aligned16(x) || !aligned16(centroids) || !aligned16(bucket_ids) || !aligned16(ws)) return SAAP_INVALID_ARG;
  if (S <= 0 || Hkv <= 0 || N <= 0 || B <= 0) return SAAP_INVALID_ARG;
  if (dtype != SAAP_F32 && dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  if (d != kD) return SAAP_UNSUPPORTED;
  const long long units = (long long)S * Hkv;
  const long long rows = units * N;
  if (rows > 0x7fffffffLL || units > 65535 || Hkv > 4095 || B >= (1 << 24)) return SAAP_UNSUPPORTED;
  if (ws_bytes < assign_workspace_bytes(rows)) return SAAP_WORKSPACE_TOO_SMALL;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const int cus = device_cus();

  if (dtype == SAAP_F32) {
    const long long grid = rows < (long long)cus * 8 ? rows : (long long)cus * 8;
    hipLaunchKernelGGL(assign_exact_f32_kernel, dim3((unsigned)grid), dim3(256), 0, hs, static_cast<const float*>(x),
                       static_cast<const float*>(centroids), bias, bucket_ids, rows, Hkv, N, B);
    return launch_status();
  }

  unsigned* n_flagged = reinterpret_cast<unsigned*>(ws);   // header words 0..Hkv, zero on entry: list lengths, arrivals
  const size_t list_cap = (size_t)S * N;                   // entries per head's list
  float* cmax = reinterpret_cast<float*>(static_cast<char*>(ws) + SAAP_WS_HEADER_BYTES);
  int32_t* flagged = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + SAAP_WS_HEADER_BYTES + 16384);
  const bf16_t* xb = static_cast<const bf16_t*>(x);
  const bf16_t* cb = static_cast<const bf16_t*>(centroids);
  // fp32 accumulation of 128 exact products: |error| <= 128 * 2^-24 * |x| |c| per score; two scores
  // are compared, and a factor 4 of head-room covers the matrix core's internal summation order.
  const float tol = 8.0f * 128.0f * 5.9604645e-8f;
  hipLaunchKernelGGL(cent_norm_kernel, dim3((unsigned)Hkv), dim3(kNormThreads), 0, hs, cb, cmax, B);
  const dim3 grid((unsigned)((N + kRowsPerWg - 1) / kRowsPerWg), (unsigned)units);
  if (bias)
    hipLaunchKernelGGL(assign_mfma_kernel<true>, grid, dim3(256), 0, hs, xb, cb, bias, cmax, bucket_ids, flagged,
                       n_flagged, list_cap, Hkv, N, B, tol);
  else
    hipLaunchKernelGGL(assign_mfma_kernel<false>, grid, dim3(256), 0, hs, xb, cb, bias, cmax, bucket_ids,
                       flagged, n_flagged, list_cap, Hkv, N, B, tol);
  unsigned* stat = reinterpret_cast<unsigned*>(cmax) + 4095;
  // workgroups per head: enough to fill the chip twice over all heads together
  const unsigned per_head = (unsigned)((cus * 2 + Hkv - 1) / Hkv);
  hipLaunchKernelGGL(assign_rescore_kernel, dim3((unsigned)Hkv, per_head), dim3(kRescoreThreads), 0, hs, xb, cb, bias, cmax,
                     bucket_ids, flagged, n_flagged, stat, list_cap, Hkv, B, tol);
  return launch_status();
}
