// classify_queries: the query assignment model f_q of arXiv 2502.08246 (Section 4, "Asymmetric
// assignment"; Section 6.1: a two-layer perceptron with a ReLU) evaluated for every query head.
//
// At decode only a handful of rows (G per KV head per sequence) meet each weight set, so the
// call is bound by streaming the weights once; the matrix cores are the instruction that does
// the (padded 16-row) products.  Two launches, three when probabilities are asked for:
//   hidden kernel   h = relu(W1 x + b1): one workgroup per (weight set, 16-row tile, 64 hidden
//                   units); h goes to the workspace in fp32.  With hidden = 0 the same kernel
//                   without the ReLU is the whole (one-layer) model.
//   output kernel   z = W2 h + b2: one workgroup of eight waves per (weight set, 16-row tile,
//                   32, 64 or 128 buckets), so that a 1024-bucket classifier for 8 KV heads fills all
//                   256 compute units with about 40 KB of loads each.  What one compute unit
//                   pulls from memory grows with the number of waves that have loads in flight,
//                   hence eight waves with few loads each rather than two with many.
//                   h is split into three bf16 planes (8+8+8 mantissa bits = the fp32 value
//                   exactly), so the matrix cores multiply exact operands and accumulate in fp32.
//   softmax kernel  one workgroup per row, in place (the decode step skips it: the selection
//                   kernel can take logits and do the softmax itself).
// Every global load is a whole 128-byte line per 8 lanes, issued before the first LDS store so
// that a workgroup's loads are all in flight together; matrix operands are read from LDS with a
// padded row pitch (no bank conflicts).  fp32 weights use v_mfma_f32_16x16x4_f32 with operands
// straight from memory (correctness configuration, not tuned).
#include "select_body.h"

namespace saap {
namespace {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;

struct MlpShape {
  int S, Hq, Hw, hidden, B;
  int rows_per_set;   // S * Hq / Hw
  int m_pad;          // rows_per_set rounded up to 16
};

// local row m of weight set w -> global query row (s*Hq + hq)
__device__ __forceinline__ int query_row(const MlpShape& sh, int w, int m) {
  const int heads = sh.Hq / sh.Hw;
  const int s = m / heads, hq = w * heads + m % heads;
  return s * sh.Hq + hq;
}

// 16-byte global load.  The batches of loads below are kept ahead of the LDS stores that consume
// them by straight-line code (clamped, unconditional stores) and a scheduling barrier, so that a
// workgroup's loads are all in flight together.  (A volatile load would do that too, but every
// volatile access is followed by a full wait.)
__device__ __forceinline__ u32x4_t load16(const void* p) { return *reinterpret_cast<const u32x4_t*>(p); }

// Decode a 1-D grid with the weight set fastest: workgroups are handed to the 8 XCDs round-robin,
// so with Hw a multiple of 8 all workgroups of a weight set share one L2.
__device__ __forceinline__ void decode_block(const MlpShape& sh, int& w, int& mt, int& slab) {
  w = blockIdx.x % sh.Hw;
  const int rest = blockIdx.x / sh.Hw;
  const int m_tiles = sh.m_pad / 16;
  mt = rest % m_tiles;
  slab = rest / m_tiles;
}

constexpr int kPitchD = kD + 8;     // LDS row pitch (bf16 elements) of d-wide tiles

// ---- bf16: hidden layer ------------------------------------------------------------------------
// LINEAR: the same product without the ReLU, written straight to the score rows: the one-layer
// model z = W x + b (sh.hidden is then the number of outputs).
template <bool LINEAR>
__global__ void __launch_bounds__(256)
mlp_hidden_bf16_kernel(const bf16_t* __restrict__ xq, const bf16_t* __restrict__ W1, const float* __restrict__ b1,
                       float* __restrict__ hbuf, MlpShape sh) {
  __shared__ __align__(16) bf16_t s_x[16 * kPitchD];
  __shared__ __align__(16) bf16_t s_w1[64 * kPitchD];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int w, mt, slab;
  decode_block(sh, w, mt, slab);
  const int rc = lane & 15, kg = lane >> 4;
  SAAP_TRACE(0);
  // coalesced loads: the 16 query rows (one piece per thread) and 64 rows of W1 (four pieces)
  const int prow = tid >> 4, pc = tid & 15;
  const int m = min(mt * 16 + prow, sh.rows_per_set - 1);
  const u32x4_t xr = load16(xq + (size_t)query_row(sh, w, m) * kD + pc * 8);
  u32x4_t wr[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int unit = min(slab * 64 + prow + 16 * i, sh.hidden - 1);
    wr[i] = load16(W1 + ((size_t)w * sh.hidden + unit) * kD + pc * 8);
  }
  // the bias of the lane's hidden unit travels with the weights: fetched after the products it would put one
  // more memory round trip in front of the stores
  const float bv = b1 ? b1[(size_t)w * sh.hidden + min(slab * 64 + wave * 16 + rc, sh.hidden - 1)] : 0.f;
  __builtin_amdgcn_sched_barrier(0);
  *reinterpret_cast<u32x4_t*>(s_x + prow * kPitchD + pc * 8) = xr;
#pragma unroll
  for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4_t*>(s_w1 + (prow + 16 * i) * kPitchD + pc * 8) = wr[i];
  __syncthreads();
  SAAP_TRACE(1);
  const int unit = slab * 64 + wave * 16 + rc;
  if (slab * 64 + wave * 16 >= sh.hidden) return;     // whole tile beyond the layer (hidden % 64 == 32)
  f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int st = 0; st < kD / 32; ++st) {
    const bf16x8_t a = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(s_x + rc * kPitchD + st * 32 + kg * 8));
    const bf16x8_t b = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(s_w1 + (wave * 16 + rc) * kPitchD + st * 32 + kg * 8));
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
  }
  // accumulator i of this lane: row 4*kg + i, hidden unit `unit`
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = mt * 16 + 4 * kg + i;
    if (row < sh.rows_per_set) {
      if constexpr (LINEAR) hbuf[(size_t)query_row(sh, w, row) * sh.hidden + unit] = acc[i] + bv;
      else hbuf[((size_t)w * sh.m_pad + row) * sh.hidden + unit] = fmaxf(acc[i] + bv, 0.f);
    }
  }
  SAAP_TRACE(2);
}

// ---- bf16: output layer ------------------------------------------------------------------------
constexpr int kOutChunk = 512;      // hidden units per LDS pass of the output kernel
// Eight waves per workgroup: what one compute unit pulls from memory grows with the number of
// waves that have loads in flight (two waves were measured at a third of the rate of eight).
// A workgroup takes SLAB = 32 buckets, or 64 when 32 would make more than one workgroup per compute
// unit (128 when 64 still would and the tiles fit).  For the matrix products wave (t, kq) takes
// bucket tile t of the SLAB/16 and every KQ-th k-step starting at kq (KQ = 8 / tiles); the KQ partial products of a tile are added
// through LDS in a fixed order.
constexpr int kOutThreads = 512;
constexpr int kOutLoads = 16 * 128 / kOutThreads;     // 16-byte loads of activations per thread

// FUSED: the selection of the decode step runs in this launch.  At batch 1 with one weight set per KV head the
// workgroups of a weight set produce exactly the logits of one bucket list; they store them write-through, count
// their arrival, and the last one to arrive runs the selection of that list (softmax, group sum, top nprobe, visit
// plan) on the spot, reading the logits past its XCD's L2.  One launch and its dependent wait less per step.
struct FusedSelect {
  unsigned* counters;     // one per weight set, a cache line apart, zero on entry and on exit
  float* probs;           // [Hq,B] or null
  int32_t* selected;      // [Hkv,nprobe]
  int Hkv, nprobe, n_sort, cap, ept, expect;
  PlanOut po;
};

template <int SLAB, bool FUSED>
__global__ void __launch_bounds__(kOutThreads)
mlp_out_bf16_kernel(const float* __restrict__ hbuf, const bf16_t* __restrict__ W2, const float* __restrict__ b2,
                    float* __restrict__ scores, MlpShape sh, FusedSelect fs) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int w, mt, slab;
  decode_block(sh, w, mt, slab);
  const int rc = lane & 15, kg = lane >> 4;
  constexpr int kTiles = SLAB / 16, KQ = 8 / kTiles;
  constexpr int kWLoads = SLAB * 64 / kOutThreads;      // 16-byte loads of weights per thread (chunk of 512)
  const int b0 = slab * SLAB;
  const int chunk_max = min(sh.hidden, kOutChunk);
  const int pitch = chunk_max + 8;
  // LDS rows per plane of h: the real rows only (4 of a 16-row tile at batch 1), which lets three
  // workgroups share a compute unit; rows of A beyond them repeat the last real row, and a row of
  // A only reaches the same row of the product, which is dropped
  const int h_rows = min(16, sh.rows_per_set);
  bf16_t* s_h = reinterpret_cast<bf16_t*>(smem);       // [3][h_rows][pitch]
  bf16_t* s_w2 = s_h + 3 * h_rows * pitch;             // [SLAB][pitch]
  const float* hrows = hbuf + ((size_t)w * sh.m_pad + mt * 16) * sh.hidden;
  const int rows_here = min(16, sh.rows_per_set - mt * 16);    // real rows of this tile (>= 1)
  // one accumulator per plane: three independent chains of matrix instructions, added at the end
  f32x4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = acc0, acc2 = acc0;
  SAAP_TRACE(0);
  // the bias of the bucket this lane will write (waves 0 .. kTiles-1), fetched with the first weights: after the
  // products it would put one more memory round trip in front of the stores
  const float bo = b2 ? b2[(size_t)w * sh.B + min(b0 + (wave % kTiles) * 16 + rc, sh.B - 1)] : 0.f;
  for (int c0 = 0; c0 < sh.hidden; c0 += kOutChunk) {
    const int kc = min(kOutChunk, sh.hidden - c0);      // multiple of 32
    // all loads of the pass first: SLAB rows of W2 (kc/8 pieces each) and 16 rows of h (kc/4 pieces)
    const int pw = kc / 8, ph = kc / 4;
    // piece index -> (row, piece of the row); a shift when the pieces per row are a power of two
    // (hidden = 256, 512, 1024: the usual case), a division otherwise
    const int pw_sh = (pw & (pw - 1)) == 0 ? 31 - __clz(pw) : -1;
    const int ph_sh = pw_sh >= 0 ? pw_sh + 1 : -1;
    auto split_w = [&](int q, int& row, int& pc) {
      if (pw_sh >= 0) { row = q >> pw_sh; pc = q & (pw - 1); } else { row = q / pw; pc = q % pw; }
    };
    auto split_h = [&](int q, int& row, int& pc) {
      if (ph_sh >= 0) { row = q >> ph_sh; pc = q & (ph - 1); } else { row = q / ph; pc = q % ph; }
    };
    u32x4_t wv[kWLoads], hv[kOutLoads];
#pragma unroll
    for (int i = 0; i < kWLoads; ++i) {
      int row, pc;
      split_w(min(tid + kOutThreads * i, SLAB * pw - 1), row, pc);
      const int b = min(b0 + row, sh.B - 1);
      wv[i] = load16(W2 + ((size_t)w * sh.B + b) * sh.hidden + c0 + pc * 8);
    }
    // only the tile's real rows are fetched
#pragma unroll
    for (int i = 0; i < kOutLoads; ++i) {
      int row, pc;
      split_h(min(tid + kOutThreads * i, rows_here * ph - 1), row, pc);
      hv[i] = load16(hrows + (size_t)row * sh.hidden + c0 + pc * 4);
    }
    __builtin_amdgcn_sched_barrier(0);
    if (c0 == 0) SAAP_TRACE(4);
    if (c0 > 0) __syncthreads();                        // the previous pass is done with the LDS tiles
    // stores use the same clamped piece index as the loads: surplus threads rewrite the last
    // piece with identical data, and the code stays free of branches
#pragma unroll
    for (int i = 0; i < kWLoads; ++i) {
      int row, pc;
      split_w(min(tid + kOutThreads * i, SLAB * pw - 1), row, pc);
      *reinterpret_cast<u32x4_t*>(s_w2 + row * pitch + pc * 8) = wv[i];
    }
    if (c0 == 0) SAAP_TRACE(5);
#pragma unroll
    for (int i = 0; i < kOutLoads; ++i) {
      int hrow_i, hpc_i;
      split_h(min(tid + kOutThreads * i, rows_here * ph - 1), hrow_i, hpc_i);
      {
        // four activations -> three planes of truncated bf16 pieces: h == p0 + p1 + p2 exactly
        uint32_t p0[4], p1[4], p2[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float hval = __uint_as_float(hv[i][j]);
          p0[j] = __float_as_uint(hval) & 0xffff0000u;
          const float r1 = hval - __uint_as_float(p0[j]);
          p1[j] = __float_as_uint(r1) & 0xffff0000u;
          const float r2 = r1 - __uint_as_float(p1[j]);
          p2[j] = __float_as_uint(r2) & 0xffff0000u;
        }
        bf16_t* dst = s_h + hrow_i * pitch + hpc_i * 4;
        *reinterpret_cast<uint2*>(dst) = make_uint2((p0[0] >> 16) | p0[1], (p0[2] >> 16) | p0[3]);
        *reinterpret_cast<uint2*>(dst + h_rows * pitch) = make_uint2((p1[0] >> 16) | p1[1], (p1[2] >> 16) | p1[3]);
        *reinterpret_cast<uint2*>(dst + 2 * h_rows * pitch) = make_uint2((p2[0] >> 16) | p2[1], (p2[2] >> 16) | p2[3]);
      }
    }
    __syncthreads();
    if (c0 == 0) SAAP_TRACE(1);
    const int tile = wave % kTiles, kq = wave / kTiles;
    const bf16_t* wrow = s_w2 + (tile * 16 + rc) * pitch + kg * 8;
    const bf16_t* hrow = s_h + min(rc, rows_here - 1) * pitch + kg * 8;
    auto lds16 = [](const bf16_t* ptr) { return __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(ptr)); };
    const int nst = kc / 32;
    int st = kq;
    // four of the wave's k-steps at a time: their sixteen LDS reads go out before the twelve
    // matrix instructions, so the read latency is paid once per group instead of once per step
    for (; st + 3 * KQ < nst; st += 4 * KQ) {
      bf16x8_t b[4], a0[4], a1[4], a2[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        b[u] = lds16(wrow + (st + KQ * u) * 32);
        a0[u] = lds16(hrow + (st + KQ * u) * 32);
        a1[u] = lds16(hrow + h_rows * pitch + (st + KQ * u) * 32);
        a2[u] = lds16(hrow + 2 * h_rows * pitch + (st + KQ * u) * 32);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        acc2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2[u], b[u], acc2, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1[u], b[u], acc1, 0, 0, 0);
        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0[u], b[u], acc0, 0, 0, 0);
      }
    }
    for (; st < nst; st += KQ) {
      const bf16x8_t b = lds16(wrow + st * 32);
      acc2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lds16(hrow + 2 * h_rows * pitch + st * 32), b, acc2, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lds16(hrow + h_rows * pitch + st * 32), b, acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lds16(hrow + st * 32), b, acc0, 0, 0, 0);
    }
  }
  // smallest pieces first; then the four k-quarters of a bucket tile, in order, through LDS
  f32x4_t acc = (acc2 + acc1) + acc0;
  __syncthreads();                                      // the operand tiles are dead
  f32x4_t* s_part = reinterpret_cast<f32x4_t*>(smem);   // [8 waves][64 lanes]
  s_part[wave * 64 + lane] = acc;
  __syncthreads();
  if constexpr (!FUSED) {
    if (wave >= kTiles) return;
  }
  if (wave < kTiles) {
    acc = s_part[wave * 64 + lane];
#pragma unroll
    for (int j = 1; j < KQ; ++j) acc += s_part[(wave + kTiles * j) * 64 + lane];
    SAAP_TRACE(2);
    const int bucket = b0 + wave * 16 + rc;
    if (bucket < sh.B) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int mm = mt * 16 + 4 * kg + i;
        if (mm < sh.rows_per_set) {
          float* dst = scores + (size_t)query_row(sh, w, mm) * sh.B + bucket;
          if constexpr (FUSED) __hip_atomic_store(dst, acc[i] + bo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          else *dst = acc[i] + bo;
        }
      }
    }
  }
  SAAP_TRACE(3);
  if constexpr (FUSED) {
    __shared__ int s_is_last;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // the logits are out
    __syncthreads();
    if (tid == 0) {
      unsigned* c = fs.counters + (size_t)w * 32;
      const unsigned old = __hip_atomic_fetch_add(c, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_is_last = old == (unsigned)(fs.expect - 1);
      if (s_is_last) __hip_atomic_store(c, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!s_is_last) return;
    // weight set w = KV head w: its G rows of logits are complete
    switch (fs.ept) {
      case 2: select_radix_body<2, true, true>(smem, w, scores, fs.probs, fs.selected, sh.Hq, fs.Hkv, sh.B, fs.nprobe, 0, fs.n_sort, fs.cap, fs.po); break;
      case 4: select_radix_body<4, true, true>(smem, w, scores, fs.probs, fs.selected, sh.Hq, fs.Hkv, sh.B, fs.nprobe, 0, fs.n_sort, fs.cap, fs.po); break;
      default: select_radix_body<8, true, true>(smem, w, scores, fs.probs, fs.selected, sh.Hq, fs.Hkv, sh.B, fs.nprobe, 0, fs.n_sort, fs.cap, fs.po); break;
    }
  }
}

// ---- fp32 (correctness configuration): operands straight from memory ------------------------------
template <bool LINEAR>
__global__ void __launch_bounds__(256)
mlp_hidden_f32_kernel(const float* __restrict__ xq, const float* __restrict__ W1, const float* __restrict__ b1,
                      float* __restrict__ hbuf, MlpShape sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int utile = blockIdx.x * 4 + wave;           // tile of 16 hidden units
  if (utile * 16 >= sh.hidden) return;
  const int mt = blockIdx.y, w = blockIdx.z;
  const int rc = lane & 15, kg = lane >> 4;
  const int m = min(mt * 16 + rc, sh.rows_per_set - 1);
  const float* xr = xq + (size_t)query_row(sh, w, m) * kD;
  const float* wr = W1 + ((size_t)w * sh.hidden + utile * 16 + rc) * kD;
  f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
  for (int st = 0; st < kD / 4; ++st)
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(xr[st * 4 + kg], wr[st * 4 + kg], acc, 0, 0, 0);
  const int unit = utile * 16 + rc;
  const float bv = b1 ? b1[(size_t)w * sh.hidden + unit] : 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = mt * 16 + 4 * kg + i;
    if constexpr (LINEAR) {
      if (row < sh.rows_per_set) hbuf[(size_t)query_row(sh, w, row) * sh.hidden + unit] = acc[i] + bv;
    } else {
      hbuf[((size_t)w * sh.m_pad + row) * sh.hidden + unit] = fmaxf(acc[i] + bv, 0.f);
    }
  }
}

__global__ void __launch_bounds__(256)
mlp_out_f32_kernel(const float* __restrict__ hbuf, const float* __restrict__ W2, const float* __restrict__ b2,
                   float* __restrict__ scores, MlpShape sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int btile = blockIdx.x * 4 + wave;           // tile of 16 buckets
  if (btile * 16 >= sh.B) return;
  const int mt = blockIdx.y, w = blockIdx.z;
  const int rc = lane & 15, kg = lane >> 4;
  const float* hp = hbuf + ((size_t)w * sh.m_pad + mt * 16 + rc) * sh.hidden;
  const float* wr = W2 + ((size_t)w * sh.B + btile * 16 + rc) * sh.hidden;
  f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
  for (int st = 0; st < sh.hidden / 4; ++st)
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(hp[st * 4 + kg], wr[st * 4 + kg], acc, 0, 0, 0);
  const int bucket = btile * 16 + rc;
  const float bv = b2 ? b2[(size_t)w * sh.B + bucket] : 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = mt * 16 + 4 * kg + i;
    if (m < sh.rows_per_set) scores[(size_t)query_row(sh, w, m) * sh.B + bucket] = acc[i] + bv;
  }
}

// Row softmax in place; the row is held in registers between the passes.
__global__ void __launch_bounds__(256) softmax_rows_kernel(float* __restrict__ scores, int B) {
  __shared__ float s_red[4];
  constexpr int kMaxPerThread = SAAP_MAX_BUCKETS / 256;
  float* row = scores + (size_t)blockIdx.x * B;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float v[kMaxPerThread];
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < kMaxPerThread; ++i) {
    const int b = tid + i * 256;
    v[i] = b < B ? row[b] : -INFINITY;
    mx = fmaxf(mx, v[i]);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
  if (lane == 0) s_red[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
  __syncthreads();
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < kMaxPerThread; ++i) {
    v[i] = __expf(v[i] - mx);      // exp(-inf) = 0 for the padding
    sum += v[i];
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
  if (lane == 0) s_red[wave] = sum;
  __syncthreads();
  sum = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
  const float inv = 1.0f / sum;
#pragma unroll
  for (int i = 0; i < kMaxPerThread; ++i) {
    const int b = tid + i * 256;
    if (b < B) row[b] = v[i] * inv;
  }
}

}  // namespace

// header | hidden activations fp32 [weight sets][rows padded to 16][hidden]; every weight set pads
// its rows to a multiple of 16 and there are at most `rows` sets of one row each
size_t classify_workspace_bytes(long long rows, int hidden) {
  return (size_t)SAAP_WS_HEADER_BYTES + (size_t)rows * 16 * hidden * sizeof(float);
}

}  // namespace saap

using namespace saap;

// The two launches of the bf16 two-layer model; with `fs` the output kernel also selects (see FusedSelect).
static int32_t launch_mlp_bf16(const void* xq, const void* W1, const float* b1, const void* W2, const float* b2,
                               float* scores, float* hbuf, const MlpShape& sh, const FusedSelect* fs, hipStream_t hs) {
  const int hidden = sh.hidden, B = sh.B, Hw = sh.Hw;
  const int m_tiles = sh.m_pad / 16;
  const unsigned g1 = (unsigned)((hidden + 63) / 64) * m_tiles * Hw;
  // 64 buckets per workgroup when 32 would give more than one workgroup per compute unit: every
  // workgroup reads its rows of the hidden activations (as many bytes as a 32-bucket slab of W2 for a
  // full 16-row tile), so fewer, wider workgroups move fewer bytes (batch 8: 11.5 -> 8.8 us)
  const bool wide = (long long)((B + 31) / 32) * m_tiles * Hw > (long long)device_cus();
  int slab_rows = wide ? 64 : 32;
  {
    // 128 buckets when 64 would still give more than one workgroup per compute unit and the tiles fit the LDS of one
    // (few rows per weight set): with one workgroup per compute unit all loads of the launch are in flight at once
    // and no second round of workgroups waits behind the first (4096 buckets, batch 1: 12.7 -> 10.9 us)
    const int rows = sh.rows_per_set < 16 ? sh.rows_per_set : 16;
    const size_t lds128 = (size_t)(3 * rows + 128) * ((hidden < kOutChunk ? hidden : kOutChunk) + 8) * sizeof(bf16_t);
    if (wide && (long long)((B + 63) / 64) * m_tiles * Hw > (long long)device_cus() && lds128 <= 150 * 1024)
      slab_rows = 128;
  }
  const unsigned g2 = (unsigned)((B + slab_rows - 1) / slab_rows) * m_tiles * Hw;
  hipLaunchKernelGGL(mlp_hidden_bf16_kernel<false>, dim3(g1), dim3(256), 0, hs, static_cast<const bf16_t*>(xq),
                     static_cast<const bf16_t*>(W1), b1, hbuf, sh);
  const int chunk = hidden < kOutChunk ? hidden : kOutChunk;
  const int h_rows = sh.rows_per_set < 16 ? sh.rows_per_set : 16;
  size_t lds = (size_t)(3 * h_rows + slab_rows) * (chunk + 8) * sizeof(bf16_t);
  const size_t lds_part = (size_t)kOutThreads * sizeof(f32x4_t);      // partial products of the eight waves
  if (lds < lds_part) lds = lds_part;
  FusedSelect f{};
  if (fs) {
    f = *fs;
    f.expect = (int)((B + slab_rows - 1) / slab_rows);
    const SelectGeometry geo = select_geometry(B, f.nprobe, f.po.off != nullptr, f.po.runs);
    f.n_sort = geo.n_sort;
    f.cap = geo.cap;
    f.po.lds_off = geo.plan_off;
    if (lds < geo.lds) lds = geo.lds;
  }
  // the same slab width with and without the selection: the logits of both calls are then equal bit for bit
  auto launch = [&](auto kernel) -> int32_t {
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return SAAP_HIP_ERROR;
    hipLaunchKernelGGL(kernel, dim3(g2), dim3(kOutThreads), lds, hs, hbuf, static_cast<const bf16_t*>(W2), b2, scores, sh, f);
    return SAAP_OK;
  };
  if (fs) {
    if (slab_rows == 128) return launch(mlp_out_bf16_kernel<128, true>);
    if (slab_rows == 64) return launch(mlp_out_bf16_kernel<64, true>);
    return launch(mlp_out_bf16_kernel<32, true>);
  }
  if (slab_rows == 128) return launch(mlp_out_bf16_kernel<128, false>);
  if (slab_rows == 64) return launch(mlp_out_bf16_kernel<64, false>);
  return launch(mlp_out_bf16_kernel<32, false>);
}

extern "C" int32_t saap_classify_queries(const void* xq, const void* W1, const float* b1, const void* W2,
                                         const float* b2, int32_t Hw, float* scores, int32_t S, int32_t Hq,
                                         int32_t Hkv, int32_t d, int32_t hidden, int32_t B, int32_t dtype,
                                         int32_t output_kind, void* ws, size_t ws_bytes, void* stream) {
  begin_call();
  const bool linear = hidden == 0;      // one-layer model z = W2 x + b2, W2 [Hw,B,d]; W1 and b1 unused
  if (!xq || (!linear && !W1) || !W2 || !scores || !ws) return SAAP_INVALID_ARG;
  if (!aligned16(xq) || !aligned16(W1) || !aligned16(W2) || !aligned16(scores) || !aligned16(ws))
    return SAAP_INVALID_ARG;
  if (S <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || hidden < 0 || B <= 0) return SAAP_INVALID_ARG;
  if (Hw != 1 && Hw != Hkv && Hw != Hq) return SAAP_INVALID_ARG;
  if (dtype != SAAP_F32 && dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  if (output_kind != SAAP_PROBS && output_kind != SAAP_LOGITS) return SAAP_INVALID_ARG;
  if (d != kD || hidden % 32 != 0 || B % 16 != 0 || B > SAAP_MAX_BUCKETS || hidden > 1536) return SAAP_UNSUPPORTED;
  MlpShape sh;
  sh.S = S; sh.Hq = Hq; sh.Hw = Hw; sh.hidden = linear ? B : hidden; sh.B = B;
  sh.rows_per_set = S * (Hq / Hw);
  sh.m_pad = (sh.rows_per_set + 15) / 16 * 16;
  const size_t need = (size_t)SAAP_WS_HEADER_BYTES + (size_t)Hw * sh.m_pad * hidden * sizeof(float);
  if (ws_bytes < need) return SAAP_WORKSPACE_TOO_SMALL;
  const int m_tiles = sh.m_pad / 16;
  if (m_tiles > 65535 || Hw > 65535) return SAAP_UNSUPPORTED;
  float* hbuf = reinterpret_cast<float*>(static_cast<char*>(ws) + SAAP_WS_HEADER_BYTES);
  hipStream_t hs = static_cast<hipStream_t>(stream);
  saap_trace_arm();
  if (linear) {
    if (dtype == SAAP_BF16) {
      const unsigned g = (unsigned)((B + 63) / 64) * m_tiles * Hw;
      hipLaunchKernelGGL(mlp_hidden_bf16_kernel<true>, dim3(g), dim3(256), 0, hs, static_cast<const bf16_t*>(xq),
                         static_cast<const bf16_t*>(W2), b2, scores, sh);
    } else {
      const dim3 g((unsigned)((B / 16 + 3) / 4), (unsigned)m_tiles, (unsigned)Hw);
      hipLaunchKernelGGL(mlp_hidden_f32_kernel<true>, g, dim3(256), 0, hs, static_cast<const float*>(xq),
                         static_cast<const float*>(W2), b2, scores, sh);
    }
  } else if (dtype == SAAP_BF16) {
    const int32_t st = launch_mlp_bf16(xq, W1, b1, W2, b2, scores, hbuf, sh, nullptr, hs);
    if (st != SAAP_OK) return st;
  } else {
    const dim3 g1((unsigned)((hidden / 16 + 3) / 4), (unsigned)m_tiles, (unsigned)Hw);
    const dim3 g2((unsigned)((B / 16 + 3) / 4), (unsigned)m_tiles, (unsigned)Hw);
    hipLaunchKernelGGL(mlp_hidden_f32_kernel<false>, g1, dim3(256), 0, hs, static_cast<const float*>(xq),
                       static_cast<const float*>(W1), b1, hbuf, sh);
    hipLaunchKernelGGL(mlp_out_f32_kernel, g2, dim3(256), 0, hs, hbuf, static_cast<const float*>(W2), b2, scores,
                       sh);
  }
  if (output_kind == SAAP_PROBS)
    hipLaunchKernelGGL(softmax_rows_kernel, dim3((unsigned)(S * Hq)), dim3(256), 0, hs, scores, B);
  return launch_status();
}

// classify_queries (logits) and the selection of the decode step in one call.  At batch 1 with one weight set per
// KV head (the benchmark setting) the selection runs inside the classifier's output launch; any other shape takes the
// separate calls, with the same results.
extern "C" int32_t saap_classify_select(const void* xq, const void* W1, const float* b1, const void* W2,
                                        const float* b2, int32_t Hw, float* logits, float* probs,
                                        int32_t* selected, const int32_t* off, const int32_t* len,
                                        int32_t resident_run, int32_t* plan, int32_t S, int32_t Hq, int32_t Hkv,
                                        int32_t d, int32_t hidden, int32_t B, int32_t nprobe, int32_t dtype,
                                        void* ws, size_t ws_bytes, void* stream) {
  begin_call();
  const bool with_plan = plan != nullptr;
  if (with_plan && (!off || !len || !aligned16(plan))) return SAAP_INVALID_ARG;
  if (!logits || !selected || !aligned16(selected)) return SAAP_INVALID_ARG;
  if (resident_run != -1 && resident_run != B) return SAAP_INVALID_ARG;
  if (nprobe < 0 || nprobe > B) return SAAP_INVALID_ARG;
  const int G = Hkv > 0 && Hq % Hkv == 0 ? Hq / Hkv : 0;
  SelectGeometry geo = select_geometry(B > 0 ? B : 1, nprobe, false, 0);
  const bool fusable = dtype == SAAP_BF16 && hidden > 0 && S == 1 && Hw == Hkv && B <= 8 * kOutThreads && nprobe > 0 &&
                       geo.n_sort < geo.n_pow2 && (G == 1 || G == 2 || G == 4 || G == 8) &&
                       (size_t)Hw * 128 <= SAAP_WS_HEADER_BYTES;
  if (!fusable) {
    int32_t st = saap_classify_queries(xq, W1, b1, W2, b2, Hw, logits, S, Hq, Hkv, d, hidden, B, dtype, SAAP_LOGITS, ws,
                                       ws_bytes, stream);
    if (st != SAAP_OK) return st;
    if (with_plan)
      return saap_select_buckets_planned(logits, SAAP_LOGITS, probs, off, len, resident_run, selected, plan, S, Hq, Hkv, B,
                                         nprobe, SAAP_GROUP_SUM, ws, ws_bytes, stream);
    return saap_select_buckets_from_logits(logits, probs, selected, S, Hq, Hkv, B, nprobe, SAAP_GROUP_SUM, ws, ws_bytes,
                                           stream);
  }
  // the checks of saap_classify_queries
  if (!xq || !W1 || !W2 || !ws) return SAAP_INVALID_ARG;
  if (!aligned16(xq) || !aligned16(W1) || !aligned16(W2) || !aligned16(logits) || !aligned16(ws) || !aligned16(probs))
    return SAAP_INVALID_ARG;
  if (Hq <= 0 || Hkv <= 0 || B <= 0) return SAAP_INVALID_ARG;
  if (d != kD || hidden % 32 != 0 || B % 16 != 0 || B > SAAP_MAX_BUCKETS || hidden > 1536) return SAAP_UNSUPPORTED;
  MlpShape sh;
  sh.S = S; sh.Hq = Hq; sh.Hw = Hw; sh.hidden = hidden; sh.B = B;
  sh.rows_per_set = S * (Hq / Hw);
  sh.m_pad = (sh.rows_per_set + 15) / 16 * 16;
  const size_t need = (size_t)SAAP_WS_HEADER_BYTES + (size_t)Hw * sh.m_pad * hidden * sizeof(float);
  if (ws_bytes < need) return SAAP_WORKSPACE_TOO_SMALL;
  float* hbuf = reinterpret_cast<float*>(static_cast<char*>(ws) + SAAP_WS_HEADER_BYTES);
  FusedSelect fs{};
  fs.counters = reinterpret_cast<unsigned*>(ws);
  fs.probs = probs; fs.selected = selected; fs.Hkv = Hkv; fs.nprobe = nprobe;
  fs.ept = B <= 2 * kOutThreads ? 2 : B <= 4 * kOutThreads ? 4 : 8;
  if (with_plan) {
    fs.po.off = off; fs.po.len = len; fs.po.plan = plan;
    fs.po.runs = B + (resident_run >= 0 ? 1 : 0);
    fs.po.resident = resident_run;
    fs.po.ps = (2 * (nprobe + (resident_run >= 0 ? 1 : 0)) + 2 + 3) & ~3;
  }
  saap_trace_arm();
  const int32_t st = launch_mlp_bf16(xq, W1, b1, W2, b2, logits, hbuf, sh, &fs, static_cast<hipStream_t>(stream));
  return st != SAAP_OK ? st : launch_status();
}
