// classify_queries: the query assignment model f_q of arXiv 2502.08246 (Section 4, "Asymmetric
// assignment"; Section 6.1: a two-layer perceptron with a ReLU) evaluated for every query head.
//
// At decode only a handful of rows (G per KV head per sequence) meet each weight set, so the
// call is bound by streaming the weights once; the matrix cores are the instruction that does
// the (padded 16-row) products:
//   fused kernel   (bf16) one workgroup per (64 buckets, 16 rows, weight set): h = relu(W1 x + b1)
//                  for all hidden units into LDS, split into three bf16 planes (8+8+8 mantissa
//                  bits = the fp32 value exactly), so the second layer again multiplies exact
//                  bf16 operands and accumulates in fp32; then z = W2 h + b2.
//   softmax kernel one workgroup per row, in place.
// fp32 weights use v_mfma_f32_16x16x4_f32 in two launches (hidden, output) with h in the
// workspace as one fp32 plane.
#include "common.h"

namespace saap {
namespace {

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

template <typename T>
__global__ void __launch_bounds__(256)
mlp_hidden_kernel(const T* __restrict__ xq, const T* __restrict__ W1, const float* __restrict__ b1,
                  void* __restrict__ hbuf, MlpShape sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int utile = blockIdx.x * 4 + wave;           // tile of 16 hidden units
  if (utile * 16 >= sh.hidden) return;
  const int mt = blockIdx.y, w = blockIdx.z;
  const int rc = lane & 15, kg = lane >> 4;
  const int m = min(mt * 16 + rc, sh.rows_per_set - 1);
  const T* xr = xq + (size_t)query_row(sh, w, m) * kD;
  const T* wr = W1 + ((size_t)w * sh.hidden + utile * 16 + rc) * kD;
  f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
  if constexpr (sizeof(T) == 2) {
#pragma unroll
    for (int st = 0; st < kD / 32; ++st) {
      const bf16x8_t a = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(xr + st * 32 + kg * 8));
      const bf16x8_t b = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(wr + st * 32 + kg * 8));
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
    }
  } else {
#pragma unroll 8
    for (int st = 0; st < kD / 4; ++st)
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(xr[st * 4 + kg], wr[st * 4 + kg], acc, 0, 0, 0);
  }
  // accumulator i of this lane: row 4*kg + i, hidden unit utile*16 + rc
  const int unit = utile * 16 + rc;
  const float bv = b1 ? b1[(size_t)w * sh.hidden + unit] : 0.f;
  const size_t plane = (size_t)sh.Hw * sh.m_pad * sh.hidden;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = mt * 16 + 4 * kg + i;
    const float hval = fmaxf(acc[i] + bv, 0.f);
    const size_t o = ((size_t)w * sh.m_pad + row) * sh.hidden + unit;
    if constexpr (sizeof(T) == 2) {
      bf16_t* hp = static_cast<bf16_t*>(hbuf);
      // three truncated bf16 pieces: hval == p0 + p1 + p2 exactly
      const uint32_t u0 = __float_as_uint(hval) & 0xffff0000u;
      const float r1 = hval - __uint_as_float(u0);
      const uint32_t u1 = __float_as_uint(r1) & 0xffff0000u;
      const float r2 = r1 - __uint_as_float(u1);
      const uint32_t u2 = __float_as_uint(r2) & 0xffff0000u;
      hp[o] = (bf16_t)(u0 >> 16);
      hp[plane + o] = (bf16_t)(u1 >> 16);
      hp[2 * plane + o] = (bf16_t)(u2 >> 16);
    } else {
      static_cast<float*>(hbuf)[o] = hval;
    }
  }
}

// Output layer.  The four waves of a workgroup share one (weight set, 16-row tile): the
// activations (all planes) are staged in LDS once, every wave streams the W2 rows of its 16
// buckets with all loads of a 16-step block issued before the first matrix instruction.
template <typename T>
__global__ void __launch_bounds__(256)
mlp_out_kernel(const void* __restrict__ hbuf, const T* __restrict__ W2, const float* __restrict__ b2,
               float* __restrict__ scores, MlpShape sh) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int btile = blockIdx.x * 4 + wave;           // tile of 16 buckets
  const int mt = blockIdx.y, w = blockIdx.z;
  const int rc = lane & 15, kg = lane >> 4;
  const size_t plane = (size_t)sh.Hw * sh.m_pad * sh.hidden;
  const size_t hrow0 = ((size_t)w * sh.m_pad + mt * 16) * sh.hidden;
  const bool active = btile * 16 < sh.B;
  f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
  if constexpr (sizeof(T) == 2) {
    // LDS image: [plane][16 rows][hidden + 8] bf16 (row pitch padded against bank conflicts)
    const int pitch = sh.hidden + 8;
    bf16_t* s_h = reinterpret_cast<bf16_t*>(smem);
    const bf16_t* hp = static_cast<const bf16_t*>(hbuf) + hrow0;
    const int pieces_per_row = sh.hidden / 8;          // 16-byte pieces
    const T* wr = W2 + ((size_t)w * sh.B + (active ? btile * 16 + rc : 0)) * sh.hidden + kg * 8;
    constexpr int kBlock = 16;                          // steps of 32 hidden units per load block
    const int steps = sh.hidden / 32;
    uint4 wreg[kBlock];
#pragma unroll
    for (int i = 0; i < kBlock; ++i)
      if (i < steps) wreg[i] = *reinterpret_cast<const uint4*>(wr + i * 32);
    const int n_pieces = 3 * 16 * pieces_per_row;
    constexpr int kStage = 12;                          // pieces in flight per thread
    for (int i0 = tid; i0 < n_pieces; i0 += 256 * kStage) {
      uint4 tmp[kStage];
#pragma unroll
      for (int k = 0; k < kStage; ++k) {
        const int i = i0 + k * 256;
        if (i < n_pieces) {
          const int pl = i / (16 * pieces_per_row), rem = i % (16 * pieces_per_row);
          const int r = rem / pieces_per_row, pc = rem % pieces_per_row;
          tmp[k] = *reinterpret_cast<const uint4*>(hp + (size_t)pl * plane + (size_t)r * sh.hidden + pc * 8);
        }
      }
#pragma unroll
      for (int k = 0; k < kStage; ++k) {
        const int i = i0 + k * 256;
        if (i < n_pieces) {
          const int pl = i / (16 * pieces_per_row), rem = i % (16 * pieces_per_row);
          const int r = rem / pieces_per_row, pc = rem % pieces_per_row;
          *reinterpret_cast<uint4*>(s_h + ((size_t)pl * 16 + r) * pitch + pc * 8) = tmp[k];
        }
      }
    }
    __syncthreads();
    for (int s0 = 0; s0 < steps; s0 += kBlock) {
#pragma unroll
      for (int i = 0; i < kBlock; ++i) {
        if (s0 + i < steps) {
          const int k = (s0 + i) * 32 + kg * 8;
          const bf16x8_t b = __builtin_bit_cast(bf16x8_t, wreg[i]);
          const bf16x8_t a0 = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(s_h + (size_t)(0 * 16 + rc) * pitch + k));
          const bf16x8_t a1 = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(s_h + (size_t)(1 * 16 + rc) * pitch + k));
          const bf16x8_t a2 = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(s_h + (size_t)(2 * 16 + rc) * pitch + k));
          // smallest pieces first: their sum is rounded least by the fp32 accumulator
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, b, acc, 0, 0, 0);
        }
      }
      if (s0 + kBlock < steps) {
#pragma unroll
        for (int i = 0; i < kBlock; ++i)
          if (s0 + kBlock + i < steps) wreg[i] = *reinterpret_cast<const uint4*>(wr + (s0 + kBlock + i) * 32);
      }
    }
  } else {
    const float* hp = static_cast<const float*>(hbuf) + hrow0 + (size_t)rc * sh.hidden;
    const T* wr = W2 + ((size_t)w * sh.B + (active ? btile * 16 + rc : 0)) * sh.hidden;
    for (int st = 0; st < sh.hidden / 4; ++st)
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(hp[st * 4 + kg], wr[st * 4 + kg], acc, 0, 0, 0);
  }
  if (!active) return;
  const int bucket = btile * 16 + rc;
  const float bv = b2 ? b2[(size_t)w * sh.B + bucket] : 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = mt * 16 + 4 * kg + i;
    if (m < sh.rows_per_set) scores[(size_t)query_row(sh, w, m) * sh.B + bucket] = acc[i] + bv;
  }
}

// Both layers in one launch (bf16).  A workgroup owns (weight set, 16-row tile, 64 buckets):
// its four waves first compute ALL hidden units of the 16 rows (each wave a quarter of the
// hidden tiles; W1 is small and comes from L2 for every workgroup but the first), leave them in
// LDS as three exact bf16 planes, then each wave multiplies its 16 W2 rows.  The W2 loads are
// issued before the first layer starts, so one memory round trip covers x, W1 and W2.
__global__ void __launch_bounds__(256)
mlp_fused_kernel(const bf16_t* __restrict__ xq, const bf16_t* __restrict__ W1, const float* __restrict__ b1,
                 const bf16_t* __restrict__ W2, const float* __restrict__ b2, float* __restrict__ scores,
                 MlpShape sh) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // 1-D grid, weight set fastest: workgroups are handed to the 8 XCDs round-robin, so with Hw a
  // multiple of 8 all workgroups of a weight set share one L2 and W1 leaves HBM once.
  const int w = blockIdx.x % sh.Hw;
  const int rest = blockIdx.x / sh.Hw;
  const int m_tiles = sh.m_pad / 16;
  const int mt = rest % m_tiles;
  const int btile = (rest / m_tiles) * 4 + wave;     // tile of 16 buckets
  const int rc = lane & 15, kg = lane >> 4;
  const bool active = btile * 16 < sh.B;
  const int pitch = sh.hidden + 8;
  bf16_t* s_h = reinterpret_cast<bf16_t*>(smem);     // [3 planes][16 rows][pitch]

  SAAP_TRACE(0);
  constexpr int kBlock = 16;                          // W2 steps (32 hidden units each) per load block
  const int steps = sh.hidden / 32;
  const bf16_t* wr = W2 + ((size_t)w * sh.B + (active ? btile * 16 + rc : 0)) * sh.hidden + kg * 8;
  uint4 wreg[kBlock];
#pragma unroll
  for (int i = 0; i < kBlock; ++i)
    if (i < steps) wreg[i] = *reinterpret_cast<const uint4*>(wr + i * 32);

  // layer 1: A = the 16 query rows, B = 16 hidden units of W1, K = d = 128 in four steps
  const int m = min(mt * 16 + rc, sh.rows_per_set - 1);
  const bf16_t* xr = xq + (size_t)query_row(sh, w, m) * kD + kg * 8;
  uint4 xa[kD / 32];
#pragma unroll
  for (int st = 0; st < kD / 32; ++st) xa[st] = *reinterpret_cast<const uint4*>(xr + st * 32);
  constexpr int kTiles = 8;                           // hidden tiles per wave per round
  const int n_utiles = sh.hidden / 16;
  for (int u0 = wave; u0 < n_utiles; u0 += 4 * kTiles) {
    uint4 w1[kTiles][kD / 32];
    float bv[kTiles];
#pragma unroll
    for (int j = 0; j < kTiles; ++j) {
      const int ut = u0 + 4 * j;
      if (ut < n_utiles) {
        const bf16_t* w1r = W1 + ((size_t)w * sh.hidden + ut * 16 + rc) * kD + kg * 8;
#pragma unroll
        for (int st = 0; st < kD / 32; ++st) w1[j][st] = *reinterpret_cast<const uint4*>(w1r + st * 32);
        bv[j] = b1 ? b1[(size_t)w * sh.hidden + ut * 16 + rc] : 0.f;
      }
    }
    SAAP_TRACE(5);
#pragma unroll
    for (int j = 0; j < kTiles; ++j) {
      const int ut = u0 + 4 * j;
      if (j == 1) SAAP_TRACE(6);
      if (ut < n_utiles) {
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int st = 0; st < kD / 32; ++st)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xa[st]),
                                                        __builtin_bit_cast(bf16x8_t, w1[j][st]), acc, 0, 0, 0);
        // accumulator i: row 4*kg + i, hidden unit ut*16 + rc; split into three exact bf16 pieces
        const int unit = ut * 16 + rc;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = 4 * kg + i;
          const float hval = fmaxf(acc[i] + bv[j], 0.f);
          const uint32_t u0b = __float_as_uint(hval) & 0xffff0000u;
          const float r1 = hval - __uint_as_float(u0b);
          const uint32_t u1b = __float_as_uint(r1) & 0xffff0000u;
          const float r2 = r1 - __uint_as_float(u1b);
          const uint32_t u2b = __float_as_uint(r2) & 0xffff0000u;
          s_h[(size_t)(0 * 16 + row) * pitch + unit] = (bf16_t)(u0b >> 16);
          s_h[(size_t)(1 * 16 + row) * pitch + unit] = (bf16_t)(u1b >> 16);
          s_h[(size_t)(2 * 16 + row) * pitch + unit] = (bf16_t)(u2b >> 16);
        }
      }
    }
  }
  SAAP_TRACE(1);
  __syncthreads();
  SAAP_TRACE(2);

  // layer 2
  f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
  for (int s0 = 0; s0 < steps; s0 += kBlock) {
#pragma unroll
    for (int i = 0; i < kBlock; ++i) {
      if (s0 + i < steps) {
        const int k = (s0 + i) * 32 + kg * 8;
        const bf16x8_t b = __builtin_bit_cast(bf16x8_t, wreg[i]);
        const bf16x8_t a0 = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(s_h + (size_t)(0 * 16 + rc) * pitch + k));
        const bf16x8_t a1 = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(s_h + (size_t)(1 * 16 + rc) * pitch + k));
        const bf16x8_t a2 = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(s_h + (size_t)(2 * 16 + rc) * pitch + k));
        // smallest pieces first: their sum is rounded least by the fp32 accumulator
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, b, acc, 0, 0, 0);
      }
    }
    if (s0 + kBlock < steps) {
#pragma unroll
      for (int i = 0; i < kBlock; ++i)
        if (s0 + kBlock + i < steps) wreg[i] = *reinterpret_cast<const uint4*>(wr + (s0 + kBlock + i) * 32);
    }
  }
  SAAP_TRACE(3);
  if (!active) return;
  const int bucket = btile * 16 + rc;
  const float bo = b2 ? b2[(size_t)w * sh.B + bucket] : 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int mm = mt * 16 + 4 * kg + i;
    if (mm < sh.rows_per_set) scores[(size_t)query_row(sh, w, mm) * sh.B + bucket] = acc[i] + bo;
  }
  SAAP_TRACE(4);
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

// header | hidden activations: up to 3 planes of [rows padded to 16 per set][hidden] (4 bytes each bounds both dtypes)
size_t classify_workspace_bytes(long long rows, int hidden) {
  // every weight set pads its rows to a multiple of 16; at most `rows` sets of one row each
  const long long padded = rows * 16;
  return (size_t)SAAP_WS_HEADER_BYTES + (size_t)padded * hidden * 6;
}

}  // namespace saap

using namespace saap;

extern "C" int32_t saap_classify_queries(const void* xq, const void* W1, const float* b1, const void* W2,
                                         const float* b2, int32_t Hw, float* scores, int32_t S, int32_t Hq,
                                         int32_t Hkv, int32_t d, int32_t hidden, int32_t B, int32_t dtype,
                                         int32_t output_kind, void* ws, size_t ws_bytes, void* stream) {
  if (!xq || !W1 || !W2 || !scores || !ws) return SAAP_INVALID_ARG;
  if (!aligned16(xq) || !aligned16(W1) || !aligned16(W2) || !aligned16(scores) || !aligned16(ws))
    return SAAP_INVALID_ARG;
  if (S <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || hidden <= 0 || B <= 0) return SAAP_INVALID_ARG;
  if (Hw != 1 && Hw != Hkv && Hw != Hq) return SAAP_INVALID_ARG;
  if (dtype != SAAP_F32 && dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  if (output_kind != SAAP_PROBS && output_kind != SAAP_LOGITS) return SAAP_INVALID_ARG;
  if (d != kD || hidden % 32 != 0 || B % 16 != 0 || B > SAAP_MAX_BUCKETS || hidden > 1536) return SAAP_UNSUPPORTED;
  MlpShape sh;
  sh.S = S; sh.Hq = Hq; sh.Hw = Hw; sh.hidden = hidden; sh.B = B;
  sh.rows_per_set = S * (Hq / Hw);
  sh.m_pad = (sh.rows_per_set + 15) / 16 * 16;
  const size_t need = (size_t)SAAP_WS_HEADER_BYTES + (size_t)Hw * sh.m_pad * hidden * (dtype == SAAP_BF16 ? 6 : 4);
  if (ws_bytes < need) return SAAP_WORKSPACE_TOO_SMALL;
  const int m_tiles = sh.m_pad / 16;
  if (m_tiles > 65535 || Hw > 65535) return SAAP_UNSUPPORTED;
  void* hbuf = static_cast<char*>(ws) + SAAP_WS_HEADER_BYTES;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const dim3 g1((unsigned)((hidden / 16 + 3) / 4), (unsigned)m_tiles, (unsigned)Hw);
  const dim3 g2((unsigned)((B / 16 + 3) / 4), (unsigned)m_tiles, (unsigned)Hw);
  if (dtype == SAAP_BF16) {
    const size_t lds = (size_t)3 * 16 * (hidden + 8) * sizeof(bf16_t);
    if (lds > 48 * 1024) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_fused_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return SAAP_HIP_ERROR;
    }
    saap_trace_arm();
    hipLaunchKernelGGL(mlp_fused_kernel, dim3(g2.x * g2.y * g2.z), dim3(256), lds, hs, static_cast<const bf16_t*>(xq),
                       static_cast<const bf16_t*>(W1), b1, static_cast<const bf16_t*>(W2), b2, scores, sh);
  } else {
    hipLaunchKernelGGL(mlp_hidden_kernel<float>, g1, dim3(256), 0, hs, static_cast<const float*>(xq),
                       static_cast<const float*>(W1), b1, hbuf, sh);
    hipLaunchKernelGGL(mlp_out_kernel<float>, g2, dim3(256), 0, hs, hbuf, static_cast<const float*>(W2), b2,
                       scores, sh);
  }
  if (output_kind == SAAP_PROBS)
    hipLaunchKernelGGL(softmax_rows_kernel, dim3((unsigned)(S * Hq)), dim3(256), 0, hs, scores, B);
  return launch_status();
}
