// Training of the query model f_q (Section 4 "Query assignment function", Eq. 1 of arXiv
// 2502.08246; Appendix "Training details": Adam):
//   z = W2 relu(W1 x + b1) + b2,  f_q(x) = softmax(z),
//   L = 1/R sum_r sum_b T[r,b] (log T[r,b] - log f_q(x_r)[b])       (T: bucket attention mass, rows of A*H_k)
// query_model_loss_grads computes L and the gradients of all four parameter tensors for a batch,
// adam_update applies one Adam step to a tensor; a training step is the first call followed by
// the second on each tensor.  All arithmetic is fp32, every sum is taken by one thread or one
// workgroup in a fixed order (no atomics), so a step is reproducible bit for bit.
//
// The five matrix products run on the matrix cores (v_mfma_f32_32x32x2_f32): a workgroup of four
// waves owns a 64x64 tile of the result, operands are staged through LDS in k-slices of 16 by
// loaders that read global memory along its contiguous dimension whichever operand is
// transposed, bounds are checked on every dimension (R, B, hidden are free).
#include "common.h"

namespace saap {
namespace {

constexpr int kTile = 64, kSlice = 16, kGemmThreads = 256;

enum { EPI_NONE = 0, EPI_BIAS = 1, EPI_BIAS_RELU = 2, EPI_MASK = 3 };

struct GemmArgs {
  const float* A;      // TA ? [K,M] : [M,K]
  const float* B;      // TB ? [N,K] : [K,N]
  float* C;            // [M,N]
  const float* bias;   // [N]   (EPI_BIAS, EPI_BIAS_RELU)
  const float* aux;    // [M,N] (EPI_MASK: C = aux > 0 ? acc : 0)
  int M, N, K;
  long long sA, sB, sC, sBias, sAux;   // strides between the weight sets (blockIdx.z), in elements
};

// C = A' B' for one 64x64 tile; A' is M x K, B' is K x N.
template <bool TA, bool TB, int EPI>
__global__ void __launch_bounds__(kGemmThreads)
gemm_kernel(GemmArgs g) {
  __shared__ float s_a[kSlice][kTile + 1];   // [k][m]
  __shared__ float s_b[kSlice][kTile + 1];   // [k][n]
  typedef __attribute__((ext_vector_type(16))) float f32x16_t;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m0 = blockIdx.y * kTile, n0 = blockIdx.x * kTile;
  const float* A = g.A + (size_t)blockIdx.z * g.sA;
  const float* B = g.B + (size_t)blockIdx.z * g.sB;
  const int wm = (wave >> 1) * 32, wn = (wave & 1) * 32;     // this wave's 32x32 corner of the tile
  const int col = lane & 31, half = lane >> 5;
  f32x16_t acc = {0};
  for (int k0 = 0; k0 < g.K; k0 += kSlice) {
    // 64 x 16 elements per operand, four per thread, read along the contiguous dimension
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + i * kGemmThreads;
      int m, k;
      if (TA) { m = e % kTile; k = e / kTile; } else { k = e % kSlice; m = e / kSlice; }
      const bool ok = m0 + m < g.M && k0 + k < g.K;
      s_a[k][m] = ok ? (TA ? A[(size_t)(k0 + k) * g.M + m0 + m] : A[(size_t)(m0 + m) * g.K + k0 + k]) : 0.f;
      int n, kb;
      if (TB) { kb = e % kSlice; n = e / kSlice; } else { n = e % kTile; kb = e / kTile; }
      const bool okb = n0 + n < g.N && k0 + kb < g.K;
      s_b[kb][n] = okb ? (TB ? B[(size_t)(n0 + n) * g.K + k0 + kb] : B[(size_t)(k0 + kb) * g.N + n0 + n]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kSlice; k += 2)
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(s_a[k + half][wm + col], s_b[k + half][wn + col], acc, 0, 0, 0);
    __syncthreads();
  }
  // register r of this lane: row 8*(r/4) + 4*half + r%4, column `col` of the wave's corner
  float* C = g.C + (size_t)blockIdx.z * g.sC;
  const int n = n0 + wn + col;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int m = m0 + wm + 8 * (r / 4) + 4 * half + (r % 4);
    if (m < g.M && n < g.N) {
      float v = acc[r];
      if (EPI == EPI_BIAS || EPI == EPI_BIAS_RELU) v += g.bias[(size_t)blockIdx.z * g.sBias + n];
      if (EPI == EPI_BIAS_RELU) v = fmaxf(v, 0.f);
      if (EPI == EPI_MASK) v = g.aux[(size_t)blockIdx.z * g.sAux + (size_t)m * g.N + n] > 0.f ? v : 0.f;
      C[(size_t)m * g.N + n] = v;
    }
  }
}

template <bool TA, bool TB, int EPI>
void gemm(const GemmArgs& g, int Hw, hipStream_t hs) {
  const dim3 grid((unsigned)((g.N + kTile - 1) / kTile), (unsigned)((g.M + kTile - 1) / kTile), (unsigned)Hw);
  hipLaunchKernelGGL((gemm_kernel<TA, TB, EPI>), grid, dim3(kGemmThreads), 0, hs, g);
}

__global__ void widen_kernel(const bf16_t* __restrict__ x, float* __restrict__ y, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) y[i] = __uint_as_float((uint32_t)x[i] << 16);
}

// Sum of a workgroup's values, in a fixed order; every thread gets it.  s_red: 256/64 + 1 floats.
__device__ __forceinline__ float block_sum(float v, float* s_red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
}
__device__ __forceinline__ float block_max(float v, float* s_red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
}

// One workgroup per row: logits z -> the row's loss and, in place, the gradient with respect to
// the logits: ((sum_b T) * softmax(z) - T) / R.
__global__ void __launch_bounds__(256)
softmax_kl_kernel(float* __restrict__ z, const float* __restrict__ T, float* __restrict__ loss_rows, int R, int B) {
  __shared__ float s_red[4];
  const size_t row = (size_t)blockIdx.y * R + blockIdx.x;
  float* zr = z + row * B;
  const float* tr = T + row * B;
  float mx = -INFINITY, tsum = 0.f;
  for (int b = threadIdx.x; b < B; b += 256) {
    mx = fmaxf(mx, zr[b]);
    tsum += tr[b];
  }
  mx = block_max(mx, s_red);
  tsum = block_sum(tsum, s_red);
  float se = 0.f;
  for (int b = threadIdx.x; b < B; b += 256) se += __expf(zr[b] - mx);
  se = block_sum(se, s_red);
  const float lse = mx + __logf(se), inv_r = 1.0f / (float)R;
  float l = 0.f;
  for (int b = threadIdx.x; b < B; b += 256) {
    const float t = tr[b], logp = zr[b] - lse;
    if (t > 0.f) l += t * (__logf(t) - logp);
    zr[b] = (tsum * __expf(logp) - t) * inv_r;
  }
  l = block_sum(l, s_red);
  if (threadIdx.x == 0) loss_rows[row] = l;
}

// loss[w] = mean over the R rows, summed in a fixed order by one workgroup
__global__ void __launch_bounds__(256)
loss_mean_kernel(const float* __restrict__ loss_rows, float* __restrict__ loss, int R) {
  __shared__ float s_red[4];
  float v = 0.f;
  for (int r = threadIdx.x; r < R; r += 256) v += loss_rows[(size_t)blockIdx.x * R + r];
  v = block_sum(v, s_red);
  if (threadIdx.x == 0) loss[blockIdx.x] = v / (float)R;
}

// out[n] = sum over the rows of X [rows, n_cols]; one thread per column, rows in order
__global__ void __launch_bounds__(256)
colsum_kernel(const float* __restrict__ X, float* __restrict__ out, int rows, int n_cols, long long sX, long long sOut) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= n_cols) return;
  const float* x = X + (size_t)blockIdx.y * sX + c;
  float v = 0.f;
  for (int r = 0; r < rows; ++r) v += x[(size_t)r * n_cols];
  out[(size_t)blockIdx.y * sOut + c] = v;
}

__global__ void __launch_bounds__(256)
adam_kernel(float* __restrict__ p, const float* __restrict__ g, float* __restrict__ m, float* __restrict__ v, size_t n,
            float lr, float beta1, float beta2, float eps, float c1, float c2) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const float gi = g[i];
  const float mi = beta1 * m[i] + (1.0f - beta1) * gi;
  const float vi = beta2 * v[i] + (1.0f - beta2) * gi * gi;
  m[i] = mi;
  v[i] = vi;
  p[i] -= lr * (mi * c1) / (sqrtf(vi * c2) + eps);
}

}  // namespace

// header | x widened [Hw,R,d] | h [Hw,R,hidden] | z then dL/dz [Hw,R,B] | dL/da [Hw,R,hidden] | row losses [Hw,R]
size_t train_workspace_bytes(long long Hw, long long R, int d, int hidden, int B) {
  return (size_t)SAAP_WS_HEADER_BYTES + (size_t)Hw * R * ((size_t)d + 2 * (size_t)hidden + B + 1) * sizeof(float);
}

}  // namespace saap

using namespace saap;

extern "C" int32_t saap_query_model_loss_grads(const void* x, const float* target, const saap_mlp_f32* params,
                                               const saap_mlp_f32* grads, float* loss, int32_t Hw, int32_t R,
                                               int32_t d, int32_t hidden, int32_t B, int32_t x_dtype, void* ws,
                                               size_t ws_bytes, void* stream) {
  if (!x || !target || !params || !grads || !loss || !ws) return SAAP_INVALID_ARG;
  if (!params->W1 || !params->b1 || !params->W2 || !params->b2 || !grads->W1 || !grads->b1 || !grads->W2 || !grads->b2)
    return SAAP_INVALID_ARG;
  if (!aligned16(x) || !aligned16(ws)) return SAAP_INVALID_ARG;
  if (Hw <= 0 || R <= 0 || d <= 0 || hidden <= 0 || B <= 0) return SAAP_INVALID_ARG;
  if (x_dtype != SAAP_F32 && x_dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  if (Hw > 65535 || R > 65535 * 64) return SAAP_UNSUPPORTED;
  if (ws_bytes < train_workspace_bytes(Hw, R, d, hidden, B)) return SAAP_WORKSPACE_TOO_SMALL;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  float* xf = reinterpret_cast<float*>(static_cast<char*>(ws) + SAAP_WS_HEADER_BYTES);
  float* h = xf + (size_t)Hw * R * d;
  float* z = h + (size_t)Hw * R * hidden;
  float* da = z + (size_t)Hw * R * B;
  float* loss_rows = da + (size_t)Hw * R * hidden;
  const float* xin = static_cast<const float*>(x);
  if (x_dtype == SAAP_BF16) {
    const size_t n = (size_t)Hw * R * d;
    hipLaunchKernelGGL(widen_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, hs, static_cast<const bf16_t*>(x),
                       xf, n);
    xin = xf;
  }
  const long long sx = (long long)R * d, sh = (long long)R * hidden, sz = (long long)R * B;
  const long long sW1 = (long long)hidden * d, sW2 = (long long)B * hidden;
  // h = relu(x W1^T + b1)
  gemm<false, true, EPI_BIAS_RELU>({xin, params->W1, h, params->b1, nullptr, R, hidden, d, sx, sW1, sh, hidden, 0}, Hw, hs);
  // z = h W2^T + b2
  gemm<false, true, EPI_BIAS>({h, params->W2, z, params->b2, nullptr, R, B, hidden, sh, sW2, sz, B, 0}, Hw, hs);
  // row losses; z becomes dL/dz
  hipLaunchKernelGGL(softmax_kl_kernel, dim3((unsigned)R, (unsigned)Hw), dim3(256), 0, hs, z, target, loss_rows, R, B);
  hipLaunchKernelGGL(loss_mean_kernel, dim3((unsigned)Hw), dim3(256), 0, hs, loss_rows, loss, R);
  // dW2 = dz^T h, db2 = column sums of dz
  gemm<true, false, EPI_NONE>({z, h, grads->W2, nullptr, nullptr, B, hidden, R, sz, sh, sW2, 0, 0}, Hw, hs);
  hipLaunchKernelGGL(colsum_kernel, dim3((unsigned)((B + 255) / 256), (unsigned)Hw), dim3(256), 0, hs, z, grads->b2, R, B,
                     sz, (long long)B);
  // da = (dz W2) where h > 0
  gemm<false, false, EPI_MASK>({z, params->W2, da, nullptr, h, R, hidden, B, sz, sW2, sh, 0, sh}, Hw, hs);
  // dW1 = da^T x, db1 = column sums of da
  gemm<true, false, EPI_NONE>({da, xin, grads->W1, nullptr, nullptr, hidden, d, R, sh, sx, sW1, 0, 0}, Hw, hs);
  hipLaunchKernelGGL(colsum_kernel, dim3((unsigned)((hidden + 255) / 256), (unsigned)Hw), dim3(256), 0, hs, da, grads->b1,
                     R, hidden, sh, (long long)hidden);
  return launch_status();
}

extern "C" int32_t saap_adam_update(float* param, const float* grad, float* m, float* v, size_t n, int32_t step,
                                    float lr, float beta1, float beta2, float eps, void* stream) {
  if (!param || !grad || !m || !v) return SAAP_INVALID_ARG;
  if (n == 0 || step < 1 || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f)) return SAAP_INVALID_ARG;
  // bias corrections 1 / (1 - beta^t), evaluated in double on the host
  const float c1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
  const float c2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
  hipLaunchKernelGGL(adam_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(stream), param,
                     grad, m, v, n, lr, beta1, beta2, eps, c1, c2);
  return launch_status();
}
