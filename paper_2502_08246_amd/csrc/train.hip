// Training of the query model f_q (Section 4 "Query assignment function", Eq. 1 of arXiv
// 2502.08246; Appendix "Training details": Adam):
//   z = W2 relu(W1 x + b1) + b2,  f_q(x) = softmax(z),
//   L = 1/R sum_r sum_b T[r,b] (log T[r,b] - log f_q(x_r)[b])       (T: bucket attention mass, rows of A*H_k)
// With batch normalisation (the model of Section 6.1) the hidden layer is
//   relu(gamma * (a - mean_r a) / sqrt(var_r a + eps) + beta),  a = W1 x + b1,
// and fold_batch_norm turns the trained layer into plain W1, b1 for inference.
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

// Column sums in a fixed order.  A workgroup owns 64 columns; its 16 waves each take a contiguous slice of
// the rows (a wave reads 64 neighbouring columns of one row at a time) and the 16 slice sums are added in
// slice order, so the result does not depend on timing.
constexpr int kBnCols = 64, kBnSlices = 16, kBnThreads = kBnCols * kBnSlices;

// sum over the slices of v, in slice order; every thread of a column gets the same bits
__device__ __forceinline__ float slice_sum(float v, float (*s_part)[kBnCols], int col, int slice) {
  __syncthreads();
  s_part[slice][col] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < kBnSlices; ++i) t += s_part[i][col];
  return t;
}

// out[n] = sum over the rows of X [rows, n_cols]
__global__ void __launch_bounds__(kBnThreads)
colsum_kernel(const float* __restrict__ X, float* __restrict__ out, int rows, int n_cols, long long sX, long long sOut) {
  __shared__ float s_part[kBnSlices][kBnCols];
  const int col = threadIdx.x % kBnCols, slice = threadIdx.x / kBnCols;
  const int c = blockIdx.x * kBnCols + col;
  const bool live = c < n_cols;
  const int per = (rows + kBnSlices - 1) / kBnSlices, r0 = slice * per, r1 = min(r0 + per, rows);
  const float* x = X + (size_t)blockIdx.y * sX + (live ? c : 0);
  float v = 0.f;
  if (live)
    for (int r = r0; r < r1; ++r) v += x[(size_t)r * n_cols];
  v = slice_sum(v, s_part, col, slice);
  if (live && slice == 0) out[(size_t)blockIdx.y * sOut + c] = v;
}

// Batch normalisation of the hidden pre-activations a [rows, n_cols] (Section 6.1 names the layer).
// Columns and rows are dealt as in colsum_kernel.  The batch mean, then the variance about it (divisor rows).
// stats [4, n_cols] per weight set: mean, 1/sqrt(var + eps), and room for the two backward sums.
// Running statistics (optional) follow run = (1 - momentum) run + momentum batch, the variance with
// divisor rows - 1.
__global__ void __launch_bounds__(kBnThreads)
bn_stats_kernel(const float* __restrict__ A, float* __restrict__ stats, float* __restrict__ run_mean,
                float* __restrict__ run_var, int rows, int n_cols, float eps, float momentum) {
  __shared__ float s_part[kBnSlices][kBnCols];
  const int col = threadIdx.x % kBnCols, slice = threadIdx.x / kBnCols;
  const int c = blockIdx.x * kBnCols + col;
  const bool live = c < n_cols;
  const int per = (rows + kBnSlices - 1) / kBnSlices, r0 = slice * per, r1 = min(r0 + per, rows);
  const float* a = A + (size_t)blockIdx.y * rows * n_cols + (live ? c : 0);
  float sum = 0.f;
  if (live)
    for (int r = r0; r < r1; ++r) sum += a[(size_t)r * n_cols];
  const float mean = slice_sum(sum, s_part, col, slice) / (float)rows;
  float sq = 0.f;
  if (live)
    for (int r = r0; r < r1; ++r) {
      const float dlt = a[(size_t)r * n_cols] - mean;
      sq += dlt * dlt;
    }
  sq = slice_sum(sq, s_part, col, slice);
  if (!live || slice != 0) return;
  float* st = stats + (size_t)blockIdx.y * 4 * n_cols;
  st[c] = mean;
  st[n_cols + c] = 1.0f / sqrtf(sq / (float)rows + eps);
  if (run_mean) {
    const size_t i = (size_t)blockIdx.y * n_cols + c;
    run_mean[i] = (1.0f - momentum) * run_mean[i] + momentum * mean;
    run_var[i] = (1.0f - momentum) * run_var[i] + momentum * (sq / (float)(rows - 1));
  }
}

// h = relu(gamma * ahat + beta), ahat = (a - mean) * rstd
__global__ void __launch_bounds__(256)
bn_relu_kernel(const float* __restrict__ A, const float* __restrict__ stats, const float* __restrict__ gamma,
               const float* __restrict__ beta, float* __restrict__ H, int rows, int n_cols) {
  const size_t per_set = (size_t)rows * n_cols;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= per_set) return;
  const int c = (int)(i % n_cols), w = blockIdx.y;
  const float* st = stats + (size_t)w * 4 * n_cols;
  const float ahat = (A[w * per_set + i] - st[c]) * st[n_cols + c];
  H[w * per_set + i] = fmaxf(gamma[(size_t)w * n_cols + c] * ahat + beta[(size_t)w * n_cols + c], 0.f);
}

// Backward sums per column, rows sliced as in bn_stats_kernel: dbeta = sum dy, dgamma = sum dy * ahat.
__global__ void __launch_bounds__(kBnThreads)
bn_backward_sums_kernel(const float* __restrict__ A, const float* __restrict__ DY, float* __restrict__ stats,
                        float* __restrict__ dgamma, float* __restrict__ dbeta, int rows, int n_cols) {
  __shared__ float s_part[kBnSlices][kBnCols];
  const int col = threadIdx.x % kBnCols, slice = threadIdx.x / kBnCols;
  const int c = blockIdx.x * kBnCols + col;
  const bool live = c < n_cols;
  const int per = (rows + kBnSlices - 1) / kBnSlices, r0 = slice * per, r1 = min(r0 + per, rows);
  const size_t base = (size_t)blockIdx.y * rows * n_cols + (live ? c : 0);
  float* st = stats + (size_t)blockIdx.y * 4 * n_cols;
  const float mean = live ? st[c] : 0.f, rstd = live ? st[n_cols + c] : 0.f;
  float sb = 0.f, sg = 0.f;
  if (live)
    for (int r = r0; r < r1; ++r) {
      const float dy = DY[base + (size_t)r * n_cols];
      sb += dy;
      sg += dy * ((A[base + (size_t)r * n_cols] - mean) * rstd);
    }
  sb = slice_sum(sb, s_part, col, slice);
  sg = slice_sum(sg, s_part, col, slice);
  if (!live || slice != 0) return;
  st[2 * n_cols + c] = sb;
  st[3 * n_cols + c] = sg;
  dbeta[(size_t)blockIdx.y * n_cols + c] = sb;
  dgamma[(size_t)blockIdx.y * n_cols + c] = sg;
}

// In place: dy -> da = gamma * rstd * (dy - dbeta / rows - ahat * dgamma / rows)
__global__ void __launch_bounds__(256)
bn_backward_kernel(const float* __restrict__ A, float* __restrict__ DY, const float* __restrict__ stats,
                   const float* __restrict__ gamma, int rows, int n_cols) {
  const size_t per_set = (size_t)rows * n_cols;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= per_set) return;
  const int c = (int)(i % n_cols), w = blockIdx.y;
  const float* st = stats + (size_t)w * 4 * n_cols;
  const float rstd = st[n_cols + c], inv_rows = 1.0f / (float)rows;
  const float ahat = (A[w * per_set + i] - st[c]) * rstd;
  const float dy = DY[w * per_set + i];
  DY[w * per_set + i] = gamma[(size_t)w * n_cols + c] * rstd * (dy - st[2 * n_cols + c] * inv_rows - ahat * st[3 * n_cols + c] * inv_rows);
}

// W1' = s W1 (row-wise), b1' = (b1 - mean) s + beta with s = gamma / sqrt(var + eps); one thread per row of W1
template <typename TO>
__global__ void __launch_bounds__(256)
bn_fold_kernel(const float* __restrict__ W1, const float* __restrict__ b1, const float* __restrict__ gamma,
               const float* __restrict__ beta, const float* __restrict__ mean, const float* __restrict__ var, float eps,
               TO* __restrict__ W1o, float* __restrict__ b1o, size_t rows_total, int d) {
  const size_t j = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (j >= rows_total) return;
  const float s = gamma[j] / sqrtf(var[j] + eps);
  b1o[j] = (b1[j] - mean[j]) * s + beta[j];
  for (int k = 0; k < d; ++k) {
    const float v = W1[j * d + k] * s;
    if constexpr (sizeof(TO) == 4) {
      W1o[j * d + k] = v;
    } else {
      W1o[j * d + k] = Vec8<bf16_t>::narrow(v);
    }
  }
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
//        | batch-norm variant: pre-activations a [Hw,R,hidden] | column statistics [Hw,4,hidden]
size_t train_workspace_bytes(long long Hw, long long R, int d, int hidden, int B) {
  return (size_t)SAAP_WS_HEADER_BYTES + (size_t)Hw * R * ((size_t)d + 3 * (size_t)hidden + B + 1) * sizeof(float) +
         (size_t)Hw * 4 * hidden * sizeof(float);
}

}  // namespace saap

using namespace saap;

// bn == nullptr: the plain model.
static int32_t loss_grads(const void* x, const float* target, const saap_mlp_f32* params, const saap_mlp_f32* grads,
                          const saap_batch_norm_f32* bn, float* loss, int32_t Hw, int32_t R, int32_t d, int32_t hidden,
                          int32_t B, int32_t x_dtype, void* ws, size_t ws_bytes, void* stream) {
  if (!x || !target || !params || !grads || !loss || !ws) return SAAP_INVALID_ARG;
  if (bn) {
    if (!bn->gamma || !bn->beta || !bn->grad_gamma || !bn->grad_beta) return SAAP_INVALID_ARG;
    if ((bn->running_mean == nullptr) != (bn->running_var == nullptr)) return SAAP_INVALID_ARG;
    if (!(bn->eps > 0.f) || !(bn->momentum >= 0.f && bn->momentum <= 1.f)) return SAAP_INVALID_ARG;
    if (R < 2) return SAAP_INVALID_ARG;   // no variance estimate from one row
  }
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
  float* pre = loss_rows + (size_t)Hw * R;          // batch-norm variant only
  float* stats = pre + (size_t)Hw * R * hidden;
  const dim3 per_col((unsigned)((hidden + kBnCols - 1) / kBnCols), (unsigned)Hw);
  const dim3 per_elem((unsigned)(((size_t)R * hidden + 255) / 256), (unsigned)Hw);
  if (!bn) {
    // h = relu(x W1^T + b1)
    gemm<false, true, EPI_BIAS_RELU>({xin, params->W1, h, params->b1, nullptr, R, hidden, d, sx, sW1, sh, hidden, 0}, Hw, hs);
  } else {
    // a = x W1^T + b1;  h = relu(gamma * normalised(a) + beta)
    gemm<false, true, EPI_BIAS>({xin, params->W1, pre, params->b1, nullptr, R, hidden, d, sx, sW1, sh, hidden, 0}, Hw, hs);
    hipLaunchKernelGGL(bn_stats_kernel, per_col, dim3(kBnThreads), 0, hs, pre, stats, bn->running_mean, bn->running_var, R, hidden,
                       bn->eps, bn->momentum);
    hipLaunchKernelGGL(bn_relu_kernel, per_elem, dim3(256), 0, hs, pre, stats, bn->gamma, bn->beta, h, R, hidden);
  }
  // z = h W2^T + b2
  gemm<false, true, EPI_BIAS>({h, params->W2, z, params->b2, nullptr, R, B, hidden, sh, sW2, sz, B, 0}, Hw, hs);
  // row losses; z becomes dL/dz
  hipLaunchKernelGGL(softmax_kl_kernel, dim3((unsigned)R, (unsigned)Hw), dim3(256), 0, hs, z, target, loss_rows, R, B);
  hipLaunchKernelGGL(loss_mean_kernel, dim3((unsigned)Hw), dim3(256), 0, hs, loss_rows, loss, R);
  // dW2 = dz^T h, db2 = column sums of dz
  gemm<true, false, EPI_NONE>({z, h, grads->W2, nullptr, nullptr, B, hidden, R, sz, sh, sW2, 0, 0}, Hw, hs);
  hipLaunchKernelGGL(colsum_kernel, dim3((unsigned)((B + kBnCols - 1) / kBnCols), (unsigned)Hw), dim3(kBnThreads), 0, hs, z,
                     grads->b2, R, B,
                     sz, (long long)B);
  // da = (dz W2) where h > 0
  gemm<false, false, EPI_MASK>({z, params->W2, da, nullptr, h, R, hidden, B, sz, sW2, sh, 0, sh}, Hw, hs);
  if (bn) {
    // through the normalisation: da holds dL/dy on entry and dL/da on exit
    hipLaunchKernelGGL(bn_backward_sums_kernel, per_col, dim3(kBnThreads), 0, hs, pre, da, stats, bn->grad_gamma, bn->grad_beta, R,
                       hidden);
    hipLaunchKernelGGL(bn_backward_kernel, per_elem, dim3(256), 0, hs, pre, da, stats, bn->gamma, R, hidden);
  }
  // dW1 = da^T x, db1 = column sums of da
  gemm<true, false, EPI_NONE>({da, xin, grads->W1, nullptr, nullptr, hidden, d, R, sh, sx, sW1, 0, 0}, Hw, hs);
  hipLaunchKernelGGL(colsum_kernel, per_col, dim3(kBnThreads), 0, hs, da, grads->b1, R, hidden, sh, (long long)hidden);
  return launch_status();
}

extern "C" int32_t saap_query_model_loss_grads(const void* x, const float* target, const saap_mlp_f32* params,
                                               const saap_mlp_f32* grads, float* loss, int32_t Hw, int32_t R,
                                               int32_t d, int32_t hidden, int32_t B, int32_t x_dtype, void* ws,
                                               size_t ws_bytes, void* stream) {
  begin_call();
  return loss_grads(x, target, params, grads, nullptr, loss, Hw, R, d, hidden, B, x_dtype, ws, ws_bytes, stream);
}

extern "C" int32_t saap_query_model_bn_loss_grads(const void* x, const float* target, const saap_mlp_f32* params,
                                                  const saap_mlp_f32* grads, const saap_batch_norm_f32* bn, float* loss,
                                                  int32_t Hw, int32_t R, int32_t d, int32_t hidden, int32_t B,
                                                  int32_t x_dtype, void* ws, size_t ws_bytes, void* stream) {
  begin_call();
  if (!bn) return SAAP_INVALID_ARG;
  return loss_grads(x, target, params, grads, bn, loss, Hw, R, d, hidden, B, x_dtype, ws, ws_bytes, stream);
}

extern "C" int32_t saap_fold_batch_norm(const float* W1, const float* b1, const float* gamma, const float* beta,
                                        const float* running_mean, const float* running_var, float eps, void* W1_out,
                                        float* b1_out, int32_t Hw, int32_t hidden, int32_t d, int32_t out_dtype,
                                        void* stream) {
  begin_call();
  if (!W1 || !b1 || !gamma || !beta || !running_mean || !running_var || !W1_out || !b1_out) return SAAP_INVALID_ARG;
  if (Hw <= 0 || hidden <= 0 || d <= 0 || !(eps > 0.f)) return SAAP_INVALID_ARG;
  if (out_dtype != SAAP_F32 && out_dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  const size_t rows = (size_t)Hw * hidden;
  const dim3 grid((unsigned)((rows + 255) / 256));
  hipStream_t hs = static_cast<hipStream_t>(stream);
  if (out_dtype == SAAP_F32)
    hipLaunchKernelGGL(bn_fold_kernel<float>, grid, dim3(256), 0, hs, W1, b1, gamma, beta, running_mean, running_var, eps,
                       static_cast<float*>(W1_out), b1_out, rows, d);
  else
    hipLaunchKernelGGL(bn_fold_kernel<bf16_t>, grid, dim3(256), 0, hs, W1, b1, gamma, beta, running_mean, running_var, eps,
                       static_cast<bf16_t*>(W1_out), b1_out, rows, d);
  return launch_status();
}

extern "C" int32_t saap_adam_update(float* param, const float* grad, float* m, float* v, size_t n, int32_t step,
                                    float lr, float beta1, float beta2, float eps, void* stream) {
  begin_call();
  if (!param || !grad || !m || !v) return SAAP_INVALID_ARG;
  if (n == 0 || step < 1 || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f)) return SAAP_INVALID_ARG;
  // bias corrections 1 / (1 - beta^t), evaluated in double on the host
  const float c1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
  const float c2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
  hipLaunchKernelGGL(adam_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(stream), param,
                     grad, m, v, n, lr, beta1, beta2, eps, c1, c2);
  return launch_status();
}
