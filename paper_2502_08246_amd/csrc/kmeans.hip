// update_centroids: the centroid step of the k-means that defines the buckets of arXiv 2502.08246
// (Section 4, "Learning the key assignment": k-means on keys; Section 3 uses the spherical
// variant; Appendix A gives the training set-up).  With saap_assign_keys (assignment step) and
// saap_build_bucket_index (grouping the features by bucket) it makes one Lloyd iteration on the
// GPU, so that centroids for any head can be produced without leaving the device.
//
// One workgroup per (KV head, bucket).  The bucket's member rows are one contiguous run per
// sequence of the grouped features; 16 lanes read one row (16 or 32 bytes each), 16 rows are in
// flight per pass, every lane adds up its 8 features over its rows in fp32 in a fixed order, the
// 16 row groups are then added in order through LDS.  Sums are therefore reproducible from run to run.
#include "common.h"

namespace saap {
namespace {

template <typename T>
__global__ void __launch_bounds__(256)
centroid_update_kernel(const T* __restrict__ x_sorted, const int32_t* __restrict__ off, const int32_t* __restrict__ len,
                       const T* __restrict__ cent_old, T* __restrict__ cent_new, int S, int Hkv, int Ncap, int B,
                       int normalize) {
  __shared__ float s_part[16][kD];
  __shared__ float s_sq[2];
  const int b = blockIdx.x, h = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = tid & 15, grp = tid >> 4;            // 16 lanes per row, 16 row groups
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
  long long count = 0;
  for (int s = 0; s < S; ++s) {
    const size_t unit = (size_t)s * Hkv + h;
    const int first = off[unit * (B + 1) + b], n = len[unit * B + b];
    count += n;
    const T* rows = x_sorted + (unit * Ncap + first) * kD + sub * 8;
    for (int r = grp; r < n; r += 16) {
      Vec8<T> v;
      v.load(rows + (size_t)r * kD);
      float f[8];
      v.to_float(f);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += f[e];
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) s_part[grp][sub * 8 + e] = acc[e];
  __syncthreads();
  const size_t crow = ((size_t)h * B + b) * kD;
  float mean = 0.f;
  if (tid < kD) {
    float t = 0.f;
#pragma unroll
    for (int g = 0; g < 16; ++g) t += s_part[g][tid];
    mean = count > 0 ? t / (float)count : 0.f;
    // squared norm of the mean: 64 lanes on DPP and row swaps, then the two waves in order
    const float sq = sum_rows(sum16(mean * mean));
    if (lane == 0) s_sq[wave] = sq;
  }
  __syncthreads();
  if (tid < kD) {
    float v;
    if (count == 0) {
      v = Vec8<T>::widen(cent_old[crow + tid]);         // a bucket without members keeps its centroid
    } else {
      v = mean;
      if (normalize) {
        const float nrm = sqrtf(s_sq[0] + s_sq[1]);
        v = nrm > 0.f ? mean / nrm : mean;
      }
    }
    cent_new[crow + tid] = Vec8<T>::narrow(v);
  }
}

}  // namespace
}  // namespace saap

using namespace saap;

extern "C" int32_t saap_update_centroids(const void* x_sorted, const int32_t* off, const int32_t* len,
                                         const void* centroids_old, void* centroids_new, int32_t S, int32_t Hkv,
                                         int32_t Ncap, int32_t B, int32_t d, int32_t dtype, int32_t normalize,
                                         void* stream) {
  begin_call();
  if (!x_sorted || !off || !len || !centroids_old || !centroids_new) return SAAP_INVALID_ARG;
  if (!aligned16(x_sorted) || !aligned16(centroids_old) || !aligned16(centroids_new)) return SAAP_INVALID_ARG;
  if (S <= 0 || Hkv <= 0 || Ncap <= 0 || B <= 0) return SAAP_INVALID_ARG;
  if (dtype != SAAP_F32 && dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  if (d != kD || B > SAAP_MAX_BUCKETS || Hkv > 65535) return SAAP_UNSUPPORTED;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const dim3 grid((unsigned)B, (unsigned)Hkv);
  if (dtype == SAAP_BF16)
    hipLaunchKernelGGL(centroid_update_kernel<bf16_t>, grid, dim3(256), 0, hs, static_cast<const bf16_t*>(x_sorted),
                       off, len, static_cast<const bf16_t*>(centroids_old), static_cast<bf16_t*>(centroids_new), S,
                       Hkv, Ncap, B, normalize);
  else
    hipLaunchKernelGGL(centroid_update_kernel<float>, grid, dim3(256), 0, hs, static_cast<const float*>(x_sorted),
                       off, len, static_cast<const float*>(centroids_old), static_cast<float*>(centroids_new), S, Hkv,
                       Ncap, B, normalize);
  return launch_status();
}
