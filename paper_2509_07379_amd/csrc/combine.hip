// Un-grouping and weighted sum (Sections II-A and V-B of the paper): for every token the k
// expert outputs are gathered from their sorted rows and summed with the gate values in the
// fixed order j = 0..k-1, then the shared experts' output is added (Fig. 1) and the result is
// rounded to bf16.  Gather-based, no atomics: bit-reproducible run to run.
#include "device_utils.h"
#include "kernels.h"

namespace moe {

namespace {

__global__ __launch_bounds__(256) void combine_kernel(const float *__restrict__ Y, int y_planes,
                                                      long long y_plane_stride,
                                                      const float *__restrict__ w,
                                                      const int32_t *__restrict__ inv_perm,
                                                      const float *__restrict__ Ys, int ys_planes,
                                                      long long ys_plane_stride, int T, int d, int k,
                                                      uint16_t *__restrict__ out) {
  const int chunks = d >> 3;  // 8 columns per thread
  const long long gid = (long long)blockIdx.x * 256 + threadIdx.x;
  if (gid >= (long long)T * chunks) return;
  const int t = (int)(gid / chunks);
  const int c = (int)(gid - (long long)t * chunks) << 3;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.0f;
  for (int j = 0; j < k; ++j) {
    const int p = inv_perm[(size_t)t * k + j];
    const float wj = w[(size_t)t * k + j];
    float y[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) y[i] = 0.0f;
    for (int s = 0; s < y_planes; ++s) {
      const float4 *src = reinterpret_cast<const float4 *>(Y + s * y_plane_stride + (size_t)p * d + c);
      float4 a = src[0], b = src[1];
      y[0] += a.x; y[1] += a.y; y[2] += a.z; y[3] += a.w;
      y[4] += b.x; y[5] += b.y; y[6] += b.z; y[7] += b.w;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = fmaf(wj, y[i], acc[i]);
  }
  for (int s = 0; s < ys_planes; ++s) {
    const float4 *src = reinterpret_cast<const float4 *>(Ys + s * ys_plane_stride + (size_t)t * d + c);
    float4 a = src[0], b = src[1];
    acc[0] += a.x; acc[1] += a.y; acc[2] += a.z; acc[3] += a.w;
    acc[4] += b.x; acc[5] += b.y; acc[6] += b.z; acc[7] += b.w;
  }
  uint4 o;
  o.x = pack_bf16x2(acc[0], acc[1]);
  o.y = pack_bf16x2(acc[2], acc[3]);
  o.z = pack_bf16x2(acc[4], acc[5]);
  o.w = pack_bf16x2(acc[6], acc[7]);
  *reinterpret_cast<uint4 *>(out + (size_t)t * d + c) = o;
}

}  // namespace

hipError_t launch_combine(const float *Y, int y_planes, long long y_plane_stride, const float *w,
                          const int32_t *inv_perm, const float *Yshared, int ys_planes,
                          long long ys_plane_stride, int T, int d, int k, uint16_t *out,
                          hipStream_t stream) {
  long long total = (long long)T * (d >> 3);
  int grid = (int)((total + 255) / 256);
  hipLaunchKernelGGL(combine_kernel, dim3(grid), dim3(256), 0, stream, Y, y_planes, y_plane_stride, w,
                     inv_perm, Yshared, Yshared ? ys_planes : 0, ys_plane_stride, T, d, k, out);
  return hipGetLastError();
}

}  // namespace moe
