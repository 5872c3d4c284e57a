// Expansion of 4-bit integer expert weights (unsigned codes in groups of 128 with scale and zero point)
// into the bf16 matrices the GPU expert cache holds for that format.  The paper evaluates quantised
// models (Section VI); a fetched expert of this form lands in a staging area next to the cache and the
// kernel below writes its slot, so the GEMM kernels read bf16.  (e4m3 and MXFP4 experts are never
// expanded in memory: every kernel reads their codes.)
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_utils.h"
#include "kernels.h"

namespace moe {

namespace {

constexpr int kThreads = 256;

// 4-bit codes (unsigned, two per byte, even column in the low nibble), groups of 128 along a row with
// one fp32 scale and one zero point each:  out = bf16_rne(fp32((code - zero) * scale)).
// One lane expands 16 codes (one 8-byte load, two 16-byte stores); cols % 128 == 0.
__global__ __launch_bounds__(kThreads) void dequant_int4_g128_kernel(const uint8_t *__restrict__ codes,
                                                                     const float *__restrict__ scales,
                                                                     const uint8_t *__restrict__ zeros,
                                                                     long long rows, int cols,
                                                                     uint16_t *__restrict__ out) {
  const int per_row = cols >> 4;          // 16-code pieces per row
  const int groups = cols >> 7;
  const long long pieces = rows * per_row;
  for (long long c = (long long)blockIdx.x * kThreads + threadIdx.x; c < pieces;
       c += (long long)gridDim.x * kThreads) {
    const long long row = c / per_row;
    const int piece = (int)(c - row * per_row);
    const long long g = row * groups + (piece >> 3);
    const float s = scales[g];
    const int z = zeros[g];
    const uint2 q = *reinterpret_cast<const uint2 *>(codes + c * 8);
    uint32_t w[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t byte = ((j < 4 ? q.x : q.y) >> ((j & 3) * 8)) & 0xFFu;
      const float lo = (float)((int)(byte & 15u) - z) * s;
      const float hi = (float)((int)(byte >> 4) - z) * s;
      w[j] = (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
    }
    uint4 *dst = reinterpret_cast<uint4 *>(out + c * 16);
    dst[0] = make_uint4(w[0], w[1], w[2], w[3]);
    dst[1] = make_uint4(w[4], w[5], w[6], w[7]);
  }
}

}  // namespace

hipError_t launch_dequant_int4_g128(const uint8_t *codes, const float *scales, const uint8_t *zeros,
                                    long long rows, int cols, uint16_t *out, hipStream_t stream) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  if (cols % 128) return hipErrorInvalidValue;
  const long long pieces = rows * (cols >> 4);
  long long blocks = (pieces + kThreads - 1) / kThreads;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(dequant_int4_g128_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, codes, scales,
                     zeros, rows, cols, out);
  return hipGetLastError();
}

}  // namespace moe
