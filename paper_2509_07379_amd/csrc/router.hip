// Gate of the MoE layer (Section II-A of the paper): logits = x . Wr^T, Top-k of n experts,
// gate values by softmax.  Also the linear stand-in for the layer-level predictor
// (Section IV-B / V-C): scores summed over the batch, top-m.
//
// The Top-k decision is an integer result, so the fp32 dot products are summed in one
// documented order that a scalar CPU replay can follow: element i belongs to lane
// (i / 8) mod 64, each lane adds its products in ascending i (bf16 x bf16 products are
// exact in fp32, so fma == mul + add), the 64 lanes are then summed by a butterfly that
// pairs lanes differing in bit 5 first and bit 0 last, and the bias is added last.
#include "device_utils.h"
#include "kernels.h"

namespace moe {

namespace {

constexpr int kRouterThreads = 256;
constexpr int kRouterWaves = kRouterThreads / 64;

__device__ __forceinline__ float dot8_ordered(const uint4 &xv, const uint4 &wv, float acc) {
  acc = fmaf(bf16_lo(xv.x), bf16_lo(wv.x), acc);
  acc = fmaf(bf16_hi(xv.x), bf16_hi(wv.x), acc);
  acc = fmaf(bf16_lo(xv.y), bf16_lo(wv.y), acc);
  acc = fmaf(bf16_hi(xv.y), bf16_hi(wv.y), acc);
  acc = fmaf(bf16_lo(xv.z), bf16_lo(wv.z), acc);
  acc = fmaf(bf16_hi(xv.z), bf16_hi(wv.z), acc);
  acc = fmaf(bf16_lo(xv.w), bf16_lo(wv.w), acc);
  acc = fmaf(bf16_hi(xv.w), bf16_hi(wv.w), acc);
  return acc;
}

// Wave-wide selection of the n_sel best of E values (one lane per expert): value descending,
// lower index on ties.  Lane j < n_sel returns the j-th selected (value, index).
__device__ __forceinline__ void wave_select(float v, int E, int n_sel, float &sel_val, int &sel_idx) {
  const int lane = lane_id();
  bool avail = lane < E;
  sel_val = 0.0f;
  sel_idx = -1;
  for (int j = 0; j < n_sel; ++j) {
    float cv = avail ? v : -INFINITY;
    int ci = avail ? lane : 64 + lane;  // unavailable lanes lose every tie
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
      float ov = __shfl_xor(cv, m);
      int oi = __shfl_xor(ci, m);
      bool take = (ov > cv) || (ov == cv && oi < ci);
      cv = take ? ov : cv;
      ci = take ? oi : ci;
    }
    if (lane == ci) avail = false;
    if (lane == j) {
      sel_val = cv;
      sel_idx = ci;
    }
  }
}

template <int TPB, int NWAVES>
__global__ __launch_bounds__(64 * NWAVES) void router_topk_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ wr, const float *__restrict__ bias,
    int bias_stride, int T, int d, int E, int k, int renormalize, float *__restrict__ logits,
    int32_t *__restrict__ ids, float *__restrict__ w, const SingleTokenDispatch one) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint4 *xs = reinterpret_cast<uint4 *>(smem);                           // [TPB][d/8]
  float *lg = reinterpret_cast<float *>(smem + (size_t)TPB * d * 2);     // [TPB][64]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t0 = blockIdx.x * TPB;
  const int nchunk = d >> 3;

  for (int c = tid; c < TPB * nchunk; c += 64 * NWAVES) {
    int tok = c / nchunk, cc = c - tok * nchunk;
    int t = min(t0 + tok, T - 1);
    xs[c] = reinterpret_cast<const uint4 *>(x + (size_t)t * d)[cc];
  }
  __syncthreads();

  for (int e = wave; e < E; e += NWAVES) {
    float acc[TPB];
#pragma unroll
    for (int q = 0; q < TPB; ++q) acc[q] = 0.0f;
    const uint4 *wrow = reinterpret_cast<const uint4 *>(wr + (size_t)e * d);
    for (int c = lane; c < nchunk; c += 64) {
      uint4 wv = wrow[c];
#pragma unroll
      for (int q = 0; q < TPB; ++q) acc[q] = dot8_ordered(xs[q * nchunk + c], wv, acc[q]);
    }
    // the TPB butterflies side by side: each level's exchanges are in flight together
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
#pragma unroll
      for (int q = 0; q < TPB; ++q) acc[q] = acc[q] + __shfl_xor(acc[q], m);
    }
#pragma unroll
    for (int q = 0; q < TPB; ++q) {
      int t = t0 + q;
      if (lane == 0 && t < T) {
        float s = acc[q];
        if (bias) s = s + bias[(size_t)t * bias_stride + e];
        lg[q * 64 + e] = s;
      }
    }
  }
  __syncthreads();

  for (int q = wave; q < TPB; q += NWAVES) {
    int t = t0 + q;
    if (t >= T) break;
    float v = lane < E ? lg[q * 64 + lane] : -INFINITY;
    if (logits && lane < E) logits[(size_t)t * E + lane] = v;
    float sv;
    int si;
    wave_select(v, E, k, sv, si);
    float top1 = __shfl(sv, 0);
    float wj;
    if (renormalize) {
      float p = lane < k ? expf(sv - top1) : 0.0f;
      wj = p / wave_sum_tree(p);
    } else {
      float p = lane < E ? expf(v - top1) : 0.0f;
      wj = expf(sv - top1) / wave_sum_tree(p);
    }
    if (lane < k) {
      ids[(size_t)t * k + lane] = si;
      w[(size_t)t * k + lane] = wj;
    }
    // One token: grouping its k assignments by expert is a rank computation inside this wave (the
    // k experts are distinct), so the call needs no grouping kernel.  Same tables as launch_dispatch.
    if (one.counts) {
      int c = 0;
      for (int j = 0; j < k; ++j) c += (__shfl(si, j) == lane) ? 1 : 0;   // lane = expert
      int incl = c;
#pragma unroll
      for (int sft = 1; sft < 64; sft <<= 1) {
        const int o = __shfl_up(incl, sft);
        if (lane >= sft) incl += o;
      }
      const int excl = incl - c;
      if (lane < E) {
        one.counts[lane] = c;
        one.offsets[lane] = excl;
        if (one.host_counts) one.host_counts[lane] = mailbox_word(c, one.seq);   // the host polls these words
      }
      if (lane == E - 1) one.offsets[E] = incl;
      const int pos = __shfl(excl, lane < k ? si : 0);   // sorted position of assignment `lane`
      if (lane < k) {
        one.perm[pos] = lane;
        one.inv_perm[lane] = pos;
      }
    }
  }
}

// scores[e] = sum_t dot(x[t], wp[e]); one wave per expert.
__global__ __launch_bounds__(kRouterThreads) void predictor_scores_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ wp, int T, int d, int E,
    float *__restrict__ scores) {
  const int lane = threadIdx.x & 63;
  const int e = blockIdx.x * kRouterWaves + (threadIdx.x >> 6);
  if (e >= E) return;
  const int nchunk = d >> 3;
  const uint4 *wrow = reinterpret_cast<const uint4 *>(wp + (size_t)e * d);
  float s = 0.0f;
  for (int t = 0; t < T; ++t) {
    const uint4 *xrow = reinterpret_cast<const uint4 *>(x + (size_t)t * d);
    float acc = 0.0f;
    for (int c = lane; c < nchunk; c += 64) acc = dot8_ordered(xrow[c], wrow[c], acc);
    s = s + wave_sum_tree(acc);
  }
  if (lane == 0) scores[e] = s;
}

// One fully connected layer of the ExpertMLP predictor (Section IV-B) for one input vector:
// out[n] = act(W[n,:] . in + bias[n]), act = ReLU(scale * z + shift) for hidden layers (batch
// normalisation in inference form), identity for the last.  One wave per neuron; the fp32 sum is
// taken in a fixed order that a scalar replay can follow: element i belongs to lane i mod 64, each
// lane adds its products in ascending i with one fused multiply-add per element, then the butterfly.
// in / out are fp32; `in` may live in pinned host memory (the state vector is built on the host).
__global__ __launch_bounds__(kRouterThreads) void mlp_layer_kernel(
    const float *__restrict__ in, const uint16_t *__restrict__ w, const float *__restrict__ bias,
    const float *__restrict__ scale, const float *__restrict__ shift, int n_in, int n_out,
    float *__restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * kRouterWaves + (threadIdx.x >> 6);
  if (n >= n_out) return;
  const uint16_t *wrow = w + (size_t)n * n_in;
  float acc = 0.0f;
  for (int i = lane; i < n_in; i += 64) acc = fmaf(in[i], bf16_to_f32(wrow[i]), acc);
  float z = wave_sum_tree(acc) + bias[n];
  if (scale) {
    z = fmaf(z, scale[n], shift[n]);
    if (!(z > 0.0f)) z = 0.0f;
  }
  if (lane == 0) out[n] = z;
}

__global__ __launch_bounds__(64) void predictor_topm_kernel(const float *__restrict__ scores, int E,
                                                            int m, int32_t *__restrict__ top_out) {
  const int lane = threadIdx.x;
  float v = lane < E ? scores[lane] : -INFINITY;
  float sv;
  int si;
  wave_select(v, E, m, sv, si);
  if (lane < m) top_out[lane] = si;
}

}  // namespace


hipError_t launch_router_topk(const uint16_t *x, const uint16_t *wr, const float *bias,
                              int bias_stride, int T, int d, int E, int k, int renormalize,
                              float *logits, int32_t *ids, float *w, hipStream_t stream,
                              const SingleTokenDispatch *one) {
  // 4 tokens per block share one pass over Wr, 8 waves take the experts in turn (a wave's time is a
  // chain of dependent loads and exchanges per expert, so more waves per token group means a shorter
  // chain); small batches (decode) use one token per block and 16 waves, so that the E dot products
  // of a token run side by side.
  SingleTokenDispatch none{};
  if (one && T != 1) return hipErrorInvalidValue;
  if (T >= 64) {
    constexpr int TPB = 4;
    size_t smem = (size_t)TPB * d * 2 + TPB * 64 * sizeof(float);
    int grid = (T + TPB - 1) / TPB;
    static bool attr_set = false;   // token vectors of d up to kMaxHidden: more than the 64 KB default
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(router_topk_kernel<TPB, 8>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize,
                                         TPB * kMaxHidden * 2 + TPB * 64 * (int)sizeof(float));
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    hipLaunchKernelGGL((router_topk_kernel<TPB, 8>), dim3(grid), dim3(512), smem, stream, x, wr, bias,
                       bias_stride, T, d, E, k, renormalize, logits, ids, w, none);
  } else {
    constexpr int TPB = 1;
    size_t smem = (size_t)TPB * d * 2 + TPB * 64 * sizeof(float);
    hipLaunchKernelGGL((router_topk_kernel<TPB, 16>), dim3(T), dim3(1024), smem, stream, x, wr, bias,
                       bias_stride, T, d, E, k, renormalize, logits, ids, w, one ? *one : none);
  }
  return hipGetLastError();
}

hipError_t launch_mlp_predictor(const float *state, const int32_t *dims, int n_fc, const uint16_t *const *w,
                                const float *const *bias, const float *const *scale, const float *const *shift,
                                float *act0, float *act1, int m, float *scores, int32_t *top_out,
                                hipStream_t stream) {
  const float *in = state;
  for (int l = 0; l < n_fc; ++l) {
    const bool last = l + 1 == n_fc;
    float *out = last ? scores : ((l & 1) ? act1 : act0);
    const int grid = (dims[l + 1] + kRouterWaves - 1) / kRouterWaves;
    hipLaunchKernelGGL(mlp_layer_kernel, dim3(grid), dim3(kRouterThreads), 0, stream, in, w[l], bias[l],
                       last ? nullptr : scale[l], last ? nullptr : shift[l], dims[l], dims[l + 1], out);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    in = out;
  }
  hipLaunchKernelGGL(predictor_topm_kernel, dim3(1), dim3(64), 0, stream, scores, dims[n_fc], m, top_out);
  return hipGetLastError();
}

hipError_t launch_predictor(const uint16_t *x, const uint16_t *wp, int T, int d, int E, int m,
                            float *scores, int32_t *top_out, hipStream_t stream) {
  int grid = (E + kRouterWaves - 1) / kRouterWaves;
  hipLaunchKernelGGL(predictor_scores_kernel, dim3(grid), dim3(kRouterThreads), 0, stream, x, wp, T,
                     d, E, scores);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL(predictor_topm_kernel, dim3(1), dim3(64), 0, stream, scores, E, m, top_out);
  return hipGetLastError();
}

}  // namespace moe
