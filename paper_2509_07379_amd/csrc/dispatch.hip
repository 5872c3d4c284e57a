// Grouping of the tokens by assigned expert (Section V-B of the paper): a stable counting sort
// of the T*k assignments a = t*k + j by expert id.  Three small kernels (one block doing all three
// phases for decode-sized inputs), no ranks taken from atomics, so the permutation is the unique
// stable one:
//   1. per-block histogram (LDS integer atomics only count),
//   2. one wave scans the block histograms per expert and the experts' totals,
//   3. every block ranks its own assignments with wave ballots and scatters.
#include "device_utils.h"
#include "kernels.h"
#include "gemm_plan.h"

namespace moe {

namespace {

__global__ __launch_bounds__(kDispatchChunk) void dispatch_hist_kernel(const int32_t *__restrict__ ids,
                                                                       int n, int E,
                                                                       int32_t *__restrict__ blk_hist) {
  __shared__ int hist[kMaxExperts];
  const int tid = threadIdx.x;
  if (tid < kMaxExperts) hist[tid] = 0;
  __syncthreads();
  const int a = blockIdx.x * kDispatchChunk + tid;
  if (a < n) atomicAdd(&hist[ids[a]], 1);
  __syncthreads();
  if (tid < E) blk_hist[(size_t)blockIdx.x * E + tid] = hist[tid];
}

// Sixteen waves share the blocks out (lane = expert): each sums its share of the block histograms, the
// sums are exchanged through LDS, and each writes the running totals of its own blocks; the first wave
// then has every expert's count in its lanes and writes counts, offsets, the host's mailbox and, if
// asked, the work plans of the layer's grouped GEMMs (one launch less on the critical path).
constexpr int kScanWaves = 16;
__global__ __launch_bounds__(64 * kScanWaves) void dispatch_scan_kernel(const int32_t *__restrict__ blk_hist,
                                                                        int nblk, int E,
                                                                        int32_t *__restrict__ blk_base,
                                                                        int32_t *__restrict__ counts,
                                                                        int32_t *__restrict__ offsets,
                                                                        long long *__restrict__ host_counts, int seq,
                                                                        const PlanParams p0, const PlanParams p1) {
  __shared__ int part[kScanWaves][64];
  const int e = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int per = (nblk + kScanWaves - 1) / kScanWaves;
  const int b_lo = min(nblk, w * per), b_hi = min(nblk, b_lo + per);
  int sum = 0;
  if (e < E) {
    // 8 independent loads in flight per lane
    for (int b0 = b_lo; b0 < b_hi; b0 += 8) {
      int h[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) h[j] = b0 + j < b_hi ? blk_hist[(size_t)(b0 + j) * E + e] : 0;
#pragma unroll
      for (int j = 0; j < 8; ++j) sum += h[j];
    }
  }
  part[w][e] = sum;
  __syncthreads();
  int run = 0, total = 0;
#pragma unroll
  for (int v = 0; v < kScanWaves; ++v) {
    const int s = part[v][e];
    if (v < w) run += s;
    total += s;
  }
  if (e < E) {
    for (int b0 = b_lo; b0 < b_hi; b0 += 8) {
      int h[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) h[j] = b0 + j < b_hi ? blk_hist[(size_t)(b0 + j) * E + e] : 0;
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (b0 + j < b_hi) {
          blk_base[(size_t)(b0 + j) * E + e] = run;
          run += h[j];
        }
    }
  }
  if (w != 0) return;
  // inclusive scan over the experts (lanes)
  int incl = total;
#pragma unroll
  for (int s = 1; s < 64; s <<= 1) {
    int o = __shfl_up(incl, s);
    if (e >= s) incl += o;
  }
  if (e < E) {
    counts[e] = total;
    offsets[e] = incl - total;
    if (host_counts) host_counts[e] = mailbox_word(total, seq);   // the host polls these words
  }
  if (e == E - 1) offsets[E] = incl;
  if (p0.out) make_plan(p0, e, total);
  if (p1.out) make_plan(p1, e, total);
}

__global__ __launch_bounds__(kDispatchChunk) void dispatch_scatter_kernel(
    const int32_t *__restrict__ ids, int n, int E, const int32_t *__restrict__ blk_base,
    const int32_t *__restrict__ offsets, int32_t *__restrict__ perm, int32_t *__restrict__ inv_perm) {
  constexpr int kWaves = kDispatchChunk / 64;
  __shared__ int wave_cnt[kWaves][kMaxExperts];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < kWaves * kMaxExperts; i += kDispatchChunk) (&wave_cnt[0][0])[i] = 0;
  __syncthreads();
  const int a = blockIdx.x * kDispatchChunk + tid;
  const bool valid = a < n;
  const int e = valid ? ids[a] : 0;
  // lanes of this wave holding the same expert (6 ballots, E <= 64)
  unsigned long long peers = __ballot(valid);
#pragma unroll
  for (int bit = 0; bit < 6; ++bit) {
    unsigned long long b = __ballot((e >> bit) & 1);
    peers &= ((e >> bit) & 1) ? b : ~b;
  }
  const unsigned long long lt = (1ull << lane) - 1ull;
  const int rank_in_wave = __popcll(peers & lt);
  if (valid && rank_in_wave == 0) wave_cnt[wave][e] = __popcll(peers);
  __syncthreads();
  if (valid) {
    int base = offsets[e] + blk_base[(size_t)blockIdx.x * E + e];
    for (int wv = 0; wv < wave; ++wv) base += wave_cnt[wv][e];
    int p = base + rank_in_wave;
    perm[p] = a;
    inv_perm[a] = p;
  }
}


// Decode-sized inputs (n <= kSmallDispatch assignments): the three phases in one block.
constexpr int kSmallDispatch = 2048;

__global__ __launch_bounds__(kDispatchChunk) void dispatch_small_kernel(
    const int32_t *__restrict__ ids, int n, int E, int32_t *__restrict__ counts,
    int32_t *__restrict__ offsets, int32_t *__restrict__ perm, int32_t *__restrict__ inv_perm,
    long long *__restrict__ host_counts, int seq, int32_t *__restrict__ active, const PlanParams p0,
    const PlanParams p1) {
  constexpr int kWaves = kDispatchChunk / 64;
  __shared__ int hist[kMaxExperts];
  __shared__ int base[kMaxExperts];       // next free sorted position of each expert
  __shared__ int wave_cnt[kWaves][kMaxExperts];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < kMaxExperts) hist[tid] = 0;
  __syncthreads();
  for (int a = tid; a < n; a += kDispatchChunk) atomicAdd(&hist[ids[a]], 1);
  __syncthreads();
  if (wave == 0) {
    int run = lane < E ? hist[lane] : 0;
    int incl = run;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
      int o = __shfl_up(incl, s);
      if (lane >= s) incl += o;
    }
    if (lane < E) {
      counts[lane] = run;
      offsets[lane] = incl - run;
      base[lane] = incl - run;
      if (host_counts) host_counts[lane] = mailbox_word(run, seq);   // the host polls these words
    }
    if (lane == E - 1) offsets[E] = incl;
    if (active) {
      // the experts that have rows, in ascending id, then -1: a launch sized for the most there can be
      // finds its groups here without the host having looked at the counts
      const unsigned long long has = __ballot(run > 0);
      if (run > 0) active[__popcll(has & ((1ull << lane) - 1ull))] = lane;
      if (lane >= __popcll(has)) active[lane] = -1;
    }
    if (p0.out) make_plan(p0, lane, run);
    if (p1.out) make_plan(p1, lane, run);
  }
  for (int c0 = 0; c0 < n; c0 += kDispatchChunk) {
    for (int i = tid; i < kWaves * kMaxExperts; i += kDispatchChunk) (&wave_cnt[0][0])[i] = 0;
    __syncthreads();  // also publishes base[] (first round) / its update (later rounds)
    const int a = c0 + tid;
    const bool valid = a < n;
    const int e = valid ? ids[a] : 0;
    unsigned long long peers = __ballot(valid);
#pragma unroll
    for (int bit = 0; bit < 6; ++bit) {
      unsigned long long b = __ballot((e >> bit) & 1);
      peers &= ((e >> bit) & 1) ? b : ~b;
    }
    const int rank_in_wave = __popcll(peers & ((1ull << lane) - 1ull));
    if (valid && rank_in_wave == 0) wave_cnt[wave][e] = __popcll(peers);
    __syncthreads();
    if (valid) {
      int p = base[e] + rank_in_wave;
      for (int wv = 0; wv < wave; ++wv) p += wave_cnt[wv][e];
      perm[p] = a;
      inv_perm[a] = p;
    }
    __syncthreads();
    if (tid < E) {
      int add = 0;
      for (int wv = 0; wv < kWaves; ++wv) add += wave_cnt[wv][tid];
      base[tid] += add;
    }
    __syncthreads();  // base[] is final and wave_cnt[] has been read before the next round clears it
  }
}

}  // namespace

hipError_t launch_dispatch(const int32_t *ids, int n, int E, int32_t *blk_hist, int32_t *blk_base,
                           int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                           long long *host_counts, int seq, hipStream_t stream, int32_t *active,
                           const PlanParams *plans) {
  const PlanParams none{};
  const PlanParams &p0 = plans ? plans[0] : none, &p1 = plans ? plans[1] : none;
  if (n <= kSmallDispatch) {
    hipLaunchKernelGGL(dispatch_small_kernel, dim3(1), dim3(kDispatchChunk), 0, stream, ids, n, E, counts, offsets,
                       perm, inv_perm, host_counts, seq, active, p0, p1);
    return hipGetLastError();
  }
  const int nblk = (n + kDispatchChunk - 1) / kDispatchChunk;
  hipLaunchKernelGGL(dispatch_hist_kernel, dim3(nblk), dim3(kDispatchChunk), 0, stream, ids, n, E,
                     blk_hist);
  hipLaunchKernelGGL(dispatch_scan_kernel, dim3(1), dim3(64 * kScanWaves), 0, stream, blk_hist, nblk, E, blk_base,
                     counts, offsets, host_counts, seq, p0, p1);
  hipLaunchKernelGGL(dispatch_scatter_kernel, dim3(nblk), dim3(kDispatchChunk), 0, stream, ids, n, E,
                     blk_base, offsets, perm, inv_perm);
  return hipGetLastError();
}

}  // namespace moe
