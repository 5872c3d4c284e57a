// Expert mat-vec for the decode stage (Section V-C of the paper): a decode step routes a
// handful of tokens, so every active expert's weights are streamed once from its cache slot
// and the kernel is bound by HBM bandwidth, not by the matrix cores.
//
//   GEMM_SWIGLU     h[p, n] = bf16( silu(x_p . Wg[n]) * (x_p . Wu[n]) )
//   GEMM_PLAIN_F32  y[p, c] = h_p . Wd[c]
//
// Per-token kernels (grouped_gemv_kernel, fused_down_combine_kernel): one wave owns R consecutive
// weight rows, each lane streams 16-byte pieces of those rows (R or 2R independent loads in flight
// per step), multiplies them with the group's token vectors held in LDS, and the 64 partial sums
// are reduced with a butterfly at the end.  Up to 8 tokens share one pass over the weights; the
// token count selects the unrolling.
// Matrix-core kernel (grouped_skinny_kernel): the same single pass for up to 16 tokens per expert
// with 16x16x32 MFMAs; it takes over where the per-token kernels are bound by their arithmetic
// (several tokens on quantised rows, long bf16 down rows, more than 8 tokens).
#include "device_utils.h"
#include "kernels.h"

namespace moe {

namespace {

constexpr int GV_MAXTOK = 8;   // tokens per pass over the weights

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Eight bf16 products added to an fp32 sum with four two-element dot instructions
// (v_dot2c_f32_bf16): no unpacking of the operands, a third of the vector instructions of an
// fma chain.  With eight tokens per pass the fma chain, not HBM, bounded the kernel.
__device__ __forceinline__ float dot2(uint32_t x, uint32_t w, float acc) {   // by value: plain scalars
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, x), __builtin_bit_cast(bf16x2, w), acc, false);
}
__device__ __forceinline__ float dot8(const u32x4 &xv, const u32x4 &wv, float acc) {
  acc = dot2(xv.x, wv.x, acc);
  acc = dot2(xv.y, wv.y, acc);
  acc = dot2(xv.z, wv.z, acc);
  acc = dot2(xv.w, wv.w, acc);
  return acc;
}

template <int MODE, int NT, int NTMAX, int GV_R, int UNR = 2>
__device__ __forceinline__ void accumulate(const u32x4 *__restrict__ xs, int seg_chunks,
                                           const u32x4 *const (&w0)[GV_R], const u32x4 *const (&w1)[GV_R],
                                           int lane, float (&acc0)[GV_R][NTMAX],
                                           float (&acc1)[GV_R][NTMAX]) {
#pragma unroll UNR
  for (int c = lane; c < seg_chunks; c += 64) {
    u32x4 wv0[GV_R], wv1[GV_R];
#pragma unroll
    for (int r = 0; r < GV_R; ++r) {
      wv0[r] = __builtin_nontemporal_load(w0[r] + c);
      if (MODE == GEMM_SWIGLU) wv1[r] = __builtin_nontemporal_load(w1[r] + c);
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      u32x4 xv = xs[t * seg_chunks + c];
#pragma unroll
      for (int r = 0; r < GV_R; ++r) {
        acc0[r][t] = dot8(xv, wv0[r], acc0[r][t]);
        if (MODE == GEMM_SWIGLU) acc1[r][t] = dot8(xv, wv1[r], acc1[r][t]);
      }
    }
  }
}

typedef float f32x2 __attribute__((ext_vector_type(2)));

// Four e4m3 codes (one 32-bit word, element 0 in the low byte) and their row's scale -> the four
// bf16 weights bf16_rne(value(code) * scale), packed in pairs: the hardware conversions of gfx950
// (OCP e4m3 to fp32, exact; fp32 to bf16, nearest even) around one fp32 multiply.
struct Pair32 { uint32_t w01, w23; };
__device__ __forceinline__ Pair32 expand4(uint32_t codes, float scale) {   // by value: plain scalars
  f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)codes, false);
  f32x2 b = __builtin_amdgcn_cvt_pk_f32_fp8((int)codes, true);
  a *= scale;
  b *= scale;
  Pair32 p;
  p.w01 = __builtin_bit_cast(uint32_t, __builtin_convertvector(a, bf16x2));
  p.w23 = __builtin_bit_cast(uint32_t, __builtin_convertvector(b, bf16x2));
  return p;
}
__device__ __forceinline__ void expand16(const u32x4 &q, float scale, u32x4 &lo, u32x4 &hi) {
  const uint32_t qx = q.x, qy = q.y, qz = q.z, qw = q.w;
  const Pair32 a = expand4(qx, scale), b = expand4(qy, scale), c = expand4(qz, scale), d = expand4(qw, scale);
  lo = u32x4{a.w01, a.w23, b.w01, b.w23};
  hi = u32x4{c.w01, c.w23, d.w01, d.w23};
}

// The same sums from 8-bit weights: a lane's 16-byte piece holds 16 codes, i.e. two of the token
// vectors' 8-element pieces; the codes are expanded once per piece and used for all NT tokens.
template <int MODE, int NT, int NTMAX, int GV_R>
__device__ __forceinline__ void accumulate_q8(const u32x4 *__restrict__ xs, int seg_chunks,
                                              const u32x4 *const (&w0)[GV_R], const u32x4 *const (&w1)[GV_R],
                                              const float (&s0)[GV_R], const float (&s1)[GV_R], int lane,
                                              float (&acc0)[GV_R][NTMAX], float (&acc1)[GV_R][NTMAX]) {
  const int pieces = seg_chunks >> 1;
#pragma unroll 2
  for (int c = lane; c < pieces; c += 64) {
    u32x4 q0[GV_R], q1[GV_R];
#pragma unroll
    for (int r = 0; r < GV_R; ++r) {
      q0[r] = __builtin_nontemporal_load(w0[r] + c);
      if (MODE == GEMM_SWIGLU) q1[r] = __builtin_nontemporal_load(w1[r] + c);
    }
#pragma unroll
    for (int r = 0; r < GV_R; ++r) {
      u32x4 lo0, hi0, lo1, hi1;
      expand16(q0[r], s0[r], lo0, hi0);
      if (MODE == GEMM_SWIGLU) expand16(q1[r], s1[r], lo1, hi1);
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const u32x4 xlo = xs[t * seg_chunks + 2 * c], xhi = xs[t * seg_chunks + 2 * c + 1];
        acc0[r][t] = dot8(xhi, hi0, dot8(xlo, lo0, acc0[r][t]));
        if (MODE == GEMM_SWIGLU) acc1[r][t] = dot8(xhi, hi1, dot8(xlo, lo1, acc1[r][t]));
      }
    }
  }
}

// 32 MXFP4 codes (one 16-byte piece = one scale block; element 0 in the low nibble of byte 0) ->
// 32 bf16 weights value(code) * scale, exact: the hardware conversion of gfx950 takes the two codes
// of one byte and the scale's exponent and returns the packed pair.
__device__ __forceinline__ uint32_t mx4_pair(uint32_t word, float scale, int byte) {   // by value: plain scalars
  bf16x2 p;
  if (byte == 0) p = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(word, scale, 0);
  else if (byte == 1) p = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(word, scale, 1);
  else if (byte == 2) p = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(word, scale, 2);
  else p = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(word, scale, 3);
  return __builtin_bit_cast(uint32_t, p);
}
__device__ __forceinline__ u32x4 mx4_expand8(uint32_t word, float scale) {
  return u32x4{mx4_pair(word, scale, 0), mx4_pair(word, scale, 1), mx4_pair(word, scale, 2), mx4_pair(word, scale, 3)};
}

// The same sums from MXFP4 weights: a lane's 16-byte piece holds the 32 codes of one scale block, i.e.
// four of the token vectors' 8-element pieces.  sc0 / sc1: the rows' scale bytes for this K segment.
template <int MODE, int NT, int NTMAX, int GV_R>
__device__ __forceinline__ void accumulate_mx4(const u32x4 *__restrict__ xs, int seg_chunks,
                                               const u32x4 *const (&w0)[GV_R], const u32x4 *const (&w1)[GV_R],
                                               const uint8_t *const (&sc0)[GV_R], const uint8_t *const (&sc1)[GV_R],
                                               int lane, float (&acc0)[GV_R][NTMAX], float (&acc1)[GV_R][NTMAX]) {
  const int pieces = seg_chunks >> 2;
#pragma unroll NT <= 2 ? 2 : 1
  for (int c = lane; c < pieces; c += 64) {
    u32x4 q0[GV_R], q1[GV_R];
    float f0[GV_R], f1[GV_R];
#pragma unroll
    for (int r = 0; r < GV_R; ++r) {
      q0[r] = __builtin_nontemporal_load(w0[r] + c);
      f0[r] = __uint_as_float((uint32_t)sc0[r][c] << 23);
      if (MODE == GEMM_SWIGLU) {
        q1[r] = __builtin_nontemporal_load(w1[r] + c);
        f1[r] = __uint_as_float((uint32_t)sc1[r][c] << 23);
      }
    }
#pragma unroll
    for (int r = 0; r < GV_R; ++r) {
      {   // gate (or down) row: expand, use for all tokens, then the up row (half as many live registers)
        const uint32_t a0 = q0[r].x, a1 = q0[r].y, a2 = q0[r].z, a3 = q0[r].w;
        const u32x4 g0 = mx4_expand8(a0, f0[r]), g1 = mx4_expand8(a1, f0[r]), g2 = mx4_expand8(a2, f0[r]),
                    g3 = mx4_expand8(a3, f0[r]);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const u32x4 *xp = xs + t * seg_chunks + 4 * c;
          acc0[r][t] = dot8(xp[3], g3, dot8(xp[2], g2, dot8(xp[1], g1, dot8(xp[0], g0, acc0[r][t]))));
        }
      }
      if (MODE == GEMM_SWIGLU) {
        const uint32_t b0 = q1[r].x, b1 = q1[r].y, b2 = q1[r].z, b3 = q1[r].w;
        const u32x4 u0 = mx4_expand8(b0, f1[r]), u1 = mx4_expand8(b1, f1[r]), u2 = mx4_expand8(b2, f1[r]),
                    u3 = mx4_expand8(b3, f1[r]);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const u32x4 *xp = xs + t * seg_chunks + 4 * c;
          acc1[r][t] = dot8(xp[3], u3, dot8(xp[2], u2, dot8(xp[1], u1, dot8(xp[0], u0, acc1[r][t]))));
        }
      }
    }
  }
}

// GV_R weight rows per wave.  Measured on MI355X: the more, smaller waves stream the weights, the
// closer the kernel gets to the HBM rate (one row per wave for rows of 4 KB and more, two for
// shorter rows); blocks that walk over several row groups were slower in every shape.
// NTHR threads per block: 256, or 1024 when many tokens share a pass (every block stages the token
// vectors of a K segment in LDS first, which for 8 tokens is as many bytes as a 4-wave block's share
// of the weights; 16 waves share one copy).
// (at least 6 waves per SIMD for the 4-wave blocks: left alone, the register allocator of the
// multi-token variants wanders between 76 and 100 registers with unrelated edits)
// QF: 0, or the format (GemmArgs::qfmt) of the quantised copies from which the experts named in
// routed.q8_mask are streamed (the second problem, the shared experts, is always bf16); with QF = 0
// the mask is ignored.
template <int MODE, int NTMAX, int GV_R, int NTHR, int QF>
__global__ __launch_bounds__(NTHR) __attribute__((amdgpu_waves_per_eu(NTHR == 256 ? ((QF == 2 || (QF && (NTMAX > 1 || GV_R > 1))) ? 4 : 6) : 4)))
void grouped_gemv_kernel(const GemmArgs routed, const GemmArgs extra,
                                                             int has_extra, int kseg, int ntcap, int n_extra_y) {
  constexpr int GV_THREADS = NTHR, GV_WAVES = NTHR / 64;
  // Grid: x = block of weight rows (as many as the routed problem needs), y = selected group of
  // the routed problem; with has_extra, the last n_extra_y values of y are further runs of gridDim.x
  // blocks for the second problem (the always-on shared experts), so that one launch streams both
  // weight sets and neither pays for the other's row count.
  // (the test is written against gridDim.y: the form with the count of routed groups costs this
  // compiler 22 more vector registers and a third of the occupancy)
  const bool is_extra = has_extra && blockIdx.y + (unsigned)n_extra_y >= gridDim.y;
  const GemmArgs &args = is_extra ? extra : routed;
  const unsigned sel = blockIdx.y;                                           // which selected group
  const unsigned bx = is_extra ? (blockIdx.y + (unsigned)n_extra_y - gridDim.y) * gridDim.x + blockIdx.x : blockIdx.x;
  extern __shared__ __align__(16) unsigned char smem[];
  u32x4 *xs = reinterpret_cast<u32x4 *>(smem);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // group of this block: the sel-th expert of the mask
  int grp = 0, row0 = args.single_row0, cnt = args.single_rows;
  if (args.offsets) {
    if (args.sel_ids) {
      // a list on the device: the gate's own id list (one token: its k experts, all distinct), or the
      // grouping kernel's list of the experts that have rows, padded with -1
      grp = args.sel_ids[sel];
      if (grp < 0) return;
    } else {
      unsigned long long m = args.group_mask;
      for (unsigned i = 0; i < sel; ++i) m &= m - 1;
      if (m == 0) return;   // fewer groups in the mask than the launch was sized for
      grp = __ffsll((long long)m) - 1;
    }
    row0 = args.offsets[grp];
    cnt = args.offsets[grp + 1] - row0;
  }
  if (cnt <= 0) return;

  const char *wptr = args.wbase + (long long)args.slot[grp] * args.wstride;
  const uint16_t *B0 = reinterpret_cast<const uint16_t *>(wptr + args.b0_off);
  const uint16_t *B1 = reinterpret_cast<const uint16_t *>(wptr + args.b1_off);
  const int n_first = (bx * GV_WAVES + wave) * GV_R;
  if ((int)bx * GV_WAVES * GV_R >= args.N) return;
  const bool q8 = QF != 0 && !is_extra && ((args.q8_mask >> grp) & 1ull);
  const char *qptr = args.qbase + (long long)args.slot[grp] * args.qstride;
  float s0[GV_R], s1[GV_R];
  if (QF == 1) {
#pragma unroll
    for (int r = 0; r < GV_R; ++r) {
      const int n = min(n_first + r, args.N - 1);
      s0[r] = q8 ? reinterpret_cast<const float *>(qptr + args.q_s0_off)[n] : 0.0f;
      s1[r] = q8 ? reinterpret_cast<const float *>(qptr + args.q_s1_off)[n] : 0.0f;
    }
  }

  for (int tok0 = 0; tok0 < cnt; tok0 += ntcap) {
    const int ntok = min(ntcap, cnt - tok0);  // ntcap <= NTMAX tokens fit the LDS buffer
    float acc0[GV_R][NTMAX], acc1[GV_R][NTMAX];
#pragma unroll
    for (int r = 0; r < GV_R; ++r)
#pragma unroll
      for (int t = 0; t < NTMAX; ++t) acc0[r][t] = acc1[r][t] = 0.0f;

    for (int k0 = 0; k0 < args.K; k0 += kseg) {
      const int seg = min(kseg, args.K - k0);
      const int seg_chunks = seg >> 3;
      __syncthreads();  // previous segment fully consumed
      for (int c = tid; c < ntok * seg_chunks; c += GV_THREADS) {
        int t = c / seg_chunks, cc = c - t * seg_chunks;
        int p = row0 + tok0 + t;
        long long srow = args.perm ? (long long)(args.perm[p] / args.k_top) : (long long)p;
        xs[c] = *reinterpret_cast<const u32x4 *>(args.A + srow * args.lda + k0 + cc * 8);
      }
      __syncthreads();
      const u32x4 *w0[GV_R], *w1[GV_R];
#pragma unroll
      for (int r = 0; r < GV_R; ++r) {
        int n = min(n_first + r, args.N - 1);
        w0[r] = reinterpret_cast<const u32x4 *>(B0 + (long long)n * args.ldb + k0);
        w1[r] = reinterpret_cast<const u32x4 *>(B1 + (long long)n * args.ldb + k0);
      }
      const uint8_t *sc0[GV_R], *sc1[GV_R];
      if (QF == 1 && q8) {   // the same rows in the 8-bit copy: K bytes per row
#pragma unroll
        for (int r = 0; r < GV_R; ++r) {
          const int n = min(n_first + r, args.N - 1);
          w0[r] = reinterpret_cast<const u32x4 *>(qptr + args.q_b0_off + (long long)n * args.ldb + k0);
          w1[r] = reinterpret_cast<const u32x4 *>(qptr + args.q_b1_off + (long long)n * args.ldb + k0);
        }
      }
      if (QF == 2 && q8) {   // MXFP4 copy: K / 2 bytes of codes and K / 32 scale bytes per row
#pragma unroll
        for (int r = 0; r < GV_R; ++r) {
          const long long n = min(n_first + r, args.N - 1);
          w0[r] = reinterpret_cast<const u32x4 *>(qptr + args.q_b0_off + ((n * args.ldb + k0) >> 1));
          w1[r] = reinterpret_cast<const u32x4 *>(qptr + args.q_b1_off + ((n * args.ldb + k0) >> 1));
          sc0[r] = reinterpret_cast<const uint8_t *>(qptr + args.q_s0_off) + ((n * args.ldb + k0) >> 5);
          sc1[r] = reinterpret_cast<const uint8_t *>(qptr + args.q_s1_off) + ((n * args.ldb + k0) >> 5);
        }
      }
#define MOE_GEMV_CASE(NT)                                                             \
  if constexpr (NT <= NTMAX) {                                                        \
    if (ntok == NT) {                                                                 \
      if (QF == 1 && q8) accumulate_q8<MODE, NT, NTMAX, GV_R>(xs, seg_chunks, w0, w1, s0, s1, lane, acc0, acc1); \
      else if (QF == 2 && q8) accumulate_mx4<MODE, NT, NTMAX, GV_R>(xs, seg_chunks, w0, w1, sc0, sc1, lane, acc0, acc1); \
      else accumulate<MODE, NT, NTMAX, GV_R>(xs, seg_chunks, w0, w1, lane, acc0, acc1); \
    }                                                                                 \
  }
      MOE_GEMV_CASE(1) MOE_GEMV_CASE(2) MOE_GEMV_CASE(3) MOE_GEMV_CASE(4)
      MOE_GEMV_CASE(5) MOE_GEMV_CASE(6) MOE_GEMV_CASE(7) MOE_GEMV_CASE(8)
#undef MOE_GEMV_CASE
    }

#pragma unroll
    for (int r = 0; r < GV_R; ++r) {
      const int n = n_first + r;
#pragma unroll
      for (int t = 0; t < NTMAX; ++t) {
        if (t >= ntok) break;
        float s0 = wave_sum_tree(acc0[r][t]);
        float s1 = (MODE == GEMM_SWIGLU) ? wave_sum_tree(acc1[r][t]) : 0.0f;
        if (lane == 0 && n < args.N) {
          const long long o = (long long)(row0 + tok0 + t) * args.ldo + n;
          if (MODE == GEMM_SWIGLU)
            reinterpret_cast<uint16_t *>(args.out)[o] = f32_to_bf16(silu(s0) * s1);
          else
            reinterpret_cast<float *>(args.out)[o] = s0;
        }
      }
    }
  }
}

// One token, down projection and weighted sum in one launch: a wave owns GV_R output
// columns and walks over the token's k experts (ids from the gate's list on the device); per expert
// the same row sums as grouped_gemv_kernel<GEMM_PLAIN_F32> (same lane order, so the same bits), then
// out[c] = bf16(fma(w_j, y_j[c], ...)) in the order j = 0 .. k-1 of the weighted-sum kernel.  Saves
// the fp32 round trip of y and one launch.
// The h vectors (one per expert, then the shared experts') pass through LDS.  stage_all: all of them
// fit the buffer side by side and are staged once, before the first weight row is streamed.
// Otherwise one vector at a time: the next one is fetched into registers (FUSED_PF pieces per thread)
// while the current expert's rows are streamed, so that the hand-over between two experts costs two
// barriers and an LDS write instead of a round trip to L2 during which no weight is in flight.
constexpr int FUSED_PF = 8;   // 16-byte pieces per thread held for the next vector: K <= 16384
template <int GV_R, int QF>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(QF ? 4 : 6)))
void fused_down_combine_kernel(const GemmArgs args, const GemmArgs extra, int has_extra,
                               const float *__restrict__ gate_w, int k_top, uint16_t *__restrict__ out,
                               int stage_all) {
  constexpr int GV_WAVES = 4;
  extern __shared__ __align__(16) unsigned char smem[];
  u32x4 *xs = reinterpret_cast<u32x4 *>(smem);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_first = (blockIdx.x * GV_WAVES + wave) * GV_R;
  const int seg_chunks = args.K >> 3;
  const int n_phases = k_top + (has_extra ? 1 : 0);
  // phase p < k_top: expert sel_ids[p], its h vector is the sorted row offsets[expert];
  // phase k_top: the shared experts' h vector
  // lane j < k of every wave looks up expert j once (id, sorted row, slot, gate value); the phases
  // read them back with a lane read, so no phase waits for a chain of dependent lookups
  int my_grp = 0, my_row = 0, my_slot = 0;
  float my_w = 0.0f;
  if (lane < k_top) {
    my_grp = args.sel_ids[lane];
    my_row = args.offsets[my_grp];
    my_slot = args.slot[my_grp];
    my_w = gate_w[lane];
  }
  auto vector_of = [&](int p, int &chunks) -> const u32x4 * {
    if (p < k_top) {
      chunks = seg_chunks;
      return reinterpret_cast<const u32x4 *>(args.A + (long long)__builtin_amdgcn_readlane(my_row, p) * args.lda);
    }
    chunks = extra.K >> 3;
    return reinterpret_cast<const u32x4 *>(extra.A + (long long)extra.single_row0 * extra.lda);
  };
  const bool prefetch = !stage_all && seg_chunks <= FUSED_PF * 256 && (!has_extra || (extra.K >> 3) <= FUSED_PF * 256);
  u32x4 pf[FUSED_PF];
  if (stage_all) {
    int base = 0;
    for (int p = 0; p < n_phases; ++p) {
      int chunks;
      const u32x4 *v = vector_of(p, chunks);
      for (int c = tid; c < chunks; c += 256) xs[base + c] = v[c];
      base += chunks;
    }
    __syncthreads();
  } else if (prefetch) {
    int chunks;
    const u32x4 *v = vector_of(0, chunks);
#pragma unroll
    for (int i = 0; i < FUSED_PF; ++i)
      if (tid + i * 256 < chunks) pf[i] = v[tid + i * 256];
  }
  float total[GV_R];
#pragma unroll
  for (int r = 0; r < GV_R; ++r) total[r] = 0.0f;
  int xs_base = 0;
  for (int p = 0; p < n_phases; ++p) {
    const bool shared_phase = p >= k_top;
    // (field by field: choosing between the two argument blocks as a whole puts both on the stack)
    const int chunks = (shared_phase ? extra.K : args.K) >> 3;
    const int n_rows = shared_phase ? extra.N : args.N;
    const long long ldb = shared_phase ? extra.ldb : args.ldb;
    const u32x4 *xv = xs;
    if (stage_all) {
      xv = xs + xs_base;
      xs_base += chunks;
    } else {
      __syncthreads();                     // the previous vector is fully consumed
      if (prefetch) {
#pragma unroll
        for (int i = 0; i < FUSED_PF; ++i)
          if (tid + i * 256 < chunks) xs[tid + i * 256] = pf[i];
      } else {
        int ch;
        const u32x4 *v = vector_of(p, ch);
        for (int c = tid; c < chunks; c += 256) xs[c] = v[c];
      }
      __syncthreads();
      if (prefetch && p + 1 < n_phases) {
        int ch;
        const u32x4 *v = vector_of(p + 1, ch);
#pragma unroll
        for (int i = 0; i < FUSED_PF; ++i)
          if (tid + i * 256 < ch) pf[i] = v[tid + i * 256];
      }
    }
    const int grp = shared_phase ? 0 : __builtin_amdgcn_readlane(my_grp, p);
    const int slot = shared_phase ? 0 : __builtin_amdgcn_readlane(my_slot, p);
    const bool q8 = QF != 0 && !shared_phase && ((args.q8_mask >> grp) & 1ull);
    const char *wptr = shared_phase ? extra.wbase + (long long)extra.slot[0] * extra.wstride + extra.b0_off
                                    : args.wbase + (long long)slot * args.wstride + args.b0_off;
    const char *qptr = args.qbase + (long long)slot * args.qstride;
    const u32x4 *w0[GV_R];
    const uint8_t *sc0[GV_R];
    float s0[GV_R];
    float acc0[GV_R][1], acc1[GV_R][1];
#pragma unroll
    for (int r = 0; r < GV_R; ++r) {
      const long long n = min(n_first + r, n_rows - 1);
      acc0[r][0] = acc1[r][0] = 0.0f;
      s0[r] = 0.0f;
      sc0[r] = nullptr;
      w0[r] = reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(wptr) + n * ldb);
      if (QF == 1 && q8) {
        w0[r] = reinterpret_cast<const u32x4 *>(qptr + args.q_b0_off + n * args.ldb);
        s0[r] = reinterpret_cast<const float *>(qptr + args.q_s0_off)[n];
      }
      if (QF == 2 && q8) {
        w0[r] = reinterpret_cast<const u32x4 *>(qptr + args.q_b0_off + ((n * args.ldb) >> 1));
        sc0[r] = reinterpret_cast<const uint8_t *>(qptr + args.q_s0_off) + ((n * args.ldb) >> 5);
      }
    }
    if (QF == 1 && q8) accumulate_q8<GEMM_PLAIN_F32, 1, 1, GV_R>(xv, chunks, w0, w0, s0, s0, lane, acc0, acc1);
    else if (QF == 2 && q8) accumulate_mx4<GEMM_PLAIN_F32, 1, 1, GV_R>(xv, chunks, w0, w0, sc0, sc0, lane, acc0, acc1);
    else accumulate<GEMM_PLAIN_F32, 1, 1, GV_R>(xv, chunks, w0, w0, lane, acc0, acc1);
    if (!shared_phase) {
      const float wj = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, my_w), p));
#pragma unroll
      for (int r = 0; r < GV_R; ++r) {
        // y = 0 + (the one plane's value), then fma(w_j, y, sum): the weighted-sum kernel's operations
        const float y = 0.0f + wave_sum_tree(acc0[r][0]);
        total[r] = fmaf(wj, y, total[r]);
      }
    } else {
      // the shared experts (one always-on group of bf16 weights): their down rows for the same
      // columns, added after the routed sum as the weighted-sum kernel adds them
#pragma unroll
      for (int r = 0; r < GV_R; ++r) total[r] = total[r] + wave_sum_tree(acc0[r][0]);
    }
  }
#pragma unroll
  for (int r = 0; r < GV_R; ++r)
    if (lane == 0 && n_first + r < args.N) out[n_first + r] = f32_to_bf16(total[r]);
}

// Several tokens per expert: the same pass over the weights with the sums taken by the matrix cores
// instead of per-token dot products, which at 8 tokens, and with 4-bit weights from 3, cost more
// issue time than the bytes take to arrive.  v_mfma_f32_16x16x32_bf16 multiplies 16 weight rows by up
// to 16 token vectors: lane l supplies 8 consecutive k of weight row l % 16 and of token l % 16 (lane
// group l / 16 selects which 8 of the 32), and receives the sums of rows 4 (l / 16) + i, i = 0..3,
// for token l % 16.  A block owns one pair of row tiles (the gate and up rows of 16 columns of h, or
// 32 columns of y); its waves cut K into slices, one each, and add their partial sums through LDS
// in wave order, so that the launch consists of many short, equal pieces.  A lane streams 32 bytes
// per row tile and step, four lanes one whole 128-byte line of a row; quantised rows are expanded to
// the same bf16 values as in the per-token kernels.  The token vectors are read from global memory
// as they are needed (a few KB per slice, shared by every block: they stay in the caches).  The sums
// are fp32 in the matrix core's order, so results agree with the per-token kernels to rounding, not
// bit for bit.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int SK_TOK = 16;       // tokens per pass over the weights
constexpr int SK_MAXWAVES = 8;   // K slices per block

__device__ __forceinline__ f32x4 mfma16(const u32x4 &w, const u32x4 &x, const f32x4 &acc) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w), __builtin_bit_cast(bf16x8, x), acc, 0, 0, 0);
}

// One K slice of NP row tile pairs.  F: format of the rows (0 bf16, 1 e4m3 + row scale, 2 MXFP4).
// pa / pb: this lane's row in the two tiles of each pair at the slice's first k, already advanced to
// the lane group's share; xl: this lane's token vector, likewise; sca / scb: MXFP4 scale bytes,
// likewise.  The token pieces of a step are loaded once and used for all 2 NP tiles: with quantised
// rows they are 2 (e4m3) or 4 (MXFP4) times the bytes of a tile's codes, and with one pair per wave
// those launches were bound by the token reads from L2, not by HBM.
template <int NP>
struct SkTiles {
  const char *pa[NP], *pb[NP];
  const uint8_t *sca[NP], *scb[NP];
  float sa[NP], sb[NP];
  f32x4 acc_a[NP], acc_b[NP];
};

template <int F, int NP>
__device__ __forceinline__ void skinny_segment(SkTiles<NP> &T, const char *__restrict__ xl, int seg) {
  constexpr int KL = F == 0 ? 16 : (F == 1 ? 32 : 64);   // k per lane and step: 32 bytes of the row
  constexpr int STEP = 4 * KL;                           // k per wave and step
  constexpr int NX = KL / 8;                             // 16-byte pieces of the token vector per step
  constexpr int D = (F == 0 && NP == 1) ? 3 : 2;         // steps whose loads are in flight or in use
  // The registers of a step.  The loads of step s + D - 1 are issued before the products of step s
  // are taken, each into its own registers: left to itself the compiler reuses one set and waits
  // for every load of a turn before it issues the next turn's.
  struct Regs {
    u32x4 a0[NP], a1[NP], b0[NP], b1[NP], x[NX];
    uint32_t sc[NP];   // MXFP4: the four scale bytes of the step (tile a: bytes 0, 1; tile b: bytes 2, 3)
  };
  auto load = [&](int ks, Regs &R) {
    const u32x4 *x = reinterpret_cast<const u32x4 *>(xl + ks * 2);   // first: they arrive first
#pragma unroll
    for (int i = 0; i < NX; ++i) R.x[i] = x[i];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const u32x4 *wa = reinterpret_cast<const u32x4 *>(T.pa[p] + (F == 0 ? ks * 2 : (F == 1 ? ks : ks >> 1)));
      const u32x4 *wb = reinterpret_cast<const u32x4 *>(T.pb[p] + (F == 0 ? ks * 2 : (F == 1 ? ks : ks >> 1)));
      R.a0[p] = __builtin_nontemporal_load(wa);
      R.a1[p] = __builtin_nontemporal_load(wa + 1);
      R.b0[p] = __builtin_nontemporal_load(wb);
      R.b1[p] = __builtin_nontemporal_load(wb + 1);
      if (F == 2) {
        const int blk = ks >> 5;   // two scale blocks of 32 codes per lane, row tile and step
        R.sc[p] = (uint32_t)T.sca[p][blk] | ((uint32_t)T.sca[p][blk + 1] << 8) | ((uint32_t)T.scb[p][blk] << 16) |
                  ((uint32_t)T.scb[p][blk + 1] << 24);
      }
    }
  };
  auto compute = [&](const Regs &R) {
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      f32x4 &acc_a = T.acc_a[p], &acc_b = T.acc_b[p];
      if (F == 0) {
        acc_a = mfma16(R.a0[p], R.x[0], acc_a);
        acc_b = mfma16(R.b0[p], R.x[0], acc_b);
        acc_a = mfma16(R.a1[p], R.x[1], acc_a);
        acc_b = mfma16(R.b1[p], R.x[1], acc_b);
      } else if (F == 1) {
        const float sa = T.sa[p], sb = T.sb[p];
        u32x4 lo, hi;
        expand16(R.a0[p], sa, lo, hi);
        acc_a = mfma16(lo, R.x[0], acc_a);
        acc_a = mfma16(hi, R.x[1], acc_a);
        expand16(R.b0[p], sb, lo, hi);
        acc_b = mfma16(lo, R.x[0], acc_b);
        acc_b = mfma16(hi, R.x[1], acc_b);
        expand16(R.a1[p], sa, lo, hi);
        acc_a = mfma16(lo, R.x[2], acc_a);
        acc_a = mfma16(hi, R.x[3], acc_a);
        expand16(R.b1[p], sb, lo, hi);
        acc_b = mfma16(lo, R.x[2], acc_b);
        acc_b = mfma16(hi, R.x[3], acc_b);
      } else {
        const uint32_t sc = R.sc[p];
        const float fa0 = __uint_as_float((sc & 0xffu) << 23), fa1 = __uint_as_float(((sc >> 8) & 0xffu) << 23);
        const float fb0 = __uint_as_float(((sc >> 16) & 0xffu) << 23), fb1 = __uint_as_float((sc >> 24) << 23);
        const u32x4 qa0 = R.a0[p], qa1 = R.a1[p], qb0 = R.b0[p], qb1 = R.b1[p];
        const uint32_t a00 = qa0.x, a01 = qa0.y, a02 = qa0.z, a03 = qa0.w, a10 = qa1.x, a11 = qa1.y, a12 = qa1.z, a13 = qa1.w;
        const uint32_t b00 = qb0.x, b01 = qb0.y, b02 = qb0.z, b03 = qb0.w, b10 = qb1.x, b11 = qb1.y, b12 = qb1.z, b13 = qb1.w;
        acc_a = mfma16(mx4_expand8(a00, fa0), R.x[0], acc_a); acc_b = mfma16(mx4_expand8(b00, fb0), R.x[0], acc_b);
        acc_a = mfma16(mx4_expand8(a01, fa0), R.x[1], acc_a); acc_b = mfma16(mx4_expand8(b01, fb0), R.x[1], acc_b);
        acc_a = mfma16(mx4_expand8(a02, fa0), R.x[2], acc_a); acc_b = mfma16(mx4_expand8(b02, fb0), R.x[2], acc_b);
        acc_a = mfma16(mx4_expand8(a03, fa0), R.x[3], acc_a); acc_b = mfma16(mx4_expand8(b03, fb0), R.x[3], acc_b);
        acc_a = mfma16(mx4_expand8(a10, fa1), R.x[4], acc_a); acc_b = mfma16(mx4_expand8(b10, fb1), R.x[4], acc_b);
        acc_a = mfma16(mx4_expand8(a11, fa1), R.x[5], acc_a); acc_b = mfma16(mx4_expand8(b11, fb1), R.x[5], acc_b);
        acc_a = mfma16(mx4_expand8(a12, fa1), R.x[6], acc_a); acc_b = mfma16(mx4_expand8(b12, fb1), R.x[6], acc_b);
        acc_a = mfma16(mx4_expand8(a13, fa1), R.x[7], acc_a); acc_b = mfma16(mx4_expand8(b13, fb1), R.x[7], acc_b);
      }
    }
  };
  // n >= 1 steps.  Start-up and the turns of the main loop issue their loads unconditionally (the
  // counts of loads in flight that the compiler derives for its waits are then the same on every
  // path); the last 2 D - 2 steps at most are drained with conditions.
  const int n = seg / STEP;
  Regs R[D];
#pragma unroll
  for (int i = 0; i < D - 1; ++i) load(min(i, n - 1) * STEP, R[i]);
  int s = 0;
  for (; s + 2 * D - 2 < n; s += D) {
#pragma unroll
    for (int i = 0; i < D; ++i) {
      load((s + i + D - 1) * STEP, R[(i + D - 1) % D]);
      compute(R[i]);
    }
  }
#pragma unroll
  for (int i = 0; i < 2 * D - 2; ++i) {
    if (s + i < n) {
      if (s + i + D - 1 < n) load((s + i + D - 1) * STEP, R[(i + D - 1) % D]);
      compute(R[i % D]);
    }
  }
}

// Grid: x = NP row tile pairs, y = selected group, the shared experts in further runs of y (as
// grouped_gemv_kernel).  blockDim.x / 64 <= SK_MAXWAVES waves = K slices.
// Requires N % 16 == 0 and K % 64 == 0 (bf16), 128 (e4m3), 256 (MXFP4).
template <int MODE, int QF, int NP>
__global__ __launch_bounds__(SK_MAXWAVES * 64) __attribute__((amdgpu_waves_per_eu(QF == 2 ? 2 : (QF == 1 ? 3 : 4))))
void grouped_skinny_kernel(const GemmArgs routed, const GemmArgs extra,
                                                                          int has_extra, int n_extra_y) {
  constexpr int PAIR = MODE == GEMM_SWIGLU ? 16 : 32;   // output columns per tile pair
  constexpr int ROWS = NP * PAIR;                       // output columns per block
  const bool is_extra = has_extra && blockIdx.y + (unsigned)n_extra_y >= gridDim.y;
  // (field by field: choosing between the two argument blocks as a whole puts both on the stack)
#define SK_ARG(f) (is_extra ? extra.f : routed.f)
  const int N = SK_ARG(N), K = SK_ARG(K), k_top = SK_ARG(k_top);
  const long long lda = SK_ARG(lda), ldb = SK_ARG(ldb), ldo = SK_ARG(ldo);
  const uint16_t *A = SK_ARG(A);
  const int32_t *perm = SK_ARG(perm), *offsets = SK_ARG(offsets);
  void *outp = SK_ARG(out);
  const unsigned sel = blockIdx.y;
  const unsigned bx = is_extra ? (blockIdx.y + (unsigned)n_extra_y - gridDim.y) * gridDim.x + blockIdx.x : blockIdx.x;
  __shared__ float red[SK_MAXWAVES][8 * NP][64];
  const int tid = threadIdx.x, lane = tid & 63, waves = blockDim.x >> 6;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: the slice bounds stay scalar
  const int r = lane & 15, g = lane >> 4;

  int grp = 0, row0 = SK_ARG(single_row0), cnt = SK_ARG(single_rows);
  if (offsets) {
    if (!is_extra && routed.sel_ids) {
      grp = routed.sel_ids[sel];
      if (grp < 0) return;   // (the list of experts with rows is padded with -1)
    } else {
      unsigned long long m = SK_ARG(group_mask);
      for (unsigned i = 0; i < sel; ++i) m &= m - 1;
      if (m == 0) return;
      grp = __ffsll((long long)m) - 1;
    }
    row0 = offsets[grp];
    cnt = offsets[grp + 1] - row0;
  }
  if (cnt <= 0) return;
  const int n0 = bx * ROWS;
  if (n0 >= N) return;   // the whole block, before any barrier

  const bool q = QF != 0 && !is_extra && ((routed.q8_mask >> grp) & 1ull);
  const int kl = !q ? 16 : (QF == 1 ? 32 : 64);
  // this wave's K slice: whole steps of 4 kl, shared out as evenly as they go
  const int steps = K / (4 * kl);
  const int k_begin = (int)((long long)steps * wave / waves) * (4 * kl);
  const int k_len = (int)((long long)steps * (wave + 1) / waves) * (4 * kl) - k_begin;
  const int slot = is_extra ? extra.slot[grp] : routed.slot[grp];
  const char *wptr = SK_ARG(wbase) + (long long)slot * SK_ARG(wstride);
  const char *qptr = routed.qbase + (long long)slot * routed.qstride;   // used with q only
  const long long b0_off = SK_ARG(b0_off);
  const long long b_off = MODE == GEMM_SWIGLU ? SK_ARG(b1_off) : b0_off;
  const long long qb_off = MODE == GEMM_SWIGLU ? routed.q_b1_off : routed.q_b0_off;
  const long long qs_off = MODE == GEMM_SWIGLU ? routed.q_s1_off : routed.q_s0_off;
  SkTiles<NP> T;
#pragma unroll
  for (int p = 0; p < NP; ++p) {
    // rows of the pair's two tiles held by this lane (clamped: tiles past the last column compute a
    // copy of the last row and store nothing)
    const long long na = min(n0 + p * PAIR + r, N - 1);
    const long long nb = MODE == GEMM_SWIGLU ? na : min(n0 + p * PAIR + 16 + r, N - 1);
    const long long ka = na * ldb + k_begin + g * kl, kb = nb * ldb + k_begin + g * kl;   // first element
    T.sca[p] = T.scb[p] = nullptr;
    T.sa[p] = T.sb[p] = 0.0f;
    if (!q) {
      T.pa[p] = wptr + b0_off + ka * 2;
      T.pb[p] = wptr + b_off + kb * 2;
    } else if (QF == 1) {
      T.pa[p] = qptr + routed.q_b0_off + ka;
      T.pb[p] = qptr + qb_off + kb;
      T.sa[p] = reinterpret_cast<const float *>(qptr + routed.q_s0_off)[na];
      T.sb[p] = reinterpret_cast<const float *>(qptr + qs_off)[nb];
    } else {
      T.pa[p] = qptr + routed.q_b0_off + (ka >> 1);
      T.pb[p] = qptr + qb_off + (kb >> 1);
      T.sca[p] = reinterpret_cast<const uint8_t *>(qptr + routed.q_s0_off) + (ka >> 5);
      T.scb[p] = reinterpret_cast<const uint8_t *>(qptr + qs_off) + (kb >> 5);
    }
  }

  for (int tok0 = 0; tok0 < cnt; tok0 += SK_TOK) {
    const int ntok = min(SK_TOK, cnt - tok0);
    // lanes past the last token read the last token's vector again; their sums are not stored
    const int p = row0 + tok0 + min(r, ntok - 1);
    const long long srow = perm ? (long long)(perm[p] / k_top) : (long long)p;
    const char *xl = reinterpret_cast<const char *>(A + srow * lda + k_begin + g * kl);
#pragma unroll
    for (int p = 0; p < NP; ++p) T.acc_a[p] = T.acc_b[p] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    if (k_len <= 0) {}   // more waves than steps: nothing to add
    else if (!q) skinny_segment<0, NP>(T, xl, k_len);
    else if (QF == 1) skinny_segment<1, NP>(T, xl, k_len);
    else skinny_segment<2, NP>(T, xl, k_len);
    if (tok0) __syncthreads();   // the previous pass's partial sums are consumed
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        red[wave][8 * p + i][lane] = T.acc_a[p][i];
        red[wave][8 * p + 4 + i][lane] = T.acc_b[p][i];
      }
    __syncthreads();
    // wave 0: the slices' sums in wave order; lane: token r, output columns 4 g .. 4 g + 3 of each tile
    if (wave == 0 && r < ntok) {
      const long long orow = (long long)(row0 + tok0 + r) * ldo;
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        float sum[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          sum[i] = red[0][8 * p + i][lane];
          for (int w = 1; w < waves; ++w) sum[i] += red[w][8 * p + i][lane];
        }
        const int ca = n0 + p * PAIR + 4 * g;
        if (MODE == GEMM_SWIGLU) {
          if (ca < N) {
            uint2 o;
            o.x = pack_bf16x2(silu(sum[0]) * sum[4], silu(sum[1]) * sum[5]);
            o.y = pack_bf16x2(silu(sum[2]) * sum[6], silu(sum[3]) * sum[7]);
            *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(outp) + orow + ca) = o;
          }
        } else {
          float *y = reinterpret_cast<float *>(outp) + orow;
          if (ca < N) *reinterpret_cast<float4 *>(y + ca) = float4{sum[0], sum[1], sum[2], sum[3]};
          if (ca + 16 < N) *reinterpret_cast<float4 *>(y + ca + 16) = float4{sum[4], sum[5], sum[6], sum[7]};
        }
      }
    }
  }
#undef SK_ARG
}

}  // namespace

// Quantised experts (e4m3 rows, MXFP4) exist in the cache in that form only: every mat-vec reads the
// codes and expands them in registers.
bool gemv_reads_copies(const GemmArgs &args) {
  return args.qbase != nullptr && args.K % (args.qfmt == 2 ? 32 : 16) == 0;
}

// One token (its row in the sorted order is offsets[expert]), args = the down projection's arguments
// with sel_ids set, gate_w [k] the token's gate values, out [N] bf16; extra: the shared experts' down
// projection (one group of one row), added last.  Requires K * 2 <= 64 KB for both.
hipError_t launch_fused_down_combine(const GemmArgs &args, const float *gate_w, int k_top, uint16_t *out,
                                     hipStream_t stream, const GemmArgs *extra) {
  if (!args.sel_ids || !args.offsets || args.K % 8 || (size_t)args.K * 2 > 65536 || k_top < 1 || k_top > 64)
    return hipErrorInvalidValue;
  if (extra && (extra->N != args.N || extra->K % 8 || (size_t)extra->K * 2 > 65536 || extra->single_rows != 1))
    return hipErrorInvalidValue;
  const int max_k = extra && extra->K > args.K ? extra->K : args.K;
  const GemmArgs &extra_args = extra ? *extra : args;
  const int has_extra = extra ? 1 : 0;
  const bool use_q = args.q8_mask != 0 && gemv_reads_copies(args);
  int rows_per_wave = (use_q && args.K >= 2048) ? 2 : (args.K >= 2048 ? 1 : 2);
  if (!use_q && args.N < 4096) rows_per_wave = 1;   // a wave walks the experts one after the other: few columns, few waves
  const int rows_per_block = 4 * rows_per_wave;
  const dim3 grid((args.N + rows_per_block - 1) / rows_per_block);
  // all h vectors side by side when that leaves room for five blocks per compute unit
  const size_t all_bytes = ((size_t)k_top * args.K + (extra ? extra->K : 0)) * 2;
  const int stage_all = all_bytes <= 28672 ? 1 : 0;
  const size_t smem = stage_all ? all_bytes : (size_t)max_k * 2;
#define MOE_FUSED_LAUNCH(R, Q)                                                                \
  do {                                                                                        \
    auto kern = fused_down_combine_kernel<R, Q>;                                              \
    static bool attr_set = false;                                                             \
    if (!attr_set) {                                                                          \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 65536);  \
      if (e != hipSuccess) return e;                                                          \
      attr_set = true;                                                                        \
    }                                                                                         \
    hipLaunchKernelGGL(kern, grid, dim3(256), smem, stream, args, extra_args, has_extra, gate_w, k_top, out, stage_all); \
  } while (0)
  const int q = use_q ? args.qfmt : 0;
  if (rows_per_wave == 2) {
    if (q == 2) MOE_FUSED_LAUNCH(2, 2);
    else if (q == 1) MOE_FUSED_LAUNCH(2, 1);
    else MOE_FUSED_LAUNCH(2, 0);
  } else {
    MOE_FUSED_LAUNCH(1, 0);
  }
#undef MOE_FUSED_LAUNCH
  return hipGetLastError();
}

hipError_t launch_grouped_gemv(GemmMode mode, const GemmArgs &args, int max_rows_per_group,
                               int n_groups_in_mask, hipStream_t stream, const GemmArgs *extra) {
  if (n_groups_in_mask <= 0 || max_rows_per_group <= 0) {
    if (!extra) return hipSuccess;
    return launch_grouped_gemv(mode, *extra, extra->single_rows, 1, stream, nullptr);
  }
  int max_tok = max_rows_per_group, max_n = args.N, max_k = args.K;
  if (extra) {
    if (extra->single_rows > max_tok) max_tok = extra->single_rows;
    if (extra->N > max_n) max_n = extra->N;
    if (extra->K > max_k) max_k = extra->K;
  }
  const bool use_q8 = args.q8_mask != 0 && gemv_reads_copies(args);
  {
    // several tokens per expert: the matrix-core kernel, where the shapes allow its steps
    const int kmul = !use_q8 ? 64 : (args.qfmt == 2 ? 256 : 128);
    const bool shapes_ok = args.N % 16 == 0 && args.K % kmul == 0 && (!extra || (extra->N % 16 == 0 && extra->K % 64 == 0));
    // Where it pays (measured, Mixtral- and Qwen-shaped experts): quantised rows (the per-token
    // kernels are bound by their dot products there), e4m3 down projections from 5 tokens; bf16
    // rows only in down projections with long rows, or past the per-token kernels' 8 tokens.
    bool pays;
    if (use_q8) pays = !(args.qfmt == 1 && mode == GEMM_PLAIN_F32 && max_tok < 5);
    // (a launch of fewer than 128 blocks of four waves leaves most of the chip without a wave: the
    // Qwen-shaped shared experts' down projection, 64 blocks, took 41 us there against 10 us per token)
    else pays = max_tok > GV_MAXTOK ||
                (mode == GEMM_PLAIN_F32 && args.K >= 4096 && (long long)(args.N / 32) * n_groups_in_mask >= 128);
    if (args.tune.skinny_forced) pays = true;
    // from 3 tokens per expert; quantised gate/up rows from 2 (MXFP4, Mixtral shape, 2 tokens: 57
    // against 70 us per launch; one token is faster per token: 37 against 41 us)
    const int min_tok = args.tune.skinny_min_tok > 0 ? args.tune.skinny_min_tok : ((use_q8 && mode == GEMM_SWIGLU) ? 2 : 3);
    if (max_tok >= min_tok && shapes_ok && pays) {
      // row tile pairs per block: quantised rows share their token pieces between two pairs, except in
      // down projections with few tokens, where the launch would be left with too few blocks
      // (MXFP4, Mixtral shape, 4 tokens: 59 against 52 us; 32 tokens: 85 against 96 us)
      const int pairs = use_q8 && (mode == GEMM_SWIGLU || max_tok > 8) ? 2 : 1;
      const int rows_per_block = pairs * (mode == GEMM_SWIGLU ? 16 : 32);
      const int bpg = (args.N + rows_per_block - 1) / rows_per_block;
      const int extra_blocks = extra ? (extra->N + rows_per_block - 1) / rows_per_block : 0;
      const int n_extra_y = (extra_blocks + bpg - 1) / bpg;
      const dim3 grid(bpg, n_groups_in_mask + n_extra_y);
      const int has_extra = extra ? 1 : 0;
      const GemmArgs &extra_args = extra ? *extra : args;
      const int qf = use_q8 ? args.qfmt : 0;
      // K slices (waves) per block: at least 8 steps each, 4 at most
      const int steps = args.K / (use_q8 ? (args.qfmt == 2 ? 256 : 128) : 64);
      int slices = steps / 8 < 1 ? 1 : (steps / 8 > 4 ? 4 : steps / 8);
      if (args.tune.skinny_waves >= 1 && args.tune.skinny_waves <= SK_MAXWAVES) slices = args.tune.skinny_waves;
      const int threads = 64 * slices;
#define MOE_SKINNY_LAUNCH(MODE, Q)                                                                         \
  do {                                                                                                     \
    if (pairs == 2)                                                                                        \
      hipLaunchKernelGGL((grouped_skinny_kernel<MODE, Q, (Q != 0 ? 2 : 1)>), grid, dim3(threads), 0, stream, args, \
                         extra_args, has_extra, n_extra_y);                                                \
    else                                                                                                   \
      hipLaunchKernelGGL((grouped_skinny_kernel<MODE, Q, 1>), grid, dim3(threads), 0, stream, args, extra_args, \
                         has_extra, n_extra_y);                                                            \
  } while (0)
      if (mode == GEMM_SWIGLU) {
        if (qf == 2) MOE_SKINNY_LAUNCH(GEMM_SWIGLU, 2);
        else if (qf == 1) MOE_SKINNY_LAUNCH(GEMM_SWIGLU, 1);
        else MOE_SKINNY_LAUNCH(GEMM_SWIGLU, 0);
      } else {
        if (qf == 2) MOE_SKINNY_LAUNCH(GEMM_PLAIN_F32, 2);
        else if (qf == 1) MOE_SKINNY_LAUNCH(GEMM_PLAIN_F32, 1);
        else MOE_SKINNY_LAUNCH(GEMM_PLAIN_F32, 0);
      }
#undef MOE_SKINNY_LAUNCH
      return hipGetLastError();
    }
  }
  const int ntcap = max_tok < GV_MAXTOK ? max_tok : GV_MAXTOK;
  int kseg = (65536 / (ntcap * 2)) / 512 * 512;   // token vectors of one K segment fit 64 KB of LDS
  if (kseg >= max_k) kseg = max_k;
  const size_t smem = (size_t)ntcap * kseg * 2;
  int rows_per_wave = max_k >= 2048 ? 1 : 2;
  if (use_q8 && max_k >= 2048) rows_per_wave = 2;   // a row is half as many bytes: two per wave keep as much in flight
  if (args.tune.gemv_rows > 0) rows_per_wave = args.tune.gemv_rows;
  if (ntcap > 2 && rows_per_wave > 2) rows_per_wave = 2;   // accumulators: rows x tokens x {gate, up}
  // quantised rows are short (K or K / 2 bytes): with several tokens 16 waves share one staged copy of
  // the token vectors (4 tokens, Mixtral shape: MXFP4 241 -> 201 us per layer, e4m3 255 -> 234 us; one
  // token is as fast with 4 waves)
  // bf16 rows with 3 or 4 tokens: a 4-wave block stages as many bytes of token vectors as half its
  // share of the weights; with large experts 16 waves per staged copy win (Mixtral shape, 8 tokens in
  // groups of at most 4: gate/up 315 -> 276 us), with small ones the finer blocks do (Qwen shape,
  // 8 tokens: 130 against 143 us per layer)
  const bool big_rows = (long long)args.N * args.K >= (1ll << 24);
  const int threads = (ntcap > 4 || (ntcap > 2 && big_rows) || (use_q8 && ntcap > 1)) ? 1024 : 256;
  const int rows_per_block = (threads / 64) * rows_per_wave;
  const int bpg = (args.N + rows_per_block - 1) / rows_per_block;
  const int extra_blocks = extra ? (extra->N + rows_per_block - 1) / rows_per_block : 0;
  const int n_extra_y = (extra_blocks + bpg - 1) / bpg;
  dim3 grid(bpg, n_groups_in_mask + n_extra_y);
  const int has_extra = extra ? 1 : 0;
  const GemmArgs &extra_args = extra ? *extra : args;
#define MOE_GEMV_LAUNCH(MODE, NTMAX)                                                          \
  do {                                                                                        \
    if (rows_per_wave == 4) MOE_GEMV_LAUNCH_R(MODE, NTMAX, (NTMAX <= 2 ? 4 : 2));             \
    else if (rows_per_wave >= 2) MOE_GEMV_LAUNCH_R(MODE, NTMAX, 2);                           \
    else MOE_GEMV_LAUNCH_R(MODE, NTMAX, 1);                                                   \
  } while (0)
#define MOE_GEMV_LAUNCH_R(MODE, NTMAX, R)                                                     \
  do {                                                                                        \
    if (use_q8 && args.qfmt == 2) MOE_GEMV_LAUNCH_Q(MODE, NTMAX, R, 2);                       \
    else if (use_q8) MOE_GEMV_LAUNCH_Q(MODE, NTMAX, R, 1);                                    \
    else MOE_GEMV_LAUNCH_Q(MODE, NTMAX, R, 0);                                                \
  } while (0)
#define MOE_GEMV_LAUNCH_Q(MODE, NTMAX, R, Q)                                                  \
  do {                                                                                        \
    /* 3 or 4 tokens on bf16 rows exist with 4 and with 16 waves; every other case with one of them */ \
    if (threads == 1024) MOE_GEMV_LAUNCH_T(MODE, NTMAX, R, Q, ((NTMAX > 2 || (Q != 0 && NTMAX > 1)) ? 1024 : 256)); \
    else MOE_GEMV_LAUNCH_T(MODE, NTMAX, R, Q, ((NTMAX > 4 || (Q != 0 && NTMAX > 1)) ? 1024 : 256)); \
  } while (0)
#define MOE_GEMV_LAUNCH_T(MODE, NTMAX, R, Q, NTHR)                                            \
  do {                                                                                        \
    auto kern = grouped_gemv_kernel<MODE, NTMAX, R, NTHR, Q>;                                  \
    static bool attr_set = false;                                                             \
    if (!attr_set) {                                                                          \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 65536);  \
      if (e != hipSuccess) return e;                                                          \
      attr_set = true;                                                                        \
    }                                                                                         \
    hipLaunchKernelGGL(kern, grid, dim3(threads), smem, stream, args, extra_args, has_extra, kseg, ntcap, \
                       n_extra_y);                                                            \
  } while (0)
  if (mode == GEMM_SWIGLU) {
    if (ntcap == 1) MOE_GEMV_LAUNCH(GEMM_SWIGLU, 1);
    else if (ntcap == 2) MOE_GEMV_LAUNCH(GEMM_SWIGLU, 2);
    else if (ntcap <= 4) MOE_GEMV_LAUNCH(GEMM_SWIGLU, 4);
    else MOE_GEMV_LAUNCH(GEMM_SWIGLU, 8);
  } else {
    if (ntcap == 1) MOE_GEMV_LAUNCH(GEMM_PLAIN_F32, 1);
    else if (ntcap == 2) MOE_GEMV_LAUNCH(GEMM_PLAIN_F32, 2);
    else if (ntcap <= 4) MOE_GEMV_LAUNCH(GEMM_PLAIN_F32, 4);
    else MOE_GEMV_LAUNCH(GEMM_PLAIN_F32, 8);
  }
#undef MOE_GEMV_LAUNCH
#undef MOE_GEMV_LAUNCH_R
#undef MOE_GEMV_LAUNCH_Q
#undef MOE_GEMV_LAUNCH_T
  return hipGetLastError();
}

}  // namespace moe
