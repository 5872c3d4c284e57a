// Grouped expert GEMM on bf16 MFMA (gfx950), the batch-per-expert operation of the prefill
// stage (Section V-B of the paper): each expert multiplies the rows routed to it by its own
// weights, read from its GPU-expert-cache slot.
//
//   GEMM_SWIGLU     H[p, n]  = bf16( silu(X_p . Wg[n]) * (X_p . Wu[n]) )   A rows gathered by perm
//   GEMM_PLAIN_F32  Y[p, c]  = H_p . Wd[c]   (fp32, one plane per K slice)
//   GEMM_PLAIN_BF16 C = A . B^T (bf16; dense stand-in for the non-MoE block)
//
// Both operands are K-contiguous ("NT"), so every lane feeds the MFMA with 8 consecutive
// bf16 of a row (one 16-byte LDS read).  Tiles are BM x BN x 64, staged through LDS with a
// 16-byte XOR swizzle and double buffering (global loads of tile i+1 are in flight while the
// MFMAs of tile i run; one barrier per K step).
//
// Ragged groups: a group of `cnt` rows is cut into ceil(cnt/BM) M-tiles of equal height
// (rounded up to 32), each wave owns every WARPS_M-th 32-row fragment, and fragments past
// the tile's last row are skipped, so a nearly empty tail tile costs a fraction of a full one
// and the skipping stays balanced over the waves.
//
// Launch: 1-D grid; hardware block b runs logical tile (b % 8) * chunk + b / 8 so that the
// blocks one XCD receives (every 8th) are consecutive logical tiles - the M-tiles sharing a
// weight tile hit the same L2.
#include "device_utils.h"
#include "kernels.h"

namespace moe {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 64;           // K elements per stage (128 bytes per row)
constexpr int ROW_BYTES = BK * 2;

__device__ __forceinline__ int swz(int row, int kc) { return row * ROW_BYTES + ((kc ^ (row & 7)) << 4); }

template <int BM, int BN, int WARPS_M, int WARPS_N, int MODE>
__global__ __launch_bounds__(64 * WARPS_M * WARPS_N) void grouped_gemm_kernel(const GemmArgs args) {
  constexpr int NTHR = 64 * WARPS_M * WARPS_N;
  constexpr int BN_OUT = (MODE == GEMM_SWIGLU) ? BN / 2 : BN;
  constexpr int FM = BM / (32 * WARPS_M);
  constexpr int FN = BN / (32 * WARPS_N);
  constexpr int FNH = (MODE == GEMM_SWIGLU) ? FN / 2 : FN;  // column fragments per half
  constexpr int CA = BM * 8 / NTHR;  // 16-byte chunks per thread, A tile
  constexpr int CB = BN * 8 / NTHR;
  constexpr int STAGE = (BM + BN) * ROW_BYTES;
  static_assert(BM % (32 * WARPS_M) == 0 && BN % (32 * WARPS_N) == 0, "tile/wave mismatch");
  static_assert((BM * 8) % NTHR == 0 && (BN * 8) % NTHR == 0, "chunk mismatch");
  static_assert(MODE != GEMM_SWIGLU || FN % 2 == 0, "SwiGLU needs gate and up fragments");

  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WARPS_M, wn = wave / WARPS_M;

  // ---------------- logical tile of this block
  const int n_tiles_n = (args.N + BN_OUT - 1) / BN_OUT;
  const int per_m = n_tiles_n * args.splitk;
  int total = 0;
  if (args.offsets) {
    for (int e = 0; e < args.n_groups; ++e)
      if ((args.group_mask >> e) & 1ull) {
        int cnt = args.offsets[e + 1] - args.offsets[e];
        total += ((cnt + BM - 1) / BM) * per_m;
      }
  } else {
    total = ((args.single_rows + BM - 1) / BM) * per_m;
  }
  const int chunk = (total + 7) >> 3;
  const int slot_in_xcd = (int)blockIdx.x >> 3;
  int l = ((int)blockIdx.x & 7) * chunk + slot_in_xcd;
  if (slot_in_xcd >= chunk || l >= total) return;

  int grp = 0, row0 = args.single_row0, cnt = args.single_rows;
  if (args.offsets) {
    for (int e = 0; e < args.n_groups; ++e) {
      if (!((args.group_mask >> e) & 1ull)) continue;
      int o = args.offsets[e], c = args.offsets[e + 1] - o;
      int tiles = ((c + BM - 1) / BM) * per_m;
      if (l < tiles) { grp = e; row0 = o; cnt = c; break; }
      l -= tiles;
    }
  }
  const int mt = (cnt + BM - 1) / BM;
  const int m_idx = l % mt;
  const int rest = l / mt;
  const int ks = rest % args.splitk;
  const int n_idx = rest / args.splitk;
  int rpt = (((cnt + mt - 1) / mt) + 31) & ~31;   // balanced tile height
  if (rpt > BM) rpt = BM;
  const int tile_row0 = m_idx * rpt;
  const int rows_valid = min(rpt, cnt - tile_row0);
  if (rows_valid <= 0) return;
  const int n0 = n_idx * BN_OUT;

  const char *wptr = args.wbase + (long long)args.slot[grp] * args.wstride;
  const uint16_t *B0 = reinterpret_cast<const uint16_t *>(wptr + args.b0_off);
  const uint16_t *B1 = reinterpret_cast<const uint16_t *>(wptr + args.b1_off);

  // K range of this slice (in BK steps)
  const int kt_total = (args.K + BK - 1) / BK;
  const int kt_begin = (int)((long long)kt_total * ks / args.splitk);
  const int kt_end = (int)((long long)kt_total * (ks + 1) / args.splitk);

  // ---------------- per-thread global sources and LDS destinations
  const uint16_t *a_src[CA];
  int a_dst[CA];
#pragma unroll
  for (int i = 0; i < CA; ++i) {
    int c = tid + i * NTHR, r = c >> 3, kc = c & 7;
    int rr = r < rows_valid ? r : 0;
    int p = row0 + tile_row0 + rr;
    long long srow = args.perm ? (long long)(args.perm[p] / args.k_top) : (long long)p;
    a_src[i] = args.A + srow * args.lda + kc * 8;
    a_dst[i] = swz(r, kc);
  }
  const uint16_t *b_src[CB];
  int b_dst[CB];
#pragma unroll
  for (int i = 0; i < CB; ++i) {
    int c = tid + i * NTHR, r = c >> 3, kc = c & 7;
    const uint16_t *base = B0;
    int rr = r;
    if (MODE == GEMM_SWIGLU && r >= BN / 2) { base = B1; rr = r - BN / 2; }
    int n = n0 + rr;
    if (n >= args.N) n = args.N - 1;
    b_src[i] = base + (long long)n * args.ldb + kc * 8;
    b_dst[i] = BM * ROW_BYTES + swz(r, kc);
  }
  const int kc_lane = tid & 7;  // this thread's 16-byte column inside the 64-wide K step

  // fragments of this wave that hold valid rows (interleaved ownership keeps them balanced)
  int fm_valid = 0;
#pragma unroll
  for (int i = 0; i < FM; ++i) fm_valid += ((i * WARPS_M + wm) * 32 < rows_valid) ? 1 : 0;

  floatx16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  uint4 ra[CA], rb[CB];
  auto load_global = [&](int kt) {
    const int k0 = kt * BK;
    const bool k_ok = k0 + kc_lane * 8 < args.K;
#pragma unroll
    for (int i = 0; i < CA; ++i)
      ra[i] = k_ok ? *reinterpret_cast<const uint4 *>(a_src[i] + k0) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < CB; ++i)
      rb[i] = k_ok ? *reinterpret_cast<const uint4 *>(b_src[i] + k0) : make_uint4(0, 0, 0, 0);
  };
  auto store_lds = [&](int stage) {
    unsigned char *s = smem + stage * STAGE;
#pragma unroll
    for (int i = 0; i < CA; ++i) *reinterpret_cast<uint4 *>(s + a_dst[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < CB; ++i) *reinterpret_cast<uint4 *>(s + b_dst[i]) = rb[i];
  };

  // LDS read offsets of this lane's fragment rows
  int a_off[FM], b_off[FN];
  const int lrow = lane & 31, lk = lane >> 5;
#pragma unroll
  for (int i = 0; i < FM; ++i) a_off[i] = (i * WARPS_M + wm) * 32 + lrow;
#pragma unroll
  for (int j = 0; j < FN; ++j) {
    if (MODE == GEMM_SWIGLU)
      b_off[j] = (j / FNH) * (BN / 2) + ((j % FNH) * WARPS_N + wn) * 32 + lrow;  // gate half | up half
    else
      b_off[j] = (j * WARPS_N + wn) * 32 + lrow;
  }

  if (kt_begin < kt_end) {
    load_global(kt_begin);
    store_lds(0);
  }
  __syncthreads();

  for (int kt = kt_begin; kt < kt_end; ++kt) {
    const int stage = (kt - kt_begin) & 1;
    if (kt + 1 < kt_end) load_global(kt + 1);
    const unsigned char *sa = smem + stage * STAGE;
    const unsigned char *sb = sa + BM * ROW_BYTES;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 af[FM], bfr[FN];
      const int kc = kk * 2 + lk;
#pragma unroll
      for (int i = 0; i < FM; ++i)
        if (i < fm_valid) af[i] = *reinterpret_cast<const bf16x8 *>(sa + swz(a_off[i], kc));
#pragma unroll
      for (int j = 0; j < FN; ++j) bfr[j] = *reinterpret_cast<const bf16x8 *>(sb + swz(b_off[j], kc));
#pragma unroll
      for (int i = 0; i < FM; ++i)
        if (i < fm_valid) {
#pragma unroll
          for (int j = 0; j < FN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
    }
    if (kt + 1 < kt_end) store_lds(stage ^ 1);
    __syncthreads();
  }

  // ---------------- epilogue.  C fragment layout of the 32x32 MFMA: lane holds column
  // (lane % 32) and rows 8*(r/4) + 4*(lane/32) + r%4 for its 16 registers r.
  const long long out_row_base = (long long)row0 + tile_row0;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    if (i >= fm_valid) continue;
    const int frow = (i * WARPS_M + wm) * 32;
#pragma unroll
    for (int j = 0; j < FNH; ++j) {
      const int col = n0 + (j * WARPS_N + wn) * 32 + lrow;
      if (col >= args.N) continue;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = frow + 8 * (r >> 2) + 4 * lk + (r & 3);
        if (row >= rows_valid) continue;
        const long long o = (out_row_base + row) * args.ldo + col;
        if (MODE == GEMM_SWIGLU) {
          float h = silu(acc[i][j][r]) * acc[i][j + FNH][r];
          reinterpret_cast<uint16_t *>(args.out)[o] = f32_to_bf16(h);
        } else if (MODE == GEMM_PLAIN_F32) {
          reinterpret_cast<float *>(args.out)[(long long)ks * args.out_split_stride + o] = acc[i][j][r];
        } else {
          reinterpret_cast<uint16_t *>(args.out)[o] = f32_to_bf16(acc[i][j][r]);
        }
      }
    }
  }
}

template <int BM, int BN, int WARPS_M, int WARPS_N, int MODE>
hipError_t launch_cfg(const GemmArgs &args, int max_rows, int n_groups_in_mask, hipStream_t stream) {
  constexpr int BN_OUT = (MODE == GEMM_SWIGLU) ? BN / 2 : BN;
  constexpr int NTHR = 64 * WARPS_M * WARPS_N;
  constexpr size_t smem = 2 * (size_t)(BM + BN) * ROW_BYTES;
  auto kern = grouped_gemm_kernel<BM, BN, WARPS_M, WARPS_N, MODE>;
  static bool attr_set = false;  // per instantiation; idempotent if two threads race
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const long long n_tiles_n = (args.N + BN_OUT - 1) / BN_OUT;
  const long long m_tiles_ub = (long long)max_rows / BM + n_groups_in_mask;
  long long ub = m_tiles_ub * n_tiles_n * args.splitk;
  if (ub <= 0) return hipSuccess;
  ub = (ub + 7) / 8 * 8;
  if (ub > 0x7FFFFFFFll) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, dim3((unsigned)ub), dim3(NTHR), smem, stream, args);
  return hipGetLastError();
}

}  // namespace

// Tile shapes.  Variant 0 picks by shape; 1.. force one (tuning hook).
static int g_variant[3] = {0, 0, 0};

void set_gemm_variant(int mode, int variant) {
  if (mode >= 0 && mode < 3) g_variant[mode] = variant;
}

template <int MODE>
static hipError_t launch_mode(const GemmArgs &args, int max_rows, int n_groups_in_mask, hipStream_t stream) {
  int v = g_variant[MODE];
  if (v == 0) v = 1;
  switch (v) {
    case 2: return launch_cfg<256, 256, 2, 2, MODE>(args, max_rows, n_groups_in_mask, stream);
    case 3: return launch_cfg<256, 256, 4, 2, MODE>(args, max_rows, n_groups_in_mask, stream);
    case 4: return launch_cfg<128, 256, 2, 2, MODE>(args, max_rows, n_groups_in_mask, stream);
    case 5: return launch_cfg<256, 128, 2, 2, MODE>(args, max_rows, n_groups_in_mask, stream);
    case 6: return launch_cfg<128, 256, 2, 4, MODE>(args, max_rows, n_groups_in_mask, stream);
    default: return launch_cfg<128, 128, 2, 2, MODE>(args, max_rows, n_groups_in_mask, stream);
  }
}

hipError_t launch_grouped_gemm(GemmMode mode, const GemmArgs &args, int max_rows, int n_groups_in_mask,
                               hipStream_t stream) {
  switch (mode) {
    case GEMM_SWIGLU: return launch_mode<GEMM_SWIGLU>(args, max_rows, n_groups_in_mask, stream);
    case GEMM_PLAIN_F32: return launch_mode<GEMM_PLAIN_F32>(args, max_rows, n_groups_in_mask, stream);
    default: return launch_mode<GEMM_PLAIN_BF16>(args, max_rows, n_groups_in_mask, stream);
  }
}

}  // namespace moe
