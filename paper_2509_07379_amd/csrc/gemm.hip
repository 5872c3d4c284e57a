// Grouped expert GEMM on bf16 MFMA (gfx950), the batch-per-expert operation of the prefill
// stage (Section V-B of the paper): each expert multiplies the rows routed to it by its own
// weights, read from its GPU-expert-cache slot.
//
//   GEMM_SWIGLU     H[p, n]  = bf16( silu(X_p . Wg[n]) * (X_p . Wu[n]) )   A rows gathered by perm
//   GEMM_PLAIN_F32  Y[p, c]  = H_p . Wd[c]   (fp32, one plane per K slice)
//   GEMM_PLAIN_BF16 C = A . B^T (bf16; dense stand-in for the non-MoE block)
//
// Both operands are K-contiguous ("NT"), so every lane feeds the MFMA with 8 consecutive
// bf16 of a row (one 16-byte LDS read).  Tiles are BM x BN x 64 in a two-stage LDS ring with
// a 16-byte XOR swizzle.  The main kernel fills the ring with direct global->LDS loads
// (global_load_lds_dwordx4: no VGPR staging, no ds_write), issued right after the barrier so
// that the loads of K step i+1 fly while the MFMAs of step i run; fragment reads of the next
// 16-wide K slice are issued before the MFMAs of the current one.  A register-staged kernel
// with zero fill covers K that is not a multiple of 64.
//
// Ragged groups: a group of `cnt` rows is cut into ceil(cnt/BM) M-tiles of equal height
// (rounded up to 32), each wave owns every WARPS_M-th 32-row fragment, and fragments past
// the tile's last row are skipped, so a nearly empty tail tile costs a fraction of a full one
// and the skipping stays balanced over the waves.
//
// Launch: 1-D grid; hardware block b runs logical tile (b % 8) * chunk + b / 8 so that the
// blocks one XCD receives (every 8th) are consecutive logical tiles - the M-tiles sharing a
// weight tile hit the same L2.
#include <type_traits>

#include "device_utils.h"
#include "kernels.h"
#include "gemm_plan.h"

namespace moe {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64;           // K elements per stage (128 bytes per row)
constexpr int ROW_BYTES = BK * 2;

// 16-byte chunk kc of a 128-byte tile row lands at chunk kc ^ ((row >> 1) & 7): the LDS has 64 banks
// (256 bytes per cycle), so the 16 rows that one b128 read phase touches (two rows per 256-byte
// line) must spread over all 16 chunk positions.
__device__ __forceinline__ int swz(int row, int kc) { return row * ROW_BYTES + ((kc ^ ((row >> 1) & 7)) << 4); }


// ---------------------------------------------------------------------------------------------
// Tile decode shared by both kernels.
struct TileInfo {
  int grp, row0, tile_row0, rows_valid, n0, ks;
  int ns;   // K slices of this tile (persistent kernel; the others use args.splitk)
};

template <int BM, int BN_OUT>
__device__ __forceinline__ bool decode_tile(const GemmArgs &args, TileInfo &t) {
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
  if (slot_in_xcd >= chunk || l >= total) return false;

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
  t.ks = rest % args.splitk;
  const int n_idx = rest / args.splitk;
  int rpt = (((cnt + mt - 1) / mt) + 31) & ~31;   // balanced tile height
  if (rpt > BM) rpt = BM;
  t.grp = grp;
  t.row0 = row0;
  t.tile_row0 = m_idx * rpt;
  t.rows_valid = min(rpt, cnt - t.tile_row0);
  t.n0 = n_idx * BN_OUT;
  return t.rows_valid > 0;
}

// Work items of the persistent kernel.  A group of cnt rows is cnt / BM full row tiles and, if rows are
// left over, one remainder tile (instead of tiles of equal height: a row tile's cost is its weight
// traffic plus its MFMAs, so two full tiles and a short one are cheaper than three of medium height).
// A full tile is cut into s_f K slices, a remainder tile into s_r; an item is (row tile, column tile,
// K slice).  Inside a group the row tiles are numbered in panels of 8 (the remainder tile is the last
// row tile): inside a panel the row tile runs fastest, then the column tile, then the K slice, so the
// blocks of an XCD that work side by side are on one K slice: they share each operand tile through
// their L2 and walk the same K range at the same time (with the K slice ahead of the column tile the
// 32 blocks of an XCD spread over all slices and re-read the rows of A once per five column tiles:
// Mixtral shape, down GEMM 483 -> 469 us).
// (args.equal_heights: the other way to cut a group, ceil(cnt / BM) tiles of equal height rounded up to 32
// rows, all of them "full" tiles as far as the numbering goes.  Equal tiles keep the blocks of an XCD in
// step with each other, which the down projection, whose both operands stream from HBM, needs more
// than it needs the cheaper cut.)
template <int BM, int BN_OUT>
__device__ __forceinline__ int group_items(const GemmArgs &args, int cnt, int s_f, int s_r) {
  const int ntn = (args.N + BN_OUT - 1) / BN_OUT;
  if (args.equal_heights) return ntn * ((cnt + BM - 1) / BM) * s_f;
  return ntn * ((cnt / BM) * s_f + ((cnt % BM) ? s_r : 0));
}

template <int BM, int BN_OUT>
__device__ __forceinline__ int count_items(const GemmArgs &args, int s_f, int s_r) {
  if (!args.offsets) return group_items<BM, BN_OUT>(args, args.single_rows, s_f, s_r);
  int total = 0;
  for (int e = 0; e < args.n_groups; ++e)
    if ((args.group_mask >> e) & 1ull)
      total += group_items<BM, BN_OUT>(args, args.offsets[e + 1] - args.offsets[e], s_f, s_r);
  return total;
}

// Item l of the launch.  plan != NULL: the first item of every group is in plan->item_begin (lane j
// looks at group j, one ballot finds l's group); otherwise the groups are walked.
template <int BM, int BN_OUT>
__device__ __forceinline__ void decode_item(const GemmArgs &args, const GemmPlan *plan, int s_f, int s_r, int lane,
                                            int l, TileInfo &t) {
  const int ntn = (args.N + BN_OUT - 1) / BN_OUT;
  int grp = 0, row0 = args.single_row0, cnt = args.single_rows;
  if (args.offsets) {
    if (plan) {
      const int end_j = plan->item_begin[min(lane + 1, kMaxExperts)];
      grp = __builtin_amdgcn_readfirstlane(__popcll(__ballot(lane < args.n_groups && end_j <= l)));
      l -= plan->item_begin[grp];
      row0 = args.offsets[grp];
      cnt = args.offsets[grp + 1] - row0;
    } else {
      for (int e = 0; e < args.n_groups; ++e) {
        if (!((args.group_mask >> e) & 1ull)) continue;
        const int o = args.offsets[e], c = args.offsets[e + 1] - o;
        const int items = group_items<BM, BN_OUT>(args, c, s_f, s_r);
        if (l < items) { grp = e; row0 = o; cnt = c; break; }
        l -= items;
      }
    }
  }
  constexpr int PANEL = 8;
  const int mf = args.equal_heights ? (cnt + BM - 1) / BM : cnt / BM;
  const int hr = args.equal_heights ? 0 : ((cnt % BM) ? 1 : 0);
  int height = BM;
  if (args.equal_heights && mf > 0) height = min(BM, (((cnt + mf - 1) / mf) + 31) & ~31);
  const int ipp = PANEL * s_f * ntn;              // items of a panel of 8 full tiles
  const int panel = min(l / ipp, mf / PANEL);
  l -= panel * ipp;
  const int pf = min(PANEL, mf - panel * PANEL);  // full tiles of this panel
  const int pr = (panel == mf / PANEL) ? hr : 0;  // ... and the remainder tile, in the group's last panel
  // inside the panel: row tile fastest, then the column tile, then the K slice (s_f == s_r whenever a
  // remainder tile shares a panel with full tiles: every tile of a launch has the same K slices)
  const int here = pf + pr;                       // row tiles of this panel, > 0 for every valid item
  const int ks = l / (here * ntn);
  const int rr = l - ks * here * ntn;
  const int n_idx = rr / here;
  const int r = rr - n_idx * here;
  const bool is_rem = r >= pf;
  const int m_idx = panel * PANEL + (is_rem ? pf : r);
  // (everything here is the same for all lanes: say so, so that it lives in scalar registers)
  t.grp = __builtin_amdgcn_readfirstlane(grp);
  t.row0 = __builtin_amdgcn_readfirstlane(row0);
  t.tile_row0 = __builtin_amdgcn_readfirstlane(m_idx * height);
  t.rows_valid = __builtin_amdgcn_readfirstlane(min(height, cnt - m_idx * height));
  t.n0 = __builtin_amdgcn_readfirstlane(n_idx * BN_OUT);
  t.ks = __builtin_amdgcn_readfirstlane(ks);
  t.ns = __builtin_amdgcn_readfirstlane(is_rem ? s_r : s_f);
}

// A value the optimiser cannot trace back: what is computed from it inside a loop stays inside.
__device__ __forceinline__ int opaque(int x) {
  asm volatile("" : "+v"(x));
  return x;
}

// fp32 -> bf16 by the hardware conversion (round to nearest even).
__device__ __forceinline__ uint16_t cvt_bf16(float f) {
  return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f));
}

template <int MODE>
__device__ __forceinline__ void store_value(char *ptr, float v, float v_up) {
  if (MODE == GEMM_SWIGLU)
    *reinterpret_cast<uint16_t *>(ptr) = cvt_bf16(silu(v) * v_up);
  else if (MODE == GEMM_PLAIN_F32)
    *reinterpret_cast<float *>(ptr) = v;
  else
    *reinterpret_cast<uint16_t *>(ptr) = cvt_bf16(v);
}

// Epilogue.  C fragment layout of the 32x32 MFMA: lane holds column (lane % 32) and rows
// 8*(r/4) + 4*(lane/32) + r%4 for its 16 registers r.  Per fragment the address is a wave-uniform
// base plus one per-lane offset that is the same for every store of the kernel, and a fragment
// that lies completely inside the tile and the matrix is stored without per-lane tests.
template <int MODE, int FM, int FN, int WARPS_M, int WARPS_N>
__device__ __forceinline__ void store_tile(const GemmArgs &args, const TileInfo &t, int wm, int wn, int lane,
                                           int fm_valid, floatx16 (&acc)[FM][FN], int i_begin = 0,
                                           int i_end = FM) {
  constexpr int FNH = (MODE == GEMM_SWIGLU) ? FN / 2 : FN;
  constexpr int ESIZE = (MODE == GEMM_PLAIN_F32) ? 4 : 2;
  lane = opaque(lane);   // the per-lane values below are re-derived per call instead of being kept alive
  const int lrow = lane & 31, lk = lane >> 5;
  const uint32_t lane_off = (uint32_t)((4 * lk) * args.ldo + lrow) * ESIZE;   // bytes
  char *plane = reinterpret_cast<char *>(args.out) +
                (MODE == GEMM_PLAIN_F32 ? (long long)t.ks * args.out_split_stride * ESIZE : 0ll);
  const long long out_row_base = (long long)t.row0 + t.tile_row0;
  const long long row_step = (long long)args.ldo * ESIZE;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    if (i < i_begin || i >= i_end || i >= fm_valid) continue;
    const int frow = (i * WARPS_M + wm) * 32;   // uniform
#pragma unroll
    for (int j = 0; j < FNH; ++j) {
      const int col0 = t.n0 + (j * WARPS_N + wn) * 32;   // uniform
      if (col0 >= args.N) continue;
      char *sp = plane + ((out_row_base + frow) * args.ldo + col0) * ESIZE;   // uniform, walks down the rows
      const bool full = frow + 32 <= t.rows_valid && col0 + 32 <= args.N;
      if (full) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          store_value<MODE>(sp + lane_off, acc[i][j][r], acc[i][(MODE == GEMM_SWIGLU) ? j + FNH : j][r]);
          sp += ((r & 3) == 3 ? 5ll : 1ll) * row_step;   // rows 0..3, 8..11, 16..19, 24..27
        }
      } else {
        const bool col_ok = col0 + lrow < args.N;
        const int rows_left = t.rows_valid - frow - 4 * lk;   // the lane's row 8*(r/4) + r%4 must be below
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          if (col_ok && 8 * (r >> 2) + (r & 3) < rows_left)
            store_value<MODE>(sp + lane_off, acc[i][j][r], acc[i][(MODE == GEMM_SWIGLU) ? j + FNH : j][r]);
          sp += ((r & 3) == 3 ? 5ll : 1ll) * row_step;
        }
      }
    }
  }
}

// Epilogue for accumulators of transposed fragments (MFMA called with the B fragment as first
// operand): lane holds output row (lane % 32) and the columns 8*(r/4) + 4*(lane/32) + r%4 of the
// fragment, i.e. four groups of four consecutive columns, so a fragment leaves in four stores of
// 8 (bf16) or 16 (fp32) bytes per lane that share one address and differ in the immediate offset.
//
// With a wave-private 4 KB LDS buffer (xp) a full fragment is first turned round in LDS: it is written
// as 32 rows of 64 (bf16) or 128 (fp32) bytes and read back so that 4 or 8 neighbouring lanes hold one
// whole row segment.  A store instruction then covers 16 or 8 rows with contiguous 64 / 128 bytes each
// instead of 32 rows with 16 / 32 bytes each; the memory pipeline takes about one cycle per cache
// line an instruction touches, and the epilogue is bound by exactly that.  16-byte pieces of a row are
// XOR-swizzled against the row number (at most 2-way bank conflicts on the 8-byte writes).
template <int MODE, int FM, int FN, int WARPS_M, int WARPS_N>
__device__ __forceinline__ void store_tile_cols(const GemmArgs &args, const TileInfo &t, int wm, int wn, int lane,
                                                int fm_valid, floatx16 (&acc)[FM][FN], int i_begin, int i_end,
                                                unsigned char *xp = nullptr) {
  constexpr int FNH = (MODE == GEMM_SWIGLU) ? FN / 2 : FN;
  constexpr int ESIZE = (MODE == GEMM_PLAIN_F32) ? 4 : 2;
  constexpr int PPR = 2 * ESIZE;          // 16-byte pieces per fragment row: 4 (bf16) or 8 (fp32)
  constexpr int RPP = 64 / PPR;           // rows per store instruction: 16 or 8
  lane = opaque(lane);   // the per-lane values below are re-derived per call instead of being kept alive
  const int lrow = lane & 31, lk = lane >> 5;
  const uint32_t lane_off = (uint32_t)(lrow * args.ldo + 4 * lk) * ESIZE;   // bytes
  // turned-round layout: this lane's row and piece of a pass, as LDS and as global byte offsets
  const int xrow = lane / PPR, xq = lane % PPR;
  const uint32_t xlane_off = (uint32_t)(xrow * args.ldo) * ESIZE + xq * 16;
  char *plane = reinterpret_cast<char *>(args.out) +
                (MODE == GEMM_PLAIN_F32 ? (long long)t.ks * args.out_split_stride * ESIZE : 0ll);
  const long long out_row_base = (long long)t.row0 + t.tile_row0;
  const bool aligned = (args.ldo * ESIZE) % 16 == 0 && (reinterpret_cast<uintptr_t>(args.out) & 15) == 0 &&
                       (MODE != GEMM_PLAIN_F32 || (args.out_split_stride * ESIZE) % 16 == 0);
  const long long row_bytes = (long long)args.ldo * ESIZE;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    if (i < i_begin || i >= i_end || i >= fm_valid) continue;
    const int frow = (i * WARPS_M + wm) * 32;   // uniform
#pragma unroll
    for (int j = 0; j < FNH; ++j) {
      const int col0 = t.n0 + (j * WARPS_N + wn) * 32;   // uniform
      if (col0 >= args.N) continue;
      char *sp = plane + ((out_row_base + frow) * args.ldo + col0) * ESIZE;   // uniform
      float v[16];
#pragma unroll
      for (int r = 0; r < 16; ++r)
        v[r] = (MODE == GEMM_SWIGLU) ? silu(acc[i][j][r]) * acc[i][j + FNH][r] : acc[i][j][r];
      const bool full = frow + 32 <= t.rows_valid && col0 + 32 <= args.N && aligned;
      if (full && xp) {
        // row pitch 16 * PPR bytes; piece index XORed with (row >> 1) & 7 (fp32: 8 pieces, two rows per
        // 64 banks) or (row >> 2) & 3 (bf16: 4 pieces, four rows per 64 banks)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          if (MODE == GEMM_PLAIN_F32) {
            f32x4 o = {v[4 * g], v[4 * g + 1], v[4 * g + 2], v[4 * g + 3]};
            *reinterpret_cast<f32x4 *>(xp + lrow * 128 + (((2 * g + lk) ^ ((lrow >> 1) & 7)) << 4)) = o;
          } else {
            u32x2 o;
            o.x = (uint32_t)cvt_bf16(v[4 * g]) | ((uint32_t)cvt_bf16(v[4 * g + 1]) << 16);
            o.y = (uint32_t)cvt_bf16(v[4 * g + 2]) | ((uint32_t)cvt_bf16(v[4 * g + 3]) << 16);
            *reinterpret_cast<u32x2 *>(xp + lrow * 64 + ((g ^ ((lrow >> 2) & 3)) << 4) + lk * 8) = o;
          }
        }
#pragma unroll
        for (int pass = 0; pass < 32 / RPP; ++pass) {
          const int row = pass * RPP + xrow;
          const int sw = (MODE == GEMM_PLAIN_F32) ? ((row >> 1) & 7) : ((row >> 2) & 3);
          const f32x4 o = *reinterpret_cast<const f32x4 *>(xp + row * (16 * PPR) + ((xq ^ sw) << 4));
          *reinterpret_cast<f32x4 *>(sp + (long long)pass * RPP * row_bytes + xlane_off) = o;
        }
      } else if (full) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          char *ptr = sp + lane_off + g * 8 * ESIZE;
          // plain (cached) stores: streaming stores were several times slower here
          if (MODE == GEMM_PLAIN_F32) {
            f32x4 o = {v[4 * g], v[4 * g + 1], v[4 * g + 2], v[4 * g + 3]};
            *reinterpret_cast<f32x4 *>(ptr) = o;
          } else {
            u32x2 o;
            o.x = (uint32_t)cvt_bf16(v[4 * g]) | ((uint32_t)cvt_bf16(v[4 * g + 1]) << 16);
            o.y = (uint32_t)cvt_bf16(v[4 * g + 2]) | ((uint32_t)cvt_bf16(v[4 * g + 3]) << 16);
            *reinterpret_cast<u32x2 *>(ptr) = o;
          }
        }
      } else if (frow + lrow < t.rows_valid) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int c = 8 * (r >> 2) + 4 * lk + (r & 3);
          if (col0 + c >= args.N) continue;
          char *ptr = sp + ((long long)lrow * args.ldo + c) * ESIZE;
          if (MODE == GEMM_PLAIN_F32)
            *reinterpret_cast<float *>(ptr) = v[r];
          else
            *reinterpret_cast<uint16_t *>(ptr) = cvt_bf16(v[r]);
        }
      }
    }
  }
}

typedef __attribute__((address_space(3))) void *lds_ptr_t;
typedef __attribute__((address_space(1))) const void *glb_ptr_t;

// ---------------------------------------------------------------------------------------------
// Main kernel: direct global->LDS loads.  Needs K % 64 == 0.
template <int BM, int BN, int WARPS_M, int WARPS_N, int MODE>
__global__ __launch_bounds__(64 * WARPS_M * WARPS_N) void grouped_gemm_dma_kernel(const GemmArgs args) {
  constexpr int NW = WARPS_M * WARPS_N;
  constexpr int BN_OUT = (MODE == GEMM_SWIGLU) ? BN / 2 : BN;
  constexpr int FM = BM / (32 * WARPS_M);
  constexpr int FN = BN / (32 * WARPS_N);
  constexpr int FNH = (MODE == GEMM_SWIGLU) ? FN / 2 : FN;
  constexpr int STAGE = (BM + BN) * ROW_BYTES;
  constexpr int GROUPS = (BM + BN) / 8;   // 8 tile rows = 1 KB = one wave-wide 16-byte load
  constexpr int GPW = GROUPS / NW;        // loads per wave per stage
  static_assert(BM % (32 * WARPS_M) == 0 && BN % (32 * WARPS_N) == 0, "tile/wave mismatch");
  static_assert(GROUPS % NW == 0, "load split mismatch");
  static_assert(MODE != GEMM_SWIGLU || FN % 2 == 0, "SwiGLU needs gate and up fragments");
  static_assert(FM <= 4, "fragment-count dispatch covers up to 4 row fragments per wave");

  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: stays in scalar registers
  const int wm = wave % WARPS_M, wn = wave / WARPS_M;

  TileInfo t;
  if (!decode_tile<BM, BN_OUT>(args, t)) return;

  const char *wptr = args.wbase + (long long)args.slot[t.grp] * args.wstride;
  const uint16_t *B0 = reinterpret_cast<const uint16_t *>(wptr + args.b0_off);
  const uint16_t *B1 = reinterpret_cast<const uint16_t *>(wptr + args.b1_off);
  const int kt_total = args.K / BK;
  const int kt_begin = (int)((long long)kt_total * t.ks / args.splitk);
  const int kt_end = (int)((long long)kt_total * (t.ks + 1) / args.splitk);

  // This lane's source of each of the wave's loads.  Load g fills tile rows 8g..8g+7 (A rows first,
  // then B rows); lane l lands at row 8g + l/8, chunk position l%8, so it fetches the chunk that the
  // swizzle maps there.
  const uint16_t *src[GPW];
#pragma unroll
  for (int i = 0; i < GPW; ++i) {
    const int g = i * NW + wave;
    const int row = g * 8 + (lane >> 3);
    const int kc = (lane & 7) ^ ((row >> 1) & 7);
    if (g * 8 < BM) {
      int rr = row < t.rows_valid ? row : 0;
      int p = t.row0 + t.tile_row0 + rr;
      long long srow = args.perm ? (long long)(args.perm[p] / args.k_top) : (long long)p;
      src[i] = args.A + srow * args.lda + kc * 8;
    } else {
      int r = row - BM;
      const uint16_t *base = B0;
      if (MODE == GEMM_SWIGLU && r >= BN / 2) { base = B1; r -= BN / 2; }
      int n = t.n0 + r;
      if (n >= args.N) n = args.N - 1;
      src[i] = base + (long long)n * args.ldb + kc * 8;
    }
  }

  int fm_valid = 0;
#pragma unroll
  for (int i = 0; i < FM; ++i) fm_valid += ((i * WARPS_M + wm) * 32 < t.rows_valid) ? 1 : 0;

  floatx16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

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

#define MOE_ISSUE(kt_, stage_)                                                                       \
  do {                                                                                               \
    _Pragma("unroll") for (int i_ = 0; i_ < GPW; ++i_)                                               \
      __builtin_amdgcn_global_load_lds((glb_ptr_t)(src[i_] + (long long)(kt_) * BK),                 \
                                       (lds_ptr_t)(smem + (stage_) * STAGE + (i_ * NW + wave) * 1024), \
                                       16, 0, 0);                                                    \
  } while (0)
#define MOE_READ_FRAGS(FMV, buf_, kk_)                                                               \
  do {                                                                                               \
    const int kc_ = (kk_) * 2 + lk;                                                                  \
    _Pragma("unroll") for (int i_ = 0; i_ < FMV; ++i_)                                               \
      af_[buf_][i_] = *reinterpret_cast<const bf16x8 *>(sa_ + swz(a_off[i_], kc_));                  \
    _Pragma("unroll") for (int j_ = 0; j_ < FN; ++j_)                                                \
      bf_[buf_][j_] = *reinterpret_cast<const bf16x8 *>(sb_ + swz(b_off[j_], kc_));                  \
  } while (0)
#define MOE_MMA_STAGE(FMV, stage_)                                                                   \
  do {                                                                                               \
    const unsigned char *sa_ = smem + (stage_) * STAGE;                                              \
    const unsigned char *sb_ = sa_ + BM * ROW_BYTES;                                                 \
    bf16x8 af_[2][FMV > 0 ? FMV : 1], bf_[2][FN];                                                    \
    if (FMV > 0) {                                                                                   \
      MOE_READ_FRAGS(FMV, 0, 0);                                                                     \
      _Pragma("unroll") for (int kk_ = 0; kk_ < BK / 16; ++kk_) {                                    \
        if (kk_ + 1 < BK / 16) MOE_READ_FRAGS(FMV, (kk_ + 1) & 1, kk_ + 1);                          \
        _Pragma("unroll") for (int i_ = 0; i_ < FMV; ++i_)                                           \
          _Pragma("unroll") for (int j_ = 0; j_ < FN; ++j_)                                          \
            acc[i_][j_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af_[kk_ & 1][i_], bf_[kk_ & 1][j_], \
                                                                  acc[i_][j_], 0, 0, 0);             \
      }                                                                                              \
    }                                                                                                \
  } while (0)
// One K step.  The loads of the next step go out first (the last step re-loads itself: harmless and
// branch-free, so the whole body is one scheduling region).  The group barriers then pin the
// software pipeline: fragments of 16-wide slice kk+1 are requested before the MFMAs of slice kk.
#define MOE_K_LOOP(FMV)                                                                              \
  do {                                                                                               \
    for (int kt = kt_begin; kt < kt_end; ++kt) {                                                     \
      const int stage_ = (kt - kt_begin) & 1;                                                        \
      const int kn_ = kt + 1 < kt_end ? kt + 1 : kt;                                                 \
      __builtin_amdgcn_s_waitcnt(0x0F70); /* vmcnt(0): this wave's loads of step kt have landed */   \
      __syncthreads();                    /* ... and everybody's; stage^1 is free again */          \
      MOE_ISSUE(kn_, stage_ ^ 1);                                                                    \
      MOE_MMA_STAGE(FMV, stage_);                                                                    \
      if (FMV > 0) {                                                                                 \
        __builtin_amdgcn_sched_group_barrier(0x020, GPW, 0);          /* global->LDS loads */        \
        __builtin_amdgcn_sched_group_barrier(0x100, FMV + FN, 0);     /* fragments of slice 0 */     \
        __builtin_amdgcn_sched_group_barrier(0x100, FMV + FN, 0);                                    \
        __builtin_amdgcn_sched_group_barrier(0x008, FMV * FN, 0);                                    \
        __builtin_amdgcn_sched_group_barrier(0x100, FMV + FN, 0);                                    \
        __builtin_amdgcn_sched_group_barrier(0x008, FMV * FN, 0);                                    \
        __builtin_amdgcn_sched_group_barrier(0x100, FMV + FN, 0);                                    \
        __builtin_amdgcn_sched_group_barrier(0x008, FMV * FN, 0);                                    \
        __builtin_amdgcn_sched_group_barrier(0x008, FMV * FN, 0);                                    \
      }                                                                                              \
    }                                                                                                \
  } while (0)

  if (kt_begin < kt_end) MOE_ISSUE(kt_begin, 0);
  switch (fm_valid) {
    case 0: MOE_K_LOOP(0); break;
    case 1: MOE_K_LOOP(1); break;
    case 2: if constexpr (FM >= 2) MOE_K_LOOP(2); break;
    case 3: if constexpr (FM >= 3) MOE_K_LOOP(3); break;
    default: if constexpr (FM >= 4) MOE_K_LOOP(4); break;
  }
#undef MOE_K_LOOP
#undef MOE_MMA_STAGE
#undef MOE_READ_FRAGS
#undef MOE_ISSUE

  store_tile<MODE, FM, FN, WARPS_M, WARPS_N>(args, t, wm, wn, lane, fm_valid, acc);
}

// ---------------------------------------------------------------------------------------------
// The same tile loop on quantised experts: the B operand is read from the expert's blob as it came over
// the host link.  Every lane fetches 16-byte pieces of the code tile into registers one K step ahead,
// expands them to bf16 weights and writes them into the swizzled LDS tile the MFMAs read; A keeps its
// direct global -> LDS loads.  The expansion is issued while the other waves' MFMAs run.
//   QF = 1 (MOE_FMT_E4M3_ROWS): e4m3 codes, one fp32 scale per B row, 64 bytes per row and K step.  The
//     weight is bf16_rne(value(code) * scale[row]) (the hardware's e4m3 -> fp32 conversion, one multiply,
//     the hardware's fp32 -> bf16 rounding), some 70 vector instructions per lane and K step.
//   QF = 2 (MOE_FMT_MXFP4): e2m1 codes, two per byte, one power-of-two scale byte per 32 codes: 32 bytes
//     of codes and 2 scale bytes per row and K step.  A lane's piece is one scale block; the hardware
//     conversion takes a byte of two codes and the scale and returns the exact bf16 pair.
// Either way the weights are the values the format defines, so the products are those of a GEMM on
// expanded weights.  Needs K % 64 == 0.
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
typedef float f32x2v __attribute__((ext_vector_type(2)));

__device__ __forceinline__ u32x4 expand8_e4m3(uint32_t c0, uint32_t c1, float scale) {
  f32x2v a = __builtin_amdgcn_cvt_pk_f32_fp8((int)c0, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)c0, true);
  f32x2v c = __builtin_amdgcn_cvt_pk_f32_fp8((int)c1, false), d = __builtin_amdgcn_cvt_pk_f32_fp8((int)c1, true);
  a *= scale; b *= scale; c *= scale; d *= scale;
  return u32x4{__builtin_bit_cast(uint32_t, __builtin_convertvector(a, bf16x2v)),
               __builtin_bit_cast(uint32_t, __builtin_convertvector(b, bf16x2v)),
               __builtin_bit_cast(uint32_t, __builtin_convertvector(c, bf16x2v)),
               __builtin_bit_cast(uint32_t, __builtin_convertvector(d, bf16x2v))};
}

__device__ __forceinline__ u32x4 expand8_mxfp4(uint32_t word, float scale) {
  typedef __bf16 pair_t __attribute__((ext_vector_type(2)));
  const pair_t p0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(word, scale, 0);
  const pair_t p1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(word, scale, 1);
  const pair_t p2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(word, scale, 2);
  const pair_t p3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(word, scale, 3);
  return u32x4{__builtin_bit_cast(uint32_t, p0), __builtin_bit_cast(uint32_t, p1), __builtin_bit_cast(uint32_t, p2),
               __builtin_bit_cast(uint32_t, p3)};
}

template <int BM, int BN, int WARPS_M, int WARPS_N, int MODE, int QF>
__global__ __launch_bounds__(64 * WARPS_M * WARPS_N) void grouped_gemm_q8_kernel(const GemmArgs args) {
  constexpr int NW = WARPS_M * WARPS_N;
  constexpr int BN_OUT = (MODE == GEMM_SWIGLU) ? BN / 2 : BN;
  constexpr int FM = BM / (32 * WARPS_M);
  constexpr int FN = BN / (32 * WARPS_N);
  constexpr int FNH = (MODE == GEMM_SWIGLU) ? FN / 2 : FN;
  constexpr int STAGE = (BM + BN) * ROW_BYTES;
  constexpr int GPA = BM / 8 / NW;    // wave-wide A loads per wave and stage (8 tile rows each)
  // 16-byte pieces of codes per lane and stage: a wave-wide load covers 16 B rows of e4m3 codes (4 lanes
  // per row) or 32 of MXFP4 codes (2 lanes per row); a piece expands to ND 16-byte chunks of the LDS row
  constexpr int RPL = QF == 2 ? 32 : 16, ND = QF == 2 ? 4 : 2, QSTEP = QF == 2 ? BK / 2 : BK;
  constexpr int NQ = BN / RPL / NW;
  static_assert(QF == 1 || QF == 2, "formats: 1 = e4m3 rows, 2 = MXFP4");
  static_assert(BM % (8 * NW) == 0 && BN % (RPL * NW) == 0, "load split mismatch");
  static_assert(FM <= 4, "fragment-count dispatch covers up to 4 row fragments per wave");

  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WARPS_M, wn = wave / WARPS_M;

  TileInfo t;
  if (!decode_tile<BM, BN_OUT>(args, t)) return;

  const char *qptr = args.qbase + (long long)args.slot[t.grp] * args.qstride;
  const int kt_total = args.K / BK;
  const int kt_begin = (int)((long long)kt_total * t.ks / args.splitk);
  const int kt_end = (int)((long long)kt_total * (t.ks + 1) / args.splitk);

  // A: load g fills tile rows 8g..8g+7; lane l lands at row 8g + l/8, chunk position l%8
  const uint16_t *a_src[GPA];
#pragma unroll
  for (int i = 0; i < GPA; ++i) {
    const int g = i * NW + wave;
    const int row = g * 8 + (lane >> 3);
    const int kc = (lane & 7) ^ ((row >> 1) & 7);
    const int rr = row < t.rows_valid ? row : 0;
    const int p = t.row0 + t.tile_row0 + rr;
    const long long srow = args.perm ? (long long)(args.perm[p] / args.k_top) : (long long)p;
    a_src[i] = args.A + srow * args.lda + kc * 8;
  }
  // B, e4m3: piece i of this lane is 16 codes of tile row 16 (i NW + wave) + l/4, columns 16 (l%4) .. +15 of
  // the K step; expanded they are the row's bf16 chunks 2 (l%4) and 2 (l%4) + 1.  MXFP4: 32 codes of tile row
  // 32 (i NW + wave) + l/2, columns 32 (l%2) .. +31, with the scale byte of that block; chunks 4 (l%2) .. +3.
  const uint8_t *q_src[NQ];
  const uint8_t *sc_src[NQ];   // MXFP4: this piece's scale byte in K step 0
  float q_scale[NQ];           // e4m3: the row's scale
  int q_dst[NQ][ND];
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    const int r = (i * NW + wave) * RPL + (QF == 2 ? lane >> 1 : lane >> 2);
    const int piece = QF == 2 ? lane & 1 : lane & 3;
    long long codes_off = args.q_b0_off, scale_off = args.q_s0_off;
    int rr = r;
    if (MODE == GEMM_SWIGLU && r >= BN / 2) { codes_off = args.q_b1_off; scale_off = args.q_s1_off; rr = r - BN / 2; }
    int n = t.n0 + rr;
    if (n >= args.N) n = args.N - 1;
    if constexpr (QF == 2) {
      q_src[i] = reinterpret_cast<const uint8_t *>(qptr + codes_off) + (long long)n * (args.K / 2) + piece * 16;
      sc_src[i] = reinterpret_cast<const uint8_t *>(qptr + scale_off) + (long long)n * (args.K / 32) + piece;
      q_scale[i] = 0.0f;
    } else {
      q_src[i] = reinterpret_cast<const uint8_t *>(qptr + codes_off) + (long long)n * args.K + piece * 16;
      sc_src[i] = nullptr;
      q_scale[i] = reinterpret_cast<const float *>(qptr + scale_off)[n];
    }
#pragma unroll
    for (int j = 0; j < ND; ++j) q_dst[i][j] = BM * ROW_BYTES + swz(r, ND * piece + j);
  }

  int fm_valid = 0;
#pragma unroll
  for (int i = 0; i < FM; ++i) fm_valid += ((i * WARPS_M + wm) * 32 < t.rows_valid) ? 1 : 0;

  floatx16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

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

  u32x4 cq[NQ];      // codes of the K step after the one in LDS
  uint32_t csc[NQ];  // MXFP4: and their scale bytes
#define MOE_Q_LOADA(kt_, stage_)                                                                     \
  do {                                                                                               \
    _Pragma("unroll") for (int i_ = 0; i_ < GPA; ++i_)                                               \
      __builtin_amdgcn_global_load_lds((glb_ptr_t)(a_src[i_] + (long long)(kt_) * BK),               \
                                       (lds_ptr_t)(smem + (stage_) * STAGE + (i_ * NW + wave) * 1024), \
                                       16, 0, 0);                                                    \
  } while (0)
#define MOE_Q_LOADQ(kt_)                                                                             \
  do {                                                                                               \
    _Pragma("unroll") for (int i_ = 0; i_ < NQ; ++i_) {                                              \
      cq[i_] = *reinterpret_cast<const u32x4 *>(q_src[i_] + (long long)(kt_) * QSTEP);               \
      if constexpr (QF == 2) csc[i_] = sc_src[i_][(long long)(kt_) * (BK / 32)];                     \
    }                                                                                                \
  } while (0)
#define MOE_Q_EXPAND(stage_)                                                                         \
  do {                                                                                               \
    _Pragma("unroll") for (int i_ = 0; i_ < NQ; ++i_) {                                              \
      const u32x4 c_ = cq[i_];                                                                       \
      unsigned char *st_ = smem + (stage_) * STAGE;                                                  \
      if constexpr (QF == 2) {                                                                       \
        const float f_ = __uint_as_float(csc[i_] << 23);                                             \
        *reinterpret_cast<u32x4 *>(st_ + q_dst[i_][0]) = expand8_mxfp4(c_.x, f_);                    \
        *reinterpret_cast<u32x4 *>(st_ + q_dst[i_][1]) = expand8_mxfp4(c_.y, f_);                    \
        *reinterpret_cast<u32x4 *>(st_ + q_dst[i_][ND - 2]) = expand8_mxfp4(c_.z, f_);               \
        *reinterpret_cast<u32x4 *>(st_ + q_dst[i_][ND - 1]) = expand8_mxfp4(c_.w, f_);               \
      } else {                                                                                       \
        *reinterpret_cast<u32x4 *>(st_ + q_dst[i_][0]) = expand8_e4m3(c_.x, c_.y, q_scale[i_]);      \
        *reinterpret_cast<u32x4 *>(st_ + q_dst[i_][1]) = expand8_e4m3(c_.z, c_.w, q_scale[i_]);      \
      }                                                                                              \
    }                                                                                                \
  } while (0)
#define MOE_Q_MMA(FMV, stage_)                                                                       \
  do {                                                                                               \
    const unsigned char *sa_ = smem + (stage_) * STAGE;                                              \
    const unsigned char *sb_ = sa_ + BM * ROW_BYTES;                                                 \
    _Pragma("unroll") for (int kk_ = 0; kk_ < BK / 16; ++kk_) {                                      \
      const int kc_ = kk_ * 2 + lk;                                                                  \
      bf16x8 af_[FMV > 0 ? FMV : 1], bf_[FN];                                                        \
      _Pragma("unroll") for (int i_ = 0; i_ < FMV; ++i_)                                             \
        af_[i_] = *reinterpret_cast<const bf16x8 *>(sa_ + swz(a_off[i_], kc_));                      \
      _Pragma("unroll") for (int j_ = 0; j_ < FN; ++j_)                                              \
        bf_[j_] = *reinterpret_cast<const bf16x8 *>(sb_ + swz(b_off[j_], kc_));                      \
      _Pragma("unroll") for (int i_ = 0; i_ < FMV; ++i_)                                             \
        _Pragma("unroll") for (int j_ = 0; j_ < FN; ++j_)                                            \
          acc[i_][j_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af_[i_], bf_[j_], acc[i_][j_], 0, 0, 0); \
    }                                                                                                \
  } while (0)
// One K step: the A tile and the codes requested in the step before have arrived; after the barrier
// nobody reads the other stage any more, so the next step's A loads go out, the codes in registers
// become its B tile and the codes of the step after that are requested; then this step's MFMAs.
// (The last step requests and expands itself again: harmless, and the loop body stays branch-free.)
#define MOE_Q_LOOP(FMV)                                                                              \
  do {                                                                                               \
    for (int kt = kt_begin; kt < kt_end; ++kt) {                                                     \
      const int stage_ = (kt - kt_begin) & 1;                                                        \
      const int kn_ = kt + 1 < kt_end ? kt + 1 : kt;                                                 \
      const int kn2_ = kt + 2 < kt_end ? kt + 2 : kn_;                                               \
      __builtin_amdgcn_s_waitcnt(0x0F70); /* vmcnt(0): this wave's A loads of step kt have landed */ \
      __syncthreads();   /* ... and everybody's, with the B tile written in the step before */       \
      MOE_Q_LOADA(kn_, stage_ ^ 1);                                                                  \
      MOE_Q_EXPAND(stage_ ^ 1);                                                                      \
      MOE_Q_LOADQ(kn2_);                                                                             \
      MOE_Q_MMA(FMV, stage_);                                                                        \
    }                                                                                                \
  } while (0)

  if (kt_begin < kt_end) {
    MOE_Q_LOADA(kt_begin, 0);
    MOE_Q_LOADQ(kt_begin);
    MOE_Q_EXPAND(0);   // (waits for the codes)
    MOE_Q_LOADQ(kt_begin + 1 < kt_end ? kt_begin + 1 : kt_begin);
  }
  switch (fm_valid) {
    case 0: MOE_Q_LOOP(0); break;
    case 1: MOE_Q_LOOP(1); break;
    case 2: if constexpr (FM >= 2) MOE_Q_LOOP(2); break;
    case 3: if constexpr (FM >= 3) MOE_Q_LOOP(3); break;
    default: if constexpr (FM >= 4) MOE_Q_LOOP(4); break;
  }
#undef MOE_Q_LOOP
#undef MOE_Q_MMA
#undef MOE_Q_EXPAND
#undef MOE_Q_LOADQ
#undef MOE_Q_LOADA
  (void)STAGE;
  store_tile<MODE, FM, FN, WARPS_M, WARPS_N>(args, t, wm, wn, lane, fm_valid, acc);
}

// ---------------------------------------------------------------------------------------------
// Short row tiles of the persistent kernel: at most 64 rows, i.e. a small group or what a group leaves
// over after its full tiles.  Such a tile has almost no MFMA work; its time is the 256-row weight tile's
// way from memory through LDS, and as the only (or first) reader of those weights it waits for HBM,
// not for L2.  So it gets a pipeline of its own in the same LDS: four stages of 40 KB ([A 64 rows]
// [B 256 rows], the same 128-byte rows and swizzle), loads three K steps ahead, one barrier per K step,
// every wave both loading and multiplying (wave (wm, wn) owns rows 32 wm.. and the same two column
// fragments as in a full tile).  Rows past the tile's last one are never fetched.  The results leave
// without the LDS transposition (there is little to store).  On entry no load may be in flight and
// nobody may still use LDS; on exit the same holds.
constexpr int kSmallTileRows = 64;

// On quantised experts (QF = 1 e4m3 blobs, 2 MXFP4 blobs; layouts and conversions as in the persistent
// kernel) a stage is [A 64 rows][codes of 256 B rows (+ MXFP4 scale dwords)], 24 KB or 18 KB, so six or
// eight stages fit and the loads run five or seven K steps ahead (one stage fewer measured the same: at
// about 1 us per K step these tiles are bound by the step itself, not by the loads in flight).
template <int MODE, int QF>
__device__ __forceinline__ void pp_small_tile(const GemmArgs &args, const TileInfo &t, unsigned char *smem,
                                              int lane, int wave) {
  constexpr int BN = 256, SA = kSmallTileRows, WARPS_M = 2, WARPS_N = 4, FN = 2;
  constexpr int FNH = (MODE == GEMM_SWIGLU) ? FN / 2 : FN;
  constexpr int SAB = SA * ROW_BYTES;          // the A part of a stage
  constexpr int SQS = SAB + BN * 32;           // MXFP4: the scale dwords, behind the codes
  constexpr int SST = SAB + (QF == 2 ? BN * 32 + 2048 : QF == 1 ? BN * 64 : BN * ROW_BYTES);   // 18 / 24 / 40 KB
  constexpr int NST = QF == 2 ? 8 : QF == 1 ? 6 : 4;   // stages (144 / 144 / 160 KB)
  // B loads (wave-wide) per wave and stage: 4 of 8 rows x 128 bytes; e4m3 2 of 16 rows x 64 bytes of codes;
  // MXFP4 one of 32 rows x 32 bytes of codes and one of scale dwords
  constexpr int NLB = QF == 2 ? 2 : QF == 1 ? 2 : BN / 8 / 8;
  constexpr int NLC = QF == 2 ? 1 : QF == 1 ? 2 : 4;   // ... of which rows of weights or codes
  constexpr int LPS = NLB + 1;                 // loads per wave and stage, with the one of A
  static_assert(NST * SST <= 160 * 1024 && NST <= 8 && (NST - 2) * LPS < 64, "stages must fit LDS and the load counter");
  const int wm = wave >> 2, wn = wave & 3;
  const int kt_total = args.K / BK;
  const int kt_begin = (int)((long long)kt_total * t.ks / t.ns);
  const int nk = (int)((long long)kt_total * (t.ks + 1) / t.ns) - kt_begin;

  // This lane's sources.  A: row group `wave` (rows 8 wave .. 8 wave + 7); B (bf16): row groups wave + 8 i.
  // Lane l lands at row 8 g + l / 8, chunk position l % 8 and fetches the chunk the swizzle maps there;
  // g & 1 is wave & 1 for all of them.  B (e4m3): 16-row groups wave + 8 i.  B (MXFP4): the 32 rows 32 wave ..,
  // lane l the half (l / 16) % 2 of row 16 (l / 32) + l % 16 (see the persistent kernel).
  const int lane_s = opaque(lane);
  const int kc16 = ((lane_s & 7) ^ ((wave & 1) * 4 + (lane_s >> 4))) * 16;
  const int a_row = wave * 8 + (lane_s >> 3);
  const int p = t.row0 + t.tile_row0 + (a_row < t.rows_valid ? a_row : 0);
  uint32_t a_voff = 0x80000000u;   // beyond the buffer's range: no memory traffic, zeros
  if (a_row < t.rows_valid) {
    const long long srow = args.perm ? (long long)(args.perm[p] / args.k_top) : (long long)a_row;
    a_voff = (uint32_t)(srow * args.lda * 2 + kc16);
  }
  const uint16_t *a_base = args.perm ? args.A : args.A + (long long)(t.row0 + t.tile_row0) * args.lda;
  __amdgpu_buffer_rsrc_t a_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(a_base), 0, 0x7FFFFFFF, 0x00020000);
  const char *wptr = QF != 0 ? args.qbase + (long long)args.slot[t.grp] * args.qstride
                             : args.wbase + (long long)args.slot[t.grp] * args.wstride + args.b0_off;
  __amdgpu_buffer_rsrc_t b_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(wptr), 0, 0x7FFFFFFF, 0x00020000);
  const long long row_bytes = QF == 2 ? args.K >> 1 : QF == 1 ? args.K : (long long)args.ldb * 2;
  const uint32_t b_voff =
      QF == 2 ? (uint32_t)(((lane_s >> 5) * 16 + (lane_s & 15)) * row_bytes + ((lane_s >> 4) & 1) * 16)
      : QF == 1 ? (uint32_t)((lane_s >> 2) * row_bytes + (((lane_s & 3) ^ ((lane_s >> 4) & 3)) << 4))
                : (uint32_t)((lane_s >> 3) * row_bytes + kc16);
  int b_soff[NLC];
#pragma unroll
  for (int i = 0; i < NLC; ++i) {
    int r = QF == 2 ? wave * 32 : QF == 1 ? (wave + 8 * i) * 16 : (wave + 8 * i) * 8;
    long long base = QF != 0 ? args.q_b0_off : 0;
    if (MODE == GEMM_SWIGLU && r >= BN / 2) {
      base = QF != 0 ? args.q_b1_off : args.b1_off - args.b0_off;
      r -= BN / 2;
    }
    b_soff[i] = (int)(base + (long long)(t.n0 + r) * row_bytes);
  }
  // MXFP4: wave w brings the scale dwords of tile rows 32 w .. 32 w + 31 (lanes 0..31)
  uint32_t q_ssrc = 0x80000000u;
  int q_ssoff = 0;
  if constexpr (QF == 2) {
    int rs = wave * 32;
    long long sbase = args.q_s0_off;
    if (MODE == GEMM_SWIGLU && rs >= BN / 2) { sbase = args.q_s1_off; rs -= BN / 2; }
    if (lane_s < 32) q_ssrc = (uint32_t)(lane_s * (args.K >> 5));
    q_ssoff = (int)(sbase + (long long)(t.n0 + rs) * (args.K >> 5));
  }
  const int lrow = lane_s & 31, lk = lane_s >> 5;
  const int a_addr = swz(wm * 32 + lrow, lk);
  int b_addr[FN], q_saddr[FN] = {};
  float q_rs[FN] = {};   // e4m3: the scales of this lane's B fragment rows
#pragma unroll
  for (int j = 0; j < FN; ++j) {
    const int brow = (MODE == GEMM_SWIGLU) ? (j / FNH) * (BN / 2) + ((j % FNH) * WARPS_N + wn) * 32 + lrow
                                           : (j * WARPS_N + wn) * 32 + lrow;
    if constexpr (QF == 2) {
      b_addr[j] = SAB + (brow >> 4) * 512 + (brow & 15) * 16 + lk * 4;
      q_saddr[j] = SQS + (brow >> 5) * 256 + (brow & 31) * 4;
    } else if constexpr (QF == 1) {
      b_addr[j] = SAB + brow * 64 + lk * 8 + (((brow >> 2) & 3) << 4);
      const long long so = (MODE == GEMM_SWIGLU && j >= FNH) ? args.q_s1_off : args.q_s0_off;
      const int n = t.n0 + (((MODE == GEMM_SWIGLU) ? j % FNH : j) * WARPS_N + wn) * 32 + lrow;
      q_rs[j] = reinterpret_cast<const float *>(wptr + so)[n];
    } else {
      b_addr[j] = SAB + swz(brow, lk);
    }
  }
  const int fm_valid = wm * 32 < t.rows_valid ? 1 : 0;

#define MOE_SISSUE(q_)                                                                               \
  do {                                                                                               \
    unsigned char *st_ = smem + ((q_) % NST) * SST;                                                  \
    const int kt_ = kt_begin + (q_);                                                                 \
    _Pragma("unroll") for (int i_ = 0; i_ < NLC; ++i_) {                                             \
      if constexpr (QF == 2)                                                                         \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, (lds_ptr_t)(st_ + SAB + wave * 1024), 16,  \
                                                 (int)b_voff, b_soff[i_] + kt_ * (BK / 2), 0, 0);    \
      else if constexpr (QF == 1)                                                                    \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, (lds_ptr_t)(st_ + SAB + (wave + 8 * i_) * 1024), 16, \
                                                 (int)b_voff, b_soff[i_] + kt_ * BK, 0, 0);          \
      else                                                                                           \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, (lds_ptr_t)(st_ + SAB + (wave + 8 * i_) * 1024), 16, \
                                                 (int)b_voff, b_soff[i_] + kt_ * ROW_BYTES, 0, 0);   \
    }                                                                                                \
    if constexpr (QF == 2)                                                                           \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, (lds_ptr_t)(st_ + SQS + wave * 256), 4, (int)q_ssrc, \
                                               q_ssoff + ((kt_ >> 1) << 2), 0, 0);                   \
    __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_ptr_t)(st_ + wave * 1024), 16, (int)a_voff, \
                                             kt_ * ROW_BYTES, 0, 0);                                 \
  } while (0)
#define MOE_SVMCNT(n_) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n_) & 15) | (((n_) >> 4) << 14))

  floatx16 acc[1][FN];
#pragma unroll
  for (int j = 0; j < FN; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[0][j][r] = 0.0f;

  for (int q = 0; q < NST - 1; ++q)
    if (q < nk) MOE_SISSUE(q);
  for (int H = 0; H < nk; ++H) {
    // this wave's loads of stage H have landed: the stages requested after it (at most NST - 2 of them:
    // the next one is requested behind the barrier) may still be in flight
    const int later = nk - 1 - H;
    __builtin_amdgcn_sched_barrier(0);
    switch (later < NST - 2 ? later : NST - 2) {
      case 0: MOE_SVMCNT(0); break;
      case 1: MOE_SVMCNT(LPS); break;
      case 2: MOE_SVMCNT(2 * LPS); break;
      case 3: MOE_SVMCNT(NST > 4 ? 3 * LPS : 0); break;
      case 4: MOE_SVMCNT(NST > 5 ? 4 * LPS : 0); break;
      case 5: MOE_SVMCNT(NST > 6 ? 5 * LPS : 0); break;
      default: MOE_SVMCNT(NST > 7 ? 6 * LPS : 0); break;
    }
    __builtin_amdgcn_s_barrier();   // ... and everybody's; the stage read in the last step is free
    __builtin_amdgcn_sched_barrier(0);
    if (H + NST - 1 < nk) MOE_SISSUE(H + NST - 1);
    if (fm_valid) {
      const unsigned char *st = smem + (H % NST) * SST;
      bf16x8 af[4], bf[FN][4];
      if constexpr (QF == 2) {
        uint32_t qc[FN][4], qs[FN];
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          qs[j] = *reinterpret_cast<const uint32_t *>(st + q_saddr[j]);
#pragma unroll
          for (int ks = 0; ks < 4; ++ks)
            qc[j][ks] = *reinterpret_cast<const uint32_t *>(st + (b_addr[j] ^ (((ks >> 1) << 8) | ((ks & 1) << 3))));
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) af[ks] = *reinterpret_cast<const bf16x8 *>(st + (a_addr ^ (ks << 5)));
        const int sh = ((kt_begin + H) & 1) * 16;
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          const float f0 = __uint_as_float(((qs[j] >> sh) & 0xFFu) << 23);
          const float f1 = __uint_as_float(((qs[j] >> (sh + 8)) & 0xFFu) << 23);
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) bf[j][ks] = __builtin_bit_cast(bf16x8, expand8_mxfp4(qc[j][ks], ks < 2 ? f0 : f1));
        }
      } else if constexpr (QF == 1) {
        u32x2 qc[FN][4];
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) qc[j][ks] = *reinterpret_cast<const u32x2 *>(st + (b_addr[j] ^ (ks << 4)));
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) af[ks] = *reinterpret_cast<const bf16x8 *>(st + (a_addr ^ (ks << 5)));
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int ks = 0; ks < 4; ++ks)
            bf[j][ks] = __builtin_bit_cast(bf16x8, expand8_e4m3(qc[j][ks].x, qc[j][ks].y, q_rs[j]));
      } else {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          af[ks] = *reinterpret_cast<const bf16x8 *>(st + (a_addr ^ (ks << 5)));
#pragma unroll
          for (int j = 0; j < FN; ++j) bf[j][ks] = *reinterpret_cast<const bf16x8 *>(st + (b_addr[j] ^ (ks << 5)));
        }
      }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[j][ks], af[ks], acc[0][j], 0, 0, 0);
    }
  }
#undef MOE_SVMCNT
#undef MOE_SISSUE
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): this wave's fragment reads are done
  __builtin_amdgcn_s_barrier();         // ... and everybody's: LDS is free
  __builtin_amdgcn_sched_barrier(0);
  store_tile_cols<MODE, 1, FN, WARPS_M, WARPS_N>(args, t, wm, wn, lane, fm_valid, acc, 0, 1, nullptr);
}

// ---------------------------------------------------------------------------------------------
// Ping-pong kernel: 256 x 256 x 64 tiles in a two-stage LDS ring, eight waves in two groups of
// four.  Waves w and w+4 of a block sit on the same SIMD; the two groups run the same loop one
// barrier interval ("tick") apart, so while one wave of a SIMD issues 16 MFMAs, its partner pulls
// its next fragments out of LDS and requests global->LDS loads.  Every wait (LDS latency, load
// completion) falls into a tick in which the SIMD's matrix pipe is fed by the other wave.
//
// A wave owns 4 x 2 fragments of 32 x 32.  One K step of 64 is two M/C tick pairs:
//   M1: read B (both fragments, 4 K slices) and A fragments 0,1      C1: 16 MFMAs on them
//   M2: read A fragments 2,3 (B stays in registers)                   C2: 16 MFMAs
//   group 0:  M1(0) C1(0) M2(0) C2(0) M1(1) ...
//   group 1:    -   M1(0) C1(0) M2(0) C2(0) ...
// The B rows of a stage are free after both groups' M1, the lower 128 A rows likewise, the upper
// 128 A rows after both M2.  Refills are spread so that every M tick requests four wave-wide loads
// per wave and each load has four to six ticks to land, although only two stages fit into LDS:
//   M2(H): B rows of stage H+2 (each group one half)
//   M1(H): group 0 the lower A rows, group 1 the upper A rows of stage H+1
// Loads move whole 128-byte lines (8 tile rows per wave-wide load): half lines would halve the L1
// fill rate.  Needs K % 64 == 0.
// QF = 2: the B operand is the experts' MXFP4 blobs (GemmArgs::qbase).  A stage's B tile is then 256 rows of
// 32 bytes of codes plus 4 scale bytes per row.  Each wave brings 32 rows of codes with one 16-byte direct
// load (lane l the half (l / 16) % 2 of row 16 (l / 32) + l % 16; in LDS the 16 first halves of a 16-row
// block are followed by its 16 second halves, which leaves the fragment reads two-way bank conflicts, the
// least that 16-byte pieces allow) and 32 rows of scales with one 4-byte load (lanes 0..31: the aligned dword
// that holds the row's two scale bytes of this K step and of its neighbour).  A lane builds its B fragment of K slice ks from one dword of codes with the hardware's scaled
// fp4 conversion (exact), so the MFMAs see the weights the format defines.  Needs K % 128 == 0 and the blob within 31 bits of byte offset.
// QF = 1: the e4m3 blobs.  A stage's B tile is 256 rows of 64 bytes of codes, two 16-byte wave-wide loads per wave
// (a load is 16 rows of four pieces; the piece at position p of row r is piece p ^ ((r >> 2) & 3) of the row's
// K step).  A lane builds a B fragment from 8 bytes of codes and its row's fp32 scale (fetched once per tile):
// the hardware's e4m3 -> fp32 conversion, one multiply, nearest-even bf16 - 16 vector instructions per
// fragment and K slice, issued in the load tick.
template <int MODE, int QF = 0>
__global__ __launch_bounds__(512) void grouped_gemm_pp_kernel(const GemmArgs args) {
  constexpr int BM = 256, BN = 256, WARPS_M = 2, WARPS_N = 4;
  constexpr int BN_OUT = (MODE == GEMM_SWIGLU) ? BN / 2 : BN;
  constexpr int FM = 4, FN = 2;
  constexpr int FNH = (MODE == GEMM_SWIGLU) ? FN / 2 : FN;
  constexpr int STAGE = (BM + BN) * ROW_BYTES;   // 64 KB
  constexpr int NL = 4;                          // wave-wide loads per wave and M tick
  constexpr int NB = QF != 0 ? 2 : NL;           // ... of a B stage (e4m3: two of codes; MXFP4: codes and scales)
  constexpr int QCODES = BM * ROW_BYTES;         // quantised B: a stage's codes (e4m3 16 KB; MXFP4 8 KB and,
  constexpr int QSCALES = QCODES + BN * 32;      // behind them, 2 KB for the scale dwords)
  static_assert(QF >= 0 && QF <= 2, "B operand: 0 = bf16, 1 = e4m3 rows, 2 = MXFP4");

  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  unsigned char *xpose = smem + 2 * STAGE + wave * 4096;   // this wave's epilogue buffer
  const int grp = wave >> 2;          // the two waves of a SIMD are in different groups
  const int wm = grp, wn = wave & 3;

  // Work items (decode_item).  With a plan the blocks take them from eight queues, one per XCD (blocks
  // go round-robin over the XCDs, so b % 8 is a block's XCD): item v of a range goes to whoever
  // increments that range's counter from v, which keeps every block busy until its range is used up,
  // whatever the tiles cost; then it goes on with the other XCDs' ranges.  Without a plan block b walks
  // the items (b % 8) * chunk + b / 8 + i * (blocks / 8).  Either way the blocks of one XCD work on
  // consecutive items at any time, and the metadata and first loads of the next item are requested
  // before the current item's results are stored.  The item after the next one travels from thread 0
  // to the block through the first word of wave 0's epilogue buffer (written at the top of an item,
  // read behind the barrier that follows, long before any wave stores results again).
  GemmPlan *const plan = args.plan;
  const bool dyn = plan != nullptr && args.plan_queue;
  const GemmPlan *const qplan = dyn ? plan : nullptr;   // the groups' first items, for the queues' item numbers
  const int s_f = __builtin_amdgcn_readfirstlane(plan ? plan->s_full : args.splitk);
  const int s_r = __builtin_amdgcn_readfirstlane(plan ? plan->s_rem : args.splitk);
  volatile int *qbox = reinterpret_cast<volatile int *>(smem + 2 * STAGE);
  const int xcd = (int)blockIdx.x & 7;
  const int nslots = (int)gridDim.x >> 3;
  int own_b = 0, own_len = 0, st_end = 0;   // this XCD's range (plan) / end of this block's range (no plan)
  int cur, nxt;                             // item being computed, item after it (-1: none)
  int pend_v = 0;                           // thread 0: its last increment of the own range's counter
  bool pend_issued = false;
#define MOE_PTAKE_OWN() __hip_atomic_fetch_add(&plan->queue[xcd * 16], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
  // an item of another XCD's range (own range used up), or -1 when every range is
  auto steal = [&]() -> int {
    for (int i = 1; i < 8; ++i) {
      const int xx = (xcd + i) & 7;
      const int b = plan->xcd_begin[xx], len = plan->xcd_begin[xx + 1] - b;
      if (len <= 0) continue;
      const int v = __hip_atomic_fetch_add(&plan->queue[xx * 16], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (v < len) return b + v;
    }
    return -1;
  };
  if (dyn) {
    own_b = __builtin_amdgcn_readfirstlane(plan->xcd_begin[xcd]);
    own_len = __builtin_amdgcn_readfirstlane(plan->xcd_begin[xcd + 1]) - own_b;
    if (tid == 0) {
      int it[2];
      for (int q = 0; q < 2; ++q) {
        int v = own_len > 0 ? MOE_PTAKE_OWN() : own_len;
        it[q] = v < own_len ? own_b + v : steal();
      }
      qbox[0] = it[0];
      qbox[1] = it[1];
    }
    __syncthreads();
    cur = qbox[0];
    nxt = qbox[1];
    __syncthreads();
    if (nxt >= 0 && own_len > 0) {   // the third item: requested now, looked at when the first one starts
      if (tid == 0) pend_v = MOE_PTAKE_OWN();
      pend_issued = true;
    }
  } else {
    const int total = count_items<BM, BN_OUT>(args, s_f, s_r);
    const int chunk = (total + 7) >> 3;
    const int slot = (int)blockIdx.x >> 3;
    st_end = min(total, (xcd + 1) * chunk);
    cur = slot < chunk && xcd * chunk + slot < st_end ? xcd * chunk + slot : -1;
    nxt = cur >= 0 && cur + nslots < st_end ? cur + nslots : -1;
  }
  cur = __builtin_amdgcn_readfirstlane(cur);
  nxt = __builtin_amdgcn_readfirstlane(nxt);
  if (cur < 0) return;

  // The last column tile is moved back so that it ends at column N - 1 (the overlap is computed
  // twice, to the same bits): every B row of a tile exists, and its offset is affine in the row.
  TileInfo t;
  decode_item<BM, BN_OUT>(args, qplan, s_f, s_r, lane, cur, t);
  t.n0 = min(t.n0, args.N - BN_OUT);

  // Row group g (0..63) is tile rows 8g..8g+7 of a stage (A rows 0..255, then B rows 0..255) and
  // one wave-wide load: lane l lands at row 8g + l/8, chunk position l%8, and fetches the chunk the
  // swizzle maps there.  Group 0 loads the lower A rows and the first half of B, group 1 the rest.
  // Sources are 32-bit byte offsets into two buffer resources (A, and the blob from its gate/down
  // rows on), so a load needs one VGPR and the K advance is a scalar offset.
  // Gathered rows (perm) are addressed from the start of A; rows in place from the tile's first row,
  // so that only a gathered source has to fit 31 bits of byte offset.
  __amdgpu_buffer_rsrc_t a_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(args.A), 0, 0x7FFFFFFF, 0x00020000);
#define MOE_PGROUP(i_) (((i_) / NL) * 32 + grp * 16 + ((i_) % NL) * 4 + (wave & 3))

  // Gathered source rows of this lane's A loads of tile tt_ (requested; used by MOE_PSRC), and the
  // byte offsets of its eight loads.  (row >> 1) & 7 of a lane's row 8g + l/8 is 4 (g & 1) + l/16,
  // and g & 1 = wave & 1 for all of a wave's row groups: one chunk offset serves all eight.
#define MOE_PPERM(tt_, out_)                                                                         \
  _Pragma("unroll") for (int i_ = 0; i_ < NL; ++i_) {                                                \
    const int row_ = MOE_PGROUP(i_) * 8 + (lane_s >> 3);                                             \
    const int rr_ = row_ < (tt_).rows_valid ? row_ : 0;                                              \
    const int p_ = (tt_).row0 + (tt_).tile_row0 + rr_;                                               \
    (out_)[i_] = args.perm ? args.perm[p_] : rr_;                                                    \
  }
#define MOE_PSRC(tt_, prow_)                                                                         \
  do {                                                                                               \
    const int kc16_ = ((lane_s & 7) ^ ((wave & 1) * 4 + (lane_s >> 4))) * 16;                        \
    _Pragma("unroll") for (int i_ = 0; i_ < NL; ++i_) {                                              \
      const long long srow_ =                                                                        \
          args.perm ? (long long)((prow_)[i_] / args.k_top) : (long long)(prow_)[i_];                \
      /* rows past the tile's last one: an offset beyond the buffer's range, which costs no memory   \
         traffic (the load returns zeros; what the MFMAs make of those rows is never stored) */      \
      src[i_] = MOE_PGROUP(i_) * 8 + (lane_s >> 3) < (tt_).rows_valid                                \
                    ? (uint32_t)(srow_ * args.lda * 2 + kc16_) : 0x80000000u;                        \
    }                                                                                                \
    if (!args.perm)                                                                                  \
      a_rsrc = __builtin_amdgcn_make_buffer_rsrc(                                                    \
          const_cast<uint16_t *>(args.A + (long long)((tt_).row0 + (tt_).tile_row0) * args.lda), 0,  \
          0x7FFFFFFF, 0x00020000);                                                                   \
    /* B rows are n0 + 8 g + l/8: one per-lane offset, the row group's part is scalar */             \
    if constexpr (QF == 2) {                                                                         \
      /* codes: K / 2 bytes per row; wave w brings tile rows 32 w .. 32 w + 31 */                    \
      src[NL] = (uint32_t)(((lane_s >> 5) * 16 + (lane_s & 15)) * (args.K >> 1) + ((lane_s >> 4) & 1) * 16); \
      {                                                                                              \
        int r_ = wave * 32;                                                                          \
        long long base_ = args.q_b0_off;                                                             \
        if (MODE == GEMM_SWIGLU && r_ >= BN / 2) { base_ = args.q_b1_off; r_ -= BN / 2; }            \
        b_soff[0] = (int)(base_ + (long long)((tt_).n0 + r_) * (args.K >> 1));                       \
      }                                                                                              \
      /* scales: the dwords of the same rows (K / 32 bytes per row) */                               \
      int rs_ = wave * 32;                                                                           \
      long long sbase_ = args.q_s0_off;                                                              \
      if (MODE == GEMM_SWIGLU && rs_ >= BN / 2) { sbase_ = args.q_s1_off; rs_ -= BN / 2; }           \
      q_ssrc = lane_s < 32 ? (uint32_t)(lane_s * (args.K >> 5)) : 0x80000000u;                       \
      q_ssoff = (int)(sbase_ + (long long)((tt_).n0 + rs_) * (args.K >> 5));                         \
    } else if constexpr (QF == 1) {                                                                  \
      /* codes: K bytes per row; load i_ of a wave brings tile rows 16 (8 i_ + wave) .. + 15 */      \
      src[NL] = (uint32_t)((lane_s >> 2) * args.K + (((lane_s & 3) ^ ((lane_s >> 4) & 3)) << 4));    \
      _Pragma("unroll") for (int i_ = 0; i_ < 2; ++i_) {                                             \
        int r_ = (i_ * 8 + wave) * 16;                                                               \
        long long base_ = args.q_b0_off;                                                             \
        if (MODE == GEMM_SWIGLU && r_ >= BN / 2) { base_ = args.q_b1_off; r_ -= BN / 2; }            \
        b_soff[i_] = (int)(base_ + (long long)((tt_).n0 + r_) * args.K);                             \
      }                                                                                              \
    } else {                                                                                         \
      src[NL] = (uint32_t)((lane_s >> 3) * args.ldb * 2 + kc16_);                                    \
      _Pragma("unroll") for (int i_ = 0; i_ < NL; ++i_) {                                            \
        int r_ = MOE_PGROUP(NL + i_) * 8 - BM;                                                       \
        long long up_ = 0;                                                                           \
        if (MODE == GEMM_SWIGLU && r_ >= BN / 2) { up_ = args.b1_off - args.b0_off; r_ -= BN / 2; }  \
        b_soff[i_] = (int)(up_ + (long long)((tt_).n0 + r_) * args.ldb * 2);                         \
      }                                                                                              \
    }                                                                                                \
  } while (0)
#define MOE_PTILE_SETUP(tt_)                                                                         \
  do {                                                                                               \
    const char *wptr_ = QF != 0 ? args.qbase + (long long)args.slot[(tt_).grp] * args.qstride        \
                                : args.wbase + (long long)args.slot[(tt_).grp] * args.wstride + args.b0_off; \
    b_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(wptr_), 0, 0x7FFFFFFF, 0x00020000); \
    const int kt_total_ = args.K / BK;                                                               \
    kt_begin = (int)((long long)kt_total_ * (tt_).ks / (tt_).ns);                                    \
    nk = (int)((long long)kt_total_ * ((tt_).ks + 1) / (tt_).ns) - kt_begin;                         \
    fm_valid = 0;                                                                                    \
    _Pragma("unroll") for (int i_ = 0; i_ < FM; ++i_)                                                \
      fm_valid += ((i_ * WARPS_M + wm) * 32 < (tt_).rows_valid) ? 1 : 0;                             \
    if constexpr (QF == 1) {                                                                         \
      _Pragma("unroll") for (int j_ = 0; j_ < FN; ++j_) {                                            \
        const long long so_ = (MODE == GEMM_SWIGLU && j_ >= FNH) ? args.q_s1_off : args.q_s0_off;    \
        const int n_ = (tt_).n0 + (((MODE == GEMM_SWIGLU) ? j_ % FNH : j_) * WARPS_N + wn) * 32 + (lane & 31); \
        q_rs[j_] = reinterpret_cast<const float *>(wptr_ + so_)[n_];                                 \
      }                                                                                              \
    }                                                                                                \
  } while (0)

  float q_rs[FN] = {};           // e4m3: the scales of this lane's B fragment rows
  __amdgpu_buffer_rsrc_t b_rsrc;
  int kt_begin, nk, fm_valid;
  uint32_t src[NL + 1];          // per-lane byte offsets: the A row groups, then one for all B rows
  int b_soff[NL];                // scalar byte offsets of the B row groups
  uint32_t q_ssrc = 0;           // MXFP4: per-lane and scalar byte offset of the scale load
  int q_ssoff = 0;
  {
    const int lane_s = opaque(lane);
    int prow[NL];
    MOE_PPERM(t, prow);
    MOE_PSRC(t, prow);
  }
  MOE_PTILE_SETUP(t);

  // this wave's A (WHICH_ = 0) or B (WHICH_ = 1) loads of stage q_
#define MOE_PISSUE(q_, WHICH_)                                                                       \
  do {                                                                                               \
    if ((WHICH_) && QF == 2) {                                                                       \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(                                                      \
          b_rsrc, (lds_ptr_t)(smem + ((q_) & 1) * STAGE + QSCALES + wave * 256), 4, (int)q_ssrc,     \
          q_ssoff + (((kt_begin + (q_)) >> 1) << 2), 0, 0);                                          \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(                                                      \
          b_rsrc, (lds_ptr_t)(smem + ((q_) & 1) * STAGE + QCODES + wave * 1024), 16, (int)src[NL],   \
          b_soff[0] + (kt_begin + (q_)) * (BK / 2), 0, 0);                                           \
    } else                                                                                           \
    if ((WHICH_) && QF == 1) {                                                                       \
      _Pragma("unroll") for (int i_ = 0; i_ < 2; ++i_)                                               \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(                                                    \
            b_rsrc, (lds_ptr_t)(smem + ((q_) & 1) * STAGE + QCODES + (i_ * 8 + wave) * 1024), 16,    \
            (int)src[NL], b_soff[i_] + (kt_begin + (q_)) * BK, 0, 0);                                \
    } else                                                                                           \
    _Pragma("unroll") for (int i_ = 0; i_ < NL; ++i_) {                                              \
      if (WHICH_)                                                                                    \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(                                                    \
            b_rsrc, (lds_ptr_t)(smem + ((q_) & 1) * STAGE + MOE_PGROUP(NL + i_) * 1024), 16,         \
            (int)src[NL], b_soff[i_] + (kt_begin + (q_)) * ROW_BYTES, 0, 0);                         \
      else                                                                                           \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(                                                    \
            a_rsrc, (lds_ptr_t)(smem + ((q_) & 1) * STAGE + MOE_PGROUP(i_) * 1024), 16,              \
            (int)src[i_], (kt_begin + (q_)) * ROW_BYTES, 0, 0);                                      \
    }                                                                                                \
  } while (0)
#define MOE_PVMCNT(n_) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n_) & 15) | (((n_) >> 4) << 14))
#define MOE_PBARRIER()                                                                               \
  do {                                                                                               \
    __builtin_amdgcn_sched_barrier(0);                                                               \
    __builtin_amdgcn_s_barrier();                                                                    \
    __builtin_amdgcn_sched_barrier(0);                                                               \
  } while (0)
#define MOE_PREAD_A(I0_, I1_)                                                                        \
  do {                                                                                               \
    _Pragma("unroll") for (int i_ = (I0_); i_ < (I1_); ++i_)                                         \
      _Pragma("unroll") for (int ks_ = 0; ks_ < 4; ++ks_)                                            \
        af_[i_ & 1][ks_] = *reinterpret_cast<const bf16x8 *>(st_ + (a_addr[i_] ^ (ks_ << 5)));       \
  } while (0)
// MFMAs of fragment i_ for K slices [KS0_, KS1_) against both B fragments
#define MOE_PMMA1(i_, ks_)                                                                           \
  _Pragma("unroll") for (int j_ = 0; j_ < FN; ++j_)                                                  \
    acc[i_][j_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf_[j_][ks_], af_[(i_) & 1][ks_], acc[i_][j_], 0, 0, 0)
// The two compute ticks of a K step, for FMV valid fragments, with the MFMAs split evenly:
//   4: {0,1} | {2,3}     3: 0 and the first half of 1 | second half of 1 and 2
//   2: 0 | 1             1: first half of 0 | second half of 0
// (fragments 0,1 are read in M1 and 2,3 in M2, whatever tick multiplies them: the A rows of fragments 2, 3 are
// the ones whose arrival group 1 certifies only at the end of ITS M1, one tick after group 0's, so no wave may
// read them before M2.  Cutting the ticks along K instead - all fragments' slices 0, 1 in M1 - reads them too
// early: tried for the e4m3 conversions, wrong sums in rows 128.. of a tile)
#define MOE_PMMA(FMV, TICK_)                                                                         \
  do {                                                                                               \
    __builtin_amdgcn_s_setprio(1);                                                                   \
    _Pragma("unroll") for (int ks_ = 0; ks_ < 4; ++ks_) {                                            \
      if (FMV == 4) {                                                                                \
        MOE_PMMA1(2 * (TICK_), ks_);                                                                 \
        MOE_PMMA1(2 * (TICK_) + 1, ks_);                                                             \
      } else if (FMV == 3) {                                                                         \
        if ((TICK_) == 0) { MOE_PMMA1(0, ks_); if (ks_ < 2) MOE_PMMA1(1, ks_); }                     \
        else { if (ks_ >= 2) MOE_PMMA1(1, ks_); MOE_PMMA1(2, ks_); }                                 \
      } else if (FMV == 2) {                                                                         \
        MOE_PMMA1((TICK_), ks_);                                                                     \
      } else if (FMV == 1) {                                                                         \
        if ((ks_ >> 1) == (TICK_)) MOE_PMMA1(0, ks_);                                                \
      }                                                                                              \
    }                                                                                                \
    __builtin_amdgcn_s_setprio(0);                                                                   \
  } while (0)
// One K step of one wave.  FMV of the wave's A fragments are valid: the others are neither read
// nor multiplied (the loop is instantiated per count, so a tick stays straight-line code).
// iss1_ / iss2_: the upper-or-lower A rows of stage H+1 / the B rows of stage H+2 are requested
// here (M1(0) requests nothing: the prologue already has); next_: stage H+1 exists.  A wave's loads
// complete in order (NL of an A stage, NB of a B stage): after M2(H) its youngest are [B(H+1)] [A(H+1)] [B(H+2)].  Group 1 has to
// certify its share at the end of its M ticks (group 0 reads in the next tick); group 0 can wait
// until the end of C2, right before its own M1(H+1).  The flags are wave-uniform: scalar branches.
#define MOE_PP_STEP(FMV, iss1_, iss2_, next_)                                                        \
  do {                                                                                               \
    const unsigned char *st_ = smem + (H & 1) * STAGE;                                               \
    /* M1 */                                                                                         \
    if (FMV > 0) {                                                                                   \
      if constexpr (QF == 2) {                                                                       \
        uint32_t qc_[FN][4], qs_[FN];                                                                \
        _Pragma("unroll") for (int j_ = 0; j_ < FN; ++j_) {                                          \
          qs_[j_] = *reinterpret_cast<const uint32_t *>(st_ + q_saddr[j_]);                          \
          _Pragma("unroll") for (int ks_ = 0; ks_ < 4; ++ks_)                                        \
            qc_[j_][ks_] = *reinterpret_cast<const uint32_t *>(                                      \
                st_ + (b_addr[j_] ^ (((ks_ >> 1) << 8) | ((ks_ & 1) << 3))));                        \
        }                                                                                            \
        MOE_PREAD_A(0, (FMV < 2 ? FMV : 2));                                                         \
        const int sh_ = ((kt_begin + H) & 1) * 16;   /* this K step's two bytes of the scale dword */ \
        _Pragma("unroll") for (int j_ = 0; j_ < FN; ++j_) {                                          \
          const float f0_ = __uint_as_float(((qs_[j_] >> sh_) & 0xFFu) << 23);                       \
          const float f1_ = __uint_as_float(((qs_[j_] >> (sh_ + 8)) & 0xFFu) << 23);                 \
          _Pragma("unroll") for (int ks_ = 0; ks_ < 4; ++ks_)                                        \
            bf_[j_][ks_] = __builtin_bit_cast(bf16x8, expand8_mxfp4(qc_[j_][ks_], ks_ < 2 ? f0_ : f1_)); \
        }                                                                                            \
      } else if constexpr (QF == 1) {                                                                \
        u32x2 qc_[FN][4];                                                                            \
        _Pragma("unroll") for (int j_ = 0; j_ < FN; ++j_)                                            \
          _Pragma("unroll") for (int ks_ = 0; ks_ < 4; ++ks_)                                        \
            qc_[j_][ks_] = *reinterpret_cast<const u32x2 *>(st_ + (b_addr[j_] ^ (ks_ << 4)));        \
        MOE_PREAD_A(0, (FMV < 2 ? FMV : 2));                                                         \
        _Pragma("unroll") for (int j_ = 0; j_ < FN; ++j_)                                            \
          _Pragma("unroll") for (int ks_ = 0; ks_ < 4; ++ks_)                                        \
            bf_[j_][ks_] = __builtin_bit_cast(bf16x8, expand8_e4m3(qc_[j_][ks_].x, qc_[j_][ks_].y, q_rs[j_])); \
      } else {                                                                                       \
        _Pragma("unroll") for (int j_ = 0; j_ < FN; ++j_)                                            \
          _Pragma("unroll") for (int ks_ = 0; ks_ < 4; ++ks_)                                        \
            bf_[j_][ks_] = *reinterpret_cast<const bf16x8 *>(st_ + (b_addr[j_] ^ (ks_ << 5)));       \
        MOE_PREAD_A(0, (FMV < 2 ? FMV : 2));                                                         \
      }                                                                                              \
    }                                                                                                \
    if (iss1_) MOE_PISSUE(H + 1, 0);                                                                 \
    if (grp) { if (next_) MOE_PVMCNT(NL + NB); else MOE_PVMCNT(0); }  /* upper A rows of stage H */  \
    __builtin_amdgcn_s_waitcnt(0xC07F);  /* lgkmcnt(0): fragments are in */                          \
    MOE_PBARRIER();                                                                                  \
    /* C1 */                                                                                         \
    if (FMV > 0) MOE_PMMA(FMV, 0);                                                                   \
    MOE_PBARRIER();                                                                                  \
    /* M2 */                                                                                         \
    if (FMV > 2) MOE_PREAD_A(2, FMV);                                                                \
    if (iss2_) MOE_PISSUE(H + 2, 1);                                                                 \
    if (grp) { if (iss2_) MOE_PVMCNT(NL + NB); else if (next_) MOE_PVMCNT(NL); else MOE_PVMCNT(0); } \
    __builtin_amdgcn_s_waitcnt(0xC07F);                                                              \
    MOE_PBARRIER();                                                                                  \
    /* C2 */                                                                                         \
    if (FMV > 0) MOE_PMMA(FMV, 1);                                                                   \
    if (!grp) { if (iss2_) MOE_PVMCNT(NB); else MOE_PVMCNT(0); }     /* all of stage H+1 */          \
    MOE_PBARRIER();                                                                                  \
  } while (0)
#define MOE_PP_LOOP(FMV)                                                                             \
  do {                                                                                               \
    bf16x8 af_[2][4], bf_[FN][4];                                                                    \
    for (int H = 0; H < nk; ++H) MOE_PP_STEP(FMV, (H > 0 && H + 1 < nk), (H + 2 < nk), (H + 1 < nk)); \
  } while (0)

// both stages' first loads of the tile set up last (stage 1 only if the tile has a second K step)
#define MOE_PPROLOGUE()                                                                              \
  do {                                                                                               \
    MOE_PISSUE(0, 1);                                                                                \
    MOE_PISSUE(0, 0);                                                                                \
    if (nk > 1) {                                                                                    \
      MOE_PISSUE(1, 1);                                                                              \
      MOE_PISSUE(1, 0);                                                                              \
    }                                                                                                \
  } while (0)

  if (t.rows_valid > kSmallTileRows) MOE_PPROLOGUE();
  for (;;) {
    const bool has_next = nxt >= 0;
    TileInfo tn = t;
    if (has_next) {
      decode_item<BM, BN_OUT>(args, qplan, s_f, s_r, lane, nxt, tn);
      tn.n0 = min(tn.n0, args.N - BN_OUT);
    }
    MOE_PVMCNT(0);   // this tile's first loads have landed (and the previous tile's stores are out)
    // the item after the next one: thread 0's increment has come back with the loads
    if (dyn && tid == 0) {
      int it = -1;
      if (has_next) it = pend_issued && pend_v < own_len ? own_b + pend_v : steal();
      qbox[0] = it;
    }

    // LDS byte offset of this lane's 16 bytes of K slice 0 inside a stage; slice ks is at ^ (ks << 5)
    // (the swizzle XORs the chunk index, and slice ks only changes bits 1..2 of it).  Derived from
    // an opaque copy of the lane id so that they live only as long as the K loop.
    int a_addr[FM], b_addr[FN];
    int q_saddr[FN] = {};   // MXFP4: this lane's scale dwords
    {
      const int lane_k = opaque(lane);
      const int lrow = lane_k & 31, lk = lane_k >> 5;
#pragma unroll
      for (int i = 0; i < FM; ++i) a_addr[i] = swz((i * WARPS_M + wm) * 32 + lrow, lk);
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        const int brow = (MODE == GEMM_SWIGLU) ? (j / FNH) * (BN / 2) + ((j % FNH) * WARPS_N + wn) * 32 + lrow
                                               : (j * WARPS_N + wn) * 32 + lrow;
        if constexpr (QF == 2) {
          // dword ks * 2 + lk of the row's codes: half ks / 2 of the row, dword 2 (ks % 2) + lk of that half
          b_addr[j] = QCODES + (brow >> 4) * 512 + (brow & 15) * 16 + lk * 4;
          q_saddr[j] = QSCALES + (brow >> 5) * 256 + (brow & 31) * 4;   // wave brow / 32 brought it, lane brow % 32
        } else if constexpr (QF == 1) {
          // 8 codes of K slice ks: half lk of piece ks, which sits at position ks ^ ((brow >> 2) & 3)
          b_addr[j] = QCODES + brow * 64 + lk * 8 + (((brow >> 2) & 3) << 4);
        } else {
          b_addr[j] = BM * ROW_BYTES + swz(brow, lk);
        }
      }
    }

    floatx16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    MOE_PBARRIER();
    int after_next;
    if (dyn) after_next = qbox[0];
    else after_next = has_next && nxt + nslots < st_end ? nxt + nslots : -1;
    after_next = __builtin_amdgcn_readfirstlane(after_next);
    if (t.rows_valid <= kSmallTileRows) {
      // A short tile (pp_small_tile): no loads were requested for it, and its last stage lies over the
      // mailbox word, which everybody has to have read first.
      MOE_PBARRIER();
      pp_small_tile<MODE, QF>(args, t, smem, lane, wave);
      if (!has_next) break;
      pend_issued = dyn && after_next >= 0 && own_len > 0;
      if (pend_issued && tid == 0) pend_v = MOE_PTAKE_OWN();
      if (tn.rows_valid > kSmallTileRows) {
        const int lane_s = opaque(lane);
        int prow_n[NL];
        MOE_PPERM(tn, prow_n);
        MOE_PSRC(tn, prow_n);
        MOE_PTILE_SETUP(tn);
        MOE_PPROLOGUE();
      }
      t = tn;
      cur = nxt;
      nxt = after_next;
      continue;
    }
    if (grp == 1) MOE_PBARRIER();   // group 1 runs one tick behind
    switch (fm_valid) {
      case 0: MOE_PP_LOOP(0); break;
      case 1: MOE_PP_LOOP(1); break;
      case 2: MOE_PP_LOOP(2); break;
      case 3: MOE_PP_LOOP(3); break;
      default: MOE_PP_LOOP(4); break;
    }
    if (grp == 0) MOE_PBARRIER();   // same number of barriers for both groups; LDS is free now

    // The next tile's gathered rows are requested, half of this tile is stored while they arrive,
    // then the next tile's first loads go out and fly while the other half is stored.
    const int fm_cur = fm_valid;
    const int lane_s = opaque(lane);
    int prow_n[NL];
    const bool next_full = has_next && tn.rows_valid > kSmallTileRows;   // a short tile sets itself up
    if (next_full) {
      MOE_PPERM(tn, prow_n);
    } else {
#pragma unroll
      for (int i = 0; i < NL; ++i) prow_n[i] = 0;
    }
    store_tile_cols<MODE, FM, FN, WARPS_M, WARPS_N>(args, t, wm, wn, lane, fm_cur, acc, 0, FM / 2, xpose);
    if (has_next) {
      // the request for the item after the next two goes out ahead of the loads, so it is back with them
      pend_issued = dyn && after_next >= 0 && own_len > 0;
      if (pend_issued && tid == 0) pend_v = MOE_PTAKE_OWN();
    }
    if (next_full) {
      MOE_PSRC(tn, prow_n);
      MOE_PTILE_SETUP(tn);
      MOE_PPROLOGUE();
    }
    store_tile_cols<MODE, FM, FN, WARPS_M, WARPS_N>(args, t, wm, wn, lane, fm_cur, acc, FM / 2, FM, xpose);
    if (!has_next) break;
    t = tn;
    cur = nxt;
    nxt = after_next;
  }
#undef MOE_PTAKE_OWN
#undef MOE_PPROLOGUE
#undef MOE_PP_LOOP
#undef MOE_PP_STEP
#undef MOE_PMMA
#undef MOE_PMMA1
#undef MOE_PREAD_A
#undef MOE_PBARRIER
#undef MOE_PVMCNT
#undef MOE_PISSUE
#undef MOE_PTILE_SETUP
#undef MOE_PSRC
#undef MOE_PPERM
#undef MOE_PGROUP
}

// ---------------------------------------------------------------------------------------------
// Register-staged kernel with zero fill of the K tail (K % 8 == 0 is enough).
template <int BM, int BN, int WARPS_M, int WARPS_N, int MODE>
__global__ __launch_bounds__(64 * WARPS_M * WARPS_N) void grouped_gemm_ktail_kernel(const GemmArgs args) {
  constexpr int NTHR = 64 * WARPS_M * WARPS_N;
  constexpr int BN_OUT = (MODE == GEMM_SWIGLU) ? BN / 2 : BN;
  constexpr int FM = BM / (32 * WARPS_M);
  constexpr int FN = BN / (32 * WARPS_N);
  constexpr int FNH = (MODE == GEMM_SWIGLU) ? FN / 2 : FN;
  constexpr int CA = BM * 8 / NTHR;  // 16-byte chunks per thread, A tile
  constexpr int CB = BN * 8 / NTHR;
  constexpr int STAGE = (BM + BN) * ROW_BYTES;

  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WARPS_M, wn = wave / WARPS_M;

  TileInfo t;
  if (!decode_tile<BM, BN_OUT>(args, t)) return;

  const char *wptr = args.wbase + (long long)args.slot[t.grp] * args.wstride;
  const uint16_t *B0 = reinterpret_cast<const uint16_t *>(wptr + args.b0_off);
  const uint16_t *B1 = reinterpret_cast<const uint16_t *>(wptr + args.b1_off);
  const int kt_total = (args.K + BK - 1) / BK;
  const int kt_begin = (int)((long long)kt_total * t.ks / args.splitk);
  const int kt_end = (int)((long long)kt_total * (t.ks + 1) / args.splitk);

  const uint16_t *a_src[CA];
  int a_dst[CA];
#pragma unroll
  for (int i = 0; i < CA; ++i) {
    int c = tid + i * NTHR, r = c >> 3, kc = c & 7;
    int rr = r < t.rows_valid ? r : 0;
    int p = t.row0 + t.tile_row0 + rr;
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
    int n = t.n0 + rr;
    if (n >= args.N) n = args.N - 1;
    b_src[i] = base + (long long)n * args.ldb + kc * 8;
    b_dst[i] = BM * ROW_BYTES + swz(r, kc);
  }
  const int kc_lane = tid & 7;

  int fm_valid = 0;
#pragma unroll
  for (int i = 0; i < FM; ++i) fm_valid += ((i * WARPS_M + wm) * 32 < t.rows_valid) ? 1 : 0;

  floatx16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  int a_off[FM], b_off[FN];
  const int lrow = lane & 31, lk = lane >> 5;
#pragma unroll
  for (int i = 0; i < FM; ++i) a_off[i] = (i * WARPS_M + wm) * 32 + lrow;
#pragma unroll
  for (int j = 0; j < FN; ++j) {
    if (MODE == GEMM_SWIGLU)
      b_off[j] = (j / FNH) * (BN / 2) + ((j % FNH) * WARPS_N + wn) * 32 + lrow;
    else
      b_off[j] = (j * WARPS_N + wn) * 32 + lrow;
  }

  u32x4 ra[CA], rb[CB];
  for (int kt = kt_begin; kt < kt_end; ++kt) {
    const int k0 = kt * BK;
    const bool k_ok = k0 + kc_lane * 8 < args.K;
    const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < CA; ++i) ra[i] = k_ok ? *reinterpret_cast<const u32x4 *>(a_src[i] + k0) : zero;
#pragma unroll
    for (int i = 0; i < CB; ++i) rb[i] = k_ok ? *reinterpret_cast<const u32x4 *>(b_src[i] + k0) : zero;
    __syncthreads();  // previous step's fragments have been read
#pragma unroll
    for (int i = 0; i < CA; ++i) *reinterpret_cast<u32x4 *>(smem + a_dst[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < CB; ++i) *reinterpret_cast<u32x4 *>(smem + b_dst[i]) = rb[i];
    __syncthreads();
    const unsigned char *sa = smem, *sb = smem + BM * ROW_BYTES;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int kc = kk * 2 + lk;
      bf16x8 bfr[FN];
#pragma unroll
      for (int j = 0; j < FN; ++j) bfr[j] = *reinterpret_cast<const bf16x8 *>(sb + swz(b_off[j], kc));
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        if (i < fm_valid) {
          bf16x8 af = *reinterpret_cast<const bf16x8 *>(sa + swz(a_off[i], kc));
#pragma unroll
          for (int j = 0; j < FN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfr[j], acc[i][j], 0, 0, 0);
        }
      }
    }
  }
  (void)STAGE;
  store_tile<MODE, FM, FN, WARPS_M, WARPS_N>(args, t, wm, wn, lane, fm_valid, acc);
}

template <int BM, int BN, int WARPS_M, int WARPS_N, int MODE>
hipError_t launch_cfg(const GemmArgs &args, int max_rows, int n_groups_in_mask, hipStream_t stream) {
  constexpr int BN_OUT = (MODE == GEMM_SWIGLU) ? BN / 2 : BN;
  constexpr int NTHR = 64 * WARPS_M * WARPS_N;
  constexpr size_t smem = 2 * (size_t)(BM + BN) * ROW_BYTES;
  auto kern = grouped_gemm_dma_kernel<BM, BN, WARPS_M, WARPS_N, MODE>;
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

template <int BM, int BN, int WARPS_M, int WARPS_N, int MODE, int QF>
hipError_t launch_q8_cfg(const GemmArgs &args, int max_rows, int n_groups_in_mask, hipStream_t stream) {
  constexpr int BN_OUT = (MODE == GEMM_SWIGLU) ? BN / 2 : BN;
  constexpr int NTHR = 64 * WARPS_M * WARPS_N;
  constexpr size_t smem = 2 * (size_t)(BM + BN) * ROW_BYTES;
  auto kern = grouped_gemm_q8_kernel<BM, BN, WARPS_M, WARPS_N, MODE, QF>;
  static bool attr_set = false;
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

static int pp_grid_blocks() {
  static int blocks = 0;
  if (!blocks) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8)
      cus = 256;
    blocks = cus / 8 * 8;
  }
  return blocks;
}

// Blocks of a persistent launch: one per compute unit (a multiple of 8, spread over the 8 XCDs), fewer
// if there cannot be that many items; a launch that runs beside other streams' small kernels leaves
// them some units, whose LDS it would otherwise fill.
static int pp_grid(const GemmArgs &args, GemmMode mode, int max_rows, int n_groups_in_mask, int slices) {
  const int bn_out = mode == GEMM_SWIGLU ? 128 : 256;
  const long long n_tiles_n = (args.N + bn_out - 1) / bn_out;
  const long long m_tiles_ub = (long long)max_rows / kPpTileRows + n_groups_in_mask;
  long long ub = m_tiles_ub * n_tiles_n * slices;
  if (ub <= 0) return 0;
  ub = (ub + 7) / 8 * 8;
  int cap = pp_grid_blocks() - (args.spare_cus > 0 ? (args.spare_cus + 7) / 8 * 8 : 0);
  if (cap < 8) cap = 8;
  return (int)(ub < cap ? ub : cap);
}

template <int MODE, int QF = 0>
hipError_t launch_pp(const GemmArgs &args, int max_rows, int n_groups_in_mask, hipStream_t stream) {
  constexpr int BM = 256, BN = 256;
  // two stages of A and B tiles + 4 KB per wave for the epilogue's transposition
  constexpr size_t smem = 2 * (size_t)(BM + BN) * ROW_BYTES + 8 * 4096;
  auto kern = grouped_gemm_pp_kernel<MODE, QF>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int grid = pp_grid(args, (GemmMode)MODE, max_rows, n_groups_in_mask,
                           args.plan ? (args.max_splitk > 0 ? args.max_splitk : 1) : args.splitk);
  if (grid <= 0) return hipSuccess;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), smem, stream, args);
  return hipGetLastError();
}

template <int MODE>
hipError_t launch_ktail(const GemmArgs &args, int max_rows, int n_groups_in_mask, hipStream_t stream) {
  constexpr int BM = 128, BN = 128;
  constexpr int BN_OUT = (MODE == GEMM_SWIGLU) ? BN / 2 : BN;
  constexpr size_t smem = (size_t)(BM + BN) * ROW_BYTES;
  const long long n_tiles_n = (args.N + BN_OUT - 1) / BN_OUT;
  const long long m_tiles_ub = (long long)max_rows / BM + n_groups_in_mask;
  long long ub = m_tiles_ub * n_tiles_n * args.splitk;
  if (ub <= 0) return hipSuccess;
  ub = (ub + 7) / 8 * 8;
  if (ub > 0x7FFFFFFFll) return hipErrorInvalidValue;
  hipLaunchKernelGGL((grouped_gemm_ktail_kernel<BM, BN, 2, 2, MODE>), dim3((unsigned)ub), dim3(256), smem, stream,
                     args);
  return hipGetLastError();
}

}  // namespace

// args.tune.gemm_variant: 0 picks by shape; a test or tuning run forces 1 = 128 x 128 tiles, 6 = 256 x 256
// tiles of the single-phase kernel, 12 = the persistent ping-pong kernel (where the shape allows it).
static bool pp_possible(GemmMode mode, const GemmArgs &args) {
  if (args.b_quant) {
    // Codes and scales are addressed from the start of the blob with 31-bit byte offsets (the scales lie in
    // front of the codes); codes travel in aligned 16-byte pieces, the MXFP4 scale bytes of two K steps as one
    // aligned dword (hence K % 128).
    if (mode == GEMM_PLAIN_BF16 || (args.qfmt != 1 && args.qfmt != 2)) return false;
    const long long row_bytes = args.qfmt == 2 ? args.K / 2 : args.K;
    const long long codes_end = (args.q_b1_off > args.q_b0_off ? args.q_b1_off : args.q_b0_off) + args.N * row_bytes;
    return args.K % (args.qfmt == 2 ? 128 : BK) == 0 && (args.q_s0_off % 4) == 0 && (args.q_s1_off % 4) == 0 &&
           (args.q_b0_off % 16) == 0 && (args.q_b1_off % 16) == 0 && codes_end < 0x7FFFFFFFll &&
           (long long)(args.perm ? args.a_rows : 256) * args.lda * 2 < 0x7FFFFFFFll &&
           args.N >= (mode == GEMM_SWIGLU ? 128 : 256);
  }
  // The ping-pong kernel addresses a gathered A from its first row (any of its a_rows rows can be
  // named by the permutation), an A used in place from the tile's first row (256 rows), and the
  // blob from its first B row, all with 31-bit byte offsets.
  return args.K % BK == 0 && (long long)(args.perm ? args.a_rows : 256) * args.lda * 2 < 0x7FFFFFFFll &&
         (args.b1_off - args.b0_off) + (long long)args.N * args.ldb * 2 < 0x7FFFFFFFll &&
         args.b1_off >= args.b0_off && args.N >= (mode == GEMM_SWIGLU ? 128 : 256);
}

int gemm_kernel_choice(GemmMode mode, const GemmArgs &args, int max_rows, int n_groups_in_mask) {
  if (args.plan) return 12;   // a layer call that runs from a plan runs on the persistent kernel throughout
  if (args.K % BK != 0) return 100;
  int v = args.tune.gemm_variant[mode];
  const bool pp_ok = pp_possible(mode, args);
  if (v == 0) {
    // 256 x 256 ping-pong tiles unless the groups are small on average, where the finer 128 x 128
    // tiles waste less of the matrix cores on empty rows
    const long long avg_rows = n_groups_in_mask > 0 ? (long long)max_rows / n_groups_in_mask : max_rows;
    v = avg_rows > 96 ? (pp_ok ? 12 : 6) : 1;
  }
  if (v == 12 && !pp_ok) v = 6;
  return v == 6 || v == 12 ? v : 1;
}

template <int MODE>
static hipError_t launch_mode(const GemmArgs &args, int max_rows, int n_groups_in_mask, hipStream_t stream) {
  if (args.b_quant) {
    // quantised experts: the persistent kernel where its shape rules allow, whatever the groups' height (its
    // short-tile pipeline also serves groups of a few rows: Mixtral shape, 16 to 50 rows per expert, e4m3
    // 389-494 against 534-563 us per layer on the 128 x 128 tiles below, MXFP4 419-510 against 476-501; 60 and 64
    // experts of 4 to 19 rows each: 5 to 10 % ahead), else the kernel that expands the codes on their way into LDS, with the tile
    // size by the groups' average height
    if (MODE == GEMM_PLAIN_BF16 || (args.qfmt != 1 && args.qfmt != 2) || !args.qbase || args.K % BK != 0)
      return hipErrorInvalidValue;
    const long long avg_rows = n_groups_in_mask > 0 ? (long long)max_rows / n_groups_in_mask : max_rows;
    const int v = args.tune.gemm_variant[MODE];
    const bool big = avg_rows > 96 && v != 1;
    if constexpr (MODE != GEMM_PLAIN_BF16) {
      if (args.plan || ((v == 0 || v == 12) && pp_possible((GemmMode)MODE, args)))
        return args.qfmt == 2 ? launch_pp<MODE, 2>(args, max_rows, n_groups_in_mask, stream)
                              : launch_pp<MODE, 1>(args, max_rows, n_groups_in_mask, stream);
    }
    if (args.plan) return hipErrorInvalidValue;
    if (args.qfmt == 2)
      return big ? launch_q8_cfg<256, 256, 2, 4, MODE, 2>(args, max_rows, n_groups_in_mask, stream)
                 : launch_q8_cfg<128, 128, 2, 2, MODE, 2>(args, max_rows, n_groups_in_mask, stream);
    return big ? launch_q8_cfg<256, 256, 2, 4, MODE, 1>(args, max_rows, n_groups_in_mask, stream)
               : launch_q8_cfg<128, 128, 2, 2, MODE, 1>(args, max_rows, n_groups_in_mask, stream);
  }
  switch (gemm_kernel_choice((GemmMode)MODE, args, max_rows, n_groups_in_mask)) {
    case 100: return launch_ktail<MODE>(args, max_rows, n_groups_in_mask, stream);
    case 6: return launch_cfg<256, 256, 2, 4, MODE>(args, max_rows, n_groups_in_mask, stream);
    case 12: return launch_pp<MODE>(args, max_rows, n_groups_in_mask, stream);
    default: return launch_cfg<128, 128, 2, 2, MODE>(args, max_rows, n_groups_in_mask, stream);
  }
}

bool prepare_gemm_plans(GemmArgs &a1, GemmArgs &a2, GemmPlan *plans, PlanParams (&params)[2]) {
  a1.plan = a2.plan = nullptr;
  a1.plan_queue = a2.plan_queue = 0;
  params[0] = PlanParams{};
  params[1] = PlanParams{};
  if (!plans || !a1.offsets || !a2.offsets) return false;
  GemmArgs *a[2] = {&a1, &a2};
  const GemmMode mode[2] = {GEMM_SWIGLU, GEMM_PLAIN_F32};
  for (int i = 0; i < 2; ++i) {
    const int v = a[i]->tune.gemm_variant[mode[i]];
    if (!pp_possible(mode[i], *a[i]) || (v != 0 && v != 12)) return false;
  }
  for (int i = 0; i < 2; ++i) {
    // every tile of the down GEMM gets the same K slices (a2.splitk): blocks that work side by side then
    // walk the same K range, whatever tiles they hold; SwiGLU needs whole sums
    const int s = mode[i] == GEMM_PLAIN_F32 && a[i]->splitk > 1 ? a[i]->splitk : 1;
    a[i]->plan = plans + i;
    a[i]->max_splitk = s;
    const int bn_out = mode[i] == GEMM_SWIGLU ? 128 : 256;
    PlanParams &p = params[i];
    p.mask = a[i]->n_groups >= 64 ? ~0ull : ((1ull << a[i]->n_groups) - 1ull);
    p.n_groups = a[i]->n_groups;
    p.ntn = (a[i]->N + bn_out - 1) / bn_out;
    p.slices = s;
    p.equal_heights = a[i]->equal_heights;
    p.out = plans + i;
  }
  return true;
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
