// Internal launcher interface between the host logic (api.hip) and the gfx950 kernels.
// Every launcher only enqueues on `stream` and returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moe {

constexpr int kMaxExperts = 64;   // one lane per expert in the wave-wide top-k
constexpr int kDispatchChunk = 256;  // assignments per dispatch block
constexpr int kMaxCacheSlots = 32767;  // GemmArgs::slot is 16 bits wide
constexpr int kMaxHidden = 16384;      // the gate's kernel stages 4 token vectors (8 d bytes) in LDS

// ---- gate: logits (fixed fp32 summation order), top-k, gate values -------------------
// x [T,d] bf16, wr [E,d] bf16, bias NULL or fp32 [t*bias_stride + e].
// Outputs: ids [T,k] (descending logit, lower id on ties), w [T,k] fp32, logits [T,E] (may be NULL).
// one (T == 1 only, else NULL): the grouping tables of launch_dispatch, written by the gate's kernel
// itself; host_counts (may be NULL) as there.
struct SingleTokenDispatch {
  int32_t *counts, *offsets, *perm, *inv_perm;
  long long *host_counts;
  int seq;
};
// A word of the host's mailbox: an expert's count with the call's number above it, written with ONE 8-byte
// store.  The host may then trust each word by itself, in whatever order the words cross the host link
// (stores of one wave to pinned host memory need not arrive in program order, fence or not).
__host__ __device__ inline long long mailbox_word(int count, int seq) {
  return (long long)(((unsigned long long)(unsigned)seq << 32) | (unsigned)count);
}
hipError_t launch_router_topk(const uint16_t *x, const uint16_t *wr, const float *bias,
                              int bias_stride, int T, int d, int E, int k, int renormalize,
                              float *logits, int32_t *ids, float *w, hipStream_t stream,
                              const SingleTokenDispatch *one = nullptr);

// Predictor stand-in: scores[e] = sum_t x[t].wp[e] (same summation order per token, tokens
// ascending), top-m ids to `top_out` (device-visible, e.g. pinned host memory).
// ExpertMLP predictor (Section IV-B): n_fc layers, dims[0..n_fc]; w[l] bf16 [dims[l+1], dims[l]],
// bias / scale / shift fp32 (scale, shift: hidden layers only); state fp32 [dims[0]] (device-visible);
// act0 / act1: fp32 scratch of max(dims) each; scores [dims[n_fc]]; top_out [m] (device-visible).
hipError_t launch_mlp_predictor(const float *state, const int32_t *dims, int n_fc, const uint16_t *const *w,
                                const float *const *bias, const float *const *scale, const float *const *shift,
                                float *act0, float *act1, int m, float *scores, int32_t *top_out,
                                hipStream_t stream);
// 4-bit expert weights -> bf16: out[r, c] = bf16_rne((code[r, c] - zeros[r, c/128]) * scales[r, c/128]);
// two codes per byte, even column in the low nibble; cols % 128 == 0.
hipError_t launch_dequant_int4_g128(const uint8_t *codes, const float *scales, const uint8_t *zeros,
                                    long long rows, int cols, uint16_t *out, hipStream_t stream);
hipError_t launch_predictor(const uint16_t *x, const uint16_t *wp, int T, int d, int E, int m,
                            float *scores, int32_t *top_out, hipStream_t stream);

struct PlanParams;

// ---- dispatch: stable counting sort of the T*k assignments by expert ------------------
// blk_hist / blk_base: [ceil(n/kDispatchChunk) * E] scratch.  counts [E], offsets [E+1],
// perm [n], inv_perm [n].  host_counts: optional device-visible mirror of counts (pinned, kMaxExperts
// 8-byte words, of which the first E are written: mailbox_word(count, seq)).
// active (optional, decode-sized inputs only: n <= 2048): [kMaxExperts] receives the ids of the experts
// that have rows, ascending, padded with -1.
hipError_t launch_dispatch(const int32_t *ids, int n, int E, int32_t *blk_hist, int32_t *blk_base,
                           int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                           long long *host_counts, int seq, hipStream_t stream, int32_t *active = nullptr,
                           const PlanParams *plans = nullptr);   // plans: NULL or two PlanParams (see below)

// Tuning and test hooks of one context (moe_tune); all zero = every choice by shape.  Host side only:
// the launchers read them, the kernels never do.
struct Tune {
  int gemm_variant[3];   // per GemmMode: 0 = by shape, 1 = 128 x 128 tiles, 6 = 256 x 256 single-phase, 12 = ping-pong
  int gemv_rows;         // weight rows per wave of the per-token mat-vec (0 = by shape, 1, 2 or 4)
  int skinny_min_tok;    // tokens per expert from which the matrix-core mat-vec is used (0 = by rule)
  int skinny_forced;     // the matrix-core mat-vec wherever the shapes allow it
  int skinny_waves;      // K slices (waves) per block of the matrix-core mat-vec (0 = by shape)
};

// Work plan of one grouped launch of the persistent GEMM, computed on the device from the groups'
// sizes (launch_gemm_plans) and read by every block of the launch.
// A group of cnt rows is cut into cnt / 256 full row tiles and one remainder tile; an item is one
// (row tile, column tile, K slice).  Blocks take items from eight queues, one per XCD, each a
// contiguous range of the item list of about equal estimated cost; a block whose own range is used
// up goes on with its neighbours'.
constexpr int kPpTileRows = 256;
struct GemmPlan {
  int n_items;
  int s_full, s_rem;                 // K slices (= fp32 output planes) of a full / a remainder row tile
  int xcd_begin[9];                  // item range of each XCD's queue
  int item_begin[kMaxExperts + 1];   // first item of each group
  int queue[8 * 16];                 // items taken from each range so far (one counter per 64-byte line)
};

// ---- grouped GEMM on bf16 MFMA --------------------------------------------------------
struct GemmArgs {
  const uint16_t *A;      // activations, row-major bf16
  int lda;                // elements between A rows
  int a_rows;             // rows of A that a gathered read (perm) can reach: the token count
  const int32_t *perm;    // non-NULL: sorted row p reads A row perm[p] / k_top (token gather)
  int k_top;
  const int32_t *offsets; // device [n_groups+1] sorted-row offsets; NULL = one group
  int single_row0, single_rows;   // the one group when offsets == NULL
  unsigned long long group_mask;  // experts that take part (bit e)
  const int32_t *sel_ids;         // mat-vec kernels: non-NULL = device list of the groups that take part
                                  // (launch index -> expert), used instead of group_mask
  int n_groups;
  const char *wbase;      // expert e's blob at wbase + slot[e] * wstride
  long long wstride;
  int16_t slot[kMaxExperts];   // cache slot of expert e (moe_config.cache_slots <= 32767)
  long long b0_off, b1_off;  // byte offsets in the blob of the B rows (gate|down) and (up)
  int ldb;                // elements between B rows (= K)
  int N;                  // output columns (SwiGLU: I; the block reads N gate rows and N up rows)
  int K;
  void *out;              // rows indexed by sorted position
  int ldo;
  int splitk;             // K slices, each written to its own output plane (the same for every tile)
  int max_splitk;         // with a plan: output planes there are room for (slices are chosen per tile class)
  GemmPlan *plan;         // device memory, or NULL.  The K slices of a tile come from it (s_full, s_rem) ...
  int equal_heights;      // persistent kernel: cut a group into row tiles of equal height instead of full tiles
                          // and a remainder
  int plan_queue;         // ... and, if set, the items are taken from its queues (the launch covers every group
                          // with rows, as the plan does); otherwise they are dealt out in a fixed order
  long long out_split_stride;  // elements between planes
  int spare_cus;          // persistent GEMM: compute units to leave to kernels of other streams
  // Quantised experts.  Expert e with bit e of q8_mask set is read from qbase + slot[e] * qstride, not
  // from a bf16 blob.  qfmt 1: e4m3 codes of the B rows at q_b0_off / q_b1_off (K bytes per row), one
  // fp32 scale per B row at q_s0_off / q_s1_off; the weight used is bf16_rne(value(code) * scale).
  // K % 16 == 0.  qfmt 2: MXFP4 (e2m1 codes, two per byte, K / 2 bytes per row at q_b*_off; one scale
  // byte per 32 columns, K / 32 bytes per row at q_s*_off; weight = value(code) * 2^(scale - 127), exact
  // in bf16).  K % 32 == 0.  The mat-vec kernels go by the mask; the GEMM kernels by b_quant.
  int qfmt;               // 0 none, 1 e4m3 with row scales, 2 MXFP4
  int b_quant;            // GEMM kernels: every expert's B operand is its quantised blob at qbase (K % 64 == 0)
  unsigned long long q8_mask;
  const char *qbase;
  long long qstride;
  long long q_b0_off, q_b1_off, q_s0_off, q_s1_off;
  Tune tune;              // host side only
};

enum GemmMode { GEMM_SWIGLU = 0, GEMM_PLAIN_F32 = 1, GEMM_PLAIN_BF16 = 2 };

// max_rows: host upper bound of the rows summed over the groups in the mask.
hipError_t launch_grouped_gemm(GemmMode mode, const GemmArgs &args, int max_rows, int n_groups_in_mask,
                               hipStream_t stream);


// What the grouping kernel needs to know to write the plan of one grouped launch: the launch's shape and
// where the plan goes (out == NULL: no plan).
struct PlanParams {
  unsigned long long mask;   // groups that take part
  int n_groups;
  int ntn;                   // column tiles of the launch
  int slices;                // K slices of every tile
  int equal_heights;         // how the groups are cut into row tiles (GemmArgs::equal_heights)
  GemmPlan *out;
};

// The plans of a prefill layer's two grouped GEMMs (gate/up: a1, down: a2, both with their offsets and
// every group in the mask): if both can run on the persistent kernel, points a1.plan / a2.plan at
// plans[0] / plans[1] (device memory), fills in params for launch_dispatch, which then writes the plans
// from the groups' sizes, and returns true; otherwise leaves both NULL.  Every tile of the down GEMM is cut
// into a2.splitk K slices, so the summation order of an output element never depends on which
// experts happened to be resident.
bool prepare_gemm_plans(GemmArgs &a1, GemmArgs &a2, GemmPlan *plans, PlanParams (&params)[2]);

// The kernel launch_grouped_gemm picks: 1 = 128 x 128 tiles, 6 = 256 x 256 single-phase, 12 = persistent
// ping-pong, 100 = the register-staged kernel for K that is no multiple of 64.
int gemm_kernel_choice(GemmMode mode, const GemmArgs &args, int max_rows, int n_groups_in_mask);

// ---- decode: bandwidth-bound expert mat-vec --------------------------------------------
// Same argument block; rows per group are few (decode batch).  SWIGLU -> bf16 h, PLAIN_F32 -> fp32 y.
// extra: optional second single-group problem (the shared experts) streamed by the same launch.
hipError_t launch_grouped_gemv(GemmMode mode, const GemmArgs &args, int max_rows_per_group,
                               int n_groups_in_mask, hipStream_t stream, const GemmArgs *extra = nullptr);

// One token: the down projection of its k experts (args.sel_ids, device), of the shared experts
// (extra, may be NULL: a single group of one row) and the weighted sum in one launch; gate_w [k] fp32
// (device), out [N] bf16.  The same bits as launch_grouped_gemv(GEMM_PLAIN_F32) followed by
// launch_combine.  Requires K * 2 <= 64 KB for both problems.
hipError_t launch_fused_down_combine(const GemmArgs &args, const float *gate_w, int k_top, uint16_t *out,
                                     hipStream_t stream, const GemmArgs *extra = nullptr);
// Whether launch_grouped_gemv reads the quantised blobs of the experts of args.q8_mask (a format is set
// and K fits its pieces), whatever the mask and the token count.
bool gemv_reads_copies(const GemmArgs &args);

// ---- combine: out[t] = sum_j w[t,j] * Y[inv_perm[t*k+j]] (+ shared), fixed order, bf16 out ----
hipError_t launch_combine(const float *Y, int y_planes, long long y_plane_stride, const float *w,
                          const int32_t *inv_perm, const float *Yshared, int ys_planes,
                          long long ys_plane_stride, int T, int d, int k, uint16_t *out,
                          hipStream_t stream);

}  // namespace moe
