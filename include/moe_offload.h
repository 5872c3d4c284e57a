/*
 * moe_offload.h - C ABI of the MI355X (gfx950) MoE-layer library.
 *
 * One Mixture-of-Experts FFN layer served from an offloaded expert pool, after the
 * inference runtime of DuoServe-MoE (Section V of the paper): every expert lives in
 * a pinned "CPU expert cache", a small "GPU expert cache" of S slots per layer (or, with
 * cfg.shared_slots, of S slots for all layers) is filled by a communication stream just
 * before the experts run (Section V-A), the
 * prefill stage pipelines "compute expert i / fetch expert i+1" (Section V-B) and the
 * decode stage prefetches the experts a per-layer predictor names and re-fetches on
 * a wrong guess (Section V-C).  The numbers a layer produces never depend on the
 * cache state.
 *
 * Conventions
 *  - "dev" pointers are device (HBM) memory, "host" pointers are host memory, and
 *    "pinned" means page-locked host memory (hipHostMalloc / torch pin_memory).
 *    All of them are owned by the CALLER and must stay valid while the ctx uses them;
 *    the library owns only bookkeeping (slot tables, events, a few KB of pinned
 *    mailboxes).  bf16 tensors are raw 16-bit patterns, row-major.
 *  - Streams are hipStream_t handles passed as void* (NULL = the default stream).
 *    Calls enqueue work and return; they block the host only where stated.  A layer
 *    call may run part of its work (the shared experts) on a stream of the library's
 *    own, forked from and joined back into compute_stream inside the call: everything
 *    a call enqueues is complete when compute_stream reaches the end of the call.
 *    Device inputs (activations, route bias, predictor inputs) are read on the stream the call is
 *    given: whatever produced them on another stream (an upload on a framework's own stream, say)
 *    must be ordered before that stream by the caller.
 *  - Every function returns 0 on success or a negative MOE_E_* code and never throws
 *    or aborts; moe_last_error() returns a thread-local message for the last failure.
 *  - One ctx serves one (compute stream, copy stream) pair at a time; calls on the
 *    same ctx must not overlap in time from several host threads.  The compute stream of a
 *    layer call must stay alive until the ctx is destroyed or the layer's cache has been used
 *    again: a later copy into a slot that the call read may record, on that stream, the event
 *    it then waits for.
 */
#ifndef MOE_OFFLOAD_H
#define MOE_OFFLOAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_OK 0
#define MOE_E_ARG (-1)         /* null/unaligned pointer, T <= 0, k > E, cache_slots < 1, bad id ... */
#define MOE_E_UNSUPPORTED (-2) /* E > 64, d % 8 != 0, I % 8 != 0, d > 16384, cache_slots > 32767 ... */
#define MOE_E_HIP (-3)         /* a HIP runtime call failed (text in moe_last_error) */
#define MOE_E_UNBOUND (-4)     /* layer not bound */
#define MOE_E_WORKSPACE (-5)   /* workspace too small */

typedef struct moe_ctx moe_ctx;

/* Shape of the layer family (Fig. 1 of the paper: Top-k of n routed experts plus
 * optional shared experts).  Experts are SwiGLU FFN blocks without biases. */
typedef struct {
  int32_t d;           /* hidden size, multiple of 8, at most 16384 (the gate stages token vectors in LDS) */
  int32_t I;           /* routed-expert intermediate size, multiple of 8 */
  int32_t E;           /* routed experts per layer, 1..64 */
  int32_t k;           /* experts per token, 1..E */
  int32_t n_layers;    /* layers that can be bound */
  int32_t cache_slots; /* S: GPU expert cache slots per layer, 1..32767 (Section V-A) */
  int32_t I_shared;    /* 0, or total intermediate size of the always-on shared experts */
  int32_t renormalize; /* 1: gate values = softmax over the k selected; 0: over all E */
  int32_t shared_slots;/* 0: every layer has its own cache of cache_slots slots; 1: ONE cache of
                          cache_slots slots serves all layers in turn (Section V-A: a GPU expert
                          cache of k experts, refilled layer after layer) */
  int32_t host_format; /* MOE_FMT_*: how an expert is stored in the CPU expert cache and travels
                          over the host link */
} moe_config;

/* moe_config.host_format.
 * MOE_FMT_BF16: the blob is the three bf16 matrices, copied straight into a slot.
 * MOE_FMT_E4M3_ROWS: 8-bit weights (the paper serves quantised models, Section VI; the format is this
 *   library's): [scale fp32: 2I rows of W_gate/W_up, then d rows of W_down][W_gate codes I x d]
 *   [W_up codes I x d][W_down codes d x I], codes = OCP e4m3 (1-4-3 bits, bias 7, max 448, 0x7F NaN);
 *   d and I multiples of 64.  A weight is bf16 nearest-even of fp32(value(code) * scale[row]).  The GPU
 *   expert cache holds an expert in this form and in no other: a slot is moe_host_blob_bytes rounded up
 *   to 256 bytes, a fetch is one copy (half the bytes of bf16 on the link and in HBM), and every kernel
 *   reads the codes as they landed.  The prefill GEMMs expand each tile of codes to those bf16 weights
 *   on its way into LDS, the decode mat-vecs in registers; the results are those of MOE_FMT_BF16 run on
 *   the expanded weights.  initial_resident names experts whose 8-bit blob the caller has put into the
 *   slot. */
#define MOE_FMT_BF16 0
#define MOE_FMT_E4M3_ROWS 1
/* MOE_FMT_INT4_G128: 4-bit weights, the storage form of AWQ / GPTQ-style quantisation: unsigned 4-bit
 *   codes, two per byte (even column in the low nibble), in groups of 128 along a row with one fp32
 *   scale and one zero point (a byte, 0..15) per group; d and I multiples of 128.  Blob:
 *   [scales of [W_gate; W_up] (2I x d/128 fp32)][scales of W_down (d x I/128 fp32)][zero points, same
 *   order (bytes)][padding to a multiple of 16][codes of [W_gate; W_up] (2I x d/2)][codes of W_down
 *   (d x I/2)].  weight = bf16 nearest-even of fp32((code - zero) * scale).  A fetched expert lands in
 *   a staging area behind the bf16 slots and a kernel expands it into its slot.  The kernels run on a
 *   stream of the library's own, each behind the copy it reads, so that the next copy does not wait for
 *   them; every call that fetched makes copy_stream wait for the last of them before it returns, so a
 *   synchronised copy_stream still means "the experts are in their slots".  Slots, matmuls and results
 *   are those of MOE_FMT_BF16 run on the expanded weights; the link carries a quarter of the bytes, HBM
 *   holds the bf16 slots.  initial_resident names experts whose expanded bf16 blob is in the slot. */
#define MOE_FMT_INT4_G128 2
/* MOE_FMT_MXFP4: the OCP microscaling 4-bit format: e2m1 codes (bit 3 sign, bits 2..1 exponent, bit 0
 *   mantissa: 0, 0.5, 1, 1.5, 2, 3, 4, 6), two per byte (even column in the low nibble); 32 consecutive
 *   values of a row share the scale 2^(s - 127), s one byte in 1..254; d and I multiples of 64.  Blob:
 *   [scale bytes of [W_gate; W_up] (2I x d/32)][scale bytes of W_down (d x I/32)][padding to a multiple
 *   of 16][codes of [W_gate; W_up] (2I x d/2)][codes of W_down (d x I/2)].  weight = value(code) *
 *   2^(s - 127), exact in bf16.  Held like MOE_FMT_E4M3_ROWS: the GPU expert cache is the blobs
 *   themselves, one per slot, rounded up to 256 bytes (about a quarter of the bytes of bf16 on the link
 *   and in HBM), a fetch is one copy, and every kernel reads the codes as they landed, expanding them
 *   with the hardware's scaled fp4 conversion: the prefill GEMMs tile by tile on the way into LDS, the
 *   decode mat-vecs in registers.  The results are those of MOE_FMT_BF16 run on the expanded weights.
 *   initial_resident names experts whose MXFP4 blob the caller has put into the slot. */
#define MOE_FMT_MXFP4 3

/* Cache counters (host side).  hits/misses count active experts per layer call.
 * prefetch_ready / prefetch_stalled: of the prefetched experts a layer call went on to use, how
 * many had landed in their slot when the call asked for them and how many had not (Section V-C:
 * a prefetch that is late stalls the computation stream), taken on the host when the call
 * enqueues its wait.  wait_ms: host time the layer calls spent blocked until the gate's counts
 * arrived (only calls that have to compare them with the cache block).  compute_ms: kernel time
 * of the layer's calls, from the events of moe_set_profiling (0 while profiling is off). */
typedef struct {
  int32_t hits, misses, prefetch_issued, prefetch_useful, prefetch_dropped, layer_calls;
  int64_t bytes_h2d;
  int32_t prefetch_ready, prefetch_stalled;
  float wait_ms, compute_ms;
} moe_stats;

/* Kernel classes timed when profiling is on (moe_set_profiling). */
enum {
  MOE_K_ROUTER = 0, MOE_K_DISPATCH, MOE_K_GEMM1, MOE_K_GEMM2, MOE_K_GEMV1, MOE_K_GEMV2,
  MOE_K_COMBINE, MOE_K_PREDICTOR, MOE_K_COUNT
};

const char *moe_last_error(void);

/* Creates the bookkeeping for cfg on the current HIP device.  *out receives the ctx. */
int moe_create(const moe_config *cfg, moe_ctx **out);
/* Destroys events and tables.  Frees nothing the caller allocated.  Blocks until the
 * device is idle. */
int moe_destroy(moe_ctx *ctx);

/* Bytes of one expert in the CPU expert cache: 6*d*I (bf16), 4*(2I+d) + 3*d*I (e4m3 rows) or
 * 15*d*I/128 rounded up to 16, plus 3*d*I/2 (int4 groups), or 3*d*I/32 rounded up to 16, plus
 * 3*d*I/2 (MXFP4). */
size_t moe_host_blob_bytes(const moe_config *cfg);
/* Bytes of one GPU expert cache (dev_slots of moe_bind_layer).  MOE_FMT_BF16: cache_slots slots of 6*d*I
 * bytes.  MOE_FMT_E4M3_ROWS, MOE_FMT_MXFP4: cache_slots slots of moe_host_blob_bytes rounded up to 256.
 * MOE_FMT_INT4_G128: cache_slots bf16 slots followed by one staging area (the blob, rounded up to 256)
 * per slot. */
size_t moe_cache_bytes(const moe_config *cfg);

/* Bytes of device workspace a layer call on T tokens needs (256-byte aligned base). */
size_t moe_workspace_bytes(const moe_config *cfg, int T);

/*
 * Attaches a layer's memory (Section V-A: CPU expert cache, GPU expert cache).
 *  host_expert_blob[E]  pinned; each moe_host_blob_bytes: W_gate (I x d), W_up (I x d), W_down (d x I),
 *                       row-major bf16 (or the 8-bit layout of cfg.host_format), one contiguous
 *                       blob per expert (= one DMA per expert).
 *  dev_router_w         [E, d] bf16 gate weight.
 *  dev_shared_blob      NULL, or 6*d*I_shared bytes in the same layout (always resident).
 *  dev_slots            moe_cache_bytes: the layer's GPU expert cache, slot s at s times the slot size (with
 *                       shared_slots: the one cache, the same pointer for every layer).
 *  initial_resident     NULL (all slots empty) or [S] expert ids / -1: slot s already holds
 *                       that expert's blob (the caller put it there): the bf16 matrices, or for
 *                       MOE_FMT_E4M3_ROWS the 8-bit blob.
 * The pointers are read, not copied.
 */
int moe_bind_layer(moe_ctx *ctx, int layer, const void *const *host_expert_blob,
                   const void *dev_router_w, const void *dev_shared_blob, void *dev_slots,
                   const int32_t *initial_resident);

/*
 * Prefetch (Sections V-B, V-C): makes the named experts of `layer` resident by copies
 * enqueued on copy_stream, ordered behind the last use of each overwritten slot.
 * Resident ids cost nothing; repeated ids are ignored.  Victim: an empty slot, else the
 * least recently used slot whose expert is not named in this request; if none is left
 * the id is dropped (counted).  host_ids[n] are plain host ints.  Does not block.
 */
int expert_cache_prefetch(moe_ctx *ctx, int layer, const int32_t *host_ids, int n,
                          void *copy_stream);

/*
 * Stand-in for the paper's layer-level predictor (Section IV-B, used as in Section V-C):
 * score[e] = sum_t x[t] . Wp[e]; the m best (score descending, lower id on ties) go to
 * pinned_topm[m] (pinned host ints, valid once `stream` has been synchronised) and, if
 * dev_scores != NULL, the E scores to dev_scores.  dev_x [T, d] bf16, dev_wp [E, d] bf16.
 * `layer` is the layer whose experts are being predicted (0 <= layer < n_layers; it need not be
 * bound): the predictor is per layer, the caller passes that layer's dev_wp.
 */
int predictor_score(moe_ctx *ctx, int layer, const void *dev_x, int T, const void *dev_wp, int m,
                    float *dev_scores, int32_t *pinned_topm, void *stream);

/*
 * The paper's predictor, ExpertMLP (Section IV-B), for one state vector: n_fc fully connected
 * layers of sizes host_dims[0] -> host_dims[1] -> ... -> host_dims[n_fc] (= number of experts).
 * Every layer but the last is followed by batch normalisation in inference form (per neuron
 * z * scale + shift) and ReLU; dropout is the identity at inference.  The last layer's outputs
 * are the experts' logits (their sigmoid is the predicted activation probability, which ranks
 * the same): the m best go to pinned_topm[m], all of them to dev_scores if != NULL.
 *   state       fp32 [host_dims[0]], device-visible (device or pinned host memory).
 *   dev_w[l]    bf16 [host_dims[l+1], host_dims[l]] row-major; dev_bias[l] fp32 [host_dims[l+1]];
 *   dev_scale[l], dev_shift[l]  fp32, for l < n_fc - 1 (the entries for the last layer are ignored).
 *   dev_act     fp32 scratch, 2 * max(host_dims) elements.
 * The host arrays of pointers are read during the call only.  2 <= n_fc <= 16.  Does not block.
 */
int predictor_mlp_score(moe_ctx *ctx, const float *state, const int32_t *host_dims, int n_fc,
                        const void *const *dev_w, const float *const *dev_bias,
                        const float *const *dev_scale, const float *const *dev_shift, float *dev_act,
                        int m, float *dev_scores, int32_t *pinned_topm, void *stream);

/*
 * State Constructor (Sections IV-A, IV-B, V-C): keeps the experts selected at each layer of the
 * current decode step and builds the predictor's input s_l = [h_l, p_l, a_{l-1,l}] as one fp32
 * vector of moe_state_dim() = L*k + M + k*M entries:
 *   h_l        the ids selected at layers 0 .. l-1, in the order recorded, each id i stored as
 *              (i + 1) / M, zero-padded to L*k entries;
 *   p_l        row l of the popularity matrix (Eq. 2);
 *   a_{l-1,l}  for each of the k experts recorded at layer l-1, its row of the affinity matrix
 *              between layers l-1 and l (Eq. 3); zeros for l = 0.
 * host_popularity [L, M] and host_affinity [L-1, M, M] (fp32, from the preprocessing phase) are
 * copied.  moe_state_record stores the k ids of a layer (any order of layers; a layer can be
 * recorded again), moe_state_clear forgets all of them (after each decode round),
 * moe_state_vector writes s_layer to host_out (plain or pinned host memory) and fails with
 * MOE_E_ARG if one of the layers 0 .. layer-1 has not been recorded.  Host-only; no GPU work.
 */
typedef struct moe_state moe_state;
int moe_state_create(int n_layers, int n_experts, int k, const float *host_popularity,
                     const float *host_affinity, moe_state **out);
int moe_state_destroy(moe_state *st);
int moe_state_dim(const moe_state *st);
int moe_state_record(moe_state *st, int layer, const int32_t *host_ids);
int moe_state_clear(moe_state *st);
int moe_state_vector(const moe_state *st, int layer, float *host_out);

/*
 * One MoE layer in the prefill stage (Section V-B): gate -> Top-k -> tokens grouped by
 * expert -> every active expert as a grouped bf16 MFMA GEMM from its cache slot -> weighted
 * sum (+ shared experts) -> dev_y [T, d] bf16.  Experts that are not resident stream
 * through the slots in ascending id, each fetched once on copy_stream while the previous
 * one computes.  Groups of any size run on the MFMA kernels: for a handful of tokens
 * moe_decode_layer gives the same result faster (and itself moves to the GEMM kernels when some
 * expert receives more than 16 tokens, 24 on MXFP4 experts).  When some routed
 * expert is not resident the call blocks the host until the gate's counts are known, and again
 * before each fetch into a slot whose last reader (an expert of this call, S fetches earlier) is
 * still computing: the copy is then enqueued with no wait in front of it, which starts it sooner
 * than a wait on the stream would.  Such a call returns when all its work is enqueued, i.e. after
 * all but the last S experts have been computed.
 *  dev_route_bias  NULL, or fp32 added to the gate logits: element [t*bias_stride + e]
 *                  (bias_stride 0 = one row for all tokens, E = one row per token).
 *  dev_workspace   >= moe_workspace_bytes(cfg, T), 256-byte aligned; holds the routing
 *                  tables afterwards (see moe_debug_routing).
 *  opt             NULL, or receives this call's own counters (hits, misses, prefetch_useful,
 *                  prefetch_ready / _stalled, bytes_h2d, wait_ms; layer_calls = 1; compute_ms = 0,
 *                  kernel times are asynchronous: moe_get_stats).  With opt the call waits for the
 *                  gate's counts before it returns even when every expert is resident.
 * When every routed expert is resident the call only enqueues: its cache counters (hits, recency)
 * are filled in once the gate's counts have reached the host, by the next call that looks at the
 * cache or its counters (expert_cache_prefetch, a layer call with a miss, moe_get_stats, ...), in
 * the order of the calls.  If a HIP call fails midway the error is returned, work already enqueued
 * still runs and the library's side stream is joined back into compute_stream; experts whose copy
 * had been enqueued count as resident, so the cache stays consistent with what the streams will do.
 */
int moe_prefill_layer(moe_ctx *ctx, int layer, const void *dev_x, int T,
                      const float *dev_route_bias, int bias_stride, void *dev_y,
                      void *dev_workspace, size_t ws_bytes, void *compute_stream,
                      void *copy_stream, moe_stats *opt);

/*
 * One MoE layer in the decode stage (Section V-C), T = batch (small).  Same contract and
 * results as moe_prefill_layer; experts run as bandwidth-bound GEMVs.  The gate's choice is
 * compared with the cache ("synchronisation point 1"): hits run first, misses are
 * re-fetched on copy_stream and run as they land.  Experts with at most 16 tokens (32 where
 * quantised copies are read) run as mat-vecs: per-token dot products for a few tokens, 16x16x32
 * MFMAs over the same single pass for more; a batch that gives some expert more goes to the GEMM
 * kernels.  The host looks at the gate's counts
 * (a short wait on a pinned mailbox) unless every expert is resident and T = 1: then the
 * mat-vec launches read the token's k experts from the gate's id list on the device and the
 * call only enqueues (its cache counters are filled in later, as for moe_prefill_layer; up to 32
 * such calls can be in flight before a call waits for the oldest one's counts).
 */
int moe_decode_layer(moe_ctx *ctx, int layer, const void *dev_x, int T,
                     const float *dev_route_bias, int bias_stride, void *dev_y,
                     void *dev_workspace, size_t ws_bytes, void *compute_stream,
                     void *copy_stream, moe_stats *opt);

/*
 * moe_decode_layer for callers that cannot allocate device memory or have nowhere to keep a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results and cache behaviour as moe_decode_layer, but the workspace is a static
 * array of MOE_STATIC_WORKSPACE_BYTES (8 MiB) that the library holds on every GPU it is loaded on
 * until the process ends (its device address is taken once per device, in moe_create).  The call
 * allocates nothing: no hipMalloc / hipFree, no events or streams are created, and kernel timing
 * (moe_set_profiling) is off for its launches.  A T for which moe_workspace_bytes(cfg, T) exceeds the
 * static size is refused with MOE_E_WORKSPACE (Mixtral-shaped layers: T <= 93, Qwen-shaped: T <= 131).
 * No part of the workspace has to start at zero: every table is written before it is read inside a
 * call, so consecutive calls may differ in T.  All calls on one GPU share the one array, whatever
 * their context or stream: two that overlap in time race on it.
 */
#define MOE_STATIC_WORKSPACE_BYTES (8u << 20)
int moe_decode_layer_static(moe_ctx *ctx, int layer, const void *dev_x, int T,
                            const float *dev_route_bias, int bias_stride, void *dev_y,
                            void *compute_stream, void *copy_stream, moe_stats *opt);
/*
 * Parity hook: copies the routing tables the last layer call left in `dev_workspace`
 * (T as in that call) to caller device buffers on `stream`; any destination may be NULL.
 * ids [T,k] i32, w [T,k] f32, counts [E], offsets [E+1], perm [T*k], inv_perm [T*k].
 */
int moe_debug_routing(moe_ctx *ctx, const void *dev_workspace, int T, int32_t *dev_ids,
                      float *dev_w, int32_t *dev_counts, int32_t *dev_offsets, int32_t *dev_perm,
                      int32_t *dev_inv_perm, void *stream);

/* Parity hook: the gate logits (bias included) of the last layer call, [T, E] fp32, copied from
 * `dev_workspace` on `stream`.  The Top-k is an integer decision taken on these values, so they are
 * defined bit for bit (Section II-A; fixed summation order, see the kernel's header). */
int moe_debug_logits(moe_ctx *ctx, const void *dev_workspace, int T, float *dev_logits, void *stream);

/* Cache counters of `layer` (or summed over all layers if layer < 0).  Blocks until the gate's counts
 * of every layer call so far have reached the host and, while profiling is on, until the kernels
 * timed so far have finished. */
int moe_get_stats(moe_ctx *ctx, int layer, moe_stats *out);
int moe_reset_stats(moe_ctx *ctx);
/*
 * Forgets which experts the slots of `layer` hold (all slots become empty), e.g. because the
 * slot memory now backs another set of experts.  Ordering against kernels that still read the
 * slots is kept: later copies into them wait for those readers.
 */
int moe_cache_invalidate(moe_ctx *ctx, int layer);
/* Expert id held by each slot of `layer` (-1 = empty) into host_slot_expert[S]. */
int moe_cache_state(moe_ctx *ctx, int layer, int32_t *host_slot_expert);

/*
 * Kernel timing.  on != 0: every kernel launch of the layer calls is bracketed by HIP
 * events on its own stream.  moe_get_kernel_times blocks until those events have
 * completed, writes the durations summed since the last call into ms[MOE_K_COUNT] /
 * launches[MOE_K_COUNT] and clears the record.
 */
int moe_set_profiling(moe_ctx *ctx, int on);
int moe_get_kernel_times(moe_ctx *ctx, float *ms, int32_t *launches);

/*
 * Plain bf16 GEMM C[M,N] = A[M,K] * B[N,K]^T on the same MFMA kernel as the experts
 * (the stand-in for the non-MoE block whose time hides the first expert fetch,
 * Section V-B).  All device pointers, C bf16.  K a multiple of 8.
 */
int moe_dense_gemm_bf16(const void *dev_a, const void *dev_b, void *dev_c, int M, int N, int K,
                        void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_OFFLOAD_H */
