// Host side of the C ABI (include/moe_offload.h): argument checks, the expert-slot cache
// (Section V-A of the paper), the stream/event ordering of prefetch, fetch and compute
// (Sections V-B and V-C), and the sequencing of the kernels of one layer.
//
// Ordering rules (the paper's "synchronisation points"):
//   - a slot is read by the compute stream only after hipStreamWaitEvent(compute, copied[slot]);
//   - a slot is overwritten by the copy stream only after hipStreamWaitEvent(copy, <event
//     recorded on the compute stream behind the last kernel that read the slot>).
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <memory>
#include <new>
#include <atomic>
#include <chrono>
#include <vector>

#include "../../include/moe_offload.h"
#include "kernels.h"
#include "moe_tuning.h"

using namespace moe;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

// Test hook (moe_inject_failure): the n-th HIP call of this thread from now on is not made and
// reports an error instead, so that the state a failed call leaves behind can be examined.
thread_local int g_fail_countdown = 0;

#define HIP_TRY(expr)                                                                      \
  do {                                                                                     \
    if (g_fail_countdown > 0 && --g_fail_countdown == 0)                                   \
      return fail(MOE_E_HIP, "injected failure instead of %s (%s:%d)", #expr, __FILE__, __LINE__); \
    hipError_t _e = (expr);                                                                \
    if (_e != hipSuccess)                                                                  \
      return fail(MOE_E_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e), __FILE__, __LINE__); \
  } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// K slices of the down projection.  Few, long tiles (Mixtral-like: K = 14336, ~320 tiles of
// 256 x 256 on 256 CUs) leave most of the last round idle; slicing K makes the tiles finer.
// The slices land in separate fp32 planes that the combine kernel adds in a fixed order.
constexpr int kMaxSplitK = 4;

// Host-side tuning and test hooks of one context (moe_tune), beside the launchers' Tune.
struct ApiTune {
  int splitk = 0;            // K slices of the down GEMM, 0 = heuristic, at most kMaxSplitK
  int no_fused_down = 0;     // a one-token call runs the down mat-vec and the weighted sum as two launches
  int host_looks_always = 0; // a one-token decode call waits for the gate on the host like any other
  int matvec_max_rows = 0;   // largest group a decode call gives to the mat-vec launches, 0 = default
  int down_sched = 0;        // down GEMM: 0 = by shape, 1 = tiles of equal height in a fixed order, 2 = full +
                             // remainder tiles from the queues, 3 = equal heights from the queues
  int up_sched = 0;          // gate/up GEMM: 0 = by shape, 1 = equal heights in a fixed order, 2 = full + remainder
                             // tiles from the queues
};

int choose_splitk(const moe_config &cfg, int T) {
  const long long rows = (long long)T * cfg.k;
  if (rows < 1024) return 1;  // decode-sized calls run the mat-vec path
  const long long tiles = (rows / 256 + (cfg.E + 1) / 2) * ((cfg.d + 255) / 256);
  long long s = (3 * 256 + tiles - 1) / tiles;  // aim at >= 3 rounds of tiles over 256 CUs
  const long long max_by_k = cfg.I / 1024;      // keep every slice >= 16 K steps
  if (s > max_by_k) s = max_by_k;
  if (s > kMaxSplitK) s = kMaxSplitK;
  return s < 1 ? 1 : (int)s;
}

struct WsLayout {
  size_t logits, ids, w, counts, offsets, active, blk_hist, blk_base, perm, inv_perm, plans, H, Hs, Y, Ys, total;
  int planes;   // fp32 planes of Y there is room for
  int splitk, nblk;
};

// The workspace has the planes the heuristic asks for; forced_splitk (a tuning hook) can only use
// fewer of them, so the size never depends on it.
WsLayout ws_layout(const moe_config &c, int T, int forced_splitk = 0) {
  WsLayout L{};
  const size_t n = (size_t)T * c.k;
  L.planes = choose_splitk(c, T);
  L.splitk = forced_splitk > 0 && forced_splitk < L.planes ? forced_splitk : L.planes;
  L.nblk = (int)((n + kDispatchChunk - 1) / kDispatchChunk);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  L.logits = take((size_t)T * c.E * 4);
  L.ids = take(n * 4);
  L.w = take(n * 4);
  L.counts = take((size_t)c.E * 4);
  L.offsets = take((size_t)(c.E + 1) * 4);
  L.active = take((size_t)kMaxExperts * 4);
  L.blk_hist = take((size_t)L.nblk * c.E * 4);
  L.blk_base = take((size_t)L.nblk * c.E * 4);
  L.perm = take(n * 4);
  L.inv_perm = take(n * 4);
  L.plans = take(2 * sizeof(GemmPlan));
  L.H = take(n * c.I * 2);
  L.Hs = take((size_t)T * c.I_shared * 2);
  L.Y = take((size_t)L.planes * n * c.d * 4);
  L.Ys = take(c.I_shared ? (size_t)T * c.d * 4 : 0);
  L.total = off;
  return L;
}

// One GPU expert cache: S slots of one blob each, with the events that order the copy stream
// against the compute stream.  Each layer has its own, or (cfg.shared_slots) all layers share one,
// the paper's cache of k experts that is refilled layer after layer (Section V-A).
struct SlotSet {
  char *slots = nullptr;
  std::vector<int> slot_expert, slot_layer;   // what a slot holds: expert of which layer (-1: empty)
  std::vector<unsigned long long> stamp;
  std::vector<char> prefetched;      // slot filled by a prefetch and not yet served
  std::vector<char> copy_pending;    // a copy into the slot was enqueued; compute has not waited yet
  std::vector<char> pf_landed;       // prefetched slot, when compute first waited for it: 1 = had landed, 2 = had not
  std::vector<char> use_kind;        // 0: never read, 1: read behind used[slot], 2: read behind group_done
  std::vector<hipEvent_t> copied, used;   // the slot can be read (fetched and, int4 pool, expanded) / has been read
  std::vector<hipEvent_t> copied_up;  // a split fetch has brought (and expanded) its gate / up matrices
  // integer 4-bit host format: the bytes of a fetch (its first piece, all of it) are in the staging area
  std::vector<hipEvent_t> landed_up, landed;
  std::vector<char> staged;          // the slot's staging area has been written before
  std::vector<char> q_valid;         // the slot holds a quantised blob that every kernel reads as it is
  std::vector<char> expand_pending;  // the expansion into the slot was enqueued; compute has not waited for it yet
  hipEvent_t group_done = nullptr;
  bool done_pending = false;         // group_done still has to be recorded, on done_stream, before it is waited for
  hipStream_t done_stream = nullptr;
  unsigned long long clock = 0;
};

struct Layer {
  bool bound = false;
  int index = 0;
  std::vector<const void *> host_blob;
  const uint16_t *router_w = nullptr;
  const char *shared_blob = nullptr;
  SlotSet *set = nullptr;            // own.get(), or the context's shared set
  std::unique_ptr<SlotSet> own;
  std::vector<int> expert_slot;      // this layer's experts -> slot of `set` (-1: not resident)
  moe_stats stats{};
};

// Workspace of moe_decode_layer_static: one array per GPU the library is loaded on, for callers that
// cannot allocate.  Host code never uses the array's name as an address: the device address is taken
// once per device with hipGetSymbolAddress (moe_create) and kept in g_static_ws.
constexpr size_t kStaticWorkspaceBytes = MOE_STATIC_WORKSPACE_BYTES;
constexpr int kMaxDevices = 64;
__device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];
void *g_static_ws[kMaxDevices] = {};

struct TimedLaunch {
  hipEvent_t start, stop;
  int kind, layer;
};

// A layer call whose cache counters wait for the gate's per-expert counts: the grouping kernel
// writes them, each with the call's number above it, into mailbox `box` (pinned host memory).
struct PendingCall {
  int layer, box, seq;
  hipStream_t stream;   // with no_event: the stream to wait for instead
  bool no_event;        // the call recorded no event behind its counts
};
constexpr int kMailboxes = 32;
constexpr int kMailboxWords = kMaxExperts;   // 8-byte words (mailbox_word): a box is 512 bytes

}  // namespace

struct moe_ctx {
  moe_config cfg{};
  int device = 0;
  size_t blob_bytes = 0;        // one slot: the bf16 blob, 6*d*I; 0 where the cache keeps experts in their quantised form only
  bool direct_q = false;        // e4m3 rows, MXFP4: every kernel reads the blob as fetched; no bf16 slot, no expansion
  size_t host_blob_bytes = 0;   // one expert in the CPU expert cache (bf16: the same; e4m3: scales + codes)
  size_t stage_stride = 0;      // e4m3: bytes of one slot's staging area behind the slots (256-aligned)
  std::vector<Layer> layers;
  std::unique_ptr<SlotSet> shared_set;   // cfg.shared_slots: the one cache all layers use
  // Mailboxes the grouping kernel fills, one per layer call in flight: the E counts, each in a word of
  // its own with the call's number.  A call that needs the counts at once waits for its own; a call that could enqueue
  // everything without them leaves an entry in `pending`, and its counters are filled in by the next
  // API call that looks at the cache (or when the mailbox is needed again).
  long long *mailboxes = nullptr;     // [kMailboxes][kMailboxWords], pinned
  hipEvent_t routed[kMailboxes] = {};
  int32_t call_no = 0;
  PendingCall pending[kMailboxes];    // ring, oldest at pend_head (a mailbox has at most one pending call)
  int pend_head = 0, pend_count = 0;
  bool timers_off = false;            // inside a call that must not create events
  int cur_layer = -1;                 // layer of the call being enqueued (for the kernel timers)
  Tune tune{};
  ApiTune api_tune{};
  float kernel_ms[MOE_K_COUNT] = {};  // harvested kernel durations not yet handed to moe_get_kernel_times
  int32_t kernel_launches[MOE_K_COUNT] = {};
  // prefill with shared experts: they run on a stream of the library's own, beside the gate, the
  // grouping and the routed experts (fork at the start of the call, join before the weighted sum)
  hipStream_t side = nullptr;
  hipEvent_t fork = nullptr, join = nullptr;
  // 8-bit host format: fetched experts are expanded into their slots on this stream, so that the
  // next copy does not queue behind the expansion; expand_tail is the completion event of the last
  // expansion no API call has joined into the copy stream yet
  hipStream_t expand = nullptr;
  hipEvent_t expand_tail = nullptr;
  float *dev_scores = nullptr;        // [64] scratch for predictor_score without dev_scores
  bool profiling = false;
  std::vector<TimedLaunch> timed;
  std::vector<hipEvent_t> event_pool;
};

namespace {

int check_cfg(const moe_config *c) {
  if (!c) return fail(MOE_E_ARG, "cfg is NULL");
  if (c->d <= 0 || c->I <= 0 || c->E <= 0 || c->k <= 0 || c->n_layers <= 0 || c->I_shared < 0)
    return fail(MOE_E_ARG, "d, I, E, k, n_layers must be positive (I_shared >= 0)");
  if (c->k > c->E) return fail(MOE_E_ARG, "k = %d exceeds E = %d", c->k, c->E);
  if (c->cache_slots < 1) return fail(MOE_E_ARG, "cache_slots = %d, need >= 1", c->cache_slots);
  if (c->cache_slots > kMaxCacheSlots)   // the kernels' argument block holds a slot index in 16 bits
    return fail(MOE_E_UNSUPPORTED, "cache_slots = %d > %d", c->cache_slots, kMaxCacheSlots);
  if (c->d > kMaxHidden)                 // the gate keeps four token vectors in LDS
    return fail(MOE_E_UNSUPPORTED, "d = %d > %d", c->d, kMaxHidden);
  if (c->E > kMaxExperts) return fail(MOE_E_UNSUPPORTED, "E = %d > %d experts", c->E, kMaxExperts);
  if (c->d % 8 || c->I % 8 || c->I_shared % 8)
    return fail(MOE_E_UNSUPPORTED, "d, I and I_shared must be multiples of 8");
  if (c->host_format < MOE_FMT_BF16 || c->host_format > MOE_FMT_MXFP4)
    return fail(MOE_E_ARG, "host_format = %d is not a known format", c->host_format);
  if (c->host_format == MOE_FMT_E4M3_ROWS && (c->d % 64 || c->I % 64))
    return fail(MOE_E_UNSUPPORTED, "MOE_FMT_E4M3_ROWS needs d and I to be multiples of 64");
  if (c->host_format == MOE_FMT_MXFP4 && (c->d % 64 || c->I % 64))
    return fail(MOE_E_UNSUPPORTED, "MOE_FMT_MXFP4 needs d and I to be multiples of 64");
  if (c->host_format == MOE_FMT_INT4_G128 && (c->d % 128 || c->I % 128))
    return fail(MOE_E_UNSUPPORTED, "MOE_FMT_INT4_G128 needs d and I to be multiples of 128");
  return MOE_OK;
}

int get_layer(moe_ctx *ctx, int layer, Layer **out, bool need_bound = true) {
  if (!ctx) return fail(MOE_E_ARG, "ctx is NULL");
  if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(MOE_E_ARG, "layer %d out of range", layer);
  *out = &ctx->layers[layer];
  if (need_bound && !(*out)->bound) return fail(MOE_E_UNBOUND, "layer %d is not bound", layer);
  return MOE_OK;
}

// ---- kernel timing ------------------------------------------------------------------------
struct Timer {
  moe_ctx *ctx;
  hipStream_t stream;
  int kind;
  hipEvent_t start = nullptr, stop = nullptr;
  Timer(moe_ctx *c, hipStream_t s, int k) : ctx(c), stream(s), kind(k) {
    if (!ctx->profiling || ctx->timers_off) return;
    auto get = [&]() -> hipEvent_t {
      if (!ctx->event_pool.empty()) {
        hipEvent_t e = ctx->event_pool.back();
        ctx->event_pool.pop_back();
        return e;
      }
      hipEvent_t e = nullptr;
      if (hipEventCreate(&e) != hipSuccess) return nullptr;
      return e;
    };
    start = get();
    stop = get();
    if (start && stop) (void)hipEventRecord(start, stream);
  }
  ~Timer() {
    if (!start || !stop) return;
    (void)hipEventRecord(stop, stream);
    ctx->timed.push_back({start, stop, kind, ctx->cur_layer});
  }
};

// Blocks until the timed launches recorded so far have completed and adds their durations to the
// context's per-class sums and to their layers' compute_ms.
int harvest_timers(moe_ctx *ctx) {
  for (auto &t : ctx->timed) {
    HIP_TRY(hipEventSynchronize(t.stop));
    float dt = 0.0f;
    HIP_TRY(hipEventElapsedTime(&dt, t.start, t.stop));
    ctx->kernel_ms[t.kind] += dt;
    ctx->kernel_launches[t.kind]++;
    if (t.layer >= 0 && t.layer < (int)ctx->layers.size()) ctx->layers[t.layer].stats.compute_ms += dt;
    ctx->event_pool.push_back(t.start);
    ctx->event_pool.push_back(t.stop);
  }
  ctx->timed.clear();
  return MOE_OK;
}

// ---- cache bookkeeping --------------------------------------------------------------------
void touch(Layer &L, int s) { L.set->stamp[s] = ++L.set->clock; }

// Section V-C, second synchronisation point: had a prefetched expert landed when compute asked for it
// (1) or does the computation stream have to wait for the copy (2)?  Taken on the host when the wait
// is enqueued, which is never later than the stream's own wait.
int prefetch_arrival(SlotSet &set, int s) {
  return hipEventQuery(set.copied[s]) == hipSuccess ? 1 : 2;
}

// A served expert that was resident: recency, hit counter and, the first time after a prefetch
// brought it in, the prefetch counters.
void account_hit(Layer &L, int s) {
  SlotSet &set = *L.set;
  touch(L, s);
  L.stats.hits++;
  if (!set.prefetched[s]) return;
  L.stats.prefetch_useful++;
  set.prefetched[s] = 0;
  const int arrival = set.pf_landed[s] ? set.pf_landed[s] : (set.copy_pending[s] ? prefetch_arrival(set, s) : 1);
  if (arrival == 1) L.stats.prefetch_ready++;
  else L.stats.prefetch_stalled++;
  set.pf_landed[s] = 0;
}


// The host needs the gate's per-expert counts of the call that owns mailbox `box`.  Waking up on the
// event costs 10-20 us; the grouping kernel writes every count together with the call's number, as one
// 8-byte word, into pinned, host-coherent memory, so the host first polls those words for a while (the
// kernel is a few microseconds away) and only then blocks.  Each word vouches for itself: with a
// separate "all written" word behind the counts the host has to rely on the order in which a wave's
// stores cross the host link, and one run in some thousand calls read two counts of a call as the zeros
// the mailbox held before.
bool counts_arrived(const moe_ctx *ctx, int box, int seq) {
  volatile const long long *w = ctx->mailboxes + (size_t)box * kMailboxWords;
  for (int e = 0; e < ctx->cfg.E; ++e)
    if ((int)((unsigned long long)w[e] >> 32) != seq) return false;
  std::atomic_thread_fence(std::memory_order_acquire);
  return true;
}
inline int mailbox_count(const long long *box_words, int e) { return (int)(unsigned)(box_words[e] & 0xFFFFFFFFll); }

hipError_t wait_for_counts(moe_ctx *ctx, int box, int seq, hipStream_t stream_instead = nullptr, bool no_event = false) {
  const auto t0 = std::chrono::steady_clock::now();
  for (int spin = 0;; ++spin) {
    if (counts_arrived(ctx, box, seq)) return hipSuccess;
    if ((spin & 255) == 255 &&
        std::chrono::steady_clock::now() - t0 > std::chrono::microseconds(300))
      break;
  }
  hipError_t e = no_event ? hipStreamSynchronize(stream_instead) : hipEventSynchronize(ctx->routed[box]);
  if (e != hipSuccess) return e;
  return counts_arrived(ctx, box, seq) ? hipSuccess : hipErrorUnknown;
}

// Cache counters of a call that was enqueued without looking at the gate's result (every expert was
// resident): hits, recency stamps and useful prefetches, exactly as if they had been taken at the call.
void account_resident_call(moe_ctx *ctx, const PendingCall &p) {
  Layer &L = ctx->layers[p.layer];
  const long long *words = ctx->mailboxes + (size_t)p.box * kMailboxWords;
  for (int e = 0; e < ctx->cfg.E; ++e)
    if (mailbox_count(words, e) > 0) {
      const int s = L.expert_slot[e];
      if (s >= 0) account_hit(L, s);   // (always: whatever changes the slots settles the pending calls first)
    }
}

// Fills in the counters of pending calls, oldest first.  block: wait for every one of them (anything
// that reads or changes recency stamps, slot contents or counters does this first, so the order of
// the stamps is the order of the calls); otherwise stop at the first whose counts are not there yet.
int settle_pending(moe_ctx *ctx, bool block) {
  while (ctx->pend_count > 0) {
    const PendingCall p = ctx->pending[ctx->pend_head];
    if (!counts_arrived(ctx, p.box, p.seq)) {
      if (!block) break;
      HIP_TRY(wait_for_counts(ctx, p.box, p.seq, p.stream, p.no_event));
    }
    account_resident_call(ctx, p);
    ctx->pend_head = (ctx->pend_head + 1) % kMailboxes;
    ctx->pend_count--;
  }
  return MOE_OK;
}

int pick_victim(const Layer &L, unsigned long long protected_mask) {
  const int S = (int)L.set->slot_expert.size();
  for (int s = 0; s < S; ++s)
    if (L.set->slot_expert[s] < 0) return s;
  int best = -1;
  for (int s = 0; s < S; ++s) {
    // (another layer's expert in a shared cache is never protected: its readers are ordered by events)
    if (L.set->slot_layer[s] == L.index && ((protected_mask >> L.set->slot_expert[s]) & 1ull)) continue;
    if (best < 0 || L.set->stamp[s] < L.set->stamp[best]) best = s;
  }
  return best;
}

// The copy into slot s may start when the slot's last reader has finished.  If it has (the usual case in
// decode: the reader ran a step ago), nothing is enqueued.  Otherwise either the copy stream waits for the
// reader's event, or (host_waits) the calling thread does and the copy is enqueued without a dependency.
// A copy behind a wait for an event that is still pending starts some 30 to 45 us after the event fires
// (the wait and the DMA are handed over by the runtime's queues); a copy that is simply next in the copy
// stream's queue starts 7 to 25 us after its predecessor.  A layer call that streams misses through the
// slots has nothing else to do on the host, and every copy it issues waits for the compute of an earlier
// expert of the same call, so it paces the copies itself (64 experts of 17 MB through 16 slots: 25.5 ->
// 21.3 ms per layer; as MXFP4 blobs of 4.6 MB: 12.4 -> 8.1 ms; copies alone 20.3 and 7.2 ms).  A prefetch
// call stays asynchronous: its copy waits on the stream.
int wait_slot_free(Layer &L, int s, hipStream_t copy_stream, bool host_waits) {
  hipEvent_t ev = nullptr;
  if (L.set->use_kind[s] == 1) ev = L.set->used[s];
  if (L.set->use_kind[s] == 2) {
    if (L.set->done_pending) {   // the last grouped launch over resident experts left the recording to us
      HIP_TRY(hipEventRecord(L.set->group_done, L.set->done_stream));
      L.set->done_pending = false;
    }
    ev = L.set->group_done;
  }
  if (!ev || hipEventQuery(ev) == hipSuccess) return MOE_OK;
  if (host_waits) HIP_TRY(hipEventSynchronize(ev));
  else HIP_TRY(hipStreamWaitEvent(copy_stream, ev, 0));
  return MOE_OK;
}

// Enqueue the copy of expert e into slot s on the copy stream, behind the slot's last reader
// (waited: that wait is already on the stream; host_waits: see wait_slot_free).
// split: the gate / up matrices and the down
// matrix travel as two copies, with copied_up[s] recorded in between, so that the first matmul
// can start while the down matrix is still on the link.
int place(moe_ctx *ctx, Layer &L, int e, int s, bool by_prefetch, hipStream_t copy_stream,
          bool waited = false, bool split = false, bool host_waits = false) {
  if (!waited) {
    int rc = wait_slot_free(L, s, copy_stream, host_waits);
    if (rc) return rc;
  }
  char *dst = L.set->slots + (size_t)s * ctx->blob_bytes;
  const char *src = static_cast<const char *>(L.host_blob[e]);
  const moe_config &c = ctx->cfg;
  // From here on the slot's old content is gone: should a step below fail, the tables call the slot
  // empty rather than name an expert whose bytes are being overwritten.
  if (L.set->slot_expert[s] >= 0) ctx->layers[L.set->slot_layer[s]].expert_slot[L.set->slot_expert[s]] = -1;
  L.set->slot_expert[s] = L.set->slot_layer[s] = -1;
  L.set->prefetched[s] = 0;
  L.set->q_valid[s] = 0;
  if (c.host_format != MOE_FMT_BF16) {
    // The quantised blob is [scales and zero points][gate codes][up codes][down codes].  e4m3 rows and
    // MXFP4 stay as they are: the blob lands in the slot.  The 4-bit integer form lands in the slot's
    // staging area on the copy stream; kernels on the expansion stream, each behind the copy it reads,
    // write the bf16 slot, and copied_up / copied are recorded there, after the expansion.
    SlotSet &set = *L.set;
    hipStream_t xs = ctx->expand;
    char *stage = set.slots + (size_t)c.cache_slots * ctx->blob_bytes + (size_t)s * ctx->stage_stride;
    const size_t Id = (size_t)c.I * c.d;
    uint16_t *w = reinterpret_cast<uint16_t *>(dst);
    size_t meta_bytes, up_codes;   // bytes in front of the codes; bytes of the gate and up codes
    if (c.host_format == MOE_FMT_E4M3_ROWS) {
      meta_bytes = (size_t)4 * (2 * c.I + c.d);
      up_codes = 2 * Id;
    } else if (c.host_format == MOE_FMT_INT4_G128) {
      meta_bytes = (15 * Id / 128 + 15) / 16 * 16;
      up_codes = Id;
    } else {
      meta_bytes = (3 * Id / 32 + 15) / 16 * 16;
      up_codes = Id;
    }
    const uint8_t *codes = reinterpret_cast<const uint8_t *>(stage + meta_bytes);
    auto expand = [&](bool down) -> int {   // MOE_FMT_INT4_G128
      const size_t n_up = 2 * Id / 128, n_dn = Id / 128;
      const float *scales = reinterpret_cast<const float *>(stage);
      const uint8_t *zeros = reinterpret_cast<const uint8_t *>(stage + 4 * (n_up + n_dn));
      if (!down) HIP_TRY(launch_dequant_int4_g128(codes, scales, zeros, 2 * c.I, c.d, w, xs));
      else HIP_TRY(launch_dequant_int4_g128(codes + up_codes, scales + n_up, zeros + n_up, c.d, c.I, w + 2 * Id, xs));
      return MOE_OK;
    };
    if (ctx->direct_q) {
      // The cache holds the quantised blob and nothing else: one copy (or two, split behind the gate / up
      // codes), readable by every kernel the moment it has landed.
      if (split) {
        HIP_TRY(hipMemcpyAsync(stage, src, meta_bytes + up_codes, hipMemcpyHostToDevice, copy_stream));
        HIP_TRY(hipEventRecord(set.copied_up[s], copy_stream));
        HIP_TRY(hipMemcpyAsync(stage + meta_bytes + up_codes, src + meta_bytes + up_codes,
                               ctx->host_blob_bytes - meta_bytes - up_codes, hipMemcpyHostToDevice, copy_stream));
      } else {
        HIP_TRY(hipMemcpyAsync(stage, src, ctx->host_blob_bytes, hipMemcpyHostToDevice, copy_stream));
      }
      HIP_TRY(hipEventRecord(set.copied[s], copy_stream));
    } else {
    // the staging area's last expansion must be over before new bytes land in it
    if (set.staged[s]) HIP_TRY(hipStreamWaitEvent(copy_stream, set.copied[s], 0));
    set.staged[s] = 1;
    set.expand_pending[s] = 1;
    int rc = MOE_OK;
    if (split) {
      HIP_TRY(hipMemcpyAsync(stage, src, meta_bytes + up_codes, hipMemcpyHostToDevice, copy_stream));
      HIP_TRY(hipEventRecord(set.landed_up[s], copy_stream));
      HIP_TRY(hipMemcpyAsync(stage + meta_bytes + up_codes, src + meta_bytes + up_codes,
                             ctx->host_blob_bytes - meta_bytes - up_codes, hipMemcpyHostToDevice, copy_stream));
      HIP_TRY(hipEventRecord(set.landed[s], copy_stream));
      HIP_TRY(hipStreamWaitEvent(xs, set.landed_up[s], 0));
      if ((rc = expand(false))) return rc;
      HIP_TRY(hipEventRecord(set.copied_up[s], xs));
      HIP_TRY(hipStreamWaitEvent(xs, set.landed[s], 0));
    } else {
      HIP_TRY(hipMemcpyAsync(stage, src, ctx->host_blob_bytes, hipMemcpyHostToDevice, copy_stream));
      HIP_TRY(hipEventRecord(set.landed[s], copy_stream));
      HIP_TRY(hipStreamWaitEvent(xs, set.landed[s], 0));
      if ((rc = expand(false))) return rc;
    }
    if ((rc = expand(true))) return rc;
    HIP_TRY(hipEventRecord(set.copied[s], xs));
    ctx->expand_tail = set.copied[s];
    }
  } else if (split) {
    const size_t up_bytes = ctx->blob_bytes / 3 * 2;   // [W_gate; W_up], then W_down
    HIP_TRY(hipMemcpyAsync(dst, src, up_bytes, hipMemcpyHostToDevice, copy_stream));
    HIP_TRY(hipEventRecord(L.set->copied_up[s], copy_stream));
    HIP_TRY(hipMemcpyAsync(dst + up_bytes, src + up_bytes, ctx->blob_bytes - up_bytes, hipMemcpyHostToDevice,
                           copy_stream));
  } else {
    HIP_TRY(hipMemcpyAsync(dst, src, ctx->blob_bytes, hipMemcpyHostToDevice, copy_stream));
  }
  if (c.host_format == MOE_FMT_BF16) HIP_TRY(hipEventRecord(L.set->copied[s], copy_stream));
  L.set->q_valid[s] = ctx->direct_q;   // forms every kernel reads as fetched
  L.set->slot_expert[s] = e;
  L.set->slot_layer[s] = L.index;
  L.expert_slot[e] = s;
  L.set->prefetched[s] = by_prefetch;
  L.set->copy_pending[s] = 1;
  L.set->pf_landed[s] = 0;
  L.set->use_kind[s] = 0;
  touch(L, s);
  L.stats.bytes_h2d += (int64_t)ctx->host_blob_bytes;
  return MOE_OK;
}

// The copy stream waits for every expansion enqueued so far: a caller that has synchronised the
// copy stream may then rely on the experts being in their slots.
int join_expand(moe_ctx *ctx, hipStream_t copy_stream) {
  if (!ctx->expand_tail) return MOE_OK;
  HIP_TRY(hipStreamWaitEvent(copy_stream, ctx->expand_tail, 0));
  ctx->expand_tail = nullptr;
  return MOE_OK;
}

// The compute stream waits until slot s can be read: its bytes have landed and, for an integer 4-bit
// pool, been expanded.
int wait_ready(Layer &L, int s, hipStream_t cs) {
  SlotSet &set = *L.set;
  if (set.copy_pending[s] && set.prefetched[s] && !set.pf_landed[s]) set.pf_landed[s] = prefetch_arrival(set, s);
  if (set.copy_pending[s] || set.expand_pending[s]) {
    HIP_TRY(hipStreamWaitEvent(cs, set.copied[s], 0));
    set.copy_pending[s] = set.expand_pending[s] = 0;
  }
  return MOE_OK;
}

GemmArgs routed_args(const moe_ctx *ctx, const Layer &L, const char *ws, const WsLayout &W, int T,
                     bool second, const void *x) {
  const moe_config &c = ctx->cfg;
  GemmArgs a{};
  a.k_top = c.k;
  a.offsets = reinterpret_cast<const int32_t *>(ws + W.offsets);
  a.n_groups = c.E;
  a.wbase = L.set->slots;
  a.wstride = (long long)ctx->blob_bytes;
  for (int e = 0; e < c.E; ++e) a.slot[e] = (int16_t)(L.expert_slot[e] < 0 ? 0 : L.expert_slot[e]);
  a.splitk = 1;
  a.tune = ctx->tune;
  if (c.host_format == MOE_FMT_E4M3_ROWS) {
    // every kernel reads the 8-bit blob as the slot holds it: [row scales][gate | up | down codes]
    const long long scale_bytes = (long long)4 * (2 * c.I + c.d), Id = (long long)c.I * c.d;
    a.qfmt = 1;
    a.qbase = L.set->slots + (size_t)c.cache_slots * ctx->blob_bytes;
    a.qstride = (long long)ctx->stage_stride;
    a.q_b0_off = scale_bytes + (second ? 2 * Id : 0);
    a.q_b1_off = scale_bytes + (second ? 2 * Id : Id);
    a.q_s0_off = second ? (long long)4 * 2 * c.I : 0;
    a.q_s1_off = second ? (long long)4 * 2 * c.I : (long long)4 * c.I;
    a.b_quant = 1;        // the GEMM kernels expand the codes on their way into LDS
  } else if (c.host_format == MOE_FMT_MXFP4) {
    // likewise the MXFP4 blob (a quarter of the bytes): [scale bytes, K/32 per row][codes, K/2 bytes per row]
    const long long Id = (long long)c.I * c.d, meta = (3 * Id / 32 + 15) / 16 * 16;
    a.qfmt = 2;
    a.qbase = L.set->slots + (size_t)c.cache_slots * ctx->blob_bytes;
    a.qstride = (long long)ctx->stage_stride;
    a.q_b0_off = meta + (second ? Id : 0);
    a.q_b1_off = meta + (second ? Id : Id / 2);
    a.q_s0_off = second ? 2 * Id / 32 : 0;
    a.q_s1_off = second ? 2 * Id / 32 : Id / 32;
    a.b_quant = 1;
  }
  if (a.qbase)
    for (int e = 0; e < c.E; ++e)
      if (L.expert_slot[e] >= 0 && L.set->q_valid[L.expert_slot[e]]) a.q8_mask |= 1ull << e;
  if (!second) {
    a.A = reinterpret_cast<const uint16_t *>(x);
    a.lda = c.d;
    a.a_rows = T;
    a.perm = reinterpret_cast<const int32_t *>(ws + W.perm);
    a.b0_off = 0;
    a.b1_off = (long long)c.I * c.d * 2;
    a.ldb = c.d;
    a.N = c.I;
    a.K = c.d;
    a.out = const_cast<char *>(ws + W.H);
    a.ldo = c.I;
  } else {
    a.A = reinterpret_cast<const uint16_t *>(ws + W.H);
    a.lda = c.I;
    a.perm = nullptr;
    a.b0_off = (long long)2 * c.I * c.d * 2;
    a.b1_off = a.b0_off;
    a.ldb = c.I;
    a.N = c.d;
    a.K = c.I;
    a.out = const_cast<char *>(ws + W.Y);
    a.ldo = c.d;
    a.splitk = W.splitk;
    a.max_splitk = W.planes;
    a.out_split_stride = (long long)T * c.k * c.d;
  }
  return a;
}

GemmArgs shared_args(const moe_ctx *ctx, const Layer &L, const char *ws, const WsLayout &W, int T,
                     bool second, const void *x) {
  const moe_config &c = ctx->cfg;
  GemmArgs a{};
  a.k_top = 1;
  a.offsets = nullptr;
  a.single_row0 = 0;
  a.single_rows = T;
  a.group_mask = 1;
  a.n_groups = 1;
  a.wbase = L.shared_blob;
  a.wstride = 0;
  a.splitk = 1;
  a.tune = ctx->tune;
  if (!second) {
    a.A = reinterpret_cast<const uint16_t *>(x);
    a.lda = c.d;
    a.b0_off = 0;
    a.b1_off = (long long)c.I_shared * c.d * 2;
    a.ldb = c.d;
    a.N = c.I_shared;
    a.K = c.d;
    a.out = const_cast<char *>(ws + W.Hs);
    a.ldo = c.I_shared;
  } else {
    a.A = reinterpret_cast<const uint16_t *>(ws + W.Hs);
    a.lda = c.I_shared;
    a.b0_off = (long long)2 * c.I_shared * c.d * 2;
    a.b1_off = a.b0_off;
    a.ldb = c.I_shared;
    a.N = c.d;
    a.K = c.I_shared;
    a.out = const_cast<char *>(ws + W.Ys);
    a.ldo = c.d;
  }
  return a;
}

// Decode groups up to this many tokens use the mat-vec launches (one pass over the weights per 16
// tokens through the matrix cores), larger ones the GEMM kernels; on quantised experts the mat-vec
// launches of MXFP4 blobs stream a quarter of the bytes per pass and stay ahead for a little longer
// (Mixtral shape, largest group 19 rows: 375 against 426 us per layer on the GEMM kernels; 29 rows: 518
// against 438; e4m3, 19 rows: 483 against 396).
constexpr int kMatvecMaxRows = 16, kMatvecMaxRowsMx4 = 24;

// Both expert matmuls of the groups in `mask`, on `stream`.
// A launch that covers every group with rows (use_queues) takes its items from the plan's queues, if
// the layer call has a plan (a1.plan, a2.plan).
int run_experts(moe_ctx *ctx, bool decode, GemmArgs a1, GemmArgs a2, unsigned long long mask,
                int n_groups, int max_rows, int max_rows_per_group, hipStream_t stream,
                const GemmArgs *s1 = nullptr, const GemmArgs *s2 = nullptr,
                hipEvent_t before_second = nullptr, bool use_queues = false) {
  a1.group_mask = a2.group_mask = mask;
  a1.plan_queue = a1.plan && use_queues;
  a2.plan_queue = a2.plan && use_queues;
  // The mat-vec kernels pass over an expert's weights once per 16 of its tokens: a decode batch that
  // gives some expert many more goes to the GEMM kernels, which stream the weights once.
  const bool from_copies = a1.q8_mask != 0 && gemv_reads_copies(a1);
  const int matvec_limit = ctx->api_tune.matvec_max_rows > 0 ? ctx->api_tune.matvec_max_rows : (from_copies && a1.qfmt == 2 ? kMatvecMaxRowsMx4 : kMatvecMaxRows);
  if (decode && max_rows_per_group <= matvec_limit) {
    {
      Timer t(ctx, stream, MOE_K_GEMV1);
      HIP_TRY(launch_grouped_gemv(GEMM_SWIGLU, a1, max_rows_per_group, n_groups, stream, s1));
    }
    if (before_second) HIP_TRY(hipStreamWaitEvent(stream, before_second, 0));
    Timer t(ctx, stream, MOE_K_GEMV2);
    HIP_TRY(launch_grouped_gemv(GEMM_PLAIN_F32, a2, max_rows_per_group, n_groups, stream, s2));
  } else {
    {
      Timer t(ctx, stream, MOE_K_GEMM1);
      HIP_TRY(launch_grouped_gemm(GEMM_SWIGLU, a1, max_rows, n_groups, stream));
    }
    if (before_second) HIP_TRY(hipStreamWaitEvent(stream, before_second, 0));
    Timer t(ctx, stream, MOE_K_GEMM2);
    HIP_TRY(launch_grouped_gemm(GEMM_PLAIN_F32, a2, max_rows, n_groups, stream));
  }
  return MOE_OK;
}

// Joins the library's side stream back into the compute stream when a layer call leaves early with
// an error after the fork: whatever the side stream was given still finishes before anything the
// caller enqueues next on the compute stream.
struct SideJoin {
  moe_ctx *ctx;
  hipStream_t cs;
  bool armed = false;
  ~SideJoin() {
    if (!armed) return;
    if (hipEventRecord(ctx->join, ctx->side) == hipSuccess) (void)hipStreamWaitEvent(cs, ctx->join, 0);
  }
};

int run_layer(moe_ctx *ctx, int layer, const void *dev_x, int T, const float *bias, int bias_stride,
              void *dev_y, void *dev_ws, size_t ws_bytes, void *compute_stream, void *copy_stream,
              bool decode, moe_stats *opt) {
  Layer *Lp = nullptr;
  int rc = get_layer(ctx, layer, &Lp);
  if (rc) return rc;
  Layer &L = *Lp;
  const moe_config &c = ctx->cfg;
  if (!dev_x || !dev_y || !dev_ws) return fail(MOE_E_ARG, "dev_x, dev_y and dev_workspace must be non-NULL");
  if (T <= 0) return fail(MOE_E_ARG, "T = %d, need > 0", T);
  if ((long long)T * c.k > 0x3FFFFFFFll) return fail(MOE_E_UNSUPPORTED, "T*k too large");
  if (!aligned(dev_x, 16) || !aligned(dev_y, 16)) return fail(MOE_E_ARG, "dev_x / dev_y need 16-byte alignment");
  if (!aligned(dev_ws, 256)) return fail(MOE_E_ARG, "dev_workspace needs 256-byte alignment");
  if (bias && bias_stride != 0 && bias_stride != c.E)
    return fail(MOE_E_ARG, "bias_stride must be 0 or E");
  const WsLayout W = ws_layout(c, T, ctx->api_tune.splitk);
  if (ws_bytes < W.total) return fail(MOE_E_WORKSPACE, "workspace %zu < %zu bytes", ws_bytes, W.total);
  hipStream_t cs = reinterpret_cast<hipStream_t>(compute_stream);
  hipStream_t ks = reinterpret_cast<hipStream_t>(copy_stream);
  char *ws = reinterpret_cast<char *>(dev_ws);
  const int S = c.cache_slots, E = c.E;
  const int n = T * c.k;
  ctx->cur_layer = layer;

  bool all_resident = true;
  for (int e = 0; e < E; ++e) all_resident &= L.expert_slot[e] >= 0;
  // A call is enqueued without looking at the gate's result when that result cannot change what is
  // launched: every expert resident, and
  //  - a prefill call (one grouped launch over all experts, sized on the device), or
  //  - one token: the mat-vec launches take the k experts from the gate's own id list on the device, so
  //    the host neither waits for the gate nor launches blocks for the other experts, or
  //  - a decode batch whose experts get few tokens each (on a layer of 16 experts or more at most 2.25
  //    assignments per expert, on a smaller one at most two thirds of one): the launches are sized for
  //    min(E, T k) groups of at most two tokens per pass over the weights, find their experts in the list the
  //    grouping kernel writes, and an expert with more tokens takes further passes.  The shared experts,
  //    which see every token, keep their own launches on the side stream, beside the gate.  (Qwen shape,
  //    per layer: 12 tokens 146 against 150 us with the host's look, 24 tokens 214 against 242, 32 tokens 253
  //    against 283; 48 tokens 334 against 306, so from there on the host looks.)
  // A decode batch on a layer of few experts takes the other path: the per-expert row counts pick a much
  // leaner mat-vec variant and the host's look at them pays (Mixtral shape, 4 tokens: 381 against
  // 398 us), while the shared experts' launches cover the host's wait.
  const bool blind_one = decode && T == 1 && !ctx->api_tune.host_looks_always;
  const bool few_per_expert = E >= 16 ? (long long)n * 4 <= (long long)E * 9 : (long long)n * 3 <= (long long)E * 2;
  const bool blind_batch = decode && T > 1 && few_per_expert && n <= 2048 &&
                           !ctx->api_tune.host_looks_always;
  const bool enqueue_blind = all_resident && (!decode || blind_one || blind_batch);

  // The counters of earlier calls that were enqueued blind: a call that looks at the cache needs them
  // all (recency stamps decide its victims); a blind call only takes what has arrived.
  rc = settle_pending(ctx, !enqueue_blind || opt != nullptr);
  if (rc) return rc;
  const moe_stats before = L.stats;
  // this call's mailbox; the call that used it 32 calls ago must have been accounted for
  const int seq = ++ctx->call_no;
  const int box = seq % kMailboxes;
  if (ctx->pend_count > 0 && ctx->pending[ctx->pend_head].box == box) {   // (the ring is full)
    rc = settle_pending(ctx, true);
    if (rc) return rc;
  }
  long long *mailbox = ctx->mailboxes + (size_t)box * kMailboxWords;

  // A prefill batch of some size: the shared experts get the library's side stream.  Their two
  // launches need nothing but x, so they fill the compute units that the gate and the grouping leave
  // idle, and their last, partly filled round of tiles overlaps the routed experts' first.
  // A decode batch (several tokens, so the host looks at the gate's result before it launches the
  // routed experts) does the same: the shared experts' mat-vecs, arithmetic-bound at 8 tokens, then
  // run beside the bandwidth-bound routed ones instead of in front of them.
  const bool shared_on_side = c.I_shared && (decode ? (!enqueue_blind || (blind_batch && !blind_one)) : T >= 256);
  SideJoin side_join{ctx, cs};
  if (shared_on_side) {
    HIP_TRY(hipEventRecord(ctx->fork, cs));   // after everything the caller queued before (x, the last call)
    HIP_TRY(hipStreamWaitEvent(ctx->side, ctx->fork, 0));
    side_join.armed = true;
  }

  // ---- the routed experts' two launches, and how a prefill call of some size deals its tiles out
  GemmArgs a1 = routed_args(ctx, L, ws, W, T, false, dev_x), a2 = routed_args(ctx, L, ws, W, T, true, dev_x);
  PlanParams plan_params[2] = {};
  bool with_plans = false;
  if (decode) {
    a2.splitk = 1;   // a decode call never cuts K into slices
  } else if (n >= 1024) {
    // Two ways to cut the groups into row tiles and to deal the tiles out.  Few groups of a few row tiles
    // each (Mixtral-like at 2048 tokens): tiles of equal height in a fixed order; the blocks of an XCD then
    // stay in step and share what they fetch, and a group's few left-over rows do not become a tile of
    // their own that waits for its weights alone (measured in one process: 1508 against 1527 us per
    // layer).  Many groups of very different size (DeepSeek-like, 48 of 64 groups under 256 rows), or groups
    // of many row tiles: full tiles plus a short remainder tile on its deeper pipeline, taken from per-XCD
    // queues (64 experts: 730 against 803 us per layer; 8 experts: ahead from about 1500 rows per group,
    // 4.86 against 5.00 ms at 8192 tokens, 18.3 against 19.1 ms at 32768); the plan of those launches is
    // written by the grouping kernel, which has the groups' sizes.
    const int by_shape = (E >= 16 || (long long)n >= 1536ll * E) ? 2 : 1;
    const int up = ctx->api_tune.up_sched ? ctx->api_tune.up_sched : by_shape;
    const int down = ctx->api_tune.down_sched ? ctx->api_tune.down_sched : by_shape;
    a1.equal_heights = up == 1;
    a2.equal_heights = down != 2;
    with_plans = prepare_gemm_plans(a1, a2, reinterpret_cast<GemmPlan *>(ws + W.plans), plan_params);
    if (up == 1) {
      a1.plan = nullptr;
      plan_params[0].out = nullptr;
    }
    if (down == 1) {
      a2.plan = nullptr;
      plan_params[1].out = nullptr;
    }
    with_plans = with_plans && (a1.plan || a2.plan);
  }

  // ---- gate, Top-k, grouping (one token: the gate's kernel writes the grouping tables itself)
  SingleTokenDispatch one{reinterpret_cast<int32_t *>(ws + W.counts), reinterpret_cast<int32_t *>(ws + W.offsets),
                          reinterpret_cast<int32_t *>(ws + W.perm), reinterpret_cast<int32_t *>(ws + W.inv_perm),
                          mailbox, seq};
  {
    Timer t(ctx, cs, MOE_K_ROUTER);
    HIP_TRY(launch_router_topk(reinterpret_cast<const uint16_t *>(dev_x), L.router_w, bias, bias_stride, T,
                               c.d, E, c.k, c.renormalize, reinterpret_cast<float *>(ws + W.logits),
                               reinterpret_cast<int32_t *>(ws + W.ids), reinterpret_cast<float *>(ws + W.w),
                               cs, T == 1 ? &one : nullptr));
  }
  if (T != 1) {
    Timer t(ctx, cs, MOE_K_DISPATCH);
    HIP_TRY(launch_dispatch(reinterpret_cast<const int32_t *>(ws + W.ids), n, E,
                            reinterpret_cast<int32_t *>(ws + W.blk_hist),
                            reinterpret_cast<int32_t *>(ws + W.blk_base),
                            reinterpret_cast<int32_t *>(ws + W.counts),
                            reinterpret_cast<int32_t *>(ws + W.offsets),
                            reinterpret_cast<int32_t *>(ws + W.perm),
                            reinterpret_cast<int32_t *>(ws + W.inv_perm), mailbox, seq, cs,
                            n <= 2048 ? reinterpret_cast<int32_t *>(ws + W.active) : nullptr,
                            with_plans ? plan_params : nullptr));
  }
  // (An event between two launches holds the second one back by a few microseconds.  A one-token call
  // that never looks at the counts itself records none: whoever needs the counts later and does not
  // find them in the mailbox waits for the stream.  Measured, Mixtral shape: 120 -> 117 us per layer.
  // Batches keep the event, they were 2 us slower without it; prefill calls measure the same either way.)
  const bool no_counts_event = blind_one && enqueue_blind;
  if (!no_counts_event) HIP_TRY(hipEventRecord(ctx->routed[box], cs));

  // ---- shared experts: independent of the routing.  When the host has to wait for the gate they
  // run first and cover that wait; in an all-resident decode call they ride in the routed launches.
  GemmArgs s1{}, s2{};
  const bool shared_in_routed_launch = c.I_shared && decode && enqueue_blind && !shared_on_side;
  if (c.I_shared) {
    s1 = shared_args(ctx, L, ws, W, T, false, dev_x);
    s2 = shared_args(ctx, L, ws, W, T, true, dev_x);
    if (shared_on_side) {
      // beside the gate and the grouping: their blocks need a little LDS on some compute unit
      s1.spare_cus = s2.spare_cus = 32;
      rc = run_experts(ctx, decode, s1, s2, 1ull, 1, T, T, ctx->side);
      if (rc) return rc;
      HIP_TRY(hipEventRecord(ctx->join, ctx->side));
      side_join.armed = false;   // from here on the ordinary join before the weighted sum does it
    } else if (!shared_in_routed_launch) {
      rc = run_experts(ctx, decode, s1, s2, 1ull, 1, T, T, cs);
      if (rc) return rc;
    }
  }
  // (an error below still has to join: the event is recorded, only the wait is missing)
  struct JoinOnExit {
    moe_ctx *ctx;
    hipStream_t cs;
    bool armed;
    ~JoinOnExit() {
      if (armed) (void)hipStreamWaitEvent(cs, ctx->join, 0);
    }
  } join_on_exit{ctx, cs, shared_on_side};

  bool combined = false;   // the weighted sum has been done by the down projection's launch
  L.stats.layer_calls++;
  if (enqueue_blind) {
    // Every expert is in a slot: nothing to decide on the host, one grouped launch.
    for (int s = 0; s < S; ++s)
      if (L.set->slot_layer[s] == L.index) {
        rc = wait_ready(L, s, cs);
        if (rc) return rc;
      }
    const unsigned long long mask = E == 64 ? ~0ull : ((1ull << E) - 1ull);
    if (blind_one) a1.sel_ids = a2.sel_ids = reinterpret_cast<const int32_t *>(ws + W.ids);
    if (blind_one && (size_t)c.I * 2 <= 65536 && (size_t)c.I_shared * 2 <= 65536 && !ctx->api_tune.no_fused_down) {
      // one token: the down mat-vec adds the k experts' rows (and the shared experts') up itself
      a1.group_mask = a2.group_mask = mask;
      {
        Timer t(ctx, cs, MOE_K_GEMV1);
        HIP_TRY(launch_grouped_gemv(GEMM_SWIGLU, a1, 1, c.k, cs, shared_in_routed_launch ? &s1 : nullptr));
      }
      Timer t(ctx, cs, MOE_K_GEMV2);
      HIP_TRY(launch_fused_down_combine(a2, reinterpret_cast<const float *>(ws + W.w), c.k,
                                        reinterpret_cast<uint16_t *>(dev_y), cs,
                                        shared_in_routed_launch ? &s2 : nullptr));
      combined = true;
    } else if (blind_batch && !blind_one) {
      a1.sel_ids = a2.sel_ids = reinterpret_cast<const int32_t *>(ws + W.active);
      a1.group_mask = a2.group_mask = mask;
      const int groups = n < E ? n : E;
      {
        Timer t(ctx, cs, MOE_K_GEMV1);
        HIP_TRY(launch_grouped_gemv(GEMM_SWIGLU, a1, 2, groups, cs, shared_in_routed_launch ? &s1 : nullptr));
      }
      Timer t(ctx, cs, MOE_K_GEMV2);
      HIP_TRY(launch_grouped_gemv(GEMM_PLAIN_F32, a2, 2, groups, cs, shared_in_routed_launch ? &s2 : nullptr));
    } else {
      rc = run_experts(ctx, decode, a1, a2, mask, blind_one ? c.k : E, n, T, cs,
                       shared_in_routed_launch ? &s1 : nullptr, shared_in_routed_launch ? &s2 : nullptr, nullptr,
                       true);
      if (rc) return rc;
    }
    // "Every reader of these slots is done" is recorded only when a copy asks for it (wait_slot_free):
    // an event between two launches holds the second one back by several microseconds, and a layer
    // whose experts are all resident is rarely copied into.
    L.set->done_pending = true;
    L.set->done_stream = cs;
    for (int s = 0; s < S; ++s)
      if (L.set->slot_layer[s] == L.index) L.set->use_kind[s] = 2;
    // The counters need the gate's counts, the launches did not: they are filled in when the mailbox
    // has arrived, by whichever later call looks at the cache (or right here if the caller wants them).
    ctx->pending[(ctx->pend_head + ctx->pend_count) % kMailboxes] = {layer, box, seq, cs, no_counts_event};
    ctx->pend_count++;
  } else {
    // "Synchronisation point 1": the gate's choice is compared with the cache.
    {
      const auto t0 = std::chrono::steady_clock::now();
      HIP_TRY(wait_for_counts(ctx, box, seq));
      L.stats.wait_ms += std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t0).count();
    }
    int counts[kMaxExperts];
    unsigned long long hit_mask = 0;
    int n_hits = 0, hit_rows = 0, hit_max = 0;
    int misses[kMaxExperts], n_miss = 0;
    for (int e = 0; e < E; ++e) {
      counts[e] = mailbox_count(mailbox, e);
      if (counts[e] <= 0) continue;
      if (L.expert_slot[e] >= 0) {
        hit_mask |= 1ull << e;
        n_hits++;
        hit_rows += counts[e];
        if (counts[e] > hit_max) hit_max = counts[e];
      } else {
        misses[n_miss++] = e;
      }
    }
    for (int e = 0; e < E; ++e)
      if ((hit_mask >> e) & 1ull) account_hit(L, L.expert_slot[e]);
    L.stats.misses += n_miss;
    if (n_hits && n_miss == 0) {
      for (int e = 0; e < E; ++e)
        if ((hit_mask >> e) & 1ull) {
          rc = wait_ready(L, L.expert_slot[e], cs);
          if (rc) return rc;
        }
      rc = run_experts(ctx, decode, a1, a2, hit_mask, n_hits, hit_rows, hit_max, cs, nullptr, nullptr, nullptr,
                       true);
      if (rc) return rc;
      HIP_TRY(hipEventRecord(L.set->group_done, cs));
      L.set->done_pending = false;
      for (int e = 0; e < E; ++e)
        if ((hit_mask >> e) & 1ull) L.set->use_kind[L.expert_slot[e]] = 2;
    } else if (n_hits) {
      // Misses will reuse these slots: run the hits one by one, each with its own "last reader"
      // event, so that the first fetch can start as soon as the first hit has been computed.
      for (int e = 0; e < E; ++e) {
        if (!((hit_mask >> e) & 1ull)) continue;
        const int s = L.expert_slot[e];
        rc = wait_ready(L, s, cs);  // only this expert's fetch: the next one may still be in flight
        if (rc) return rc;
        rc = run_experts(ctx, decode, a1, a2, 1ull << e, 1, counts[e], counts[e], cs);
        if (rc) return rc;
        HIP_TRY(hipEventRecord(L.set->used[s], cs));
        L.set->use_kind[s] = 1;
      }
    }
    // Misses stream through the slots in ascending id: fetch on the copy stream (once the victim's
    // last reader, an expert of this call S fetches earlier, has been computed: the calling thread
    // waits for that, see wait_slot_free), compute as soon as the copy has landed.  The last fetch is
    // split so that only the down projection and the weighted sum run after it.
    for (int i = 0; i < n_miss; ++i) {
      const int e = misses[i];
      const int s = pick_victim(L, 0ull);
      const bool last = i + 1 == n_miss;
      rc = place(ctx, L, e, s, false, ks, false, last, true);
      if (rc) return rc;
      a1.slot[e] = a2.slot[e] = (int16_t)s;
      if (a1.qbase && L.set->q_valid[s]) {   // fetched just now, as a quantised blob
        a1.q8_mask |= 1ull << e;
        a2.q8_mask |= 1ull << e;
      }
      SlotSet &set = *L.set;
      HIP_TRY(hipStreamWaitEvent(cs, last ? set.copied_up[s] : set.copied[s], 0));
      set.copy_pending[s] = set.expand_pending[s] = 0;
      rc = run_experts(ctx, decode, a1, a2, 1ull << e, 1, counts[e], counts[e], cs, nullptr, nullptr,
                       last ? set.copied[s] : nullptr);
      if (rc) return rc;
      HIP_TRY(hipEventRecord(L.set->used[s], cs));
      L.set->use_kind[s] = 1;
    }
  }

  // ---- weighted sum per token (+ shared experts)
  if (shared_on_side) {
    join_on_exit.armed = false;
    HIP_TRY(hipStreamWaitEvent(cs, ctx->join, 0));
  }
  if (!combined) {
    Timer t(ctx, cs, MOE_K_COMBINE);
    HIP_TRY(launch_combine(reinterpret_cast<const float *>(ws + W.Y), a2.splitk, (long long)n * c.d,
                           reinterpret_cast<const float *>(ws + W.w),
                           reinterpret_cast<const int32_t *>(ws + W.inv_perm),
                           c.I_shared ? reinterpret_cast<const float *>(ws + W.Ys) : nullptr, 1, 0, T, c.d,
                           c.k, reinterpret_cast<uint16_t *>(dev_y), cs));
  }
  if (opt) {
    // the caller wants this call's counters now: wait for the gate's counts if they are still out
    rc = settle_pending(ctx, true);
    if (rc) return rc;
    const moe_stats &a = L.stats;
    *opt = moe_stats{};
    opt->hits = a.hits - before.hits;
    opt->misses = a.misses - before.misses;
    opt->prefetch_useful = a.prefetch_useful - before.prefetch_useful;
    opt->prefetch_ready = a.prefetch_ready - before.prefetch_ready;
    opt->prefetch_stalled = a.prefetch_stalled - before.prefetch_stalled;
    opt->layer_calls = 1;
    opt->bytes_h2d = a.bytes_h2d - before.bytes_h2d;
    opt->wait_ms = a.wait_ms - before.wait_ms;
  }
  return MOE_OK;
}

}  // namespace

// ============================================================================================
extern "C" {

const char *moe_last_error(void) { return g_err; }

static int create_parts(moe_ctx *ctx, const moe_config *cfg) {
  HIP_TRY(hipGetDevice(&ctx->device));
  if (ctx->device >= 0 && ctx->device < kMaxDevices && !g_static_ws[ctx->device]) {
    void *p = nullptr;   // this device's copy of the static workspace
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    g_static_ws[ctx->device] = p;
  }
  ctx->layers.resize(cfg->n_layers);
  HIP_TRY(hipHostMalloc(reinterpret_cast<void **>(&ctx->mailboxes),
                        (size_t)kMailboxes * kMailboxWords * sizeof(long long), 0));
  memset(ctx->mailboxes, 0, (size_t)kMailboxes * kMailboxWords * sizeof(long long));
  for (int i = 0; i < kMailboxes; ++i) HIP_TRY(hipEventCreateWithFlags(&ctx->routed[i], hipEventDisableTiming));
  if (cfg->I_shared) {
    HIP_TRY(hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking));
    HIP_TRY(hipEventCreateWithFlags(&ctx->fork, hipEventDisableTiming));
    HIP_TRY(hipEventCreateWithFlags(&ctx->join, hipEventDisableTiming));
  }
  if (cfg->host_format == MOE_FMT_INT4_G128) HIP_TRY(hipStreamCreateWithFlags(&ctx->expand, hipStreamNonBlocking));
  HIP_TRY(hipMalloc(reinterpret_cast<void **>(&ctx->dev_scores), kMaxExperts * sizeof(float)));
  return MOE_OK;
}

int moe_create(const moe_config *cfg, moe_ctx **out) {
  if (!out) return fail(MOE_E_ARG, "out is NULL");
  *out = nullptr;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  int ndev = 0;
  HIP_TRY(hipGetDeviceCount(&ndev));
  if (ndev < 1) return fail(MOE_E_HIP, "no HIP device");
  moe_ctx *ctx = new (std::nothrow) moe_ctx();
  if (!ctx) return fail(MOE_E_ARG, "out of host memory");
  ctx->cfg = *cfg;
  ctx->direct_q = cfg->host_format == MOE_FMT_E4M3_ROWS || cfg->host_format == MOE_FMT_MXFP4;
  ctx->blob_bytes = ctx->direct_q ? 0 : (size_t)6 * cfg->d * cfg->I;
  ctx->host_blob_bytes = moe_host_blob_bytes(cfg);
  ctx->stage_stride = cfg->host_format != MOE_FMT_BF16 ? (ctx->host_blob_bytes + 255) / 256 * 256 : 0;
  rc = create_parts(ctx, cfg);
  if (rc) {
    // what has been created so far is released again; the message of the failure is kept
    char msg[sizeof(g_err)];
    memcpy(msg, g_err, sizeof(msg));
    (void)moe_destroy(ctx);
    memcpy(g_err, msg, sizeof(msg));
    return rc;
  }
  *out = ctx;
  return MOE_OK;
}

int moe_destroy(moe_ctx *ctx) {
  if (!ctx) return MOE_OK;
  (void)hipDeviceSynchronize();
  ctx->pend_count = 0;
  auto destroy_set = [](SlotSet *set) {
    if (!set) return;
    for (hipEvent_t e : set->copied) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : set->copied_up) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : set->used) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : set->landed_up) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : set->landed) if (e) (void)hipEventDestroy(e);
    if (set->group_done) (void)hipEventDestroy(set->group_done);
  };
  for (Layer &L : ctx->layers) destroy_set(L.own.get());
  destroy_set(ctx->shared_set.get());
  for (auto &t : ctx->timed) {
    (void)hipEventDestroy(t.start);
    (void)hipEventDestroy(t.stop);
  }
  for (hipEvent_t e : ctx->event_pool) (void)hipEventDestroy(e);
  for (hipEvent_t e : ctx->routed) if (e) (void)hipEventDestroy(e);
  if (ctx->fork) (void)hipEventDestroy(ctx->fork);
  if (ctx->join) (void)hipEventDestroy(ctx->join);
  if (ctx->side) {
    (void)hipStreamSynchronize(ctx->side);
    (void)hipStreamDestroy(ctx->side);
  }
  if (ctx->expand) (void)hipStreamDestroy(ctx->expand);
  if (ctx->mailboxes) (void)hipHostFree(ctx->mailboxes);
  if (ctx->dev_scores) (void)hipFree(ctx->dev_scores);
  delete ctx;
  return MOE_OK;
}

size_t moe_host_blob_bytes(const moe_config *cfg) {
  if (check_cfg(cfg)) return 0;
  const size_t dI = (size_t)cfg->d * cfg->I;
  if (cfg->host_format == MOE_FMT_E4M3_ROWS) return (size_t)4 * (2 * cfg->I + cfg->d) + 3 * dI;
  if (cfg->host_format == MOE_FMT_INT4_G128) return (15 * dI / 128 + 15) / 16 * 16 + 3 * dI / 2;
  if (cfg->host_format == MOE_FMT_MXFP4) return (3 * dI / 32 + 15) / 16 * 16 + 3 * dI / 2;
  return 6 * dI;
}

size_t moe_cache_bytes(const moe_config *cfg) {
  if (check_cfg(cfg)) return 0;
  const size_t slot = cfg->host_format == MOE_FMT_E4M3_ROWS || cfg->host_format == MOE_FMT_MXFP4 ? 0 : (size_t)6 * cfg->d * cfg->I;
  const size_t stage = cfg->host_format != MOE_FMT_BF16 ? (moe_host_blob_bytes(cfg) + 255) / 256 * 256 : 0;
  return (size_t)cfg->cache_slots * (slot + stage);
}

size_t moe_workspace_bytes(const moe_config *cfg, int T) {
  if (check_cfg(cfg) || T <= 0) return 0;
  return ws_layout(*cfg, T).total;
}

int moe_bind_layer(moe_ctx *ctx, int layer, const void *const *host_expert_blob, const void *dev_router_w,
                   const void *dev_shared_blob, void *dev_slots, const int32_t *initial_resident) {
  Layer *Lp = nullptr;
  int rc = get_layer(ctx, layer, &Lp, false);
  if (rc) return rc;
  const moe_config &c = ctx->cfg;
  if (!host_expert_blob || !dev_router_w || !dev_slots) return fail(MOE_E_ARG, "NULL pointer in moe_bind_layer");
  if (c.I_shared && !dev_shared_blob) return fail(MOE_E_ARG, "I_shared > 0 but dev_shared_blob is NULL");
  if (!aligned(dev_router_w, 16) || !aligned(dev_slots, 16) || !aligned(dev_shared_blob, 16))
    return fail(MOE_E_ARG, "device pointers need 16-byte alignment");
  for (int e = 0; e < c.E; ++e)
    if (!host_expert_blob[e]) return fail(MOE_E_ARG, "host_expert_blob[%d] is NULL", e);
  const int S = c.cache_slots;
  rc = settle_pending(ctx, true);
  if (rc) return rc;
  if (initial_resident) {
    unsigned long long seen = 0;
    for (int s = 0; s < S; ++s) {
      int e = initial_resident[s];
      if (e < -1 || e >= c.E) return fail(MOE_E_ARG, "initial_resident[%d] = %d out of range", s, e);
      if (e >= 0 && ((seen >> e) & 1ull)) return fail(MOE_E_ARG, "expert %d named twice in initial_resident", e);
      if (e >= 0) seen |= 1ull << e;
    }
  }
  Layer &L = *Lp;
  L.index = layer;
  const bool shared = c.shared_slots != 0;
  if (shared && ctx->shared_set && ctx->shared_set->slots != reinterpret_cast<char *>(dev_slots))
    return fail(MOE_E_ARG, "shared_slots: every layer must be bound to the same dev_slots");
  std::unique_ptr<SlotSet> &holder = shared ? ctx->shared_set : L.own;
  const bool fresh = !holder;
  if (fresh) {
    holder.reset(new (std::nothrow) SlotSet());
    if (!holder) return fail(MOE_E_HIP, "out of host memory");
    SlotSet &set = *holder;
    set.copied.assign(S, nullptr);
    set.copied_up.assign(S, nullptr);
    set.used.assign(S, nullptr);
    for (int s = 0; s < S; ++s) {
      HIP_TRY(hipEventCreateWithFlags(&set.copied[s], hipEventDisableTiming));
      HIP_TRY(hipEventCreateWithFlags(&set.copied_up[s], hipEventDisableTiming));
      HIP_TRY(hipEventCreateWithFlags(&set.used[s], hipEventDisableTiming));
    }
    HIP_TRY(hipEventCreateWithFlags(&set.group_done, hipEventDisableTiming));
    set.staged.assign(S, 0);
    set.q_valid.assign(S, 0);
    set.expand_pending.assign(S, 0);
    if (c.host_format == MOE_FMT_INT4_G128) {   // the only format with an expansion behind the copy
      set.landed_up.assign(S, nullptr);
      set.landed.assign(S, nullptr);
      for (int s = 0; s < S; ++s) {
        HIP_TRY(hipEventCreateWithFlags(&set.landed_up[s], hipEventDisableTiming));
        HIP_TRY(hipEventCreateWithFlags(&set.landed[s], hipEventDisableTiming));
      }
    }
  }
  L.set = holder.get();
  SlotSet &set = *L.set;
  L.host_blob.assign(host_expert_blob, host_expert_blob + c.E);
  L.router_w = reinterpret_cast<const uint16_t *>(dev_router_w);
  L.shared_blob = reinterpret_cast<const char *>(dev_shared_blob);
  L.expert_slot.assign(c.E, -1);
  L.stats = moe_stats{};
  if (fresh || !shared) {
    // (re)binding a layer of its own cache resets that cache; a shared cache is set up by the first
    // layer that is bound and only claimed slot by slot by the others
    set.slots = reinterpret_cast<char *>(dev_slots);
    set.slot_expert.assign(S, -1);
    set.slot_layer.assign(S, -1);
    set.stamp.assign(S, 0);
    set.prefetched.assign(S, 0);
    set.copy_pending.assign(S, 0);
    set.pf_landed.assign(S, 0);
    set.use_kind.assign(S, 0);
    set.q_valid.assign(S, 0);
    // (staged / expand_pending keep their values: they order new copies behind expansions that may
    // still be running on the library's own stream, whatever the slots are taken to hold now)
    set.clock = 0;
  } else {
    for (int s = 0; s < S; ++s)   // rebinding a layer of a shared cache drops what it held there
      if (set.slot_layer[s] == layer) {
        set.slot_expert[s] = set.slot_layer[s] = -1;
        set.prefetched[s] = 0;
        set.stamp[s] = 0;
      }
  }
  if (initial_resident)
    for (int s = 0; s < S; ++s)
      if (initial_resident[s] >= 0) {
        if (set.slot_expert[s] >= 0) ctx->layers[set.slot_layer[s]].expert_slot[set.slot_expert[s]] = -1;
        set.slot_expert[s] = initial_resident[s];
        set.slot_layer[s] = layer;
        set.q_valid[s] = ctx->direct_q ? 1 : 0;   // what the caller put there: the blob as the slots hold it
        L.expert_slot[initial_resident[s]] = s;
      }
  L.bound = true;
  return MOE_OK;
}

int expert_cache_prefetch(moe_ctx *ctx, int layer, const int32_t *host_ids, int n, void *copy_stream) {
  Layer *Lp = nullptr;
  int rc = get_layer(ctx, layer, &Lp);
  if (rc) return rc;
  Layer &L = *Lp;
  if (n < 0 || (n > 0 && !host_ids)) return fail(MOE_E_ARG, "bad id list");
  rc = settle_pending(ctx, true);   // the victims depend on the recency stamps of every call so far
  if (rc) return rc;
  unsigned long long protected_mask = 0;
  for (int i = 0; i < n; ++i) {
    if (host_ids[i] < 0 || host_ids[i] >= ctx->cfg.E) return fail(MOE_E_ARG, "expert id %d out of range", host_ids[i]);
    protected_mask |= 1ull << host_ids[i];
  }
  unsigned long long seen = 0;
  hipStream_t ks = reinterpret_cast<hipStream_t>(copy_stream);
  for (int i = 0; i < n; ++i) {
    const int e = host_ids[i];
    if ((seen >> e) & 1ull) continue;
    seen |= 1ull << e;
    int s = L.expert_slot[e];
    if (s >= 0) {
      touch(L, s);
      continue;
    }
    s = pick_victim(L, protected_mask);
    if (s < 0) {
      L.stats.prefetch_dropped++;
      continue;
    }
    rc = place(ctx, L, e, s, true, ks);
    if (rc) return rc;
    L.stats.prefetch_issued++;
  }
  return join_expand(ctx, ks);
}

int predictor_score(moe_ctx *ctx, int layer, const void *dev_x, int T, const void *dev_wp, int m,
                    float *dev_scores, int32_t *pinned_topm, void *stream) {
  if (!ctx) return fail(MOE_E_ARG, "ctx is NULL");
  if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(MOE_E_ARG, "layer %d out of range", layer);
  ctx->cur_layer = layer;
  if (!dev_x || !dev_wp || !pinned_topm) return fail(MOE_E_ARG, "NULL pointer in predictor_score");
  if (T <= 0 || m <= 0 || m > ctx->cfg.E) return fail(MOE_E_ARG, "need T > 0 and 1 <= m <= E");
  if (!aligned(dev_x, 16) || !aligned(dev_wp, 16)) return fail(MOE_E_ARG, "16-byte alignment needed");
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  Timer t(ctx, s, MOE_K_PREDICTOR);
  HIP_TRY(launch_predictor(reinterpret_cast<const uint16_t *>(dev_x), reinterpret_cast<const uint16_t *>(dev_wp),
                           T, ctx->cfg.d, ctx->cfg.E, m, dev_scores ? dev_scores : ctx->dev_scores,
                           pinned_topm, s));
  return MOE_OK;
}

int predictor_mlp_score(moe_ctx *ctx, const float *state, const int32_t *host_dims, int n_fc,
                        const void *const *dev_w, const float *const *dev_bias,
                        const float *const *dev_scale, const float *const *dev_shift, float *dev_act,
                        int m, float *dev_scores, int32_t *pinned_topm, void *stream) {
  if (!ctx) return fail(MOE_E_ARG, "ctx is NULL");
  if (!state || !host_dims || !dev_w || !dev_bias || !dev_scale || !dev_shift || !dev_act || !pinned_topm)
    return fail(MOE_E_ARG, "NULL pointer in predictor_mlp_score");
  if (n_fc < 2 || n_fc > 16) return fail(MOE_E_ARG, "n_fc = %d, need 2..16", n_fc);
  int maxd = 0;
  for (int l = 0; l <= n_fc; ++l) {
    if (host_dims[l] <= 0) return fail(MOE_E_ARG, "host_dims[%d] = %d", l, host_dims[l]);
    if (host_dims[l] > maxd) maxd = host_dims[l];
  }
  if (host_dims[n_fc] > kMaxExperts) return fail(MOE_E_UNSUPPORTED, "more than %d outputs", kMaxExperts);
  if (m <= 0 || m > host_dims[n_fc]) return fail(MOE_E_ARG, "need 1 <= m <= number of outputs");
  const uint16_t *w[16];
  for (int l = 0; l < n_fc; ++l) {
    if (!dev_w[l] || !dev_bias[l] || (l + 1 < n_fc && (!dev_scale[l] || !dev_shift[l])))
      return fail(MOE_E_ARG, "NULL parameter pointer of layer %d", l);
    w[l] = reinterpret_cast<const uint16_t *>(dev_w[l]);
  }
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  Timer t(ctx, s, MOE_K_PREDICTOR);
  HIP_TRY(launch_mlp_predictor(state, host_dims, n_fc, w, dev_bias, dev_scale, dev_shift, dev_act, dev_act + maxd, m,
                               dev_scores ? dev_scores : ctx->dev_scores, pinned_topm, s));
  return MOE_OK;
}

// ---- State Constructor: host bookkeeping only ---------------------------------------------
}  // extern "C"
struct moe_state {
  int L = 0, M = 0, k = 0;
  std::vector<float> P, A;          // [L, M], [L-1, M, M]
  std::vector<int32_t> ids;         // [L, k]
  std::vector<char> have;           // [L]
};
extern "C" {

int moe_state_create(int n_layers, int n_experts, int k, const float *host_popularity,
                     const float *host_affinity, moe_state **out) {
  if (!out || !host_popularity || (n_layers > 1 && !host_affinity)) return fail(MOE_E_ARG, "NULL argument");
  if (n_layers <= 0 || n_experts <= 0 || k <= 0 || k > n_experts) return fail(MOE_E_ARG, "bad sizes");
  moe_state *st = new (std::nothrow) moe_state();
  if (!st) return fail(MOE_E_HIP, "out of host memory");
  st->L = n_layers;
  st->M = n_experts;
  st->k = k;
  st->P.assign(host_popularity, host_popularity + (size_t)n_layers * n_experts);
  if (n_layers > 1)
    st->A.assign(host_affinity, host_affinity + (size_t)(n_layers - 1) * n_experts * n_experts);
  st->ids.assign((size_t)n_layers * k, 0);
  st->have.assign(n_layers, 0);
  *out = st;
  return MOE_OK;
}

int moe_state_destroy(moe_state *st) {
  delete st;
  return MOE_OK;
}

int moe_state_dim(const moe_state *st) { return st ? st->L * st->k + st->M + st->k * st->M : 0; }

int moe_state_record(moe_state *st, int layer, const int32_t *host_ids) {
  if (!st || !host_ids) return fail(MOE_E_ARG, "NULL argument");
  if (layer < 0 || layer >= st->L) return fail(MOE_E_ARG, "layer %d out of range", layer);
  for (int q = 0; q < st->k; ++q)
    if (host_ids[q] < 0 || host_ids[q] >= st->M) return fail(MOE_E_ARG, "expert id %d out of range", host_ids[q]);
  for (int q = 0; q < st->k; ++q) st->ids[(size_t)layer * st->k + q] = host_ids[q];
  st->have[layer] = 1;
  return MOE_OK;
}

int moe_state_clear(moe_state *st) {
  if (!st) return fail(MOE_E_ARG, "NULL argument");
  st->have.assign(st->L, 0);
  return MOE_OK;
}

int moe_state_vector(const moe_state *st, int layer, float *host_out) {
  if (!st || !host_out) return fail(MOE_E_ARG, "NULL argument");
  if (layer < 0 || layer >= st->L) return fail(MOE_E_ARG, "layer %d out of range", layer);
  for (int j = 0; j < layer; ++j)
    if (!st->have[j]) return fail(MOE_E_ARG, "layer %d has not been recorded in this decode step", j);
  const int L = st->L, M = st->M, k = st->k;
  const int dim = L * k + M + k * M;
  for (int i = 0; i < dim; ++i) host_out[i] = 0.0f;
  for (int j = 0; j < layer; ++j)
    for (int q = 0; q < k; ++q)
      host_out[j * k + q] = (float)((double)(st->ids[(size_t)j * k + q] + 1) / (double)M);
  for (int i = 0; i < M; ++i) host_out[L * k + i] = st->P[(size_t)layer * M + i];
  if (layer > 0)
    for (int q = 0; q < k; ++q) {
      const int e = st->ids[(size_t)(layer - 1) * k + q];
      const float *row = st->A.data() + ((size_t)(layer - 1) * M + e) * M;
      for (int i = 0; i < M; ++i) host_out[L * k + M + q * M + i] = row[i];
    }
  return MOE_OK;
}

int moe_prefill_layer(moe_ctx *ctx, int layer, const void *dev_x, int T, const float *dev_route_bias,
                      int bias_stride, void *dev_y, void *dev_workspace, size_t ws_bytes,
                      void *compute_stream, void *copy_stream, moe_stats *opt) {
  int rc = run_layer(ctx, layer, dev_x, T, dev_route_bias, bias_stride, dev_y, dev_workspace, ws_bytes,
                     compute_stream, copy_stream, false, opt);
  return rc ? rc : join_expand(ctx, reinterpret_cast<hipStream_t>(copy_stream));
}

int moe_decode_layer(moe_ctx *ctx, int layer, const void *dev_x, int T, const float *dev_route_bias,
                     int bias_stride, void *dev_y, void *dev_workspace, size_t ws_bytes,
                     void *compute_stream, void *copy_stream, moe_stats *opt) {
  int rc = run_layer(ctx, layer, dev_x, T, dev_route_bias, bias_stride, dev_y, dev_workspace, ws_bytes,
                     compute_stream, copy_stream, true, opt);
  return rc ? rc : join_expand(ctx, reinterpret_cast<hipStream_t>(copy_stream));
}

int moe_decode_layer_static(moe_ctx *ctx, int layer, const void *dev_x, int T, const float *dev_route_bias,
                            int bias_stride, void *dev_y, void *compute_stream, void *copy_stream,
                            moe_stats *opt) {
  if (!ctx) return fail(MOE_E_ARG, "ctx is NULL");
  if (T <= 0) return fail(MOE_E_ARG, "T = %d, need > 0", T);
  void *ws = ctx->device >= 0 && ctx->device < kMaxDevices ? g_static_ws[ctx->device] : nullptr;
  if (!ws) return fail(MOE_E_UNSUPPORTED, "no static workspace on device %d", ctx->device);
  const size_t need = ws_layout(ctx->cfg, T, ctx->api_tune.splitk).total;
  if (need > kStaticWorkspaceBytes)
    return fail(MOE_E_WORKSPACE, "T = %d needs %zu bytes of workspace, the static one holds %zu: use moe_decode_layer",
                T, need, kStaticWorkspaceBytes);
  ctx->timers_off = true;   // a timer would have to create events
  int rc = run_layer(ctx, layer, dev_x, T, dev_route_bias, bias_stride, dev_y, ws, kStaticWorkspaceBytes,
                     compute_stream, copy_stream, true, opt);
  ctx->timers_off = false;
  return rc ? rc : join_expand(ctx, reinterpret_cast<hipStream_t>(copy_stream));
}

int moe_debug_routing(moe_ctx *ctx, const void *dev_workspace, int T, int32_t *dev_ids, float *dev_w,
                      int32_t *dev_counts, int32_t *dev_offsets, int32_t *dev_perm, int32_t *dev_inv_perm,
                      void *stream) {
  if (!ctx || !dev_workspace || T <= 0) return fail(MOE_E_ARG, "bad argument to moe_debug_routing");
  const moe_config &c = ctx->cfg;
  const WsLayout W = ws_layout(c, T);
  const char *ws = reinterpret_cast<const char *>(dev_workspace);
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  const size_t n = (size_t)T * c.k;
  if (dev_ids) HIP_TRY(hipMemcpyAsync(dev_ids, ws + W.ids, n * 4, hipMemcpyDeviceToDevice, s));
  if (dev_w) HIP_TRY(hipMemcpyAsync(dev_w, ws + W.w, n * 4, hipMemcpyDeviceToDevice, s));
  if (dev_counts) HIP_TRY(hipMemcpyAsync(dev_counts, ws + W.counts, (size_t)c.E * 4, hipMemcpyDeviceToDevice, s));
  if (dev_offsets)
    HIP_TRY(hipMemcpyAsync(dev_offsets, ws + W.offsets, (size_t)(c.E + 1) * 4, hipMemcpyDeviceToDevice, s));
  if (dev_perm) HIP_TRY(hipMemcpyAsync(dev_perm, ws + W.perm, n * 4, hipMemcpyDeviceToDevice, s));
  if (dev_inv_perm) HIP_TRY(hipMemcpyAsync(dev_inv_perm, ws + W.inv_perm, n * 4, hipMemcpyDeviceToDevice, s));
  return MOE_OK;
}

int moe_debug_logits(moe_ctx *ctx, const void *dev_workspace, int T, float *dev_logits, void *stream) {
  if (!ctx || !dev_workspace || !dev_logits || T <= 0) return fail(MOE_E_ARG, "bad argument to moe_debug_logits");
  const WsLayout W = ws_layout(ctx->cfg, T);
  HIP_TRY(hipMemcpyAsync(dev_logits, reinterpret_cast<const char *>(dev_workspace) + W.logits,
                         (size_t)T * ctx->cfg.E * 4, hipMemcpyDeviceToDevice, reinterpret_cast<hipStream_t>(stream)));
  return MOE_OK;
}

int moe_get_stats(moe_ctx *ctx, int layer, moe_stats *out) {
  if (!ctx || !out) return fail(MOE_E_ARG, "NULL argument");
  if (layer >= ctx->cfg.n_layers) return fail(MOE_E_ARG, "layer %d out of range", layer);
  int rc = settle_pending(ctx, true);
  if (rc) return rc;
  if ((rc = harvest_timers(ctx))) return rc;
  moe_stats acc{};
  for (int l = 0; l < ctx->cfg.n_layers; ++l) {
    if (layer >= 0 && l != layer) continue;
    const moe_stats &s = ctx->layers[l].stats;
    acc.hits += s.hits;
    acc.misses += s.misses;
    acc.prefetch_issued += s.prefetch_issued;
    acc.prefetch_useful += s.prefetch_useful;
    acc.prefetch_dropped += s.prefetch_dropped;
    acc.layer_calls += s.layer_calls;
    acc.bytes_h2d += s.bytes_h2d;
    acc.prefetch_ready += s.prefetch_ready;
    acc.prefetch_stalled += s.prefetch_stalled;
    acc.wait_ms += s.wait_ms;
    acc.compute_ms += s.compute_ms;
  }
  *out = acc;
  return MOE_OK;
}

int moe_reset_stats(moe_ctx *ctx) {
  if (!ctx) return fail(MOE_E_ARG, "ctx is NULL");
  int rc = settle_pending(ctx, true);
  if (rc) return rc;
  if ((rc = harvest_timers(ctx))) return rc;
  for (Layer &L : ctx->layers) L.stats = moe_stats{};
  return MOE_OK;
}

int moe_cache_invalidate(moe_ctx *ctx, int layer) {
  Layer *Lp = nullptr;
  int rc = get_layer(ctx, layer, &Lp);
  if (rc) return rc;
  Layer &L = *Lp;
  rc = settle_pending(ctx, true);
  if (rc) return rc;
  for (size_t s = 0; s < L.set->slot_expert.size(); ++s) {
    if (L.set->slot_layer[s] != L.index) continue;   // a shared cache: only what this layer holds
    L.expert_slot[L.set->slot_expert[s]] = -1;
    L.set->slot_expert[s] = L.set->slot_layer[s] = -1;
    L.set->prefetched[s] = 0;
    L.set->stamp[s] = 0;
  }
  return MOE_OK;
}

int moe_cache_state(moe_ctx *ctx, int layer, int32_t *host_slot_expert) {
  Layer *Lp = nullptr;
  int rc = get_layer(ctx, layer, &Lp);
  if (rc) return rc;
  if (!host_slot_expert) return fail(MOE_E_ARG, "NULL argument");
  rc = settle_pending(ctx, true);
  if (rc) return rc;
  for (int s = 0; s < ctx->cfg.cache_slots; ++s)
    host_slot_expert[s] = Lp->set->slot_layer[s] == layer ? Lp->set->slot_expert[s] : -1;
  return MOE_OK;
}

int moe_set_profiling(moe_ctx *ctx, int on) {
  if (!ctx) return fail(MOE_E_ARG, "ctx is NULL");
  ctx->profiling = on != 0;
  return MOE_OK;
}

int moe_get_kernel_times(moe_ctx *ctx, float *ms, int32_t *launches) {
  if (!ctx || !ms || !launches) return fail(MOE_E_ARG, "NULL argument");
  int rc = harvest_timers(ctx);
  if (rc) return rc;
  for (int i = 0; i < MOE_K_COUNT; ++i) {
    ms[i] = ctx->kernel_ms[i];
    launches[i] = ctx->kernel_launches[i];
    ctx->kernel_ms[i] = 0.0f;
    ctx->kernel_launches[i] = 0;
  }
  return MOE_OK;
}

int moe_inject_failure(int nth_hip_call) {
  g_fail_countdown = nth_hip_call > 0 ? nth_hip_call : 0;
  return MOE_OK;
}

int moe_debug_gemm_choice(int mode, int gathered, long long a_rows, int lda, int N, int ldb, int K,
                          long long b1_minus_b0, int max_rows, int n_groups) {
  GemmArgs a{};
  static const int32_t some_perm = 0;
  a.perm = gathered ? &some_perm : nullptr;
  a.a_rows = (int)a_rows;
  a.lda = lda;
  a.N = N;
  a.ldb = ldb;
  a.K = K;
  a.b0_off = 0;
  a.b1_off = b1_minus_b0;
  if (mode < 0 || mode > 2) return fail(MOE_E_ARG, "mode %d", mode);
  return gemm_kernel_choice((GemmMode)mode, a, max_rows, n_groups);
}

int moe_debug_plans(moe_ctx *ctx, const void *dev_workspace, int T, int32_t *host_out, void *stream) {
  if (!ctx || !dev_workspace || !host_out || T <= 0) return fail(MOE_E_ARG, "bad argument to moe_debug_plans");
  const WsLayout W = ws_layout(ctx->cfg, T, ctx->api_tune.splitk);
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  HIP_TRY(hipMemcpyAsync(host_out, reinterpret_cast<const char *>(dev_workspace) + W.plans, 2 * sizeof(GemmPlan),
                         hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  return MOE_OK;
}

int moe_tune(moe_ctx *ctx, int mode, int variant) {
  if (!ctx) return fail(MOE_E_ARG, "ctx is NULL");
  if (mode < 0 || mode > 12 || variant < 0) return fail(MOE_E_ARG, "bad mode/variant");
  switch (mode) {
    case 12: ctx->api_tune.up_sched = variant; return MOE_OK;
    case 11: ctx->api_tune.down_sched = variant; return MOE_OK;
    case 10: ctx->tune.skinny_waves = variant; return MOE_OK;
    case 9: ctx->api_tune.matvec_max_rows = variant; return MOE_OK;
    case 8:
      ctx->tune.skinny_min_tok = variant;
      ctx->tune.skinny_forced = variant == 1;   // 1: every launch with a token or more, whatever the format
      return MOE_OK;
    case 7: ctx->api_tune.no_fused_down = variant != 0; return MOE_OK;
    case 6: return fail(MOE_E_ARG, "mode 6 is not in use");
    case 5: ctx->api_tune.host_looks_always = variant == 0; return MOE_OK;
    case 4:
      if (variant != 0 && variant != 1 && variant != 2 && variant != 4)
        return fail(MOE_E_ARG, "rows per wave of the mat-vec kernels: 0 (by shape), 1, 2 or 4");
      ctx->tune.gemv_rows = variant;
      return MOE_OK;
    case 3:
      if (variant > kMaxSplitK) return fail(MOE_E_ARG, "at most %d K slices", kMaxSplitK);
      ctx->api_tune.splitk = variant;
      return MOE_OK;
    default:
      if (variant != 0 && variant != 1 && variant != 6 && variant != 12)
        return fail(MOE_E_ARG, "GEMM variants: 0 (by shape), 1, 6, 12");
      ctx->tune.gemm_variant[mode] = variant;
      return MOE_OK;
  }
}

int moe_dense_gemm_bf16(const void *dev_a, const void *dev_b, void *dev_c, int M, int N, int K, void *stream) {
  if (!dev_a || !dev_b || !dev_c) return fail(MOE_E_ARG, "NULL pointer in moe_dense_gemm_bf16");
  if (M <= 0 || N <= 0 || K <= 0 || K % 8) return fail(MOE_E_ARG, "M, N, K must be positive and K a multiple of 8");
  if (!aligned(dev_a, 16) || !aligned(dev_b, 16) || !aligned(dev_c, 16)) return fail(MOE_E_ARG, "16-byte alignment needed");
  GemmArgs a{};
  a.A = reinterpret_cast<const uint16_t *>(dev_a);
  a.lda = K;
  a.k_top = 1;
  a.single_rows = M;
  a.group_mask = 1;
  a.n_groups = 1;
  a.wbase = reinterpret_cast<const char *>(dev_b);
  a.ldb = K;
  a.N = N;
  a.K = K;
  a.out = dev_c;
  a.ldo = N;
  a.splitk = 1;
  HIP_TRY(launch_grouped_gemm(GEMM_PLAIN_BF16, a, M, 1, reinterpret_cast<hipStream_t>(stream)));
  return MOE_OK;
}

}  // extern "C"
