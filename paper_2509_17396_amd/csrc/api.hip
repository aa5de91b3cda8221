// C ABI of libepicache: host-side validation, workspace layout and the launch
// sequence of one eviction step (paper Alg. 1 phase A3).  No kernel lives here.
#include <math.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "epicache_internal.h"

namespace epicache {

static size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

// Compute units of the one target of this build, MI355X (gfx950): 8 XCDs x 32.  It only steers the split
// heuristic below (how many key splits fill whole rounds of resident workgroups); results never depend on it.
constexpr int kComputeUnits = 256;

// Number of key splits for a kernel whose grid is `base` workgroups per split: the split count
// (at most 32, at least 4 key tiles each) whose workgroup count fills whole rounds of the `slots`
// workgroups the chip holds at once; `penalty` per split favours fewer splits.
static void pick_splits(int64_t base, int64_t slots, int tiles, double penalty, int* n_splits,
                        int* tiles_per_split) {
  const int cap = tiles / 4 > 1 ? (tiles / 4 < 32 ? tiles / 4 : 32) : 1;
  double best = -1.0;
  int best_tps = tiles;
  for (int s = 1; s <= cap; s++) {
    const int tps = (tiles + s - 1) / s;
    const int eff_s = (tiles + tps - 1) / tps;
    const double rounds = (double)(base * eff_s) / (double)slots;
    const double fill = rounds / (double)(int64_t)(rounds + 0.999999);
    const double score = fill - penalty * eff_s;
    if (score > best) best = score, best_tps = tps;
  }
  *tiles_per_split = best_tps;
  *n_splits = (tiles + best_tps - 1) / best_tps;
}

int make_plan(const epicache_params* prm, Plan* out) {
  if (!prm || !out) return EPICACHE_ERR_INVALID_ARG;
  if (prm->struct_size != sizeof(epicache_params)) return EPICACHE_ERR_INVALID_ARG;
  if (prm->n_batch < 1 || prm->n_q_heads < 1 || prm->n_kv_heads < 1 || prm->head_dim < 1 ||
      prm->n_cached < 0 || prm->n_block < 0 || prm->budget < 1 || prm->patch_len < 1)
    return EPICACHE_ERR_INVALID_ARG;
  if (prm->n_q_heads % prm->n_kv_heads != 0) return EPICACHE_ERR_INVALID_ARG;
  if (prm->dtype != EPICACHE_DTYPE_F32 && prm->dtype != EPICACHE_DTYPE_BF16)
    return EPICACHE_ERR_INVALID_ARG;
  if (prm->reduce != EPICACHE_REDUCE_MAX && prm->reduce != EPICACHE_REDUCE_SUM)
    return EPICACHE_ERR_INVALID_ARG;
  if (!(prm->softmax_scale >= 0.0f) || isinf(prm->softmax_scale)) return EPICACHE_ERR_INVALID_ARG;
  if (prm->softmax_scale > 1.0e6f) return EPICACHE_ERR_UNSUPPORTED;  // the kernels' sentinels times the scale stay finite
  if ((prm->causal_patch != 0 && prm->causal_patch != 1) || prm->reserved != 0) return EPICACHE_ERR_INVALID_ARG;
  const int64_t N64 = (int64_t)prm->n_cached + prm->n_block;
  if (N64 < 1) return EPICACHE_ERR_INVALID_ARG;
  const int64_t rows64 = N64 + (prm->causal_patch ? prm->patch_len : 0);  // K rows a head must hold

  Plan pl;
  memset(&pl, 0, sizeof(pl));
  pl.nb = prm->n_batch;
  pl.Hq = prm->n_q_heads;
  pl.Hkv = prm->n_kv_heads;
  pl.G = pl.Hq / pl.Hkv;
  pl.d = prm->head_dim;
  pl.p = prm->patch_len;
  pl.M = prm->budget;
  pl.dtype = prm->dtype;
  pl.reduce = prm->reduce;
  pl.causal_patch = prm->causal_patch;
  pl.elem = prm->dtype == EPICACHE_DTYPE_F32 ? 4 : 2;
  pl.qsb = prm->q_stride_b, pl.qsh = prm->q_stride_h, pl.qst = prm->q_stride_t;
  pl.ksb = prm->kv_stride_b, pl.ksh = prm->kv_stride_h, pl.kst = prm->kv_stride_t;

  // strides: innermost axis contiguous, rows must not overlap, 16-byte friendly
  const int64_t strides[6] = {pl.qsb, pl.qsh, pl.qst, pl.ksb, pl.ksh, pl.kst};
  for (int i = 0; i < 6; i++)
    if (strides[i] < 0 || strides[i] % 8 != 0) return EPICACHE_ERR_INVALID_ARG;
  if (pl.qst < pl.d || pl.kst < pl.d) return EPICACHE_ERR_INVALID_ARG;
  if (pl.qst > (1 << 20) || pl.kst > (1 << 20)) return EPICACHE_ERR_UNSUPPORTED;  // 32-bit row offsets in the kernels
  if (pl.qsh < pl.qst * (int64_t)(pl.p - 1) + pl.d) return EPICACHE_ERR_INVALID_ARG;
  if (pl.ksh < pl.kst * (rows64 - 1) + pl.d) return EPICACHE_ERR_INVALID_ARG;
  if (pl.nb > 1 && (pl.qsb < pl.qsh * (int64_t)(pl.Hq - 1) + pl.qst * (int64_t)(pl.p - 1) + pl.d ||
                    pl.ksb < pl.ksh * (int64_t)(pl.Hkv - 1) + pl.kst * (rows64 - 1) + pl.d))
    return EPICACHE_ERR_INVALID_ARG;

  // supported envelope
  if (pl.d % 8 != 0 || pl.d < 8 || pl.d > 256) return EPICACHE_ERR_UNSUPPORTED;
  if (N64 > (1 << 24)) return EPICACHE_ERR_UNSUPPORTED;
  const int64_t R64 = (int64_t)pl.G * pl.p;
  if (R64 > 16384) return EPICACHE_ERR_UNSUPPORTED;  // pass 2 keeps one normaliser per row in LDS, next to two tiles
  const int64_t nbh = (int64_t)pl.nb * pl.Hkv;
  if (nbh > 65535) return EPICACHE_ERR_UNSUPPORTED;

  pl.N = (int)N64;
  pl.R = (int)R64;
  pl.Rpad = (pl.R + 63) / 64 * 64;
  pl.n_keep = pl.M < pl.N ? pl.M : pl.N;
  const float scale = prm->softmax_scale > 0.0f ? prm->softmax_scale : 1.0f / sqrtf((float)pl.d);
  pl.c2 = scale * 1.44269504088896340736f;

  pl.use_mfma = (pl.dtype == EPICACHE_DTYPE_BF16 && (pl.d == 128 || pl.d == 64)) ? 1 : 0;
  if (pl.use_mfma) {
    const int tiles = (pl.N + kKeyTile - 1) / kKeyTile;
    // rows per workgroup: 256 (4 waves x 64) or 192 (2 waves x 96), whichever pads R less
    if (pl.R <= 32) pl.stats_rows_per_wg = 32;
    else if (pl.R <= 64) pl.stats_rows_per_wg = 64;
    else if (pl.R <= 128) pl.stats_rows_per_wg = 128;
    else pl.stats_rows_per_wg = ((pl.R + 191) / 192 * 192 < (pl.R + 255) / 256 * 256) ? 192 : 256;
    const int64_t base = nbh * ((pl.R + pl.stats_rows_per_wg - 1) / pl.stats_rows_per_wg);
    // workgroups that fit the chip at once: 8 waves per CU (2 per SIMD)
    const int nw = pl.stats_rows_per_wg == 192 ? 2 : pl.stats_rows_per_wg == 64 ? 2 : pl.stats_rows_per_wg == 32 ? 1 : 4;
    const int64_t slots = kComputeUnits * (8 / nw);
    pick_splits(base, slots, tiles, 0.004, &pl.n_splits, &pl.tiles_per_split);
    // the streaming reduction re-derives every row's log-sum-exp per workgroup: fewer, longer splits
    pick_splits(nbh, slots, tiles, 0.03, &pl.reduce_splits, &pl.reduce_tiles_per_split);
  } else {
    pl.n_splits = 1;
    pl.tiles_per_split = 0;
    pl.reduce_splits = 1;
    pl.reduce_tiles_per_split = 0;
  }

  size_t off = 0;
  pl.off_stats = off;
  off += align256((size_t)nbh * pl.n_splits * pl.Rpad * sizeof(float2));
  pl.off_nlse = off;  // one combined normaliser per scoring row, between the two scoring passes
  off += align256((size_t)nbh * pl.Rpad * sizeof(float));
  pl.off_scores = off;
  off += align256((size_t)nbh * pl.N * sizeof(float));
  pl.off_keep = off;
  off += align256((size_t)nbh * pl.n_keep * sizeof(int32_t));
  pl.off_lse = off;  // row normalisers of the attention-fused step
  off += align256((size_t)pl.nb * pl.Hq * pl.p * sizeof(float));
  pl.ws_total = off;
  const size_t keydiff = align256(keydiff_workspace_bytes(pl));
  if (pl.ws_total < keydiff) pl.ws_total = keydiff;
  pl.keep_stride = pl.n_keep;
  *out = pl;
  return EPICACHE_OK;
}

// Plan of a ragged call: N and M are the upper bounds, the keep rows are pitched for the selection
// rule, and the workspace gains the per-head threshold records.
static int make_ragged_plan(const epicache_params* prm, int32_t select, Plan* out) {
  Plan pl;
  int st = make_plan(prm, &pl);
  if (st != EPICACHE_OK) return st;
  if (select != EPICACHE_SELECT_PER_HEAD && select != EPICACHE_SELECT_POOLED) return EPICACHE_ERR_INVALID_ARG;
  const int64_t nbh = (int64_t)pl.nb * pl.Hkv;
  if (select == EPICACHE_SELECT_POOLED) {
    if (pl.Hkv > 1024 || (int64_t)pl.Hkv * pl.N >= (int64_t(1) << 31)) return EPICACHE_ERR_UNSUPPORTED;
    const int64_t pooled = (int64_t)pl.Hkv * pl.M;
    pl.keep_stride = (int)(pooled < pl.N ? pooled : pl.N);
  } else {
    pl.keep_stride = pl.n_keep;
  }
  size_t off = pl.off_keep;
  off += align256((size_t)nbh * pl.keep_stride * sizeof(int32_t));
  pl.off_lse = off;
  off += align256((size_t)pl.nb * pl.Hq * pl.p * sizeof(float));
  pl.off_select = off;
  off += align256(select_ragged_record_bytes(pl));
  if (pl.ws_total < off) pl.ws_total = off;
  *out = pl;
  return EPICACHE_OK;
}

static bool misaligned(const void* ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15) != 0; }

static int run_score(const Plan& pl, const void* q, const void* k, float* scores, char* ws,
                     hipStream_t stream) {
  float2* stats = reinterpret_cast<float2*>(ws + pl.off_stats);
  float* nlse = reinterpret_cast<float*>(ws + pl.off_nlse);
  hipError_t e = pl.use_mfma ? launch_score_mfma(pl, q, k, scores, stats, nlse, false, stream)
                             : launch_score_generic(pl, q, k, scores, stats, false, stream);
  return e == hipSuccess ? EPICACHE_OK : EPICACHE_ERR_DEVICE;
}

// Scoring with the caller's row normalisers: they take the place of pass 1 (one (max, sum) pair per row).
static int run_score_lse(const Plan& pl, const void* q, const void* k, const float* row_lse, float* scores,
                         char* ws, hipStream_t stream) {
  Plan p1 = pl;
  p1.n_splits = 1;
  float2* stats = reinterpret_cast<float2*>(ws + pl.off_stats);
  if (launch_lse_to_stats(p1, row_lse, stats, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
  float* nlse = reinterpret_cast<float*>(ws + pl.off_nlse);
  hipError_t e = p1.use_mfma ? launch_score_mfma(p1, q, k, scores, stats, nlse, true, stream)
                             : launch_score_generic(p1, q, k, scores, stats, true, stream);
  return e == hipSuccess ? EPICACHE_OK : EPICACHE_ERR_DEVICE;
}

// ---- App. A.2 "SnapKV": the last w = patch_len context rows are the observation window.  The plan of the
// scoring and selection inside: N - w rows scored under the causal mask of the window (its keys follow those
// rows, which is the causal_patch layout), M - w of them kept.
struct SnapkvPlan {
  Plan outer;   // all N context rows, budget M: the compaction
  Plan inner;   // the N - w rows before the window, budget M - w: scoring and selection
  bool evicts;  // N > M
  bool scores;  // there are rows before the window
  size_t off_scores, off_keep, total;
};

static int make_snapkv_plan(const epicache_params* prm, SnapkvPlan* out) {
  SnapkvPlan sp;
  int st = make_plan(prm, &sp.outer);
  if (st != EPICACHE_OK) return st;
  if (prm->causal_patch) return EPICACHE_ERR_INVALID_ARG;  // the call applies the window's causal mask itself
  const Plan& po = sp.outer;
  const int w = po.p;
  sp.evicts = po.N > po.M;
  sp.scores = po.N > w;
  if (sp.evicts && po.M <= w) return EPICACHE_ERR_INVALID_ARG;  // the budget must exceed the window it always keeps
  const int64_t nbh = (int64_t)po.nb * po.Hkv;
  if (sp.scores) {
    epicache_params pi = *prm;
    const int n_before = po.N - w;
    pi.n_cached = prm->n_cached < n_before ? prm->n_cached : n_before;
    pi.n_block = n_before - pi.n_cached;
    pi.budget = sp.evicts ? po.M - w : po.M;
    pi.causal_patch = 1;
    st = make_plan(&pi, &sp.inner);
    if (st != EPICACHE_OK) return st;
    sp.off_scores = sp.inner.off_scores;
    sp.off_keep = sp.inner.off_keep;
  } else {
    sp.inner = po;
    sp.off_scores = sp.off_keep = 0;
  }
  sp.total = sp.off_keep + align256((size_t)nbh * po.n_keep * sizeof(int32_t));
  *out = sp;
  return EPICACHE_OK;
}

// ---- App. A.2 "KVzip": the patch is the whole block behind an instruction, thousands of tokens per query
// head.  The patch tokens are scored kChunkRows / G at a time with the kernels of epicache_score and the chunk
// results are combined with the reduction.
constexpr int kLongPatchChunkRows = 4096;  // scoring rows (G x tokens) per chunk

struct LongPatchPlan {
  Plan body, tail;      // a full chunk of patch tokens; the last, shorter chunk (n_tail_tokens > 0)
  Plan whole;           // N, M, n_keep of the step (taken from `body`)
  int chunk_tokens, n_body, n_tail_tokens;
  size_t off_tmp, off_scores, off_keep, total;
};

static int make_long_patch_plan(const epicache_params* prm, LongPatchPlan* out) {
  if (!prm) return EPICACHE_ERR_INVALID_ARG;
  if (prm->struct_size != sizeof(epicache_params)) return EPICACHE_ERR_INVALID_ARG;
  if (prm->patch_len < 1 || prm->n_q_heads < 1 || prm->n_kv_heads < 1 || prm->n_q_heads % prm->n_kv_heads != 0)
    return EPICACHE_ERR_INVALID_ARG;
  if (prm->causal_patch) return EPICACHE_ERR_INVALID_ARG;  // chunks would need the patch keys of earlier chunks
  if (prm->patch_len > (1 << 20)) return EPICACHE_ERR_UNSUPPORTED;
  const int G = prm->n_q_heads / prm->n_kv_heads;
  LongPatchPlan lp;
  int pc = kLongPatchChunkRows / G;
  if (pc >= 64) pc = pc / 64 * 64;  // whole 64-row tiles inside one query head
  if (pc < 1) pc = 1;
  if (pc > prm->patch_len) pc = prm->patch_len;
  lp.chunk_tokens = pc;
  lp.n_body = prm->patch_len / pc;
  lp.n_tail_tokens = prm->patch_len % pc;
  // the strides must hold the whole patch, not just one chunk
  if (prm->q_stride_t >= 0 && prm->q_stride_h < prm->q_stride_t * (int64_t)(prm->patch_len - 1) + prm->head_dim)
    return EPICACHE_ERR_INVALID_ARG;
  if (prm->n_batch > 1 && prm->q_stride_b < prm->q_stride_h * (int64_t)(prm->n_q_heads - 1) +
                                                prm->q_stride_t * (int64_t)(prm->patch_len - 1) + prm->head_dim)
    return EPICACHE_ERR_INVALID_ARG;
  epicache_params pb = *prm;
  pb.patch_len = pc;
  int st = make_plan(&pb, &lp.body);
  if (st != EPICACHE_OK) return st;
  lp.tail = lp.body;
  if (lp.n_tail_tokens) {
    pb.patch_len = lp.n_tail_tokens;
    st = make_plan(&pb, &lp.tail);
    if (st != EPICACHE_OK) return st;
  }
  lp.whole = lp.body;
  const int64_t nbh = (int64_t)lp.body.nb * lp.body.Hkv;
  lp.off_tmp = lp.body.off_scores > lp.tail.off_scores ? lp.body.off_scores : lp.tail.off_scores;
  lp.off_scores = lp.off_tmp + align256((size_t)nbh * lp.body.N * sizeof(float));
  lp.off_keep = lp.off_scores + align256((size_t)nbh * lp.body.N * sizeof(float));
  lp.total = lp.off_keep + align256((size_t)nbh * lp.body.n_keep * sizeof(int32_t));
  *out = lp;
  return EPICACHE_OK;
}

// scores of the whole patch: chunk 0 writes `scores`, every later chunk goes to `tmp` and is folded in
static int run_score_long_patch(const LongPatchPlan& lp, const void* q, const void* k, float* scores, char* ws,
                                hipStream_t stream) {
  float* tmp = reinterpret_cast<float*>(ws + lp.off_tmp);
  const int n_chunks = lp.n_body + (lp.n_tail_tokens ? 1 : 0);
  for (int c = 0; c < n_chunks; c++) {
    const Plan& pc = c < lp.n_body ? lp.body : lp.tail;
    const char* qc = static_cast<const char*>(q) + (size_t)c * lp.chunk_tokens * pc.qst * pc.elem;
    int st = run_score(pc, qc, k, c == 0 ? scores : tmp, ws, stream);
    if (st != EPICACHE_OK) return st;
    if (c > 0 && launch_combine_scores(lp.whole, scores, tmp, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
  }
  return EPICACHE_OK;
}

// Workspace of epicache_evict_step_static: one array per GPU, held from the moment the code object is
// loaded until the process ends.  Host code never uses the array's name as an address: its device address
// is looked up once per device (static_scratch) and that pointer is what the kernels receive.
constexpr size_t kStaticScratchBytes = EPICACHE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex scratch_mutex;
static void* scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, null until looked up

// Device address of the current device's copy of `scratch`; null if the lookup fails.
static void* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    scratch_ptr[dev] = ptr;
  }
  return scratch_ptr[dev];
}

// ---- the step as a two-stream pipeline over chunks of the batch (epicache_evict_step_overlapped)
constexpr int kMaxOverlapChunks = 64;

struct OverlapPlan {
  Plan whole;            // the step as one launch: validation, N, M
  Plan body, tail;       // a chunk of chunk_nb batch items; the last chunk (tail_nb items, 1..chunk_nb)
  int n_chunks, chunk_nb, tail_nb;
  size_t total;          // bytes: every chunk has its own workspace slice
};

// select < 0: the uniform step; otherwise the ragged step with that selection rule (plans with its keep pitch and
// threshold records)
static int make_overlap_plan(const epicache_params* prm, int32_t n_chunks, bool with_lse, int32_t select,
                             OverlapPlan* out) {
  OverlapPlan op;
  auto plan_of = [&](const epicache_params* p, Plan* pl) {
    return select < 0 ? make_plan(p, pl) : make_ragged_plan(p, select, pl);
  };
  int st = plan_of(prm, &op.whole);
  if (st != EPICACHE_OK) return st;
  if (n_chunks < 0 || n_chunks > kMaxOverlapChunks) return EPICACHE_ERR_INVALID_ARG;
  const Plan& pw = op.whole;
  int n = n_chunks;
  if (n == 0) {
    // Overlap pays where the scoring is bound by arithmetic and leaves HBM idle: the MFMA path with at least
    // 256 scoring rows per KV head.  Chunks of some 64 (batch item, head) pairs keep every scoring launch at half
    // a round of resident workgroups or more, and a chunk should score for a tenth of a millisecond or so
    // (1.25e11 flops in the two passes), or its launches cost more than the overlap returns.
    const int64_t nbh = (int64_t)pw.nb * pw.Hkv;
    n = 1;
    if (pw.use_mfma && pw.R >= 256 && pw.N > pw.M) {
      const double flops = (with_lse ? 2.0 : 4.0) * pw.R * (double)pw.N * pw.d * (double)nbh;  // one pass or two
      const double by_work = flops / 1.25e11;
      n = (int)(nbh / 64);
      if ((double)n > by_work) n = (int)by_work;
    }
    if (n < 1) n = 1;
    if (n > kMaxOverlapChunks) n = kMaxOverlapChunks;
  }
  if (n > pw.nb) n = pw.nb;
  op.chunk_nb = (pw.nb + n - 1) / n;
  op.n_chunks = (pw.nb + op.chunk_nb - 1) / op.chunk_nb;
  op.tail_nb = pw.nb - (op.n_chunks - 1) * op.chunk_nb;
  epicache_params pc = *prm;
  pc.n_batch = op.chunk_nb;
  st = plan_of(&pc, &op.body);
  if (st != EPICACHE_OK) return st;
  op.tail = op.body;
  if (op.tail_nb != op.chunk_nb) {
    pc.n_batch = op.tail_nb;
    st = plan_of(&pc, &op.tail);
    if (st != EPICACHE_OK) return st;
  }
  op.total = (size_t)(op.n_chunks - 1) * op.body.ws_total + op.tail.ws_total;
  *out = op;
  return EPICACHE_OK;
}

// Events that order the two streams of epicache_evict_step_overlapped: one per chunk (scores done ->
// selection and compaction may start) and one for the join.  Created once per device, kept until the process ends.  A wait
// refers to the record that precedes it at the time it is enqueued, so the pool can be reused by the next call
// while the previous one is still running; the mutex is held from a call's first record to its last wait, so
// two host threads never interleave their records and waits.
struct OverlapEvents {
  hipEvent_t chunk[kMaxOverlapChunks];
  hipEvent_t join;
  bool ready;
};
static std::mutex overlap_mutex;
static OverlapEvents overlap_events[kMaxDevices];

// call with overlap_mutex held; null if the device is out of range or an event cannot be created
static OverlapEvents* overlap_event_pool() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  OverlapEvents& ev = overlap_events[dev];
  if (!ev.ready) {
    hipEvent_t made[kMaxOverlapChunks + 1];
    int n = 0;
    for (; n <= kMaxOverlapChunks; n++)
      if (hipEventCreateWithFlags(&made[n], hipEventDisableTiming) != hipSuccess) break;
    if (n <= kMaxOverlapChunks) {
      (void)hipGetLastError();
      for (int i = 0; i < n; i++) (void)hipEventDestroy(made[i]);
      return nullptr;
    }
    for (int i = 0; i < kMaxOverlapChunks; i++) ev.chunk[i] = made[i];
    ev.join = made[kMaxOverlapChunks];
    ev.ready = true;
  }
  return &ev;
}

// The chunks of an overlapped step: score(c) on `main_stream`, rest(c) (selection and compaction) on `aux_stream`
// behind an event that follows score(c); at the end `main_stream` waits for the last rest().  With a single chunk
// or a single stream everything runs on `main_stream` in order.
template <class ScoreFn, class RestFn>
static int run_chunks_on_two_streams(int n_chunks, hipStream_t main_stream, hipStream_t aux_stream, ScoreFn score,
                                     RestFn rest) {
  const bool two_streams = main_stream != aux_stream && n_chunks > 1;
  // Under stream capture the events only shape the graph's edges and are not needed once the call returns: they
  // are created for the call and destroyed at its end, so that the pool's events never belong to a capture.
  std::unique_lock<std::mutex> lock(overlap_mutex, std::defer_lock);
  OverlapEvents* ev = nullptr;
  OverlapEvents capture_events;
  bool capturing = false;
  if (two_streams) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(main_stream, &cs) != hipSuccess) {
      (void)hipGetLastError();
      cs = hipStreamCaptureStatusNone;
    }
    capturing = cs == hipStreamCaptureStatusActive;
    if (capturing) {
      int made = 0;
      for (; made <= n_chunks; made++) {
        hipEvent_t* slot = made < n_chunks ? &capture_events.chunk[made] : &capture_events.join;
        if (hipEventCreateWithFlags(slot, hipEventDisableTiming) != hipSuccess) break;
      }
      if (made <= n_chunks) {
        (void)hipGetLastError();
        for (int i = 0; i < made; i++) (void)hipEventDestroy(capture_events.chunk[i]);
        return EPICACHE_ERR_DEVICE;
      }
      ev = &capture_events;
    } else {
      lock.lock();
      ev = overlap_event_pool();
      if (!ev) return EPICACHE_ERR_DEVICE;
    }
  }
  int result = EPICACHE_OK;
  bool forked = false;
  for (int c = 0; c < n_chunks && result == EPICACHE_OK; c++) {
    result = score(c, main_stream);
    if (result != EPICACHE_OK) break;
    hipStream_t rest_stream = main_stream;
    if (two_streams) {
      // selection and compaction of this chunk wait for its scores only; the next chunk's scoring does not wait
      // for them
      if (hipEventRecord(ev->chunk[c], main_stream) != hipSuccess ||
          hipStreamWaitEvent(aux_stream, ev->chunk[c], 0) != hipSuccess) {
        result = EPICACHE_ERR_DEVICE;
        break;
      }
      forked = true;
      rest_stream = aux_stream;
    }
    result = rest(c, rest_stream);
  }
  if (forked) {
    // join, also after a failed launch: whatever follows on the caller's stream is ordered after the work enqueued
    // on the other stream so far
    if (hipEventRecord(ev->join, aux_stream) != hipSuccess ||
        hipStreamWaitEvent(main_stream, ev->join, 0) != hipSuccess)
      result = EPICACHE_ERR_DEVICE;
  }
  if (capturing) {
    for (int i = 0; i < n_chunks; i++) (void)hipEventDestroy(capture_events.chunk[i]);
    (void)hipEventDestroy(capture_events.join);
  }
  return result;
}

}  // namespace epicache

using namespace epicache;

extern "C" {

int epicache_workspace_size(const epicache_params* params, size_t* bytes_out) {
  if (!bytes_out) return EPICACHE_ERR_INVALID_ARG;
  Plan pl;
  int st = make_plan(params, &pl);
  if (st != EPICACHE_OK) return st;
  *bytes_out = pl.ws_total;
  return EPICACHE_OK;
}

int epicache_score(const epicache_params* params, const void* q, const void* k, float* scores,
                   void* workspace, size_t workspace_bytes, void* hip_stream) {
  Plan pl;
  int st = make_plan(params, &pl);
  if (st != EPICACHE_OK) return st;
  if (!q || !k || !scores || !workspace) return EPICACHE_ERR_INVALID_ARG;
  if (misaligned(q) || misaligned(k) || misaligned(scores) || misaligned(workspace))
    return EPICACHE_ERR_INVALID_ARG;
  if (workspace_bytes < pl.off_scores) return EPICACHE_ERR_WORKSPACE_TOO_SMALL;
  return run_score(pl, q, k, scores, static_cast<char*>(workspace), (hipStream_t)hip_stream);
}

int epicache_score_lse(const epicache_params* params, const void* q, const void* k,
                       const float* row_lse, float* scores, void* workspace, size_t workspace_bytes,
                       void* hip_stream) {
  Plan pl;
  int st = make_plan(params, &pl);
  if (st != EPICACHE_OK) return st;
  if (!q || !k || !row_lse || !scores || !workspace) return EPICACHE_ERR_INVALID_ARG;
  if (pl.causal_patch) return EPICACHE_ERR_INVALID_ARG;  // the supplied normaliser already fixes the denominator
  if (misaligned(q) || misaligned(k) || misaligned(row_lse) || misaligned(scores) || misaligned(workspace))
    return EPICACHE_ERR_INVALID_ARG;
  if (workspace_bytes < pl.off_scores) return EPICACHE_ERR_WORKSPACE_TOO_SMALL;
  return run_score_lse(pl, q, k, row_lse, scores, static_cast<char*>(workspace), (hipStream_t)hip_stream);
}

int epicache_patch_attention(const epicache_params* params, const void* q, const void* k, const void* v,
                             void* out, float* lse_out, void* hip_stream) {
  Plan pl;
  int st = make_plan(params, &pl);
  if (st != EPICACHE_OK) return st;
  if (!q || !k || !v || !out || !lse_out) return EPICACHE_ERR_INVALID_ARG;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(lse_out))
    return EPICACHE_ERR_INVALID_ARG;
  if (out == q || out == k || out == v) return EPICACHE_ERR_INVALID_ARG;
  if ((int64_t)pl.nb * pl.Hq * pl.p > INT32_MAX) return EPICACHE_ERR_UNSUPPORTED;
  hipError_t e = launch_patch_attention(pl, q, k, v, out, lse_out, (hipStream_t)hip_stream);
  return e == hipSuccess ? EPICACHE_OK : EPICACHE_ERR_DEVICE;
}

int epicache_patch_attention_ragged(const epicache_params* params, const void* q, const void* k, const void* v,
                                    const int32_t* n_ctx, void* out, float* lse_out, void* hip_stream) {
  Plan pl;
  int st = make_plan(params, &pl);
  if (st != EPICACHE_OK) return st;
  if (!q || !k || !v || !n_ctx || !out || !lse_out) return EPICACHE_ERR_INVALID_ARG;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(n_ctx) || misaligned(out) || misaligned(lse_out))
    return EPICACHE_ERR_INVALID_ARG;
  if (out == q || out == k || out == v) return EPICACHE_ERR_INVALID_ARG;
  if ((int64_t)pl.nb * pl.Hq * pl.p > INT32_MAX) return EPICACHE_ERR_UNSUPPORTED;
  pl.n_ctx = n_ctx;
  hipError_t e = launch_patch_attention(pl, q, k, v, out, lse_out, (hipStream_t)hip_stream);
  return e == hipSuccess ? EPICACHE_OK : EPICACHE_ERR_DEVICE;
}

int epicache_evict_step_attn(const epicache_params* params, const void* q, void* k, void* v, void* out,
                             float* scores_opt, int32_t* keep_idx_opt, void* workspace, size_t workspace_bytes,
                             void* hip_stream) {
  Plan pl;
  int st = make_plan(params, &pl);
  if (st != EPICACHE_OK) return st;
  if (!q || !k || !v || !out || !workspace) return EPICACHE_ERR_INVALID_ARG;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(workspace) ||
      misaligned(scores_opt) || misaligned(keep_idx_opt))
    return EPICACHE_ERR_INVALID_ARG;
  if (k == v || out == q || out == k || out == v) return EPICACHE_ERR_INVALID_ARG;
  if ((int64_t)pl.nb * pl.Hq * pl.p > INT32_MAX) return EPICACHE_ERR_UNSUPPORTED;
  if (workspace_bytes < pl.ws_total) return EPICACHE_ERR_WORKSPACE_TOO_SMALL;
  char* ws = static_cast<char*>(workspace);
  hipStream_t stream = (hipStream_t)hip_stream;
  float* lse = reinterpret_cast<float*>(ws + pl.off_lse);
  // the patch's pass through the layer: its output, and the normaliser of every scoring row ...
  if (launch_patch_attention(pl, q, k, v, out, lse, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
  // ... which already fix the denominator (context keys, plus the patch's own with causal_patch), so the
  // scoring needs one pass over the context keys
  float* scores = scores_opt ? scores_opt : reinterpret_cast<float*>(ws + pl.off_scores);
  int32_t* keep = keep_idx_opt ? keep_idx_opt : reinterpret_cast<int32_t*>(ws + pl.off_keep);
  Plan ps = pl;
  ps.causal_patch = 0;
  if (pl.N <= pl.M) {  // nothing to evict
    if (scores_opt) {
      st = run_score_lse(ps, q, k, lse, scores, ws, stream);
      if (st != EPICACHE_OK) return st;
    }
    if (keep_idx_opt && launch_iota_keep(pl, keep, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
    return EPICACHE_OK;
  }
  st = run_score_lse(ps, q, k, lse, scores, ws, stream);
  if (st != EPICACHE_OK) return st;
  if (launch_topk(pl, scores, keep, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
  if (launch_compact(pl, keep, k, v, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
  return EPICACHE_OK;
}

int epicache_score_keydiff(const epicache_params* params, const void* k, const int32_t* n_ctx_opt,
                           float* scores, void* workspace, size_t workspace_bytes, void* hip_stream) {
  Plan pl;
  int st = make_plan(params, &pl);
  if (st != EPICACHE_OK) return st;
  if (!k || !scores || !workspace) return EPICACHE_ERR_INVALID_ARG;
  if (misaligned(k) || misaligned(n_ctx_opt) || misaligned(scores) || misaligned(workspace))
    return EPICACHE_ERR_INVALID_ARG;
  if (workspace_bytes < keydiff_workspace_bytes(pl)) return EPICACHE_ERR_WORKSPACE_TOO_SMALL;
  pl.n_ctx = n_ctx_opt;
  hipError_t e = launch_score_keydiff(pl, k, scores, workspace, (hipStream_t)hip_stream);
  return e == hipSuccess ? EPICACHE_OK : EPICACHE_ERR_DEVICE;
}

int epicache_topk(const epicache_params* params, const float* scores, int32_t* keep_idx,
                  void* workspace, size_t workspace_bytes, void* hip_stream) {
  (void)workspace;
  (void)workspace_bytes;  // the selection keeps its state on chip
  Plan pl;
  int st = make_plan(params, &pl);
  if (st != EPICACHE_OK) return st;
  if (!scores || !keep_idx) return EPICACHE_ERR_INVALID_ARG;
  if (misaligned(scores) || misaligned(keep_idx)) return EPICACHE_ERR_INVALID_ARG;
  hipError_t e = launch_topk(pl, scores, keep_idx, (hipStream_t)hip_stream);
  return e == hipSuccess ? EPICACHE_OK : EPICACHE_ERR_DEVICE;
}

int epicache_compact(const epicache_params* params, const int32_t* keep_idx, void* k, void* v,
                     void* workspace, size_t workspace_bytes, void* hip_stream) {
  (void)workspace;
  (void)workspace_bytes;  // in-place gather, no staging buffer
  Plan pl;
  int st = make_plan(params, &pl);
  if (st != EPICACHE_OK) return st;
  if (!keep_idx || !k || !v) return EPICACHE_ERR_INVALID_ARG;
  if (misaligned(keep_idx) || misaligned(k) || misaligned(v)) return EPICACHE_ERR_INVALID_ARG;
  if (k == v) return EPICACHE_ERR_INVALID_ARG;
  hipError_t e = launch_compact(pl, keep_idx, k, v, (hipStream_t)hip_stream);
  return e == hipSuccess ? EPICACHE_OK : EPICACHE_ERR_DEVICE;
}

static int evict_step_impl(const epicache_params* params, const void* q, void* k, void* v,
                           const float* row_lse, bool with_lse, float* scores_opt, int32_t* keep_idx_opt,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  Plan pl;
  int st = make_plan(params, &pl);
  if (st != EPICACHE_OK) return st;
  if (!q || !k || !v || !workspace || (with_lse && !row_lse)) return EPICACHE_ERR_INVALID_ARG;
  if (with_lse && pl.causal_patch) return EPICACHE_ERR_INVALID_ARG;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(workspace) ||
      misaligned(scores_opt) || misaligned(keep_idx_opt) || misaligned(row_lse))
    return EPICACHE_ERR_INVALID_ARG;
  if (k == v) return EPICACHE_ERR_INVALID_ARG;
  const size_t need = !scores_opt ? (!keep_idx_opt ? pl.ws_total : pl.off_keep) :
                      (!keep_idx_opt ? pl.ws_total : pl.off_scores);
  if (workspace_bytes < need) return EPICACHE_ERR_WORKSPACE_TOO_SMALL;
  char* ws = static_cast<char*>(workspace);
  hipStream_t stream = (hipStream_t)hip_stream;
  float* scores = scores_opt ? scores_opt : reinterpret_cast<float*>(ws + pl.off_scores);
  int32_t* keep = keep_idx_opt ? keep_idx_opt : reinterpret_cast<int32_t*>(ws + pl.off_keep);
  auto score = [&]() -> int {
    return with_lse ? run_score_lse(pl, q, k, row_lse, scores, ws, stream) : run_score(pl, q, k, scores, ws, stream);
  };

  if (pl.N <= pl.M) {  // nothing to evict: the cache is still filling up (App. A.3)
    if (scores_opt) {
      st = score();
      if (st != EPICACHE_OK) return st;
    }
    if (keep_idx_opt && launch_iota_keep(pl, keep, stream) != hipSuccess)
      return EPICACHE_ERR_DEVICE;
    return EPICACHE_OK;
  }
  st = score();
  if (st != EPICACHE_OK) return st;
  if (launch_topk(pl, scores, keep, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
  if (launch_compact(pl, keep, k, v, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
  return EPICACHE_OK;
}

int epicache_evict_step(const epicache_params* params, const void* q, void* k, void* v,
                        float* scores_opt, int32_t* keep_idx_opt, void* workspace,
                        size_t workspace_bytes, void* hip_stream) {
  return evict_step_impl(params, q, k, v, nullptr, false, scores_opt, keep_idx_opt, workspace,
                         workspace_bytes, hip_stream);
}

int epicache_evict_step_static(const epicache_params* params, const void* q, void* k, void* v,
                               float* scores_opt, int32_t* keep_idx_opt, void* hip_stream) {
  Plan pl;
  int st = make_plan(params, &pl);
  if (st != EPICACHE_OK) return st;
  // only the parts of the workspace that the caller does not supply have to fit the array
  const size_t need = !scores_opt ? (!keep_idx_opt ? pl.ws_total : pl.off_keep) :
                      (!keep_idx_opt ? pl.ws_total : pl.off_scores);
  if (need > kStaticScratchBytes) return EPICACHE_ERR_WORKSPACE_TOO_SMALL;
  void* ws = static_scratch();
  if (!ws) return EPICACHE_ERR_DEVICE;
  return evict_step_impl(params, q, k, v, nullptr, false, scores_opt, keep_idx_opt, ws,
                         kStaticScratchBytes, hip_stream);
}

int epicache_overlapped_workspace_size(const epicache_params* params, int32_t n_chunks, int32_t with_row_lse,
                                       size_t* bytes_out, int32_t* n_chunks_out) {
  if (!bytes_out) return EPICACHE_ERR_INVALID_ARG;
  OverlapPlan op;
  int st = make_overlap_plan(params, n_chunks, with_row_lse != 0, -1, &op);
  if (st != EPICACHE_OK) return st;
  *bytes_out = op.total;
  if (n_chunks_out) *n_chunks_out = op.n_chunks;
  return EPICACHE_OK;
}

int epicache_evict_step_overlapped(const epicache_params* params, const void* q, void* k, void* v,
                                   const float* row_lse_opt, float* scores_opt, int32_t* keep_idx_opt,
                                   int32_t n_chunks, void* workspace, size_t workspace_bytes, void* hip_stream,
                                   void* hip_stream_aux) {
  OverlapPlan op;
  int st = make_overlap_plan(params, n_chunks, row_lse_opt != nullptr, -1, &op);
  if (st != EPICACHE_OK) return st;
  if (!q || !k || !v || !workspace) return EPICACHE_ERR_INVALID_ARG;
  if (row_lse_opt && op.whole.causal_patch) return EPICACHE_ERR_INVALID_ARG;  // as epicache_score_lse
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(workspace) || misaligned(scores_opt) ||
      misaligned(keep_idx_opt) || misaligned(row_lse_opt))
    return EPICACHE_ERR_INVALID_ARG;
  if (k == v) return EPICACHE_ERR_INVALID_ARG;
  if (workspace_bytes < op.total) return EPICACHE_ERR_WORKSPACE_TOO_SMALL;
  const Plan& pw = op.whole;
  hipStream_t main_stream = (hipStream_t)hip_stream, aux_stream = (hipStream_t)hip_stream_aux;
  char* ws = static_cast<char*>(workspace);

  struct Chunk {
    const Plan* pl;
    const char* q;
    char *k, *v, *ws;
    float* scores;
    int32_t* keep;
    const float* lse;
  };
  auto chunk = [&](int c) {
    Chunk ch;
    ch.pl = c + 1 < op.n_chunks ? &op.body : &op.tail;
    const int64_t b0 = (int64_t)c * op.chunk_nb;  // first batch item of the chunk
    ch.q = static_cast<const char*>(q) + b0 * pw.qsb * pw.elem;
    ch.k = static_cast<char*>(k) + b0 * pw.ksb * pw.elem;
    ch.v = static_cast<char*>(v) + b0 * pw.ksb * pw.elem;
    ch.ws = ws + (size_t)c * op.body.ws_total;
    ch.scores = scores_opt ? scores_opt + b0 * pw.Hkv * pw.N : reinterpret_cast<float*>(ch.ws + ch.pl->off_scores);
    ch.keep = keep_idx_opt ? keep_idx_opt + b0 * pw.Hkv * pw.n_keep
                           : reinterpret_cast<int32_t*>(ch.ws + ch.pl->off_keep);
    // the caller's normalisers of this chunk's rows ([n_batch, n_q_heads, patch_len], dense)
    ch.lse = row_lse_opt ? row_lse_opt + b0 * pw.Hq * pw.p : nullptr;
    return ch;
  };
  auto score = [&](int c, hipStream_t stream) -> int {
    const Chunk ch = chunk(c);
    return ch.lse ? run_score_lse(*ch.pl, ch.q, ch.k, ch.lse, ch.scores, ch.ws, stream)
                  : run_score(*ch.pl, ch.q, ch.k, ch.scores, ch.ws, stream);
  };
  if (pw.N <= pw.M) {  // nothing to evict: as epicache_evict_step, chunk by chunk on the caller's stream
    for (int c = 0; c < op.n_chunks; c++) {
      if (scores_opt) {
        st = score(c, main_stream);
        if (st != EPICACHE_OK) return st;
      }
      const Chunk ch = chunk(c);
      if (keep_idx_opt && launch_iota_keep(*ch.pl, ch.keep, main_stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
    }
    return EPICACHE_OK;
  }
  auto select_and_compact = [&](int c, hipStream_t stream) -> int {
    const Chunk ch = chunk(c);
    if (launch_topk(*ch.pl, ch.scores, ch.keep, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
    if (launch_compact(*ch.pl, ch.keep, ch.k, ch.v, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
    return EPICACHE_OK;
  };
  return run_chunks_on_two_streams(op.n_chunks, main_stream, aux_stream, score, select_and_compact);
}

int epicache_ragged_overlapped_workspace_size(const epicache_params* params, int32_t select, int32_t n_chunks,
                                              int32_t with_row_lse, size_t* bytes_out, int32_t* keep_capacity_out,
                                              int32_t* n_chunks_out) {
  if (!bytes_out) return EPICACHE_ERR_INVALID_ARG;
  OverlapPlan op;
  int st = make_overlap_plan(params, n_chunks, with_row_lse != 0, select, &op);
  if (st != EPICACHE_OK) return st;
  *bytes_out = op.total;
  if (keep_capacity_out) *keep_capacity_out = op.whole.keep_stride;
  if (n_chunks_out) *n_chunks_out = op.n_chunks;
  return EPICACHE_OK;
}

int epicache_evict_step_ragged_overlapped(const epicache_params* params, int32_t select, const void* q, void* k,
                                          void* v, const int32_t* n_ctx, const int32_t* budgets,
                                          const float* row_lse_opt, int32_t* n_kept, float* scores_opt,
                                          int32_t* keep_idx_opt, int32_t n_chunks, void* workspace,
                                          size_t workspace_bytes, void* hip_stream, void* hip_stream_aux) {
  OverlapPlan op;
  int st = make_overlap_plan(params, n_chunks, row_lse_opt != nullptr, select, &op);
  if (st != EPICACHE_OK) return st;
  if (!q || !k || !v || !n_ctx || !n_kept || !workspace) return EPICACHE_ERR_INVALID_ARG;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(n_ctx) || misaligned(budgets) ||
      misaligned(row_lse_opt) || misaligned(n_kept) || misaligned(scores_opt) || misaligned(keep_idx_opt) ||
      misaligned(workspace))
    return EPICACHE_ERR_INVALID_ARG;
  const Plan& pw = op.whole;
  if (k == v || (row_lse_opt && pw.causal_patch)) return EPICACHE_ERR_INVALID_ARG;
  if (workspace_bytes < op.total) return EPICACHE_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t main_stream = (hipStream_t)hip_stream, aux_stream = (hipStream_t)hip_stream_aux;
  char* ws = static_cast<char*>(workspace);

  struct Chunk {
    Plan pl;  // with this chunk's lengths
    const char* q;
    char *k, *v, *ws;
    float* scores;
    int32_t *keep, *n_kept;
    const int32_t* budgets;
    const float* lse;
  };
  auto chunk = [&](int c) {
    Chunk ch;
    ch.pl = c + 1 < op.n_chunks ? op.body : op.tail;
    const int64_t b0 = (int64_t)c * op.chunk_nb;
    ch.pl.n_ctx = n_ctx + b0 * pw.Hkv;
    ch.q = static_cast<const char*>(q) + b0 * pw.qsb * pw.elem;
    ch.k = static_cast<char*>(k) + b0 * pw.ksb * pw.elem;
    ch.v = static_cast<char*>(v) + b0 * pw.ksb * pw.elem;
    ch.ws = ws + (size_t)c * op.body.ws_total;
    ch.scores = scores_opt ? scores_opt + b0 * pw.Hkv * pw.N : reinterpret_cast<float*>(ch.ws + ch.pl.off_scores);
    ch.keep = keep_idx_opt ? keep_idx_opt + b0 * pw.Hkv * pw.keep_stride
                           : reinterpret_cast<int32_t*>(ch.ws + ch.pl.off_keep);
    ch.n_kept = n_kept + b0 * pw.Hkv;
    ch.budgets = budgets ? budgets + b0 : nullptr;
    ch.lse = row_lse_opt ? row_lse_opt + b0 * pw.Hq * pw.p : nullptr;
    return ch;
  };
  auto score = [&](int c, hipStream_t stream) -> int {
    const Chunk ch = chunk(c);
    return ch.lse ? run_score_lse(ch.pl, ch.q, ch.k, ch.lse, ch.scores, ch.ws, stream)
                  : run_score(ch.pl, ch.q, ch.k, ch.scores, ch.ws, stream);
  };
  auto select_and_compact = [&](int c, hipStream_t stream) -> int {
    Chunk ch = chunk(c);
    if (launch_select_ragged(ch.pl, select, ch.scores, ch.budgets, ch.keep, ch.n_kept, ch.ws + ch.pl.off_select,
                             stream) != hipSuccess)
      return EPICACHE_ERR_DEVICE;
    ch.pl.n_kept = ch.n_kept;
    if (launch_compact(ch.pl, ch.keep, ch.k, ch.v, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
    return EPICACHE_OK;
  };
  return run_chunks_on_two_streams(op.n_chunks, main_stream, aux_stream, score, select_and_compact);
}

int epicache_evict_step_lse(const epicache_params* params, const void* q, void* k, void* v,
                            const float* row_lse, float* scores_opt, int32_t* keep_idx_opt,
                            void* workspace, size_t workspace_bytes, void* hip_stream) {
  return evict_step_impl(params, q, k, v, row_lse, true, scores_opt, keep_idx_opt, workspace,
                         workspace_bytes, hip_stream);
}

int epicache_snapkv_workspace_size(const epicache_params* params, size_t* bytes_out) {
  if (!bytes_out) return EPICACHE_ERR_INVALID_ARG;
  SnapkvPlan sp;
  int st = make_snapkv_plan(params, &sp);
  if (st != EPICACHE_OK) return st;
  *bytes_out = sp.total;
  return EPICACHE_OK;
}

int epicache_evict_step_snapkv(const epicache_params* params, const void* q_window, void* k, void* v,
                               float* scores_opt, int32_t* keep_idx_opt, void* workspace, size_t workspace_bytes,
                               void* hip_stream) {
  SnapkvPlan sp;
  int st = make_snapkv_plan(params, &sp);
  if (st != EPICACHE_OK) return st;
  if (!q_window || !k || !v || !workspace) return EPICACHE_ERR_INVALID_ARG;
  if (misaligned(q_window) || misaligned(k) || misaligned(v) || misaligned(workspace) || misaligned(scores_opt) ||
      misaligned(keep_idx_opt))
    return EPICACHE_ERR_INVALID_ARG;
  if (k == v) return EPICACHE_ERR_INVALID_ARG;
  if (workspace_bytes < sp.total) return EPICACHE_ERR_WORKSPACE_TOO_SMALL;
  char* ws = static_cast<char*>(workspace);
  hipStream_t stream = (hipStream_t)hip_stream;
  float* scores = scores_opt ? scores_opt : reinterpret_cast<float*>(ws + sp.off_scores);
  int32_t* keep = keep_idx_opt ? keep_idx_opt : reinterpret_cast<int32_t*>(ws + sp.off_keep);
  const Plan& po = sp.outer;
  if (!sp.evicts) {  // the cache is still filling up: everything stays
    if (scores_opt && sp.scores) {
      st = run_score(sp.inner, q_window, k, scores, ws, stream);
      if (st != EPICACHE_OK) return st;
    }
    if (keep_idx_opt && launch_iota_keep(po, keep, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
    return EPICACHE_OK;
  }
  // N > M > w: score the rows before the window, keep the best M - w of them and the window itself
  st = run_score(sp.inner, q_window, k, scores, ws, stream);
  if (st != EPICACHE_OK) return st;
  Plan sel = sp.inner;
  sel.keep_stride = po.n_keep;  // the selection fills the first M - w entries of rows that are M long
  if (launch_topk(sel, scores, keep, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
  if (launch_append_rows(po, keep, po.M - po.p, po.p, po.N - po.p, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
  if (launch_compact(po, keep, k, v, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
  return EPICACHE_OK;
}

int epicache_kvzip_workspace_size(const epicache_params* params, size_t* bytes_out) {
  if (!bytes_out) return EPICACHE_ERR_INVALID_ARG;
  LongPatchPlan lp;
  int st = make_long_patch_plan(params, &lp);
  if (st != EPICACHE_OK) return st;
  *bytes_out = lp.total;
  return EPICACHE_OK;
}

int epicache_score_kvzip(const epicache_params* params, const void* q, const void* k, float* scores,
                         void* workspace, size_t workspace_bytes, void* hip_stream) {
  LongPatchPlan lp;
  int st = make_long_patch_plan(params, &lp);
  if (st != EPICACHE_OK) return st;
  if (!q || !k || !scores || !workspace) return EPICACHE_ERR_INVALID_ARG;
  if (misaligned(q) || misaligned(k) || misaligned(scores) || misaligned(workspace)) return EPICACHE_ERR_INVALID_ARG;
  if (workspace_bytes < lp.off_scores) return EPICACHE_ERR_WORKSPACE_TOO_SMALL;
  return run_score_long_patch(lp, q, k, scores, static_cast<char*>(workspace), (hipStream_t)hip_stream);
}

int epicache_evict_step_kvzip(const epicache_params* params, const void* q, void* k, void* v, float* scores_opt,
                              int32_t* keep_idx_opt, void* workspace, size_t workspace_bytes, void* hip_stream) {
  LongPatchPlan lp;
  int st = make_long_patch_plan(params, &lp);
  if (st != EPICACHE_OK) return st;
  if (!q || !k || !v || !workspace) return EPICACHE_ERR_INVALID_ARG;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(workspace) || misaligned(scores_opt) ||
      misaligned(keep_idx_opt))
    return EPICACHE_ERR_INVALID_ARG;
  if (k == v) return EPICACHE_ERR_INVALID_ARG;
  if (workspace_bytes < lp.total) return EPICACHE_ERR_WORKSPACE_TOO_SMALL;
  char* ws = static_cast<char*>(workspace);
  hipStream_t stream = (hipStream_t)hip_stream;
  float* scores = scores_opt ? scores_opt : reinterpret_cast<float*>(ws + lp.off_scores);
  int32_t* keep = keep_idx_opt ? keep_idx_opt : reinterpret_cast<int32_t*>(ws + lp.off_keep);
  const Plan& pw = lp.whole;
  if (pw.N <= pw.M) {  // nothing to evict
    if (scores_opt) {
      st = run_score_long_patch(lp, q, k, scores, ws, stream);
      if (st != EPICACHE_OK) return st;
    }
    if (keep_idx_opt && launch_iota_keep(pw, keep, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
    return EPICACHE_OK;
  }
  st = run_score_long_patch(lp, q, k, scores, ws, stream);
  if (st != EPICACHE_OK) return st;
  if (launch_topk(pw, scores, keep, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
  if (launch_compact(pw, keep, k, v, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
  return EPICACHE_OK;
}

int epicache_ragged_workspace_size(const epicache_params* params, int32_t select, size_t* bytes_out,
                                   int32_t* keep_capacity_out) {
  if (!bytes_out || !keep_capacity_out) return EPICACHE_ERR_INVALID_ARG;
  Plan pl;
  int st = make_ragged_plan(params, select, &pl);
  if (st != EPICACHE_OK) return st;
  *bytes_out = pl.ws_total;
  *keep_capacity_out = pl.keep_stride;
  return EPICACHE_OK;
}

int epicache_score_ragged(const epicache_params* params, const void* q, const void* k, const int32_t* n_ctx,
                          const float* row_lse_opt, float* scores, void* workspace, size_t workspace_bytes,
                          void* hip_stream) {
  Plan pl;
  int st = make_plan(params, &pl);
  if (st != EPICACHE_OK) return st;
  if (!q || !k || !n_ctx || !scores || !workspace) return EPICACHE_ERR_INVALID_ARG;
  if (misaligned(q) || misaligned(k) || misaligned(n_ctx) || misaligned(row_lse_opt) || misaligned(scores) ||
      misaligned(workspace))
    return EPICACHE_ERR_INVALID_ARG;
  if (row_lse_opt && pl.causal_patch) return EPICACHE_ERR_INVALID_ARG;
  if (workspace_bytes < pl.off_scores) return EPICACHE_ERR_WORKSPACE_TOO_SMALL;
  pl.n_ctx = n_ctx;
  char* ws = static_cast<char*>(workspace);
  hipStream_t stream = (hipStream_t)hip_stream;
  return row_lse_opt ? run_score_lse(pl, q, k, row_lse_opt, scores, ws, stream) : run_score(pl, q, k, scores, ws, stream);
}

int epicache_select_ragged(const epicache_params* params, int32_t select, const float* scores,
                           const int32_t* n_ctx, const int32_t* budgets, int32_t* keep_idx, int32_t* n_kept,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  Plan pl;
  int st = make_ragged_plan(params, select, &pl);
  if (st != EPICACHE_OK) return st;
  if (!scores || !n_ctx || !keep_idx || !n_kept || !workspace) return EPICACHE_ERR_INVALID_ARG;
  if (misaligned(scores) || misaligned(n_ctx) || misaligned(budgets) || misaligned(keep_idx) ||
      misaligned(n_kept) || misaligned(workspace))
    return EPICACHE_ERR_INVALID_ARG;
  if (workspace_bytes < pl.ws_total) return EPICACHE_ERR_WORKSPACE_TOO_SMALL;
  pl.n_ctx = n_ctx;
  hipError_t e = launch_select_ragged(pl, select, scores, budgets, keep_idx, n_kept,
                                      static_cast<char*>(workspace) + pl.off_select, (hipStream_t)hip_stream);
  return e == hipSuccess ? EPICACHE_OK : EPICACHE_ERR_DEVICE;
}

int epicache_compact_ragged(const epicache_params* params, int32_t select, const int32_t* keep_idx,
                            const int32_t* n_kept, void* k, void* v, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
  (void)workspace;
  (void)workspace_bytes;  // in-place gather, no staging buffer
  Plan pl;
  int st = make_ragged_plan(params, select, &pl);
  if (st != EPICACHE_OK) return st;
  if (!keep_idx || !n_kept || !k || !v) return EPICACHE_ERR_INVALID_ARG;
  if (misaligned(keep_idx) || misaligned(n_kept) || misaligned(k) || misaligned(v)) return EPICACHE_ERR_INVALID_ARG;
  if (k == v) return EPICACHE_ERR_INVALID_ARG;
  pl.n_kept = n_kept;
  hipError_t e = launch_compact(pl, keep_idx, k, v, (hipStream_t)hip_stream);
  return e == hipSuccess ? EPICACHE_OK : EPICACHE_ERR_DEVICE;
}

int epicache_evict_step_ragged(const epicache_params* params, int32_t select, const void* q, void* k, void* v,
                               const int32_t* n_ctx, const int32_t* budgets, const float* row_lse_opt,
                               int32_t* n_kept, float* scores_opt, int32_t* keep_idx_opt, void* workspace,
                               size_t workspace_bytes, void* hip_stream) {
  Plan pl;
  int st = make_ragged_plan(params, select, &pl);
  if (st != EPICACHE_OK) return st;
  if (!q || !k || !v || !n_ctx || !n_kept || !workspace) return EPICACHE_ERR_INVALID_ARG;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(n_ctx) || misaligned(budgets) ||
      misaligned(row_lse_opt) || misaligned(n_kept) || misaligned(scores_opt) || misaligned(keep_idx_opt) ||
      misaligned(workspace))
    return EPICACHE_ERR_INVALID_ARG;
  if (k == v || (row_lse_opt && pl.causal_patch)) return EPICACHE_ERR_INVALID_ARG;
  if (workspace_bytes < pl.ws_total) return EPICACHE_ERR_WORKSPACE_TOO_SMALL;
  char* ws = static_cast<char*>(workspace);
  hipStream_t stream = (hipStream_t)hip_stream;
  float* scores = scores_opt ? scores_opt : reinterpret_cast<float*>(ws + pl.off_scores);
  int32_t* keep = keep_idx_opt ? keep_idx_opt : reinterpret_cast<int32_t*>(ws + pl.off_keep);
  pl.n_ctx = n_ctx;
  st = row_lse_opt ? run_score_lse(pl, q, k, row_lse_opt, scores, ws, stream) : run_score(pl, q, k, scores, ws, stream);
  if (st != EPICACHE_OK) return st;
  if (launch_select_ragged(pl, select, scores, budgets, keep, n_kept, ws + pl.off_select, stream) != hipSuccess)
    return EPICACHE_ERR_DEVICE;
  pl.n_kept = n_kept;
  if (launch_compact(pl, keep, k, v, stream) != hipSuccess) return EPICACHE_ERR_DEVICE;
  return EPICACHE_OK;
}

int epicache_episode_medoids(const float* embeddings, const int32_t* assignment, int32_t n_segments,
                             int32_t n_episodes, int32_t dim, float* centroids_out, int32_t* medoid_out,
                             void* hip_stream) {
  if (!embeddings || !assignment || !centroids_out || !medoid_out) return EPICACHE_ERR_INVALID_ARG;
  if (n_segments < 1 || n_episodes < 1 || dim < 1) return EPICACHE_ERR_INVALID_ARG;
  if (dim > 8192 || n_episodes > 65535) return EPICACHE_ERR_UNSUPPORTED;  // centroid in LDS, one workgroup each
  hipError_t e = launch_episode_medoids(embeddings, assignment, n_segments, n_episodes, dim, centroids_out,
                                        medoid_out, (hipStream_t)hip_stream);
  return e == hipSuccess ? EPICACHE_OK : EPICACHE_ERR_DEVICE;
}

int epicache_match_queries(const float* queries, const float* centroids, int32_t n_queries, int32_t n_episodes,
                           int32_t dim, float tau, int32_t* episode_out, float* cosine_out_opt,
                           void* hip_stream) {
  if (!queries || !centroids || !episode_out) return EPICACHE_ERR_INVALID_ARG;
  if (n_queries < 1 || n_episodes < 1 || dim < 1 || tau != tau) return EPICACHE_ERR_INVALID_ARG;
  hipError_t e = launch_match_queries(queries, centroids, n_queries, n_episodes, dim, tau, episode_out,
                                      cosine_out_opt, (hipStream_t)hip_stream);
  return e == hipSuccess ? EPICACHE_OK : EPICACHE_ERR_DEVICE;
}

int epicache_layer_budgets(const double* sensitivity, int32_t n_layers, double alpha, int32_t budget,
                           int32_t* budgets_out) {
  if (!sensitivity || !budgets_out || n_layers < 1 || budget < 1) return EPICACHE_ERR_INVALID_ARG;
  if (!(alpha >= 0.0) || isinf(alpha)) return EPICACHE_ERR_INVALID_ARG;
  if ((int64_t)n_layers * budget > INT32_MAX) return EPICACHE_ERR_UNSUPPORTED;
  std::vector<double> w(n_layers);
  double wsum = 0.0;
  for (int l = 0; l < n_layers; l++) {
    if (!(sensitivity[l] >= 0.0) || isinf(sensitivity[l])) return EPICACHE_ERR_INVALID_ARG;
    w[l] = pow(sensitivity[l], alpha);
    wsum += w[l];
  }
  const int64_t total = (int64_t)n_layers * budget;
  if (!(wsum > 0.0) || isinf(wsum)) {  // nothing to go by: uniform
    for (int l = 0; l < n_layers; l++) budgets_out[l] = budget;
    return EPICACHE_OK;
  }
  std::vector<double> frac(n_layers);
  int64_t given = 0;
  for (int l = 0; l < n_layers; l++) {
    const double quota = w[l] / wsum * (double)total;  // Eq. 6
    const double fl = floor(quota);
    budgets_out[l] = (int32_t)fl;
    frac[l] = quota - fl;
    given += budgets_out[l];
  }
  for (int64_t left = total - given; left > 0; left--) {  // largest remainder first, ties to the lower layer
    int best = 0;
    for (int l = 1; l < n_layers; l++)
      if (frac[l] > frac[best]) best = l;
    budgets_out[best] += 1;
    frac[best] = -1.0;
  }
  for (int l = 0; l < n_layers; l++) {  // no layer without a row
    if (budgets_out[l] >= 1) continue;
    int big = 0;
    for (int j = 1; j < n_layers; j++)
      if (budgets_out[j] > budgets_out[big]) big = j;
    budgets_out[big] -= 1;
    budgets_out[l] = 1;
  }
  return EPICACHE_OK;
}

const char* epicache_status_string(int status) {
  switch (status) {
    case EPICACHE_OK: return "ok";
    case EPICACHE_ERR_INVALID_ARG: return "invalid argument";
    case EPICACHE_ERR_UNSUPPORTED: return "unsupported configuration";
    case EPICACHE_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case EPICACHE_ERR_DEVICE: return "HIP runtime error";
    default: return "unknown status";
  }
}

const char* epicache_version(void) { return "0.1.0"; }

}  // extern "C"
