// Internal declarations shared by the HIP translation units of libepicache.
// Not part of the C ABI (see include/epicache.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "epicache.h"

namespace epicache {

// Everything the launchers need, derived once on the host from epicache_params.
struct Plan {
  int nb, Hq, Hkv, G, d, p;
  int N;        // context rows scored: n_cached + n_block
  int R;        // rows that vote for one KV head: G * p
  int Rpad;     // R rounded up to 64
  int M;        // budget
  int n_keep;   // min(M, N)
  int dtype, reduce;
  int causal_patch;  // the p rows after a head's context are the patch's keys, seen causally by the queries
  int elem;     // bytes per element of Q/K/V
  float c2;     // softmax scale * log2(e): logits are handled in base 2
  int64_t qsb, qsh, qst, ksb, ksh, kst;  // strides in elements
  // score kernels
  int use_mfma;     // bf16 MFMA path (d == 64 or 128), else the generic path
  int stats_rows_per_wg;  // query rows per workgroup of the row-statistics pass
  int n_splits;     // key splits of the row-statistics pass
  int tiles_per_split;
  int reduce_splits;  // key splits of the streaming reduction pass
  int reduce_tiles_per_split;
  // workspace layout (byte offsets, 256-aligned)
  size_t off_stats, off_nlse, off_scores, off_keep, off_lse, ws_total;
  // ragged batches: device arrays indexed by b * Hkv + h, null in the uniform calls
  const int32_t* n_ctx;   // context rows per (b, h), at most N; N is then the pitch of a score row
  const int32_t* n_kept;  // rows kept per (b, h), read by the compaction
  int keep_stride;        // pitch of a row of kept indices (n_keep in the uniform calls)
  size_t off_select;      // per-(b, h) threshold records of the ragged selection
};

// Context rows of (b, h): the per-head length of a ragged batch, clamped to what the strides were checked for.
__device__ __forceinline__ int ctx_rows(const Plan& pl, int bh) {
  if (!pl.n_ctx) return pl.N;
  const int n = pl.n_ctx[bh];
  return n < 0 ? 0 : (n > pl.N ? pl.N : n);
}

constexpr int kKeyTile = 64;     // keys staged per LDS tile in the statistics pass
constexpr int kKeysPerWG = 256;  // keys per workgroup in the reduction pass

int make_plan(const epicache_params* prm, Plan* out);

// Each launcher enqueues on `stream` and returns a hipError_t.
// `stats_ready`: the row statistics are already in `stats` (one split); only the reduction pass runs.
hipError_t launch_score_generic(const Plan& pl, const void* q, const void* k, float* scores,
                                float2* stats, bool stats_ready, hipStream_t stream);
// `nlse` [nb * Hkv, Rpad]: minus the base-2 log-sum-exp of every scoring row, written between the two passes
hipError_t launch_score_mfma(const Plan& pl, const void* q, const void* k, float* scores,
                             float2* stats, float* nlse, bool stats_ready, hipStream_t stream);
hipError_t launch_lse_to_stats(const Plan& pl, const float* row_lse, float2* stats, hipStream_t stream);
hipError_t launch_topk(const Plan& pl, const float* scores, int32_t* keep, hipStream_t stream);
hipError_t launch_iota_keep(const Plan& pl, int32_t* keep, hipStream_t stream);
// keep[bh][first + j] = row0 + j, j < count (rows of pitch pl.keep_stride): rows retained unconditionally
hipError_t launch_append_rows(const Plan& pl, int32_t* keep, int first, int count, int row0, hipStream_t stream);
// dst = reduce(dst, src) elementwise over [nb, Hkv, N] scores (pl.reduce)
hipError_t launch_combine_scores(const Plan& pl, float* dst, const float* src, hipStream_t stream);
hipError_t launch_compact(const Plan& pl, const int32_t* keep, void* k, void* v,
                          hipStream_t stream);
size_t select_ragged_record_bytes(const Plan& pl);
// KeyDiff scoring: chunk sums of the keys live at the start of the workspace.
size_t keydiff_workspace_bytes(const Plan& pl);
hipError_t launch_score_keydiff(const Plan& pl, const void* k, float* scores, void* workspace,
                                hipStream_t stream);
// Ragged selection: per-(b, h) (select == per head) or per-b pooled thresholds, then the kept indices.
hipError_t launch_select_ragged(const Plan& pl, int select, const float* scores, const int32_t* budgets,
                                int32_t* keep, int32_t* n_kept, void* records, hipStream_t stream);

// Attention output and log-sum-exp of the patch queries (dense out [nb, Hq, p, d], lse [nb, Hq, p]).
hipError_t launch_patch_attention(const Plan& pl, const void* q, const void* k, const void* v, void* out,
                                  float* lse, hipStream_t stream);
// Episode geometry on fp32 embeddings: cluster centroids + centroid-closest members, query matching.
hipError_t launch_episode_medoids(const float* emb, const int32_t* assign, int K, int E, int D,
                                  float* centroids, int32_t* medoid, hipStream_t stream);
hipError_t launch_match_queries(const float* queries, const float* centroids, int nq, int E, int D, float tau,
                                int32_t* episode, float* cosine_opt, hipStream_t stream);

}  // namespace epicache
