// Internal plan shared by the host API and the gfx950 kernels of libspeckv.
// Not part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstdlib>
#include <cstring>

#include "speckv.h"

namespace speckv {

constexpr int kMaxSeqs = SPECKV_MAX_SEQS;

// Per-sequence prefix tables, passed to kernels by value (kernarg segment).
struct SeqTab {
  int32_t n_seqs;
  int32_t cu[kMaxSeqs + 1];   // token prefix sums
  int32_t ck[kMaxSeqs + 1];   // prefix sums of n_keep_s
  int32_t cc[kMaxSeqs + 1];   // prefix sums of the unmasked key chunks (scoring grid)
  int32_t tail0[kMaxSeqs];    // first key of the masked tail: keys below it are visible to every row
};

struct Dims {
  int32_t L, S, Hq, Hkv, G, D, elt;       // elt = bytes per element (2 bf16 / f16, 4 f32)
  int32_t dt;                              // speckv_dtype of q, k, v
  int32_t w, a, R, M;                      // M = G * R rows per KV group
  int32_t pool_k, c_max;
  int32_t reduce_max;                      // 1: max over the rows of a head instead of the sum
  int32_t head_max;                        // 1: heads (and layers) combined by max instead of sum
  int32_t pool_avg;                        // 1: zero-padded mean instead of the clipped max
  int32_t weight_rows;                     // 1: window row i scaled by (i + 1) / n_window (Alg. 2)
  float sm_scale;
  int64_t q_sl, q_ss, q_sr, q_sh;          // element strides
  int64_t kv_sl, kv_st, kv_sh;
  int64_t T, KT;                           // total tokens, total kept rows
  const int32_t *n_dev;                    // device-side token count of a one-sequence call, or null
};

// Geometry of the scoring launches (Alg. 1 CrossAttention + reduce).
struct ScoreGeom {
  int32_t MB;         // 32-row blocks per wave
  int32_t NW;         // waves per workgroup
  int32_t RSB;        // rows per workgroup = NW * MB * 32
  int32_t RS;         // row super-blocks per KV group
  int32_t Rp;         // observation rows per head, padded to a multiple of 32
  int32_t HPS;        // whole heads per super-block (when a head fits), else 1
  int32_t PPH;        // super-blocks per head (1 when a head fits)
  int32_t KC;         // keys per chunk (multiple of the LDS tile)
  int32_t n_fast_chunks;   // unmasked chunks over all sequences = cc[S]
  int32_t n_chunks;        // n_fast_chunks + one masked tail chunk per sequence
};

struct Plan {
  Dims d;
  SeqTab t;
  ScoreGeom g;
  // workspace carve-up (byte offsets, 256-aligned)
  size_t off_part, off_lse, off_planes, off_pooled, off_pooled2, off_sel, total;
  size_t off_ada_hist, off_ada_state, total_ada;   // extra scratch of the shared-budget selection
  // selection of long rows in calls with few rows: parts per row (1: not split), keys per part, scratch
  int32_t sel_parts, sel_part_len;
  size_t off_sel_hist, off_sel_state;
  // first-digit histograms of the pooled rows (2048 counters per row), filled by the pooling kernel
  // of a fused call so that selection starts at the second read; hist0_words == 0: not used
  size_t off_hist0;
  int64_t hist0_words;
};

inline __host__ __device__ int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// Tokens of sequence s as the kernels see them.  Normally the host's length; with a device-side
// count (one-sequence calls only) that count, clamped to [max(1, n_window), host length].  The
// host length stays the row stride of every layout and the bound of every grid.
__device__ inline int live_len(const Dims &d, const SeqTab &t, int s) {
  const int n_host = t.cu[s + 1] - t.cu[s];
  if (d.n_dev == nullptr) return n_host;
  const int lo = d.w > 1 ? d.w : 1;
  const int v = *d.n_dev;
  return v < lo ? lo : (v > n_host ? n_host : v);
}
// First key of the masked tail for a live length n: keys below it are whole LDS tiles (kt keys)
// that every observation row may see (key <= n - n_window).
__device__ inline int live_tail0(const Dims &d, const SeqTab &t, int s, int n, int kt) {
  if (d.n_dev == nullptr) return t.tail0[s];
  const int visible = n - d.w + 1 < n ? n - d.w + 1 : n;
  return visible / kt * kt;
}

// Raises a kernel's dynamic LDS limit; the runtime call is made once per (device, kernel, size)
// and remembered (score.hip).
hipError_t allow_dynamic_lds(const void *kernel, size_t bytes);

// Kernel launchers (each returns the hipError of its launches).
hipError_t launch_compact(const Plan &pl, const void *k, const void *v, const int32_t *idx,
                          void *k_out, void *v_out, hipStream_t st);
// `events`, when not null, holds 4 hipEvent_t recorded before pass 1, before the merge of the
// row statistics, before pass 2 and after pass 2.
// `lse_in`, when not null, holds natural-log row normalisers [L][S][R][Hq]; the row-statistics
// sweep is skipped and only the column reduction runs.
// `clear`, when not null, is scratch of clear_words 32-bit words that the call leaves zeroed (done
// by the small kernel between the sweeps: the fused calls need zeroed counters for the pooling
// kernel and must not use a memset, which a captured graph may not contain).
// ints behind the partial pairs of the row-statistics sweep (one short list per chunk workgroup)
int64_t score_fail_words(const Plan &pl);
// Workgroups of one scoring sweep: chunk workgroups ((layer, head, chunk) items rounded up to a
// multiple of 8, times the row super-blocks) plus one masked tail per (unit, sequence).
inline int64_t score_chunk_workgroups(const Dims &d, const ScoreGeom &g) {
  return ((int64_t)g.n_fast_chunks * d.L * d.Hkv + 7) / 8 * 8 * g.RS;
}
// True when the key-tile row-statistics sweep sums against fixed reference exponents and a repair
// launch follows it.  That pays when the sweep runs for several rounds of workgroups; in a
// one-round sweep the repair launch (a few microseconds when it has nothing to do, a segment's
// duration when it has) costs more than the first sweep gains.
// The environment can override the choice (read on every call so that a test can switch it):
// SPECKV_ROW_STATISTICS=fixed (always) or online (never).
inline bool score_rows_fixed_reference(const Dims &d, const ScoreGeom &g) {
  const char *e = std::getenv("SPECKV_ROW_STATISTICS");
  if (e != nullptr && std::strcmp(e, "fixed") == 0) return true;
  if (e != nullptr && std::strcmp(e, "online") == 0) return false;
  return score_chunk_workgroups(d, g) + (int64_t)d.L * d.Hkv * g.RS * d.S > 2 * 256;
}
hipError_t launch_score(const Plan &pl, const void *q, const void *k, float2 *part, float *lse,
                        float *planes, hipStream_t st, hipEvent_t *events = nullptr,
                        const float *lse_in = nullptr, uint32_t *clear = nullptr, int64_t clear_words = 0);
// True when sweep `pass` (1 row statistics, 2 column reduction) over the unmasked chunks of this
// plan runs in the Q-stationary kernel (score_qs.hip) rather than the tile-streaming one
// (score_sweep.h); diagnostics only.
bool score_uses_qs(const Plan &pl, int pass);
// Row `lr` of super-block `rs` -> (head in group, observation row); false for padding rows.
// Heads never share a 32-row block: each head's R rows are padded to Rp, and a super-block holds
// either HPS whole heads or one of the PPH slices of a single head.
__host__ __device__ inline bool decode_row(const Dims &d, const ScoreGeom &g, int rs, int lr, int *hh, int *i) {
  if (g.PPH == 1) {
    *hh = rs * g.HPS + lr / g.Rp;
    *i = lr % g.Rp;
    return lr < g.HPS * g.Rp && *hh < d.G && *i < d.R;
  }
  *hh = rs / g.PPH;
  *i = (rs % g.PPH) * g.RSB + lr;
  return *i < d.R;
}

// out rows = (layer, seq, head): pooled/raw in the "scores" layout from RS planes.
// hist0, when not null: [rows][2048] zeroed counters; the kernel adds the first-digit histogram of
// every row's pooled scores (the non-window entries), for launch_select.
hipError_t launch_reduce_pool(const Plan &pl, const float *planes, float *raw, float *pooled,
                              hipStream_t st, uint32_t *hist0 = nullptr);
// single output row summing every plane of a one-sequence call (prompt-token selection)
hipError_t launch_reduce_pool_all(const Plan &pl, const float *planes, float *raw, float *pooled,
                                  hipStream_t st);
// max-pool (kernel pool_k, clipped to [0, n_in - n_window)) of one row of n_in scores
hipError_t launch_pool_row(const float *in, float *out, int32_t n_in, int32_t n_window, int32_t pool_k,
                           hipStream_t st);
// hist / state: scratch of the split-row path (off_sel_hist, off_sel_state); with either null, or when
// the plan does not split rows (sel_parts == 1), every row is ranked by one workgroup.
// hist0, when not null: the rows' first-digit histograms from launch_reduce_pool (one-workgroup path).
hipError_t launch_select(const Plan &pl, const float *pooled, int32_t *idx, uint32_t *hist, uint32_t *state,
                         hipStream_t st, const uint32_t *hist0 = nullptr);
// Shared layer budget: head offsets from a layer-wide threshold, then per-head selection.
// hist: L*S*Hkv*2048 uint32, state: L*S*(2 + 3*Hkv) uint32 of scratch.
hipError_t launch_select_ada(const Plan &pl, int32_t c_floor, const float *pooled, int32_t *idx,
                             int32_t *head_off, uint32_t *hist, uint32_t *state, hipStream_t st);
hipError_t launch_compact_ada(const Plan &pl, const void *k, const void *v, const int32_t *idx,
                              const int32_t *head_off, void *k_out, void *v_out, hipStream_t st);
hipError_t launch_select_row(const float *pooled_row, int32_t m, int32_t count, int32_t *sel,
                             hipStream_t st);
hipError_t launch_expand(const int32_t *sel, int32_t count, int32_t n_in, int32_t n_window,
                         int32_t n_neighbor, const int32_t *token_ids, int32_t *idx_out,
                         int32_t *ids_out, int32_t *count_out, hipStream_t st);

}  // namespace speckv
