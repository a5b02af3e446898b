// Host side of libspeckv: argument validation, launch planning, workspace carve-up and the
// extern "C" entry points declared in speckv.h.  Nothing here touches the device except
// kernel launches on the caller's stream.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>

#include "speckv_internal.h"

namespace speckv {
namespace {

constexpr int64_t kTokenLimit = (int64_t)1 << 30;   // total tokens per call
constexpr int kTargetWorkgroups = 1024;             // scoring grid: at least about 4 workgroups per CU
constexpr int kChunkFloor = 8192;                   // chunks are not shortened below this to balance the grid
constexpr int kWorkgroupCost = 190;                 // fixed cost of a scoring workgroup, in keys (measured)
constexpr int kCUs = 256;                           // compute units of an MI355X
constexpr int kChunkAlign = 256;                    // chunk = whole LDS key tiles (the largest tile)
constexpr int kSelSplitMinKeys = 1 << 18;            // rows at least this long may be ranked by several workgroups
constexpr int kSelSplitWorkgroups = 512;            // ... when the call has fewer than half this many rows
constexpr int kSelSplitMaxParts = 64;
constexpr int kChunkMin = 512;                      // shortest chunk
constexpr int kChunkSmallCap = 4096;                // longest chunk that small problems are given

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Fills the dimension and per-sequence tables.  Returns SPECKV_OK or the reason.
speckv_status build_plan(const speckv_params *p, Plan *pl, bool one_row_per_call, int32_t top_k) {
  if (p == nullptr) return SPECKV_ERR_INVALID_ARG;
  std::memset(pl, 0, sizeof(*pl));
  Dims &d = pl->d;
  if (p->n_seqs < 1 || p->n_layers < 1 || p->n_kv_heads < 1 || p->n_q_heads < 1) return SPECKV_ERR_INVALID_ARG;
  if (p->n_q_heads % p->n_kv_heads != 0) return SPECKV_ERR_INVALID_ARG;
  if (p->n_window < 0 || p->n_lookahead < 0 || p->n_window + (int64_t)p->n_lookahead < 1) return SPECKV_ERR_INVALID_ARG;
  if (p->pool_k < 1 || p->c_max < 0) return SPECKV_ERR_INVALID_ARG;
  if (!(p->sm_scale > 0.f) || !std::isfinite(p->sm_scale)) return SPECKV_ERR_INVALID_ARG;
  if (p->dtype != SPECKV_BF16 && p->dtype != SPECKV_F32 && p->dtype != SPECKV_F16) return SPECKV_ERR_INVALID_ARG;
  if (p->reduce_op != SPECKV_REDUCE_SUM && p->reduce_op != SPECKV_REDUCE_MAX) return SPECKV_ERR_INVALID_ARG;
  if (p->pool_op != SPECKV_POOL_MAX && p->pool_op != SPECKV_POOL_AVG) return SPECKV_ERR_INVALID_ARG;
  if (p->n_seqs > SPECKV_MAX_SEQS) return SPECKV_ERR_UNSUPPORTED;
  if (p->head_dim != 64 && p->head_dim != 128) return SPECKV_ERR_UNSUPPORTED;
  if (p->pool_k > SPECKV_MAX_POOL_K) return SPECKV_ERR_UNSUPPORTED;
  if (one_row_per_call && p->n_seqs != 1) return SPECKV_ERR_UNSUPPORTED;

  d.L = p->n_layers; d.S = p->n_seqs; d.Hq = p->n_q_heads; d.Hkv = p->n_kv_heads;
  d.G = d.Hq / d.Hkv; d.D = p->head_dim; d.elt = p->dtype == SPECKV_F32 ? 4 : 2; d.dt = p->dtype;
  d.w = p->n_window; d.a = p->n_lookahead; d.R = d.w + d.a;
  d.pool_k = p->pool_k; d.c_max = p->c_max; d.sm_scale = p->sm_scale;
  d.reduce_max = p->reduce_op == SPECKV_REDUCE_MAX; d.pool_avg = p->pool_op == SPECKV_POOL_AVG;
  d.head_max = 0; d.weight_rows = 0;
  if ((int64_t)d.G * d.R > SPECKV_MAX_GROUP_ROWS) return SPECKV_ERR_UNSUPPORTED;
  d.M = d.G * d.R;
  d.q_sl = p->q_stride_layer; d.q_ss = p->q_stride_seq; d.q_sr = p->q_stride_row; d.q_sh = p->q_stride_head;
  d.kv_sl = p->kv_stride_layer; d.kv_st = p->kv_stride_token; d.kv_sh = p->kv_stride_head;
  const int64_t strides[7] = {d.q_sl, d.q_ss, d.q_sr, d.q_sh, d.kv_sl, d.kv_st, d.kv_sh};
  for (int64_t sv : strides)
    if (sv < 0 || (sv * d.elt) % 16 != 0) return SPECKV_ERR_INVALID_ARG;
  if (d.q_sr < d.D || d.q_sh < d.D || d.kv_st < d.D || d.kv_sh < d.D) return SPECKV_ERR_INVALID_ARG;
  if (d.kv_st * d.elt >= ((int64_t)1 << 23)) return SPECKV_ERR_UNSUPPORTED;   // 32-bit offsets inside a 128-key tile

  SeqTab &t = pl->t;
  t.n_seqs = d.S;
  t.cu[0] = 0; t.ck[0] = 0;
  if (p->cu_seqlens == nullptr) {
    if (d.S != 1) return SPECKV_ERR_INVALID_ARG;
    if (p->n_in < 1 || p->n_in > kTokenLimit) return p->n_in < 1 ? SPECKV_ERR_INVALID_ARG : SPECKV_ERR_UNSUPPORTED;
    t.cu[1] = (int32_t)p->n_in;
  } else {
    if (p->cu_seqlens[0] != 0) return SPECKV_ERR_INVALID_ARG;
    for (int s = 0; s < d.S; ++s) {
      if (p->cu_seqlens[s + 1] < p->cu_seqlens[s]) return SPECKV_ERR_INVALID_ARG;
      if ((int64_t)p->cu_seqlens[s + 1] > kTokenLimit) return SPECKV_ERR_UNSUPPORTED;
      t.cu[s + 1] = p->cu_seqlens[s + 1];
    }
  }
  for (int s = 0; s < d.S; ++s) {
    const int n_s = t.cu[s + 1] - t.cu[s];
    if (n_s < 1 || n_s < d.w) return SPECKV_ERR_INVALID_ARG;
    const int m = n_s - d.w;
    t.ck[s + 1] = t.ck[s] + (d.c_max < m ? d.c_max : m) + d.w;
  }
  d.T = t.cu[d.S];
  d.KT = t.ck[d.S];
  // a device-side token count replaces the host's length inside the kernels (one sequence only)
  d.n_dev = p->n_in_dev;
  if (d.n_dev != nullptr) {
    if (d.S != 1 || one_row_per_call) return SPECKV_ERR_UNSUPPORTED;
    if (reinterpret_cast<uintptr_t>(d.n_dev) & 3u) return SPECKV_ERR_INVALID_ARG;
  }

  // scoring geometry.  Every head's R rows are padded to Rp (a multiple of the 32-row MFMA block)
  // so that no block mixes heads; (waves, blocks per wave): small groups use 4 waves, larger ones
  // 8 waves so that two waves share each SIMD and the matrix and vector pipes overlap across them.
  ScoreGeom &g = pl->g;
  g.Rp = (d.R + 31) / 32 * 32;
  const int64_t m_pad = (int64_t)d.G * g.Rp;
  if (m_pad <= 128) { g.NW = 4; g.MB = 1; }
  else if (m_pad <= 256 || d.D * d.elt > 256) { g.NW = 8; g.MB = 1; }
  else { g.NW = 8; g.MB = 2; }
  g.RSB = g.NW * g.MB * 32;
  if (g.Rp <= g.RSB) {            // whole heads per super-block, spread evenly over the super-blocks
    const int fit = g.RSB / g.Rp;
    g.PPH = 1; g.RS = (d.G + fit - 1) / fit; g.HPS = (d.G + g.RS - 1) / g.RS;
  } else {                        // one head spread over PPH super-blocks
    g.HPS = 1; g.PPH = (g.Rp + g.RSB - 1) / g.RSB; g.RS = d.G * g.PPH;
  }
  const int64_t units = (int64_t)d.L * d.Hkv * g.RS;
  if (units > (int64_t)1 << 24) return SPECKV_ERR_UNSUPPORTED;       // grid sizes stay far below 2^31
  // Keys [0, tail0) of a sequence are complete LDS tiles visible to every observation row
  // (key <= m); they are cut into chunks of KC keys.  The rest is one masked tail chunk.
  const int rowb = d.D * d.elt;
  const int kt = rowb <= 128 ? 256 : rowb <= 256 ? 128 : 64;          // keys per LDS tile of the scoring kernels
  int64_t fast_keys = 0;
  for (int s = 0; s < d.S; ++s) {
    const int n_s = t.cu[s + 1] - t.cu[s];
    const int visible_to_all = n_s - d.w + 1 < n_s ? n_s - d.w + 1 : n_s;    // keys 0..m, clipped
    t.tail0[s] = visible_to_all / kt * kt;
    fast_keys += t.tail0[s];
  }
  // Chunk length.  A workgroup pays for loading its Q fragments and row normalisers (about
  // kWorkgroupCost keys' worth of time), so chunks should not be short; but the grid runs in rounds
  // of one workgroup per CU, so few or unequal workgroups (ragged batches) leave CUs idle at the
  // end.  Start from about four workgroups per CU and halve the chunk while a simple model of the
  // sweep's duration (in key-times per CU) improves; tiny problems get longer chunks (up to 4096
  // keys) as long as one workgroup per CU remains.
  const int64_t many = (kTargetWorkgroups + units - 1) / units, few = (kCUs + units - 1) / units;
  auto sweep_time = [&](int64_t kc_) {
    int64_t chunks = 0;
    bool equal = true;
    for (int s = 0; s < d.S; ++s) {
      chunks += (t.tail0[s] + kc_ - 1) / kc_;
      if (t.tail0[s] % kc_ != 0) equal = false;
    }
    const double n_wg = (double)chunks * (double)units;
    const double rounds = std::ceil(n_wg / kCUs) * (double)(kc_ + kWorkgroupCost);
    if (equal) return rounds;                                   // identical workgroups: whole rounds
    const double spread = ((double)fast_keys * (double)units + n_wg * kWorkgroupCost) / kCUs +
                          0.75 * (double)(kc_ + kWorkgroupCost);  // even spread plus a ragged last round
    return rounds < spread ? rounds : spread;
  };
  int64_t kc = align_up((fast_keys + many - 1) / many, kChunkAlign);
  if (kc > kChunkFloor) {
    double best = sweep_time(kc);
    for (int64_t cand = (int64_t)1 << 20; cand >= kChunkFloor; cand >>= 1) {
      if (cand >= kc) continue;
      const double tm = sweep_time(cand);
      if (tm < best) { best = tm; kc = cand; }
    }
  }
  int64_t kc_few = align_up((fast_keys + few - 1) / few, kChunkAlign);
  if (kc_few > kChunkSmallCap) kc_few = kChunkSmallCap;
  if (kc < kc_few) kc = kc_few;
  if (kc < kChunkMin) kc = kChunkMin;
  // The masked tails run as workgroups of the same launch (one per unit and sequence).  When the
  // chunk workgroups alone fit one round of the CUs but not together with the tails, the chunk
  // workgroups that have to wait for a tail's CU finish a tail's duration after all others;
  // chunks up to a quarter longer that bring everything into one round are cheaper.
  {
    auto chunk_wgs = [&](int64_t kc_) {
      int64_t chunks = 0;
      for (int s = 0; s < d.S; ++s) chunks += (t.tail0[s] + kc_ - 1) / kc_;
      return chunks * units;
    };
    const int64_t tails = units * d.S;
    if (chunk_wgs(kc) <= kCUs && chunk_wgs(kc) + tails > kCUs) {
      for (int64_t longer = kc + kt; longer <= kc + kc / 4; longer += kt)
        if (chunk_wgs(longer) + tails <= kCUs) { kc = longer; break; }
    }
  }
  g.KC = (int32_t)kc;
  t.cc[0] = 0;
  for (int s = 0; s < d.S; ++s) t.cc[s + 1] = t.cc[s] + (t.tail0[s] + g.KC - 1) / g.KC;
  g.n_fast_chunks = t.cc[d.S];
  g.n_chunks = g.n_fast_chunks + d.S;

  // workspace carve-up
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = (size_t)align_up((int64_t)(off + bytes), 256); return o; };
  // partial pairs of the row-statistics sweep, and behind them the segments its chunk workgroups
  // leave for the repair launch (score_fail_words ints)
  pl->off_part = take((size_t)units * g.n_chunks * g.RSB * sizeof(float2) + (size_t)score_fail_words(*pl) * sizeof(int32_t));
  pl->off_lse = take((size_t)d.L * d.Hkv * d.S * g.RS * g.RSB * sizeof(float));
  pl->off_planes = take((size_t)g.RS * d.L * d.Hkv * d.T * sizeof(float));
  pl->off_pooled = take(one_row_per_call ? (size_t)d.T * sizeof(float) : (size_t)d.L * d.Hkv * d.T * sizeof(float));
  pl->off_pooled2 = take(one_row_per_call ? (size_t)d.T * sizeof(float) : 0);
  pl->off_sel = take(one_row_per_call ? (size_t)(top_k > 0 ? top_k : 0) * sizeof(int32_t) : 0);
  // Selection: one workgroup per row unless the call has few, long rows; then each row is cut into
  // parts so that about kSelSplitWorkgroups workgroups share the ranking.
  pl->sel_parts = 1; pl->sel_part_len = 0; pl->off_sel_hist = 0; pl->off_sel_state = 0;
  if (!one_row_per_call) {
    const int64_t rows = (int64_t)d.L * d.S * d.Hkv;
    int max_m = 0;
    for (int s = 0; s < d.S; ++s) max_m = std::max(max_m, t.cu[s + 1] - t.cu[s] - d.w);
    if (max_m >= kSelSplitMinKeys && rows * 2 <= kSelSplitWorkgroups) {
      int parts = (int)(kSelSplitWorkgroups / rows);
      if (parts > kSelSplitMaxParts) parts = kSelSplitMaxParts;
      pl->sel_part_len = (int32_t)align_up((max_m + parts - 1) / parts, 1024);
      pl->sel_parts = (max_m + pl->sel_part_len - 1) / pl->sel_part_len;
      pl->off_sel_hist = take((size_t)rows * pl->sel_parts * 2048 * sizeof(uint32_t));
      pl->off_sel_state = take((size_t)rows * (2 + 2 * (size_t)pl->sel_parts) * sizeof(uint32_t));
    }
  }
  // first-digit histograms of the pooled rows for the one-workgroup selection of the fused calls
  pl->off_hist0 = 0; pl->hist0_words = 0;
  if (!one_row_per_call && pl->sel_parts == 1) {
    pl->hist0_words = (int64_t)d.L * d.S * d.Hkv * 2048;
    pl->off_hist0 = take((size_t)pl->hist0_words * sizeof(uint32_t));
  }
  pl->total = off;
  pl->off_ada_hist = take((size_t)d.L * d.S * d.Hkv * 2048 * sizeof(uint32_t));
  pl->off_ada_state = take((size_t)d.L * d.S * (2 + 3 * (size_t)d.Hkv) * sizeof(uint32_t));
  pl->total_ada = off;
  return SPECKV_OK;
}

speckv_status check_ws(const Plan &pl, const void *ws, size_t ws_bytes) {
  if (ws == nullptr || (reinterpret_cast<uintptr_t>(ws) & 255u) != 0 || ws_bytes < pl.total) return SPECKV_ERR_WORKSPACE;
  return SPECKV_OK;
}

speckv_status from_hip(hipError_t e) { return e == hipSuccess ? SPECKV_OK : SPECKV_ERR_RUNTIME; }

// Scratch of speckv_compress_static: one array per GPU, part of the library's code object, so a
// caller that may not allocate (HIP graph capture, a serving loop) still has a workspace.  The
// name below is only a host-side handle; the device address is looked up once per device with
// hipGetSymbolAddress and that pointer is what the kernels and every other host use get.
static __device__ __align__(256) unsigned char scratch[SPECKV_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

speckv_status static_scratch(void **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SPECKV_ERR_RUNTIME;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return SPECKV_ERR_RUNTIME;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return SPECKV_OK;
}

}  // namespace
}  // namespace speckv

using namespace speckv;

extern "C" {

const char *speckv_status_string(speckv_status status) {
  switch (status) {
    case SPECKV_OK: return "ok";
    case SPECKV_ERR_INVALID_ARG: return "invalid argument";
    case SPECKV_ERR_UNSUPPORTED: return "unsupported configuration";
    case SPECKV_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SPECKV_ERR_RUNTIME: return "HIP runtime error";
  }
  return "unknown status";
}

int64_t speckv_n_keep(const speckv_params *p, int32_t seq) {
  Plan pl;
  if (build_plan(p, &pl, false, 0) != SPECKV_OK || seq < 0 || seq >= pl.d.S) return -1;
  return pl.t.ck[seq + 1] - pl.t.ck[seq];
}

int64_t speckv_total_keep(const speckv_params *p) {
  Plan pl;
  if (build_plan(p, &pl, false, 0) != SPECKV_OK) return -1;
  return pl.d.KT;
}

speckv_status speckv_plan_info(const speckv_params *p, int64_t info[SPECKV_PLAN_INFO_WORDS]) {
  Plan pl;
  speckv_status st = build_plan(p, &pl, false, 0);
  if (st != SPECKV_OK) return st;
  if (info == nullptr) return SPECKV_ERR_INVALID_ARG;
  const int rowb = pl.d.D * pl.d.elt;
  info[0] = pl.g.NW; info[1] = pl.g.MB; info[2] = pl.g.RS; info[3] = pl.g.KC; info[4] = pl.g.n_fast_chunks;
  info[5] = rowb <= 128 ? 256 : rowb <= 256 ? 128 : 64;
  info[6] = pl.sel_parts; info[7] = pl.sel_part_len;
  info[8] = (score_uses_qs(pl, 1) ? 1 : 0) | (score_uses_qs(pl, 2) ? 2 : 0);
  info[9] = pl.d.reduce_max;
  info[10] = (!score_uses_qs(pl, 1) && pl.g.n_fast_chunks > 0 && score_rows_fixed_reference(pl.d, pl.g)) ? 1 : 0;
  return SPECKV_OK;
}

size_t speckv_workspace_bytes(const speckv_params *p) {
  Plan pl;
  if (build_plan(p, &pl, false, 0) != SPECKV_OK) return 0;
  return pl.total;
}

size_t speckv_select_workspace_bytes(const speckv_params *p) {
  Plan pl;
  if (build_plan(p, &pl, false, 0) != SPECKV_OK || pl.sel_parts <= 1) return 0;
  return (size_t)align_up((int64_t)(pl.off_sel_state - pl.off_sel_hist), 256) + (pl.total - pl.off_sel_state);
}

size_t specpc_workspace_bytes(const speckv_params *p, int32_t top_k) {
  Plan pl;
  if (p == nullptr || top_k < 0) return 0;
  speckv_params eff = *p;                 // as in specpc_select_tokens: always sum / max pooling
  eff.reduce_op = SPECKV_REDUCE_SUM;
  eff.pool_op = SPECKV_POOL_MAX;
  if (build_plan(&eff, &pl, true, top_k) != SPECKV_OK) return 0;
  return pl.total;
}

static speckv_status score_impl(const speckv_params *p, const void *q, const void *k, const float *lse_in,
                                bool want_lse, float *pooled, float *raw, void *workspace,
                                size_t workspace_bytes, void *stream) {
  Plan pl;
  speckv_status st = build_plan(p, &pl, false, 0);
  if (st != SPECKV_OK) return st;
  if (q == nullptr || k == nullptr || pooled == nullptr || (want_lse && lse_in == nullptr)) return SPECKV_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || (reinterpret_cast<uintptr_t>(pooled) & 3u) ||
      (reinterpret_cast<uintptr_t>(raw) & 3u) || (reinterpret_cast<uintptr_t>(lse_in) & 3u)) return SPECKV_ERR_INVALID_ARG;
  if ((st = check_ws(pl, workspace, workspace_bytes)) != SPECKV_OK) return st;
  char *ws = static_cast<char *>(workspace);
  hipStream_t hs = static_cast<hipStream_t>(stream);
  float *planes = reinterpret_cast<float *>(ws + pl.off_planes);
  hipError_t e = launch_score(pl, q, k, reinterpret_cast<float2 *>(ws + pl.off_part),
                              reinterpret_cast<float *>(ws + pl.off_lse), planes, hs, nullptr, lse_in);
  if (e != hipSuccess) return SPECKV_ERR_RUNTIME;
  return from_hip(launch_reduce_pool(pl, planes, raw, pooled, hs));
}

speckv_status speckv_score(const speckv_params *p, const void *q, const void *k, float *pooled,
                           float *raw, void *workspace, size_t workspace_bytes, void *stream) {
  return score_impl(p, q, k, nullptr, false, pooled, raw, workspace, workspace_bytes, stream);
}

speckv_status speckv_score_lse(const speckv_params *p, const void *q, const void *k, const float *lse_in,
                               float *pooled, float *raw, void *workspace, size_t workspace_bytes,
                               void *stream) {
  return score_impl(p, q, k, lse_in, true, pooled, raw, workspace, workspace_bytes, stream);
}

speckv_status speckv_select(const speckv_params *p, const float *pooled, int32_t *idx,
                            void *workspace, size_t workspace_bytes, void *stream) {
  Plan pl;
  speckv_status st = build_plan(p, &pl, false, 0);
  if (st != SPECKV_OK) return st;
  if (pooled == nullptr || idx == nullptr) return SPECKV_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(pooled) & 3u) || (reinterpret_cast<uintptr_t>(idx) & 3u)) return SPECKV_ERR_INVALID_ARG;
  // The workspace is optional here: without it every row is ranked by one workgroup (scratch in
  // LDS); with one of speckv_select_workspace_bytes, calls with few and very long rows spread each
  // row over several workgroups.  Layout: the parts' histograms, then the search state.
  uint32_t *hist = nullptr, *state = nullptr;
  if (workspace != nullptr && pl.sel_parts > 1) {
    const size_t hist_bytes = (size_t)align_up((int64_t)(pl.off_sel_state - pl.off_sel_hist), 256);
    const size_t need = hist_bytes + (pl.total - pl.off_sel_state);
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || workspace_bytes < need) return SPECKV_ERR_WORKSPACE;
    hist = reinterpret_cast<uint32_t *>(static_cast<char *>(workspace));
    state = reinterpret_cast<uint32_t *>(static_cast<char *>(workspace) + hist_bytes);
  }
  return from_hip(launch_select(pl, pooled, idx, hist, state, static_cast<hipStream_t>(stream)));
}

speckv_status speckv_compact(const speckv_params *p, const void *k, const void *v, const int32_t *idx,
                             void *k_out, void *v_out, void *stream) {
  Plan pl;
  speckv_status st = build_plan(p, &pl, false, 0);
  if (st != SPECKV_OK) return st;
  if (k == nullptr || idx == nullptr || k_out == nullptr) return SPECKV_ERR_INVALID_ARG;
  if ((v == nullptr) != (v_out == nullptr)) return SPECKV_ERR_INVALID_ARG;
  if (!aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out) ||
      (reinterpret_cast<uintptr_t>(idx) & 3u)) return SPECKV_ERR_INVALID_ARG;
  return from_hip(launch_compact(pl, k, v, idx, k_out, v_out, static_cast<hipStream_t>(stream)));
}

static speckv_status compress_impl(const speckv_params *p, const void *q, const void *k, const void *v,
                                   int32_t *idx, void *k_out, void *v_out, void *workspace,
                                   size_t workspace_bytes, void *stream, hipEvent_t *ev,
                                   const float *lse_in = nullptr) {
  Plan pl;
  speckv_status st = build_plan(p, &pl, false, 0);
  if (st != SPECKV_OK) return st;
  if (q == nullptr || k == nullptr || idx == nullptr || k_out == nullptr) return SPECKV_ERR_INVALID_ARG;
  if ((v == nullptr) != (v_out == nullptr)) return SPECKV_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out) ||
      (reinterpret_cast<uintptr_t>(idx) & 3u)) return SPECKV_ERR_INVALID_ARG;
  if ((st = check_ws(pl, workspace, workspace_bytes)) != SPECKV_OK) return st;
  char *ws = static_cast<char *>(workspace);
  hipStream_t hs = static_cast<hipStream_t>(stream);
  float *planes = reinterpret_cast<float *>(ws + pl.off_planes);
  float *pooled = reinterpret_cast<float *>(ws + pl.off_pooled);
  // the pooling kernel also counts the first selection digit of every row (counters zeroed by the
  // kernel between the sweeps), so that selection starts at its second read of the pooled scores
  uint32_t *hist0 = pl.hist0_words > 0 ? reinterpret_cast<uint32_t *>(ws + pl.off_hist0) : nullptr;
  hipError_t e = launch_score(pl, q, k, reinterpret_cast<float2 *>(ws + pl.off_part),
                              reinterpret_cast<float *>(ws + pl.off_lse), planes, hs, ev, lse_in, hist0, pl.hist0_words);
  if (e != hipSuccess) return SPECKV_ERR_RUNTIME;
  if ((e = launch_reduce_pool(pl, planes, nullptr, pooled, hs, hist0)) != hipSuccess) return SPECKV_ERR_RUNTIME;
  if (ev && hipEventRecord(ev[4], hs) != hipSuccess) return SPECKV_ERR_RUNTIME;
  if ((e = launch_select(pl, pooled, idx, reinterpret_cast<uint32_t *>(ws + pl.off_sel_hist),
                         reinterpret_cast<uint32_t *>(ws + pl.off_sel_state), hs, hist0)) != hipSuccess) return SPECKV_ERR_RUNTIME;
  if (ev && hipEventRecord(ev[5], hs) != hipSuccess) return SPECKV_ERR_RUNTIME;
  if ((e = launch_compact(pl, k, v, idx, k_out, v_out, hs)) != hipSuccess) return SPECKV_ERR_RUNTIME;
  if (ev && hipEventRecord(ev[6], hs) != hipSuccess) return SPECKV_ERR_RUNTIME;
  return SPECKV_OK;
}

speckv_status speckv_compress(const speckv_params *p, const void *q, const void *k, const void *v,
                              int32_t *idx, void *k_out, void *v_out, void *workspace,
                              size_t workspace_bytes, void *stream) {
  return compress_impl(p, q, k, v, idx, k_out, v_out, workspace, workspace_bytes, stream, nullptr);
}

speckv_status speckv_compress_static(const speckv_params *p, const void *q, const void *k, const void *v,
                                     int32_t *idx, void *k_out, void *v_out, void *stream) {
  Plan pl;
  speckv_status st = build_plan(p, &pl, false, 0);
  if (st != SPECKV_OK) return st;
  if (pl.total > (size_t)SPECKV_STATIC_SCRATCH_BYTES) return SPECKV_ERR_WORKSPACE;   // problem too large for the fixed scratch
  void *ws = nullptr;
  if ((st = static_scratch(&ws)) != SPECKV_OK) return st;
  return compress_impl(p, q, k, v, idx, k_out, v_out, ws, (size_t)SPECKV_STATIC_SCRATCH_BYTES, stream, nullptr);
}

speckv_status speckv_compress_lse(const speckv_params *p, const void *q, const void *k, const void *v,
                                  const float *lse_in, int32_t *idx, void *k_out, void *v_out,
                                  void *workspace, size_t workspace_bytes, void *stream) {
  if (lse_in == nullptr || (reinterpret_cast<uintptr_t>(lse_in) & 3u)) return SPECKV_ERR_INVALID_ARG;
  return compress_impl(p, q, k, v, idx, k_out, v_out, workspace, workspace_bytes, stream, nullptr, lse_in);
}

speckv_status speckv_compress_events(const speckv_params *p, const void *q, const void *k, const void *v,
                                     int32_t *idx, void *k_out, void *v_out, void *workspace,
                                     size_t workspace_bytes, void *stream, void **events, int32_t n_events) {
  if (events == nullptr || n_events != SPECKV_N_STAGE_EVENTS) return SPECKV_ERR_INVALID_ARG;
  for (int i = 0; i < n_events; ++i)
    if (events[i] == nullptr) return SPECKV_ERR_INVALID_ARG;
  return compress_impl(p, q, k, v, idx, k_out, v_out, workspace, workspace_bytes, stream,
                       reinterpret_cast<hipEvent_t *>(events));
}

size_t speckv_ada_workspace_bytes(const speckv_params *p) {
  Plan pl;
  if (build_plan(p, &pl, false, 0) != SPECKV_OK || pl.d.Hkv > SPECKV_MAX_ADA_HEADS) return 0;
  return pl.total_ada;
}

static speckv_status ada_plan(const speckv_params *p, int32_t c_floor, Plan *pl) {
  speckv_status st = build_plan(p, pl, false, 0);
  if (st != SPECKV_OK) return st;
  if (c_floor < 0) return SPECKV_ERR_INVALID_ARG;
  if (pl->d.Hkv > SPECKV_MAX_ADA_HEADS) return SPECKV_ERR_UNSUPPORTED;
  return SPECKV_OK;
}

speckv_status speckv_select_ada(const speckv_params *p, int32_t c_floor, const float *pooled, int32_t *idx,
                                int32_t *head_off, void *workspace, size_t workspace_bytes, void *stream) {
  Plan pl;
  speckv_status st = ada_plan(p, c_floor, &pl);
  if (st != SPECKV_OK) return st;
  if (pooled == nullptr || idx == nullptr || head_off == nullptr) return SPECKV_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(pooled) & 3u) || (reinterpret_cast<uintptr_t>(idx) & 3u) ||
      (reinterpret_cast<uintptr_t>(head_off) & 3u)) return SPECKV_ERR_INVALID_ARG;
  if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 ||
      workspace_bytes < pl.total_ada) return SPECKV_ERR_WORKSPACE;
  char *ws = static_cast<char *>(workspace);
  return from_hip(launch_select_ada(pl, c_floor, pooled, idx, head_off,
                                    reinterpret_cast<uint32_t *>(ws + pl.off_ada_hist),
                                    reinterpret_cast<uint32_t *>(ws + pl.off_ada_state),
                                    static_cast<hipStream_t>(stream)));
}

speckv_status speckv_compact_ada(const speckv_params *p, const void *k, const void *v, const int32_t *idx,
                                 const int32_t *head_off, void *k_out, void *v_out, void *stream) {
  Plan pl;
  speckv_status st = ada_plan(p, 0, &pl);
  if (st != SPECKV_OK) return st;
  if (k == nullptr || idx == nullptr || head_off == nullptr || k_out == nullptr) return SPECKV_ERR_INVALID_ARG;
  if ((v == nullptr) != (v_out == nullptr)) return SPECKV_ERR_INVALID_ARG;
  if (!aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out) ||
      (reinterpret_cast<uintptr_t>(idx) & 3u) || (reinterpret_cast<uintptr_t>(head_off) & 3u)) return SPECKV_ERR_INVALID_ARG;
  return from_hip(launch_compact_ada(pl, k, v, idx, head_off, k_out, v_out, static_cast<hipStream_t>(stream)));
}

speckv_status speckv_compress_ada(const speckv_params *p, int32_t c_floor, const void *q, const void *k,
                                  const void *v, int32_t *idx, int32_t *head_off, void *k_out, void *v_out,
                                  void *workspace, size_t workspace_bytes, void *stream) {
  Plan pl;
  speckv_status st = ada_plan(p, c_floor, &pl);
  if (st != SPECKV_OK) return st;
  if (q == nullptr || k == nullptr || idx == nullptr || head_off == nullptr || k_out == nullptr) return SPECKV_ERR_INVALID_ARG;
  if ((v == nullptr) != (v_out == nullptr)) return SPECKV_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out) ||
      (reinterpret_cast<uintptr_t>(idx) & 3u) || (reinterpret_cast<uintptr_t>(head_off) & 3u)) return SPECKV_ERR_INVALID_ARG;
  if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 ||
      workspace_bytes < pl.total_ada) return SPECKV_ERR_WORKSPACE;
  char *ws = static_cast<char *>(workspace);
  hipStream_t hs = static_cast<hipStream_t>(stream);
  float *planes = reinterpret_cast<float *>(ws + pl.off_planes);
  float *pooled = reinterpret_cast<float *>(ws + pl.off_pooled);
  hipError_t e = launch_score(pl, q, k, reinterpret_cast<float2 *>(ws + pl.off_part),
                              reinterpret_cast<float *>(ws + pl.off_lse), planes, hs);
  if (e != hipSuccess) return SPECKV_ERR_RUNTIME;
  if ((e = launch_reduce_pool(pl, planes, nullptr, pooled, hs)) != hipSuccess) return SPECKV_ERR_RUNTIME;
  if ((e = launch_select_ada(pl, c_floor, pooled, idx, head_off, reinterpret_cast<uint32_t *>(ws + pl.off_ada_hist),
                             reinterpret_cast<uint32_t *>(ws + pl.off_ada_state), hs)) != hipSuccess) return SPECKV_ERR_RUNTIME;
  return from_hip(launch_compact_ada(pl, k, v, idx, head_off, k_out, v_out, hs));
}

static speckv_status select_tokens_impl(const speckv_params *p, int32_t top_k, int32_t n_neighbor,
                                        const void *q, const void *k, const int32_t *token_ids,
                                        int32_t *idx_out, int32_t *ids_out, int32_t *count_out,
                                        void *workspace, size_t workspace_bytes, void *stream, hipEvent_t *ev) {
  if (p == nullptr || top_k < 0 || n_neighbor < 0) return SPECKV_ERR_INVALID_ARG;
  // the reduced form is defined with sum aggregation and max pooling whatever the caller's ops say
  speckv_params eff = *p;
  eff.reduce_op = SPECKV_REDUCE_SUM;
  eff.pool_op = SPECKV_POOL_MAX;
  Plan pl;
  speckv_status st = build_plan(&eff, &pl, true, top_k);
  if (st != SPECKV_OK) return st;
  if (q == nullptr || k == nullptr || token_ids == nullptr || idx_out == nullptr || ids_out == nullptr ||
      count_out == nullptr) return SPECKV_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k)) return SPECKV_ERR_INVALID_ARG;
  if ((st = check_ws(pl, workspace, workspace_bytes)) != SPECKV_OK) return st;
  char *ws = static_cast<char *>(workspace);
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const int n_in = (int)pl.d.T, m = n_in - pl.d.w;
  const int count = top_k < m ? top_k : m;
  float *planes = reinterpret_cast<float *>(ws + pl.off_planes);
  float *pooled = reinterpret_cast<float *>(ws + pl.off_pooled);
  int32_t *sel = reinterpret_cast<int32_t *>(ws + pl.off_sel);
  hipError_t e = launch_score(pl, q, k, reinterpret_cast<float2 *>(ws + pl.off_part),
                              reinterpret_cast<float *>(ws + pl.off_lse), planes, hs, ev);
  if (e != hipSuccess) return SPECKV_ERR_RUNTIME;
  if ((e = launch_reduce_pool_all(pl, planes, nullptr, pooled, hs)) != hipSuccess) return SPECKV_ERR_RUNTIME;
  if (ev && hipEventRecord(ev[4], hs) != hipSuccess) return SPECKV_ERR_RUNTIME;
  if ((e = launch_select_row(pooled, m, count, sel, hs)) != hipSuccess) return SPECKV_ERR_RUNTIME;
  if (ev && hipEventRecord(ev[5], hs) != hipSuccess) return SPECKV_ERR_RUNTIME;
  if ((e = launch_expand(sel, count, n_in, pl.d.w, n_neighbor, token_ids, idx_out, ids_out, count_out, hs)) != hipSuccess)
    return SPECKV_ERR_RUNTIME;
  if (ev && hipEventRecord(ev[6], hs) != hipSuccess) return SPECKV_ERR_RUNTIME;
  return SPECKV_OK;
}

speckv_status specpc_select_tokens(const speckv_params *p, int32_t top_k, int32_t n_neighbor,
                                   const void *q, const void *k, const int32_t *token_ids,
                                   int32_t *idx_out, int32_t *ids_out, int32_t *count_out,
                                   void *workspace, size_t workspace_bytes, void *stream) {
  return select_tokens_impl(p, top_k, n_neighbor, q, k, token_ids, idx_out, ids_out, count_out, workspace,
                            workspace_bytes, stream, nullptr);
}

speckv_status specpc_select_tokens_events(const speckv_params *p, int32_t top_k, int32_t n_neighbor,
                                          const void *q, const void *k, const int32_t *token_ids,
                                          int32_t *idx_out, int32_t *ids_out, int32_t *count_out,
                                          void *workspace, size_t workspace_bytes, void *stream,
                                          void **events, int32_t n_events) {
  if (events == nullptr || n_events != SPECKV_N_STAGE_EVENTS) return SPECKV_ERR_INVALID_ARG;
  for (int i = 0; i < n_events; ++i)
    if (events[i] == nullptr) return SPECKV_ERR_INVALID_ARG;
  return select_tokens_impl(p, top_k, n_neighbor, q, k, token_ids, idx_out, ids_out, count_out, workspace,
                            workspace_bytes, stream, reinterpret_cast<hipEvent_t *>(events));
}

// Parameters of the layers that take part: the first l_skip layers are dropped by moving the base
// pointers, and the reduction becomes a max over rows, heads and layers with weighted window rows.
static speckv_status alg2_plan(const speckv_params *p, int32_t l_skip, Plan *pl, speckv_params *eff) {
  if (p == nullptr || l_skip < 0) return SPECKV_ERR_INVALID_ARG;
  if (l_skip >= p->n_layers) return SPECKV_ERR_INVALID_ARG;
  *eff = *p;
  eff->n_layers = p->n_layers - l_skip;
  eff->reduce_op = SPECKV_REDUCE_MAX;
  eff->pool_op = SPECKV_POOL_AVG;
  const int32_t m_cap = p->c_max < 0 ? 0 : p->c_max;
  speckv_status st = build_plan(eff, pl, true, m_cap);
  if (st != SPECKV_OK) return st;
  pl->d.head_max = 1;
  pl->d.weight_rows = 1;
  return SPECKV_OK;
}

size_t specpc_compress_workspace_bytes(const speckv_params *p, int32_t l_skip) {
  Plan pl;
  speckv_params eff;
  if (alg2_plan(p, l_skip, &pl, &eff) != SPECKV_OK) return 0;
  return pl.total;
}

speckv_status specpc_compress_prompt(const speckv_params *p, int32_t l_skip, int32_t n_neighbor,
                                     const void *q, const void *k, const int32_t *token_ids,
                                     int32_t *idx_out, int32_t *ids_out, int32_t *count_out,
                                     void *workspace, size_t workspace_bytes, void *stream) {
  Plan pl;
  speckv_params eff;
  speckv_status st = alg2_plan(p, l_skip, &pl, &eff);
  if (st != SPECKV_OK) return st;
  if (n_neighbor < 1) return SPECKV_ERR_INVALID_ARG;
  if (n_neighbor > SPECKV_MAX_POOL_K) return SPECKV_ERR_UNSUPPORTED;
  if (q == nullptr || k == nullptr || token_ids == nullptr || idx_out == nullptr || ids_out == nullptr ||
      count_out == nullptr) return SPECKV_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k)) return SPECKV_ERR_INVALID_ARG;
  if ((st = check_ws(pl, workspace, workspace_bytes)) != SPECKV_OK) return st;
  char *ws = static_cast<char *>(workspace);
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const Dims &d = pl.d;
  const char *q0 = static_cast<const char *>(q) + (int64_t)l_skip * d.q_sl * d.elt;
  const char *k0 = static_cast<const char *>(k) + (int64_t)l_skip * d.kv_sl * d.elt;
  const int n_in = (int)d.T, m = n_in - d.w;
  const int count = d.c_max < m ? d.c_max : m;
  float *planes = reinterpret_cast<float *>(ws + pl.off_planes);
  float *smooth = reinterpret_cast<float *>(ws + pl.off_pooled);
  float *spread = reinterpret_cast<float *>(ws + pl.off_pooled2);
  int32_t *sel = reinterpret_cast<int32_t *>(ws + pl.off_sel);
  hipError_t e = launch_score(pl, q0, k0, reinterpret_cast<float2 *>(ws + pl.off_part),
                              reinterpret_cast<float *>(ws + pl.off_lse), planes, hs);
  if (e != hipSuccess) return SPECKV_ERR_RUNTIME;
  if ((e = launch_reduce_pool_all(pl, planes, nullptr, smooth, hs)) != hipSuccess) return SPECKV_ERR_RUNTIME;
  if ((e = launch_pool_row(smooth, spread, n_in, d.w, n_neighbor, hs)) != hipSuccess) return SPECKV_ERR_RUNTIME;
  if ((e = launch_select_row(spread, m, count, sel, hs)) != hipSuccess) return SPECKV_ERR_RUNTIME;
  return from_hip(launch_expand(sel, count, n_in, d.w, 0, token_ids, idx_out, ids_out, count_out, hs));
}

}  // extern "C"
