// Pooling, top-C selection and index expansion.
//
//  * reduce_pool: sums the partial score planes the scoring kernels wrote, emits the raw
//    importance (Eq. 1, summed over queries and the GQA group) and its 1-D max-pool with
//    kernel k over the non-window candidates (Alg. 1 pooling step; table: Max, k = 7).
//  * select: the C largest pooled scores per (layer, sequence, KV head), ties to the
//    smaller index, ascending, then the window m..n_in-1 (Alg. 1 "Select KVs").
//    MSD radix select on order-preserving 32-bit keys (11 + 11 + 10 bits, LDS
//    histograms), then an ordered compaction that ranks candidates with wavefront
//    prefix sums.  One workgroup per row; every step is deterministic.  A workgroup is
//    bound by its vector ALU, so the per-element work is kept minimal: 128-bit loads,
//    digits taken from the raw float bits, float compares against the threshold.
//  * shared layer budget: per-head counts from one layer-wide threshold (histogram and
//    decision kernels per digit), then the same row select with each head's own count.
//  * expand: widens selected tokens to +-n_neighbor, unites them with the window and
//    emits the sorted set with the token ids gathered (Sec. 4.2 prompt compression).
#include "speckv_internal.h"

namespace speckv {
namespace {

// ----------------------------------------------------------------------------------
// reduce + pool
// ----------------------------------------------------------------------------------
constexpr int kPoolThreads = 256;
constexpr int kPoolTile = 1024;

// How the partial planes of one output row are merged: value = outer over groups of
// (inner over the n_inner consecutive planes of a group); each op is a sum or a max.
struct PlaneMerge {
  int n_outer, n_inner;
  int inner_max, outer_max;
  int64_t plane_stride;
};

// Merges the planes per key, writes raw (optional) and pooled for one row tile.
__device__ inline void reduce_pool_tile(const float *__restrict__ in, PlaneMerge pm,
                                        float *__restrict__ raw, float *__restrict__ pooled,
                                        int n_s, int n_row, int m, int pool_k, int pool_avg, int j0,
                                        float *tile) {
  // window of key j: j - half .. j + after (symmetric for odd kernels; an even kernel looks one
  // position further back than ahead, the library convention with padding k / 2)
  const int half = pool_k / 2, after = (pool_k - 1) / 2;
  const int span = kPoolTile + 2 * half;
  for (int x = threadIdx.x; x < span; x += kPoolThreads) {
    const int jj = j0 - half + x;
    float acc = 0.f;
    if (jj >= 0 && jj < n_s) {
      const float *p = in + jj;
      for (int o = 0; o < pm.n_outer; ++o) {
        float v = 0.f;                                   // scores are non-negative: 0 is neutral for max
        for (int q = 0; q < pm.n_inner; ++q) {
          const float y = p[(int64_t)(o * pm.n_inner + q) * pm.plane_stride];
          v = pm.inner_max ? fmaxf(v, y) : v + y;
        }
        acc = pm.outer_max ? fmaxf(acc, v) : acc + v;
      }
    }
    tile[x] = acc;
  }
  __syncthreads();
  for (int x = threadIdx.x; x < kPoolTile; x += kPoolThreads) {
    const int j = j0 + x;
    if (j >= n_row) break;                                  // entries past the live length read as zero
    const float center = tile[x + half];
    if (raw != nullptr) raw[j] = center;
    float best = 0.f;
    if (j < m) {
      const int lo = max(0, j - half), hi = min(m - 1, j + after);
      best = tile[lo - j0 + half];
      if (pool_avg) {
        for (int jj = lo + 1; jj <= hi; ++jj) best += tile[jj - j0 + half];
        best /= (float)pool_k;                            // zeros outside [0, m) count in the divisor
      } else {
        for (int jj = lo + 1; jj <= hi; ++jj) best = fmaxf(best, tile[jj - j0 + half]);
      }
    }
    pooled[j] = best;
  }
}

__global__ __launch_bounds__(kPoolThreads) void reduce_pool_kernel(
    Dims d, SeqTab t, PlaneMerge pm, const float *__restrict__ planes,
    float *__restrict__ raw, float *__restrict__ pooled, int tiles_per_row) {
  __shared__ float tile[kPoolTile + SPECKV_MAX_POOL_K + 1];
  const int unit = blockIdx.x / tiles_per_row;
  const int j0 = (blockIdx.x - unit * tiles_per_row) * kPoolTile;
  const int g = unit % d.Hkv;
  const int s = (unit / d.Hkv) % d.S;
  const int layer = unit / (d.Hkv * d.S);
  const int n_row = t.cu[s + 1] - t.cu[s];
  if (j0 >= n_row) return;
  const int n_s = live_len(d, t, s);
  const int64_t base = (int64_t)layer * d.Hkv * d.T + (int64_t)d.Hkv * t.cu[s] + (int64_t)g * n_row;
  reduce_pool_tile(planes + base, pm, raw ? raw + base : nullptr, pooled + base, n_s, n_row, n_s - d.w,
                   d.pool_k, d.pool_avg, j0, tile);
}

// One output row that merges every plane (all layers, heads, row super-blocks) of a
// single-sequence call: planes are consecutive rows of n_in floats, all merged by one op (sum or
// max).  There can be hundreds of planes, so a workgroup takes a short tile of keys and its four
// wavefronts each merge a quarter of the planes; the quarters are combined in a fixed order.
constexpr int kAllTile = 64, kAllSlices = 4;

__global__ __launch_bounds__(kAllTile * kAllSlices) void reduce_pool_all_kernel(
    int n_in, int n_window, int pool_k, int pool_avg, PlaneMerge pm, const float *__restrict__ planes,
    float *__restrict__ raw, float *__restrict__ pooled) {
  __shared__ float part[kAllSlices][kAllTile + SPECKV_MAX_POOL_K + 1];
  const int j0 = blockIdx.x * kAllTile;
  if (j0 >= n_in) return;
  const int half = pool_k / 2, after = (pool_k - 1) / 2, span = kAllTile + 2 * half;   // see reduce_pool_tile
  const int slice = threadIdx.x / kAllTile, lane = threadIdx.x % kAllTile;
  const int n_planes = pm.n_outer * pm.n_inner;
  const int per_slice = (n_planes + kAllSlices - 1) / kAllSlices;
  const int o0 = slice * per_slice, o1 = min(n_planes, o0 + per_slice);
  for (int x = lane; x < span; x += kAllTile) {
    const int jj = j0 - half + x;
    float acc = 0.f;                                       // scores are non-negative: 0 is neutral for max
    if (jj >= 0 && jj < n_in) {
      const float *p = planes + jj;
#pragma unroll 8
      for (int o = o0; o < o1; ++o) {
        const float y = p[(int64_t)o * pm.plane_stride];
        acc = pm.outer_max ? fmaxf(acc, y) : acc + y;
      }
    }
    part[slice][x] = acc;
  }
  __syncthreads();
  float *tile = part[0];
  for (int x = threadIdx.x; x < span; x += kAllTile * kAllSlices) {
    float v = part[0][x];
#pragma unroll
    for (int s2 = 1; s2 < kAllSlices; ++s2) v = pm.outer_max ? fmaxf(v, part[s2][x]) : v + part[s2][x];
    tile[x] = v;
  }
  __syncthreads();
  const int m = n_in - n_window;
  for (int x = threadIdx.x; x < kAllTile; x += kAllTile * kAllSlices) {
    const int j = j0 + x;
    if (j >= n_in) break;
    if (raw != nullptr) raw[j] = tile[x + half];
    float best = 0.f;
    if (j < m) {
      const int lo = max(0, j - half), hi = min(m - 1, j + after);
      best = tile[lo - j0 + half];
      if (pool_avg) {
        for (int jj = lo + 1; jj <= hi; ++jj) best += tile[jj - j0 + half];
        best /= (float)pool_k;                            // zeros outside [0, m) count in the divisor
      } else {
        for (int jj = lo + 1; jj <= hi; ++jj) best = fmaxf(best, tile[jj - j0 + half]);
      }
    }
    pooled[j] = best;
  }
}

// ----------------------------------------------------------------------------------
// radix select
// ----------------------------------------------------------------------------------
constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelVec = 4;         // 128-bit vectors a thread ranks per tile of the emission pass
constexpr int kHistCopies = 8;
constexpr int kHistUnroll = 4;     // independent 128-bit loads in flight per thread in the histogram passes

// Ordered key of a float (larger float, larger key): with u its bits and -0 taken as +0,
// key = u | 0x80000000 for a positive number and ~u for a negative one.  `prefix` values below
// are leading bits of such keys.
// The histogram passes work on the raw float bits (fewer operations per element than the ordered
// key); only the bin index is translated when the bins are read in descending order.
// Ordered digit D of level `pass` (0, 1, 2) -> digit of the raw bits; `neg`: the number is negative.
__device__ __forceinline__ int raw_digit(int D, int pass, int nb, bool neg) {
  if (pass == 0) return D >= 1024 ? D - 1024 : 2047 - D;
  return neg ? nb - 1 - D : D;
}
// Raw float bits (under `mask`) of the numbers whose ordered key starts with `prefix`.
__device__ __forceinline__ uint32_t raw_prefix_of(uint32_t prefix, uint32_t mask) {
  return (prefix & 0x80000000u) ? (prefix ^ 0x80000000u) : (~prefix & mask);
}
// Raw bits of x with -0 turned into +0 (the two compare equal and must share a bin).
__device__ __forceinline__ uint32_t raw_bits(float x) { return __float_as_uint(x + 0.0f); }

struct SelShared {
  uint32_t hist[kHistCopies * 2048];   // one copy per lane residue: spreads atomics that hit one bin
  uint32_t wave_tot[2][kSelWaves];
  uint32_t prefix, remaining;
};

// Exclusive prefix sum of v over the workgroup in thread order; *total gets the sum.
// Uses wavefront shuffles for the in-wave scan and LDS for the 16 wave totals.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *wave_tot, uint32_t *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t inc = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t up = __shfl_up(inc, off, 64);
    if (lane >= off) inc += up;
  }
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int w2 = 0; w2 < kSelWaves; ++w2) {
    const uint32_t x = wave_tot[w2];
    if (w2 < wave) before += x;
    all += x;
  }
  *total = all;
  return before + inc - v;
}

// A row split for 128-bit access: `lead` scalars up to the first 16-byte boundary, nv float4
// vectors, then the scalars from tail0 to the end.
struct RowSplit { int lead, nv, tail0; };
__device__ __forceinline__ RowSplit split_row(const float *x, int m) {
  RowSplit rs;
  rs.lead = min((int)((4u - ((uint32_t)(reinterpret_cast<uintptr_t>(x) >> 2) & 3u)) & 3u), m);
  rs.nv = (m - rs.lead) >> 2;
  rs.tail0 = rs.lead + 4 * rs.nv;
  return rs;
}

// Histogram of one radix digit of the entries of x[0..m) whose ordered key starts with `prefix`
// (bits under `mask`), into the kHistCopies copies of sh.hist (cleared first), indexed by the digit
// of the RAW bits (see raw_digit).  The loads are unconditional (index clamped) so that kHistUnroll
// vectors per thread are in flight.
__device__ __forceinline__ void histogram_pass(const float *__restrict__ x, int m, RowSplit rs,
                                               uint32_t prefix, uint32_t mask, int shift, int nb,
                                               SelShared &sh) {
  const int tid = threadIdx.x;
  for (int b = tid; b < kHistCopies * 2048; b += kSelThreads) sh.hist[b] = 0;
  __syncthreads();
  uint32_t *h = sh.hist + (tid % kHistCopies) * 2048;
  const uint32_t rawp = raw_prefix_of(prefix, mask);
  const float4 *xv = reinterpret_cast<const float4 *>(x + rs.lead);
  for (int v0 = 0; v0 < rs.nv; v0 += kSelThreads * kHistUnroll) {
    float4 val[kHistUnroll];
#pragma unroll
    for (int u = 0; u < kHistUnroll; ++u) val[u] = xv[min(v0 + u * kSelThreads + tid, rs.nv - 1)];
#pragma unroll
    for (int u = 0; u < kHistUnroll; ++u) {
      const bool ok = v0 + u * kSelThreads + tid < rs.nv;
      const float e4[4] = {val[u].x, val[u].y, val[u].z, val[u].w};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint32_t u = raw_bits(e4[c]);
        if (ok && ((u ^ rawp) & mask) == 0) atomicAdd(&h[(u >> shift) & (nb - 1)], 1u);
      }
    }
  }
  if (tid < rs.lead + (m - rs.tail0)) {
    const uint32_t u = raw_bits(x[tid < rs.lead ? tid : rs.tail0 + (tid - rs.lead)]);
    if (((u ^ rawp) & mask) == 0) atomicAdd(&h[(u >> shift) & (nb - 1)], 1u);
  }
  __syncthreads();
}

// Ordered key of the count-th largest entry of x[0..m) (1 <= count <= m) and how many of the
// entries equal to it belong to the `count` largest.
__device__ __forceinline__ void radix_threshold(const float *__restrict__ x, int m, RowSplit rs, int count,
                                                SelShared &sh, uint32_t *thr_key, uint32_t *need_eq_out) {
  const int tid = threadIdx.x;
  uint32_t prefix = 0, mask = 0, remaining = (uint32_t)count;
#pragma unroll
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = pass == 0 ? 21 : pass == 1 ? 10 : 0;       // digits of 11, 11 and 10 bits
    const int nb = pass == 2 ? 1024 : 2048;
    histogram_pass(x, m, rs, prefix, mask, shift, nb, sh);
    // thread t owns the bins nb-1-2t and nb-2-2t: scanning threads in order walks the
    // bins from the largest digit down.
    const int b0 = nb - 1 - 2 * tid, b1 = nb - 2 - 2 * tid;
    const bool neg = (prefix & 0x80000000u) == 0;
    const int r0 = raw_digit(b0, pass, nb, neg), r1 = raw_digit(b1, pass, nb, neg);
    uint32_t c0 = 0, c1 = 0;
#pragma unroll
    for (int cp = 0; cp < kHistCopies; ++cp) {
      if (b0 >= 0) c0 += sh.hist[cp * 2048 + r0];
      if (b1 >= 0) c1 += sh.hist[cp * 2048 + r1];
    }
    uint32_t total;
    const uint32_t above = block_exclusive_scan(c0 + c1, sh.wave_tot[0], &total);
    if (above < remaining && remaining <= above + c0) {
      sh.prefix = prefix | ((uint32_t)b0 << shift);
      sh.remaining = remaining - above;
    } else if (above + c0 < remaining && remaining <= above + c0 + c1) {
      sh.prefix = prefix | ((uint32_t)b1 << shift);
      sh.remaining = remaining - above - c0;
    }
    __syncthreads();
    prefix = sh.prefix;
    remaining = sh.remaining;
    mask |= (uint32_t)(nb - 1) << shift;
    __syncthreads();
  }
  *thr_key = prefix;
  *need_eq_out = remaining;
}

// Writes, ascending, the indices of the entries of x[0..m) above the threshold key and of the
// first need_eq entries equal to it (compared as floats: the same order as the keys, with -0
// equal to +0).
// x may be a slice of a longer row: index_base is the row index of x[0] and run_gt / run_eq
// start at the numbers of entries above / equal to the threshold that precede the slice.
__device__ __forceinline__ void emit_selected(const float *__restrict__ x, int m, RowSplit rs,
                                              uint32_t thr_key, uint32_t need_eq,
                                              int32_t *__restrict__ out, SelShared &sh,
                                              uint32_t run_gt = 0, uint32_t run_eq = 0, int index_base = 0) {
  const int tid = threadIdx.x;
  const float thr = __uint_as_float(raw_prefix_of(thr_key, 0xffffffffu));
  // the scalars before the first vector: every thread tracks the counts, thread 0 writes
  for (int j = 0; j < rs.lead; ++j) {
    const float xj = x[j];
    const bool is_gt = xj > thr, is_eq = xj == thr;
    if (tid == 0 && (is_gt || (is_eq && run_eq < need_eq))) out[run_gt + min(run_eq, need_eq)] = index_base + j;
    run_gt += is_gt;
    run_eq += is_eq;
  }
  if (rs.nv > 0) {
    // a thread ranks kSelVec adjacent vectors per tile; the values of the next tile are
    // requested before the current tile is ranked
    const float4 *xv = reinterpret_cast<const float4 *>(x + rs.lead);
    constexpr int kTileVec = kSelThreads * kSelVec;
    float4 val[kSelVec], nxt[kSelVec];
#pragma unroll
    for (int e = 0; e < kSelVec; ++e) val[e] = xv[min(tid * kSelVec + e, rs.nv - 1)];
    int buf = 0;
    for (int v0 = 0; v0 < rs.nv; v0 += kTileVec, buf ^= 1) {
      const int vb = v0 + tid * kSelVec;
#pragma unroll
      for (int e = 0; e < kSelVec; ++e) nxt[e] = xv[min(vb + kTileVec + e, rs.nv - 1)];
      uint32_t gt_bits = 0, eq_bits = 0;
#pragma unroll
      for (int e = 0; e < kSelVec; ++e) {
        const float e4[4] = {val[e].x, val[e].y, val[e].z, val[e].w};
        uint32_t g4 = 0, q4 = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          g4 |= e4[c] > thr ? 1u << c : 0u;
          q4 |= e4[c] == thr ? 1u << c : 0u;
        }
        if (vb + e < rs.nv) { gt_bits |= g4 << (4 * e); eq_bits |= q4 << (4 * e); }
      }
      const uint32_t cg = __popc(gt_bits), ce = __popc(eq_bits);
      // one scan for both counts: gt in the low 16 bits, eq in the high 16 bits
      // (a tile holds at most 16384 entries, so neither field can overflow)
      uint32_t total;
      const uint32_t before = block_exclusive_scan(cg | (ce << 16), sh.wave_tot[buf], &total);
      uint32_t gt_before = run_gt + (before & 0xffffu), eq_before = run_eq + (before >> 16);
      if ((gt_bits | eq_bits) != 0) {
#pragma unroll
        for (int b = 0; b < 4 * kSelVec; ++b) {
          const bool is_gt = (gt_bits >> b) & 1u, is_eq = (eq_bits >> b) & 1u;
          if (is_gt || (is_eq && eq_before < need_eq))
            out[gt_before + min(eq_before, need_eq)] = index_base + rs.lead + 4 * vb + b;
          gt_before += is_gt;
          eq_before += is_eq;
        }
      }
      run_gt += total & 0xffffu;
      run_eq += total >> 16;
#pragma unroll
      for (int e = 0; e < kSelVec; ++e) val[e] = nxt[e];
    }
  }
  for (int j = rs.tail0; j < m; ++j) {
    const float xj = x[j];
    const bool is_gt = xj > thr, is_eq = xj == thr;
    if (tid == 0 && (is_gt || (is_eq && run_eq < need_eq))) out[run_gt + min(run_eq, need_eq)] = index_base + j;
    run_gt += is_gt;
    run_eq += is_eq;
  }
}

// Writes the `count` (1 <= count <= m) indices of the largest x[0..m) to out, ascending,
// equal values taken from the low-index end.
__device__ __forceinline__ void select_top_row(const float *__restrict__ x, int m, int count,
                                               int32_t *__restrict__ out, SelShared &sh) {
  const RowSplit rs = split_row(x, m);
  uint32_t thr_key, need_eq;
  radix_threshold(x, m, rs, count, sh, &thr_key, &need_eq);
  emit_selected(x, m, rs, thr_key, need_eq, out, sh);
}

__global__ __launch_bounds__(kSelThreads) void select_kernel(Dims d, SeqTab t,
                                                             const float *__restrict__ pooled,
                                                             int32_t *__restrict__ idx) {
  __shared__ SelShared sh;
  const int unit = blockIdx.x;
  const int g = unit % d.Hkv;
  const int s = (unit / d.Hkv) % d.S;
  const int layer = unit / (d.Hkv * d.S);
  const int n_row = t.cu[s + 1] - t.cu[s];
  const int m = live_len(d, t, s) - d.w;
  const int n_keep = t.ck[s + 1] - t.ck[s];
  const int count = min(n_keep - d.w, m);                 // a live prompt shorter than the host's bound keeps fewer
  const float *row = pooled + (int64_t)layer * d.Hkv * d.T + (int64_t)d.Hkv * t.cu[s] + (int64_t)g * n_row;
  int32_t *out = idx + (int64_t)layer * d.Hkv * d.KT + (int64_t)d.Hkv * t.ck[s] + (int64_t)g * n_keep;
  for (int x = threadIdx.x; x < d.w; x += kSelThreads) out[count + x] = m + x;   // window, last
  for (int x = count + d.w + threadIdx.x; x < n_keep; x += kSelThreads) out[x] = -1;   // unused slots
  if (count > 0) select_top_row(row, m, count, out, sh);
}

__global__ __launch_bounds__(kSelThreads) void select_row_kernel(const float *__restrict__ row,
                                                                 int m, int count,
                                                                 int32_t *__restrict__ sel) {
  __shared__ SelShared sh;
  if (count > 0) select_top_row(row, m, count, sel, sh);
}

// ----------------------------------------------------------------------------------
// long rows, few rows: a row split over several workgroups
// ----------------------------------------------------------------------------------
// One workgroup ranks about 128K keys in 55 us; a call with a handful of rows of a million keys
// would leave the other CUs idle for most of a millisecond.  Such rows are cut into P parts.
// Per digit, msel_hist_kernel histograms every part and msel_decide_kernel (one workgroup per
// row) adds the parts, extends the threshold prefix and keeps, per part, the number of keys above
// it; after the last digit it also knows the keys equal to the threshold per part, so that
// msel_emit_kernel can place every part's output without another counting pass.
// State per row: [0] prefix, [1] remaining, [2 .. 2+P) keys above per part, [2+P .. 2+2P) equal.
struct RowRef { const float *x; int32_t *out; int m, count, n_keep; };
__device__ __forceinline__ RowRef row_of(const Dims &d, const SeqTab &t, int row, const float *pooled,
                                         int32_t *idx) {
  const int g = row % d.Hkv;
  const int s = (row / d.Hkv) % d.S;
  const int layer = row / (d.Hkv * d.S);
  const int n_row = t.cu[s + 1] - t.cu[s];
  const int n_keep = t.ck[s + 1] - t.ck[s];
  RowRef r;
  r.x = pooled + (int64_t)layer * d.Hkv * d.T + (int64_t)d.Hkv * t.cu[s] + (int64_t)g * n_row;
  r.out = idx ? idx + (int64_t)layer * d.Hkv * d.KT + (int64_t)d.Hkv * t.ck[s] + (int64_t)g * n_keep : nullptr;
  r.m = live_len(d, t, s) - d.w;
  r.count = min(n_keep - d.w, r.m);
  r.n_keep = n_keep;
  return r;
}

__global__ __launch_bounds__(kSelThreads) void msel_hist_kernel(Dims d, SeqTab t, const float *__restrict__ pooled,
                                                                int level, int P, int part_len,
                                                                const uint32_t *__restrict__ state,
                                                                uint32_t *__restrict__ hist) {
  __shared__ SelShared sh;
  const int tid = threadIdx.x;
  const int row = blockIdx.x / P, part = blockIdx.x % P;
  const RowRef r = row_of(d, t, row, pooled, nullptr);
  const int start = part * part_len;
  const int len = max(0, min(part_len, r.m - start));
  const int shift = level == 0 ? 21 : level == 1 ? 10 : 0, nb = level == 2 ? 1024 : 2048;
  const uint32_t mask = level == 0 ? 0u : level == 1 ? 0xffe00000u : 0xfffffc00u;
  const uint32_t prefix = level == 0 ? 0u : state[(int64_t)row * (2 + 2 * P)];
  const float *x = r.x + start;
  histogram_pass(x, len, split_row(x, len), prefix, mask, shift, nb, sh);
  uint32_t *out = hist + (int64_t)blockIdx.x * 2048;
  const bool neg = (prefix & 0x80000000u) == 0;
  for (int b = tid; b < 2048; b += kSelThreads) {       // b: ordered digit
    uint32_t c = 0;
    if (b < nb) {
      const int rd = raw_digit(b, level, nb, neg);
#pragma unroll
      for (int cp = 0; cp < kHistCopies; ++cp) c += sh.hist[cp * 2048 + rd];
    }
    out[b] = c;
  }
}

__global__ __launch_bounds__(kSelThreads) void msel_decide_kernel(Dims d, SeqTab t, int level, int P,
                                                                  uint32_t *__restrict__ state,
                                                                  const uint32_t *__restrict__ hist) {
  __shared__ uint32_t wave_tot[kSelWaves];
  __shared__ uint32_t found[2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = blockIdx.x;
  const RowRef r = row_of(d, t, row, nullptr, nullptr);
  if (r.count <= 0) return;
  uint32_t *st = state + (int64_t)row * (2 + 2 * P);
  const uint32_t *hs = hist + (int64_t)row * P * 2048;
  const int shift = level == 0 ? 21 : level == 1 ? 10 : 0, nb = level == 2 ? 1024 : 2048;
  const uint32_t remaining = level == 0 ? (uint32_t)r.count : st[1];
  // thread t owns the bins nb-1-2t and nb-2-2t of the row's histogram (the parts added up)
  const int b0 = nb - 1 - 2 * tid, b1 = nb - 2 - 2 * tid;
  uint32_t c0 = 0, c1 = 0;
  if (b0 >= 0)
    for (int p = 0; p < P; ++p) {
      c0 += hs[(int64_t)p * 2048 + b0];
      if (b1 >= 0) c1 += hs[(int64_t)p * 2048 + b1];
    }
  uint32_t total;
  const uint32_t above = block_exclusive_scan(c0 + c1, wave_tot, &total);
  if (above < remaining && remaining <= above + c0) {
    found[0] = (uint32_t)b0;
    found[1] = remaining - above;
  } else if (above + c0 < remaining && remaining <= above + c0 + c1) {
    found[0] = (uint32_t)b1;
    found[1] = remaining - above - c0;
  }
  __syncthreads();
  const int digit = (int)found[0];
  // per part: keys above the extended prefix (one wavefront per part), keys equal to it
  for (int p = wave; p < P; p += kSelWaves) {
    uint32_t gt = 0;
    for (int b = digit + 1 + lane; b < nb; b += 64) gt += hs[(int64_t)p * 2048 + b];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) gt += __shfl_down(gt, off, 64);
    if (lane == 0) {
      st[2 + p] = (level == 0 ? 0u : st[2 + p]) + gt;
      st[2 + P + p] = hs[(int64_t)p * 2048 + digit];
    }
  }
  if (tid == 0) {
    st[0] = (level == 0 ? 0u : st[0]) | ((uint32_t)digit << shift);
    st[1] = found[1];
  }
}

__global__ __launch_bounds__(kSelThreads) void msel_emit_kernel(Dims d, SeqTab t, const float *__restrict__ pooled,
                                                                int P, int part_len,
                                                                const uint32_t *__restrict__ state,
                                                                int32_t *__restrict__ idx) {
  __shared__ SelShared sh;
  const int row = blockIdx.x / P, part = blockIdx.x % P;
  const RowRef r = row_of(d, t, row, pooled, idx);
  if (part == 0) {
    for (int x = threadIdx.x; x < d.w; x += kSelThreads) r.out[r.count + x] = r.m + x;   // window, last
    for (int x = r.count + d.w + threadIdx.x; x < r.n_keep; x += kSelThreads) r.out[x] = -1;   // unused slots
  }
  const int start = part * part_len;
  const int len = min(part_len, r.m - start);
  if (r.count <= 0 || len <= 0) return;
  const uint32_t *st = state + (int64_t)row * (2 + 2 * P);
  uint32_t gt0 = 0, eq0 = 0;
  for (int q = 0; q < part; ++q) { gt0 += st[2 + q]; eq0 += st[2 + P + q]; }
  const float *x = r.x + start;
  emit_selected(x, len, split_row(x, len), st[0], st[1], r.out, sh, gt0, eq0, start);
}

// ----------------------------------------------------------------------------------
// layer budget shared across KV heads
// ----------------------------------------------------------------------------------
// The heads' counts follow from one layer-wide threshold: the largest key t for which
//   F(t) = sum over heads of max(0, #{keys of the head >= t} - floor)
// still reaches the number of slots left after the floors.  t is found digit by digit like
// the per-row radix select, with one histogram per head (kept in the workspace) and a small
// decision kernel per digit.  Search state per (layer, sequence): [0] prefix of t,
// [2 .. 2+Hkv) keys above the prefix per head, [2+Hkv .. 2+2Hkv) keys equal to t per head,
// [2+2Hkv .. 2+3Hkv) how many of a head's keys equal to t it keeps, with bit 31 set when t is also the
// head's own threshold (otherwise its floor reaches below t and the head runs its own radix search).
__host__ __device__ constexpr int kAdaStateWords(int hkv) { return 2 + 3 * hkv; }
__device__ __forceinline__ int ada_shift(int level) { return level == 0 ? 21 : level == 1 ? 10 : 0; }
__device__ __forceinline__ int ada_bins(int level) { return level == 2 ? 1024 : 2048; }

__global__ __launch_bounds__(kSelThreads) void ada_hist_kernel(Dims d, SeqTab t,
                                                               const float *__restrict__ pooled, int level,
                                                               const uint32_t *__restrict__ state,
                                                               uint32_t *__restrict__ hist) {
  __shared__ SelShared sh;
  const int tid = threadIdx.x;
  const int unit = blockIdx.x;
  const int g = unit % d.Hkv;
  const int ls = unit / d.Hkv;
  const int s = ls % d.S;
  const int layer = ls / d.S;
  const int n_s = t.cu[s + 1] - t.cu[s];
  const int m = n_s - d.w;
  const float *x = pooled + (int64_t)layer * d.Hkv * d.T + (int64_t)d.Hkv * t.cu[s] + (int64_t)g * n_s;
  const int shift = ada_shift(level), nb = ada_bins(level);
  const uint32_t mask = level == 0 ? 0u : level == 1 ? 0xffe00000u : 0xfffffc00u;
  const uint32_t prefix = level == 0 ? 0u : state[(int64_t)ls * kAdaStateWords(d.Hkv)];
  histogram_pass(x, max(m, 0), split_row(x, max(m, 0)), prefix, mask, shift, nb, sh);
  uint32_t *out = hist + (int64_t)unit * 2048;
  const bool neg = (prefix & 0x80000000u) == 0;
  for (int b = tid; b < 2048; b += kSelThreads) {       // b: ordered digit
    uint32_t c = 0;
    if (b < nb) {
      const int r = raw_digit(b, level, nb, neg);
#pragma unroll
      for (int cp = 0; cp < kHistCopies; ++cp) c += sh.hist[cp * 2048 + r];
    }
    out[b] = c;
  }
}

__global__ __launch_bounds__(kSelThreads) void ada_decide_kernel(Dims d, SeqTab t, int c_floor, int level,
                                                                 uint32_t *__restrict__ state,
                                                                 uint32_t *__restrict__ hist,
                                                                 int32_t *__restrict__ head_off) {
  __shared__ uint32_t wave_tot[kSelWaves];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ls = blockIdx.x;
  const int s = ls % d.S;
  const int H = d.Hkv;
  const int m = t.cu[s + 1] - t.cu[s] - d.w;
  const int C = min(d.c_max, m);
  const int f = min(c_floor, C);
  const unsigned long long need = (unsigned long long)H * (unsigned)(C - f);
  uint32_t *hs = hist + (int64_t)ls * H * 2048;
  uint32_t *st = state + (int64_t)ls * kAdaStateWords(H);
  const int shift = ada_shift(level), nb = ada_bins(level);

  // (i) each head's histogram becomes inclusive suffix sums (keys with this digit or a larger one)
  const int per = nb / 64;
  for (int h = wave; h < H; h += kSelWaves) {
    uint32_t *hh = hs + (int64_t)h * 2048 + lane * per;
    uint32_t v[32];
    uint32_t sum = 0;
#pragma unroll
    for (int i = 31; i >= 0; --i) {
      if (i < per) { sum += hh[i]; v[i] = sum; }
    }
    uint32_t run = sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t up = __shfl_down(run, off, 64);
      if (lane + off < 64) run += up;
    }
    const uint32_t higher = run - sum;
#pragma unroll
    for (int i = 0; i < 32; ++i)
      if (i < per) hh[i] = v[i] + higher;
  }
  __syncthreads();

  // (ii) F at the digits nb-1-2t and nb-2-2t; F does not grow with the digit, so the digits
  // that reach `need` are the lowest ones and their number gives the digit of t.
  const int b0 = nb - 1 - 2 * tid, b1 = nb - 2 - 2 * tid;
  unsigned long long F0 = 0, F1 = 0;
  if (b0 >= 0) {
    for (int h = 0; h < H; ++h) {
      const uint32_t above = level == 0 ? 0u : st[2 + h];
      const uint32_t c0 = above + hs[(int64_t)h * 2048 + b0];
      const uint32_t c1 = b1 >= 0 ? above + hs[(int64_t)h * 2048 + b1] : 0u;
      F0 += c0 > (uint32_t)f ? c0 - (uint32_t)f : 0u;
      F1 += c1 > (uint32_t)f ? c1 - (uint32_t)f : 0u;
    }
  }
  const uint32_t hits = (b0 >= 0 && F0 >= need ? 1u : 0u) + (b1 >= 0 && F1 >= need ? 1u : 0u);
  uint32_t n_hits;
  (void)block_exclusive_scan(hits, wave_tot, &n_hits);
  const int digit = (int)n_hits - 1;          // F(0) >= need always, so n_hits >= 1

  // (iii) per head: keys above the extended prefix, and keys equal to it
  if (tid < H) {
    const uint32_t ge = hs[(int64_t)tid * 2048 + digit];
    const uint32_t gt = digit + 1 < nb ? hs[(int64_t)tid * 2048 + digit + 1] : 0u;
    st[2 + tid] = (level == 0 ? 0u : st[2 + tid]) + gt;
    st[2 + H + tid] = ge - gt;
  }
  if (tid == 0) st[0] = (level == 0 ? 0u : st[0]) | ((uint32_t)digit << shift);
  if (level < 2) return;
  __syncthreads();
  // (iv) t is complete: heads above their floor keep every key larger than t; the slots still
  // open go to keys equal to t that no floor has taken, heads in order.
  if (tid == 0) {
    long long open = (long long)need;
    for (int h = 0; h < H; ++h) {
      const long long gt = st[2 + h];
      open -= gt > f ? gt - f : 0;
    }
    int32_t *ho = head_off + (int64_t)ls * (H + 1);
    int off = 0;
    for (int h = 0; h < H; ++h) {
      const long long gt = st[2 + h], eq = st[2 + H + h];
      long long avail = gt + eq - f < eq ? gt + eq - f : eq;
      if (avail < 0) avail = 0;
      const long long take = avail < open ? avail : open;
      open -= take;
      ho[h] = off;
      off += (int)((gt > f ? gt : f) + take) + d.w;
      // the head keeps its keys above t and (floor part + take) of those equal to t, if its
      // floor does not reach below t
      const long long ties = (gt < f ? f - gt : 0) + take;
      st[2 + 2 * H + h] = gt + eq >= f ? (0x80000000u | (uint32_t)ties) : 0u;
    }
    ho[H] = off;
  }
}

__global__ __launch_bounds__(kSelThreads) void select_ada_kernel(Dims d, SeqTab t,
                                                                 const float *__restrict__ pooled,
                                                                 const int32_t *__restrict__ head_off,
                                                                 const uint32_t *__restrict__ state,
                                                                 int32_t *__restrict__ idx) {
  __shared__ SelShared sh;
  const int unit = blockIdx.x;
  const int g = unit % d.Hkv;
  const int ls = unit / d.Hkv;
  const int s = ls % d.S;
  const int layer = ls / d.S;
  const int n_s = t.cu[s + 1] - t.cu[s];
  const int m = n_s - d.w;
  const int32_t *ho = head_off + (int64_t)ls * (d.Hkv + 1);
  const int start = ho[g];
  const int count = min(max(ho[g + 1] - start - d.w, 0), m);
  const float *row = pooled + (int64_t)layer * d.Hkv * d.T + (int64_t)d.Hkv * t.cu[s] + (int64_t)g * n_s;
  int32_t *out = idx + (int64_t)layer * d.Hkv * d.KT + (int64_t)d.Hkv * t.ck[s] + start;
  for (int x = threadIdx.x; x < d.w; x += kSelThreads) out[count + x] = m + x;
  if (count <= 0) return;
  const uint32_t *st = state + (int64_t)ls * kAdaStateWords(d.Hkv);
  const uint32_t known = st[2 + 2 * d.Hkv + g];
  if (known & 0x80000000u) emit_selected(row, m, split_row(row, m), st[0], known & 0x7fffffffu, out, sh);
  else select_top_row(row, m, count, out, sh);
}

// ----------------------------------------------------------------------------------
// neighbour expansion (single workgroup)
// ----------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelThreads) void expand_kernel(
    const int32_t *__restrict__ sel, int count, int n_in, int n_window, int nb,
    const int32_t *__restrict__ token_ids, int32_t *__restrict__ idx_out,
    int32_t *__restrict__ ids_out, int32_t *__restrict__ count_out) {
  __shared__ uint32_t wave_tot[2][kSelWaves];
  const int tid = threadIdx.x;
  uint32_t written = 0;
  int buf = 0;
  // `sel` is ascending, so interval r = [t_r - nb, t_r + nb] only has to be trimmed
  // against the end of interval r-1 to make the union duplicate-free.
  for (int r0 = 0; r0 < count; r0 += kSelThreads, buf ^= 1) {
    const int r = r0 + tid;
    int start = 0, fresh = 0;
    if (r < count) {
      const int tok = sel[r];
      const int lo = max(0, tok - nb), hi = min(n_in - 1, tok + nb);
      const int prev_hi = r > 0 ? min(n_in - 1, sel[r - 1] + nb) : -1;
      start = max(lo, prev_hi + 1);
      fresh = max(0, hi - start + 1);
    }
    uint32_t total;
    uint32_t pos = written + block_exclusive_scan((uint32_t)fresh, wave_tot[buf], &total);
    for (int e = 0; e < fresh; ++e) {
      idx_out[pos + e] = start + e;
      ids_out[pos + e] = token_ids[start + e];
    }
    written += total;
  }
  const int m = n_in - n_window;
  const int last_hi = count > 0 ? min(n_in - 1, sel[count - 1] + nb) : -1;
  const int wstart = max(m, last_hi + 1);
  for (int j = wstart + tid; j < n_in; j += kSelThreads) {
    idx_out[written + (j - wstart)] = j;
    ids_out[written + (j - wstart)] = token_ids[j];
  }
  if (tid == 0) *count_out = (int32_t)written + max(0, n_in - wstart);
}

}  // namespace

hipError_t launch_reduce_pool(const Plan &pl, const float *planes, float *raw, float *pooled,
                              hipStream_t st) {
  const Dims &d = pl.d;
  int max_n = 0;
  for (int s = 0; s < d.S; ++s) max_n = max(max_n, pl.t.cu[s + 1] - pl.t.cu[s]);
  const int tiles = (max_n + kPoolTile - 1) / kPoolTile;
  const int64_t blocks = (int64_t)d.L * d.S * d.Hkv * tiles;
  // planes of one head (PPH slices) merge like the rows of a head; heads merge by sum or max
  PlaneMerge pm;
  pm.n_inner = pl.g.PPH;
  pm.n_outer = pl.g.RS / pl.g.PPH;
  pm.inner_max = d.reduce_max;
  pm.outer_max = d.reduce_max && d.head_max;
  pm.plane_stride = (int64_t)d.L * d.Hkv * d.T;
  hipLaunchKernelGGL(reduce_pool_kernel, dim3((unsigned)blocks), dim3(kPoolThreads), 0, st, d, pl.t,
                     pm, planes, raw, pooled, tiles);
  return hipGetLastError();
}

hipError_t launch_reduce_pool_all(const Plan &pl, const float *planes, float *raw, float *pooled,
                                  hipStream_t st) {
  const Dims &d = pl.d;
  const int n_in = (int)d.T;
  const int tiles = (n_in + kAllTile - 1) / kAllTile;
  // every plane (row super-block, layer, head) merges with one op: all sums, or all maxima
  PlaneMerge pm;
  pm.n_inner = 1;
  pm.n_outer = pl.g.RS * d.L * d.Hkv;
  pm.inner_max = 0;
  pm.outer_max = d.reduce_max && d.head_max;
  pm.plane_stride = n_in;
  hipLaunchKernelGGL(reduce_pool_all_kernel, dim3(tiles), dim3(kAllTile * kAllSlices), 0, st, n_in, d.w,
                     d.pool_k, d.pool_avg, pm, planes, raw, pooled);
  return hipGetLastError();
}

hipError_t launch_pool_row(const float *in, float *out, int32_t n_in, int32_t n_window, int32_t pool_k,
                           hipStream_t st) {
  const int tiles = (n_in + kAllTile - 1) / kAllTile;
  PlaneMerge pm;
  pm.n_inner = 1; pm.n_outer = 1; pm.inner_max = 0; pm.outer_max = 0; pm.plane_stride = n_in;
  hipLaunchKernelGGL(reduce_pool_all_kernel, dim3(tiles), dim3(kAllTile * kAllSlices), 0, st, n_in, n_window,
                     pool_k, 0, pm, in, (float *)nullptr, out);
  return hipGetLastError();
}

hipError_t launch_select(const Plan &pl, const float *pooled, int32_t *idx, uint32_t *hist, uint32_t *state,
                         hipStream_t st) {
  const Dims &d = pl.d;
  const int64_t rows = (int64_t)d.L * d.S * d.Hkv;
  if (pl.sel_parts > 1 && hist != nullptr && state != nullptr) {
    const int P = pl.sel_parts;
    const dim3 wide((unsigned)(rows * P)), one((unsigned)rows), block(kSelThreads);
    for (int level = 0; level < 3; ++level) {
      hipLaunchKernelGGL(msel_hist_kernel, wide, block, 0, st, d, pl.t, pooled, level, P, pl.sel_part_len,
                         state, hist);
      hipLaunchKernelGGL(msel_decide_kernel, one, block, 0, st, d, pl.t, level, P, state, hist);
    }
    hipLaunchKernelGGL(msel_emit_kernel, wide, block, 0, st, d, pl.t, pooled, P, pl.sel_part_len, state, idx);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(select_kernel, dim3((unsigned)rows), dim3(kSelThreads), 0, st, d, pl.t, pooled, idx);
  return hipGetLastError();
}

hipError_t launch_select_ada(const Plan &pl, int32_t c_floor, const float *pooled, int32_t *idx,
                             int32_t *head_off, uint32_t *hist, uint32_t *state, hipStream_t st) {
  const Dims &d = pl.d;
  const unsigned pairs = (unsigned)(d.L * d.S);
  for (int level = 0; level < 3; ++level) {
    hipLaunchKernelGGL(ada_hist_kernel, dim3(pairs * d.Hkv), dim3(kSelThreads), 0, st, d, pl.t, pooled,
                       level, state, hist);
    hipLaunchKernelGGL(ada_decide_kernel, dim3(pairs), dim3(kSelThreads), 0, st, d, pl.t, c_floor, level,
                       state, hist, head_off);
  }
  hipLaunchKernelGGL(select_ada_kernel, dim3(pairs * d.Hkv), dim3(kSelThreads), 0, st, d, pl.t, pooled,
                     head_off, state, idx);
  return hipGetLastError();
}

hipError_t launch_select_row(const float *pooled_row, int32_t m, int32_t count, int32_t *sel,
                             hipStream_t st) {
  hipLaunchKernelGGL(select_row_kernel, dim3(1), dim3(kSelThreads), 0, st, pooled_row, m, count, sel);
  return hipGetLastError();
}

hipError_t launch_expand(const int32_t *sel, int32_t count, int32_t n_in, int32_t n_window,
                         int32_t n_neighbor, const int32_t *token_ids, int32_t *idx_out,
                         int32_t *ids_out, int32_t *count_out, hipStream_t st) {
  hipLaunchKernelGGL(expand_kernel, dim3(1), dim3(kSelThreads), 0, st, sel, count, n_in, n_window,
                     n_neighbor, token_ids, idx_out, ids_out, count_out);
  return hipGetLastError();
}

}  // namespace speckv
