// Pooling, top-C selection and index expansion.
//
//  * reduce_pool: sums the partial score planes the scoring kernels wrote, emits the raw
//    importance (Eq. 1, summed over queries and the GQA group) and its 1-D max-pool with
//    kernel k over the non-window candidates (Alg. 1 pooling step; table: Max, k = 7).
//  * select: the C largest pooled scores per (layer, sequence, KV head), ties to the
//    smaller index, ascending, then the window m..n_in-1 (Alg. 1 "Select KVs").
//    MSD radix select on order-preserving 32-bit keys (digits of 11 + 11 + 10 bits).  One
//    workgroup per row; every step is deterministic.  The histogram of the first digit comes
//    from the pooling kernel in the fused calls (else from one read of the row); rows of up to
//    about 229K entries are then read once more: entries above the threshold's bin are
//    selected outright, the few inside it settle the other two digits in LDS.  Longer rows, and
//    rows with more than 4096 entries in that bin, take one read per digit plus an ordered
//    compaction.  A workgroup is bound by its vector ALU, so the per-element work is kept
//    minimal: 128-bit loads, float compares against the bin's bounds, digits from raw bits.
//  * shared layer budget: per-head counts from one layer-wide threshold (histogram and
//    decision kernels per digit), then the same row select with each head's own count.
//  * expand: widens selected tokens to +-n_neighbor, unites them with the window and
//    emits the sorted set with the token ids gathered (Sec. 4.2 prompt compression).
#include "speckv_internal.h"

namespace speckv {
namespace {

// Raw bits of x with -0 turned into +0 (the two compare equal and must share a bin).
__device__ __forceinline__ uint32_t raw_bits(float x) { return __float_as_uint(x + 0.0f); }
// Ordered key of a float (larger float, larger key): key = u | 0x80000000 for a positive number
// with bits u and ~u for a negative one.  The selection works on digits of this key.
__device__ __forceinline__ uint32_t ordered_key(float x) {
  const uint32_t u = raw_bits(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

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
                                        float *tile, uint32_t *first_digit = nullptr) {
  // window of key j: j - half .. j + after (symmetric for odd kernels; an even kernel looks one
  // position further back than ahead, the library convention with padding k / 2)
  const int half = pool_k / 2, after = (pool_k - 1) / 2;
  const int span = kPoolTile + 2 * half;
  constexpr int kPerThread = (kPoolTile + SPECKV_MAX_POOL_K + kPoolThreads - 1) / kPoolThreads;
  if (pm.n_inner == 1 && pm.n_outer <= 2) {
    // one or two planes (the usual case): every load of the thread is issued before the first is used
    float r0[kPerThread], r1[kPerThread];
#pragma unroll
    for (int u = 0; u < kPerThread; ++u) {
      const int x = threadIdx.x + u * kPoolThreads, jj = j0 - half + x;
      const bool ok = x < span && jj >= 0 && jj < n_s;
      r0[u] = ok ? in[jj] : 0.f;
      r1[u] = ok && pm.n_outer == 2 ? in[jj + pm.plane_stride] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < kPerThread; ++u) {
      const int x = threadIdx.x + u * kPoolThreads;
      const float a0 = pm.inner_max ? fmaxf(0.f, r0[u]) : r0[u], a1 = pm.inner_max ? fmaxf(0.f, r1[u]) : r1[u];
      if (x < span) tile[x] = pm.outer_max ? fmaxf(fmaxf(0.f, a0), a1) : 0.f + a0 + a1;
    }
  } else
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
      if (first_digit != nullptr) atomicAdd(&first_digit[ordered_key(best) >> 21], 1u);   // selection's first digit
    }
    pooled[j] = best;
  }
}

__global__ __launch_bounds__(kPoolThreads) void reduce_pool_kernel(
    Dims d, SeqTab t, PlaneMerge pm, const float *__restrict__ planes,
    float *__restrict__ raw, float *__restrict__ pooled, int tiles_per_row, uint32_t *__restrict__ hist0) {
  __shared__ float tile[kPoolTile + SPECKV_MAX_POOL_K + 1];
  __shared__ uint32_t first_digit[2048];
  const int unit = blockIdx.x / tiles_per_row;
  const int j0 = (blockIdx.x - unit * tiles_per_row) * kPoolTile;
  const int g = unit % d.Hkv;
  const int s = (unit / d.Hkv) % d.S;
  const int layer = unit / (d.Hkv * d.S);
  const int n_row = t.cu[s + 1] - t.cu[s];
  if (j0 >= n_row) return;
  const int n_s = live_len(d, t, s);
  const int64_t base = (int64_t)layer * d.Hkv * d.T + (int64_t)d.Hkv * t.cu[s] + (int64_t)g * n_row;
  // with hist0: the tile's histogram of the first selection digit is built in LDS (cleared here; the
  // barrier inside reduce_pool_tile orders the clearing before the counting) and added to the row's
  if (hist0 != nullptr)
    for (int b = threadIdx.x; b < 2048; b += kPoolThreads) first_digit[b] = 0;
  reduce_pool_tile(planes + base, pm, raw ? raw + base : nullptr, pooled + base, n_s, n_row, n_s - d.w,
                   d.pool_k, d.pool_avg, j0, tile, hist0 != nullptr ? first_digit : nullptr);
  if (hist0 != nullptr) {
    __syncthreads();
    for (int b = threadIdx.x; b < 2048; b += kPoolThreads) {
      const uint32_t c = first_digit[b];
      if (c != 0) atomicAdd(&hist0[(int64_t)unit * 2048 + b], c);
    }
  }
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

struct SelShared {
  uint32_t hist[kHistCopies * 2048];   // one copy per lane residue: spreads atomics that hit one bin
  uint32_t wave_tot[2][kSelWaves];
  uint32_t prefix, remaining, bin_count;
};

// Inclusive prefix sum over the 64 lanes of a wavefront with data-parallel-primitive moves:
// shifts by 1, 2, 4, 8 inside each row of 16 lanes (lanes without a source add 0), then lane 15 of
// rows 0 and 2 is added to rows 1 and 3, then lane 31 to rows 2 and 3.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
  int x = (int)v;
  x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, false);   // row_shr:1
  x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, false);   // row_shr:2
  x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, false);   // row_shr:4
  x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, false);   // row_shr:8
  x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
  x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
  return (uint32_t)x;
}

// Exclusive prefix sum of v over the wavefront; *total gets the sum.
__device__ __forceinline__ uint32_t wave_exclusive_scan(uint32_t v, uint32_t *total) {
  const uint32_t inc = wave_inclusive_scan(v);
  *total = (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
  return inc - v;
}

// Exclusive prefix sum of v over the workgroup in thread order; *total gets the sum.
// Wavefront scans, then LDS for the 16 wave totals.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *wave_tot, uint32_t *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t inc = wave_inclusive_scan(v);
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

// c0, c1: this thread's counts of the entries with digit nb-1-2t and nb-2-2t (ordered digits of
// level `pass`, t the thread) among the entries that share `prefix`.  Extends `prefix` by the digit
// that holds the remaining-th largest of them, reduces `remaining` to its rank among the entries
// with that digit and returns how many entries have it.
__device__ __forceinline__ uint32_t decide_from_counts(SelShared &sh, int pass, uint32_t c0, uint32_t c1,
                                                       uint32_t &prefix, uint32_t &mask, uint32_t &remaining) {
  const int tid = threadIdx.x;
  const int shift = pass == 0 ? 21 : pass == 1 ? 10 : 0;       // digits of 11, 11 and 10 bits
  const int nb = pass == 2 ? 1024 : 2048;
  const int b0 = nb - 1 - 2 * tid, b1 = nb - 2 - 2 * tid;      // scanning threads in order walks the bins downwards
  uint32_t total;
  const uint32_t above = block_exclusive_scan(c0 + c1, sh.wave_tot[0], &total);
  if (above < remaining && remaining <= above + c0) {
    sh.prefix = prefix | ((uint32_t)b0 << shift);
    sh.remaining = remaining - above;
    sh.bin_count = c0;
  } else if (above + c0 < remaining && remaining <= above + c0 + c1) {
    sh.prefix = prefix | ((uint32_t)b1 << shift);
    sh.remaining = remaining - above - c0;
    sh.bin_count = c1;
  }
  __syncthreads();
  prefix = sh.prefix;
  remaining = sh.remaining;
  const uint32_t in_bin = sh.bin_count;
  mask |= (uint32_t)(nb - 1) << shift;
  __syncthreads();
  return in_bin;
}

// The same after histogram_pass for digit `pass`: the counts come from the LDS histogram.
__device__ __forceinline__ uint32_t decide_digit(SelShared &sh, int pass, uint32_t &prefix, uint32_t &mask,
                                                 uint32_t &remaining) {
  const int tid = threadIdx.x;
  const int nb = pass == 2 ? 1024 : 2048;
  const int b0 = nb - 1 - 2 * tid, b1 = nb - 2 - 2 * tid;
  const bool neg = (prefix & 0x80000000u) == 0;
  const int r0 = raw_digit(b0, pass, nb, neg), r1 = raw_digit(b1, pass, nb, neg);
  uint32_t c0 = 0, c1 = 0;
#pragma unroll
  for (int cp = 0; cp < kHistCopies; ++cp) {
    if (b0 >= 0) c0 += sh.hist[cp * 2048 + r0];
    if (b1 >= 0) c1 += sh.hist[cp * 2048 + r1];
  }
  return decide_from_counts(sh, pass, c0, c1, prefix, mask, remaining);
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
      const uint32_t gt_before = run_gt + (before & 0xffffu), eq_before = run_eq + (before >> 16);
      // selected entries are rare: only the set bits are visited
      for (uint32_t rest = gt_bits | eq_bits; rest != 0; rest &= rest - 1) {
        const int b = __ffs(rest) - 1;
        const uint32_t below = (1u << b) - 1u;
        const uint32_t gt_b = gt_before + __popc(gt_bits & below), eq_b = eq_before + __popc(eq_bits & below);
        if (((gt_bits >> b) & 1u) || eq_b < need_eq) out[gt_b + min(eq_b, need_eq)] = index_base + rs.lead + 4 * vb + b;
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

// ---- rows of up to kFastMaxVec vectors: one more read once a digit or two are decided ----
// With the leading digit(s) of the threshold decided, the keys that start the same way form one
// range of floats.  Entries above it are selected whatever the other digits turn out to be
// ("winners"); only the entries inside it ("candidates", usually a small fraction of the row) decide
// the rest of the threshold.  So the row is read just once more:
//   1. every wavefront classifies a contiguous part of the row, tile by tile (two float compares
//      per entry), and leaves per thread and tile a word of winner and candidate bits in LDS - no
//      scans, no barriers;
//   2. after one exchange of the wavefronts' totals each wavefront walks its words again (LDS only),
//      turns the bit counts into positions with one wavefront scan and appends its candidates to an
//      LDS list in index order (index, winners before); the candidates' keys are then gathered by
//      all threads together (the row is in cache);
//   3. the remaining digits of the threshold are found on that list;
//   4. every output position follows from counts that are already there:
//        a selected candidate goes to  (winners before it) + (selected candidates before it),
//        a winner to                   (winners before it) + (selected candidates with a smaller index).
//      For the latter the selected candidates are counted per range (the entries one wavefront holds
//      in one tile: consecutive indices); a winner adds the ranges before its own and searches the
//      few selected candidates of its own range.
constexpr int kFastSlots = 16;                                   // per wavefront: leading scalars, 14 tiles, trailing scalars
constexpr int kWaveTileVec = 64 * kSelVec;                       // 128-bit vectors per wavefront tile
constexpr int kFastMaxVec = (kFastSlots - 2) * kWaveTileVec * kSelWaves;
constexpr int kFastRanges = kFastSlots * kSelWaves;
constexpr int kCandCap = 4096;                                   // candidates the LDS list holds

struct FastShared {
  uint32_t marks[kFastSlots][kSelThreads + 1];   // per thread and slot: winner bits (low 16) and candidate bits, later
                                                 // winner bits and the winners before them in the wavefront's part
                                                 // (rows padded by one word: step 2 reads across slots)
  uint32_t ckey[kCandCap];                    // candidates in index order: ordered key (later: indices of the
                                              //   selected candidates, ascending),
  int32_t cidx[kCandCap];                     //   index in the row,
  uint32_t cgtb[kCandCap];                    //   winners before it (low 24 bits), its range (high 8 bits)
  uint32_t hist[2048];
  uint32_t range_sel[kFastRanges + 1];        // selected candidates before each range (wavefront-major)
  uint32_t wave_cnt[kSelWaves];               // winners (low 16 bits) and candidates per wavefront
  uint32_t wave_tot[2][kSelWaves];
  uint32_t found[2];
};
constexpr size_t kSelLdsBytes = sizeof(FastShared) > sizeof(SelShared) ? sizeof(FastShared) : sizeof(SelShared);

// Smallest and largest float whose ordered key starts with the `bits` (11 or 22) leading bits of
// `prefix`.  Ranges that hold NaN patterns are cut at the infinities, and a range that would end at
// -0 ends at the largest negative number instead (zero of either sign has the key of +0).
__device__ __forceinline__ void prefix_bounds(uint32_t prefix, int bits, float *lo, float *hi) {
  const uint32_t low = 0xffffffffu >> bits;                     // the key bits the prefix leaves open
  const uint32_t k_lo = prefix & ~low, k_hi = prefix | low;     // smallest / largest key of the range
  if (prefix & 0x80000000u) {                                   // positive numbers: bits = key without the top bit
    *lo = __uint_as_float(min(k_lo ^ 0x80000000u, 0x7f800000u));
    *hi = __uint_as_float(min(k_hi ^ 0x80000000u, 0x7f800000u));
  } else {                                                      // negative numbers: bits = ~key
    *lo = __uint_as_float(min(~k_lo, 0xff800000u));
    *hi = __uint_as_float(min(max(~k_hi, 0x80000001u), 0xff800000u));
  }
}

// The threshold's key starts with the `bits` (11: one digit decided, 22: two) leading bits of
// `prefix`.  Writes the `take` largest of the entries whose key starts the same way plus every
// larger entry, indices ascending, ties to the lower index (see above).  rs.nv <= kFastMaxVec and
// at most kCandCap entries share the prefix.
__device__ __forceinline__ void select_after_prefix(const float *__restrict__ x, int m, RowSplit rs,
                                                    uint32_t prefix, int bits, uint32_t take,
                                                    int32_t *__restrict__ out, FastShared &fs) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  float lo_f, hi_f;
  prefix_bounds(prefix, bits, &lo_f, &hi_f);
  // the wavefront's part of the vectors: whole tiles, the same number for every wavefront
  const int part_vec = ((rs.nv + kSelWaves - 1) / kSelWaves + kWaveTileVec - 1) / kWaveTileVec * kWaveTileVec;
  const int v_begin = min(wv * part_vec, rs.nv), v_end = min(v_begin + part_vec, rs.nv);
  const int n_tiles = (v_end - v_begin + kWaveTileVec - 1) / kWaveTileVec;
  const bool has_lead = wv == 0 && rs.lead > 0, has_tail = wv == kSelWaves - 1 && m > rs.tail0;
  // row index of bit 0 of the word of lane `ln` of this wavefront in a slot
  auto index0 = [&](int slot, int ln) {
    if (slot == 0) return ln;
    if (slot == kFastSlots - 1) return rs.tail0 + ln;
    return rs.lead + 4 * (v_begin + (slot - 1) * kWaveTileVec + ln * kSelVec);
  };

  // ---- 1. classification
  uint32_t mine = 0;                            // this thread's winners (low 16 bits) and candidates
  auto classify_scalar = [&](int slot, int first, int n) {
    uint32_t w = 0;
    if (lane < n) {
      const float xv = x[first + lane];
      w = (xv > hi_f ? 1u : 0u) | ((xv >= lo_f && xv <= hi_f) ? 1u << 16 : 0u);
    }
    fs.marks[slot][tid] = w;
    mine += w;
  };
  if (has_lead) classify_scalar(0, 0, rs.lead);
  if (n_tiles > 0) {
    // the values of the next tile are requested before the current tile is classified
    const float4 *xv = reinterpret_cast<const float4 *>(x + rs.lead);
    float4 val[kSelVec], nxt[kSelVec];
#pragma unroll
    for (int e = 0; e < kSelVec; ++e) val[e] = xv[min(v_begin + lane * kSelVec + e, rs.nv - 1)];
    for (int tile = 0; tile < n_tiles; ++tile) {
      const int vb = v_begin + tile * kWaveTileVec + lane * kSelVec;
#pragma unroll
      for (int e = 0; e < kSelVec; ++e) nxt[e] = xv[min(vb + kWaveTileVec + e, rs.nv - 1)];
      uint32_t gt_bits = 0, ge_bits = 0;
#pragma unroll
      for (int e = 0; e < kSelVec; ++e) {
        const float e4[4] = {val[e].x, val[e].y, val[e].z, val[e].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          gt_bits |= e4[c] > hi_f ? 1u << (4 * e + c) : 0u;
          ge_bits |= e4[c] >= lo_f ? 1u << (4 * e + c) : 0u;
        }
      }
      const int n_valid = min(max(v_end - vb, 0), kSelVec);                 // vectors of this thread inside the part
      const uint32_t valid = (1u << (4 * n_valid)) - 1u;
      gt_bits &= valid;
      const uint32_t c_bits = ge_bits & ~gt_bits & valid;
      fs.marks[1 + tile][tid] = gt_bits | (c_bits << 16);
      mine += __popc(gt_bits) | (__popc(c_bits) << 16);
#pragma unroll
      for (int e = 0; e < kSelVec; ++e) val[e] = nxt[e];
    }
  }
  if (has_tail) classify_scalar(kFastSlots - 1, rs.tail0, m - rs.tail0);
  // a part holds fewer than 2^16 entries, so the packed counts cannot overflow
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mine += __shfl_xor(mine, off, 64);
  if (lane == 0) fs.wave_cnt[wv] = mine;
  for (int b = tid; b <= kFastRanges; b += kSelThreads) fs.range_sel[b] = 0;
  __syncthreads();
  uint32_t gt_base = 0, c_base = 0, c_all = 0;   // winners / candidates before this wavefront's part; all candidates
#pragma unroll
  for (int w2 = 0; w2 < kSelWaves; ++w2) {
    const uint32_t v = fs.wave_cnt[w2];
    if (w2 < wv) { gt_base += v & 0xffffu; c_base += v >> 16; }
    c_all += v >> 16;
  }

  // ---- 2. positions inside the wavefront's part; candidates to the list (their keys follow)
  {
    uint32_t run_gt = 0, run_c = c_base;
    // one word of lane `ln`: the winners before it become its upper half, its candidates are listed
    auto place_word = [&](int slot, int ln, uint32_t g_before, uint32_t c_before) {
      const uint32_t w = fs.marks[slot][wv * 64 + ln];
      const uint32_t gt_bits = w & 0xffffu, c_bits = w >> 16;
      fs.marks[slot][wv * 64 + ln] = gt_bits | (g_before << 16);
      for (uint32_t rest = c_bits; rest != 0; rest &= rest - 1) {          // candidates are few
        const int b = __ffs(rest) - 1;
        const uint32_t below = (1u << b) - 1u;
        const uint32_t cpos = c_before + __popc(c_bits & below);
        if (cpos < (uint32_t)kCandCap) {
          fs.cidx[cpos] = index0(slot, ln) + b;
          fs.cgtb[cpos] = (gt_base + g_before + __popc(gt_bits & below)) | ((uint32_t)(wv * kFastSlots + slot) << 24);
        }
      }
    };
    auto place_scalar = [&](int slot) {
      const uint32_t w = fs.marks[slot][tid];
      uint32_t total;
      const uint32_t before = wave_exclusive_scan((w & 1u) | (w & 0x10000u), &total);
      place_word(slot, lane, run_gt + (before & 0xffffu), run_c + (before >> 16));
      run_gt += total & 0xffffu;
      run_c += total >> 16;
    };
    if (has_lead) place_scalar(0);
    if (n_tiles > 0) {
      // The wavefront's n_tiles * 64 words form one sequence in index order (tile, lane).  Lane l takes
      // the n_tiles consecutive words from n_tiles * l on, so that one wavefront scan serves all tiles.
      uint32_t sum = 0;
      for (int i = 0; i < n_tiles; ++i) {
        const int f = n_tiles * lane + i;
        const uint32_t w = fs.marks[1 + (f >> 6)][wv * 64 + (f & 63)];
        sum += __popc(w & 0xffffu) | (__popc(w >> 16) << 16);
      }
      uint32_t total;
      const uint32_t before = wave_exclusive_scan(sum, &total);
      uint32_t g_run = run_gt + (before & 0xffffu), c_run = run_c + (before >> 16);
      for (int i = 0; i < n_tiles; ++i) {
        const int f = n_tiles * lane + i;
        const uint32_t w = fs.marks[1 + (f >> 6)][wv * 64 + (f & 63)];
        place_word(1 + (f >> 6), f & 63, g_run, c_run);
        g_run += __popc(w & 0xffffu);
        c_run += __popc(w >> 16);
      }
      run_gt += total & 0xffffu;
      run_c += total >> 16;
    }
    if (has_tail) place_scalar(kFastSlots - 1);
  }
  __syncthreads();
  const int nc = (int)min(c_all, (uint32_t)kCandCap);
  for (int c = tid; c < nc; c += kSelThreads) fs.ckey[c] = ordered_key(x[fs.cidx[c]]);   // read again: cache hits

  // ---- 3. the rest of the threshold: the r-th largest of the nc listed keys, by the digits that
  // are still open (11 and 10 bits, or the last 10 bits only)
  const uint32_t r = min(take, (uint32_t)nc);
  int buf = 0;
  if (nc > 0) {
    uint32_t total;
    if (bits == 11) {
      for (int b = tid; b < 2048; b += kSelThreads) fs.hist[b] = 0;
      __syncthreads();
      for (int c = tid; c < nc; c += kSelThreads) atomicAdd(&fs.hist[(fs.ckey[c] >> 10) & 2047u], 1u);
      __syncthreads();
      const int b0 = 2047 - 2 * tid, b1 = 2046 - 2 * tid;
      const uint32_t c0 = fs.hist[b0], c1 = fs.hist[b1];
      const uint32_t above = block_exclusive_scan(c0 + c1, fs.wave_tot[buf], &total);
      buf ^= 1;
      if (above < r && r <= above + c0) { fs.found[0] = (uint32_t)b0; fs.found[1] = r - above; }
      else if (above + c0 < r && r <= above + c0 + c1) { fs.found[0] = (uint32_t)b1; fs.found[1] = r - above - c0; }
    } else if (tid == 0) {
      fs.found[0] = (prefix >> 10) & 2047u;     // the second digit is part of the prefix
      fs.found[1] = r;
    }
    __syncthreads();
    const uint32_t d1 = fs.found[0], r1 = fs.found[1];
    fs.hist[tid] = 0;                           // 1024 bins, one per thread
    __syncthreads();
    for (int c = tid; c < nc; c += kSelThreads) {
      const uint32_t k = fs.ckey[c];
      if (((k >> 10) & 2047u) == d1) atomicAdd(&fs.hist[k & 1023u], 1u);
    }
    __syncthreads();
    {
      const int b0 = 1023 - tid;
      const uint32_t c0 = fs.hist[b0];
      const uint32_t above = block_exclusive_scan(c0, fs.wave_tot[buf], &total);
      buf ^= 1;
      if (above < r1 && r1 <= above + c0) { fs.found[0] = (uint32_t)b0; fs.found[1] = r1 - above; }
    }
    __syncthreads();
    const uint32_t thr21 = (d1 << 10) | fs.found[0], need_eq = fs.found[1];

    // selected candidates, in list (= index) order; their indices overwrite the keys (position <=
    // list position, and every key of a round is read before the round's scan)
    uint32_t run_sg = 0, run_eq = 0;
    for (int c0 = 0; c0 < nc; c0 += kSelThreads) {
      const int c = c0 + tid;
      const uint32_t k21 = c < nc ? fs.ckey[c] & 0x1fffffu : 0u;
      const bool is_gt = c < nc && k21 > thr21, is_eq = c < nc && k21 == thr21;
      const uint32_t before = block_exclusive_scan((is_gt ? 1u : 0u) | (is_eq ? 1u << 16 : 0u), fs.wave_tot[buf], &total);
      buf ^= 1;
      const uint32_t eq_b = run_eq + (before >> 16);
      if (is_gt || (is_eq && eq_b < need_eq)) {
        const uint32_t pos = run_sg + (before & 0xffffu) + min(eq_b, need_eq);
        const int32_t j = fs.cidx[c];
        const uint32_t gr = fs.cgtb[c];
        fs.ckey[pos] = (uint32_t)j;
        out[(gr & 0xffffffu) + pos] = j;
        atomicAdd(&fs.range_sel[gr >> 24], 1u);
      }
      run_sg += total & 0xffffu;
      run_eq += total >> 16;
    }
  }
  __syncthreads();
  // counts per range -> selected candidates before each range (one wavefront, 4 ranges per lane)
  static_assert(kFastRanges == 256, "four ranges per lane");
  if (tid < 64) {
    uint32_t v[4], sum = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[i] = fs.range_sel[4 * tid + i]; sum += v[i]; }
    uint32_t all;
    uint32_t run = wave_exclusive_scan(sum, &all);
#pragma unroll
    for (int i = 0; i < 4; ++i) { fs.range_sel[4 * tid + i] = run; run += v[i]; }
    if (tid == 63) fs.range_sel[kFastRanges] = all;
  }
  __syncthreads();

  // ---- 4. winners: position = winners before + selected candidates with a smaller index (those of
  // earlier ranges, plus those of the wavefront's own range that precede the winner)
  const int32_t *sidx = reinterpret_cast<const int32_t *>(fs.ckey);
  auto emit_winners = [&](int slot) {
    const uint32_t mk = fs.marks[slot][tid];
    uint32_t bits = mk & 0xffffu;
    if (bits == 0) return;
    const int s0 = (int)fs.range_sel[wv * kFastSlots + slot], s1 = (int)fs.range_sel[wv * kFastSlots + slot + 1];
    uint32_t pos = gt_base + (mk >> 16);
    const int j0 = index0(slot, lane);
    // selected candidates of the range before the thread's first winner: binary search; the
    // thread's other winners follow within 16 indices, so the count is advanced one by one
    int lo = s0, hi = s1;
    const int first = j0 + (__ffs(bits) - 1);
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (sidx[mid] < first) lo = mid + 1; else hi = mid;
    }
    for (; bits != 0; bits &= bits - 1) {
      const int j = j0 + (__ffs(bits) - 1);
      while (lo < s1 && sidx[lo] < j) ++lo;
      out[pos + (uint32_t)lo] = j;
      ++pos;
    }
  };
  if (has_lead) emit_winners(0);
  for (int tile = 0; tile < n_tiles; ++tile) emit_winners(1 + tile);
  if (has_tail) emit_winners(kFastSlots - 1);
}

// Writes the `count` (1 <= count <= m) indices of the largest x[0..m) to out, ascending,
// equal values taken from the low-index end.  lds: kSelLdsBytes of LDS.  first_digit, when not
// null: the row's histogram of the first digit (2048 counters by ordered digit), already counted.
__device__ __forceinline__ void select_top_row(const float *__restrict__ x, int m, int count,
                                               int32_t *__restrict__ out, unsigned char *lds,
                                               const uint32_t *__restrict__ first_digit = nullptr) {
  SelShared &sh = *reinterpret_cast<SelShared *>(lds);
  const RowSplit rs = split_row(x, m);
  uint32_t prefix = 0, mask = 0, remaining = (uint32_t)count;
  uint32_t in_bin;
  if (first_digit != nullptr) {
    const int tid = threadIdx.x;
    in_bin = decide_from_counts(sh, 0, first_digit[2047 - 2 * tid], first_digit[2046 - 2 * tid], prefix, mask, remaining);
  } else {
    histogram_pass(x, m, rs, prefix, mask, 21, 2048, sh);
    in_bin = decide_digit(sh, 0, prefix, mask, remaining);
  }
  if (rs.nv <= kFastMaxVec && in_bin <= (uint32_t)kCandCap) {
    select_after_prefix(x, m, rs, prefix, 11, remaining, out, *reinterpret_cast<FastShared *>(lds));
    return;
  }
  histogram_pass(x, m, rs, prefix, mask, 10, 2048, sh);
  in_bin = decide_digit(sh, 1, prefix, mask, remaining);
  if (rs.nv <= kFastMaxVec && in_bin <= (uint32_t)kCandCap) {
    select_after_prefix(x, m, rs, prefix, 22, remaining, out, *reinterpret_cast<FastShared *>(lds));
    return;
  }
  histogram_pass(x, m, rs, prefix, mask, 0, 1024, sh);
  (void)decide_digit(sh, 2, prefix, mask, remaining);
  emit_selected(x, m, rs, prefix, remaining, out, sh);
}

__global__ __launch_bounds__(kSelThreads) void select_kernel(Dims d, SeqTab t,
                                                             const float *__restrict__ pooled,
                                                             int32_t *__restrict__ idx,
                                                             const uint32_t *__restrict__ hist0) {
  extern __shared__ __attribute__((aligned(16))) unsigned char sel_lds[];
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
  if (count > 0) select_top_row(row, m, count, out, sel_lds, hist0 != nullptr ? hist0 + (int64_t)unit * 2048 : nullptr);
}

__global__ __launch_bounds__(kSelThreads) void select_row_kernel(const float *__restrict__ row,
                                                                 int m, int count,
                                                                 int32_t *__restrict__ sel) {
  extern __shared__ __attribute__((aligned(16))) unsigned char sel_lds[];
  if (count > 0) select_top_row(row, m, count, sel, sel_lds);
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
  const int n_s = t.cu[s + 1] - t.cu[s];                  // row stride
  const int m = live_len(d, t, s) - d.w;
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
  const int m = live_len(d, t, s) - d.w;
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
  extern __shared__ __attribute__((aligned(16))) unsigned char sel_lds[];
  const int unit = blockIdx.x;
  const int g = unit % d.Hkv;
  const int ls = unit / d.Hkv;
  const int s = ls % d.S;
  const int layer = ls / d.S;
  const int n_s = t.cu[s + 1] - t.cu[s];                  // row stride
  const int m = live_len(d, t, s) - d.w;
  const int32_t *ho = head_off + (int64_t)ls * (d.Hkv + 1);
  const int start = ho[g];
  const int count = min(max(ho[g + 1] - start - d.w, 0), m);
  const float *row = pooled + (int64_t)layer * d.Hkv * d.T + (int64_t)d.Hkv * t.cu[s] + (int64_t)g * n_s;
  int32_t *out = idx + (int64_t)layer * d.Hkv * d.KT + (int64_t)d.Hkv * t.ck[s] + start;
  for (int x = threadIdx.x; x < d.w; x += kSelThreads) out[count + x] = m + x;
  if (g == d.Hkv - 1) {     // a live prompt shorter than the host's bound leaves slots behind the last head unused
    const int used = ho[d.Hkv], slots = d.Hkv * (t.ck[s + 1] - t.ck[s]);
    for (int x = used + threadIdx.x; x < slots; x += kSelThreads) out[x - start] = -1;
  }
  if (count <= 0) return;
  const uint32_t *st = state + (int64_t)ls * kAdaStateWords(d.Hkv);
  const uint32_t known = st[2 + 2 * d.Hkv + g];
  if (known & 0x80000000u)
    emit_selected(row, m, split_row(row, m), st[0], known & 0x7fffffffu, out, *reinterpret_cast<SelShared *>(sel_lds));
  else select_top_row(row, m, count, out, sel_lds);
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
                              hipStream_t st, uint32_t *hist0) {
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
                     pm, planes, raw, pooled, tiles, hist0);
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
                         hipStream_t st, const uint32_t *hist0) {
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
  const hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(select_kernel), kSelLdsBytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(select_kernel, dim3((unsigned)rows), dim3(kSelThreads), kSelLdsBytes, st, d, pl.t, pooled, idx, hist0);
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
  const hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(select_ada_kernel), kSelLdsBytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(select_ada_kernel, dim3(pairs * d.Hkv), dim3(kSelThreads), kSelLdsBytes, st, d, pl.t, pooled,
                     head_off, state, idx);
  return hipGetLastError();
}

hipError_t launch_select_row(const float *pooled_row, int32_t m, int32_t count, int32_t *sel,
                             hipStream_t st) {
  const hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(select_row_kernel), kSelLdsBytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(select_row_kernel, dim3(1), dim3(kSelThreads), kSelLdsBytes, st, pooled_row, m, count, sel);
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
