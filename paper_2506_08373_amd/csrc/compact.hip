// KV-cache compaction: cache <- K[i_cache], V[i_cache]  (Alg. 1, last step).
//
// Pure gather, bound by HBM bandwidth.  One launch covers every layer, sequence and KV
// head, K and V together.  A row of d elements is moved by rowbytes/16 adjacent lanes,
// each with one non-temporal 128-bit load and store per tensor.  One row per thread group
// measured best (occupancy hides the latency; more rows per thread only cost registers).
#include "speckv_internal.h"

namespace speckv {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 1;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // one 128-bit lane access

template <bool HAS_V>
__global__ __launch_bounds__(kThreads) void compact_kernel(
    Dims d, SeqTab t, const char *__restrict__ k, const char *__restrict__ v,
    const int32_t *__restrict__ idx, char *__restrict__ k_out, char *__restrict__ v_out,
    int blocks_per_unit, int lpr_shift) {
  const int unit = blockIdx.x / blocks_per_unit;
  const int blk = blockIdx.x - unit * blocks_per_unit;
  const int g = unit % d.Hkv;
  const int s = (unit / d.Hkv) % d.S;
  const int layer = unit / (d.Hkv * d.S);
  const int n_keep = t.ck[s + 1] - t.ck[s];
  const int n_s = live_len(d, t, s);
  const int rows_per_step = kThreads >> lpr_shift;
  const int r0 = blk * rows_per_step * kUnroll;
  if (r0 >= n_keep) return;

  const int part = threadIdx.x & ((1 << lpr_shift) - 1);
  const int row_in_step = threadIdx.x >> lpr_shift;
  const int64_t rowbytes = (int64_t)d.D * d.elt;
  const int64_t out_row0 = (int64_t)layer * d.Hkv * d.KT + (int64_t)d.Hkv * t.ck[s] + (int64_t)g * n_keep;
  const int32_t *idx_row = idx + out_row0;
  const int64_t src_base = ((int64_t)layer * d.kv_sl + (int64_t)g * d.kv_sh) * d.elt + (int64_t)part * 16;
  const int64_t tok_bytes = d.kv_st * d.elt;

  u32x4 kv[kUnroll], vv[kUnroll];
  int rr[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const int r = r0 + u * rows_per_step + row_in_step;
    rr[u] = r;
    kv[u] = (u32x4)(0u);
    vv[u] = (u32x4)(0u);
    if (r < n_keep) {
      const int j = idx_row[r];
      if ((unsigned)j < (unsigned)n_s) {   // an index outside the sequence gives a zero row
        const int64_t off = src_base + (int64_t)(t.cu[s] + j) * tok_bytes;
        kv[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(k + off));
        if (HAS_V) vv[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(v + off));
      }
    }
  }
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    if (rr[u] < n_keep) {
      const int64_t off = (out_row0 + rr[u]) * rowbytes + (int64_t)part * 16;
      __builtin_nontemporal_store(kv[u], reinterpret_cast<u32x4 *>(k_out + off));
      if (HAS_V) __builtin_nontemporal_store(vv[u], reinterpret_cast<u32x4 *>(v_out + off));
    }
  }
}

// Shared layer budget: the heads of a (layer, sequence) block own row ranges given by head_off.
template <bool HAS_V>
__global__ __launch_bounds__(kThreads) void compact_ada_kernel(
    Dims d, SeqTab t, const char *__restrict__ k, const char *__restrict__ v,
    const int32_t *__restrict__ idx, const int32_t *__restrict__ head_off, char *__restrict__ k_out,
    char *__restrict__ v_out, int blocks_per_unit, int lpr_shift) {
  const int ls = blockIdx.x / blocks_per_unit;
  const int blk = blockIdx.x - ls * blocks_per_unit;
  const int s = ls % d.S;
  const int layer = ls / d.S;
  const int rows = d.Hkv * (t.ck[s + 1] - t.ck[s]);
  const int n_s = live_len(d, t, s);
  const int r = blk * (kThreads >> lpr_shift) + (threadIdx.x >> lpr_shift);
  if (r >= rows) return;
  // head of row r: the last g with head_off[g] <= r
  const int32_t *ho = head_off + (int64_t)ls * (d.Hkv + 1);
  int lo = 0, hi = d.Hkv;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (ho[mid] <= r) lo = mid; else hi = mid;
  }
  const int g = lo;
  const int part = threadIdx.x & ((1 << lpr_shift) - 1);
  const int64_t rowbytes = (int64_t)d.D * d.elt;
  const int64_t out_row = (int64_t)layer * d.Hkv * d.KT + (int64_t)d.Hkv * t.ck[s] + r;
  const int j = idx[out_row];
  u32x4 kv = (u32x4)(0u), vv = (u32x4)(0u);
  if ((unsigned)j < (unsigned)n_s) {
    const int64_t off = ((int64_t)layer * d.kv_sl + (int64_t)g * d.kv_sh + (int64_t)(t.cu[s] + j) * d.kv_st) * d.elt +
                        (int64_t)part * 16;
    kv = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(k + off));
    if (HAS_V) vv = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(v + off));
  }
  const int64_t off = out_row * rowbytes + (int64_t)part * 16;
  __builtin_nontemporal_store(kv, reinterpret_cast<u32x4 *>(k_out + off));
  if (HAS_V) __builtin_nontemporal_store(vv, reinterpret_cast<u32x4 *>(v_out + off));
}

}  // namespace

hipError_t launch_compact_ada(const Plan &pl, const void *k, const void *v, const int32_t *idx,
                              const int32_t *head_off, void *k_out, void *v_out, hipStream_t st) {
  const Dims &d = pl.d;
  const int rowbytes = d.D * d.elt;
  int lpr_shift = 0;
  while ((16 << lpr_shift) < rowbytes) ++lpr_shift;
  const int rows_per_block = kThreads >> lpr_shift;
  int64_t max_rows = 0;
  for (int s = 0; s < d.S; ++s) max_rows = max(max_rows, (int64_t)d.Hkv * (pl.t.ck[s + 1] - pl.t.ck[s]));
  if (max_rows == 0) return hipSuccess;
  const int64_t bpu = (max_rows + rows_per_block - 1) / rows_per_block;
  const int64_t blocks = (int64_t)d.L * d.S * bpu;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  dim3 grid((unsigned)blocks), block(kThreads);
  if (v != nullptr) {
    hipLaunchKernelGGL(compact_ada_kernel<true>, grid, block, 0, st, d, pl.t, (const char *)k,
                       (const char *)v, idx, head_off, (char *)k_out, (char *)v_out, (int)bpu, lpr_shift);
  } else {
    hipLaunchKernelGGL(compact_ada_kernel<false>, grid, block, 0, st, d, pl.t, (const char *)k,
                       (const char *)nullptr, idx, head_off, (char *)k_out, (char *)nullptr, (int)bpu,
                       lpr_shift);
  }
  return hipGetLastError();
}

hipError_t launch_compact(const Plan &pl, const void *k, const void *v, const int32_t *idx,
                          void *k_out, void *v_out, hipStream_t st) {
  const Dims &d = pl.d;
  const int rowbytes = d.D * d.elt;
  int lpr_shift = 0;
  while ((16 << lpr_shift) < rowbytes) ++lpr_shift;   // lanes per row = rowbytes / 16 (power of two)
  const int rows_per_block = (kThreads >> lpr_shift) * kUnroll;
  int max_keep = 0;
  for (int s = 0; s < d.S; ++s) max_keep = max(max_keep, pl.t.ck[s + 1] - pl.t.ck[s]);
  if (max_keep == 0) return hipSuccess;
  const int bpu = (max_keep + rows_per_block - 1) / rows_per_block;
  const int64_t blocks = (int64_t)d.L * d.S * d.Hkv * bpu;
  dim3 grid((unsigned)blocks), block(kThreads);
  if (v != nullptr) {
    hipLaunchKernelGGL(compact_kernel<true>, grid, block, 0, st, d, pl.t, (const char *)k,
                       (const char *)v, idx, (char *)k_out, (char *)v_out, bpu, lpr_shift);
  } else {
    hipLaunchKernelGGL(compact_kernel<false>, grid, block, 0, st, d, pl.t, (const char *)k,
                       (const char *)nullptr, idx, (char *)k_out, (char *)nullptr, bpu, lpr_shift);
  }
  return hipGetLastError();
}

}  // namespace speckv
