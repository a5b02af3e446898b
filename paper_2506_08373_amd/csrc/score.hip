// Importance scoring: the kernels between the two sweeps and the host entry that strings the
// sweeps together (Sec. 3.1 Eq. 1; Alg. 1 CrossAttention and reduce steps).  The sweeps themselves
// are in score_sweep.h (compiled in score_rows.hip and score_cols.hip) and score_qs.hip.
#include <map>
#include <mutex>
#include <utility>

#include "score_common.h"

namespace speckv {
namespace {

// Merges the per-chunk (max2, sum) pairs of each row into lse2 = max2 + log2(sum).
// A block covers 64 rows; its 4 waves split the chunks and merge their partial pairs in LDS.
constexpr int kMergeRows = 64, kMergeSlices = 4;

// Zeroes A.clear (if any), the work spread over every thread of the grid.
__device__ inline void clear_scratch(const ScoreArgs &A) {
  if (A.clear == nullptr) return;
  const int64_t n_threads = (int64_t)gridDim.x * gridDim.y * blockDim.x;
  const int64_t id = ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * blockDim.x + threadIdx.x;
  for (int64_t i = id; i < A.clear_words; i += n_threads) A.clear[i] = 0u;
}

__device__ inline void merge_pair(float &m, float &l, float m2, float l2) {
  const float mm = fmaxf(m, m2);
  l = l * exp2f(m - mm) + l2 * exp2f(m2 - mm);
  m = mm;
}

__global__ __launch_bounds__(kMergeRows * kMergeSlices) void lse_combine_kernel(ScoreArgs A) {
  clear_scratch(A);
  __shared__ float2 partial[kMergeSlices][kMergeRows];
  const Dims &d = A.d;
  const int RSB = A.g.RSB;
  const int blocks_per_unit = RSB / kMergeRows;
  const int unit = blockIdx.x / blocks_per_unit;     // (layer, head, row super-block)
  const int r = (blockIdx.x % blocks_per_unit) * kMergeRows + (threadIdx.x % kMergeRows);
  const int slice = threadIdx.x / kMergeRows;
  const int s = blockIdx.y;
  const int rs = unit % A.g.RS;
  const int lh = unit / A.g.RS;                       // layer * Hkv + head
  const int c0 = A.t.cc[s], c1 = A.t.cc[s + 1];
  const float2 *pp = A.part + ((int64_t)unit * A.g.n_chunks) * RSB + r;
  float mm = kNegBig, ll = 0.f;
#pragma unroll 4
  for (int c = c0 + slice; c < c1; c += kMergeSlices) {
    const float2 v = pp[(int64_t)c * RSB];
    merge_pair(mm, ll, v.x, v.y);
  }
  if (slice == 0) {                                   // the sequence's masked tail chunk
    const float2 v = pp[(int64_t)(A.g.n_fast_chunks + s) * RSB];
    merge_pair(mm, ll, v.x, v.y);
  }
  partial[slice][threadIdx.x % kMergeRows] = make_float2(mm, ll);
  __syncthreads();
  if (slice == 0) {
#pragma unroll
    for (int k2 = 1; k2 < kMergeSlices; ++k2) {
      const float2 v = partial[k2][threadIdx.x];
      merge_pair(mm, ll, v.x, v.y);
    }
    A.lse[((int64_t)lh * d.S + s) * ((int64_t)A.g.RS * RSB) + rs * RSB + r] = mm + log2f(ll);
  }
}

// Converts caller-supplied natural-log normalisers [L][S][R][Hq] into the padded log2 layout
// the column-reduction sweep reads.
__global__ __launch_bounds__(256) void lse_import_kernel(ScoreArgs A) {
  clear_scratch(A);
  const Dims &d = A.d;
  const int RSB = A.g.RSB;
  const int unit = blockIdx.x;            // (layer, head, row super-block)
  const int s = blockIdx.y;
  const int rs = unit % A.g.RS;
  const int lh = unit / A.g.RS;           // layer * Hkv + head
  const int g = lh % d.Hkv, layer = lh / d.Hkv;
  for (int lr = threadIdx.x; lr < RSB; lr += blockDim.x) {
    int hh, i;
    float v = 0.f;
    if (decode_row(d, A.g, rs, lr, &hh, &i))
      v = A.lse_in[(((int64_t)layer * d.S + s) * d.R + i) * d.Hq + g * d.G + hh] * 1.4426950408889634f;
    A.lse[((int64_t)lh * d.S + s) * ((int64_t)A.g.RS * RSB) + rs * RSB + lr] = v;
  }
}

}  // namespace

// Raises a kernel's dynamic LDS limit; the runtime call is made once per (device, kernel, size)
// and remembered, so a fused call does not pay for it on every launch.
hipError_t allow_dynamic_lds(const void *kernel, size_t bytes) {
  static std::mutex mu;
  static std::map<std::pair<int, const void *>, size_t> granted;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> lock(mu);
  size_t &have = granted[std::make_pair(dev, kernel)];
  if (have >= bytes && have != 0) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess) have = bytes;
  return e;
}

int64_t score_fail_words(const Plan &pl) { return score_chunk_workgroups(pl.d, pl.g) * kFailWaves * kFailWords; }

bool score_uses_qs(const Plan &pl, int pass) {
  ScoreArgs A;
  A.d = pl.d; A.t = pl.t; A.g = pl.g;
  A.q = nullptr; A.k = nullptr; A.part = nullptr; A.lse = nullptr; A.planes = nullptr; A.lse_in = nullptr; A.chunk_blocks = 0; A.clear = nullptr; A.clear_words = 0; A.fail = nullptr;
  return qs_supported(A, pass);
}

hipError_t launch_score(const Plan &pl, const void *q, const void *k, float2 *part, float *lse,
                        float *planes, hipStream_t st, hipEvent_t *events, const float *lse_in,
                        uint32_t *clear, int64_t clear_words) {
  ScoreArgs A;
  A.d = pl.d; A.t = pl.t; A.g = pl.g;
  A.q = (const char *)q; A.k = (const char *)k;
  A.part = part; A.lse = lse; A.planes = planes; A.lse_in = lse_in; A.chunk_blocks = 0;
  A.clear = clear; A.clear_words = clear != nullptr ? clear_words : 0;
  A.fail = reinterpret_cast<int32_t *>(part + (int64_t)A.d.L * A.d.Hkv * A.g.RS * A.g.n_chunks * A.g.RSB);
  hipEvent_t *ev = events;
  hipError_t e;
  if (ev && (e = hipEventRecord(ev[0], st)) != hipSuccess) return e;
  if (A.lse_in == nullptr && (e = launch_row_statistics_sweep(A, st)) != hipSuccess) return e;
  if (ev && (e = hipEventRecord(ev[1], st)) != hipSuccess) return e;
  if (A.lse_in == nullptr) {
    hipLaunchKernelGGL(lse_combine_kernel, dim3(A.d.L * A.d.Hkv * A.g.RS * (A.g.RSB / kMergeRows), A.d.S),
                       dim3(kMergeRows * kMergeSlices), 0, st, A);
  } else {
    hipLaunchKernelGGL(lse_import_kernel, dim3(A.d.L * A.d.Hkv * A.g.RS, A.d.S), dim3(256), 0, st, A);
  }
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (ev && (e = hipEventRecord(ev[2], st)) != hipSuccess) return e;
  if ((e = launch_column_sweep(A, st)) != hipSuccess) return e;
  if (ev && (e = hipEventRecord(ev[3], st)) != hipSuccess) return e;
  return hipSuccess;
}

}  // namespace speckv
