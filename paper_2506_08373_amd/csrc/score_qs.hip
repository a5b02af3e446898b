// Scoring sweeps with the query rows stationary in LDS (Sec. 3.1 Eq. 1; Alg. 1 CrossAttention
// and reduce steps; App. C.2 for the GQA group).  An alternative to the tile-streaming kernel of
// score_sweep.h for the unmasked chunks of large groups: by default it runs the row-statistics sweep at
// d = 64; SPECKV_SCORE_KERNEL=qs selects it for every sweep it supports.
//
// Same mathematics (pass 1: per-row (reference, sum of exp2) over a chunk of keys; pass 2:
// per-key sum over the rows of 2^(c*S - lse2)), different dataflow:
//
//   * the M = G*R stacked query rows of the KV group (up to 512 rows, 128 KiB at d = 128) are
//     written to LDS once per workgroup, in the swizzled 16-byte-chunk layout of Tile<>;
//   * each of the eight waves (two per SIMD) owns every eighth 64-key step of the chunk and loads
//     the MFMA fragments of its keys straight from global memory into registers: no key tile in
//     LDS, no workgroup barrier inside the sweep, no cross-wave merge.  The next step's keys are
//     requested right after the last MFMAs of the current one; the other wave on the SIMD runs
//     meanwhile;
//   * per step a wave walks over the 32-row blocks of Q: K is the A operand, so a lane holds
//     16 keys of ONE query row per 32x32 block.  The row's normaliser (pass 2) or running
//     reference (pass 1) is a single value per lane and block;
//   * a wave alternates between a matrix phase (the block's MFMAs) and a vector phase (its
//     softmax arithmetic); without barriers the two waves of a SIMD drift into opposite phases;
//   * pass 2 accumulates the lane's 16 keys over all row blocks and folds the 32 lanes of a
//     half once per step (reduce-scatter over lane bits 4..1, then one pair add): the wave
//     writes complete column sums of its 64 keys;
//   * pass 1 keeps (reference, sum) per (wave, row) in LDS.  The sum is taken against the
//     reference that is already there; only when a block overflows that reference (any partial
//     sum not below 2^100, which includes the very first block, whose reference is "nothing seen
//     yet") the block is redone with the usual online maximum step.  The eight waves' pairs are
//     merged once at the end of the chunk.
//
// No atomics: results are bit-reproducible.  The masked tail of every sequence and the
// geometries this kernel is not built for stay with the tile-streaming kernel.
#include <cstdlib>
#include <cstring>
#include <type_traits>

#include "score_common.h"

namespace speckv {
namespace {

constexpr int kQsWaves = 8;     // two waves per SIMD: one in its matrix phase while the other does vector work
constexpr int kQsKB = 2;        // 32-key blocks per wave and step
constexpr int kQsMinBlocks = 8; // fewer row blocks per workgroup: the tile-streaming kernel is used
constexpr float kQsOverflow = 1.2676506e30f;   // 2^100: a block sum this large redoes its block

template <int D>
constexpr size_t qs_lds_bytes(int nb2, int pass) {
  return (size_t)nb2 * 32 * D * 2 + (pass == 1 ? (size_t)kQsWaves * nb2 * 32 * sizeof(float2)
                                               : (size_t)nb2 * 32 * sizeof(float));
}

// Sum (or max) of v[0..15] over the 32 lanes of each half.  Returns, in lane l, the result for
// register index (l % 32) / 2; lanes l and l ^ 1 hold the same value.
template <bool IS_MAX>
__device__ __forceinline__ float fold32(const float (&v)[16], int l32) {
  float w8[8], w4[4], w2[2];
  {
    const bool low = (l32 & 16) == 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float recv = __shfl_xor(low ? v[8 + j] : v[j], 16, 64);
      const float own = low ? v[j] : v[8 + j];
      w8[j] = IS_MAX ? fmaxf(own, recv) : own + recv;
    }
  }
  {
    const bool low = (l32 & 8) == 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float recv = __shfl_xor(low ? w8[4 + j] : w8[j], 8, 64);
      const float own = low ? w8[j] : w8[4 + j];
      w4[j] = IS_MAX ? fmaxf(own, recv) : own + recv;
    }
  }
  {
    const bool low = (l32 & 4) == 0;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const float recv = __shfl_xor(low ? w4[2 + j] : w4[j], 4, 64);
      const float own = low ? w4[j] : w4[2 + j];
      w2[j] = IS_MAX ? fmaxf(own, recv) : own + recv;
    }
  }
  const bool low = (l32 & 2) == 0;
  const float recv = __shfl_xor(low ? w2[1] : w2[0], 2, 64);
  const float own = low ? w2[0] : w2[1];
  const float w1 = IS_MAX ? fmaxf(own, recv) : own + recv;
  const float other = __shfl_xor(w1, 1, 64);
  return IS_MAX ? fmaxf(w1, other) : w1 + other;
}

//   PASS  1: row statistics, 2: column reduction
//   RED   (pass 2) 0: sum over the rows of a head, 1: max over the rows of a head
template <int DT, int D, int PASS, int RED>
__global__ __launch_bounds__(kQsWaves * 64) void score_qs_kernel(ScoreArgs A) {
  constexpr int NW = kQsWaves, KB = kQsKB, STEP = KB * 32;
  using TL = Tile<2, D>;
  constexpr int ROWB = TL::ROWB, NCS = TL::NCS, C16 = TL::C16;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  const Dims &d = A.d;
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);

  // (layer, head, chunk, row super-block) of this workgroup: the RS super-blocks that sweep the
  // same keys get linear ids 8 apart, i.e. the same XCD and its L2 (see score_sweep.h)
  const int per_group = 8 * A.g.RS;
  const int grp = blockIdx.x / per_group, within = blockIdx.x % per_group;
  const int item = grp * 8 + (within & 7);
  if (item >= A.g.n_fast_chunks * d.L * d.Hkv) return;
  const int chunk = item % A.g.n_fast_chunks;
  const int unit = (item / A.g.n_fast_chunks) * A.g.RS + (within >> 3);
  int s = 0;
  while (s + 1 < d.S && A.t.cc[s + 1] <= chunk) ++s;
  const int n_host = A.t.cu[s + 1] - A.t.cu[s];          // row stride of the score layouts
  const int n_live = live_len(d, A.t, s);                 // tokens that exist (device-side count honoured)
  const int key_begin = (chunk - A.t.cc[s]) * A.g.KC;
  const int key_end = min(live_tail0(d, A.t, s, n_live, TL::KT), key_begin + A.g.KC);
  const int rs = unit % A.g.RS;
  const int g = (unit / A.g.RS) % d.Hkv;
  const int layer = unit / (A.g.RS * d.Hkv);
  const int RSB = A.g.RSB;
  const float c2 = d.sm_scale * 1.4426950408889634f;

  // row blocks that hold rows, rounded up to an even count (the loop below is unrolled by two);
  // the rows of the padding block are zero and contribute nothing
  int nblk;
  if (A.g.PPH == 1) nblk = min(A.g.HPS, d.G - rs * A.g.HPS) * (A.g.Rp / 32);
  else nblk = (min(RSB, d.R - (rs % A.g.PPH) * RSB) + 31) / 32;
  const int nb2 = __builtin_amdgcn_readfirstlane((nblk + 1) & ~1);
  const int nrows = nb2 * 32;

  unsigned char *qlds = smem;
  float *nl_lds = reinterpret_cast<float *>(smem + (size_t)nrows * ROWB);          // pass 2
  float2 *st_lds = reinterpret_cast<float2 *>(smem + (size_t)nrows * ROWB);        // pass 1: [NW][nb2][32]

  // ---- stationary operand: the group's query rows, 16-byte chunk c of row r at slot c ^ swizzle(r)
  for (int x = tid; x < nrows * C16; x += NW * 64) {
    const int row = x / C16, c = x % C16;
    int hh, i;
    u32x4 v = (u32x4)(0u);
    if (decode_row(d, A.g, rs, row, &hh, &i)) {
      const char *qp = A.q + ((int64_t)layer * d.q_sl + (int64_t)s * d.q_ss + (int64_t)i * d.q_sr +
                              (int64_t)(g * d.G + hh) * d.q_sh) * 2 + c * 16;
      v = *reinterpret_cast<const u32x4 *>(qp);
    }
    *reinterpret_cast<u32x4 *>(qlds + row * ROWB + ((c ^ TL::swizzle(row)) * 16)) = v;
  }
  if (PASS == 2) {
    const float *lp = A.lse + (((int64_t)layer * d.Hkv + g) * d.S + s) * ((int64_t)A.g.RS * RSB) + rs * RSB;
    for (int row = tid; row < nrows; row += NW * 64) {
      int hh, i;
      float v = -INFINITY;                                 // padding rows contribute 2^-inf = 0
      if (decode_row(d, A.g, rs, row, &hh, &i)) {
        v = -lp[row];
        if (d.weight_rows && i < d.w) v += log2f((float)(i + 1) / (float)d.w);   // row weight folded in
      }
      nl_lds[row] = v;
    }
  } else {
    for (int x = tid; x < NW * nb2 * 32; x += NW * 64) st_lds[x] = make_float2(kNegBig, 0.f);
  }
  __syncthreads();

  // ---- this wave's keys: steps wv, wv + NW, ... of STEP keys each
  const int nsteps = max(0, key_end - key_begin) / STEP;    // chunks are whole LDS tiles of >= 128 keys
  const char *kbase = A.k + ((int64_t)layer * d.kv_sl + (int64_t)A.t.cu[s] * d.kv_st + (int64_t)g * d.kv_sh) * 2;
  const int64_t tokb = d.kv_st * 2;
  uint32_t kofs[KB];                                        // the lane's byte offset inside a step
#pragma unroll
  for (int kb = 0; kb < KB; ++kb) kofs[kb] = (uint32_t)(kb * 32 + l32) * (uint32_t)tokb + (uint32_t)(half * NCS * 16);
  uint32_t foff[NCS];                                       // the lane's fragment chunks of row l32 of a block
#pragma unroll
  for (int cs = 0; cs < NCS; ++cs) foff[cs] = l32 * ROWB + (((half * NCS + cs) ^ TL::swizzle(l32)) * 16);
  float2 *st_mine = st_lds + ((size_t)wv * nb2) * 32 + l32;   // both lane halves share a row's pair

  float *plane_out = nullptr;
  if (PASS == 2)
    plane_out = A.planes + ((int64_t)rs * d.L + layer) * d.Hkv * d.T + (int64_t)d.Hkv * A.t.cu[s] + (int64_t)g * n_host;
  const int blocks_per_head = (A.g.PPH == 1 ? A.g.Rp : RSB) / 32;
  const bool head_max = d.head_max != 0;

  u32x4 kf[KB][NCS];                     // key fragments of the current step
  u32x4 qe[NCS], qo[NCS];                // Q fragments of an even / odd row block
  f32x16 acc[KB];                        // scores of one row block
  float se_x = 0.f, se_y = 0.f, so_x = 0.f, so_y = 0.f;   // pass 1: (reference, sum); pass 2: .x = -lse2
  float colacc[KB][16];                  // pass 2: per key, over the row blocks (of a head when RED)
  float total[KB];                       // pass 2, RED: folded heads so far
#pragma unroll
  for (int kb = 0; kb < KB; ++kb) {
    total[kb] = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) colacc[kb][i] = 0.f;
  }

  auto load_k = [&](int step) __attribute__((always_inline)) {
    const char *base = kbase + (int64_t)(key_begin + step * STEP) * tokb;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int cs = 0; cs < NCS; ++cs)
        kf[kb][cs] = *reinterpret_cast<const u32x4 *>(base + kofs[kb] + cs * 16);
  };
  auto load_q = [&](u32x4(&dst)[NCS], int rb) __attribute__((always_inline)) {
#pragma unroll
    for (int cs = 0; cs < NCS; ++cs)
      dst[cs] = *reinterpret_cast<const u32x4 *>(qlds + rb * (32 * ROWB) + foff[cs]);
  };
  auto load_state = [&](float &x, float &y, int rb) __attribute__((always_inline)) {
    if (PASS == 2) {
      x = nl_lds[rb * 32 + l32];
    } else {
      const float2 v = st_mine[rb * 32];
      x = v.x; y = v.y;
    }
  };
  auto mma = [&](const u32x4(&qf)[NCS]) __attribute__((always_inline)) {
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) acc[kb] = (f32x16){0};
#pragma unroll
    for (int cs = 0; cs < NCS; ++cs)
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) acc[kb] = mma_chunk<DT>(kf[kb][cs], qf[cs], acc[kb]);
  };
  // turns the scores of row block rb into probabilities; sx, sy: the block's state (see above)
  auto soft = [&](float sx, float sy, int rb) __attribute__((always_inline)) {
    if (PASS == 1) {
      const float nref = -sx;
      float sum = 0.f;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {                    // per key block: multiply-adds, exp2, a tree of adds
        float x[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = fmaf(acc[kb][i], c2, nref);
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = __builtin_amdgcn_exp2f(x[i]);
        sum += (((x[0] + x[1]) + (x[2] + x[3])) + ((x[4] + x[5]) + (x[6] + x[7]))) +
               (((x[8] + x[9]) + (x[10] + x[11])) + ((x[12] + x[13]) + (x[14] + x[15])));
      }
      sum = add_other_half(sum);                           // the row's keys of both lane halves
      float ref = sx, l = sy + sum;
      if (__builtin_amdgcn_ballot_w64(!(sum < kQsOverflow)) != 0) {
        // some row's reference is too low for this block (or it has none yet): online maximum step
        float tmax = acc[0][0];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, acc[kb][i]);
        const float mnew = fmaxf(sx, max_other_half(tmax) * c2);
        const float nm = -mnew;
        float sum2 = 0.f;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) sum2 += __builtin_amdgcn_exp2f(fmaf(acc[kb][i], c2, nm));
        l = fmaf(sy, __builtin_amdgcn_exp2f(sx - mnew), add_other_half(sum2));
        ref = mnew;
      }
      st_mine[rb * 32] = make_float2(ref, l);              // both halves write the same pair
    } else {
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = __builtin_amdgcn_exp2f(fmaf(acc[kb][i], c2, sx));
          colacc[kb][i] = RED == 0 ? colacc[kb][i] + p : fmaxf(colacc[kb][i], p);
        }
      if (RED == 1 && ((rb + 1) % blocks_per_head == 0 || rb + 1 == nb2)) {
        // the head is complete: its per-key maximum joins the other heads' (sum, or max for Alg. 2)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
          const float hm = fold32<true>(colacc[kb], l32);
          total[kb] = head_max ? fmaxf(total[kb], hm) : total[kb] + hm;
#pragma unroll
          for (int i = 0; i < 16; ++i) colacc[kb][i] = 0.f;
        }
      }
    }
  };
  // complete column values of the step's keys (pass 2)
  auto store_step = [&](int step) __attribute__((always_inline)) {
    const int i = l32 >> 1;                                  // register index the fold leaves in this lane
    const int key0 = key_begin + step * STEP + 8 * (i >> 2) + 4 * half + (i & 3);
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
      float v;
      if (RED == 0) {
        v = fold32<false>(colacc[kb], l32);
#pragma unroll
        for (int j = 0; j < 16; ++j) colacc[kb][j] = 0.f;
      } else {
        v = total[kb];
        total[kb] = 0.f;
      }
      if ((l32 & 1) == 0) plane_out[key0 + kb * 32] = v;
    }
  };

  // A wave alternates between a matrix phase (the block's 8*KB MFMAs) and a vector phase (its
  // softmax arithmetic); the second wave on the SIMD runs the other phase meanwhile.  Q fragments
  // and block states are fetched from LDS one row block ahead; the keys of the following step are
  // requested as soon as the last MFMAs of this one are issued.
  if (wv < nsteps) {
    load_k(wv);
    load_q(qe, 0);
    load_state(se_x, se_y, 0);
    for (int step = wv; step < nsteps; step += NW) {
      for (int rb = 0; rb < nb2; rb += 2) {
        load_q(qo, rb + 1);
        load_state(so_x, so_y, rb + 1);
        mma(qe);
        soft(se_x, se_y, rb);
        const int nxt = rb + 2 < nb2 ? rb + 2 : 0;
        load_q(qe, nxt);
        mma(qo);
        if (rb + 2 >= nb2 && step + NW < nsteps) load_k(step + NW);
        load_state(se_x, se_y, nxt);       // after block rb's state was written (nb2 may be 2)
        soft(so_x, so_y, rb + 1);
      }
      if (PASS == 2) store_step(step);
    }
  }

  if (PASS == 1) {
    // merge the waves' and lane halves' (reference, sum) pairs of every row: one pair per chunk
    __syncthreads();
    float2 *pp = A.part + ((int64_t)unit * A.g.n_chunks + chunk) * RSB;
    for (int row = tid; row < RSB; row += NW * 64) {
      float mm = kNegBig, ll = 0.f;
      if (row < nrows) {
        const int rb = row >> 5, r32 = row & 31;
#pragma unroll
        for (int x = 0; x < NW; ++x) {
          const float2 v = st_lds[((size_t)x * nb2 + rb) * 32 + r32];
          const float m2 = fmaxf(mm, v.x);
          ll = ll * __builtin_amdgcn_exp2f(mm - m2) + v.y * __builtin_amdgcn_exp2f(v.x - m2);
          mm = m2;
        }
      }
      pp[row] = make_float2(mm, ll);
    }
  }
}

template <int DT, int D>
hipError_t qs_launch(const ScoreArgs &A, int pass, size_t lds, dim3 grid, hipStream_t st) {
  const dim3 block(kQsWaves * 64);
  auto go = [&](auto kernel) {
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kernel, grid, block, lds, st, A);
    return hipGetLastError();
  };
  if (pass == 1) return go(score_qs_kernel<DT, D, 1, 0>);
  return A.d.reduce_max ? go(score_qs_kernel<DT, D, 2, 1>) : go(score_qs_kernel<DT, D, 2, 0>);
}

// largest number of row blocks (rounded up to even) any workgroup of the launch holds
int qs_max_blocks(const ScoreArgs &A) {
  int nblk;
  if (A.g.PPH == 1) nblk = A.g.HPS * (A.g.Rp / 32);
  else nblk = (std::min(A.g.RSB, (int)A.d.R) + 31) / 32;
  return (nblk + 1) & ~1;
}

}  // namespace

bool qs_supported(const ScoreArgs &A, int pass) {
  // Default: only the row-statistics sweep at d = 64, where the vector pipe is the limit and this
  // kernel's reference-exponent step (no maximum search) measures 12 % faster than the online step
  // of the tile-streaming kernel.  Everywhere else the two dataflows end at the same matrix-pipe
  // utilisation and the tile-streaming kernel is equal or slightly ahead.  The environment can
  // override the choice: SPECKV_SCORE_KERNEL=tile (never), qs (both sweeps), qs1 / qs2 (that sweep
  // only).  Read on every call so that a test can switch it.
  const char *e = std::getenv("SPECKV_SCORE_KERNEL");
  bool want = pass == 1 && A.d.D == 64;
  if (e != nullptr && e[0] != '\0') {
    if (std::strcmp(e, "tile") == 0) want = false;
    else if (std::strcmp(e, "qs") == 0) want = true;
    else if (std::strcmp(e, "qs1") == 0) want = pass == 1;
    else if (std::strcmp(e, "qs2") == 0) want = pass == 2;
  }
  if (!want) return false;
  if (A.d.dt == SPECKV_F32 || A.g.n_fast_chunks <= 0) return false;
  const int nb2 = qs_max_blocks(A);
  if (nb2 < kQsMinBlocks || nb2 * 32 > A.g.RSB) return false;
  const size_t lds = A.d.D == 128 ? qs_lds_bytes<128>(nb2, 1) : qs_lds_bytes<64>(nb2, 1);
  return lds <= (size_t)160 * 1024;
}

hipError_t launch_qs_sweep(const ScoreArgs &A, int pass, hipStream_t st) {
  const int nb2 = qs_max_blocks(A);
  const int64_t items = (int64_t)A.g.n_fast_chunks * A.d.L * A.d.Hkv;
  const int64_t wgs = (items + 7) / 8 * 8 * A.g.RS;
  if (wgs > 0x7fffffffLL) return hipErrorInvalidValue;
  const dim3 grid((unsigned)wgs);
  const bool d128 = A.d.D == 128;
  const size_t lds = d128 ? qs_lds_bytes<128>(nb2, pass) : qs_lds_bytes<64>(nb2, pass);
  if (A.d.dt == SPECKV_BF16)
    return d128 ? qs_launch<kBf16, 128>(A, pass, lds, grid, st) : qs_launch<kBf16, 64>(A, pass, lds, grid, st);
  return d128 ? qs_launch<kF16, 128>(A, pass, lds, grid, st) : qs_launch<kF16, 64>(A, pass, lds, grid, st);
}

}  // namespace speckv
