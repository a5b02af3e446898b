// Importance scoring on the gfx950 matrix cores (Sec. 3.1 Eq. 1; Alg. 1 CrossAttention and
// reduce steps; App. C.2 for the GQA group).
//
// For one (layer, sequence, KV head) the logits are S = Qg . K^T with Qg the M = G*R stacked
// observation rows of the G query heads that share the KV head (row r = head_in_group*R + i)
// and K the n_in prompt keys of that head.  The importance of key j is the column sum of the
// row softmax of sm_scale*S.  A column sum needs every row's normaliser first, so S is
// computed twice and never stored:
//
//   pass 1  row statistics: per row a pair (reference exponent, sum of 2^(c*S - reference)) over
//           the keys of one chunk, the reference either the running maximum or fixed per chunk
//           (see score_body); a small kernel merges the chunks into
//           lse2[row] = log2 sum_j 2^(c*S[row,j]), c = sm_scale*log2(e).
//   pass 2  column sums: raw[j] = sum_rows 2^(c*S[row,j] - lse2[row]).
//
// Work split: a workgroup owns RSB = NW*MB*32 rows (all of them when M <= RSB) and one chunk of
// keys.  Each wave keeps the MFMA fragments of its MB 32-row blocks of Q in registers for the
// whole sweep; K tiles of KT keys stream HBM -> LDS directly (global_load_lds, double buffered,
// no staging registers).  The LDS tile is unpadded; the 16-byte chunks of a row are stored at
// slot = chunk ^ swizzle(row) so that the 128-bit fragment reads of 16 consecutive keys hit 16
// different bank groups.  Every wave reads all K fragments of a tile.
// Pass 1 multiplies with K as the A operand, so a lane holds 16 keys of ONE query row and the
// row statistics stay in two registers per row block; pass 2 multiplies with Q as the A operand,
// so a lane holds 16 rows of ONE key and the column sum is an in-lane add, one cross-half add and
// a cross-wave add through LDS.  No atomics anywhere: results are bit-reproducible.
//
// MFMA operand layout used (v_mfma_f32_32x32x16_bf16, v_mfma_f32_32x32x16_f16, v_mfma_f32_32x32x2_f32): lane l holds
// row (A) or column (B) l%32 and the k-slice selected by l/32; the result register i of lane l
// is element (8*(i/4) + 4*(l/32) + i%4, l%32).  Both operands take their k-slices from the same
// 16-byte chunks of the head dimension (half l/32 reads chunks [half*NCS, half*NCS+NCS)), so the
// contraction is over all d channels whatever order the hardware assigns inside a slice.
//
// This header holds the sweep kernels and their launcher.  It is compiled into two translation
// units, one per sweep (score_rows.hip, score_cols.hip), because the two want different
// instruction scheduling strategies from the compiler (see build.py).
#pragma once
#include <type_traits>
#include <utility>

#include "score_common.h"

namespace speckv {
namespace {


template <int ELT, int D, int MB, int NW>
constexpr size_t score_lds_bytes() {
  using TL = Tile<ELT, D>;
  return (size_t)2 * TL::TILE_BYTES + (size_t)2 * NW * MB * TL::KT * sizeof(float);
}

// One workgroup's sweep over a chunk of keys; bid = its index among the workgroups of its kind.
//   PASS    1: row statistics, 2: column reduction
//   RED     (pass 2) 0: sum over the rows of a head, 1: max over the rows of a head;
//           (pass 1) 0: online step on every key block, 1: fixed reference exponents with a
//           repair launch behind the sweep (see below; for sweeps of several rounds of workgroups)
//   MASKED  false: every tile of the chunk is complete and visible to every row (key <= m), the
//           loop body is straight-line code without any bounds or mask logic;
//           true: the tail of a sequence (keys that window rows may not see, end of sequence)
//   REPAIR  (pass 1, unmasked) false: the whole chunk against fixed references; every wavefront
//           leaves the segments (kAnchorTiles tiles) in which one of its sums overflowed out of
//           its pairs and lists them in A.fail;  true: segment `seg` alone with the online step,
//           its pairs merged into the ones already written; wavefronts that do not take part
//           (the segment is not on their list) only help to load the key tiles
template <int DT, int D, int MB, int NW, int PASS, int RED, bool MASKED, bool REPAIR = false>
__device__ __forceinline__ void score_body(const ScoreArgs &A, const int bid, const int seg = 0,
                                           const bool wave_takes_part = true) {
  static_assert(!REPAIR || (PASS == 1 && !MASKED), "only the row-statistics sweep is repaired");
  constexpr int ELT = elt_bytes(DT);
  using TL = Tile<ELT, D>;
  constexpr int ROWB = TL::ROWB, NCS = TL::NCS, KT = TL::KT, TILE_BYTES = TL::TILE_BYTES;
  constexpr int RSB = NW * MB * 32;
  constexpr int SEG_PER_WAVE = TILE_BYTES / 1024 / NW;   // 1 KiB (one wave-wide 128-bit load) segments
  constexpr int RPS = 1024 / ROWB;                        // tile rows per segment
  static_assert(TILE_BYTES % (1024 * NW) == 0, "tile load must divide evenly over the waves");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  unsigned char *kbuf = smem;
  float *csum = reinterpret_cast<float *>(smem + 2 * TILE_BYTES);

  const Dims &d = A.d;
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  int unit, s, chunk, key_begin, key_end;
  if (MASKED) {
    const int units = d.L * d.Hkv * A.g.RS;
    unit = bid % units;
    s = bid / units;
    chunk = A.g.n_fast_chunks + s;
  } else {
    // 1-D grid.  Workgroups go to the 8 XCDs round-robin by their linear id and each XCD has its
    // own L2, so the RS row super-blocks that sweep the SAME keys of a (layer, head) get ids 8
    // apart: same XCD, dispatched together, and the keys come from HBM once instead of RS times.
    const int per_group = 8 * A.g.RS;
    const int grp = bid / per_group, within = bid % per_group;
    const int item = grp * 8 + (within & 7);            // (layer, head, chunk), chunk fastest
    if (item >= A.g.n_fast_chunks * d.L * d.Hkv) return;
    chunk = item % A.g.n_fast_chunks;
    unit = (item / A.g.n_fast_chunks) * A.g.RS + (within >> 3);
    s = 0;
    while (s + 1 < d.S && A.t.cc[s + 1] <= chunk) ++s;
  }
  const int n_host = A.t.cu[s + 1] - A.t.cu[s];          // row stride of the score layouts
  const int n_s = live_len(d, A.t, s);                    // tokens that exist (device-side count honoured)
  const int tail0 = live_tail0(d, A.t, s, n_s, KT);
  if (MASKED) {
    key_begin = tail0;
    key_end = n_s;
  } else {
    key_begin = (chunk - A.t.cc[s]) * A.g.KC;
    key_end = min(tail0, key_begin + A.g.KC);             // a chunk past a shorter live prompt is empty
  }
  const int rs = unit % A.g.RS;
  const int g = (unit / A.g.RS) % d.Hkv;
  const int layer = unit / (A.g.RS * d.Hkv);
  const int m = n_s - d.w;
  const int ntiles = (key_end - key_begin + KT - 1) / KT;
  const float c2 = d.sm_scale * 1.4426950408889634f;

  // 32-row block b of the super-block belongs to wave b % NW (its row block b / NW), so that a
  // partly filled super-block still spreads its blocks evenly over the SIMDs.  Blocks past the
  // last valid row are skipped: nact = how many of this wave's MB blocks hold rows.
  int nblk;
  if (A.g.PPH == 1) nblk = min(A.g.HPS, d.G - rs * A.g.HPS) * (A.g.Rp / 32);
  else nblk = (min(RSB, d.R - (rs % A.g.PPH) * RSB) + 31) / 32;
  const int nact = wave_takes_part ? __builtin_amdgcn_readfirstlane(max(0, min(MB, (nblk - wv + NW - 1) / NW))) : 0;
  // Maximum over the query rows, full super-block, an even number of blocks per head: the wave
  // takes two neighbouring blocks (2 wv and 2 wv + 1, the same head) instead, merges their
  // column maxima in registers and hands one value per key to the flush, not two.  A maximum
  // does not depend on the order, so the result is the same bit for bit.
  const int blocks_per_head = (A.g.PPH == 1 ? A.g.Rp : RSB) / 32;
  const bool paired = PASS == 2 && RED == 1 && !MASKED && MB == 2 && nblk == NW * MB && blocks_per_head % 2 == 0;
  auto block_of = [&](int rb) { return paired ? wv * MB + rb : rb * NW + wv; };
  if (PASS == 2)   // slots of skipped blocks must read as zero when the tile partials are merged
    for (int x = tid; x < 2 * NW * MB * KT; x += NW * 64) csum[x] = 0.f;

  // head and first observation row of each of this wave's 32-row blocks (a block never mixes
  // heads, so one division per block replaces one per row)
  int blk_head[MB], blk_i0[MB];
#pragma unroll
  for (int rb = 0; rb < MB; ++rb) {
    int hh, i0;
    const bool ok = decode_row(d, A.g, rs, block_of(rb) * 32, &hh, &i0);
    blk_head[rb] = ok ? hh : -1;       // -1: the whole block is padding
    blk_i0[rb] = i0;
  }
#define SPECKV_ROW_VALID(rb_, r32_) (blk_head[rb_] >= 0 && blk_i0[rb_] + (r32_) < d.R)

  // ---- K tile staging: each wave issues SEG_PER_WAVE wave-wide 128-bit loads that land in LDS
  // at lds_base + lane*16; the lane picks the global chunk that belongs in its (row, slot).
  const char *kbase = A.k + ((int64_t)layer * d.kv_sl + (int64_t)A.t.cu[s] * d.kv_st + (int64_t)g * d.kv_sh) * ELT;
  const int64_t tokb = d.kv_st * ELT;
  const int st_row = (lane * 16) / ROWB, st_slot = ((lane * 16) % ROWB) / 16;
  // unmasked sweep: the lane's byte offset inside a tile never changes, only the (uniform) tile
  // base moves, so the loads use a scalar base plus a 32-bit lane offset
  uint32_t loff[SEG_PER_WAVE];
#pragma unroll
  for (int it = 0; it < SEG_PER_WAVE; ++it) {
    const int r_ = (it * NW + wv) * RPS + st_row;
    loff[it] = (uint32_t)r_ * (uint32_t)tokb + (uint32_t)((st_slot ^ TL::swizzle(r_)) * 16);
  }
#define SPECKV_LOAD_TILE(tile_, buf_)                                                         \
  {                                                                                           \
    const int k0_ = key_begin + (tile_) * KT;                                                 \
    const char *tbase_ = kbase + (int64_t)k0_ * tokb;                                         \
    _Pragma("unroll") for (int it = 0; it < SEG_PER_WAVE; ++it) {                             \
      const int seg_ = it * NW + wv;                                                          \
      const char *src_;                                                                       \
      if (MASKED) {                                                                           \
        const int r_ = seg_ * RPS + st_row;                                                   \
        /* rows past the end of the sequence re-read its last key; they are masked later */   \
        src_ = kbase + (int64_t)min(k0_ + r_, n_s - 1) * tokb + (st_slot ^ TL::swizzle(r_)) * 16; \
      } else {                                                                                \
        src_ = tbase_ + loff[it];                                                             \
      }                                                                                       \
      __builtin_amdgcn_global_load_lds(                                                       \
          (const __attribute__((address_space(1))) void *)src_,                               \
          (__attribute__((address_space(3))) void *)(kbuf + (buf_) * TILE_BYTES + seg_ * 1024), 16, 0, 0); \
    }                                                                                         \
  }
  // the first tile is requested before anything else is loaded, so that its latency overlaps
  // with the Q fragment and row normaliser loads below
  const int first_tile = REPAIR ? seg * kAnchorTiles : 0;
  if (ntiles > first_tile) SPECKV_LOAD_TILE(first_tile, 0)

  // ---- Q fragments of this wave's row blocks, resident for the whole sweep
  u32x4 qf[MB][NCS];
#pragma unroll
  for (int rb = 0; rb < MB; ++rb) {
    const bool valid = SPECKV_ROW_VALID(rb, l32);
    const int hh = blk_head[rb], i = blk_i0[rb] + l32;
    const char *qp = A.q + ((int64_t)layer * d.q_sl + (int64_t)s * d.q_ss + (int64_t)(valid ? i : 0) * d.q_sr +
                            (int64_t)(g * d.G + (valid ? hh : 0)) * d.q_sh) * ELT + (half * NCS) * 16;
#pragma unroll
    for (int cs = 0; cs < NCS; ++cs)
      qf[rb][cs] = valid ? *reinterpret_cast<const u32x4 *>(qp + cs * 16) : (u32x4)(0u);
  }

  // ---- per-pass row state
  float mrun[MB], lrun[MB];          // pass 1: lane = one query row per row block
  float nlse[MB][16];                // pass 2: lane = 16 rows per row block
  if (PASS == 1) {
#pragma unroll
    for (int rb = 0; rb < MB; ++rb) { mrun[rb] = kNegBig; lrun[rb] = 0.f; }
  } else {
    const float *lp = A.lse + (((int64_t)layer * d.Hkv + g) * d.S + s) * ((int64_t)A.g.RS * RSB);
#pragma unroll
    for (int rb = 0; rb < MB; ++rb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int r32 = 8 * (i >> 2) + 4 * half + (i & 3);
        const int lr = block_of(rb) * 32 + r32;
        const bool valid = SPECKV_ROW_VALID(rb, r32);
        const int io = blk_i0[rb] + r32;
        float v = -lp[rs * RSB + lr];                       // the lse buffer covers the padded rows
        if (d.weight_rows && io < d.w) v += log2f((float)(io + 1) / (float)d.w);   // row weight folded in
        nlse[rb][i] = valid ? v : -INFINITY;                // padded rows contribute 2^-inf = 0
      }
  }

  // ---- masked sweep: last key each row may see (window row i sees keys <= m + i, a lookahead
  // row the whole prompt), computed once instead of per score
  int last1[MB];                     // pass 1: the lane's own query row per row block
  int last2[MB][16];                 // pass 2: the 16 rows a lane holds per row block
  if (MASKED) {
#pragma unroll
    for (int rb = 0; rb < MB; ++rb) {
      if (PASS == 1) {
        const int io = blk_i0[rb] + l32;
        last1[rb] = io < d.w ? m + io : n_s - 1;
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int io = blk_i0[rb] + 8 * (i >> 2) + 4 * half + (i & 3);
          last2[rb][i] = io < d.w ? m + io : n_s - 1;
        }
      }
    }
  }

  // per-lane LDS offsets of the fragment chunks of key row l32 (same for every 32-key block)
  uint32_t foff[NCS];
#pragma unroll
  for (int cs = 0; cs < NCS; ++cs) foff[cs] = l32 * ROWB + (((half * NCS + cs) ^ TL::swizzle(l32)) * 16);
#define SPECKV_LOAD_BFRAG(dst_, buf_, kb_)                                                     \
  _Pragma("unroll") for (int cs = 0; cs < NCS; ++cs)                                          \
    dst_[cs] = *reinterpret_cast<const u32x4 *>(kbuf + (buf_) * TILE_BYTES + (kb_) * 32 * ROWB + foff[cs]);

  // cross-wave merge of the column partials of one finished tile (pass 2)
  float *plane_out = nullptr;
  if (PASS == 2)
    plane_out = A.planes + ((int64_t)rs * d.L + layer) * d.Hkv * d.T + (int64_t)d.Hkv * A.t.cu[s] + (int64_t)g * n_host;
  const bool head_max = d.head_max != 0;
  const int slots_per_head = paired ? blocks_per_head / 2 : blocks_per_head;
#define SPECKV_FLUSH_TILE(tile_)                                                             \
  if (tid < KT) {                                                                            \
    const int key_ = key_begin + (tile_) * KT + tid;                                         \
    if (key_ < key_end) {                                                                    \
      const float *cp_ = csum + (size_t)((tile_) & 1) * NW * MB * KT + tid;                  \
      float total_ = 0.f;                                                                    \
      if (RED == 0) {                                                                        \
        _Pragma("unroll") for (int w2 = 0; w2 < NW; ++w2) total_ += cp_[w2 * KT];            \
      } else {                                                                               \
        /* per block (or block pair) maxima: max within a head, then heads added (or maxed) */ \
        float cur_ = 0.f;                                                                    \
        int in_head_ = 0;                                                                    \
        _Pragma("unroll") for (int b2 = 0; b2 < NW * MB; ++b2) {                             \
          if (paired && b2 >= NW) break;                                                     \
          if (in_head_ == slots_per_head) {                                                  \
            total_ = head_max ? fmaxf(total_, cur_) : total_ + cur_;                         \
            cur_ = 0.f;                                                                      \
            in_head_ = 0;                                                                    \
          }                                                                                  \
          cur_ = fmaxf(cur_, cp_[b2 * KT]);                                                  \
          ++in_head_;                                                                        \
        }                                                                                    \
        total_ = head_max ? fmaxf(total_, cur_) : total_ + cur_;                             \
      }                                                                                      \
      plane_out[key_] = total_;                                                              \
    }                                                                                        \
  }

  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  // Row statistics of an unmasked chunk.  The chunk's first 32-key block gives each row its reference
  // exponent (the block's maximum, found by the online step); every later block only adds
  // 2^(score - reference) to the row's sum: no maximum search, no rescaling.  After every segment the
  // sum's own exponent moves into the reference (a few integer and float operations, no branch),
  // which keeps the sum near 2^-shift with shift = 100 - ceil(log2(keys per chunk)): a term that
  // underflows (below 2^-126) beside it is less than 2^-25 / (keys per chunk) of the sum, so all
  // of a chunk's keys together stay below fp32 resolution, and a score may exceed everything the
  // row has seen before its segment by 126 + shift binary orders (146 nats for 32K-key chunks)
  // before the sum overflows.  An overflow is sticky (infinity stays infinity), so it is looked for
  // once per segment of kAnchorTiles tiles (kAnchorLimit; also NaN): the wavefront then goes back
  // to the pairs it had before the segment, notes the segment on its list in A.fail and goes on;
  // the repair launch behind this one (REPAIR) sweeps the noted segments with the online step on
  // every block and adds their pairs.  (The same second sweep as code inside this kernel, inlined,
  // outlined or as a compact loop, costs the first sweep the 3 % it is there to gain.)
  const int anchor_shift = 100 - (32 - __builtin_clz((unsigned)max(A.g.KC, 2) - 1u));
  int fresh_tile = 0;                // the tile whose first block finds the reference (no pair yet)

  // one tile of the sweep; the LDS buffer index is a compile-time constant so that every LDS
  // address below is a register plus an immediate
  auto do_tile = [&](int tile, auto buf_c, auto anchored_c) {
    constexpr int buf = decltype(buf_c)::value;
    if (tile + 1 < ntiles) SPECKV_LOAD_TILE(tile + 1, buf ^ 1)
    if (PASS == 2 && tile > 0) SPECKV_FLUSH_TILE(tile - 1)
    const int tk0 = key_begin + tile * KT;
    if (!MASKED) {
      // Per 32-key block the MB accumulator chains of this wave are interleaved MFMA by MFMA
      // (no back-to-back dependent MFMAs); the fragments of the next block are fetched while
      // the vector pipe turns the scores into probabilities.  The second wave on the SIMD
      // runs its MFMAs underneath that vector work.
      // NACT = number of active row blocks of this wave (compile-time copy of nact)
      // anchored: row statistics against the fixed reference (see above), else the online step
      auto fast_tile = [&](auto nact_c, auto anchored_c) {
        constexpr int NACT = decltype(nact_c)::value;
        constexpr bool anchored = decltype(anchored_c)::value;
        u32x4 bf[NCS];
        SPECKV_LOAD_BFRAG(bf, buf, 0)
#pragma unroll
        for (int kb = 0; kb < KT / 32; ++kb) {
          f32x16 acc[NACT];
#pragma unroll
          for (int rb = 0; rb < NACT; ++rb) acc[rb] = (f32x16){0};
          // pass 2: the compiler may not move vector work of the neighbouring key blocks across the
          // MFMA chains or the fragment loads (measured: the column sweep 1.5 % faster, the step 0.5 %
          // since the chip is power-limited; the same barriers cost the row-statistics sweep 5 %;
          // wave priorities (s_setprio) around the MFMAs do no more than the barrier they imply)
          if (PASS == 2) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int cs = 0; cs < NCS; ++cs)
#pragma unroll
            for (int rb = 0; rb < NACT; ++rb)
              acc[rb] = PASS == 1 ? mma_chunk<DT>(bf[cs], qf[rb][cs], acc[rb]) : mma_chunk<DT>(qf[rb][cs], bf[cs], acc[rb]);
          if (PASS == 2) __builtin_amdgcn_sched_barrier(0);
          if (kb + 1 < KT / 32) SPECKV_LOAD_BFRAG(bf, buf, kb + 1)
          if (PASS == 2) __builtin_amdgcn_sched_barrier(0);
          if (PASS == 1 && anchored && !(kb == 0 && tile == fresh_tile)) {
#pragma unroll
            for (int rb = 0; rb < NACT; ++rb) {
              const float nm = -mrun[rb];
              float sum = 0.f;
#pragma unroll
              for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(fmaf(acc[rb][i], c2, nm));
              lrun[rb] += sum;
            }
          } else if (PASS == 1) {
#pragma unroll
            for (int rb = 0; rb < NACT; ++rb) {
              // branch-free online softmax step for the lane's query row
              float tmax = fmaxf(fmaxf(acc[rb][0], acc[rb][1]), acc[rb][2]);
#pragma unroll
              for (int i = 3; i < 15; i += 2) tmax = fmaxf(fmaxf(tmax, acc[rb][i]), acc[rb][i + 1]);
              tmax = fmaxf(tmax, acc[rb][15]);
              const float mnew = fmaxf(mrun[rb], tmax * c2);
              const float scale = __builtin_amdgcn_exp2f(mrun[rb] - mnew);
              const float nm = -mnew;
              float sum = 0.f;
#pragma unroll
              for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(fmaf(acc[rb][i], c2, nm));
              lrun[rb] = fmaf(lrun[rb], scale, sum);
              mrun[rb] = mnew;
              if (anchored) {      // the chunk's first block: move the reference up for the blocks that follow
                lrun[rb] = __builtin_ldexpf(lrun[rb], -anchor_shift);
                mrun[rb] += (float)anchor_shift;
              }
            }
          } else {
            // the 16 probabilities of a row block: all multiply-adds, then all exp2, then the reduction
            // as a tree, so that no instruction waits on the one issued just before it (against
            // two batches of 8 with a serial sum: the column sweep 2.4 % faster, the step 0.8 %)
            float colsum = 0.f;
#pragma unroll
            for (int rb = 0; rb < NACT; ++rb) {
              if (RED == 1 && !(paired && rb > 0)) colsum = 0.f;
              float x[16];
#pragma unroll
              for (int i = 0; i < 16; ++i) x[i] = fmaf(acc[rb][i], c2, nlse[rb][i]);
#pragma unroll
              for (int i = 0; i < 16; ++i) x[i] = __builtin_amdgcn_exp2f(x[i]);
              __builtin_amdgcn_sched_barrier(0);
              if (RED == 0) {
                colsum += (((x[0] + x[1]) + (x[2] + x[3])) + ((x[4] + x[5]) + (x[6] + x[7]))) +
                          (((x[8] + x[9]) + (x[10] + x[11])) + ((x[12] + x[13]) + (x[14] + x[15])));
              } else {
                const float t0 = fmaxf(fmaxf(x[0], x[1]), x[2]), t1 = fmaxf(fmaxf(x[3], x[4]), x[5]);
                const float t2 = fmaxf(fmaxf(x[6], x[7]), x[8]), t3 = fmaxf(fmaxf(x[9], x[10]), x[11]);
                const float t4 = fmaxf(fmaxf(x[12], x[13]), x[14]);
                colsum = fmaxf(fmaxf(colsum, fmaxf(fmaxf(t0, t1), t2)), fmaxf(fmaxf(t3, t4), x[15]));
              }
              __builtin_amdgcn_sched_barrier(0);
              if (RED == 1 && !paired) {   // one value per 32-row block: blocks of a head are merged at the flush
                colsum = max_other_half(colsum);
                if (half == 0) csum[(size_t)buf * NW * MB * KT + (rb * NW + wv) * KT + kb * 32 + l32] = colsum;
              }
            }
            if (RED == 0) {
              colsum = add_other_half(colsum);
              if (half == 0) csum[(size_t)buf * NW * MB * KT + wv * KT + kb * 32 + l32] = colsum;
            } else if (paired) {       // the maximum over both blocks of the pair, slot wv
              colsum = max_other_half(colsum);
              if (half == 0) csum[(size_t)buf * NW * MB * KT + wv * KT + kb * 32 + l32] = colsum;
            }
          }
        }
      };
      if (nact == MB) fast_tile(std::integral_constant<int, MB>{}, anchored_c);
      else if (MB > 1 && nact == 1) fast_tile(std::integral_constant<int, 1>{}, anchored_c);
    } else {
      // Tail tiles: keys above m are hidden from some window rows; keys >= n_s do not exist.
#pragma unroll 1
      for (int kb = 0; kb < KT / 32; ++kb) {
        if (tk0 + kb * 32 >= key_end) break;               // nothing but padding from here on
        u32x4 bf[NCS];
        SPECKV_LOAD_BFRAG(bf, buf, kb)
        if (PASS == 1) {
#pragma unroll
          for (int rb = 0; rb < MB; ++rb) {
            if (rb >= nact) continue;
            f32x16 acc = {0};
#pragma unroll
            for (int cs = 0; cs < NCS; ++cs) acc = mma_chunk<DT>(bf[cs], qf[rb][cs], acc);
            // lane: query row (wv*MB+rb)*32 + l32; keys tk0 + kb*32 + 8*(i/4) + 4*half + i%4
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int key = tk0 + kb * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
              if (key > last1[rb]) acc[i] = -INFINITY;
            }
            float tmax = acc[0];
#pragma unroll
            for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, acc[i]);
            const float mnew = fmaxf(mrun[rb], tmax * c2);
            const float scale = __builtin_amdgcn_exp2f(mrun[rb] - mnew);
            const float nm = -mnew;
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(fmaf(acc[i], c2, nm));
            lrun[rb] = fmaf(lrun[rb], scale, sum);
            mrun[rb] = mnew;
          }
        } else {
          float colsum = 0.f;
          const int key = tk0 + kb * 32 + l32;
#pragma unroll
          for (int rb = 0; rb < MB; ++rb) {
            if (rb >= nact) continue;
            f32x16 acc = {0};
#pragma unroll
            for (int cs = 0; cs < NCS; ++cs) acc = mma_chunk<DT>(qf[rb][cs], bf[cs], acc);
            // lane: key tk0 + kb*32 + l32; rows (wv*MB+rb)*32 + 8*(i/4) + 4*half + i%4
            float p[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) p[i] = __builtin_amdgcn_exp2f(fmaf(acc[i], c2, nlse[rb][i]));
#pragma unroll
            for (int i = 0; i < 16; ++i)
              if (key > last2[rb][i]) p[i] = 0.f;
            if (RED == 0) {
#pragma unroll
              for (int i = 0; i < 16; ++i) colsum += p[i];
            } else {
              float cm = 0.f;
#pragma unroll
              for (int i = 0; i < 16; ++i) cm = fmaxf(cm, p[i]);
              cm = max_other_half(cm);
              if (half == 0) csum[(size_t)buf * NW * MB * KT + (rb * NW + wv) * KT + kb * 32 + l32] = cm;
            }
          }
          if (RED == 0) {
            colsum = add_other_half(colsum);
            if (half == 0) csum[(size_t)buf * NW * MB * KT + wv * KT + kb * 32 + l32] = colsum;
          }
        }
      }
    }
    // the next tile must have landed in LDS, and every wave must be done with this one
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  };
  // tiles [t0, t1), t0 even (its tile sits in LDS buffer 0)
  auto run_tiles = [&](int t0, int t1, auto anchored_c) {
    for (int tile = t0; tile < t1; tile += 2) {
      do_tile(tile, std::integral_constant<int, 0>{}, anchored_c);
      if (tile + 1 < t1) do_tile(tile + 1, std::integral_constant<int, 1>{}, anchored_c);
    }
  };
  if constexpr (REPAIR) {
    run_tiles(first_tile, min(ntiles, first_tile + kAnchorTiles), std::false_type{});
  } else if constexpr (PASS == 1 && !MASKED && RED == 1) {
    int n_failed = 0;
    int listed[kFailListed + 1];       // uniform: lives in scalar registers
#pragma unroll
    for (int i = 0; i <= kFailListed; ++i) listed[i] = 0;
    for (int t0 = 0; t0 < ntiles; t0 += kAnchorTiles) {
      const int t1 = min(ntiles, t0 + kAnchorTiles);
      float m_before[MB], l_before[MB];
#pragma unroll
      for (int rb = 0; rb < MB; ++rb) { m_before[rb] = mrun[rb]; l_before[rb] = lrun[rb]; }
      run_tiles(t0, t1, std::true_type{});
      bool out_of_range = false;
#pragma unroll
      for (int rb = 0; rb < MB; ++rb) out_of_range |= !(lrun[rb] < kAnchorLimit);
      // The decision is the wavefront's own (its rows are nobody else's): no barrier, no exchange.
      // (A full list: every later segment is left to the repair as well, overflowed or not.)
      if (__builtin_amdgcn_ballot_w64(out_of_range) != 0 || n_failed > kFailListed) {            // rare
#pragma unroll
        for (int rb = 0; rb < MB; ++rb) { mrun[rb] = m_before[rb]; lrun[rb] = l_before[rb]; }
        if (fresh_tile == t0) fresh_tile = t1;         // still no pair: the next segment finds the reference
#pragma unroll
        for (int i = 0; i <= kFailListed; ++i)
          if (i == n_failed) listed[i] = t0 / kAnchorTiles;
        ++n_failed;
      } else {                                         // the sum's exponent above 2^-shift goes into the reference
#pragma unroll
        for (int rb = 0; rb < MB; ++rb) {
          const int up = lrun[rb] > 0.f ? max(__builtin_amdgcn_frexp_expf(lrun[rb]) + anchor_shift, 0) : 0;
          lrun[rb] = __builtin_ldexpf(lrun[rb], -up);
          mrun[rb] += (float)up;
        }
      }
    }
    if (lane <= kFailListed + 1) {
      int32_t *mine = A.fail + ((int64_t)bid * NW + wv) * kFailWords;
      int v = n_failed;
#pragma unroll
      for (int i = 0; i <= kFailListed; ++i)
        if (lane == i + 1) v = listed[i];
      mine[lane] = v;                  // [0] count, [1 ..] segments, the last one the start of the rest
    }
  } else {
    run_tiles(0, ntiles, std::false_type{});
  }

  if (PASS == 1) {
    // an empty chunk (a sequence without masked tail) leaves the neutral pair (-big, 0)
    float2 *pp = A.part + ((int64_t)unit * A.g.n_chunks + chunk) * RSB;
#pragma unroll
    for (int rb = 0; rb < MB; ++rb) {
      // A sum taken against a fixed reference can be many binary orders away from 1.  Its exponent
      // moves into the reference first, so that every pair handed on has a sum in [0.5, 1) (or 0)
      // and merging two pairs never multiplies a large sum by a factor that underflows.
      int e2;
      const float lf = __builtin_frexpf(lrun[rb], &e2);
      const float mf = mrun[rb] + (float)e2;
      const float mo = __shfl_xor(mf, 32, 64), lo = __shfl_xor(lf, 32, 64);
      const float mm = fmaxf(mf, mo);
      const float ll = lf * __builtin_amdgcn_exp2f(mf - mm) + lo * __builtin_amdgcn_exp2f(mo - mm);
      if (half == 0) {
        float2 *slot = &pp[(rb * NW + wv) * 32 + l32];
        if (REPAIR) {                // add to what the first sweep (and earlier repairs) left there
          const float2 have = *slot;
          const float m2 = fmaxf(have.x, mm);
          *slot = make_float2(m2, have.y * __builtin_amdgcn_exp2f(have.x - m2) + ll * __builtin_amdgcn_exp2f(mm - m2));
        } else {
          *slot = make_float2(mm, ll);
        }
      }
    }
  } else if (ntiles > 0) {
    SPECKV_FLUSH_TILE(ntiles - 1)
  }
}

#undef SPECKV_ROW_VALID
#undef SPECKV_LOAD_TILE
#undef SPECKV_LOAD_BFRAG
#undef SPECKV_FLUSH_TILE

// A kernel with TAIL_ONLY = false is a whole sweep in one launch: its first A.chunk_blocks
// workgroups run one unmasked chunk each, the ones behind them the sequences' masked tails (one per
// (unit, sequence)).  A tail is a short latency chain; behind the chunks it fills the CUs that the
// last round of chunk workgroups frees one by one (ragged batches: 1 % faster than tails in front,
// equal-length grids: the same).  TAIL_ONLY = true is the tails alone (calls without a complete
// chunk, and the tails behind a Q-stationary sweep).
template <int DT, int D, int MB, int NW, int PASS, int RED, bool TAIL_ONLY>
__device__ __forceinline__ void score_dispatch(const ScoreArgs &A) {
  const int bid = blockIdx.x;
  if (TAIL_ONLY) score_body<DT, D, MB, NW, PASS, RED, true>(A, bid);
  else if (bid < A.chunk_blocks) score_body<DT, D, MB, NW, PASS, RED, false>(A, bid);
  else score_body<DT, D, MB, NW, PASS, RED, true>(A, bid - A.chunk_blocks);
}

// The row-statistics sweep is compiled for exactly two waves per SIMD (the register allocator
// then schedules its softmax arithmetic more freely); the column sweep does better without.
template <int DT, int D, int MB, int NW, int PASS, int RED, bool TAIL_ONLY>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void score_kernel_rows(ScoreArgs A) {
  score_dispatch<DT, D, MB, NW, PASS, RED, TAIL_ONLY>(A);
}

template <int DT, int D, int MB, int NW, int PASS, int RED, bool TAIL_ONLY>
__global__ __launch_bounds__(NW * 64) void score_kernel_cols(ScoreArgs A) {
  score_dispatch<DT, D, MB, NW, PASS, RED, TAIL_ONLY>(A);
}

// The launch behind a row-statistics sweep: a chunk workgroup's twin reads the lists its wavefronts
// left and repeats the listed segments, in ascending order, with the online step (normally there
// are none and it returns).  Every thread walks all NW lists, so the order needs no exchange.
template <int DT, int D, int MB, int NW>
__global__ __launch_bounds__(NW * 64) void score_kernel_rows_repair(ScoreArgs A) {
  const int bid = blockIdx.x;
  const int per_group = 8 * A.g.RS;
  const int item = (bid / per_group) * 8 + ((bid % per_group) & 7);
  if (item >= A.g.n_fast_chunks * A.d.L * A.d.Hkv) return;        // padding of the grid: no lists written
  const int32_t *lists = A.fail + (int64_t)bid * NW * kFailWords;
  const int wv = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  int count[NW], at[NW];
  int total = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) { count[w] = lists[w * kFailWords]; at[w] = 0; total += count[w]; }
  if (total == 0) return;
  auto listed = [&](int w, int i) {
    return i <= kFailListed ? lists[w * kFailWords + 1 + i] : lists[w * kFailWords + 1 + kFailListed] + (i - kFailListed);
  };
  for (;;) {
    int next = 0x7fffffff;
#pragma unroll
    for (int w = 0; w < NW; ++w)
      if (at[w] < count[w]) next = min(next, listed(w, at[w]));
    if (next == 0x7fffffff) break;
    bool mine = false;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const bool has = at[w] < count[w] && listed(w, at[w]) == next;
      if (has) ++at[w];
      if (w == wv) mine = has;
    }
    score_body<DT, D, MB, NW, 1, 0, false, true>(A, bid, next, mine);
    __syncthreads();
  }
}

template <typename K>
hipError_t launch_one(K kernel, const ScoreArgs &A, dim3 grid, dim3 block, size_t lds, hipStream_t st) {
  hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kernel, grid, block, lds, st, A);
  return hipGetLastError();
}

template <int DT, int D, int MB, int NW, int PASS, int RED>
hipError_t launch_sweep(const ScoreArgs &A0, size_t lds, hipStream_t st) {
  ScoreArgs A = A0;
  const int64_t tails = (int64_t)A.d.L * A.d.Hkv * A.g.RS * A.d.S;
  if (tails > 0x7fffffffLL) return hipErrorInvalidValue;
  const dim3 block(NW * 64);
  A.chunk_blocks = 0;
  if (A.g.n_fast_chunks > 0 && !qs_supported(A, PASS)) {
    const int64_t items = (int64_t)A.g.n_fast_chunks * A.d.L * A.d.Hkv;
    const int64_t chunk_wgs = (items + 7) / 8 * 8 * A.g.RS;
    if (chunk_wgs + tails > 0x7fffffffLL) return hipErrorInvalidValue;
    A.chunk_blocks = (int)chunk_wgs;
    const dim3 grid((unsigned)(chunk_wgs + tails));
    if constexpr (PASS == 1) {
      hipError_t e;
      if constexpr (NW == 8) e = launch_one(score_kernel_rows<DT, D, MB, NW, PASS, RED, false>, A, grid, block, lds, st);
      else e = launch_one(score_kernel_cols<DT, D, MB, NW, PASS, RED, false>, A, grid, block, lds, st);
      if (e != hipSuccess || RED == 0) return e;
      return launch_one(score_kernel_rows_repair<DT, D, MB, NW>, A, dim3((unsigned)chunk_wgs), block, lds, st);
    } else {
      return launch_one(score_kernel_cols<DT, D, MB, NW, PASS, RED, false>, A, grid, block, lds, st);
    }
  }
  if (A.g.n_fast_chunks > 0) {
    const hipError_t e = launch_qs_sweep(A, PASS, st);
    if (e != hipSuccess) return e;
  }
  return launch_one(score_kernel_cols<DT, D, MB, NW, PASS, RED, true>, A, dim3((unsigned)tails), block, lds, st);
}

// Sweep PASS (1 row statistics, 2 column reduction) for the number type, head dimension and
// workgroup geometry of A.
template <int DT, int D, int MB, int NW, int PASS>
hipError_t sweep_for_geometry(const ScoreArgs &A, hipStream_t st) {
  const size_t lds = score_lds_bytes<elt_bytes(DT), D, MB, NW>();
  if constexpr (PASS == 1) {
    if (score_rows_fixed_reference(A.d, A.g)) return launch_sweep<DT, D, MB, NW, 1, 1>(A, lds, st);
    return launch_sweep<DT, D, MB, NW, 1, 0>(A, lds, st);
  }
  else return A.d.reduce_max ? launch_sweep<DT, D, MB, NW, 2, 1>(A, lds, st) : launch_sweep<DT, D, MB, NW, 2, 0>(A, lds, st);
}

template <int DT, int D, int PASS>
hipError_t sweep_for_type(const ScoreArgs &A, hipStream_t st) {
  switch (A.g.NW * 10 + A.g.MB) {
    case 41: return sweep_for_geometry<DT, D, 1, 4, PASS>(A, st);
    case 81: return sweep_for_geometry<DT, D, 1, 8, PASS>(A, st);
    case 82:
      if constexpr (D * elt_bytes(DT) <= 256) return sweep_for_geometry<DT, D, 2, 8, PASS>(A, st);
      return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
  }
}

template <int PASS>
hipError_t dispatch_sweep(const ScoreArgs &A, hipStream_t st) {
  switch (A.d.dt) {
    case SPECKV_BF16: return A.d.D == 128 ? sweep_for_type<kBf16, 128, PASS>(A, st) : sweep_for_type<kBf16, 64, PASS>(A, st);
    case SPECKV_F16: return A.d.D == 128 ? sweep_for_type<kF16, 128, PASS>(A, st) : sweep_for_type<kF16, 64, PASS>(A, st);
    default: return A.d.D == 128 ? sweep_for_type<kF32, 128, PASS>(A, st) : sweep_for_type<kF32, 64, PASS>(A, st);
  }
}

}  // namespace
}  // namespace speckv
