// Definitions shared by the scoring kernels (Sec. 3.1 Eq. 1; Alg. 1 CrossAttention and reduce
// steps): MFMA wrappers per number type, the swizzled 16-byte-chunk row layout used for operand
// tiles in LDS, and the argument block of the sweeps.  Not part of the C ABI.
#pragma once

#include "speckv_internal.h"

namespace speckv {

// Argument block of the scoring sweeps.
struct ScoreArgs {
  Dims d;
  SeqTab t;
  ScoreGeom g;
  const char *q;
  const char *k;
  float2 *part;     // [unit][chunk][RSB] (max2, sum) per row, unit = (layer, head, row super-block)
  float *lse;       // [layer][head][seq][RS*RSB]
  const float *lse_in;   // optional caller-supplied natural-log normalisers [L][S][R][Hq]
  float *planes;    // [RS][layer][Hkv*T]
  uint32_t *clear;  // optional scratch the kernel between the sweeps zeroes (clear_words words)
  int64_t clear_words;
  int chunk_blocks; // whole-sweep launches: workgroups that run unmasked chunks; the masked tails follow them
  int32_t *fail;    // row-statistics sweep: kFailWords ints per chunk workgroup (see score_sweep.h)
};

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // one 128-bit lane access

constexpr float kNegBig = -1.0e30f;    // finite stand-in for "no key seen yet"
// Row statistics against a fixed reference (score_sweep.h): a segment of kAnchorTiles tiles after
// which a row sum has reached 2^126 (or is not a number) is repeated with the online step.
constexpr int kAnchorTiles = 2;
// What each wavefront of a chunk workgroup of the row-statistics sweep leaves for the repair
// launch: [0] the number of segments to repeat, [1 .. kFailListed] the first ones by number,
// [kFailWords - 1] the segment from which on every segment is to be repeated when there are more
// than that.  A workgroup has kFailWaves such lists (the most waves a workgroup has).
constexpr int kFailWords = 8, kFailListed = 6, kFailWaves = 8;
constexpr float kAnchorLimit = 8.507059e37f;


// x + (x of the lane 32 away), in every lane, without going through LDS (v_permlane32_swap).
__device__ inline float add_other_half(float x) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}


__device__ inline float max_other_half(float x) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Number types (values of speckv_dtype) and their element size.
constexpr int kBf16 = SPECKV_BF16, kF32 = SPECKV_F32, kF16 = SPECKV_F16;
constexpr int elt_bytes(int dt) { return dt == kF32 ? 4 : 2; }

// One 16-byte chunk of the head dimension per lane half: 8 bf16/f16 or 4 f32 products per row pair.
template <int DT>
__device__ inline f32x16 mma_chunk(u32x4 a, u32x4 b, f32x16 acc);

template <>
__device__ inline f32x16 mma_chunk<kBf16>(u32x4 a, u32x4 b, f32x16 acc) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}

template <>
__device__ inline f32x16 mma_chunk<kF16>(u32x4 a, u32x4 b, f32x16 acc) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                __builtin_bit_cast(f16x8, b), acc, 0, 0, 0);
}

template <>
__device__ inline f32x16 mma_chunk<kF32>(u32x4 a, u32x4 b, f32x16 acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
  return acc;
}

template <int ELT, int D>
struct Tile {
  static constexpr int ROWB = D * ELT;          // bytes per key / query row
  static constexpr int C16 = ROWB / 16;         // 16-byte chunks per row
  static constexpr int NCS = C16 / 2;           // chunk steps (each lane half owns NCS chunks)
  static constexpr int KT = ROWB <= 128 ? 256 : ROWB <= 256 ? 128 : 64;   // keys per LDS tile (32 KiB)
  static constexpr int TILE_BYTES = KT * ROWB;
  static constexpr int RPB = ROWB >= 256 ? 1 : 256 / ROWB;   // rows per 256-byte bank sweep
  static constexpr int SWZ = (C16 < 16 ? C16 : 16) - 1;      // xor mask applied to the chunk index
  __device__ static inline int swizzle(int row) { return (row / RPB) & SWZ; }
};

}  // namespace

// Column-reduction and row-statistics sweeps over the unmasked chunks with the group's query
// rows stationary in LDS and each wave streaming its own keys through registers (score_qs.hip).
// Returns false when the geometry is outside what that kernel is built for; then nothing was
// launched and the caller uses the tile-streaming kernel.
// The two sweeps over all chunks and masked tails of a call (score_rows.hip, score_cols.hip).
hipError_t launch_row_statistics_sweep(const ScoreArgs &A, hipStream_t st);
hipError_t launch_column_sweep(const ScoreArgs &A, hipStream_t st);
bool qs_supported(const ScoreArgs &A, int pass);
hipError_t launch_qs_sweep(const ScoreArgs &A, int pass, hipStream_t st);

}  // namespace speckv
