// Ceiling probe: what this GPU sustains for the instruction mix of the scoring sweeps when nothing
// has to be fetched.  One 32x32 score tile at d = 128 is 8 bf16 MFMAs (32x32x16) plus, per lane, 16
// times (fused multiply-add, exp2, add): the softmax arithmetic of Eq. 1 (Sec. 3.1) on the tile the
// MFMAs of the previous iteration produced.  Three register-resident loops with that mix:
//
//   kind 0  the MFMAs alone
//   kind 1  MFMAs + softmax arithmetic
//   kind 2  kind 1 with the B operands re-read from LDS every second tile (512 bytes of LDS
//           traffic per MFMA, what the sweeps do)
//
// 256 workgroups of 512 threads (two waves per SIMD on every CU).  The operands come from a
// caller-provided buffer so that the data-dependent power draw can be seen: random bf16 values
// and all zeros give very different clocks.  The caller times the launch and converts
// waves * iters * 8 * 32768 flops into TFLOP/s.  Diagnostics only; not on the product path.
#include "speckv_internal.h"

namespace speckv {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kProbeThreads = 512;
constexpr int kProbeGrid = 256;

template <int LDS_EVERY, int SOFTMAX>
__global__ __launch_bounds__(kProbeThreads) void probe_kernel(const u32x4 *__restrict__ in, float *__restrict__ out,
                                                              int iters) {
  __shared__ u32x4 lb[2048];   // 32 KiB, as large as one key tile of the sweeps
  for (int i = threadIdx.x; i < 2048; i += kProbeThreads) lb[i] = in[(i * 7 + 3) & 4095];
  __syncthreads();
  u32x4 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = in[(threadIdx.x + i * 64) & 4095];
    b[i] = in[(threadIdx.x + 517 + i * 64) & 4095];
  }
  const int lane = threadIdx.x & 63;
  float l[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) l[j] = -0.25f * (float)((lane + j) & 31);
  const float c = 0.01f;
  float sum = 0.f;
  f32x16 prev;
#pragma unroll
  for (int j = 0; j < 16; ++j) prev[j] = (float)(lane + j);
  for (int it = 0; it < iters; ++it) {
    if (LDS_EVERY > 0 && (it % LDS_EVERY) == 0) {
#pragma unroll
      for (int i = 0; i < 8; ++i) b[i] = lb[((it * 8 + i) * 64 + lane) & 2047];
    }
    f32x16 acc = {0};
#pragma unroll
    for (int i = 0; i < 8; ++i)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[i]),
                                                    acc, 0, 0, 0);
    if (SOFTMAX) {
#pragma unroll
      for (int j = 0; j < 16; ++j) sum += __builtin_amdgcn_exp2f(fmaf(prev[j], c, l[j]));
    } else {
      sum += prev[0];
    }
    prev = acc;
  }
  out[blockIdx.x * kProbeThreads + threadIdx.x] = sum;
}

}  // namespace
}  // namespace speckv

using namespace speckv;

extern "C" speckv_status speckv_probe_ceiling(int32_t kind, int32_t iters, const void *operands, void *out,
                                              void *stream, int64_t *flops) {
  if (kind < 0 || kind > 2 || iters < 1 || operands == nullptr || out == nullptr || flops == nullptr)
    return SPECKV_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(operands) & 15u) || (reinterpret_cast<uintptr_t>(out) & 3u)) return SPECKV_ERR_INVALID_ARG;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const u32x4 *in = static_cast<const u32x4 *>(operands);
  float *o = static_cast<float *>(out);
  const dim3 grid(kProbeGrid), block(kProbeThreads);
  if (kind == 0) hipLaunchKernelGGL((probe_kernel<0, 0>), grid, block, 0, hs, in, o, iters);
  else if (kind == 1) hipLaunchKernelGGL((probe_kernel<0, 1>), grid, block, 0, hs, in, o, iters);
  else hipLaunchKernelGGL((probe_kernel<2, 1>), grid, block, 0, hs, in, o, iters);
  *flops = (int64_t)kProbeGrid * (kProbeThreads / 64) * iters * 8 * 32768;
  return hipGetLastError() == hipSuccess ? SPECKV_OK : SPECKV_ERR_RUNTIME;
}
