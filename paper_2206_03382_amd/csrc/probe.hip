// Measurement aid, built into its own library (libmoe_probe.so) and used by bench.py only: what the matrix cores alone
// sustain on this board.  Every wave of the grid keeps 16 accumulator tiles in registers (the expert GEMM's 128 x 128
// wave tile) and issues `iters` rounds of 32 v_mfma_f32_32x32x16_bf16 on operand fragments that never change, with no
// memory traffic at all.  The operands are random bf16 values (uniform sign and mantissa, magnitudes in [0.5, 1)) or
// all ones: the power a matrix core draws, and with it the clock the board's power limit allows, depends on the bits
// that toggle.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/moe_mi355x_probe.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
constexpr int kThreads = 256;

__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

__global__ __launch_bounds__(kThreads) void mfma_sustained_kernel(int iters, int random_operands, float* __restrict__ sink) {
  const uint32_t tid = blockIdx.x * kThreads + threadIdx.x;
  bf16x8 a[2][4], b[2][4];
#pragma unroll
  for (int p = 0; p < 2; ++p)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      u32x4 wa, wb;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t ha = probe_hash((tid * 64 + p * 8 + i) * 4 + u), hb = probe_hash((tid * 64 + 32 + p * 8 + i) * 4 + u);
        wa[u] = random_operands ? (0x3f003f00u | (ha & 0x80ff80ffu)) : 0x3f803f80u;
        wb[u] = random_operands ? (0x3f003f00u | (hb & 0x80ff80ffu)) : 0x3f803f80u;
      }
      a[p][i] = __builtin_bit_cast(bf16x8, wa);
      b[p][i] = __builtin_bit_cast(bf16x8, wb);
    }
  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
      for (int m = 0; m < 16; ++m)
        acc[m >> 2][m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[p][m & 3], a[p][m >> 2], acc[m >> 2][m & 3], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) sum += acc[i][j][v];
  if (sum == 12345.678f) sink[tid] = sum;                           // keeps the loop alive; never true in practice
}

}  // namespace

extern "C" int moe_probe_mfma_sustained(int blocks, int iters, int random_operands, float* sink, double* flop_per_launch,
                                        void* stream) {
  if (blocks < 1 || blocks > 65536 || iters < 1 || iters > (1 << 20) || !sink) return 1;
  if (flop_per_launch) *flop_per_launch = (double)blocks * 4.0 * iters * 32.0 * 2.0 * 32 * 32 * 16;
  mfma_sustained_kernel<<<dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream>>>(iters, random_operands, sink);
  return hipGetLastError() == hipSuccess ? 0 : 4;
}
