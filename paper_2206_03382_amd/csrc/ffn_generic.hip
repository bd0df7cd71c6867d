// Grouped GEMM with fused bias + activation epilogue, plain fp32 FMA version.
// Serves the fp32 storage type (where the matrix cores' reduced-precision formats are not wanted) and bf16 shapes
// the MFMA kernel does not cover.  out[e] = epilogue(A[e] (rows_e x K) * B[e] (K x N) + bias[e]); each output element
// is one ascending-k fp32 FMA chain, so results are reproducible.
#include "common.h"

namespace moe {

// TS x TS outputs per thread, 16 x 16 threads: 64 x 64 tiles, or 32 x 32 tiles for launches that would otherwise leave
// most compute units without a block (the arithmetic of an output element is the same chain either way).
template <typename ET, int TS>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const ET* __restrict__ A, const ET* __restrict__ B,
                                                           const ET* __restrict__ bias, int act,
                                                           const int32_t* __restrict__ counts, int64_t C, int K, int N,
                                                           ET* __restrict__ out) {
  constexpr int BM = 16 * TS, BN = 16 * TS, BK = 64;              // long K-steps: few round trips to memory per tile
  constexpr int PF = BM * BK / 256;                               // elements of each operand tile per thread
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN];
  const int e = blockIdx.z;
  int64_t rows = C;
  if (counts) { const int64_t c = counts[e]; rows = c < C ? (c > 0 ? c : 0) : C; }
  const int64_t m0 = (int64_t)blockIdx.y * BM;
  if (m0 >= rows) return;
  const int n0 = blockIdx.x * BN;
  const ET* Ae = A + (int64_t)e * C * K;
  const ET* Be = B + (int64_t)e * K * N;
  const int tid = threadIdx.x, ty = tid / 16, tx = tid % 16;
  float acc[TS][TS];
#pragma unroll
  for (int i = 0; i < TS; ++i)
#pragma unroll
    for (int j = 0; j < TS; ++j) acc[i][j] = 0.f;

  // the next K-step's operands are fetched into registers while this one is computed from LDS
  float pa[PF], pb[PF];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < PF; ++i) {
      const int id = tid + i * 256;
      const int r = id / BK, kk = id % BK;                 // A tile: BM rows x BK k
      const int64_t row = m0 + r;
      pa[i] = (row < rows && k0 + kk < K) ? load_as_f32<ET>(Ae + row * K + k0 + kk) : 0.f;
      const int kb = id / BN, c = id % BN;                 // B tile: BK k x BN cols
      pb[i] = (k0 + kb < K && n0 + c < N) ? load_as_f32<ET>(Be + (int64_t)(k0 + kb) * N + n0 + c) : 0.f;
    }
  };
  fetch(0);
  for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
    for (int i = 0; i < PF; ++i) {
      const int id = tid + i * 256;
      As[id % BK][id / BK] = pa[i];
      Bs[id / BN][id % BN] = pb[i];
    }
    __syncthreads();
    if (k0 + BK < K) fetch(k0 + BK);
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[TS], b[TS];
#pragma unroll
      for (int i = 0; i < TS; ++i) a[i] = As[kk][ty * TS + i];
#pragma unroll
      for (int j = 0; j < TS; ++j) b[j] = Bs[kk][tx * TS + j];
#pragma unroll
      for (int i = 0; i < TS; ++i)
#pragma unroll
        for (int j = 0; j < TS; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < TS; ++i) {
    const int64_t row = m0 + ty * TS + i;
    if (row >= rows) continue;
#pragma unroll
    for (int j = 0; j < TS; ++j) {
      const int col = n0 + tx * TS + j;
      if (col >= N) continue;
      float v = acc[i][j];
      if (bias) v += load_as_f32<ET>(bias + (int64_t)e * N + col);
      if (act >= 0) v = apply_act(v, act);
      store_from_f32<ET>(out + ((int64_t)e * C + row) * N + col, v);
    }
  }
}

hipError_t launch_grouped_gemm_generic(const void* A, const void* B, const void* bias, int act, int dtype,
                                       const int32_t* counts, int64_t E, int64_t C, int64_t K, int64_t N, void* out,
                                       hipStream_t s) {
  const dim3 block(256);
  const bool small = ceil_div(N, 64) * ceil_div(C, 64) * E < 512;   // fewer than two 64 x 64 tiles per compute unit
  const int ts = small ? 32 : 64;
  const dim3 grid((unsigned)ceil_div(N, ts), (unsigned)ceil_div(C, ts), (unsigned)E);
#define MOE_LAUNCH_GENERIC(ET, TS) gemm_generic_kernel<ET, TS><<<grid, block, 0, s>>>((const ET*)A, (const ET*)B, (const ET*)bias, act, counts, C, (int)K, (int)N, (ET*)out)
  if (dtype == MOE_F32) { if (small) MOE_LAUNCH_GENERIC(float, 2); else MOE_LAUNCH_GENERIC(float, 4); }
  else { if (small) MOE_LAUNCH_GENERIC(uint16_t, 2); else MOE_LAUNCH_GENERIC(uint16_t, 4); }
#undef MOE_LAUNCH_GENERIC
  return hipGetLastError();
}

}  // namespace moe
