// Grouped GEMM with fused bias + activation epilogue, plain fp32 FMA version.
// Serves the fp32 storage type (where the matrix cores' reduced-precision formats are not wanted) and bf16 shapes
// the MFMA kernel does not cover.  out[e] = epilogue(A[e] (rows_e x K) * B[e] (K x N) + bias[e]); each output element
// is one ascending-k fp32 FMA chain, so results are reproducible.
#include "common.h"

namespace moe {

template <typename ET>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const ET* __restrict__ A, const ET* __restrict__ B,
                                                           const ET* __restrict__ bias, int act,
                                                           const int32_t* __restrict__ counts, int64_t C, int K, int N,
                                                           ET* __restrict__ out) {
  constexpr int BM = 64, BN = 64, BK = 16;
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
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  // the next K-step's operands are fetched into registers while this one is computed from LDS
  float pa[4], pb[4];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + i * 256;
      const int r = id / BK, kk = id % BK;                 // A tile: 64 rows x 16 k
      const int64_t row = m0 + r;
      pa[i] = (row < rows && k0 + kk < K) ? load_as_f32<ET>(Ae + row * K + k0 + kk) : 0.f;
      const int kb = id / BN, c = id % BN;                 // B tile: 16 k x 64 cols
      pb[i] = (k0 + kb < K && n0 + c < N) ? load_as_f32<ET>(Be + (int64_t)(k0 + kb) * N + n0 + c) : 0.f;
    }
  };
  fetch(0);
  for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + i * 256;
      As[id % BK][id / BK] = pa[i];
      Bs[id / BN][id % BN] = pb[i];
    }
    __syncthreads();
    if (k0 + BK < K) fetch(k0 + BK);
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t row = m0 + ty * 4 + i;
    if (row >= rows) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + tx * 4 + j;
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
  const dim3 grid((unsigned)ceil_div(N, 64), (unsigned)ceil_div(C, 64), (unsigned)E), block(256);
  if (dtype == MOE_F32)
    gemm_generic_kernel<float><<<grid, block, 0, s>>>((const float*)A, (const float*)B, (const float*)bias, act, counts, C, (int)K, (int)N, (float*)out);
  else
    gemm_generic_kernel<uint16_t><<<grid, block, 0, s>>>((const uint16_t*)A, (const uint16_t*)B, (const uint16_t*)bias, act, counts, C, (int)K, (int)N, (uint16_t*)out);
  return hipGetLastError();
}

}  // namespace moe
