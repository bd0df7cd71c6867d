// Backward of the local experts' feed-forward layer (arXiv 2206.03382 Sec. 3.2: the backward pass runs "the backward
// computation of the expert" between the two all-to-alls):  y = act(z W1 + b1) W2 + b2  per expert, so
//   dH = dY W2^T,  dP = dH * act'(z W1 + b1),  dZ = dP W1^T,  dW1 = Z^T dP,  db1 = colsum dP,  dW2 = hidden^T dY,
//   db2 = colsum dY,  over the rows of an expert that exist.
// bf16 shapes the matrix-core GEMM takes (M and H multiples of 256) use its transposed-operand layouts: the weights
// are read as stored for the products with W^T, the activations as stored for the weight gradients (reduction over an
// expert's slots up to its fill), and act' is applied in the epilogue of the dH product; nothing is copied.
// Other shapes and fp32 run every product on the plain grouped GEMM (C[e] = A[e] (rows x K) * B[e] (K x N), both
// row-major) after writing out transposed what the chain rule wants transposed (weights [K,N] -> [N,K]; activations
// [C,W] -> [W,Cp] with the rows past the fill zeroed and the row count padded to the GEMM's K step).
#include "common.h"

namespace moe {

namespace {

constexpr int kPadK = 64;                                  // K step of the matrix-core GEMM

__device__ __forceinline__ int64_t live_rows(const int32_t* limit, int e, int64_t R) {
  if (!limit) return R;
  const int64_t c = limit[e];
  return c < R ? (c > 0 ? c : 0) : R;
}

// dst[e, c, r] = src[e, r, c] for r < live rows of e, 0 for live <= r < Rp.   src [E,R,W], dst [E,W,Rp].
template <typename ET>
__global__ __launch_bounds__(256) void transpose_pad_kernel(const ET* __restrict__ src, const int32_t* __restrict__ limit,
                                                            int64_t R, int64_t W, int64_t Rp, ET* __restrict__ dst) {
  __shared__ ET tile[64][64 + 2];
  const int e = blockIdx.z;
  const int64_t r0 = (int64_t)blockIdx.x * 64, c0 = (int64_t)blockIdx.y * 64;
  const int64_t rows = live_rows(limit, e, R);
  const int ty = threadIdx.x >> 6, tx = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int64_t r = r0 + ty * 16 + i, c = c0 + tx;
    tile[ty * 16 + i][tx] = (r < rows && c < W) ? src[((int64_t)e * R + r) * W + c] : ET(0);
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int64_t c = c0 + ty * 16 + i, r = r0 + tx;
    if (c < W && r < Rp) dst[((int64_t)e * W + c) * Rp + r] = tile[tx][ty * 16 + i];
  }
}

// dst[e, r, :] = src[e, r, :] for r < live rows of e, 0 for live <= r < Cp.   src [E,C,W], dst [E,Cp,W]; 16-byte pieces.
__global__ __launch_bounds__(256) void pad_rows_kernel(const uint4* __restrict__ src, const int32_t* __restrict__ limit,
                                                       int64_t E, int64_t C, int64_t Cp, int cpr, uint4* __restrict__ dst) {
  const int64_t n = E * Cp * cpr;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t row = i / cpr, ch = i % cpr;
    const int e = (int)(row / Cp);
    const int64_t r = row % Cp;
    dst[i] = r < live_rows(limit, e, C) ? src[((int64_t)e * C + r) * cpr + ch] : make_uint4(0, 0, 0, 0);
  }
}

// dP = dH * act'(pre) in place over the live rows, 16 bytes per thread.   dH, pre [E,C,H] as rows of cpr pieces.
template <typename ET>
__global__ __launch_bounds__(256) void act_backward_kernel(uint4* __restrict__ dH, const uint4* __restrict__ pre,
                                                           const int32_t* __restrict__ limit, int act, int64_t E, int64_t C,
                                                           int cpr) {
  constexpr int N = Vec16<ET>::N;
  const int64_t n = E * C * cpr;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t row = i / cpr;
    const int e = (int)(row / C);
    if (row % C >= live_rows(limit, e, C)) continue;
    float g[N], p[N];
    Vec16<ET>::unpack(dH[i], g);
    Vec16<ET>::unpack(pre[i], p);
#pragma unroll
    for (int u = 0; u < N; ++u) g[u] *= apply_act_grad(p[u], act);
    dH[i] = Vec16<ET>::pack(g);
  }
}

// out[e, c] = sum over the live rows r of src[e, r, c], fp32, in a fixed order: 32 interleaved row classes, each summed
// in ascending row order by one thread (16-byte pieces, 8 pieces = 64 or 32 columns per block), then added in class
// order.   src [E,C,W] as rows of cpr pieces, out [E,W].
template <typename ET>
__global__ __launch_bounds__(256) void colsum_kernel(const uint4* __restrict__ src, const int32_t* __restrict__ limit,
                                                     int64_t C, int cpr, ET* __restrict__ out) {
  constexpr int N = Vec16<ET>::N;
  __shared__ float part[32][8 * N + 1];
  const int e = blockIdx.y;
  const int rc = threadIdx.x >> 3, pc = threadIdx.x & 7;
  const int64_t piece = (int64_t)blockIdx.x * 8 + pc;
  const int64_t rows = live_rows(limit, e, C);
  float s[N];
#pragma unroll
  for (int u = 0; u < N; ++u) s[u] = 0.f;
  if (piece < cpr) {
#pragma unroll 4
    for (int64_t r = rc; r < rows; r += 32) {
      float f[N];
      Vec16<ET>::unpack(src[((int64_t)e * C + r) * cpr + piece], f);
#pragma unroll
      for (int u = 0; u < N; ++u) s[u] += f[u];
    }
  }
#pragma unroll
  for (int u = 0; u < N; ++u) part[rc][pc * N + u] = s[u];
  __syncthreads();
  if (threadIdx.x < 8 * N) {
    const int64_t col = (int64_t)blockIdx.x * 8 * N + threadIdx.x;
    if (col < (int64_t)cpr * N) {
      float t = 0.f;
#pragma unroll
      for (int k = 0; k < 32; ++k) t += part[k][threadIdx.x];
      store_from_f32<ET>(out + (int64_t)e * cpr * N + col, t);
    }
  }
}

inline size_t align256(size_t v) { return (v + 255) / 256 * 256; }

template <typename ET>
hipError_t transpose_pad(const void* src, const int32_t* limit, int64_t E, int64_t R, int64_t W, int64_t Rp, void* dst, hipStream_t s) {
  const dim3 grid((unsigned)ceil_div(Rp, 64), (unsigned)ceil_div(W, 64), (unsigned)E);
  transpose_pad_kernel<ET><<<grid, dim3(256), 0, s>>>((const ET*)src, limit, R, W, Rp, (ET*)dst);
  return hipGetLastError();
}

}  // namespace

FfnBackwardWorkspace ffn_backward_layout(int64_t E, int64_t C, int64_t M, int64_t H, int dtype) {
  const size_t es = dtype == MOE_F32 ? 4 : 2;
  const int64_t Cp = ceil_div(C, kPadK) * kPadK;
  FfnBackwardWorkspace w;
  size_t o = 0;
  w.pre = o;  o += align256((size_t)E * C * H * es);
  w.dP = o;   o += align256((size_t)E * C * H * es);
  w.Wt = o;   o += align256((size_t)E * M * H * es);       // W2^T, then W1^T
  w.At = o;   o += align256((size_t)E * (M > H ? M : H) * Cp * es);   // hidden^T, then Z^T
  w.Bp = o;   o += align256((size_t)E * Cp * (M > H ? M : H) * es);   // padded dY, then padded dP
  w.total = o;
  w.Cp = Cp;
  return w;
}

template <typename ET>
static hipError_t ffn_backward_t(const void* Z, const void* W1, const void* b1, const void* W2, const void* saved_pre,
                                 const void* hidden, const void* dY, int act, int dtype, const int32_t* counts, int64_t E, int64_t C, int64_t M,
                                 int64_t H, char* ws, void* dZ, void* dW1, void* db1, void* dW2, void* db2, hipStream_t s,
                                 const int32_t* gather, int64_t gather_rows) {
  const FfnBackwardWorkspace w = ffn_backward_layout(E, C, M, H, dtype);
  const int64_t Cp = w.Cp;
  const int es = (int)sizeof(ET);
  void *dP = ws + w.dP, *Wt = ws + w.Wt, *At = ws + w.At, *Bp = ws + w.Bp;
  const void* pre = saved_pre ? saved_pre : ws + w.pre;
  hipError_t err;
#define MOE_TRY(x) do { err = (x); if (err != hipSuccess) return err; } while (0)
  // pre-activations: the caller's (kept by the training forward), else recomputed
  if (!saved_pre) {
    if (gather) return hipErrorInvalidValue;                       // a fused-dispatch training forward always keeps them
    MOE_TRY(launch_grouped_gemm(Z, W1, b1, -1, dtype, counts, E, C, M, H, ws + w.pre, s));
  }
  auto colsums = [&]() -> hipError_t {
    if (db1) {
      const int cprH = (int)(H * es / 16);
      colsum_kernel<ET><<<dim3((unsigned)ceil_div(cprH, 8), (unsigned)E), dim3(256), 0, s>>>((const uint4*)dP, counts, C, cprH, (ET*)db1);
    }
    if (db2) {
      const int cprM = (int)(M * es / 16);
      colsum_kernel<ET><<<dim3((unsigned)ceil_div(cprM, 8), (unsigned)E), dim3(256), 0, s>>>((const uint4*)dY, counts, C, cprM, (ET*)db2);
    }
    return hipGetLastError();
  };
  if (dtype == MOE_BF16 && grouped_gemm_mfma_supports_backward(E, C, M, H)) {
    // dP = (dY W2^T) * act'(pre);  dZ = dP W1^T;  dW2 = hidden^T dY;  dW1 = Z^T dP  (At / Bp hold the last K-steps)
    MOE_TRY(launch_grouped_gemm_mfma_nt(dY, W2, counts, E, C, M, H, dP, pre, act, s));
    if (dZ) MOE_TRY(launch_grouped_gemm_mfma_nt(dP, W1, counts, E, C, H, M, dZ, nullptr, -1, s));
    if (dW2) MOE_TRY(launch_grouped_gemm_mfma_tn(hidden, dY, counts, E, C, H, M, At, Bp, dW2, s));
    if (dW1) MOE_TRY(launch_grouped_gemm_mfma_tn(Z, dP, counts, E, C, M, H, At, Bp, dW1, s, gather, gather_rows));
    return colsums();
  }
  if (gather) return hipErrorInvalidValue;                         // the plain products below need the dispatched rows
  // dH = dY W2^T, then dP = dH * act'(pre)
  MOE_TRY(transpose_pad<ET>(W2, nullptr, E, H, M, H, Wt, s));                          // [E,H,M] -> [E,M,H]
  MOE_TRY(launch_grouped_gemm(dY, Wt, nullptr, -1, dtype, counts, E, C, M, H, dP, s));
  {
    const int cprH = (int)(H * es / 16);
    const int64_t n = E * C * cprH, blocks = ceil_div(n, 256 * 4);
    act_backward_kernel<ET><<<dim3((unsigned)(blocks < 16384 ? blocks : 16384)), dim3(256), 0, s>>>((uint4*)dP, (const uint4*)pre, counts, act, E, C, cprH);
    MOE_TRY(hipGetLastError());
  }
  // dZ = dP W1^T
  if (dZ) {
    MOE_TRY(transpose_pad<ET>(W1, nullptr, E, M, H, M, Wt, s));                        // [E,M,H] -> [E,H,M]
    MOE_TRY(launch_grouped_gemm(dP, Wt, nullptr, -1, dtype, counts, E, C, H, M, dZ, s));
  }
  auto pad_rows = [&](const void* src, int64_t W, void* dst) -> hipError_t {
    const int cpr = (int)(W * es / 16);
    const int64_t n = E * Cp * cpr, blocks = ceil_div(n, 256 * 4);
    pad_rows_kernel<<<dim3((unsigned)(blocks < 16384 ? blocks : 16384)), dim3(256), 0, s>>>((const uint4*)src, counts, E, C, Cp, cpr, (uint4*)dst);
    return hipGetLastError();
  };
  // dW2[e] = hidden[e]^T dY[e]  (H x Cp times Cp x M)
  if (dW2) {
    MOE_TRY(transpose_pad<ET>(hidden, counts, E, C, H, Cp, At, s));
    MOE_TRY(pad_rows(dY, M, Bp));
    MOE_TRY(launch_grouped_gemm(At, Bp, nullptr, -1, dtype, nullptr, E, H, Cp, M, dW2, s));
  }
  // dW1[e] = Z[e]^T dP[e]  (M x Cp times Cp x H)
  if (dW1) {
    MOE_TRY(transpose_pad<ET>(Z, counts, E, C, M, Cp, At, s));
    MOE_TRY(pad_rows(dP, H, Bp));
    MOE_TRY(launch_grouped_gemm(At, Bp, nullptr, -1, dtype, nullptr, E, M, Cp, H, dW1, s));
  }
  MOE_TRY(colsums());
#undef MOE_TRY
  return hipSuccess;
}

bool ffn_backward_gather_supports(int64_t E, int64_t C, int64_t M, int64_t H, int64_t gather_rows, int dtype) {
  return dtype == MOE_BF16 && grouped_gemm_mfma_supports_backward(E, C, M, H) && gather_rows > 0 &&
         gather_rows * M * 2 < ((int64_t)1 << 32);
}

hipError_t launch_expert_ffn_backward(const void* Z, const void* W1, const void* b1, const void* W2, const void* pre,
                                      const void* hidden, const void* dY, int act, int dtype, const int32_t* counts, int64_t E,
                                      int64_t C, int64_t M, int64_t H, void* ws, void* dZ, void* dW1, void* db1, void* dW2,
                                      void* db2, hipStream_t s, const int32_t* gather, int64_t gather_rows) {
  if (dtype == MOE_F32)
    return ffn_backward_t<float>(Z, W1, b1, W2, pre, hidden, dY, act, dtype, counts, E, C, M, H, (char*)ws, dZ, dW1, db1, dW2, db2, s,
                                 gather, gather_rows);
  return ffn_backward_t<uint16_t>(Z, W1, b1, W2, pre, hidden, dY, act, dtype, counts, E, C, M, H, (char*)ws, dZ, dW1, db1, dW2, db2, s,
                                  gather, gather_rows);
}

}  // namespace moe
