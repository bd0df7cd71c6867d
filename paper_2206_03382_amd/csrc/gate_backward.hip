// Backward of the gating function (arXiv 2206.03382 Sec. 2.1 gate; Sec. 3.2: the backward pass mirrors the forward).
//   gate_backward_kernel   : d gate_w [T,k] -> d logits [T,E] through (renormalised) softmax-at-the-chosen-experts
//   gate_dx_kernel         : dx[t,:] (+)= sum_e dlogits[t,e] Wg[:,e]
//   gate_dw_partial/reduce : dWg[m,e] = sum_t x[t,m] dlogits[t,e], token slices summed in a fixed order; dbias likewise
// The chosen experts and the slots are integer decisions and carry no gradient.  Small, HBM-bound kernels.
#include "common.h"

namespace moe {

namespace {

constexpr int kDwSlice = 64;                               // tokens per partial sum of dWg

// One thread per token.  p = softmax(logits); g_j = p[idx_j]; gate_w = g / sum g (normalize) or g.
__global__ __launch_bounds__(256) void gate_backward_kernel(const float* __restrict__ logits, const int32_t* __restrict__ idx,
                                                            const float* __restrict__ dgate_w, int64_t T, int E, int k,
                                                            int normalize, float* __restrict__ dlogits) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  const float* row = logits + t * E;
  float mx = row[0];
  for (int e = 1; e < E; ++e) mx = fmaxf(mx, row[e]);
  float se = 0.f;
  for (int e = 0; e < E; ++e) se += expf(row[e] - mx);
  const float inv = 1.0f / se;
  const int32_t* id = idx + t * k;
  const float* dw = dgate_w + t * k;
  auto g_of = [&](int j) { const int e = id[j]; return ((unsigned)e < (unsigned)E) ? expf(row[e] - mx) * inv : 0.f; };
  float S = 1.f, c1 = 0.f;
  if (normalize) {
    S = 0.f;
    for (int j = 0; j < k; ++j) S += g_of(j);
    for (int j = 0; j < k; ++j) c1 += dw[j] * (g_of(j) / S);
  }
  // dg_j = (dw_j - c1) / S;   c = sum_j g_j dg_j = sum_e p_e dp_e
  float c = 0.f;
  for (int j = 0; j < k; ++j) c += g_of(j) * ((dw[j] - c1) / S);
  float* out = dlogits + t * E;
  for (int e = 0; e < E; ++e) out[e] = -(expf(row[e] - mx) * inv) * c;
  for (int j = 0; j < k; ++j) {                              // the chosen experts of a token are distinct
    const int e = id[j];
    if ((unsigned)e < (unsigned)E) out[e] += g_of(j) * ((dw[j] - c1) / S);
  }
}

constexpr int kDwThreads = 128;                            // threads (row pieces) per block of the dWg partial kernel
constexpr int kDxTokens = 16;                              // tokens per block of the dx kernel

// Eight consecutive entries of row `row` of Wg [M,E] starting at expert e0, as floats (0 past E).  With E a multiple of
// the 16-byte piece the row pieces are fetched whole.
template <typename ET>
__device__ __forceinline__ void wg_row8(const ET* __restrict__ Wg, int64_t row, int E, int e0, bool vec, float (&out)[8]) {
  constexpr int N = Vec16<ET>::N;
  if (vec) {
    const uint4* p = reinterpret_cast<const uint4*>(Wg + row * E + e0);
#pragma unroll
    for (int h = 0; h < 8 / N; ++h) {
      float f[N];
      Vec16<ET>::unpack(p[h], f);
#pragma unroll
      for (int i = 0; i < N; ++i) out[h * N + i] = f[i];
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) out[i] = e0 + i < E ? load_as_f32<ET>(Wg + row * E + e0 + i) : 0.f;
  }
}

// dx[t,m] = (accumulate ? dx[t,m] : 0) + sum_e dlogits[t,e] Wg[m,e].  A thread owns one 16-byte piece of the rows (N
// consecutive m) for kDxTokens tokens: the pieces of all its tokens are fetched at once and stay in registers while
// its N rows of Wg pass by, 8 experts at a time; the block's dlogits go through LDS.
template <typename ET>
__global__ __launch_bounds__(256) void gate_dx_kernel(const float* __restrict__ dlogits, const ET* __restrict__ Wg, int64_t T,
                                                      int cpr, int E, int accumulate, uint4* __restrict__ dx) {
  constexpr int N = Vec16<ET>::N;
  __shared__ float dls[kDxTokens][8];
  const int64_t t0 = (int64_t)blockIdx.x * kDxTokens;
  const int piece = blockIdx.y * 256 + threadIdx.x;
  const bool live = piece < cpr;                            // every thread joins the barriers
  const bool vec = (E % 8) == 0 && (reinterpret_cast<uintptr_t>(Wg) & 15) == 0;
  float acc[kDxTokens][N];
#pragma unroll
  for (int tt = 0; tt < kDxTokens; ++tt) {
    if (live && accumulate && t0 + tt < T) Vec16<ET>::unpack(dx[(t0 + tt) * cpr + piece], acc[tt]);
    else {
#pragma unroll
      for (int u = 0; u < N; ++u) acc[tt][u] = 0.f;
    }
  }
  for (int e0 = 0; e0 < E; e0 += 8) {
    __syncthreads();                                        // the previous chunk's dlogits have been read
    if (threadIdx.x < kDxTokens * 8) {
      const int tt = threadIdx.x >> 3, i = threadIdx.x & 7;
      dls[tt][i] = (t0 + tt < T && e0 + i < E) ? dlogits[(t0 + tt) * E + e0 + i] : 0.f;
    }
    __syncthreads();
    if (live) {
      float wr[N][8];
#pragma unroll
      for (int u = 0; u < N; ++u) wg_row8<ET>(Wg, (int64_t)piece * N + u, E, e0, vec, wr[u]);
#pragma unroll
      for (int tt = 0; tt < kDxTokens; ++tt) {
#pragma unroll
        for (int u = 0; u < N; ++u)
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[tt][u] = fmaf(dls[tt][i], wr[u][i], acc[tt][u]);
      }
    }
  }
  if (live) {
#pragma unroll
    for (int tt = 0; tt < kDxTokens; ++tt)
      if (t0 + tt < T) dx[(t0 + tt) * cpr + piece] = Vec16<ET>::pack(acc[tt]);
  }
}

// partial[s][m][e] = sum over the tokens of slice s (ascending) of x[t,m] dlogits[t,e].  A thread owns one 16-byte piece
// of the rows (N consecutive m) and 8 experts; the slice's dlogits go through LDS and the rows are fetched 16 at a time.
template <typename ET>
__global__ __launch_bounds__(kDwThreads) void gate_dw_partial_kernel(const uint4* __restrict__ x, const float* __restrict__ dlogits,
                                                              int64_t T, int cpr, int E, float* __restrict__ partial) {
  constexpr int N = Vec16<ET>::N;
  __shared__ float dls[kDwSlice][8];
  const int piece = blockIdx.x * kDwThreads + threadIdx.x;
  const int64_t s = blockIdx.y, t0 = s * kDwSlice;
  const int e0 = blockIdx.z * 8;
  for (int i = threadIdx.x; i < kDwSlice * 8; i += kDwThreads) {
    const int tt = i >> 3, ei = i & 7;
    dls[tt][ei] = (t0 + tt < T && e0 + ei < E) ? dlogits[(t0 + tt) * E + e0 + ei] : 0.f;   // zeros past T: those rows add nothing
  }
  __syncthreads();
  if (piece >= cpr) return;
  float acc[N][8];
#pragma unroll
  for (int u = 0; u < N; ++u)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[u][i] = 0.f;
  for (int tb = 0; tb < kDwSlice; tb += 16) {
    uint4 xr[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int64_t t = t0 + tb + q;
      xr[q] = x[(t < T ? t : T - 1) * cpr + piece];         // past T: a valid row, multiplied by zeros
    }
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      float xv[N];
      Vec16<ET>::unpack(xr[q], xv);
#pragma unroll
      for (int u = 0; u < N; ++u)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[u][i] = fmaf(xv[u], dls[tb + q][i], acc[u][i]);
    }
  }
  const int64_t M = (int64_t)cpr * N;
#pragma unroll
  for (int u = 0; u < N; ++u) {
    float* dst = partial + ((int64_t)s * M + (int64_t)piece * N + u) * E + e0;
    if ((E & 7) == 0) {                                     // eight experts = 32 contiguous, aligned bytes
      reinterpret_cast<float4*>(dst)[0] = make_float4(acc[u][0], acc[u][1], acc[u][2], acc[u][3]);
      reinterpret_cast<float4*>(dst)[1] = make_float4(acc[u][4], acc[u][5], acc[u][6], acc[u][7]);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (e0 + i < E) dst[i] = acc[u][i];
    }
  }
}

// dWg[i] = sum over slices, in slice order, of partial[s][i]   (i over M*E)
template <typename ET>
__global__ __launch_bounds__(256) void gate_dw_reduce_kernel(const float* __restrict__ partial, int64_t n, int slices,
                                                             ET* __restrict__ dWg) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float s = 0.f;
  int k = 0;
  for (; k + 8 <= slices; k += 8) {                         // eight loads in flight, added in slice order
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = partial[(int64_t)(k + u) * n + i];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  for (; k < slices; ++k) s += partial[(int64_t)k * n + i];
  store_from_f32<ET>(dWg + i, s);
}

// dbias[e] = sum_t dlogits[t,e]: one block per expert, 256 interleaved token classes summed in ascending order (eight
// loads in flight), then a fixed tree.
__global__ __launch_bounds__(256) void gate_dbias_kernel(const float* __restrict__ dlogits, int64_t T, int E,
                                                         float* __restrict__ dbias) {
  __shared__ float part[256];
  const int e = blockIdx.x;
  float s = 0.f;
  int64_t t = threadIdx.x;
  for (; t + 7 * 256 < T; t += 8 * 256) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = dlogits[(t + u * 256) * E + e];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  for (; t < T; t += 256) s += dlogits[t * E + e];
  part[threadIdx.x] = s;
  __syncthreads();
  for (int off = 128; off >= 1; off >>= 1) {
    if (threadIdx.x < off) part[threadIdx.x] += part[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) dbias[e] = part[0];
}

}  // namespace

size_t gate_backward_workspace_bytes(int64_t T, int64_t M, int64_t E) {
  return align_up((size_t)T * E * 4, 256) + align_up((size_t)ceil_div(T, kDwSlice) * M * E * 4, 256);
}

template <typename ET>
static hipError_t gate_backward_t(const void* x, const void* Wg, const float* logits, const int32_t* idx, const float* dgate_w,
                                  int normalize, int64_t T, int64_t M, int64_t E, int k, char* ws, void* dx, int accumulate_dx,
                                  void* dWg, float* dbias, float* dlogits_out, hipStream_t s) {
  float* dl = dlogits_out ? dlogits_out : (float*)ws;
  float* partial = (float*)(ws + align_up((size_t)T * E * 4, 256));
  hipError_t err;
  gate_backward_kernel<<<dim3((unsigned)ceil_div(T, 256)), dim3(256), 0, s>>>(logits, idx, dgate_w, T, (int)E, k, normalize, dl);
  if ((err = hipGetLastError()) != hipSuccess) return err;
  if (dx) {
    const int cpr = (int)(M * sizeof(ET) / 16);
    gate_dx_kernel<ET><<<dim3((unsigned)ceil_div(T, kDxTokens), (unsigned)ceil_div(cpr, 256)), dim3(256), 0, s>>>(dl, (const ET*)Wg, T, cpr, (int)E, accumulate_dx, (uint4*)dx);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  if (dWg) {
    const int slices = (int)ceil_div(T, kDwSlice);
    const int cprx = (int)(M * sizeof(ET) / 16);
    gate_dw_partial_kernel<ET><<<dim3((unsigned)ceil_div(cprx, kDwThreads), (unsigned)slices, (unsigned)ceil_div(E, 8)), dim3(kDwThreads), 0, s>>>(
        (const uint4*)x, dl, T, cprx, (int)E, partial);
    if ((err = hipGetLastError()) != hipSuccess) return err;
    const int64_t n = M * E;
    gate_dw_reduce_kernel<ET><<<dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s>>>(partial, n, slices, (ET*)dWg);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  if (dbias) {
    gate_dbias_kernel<<<dim3((unsigned)E), dim3(256), 0, s>>>(dl, T, (int)E, dbias);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  return hipSuccess;
}

hipError_t launch_gate_backward(const void* x, const void* Wg, const float* logits, const int32_t* idx, const float* dgate_w,
                                int normalize, int dtype, int64_t T, int64_t M, int64_t E, int k, void* ws, void* dx,
                                int accumulate_dx, void* dWg, float* dbias, float* dlogits, hipStream_t s) {
  if (dtype == MOE_F32)
    return gate_backward_t<float>(x, Wg, logits, idx, dgate_w, normalize, T, M, E, k, (char*)ws, dx, accumulate_dx, dWg, dbias, dlogits, s);
  return gate_backward_t<uint16_t>(x, Wg, logits, idx, dgate_w, normalize, T, M, E, k, (char*)ws, dx, accumulate_dx, dWg, dbias, dlogits, s);
}

}  // namespace moe
