// Backward of the gating function (arXiv 2206.03382 Sec. 2.1 gate; Sec. 3.2: the backward pass mirrors the forward).
//   gate_backward_kernel   : d gate_w [T,k] -> d logits [T,E] through (renormalised) softmax-at-the-chosen-experts
//   gate_dx_kernel         : dx[t,:] (+)= sum_e dlogits[t,e] Wg[:,e]
//   gate_dw_partial/reduce : dWg[m,e] = sum_t x[t,m] dlogits[t,e], token slices summed in a fixed order; dbias likewise
// The chosen experts and the slots are integer decisions and carry no gradient.  Small, HBM-bound kernels.
#include "common.h"

namespace moe {

namespace {

constexpr int kDwSlice = 128;                              // tokens per partial sum of dWg

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

// dx[t,m] = (accumulate ? dx[t,m] : 0) + sum_e dlogits[t,e] Wg[m,e].  One thread per (t, 16-byte piece of the row).
template <typename ET>
__global__ __launch_bounds__(256) void gate_dx_kernel(const float* __restrict__ dlogits, const ET* __restrict__ Wg, int64_t T,
                                                      int cpr, int E, int accumulate, uint4* __restrict__ dx) {
  constexpr int N = Vec16<ET>::N;
  const int64_t t = blockIdx.x;
  const int piece = blockIdx.y * 256 + threadIdx.x;
  if (piece >= cpr) return;
  const float* dl = dlogits + t * E;
  const ET* w = Wg + (int64_t)piece * N * E;                // rows piece*N .. piece*N + N-1 of Wg, E values each
  float acc[N];
  if (accumulate) Vec16<ET>::unpack(dx[t * cpr + piece], acc);
  else {
#pragma unroll
    for (int u = 0; u < N; ++u) acc[u] = 0.f;
  }
  if ((E % N) == 0 && (reinterpret_cast<uintptr_t>(Wg) & 15) == 0) {    // rows of Wg are whole 16-byte pieces
    const uint4* wv = reinterpret_cast<const uint4*>(w);
    const int rp = E / N;                                   // pieces per row
    for (int q = 0; q < rp; ++q) {
      float d[N];
#pragma unroll
      for (int i = 0; i < N; ++i) d[i] = dl[q * N + i];
#pragma unroll
      for (int u = 0; u < N; ++u) {
        float f[N];
        Vec16<ET>::unpack(wv[u * rp + q], f);
#pragma unroll
        for (int i = 0; i < N; ++i) acc[u] = fmaf(d[i], f[i], acc[u]);
      }
    }
  } else {
    for (int e = 0; e < E; ++e) {
      const float d = dl[e];
#pragma unroll
      for (int u = 0; u < N; ++u) acc[u] = fmaf(d, load_as_f32<ET>(w + u * E + e), acc[u]);
    }
  }
  dx[t * cpr + piece] = Vec16<ET>::pack(acc);
}

// partial[s][m][e] = sum over the tokens of slice s of x[t,m] dlogits[t,e]; thread = m, 8 experts per pass.
template <typename ET>
__global__ __launch_bounds__(256) void gate_dw_partial_kernel(const ET* __restrict__ x, const float* __restrict__ dlogits,
                                                              int64_t T, int M, int E, float* __restrict__ partial) {
  const int m = blockIdx.x * 256 + threadIdx.x;
  const int64_t s = blockIdx.y, t0 = s * kDwSlice, t1 = (t0 + kDwSlice) < T ? (t0 + kDwSlice) : T;
  const int e0 = blockIdx.z * 8;
  if (m >= M) return;
  float acc[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) acc[u] = 0.f;
#pragma unroll 4
  for (int64_t t = t0; t < t1; ++t) {
    const float xv = load_as_f32<ET>(x + t * M + m);
    const float* dl = dlogits + t * E + e0;
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (e0 + u < E) acc[u] = fmaf(xv, dl[u], acc[u]);
  }
#pragma unroll
  for (int u = 0; u < 8; ++u)
    if (e0 + u < E) partial[((int64_t)s * M + m) * E + e0 + u] = acc[u];
}

// dWg[i] = sum over slices, in slice order, of partial[s][i]   (i over M*E)
template <typename ET>
__global__ __launch_bounds__(256) void gate_dw_reduce_kernel(const float* __restrict__ partial, int64_t n, int slices,
                                                             ET* __restrict__ dWg) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float s = 0.f;
  for (int k = 0; k < slices; ++k) s += partial[(int64_t)k * n + i];
  store_from_f32<ET>(dWg + i, s);
}

// dbias[e] = sum_t dlogits[t,e]: one block per expert, 256 interleaved token classes summed in order, then a fixed tree.
__global__ __launch_bounds__(256) void gate_dbias_kernel(const float* __restrict__ dlogits, int64_t T, int E,
                                                         float* __restrict__ dbias) {
  __shared__ float part[256];
  const int e = blockIdx.x;
  float s = 0.f;
  for (int64_t t = threadIdx.x; t < T; t += 256) s += dlogits[t * E + e];
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
    gate_dx_kernel<ET><<<dim3((unsigned)T, (unsigned)ceil_div(cpr, 256)), dim3(256), 0, s>>>(dl, (const ET*)Wg, T, cpr, (int)E, accumulate_dx, (uint4*)dx);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  if (dWg) {
    const int slices = (int)ceil_div(T, kDwSlice);
    gate_dw_partial_kernel<ET><<<dim3((unsigned)ceil_div(M, 256), (unsigned)slices, (unsigned)ceil_div(E, 8)), dim3(256), 0, s>>>(
        (const ET*)x, dl, T, (int)M, (int)E, partial);
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
