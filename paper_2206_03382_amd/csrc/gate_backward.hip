// Backward of the gating function (arXiv 2206.03382 Sec. 2.1 gate; Sec. 3.2: the backward pass mirrors the forward).
//   gate_backward_kernel   : d gate_w [T,k] -> d logits [T,E] through (renormalised) softmax-at-the-chosen-experts
//   gate_dx_kernel         : dx[t,:] (+)= sum_e dlogits[t,e] Wg[:,e]
//   gate_dw_partial/reduce : dWg[m,e] = sum_t x[t,m] dlogits[t,e], token slices summed in a fixed order; dbias likewise
// The chosen experts and the slots are integer decisions and carry no gradient.  Small, HBM-bound kernels.
#include "common.h"

namespace moe {

namespace {

constexpr int kDwSlice = 64;                               // tokens per partial sum of dWg

constexpr int kGbTokens = 64;                              // tokens (= threads) per block of the dlogits kernel (16 for wide gates)

// One thread per token.  p = softmax(logits); g_j = p[idx_j]; gate_w = g / sum g (normalize) or g.  The block's rows of
// logits come in, and its rows of dlogits go out, through LDS (rows padded by one float) so that global accesses are
// contiguous however many experts a row has.
__global__ __launch_bounds__(kGbTokens) void gate_backward_kernel(const float* __restrict__ logits, const int32_t* __restrict__ idx,
                                                                  const float* __restrict__ dgate_w, int64_t T, int E, int k,
                                                                  int normalize, float* __restrict__ dlogits) {
  extern __shared__ float rows[];                           // [tokens of the block][E + 1]
  const int tb = blockDim.x;                                // tokens (= threads) per block
  const int64_t t0 = (int64_t)blockIdx.x * tb;
  const int nt = (int)((T - t0) < tb ? (T - t0) : tb);
  const int ld = E + 1;
  for (int i = threadIdx.x; i < nt * E; i += tb) rows[(i / E) * ld + i % E] = logits[t0 * E + i];
  __syncthreads();
  float own_mx = 0.f, own_inv = 0.f, own_c1 = 0.f, own_S = 1.f;
  if ((int)threadIdx.x < nt) {
    const int64_t t = t0 + threadIdx.x;
    float* row = rows + threadIdx.x * ld;
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
    // every entry's -p_e c now; the chosen experts' own terms are added once the block's rows are in memory, from the
    // logits re-read at the k chosen entries
    for (int e = 0; e < E; ++e) row[e] = -(expf(row[e] - mx) * inv) * c;
    own_mx = mx; own_inv = inv; own_c1 = c1; own_S = S;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < nt * E; i += tb) dlogits[t0 * E + i] = rows[(i / E) * ld + i % E];
  __syncthreads();                                          // the rows are in memory, visible to the whole block
  if ((int)threadIdx.x < nt) {
    const int64_t t = t0 + threadIdx.x;
    for (int j = 0; j < k; ++j) {                            // the chosen experts of a token are distinct
      const int e = idx[t * k + j];
      if ((unsigned)e >= (unsigned)E) continue;
      const float g = expf(logits[t * E + e] - own_mx) * own_inv;
      dlogits[t * E + e] += g * ((dgate_w[t * k + j] - own_c1) / own_S);
    }
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

// partial[s][m][e] = sum over the tokens of slice s (ascending) of x[t,m] dlogits[t,e], and (blocks of the first row
// pieces) pbias[s][e] = sum over the slice of dlogits[t,e].  A thread owns one 16-byte piece of the rows (N consecutive m)
// and EC experts; a slice is walked in runs of 64 tokens whose dlogits go through LDS, rows fetched 16 at a time.
template <typename ET, int EC>
__global__ __launch_bounds__(kDwThreads) void gate_dw_partial_kernel(const uint4* __restrict__ x, const float* __restrict__ dlogits,
                                                                     int64_t T, int cpr, int E, int slice_len,
                                                                     float* __restrict__ partial, float* __restrict__ pbias) {
  constexpr int N = Vec16<ET>::N;
  __shared__ float dls[kDwSlice][EC];
  const int e0 = blockIdx.x * EC;                           // expert chunk fastest: the blocks that share rows of x run together
  const int64_t s = blockIdx.y;
  const int piece = blockIdx.z * kDwThreads + threadIdx.x;
  const bool live = piece < cpr;
  float acc[N][EC];
#pragma unroll
  for (int u = 0; u < N; ++u)
#pragma unroll
    for (int i = 0; i < EC; ++i) acc[u][i] = 0.f;
  float bsum = 0.f;                                         // threads 0 .. EC-1 of the first piece block: column sums
  for (int sub = 0; sub < slice_len; sub += kDwSlice) {
    const int64_t t0 = s * slice_len + sub;
    __syncthreads();                                        // the previous run's dlogits have been read
    for (int i = threadIdx.x; i < kDwSlice * EC; i += kDwThreads) {
      const int tt = i / EC, ei = i % EC;
      dls[tt][ei] = (t0 + tt < T && e0 + ei < E) ? dlogits[(t0 + tt) * E + e0 + ei] : 0.f;   // zeros past T add nothing
    }
    __syncthreads();
    if (blockIdx.z == 0 && threadIdx.x < EC) {
#pragma unroll 8
      for (int tt = 0; tt < kDwSlice; ++tt) bsum += dls[tt][threadIdx.x];
    }
    if (!live || t0 >= T) continue;
    for (int tb = 0; tb < kDwSlice; tb += 16) {
      uint4 xr[16];
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int64_t t = t0 + tb + q;
        xr[q] = x[(t < T ? t : T - 1) * cpr + piece];       // past T: a valid row, multiplied by zeros
      }
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        float xv[N];
        Vec16<ET>::unpack(xr[q], xv);
#pragma unroll
        for (int u = 0; u < N; ++u)
#pragma unroll
          for (int i = 0; i < EC; ++i) acc[u][i] = fmaf(xv[u], dls[tb + q][i], acc[u][i]);
      }
    }
  }
  if (blockIdx.z == 0 && threadIdx.x < EC && e0 + threadIdx.x < E) pbias[s * E + e0 + threadIdx.x] = bsum;
  if (!live) return;
  const int64_t M = (int64_t)cpr * N;
#pragma unroll
  for (int u = 0; u < N; ++u) {
    float* dst = partial + ((int64_t)s * M + (int64_t)piece * N + u) * E + e0;
    if ((E % EC) == 0) {                                    // EC experts = EC * 4 contiguous, 16-byte aligned bytes
#pragma unroll
      for (int i = 0; i < EC; i += 4)
        reinterpret_cast<float4*>(dst)[i / 4] = make_float4(acc[u][i], acc[u][i + 1], acc[u][i + 2], acc[u][i + 3]);
    } else {
#pragma unroll
      for (int i = 0; i < EC; ++i)
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

// dbias[e] = sum over slices, in slice order, of pbias[s][e]
__global__ __launch_bounds__(256) void gate_dbias_reduce_kernel(const float* __restrict__ pbias, int E, int slices,
                                                                float* __restrict__ dbias) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= E) return;
  float s = 0.f;
  int k = 0;
  for (; k + 8 <= slices; k += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = pbias[(int64_t)(k + u) * E + e];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  for (; k < slices; ++k) s += pbias[(int64_t)k * E + e];
  dbias[e] = s;
}

// dst [rows, Ep] bf16 = src [rows, E] (fp32 or bf16) with the columns E .. Ep-1 zero; Ep a multiple of 8.  One thread
// per 8 output columns.  Operands of the matrix-core product below (its reduction runs in steps of 64 experts).
template <typename ST>
__global__ __launch_bounds__(256) void pad_to_bf16_kernel(const ST* __restrict__ src, int64_t rows, int E, int Ep,
                                                          uint4* __restrict__ dst) {
  const int gpr = Ep / 8;
  const int64_t n = rows * gpr;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / gpr;
    const int e0 = (int)(i % gpr) * 8;
    float f[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) f[u] = e0 + u < E ? load_as_f32<ST>(src + r * E + e0 + u) : 0.f;
    dst[i] = Vec16<uint16_t>::pack(f);
  }
}

// Tokens per partial sum: 64 up to 16384 tokens, then as many as keep the number of slices at 256 (the partial sums
// are written and read once, so their size is what the reduction costs).
inline int64_t dw_slice_len(int64_t T) { return kDwSlice * (ceil_div(T, (int64_t)kDwSlice * 256) > 1 ? ceil_div(T, (int64_t)kDwSlice * 256) : 1); }

}  // namespace

size_t gate_backward_workspace_bytes(int64_t T, int64_t M, int64_t E) {
  const size_t slices = (size_t)ceil_div(T, dw_slice_len(T));
  return align_up((size_t)T * E * 4, 256) + align_up(slices * M * E * 4, 256) + align_up(slices * E * 4, 256) +
         align_up((size_t)T * (ceil_div(E, 64) * 64) * 2, 256) + align_up((size_t)M * (ceil_div(E, 64) * 64) * 2, 256);
  // dlogits, partial dWg, partial dbias; dlogits and Wg in bf16 with the experts padded to a multiple of 64
}

template <typename ET>
static hipError_t gate_backward_t(const void* x, const void* Wg, const float* logits, const int32_t* idx, const float* dgate_w,
                                  int normalize, int64_t T, int64_t M, int64_t E, int k, char* ws, void* dx, int accumulate_dx,
                                  void* dWg, float* dbias, float* dlogits_out, hipStream_t s) {
  const int64_t slice_len = dw_slice_len(T);
  const int slices = (int)ceil_div(T, slice_len);
  float* dl = dlogits_out ? dlogits_out : (float*)ws;
  float* partial = (float*)(ws + align_up((size_t)T * E * 4, 256));
  float* pbias = (float*)(ws + align_up((size_t)T * E * 4, 256) + align_up((size_t)slices * M * E * 4, 256));
  hipError_t err;
  const int gb_tokens = E <= 240 ? kGbTokens : 16;              // LDS rows: at most 61 KB (gates up to 240 experts) or 33 KB
  gate_backward_kernel<<<dim3((unsigned)ceil_div(T, gb_tokens)), dim3(gb_tokens), (size_t)gb_tokens * (E + 1) * sizeof(float), s>>>(
      logits, idx, dgate_w, T, (int)E, k, normalize, dl);
  if ((err = hipGetLastError()) != hipSuccess) return err;
  // Wide bf16 gates: dx (+)= dlogits Wg^T is a [T,E] x [E,M] product, run on the matrix cores with dlogits rounded to
  // bf16 (Wg [M,E] is the transposed operand as stored; the accumulate form adds dx in the epilogue).  The reduction
  // runs in steps of 64 experts: other expert counts get zero-padded copies of both operands.
  const int64_t Ep = ceil_div(E, 64) * 64;
  const bool dx_mfma = dx && sizeof(ET) == 2 && E >= 32 && M % 256 == 0 && (reinterpret_cast<uintptr_t>(Wg) & 15) == 0 &&
                       grouped_gemm_mfma_supports_nt(T, Ep, M);
  if (dx_mfma) {
    char* extra = ws + align_up((size_t)T * E * 4, 256) + align_up((size_t)slices * M * E * 4, 256) + align_up((size_t)slices * E * 4, 256);
    uint16_t* dl16 = (uint16_t*)extra;
    uint16_t* wg16 = (uint16_t*)(extra + align_up((size_t)T * Ep * 2, 256));
    auto blocks_for = [](int64_t n) { const int64_t b = ceil_div(n, 256 * 4); return (unsigned)(b < 8192 ? (b > 0 ? b : 1) : 8192); };
    pad_to_bf16_kernel<float><<<dim3(blocks_for(T * Ep / 8)), dim3(256), 0, s>>>(dl, T, (int)E, (int)Ep, (uint4*)dl16);
    if ((err = hipGetLastError()) != hipSuccess) return err;
    const void* wgt = Wg;
    if (Ep != E) {
      pad_to_bf16_kernel<uint16_t><<<dim3(blocks_for(M * Ep / 8)), dim3(256), 0, s>>>((const uint16_t*)Wg, M, (int)E, (int)Ep, (uint4*)wg16);
      if ((err = hipGetLastError()) != hipSuccess) return err;
      wgt = wg16;
    }
    if ((err = launch_grouped_gemm_mfma_nt(dl16, wgt, nullptr, 1, T, Ep, M, dx, accumulate_dx ? dx : nullptr, -1, s)) != hipSuccess) return err;
  } else if (dx) {
    const int cpr = (int)(M * sizeof(ET) / 16);
    gate_dx_kernel<ET><<<dim3((unsigned)ceil_div(T, kDxTokens), (unsigned)ceil_div(cpr, 256)), dim3(256), 0, s>>>(dl, (const ET*)Wg, T, cpr, (int)E, accumulate_dx, (uint4*)dx);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  if (dWg || dbias) {
    // the partial sums serve both: one pass over x and dlogits (without dWg only the first row pieces are visited)
    const int cprx = dWg ? (int)(M * sizeof(ET) / 16) : 0;        // no row pieces: x and the partial sums stay untouched
    const unsigned zblocks = dWg ? (unsigned)ceil_div(cprx, kDwThreads) : 1u;
    if (E > 8)
      gate_dw_partial_kernel<ET, 16><<<dim3((unsigned)ceil_div(E, 16), (unsigned)slices, zblocks), dim3(kDwThreads), 0, s>>>(
          (const uint4*)x, dl, T, cprx, (int)E, (int)slice_len, partial, pbias);
    else
      gate_dw_partial_kernel<ET, 8><<<dim3(1, (unsigned)slices, zblocks), dim3(kDwThreads), 0, s>>>(
          (const uint4*)x, dl, T, cprx, (int)E, (int)slice_len, partial, pbias);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  if (dWg) {
    const int64_t n = M * E;
    gate_dw_reduce_kernel<ET><<<dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s>>>(partial, n, slices, (ET*)dWg);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  if (dbias) {
    gate_dbias_reduce_kernel<<<dim3((unsigned)ceil_div(E, 256)), dim3(256), 0, s>>>(pbias, (int)E, slices, dbias);
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
