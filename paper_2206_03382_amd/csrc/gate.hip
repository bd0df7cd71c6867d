// Gating function and capacity-limited slot assignment (arXiv 2206.03382 Sec. 2.1, Eq. 1; Appendix B names the
// location scan).  Four kernels:
//   gate_logits_kernel : logits = x * Wg + bias on the fp64 matrix cores (order-independent after rounding to fp32)
//   gate_topk_kernel   : per token softmax + k rounds of (value, index) argmax in a sub-wave group; per-block,
//                        per-rank, per-expert arrival counters
//   gate_scan_kernel   : per expert, exclusive scan of the counters in arrival order (rank, block); totals;
//                        marks unfilled slots of slot_src with -1
//   gate_assign_kernel : per token and rank, position inside its block + scanned offset -> loc, slot_src
// No order-dependent atomics: every integer output is a pure function of the logits.
#include "common.h"

namespace moe {

typedef __attribute__((ext_vector_type(4))) double f64x4;

// ---------------------------------------------------------------------------------------------------------------
// logits[t,e] = sum_m x[t,m] Wg[m,e] + bias[e], fp64 accumulate (v_mfma_f64_16x16x4_f64), one rounding to fp32.
// A wave owns 16 tokens and NT tiles of 16 experts.  Operand layout of the instruction: A lane l holds
// (row l%16, k l/16), B lane l holds (k l/16, col l%16), D lane l register v holds (row 4v + l/16, col l%16).
// A lane keeps 8 consecutive x values (k = kq*8 .. kq*8+7 of a 32-wide chunk); MFMA step s uses k = kq*8+s for
// both operands, so the chunk's 32 k-values are covered exactly once.
// ---------------------------------------------------------------------------------------------------------------
// Eight consecutive x values of one lane, kept raw while in flight and widened when used.
template <typename XT> struct Raw8;
template <> struct Raw8<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float* p) { a = *reinterpret_cast<const float4*>(p); b = *reinterpret_cast<const float4*>(p + 4); }
  __device__ __forceinline__ void zero() { a = make_float4(0.f, 0.f, 0.f, 0.f); b = a; }
  __device__ __forceinline__ void widen(float (&v)[8]) const {
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
};
template <> struct Raw8<uint16_t> {
  uint4 a;
  __device__ __forceinline__ void load(const uint16_t* p) { a = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void zero() { a = make_uint4(0, 0, 0, 0); }
  __device__ __forceinline__ void widen(float (&v)[8]) const {
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

template <typename XT, int NT>
__global__ __launch_bounds__(256) void gate_logits_kernel(const XT* __restrict__ x, const XT* __restrict__ Wg,
                                                          const float* __restrict__ bias, int64_t T, int M, int E,
                                                          int e_base, float* __restrict__ logits) {
  // Wg is staged through LDS as fp64 in chunks of BK rows (32 KB whatever NT is).  x goes straight from global memory
  // to registers; with one wave per SIMD nothing else hides its latency, so each lane keeps PF passes (PF * 32 k) of
  // its row in flight in a register ring.
  constexpr int EN = NT * 16, BK = 4096 / EN, PF = 8;
  static_assert((PF * 32) % BK == 0, "LDS chunks must tile the register ring");
  __shared__ double wlds[BK][EN];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int m = lane & 15, kq = lane >> 4;
  const int64_t t0 = ((int64_t)blockIdx.x * 4 + wave) * 16;
  const int64_t trow = (t0 + m < T) ? (t0 + m) : (T - 1);
  const XT* xrow = x + trow * (int64_t)M + kq * 8;
  f64x4 acc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) acc[nt] = f64x4{0.0, 0.0, 0.0, 0.0};

  // this thread's 16 elements of a Wg chunk, fetched one chunk ahead so that their latency hides behind the MFMAs
  constexpr int WPT = BK * EN / 256;
  XT wraw[WPT];
  auto wg_fetch = [&](int kchunk) {
#pragma unroll
    for (int i = 0; i < WPT; ++i) {
      const int id = threadIdx.x + i * 256, kk = kchunk + id / EN, e = e_base + id % EN;
      wraw[i] = (kk < M && e < E) ? Wg[(int64_t)kk * E + e] : XT(0);
    }
  };
  wg_fetch(0);

  Raw8<XT> ring[PF];
#pragma unroll
  for (int j = 0; j < PF; ++j) {
    if (j * 32 + kq * 8 < M) ring[j].load(xrow + j * 32); else ring[j].zero();
  }

  for (int kbase = 0; kbase < M; kbase += PF * 32) {
#pragma unroll
    for (int j = 0; j < PF; ++j) {
      const int k0 = kbase + j * 32;                   // this pass covers k0 .. k0+31 (uniform across the block)
      if (k0 >= M) break;
      if ((j * 32) % BK == 0) {                        // refill the LDS chunk of Wg that starts here
        __syncthreads();
#pragma unroll
        for (int i = 0; i < WPT; ++i) {
          const int id = threadIdx.x + i * 256;
          wlds[id / EN][id % EN] = (double)load_as_f32<XT>(&wraw[i]);
        }
        __syncthreads();
        wg_fetch(k0 + BK);
      }
      float xv[8];
      ring[j].widen(xv);
      const int kn = k0 + PF * 32 + kq * 8;            // refill the ring slot with the pass PF ahead
      if (kn < M) ring[j].load(xrow + k0 + PF * 32); else ring[j].zero();
      const int r0 = (j * 32) % BK + kq * 8;
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const double a = (double)xv[s];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          const double b = wlds[r0 + s][nt * 16 + m];
          acc[nt] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[nt], 0, 0, 0);
        }
      }
    }
  }
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int e = e_base + nt * 16 + m;
    if (e >= E) continue;
    const double be = bias ? (double)bias[e] : 0.0;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int64_t t = t0 + 4 * v + kq;
      if (t < T) logits[t * E + e] = (float)(acc[nt][v] + be);
    }
  }
}

template <typename XT>
static hipError_t launch_gate_logits_t(const XT* x, const XT* Wg, const float* bias, int64_t T, int64_t M, int64_t E,
                                       float* logits, hipStream_t s) {
  const dim3 grid((unsigned)ceil_div(T, 64)), block(256);
  for (int64_t e_base = 0; e_base < E; e_base += 128) {
    const int64_t rem = E - e_base;
    if (rem <= 16) gate_logits_kernel<XT, 1><<<grid, block, 0, s>>>(x, Wg, bias, T, (int)M, (int)E, (int)e_base, logits);
    else if (rem <= 32) gate_logits_kernel<XT, 2><<<grid, block, 0, s>>>(x, Wg, bias, T, (int)M, (int)E, (int)e_base, logits);
    else if (rem <= 64) gate_logits_kernel<XT, 4><<<grid, block, 0, s>>>(x, Wg, bias, T, (int)M, (int)E, (int)e_base, logits);
    else gate_logits_kernel<XT, 8><<<grid, block, 0, s>>>(x, Wg, bias, T, (int)M, (int)E, (int)e_base, logits);
  }
  return hipGetLastError();
}

hipError_t launch_gate_logits(const void* x, const void* Wg, const float* bias, int dtype, int64_t T, int64_t M,
                              int64_t E, float* logits, hipStream_t s) {
  if (dtype == MOE_F32) return launch_gate_logits_t<float>((const float*)x, (const float*)Wg, bias, T, M, E, logits, s);
  return launch_gate_logits_t<uint16_t>((const uint16_t*)x, (const uint16_t*)Wg, bias, T, M, E, logits, s);
}

// ---------------------------------------------------------------------------------------------------------------
// softmax + top-k.  A group of G lanes (power of two, <= 64) owns one token; lane gl holds experts gl, gl+G, ...
// (V per lane).  Selection is k rounds of argmax on (value, index): larger value wins, equal values -> lower
// index, so the result is unique and independent of the reduction tree.
// ---------------------------------------------------------------------------------------------------------------
template <int V>
__global__ __launch_bounds__(256) void gate_topk_kernel(const float* __restrict__ logits, int64_t T, int E, int k, int G,
                                                        int normalize, int32_t* __restrict__ idx,
                                                        float* __restrict__ gate_w, int32_t* __restrict__ block_counts,
                                                        int NB) {
  extern __shared__ int hist[];                        // [k][E] arrivals of this block's tokens
  for (int i = threadIdx.x; i < k * E; i += 256) hist[i] = 0;
  __syncthreads();
  const int groups = 256 / G, g = threadIdx.x / G, gl = threadIdx.x % G;
  const float NEG_INF = -__builtin_inff();
  const int passes = (kGateTokensPerBlock + groups - 1) / groups;
  for (int it = 0; it < passes; ++it) {
    const int tb = it * groups + g;                    // token of this block handled by this lane group in this pass
    const int64_t t = (int64_t)blockIdx.x * kGateTokensPerBlock + tb;
    const bool valid = tb < kGateTokensPerBlock && t < T;
    float v[V];
#pragma unroll
    for (int vi = 0; vi < V; ++vi) {
      const int e = gl + G * vi;
      v[vi] = (valid && e < E) ? logits[t * E + e] : NEG_INF;
    }
    float mx = v[0];
#pragma unroll
    for (int vi = 1; vi < V; ++vi) mx = fmaxf(mx, v[vi]);
    for (int off = G >> 1; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    float se = 0.f;
#pragma unroll
    for (int vi = 0; vi < V; ++vi) se += expf(v[vi] - mx);
    for (int off = G >> 1; off >= 1; off >>= 1) se += __shfl_xor(se, off);

    int si[V];
    float sw[V];
#pragma unroll
    for (int vi = 0; vi < V; ++vi) { si[vi] = 0; sw[vi] = 0.f; }
    float denom = 0.f;
    for (int j = 0; j < k; ++j) {
      float bv = v[0];
      int be = gl;
#pragma unroll
      for (int vi = 1; vi < V; ++vi)
        if (v[vi] > bv) { bv = v[vi]; be = gl + G * vi; }
      for (int off = G >> 1; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(bv, off);
        const int oe = __shfl_xor(be, off);
        if (ov > bv || (ov == bv && oe < be)) { bv = ov; be = oe; }
      }
      be = be < E ? be : E - 1;                        // only reachable with non-finite logits; keeps indices in range
      const float pj = expf(bv - mx) / se;
      denom += pj;
#pragma unroll
      for (int vi = 0; vi < V; ++vi) {
        if (be == gl + G * vi) v[vi] = NEG_INF;        // the chosen expert leaves the pool
        if (j == gl + G * vi) { si[vi] = be; sw[vi] = pj; }
      }
      if (valid && gl == 0) atomicAdd(&hist[j * E + be], 1);
    }
    if (valid) {
#pragma unroll
      for (int vi = 0; vi < V; ++vi) {
        const int j = gl + G * vi;
        if (j < k) {
          idx[t * k + j] = si[vi];
          gate_w[t * k + j] = normalize ? sw[vi] / denom : sw[vi];
        }
      }
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < k * E; i += 256) {
    const int j = i / E, e = i % E;
    block_counts[((int64_t)j * NB + blockIdx.x) * E + e] = hist[i];
  }
}

// One block per expert: exclusive scan of block_counts[(j, b), e] over (j, b) in place; totals -> counts[e];
// slots [min(total, C), C) of slot_src[e] are marked unfilled.
__global__ __launch_bounds__(256) void gate_scan_kernel(int32_t* __restrict__ block_counts, int L, int E, int64_t C,
                                                        int32_t* __restrict__ counts, int32_t* __restrict__ slot_src) {
  __shared__ int part[256];
  const int e = blockIdx.x, tid = threadIdx.x;
  const int per = (L + 255) / 256;
  const int start = min(tid * per, L), stop = min(start + per, L);
  int sum = 0;
  for (int i = start; i < stop; ++i) sum += block_counts[(int64_t)i * E + e];
  part[tid] = sum;
  __syncthreads();
  for (int off = 1; off < 256; off <<= 1) {            // inclusive Hillis-Steele scan of the 256 partial sums
    const int add = (tid >= off) ? part[tid - off] : 0;
    __syncthreads();
    part[tid] += add;
    __syncthreads();
  }
  int run = part[tid] - sum;
  for (int i = start; i < stop; ++i) {
    const int c = block_counts[(int64_t)i * E + e];
    block_counts[(int64_t)i * E + e] = run;
    run += c;
  }
  const int total = part[255];
  if (tid == 0) counts[e] = total;
  if (slot_src) {
    const int64_t first = total < C ? total : C;
    for (int64_t c = first + tid; c < C; c += 256) slot_src[(int64_t)e * C + c] = -1;
  }
}

// One wave per block of 64 tokens, one lane per token: position among the block's earlier tokens with the same
// (rank, expert), found by grouping the lanes by expert with ballots (one round per distinct expert in the wave).
__global__ __launch_bounds__(kGateTokensPerBlock) void gate_assign_kernel(const int32_t* __restrict__ idx,
                                                                          const int32_t* __restrict__ block_off, int64_t T,
                                                                          int E, int k, int64_t C, int NB,
                                                                          int32_t* __restrict__ loc,
                                                                          int32_t* __restrict__ slot_src) {
  const int lane = threadIdx.x;
  const int64_t t = (int64_t)blockIdx.x * kGateTokensPerBlock + lane;
  const bool valid = t < T;
  const unsigned long long below = (1ull << lane) - 1ull;
  for (int j = 0; j < k; ++j) {
    const int e = valid ? idx[t * k + j] : -1;
    unsigned long long remaining = __ballot(valid);
    int r = 0;
    while (remaining) {
      const int leader = __ffsll((long long)remaining) - 1;
      const int e0 = __shfl(e, leader);
      const unsigned long long same = __ballot(valid && e == e0);
      if (e == e0) r = __popcll(same & below);
      remaining &= ~same;
    }
    if (valid) {
      const int l = block_off[((int64_t)j * NB + blockIdx.x) * E + e] + r;
      loc[t * k + j] = l;
      if (slot_src && l < C) slot_src[(int64_t)e * C + l] = (int32_t)t;
    }
  }
}

hipError_t launch_gate_topk(const float* logits, int64_t T, int64_t E, int k, int64_t C, int normalize, int32_t* idx,
                            float* gate_w, int32_t* loc, int32_t* counts, int32_t* slot_src, int32_t* block_counts,
                            hipStream_t s) {
  const int NB = (int)ceil_div(T, kGateTokensPerBlock);
  int G = 1;
  while (G < E && G < 64) G <<= 1;
  const int V = (int)ceil_div(E, G);
  const size_t shmem = (size_t)k * E * sizeof(int);
  const dim3 grid(NB), block(256);
  if (V == 1) gate_topk_kernel<1><<<grid, block, shmem, s>>>(logits, T, (int)E, k, G, normalize, idx, gate_w, block_counts, NB);
  else if (V == 2) gate_topk_kernel<2><<<grid, block, shmem, s>>>(logits, T, (int)E, k, G, normalize, idx, gate_w, block_counts, NB);
  else if (V <= 4) gate_topk_kernel<4><<<grid, block, shmem, s>>>(logits, T, (int)E, k, G, normalize, idx, gate_w, block_counts, NB);
  else gate_topk_kernel<8><<<grid, block, shmem, s>>>(logits, T, (int)E, k, G, normalize, idx, gate_w, block_counts, NB);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  gate_scan_kernel<<<dim3((unsigned)E), block, 0, s>>>(block_counts, k * NB, (int)E, C, counts, slot_src);
  err = hipGetLastError();
  if (err != hipSuccess) return err;
  gate_assign_kernel<<<grid, dim3(kGateTokensPerBlock), 0, s>>>(idx, block_counts, T, (int)E, k, C, NB, loc, slot_src);
  return hipGetLastError();
}

}  // namespace moe
