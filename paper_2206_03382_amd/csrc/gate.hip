// Gating function and capacity-limited slot assignment (arXiv 2206.03382 Sec. 2.1, Eq. 1; Appendix B names the
// location scan).  Four kernels:
//   gate_logits_kernel : logits = x * Wg + bias on the fp64 matrix cores (order-independent after rounding to fp32)
//   gate_topk_kernel   : per token softmax + k rounds of (value, index) argmax in a sub-wave group; per-block,
//                        per-rank, per-expert arrival counters
//   gate_scan_kernel   : per expert, exclusive scan of the counters in arrival order (rank, block); totals;
//                        marks unfilled slots of slot_src with -1
//   gate_assign_kernel : per token and rank, position inside its block + scanned offset -> loc, slot_src
// No order-dependent atomics: every integer output is a pure function of the logits.
// Further down: the dynamic capacity factor and slot sources for a capacity chosen after routing (Sec. 4.1), the cosine
// router (Appendix), and the token order of batch prioritized routing (Sec. 3.2 / Appendix ablation).
#include "common.h"

namespace moe {

// token tiles (of 16) per wave for gates of at most 16 experts: 4 measured best on MI355X (2: +5 %, 1: +10 % time)
constexpr int kNarrowGateTilesPerWave = 4;
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
  __device__ __forceinline__ void keep_if(uint32_t m) {            // m = all ones keeps the values, 0 makes them +0
    a.x = __uint_as_float(__float_as_uint(a.x) & m); a.y = __uint_as_float(__float_as_uint(a.y) & m);
    a.z = __uint_as_float(__float_as_uint(a.z) & m); a.w = __uint_as_float(__float_as_uint(a.w) & m);
    b.x = __uint_as_float(__float_as_uint(b.x) & m); b.y = __uint_as_float(__float_as_uint(b.y) & m);
    b.z = __uint_as_float(__float_as_uint(b.z) & m); b.w = __uint_as_float(__float_as_uint(b.w) & m);
  }
  __device__ __forceinline__ void widen(float (&v)[8]) const {
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
};
template <> struct Raw8<uint16_t> {
  uint4 a;
  __device__ __forceinline__ void load(const uint16_t* p) { a = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void zero() { a = make_uint4(0, 0, 0, 0); }
  __device__ __forceinline__ void keep_if(uint32_t m) { a.x &= m; a.y &= m; a.z &= m; a.w &= m; }
  __device__ __forceinline__ void widen(float (&v)[8]) const {
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

template <typename XT, int NT, int KS, int TW, bool VECW>
__global__ __launch_bounds__(256) void gate_logits_kernel(const XT* __restrict__ x, const XT* __restrict__ Wg,
                                                          const float* __restrict__ bias, int64_t T, int M, int Mq, int E,
                                                          int e_base, float* __restrict__ logits) {
  // The block's four waves are 4/KS token groups times KS splits of the reduction; a wave owns TW tiles of 16 tokens.
  // Split ks owns k in [ks*Mq, (ks+1)*Mq) (Mq a multiple of BKW); the partial sums are added in split order at the
  // end.  Narrow gates (few experts) have one accumulator tile per 16 tokens, a serial chain of dependent MFMAs: TW
  // token tiles per wave and several waves per SIMD give the matrix pipe independent chains to interleave, and the
  // TW tiles share every Wg operand read.
  // Wg is staged through LDS as fp64, BKW rows per split at a time (32 KB in all whatever NT is).  x goes straight
  // from global memory to registers through a ring of PF passes (PF * 32 k) per lane and token tile.
  constexpr int EN = NT * 16, ENP = EN + 1, BKW = 4096 / (KS * EN), PF = 8 / TW, TG = 4 / KS;
  static_assert(BKW % 32 == 0 && ((PF * 32) % BKW == 0 || BKW % (PF * 32) == 0), "LDS chunks must hold whole passes");
  // rows are padded by one double: the 64-byte pieces that the staging threads write and the 4 rows x 16 columns that
  // an MFMA operand read gathers then both spread evenly over the LDS banks
  __shared__ double wlds[KS * BKW * ENP];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ks = wave % KS, tg = wave / KS;
  const int m = lane & 15, kq = lane >> 4;
  const int64_t t0 = ((int64_t)blockIdx.x * TG + tg) * (16 * TW);
  const int kfirst = ks * Mq;                                       // first k of this wave's split
  const XT* xrow[TW];
#pragma unroll
  for (int w = 0; w < TW; ++w) {
    const int64_t t = t0 + w * 16 + m;
    xrow[w] = x + (t < T ? t : T - 1) * (int64_t)M + kfirst + kq * 8;
  }
  f64x4 acc[TW][NT];
#pragma unroll
  for (int w = 0; w < TW; ++w)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[w][nt] = f64x4{0.0, 0.0, 0.0, 0.0};

  // this thread's part of a Wg chunk (rows kl .. kl+BKW-1 of every split), fetched one chunk ahead so that its latency
  // hides behind the MFMAs.  VECW (E a multiple of the 16-byte vector, Wg 16-byte aligned): 16-byte pieces of a row;
  // otherwise single elements.
  constexpr int VEC = VECW ? 16 / (int)sizeof(XT) : 1;
  constexpr int WPT = KS * BKW * EN / (256 * VEC);
  constexpr int WORDS = VECW ? 4 : 1;                  // raw 32-bit words of one piece
  static_assert(WPT >= 1, "every thread stages at least one piece");
  uint32_t wraw[WPT][WORDS];
  // branch-free (dead pieces re-read the start of Wg and are masked to zero): a load inside a divergent branch would be
  // waited for on the spot, together with every x load in flight
  auto wg_fetch = [&](int kl) {
#pragma unroll
    for (int i = 0; i < WPT; ++i) {
      const int id = (threadIdx.x + i * 256) * VEC, q = id / (BKW * EN), r = (id / EN) % BKW, e = e_base + id % EN;
      const int kk = q * Mq + kl + r;
      const bool live = kl + r < Mq && kk < M && e < E;
      const XT* src = Wg + (live ? (int64_t)kk * E + e : 0);
      const uint32_t keep = live ? 0xffffffffu : 0u;
      if (VECW) {
        const uint4 v = *reinterpret_cast<const uint4*>(src);
        wraw[i][0] = v.x & keep; wraw[i][WORDS > 1 ? 1 : 0] = v.y & keep; wraw[i][WORDS > 2 ? 2 : 0] = v.z & keep;
        wraw[i][WORDS > 3 ? 3 : 0] = v.w & keep;
      } else if (sizeof(XT) == 2) {
        wraw[i][0] = (uint32_t)*reinterpret_cast<const uint16_t*>(src) & keep;
      } else {
        wraw[i][0] = *reinterpret_cast<const uint32_t*>(src) & keep;
      }
    }
  };
  auto wg_stage = [&]() {
#pragma unroll
    for (int i = 0; i < WPT; ++i) {
      const int id = (threadIdx.x + i * 256) * VEC;
      double* dst = wlds + (id / EN) * ENP + id % EN;
      if (sizeof(XT) == 2) {                           // bf16: even element in the low half of a word
        if (VECW) {
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            dst[2 * u] = (double)__uint_as_float(wraw[i][u % WORDS] << 16);
            dst[2 * u + 1] = (double)__uint_as_float(wraw[i][u % WORDS] & 0xffff0000u);
          }
        } else dst[0] = (double)__uint_as_float(wraw[i][0] << 16);
      } else {
#pragma unroll
        for (int u = 0; u < VEC; ++u) dst[u] = (double)__uint_as_float(wraw[i][u % WORDS]);
      }
    }
  };
  wg_fetch(0);

  Raw8<XT> ring[TW][PF];
#pragma unroll
  for (int j = 0; j < PF; ++j)
#pragma unroll
    for (int w = 0; w < TW; ++w) {
      const bool live = j * 32 + kq * 8 < Mq && kfirst + j * 32 + kq * 8 < M;
      ring[w][j].load(xrow[w] + (live ? j * 32 : -(kfirst + kq * 8)));       // dead lanes re-read the row's start
      ring[w][j].keep_if(live ? 0xffffffffu : 0u);
    }

  const double* wmine = wlds + ks * BKW * ENP;
  for (int kbase = 0; kbase < Mq; kbase += PF * 32) {
#pragma unroll
    for (int j = 0; j < PF; ++j) {
      const int kl = kbase + j * 32;                   // this pass covers kl .. kl+31 of the split (uniform across the block)
      if (kl >= Mq) break;
      if (kl % BKW == 0) {                             // refill the LDS chunk of Wg that starts here
        __syncthreads();
        wg_stage();
        __syncthreads();
        wg_fetch(kl + BKW);
      }
      float xv[TW][8];
      const int kn = kl + PF * 32 + kq * 8;            // refill the ring slot with the pass PF ahead
#pragma unroll
      for (int w = 0; w < TW; ++w) {
        ring[w][j].widen(xv[w]);
        // branch-free (dead lanes re-read the row's start), so that the compiler can count the loads in flight and
        // the wait for the next Wg chunk does not drain this prefetch
        const bool live = kn < Mq && kfirst + kn < M;
        ring[w][j].load(xrow[w] + (live ? kl + PF * 32 : -(kfirst + kq * 8)));
        ring[w][j].keep_if(live ? 0xffffffffu : 0u);
      }
      const int r0 = kl % BKW + kq * 8;
#pragma unroll
      for (int s = 0; s < 8; ++s) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          const double b = wmine[(r0 + s) * ENP + nt * 16 + m];
#pragma unroll
          for (int w = 0; w < TW; ++w) acc[w][nt] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)xv[w][s], b, acc[w][nt], 0, 0, 0);
        }
      }
    }
  }
  if (KS > 1) {                                        // partial sums of splits 1 .. KS-1 go through LDS to split 0
    double* red = wlds;                                // [KS-1][TG][TW][NT][64 lanes][4]
    static_assert((KS - 1) * TG * TW * NT * 256 <= KS * BKW * ENP, "the partial sums must fit into the staging buffer");
    __syncthreads();
    if (ks > 0) {
#pragma unroll
      for (int w = 0; w < TW; ++w)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int v = 0; v < 4; ++v) red[(((((ks - 1) * TG + tg) * TW + w) * NT + nt) * 64 + lane) * 4 + v] = acc[w][nt][v];
    }
    __syncthreads();
    if (ks > 0) return;
#pragma unroll
    for (int q = 1; q < KS; ++q)
#pragma unroll
      for (int w = 0; w < TW; ++w)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int v = 0; v < 4; ++v) acc[w][nt][v] += red[(((((q - 1) * TG + tg) * TW + w) * NT + nt) * 64 + lane) * 4 + v];
  }
#pragma unroll
  for (int w = 0; w < TW; ++w)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int e = e_base + nt * 16 + m;
      if (e >= E) continue;
      const double be = bias ? (double)bias[e] : 0.0;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int64_t t = t0 + w * 16 + 4 * v + kq;
        if (t < T) logits[t * E + e] = (float)(acc[w][nt][v] + be);
      }
    }
}

template <typename XT, int NT, int KS, int TW>
static void launch_gate_logits_one(const XT* x, const XT* Wg, const float* bias, int64_t T, int64_t M, int64_t E,
                                   int64_t e_base, float* logits, hipStream_t s) {
  constexpr int BKW = 4096 / (KS * NT * 16);
  const int Mq = (int)(ceil_div(ceil_div(M, KS), BKW) * BKW);       // k per split, a whole number of LDS chunks
  const dim3 grid((unsigned)ceil_div(T, 16 * TW * (4 / KS))), block(256);
  constexpr int VEC = 16 / (int)sizeof(XT);
  const bool vecw = E % VEC == 0 && e_base % VEC == 0 && ((uintptr_t)Wg & 15) == 0;
  if (vecw) gate_logits_kernel<XT, NT, KS, TW, true><<<grid, block, 0, s>>>(x, Wg, bias, T, (int)M, Mq, (int)E, (int)e_base, logits);
  else gate_logits_kernel<XT, NT, KS, TW, false><<<grid, block, 0, s>>>(x, Wg, bias, T, (int)M, Mq, (int)E, (int)e_base, logits);
}

template <typename XT>
static hipError_t launch_gate_logits_t(const XT* x, const XT* Wg, const float* bias, int64_t T, int64_t M, int64_t E,
                                       float* logits, hipStream_t s) {
  for (int64_t e_base = 0; e_base < E; e_base += 128) {
    const int64_t rem = E - e_base;
    if (rem <= 16) launch_gate_logits_one<XT, 1, 4, kNarrowGateTilesPerWave>(x, Wg, bias, T, M, E, e_base, logits, s);
    else if (rem <= 32) launch_gate_logits_one<XT, 2, 4, 2>(x, Wg, bias, T, M, E, e_base, logits, s);
    else if (rem <= 64) launch_gate_logits_one<XT, 4, 2, 2>(x, Wg, bias, T, M, E, e_base, logits, s);
    else launch_gate_logits_one<XT, 8, 1, 1>(x, Wg, bias, T, M, E, e_base, logits, s);
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
__global__ __launch_bounds__(1024) void gate_topk_kernel(const float* __restrict__ logits, int64_t T, int E, int k, int G,
                                                        int normalize, int32_t* __restrict__ idx,
                                                        float* __restrict__ gate_w, int32_t* __restrict__ block_counts,
                                                        int NB, const int32_t* __restrict__ perm) {
  extern __shared__ int hist[];                        // [k][E] arrivals of this block's tokens
  for (int i = threadIdx.x; i < k * E; i += blockDim.x) hist[i] = 0;
  __syncthreads();
  const int groups = blockDim.x / G, g = threadIdx.x / G, gl = threadIdx.x % G;   // blockDim.x is a multiple of 64 >= G
  const float NEG_INF = -__builtin_inff();
  const int passes = (kGateTokensPerBlock + groups - 1) / groups;
  for (int it = 0; it < passes; ++it) {
    const int tb = it * groups + g;                    // token of this block handled by this lane group in this pass
    const int64_t tv = (int64_t)blockIdx.x * kGateTokensPerBlock + tb;   // position in arrival order
    const bool valid = tb < kGateTokensPerBlock && tv < T;
    int64_t t = tv;                                                     // the token that arrives at that position
    if (valid && perm) { const int32_t p = perm[tv]; t = ((uint32_t)p < (uint64_t)T) ? p : tv; }   // clamp: never out of range
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
  for (int i = threadIdx.x; i < k * E; i += blockDim.x) {
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
                                                                          int32_t* __restrict__ slot_src,
                                                                          const int32_t* __restrict__ perm) {
  const int lane = threadIdx.x;
  const int64_t tv = (int64_t)blockIdx.x * kGateTokensPerBlock + lane;   // position in arrival order
  const bool valid = tv < T;
  int64_t t = tv;
  if (valid && perm) { const int32_t p = perm[tv]; t = ((uint32_t)p < (uint64_t)T) ? p : tv; }
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
                            hipStream_t s, const int32_t* perm) {
  const int NB = (int)ceil_div(T, kGateTokensPerBlock);
  // lane group per token: up to 16 experts one value per lane; from there on 16 lanes with up to 8 values each (4 tokens
  // per wave and 4 cross-lane steps per reduction instead of 6), and a whole wave beyond 128 experts
  int G = 1;
  while (G < E && G < 16) G <<= 1;
  if (E > 128) G = 64;
  const int V = (int)ceil_div(E, G);
  const size_t shmem = (size_t)k * E * sizeof(int);
  // one lane group per token: as many threads as the block's 64 tokens need, so that (up to 16 experts) every token's
  // logits are fetched in one round instead of one dependent round trip per pass
  const dim3 grid(NB), block(256);
  const dim3 tblock((unsigned)(64 * G < 256 ? 256 : (64 * G > 1024 ? 1024 : 64 * G)));
  if (V == 1) gate_topk_kernel<1><<<grid, tblock, shmem, s>>>(logits, T, (int)E, k, G, normalize, idx, gate_w, block_counts, NB, perm);
  else if (V == 2) gate_topk_kernel<2><<<grid, tblock, shmem, s>>>(logits, T, (int)E, k, G, normalize, idx, gate_w, block_counts, NB, perm);
  else if (V <= 4) gate_topk_kernel<4><<<grid, tblock, shmem, s>>>(logits, T, (int)E, k, G, normalize, idx, gate_w, block_counts, NB, perm);
  else gate_topk_kernel<8><<<grid, tblock, shmem, s>>>(logits, T, (int)E, k, G, normalize, idx, gate_w, block_counts, NB, perm);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  gate_scan_kernel<<<dim3((unsigned)E), block, 0, s>>>(block_counts, k * NB, (int)E, C, counts, slot_src);
  err = hipGetLastError();
  if (err != hipSuccess) return err;
  gate_assign_kernel<<<grid, dim3(kGateTokensPerBlock), 0, s>>>(idx, block_counts, T, (int)E, k, C, NB, loc, slot_src, perm);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------------
// Dynamic capacity factor (Sec. 4.1): out[0] = capacity to use, out[1] = needed capacity = max_e counts[e].
// bound > 0: capacity that the factor's upper bound gives (setting < 0); bound = 0: no upper bound (setting = 0).
// ---------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void dynamic_capacity_kernel(const int32_t* __restrict__ counts, int E, int64_t bound,
                                                               int64_t fixed, int64_t* __restrict__ out,
                                                               int32_t* __restrict__ fills) {
  // fixed > 0: that capacity whatever the arrivals are (a static factor); else the needed capacity, at most `bound`
  // (if bound > 0).  fills (optional): min(counts[e], chosen capacity) per expert.
  __shared__ int part[4];
  __shared__ int64_t chosen;
  int m = 0;
  for (int e = threadIdx.x; e < E; e += 256) m = max(m, counts[e]);
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) m = max(m, __shfl_xor(m, d, 64));
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    const int64_t needed = max(max(part[0], part[1]), max(part[2], part[3]));
    int64_t C = fixed > 0 ? fixed : needed;
    if (bound > 0 && C > bound) C = bound;
    if (C < 1) C = 1;                                   // an empty layer still has one (unfilled) slot per expert
    out[0] = C;
    out[1] = needed;
    chosen = C;
  }
  __syncthreads();
  if (fills) {
    const int64_t C = chosen;
    for (int e = threadIdx.x; e < E; e += 256) {
      const int64_t c = counts[e];
      fills[e] = (int32_t)(c < C ? (c > 0 ? c : 0) : C);
    }
  }
}

hipError_t launch_dynamic_capacity(const int32_t* counts, int64_t E, int64_t bound, int64_t* out, hipStream_t s,
                                   int64_t fixed, int32_t* fills) {
  dynamic_capacity_kernel<<<dim3(1), dim3(256), 0, s>>>(counts, (int)E, bound, fixed, out, fills);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------------
// slot_src[e,c] for a capacity chosen after the arrivals were counted: -1 everywhere, then every kept choice writes
// its token (loc is unique per expert, so no two writes meet).
// ---------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fill_i32_kernel(int32_t* __restrict__ p, int64_t n, int32_t v) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = v;
}

// C_dev (optional): the capacity chosen on the device; slots then sit `stride` apart per expert (the caller's bound)
__global__ __launch_bounds__(256) void slot_sources_kernel(const int32_t* __restrict__ idx, const int32_t* __restrict__ loc,
                                                           int64_t pairs, int k, int E, int64_t C, int64_t stride,
                                                           const int64_t* __restrict__ C_dev,
                                                           int32_t* __restrict__ slot_src) {
  if (C_dev) { const int64_t c = *C_dev; C = c < C ? c : C; }
  for (int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x; p < pairs; p += (int64_t)gridDim.x * 256) {
    const int e = idx[p], l = loc[p];
    if (l >= 0 && l < C && (unsigned)e < (unsigned)E) slot_src[(int64_t)e * stride + l] = (int32_t)(p / k);
  }
}

hipError_t launch_slot_sources(const int32_t* idx, const int32_t* loc, int64_t T, int64_t E, int k, int64_t C,
                               int32_t* slot_src, hipStream_t s, const int64_t* C_dev) {
  const int64_t n = E * C, fb = ceil_div(n, 256 * 4);
  fill_i32_kernel<<<dim3((unsigned)(fb < 8192 ? fb : 8192)), dim3(256), 0, s>>>(slot_src, n, -1);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  const int64_t pairs = T * k, sb = ceil_div(pairs, 256);
  slot_sources_kernel<<<dim3((unsigned)(sb < 8192 ? sb : 8192)), dim3(256), 0, s>>>(idx, loc, pairs, k, (int)E, C, C, C_dev, slot_src);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------------
// Cosine router (Appendix, "A New Cosine Router"): logits[t,e] = cos(W x_t, M_e) / tau.  The projection W x runs on the
// fp64 matrix-core kernel above (rounded once to fp32); the cosine itself is a handful of fp64 operations per pair.
// ---------------------------------------------------------------------------------------------------------------
// One block per expert: MeT[d][e] = Me[e][d] widened to fp64, norm[e] = max(||Me[e]||, 1e-12).
__global__ __launch_bounds__(256) void cosine_prepare_kernel(const float* __restrict__ Me, int E, int D,
                                                             double* __restrict__ MeT, double* __restrict__ norm) {
  __shared__ double part[256];
  const int e = blockIdx.x;
  double s = 0.0;
  for (int d = threadIdx.x; d < D; d += 256) {
    const double v = (double)Me[(int64_t)e * D + d];
    MeT[(int64_t)d * E + e] = v;
    s += v * v;
  }
  part[threadIdx.x] = s;
  __syncthreads();
  for (int off = 128; off >= 1; off >>= 1) {              // fixed tree: the same sum on every run
    if (threadIdx.x < off) part[threadIdx.x] += part[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) norm[e] = fmax(sqrt(part[0]), 1e-12);
}

// One wave per token, one lane per expert: the token's projection is fetched 64 values at a time and broadcast lane by
// lane; every lane accumulates its expert's dot product and the token's squared norm in fp64, in ascending d.
__global__ __launch_bounds__(256) void cosine_logits_kernel(const float* __restrict__ proj, const double* __restrict__ MeT,
                                                            const double* __restrict__ norm, double tau, int64_t T, int D,
                                                            int E, float* __restrict__ logits) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  for (int64_t t = wave; t < T; t += nwaves) {
    for (int e0 = 0; e0 < E; e0 += 64) {
      const int e = e0 + lane;
      const int ec = e < E ? e : E - 1;                   // lanes past the last expert repeat it and store nothing
      double dot = 0.0, nx2 = 0.0;
      for (int d0 = 0; d0 < D; d0 += 64) {
        const float pv = (d0 + lane < D) ? proj[t * D + d0 + lane] : 0.f;
        const int n = (D - d0) < 64 ? (D - d0) : 64;
        for (int dd = 0; dd < n; ++dd) {
          const double sd = (double)__uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(pv), dd));
          dot = fma(sd, MeT[(int64_t)(d0 + dd) * E + ec], dot);
          nx2 = fma(sd, sd, nx2);
        }
      }
      if (e < E) logits[t * E + e] = (float)((dot / (fmax(sqrt(nx2), 1e-12) * norm[e])) / tau);
    }
  }
}

hipError_t launch_gate_logits_cosine(const void* x, const void* Wp, const float* Me, double tau, int dtype, int64_t T,
                                     int64_t M, int64_t D, int64_t E, float* logits, float* proj, double* MeT, double* norm,
                                     hipStream_t s) {
  hipError_t err = launch_gate_logits(x, Wp, nullptr, dtype, T, M, D, proj, s);
  if (err != hipSuccess) return err;
  cosine_prepare_kernel<<<dim3((unsigned)E), dim3(256), 0, s>>>(Me, (int)E, (int)D, MeT, norm);
  err = hipGetLastError();
  if (err != hipSuccess) return err;
  const int64_t blocks = ceil_div(T, 4);
  cosine_logits_kernel<<<dim3((unsigned)(blocks < 16384 ? blocks : 16384)), dim3(256), 0, s>>>(proj, MeT, norm, tau, T, (int)D, (int)E, logits);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------------
// Batch prioritized routing (named in Sec. 3.2 and the Appendix's routing ablation): tokens take their slots in order
// of decreasing priority, priority = the token's largest routing probability 1 / sum_e exp(l_e - l_max), computed in
// fp64 and rounded to fp32 so that the order is a decision on an exactly comparable key; ties -> lower token.
// ---------------------------------------------------------------------------------------------------------------
// The sort key is one 64-bit integer per token: the fp32 priority's bit pattern (priorities are positive, so the
// pattern orders like the value) above the complemented token index, so that "goes before" is a single comparison.
__global__ __launch_bounds__(256) void bpr_key_kernel(const float* __restrict__ logits, int64_t T, int E,
                                                      uint64_t* __restrict__ key) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  const float* row = logits + t * E;
  float mx = row[0];
  for (int e = 1; e < E; ++e) mx = fmaxf(mx, row[e]);
  double se = 0.0;
  for (int e = 0; e < E; ++e) se += exp((double)row[e] - (double)mx);
  const float prio = (float)(1.0 / se);
  key[t] = ((uint64_t)__float_as_uint(prio) << 32) | (uint64_t)(0xffffffffu - (uint32_t)t);
}

// Position of every token in the order by counting the tokens that go before it: O(T^2) comparisons, exact and
// deterministic (integer atomics).  Block (x, y) counts, for 256 tokens, the keys of slice y that are larger.
constexpr int kBprSlice = 2048;
__global__ __launch_bounds__(256) void bpr_count_kernel(const uint64_t* __restrict__ key, int64_t T, int32_t* __restrict__ before) {
  __shared__ uint64_t tile[kBprSlice];
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t base = (int64_t)blockIdx.y * kBprSlice;
  for (int i = threadIdx.x; i < kBprSlice; i += 256) tile[i] = base + i < T ? key[base + i] : 0ull;   // 0 is below every key
  __syncthreads();
  if (t >= T) return;
  const uint64_t mine = key[t];
  int n = 0;
#pragma unroll 16
  for (int i = 0; i < kBprSlice; ++i) n += tile[i] > mine ? 1 : 0;
  if (n) atomicAdd(&before[t], n);
}

__global__ __launch_bounds__(256) void bpr_scatter_kernel(const int32_t* __restrict__ before, int64_t T, int32_t* __restrict__ perm) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t < T && (uint32_t)before[t] < (uint64_t)T) perm[before[t]] = (int32_t)t;
}

hipError_t launch_bpr_order(const float* logits, int64_t T, int64_t E, uint64_t* key, int32_t* before, int32_t* perm,
                            hipStream_t s) {
  const dim3 grid((unsigned)ceil_div(T, 256)), block(256);
  bpr_key_kernel<<<grid, block, 0, s>>>(logits, T, (int)E, key);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  fill_i32_kernel<<<dim3((unsigned)ceil_div(T, 1024)), block, 0, s>>>(before, T, 0);
  err = hipGetLastError();
  if (err != hipSuccess) return err;
  bpr_count_kernel<<<dim3((unsigned)ceil_div(T, 256), (unsigned)ceil_div(T, kBprSlice)), block, 0, s>>>(key, T, before);
  err = hipGetLastError();
  if (err != hipSuccess) return err;
  bpr_scatter_kernel<<<grid, block, 0, s>>>(before, T, perm);
  return hipGetLastError();
}

}  // namespace moe
