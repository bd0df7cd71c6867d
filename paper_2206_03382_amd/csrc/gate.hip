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
// Value of the partner lane in one step of a reduction over a group of lanes.  Steps 1 and 2 swap within quads, steps 4
// and 8 read the mirrored lane of the other half of 8 / 16 lanes (data-parallel primitives, no LDS traffic); the mirror
// is as good as an xor partner wherever the lanes of each half already agree, which holds in a reduction whose steps run
// in ascending order.  Steps 16 and 32 go through the cross-lane permute.
template <int OFF> __device__ __forceinline__ int group_partner(int v) {
  if constexpr (OFF == 1) return __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, false);        // quad_perm [1,0,3,2]
  else if constexpr (OFF == 2) return __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, false);   // quad_perm [2,3,0,1]
  else if constexpr (OFF == 4) return __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, false);  // row_half_mirror
  else if constexpr (OFF == 8) return __builtin_amdgcn_update_dpp(0, v, 0x140, 0xf, 0xf, false);  // row_mirror
  else return __shfl_xor(v, OFF, 64);
}
template <int OFF> __device__ __forceinline__ float group_partner(float v) {
  return __int_as_float(group_partner<OFF>(__float_as_int(v)));
}

template <int G> __device__ __forceinline__ float group_max(float v) {
  if constexpr (G > 1) v = fmaxf(v, group_partner<1>(v));
  if constexpr (G > 2) v = fmaxf(v, group_partner<2>(v));
  if constexpr (G > 4) v = fmaxf(v, group_partner<4>(v));
  if constexpr (G > 8) v = fmaxf(v, group_partner<8>(v));
  if constexpr (G > 16) v = fmaxf(v, group_partner<16>(v));
  if constexpr (G > 32) v = fmaxf(v, group_partner<32>(v));
  return v;
}
template <int G> __device__ __forceinline__ float group_sum(float v) {
  if constexpr (G > 1) v += group_partner<1>(v);
  if constexpr (G > 2) v += group_partner<2>(v);
  if constexpr (G > 4) v += group_partner<4>(v);
  if constexpr (G > 8) v += group_partner<8>(v);
  if constexpr (G > 16) v += group_partner<16>(v);
  if constexpr (G > 32) v += group_partner<32>(v);
  return v;
}
template <int OFF> __device__ __forceinline__ void argmax_step(float& bv, int& be) {
  const float ov = group_partner<OFF>(bv);
  const int oe = group_partner<OFF>(be);
  if (ov > bv || (ov == bv && oe < be)) { bv = ov; be = oe; }
}
template <int G> __device__ __forceinline__ void group_argmax(float& bv, int& be) {
  if constexpr (G > 1) argmax_step<1>(bv, be);
  if constexpr (G > 2) argmax_step<2>(bv, be);
  if constexpr (G > 4) argmax_step<4>(bv, be);
  if constexpr (G > 8) argmax_step<8>(bv, be);
  if constexpr (G > 16) argmax_step<16>(bv, be);
  if constexpr (G > 32) argmax_step<32>(bv, be);
}

// The decisions of one token, taken by its group of G lanes on v[vi] = logit of expert gl + G vi (-inf past E; consumed).
// Slot vi of lane gl receives choice j = gl + G vi: si = expert, sw = its softmax probability (not yet renormalised);
// denom = the sum of the k probabilities.  With `check` the k + 1 largest values are ordered and the result says whether
// some pair of neighbours is closer than `tol2` (twice the error bound of the logits) plus rounding slack (two units in
// the last place of the larger one); theta = the smallest value looked at.
template <int G, int V>
__device__ __forceinline__ bool token_topk(float (&v)[V], int gl, int E, int k, bool check, float tol2, int (&si)[V], float (&sw)[V],
                                           float& denom, float& theta) {
  const float NEG_INF = -__builtin_inff();
  float mx = v[0];
#pragma unroll
  for (int vi = 1; vi < V; ++vi) mx = fmaxf(mx, v[vi]);
  mx = group_max<G>(mx);
  float se = 0.f;
#pragma unroll
  for (int vi = 0; vi < V; ++vi) se += expf(v[vi] - mx);
  se = group_sum<G>(se);
#pragma unroll
  for (int vi = 0; vi < V; ++vi) { si[vi] = 0; sw[vi] = 0.f; }
  denom = 0.f;
  bool close = false;
  float prev = 0.f;
  const int rounds = (check && k < E) ? k + 1 : k;
  for (int j = 0; j < rounds; ++j) {
    float bv = v[0];
    int be = gl;
#pragma unroll
    for (int vi = 1; vi < V; ++vi)
      if (v[vi] > bv) { bv = v[vi]; be = gl + G * vi; }
    group_argmax<G>(bv, be);
    be = be < E ? be : E - 1;                          // only reachable with non-finite logits; keeps indices in range
    if (check && j > 0) close = close || !(prev - bv > tol2 + 4.8e-7f * fmaxf(fabsf(prev), fabsf(bv)));
    prev = bv;
    theta = bv;
#pragma unroll
    for (int vi = 0; vi < V; ++vi)
      if (be == gl + G * vi) v[vi] = NEG_INF;          // the chosen expert leaves the pool
    if (j < k) {
      const float pj = expf(bv - mx) / se;
      denom += pj;
#pragma unroll
      for (int vi = 0; vi < V; ++vi)
        if (j == gl + G * vi) { si[vi] = be; sw[vi] = pj; }
    }
  }
  return close;
}

// The ballot of a predicate over this lane's group of G lanes (G = 16: four groups per wave; G = 64: the wave)
template <int G> __device__ __forceinline__ unsigned long long group_ballot(bool p, int grp) {
  const unsigned long long b = __ballot(p);
  return G == 64 ? b : (b >> (G * grp)) & ((1ull << (G & 63)) - 1ull);
}

// sum over m of x[t, m] * Wt[e, m] in fp64 by a group of G lanes, for two experts at once (every product of two bf16
// values is exact in fp32; lane gl adds the 16-byte pieces gl, gl + G, ... in ascending order, then a fixed butterfly adds
// the G partial sums); all lanes of the group get both sums.  Four pieces are fetched per round so that their latencies
// overlap.
template <int G>
__device__ __forceinline__ void group_dot2_fp64(const uint16_t* __restrict__ xr, const uint16_t* __restrict__ wa,
                                                const uint16_t* __restrict__ wb, int M, int gl, double& sa, double& sb) {
  double acc_a = 0.0, acc_b = 0.0;
  const int pieces = M >> 3;
  for (int p0 = 0; p0 < pieces; p0 += 4 * G) {
    uint4 xv[4], av[4], bv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int p = p0 + G * u + gl;
      const int q = p < pieces ? p : 0;                  // pieces past the row's end re-read its start and are zeroed
      xv[u] = *reinterpret_cast<const uint4*>(xr + q * 8);
      av[u] = *reinterpret_cast<const uint4*>(wa + q * 8);
      bv[u] = *reinterpret_cast<const uint4*>(wb + q * 8);
      if (p >= pieces) xv[u] = make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t xa[4] = {xv[u].x, xv[u].y, xv[u].z, xv[u].w};
      const uint32_t aa[4] = {av[u].x, av[u].y, av[u].z, av[u].w};
      const uint32_t ba[4] = {bv[u].x, bv[u].y, bv[u].z, bv[u].w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float xl = __uint_as_float(xa[q] << 16), xh = __uint_as_float(xa[q] & 0xffff0000u);
        acc_a += (double)(xl * __uint_as_float(aa[q] << 16));
        acc_a += (double)(xh * __uint_as_float(aa[q] & 0xffff0000u));
        acc_b += (double)(xl * __uint_as_float(ba[q] << 16));
        acc_b += (double)(xh * __uint_as_float(ba[q] & 0xffff0000u));
      }
    }
  }
#pragma unroll
  for (int d = G / 2; d >= 1; d >>= 1) {
    acc_a += __shfl_xor(acc_a, d, 64);
    acc_b += __shfl_xor(acc_b, d, 64);
  }
  sa = acc_a;
  sb = acc_b;
}

// Exact decisions for one token whose approximate logits (within tol2 / 2 of the exactly rounded ones) left its top k
// open; run by a group of G lanes (a wave, or a quarter of one for gates of at most 128 experts: four tokens are then
// repaired side by side).  theta = the (k+1)-th largest approximate logit.  Every expert that can still reach the top k
// (approximate logit within tol2 of theta) is looked at; those that have another such expert within tol2 get their logit
// recomputed in fp64 from x and Wt and stored (an expert farther than that from every other keeps its place whatever the
// true values are); then the token is decided again on the repaired row.  hist: the block's packed arrival counters.
// `on` = this group has a token (groups without one run along with nothing to do).
template <int G>
__device__ __forceinline__ void repair_token(bool on, int64_t t, float theta, float tol2, int lane, float* __restrict__ logits,
                                             int E, int k, int normalize, int32_t* __restrict__ idx, float* __restrict__ gate_w,
                                             int* hist, const uint16_t* __restrict__ x, const uint16_t* __restrict__ Wt,
                                             const float* __restrict__ bias, int M, int Mp) {
  const float NEG_INF = -__builtin_inff();
  const int grp = lane / G, gl = lane % G;
  const float reach = theta - tol2 - 4.8e-7f * fabsf(theta);         // experts below this cannot be among the k largest
  float rv[8];
#pragma unroll
  for (int vi = 0; vi < 8; ++vi) {
    const int e = gl + G * vi;
    rv[vi] = (on && e < E) ? logits[t * E + e] : NEG_INF;
  }
  bool need[8];
#pragma unroll
  for (int vi = 0; vi < 8; ++vi) need[vi] = false;
#pragma unroll
  for (int vi = 0; vi < 8; ++vi) {
    unsigned long long todo = group_ballot<G>(on && rv[vi] >= reach, grp);
    while (todo) {
      const int l = __builtin_ctzll(todo);
      todo &= todo - 1;
      const float val = __shfl(rv[vi], grp * G + l, 64);
      bool near = false;
#pragma unroll
      for (int vj = 0; vj < 8; ++vj)
        near = near || (rv[vj] >= reach && !(vj == vi && gl == l) &&
                        fabsf(rv[vj] - val) <= tol2 + 4.8e-7f * fmaxf(fabsf(rv[vj]), fabsf(val)));
      if (group_ballot<G>(near, grp) != 0ull && gl == l) need[vi] = true;
    }
  }
  // the marked experts, two at a time (one pending until its partner turns up)
  const uint16_t* xr = x + (on ? t : 0) * (int64_t)M;
  int pend_e = -1, pend_l = 0, pend_vi = 0;
  auto put = [&](int e, int l, int vi, double sum) __attribute__((always_inline)) {
    const float val = (float)(sum + (bias ? (double)bias[e] : 0.0));
#pragma unroll
    for (int vj = 0; vj < 8; ++vj)
      if (vj == vi && gl == l) rv[vj] = val;
    if (gl == l) logits[t * E + e] = val;
  };
#pragma unroll
  for (int vi = 0; vi < 8; ++vi) {
    unsigned long long todo = group_ballot<G>(need[vi], grp);
    while (todo) {
      const int l = __builtin_ctzll(todo);
      todo &= todo - 1;
      const int e = l + G * vi;
      if (pend_e < 0) { pend_e = e; pend_l = l; pend_vi = vi; continue; }
      double sa, sb;
      group_dot2_fp64<G>(xr, Wt + (int64_t)pend_e * Mp, Wt + (int64_t)e * Mp, M, gl, sa, sb);
      put(pend_e, pend_l, pend_vi, sa);
      put(e, l, vi, sb);
      pend_e = -1;
    }
  }
  if (pend_e >= 0) {
    double sa, sb;
    group_dot2_fp64<G>(xr, Wt + (int64_t)pend_e * Mp, Wt + (int64_t)pend_e * Mp, M, gl, sa, sb);
    put(pend_e, pend_l, pend_vi, sa);
  }
  int si[8];
  float sw[8], denom, th;
  token_topk<G, 8>(rv, gl, E, k, false, 0.f, si, sw, denom, th);
  if (on) {
#pragma unroll
    for (int vi = 0; vi < 8; ++vi) {
      const int j = gl + G * vi;
      if (j < k) {
        idx[t * k + j] = si[vi];
        gate_w[t * k + j] = normalize ? sw[vi] / denom : sw[vi];
        atomicAdd(&hist[(j * E + si[vi]) >> 2], 1 << (8 * ((j * E + si[vi]) & 3)));
      }
    }
  }
}

// One block per 64 tokens (in arrival order).  Phase 1: every token's decisions from its logits.  With `margin` (the
// logits came from the fast kernel and are only known to within margin[t]) a token whose k + 1 largest logits are not
// separated by more than twice that bound is set aside.  Phase 2: one wave per token set aside repairs it (repair_token):
// the decisions then equal those taken on exactly rounded logits.  Phase 3: the block's per-(rank, expert) arrival counters go to memory.
template <int G, int V>
__global__ __launch_bounds__(1024) void gate_topk_kernel(float* __restrict__ logits, int64_t T, int E, int k,
                                                        int normalize, int32_t* __restrict__ idx,
                                                        float* __restrict__ gate_w, int32_t* __restrict__ block_counts,
                                                        int NB, const int32_t* __restrict__ perm,
                                                        const float* __restrict__ margin, const uint16_t* __restrict__ x,
                                                        const uint16_t* __restrict__ Wt, const float* __restrict__ bias,
                                                        int M, int Mp) {
  extern __shared__ int smem_i[];
  // [k][E] arrivals of this block's tokens: at most 64 each, so four 8-bit counters share a word (integer atomics on the
  // word: the sums do not depend on the order)
  int* hist = smem_i;
  const int hist_words = (k * E + 3) >> 2;
  int* aside_tok = smem_i + hist_words;                // [64] block-local tokens set aside
  float* aside_theta = reinterpret_cast<float*>(aside_tok + kGateTokensPerBlock);
  int* aside_n = aside_tok + 2 * kGateTokensPerBlock;
  for (int i = threadIdx.x; i < hist_words; i += blockDim.x) hist[i] = 0;
  if (threadIdx.x == 0) *aside_n = 0;
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
    int si[V];
    float sw[V], denom, theta;
    const bool check = margin != nullptr;
    const float tol2 = (check && valid) ? 2.0f * margin[t] : 0.f;
    bool publish = valid;
    const bool close = token_topk<G, V>(v, gl, E, k, check, tol2, si, sw, denom, theta);
    if (check && valid && close) {                     // uniform over the token's lanes
      publish = false;
      if (gl == 0) {
        const int slot = atomicAdd(aside_n, 1);
        aside_tok[slot] = tb;
        aside_theta[slot] = theta;
      }
    }
    if (publish) {
#pragma unroll
      for (int vi = 0; vi < V; ++vi) {
        const int j = gl + G * vi;
        if (j < k) {
          idx[t * k + j] = si[vi];
          gate_w[t * k + j] = normalize ? sw[vi] / denom : sw[vi];
          atomicAdd(&hist[(j * E + si[vi]) >> 2], 1 << (8 * ((j * E + si[vi]) & 3)));
        }
      }
    }
  }
  __syncthreads();
  if (margin) {
    const int n_aside = *aside_n;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    for (int i = wave; i < n_aside; i += nwaves)
      repair_token<64>(true, (int64_t)blockIdx.x * kGateTokensPerBlock + aside_tok[i], aside_theta[i],
                       2.0f * margin[(int64_t)blockIdx.x * kGateTokensPerBlock + aside_tok[i]], lane, logits, E, k, normalize, idx,
                       gate_w, hist, x, Wt, bias, M, Mp);
    __syncthreads();
  }
  for (int i = threadIdx.x; i < k * E; i += blockDim.x) {
    const int j = i / E, e = i % E;
    block_counts[((int64_t)e * k + j) * NB + blockIdx.x] = (hist[i >> 2] >> (8 * (i & 3))) & 0xff;
  }
}

// softmax + top-k with one lane per token, for k <= 32: the kernel of choice for wide gates.  A wave owns 64 consecutive
// tokens (one block of the arrival counters).  Its logits pass through LDS 32 experts at a time (rows padded to 33 words:
// the transposed reads are conflict-free); every lane walks its own row in ascending expert order and keeps the N = KMAX+1
// largest values seen so far, sorted, in registers: a new value moves in above every smaller one (strictly smaller: an
// equal value met later, i.e. a higher index, stays below) and the entries from there on shift down by one, so the list ends as the top k in the order the selection
// rule asks for, and its (k+1)-th entry serves the near-tie check.  The softmax denominator is kept chunk by chunk
// relative to the running maximum.  The four waves of a block work independently (no barrier).
template <int KMAX, bool VEC4>
__global__ __launch_bounds__(256) void gate_topk_lane_kernel(float* __restrict__ logits, int64_t T, int E, int k, int normalize,
                                                             int32_t* __restrict__ idx, float* __restrict__ gate_w,
                                                             int32_t* __restrict__ block_counts, int NB,
                                                             const float* __restrict__ margin, const uint16_t* __restrict__ x,
                                                             const uint16_t* __restrict__ Wt, const float* __restrict__ bias,
                                                             int M, int Mp) {
  constexpr int N = KMAX + 1, CW = 32, LDW = CW + 1;
  extern __shared__ int smem_i[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int hist_words = (k * E + 3) >> 2;
  const int per_wave = kGateTokensPerBlock * LDW + hist_words;
  float* tile = reinterpret_cast<float*>(smem_i + wave * per_wave);   // [64 tokens][33]
  int* hist = smem_i + wave * per_wave + kGateTokensPerBlock * LDW;   // packed [k][E] arrival counters of this wave's tokens
  const int b = blockIdx.x * 4 + wave;                                // block of 64 tokens
  if (b >= NB) return;                                                // waves are independent: no barrier below
  const int64_t t0 = (int64_t)b * kGateTokensPerBlock;
  const int64_t t = t0 + lane;
  const bool valid = t < T;
  const float NEG_INF = -__builtin_inff();
  for (int i = lane; i < hist_words; i += 64) hist[i] = 0;

  float L[N];
  int I[N];
#pragma unroll
  for (int i = 0; i < N; ++i) { L[i] = NEG_INF; I[i] = 0x7fffffff; }
  float mx = NEG_INF, se = 0.f;
  for (int e0 = 0; e0 < E; e0 += CW) {
    // tile[row][c] = logits[t0 + row][e0 + c]  (-inf outside the matrix)
    if (VEC4) {                                                        // E % 4 == 0: 16-byte pieces, 8 rows x 128 bytes per load
      const int c4 = (lane & 7) * 4;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int row = (lane >> 3) + 8 * i;
        float4 v = make_float4(NEG_INF, NEG_INF, NEG_INF, NEG_INF);
        if (t0 + row < T && e0 + c4 < E) v = *reinterpret_cast<const float4*>(logits + (t0 + row) * E + e0 + c4);
        float* d = tile + row * LDW + c4;
        d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
      }
    } else {
      const int c = lane & 31;
#pragma unroll 8
      for (int i = 0; i < 32; ++i) {
        const int row = (lane >> 5) + 2 * i;
        tile[row * LDW + c] = (t0 + row < T && e0 + c < E) ? logits[(t0 + row) * E + e0 + c] : NEG_INF;
      }
    }
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);                                // lgkmcnt(0): the tile is in LDS before any lane reads it
    float row[CW];
#pragma unroll
    for (int c = 0; c < CW; ++c) row[c] = tile[lane * LDW + c];
    float cm = row[0];
#pragma unroll
    for (int c = 1; c < CW; ++c) cm = fmaxf(cm, row[c]);
    if (cm > mx) { se *= __expf(mx - cm); mx = cm; }                   // (0 * exp(-inf) = 0 on the first chunk)
#pragma unroll
    for (int c = 0; c < CW; ++c) {
      float v = row[c];
      int e = e0 + c;
      se += __expf(v - mx);
      bool g = false;                                                  // once the value has moved in, everything below shifts down
#pragma unroll
      for (int i = 0; i < N; ++i) {
        g = g || v > L[i];
        const float tv = g ? L[i] : v;
        const int ti = g ? I[i] : e;
        L[i] = g ? v : L[i];
        I[i] = g ? e : I[i];
        v = tv;
        e = ti;
      }
    }
    __builtin_amdgcn_wave_barrier();                                   // every lane has read its row before the next chunk lands
  }
  // near-tie check on the k + 1 largest
  bool close = false;
  const bool check = margin != nullptr;
  const float tol2 = (check && valid) ? 2.0f * margin[t] : 0.f;
  float theta = NEG_INF;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    if (i < k || (i == k && k < E)) {
      theta = L[i];
      if (check && i > 0) close = close || !(L[i - 1] - L[i] > tol2 + 4.8e-7f * fmaxf(fabsf(L[i - 1]), fabsf(L[i])));
    }
  }
  const bool aside = check && valid && close;
  if (valid && !aside) {
    float p[KMAX], denom = 0.f;
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
      p[j] = 0.f;
      if (j < k) { p[j] = expf(L[j] - mx) / se; denom += p[j]; }
    }
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
      if (j < k) {
        const int e = I[j] < E ? I[j] : E - 1;                         // only reachable with non-finite logits
        idx[t * k + j] = e;
        gate_w[t * k + j] = normalize ? p[j] / denom : p[j];
        atomicAdd(&hist[(j * E + e) >> 2], 1 << (8 * ((j * E + e) & 3)));
      }
    }
  }
  // the wave repairs its open tokens: four side by side, a quarter of the wave each, for gates of at most 128 experts
  // (their list goes through the tile's LDS, which is free now), one by one with the whole wave otherwise
  const unsigned long long open = __ballot(aside);
  if (open) {
    if (E <= 128) {
      int* list = reinterpret_cast<int*>(tile);
      if (aside) list[__popcll(open & ((1ull << lane) - 1ull))] = lane;
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_s_waitcnt(0xc07f);
      const int n_open = __popcll(open), grp = lane >> 4;
      for (int i0 = 0; i0 < n_open; i0 += 4) {
        const bool on = i0 + grp < n_open;
        const int src = on ? list[i0 + grp] : 0;
        repair_token<16>(on, t0 + src, __shfl(theta, src, 64), __shfl(tol2, src, 64), lane, logits, E, k, normalize, idx, gate_w, hist,
                         x, Wt, bias, M, Mp);
      }
    } else {
      unsigned long long todo = open;
      while (todo) {
        const int l = __builtin_ctzll(todo);
        todo &= todo - 1;
        repair_token<64>(true, t0 + l, __shfl(theta, l, 64), __shfl(tol2, l, 64), lane, logits, E, k, normalize, idx, gate_w, hist, x,
                         Wt, bias, M, Mp);
      }
    }
  }
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);
  for (int i = lane; i < k * E; i += 64) {
    const int j = i / E, e = i % E;
    block_counts[((int64_t)e * k + j) * NB + b] = (hist[i >> 2] >> (8 * (i & 3))) & 0xff;
  }
}

// One block per expert: exclusive scan of block_counts[e, (j, b)] (an expert's counters are contiguous, in arrival order
// (rank j, block b)) in place; totals -> counts[e];
// slots [min(total, C), C) of slot_src[e] are marked unfilled.
__global__ __launch_bounds__(256) void gate_scan_kernel(int32_t* __restrict__ block_counts, int L, int E, int64_t C,
                                                        int32_t* __restrict__ counts, int32_t* __restrict__ slot_src) {
  __shared__ int part[256];
  const int e = blockIdx.x, tid = threadIdx.x;
  const int per = (L + 255) / 256;
  const int start = min(tid * per, L), stop = min(start + per, L);
  int sum = 0;
  for (int i = start; i < stop; ++i) sum += block_counts[(int64_t)e * L + i];
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
    const int c = block_counts[(int64_t)e * L + i];
    block_counts[(int64_t)e * L + i] = run;
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
      const int l = block_off[((int64_t)e * k + j) * NB + blockIdx.x] + r;
      loc[t * k + j] = l;
      if (slot_src && l < C) slot_src[(int64_t)e * C + l] = (int32_t)t;
    }
  }
}

hipError_t launch_gate_topk(float* logits, int64_t T, int64_t E, int k, int64_t C, int normalize, int32_t* idx,
                            float* gate_w, int32_t* loc, int32_t* counts, int32_t* slot_src, int32_t* block_counts,
                            hipStream_t s, const int32_t* perm, const GateRepair* repair) {
  const int NB = (int)ceil_div(T, kGateTokensPerBlock);
  // lane group per token: up to 16 experts one value per lane; from there on 16 lanes with up to 8 logits each (4 tokens
  // per wave), and a whole wave beyond 128 experts
  int G = 1;
  while (G < E && G < 16) G <<= 1;
  if (E > 128) G = 64;
  const int V = (int)ceil_div(E, G);
  const size_t shmem = (((size_t)k * E + 3) / 4 + 2 * kGateTokensPerBlock + 1) * sizeof(int);
  // one lane group per token: as many threads as the block's 64 tokens need, so that (up to 16 experts) every token's
  // logits are fetched in one round instead of one dependent round trip per pass
  const dim3 grid(NB), block(256);
  const dim3 tblock((unsigned)(64 * G < 256 ? 256 : (64 * G > 1024 ? 1024 : 64 * G)));
  const float* margin = repair ? repair->margin : nullptr;
  const uint16_t* rx = repair ? (const uint16_t*)repair->x : nullptr;
  const uint16_t* rw = repair ? repair->Wt : nullptr;
  const float* rb = repair ? repair->bias : nullptr;
  const int rM = repair ? (int)repair->M : 0, rMp = repair ? (int)repair->Mp : 0;
#define MOE_TOPK(GG, VV) gate_topk_kernel<GG, VV><<<grid, tblock, shmem, s>>>(logits, T, (int)E, k, normalize, idx, gate_w, block_counts, NB, perm, margin, rx, rw, rb, rM, rMp)
#define MOE_TOPK_LANE(KM)                                                                                                     \
  do {                                                                                                                        \
    const size_t lsh = 4 * ((size_t)kGateTokensPerBlock * 33 + ((size_t)k * E + 3) / 4) * sizeof(int);                        \
    const dim3 lgrid((unsigned)ceil_div(NB, 4));                                                                              \
    if (E % 4 == 0) gate_topk_lane_kernel<KM, true><<<lgrid, block, lsh, s>>>(logits, T, (int)E, k, normalize, idx, gate_w, block_counts, NB, margin, rx, rw, rb, rM, rMp); \
    else gate_topk_lane_kernel<KM, false><<<lgrid, block, lsh, s>>>(logits, T, (int)E, k, normalize, idx, gate_w, block_counts, NB, margin, rx, rw, rb, rM, rMp); \
  } while (0)
  // wide gates with few choices: one lane per token (its LDS footprint, 4 waves x (8.25 KB + k E bytes), must fit 64 KB);
  // tokens in a caller-given order (perm) keep the lane-group kernel
  const bool lane_kernel = !perm && E > 16 && k <= 32 && (size_t)k * E <= 7936;
  if (lane_kernel) {
    if (k <= 1) MOE_TOPK_LANE(1); else if (k <= 2) MOE_TOPK_LANE(2); else if (k <= 4) MOE_TOPK_LANE(4);
    else if (k <= 8) MOE_TOPK_LANE(8); else if (k <= 16) MOE_TOPK_LANE(16); else MOE_TOPK_LANE(32);
  }
  else if (G == 1) MOE_TOPK(1, 1);
  else if (G == 2) MOE_TOPK(2, 1);
  else if (G == 4) MOE_TOPK(4, 1);
  else if (G == 8) MOE_TOPK(8, 1);
  else if (G == 16) { if (V == 1) MOE_TOPK(16, 1); else if (V == 2) MOE_TOPK(16, 2); else if (V <= 4) MOE_TOPK(16, 4); else MOE_TOPK(16, 8); }
  else { if (V <= 4) MOE_TOPK(64, 4); else MOE_TOPK(64, 8); }
#undef MOE_TOPK
#undef MOE_TOPK_LANE
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
// The sort key is the complement of the fp32 priority's bit pattern (priorities are positive, so the pattern orders like
// the value): ascending keys = descending priority.  A stable sort keeps equal priorities in token order.
__global__ __launch_bounds__(256) void bpr_key_kernel(const float* __restrict__ logits, int64_t T, int E,
                                                      uint32_t* __restrict__ key, int32_t* __restrict__ val) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  const float* row = logits + t * E;
  float mx = row[0];
  for (int e = 1; e < E; ++e) mx = fmaxf(mx, row[e]);
  double se = 0.0;
  for (int e = 0; e < E; ++e) se += exp((double)row[e] - (double)mx);
  const float prio = (float)(1.0 / se);
  key[t] = ~__float_as_uint(prio);
  val[t] = (int32_t)t;
}

// Stable least-significant-digit radix sort of (key, token) pairs, three passes of 11, 11 and 10 bits.  A block owns a
// tile of 2048 consecutive pairs.  Pass: per-tile digit histograms -> one exclusive scan over (digit, tile) -> stable
// scatter (a pair's place = start of its (digit, tile) run + the number of pairs of that digit before it in the tile).
// Integer arithmetic only; every result is a pure function of the keys.
constexpr int kSortTile = 2048, kSortBins = 2048;

__global__ __launch_bounds__(256) void radix_hist_kernel(const uint32_t* __restrict__ key, int64_t n, int shift, int bins, int tiles,
                                                         uint32_t* __restrict__ hist) {
  __shared__ uint32_t h[kSortBins];
  for (int i = threadIdx.x; i < bins; i += 256) h[i] = 0;
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * kSortTile;
  for (int i = threadIdx.x; i < kSortTile; i += 256)
    if (base + i < n) atomicAdd(&h[(key[base + i] >> shift) & (bins - 1)], 1u);
  __syncthreads();
  for (int i = threadIdx.x; i < bins; i += 256) hist[(int64_t)i * tiles + blockIdx.x] = h[i];
}

// exclusive scan of hist[0 .. m) in place, one block (the array holds bins x tiles counters: small next to the keys), 8192
// counters per round: eight consecutive ones per thread, a shuffle scan inside each wave, the 16 wave totals through LDS
__global__ __launch_bounds__(1024) void radix_scan_kernel(uint32_t* __restrict__ hist, int64_t m) {
  __shared__ uint32_t wave_tot[16];
  __shared__ uint32_t carry_s;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  for (int64_t r0 = 0; r0 < m; r0 += 8192) {
    const int64_t start = r0 + (int64_t)threadIdx.x * 8;
    uint32_t v[8], sum = 0;
    if (start + 8 <= m) {                                // the array is 256-byte aligned and start a multiple of 8
      const uint4 a = *reinterpret_cast<const uint4*>(hist + start), b = *reinterpret_cast<const uint4*>(hist + start + 4);
      v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = start + i < m ? hist[start + i] : 0u;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) sum += v[i];
    uint32_t inc = sum;                                  // inclusive scan of the sums over the wave
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t t = __shfl_up(inc, d, 64);
      if (lane >= d) inc += t;
    }
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    uint32_t run = carry_s + inc - sum;
    for (int w = 0; w < wave; ++w) run += wave_tot[w];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (start + i < m) hist[start + i] = run;
      run += v[i];
    }
    __syncthreads();
    if (threadIdx.x == 1023) carry_s = run;               // the last thread's running sum = everything so far
    __syncthreads();
  }
}

__global__ __launch_bounds__(256) void radix_scatter_kernel(const uint32_t* __restrict__ key_in, const int32_t* __restrict__ val_in,
                                                            int64_t n, int shift, int bins, int tiles,
                                                            const uint32_t* __restrict__ offsets, uint32_t* __restrict__ key_out,
                                                            int32_t* __restrict__ val_out) {
  __shared__ uint32_t before[kSortBins];                  // pairs of each digit in the tile's earlier sub-tiles
  __shared__ uint16_t cnt[4][kSortBins];                  // pairs of each digit in each wave of the current sub-tile
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < bins; i += 256) { before[i] = 0; cnt[0][i] = 0; cnt[1][i] = 0; cnt[2][i] = 0; cnt[3][i] = 0; }
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * kSortTile;
  const int nbits = bins == 2048 ? 11 : 10;
  for (int sub = 0; sub < kSortTile / 256; ++sub) {      // sub-tiles in order; within one: wave by wave, lane by lane
    const int64_t i = base + sub * 256 + threadIdx.x;
    const bool live = i < n;
    const uint32_t k = live ? key_in[i] : 0u;
    const int32_t v = live ? val_in[i] : 0;
    const int d = (int)((k >> shift) & (uint32_t)(bins - 1));
    // lanes of this wave with the same digit: intersect, bit by bit, the ballots that agree with this lane's bit
    unsigned long long peers = __ballot(live);
    for (int bit = 0; bit < nbits; ++bit) {
      const unsigned long long set = __ballot((d >> bit) & 1);
      peers &= ((d >> bit) & 1) ? set : ~set;
    }
    const int rank_in_wave = __popcll(peers & ((1ull << lane) - 1ull));
    if (live && rank_in_wave == 0) cnt[wave][d] = (uint16_t)__popcll(peers);   // the group's first lane reports its size
    __syncthreads();
    if (live) {
      uint32_t r = before[d] + rank_in_wave;
      for (int w = 0; w < wave; ++w) r += cnt[w][d];
      const int64_t dst = (int64_t)offsets[(int64_t)d * tiles + blockIdx.x] + r;
      key_out[dst] = k;
      val_out[dst] = v;
    }
    __syncthreads();
    for (int q = threadIdx.x; q < bins; q += 256) {
      before[q] += (uint32_t)cnt[0][q] + cnt[1][q] + cnt[2][q] + cnt[3][q];
      cnt[0][q] = 0; cnt[1][q] = 0; cnt[2][q] = 0; cnt[3][q] = 0;
    }
    __syncthreads();
  }
}

size_t bpr_order_workspace_bytes(int64_t T) {
  const int64_t tiles = ceil_div(T, kSortTile);
  return 4 * align_up((size_t)T * 4, 256) + align_up((size_t)kSortBins * tiles * 4, 256);
}

// perm[i] = the token that arrives i-th under batch prioritized routing; returns it through *perm (a piece of ws)
hipError_t launch_bpr_order(const float* logits, int64_t T, int64_t E, void* ws, const int32_t** perm, hipStream_t s) {
  const int64_t tiles = ceil_div(T, kSortTile);
  const size_t piece = align_up((size_t)T * 4, 256);
  char* base = (char*)ws;
  uint32_t* key[2] = {(uint32_t*)base, (uint32_t*)(base + piece)};
  int32_t* val[2] = {(int32_t*)(base + 2 * piece), (int32_t*)(base + 3 * piece)};
  uint32_t* hist = (uint32_t*)(base + 4 * piece);
  bpr_key_kernel<<<dim3((unsigned)ceil_div(T, 256)), dim3(256), 0, s>>>(logits, T, (int)E, key[0], val[0]);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  const int shifts[3] = {0, 11, 22}, binsv[3] = {2048, 2048, 1024};
  int cur = 0;
  for (int p = 0; p < 3; ++p) {
    radix_hist_kernel<<<dim3((unsigned)tiles), dim3(256), 0, s>>>(key[cur], T, shifts[p], binsv[p], (int)tiles, hist);
    radix_scan_kernel<<<dim3(1), dim3(1024), 0, s>>>(hist, (int64_t)binsv[p] * tiles);
    radix_scatter_kernel<<<dim3((unsigned)tiles), dim3(256), 0, s>>>(key[cur], val[cur], T, shifts[p], binsv[p], (int)tiles, hist,
                                                                     key[cur ^ 1], val[cur ^ 1]);
    err = hipGetLastError();
    if (err != hipSuccess) return err;
    cur ^= 1;
  }
  *perm = val[cur];
  return hipSuccess;
}

}  // namespace moe
