// Gate logits at memory speed with routing decisions that stay exact (arXiv 2206.03382 Sec. 2.1: the gating function's
// linear layer; the choice of experts taken on it must not depend on a summation order).
//
// The exact kernel (gate.hip) sums every dot product in fp64, which binds the stage to the chip's slow fp64 units.  Here
// the bf16 tokens and gate weights go through the bf16 matrix cores, in blocked fp32 sums that keep a rigorous bound:
//   * a product of two bf16 values is exact in fp32;
//   * a chain of CH (1 or 2) v_mfma_f32_16x16x32_bf16 that starts from a zero accumulator adds 32 CH such products in fp32:
//     whatever order and rounding the hardware uses, 32 CH additions that each err by at most one unit in the last place
//     of a partial sum bounded by sum |x w| give  |error| <= 32 CH 2^-23 sum_{chunk} |x_m w_me|;
//   * eight chunk results are added in fp32 by the vector unit (round to nearest: 2^-24 each), and those sums are added
//     in fp32 again (ceil(chunks / 8) additions), then the bias: every partial sum is bounded by sum_m |x_m w_me| + |b_e|.
// So  |logit' - exact sum| <= B_t = (32 CH 2^-23 + (10 + ceil(chunks / 8)) 2^-24) (|x_t| max_e |w_e| + max_e |b_e|)
// by Cauchy-Schwarz over the whole row.  B_t is written per token (`margin`); |x_t|^2 comes from the matrix cores too
// (the diagonal of X X^T, accumulated beside the logits).  The top-k kernel orders a token's k+1 largest logits and accepts
// them only if every gap between neighbours exceeds 2 B_t (plus the rounding of the exactly rounded value itself); the few
// tokens that fail have the dot products of the experts in question recomputed in fp64 (gate.hip), which reproduces what
// the exact kernel would have decided.
//
// Layout: gate_prepare_kernel writes Wt [E, Mp] = Wg^T (k contiguous, rows zero-padded to a multiple of 128) and the
// experts' norms once per call.  gate_logits_fast_kernel: a block of four waves shares 128-wide k-chunks of Wt in LDS
// (double buffered, filled by direct global->LDS loads, pieces XOR-swizzled: conflict-free 16-byte operand reads); a wave owns TW tiles of 16 tokens
// whose rows go straight from global memory into the A operand (lane = token l % 16, 8 consecutive k at 8 (l / 16)),
// through a ring of R steps of prefetch.
#include <type_traits>

#include "common.h"

namespace moe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

namespace {

constexpr int kChunk = 128;                 // Wt rows are zero-padded to a multiple of this many k
constexpr float kUlp = 1.1920929e-07f;      // 2^-23

// Direct global->LDS load of 16 bytes per lane from base + voff: lane l's data lands at lds_addr + 16 l.  Written as
// inline assembly so that the compiler does not order it against the LDS reads of the other buffer; completion is tracked
// by hand (s_waitcnt vmcnt + barrier before the buffer is read).
__device__ __forceinline__ void global_to_lds_16(const void* base, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(base), "s"(lds_addr) : "memory", "m0");
}

// Wt[e, m] = Wg[m, e] for m < M, 0 for M <= m < Mp; wnorm[e] = |w_e|_2 rounded up.  One block per expert.
__global__ __launch_bounds__(256) void gate_prepare_kernel(const uint16_t* __restrict__ Wg, int M, int Mp, int E,
                                                           uint16_t* __restrict__ Wt, float* __restrict__ wnorm) {
  __shared__ float part[256];
  const int e = blockIdx.x;
  float s = 0.f;
  for (int m = threadIdx.x; m < Mp; m += 256) {
    const uint16_t w = m < M ? Wg[(int64_t)m * E + e] : (uint16_t)0;
    Wt[(int64_t)e * Mp + m] = w;
    const float f = bf16_bits_to_f32(w);
    s = fmaf(f, f, s);
  }
  part[threadIdx.x] = s;
  __syncthreads();
  for (int off = 128; off >= 1; off >>= 1) {
    if ((int)threadIdx.x < off) part[threadIdx.x] += part[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) wnorm[e] = sqrtf(part[0]) * 1.001f;
}

// NT tiles of 16 experts per pass, TW tiles of 16 tokens per wave, R K-steps (of 32) of token prefetch, KCH k per LDS
// chunk of Wt, CH matrix-core instructions chained before their sum leaves the matrix cores (the error bound grows with
// CH, the vector unit's work shrinks with it).
// EH: waves that share a token tile and split the pass's experts between them (EH x NT tiles of 16 experts in LDS): a
// wave then reads NT instead of EH x NT operand fragments from LDS per K-step (LDS bandwidth is what binds the widest
// gates) and the tokens' rows, fetched by EH waves, come from the cache the second time.
template <int NT, int TW, int R, int KCH, int CH, int EH>
__global__ __launch_bounds__(256, 2) void gate_logits_fast_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ Wt,
                                                                  const float* __restrict__ wnorm, const float* __restrict__ bias,
                                                                  int64_t T, int M, int Mp, int E, int e_base, float bound,
                                                                  float* __restrict__ logits, float* __restrict__ margin) {
  constexpr int EN = NT * EH * 16;                                  // experts of this pass
  constexpr int CS = KCH / 32;                                      // K-steps per chunk
  constexpr int SLOTS = KCH / 8;                                    // 16-byte pieces of a chunk row
  constexpr int WI = EN * KCH * 2 / 4096;                           // direct loads (1 KB each) per wave and chunk
  static_assert(KCH == 128 && WI >= 1, "a 1 KB direct load covers four 256-byte rows");
  static_assert(R % CS == 0 || CS % R == 0, "chunk boundaries fall on whole prefetch groups");
  static_assert(R % CH == 0 && CS % CH == 0, "chains do not straddle groups or chunks");
  // Wt chunks in LDS, double buffered: [EN rows][16 pieces of 8 k], piece p of row e stored at position p ^ (e % 16), so
  // that the 16 lanes of an operand read (16 consecutive rows, same p) cover all banks once.  Filled by direct loads.
  __shared__ __attribute__((aligned(1024))) uint16_t wl[2][EN * KCH];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane & 15, kq = lane >> 4;
  const int eh = wave % EH;                                         // this wave's share of the experts: tiles eh*NT .. eh*NT+NT-1
  const int64_t t0 = ((int64_t)blockIdx.x * (4 / EH) + wave / EH) * (16 * TW);
  const int steps = Mp / 32, chunks = Mp / KCH, full_steps = M / 32;   // steps whose 32 k all lie inside the row

  const uint16_t* xp[TW];                                           // this lane's 8 k of K-step 0 (rows past the end repeat the last)
#pragma unroll
  for (int w = 0; w < TW; ++w) {
    const int64_t t = t0 + w * 16 + r;
    xp[w] = x + (t < T ? t : T - 1) * (int64_t)M + kq * 8;
  }
  // this wave's direct loads of a chunk: load i fills the 1 KB block i*4 + wave = rows 4 (i*4 + wave) .. +3; lane l brings
  // the piece that belongs at position l % 16 of row +l/16.  Rows past E repeat the last expert (their logits are never
  // stored).  The byte offsets do not depend on the chunk: only the base moves.
  uint32_t woff[WI];
#pragma unroll
  for (int i = 0; i < WI; ++i) {
    const int row = (i * 4 + wave) * 4 + (lane >> 4);
    const int e = e_base + row < E ? e_base + row : E - 1;
    woff[i] = (uint32_t)(((int64_t)e * Mp + (((lane & 15) ^ (row & 15)) << 3)) * 2);
  }
  const uint32_t wl_addr = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char*)&wl[0][0]);
  auto w_issue = [&](int c) __attribute__((always_inline)) {         // chunk c -> buffer c & 1
#pragma unroll
    for (int i = 0; i < WI; ++i)
      global_to_lds_16(Wt + (int64_t)c * KCH, woff[i], wl_addr + (uint32_t)((c & 1) * EN * KCH * 2 + (i * 4 + wave) * 1024));
  };
  // x ring: slot j holds K-step s with s % R == j.  FAST: the step lies wholly inside the row (no predicate; the
  // offset from xp is a compile-time constant).  Otherwise pieces past the row's end read its start and are zeroed.
  uint4 ring[TW][R];
  auto x_fetch = [&](auto fast_tag, int j, int s_rel, int s) __attribute__((always_inline)) {
    constexpr bool FAST = decltype(fast_tag)::value;
#pragma unroll
    for (int w = 0; w < TW; ++w) {
      if (FAST) {
        ring[w][j] = *reinterpret_cast<const uint4*>(xp[w] + s_rel * 32);
      } else {
        const bool live = s * 32 + kq * 8 < M;
        const uint4 v = *reinterpret_cast<const uint4*>(live ? xp[w] + s_rel * 32 : xp[w] - kq * 8);
        const uint32_t keep = live ? 0xffffffffu : 0u;
        ring[w][j] = make_uint4(v.x & keep, v.y & keep, v.z & keep, v.w & keep);
      }
    }
  };

  f32x4 acc[TW][NT], sup[TW][NT];                                   // sums of super-chunks; of the current super-chunk's chunks
  f32x4 xx[TW];                                                     // X X^T of the token tile: its diagonal is |x_t|^2
#pragma unroll
  for (int w = 0; w < TW; ++w) {
    xx[w] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) { acc[w][nt] = f32x4{0.f, 0.f, 0.f, 0.f}; sup[w][nt] = f32x4{0.f, 0.f, 0.f, 0.f}; }
  }

  w_issue(0);
#pragma unroll
  for (int j = 0; j < R; ++j) x_fetch(std::false_type{}, j, j, j);
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(R * TW) : "memory");   // loads return in order: chunk 0 of Wt has landed
  __syncthreads();

  const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
  // fp32 sums of the current chain and of the one before it.  A chain's sum is added to its super-chunk one chain late,
  // behind the first matrix-core instruction of the next chain (by then it has long left the pipeline), and the addition
  // is pinned there: left to itself the compiler keeps every chain's sum of a whole prefetch group alive and adds them
  // all at the group's end, which costs 32 registers per chain.
  static_assert((R / CH) % 2 == 0, "chains alternate between two accumulators across prefetch groups");
  f32x4 part[2][TW][NT];
#pragma unroll
  for (int w = 0; w < TW; ++w)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) part[1][w][nt] = zero;
  auto group = [&](auto fast_tag, int s0) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < R; ++j) {
      const int s = s0 + j;                                         // uniform over the block
      const int c = s / CS;
      const uint16_t* wbuf = wl[c & 1];
      // first step of a chunk: the other buffer is free (every wave is past the last barrier): start the next chunk
      if (s % CS == 0 && c + 1 < chunks) w_issue(c + 1);
      bf16x8 a[TW];
#pragma unroll
      for (int w = 0; w < TW; ++w) {
        a[w] = __builtin_bit_cast(bf16x8, ring[w][j]);
        xx[w] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[w], a[w], xx[w], 0, 0, 0);
      }
      x_fetch(fast_tag, j, j + R, s + R);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const bf16x8 b = *reinterpret_cast<const bf16x8*>(&wbuf[((eh * NT + nt) * 16 + r) * KCH + ((((s % CS) * 4 + kq) ^ r) << 3)]);
#pragma unroll
        for (int w = 0; w < TW; ++w) {
          const int p = (j / CH) & 1;                               // compile-time: j is an unrolled index
          part[p][w][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[w], b, j % CH == 0 ? zero : part[p][w][nt], 0, 0, 0);
          if (j % CH == 0) {                                        // the chain before this one (zeros before the very first)
#pragma unroll
            for (int v = 0; v < 4; ++v) sup[w][nt][v] += part[p ^ 1][w][nt][v];
            asm volatile("" : "+v"(sup[w][nt]));
          }
        }
      }
      if ((s + 1) % (8 * CH) == 0) {                                // eight chains make a super-chunk (the latest one joins the next)
#pragma unroll
        for (int w = 0; w < TW; ++w)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[w][nt][v] += sup[w][nt][v];
            sup[w][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
          }
      }
      if ((s + 1) % CS == 0 && c + 1 < chunks) {                    // last step of a chunk: the next one must have landed
        // its direct loads were issued CS steps ago, followed by CS x TW token loads; loads return in order
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(CS * TW) : "memory");
        __syncthreads();
      }
    }
#pragma unroll
    for (int w = 0; w < TW; ++w) xp[w] += R * 32;
  };
  int s0 = 0;
  for (; s0 + 2 * R <= full_steps; s0 += R) group(std::true_type{}, s0);      // this group and the one it prefetches are full
  for (; s0 < steps; s0 += R) group(std::false_type{}, s0);                  // steps is a multiple of R (the launcher sees to it)

  // the last chain's sum (R / CH is even: it sits in the second accumulator)
#pragma unroll
  for (int w = 0; w < TW; ++w)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int v = 0; v < 4; ++v) sup[w][nt][v] += part[1][w][nt][v];
  // logits: lane holds expert column nt*16 + r of token rows 4 kq + v
#pragma unroll
  for (int w = 0; w < TW; ++w)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int e = e_base + (eh * NT + nt) * 16 + r;
      if (e >= E) continue;
      const float be = bias ? bias[e] : 0.f;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int64_t t = t0 + w * 16 + 4 * kq + v;
        if (t < T) logits[t * E + e] = (acc[w][nt][v] + sup[w][nt][v]) + be;     // the last, partial super-chunk; then the bias
      }
    }
  if (margin && eh == 0) {
    float wmax = 0.f, bmax = 0.f;
    for (int e = 0; e < E; ++e) {
      wmax = fmaxf(wmax, wnorm[e]);
      if (bias) bmax = fmaxf(bmax, fabsf(bias[e]));
    }
    // |x_t|^2 of token row i sits on the diagonal: lane (r = i, kq = i / 4), register i % 4
#pragma unroll
    for (int w = 0; w < TW; ++w) {
      const int64_t t = t0 + w * 16 + r;
      if (kq == (r >> 2) && t < T) {
        float n = xx[w][0];
#pragma unroll
        for (int v = 1; v < 4; ++v) n = (r & 3) == v ? xx[w][v] : n;
        margin[t] = bound * (sqrtf(n * 1.002f) * wmax + bmax);
      }
    }
  }
}

template <int NT, int TW, int R, int KCH, int CH, int EH>
void launch_fast_one(const uint16_t* x, const uint16_t* Wt, const float* wnorm, const float* bias, int64_t T, int M, int Mp, int E,
                     int e_base, float* logits, float* margin, hipStream_t s) {
  const dim3 grid((unsigned)ceil_div(T, (64 / EH) * TW)), block(256);
  // error bound of a logit per unit of |x| |w| + |b|: the chunk's matrix-core sum (one unit in the last place per term),
  // eight chunk results, the super-chunks, the bias (round to nearest each), with slack for the norms' own rounding
  const int chunks = Mp / (32 * CH);
  const float bound = (float)((32.0 * CH * (double)kUlp + (10.0 + (chunks + 7) / 8) * 0.5 * (double)kUlp) * 1.01);
  gate_logits_fast_kernel<NT, TW, R, KCH, CH, EH><<<grid, block, 0, s>>>(x, Wt, wnorm, bias, T, M, Mp, E, e_base, bound, logits, margin);
}

}  // namespace

size_t gate_fast_workspace_bytes(int64_t T, int64_t M, int64_t E) {
  const int64_t Mp = ceil_div(M, kChunk) * kChunk;
  return align_up((size_t)E * Mp * 2, 256) + align_up((size_t)E * 4, 256) + align_up((size_t)T * 4, 256);
}

GateFastWorkspace gate_fast_layout(void* ws, int64_t T, int64_t M, int64_t E) {
  GateFastWorkspace w;
  w.Mp = ceil_div(M, kChunk) * kChunk;
  char* base = (char*)ws;
  w.Wt = (uint16_t*)base;
  w.wnorm = (float*)(base + align_up((size_t)E * w.Mp * 2, 256));
  w.margin = (float*)((char*)w.wnorm + align_up((size_t)E * 4, 256));
  return w;
}

bool gate_logits_fast_supports(int dtype, int64_t T, int64_t M, int64_t E) {
  // 32-bit byte offsets inside Wt
  return dtype == MOE_BF16 && M % 8 == 0 && E <= 512 && E * (M + kChunk) * 2 < ((int64_t)1 << 31) && T <= ((int64_t)1 << 30);
}

// logits' (fp32, within margin[t] of the exactly rounded sums) and margin [T]; ws laid out by gate_fast_layout.
hipError_t launch_gate_logits_fast(const void* x, const void* Wg, const float* bias, int64_t T, int64_t M, int64_t E,
                                   float* logits, const GateFastWorkspace& w, hipStream_t s) {
  const int Mp = (int)w.Mp;
  gate_prepare_kernel<<<dim3((unsigned)E), dim3(256), 0, s>>>((const uint16_t*)Wg, (int)M, Mp, (int)E, w.Wt, w.wnorm);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  const uint16_t* xb = (const uint16_t*)x;
  for (int64_t e_base = 0; e_base < E; e_base += 128) {
    const int64_t rem = E - e_base;
    float* mg = e_base == 0 ? w.margin : nullptr;         // the bound does not depend on the pass
    // tokens per block 64 TW: small batches take narrow blocks so that the grid still covers the chip twice
    const bool wide = T >= 65536;
    const int steps = Mp / 32;                             // a multiple of 4; the prefetch ring must divide it
#define MOE_FAST(NT, TW, R, CH, EH) launch_fast_one<NT, TW, R, kChunk, CH, EH>(xb, w.Wt, w.wnorm, bias, T, (int)M, Mp, (int)E, (int)e_base, logits, mg, s)
#define MOE_FAST_R(NT, TW, RMAX, CH, EH)                                                  \
  do {                                                                                    \
    if (RMAX >= 16 && steps % 16 == 0) MOE_FAST(NT, TW, (RMAX >= 16 ? 16 : 4), CH, EH);   \
    else if (RMAX >= 8 && steps % 8 == 0) MOE_FAST(NT, TW, (RMAX >= 8 ? 8 : 4), CH, EH);  \
    else MOE_FAST(NT, TW, 4, CH, EH);                                                     \
  } while (0)
    if (rem <= 16) { if (wide) MOE_FAST_R(1, 2, 8, 1, 1); else MOE_FAST_R(1, 1, 16, 1, 1); }
    else if (rem <= 32) { if (wide) MOE_FAST_R(2, 2, 4, 1, 1); else MOE_FAST_R(2, 1, 8, 1, 1); }
    else if (rem <= 64) { if (wide) MOE_FAST_R(4, 2, 4, 2, 1); else MOE_FAST_R(4, 1, 8, 2, 1); }
    else MOE_FAST_R(8, 1, 8, 1, 1);                                 // single chains: the tighter bound halves the near-tie repairs of wide top-k
#undef MOE_FAST_R
#undef MOE_FAST
  }
  return hipGetLastError();
}

}  // namespace moe
