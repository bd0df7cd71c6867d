// Grouped bf16 GEMM on the gfx950 matrix cores for the local experts' feed-forward layer
// (arXiv 2206.03382 Sec. 2.1; one [C, K] slab per expert, the layout of Sec. 4.2 "Flexible All-to-All").
//
//   out[e] = epilogue(A[e] (rows_e x K) * B[e] (K x N) + bias[e]),  A [E,C,K], B [E,K,N], out [E,C,N], all bf16,
//   fp32 accumulation, rows_e = min(counts[e], C) (or C).  Requires K % 64 == 0 and N % 256 == 0.
//
// Tiling: one 512-thread block (8 waves, 2 per SIMD) owns a 256 x 256 output tile; waves form a 2 x 4 grid, each
// owning 128 x 64 as 4 x 2 tiles of v_mfma_f32_32x32x16_bf16.  K advances in steps of 64 through a two-stage LDS
// ring (2 x 64 KB) filled by direct global->LDS loads (16 bytes per lane, no staging registers).
//
// LDS layouts (both written by the direct loads, which place lane l's 16 bytes at base + 16 l):
//   A tile  [256 rows][8 chunks of 8 k]:   chunk g of row r is stored at chunk position g ^ ((r / 2) % 8), so the 16 lanes
//           that share an LDS cycle of a ds_read_b128 (16 consecutive rows, same g) cover all 64 banks once.
//   B tile  [64 k][32 chunks of 8 n]:      chunk c of row k is stored at position c ^ (4 (k % 4)); the two 16-lane
//           blocks of a ds_read_b64_tr_b16 that share a cycle (4 k rows x 32 bytes each) then cover all banks once.
// B is K x N with N contiguous, but the matrix cores want k-contiguous operands: ds_read_b64_tr_b16 transposes
// 4 k x 16 n sub-blocks on the way out of LDS (source lane s of a 16-lane block supplies row k0 + s/4,
// columns n0 + 4 (s%4) .. +3; result lane l holds column n0 + l, rows k0 .. k0+3).
//
// The two MFMA operands are passed swapped (B fragment first), so that a lane's accumulator registers hold four
// consecutive output columns of one row: D'[n][m] with m = lane % 32, n = 8 (v/4) + 4 (lane/32) + v % 4.
#include "common.h"

namespace moe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(8))) short short8v;
typedef __attribute__((ext_vector_type(16))) float f32x16;

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kThreads = 512;
constexpr int kStageBytes = 65536;          // A tile 32 KB + B tile 32 KB
constexpr int kATileBytes = 32768;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

// Direct global->LDS load of 16 bytes per lane: lane l's data lands at lds_addr + 16 l.  Written as inline assembly so
// that the compiler does not serialise the prefetch against the LDS reads of the other stage; completion is tracked
// by hand (s_waitcnt vmcnt(0) + barrier before a stage is read).
__device__ __forceinline__ void global_to_lds_16(const char* src, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(lds_addr) : "memory", "m0");
}

// Branch-free activations for the bf16 epilogue.  erf by the 5-term rational/exponential form of Abramowitz & Stegun
// 7.1.26 (absolute error < 1.5e-7, far below bf16 resolution).
__device__ __forceinline__ float fast_erf(float x) {
  const float ax = fabsf(x);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  const float r = 1.0f - p * t * __expf(-ax * ax);
  return copysignf(r, x);
}

template <int ACT> __device__ __forceinline__ float epilogue_act(float v) {
  if (ACT == MOE_ACT_RELU) return fmaxf(v, 0.f);
  if (ACT == MOE_ACT_GELU) return 0.5f * v * (1.0f + fast_erf(v * 0.70710678118654752440f));
  if (ACT == MOE_ACT_SILU) return v * __builtin_amdgcn_rcpf(1.0f + __expf(-v));
  return v;
}

}  // namespace

#define PHASE_BARRIER()                        \
  do {                                         \
    __builtin_amdgcn_sched_barrier(0);         \
    asm volatile("s_barrier" ::: "memory");    \
    __builtin_amdgcn_sched_barrier(0);         \
  } while (0)

// ---- main loop -------------------------------------------------------------------------------------------------
// Two groups of four waves (one wave of each group per SIMD) run one phase apart.  A K-step of 64 is two halves; each
// half is a MEM phase (LDS -> fragment registers) followed by a COMPUTE phase (16 MFMAs); every phase ends with a
// workgroup barrier, so between two barriers one wave per SIMD feeds the matrix core while the other moves data.
// Global phase numbering (g0 = group 0, g1 = group 1), K-step kt:
//   4kt   : g0 MEM(kt, 1st half)      g1 COMPUTE(kt-1, 2nd half)
//   4kt+1 : g0 COMPUTE(kt, 1st half)  g1 MEM(kt, 1st half)
//   4kt+2 : g0 MEM(kt, 2nd half)      g1 COMPUTE(kt, 1st half)
//   4kt+3 : g0 COMPUTE(kt, 2nd half)  g1 MEM(kt, 2nd half)
// Issuing a direct-to-LDS load blocks the issuing wave while the address unit is busy, so the 8 loads a wave
// contributes to K-step kt+1 are spread 3/3/2 over phases 4kt, 4kt+1, 4kt+2, between LDS reads or MFMAs.  They are
// waited for (s_waitcnt vmcnt(0)) before the barrier that ends phase 4kt+3; the stage they fill was last read in
// phase 4kt-1.
template <bool FULL>
__device__ __forceinline__ void tile_main_loop(char* smem, const char* const (&a_src)[4], const char* const (&b_src)[4],
                                               int64_t a_step, int64_t b_step, const int (&a_off)[4],
                                               const int (&b_off)[2], int a_swz, int kg, int ni, int grp, int wave,
                                               int K, f32x16 (&acc)[4][2]) {
  bf16x8 af[2][4], bfr[2][2];
  const uint32_t smem_addr = (uint32_t)(uintptr_t)LDS_PTR(char, smem);
  const int KT = K / BK;

  auto load_frags = [&](const char* stage, int s, bf16x8 (&a)[4], bf16x8 (&b)[2]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (FULL || i < ni) a[i] = *LDS_PTR(bf16x8, stage + a_off[i] + (((2 * s + kg) ^ a_swz) << 4));
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(short4v, stage + b_off[j] + (16 * s) * 512));
      const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(short4v, stage + b_off[j] + (16 * s + 4) * 512));
      b[j] = __builtin_bit_cast(bf16x8, (short8v)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
  };
  // MFMAs of sub-tile rows [i0, i0+2)
  auto mma2 = [&](int i0, const bf16x8 (&a)[4], const bf16x8 (&b)[2]) {
#pragma unroll
    for (int i = i0; i < i0 + 2; ++i)
      if (FULL || i < ni) {
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
      }
  };
  // load number idx (0..7: A0 B0 A1 B1 A2 B2 A3 B3) of K-step `tile`; does nothing past the last K-step
  auto dma = [&](int idx, int tile) {
    if (tile >= KT) return;
    const int q = idx >> 1;
    const uint32_t dst = smem_addr + (tile & 1) * kStageBytes + (q * 8 + wave) * 1024;
    if (idx & 1) global_to_lds_16(b_src[q] + tile * b_step, dst + kATileBytes);
    else global_to_lds_16(a_src[q] + tile * a_step, dst);
  };
#define PIN() __builtin_amdgcn_sched_barrier(0)

#pragma unroll
  for (int idx = 0; idx < 8; ++idx) dma(idx, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  PHASE_BARRIER();

  if (grp == 0) {
    for (int kt = 0; kt < KT; ++kt) {
      const char* cur = smem + (kt & 1) * kStageBytes;
      // phase 4kt: MEM, first half
      load_frags(cur, 0, af[0], bfr[0]);
      PIN(); dma(0, kt + 1); PIN();
      load_frags(cur, 1, af[1], bfr[1]);
      PIN(); dma(1, kt + 1); dma(2, kt + 1);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      PHASE_BARRIER();
      // phase 4kt+1: COMPUTE, first half
      mma2(0, af[0], bfr[0]); PIN(); dma(3, kt + 1); PIN();
      mma2(2, af[0], bfr[0]); PIN(); dma(4, kt + 1); PIN();
      mma2(0, af[1], bfr[1]); PIN(); dma(5, kt + 1); PIN();
      mma2(2, af[1], bfr[1]);
      PHASE_BARRIER();
      // phase 4kt+2: MEM, second half
      load_frags(cur, 2, af[0], bfr[0]);
      PIN(); dma(6, kt + 1); PIN();
      load_frags(cur, 3, af[1], bfr[1]);
      PIN(); dma(7, kt + 1);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      PHASE_BARRIER();
      // phase 4kt+3: COMPUTE, second half
      mma2(0, af[0], bfr[0]);
      mma2(2, af[0], bfr[0]);
      mma2(0, af[1], bfr[1]);
      mma2(2, af[1], bfr[1]);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      PHASE_BARRIER();
    }
    PHASE_BARRIER();
  } else {
    dma(0, 1); dma(1, 1); dma(2, 1);                                // phase 0: group 1 has nothing to compute yet
    PHASE_BARRIER();
    for (int kt = 0; kt < KT; ++kt) {
      const char* cur = smem + (kt & 1) * kStageBytes;
      // phase 4kt+1: MEM, first half
      load_frags(cur, 0, af[0], bfr[0]);
      PIN(); dma(3, kt + 1); PIN();
      load_frags(cur, 1, af[1], bfr[1]);
      PIN(); dma(4, kt + 1); dma(5, kt + 1);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      PHASE_BARRIER();
      // phase 4kt+2: COMPUTE, first half
      mma2(0, af[0], bfr[0]); PIN(); dma(6, kt + 1); PIN();
      mma2(2, af[0], bfr[0]); PIN(); dma(7, kt + 1); PIN();
      mma2(0, af[1], bfr[1]);
      mma2(2, af[1], bfr[1]);
      PHASE_BARRIER();
      // phase 4kt+3: MEM, second half
      load_frags(cur, 2, af[0], bfr[0]);
      load_frags(cur, 3, af[1], bfr[1]);
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
      PHASE_BARRIER();
      // phase 4(kt+1): COMPUTE, second half; first loads of K-step kt+2 (its stage was last read in phase 4kt+3)
      mma2(0, af[0], bfr[0]); PIN(); dma(0, kt + 2); PIN();
      mma2(2, af[0], bfr[0]); PIN(); dma(1, kt + 2); PIN();
      mma2(0, af[1], bfr[1]); PIN(); dma(2, kt + 2); PIN();
      mma2(2, af[1], bfr[1]);
      PHASE_BARRIER();
    }
  }
#undef PIN
}

template <int ACT>
__global__ __launch_bounds__(kThreads) void grouped_gemm_mfma_kernel(const uint16_t* __restrict__ A,
                                                                     const uint16_t* __restrict__ B,
                                                                     const uint16_t* __restrict__ bias,
                                                                     const int32_t* __restrict__ counts, int E, int64_t C,
                                                                     int K, int N, int MT, int NT,
                                                                     uint16_t* __restrict__ out) {
  __shared__ __attribute__((aligned(1024))) char smem[2 * kStageBytes];

  // ---- which tile: spread consecutive logical tiles over one XCD (blocks are dealt round-robin to the 8 XCDs) ----
  const int total = E * MT * NT;
  const int b = blockIdx.x;
  const int per = total / 8, rem = total % 8, xcd = b % 8, within = b / 8;
  const int pid = xcd * per + (xcd < rem ? xcd : rem) + within;
  const int e = pid / (MT * NT);
  const int mt = (pid / NT) % MT, nt = pid % NT;
  int64_t rows = C;
  if (counts) { const int64_t c = counts[e]; rows = c < C ? (c > 0 ? c : 0) : C; }
  const int64_t m0 = (int64_t)mt * BM;
  if (m0 >= rows) return;
  const int n0 = nt * BN;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave >> 2, wn = wave & 3;

  // ---- global sources of this lane's direct-to-LDS loads ---------------------------------------------------------
  // A: 1 KB block q*8+wave of the tile = rows 8(q*8+wave) .. +7, lane l writes row +l/8, chunk position l%8.
  // B: 1 KB block q*8+wave = k-rows 2(q*8+wave), +1, lane l writes k-row +l/32, chunk position l%32.
  const char* Ae = (const char*)(A + (int64_t)e * C * K);
  const char* Be = (const char*)(B + (int64_t)e * K * N);
  const char* a_src[4];
  const char* b_src[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int r = q * 64 + wave * 8 + (lane >> 3);
    int64_t row = m0 + r;
    row = row < C ? row : C - 1;                                    // rows past the slab are clamped (never stored)
    const int g = (lane & 7) ^ ((r >> 1) & 7);                      // global chunk that lands at position lane % 8
    a_src[q] = Ae + (row * K + g * 8) * 2;
    const int kr = q * 16 + wave * 2 + (lane >> 5);
    const int c = (lane & 31) ^ (4 * (kr & 3));
    b_src[q] = Be + ((int64_t)kr * N + n0 + c * 8) * 2;
  }
  const int64_t a_step = (int64_t)BK * 2, b_step = (int64_t)BK * N * 2;

  // ---- LDS read offsets of this lane's MFMA fragments ------------------------------------------------------------
  const int kg = lane >> 5;
  const int a_swz = ((lane & 31) >> 1) & 7;                         // ((row >> 1) & 7): tile-row offsets are multiples of 32
  int a_off[4];                                                     // + ((2 s + kg) ^ a_swz) * 16
#pragma unroll
  for (int i = 0; i < 4; ++i) a_off[i] = (wm * 128 + i * 32 + (lane & 31)) * 128;
  int b_off[2];                                                     // + (16 s + 4 rd) * 512
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int c = wn * 8 + j * 4 + ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1);
    const int swz = 4 * ((lane >> 2) & 3);                          // 4 (k & 3), k & 3 = (lane % 16) / 4
    b_off[j] = kATileBytes + (kg * 8 + ((lane & 15) >> 2)) * 512 + ((c ^ swz) << 4) + ((lane & 1) << 3);
  }
  // 32-row sub-tiles of this wave that hold real rows (the last row tile of an expert is usually ragged)
  const int64_t wave_rows = rows - m0 - wm * 128;
  const int ni = wave_rows >= 128 ? 4 : (wave_rows <= 0 ? 0 : (int)((wave_rows + 31) >> 5));

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  if (ni == 4) tile_main_loop<true>(smem, a_src, b_src, a_step, b_step, a_off, b_off, a_swz, kg, ni, wm, wave, K, acc);
  else tile_main_loop<false>(smem, a_src, b_src, a_step, b_step, a_off, b_off, a_swz, kg, ni, wm, wave, K, acc);

  // ---- epilogue: bias, activation, bf16, 8-byte stores (4 consecutive columns per lane and register group) -------
  uint16_t* oute = out + (int64_t)e * C * N;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t row = m0 + wm * 128 + i * 32 + (lane & 31);
    if (row >= rows) continue;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = n0 + wn * 64 + j * 32 + 8 * g + 4 * kg;
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = acc[i][j][4 * g + u];
        if (bias) {
          const uint2 bb = *reinterpret_cast<const uint2*>(bias + (int64_t)e * N + col);
          v[0] += __uint_as_float(bb.x << 16); v[1] += __uint_as_float(bb.x & 0xffff0000u);
          v[2] += __uint_as_float(bb.y << 16); v[3] += __uint_as_float(bb.y & 0xffff0000u);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = epilogue_act<ACT>(v[u]);
        uint2 pk;
        pk.x = (uint32_t)f32_to_bf16_bits(v[0]) | ((uint32_t)f32_to_bf16_bits(v[1]) << 16);
        pk.y = (uint32_t)f32_to_bf16_bits(v[2]) | ((uint32_t)f32_to_bf16_bits(v[3]) << 16);
        *reinterpret_cast<uint2*>(oute + row * N + col) = pk;
      }
    }
  }
}

bool grouped_gemm_mfma_supports(int64_t E, int64_t C, int64_t K, int64_t N) {
  if (K % BK != 0 || N % BN != 0) return false;
  const int64_t tiles = E * ceil_div(C, BM) * (N / BN);
  return tiles < ((int64_t)1 << 30) && C * K < ((int64_t)1 << 40);
}

hipError_t launch_grouped_gemm_mfma(const void* A, const void* B, const void* bias, int act, const int32_t* counts,
                                    int64_t E, int64_t C, int64_t K, int64_t N, void* out, hipStream_t s) {
  const int MT = (int)ceil_div(C, BM), NT = (int)(N / BN);
  const dim3 grid((unsigned)(E * MT * NT)), block(kThreads);
#define MOE_LAUNCH_GEMM(ACT)                                                                                          \
  grouped_gemm_mfma_kernel<ACT><<<grid, block, 0, s>>>((const uint16_t*)A, (const uint16_t*)B, (const uint16_t*)bias, \
                                                       counts, (int)E, C, (int)K, (int)N, MT, NT, (uint16_t*)out)
  switch (act) {
    case MOE_ACT_RELU: MOE_LAUNCH_GEMM(MOE_ACT_RELU); break;
    case MOE_ACT_GELU: MOE_LAUNCH_GEMM(MOE_ACT_GELU); break;
    case MOE_ACT_SILU: MOE_LAUNCH_GEMM(MOE_ACT_SILU); break;
    default: MOE_LAUNCH_GEMM(-1); break;
  }
#undef MOE_LAUNCH_GEMM
  return hipGetLastError();
}

}  // namespace moe
