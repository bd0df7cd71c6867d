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
//   A tile  [256 rows][8 chunks of 8 k]:   chunk g of row r is stored at chunk position g ^ (r % 8), so the 8 lanes
//           that share an LDS cycle of a ds_read_b128 (8 consecutive rows, same g) hit 8 different bank groups.
//   B tile  [64 k][32 chunks of 8 n]:      chunk c of row k is stored at position c ^ (2 (k % 4)); the 16-lane
//           block of a ds_read_b64_tr_b16 (4 k rows x 32 bytes) then covers all banks once.
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

__device__ __forceinline__ void load_tile_async(const char* const (&a_src)[4], const char* const (&b_src)[4],
                                                uint32_t stage_addr, int wave) {
#pragma unroll
  for (int q = 0; q < 4; ++q) global_to_lds_16(a_src[q], stage_addr + (q * 8 + wave) * 1024);
#pragma unroll
  for (int q = 0; q < 4; ++q) global_to_lds_16(b_src[q], stage_addr + kATileBytes + (q * 8 + wave) * 1024);
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
  const char* Ae = (const char*)(A + (int64_t)e * C * K);
  const char* Be = (const char*)(B + (int64_t)e * K * N);
  const char* a_src[4];
  const char* b_src[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int r = q * 64 + wave * 8 + (lane >> 3);                  // tile row written by this lane
    int64_t row = m0 + r;
    row = row < C ? row : C - 1;                                    // rows past the slab are clamped (never stored)
    const int g = (lane & 7) ^ (lane >> 3);                         // global chunk that lands at position lane % 8
    a_src[q] = Ae + (row * K + g * 8) * 2;
    const int kr = q * 16 + wave * 2 + (lane >> 5);                 // tile k-row written by this lane
    const int c = (lane & 31) ^ (2 * (kr & 3));
    b_src[q] = Be + ((int64_t)kr * N + n0 + c * 8) * 2;
  }
  const int64_t a_step = (int64_t)BK * 2, b_step = (int64_t)BK * N * 2;

  // ---- LDS read offsets of this lane's MFMA fragments ------------------------------------------------------------
  int a_off[4];                                                     // + ((2 s + kg) ^ (lane & 7)) * 16
#pragma unroll
  for (int i = 0; i < 4; ++i) a_off[i] = (wm * 128 + i * 32 + (lane & 31)) * 128;
  const int kg = lane >> 5;
  int b_off[2];                                                     // + (16 s + 4 rd) * 512
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int c = wn * 8 + j * 4 + ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1);
    const int swz = 2 * ((lane >> 2) & 3);
    b_off[j] = kATileBytes + (kg * 8 + ((lane & 15) >> 2)) * 512 + ((c ^ swz) << 4) + ((lane & 1) << 3);
  }

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int KT = K / BK;
  const uint32_t smem_addr = (uint32_t)(uintptr_t)LDS_PTR(char, smem);
  load_tile_async(a_src, b_src, smem_addr, wave);
  __builtin_amdgcn_s_waitcnt(0x0F70);                               // vmcnt(0)
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    char* cur = smem + (kt & 1) * kStageBytes;
    if (kt + 1 < KT) {
#pragma unroll
      for (int q = 0; q < 4; ++q) { a_src[q] += a_step; b_src[q] += b_step; }
      load_tile_async(a_src, b_src, smem_addr + ((kt + 1) & 1) * kStageBytes, wave);
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      bf16x8 af[4], bfr[2];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        af[i] = *LDS_PTR(bf16x8, cur + a_off[i] + (((2 * s + kg) ^ (lane & 7)) << 4));
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(short4v, cur + b_off[j] + (16 * s) * 512));
        const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(short4v, cur + b_off[j] + (16 * s + 4) * 512));
        const short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        bfr[j] = __builtin_bit_cast(bf16x8, both);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                             // next stage has landed (this wave's part)
    __syncthreads();                                                // ... and everyone is done reading `cur`
  }

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
