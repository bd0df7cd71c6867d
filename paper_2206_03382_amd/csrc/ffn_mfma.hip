// Grouped bf16 GEMM on the gfx950 matrix cores for the local experts' feed-forward layer
// (arXiv 2206.03382 Sec. 2.1; one [C, K] slab per expert, the layout of Sec. 4.2 "Flexible All-to-All").
//
//   out[e] = epilogue(A[e] (rows_e x K) * B[e] (K x N) + bias[e]),  A [E,C,K], B [E,K,N], out [E,C,N], all bf16,
//   fp32 accumulation, rows_e = min(counts[e], C) (or C).  Requires K % 64 == 0 and N % 256 == 0.
//
// Tiling: one 256-thread block (4 waves, one per SIMD) owns a 256 x 256 output tile; waves form a 2 x 2 grid, each
// owning 128 x 128 as 4 x 4 tiles of v_mfma_f32_32x32x16_bf16 (256 accumulator registers per lane).  Large wave tiles
// keep LDS->register traffic, the scarce resource on this chip, at 2 x 128 x 2 bytes per k per wave.  K advances in
// steps of 64 through a two-stage LDS ring (2 x 64 KB) filled by direct global->LDS loads (16 bytes per lane, no
// staging registers).  Within a wave every MFMA is followed by at most one LDS read or one direct load, so the
// data movement of the next sub-step hides in the shadow of the current sub-step's MFMAs; one workgroup barrier per
// K-step hands the LDS stages over.
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
// Operand layouts (MODE).  The forward products read A row-major with k contiguous and B row-major with n contiguous
// (kNN).  The backward needs the other two combinations and gets them without any transposed copy in memory:
//   kNT: B is given as [N, K] (k contiguous, e.g. a weight matrix used transposed): its tile is staged and read
//        exactly like an A tile ([256 n][8 chunks of 8 k], ds_read_b128);
//   kTN: A is given as [K, rows] (rows contiguous, e.g. activations used transposed for a weight gradient): its tile
//        is staged and read exactly like a B tile ([64 k][32 chunks of 8 m], transposing reads).  Here the reduction
//        runs over an expert's slots, so its length differs per expert: K-steps up to the last whole one come from
//        the operands themselves and the last one from two small side buffers [E, 64, rows] / [E, 64, N] that hold
//        the remaining slots followed by zeros (written by tail_rows_kernel below), so no read ever touches a slot
//        past the fill.
//
// The two MFMA operands are passed swapped (B fragment first), so that a lane's accumulator registers hold four
// consecutive output columns of one row: D'[n][m] with m = lane % 32, n = 8 (v/4) + 4 (lane/32) + v % 4.  The
// epilogue packs them to 8 bytes, transposes the wave's 128 x 128 tile through LDS and stores whole 256-byte row pieces.
#include <type_traits>

#include "common.h"

namespace moe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(8))) short short8v;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kThreads = 256;
constexpr int kStageBytes = 65536;          // A tile 32 KB + B tile 32 KB
constexpr int kATileBytes = 32768;
constexpr int kLoadsPerWave = 16;           // 64 KB per K-step / (4 waves x 1 KB per wave-load)
constexpr int kMaxExperts = 512;            // the tile search keeps one register per 64 experts
constexpr int kNN = 0, kNT = 1, kTN = 2;    // operand layouts, see the head of this file

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))
#define PIN() __builtin_amdgcn_sched_barrier(0)

// Direct global->LDS load of 16 bytes per lane from base + voff: lane l's data lands at lds_addr + 16 l.  Written as
// inline assembly so that the compiler does not serialise the prefetch against the LDS reads of the other stage;
// completion is tracked by hand (s_waitcnt vmcnt + barrier before a stage is read).
__device__ __forceinline__ void global_to_lds_16(const char* base, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(base), "s"(lds_addr) : "memory", "m0");
}

// Branch-free activations for the bf16 epilogue.  gelu(v) = v Phi(v) with Phi(-y) = erfc(y / sqrt 2) / 2 for y = |v|:
// e = 2^-P(y) with a degree-5 polynomial P fitted to -log2 erfc(y / sqrt 2) (weighted least squares on [0, 9] with P(0) = 0;
// |gelu error| < 6e-7 everywhere, three orders below bf16 resolution), then Phi = 1 - e/2 for
// v >= 0 and e/2 for v < 0.  One exponential, no division.
constexpr float kGeluC1 = 1.151000500e+00f, kGeluC2 = 4.595958591e-01f, kGeluC3 = 5.214662850e-02f,
                kGeluC4 = -7.198722102e-03f, kGeluC5 = 4.881033092e-04f;
__device__ __forceinline__ float fast_gelu(float v) {
  const float y = fabsf(v);
  float p = fmaf(kGeluC5, y, kGeluC4);
  p = fmaf(p, y, kGeluC3);
  p = fmaf(p, y, kGeluC2);
  p = fmaf(p, y, kGeluC1);
  const float e = __builtin_amdgcn_exp2f(-(p * y));
  const float d = copysignf(fmaf(-0.5f, e, 0.5f), v);              // Phi(v) - 1/2
  return v * (0.5f + d);
}

// gelu'(v) = Phi(v) + v phi(v) with the same Phi and phi(v) = exp2(-v^2 / (2 ln 2)) / sqrt(2 pi): two exponentials,
// |error| < 3e-6.
constexpr float kHalfLog2e = 0.72134752f, kInvSqrt2Pi = 0.39894228f;
__device__ __forceinline__ float fast_gelu_grad(float v) {
  const float y = fabsf(v);
  float p = fmaf(kGeluC5, y, kGeluC4);
  p = fmaf(p, y, kGeluC3);
  p = fmaf(p, y, kGeluC2);
  p = fmaf(p, y, kGeluC1);
  const float e = __builtin_amdgcn_exp2f(-(p * y));
  const float d = copysignf(fmaf(-0.5f, e, 0.5f), v);              // Phi(v) - 1/2
  const float dens = __builtin_amdgcn_exp2f(-kHalfLog2e * v * v) * kInvSqrt2Pi;
  return fmaf(v, dens, 0.5f + d);
}

// act'(p) for the epilogue that turns dH into dP (bf16 results: relative error far below the output resolution)
template <int ACT> __device__ __forceinline__ float epilogue_act_grad(float p) {
  if (ACT == MOE_ACT_RELU) return p > 0.f ? 1.f : 0.f;
  if (ACT == MOE_ACT_GELU) return fast_gelu_grad(p);
  const float sg = __builtin_amdgcn_rcpf(1.0f + __expf(-p));        // SiLU
  return sg * fmaf(p, 1.f - sg, 1.f);
}

template <int ACT> __device__ __forceinline__ float epilogue_act(float v) {
  if (ACT == MOE_ACT_RELU) return fmaxf(v, 0.f);
  if (ACT == MOE_ACT_GELU) return fast_gelu(v);
  if (ACT == MOE_ACT_SILU) return v * __builtin_amdgcn_rcpf(1.0f + __expf(-v));
  return v;
}

struct Frags {
  bf16x8 a[4], b[4];
};

// Inclusive prefix sum over the 64 lanes with data-parallel primitives (shifts inside rows of 16 lanes, then the rows'
// totals broadcast forward): no trip through the LDS crossbar, a few cycles per step.
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);    // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);    // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);    // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);    // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
  return v;
}

}  // namespace

// ---- main loop -------------------------------------------------------------------------------------------------
// K-step kt (64 wide) is four sub-steps of 16 MFMAs.  While sub-step s computes from one fragment buffer, the 12 LDS
// reads of sub-step s+1 fill the other.  The direct loads of K-step kt+2 go into the stage K-step kt is read from, so
// they may start only after the barrier that follows the last read of that stage (issued during sub-step 2): 8 of a
// wave's 16 loads are issued in sub-step 3 of K-step kt, the other 8 in sub-step 0 of K-step kt+1, and they are
// waited for before the barrier of K-step kt+1, two sub-steps later.
// GK (kTN only): the k-rows of A are gathered.  K-step t's row 2 (4 q + wave) + kg is row gk.rows[64 t + ...] of the
// matrix at a_base (row length gk.row_bytes); a_voff[0] then holds the lane's offset into the side buffer for q = 0.
struct GatherK {
  const int32_t* rows;          // this expert's slot -> row map (uniform)
  uint32_t row_bytes;           // bytes per row of the gathered matrix
  uint32_t nrows;               // rows of the gathered matrix (indices outside read row 0)
  uint32_t col;                 // per lane: byte offset of its 16-byte piece inside a row
  uint32_t tail_step;           // bytes between the side buffer's k-rows of consecutive q
};
template <int NI, int MODE, bool GK = false>
__device__ __forceinline__ void tile_main_loop(char* smem, const char* a_base, const char* b_base, const char* a_last,
                                               const char* b_last, const uint32_t (&a_voff)[8],
                                               const uint32_t (&b_voff)[8], int64_t a_step, int64_t b_step,
                                               const int (&a_off)[4], const int (&b_off)[4], int a_swz, int kg,
                                               int a_mask, int wave, int KT, const uint16_t* bias_w,
                                               f32x16 (&acc)[4][4], const GatherK& gk = GatherK{}) {
  constexpr bool FULL = NI == 4;
  constexpr bool TRA = MODE == kTN;          // A through transposing reads (two per fragment)
  constexpr bool TRB = MODE != kNT;          // B through transposing reads
  constexpr int NRA = TRA ? 8 : 4, NRB = TRB ? 8 : 4, NR = NRA + NRB;   // LDS reads per sub-step
  Frags f[2];
  const uint32_t smem_addr = (uint32_t)(uintptr_t)LDS_PTR(char, smem);

  // read number r (0 .. NR-1) of sub-step s from `stage` into fragment buffer `d`: first A's, then B's.  A direct read
  // fetches a lane's 8 k of one row (ds_read_b128); a transposed fragment takes two reads of 4 k each.
  auto read_direct = [&](const char* stage, int off, int s) -> bf16x8 {
    return *LDS_PTR(bf16x8, stage + off + (((2 * s + kg) ^ a_swz) << 4));
  };
  auto read_tr = [&](const char* stage, int off, int s, int half) -> short4v {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(short4v, stage + off + (16 * s + 4 * half) * 512));
  };
  auto join = [](short4v lo, short4v hi) -> bf16x8 {
    return __builtin_bit_cast(bf16x8, (short8v)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };
  auto read = [&](const char* stage, int s, int r, Frags& d, short4v (&lo)[8]) {
    if (r < NRA) {
      if (!TRA) {
        if (r < NI) d.a[r] = read_direct(stage, a_off[r], s);
      } else {
        const int i = r >> 1;
        if ((r & 1) == 0) lo[i] = read_tr(stage, a_off[i], s, 0);
        else d.a[i] = join(lo[i], read_tr(stage, a_off[i], s, 1));
      }
    } else if (NI > 0) {
      const int rb = r - NRA;
      if (!TRB) {
        d.b[rb] = read_direct(stage, b_off[rb], s);
      } else {
        const int j = rb >> 1;
        if ((rb & 1) == 0) lo[4 + j] = read_tr(stage, b_off[j], s, 0);
        else d.b[j] = join(lo[4 + j], read_tr(stage, b_off[j], s, 1));
      }
    }
  };
  // direct load number idx (0..15: A0..A7, B0..B7) of K-step `tile` (the caller guarantees tile < KT).  With a
  // transposed A the last K-step comes from the zero-padded side buffers.
  // gathered A: the eight row indices of one K-step are fetched a K-step before they are needed (plain loads, so the
  // wait the compiler puts before their use falls behind the barrier's own wait) and turned into offsets in place.
  // The last K-step comes from the zero-padded side buffer instead (tail).
  auto gather_fetch = [&](int tile, uint32_t (&g)[8]) {
    const int32_t* p = gk.rows + (int64_t)tile * BK + wave * 2 + kg;
#pragma unroll
    for (int q = 0; q < 8; ++q) g[q] = (uint32_t)p[8 * q];
  };
  auto gather_offsets = [&](bool tail, uint32_t (&g)[8]) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      if (tail) {
        g[q] = a_voff[0] + q * gk.tail_step;
      } else {
        const uint32_t r = g[q] < gk.nrows ? g[q] : 0u;
        g[q] = r * gk.row_bytes + gk.col;
      }
    }
  };
  uint32_t gv[8];
  auto dma = [&](int idx, int tile) {
    const int q = idx & 7;
    const uint32_t dst = smem_addr + (tile & 1) * kStageBytes + (q * 4 + wave) * 1024;
    const bool last = MODE == kTN && tile == KT - 1;
    if (idx < 8) {
      if (GK) {
        global_to_lds_16(last ? a_last : a_base, gv[q], dst);
      } else {
        const char* src = last ? a_last : a_base + tile * a_step;
        if (FULL || ((a_mask >> q) & 1)) global_to_lds_16(src, a_voff[q], dst);   // skip rows past the slab's fill
      }
    } else {
      const char* src = last ? b_last : b_base + tile * b_step;
      global_to_lds_16(src, b_voff[q], dst + kATileBytes);
    }
  };
  auto mfma = [&](int m, const Frags& c) {
    const int i = m >> 2, j = m & 3;
    if (i < NI) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(c.b[j], c.a[i], acc[i][j], 0, 0, 0);
  };
  // one sub-step: 16 MFMAs from `c`, interleaved with the NR reads of (stage, s_next) into `n` (if READS) and with the
  // direct loads dma_first .. dma_first+7 of K-step dma_tile (if DMA); both switches are compile-time so that the
  // steady-state loop body is branch-free
  auto substep = [&](auto reads_tag, auto dma_tag, const Frags& c, Frags& n, const char* stage, int s_next, int dma_first,
                     int dma_tile) {
    constexpr bool READS = decltype(reads_tag)::value, DMA = decltype(dma_tag)::value;
    short4v lo[8];
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      mfma(m, c);
      PIN();
      if (READS && m < NR) read(stage, s_next, m, n, lo);
      if (DMA && (m & 1) == 1) dma(dma_first + (m >> 1), dma_tile);
      PIN();
    }
  };
  using T_ = std::true_type;
  using F_ = std::false_type;
  // one K-step; DMA0: second half of the loads of K-step kt+1 (sub-step 0), DMA3: first half of K-step kt+2
  // (sub-step 3), NEXT: a K-step kt+1 exists
  // TAIL (gathered A only): K-step kt+2 is the last one
  auto kstep = [&](auto dma0_tag, auto dma3_tag, auto next_tag, int kt, auto tail_tag) {
    constexpr bool TAIL = decltype(tail_tag)::value;
    const char* cur = smem + (kt & 1) * kStageBytes;
    const char* nxt = smem + ((kt + 1) & 1) * kStageBytes;
    if (GK && decltype(dma3_tag)::value && !TAIL) { gather_fetch(kt + 2, gv); PIN(); }
    substep(T_{}, dma0_tag, f[0], f[1], cur, 1, 8, kt + 1);
    substep(T_{}, F_{}, f[1], f[0], cur, 2, 0, 0);
    substep(T_{}, F_{}, f[0], f[1], cur, 3, 0, 0);
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");      // K-step kt+1 has landed; reads of `cur` are done
    PIN();
    asm volatile("s_barrier" ::: "memory");
    PIN();
    if (GK && decltype(dma3_tag)::value) { gather_offsets(TAIL, gv); PIN(); }   // nothing else is in flight here
    substep(next_tag, dma3_tag, f[1], f[0], nxt, 0, 0, kt + 2);
  };

  uint32_t gv1[8];
  if (GK) {                                                         // both K-steps' indices before any direct load is in flight
    if (KT > 1) gather_fetch(0, gv);
    if (KT > 2) gather_fetch(1, gv1);
    gather_offsets(KT == 1, gv);
  }
#pragma unroll
  for (int idx = 0; idx < kLoadsPerWave; ++idx) dma(idx, 0);
  if (KT > 1) {
    if (GK) {
      gather_offsets(KT == 2, gv1);
#pragma unroll
      for (int q = 0; q < 8; ++q) gv[q] = gv1[q];
    }
#pragma unroll
    for (int idx = 0; idx < kLoadsPerWave; ++idx) dma(idx, 1);
  }
  // while the first stages are in flight: the accumulators start from the bias (register 4 g + u of tile (i, j) is
  // column 32 j + 8 g + 4 kg + u of the wave's 128), or from zero
#pragma unroll
  for (int j = 0; j < 4; ++j) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      float b0 = 0.f, b1 = 0.f, b2 = 0.f, b3 = 0.f;
      if (bias_w) {
        const u32x2 bb = *reinterpret_cast<const u32x2*>(bias_w + j * 32 + 8 * g + 4 * kg);
        b0 = __uint_as_float(bb.x << 16); b1 = __uint_as_float(bb.x & 0xffff0000u);
        b2 = __uint_as_float(bb.y << 16); b3 = __uint_as_float(bb.y & 0xffff0000u);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (i < NI) { acc[i][j][4 * g] = b0; acc[i][j][4 * g + 1] = b1; acc[i][j][4 * g + 2] = b2; acc[i][j][4 * g + 3] = b3; }
      }
    }
  }
  PIN();
  if (KT > 1) {
    if (FULL) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");     // loads return in order: K-step 0 has landed
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");           // ragged tiles issue fewer loads: wait for all
  } else {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  PIN();
  asm volatile("s_barrier" ::: "memory");
  PIN();
  {
    short4v lo[8];
#pragma unroll
    for (int r = 0; r < NR; ++r) read(smem, 0, r, f[0], lo);
  }
  PIN();

  if (KT >= 3) {
    if (GK) {                                                        // the K-step that loads the last one is peeled as well
      if (KT == 3) kstep(F_{}, T_{}, T_{}, 0, T_{});
      else kstep(F_{}, T_{}, T_{}, 0, F_{});
      for (int kt = 1; kt < KT - 3; ++kt) kstep(T_{}, T_{}, T_{}, kt, F_{});
      if (KT > 3) kstep(T_{}, T_{}, T_{}, KT - 3, T_{});
    } else {
      kstep(F_{}, T_{}, T_{}, 0, F_{});                              // K-step 1 was loaded whole in the prologue
      for (int kt = 1; kt < KT - 2; ++kt) kstep(T_{}, T_{}, T_{}, kt, F_{});
    }
    kstep(T_{}, F_{}, T_{}, KT - 2, F_{});                           // no K-step KT to load
    kstep(F_{}, F_{}, F_{}, KT - 1, F_{});
  } else if (KT == 2) {
    kstep(F_{}, F_{}, T_{}, 0, F_{});
    kstep(F_{}, F_{}, F_{}, 1, F_{});
  } else {
    kstep(F_{}, F_{}, F_{}, 0, F_{});
  }
}

// A weight-gradient product (kTN) reduces over an expert's slots: K-steps of 64 slots, the last one (whole or not) read
// from the side buffers, which also covers an expert without any slot (one K-step of zeros).
__host__ __device__ inline int slot_ksteps(int64_t fill) { return fill > 0 ? (int)((fill + BK - 1) / BK) : 1; }

// Tiles per group of the block numbering (log2): 32 when the launch has several rounds of tiles for every compute unit;
// fewer when it has not, so that the groups, which are dealt whole to the XCDs, still spread evenly over them.
__host__ __device__ inline int group_size_log2(int64_t live_tiles) { return live_tiles >= 1024 ? 5 : (live_tiles >= 512 ? 4 : 3); }

// Blocks to launch so that every tile is reached whatever the fills turn out to be and whichever group size they select.
static inline unsigned tile_grid(int64_t E, int64_t MT, int64_t NT) {
  int64_t blocks = 0;
  for (int gs = 3; gs <= 5; ++gs) {
    const int64_t G = (int64_t)1 << gs, groups = E * ceil_div(MT * NT, G);      // upper bound: every expert full
    const int64_t b = ceil_div(groups, 8) * 8 * G;                              // G blocks per group, groups dealt to 8 XCDs
    blocks = b > blocks ? b : blocks;
  }
  return (unsigned)blocks;
}

// Which tile block number b works on (see the numbering described in the kernel below).  Returns kTileNone past the last
// live group, kTileIdle for an idle slot of a short group, kTileLive otherwise with the expert, its row and column tile and
// the expert's number of real rows.
constexpr int kTileLive = 0, kTileIdle = 1, kTileNone = 2;
__device__ __forceinline__ int find_tile(int b, int lane, int E, int64_t C, const int32_t* __restrict__ counts, int NT,
                                         int& e_out, int& mt_out, int& nt_out, int& rows_out) {
  auto live_rows = [&](int el) -> int {                             // rows of expert el that exist (its fill, at most C)
    if (el >= E) return 0;
    int64_t r = C;
    if (counts) { const int64_t c = counts[el]; r = c < C ? (c > 0 ? c : 0) : C; }
    return (int)r;
  };
  constexpr int kChunks = kMaxExperts / 64;
  int rowsv[kChunks], mtv[kChunks];                                 // lane l of chunk c: rows / live row tiles of expert 64 c + l
#pragma unroll
  for (int c = 0; c < kChunks; ++c) rowsv[c] = c * 64 < E ? live_rows(c * 64 + lane) : 0;      // all loads in flight at once
#pragma unroll
  for (int c = 0; c < kChunks; ++c) mtv[c] = (rowsv[c] + BM - 1) / BM;
  int live_tiles = 0;                                               // live tiles of all experts
#pragma unroll
  for (int c = 0; c < kChunks; ++c) {
    if (c * 64 >= E) break;
    live_tiles += __builtin_amdgcn_readlane(wave_inclusive_scan(mtv[c] * NT), 63);
  }
  const int gs = group_size_log2(live_tiles), G = 1 << gs;          // tiles per group
  const int group = ((b / 8) >> gs) * 8 + b % 8, slot = (b / 8) & (G - 1);
  int total_full = 0;                                               // full groups of all experts
#pragma unroll
  for (int c = 0; c < kChunks; ++c) {
    if (c * 64 >= E) break;
    total_full += __builtin_amdgcn_readlane(wave_inclusive_scan((mtv[c] * NT) >> gs), 63);
  }
  const bool short_group = group >= total_full;
  const int target = short_group ? group - total_full : group;
  int e = -1, mte = 0, rank = 0, rows_e = 0;                        // expert, its live row tiles, group's rank among its own, its rows
  int base = 0;
#pragma unroll
  for (int c = 0; c < kChunks; ++c) {
    if (c * 64 >= E || e >= 0) break;
    const int mt_l = mtv[c];
    const int ng_l = short_group ? (((mt_l * NT) & (G - 1)) != 0 ? 1 : 0) : (mt_l * NT) >> gs;
    const int inc = wave_inclusive_scan(ng_l);                      // inclusive prefix sum over the wave
    const int tot = __builtin_amdgcn_readlane(inc, 63);
    if (target < base + tot) {
      const unsigned long long hit = __ballot(base + inc > target);
      const int l = __builtin_amdgcn_readfirstlane(__builtin_ctzll(hit));
      e = c * 64 + l;                                               // the same in every lane: keep them in scalar registers
      mte = __builtin_amdgcn_readlane(mt_l, l);
      rows_e = __builtin_amdgcn_readlane(rowsv[c], l);
      rank = target - (base + __builtin_amdgcn_readlane(inc - ng_l, l));
    }
    base += tot;
  }
  if (e < 0) return kTileNone;                                      // past the last live group
  const int q = ((short_group ? (mte * NT) >> gs : rank) << gs) + slot;
  if (q >= mte * NT) return kTileIdle;                              // idle slot of a short group
  const int full = (NT / 8) * mte * 8;                              // live tiles of this expert in full 8-column blocks
  int mt, nt;
  if (q < full) { mt = (q % (mte * 8)) / 8; nt = (q / (mte * 8)) * 8 + q % 8; }
  else { const int w = NT % 8, r = q - full; mt = r / w; nt = (NT / 8) * 8 + r % w; }
  e_out = e; mt_out = mt; nt_out = nt; rows_out = rows_e;
  return kTileLive;
}

// GRAD (kNT only): the epilogue multiplies by act'(pre) read from `pre` [E,C,N], i.e. the product is the gradient with
// respect to the pre-activations of a layer whose activation is ACT; with ACT < 0 it adds `pre` instead (a product
// accumulated onto an existing matrix; `pre` may then be `out` itself, every element being read before it is written
// by the same lane).
// DUAL (kNN with an activation only): the values before the activation are written to `pre_out` as well.
// GK (kTN only): A's k-rows (slots) are gathered through `gather` [E, K] from the matrix A [gather_rows, C] (the token
// matrix, for the first layer's weight gradient when the dispatch buffer was never written).
template <int ACT, int MODE, bool GRAD, bool DUAL = false, bool GK = false>
__global__ __launch_bounds__(kThreads) void grouped_gemm_mfma_kernel(const uint16_t* __restrict__ A,
                                                                     const uint16_t* __restrict__ B,
                                                                     const uint16_t* __restrict__ bias,
                                                                     const int32_t* __restrict__ counts,
                                                                     const int32_t* __restrict__ gather, int gather_rows,
                                                                     int E, int64_t C, int K, int N, int MT, int NT,
                                                                     uint16_t* out,                 // may alias `pre`
                                                                     const int32_t* __restrict__ kfill,
                                                                     const uint16_t* __restrict__ a_tail,
                                                                     const uint16_t* __restrict__ b_tail,
                                                                     const uint16_t* pre,
                                                                     uint16_t* __restrict__ pre_out) {
  __shared__ __attribute__((aligned(1024))) char smem[2 * kStageBytes];

  // ---- which tile -------------------------------------------------------------------------------------------------
  // An expert's live tiles (row tiles below its fill x all column tiles) are numbered by blocks of 8 tile columns and,
  // inside a block, row by row: 32 consecutive numbers are 4 row tiles x 8 column tiles that share A rows and B
  // columns.  Each expert's numbering is cut into groups of 32; the full groups of all experts are numbered first,
  // then the short last groups (ragged tails), and this sequence is dealt round-robin to the 8 XCDs: hardware deals
  // blocks round-robin, so block b runs on XCD b % 8, whose 32 CUs hold one group at a time in their own L2.  Counting
  // only live groups, full ones first, keeps the XCDs evenly loaded whatever the experts' fills are.  Every wave finds
  // its group by prefix sums over the experts' group counts, 64 experts per step.  A launch with few live tiles (a
  // couple of rounds per compute unit or less) cuts groups of 16 or 8 instead: whole groups go to one XCD, and with 32
  // per group a handful of them would leave some XCDs with twice the work of others.
  const int lane = threadIdx.x & 63;
  int e, mt, nt, rows_e;
  if (find_tile(blockIdx.x, lane, E, C, counts, NT, e, mt, nt, rows_e) != kTileLive) return;
  const int64_t rows = rows_e;                                      // already here from the search: no second trip to memory
  const int64_t m0 = (int64_t)mt * BM;
  if (m0 >= rows) return;                                           // cannot happen (mt < mte); keeps every access in the slab
  const int n0 = nt * BN;

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  // ---- global sources of this lane's direct-to-LDS loads (32-bit offsets from per-expert scalar bases) -------------
  // Row-major operand with k contiguous (A of kNN/kNT, B of kNT): 1 KB block q*4+wave of the tile = rows
  //   8(q*4+wave) .. +7, lane l writes row +l/8, chunk position l%8.
  // Operand with k as the slow index (B of kNN/kTN, A of kTN): 1 KB block q*4+wave = k-rows 2(q*4+wave), +1, lane l
  //   writes k-row +l/32, chunk position l%32.
  // With `gather` (the slot -> token map [E, C] of the dispatch), A is the token matrix [gather_rows, K] itself and row r
  // of expert e's slab is token gather[e, r]: the dispatch buffer is never written or read.  Unfilled slots (-1) read
  // token 0; their output rows lie past the expert's fill and are never used.
  const char* a_base;
  const char* b_base;
  const char* a_last = nullptr;
  const char* b_last = nullptr;
  int KT = K / BK;
  if (MODE == kTN) {                                                // A [E, K slots, C], B [E, K slots, N]
    a_base = GK ? (const char*)A : (const char*)(A + (int64_t)e * K * C);
    b_base = (const char*)(B + (int64_t)e * K * N);
    int64_t fill = K;
    if (kfill) { const int64_t c = kfill[e]; fill = c < K ? (c > 0 ? c : 0) : K; }
    KT = slot_ksteps(fill);
    a_last = (const char*)(a_tail + (int64_t)e * BK * C);
    b_last = (const char*)(b_tail + (int64_t)e * BK * N);
  } else {
    a_base = gather ? (const char*)A : (const char*)(A + (int64_t)e * C * K);
    b_base = (const char*)(B + (int64_t)e * K * N);
  }
  uint32_t a_voff[8], b_voff[8];
  int a_mask = 0;                                                   // bit q: A block q of this wave holds at least one real row
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int r = (q * 4 + wave) * 8 + (lane >> 3);                 // row of a k-contiguous tile
    const int g = (lane & 7) ^ ((r >> 1) & 7);                      // global chunk that lands at position lane % 8
    const int kr = (q * 4 + wave) * 2 + (lane >> 5);                // k-row of a k-slow tile
    const int c = (lane & 31) ^ (4 * (kr & 3));
    if (MODE == kTN) {
      a_mask |= 1 << q;
      a_voff[q] = (uint32_t)(((int64_t)kr * C + m0 + c * 8) * 2);
    } else {
      if (m0 + (q * 4 + wave) * 8 < rows) a_mask |= 1 << q;
      int64_t row = m0 + r;
      row = row < C ? row : C - 1;                                  // rows past the slab are clamped (never stored)
      if (gather) {
        const int t = gather[(int64_t)e * C + row];
        row = (unsigned)t < (unsigned)gather_rows ? t : 0;
      }
      a_voff[q] = (uint32_t)((row * K + g * 8) * 2);
    }
    if (MODE == kNT) b_voff[q] = (uint32_t)(((int64_t)(n0 + r) * K + g * 8) * 2);
    else b_voff[q] = (uint32_t)(((int64_t)kr * N + n0 + c * 8) * 2);
  }
  const int64_t a_step = MODE == kTN ? (int64_t)BK * C * 2 : (int64_t)BK * 2;
  const int64_t b_step = MODE == kNT ? (int64_t)BK * 2 : (int64_t)BK * N * 2;

  // ---- LDS read offsets of this lane's MFMA fragments ------------------------------------------------------------
  // direct (k-contiguous tile): row * 128, + ((2 s + kg) ^ a_swz) * 16 per sub-step s
  // transposed (k-slow tile):   k-row * 512 + swizzled 16-byte chunk + 8-byte half, + (16 s + 4 half) * 512
  const int kg = lane >> 5;
  const int a_swz = ((lane & 31) >> 1) & 7;                         // ((row >> 1) & 7): tile-row offsets are multiples of 32
  auto direct_off = [&](int w, int t) { return (w * 128 + t * 32 + (lane & 31)) * 128; };
  auto tr_off = [&](int w, int t) {
    const int c = w * 16 + t * 4 + ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1);
    const int swz = 4 * ((lane >> 2) & 3);                          // 4 (k & 3), k & 3 = (lane % 16) / 4
    return (kg * 8 + ((lane & 15) >> 2)) * 512 + ((c ^ swz) << 4) + ((lane & 1) << 3);
  };
  int a_off[4], b_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a_off[i] = MODE == kTN ? tr_off(wm, i) : direct_off(wm, i);
    b_off[i] = kATileBytes + (MODE == kNT ? direct_off(wn, i) : tr_off(wn, i));
  }
  // 32-row sub-tiles of this wave that hold real rows (the last row tile of an expert is usually ragged)
  const int64_t wave_rows = rows - m0 - wm * 128;
  const int ni = wave_rows >= 128 ? 4 : (wave_rows <= 0 ? 0 : (int)((wave_rows + 31) >> 5));

  f32x16 acc[4][4];
  const uint16_t* bias_w = bias ? bias + (int64_t)e * N + n0 + wn * 128 : nullptr;

  // the number of live sub-tiles is a template argument, so that the loop body of a ragged tile is as branch-free as a
  // full one's (a wave with no rows still loads its share of B and joins the barriers)
#define MOE_TILE_LOOP(NI) tile_main_loop<NI, MODE>(smem, a_base, b_base, a_last, b_last, a_voff, b_voff, a_step, b_step, a_off, b_off, a_swz, kg, a_mask, wave, KT, bias_w, acc)
  if (MODE == kTN && GK) {
    GatherK gk;
    gk.rows = gather + (int64_t)e * K;
    gk.row_bytes = (uint32_t)(C * 2);
    gk.nrows = (uint32_t)gather_rows;
    gk.col = a_voff[0] - (uint32_t)((wave * 2 + kg) * C * 2);       // (m0 + 8 c) * 2: the k-row term taken out again
    gk.tail_step = (uint32_t)(8 * C * 2);
    tile_main_loop<4, MODE, true>(smem, a_base, b_base, a_last, b_last, a_voff, b_voff, a_step, b_step, a_off, b_off, a_swz, kg,
                                  a_mask, wave, KT, bias_w, acc, gk);
  } else if (MODE == kTN) {                                         // output rows are a weight dimension: never ragged
    MOE_TILE_LOOP(4);
  } else {
    switch (ni) {
      case 4: MOE_TILE_LOOP(4); break;
      case 3: MOE_TILE_LOOP(3); break;
      case 2: MOE_TILE_LOOP(2); break;
      case 1: MOE_TILE_LOOP(1); break;
      default: MOE_TILE_LOOP(0); break;
    }
  }
#undef MOE_TILE_LOOP

  // ---- epilogue: activation, bf16; transposed through LDS so that global stores are 16 bytes per lane and a
  // wave's store covers 4 rows x 256 contiguous bytes.  After the last barrier of the main loop no wave reads the
  // stages and no direct load is in flight, so wave w may use the 32 KB at smem + 32 KB * w as its own
  // [128 rows][16 chunks of 8 columns]; chunk c of row r sits at position c ^ (r % 16), which makes both the 8-byte
  // writes (32 rows per instruction) and the 16-byte row-contiguous reads conflict-free.
  // A DUAL kernel writes the tile twice: first the values before the activation (what a training step keeps for the
  // backward pass), then the activated ones.
  char* wtile = smem + wave * 32768;
  const int64_t out_at = ((int64_t)e * C + m0 + wm * 128) * N + n0 + wn * 128;
  const int64_t live = rows - m0 - wm * 128;                        // rows of this wave's tile that exist
  auto write_tile = [&](auto raw_tag, uint16_t* dst) {
    constexpr bool RAW = decltype(raw_tag)::value;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (i >= ni) break;
      const int r = i * 32 + (lane & 31);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float v[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) v[u] = acc[i][j][4 * g + u];
#pragma unroll
          for (int u = 0; u < 4; ++u) v[u] = epilogue_act<(GRAD || RAW) ? -1 : ACT>(v[u]);
          u32x2 pk;
          pk.x = pack_bf16x2(v[0], v[1]);
          pk.y = pack_bf16x2(v[2], v[3]);
          *LDS_PTR(u32x2, wtile + r * 256 + (((4 * j + g) ^ (r & 15)) << 4) + 8 * kg) = pk;
        }
      }
    }
    uint16_t* oute = dst + out_at;
    for (int it0 = 0; it0 < 32; it0 += 8) {
      if (it0 * 4 >= ni * 32) break;
      uint4 pv8[8];
      if (GRAD && !RAW) {                                           // this batch's pre-activations, all loads in flight at once
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int r = (it0 + u) * 4 + (lane >> 4);
          const int rr = r < live ? r : 0;                          // rows past the fill: any valid row, result unused
          pv8[u] = *reinterpret_cast<const uint4*>(pre + out_at + (int64_t)rr * N + (((lane & 15) ^ (rr & 15)) << 3));
        }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int r = (it0 + u) * 4 + (lane >> 4);
        u32x4 q = *LDS_PTR(u32x4, wtile + r * 256 + ((lane & 15) << 4));
        if (r < live) {
          const int64_t at = (int64_t)r * N + (((lane & 15) ^ (r & 15)) << 3);
          if (GRAD && !RAW) {                                       // times act'(pre), both factors as stored (bf16); or plus `pre`
            float g[8], pv[8];
            Vec16<uint16_t>::unpack(__builtin_bit_cast(uint4, q), g);
            Vec16<uint16_t>::unpack(pv8[u], pv);
#pragma unroll
            for (int v = 0; v < 8; ++v) g[v] = ACT < 0 ? g[v] + pv[v] : g[v] * epilogue_act_grad<ACT>(pv[v]);
            q = __builtin_bit_cast(u32x4, Vec16<uint16_t>::pack(g));
          }
          *reinterpret_cast<u32x4*>(oute + at) = q;
        }
      }
    }
  };
  if (DUAL) write_tile(std::true_type{}, pre_out);
  write_tile(std::false_type{}, out);
}

// dst[e, j, :] = src[e, 64 (KT_e - 1) + j, :] if that slot is below the expert's fill, else 0, for j < 64: the last
// K-step of a kTN product.   src [E, C, W], dst [E, 64, W]; 16-byte pieces, one block per (expert, 4 slots).
__global__ __launch_bounds__(256) void tail_rows_kernel(const uint4* __restrict__ src, const int32_t* __restrict__ kfill,
                                                        int64_t C, int cpr, uint4* __restrict__ dst,
                                                        const int32_t* __restrict__ gather, int64_t gather_rows) {
  const int e = blockIdx.y;
  int64_t fill = C;
  if (kfill) { const int64_t c = kfill[e]; fill = c < C ? (c > 0 ? c : 0) : C; }
  const int64_t first = (int64_t)(slot_ksteps(fill) - 1) * BK;
  const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t slot = first + j;
  int64_t row = (int64_t)e * C + slot;
  if (gather && slot < fill) {                                      // the slot's row of the gathered matrix
    const int64_t t = gather[row];
    row = t >= 0 && t < gather_rows ? t : 0;
  }
  for (int ch = threadIdx.x & 63; ch < cpr; ch += 64)
    dst[((int64_t)e * BK + j) * cpr + ch] = slot < fill ? src[row * cpr + ch] : make_uint4(0, 0, 0, 0);
}

bool grouped_gemm_mfma_supports(int64_t E, int64_t C, int64_t K, int64_t N, int64_t gather_rows) {
  if (K % BK != 0 || N % BN != 0 || E > kMaxExperts) return false;
  const int64_t tiles = E * ceil_div(C, BM) * (N / BN);
  // 32-bit byte offsets inside one expert's A slab (or the whole token matrix when gathering) and B matrix
  const int64_t a_rows = gather_rows > 0 ? gather_rows : C;
  return tiles < ((int64_t)1 << 30) && a_rows * K * 2 < ((int64_t)1 << 32) && K * N * 2 < ((int64_t)1 << 32) &&
         gather_rows < ((int64_t)1 << 31);
}

hipError_t launch_grouped_gemm_mfma(const void* A, const void* B, const void* bias, int act, const int32_t* counts,
                                    int64_t E, int64_t C, int64_t K, int64_t N, void* out, hipStream_t s,
                                    const int32_t* gather, int64_t gather_rows, void* pre_out) {
  const int MT = (int)ceil_div(C, BM), NT = (int)(N / BN);
  const dim3 grid(tile_grid(E, MT, NT)), block(kThreads);
#define MOE_LAUNCH_GEMM(ACT, DUAL)                                                                                    \
  grouped_gemm_mfma_kernel<ACT, kNN, false, DUAL><<<grid, block, 0, s>>>(                                             \
      (const uint16_t*)A, (const uint16_t*)B, (const uint16_t*)bias, counts, gather, (int)gather_rows, (int)E, C,     \
      (int)K, (int)N, MT, NT, (uint16_t*)out, nullptr, nullptr, nullptr, nullptr,                                       \
      (uint16_t*)pre_out)
  if (pre_out && act >= 0) {
    switch (act) {
      case MOE_ACT_RELU: MOE_LAUNCH_GEMM(MOE_ACT_RELU, true); break;
      case MOE_ACT_GELU: MOE_LAUNCH_GEMM(MOE_ACT_GELU, true); break;
      default: MOE_LAUNCH_GEMM(MOE_ACT_SILU, true); break;
    }
  } else {
    switch (act) {
      case MOE_ACT_RELU: MOE_LAUNCH_GEMM(MOE_ACT_RELU, false); break;
      case MOE_ACT_GELU: MOE_LAUNCH_GEMM(MOE_ACT_GELU, false); break;
      case MOE_ACT_SILU: MOE_LAUNCH_GEMM(MOE_ACT_SILU, false); break;
      default: MOE_LAUNCH_GEMM(-1, false); break;
    }
  }
#undef MOE_LAUNCH_GEMM
  return hipGetLastError();
}

// out[e] = A[e] (rows_e x K) * Bt[e]^T, Bt [E, N, K]; with `pre` [E, C, N] the result is multiplied by act'(pre), or,
// with act < 0, has `pre` added (pre == out accumulates in place).
hipError_t launch_grouped_gemm_mfma_nt(const void* A, const void* Bt, const int32_t* counts, int64_t E, int64_t C,
                                       int64_t K, int64_t N, void* out, const void* pre, int act, hipStream_t s) {
  const int MT = (int)ceil_div(C, BM), NT = (int)(N / BN);
  const dim3 grid(tile_grid(E, MT, NT)), block(kThreads);
#define MOE_LAUNCH_GEMM(ACT, GRAD)                                                                                    \
  grouped_gemm_mfma_kernel<ACT, kNT, GRAD><<<grid, block, 0, s>>>(                                                    \
      (const uint16_t*)A, (const uint16_t*)Bt, nullptr, counts, nullptr, 0, (int)E, C, (int)K, (int)N, MT, NT,        \
      (uint16_t*)out, nullptr, nullptr, nullptr, (const uint16_t*)pre, nullptr)
  if (!pre) MOE_LAUNCH_GEMM(-1, false);
  else if (act < 0) MOE_LAUNCH_GEMM(-1, true);                      // out = product + pre
  else switch (act) {
    case MOE_ACT_RELU: MOE_LAUNCH_GEMM(MOE_ACT_RELU, true); break;
    case MOE_ACT_GELU: MOE_LAUNCH_GEMM(MOE_ACT_GELU, true); break;
    default: MOE_LAUNCH_GEMM(MOE_ACT_SILU, true); break;
  }
#undef MOE_LAUNCH_GEMM
  return hipGetLastError();
}

// out[e] (R x N) = At[e]^T * B[e] over the first min(kfill[e], C) of the C slots; At [E, C, R], B [E, C, N], R and N
// multiples of 256.  a_tail [E, 64, R] and b_tail [E, 64, N] are scratch for the zero-padded last K-step.
// With `gather` [E, C] (slot -> row, as the dispatch builds it) At is one matrix [gather_rows, R] and slot c of expert e
// is its row gather[e, c]; gather_rows * R * 2 must stay below 2^32.
hipError_t launch_grouped_gemm_mfma_tn(const void* At, const void* B, const int32_t* kfill, int64_t E, int64_t C, int64_t R,
                                       int64_t N, void* a_tail, void* b_tail, void* out, hipStream_t s,
                                       const int32_t* gather, int64_t gather_rows) {
  const int cprR = (int)(R / 8), cprN = (int)(N / 8);
  tail_rows_kernel<<<dim3(BK / 4, (unsigned)E), dim3(256), 0, s>>>((const uint4*)At, kfill, C, cprR, (uint4*)a_tail, gather, gather_rows);
  tail_rows_kernel<<<dim3(BK / 4, (unsigned)E), dim3(256), 0, s>>>((const uint4*)B, kfill, C, cprN, (uint4*)b_tail, nullptr, 0);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  const int MT = (int)(R / BM), NT = (int)(N / BN);
  const dim3 grid(tile_grid(E, MT, NT)), block(kThreads);
  if (gather)
    grouped_gemm_mfma_kernel<-1, kTN, false, false, true><<<grid, block, 0, s>>>(
        (const uint16_t*)At, (const uint16_t*)B, nullptr, nullptr, gather, (int)gather_rows, (int)E, R, (int)C, (int)N, MT, NT,
        (uint16_t*)out, kfill, (const uint16_t*)a_tail, (const uint16_t*)b_tail, nullptr, nullptr);
  else
    grouped_gemm_mfma_kernel<-1, kTN, false><<<grid, block, 0, s>>>(
        (const uint16_t*)At, (const uint16_t*)B, nullptr, nullptr, nullptr, 0, (int)E, R, (int)C, (int)N, MT, NT,
        (uint16_t*)out, kfill, (const uint16_t*)a_tail, (const uint16_t*)b_tail, nullptr, nullptr);
  return hipGetLastError();
}

// One [rows, K] x [N, K]^T product (a single "expert"): shapes the kNT layout takes.
bool grouped_gemm_mfma_supports_nt(int64_t rows, int64_t K, int64_t N) {
  return grouped_gemm_mfma_supports(1, rows, K, N, 0) && N * K * 2 < ((int64_t)1 << 32);
}

// Shapes for which the whole backward of the expert layer runs on the three layouts above.
bool grouped_gemm_mfma_supports_backward(int64_t E, int64_t C, int64_t M, int64_t H) {
  const int64_t W = M > H ? M : H;
  const int64_t tiles = E * ceil_div(C > W ? C : W, BM) * (W / BN);
  return M % BN == 0 && H % BN == 0 && E <= kMaxExperts && tiles < ((int64_t)1 << 30) &&
         C * W * 2 < ((int64_t)1 << 32) && M * H * 2 < ((int64_t)1 << 32);
}

}  // namespace moe
