// Shared device helpers and internal launcher declarations of the MoE hot-path library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/moe_mi355x.h"

namespace moe {

constexpr int kWave = 64;            // CDNA wavefront width
constexpr int kGateTokensPerBlock = 64;    // tokens whose arrivals one gate block counts and ranks (one wave in assign)

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even fp32 -> bf16 bit pattern (NaN stays NaN)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// two fp32 -> packed bf16 pair (low half = a), round-to-nearest-even in hardware (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

template <typename T> __device__ __forceinline__ float load_as_f32(const T* p);
template <> __device__ __forceinline__ float load_as_f32<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_as_f32<uint16_t>(const uint16_t* p) { return bf16_bits_to_f32(*p); }

template <typename T> __device__ __forceinline__ void store_from_f32(T* p, float v);
template <> __device__ __forceinline__ void store_from_f32<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_from_f32<uint16_t>(uint16_t* p, float v) { *p = f32_to_bf16_bits(v); }

__device__ __forceinline__ float apply_act(float v, int act) {
  if (act == MOE_ACT_RELU) return v > 0.f ? v : 0.f;
  if (act == MOE_ACT_GELU) return 0.5f * v * (1.0f + erff(v * 0.70710678118654752440f));
  return v / (1.0f + __expf(-v));
}

// derivative of the activation at pre-activation p
__device__ __forceinline__ float apply_act_grad(float p, int act) {
  if (act == MOE_ACT_RELU) return p > 0.f ? 1.f : 0.f;
  if (act == MOE_ACT_GELU) return 0.5f * (1.f + erff(p * 0.70710678118654752440f)) + p * expf(-0.5f * p * p) * 0.39894228040143267794f;
  const float sg = 1.f / (1.f + expf(-p));                  // SiLU
  return sg * (1.f + p * (1.f - sg));
}

// 16 bytes of `ET` as floats and back
template <typename ET> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[4]) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
  static __device__ __forceinline__ uint4 pack(const float (&f)[4]) {
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
  }
};
template <> struct Vec16<uint16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[8]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ uint4 pack(const float (&f)[8]) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(f[2 * i], f[2 * i + 1]);
    return make_uint4(w[0], w[1], w[2], w[3]);
  }
};

// 16-byte load of data that is read once (streamed rows): the nontemporal hint keeps it from displacing reusable lines
// and measurably raises read bandwidth on this chip (6.0 -> 6.7 TB/s on a plain read stream).
__device__ __forceinline__ uint4 load_stream(const uint4* p) {
  typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t a, size_t b) { return (a + b - 1) / b * b; }

// ---- launchers (defined in gate.hip / dispatch.hip / ffn_*.hip / api.hip); arguments are already validated --------
hipError_t launch_gate_logits(const void* x, const void* Wg, const float* bias, int dtype, int64_t T, int64_t M,
                              int64_t E, float* logits, hipStream_t s);
hipError_t launch_gate_logits_cosine(const void* x, const void* Wp, const float* Me, double tau, int dtype, int64_t T,
                                     int64_t M, int64_t D, int64_t E, float* logits, float* proj, double* MeT, double* norm,
                                     hipStream_t s);
// Fast gate logits (gate_fast.hip): workspace pieces and what the top-k kernel needs to repair near-ties exactly
struct GateFastWorkspace {
  uint16_t* Wt;                                           // [E, Mp] = Wg^T, rows zero-padded
  float* wnorm;                                           // [E]
  float* margin;                                          // [T] error bound of a token's logits
  int64_t Mp;
};
struct GateRepair {
  const float* margin;
  const void* x;
  const uint16_t* Wt;
  const float* bias;
  int64_t M, Mp;
};
size_t gate_fast_workspace_bytes(int64_t T, int64_t M, int64_t E);
GateFastWorkspace gate_fast_layout(void* ws, int64_t T, int64_t M, int64_t E);
bool gate_logits_fast_supports(int dtype, int64_t T, int64_t M, int64_t E);
hipError_t launch_gate_logits_fast(const void* x, const void* Wg, const float* bias, int64_t T, int64_t M, int64_t E,
                                   float* logits, const GateFastWorkspace& w, hipStream_t s);
// `repair` (optional): the logits are approximate to within repair->margin[t]; near-ties are then recomputed in fp64 and
// written back into `logits` (not combinable with `perm`)
hipError_t launch_gate_topk(float* logits, int64_t T, int64_t E, int k, int64_t C, int normalize, int32_t* idx,
                            float* gate_w, int32_t* loc, int32_t* counts, int32_t* slot_src, int32_t* block_counts,
                            hipStream_t s, const int32_t* perm = nullptr, const GateRepair* repair = nullptr);
size_t bpr_order_workspace_bytes(int64_t T);
hipError_t launch_bpr_order(const float* logits, int64_t T, int64_t E, void* ws, const int32_t** perm, hipStream_t s);
hipError_t launch_decode_backward(const void* d_out, const void* Y, int dtype, const int32_t* idx, const int32_t* loc,
                                  const float* gate_w, const int32_t* slot_src, int64_t T, int64_t M, int64_t E, int k,
                                  int64_t C, void* dY, float* dgate_w, hipStream_t s, bool fill_unfilled = true);
// out[0] = capacity: `fixed` if > 0, else max_e counts[e]; never above `bound` (if > 0); out[1] = max_e counts[e];
// fills[e] (optional) = min(counts[e], out[0])
hipError_t launch_dynamic_capacity(const int32_t* counts, int64_t E, int64_t bound, int64_t* out, hipStream_t s,
                                   int64_t fixed = 0, int32_t* fills = nullptr);
// C_dev (optional, device): only choices with loc < min(*C_dev, C) are kept; slot_src keeps its [E, C] layout
hipError_t launch_slot_sources(const int32_t* idx, const int32_t* loc, int64_t T, int64_t E, int k, int64_t C,
                               int32_t* slot_src, hipStream_t s, const int64_t* C_dev = nullptr);
// C_dev (optional, device): as for launch_slot_sources (slot_src must have been built with the same C_dev)
hipError_t launch_encode(const void* x, int dtype, const int32_t* idx, const int32_t* loc, const int32_t* slot_src,
                         int64_t T, int64_t M, int64_t E, int k, int64_t C, void* Z, hipStream_t s,
                         bool fill_unfilled = true, const int64_t* C_dev = nullptr);
// C_dev (optional, device): only choices with loc < min(*C_dev, C) are kept; Y keeps its [E, C, M] layout
hipError_t launch_decode(const void* Y, int dtype, const int32_t* idx, const int32_t* loc, const float* gate_w,
                         int64_t T, int64_t M, int64_t E, int k, int64_t C, void* out, hipStream_t s,
                         const int64_t* C_dev = nullptr);
// One grouped GEMM: out[e] = epilogue(A[e] (rows_e x K) * B[e] (K x N) + bias[e]); A [E,C,K], B [E,K,N], out [E,C,N].
// act < 0 means no activation.  With `pre_out` [E,C,N] the values before the activation are written there as well.
hipError_t launch_grouped_gemm(const void* A, const void* B, const void* bias, int act, int dtype, const int32_t* counts,
                               int64_t E, int64_t C, int64_t K, int64_t N, void* out, hipStream_t s, void* pre_out = nullptr);

// Matrix-core GEMM with transposed operands (ffn_mfma.hip), bf16 only; see there for the argument meaning.
bool grouped_gemm_mfma_supports_backward(int64_t E, int64_t C, int64_t M, int64_t H);
bool grouped_gemm_mfma_supports_nt(int64_t rows, int64_t K, int64_t N);
hipError_t launch_grouped_gemm_mfma_nt(const void* A, const void* Bt, const int32_t* counts, int64_t E, int64_t C,
                                       int64_t K, int64_t N, void* out, const void* pre, int act, hipStream_t s);
hipError_t launch_grouped_gemm_mfma_tn(const void* At, const void* B, const int32_t* kfill, int64_t E, int64_t C, int64_t R,
                                       int64_t N, void* a_tail, void* b_tail, void* out, hipStream_t s,
                                       const int32_t* gather = nullptr, int64_t gather_rows = 0);

size_t gate_backward_workspace_bytes(int64_t T, int64_t M, int64_t E);
hipError_t launch_gate_backward(const void* x, const void* Wg, const float* logits, const int32_t* idx, const float* dgate_w,
                                int normalize, int dtype, int64_t T, int64_t M, int64_t E, int k, void* ws, void* dx,
                                int accumulate_dx, void* dWg, float* dbias, float* dlogits, hipStream_t s);

// Backward of the expert feed-forward layer (ffn_backward.hip): byte offsets of its workspace pieces
struct FfnBackwardWorkspace {
  size_t pre, dP, Wt, At, Bp, total;
  int64_t Cp;                                             // capacity padded to the GEMM's K step
};
FfnBackwardWorkspace ffn_backward_layout(int64_t E, int64_t C, int64_t M, int64_t H, int dtype);
hipError_t launch_expert_ffn_backward(const void* Z, const void* W1, const void* b1, const void* W2, const void* pre,
                                      const void* hidden, const void* dY, int act, int dtype, const int32_t* counts, int64_t E,
                                      int64_t C, int64_t M, int64_t H, void* ws, void* dZ, void* dW1, void* db1, void* dW2,
                                      void* db2, hipStream_t s, const int32_t* gather = nullptr, int64_t gather_rows = 0);
// With `gather` [E, C] (slot -> token) `Z` is the token matrix [gather_rows, M] itself (fused dispatch: the slabs of
// dispatched rows were never written); needs saved pre-activations and shapes the matrix-core backward takes.
bool ffn_backward_gather_supports(int64_t E, int64_t C, int64_t M, int64_t H, int64_t gather_rows, int dtype);

}  // namespace moe
