// C ABI of the MoE hot-path library: argument validation, workspace layout, stage sequencing.
#include <cmath>
#include <mutex>

#include "common.h"

namespace moe {
hipError_t launch_grouped_gemm_generic(const void* A, const void* B, const void* bias, int act, int dtype,
                                       const int32_t* counts, int64_t E, int64_t C, int64_t K, int64_t N, void* out,
                                       hipStream_t s);
hipError_t launch_grouped_gemm_mfma(const void* A, const void* B, const void* bias, int act, const int32_t* counts,
                                    int64_t E, int64_t C, int64_t K, int64_t N, void* out, hipStream_t s,
                                    const int32_t* gather = nullptr, int64_t gather_rows = 0, void* pre_out = nullptr);
bool grouped_gemm_mfma_supports(int64_t E, int64_t C, int64_t K, int64_t N, int64_t gather_rows = 0);

hipError_t launch_grouped_gemm(const void* A, const void* B, const void* bias, int act, int dtype, const int32_t* counts,
                               int64_t E, int64_t C, int64_t K, int64_t N, void* out, hipStream_t s, void* pre_out) {
  if (act < 0) pre_out = nullptr;                                   // nothing to tell apart
  if (dtype == MOE_BF16 && grouped_gemm_mfma_supports(E, C, K, N))
    return launch_grouped_gemm_mfma(A, B, bias, act, counts, E, C, K, N, out, s, nullptr, 0, pre_out);
  if (pre_out) {                                                    // the plain kernel has one output: run it twice
    const hipError_t err = launch_grouped_gemm_generic(A, B, bias, -1, dtype, counts, E, C, K, N, pre_out, s);
    if (err != hipSuccess) return err;
  }
  return launch_grouped_gemm_generic(A, B, bias, act, dtype, counts, E, C, K, N, out, s);
}

namespace {

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline bool dtype_ok(int d) { return d == MOE_F32 || d == MOE_BF16; }
inline bool act_ok(int a) { return a == MOE_ACT_RELU || a == MOE_ACT_GELU || a == MOE_ACT_SILU; }
inline size_t esize(int d) { return d == MOE_F32 ? 4 : 2; }
constexpr int64_t kMaxDim = (int64_t)1 << 30;

inline int gate_shape_status(int64_t T, int64_t E, int k) {
  if (T < 1 || E < 1 || k < 1 || k > E || T > kMaxDim) return MOE_INVALID_ARG;
  if (E > 512 || (int64_t)k * E > 16384) return MOE_UNSUPPORTED;
  return MOE_OK;
}

inline int row_shape_status(int64_t M) {
  if (M < 1 || M > kMaxDim) return MOE_INVALID_ARG;
  if (M % 8 != 0) return MOE_UNSUPPORTED;
  return MOE_OK;
}

// The gating function from the tokens: logits, then decisions and slots.  bf16 gates take the fast logits kernel and
// the top-k kernel's exact repair of near-ties; everything else the fp64 logits kernel.  Workspace: the arrival
// counters, then (fast path) the transposed gate weights, their norms and the per-token error bounds.
bool gate_uses_fast_logits(int dtype, int64_t T, int64_t M, int64_t E) { return gate_logits_fast_supports(dtype, T, M, E); }

size_t gate_route_workspace(int64_t T, int64_t M, int64_t E, int k, int dtype) {
  size_t n = align_up(moe_gate_workspace_bytes(T, E, k), 256);
  if (gate_uses_fast_logits(dtype, T, M, E)) n += gate_fast_workspace_bytes(T, M, E);
  return n;
}

template <typename F>
hipError_t run_gate(const void* x, const void* Wg, const float* bias, int dtype, int64_t T, int64_t M, int64_t E, int k, int64_t C,
                    int normalize, float* logits, int32_t* idx, float* gate_w, int32_t* loc, int32_t* counts, int32_t* slot_src,
                    void* ws, hipStream_t s, F&& after_logits) {
  int32_t* counters = (int32_t*)ws;
  if (gate_uses_fast_logits(dtype, T, M, E)) {
    const GateFastWorkspace f = gate_fast_layout((char*)ws + align_up(moe_gate_workspace_bytes(T, E, k), 256), T, M, E);
    hipError_t err = launch_gate_logits_fast(x, Wg, bias, T, M, E, logits, f, s);
    if (err != hipSuccess) return err;
    if (!after_logits()) return hipErrorUnknown;
    const GateRepair repair = {f.margin, x, f.Wt, bias, M, f.Mp};
    return launch_gate_topk(logits, T, E, k, C, normalize, idx, gate_w, loc, counts, slot_src, counters, s, nullptr, &repair);
  }
  hipError_t err = launch_gate_logits(x, Wg, bias, dtype, T, M, E, logits, s);
  if (err != hipSuccess) return err;
  if (!after_logits()) return hipErrorUnknown;
  return launch_gate_topk(logits, T, E, k, C, normalize, idx, gate_w, loc, counts, slot_src, counters, s);
}

struct LayerWorkspace {
  size_t logits, idx, loc, gate_w, counts, slot_src, gate_ws, Z, hidden, Y, total;
};

LayerWorkspace layer_layout(int64_t T, int64_t M, int64_t H, int64_t E, int k, int64_t C, int dtype) {
  LayerWorkspace w;
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t at = off; off = align_up(off + bytes, 256); return at; };
  w.logits = take((size_t)T * E * 4);
  w.idx = take((size_t)T * k * 4);
  w.loc = take((size_t)T * k * 4);
  w.gate_w = take((size_t)T * k * 4);
  w.counts = take((size_t)E * 4);
  w.slot_src = take((size_t)E * C * 4);
  w.gate_ws = take(gate_route_workspace(T, M, E, k, dtype));
  w.Z = take((size_t)E * C * M * esize(dtype));
  w.hidden = take((size_t)E * C * H * esize(dtype));
  w.Y = take((size_t)E * C * M * esize(dtype));
  w.total = off;
  return w;
}


// Scratch of the entry point that allocates nothing (moe_gate_topk_static): the gate's per-block arrival counters live
// in a file-scope device array instead of a caller's workspace.  Every GPU the library runs on holds its own copy at its
// own address; host code must use the address hipGetSymbolAddress returns for the current device, never the array's name.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up once per device), or nullptr on failure.
void* static_scratch_ptr() {
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    g_scratch_ptr[device] = p;
  }
  return g_scratch_ptr[device];
}

}  // namespace
}  // namespace moe

using namespace moe;

extern "C" {

const char* moe_status_string(int status) {
  switch (status) {
    case MOE_OK: return "ok";
    case MOE_INVALID_ARG: return "invalid argument";
    case MOE_UNSUPPORTED: return "unsupported shape, dtype or alignment";
    case MOE_WORKSPACE_TOO_SMALL: return "workspace too small";
    case MOE_HIP_ERROR: return "HIP runtime error";
    case MOE_SCRATCH_TOO_SMALL: return "problem too large for the library's static scratch buffer";
    default: return "unknown status";
  }
}

int64_t moe_capacity(int64_t T, int64_t E, int k, double f) {
  if (T < 1 || E < 1 || k < 1 || k > E || !(f > 0.0)) return -1;
  return (int64_t)std::ceil((double)k * f * (double)T / (double)E);
}

size_t moe_gate_workspace_bytes(int64_t T, int64_t E, int k) {
  if (gate_shape_status(T, E, k) != MOE_OK) return 0;
  return (size_t)k * (size_t)ceil_div(T, kGateTokensPerBlock) * (size_t)E * sizeof(int32_t);
}

size_t moe_layer_workspace_bytes(int64_t T, int64_t M, int64_t H, int64_t E, int k, int64_t C, int dtype) {
  if (gate_shape_status(T, E, k) != MOE_OK || row_shape_status(M) != MOE_OK || row_shape_status(H) != MOE_OK || C < 1 ||
      C > kMaxDim || !dtype_ok(dtype))
    return 0;
  return layer_layout(T, M, H, E, k, C, dtype).total;
}

int moe_gate_logits(const void* x, const void* Wg, const float* gate_bias, int dtype, int64_t T, int64_t M, int64_t E,
                    float* logits, void* stream) {
  if (!x || !Wg || !logits || !dtype_ok(dtype) || T < 1 || E < 1 || T > kMaxDim || E > kMaxDim) return MOE_INVALID_ARG;
  if (int st = row_shape_status(M)) return st;
  if (!aligned(x, 16) || !aligned(Wg, 2) || !aligned(logits, 4)) return MOE_UNSUPPORTED;
  return launch_gate_logits(x, Wg, gate_bias, dtype, T, M, E, logits, (hipStream_t)stream) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
}

size_t moe_cosine_gate_workspace_bytes(int64_t T, int64_t D, int64_t E) {
  if (T < 1 || T > kMaxDim || D < 1 || D > 4096 || E < 1 || E > 512) return 0;
  return align_up((size_t)T * D * 4, 256) + align_up((size_t)D * E * 8, 256) + align_up((size_t)E * 8, 256);
}

int moe_gate_logits_cosine(const void* x, const void* Wp, const float* Me, double tau, int dtype, int64_t T, int64_t M,
                           int64_t D, int64_t E, float* logits, void* ws, size_t ws_bytes, void* stream) {
  if (!x || !Wp || !Me || !logits || !ws || !dtype_ok(dtype) || !(tau > 0.0) || T < 1 || T > kMaxDim || E < 1 || D < 1)
    return MOE_INVALID_ARG;
  if (int st = row_shape_status(M)) return st;
  if (E > 512 || D > 4096 || !aligned(x, 16) || !aligned(ws, 256)) return MOE_UNSUPPORTED;
  if (ws_bytes < moe_cosine_gate_workspace_bytes(T, D, E)) return MOE_WORKSPACE_TOO_SMALL;
  char* base = (char*)ws;
  float* proj = (float*)base;
  double* MeT = (double*)(base + align_up((size_t)T * D * 4, 256));
  double* norm = (double*)((char*)MeT + align_up((size_t)D * E * 8, 256));
  const double tau_eff = tau < 0.01 ? 0.01 : tau;                   // the temperature is never below 0.01
  return launch_gate_logits_cosine(x, Wp, Me, tau_eff, dtype, T, M, D, E, logits, proj, MeT, norm, (hipStream_t)stream) == hipSuccess
             ? MOE_OK : MOE_HIP_ERROR;
}

int moe_gate_topk(const float* logits, int64_t T, int64_t E, int k, int64_t C, int normalize, int32_t* idx, float* gate_w,
                  int32_t* loc, int32_t* counts, int32_t* slot_src, void* ws, size_t ws_bytes, void* stream) {
  if (!logits || !idx || !gate_w || !loc || !counts || !ws || C < 1 || C > kMaxDim) return MOE_INVALID_ARG;
  if (int st = gate_shape_status(T, E, k)) return st;
  if (!aligned(ws, 16) || !aligned(logits, 16)) return MOE_UNSUPPORTED;
  if (ws_bytes < moe_gate_workspace_bytes(T, E, k)) return MOE_WORKSPACE_TOO_SMALL;
  return launch_gate_topk(const_cast<float*>(logits), T, E, k, C, normalize, idx, gate_w, loc, counts, slot_src, (int32_t*)ws,
                          (hipStream_t)stream) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
}

size_t moe_gate_route_workspace_bytes(int64_t T, int64_t M, int64_t E, int k, int dtype) {
  if (gate_shape_status(T, E, k) != MOE_OK || row_shape_status(M) != MOE_OK || !dtype_ok(dtype)) return 0;
  return gate_route_workspace(T, M, E, k, dtype);
}

int moe_gate_route(const void* x, const void* Wg, const float* gate_bias, int dtype, int64_t T, int64_t M, int64_t E, int k,
                   int64_t C, int normalize, float* logits, int32_t* idx, float* gate_w, int32_t* loc, int32_t* counts,
                   int32_t* slot_src, void* ws, size_t ws_bytes, void* stream) {
  if (!x || !Wg || !logits || !idx || !gate_w || !loc || !counts || !ws || !dtype_ok(dtype) || C < 1 || C > kMaxDim) return MOE_INVALID_ARG;
  if (int st = gate_shape_status(T, E, k)) return st;
  if (int st = row_shape_status(M)) return st;
  if (!aligned(x, 16) || !aligned(Wg, 2) || !aligned(ws, 256) || !aligned(logits, 16)) return MOE_UNSUPPORTED;
  if (ws_bytes < gate_route_workspace(T, M, E, k, dtype)) return MOE_WORKSPACE_TOO_SMALL;
  return run_gate(x, Wg, gate_bias, dtype, T, M, E, k, C, normalize, logits, idx, gate_w, loc, counts, slot_src, ws,
                  (hipStream_t)stream, [] { return true; }) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
}

size_t moe_gate_topk_static_max_bytes(void) { return kStaticScratchBytes; }

int moe_gate_topk_static(const float* logits, int64_t T, int64_t E, int k, int64_t C, int normalize, int32_t* idx, float* gate_w,
                         int32_t* loc, int32_t* counts, int32_t* slot_src, void* stream) {
  if (!logits || !idx || !gate_w || !loc || !counts || C < 1 || C > kMaxDim) return MOE_INVALID_ARG;
  if (int st = gate_shape_status(T, E, k)) return st;
  if (!aligned(logits, 16)) return MOE_UNSUPPORTED;
  if (moe_gate_workspace_bytes(T, E, k) > kStaticScratchBytes) return MOE_SCRATCH_TOO_SMALL;
  void* ws = static_scratch_ptr();
  if (!ws) return MOE_HIP_ERROR;
  // the kernels write every counter they later read, so the last call's contents need no clearing
  return launch_gate_topk(const_cast<float*>(logits), T, E, k, C, normalize, idx, gate_w, loc, counts, slot_src, (int32_t*)ws,
                          (hipStream_t)stream) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
}

int moe_dynamic_capacity(const int32_t* counts, int64_t T, int64_t E, int k, double capacity_setting, int64_t* C_out,
                         void* stream) {
  if (!counts || !C_out || !(capacity_setting <= 0.0)) return MOE_INVALID_ARG;    // positive settings: moe_capacity
  if (int st = gate_shape_status(T, E, k)) return st;
  int64_t bound = 0;
  if (capacity_setting < 0.0) {
    bound = moe_capacity(T, E, k, -capacity_setting);
    if (bound < 1 || bound > kMaxDim) return MOE_INVALID_ARG;
  }
  return launch_dynamic_capacity(counts, E, bound, C_out, (hipStream_t)stream) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
}

int moe_slot_sources(const int32_t* idx, const int32_t* loc, int64_t T, int64_t E, int k, int64_t C, int32_t* slot_src,
                     void* stream) {
  if (!idx || !loc || !slot_src || C < 1 || C > kMaxDim || E * C > kMaxDim) return MOE_INVALID_ARG;
  if (int st = gate_shape_status(T, E, k)) return st;
  return launch_slot_sources(idx, loc, T, E, k, C, slot_src, (hipStream_t)stream) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
}

size_t moe_gate_bpr_workspace_bytes(int64_t T, int64_t E, int k) {
  const size_t g = moe_gate_workspace_bytes(T, E, k);
  if (g == 0) return 0;
  return align_up(g, 256) + bpr_order_workspace_bytes(T);
}

int moe_gate_topk_bpr(const float* logits, int64_t T, int64_t E, int k, int64_t C, int normalize, int32_t* idx, float* gate_w,
                      int32_t* loc, int32_t* counts, int32_t* slot_src, void* ws, size_t ws_bytes, void* stream) {
  if (!logits || !idx || !gate_w || !loc || !counts || !ws || C < 1 || C > kMaxDim) return MOE_INVALID_ARG;
  if (int st = gate_shape_status(T, E, k)) return st;
  if (!aligned(ws, 256) || !aligned(logits, 16)) return MOE_UNSUPPORTED;
  if (ws_bytes < moe_gate_bpr_workspace_bytes(T, E, k)) return MOE_WORKSPACE_TOO_SMALL;
  hipStream_t s = (hipStream_t)stream;
  const int32_t* perm = nullptr;
  if (launch_bpr_order(logits, T, E, (char*)ws + align_up(moe_gate_workspace_bytes(T, E, k), 256), &perm, s) != hipSuccess) return MOE_HIP_ERROR;
  return launch_gate_topk(const_cast<float*>(logits), T, E, k, C, normalize, idx, gate_w, loc, counts, slot_src, (int32_t*)ws, s, perm) == hipSuccess
             ? MOE_OK : MOE_HIP_ERROR;
}

int moe_encode(const void* x, int dtype, const int32_t* idx, const int32_t* loc, const int32_t* slot_src, int64_t T,
               int64_t M, int64_t E, int k, int64_t C, void* Z, void* stream) {
  if (!x || !idx || !loc || !Z || !dtype_ok(dtype) || T < 1 || E < 1 || k < 1 || k > E || C < 1 || T > kMaxDim ||
      E > kMaxDim || C > kMaxDim)
    return MOE_INVALID_ARG;
  if (int st = row_shape_status(M)) return st;
  if (!aligned(x, 16) || !aligned(Z, 16)) return MOE_UNSUPPORTED;
  return launch_encode(x, dtype, idx, loc, slot_src, T, M, E, k, C, Z, (hipStream_t)stream) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
}

int moe_expert_ffn(const void* Z, const void* W1, const void* b1, const void* W2, const void* b2, int act, int dtype,
                   const int32_t* counts, int64_t E, int64_t C, int64_t M, int64_t H, void* hidden, void* Y, void* stream) {
  if (!Z || !W1 || !W2 || !hidden || !Y || !dtype_ok(dtype) || !act_ok(act) || E < 1 || C < 1 || E > 65535 || C > kMaxDim)
    return MOE_INVALID_ARG;
  if (int st = row_shape_status(M)) return st;
  if (int st = row_shape_status(H)) return st;
  if (!aligned(Z, 16) || !aligned(W1, 16) || !aligned(W2, 16) || !aligned(hidden, 16) || !aligned(Y, 16)) return MOE_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  if (launch_grouped_gemm(Z, W1, b1, act, dtype, counts, E, C, M, H, hidden, s) != hipSuccess) return MOE_HIP_ERROR;
  if (launch_grouped_gemm(hidden, W2, b2, -1, dtype, counts, E, C, H, M, Y, s) != hipSuccess) return MOE_HIP_ERROR;
  return MOE_OK;
}

int moe_expert_ffn_train(const void* Z, const void* W1, const void* b1, const void* W2, const void* b2, int act, int dtype,
                         const int32_t* counts, int64_t E, int64_t C, int64_t M, int64_t H, void* pre, void* hidden, void* Y,
                         void* stream) {
  if (!Z || !W1 || !W2 || !pre || !hidden || !Y || !dtype_ok(dtype) || !act_ok(act) || E < 1 || C < 1 || E > 65535 || C > kMaxDim)
    return MOE_INVALID_ARG;
  if (int st = row_shape_status(M)) return st;
  if (int st = row_shape_status(H)) return st;
  if (!aligned(Z, 16) || !aligned(W1, 16) || !aligned(W2, 16) || !aligned(pre, 16) || !aligned(hidden, 16) || !aligned(Y, 16))
    return MOE_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  if (launch_grouped_gemm(Z, W1, b1, act, dtype, counts, E, C, M, H, hidden, s, pre) != hipSuccess) return MOE_HIP_ERROR;
  if (launch_grouped_gemm(hidden, W2, b2, -1, dtype, counts, E, C, H, M, Y, s) != hipSuccess) return MOE_HIP_ERROR;
  return MOE_OK;
}

int moe_expert_ffn_gather(const void* x, const int32_t* slot_src, int64_t T, const void* W1, const void* b1, const void* W2,
                          const void* b2, int act, int dtype, const int32_t* counts, int64_t E, int64_t C, int64_t M, int64_t H,
                          void* hidden, void* Y, void* stream) {
  if (!x || !slot_src || !W1 || !W2 || !hidden || !Y || !dtype_ok(dtype) || !act_ok(act) || T < 1 || T > kMaxDim || E < 1 ||
      C < 1 || E > 65535 || C > kMaxDim)
    return MOE_INVALID_ARG;
  if (int st = row_shape_status(M)) return st;
  if (int st = row_shape_status(H)) return st;
  if (!aligned(x, 16) || !aligned(W1, 16) || !aligned(W2, 16) || !aligned(hidden, 16) || !aligned(Y, 16)) return MOE_UNSUPPORTED;
  if (dtype != MOE_BF16 || !grouped_gemm_mfma_supports(E, C, M, H, T)) return MOE_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  if (launch_grouped_gemm_mfma(x, W1, b1, act, counts, E, C, M, H, hidden, s, slot_src, T) != hipSuccess) return MOE_HIP_ERROR;
  if (launch_grouped_gemm(hidden, W2, b2, -1, dtype, counts, E, C, H, M, Y, s) != hipSuccess) return MOE_HIP_ERROR;
  return MOE_OK;
}

int moe_decode(const void* Y, int dtype, const int32_t* idx, const int32_t* loc, const float* gate_w, int64_t T, int64_t M,
               int64_t E, int k, int64_t C, void* out, void* stream) {
  if (!Y || !idx || !loc || !gate_w || !out || !dtype_ok(dtype) || T < 1 || E < 1 || k < 1 || k > E || C < 1 ||
      T > kMaxDim || E > kMaxDim || C > kMaxDim)
    return MOE_INVALID_ARG;
  if (int st = row_shape_status(M)) return st;
  if (!aligned(Y, 16) || !aligned(out, 16)) return MOE_UNSUPPORTED;
  return launch_decode(Y, dtype, idx, loc, gate_w, T, M, E, k, C, out, (hipStream_t)stream) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
}

size_t moe_gate_backward_workspace_bytes(int64_t T, int64_t M, int64_t E, int k) {
  if (gate_shape_status(T, E, k) != MOE_OK || row_shape_status(M) != MOE_OK) return 0;
  return gate_backward_workspace_bytes(T, M, E);
}

int moe_gate_backward(const void* x, const void* Wg, const float* logits, const int32_t* idx, const float* dgate_w, int normalize,
                      int dtype, int64_t T, int64_t M, int64_t E, int k, void* ws, size_t ws_bytes, void* dx, int accumulate_dx,
                      void* dWg, float* dbias, float* dlogits, void* stream) {
  if (!logits || !idx || !dgate_w || !ws || !dtype_ok(dtype) || (!dx && !dWg && !dbias && !dlogits) || (dx && !Wg) ||
      (dWg && !x))
    return MOE_INVALID_ARG;
  if (int st = gate_shape_status(T, E, k)) return st;
  if (int st = row_shape_status(M)) return st;
  if (!aligned(ws, 256) || (dx && !aligned(dx, 16)) || (dWg && !aligned(x, 16))) return MOE_UNSUPPORTED;   // rows go in 16-byte pieces
  if (ws_bytes < gate_backward_workspace_bytes(T, M, E)) return MOE_WORKSPACE_TOO_SMALL;
  return launch_gate_backward(x, Wg, logits, idx, dgate_w, normalize, dtype, T, M, E, k, ws, dx, accumulate_dx, dWg, dbias, dlogits,
                              (hipStream_t)stream) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
}

size_t moe_ffn_backward_workspace_bytes(int64_t E, int64_t C, int64_t M, int64_t H, int dtype) {
  if (!dtype_ok(dtype) || E < 1 || C < 1 || E > 65535 || C > kMaxDim || row_shape_status(M) || row_shape_status(H)) return 0;
  return ffn_backward_layout(E, C, M, H, dtype).total;
}

int moe_expert_ffn_backward(const void* Z, const void* W1, const void* b1, const void* W2, const void* pre, const void* hidden,
                            const void* dY, int act, int dtype, const int32_t* counts, int64_t E, int64_t C, int64_t M, int64_t H,
                            void* ws, size_t ws_bytes, void* dZ, void* dW1, void* db1, void* dW2, void* db2, void* stream) {
  if (!Z || !W1 || !W2 || !hidden || !dY || !ws || !dtype_ok(dtype) || !act_ok(act) || E < 1 || C < 1 || E > 65535 ||
      C > kMaxDim || (!dZ && !dW1 && !db1 && !dW2 && !db2))
    return MOE_INVALID_ARG;
  if (int st = row_shape_status(M)) return st;
  if (int st = row_shape_status(H)) return st;
  for (const void* p : {Z, W1, W2, pre, hidden, dY, (const void*)ws, (const void*)dZ, (const void*)dW1, (const void*)dW2})
    if (p && !aligned(p, 16)) return MOE_UNSUPPORTED;
  if (ws_bytes < ffn_backward_layout(E, C, M, H, dtype).total) return MOE_WORKSPACE_TOO_SMALL;
  return launch_expert_ffn_backward(Z, W1, b1, W2, pre, hidden, dY, act, dtype, counts, E, C, M, H, ws, dZ, dW1, db1, dW2, db2,
                                    (hipStream_t)stream) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
}

int moe_encode_backward(const void* dZ, int dtype, const int32_t* idx, const int32_t* loc, int64_t T, int64_t M, int64_t E,
                        int k, int64_t C, void* dx, void* stream) {
  if (!dZ || !idx || !loc || !dx || !dtype_ok(dtype) || T < 1 || E < 1 || k < 1 || k > E || C < 1 || T > kMaxDim ||
      E > kMaxDim || C > kMaxDim)
    return MOE_INVALID_ARG;
  if (int st = row_shape_status(M)) return st;
  if (!aligned(dZ, 16) || !aligned(dx, 16)) return MOE_UNSUPPORTED;
  // the sum of a token's kept slot rows: decode with unit weights
  return launch_decode(dZ, dtype, idx, loc, nullptr, T, M, E, k, C, dx, (hipStream_t)stream) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
}

int moe_decode_backward(const void* d_out, const void* Y, int dtype, const int32_t* idx, const int32_t* loc,
                        const float* gate_w, const int32_t* slot_src, int64_t T, int64_t M, int64_t E, int k, int64_t C,
                        void* dY, float* dgate_w, void* stream) {
  if (!d_out || !idx || !loc || !dtype_ok(dtype) || T < 1 || E < 1 || k < 1 || k > E || C < 1 || T > kMaxDim ||
      E > kMaxDim || C > kMaxDim || (!dY && !dgate_w) || (dY && (!gate_w || !slot_src)) || (dgate_w && !Y))
    return MOE_INVALID_ARG;
  if (int st = row_shape_status(M)) return st;
  if (!aligned(d_out, 16) || (dY && !aligned(dY, 16)) || (Y && !aligned(Y, 16))) return MOE_UNSUPPORTED;
  return launch_decode_backward(d_out, Y, dtype, idx, loc, gate_w, slot_src, T, M, E, k, C, dY, dgate_w,
                                (hipStream_t)stream) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
}

}  // extern "C"

namespace {
// State a training step keeps between moe_layer_forward_train and moe_layer_backward, followed by the backward's scratch.
struct TrainState {
  size_t logits, idx, loc, gate_w, counts, slot_src, gate_ws, Z, pre, hidden, Y;     // written by the forward
  size_t dgate_w, dY, dZ, ffn_ws, gate_bwd_ws, total;                                // scratch of the backward
  bool fused;                                                                        // no Z: rows are read through slot_src
};

// The training step reads the experts' input rows straight from the token matrix through the slot -> token map (first
// GEMM of the forward, first layer's weight gradient of the backward) wherever the matrix-core kernels take the shape.
bool train_fuses_dispatch(int64_t T, int64_t M, int64_t H, int64_t E, int64_t C, int dtype) {
  return dtype == MOE_BF16 && grouped_gemm_mfma_supports(E, C, M, H, T) && ffn_backward_gather_supports(E, C, M, H, T, dtype);
}

TrainState train_layout(int64_t T, int64_t M, int64_t H, int64_t E, int k, int64_t C, int dtype) {
  TrainState w;
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t at = off; off = align_up(off + bytes, 256); return at; };
  const size_t es = esize(dtype);
  w.logits = take((size_t)T * E * 4);
  w.idx = take((size_t)T * k * 4);
  w.loc = take((size_t)T * k * 4);
  w.gate_w = take((size_t)T * k * 4);
  w.counts = take((size_t)E * 4);
  w.slot_src = take((size_t)E * C * 4);
  w.gate_ws = take(gate_route_workspace(T, M, E, k, dtype));
  w.fused = train_fuses_dispatch(T, M, H, E, C, dtype);
  w.Z = take(w.fused ? 0 : (size_t)E * C * M * es);                 // fused dispatch: the slabs of dispatched rows never exist
  w.pre = take((size_t)E * C * H * es);
  w.hidden = take((size_t)E * C * H * es);
  w.Y = take((size_t)E * C * M * es);
  w.dgate_w = take((size_t)T * k * 4);
  w.dY = take((size_t)E * C * M * es);
  w.dZ = take((size_t)E * C * M * es);
  w.ffn_ws = take(ffn_backward_layout(E, C, M, H, dtype).total);
  w.gate_bwd_ws = take(gate_backward_workspace_bytes(T, M, E));
  w.total = off;
  return w;
}

int layer_forward(const void* x, const void* Wg, const float* gate_bias, const void* W1, const void* b1, const void* W2,
                  const void* b2, int64_t T, int64_t M, int64_t H, int64_t E, int k, double f, int normalize, int act, int dtype,
                  void* out, int32_t* idx, int32_t* loc, float* gate_w, int32_t* counts, float* logits, void* ws,
                  size_t ws_bytes, void* stream, void* const* stage_events, bool fuse_dispatch) {
  if (!x || !Wg || !W1 || !W2 || !out || !ws || !dtype_ok(dtype) || !act_ok(act) || !(f > 0.0)) return MOE_INVALID_ARG;
  if (int st = gate_shape_status(T, E, k)) return st;
  if (int st = row_shape_status(M)) return st;
  if (int st = row_shape_status(H)) return st;
  const int64_t C = moe_capacity(T, E, k, f);
  if (C < 1 || C > kMaxDim) return MOE_INVALID_ARG;
  if (!aligned(x, 16) || !aligned(W1, 16) || !aligned(W2, 16) || !aligned(out, 16) || !aligned(ws, 256)) return MOE_UNSUPPORTED;
  const LayerWorkspace w = layer_layout(T, M, H, E, k, C, dtype);
  if (ws_bytes < w.total) return MOE_WORKSPACE_TOO_SMALL;
  if (stage_events)
    for (int i = 0; i < MOE_NUM_STAGE_EVENTS; ++i)
      if (!stage_events[i]) return MOE_INVALID_ARG;

  char* base = (char*)ws;
  float* d_logits = logits ? logits : (float*)(base + w.logits);
  int32_t* d_idx = idx ? idx : (int32_t*)(base + w.idx);
  int32_t* d_loc = loc ? loc : (int32_t*)(base + w.loc);
  float* d_gw = gate_w ? gate_w : (float*)(base + w.gate_w);
  int32_t* d_counts = counts ? counts : (int32_t*)(base + w.counts);
  int32_t* d_src = (int32_t*)(base + w.slot_src);
  void* d_gws = base + w.gate_ws;
  void* d_Z = base + w.Z;
  void* d_hidden = base + w.hidden;
  void* d_Y = base + w.Y;
  hipStream_t s = (hipStream_t)stream;
  int stage = 0;
  auto mark = [&]() -> bool { return !stage_events || hipEventRecord((hipEvent_t)stage_events[stage++], s) == hipSuccess; };

  if (!mark()) return MOE_HIP_ERROR;
  if (run_gate(x, Wg, gate_bias, dtype, T, M, E, k, C, normalize, d_logits, d_idx, d_gw, d_loc, d_counts, d_src, d_gws, s, mark) != hipSuccess ||
      !mark())
    return MOE_HIP_ERROR;
  if (fuse_dispatch && dtype == MOE_BF16 && grouped_gemm_mfma_supports(E, C, M, H, T)) {
    // the first expert GEMM gathers its rows from x through slot_src: the dispatch buffer is never materialised
    if (!mark()) return MOE_HIP_ERROR;
    if (launch_grouped_gemm_mfma(x, W1, b1, act, d_counts, E, C, M, H, d_hidden, s, d_src, T) != hipSuccess || !mark())
      return MOE_HIP_ERROR;
  } else {
    // the dispatch buffer is internal here and the expert GEMM skips rows past an expert's fill: no zero rows needed
    if (launch_encode(x, dtype, d_idx, d_loc, d_src, T, M, E, k, C, d_Z, s, false) != hipSuccess || !mark()) return MOE_HIP_ERROR;
    if (launch_grouped_gemm(d_Z, W1, b1, act, dtype, d_counts, E, C, M, H, d_hidden, s) != hipSuccess || !mark()) return MOE_HIP_ERROR;
  }
  if (launch_grouped_gemm(d_hidden, W2, b2, -1, dtype, d_counts, E, C, H, M, d_Y, s) != hipSuccess || !mark()) return MOE_HIP_ERROR;
  if (launch_decode(d_Y, dtype, d_idx, d_loc, d_gw, T, M, E, k, C, out, s) != hipSuccess || !mark()) return MOE_HIP_ERROR;
  return MOE_OK;
}
}  // namespace

extern "C" {

int moe_layer_forward(const void* x, const void* Wg, const float* gate_bias, const void* W1, const void* b1, const void* W2,
                      const void* b2, int64_t T, int64_t M, int64_t H, int64_t E, int k, double f, int normalize, int act,
                      int dtype, void* out, int32_t* idx, int32_t* loc, float* gate_w, int32_t* counts, float* logits,
                      void* ws, size_t ws_bytes, void* stream, void* const* stage_events) {
  return layer_forward(x, Wg, gate_bias, W1, b1, W2, b2, T, M, H, E, k, f, normalize, act, dtype, out, idx, loc, gate_w, counts,
                       logits, ws, ws_bytes, stream, stage_events, false);
}

int moe_layer_forward_fused(const void* x, const void* Wg, const float* gate_bias, const void* W1, const void* b1,
                            const void* W2, const void* b2, int64_t T, int64_t M, int64_t H, int64_t E, int k, double f,
                            int normalize, int act, int dtype, void* out, int32_t* idx, int32_t* loc, float* gate_w,
                            int32_t* counts, float* logits, void* ws, size_t ws_bytes, void* stream,
                            void* const* stage_events) {
  return layer_forward(x, Wg, gate_bias, W1, b1, W2, b2, T, M, H, E, k, f, normalize, act, dtype, out, idx, loc, gate_w, counts,
                       logits, ws, ws_bytes, stream, stage_events, true);
}

namespace {
struct DynamicWorkspace {
  size_t logits, idx, loc, gate_w, counts, fills, C_dev, slot_src, gate_ws, cosine_ws, Z, hidden, Y, total;
};

DynamicWorkspace dynamic_layout(int64_t T, int64_t M, int64_t H, int64_t E, int k, int64_t C_max, int dtype, int router, int64_t D,
                                int bpr) {
  DynamicWorkspace w;
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t at = off; off = align_up(off + bytes, 256); return at; };
  w.logits = take((size_t)T * E * 4);
  w.idx = take((size_t)T * k * 4);
  w.loc = take((size_t)T * k * 4);
  w.gate_w = take((size_t)T * k * 4);
  w.counts = take((size_t)E * 4);
  w.fills = take((size_t)E * 4);
  w.C_dev = take(2 * sizeof(int64_t));
  w.slot_src = take((size_t)E * C_max * 4);
  w.gate_ws = take(bpr ? moe_gate_bpr_workspace_bytes(T, E, k) : gate_route_workspace(T, M, E, k, dtype));
  w.cosine_ws = take(router == MOE_ROUTER_COSINE ? moe_cosine_gate_workspace_bytes(T, D, E) : 0);
  w.Z = take((size_t)E * C_max * M * esize(dtype));
  w.hidden = take((size_t)E * C_max * H * esize(dtype));
  w.Y = take((size_t)E * C_max * M * esize(dtype));
  w.total = off;
  return w;
}

int dynamic_shape_status(int64_t T, int64_t M, int64_t H, int64_t E, int k, int64_t C_max, int dtype, int router, int64_t D, int bpr) {
  if (!dtype_ok(dtype) || C_max < 1 || C_max > kMaxDim || (router != MOE_ROUTER_LINEAR && router != MOE_ROUTER_COSINE))
    return MOE_INVALID_ARG;
  if (int st = gate_shape_status(T, E, k)) return st;
  if (int st = row_shape_status(M)) return st;
  if (int st = row_shape_status(H)) return st;
  if (E * C_max > kMaxDim) return MOE_INVALID_ARG;
  if (router == MOE_ROUTER_COSINE && (D < 1 || moe_cosine_gate_workspace_bytes(T, D, E) == 0)) return D < 1 ? MOE_INVALID_ARG : MOE_UNSUPPORTED;
  if (bpr && moe_gate_bpr_workspace_bytes(T, E, k) == 0) return MOE_UNSUPPORTED;
  return MOE_OK;
}
}  // namespace

size_t moe_layer_dynamic_workspace_bytes(int64_t T, int64_t M, int64_t H, int64_t E, int k, int64_t C_max, int dtype, int router,
                                         int64_t D, int bpr) {
  if (dynamic_shape_status(T, M, H, E, k, C_max, dtype, router, D, bpr) != MOE_OK) return 0;
  return dynamic_layout(T, M, H, E, k, C_max, dtype, router, D, bpr).total;
}

int moe_layer_forward_dynamic(const void* x, const void* Wg, const float* gate_bias, const void* W1, const void* b1, const void* W2,
                              const void* b2, int64_t T, int64_t M, int64_t H, int64_t E, int k, double capacity_setting,
                              int64_t C_max, int normalize, int act, int dtype, int router, const float* Me, int64_t D, double tau,
                              int bpr, void* out, int32_t* idx, int32_t* loc, float* gate_w, int32_t* counts, float* logits,
                              int64_t* C_out, void* ws, size_t ws_bytes, void* stream) {
  if (!x || !Wg || !W1 || !W2 || !out || !ws || !act_ok(act) || capacity_setting != capacity_setting) return MOE_INVALID_ARG;
  if (int st = dynamic_shape_status(T, M, H, E, k, C_max, dtype, router, D, bpr)) return st;
  if (router == MOE_ROUTER_COSINE && (!Me || gate_bias || !(tau > 0.0))) return MOE_INVALID_ARG;
  if (!aligned(x, 16) || !aligned(W1, 16) || !aligned(W2, 16) || !aligned(out, 16) || !aligned(ws, 256) || (C_out && !aligned(C_out, 8)))
    return MOE_UNSUPPORTED;
  // what the host knows of the capacity: a fixed one (positive setting) or an upper bound (the caller's C_max and, for a
  // negative setting, what Eq. 1 gives for the factor -setting)
  int64_t fixed = 0, bound = C_max;
  if (capacity_setting > 0.0) {
    fixed = moe_capacity(T, E, k, capacity_setting);
    if (fixed < 1 || fixed > C_max) return MOE_INVALID_ARG;            // the buffers the caller sized cannot hold it
  } else if (capacity_setting < 0.0) {
    const int64_t b = moe_capacity(T, E, k, -capacity_setting);
    if (b < 1) return MOE_INVALID_ARG;
    bound = b < C_max ? b : C_max;
  }
  const DynamicWorkspace w = dynamic_layout(T, M, H, E, k, C_max, dtype, router, D, bpr);
  if (ws_bytes < w.total) return MOE_WORKSPACE_TOO_SMALL;
  char* base = (char*)ws;
  float* d_logits = logits ? logits : (float*)(base + w.logits);
  int32_t* d_idx = idx ? idx : (int32_t*)(base + w.idx);
  int32_t* d_loc = loc ? loc : (int32_t*)(base + w.loc);
  float* d_gw = gate_w ? gate_w : (float*)(base + w.gate_w);
  int32_t* d_counts = counts ? counts : (int32_t*)(base + w.counts);
  int32_t* d_fills = (int32_t*)(base + w.fills);
  int64_t* d_C = C_out ? C_out : (int64_t*)(base + w.C_dev);
  int32_t* d_src = (int32_t*)(base + w.slot_src);
  hipStream_t s = (hipStream_t)stream;

  // arrivals do not depend on the capacity: count them first (no slot sources yet), then choose the capacity on the device.
  // The plain linear router takes the fast logits with exact repair of near-ties; the cosine router and batch prioritized
  // routing (whose token order is itself decided on the logits) take logits that are exactly rounded throughout.
  int st;
  if (router == MOE_ROUTER_LINEAR && !bpr) {
    st = run_gate(x, Wg, gate_bias, dtype, T, M, E, k, C_max, normalize, d_logits, d_idx, d_gw, d_loc, d_counts, nullptr,
                  base + w.gate_ws, s, [] { return true; }) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
  } else {
    if (router == MOE_ROUTER_COSINE)
      st = moe_gate_logits_cosine(x, Wg, Me, tau, dtype, T, M, D, E, d_logits, base + w.cosine_ws, moe_cosine_gate_workspace_bytes(T, D, E), stream);
    else
      st = launch_gate_logits(x, Wg, gate_bias, dtype, T, M, E, d_logits, s) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
    if (st != MOE_OK) return st;
    if (bpr)
      st = moe_gate_topk_bpr(d_logits, T, E, k, C_max, normalize, d_idx, d_gw, d_loc, d_counts, nullptr, base + w.gate_ws,
                             moe_gate_bpr_workspace_bytes(T, E, k), stream);
    else
      st = launch_gate_topk(d_logits, T, E, k, C_max, normalize, d_idx, d_gw, d_loc, d_counts, nullptr, (int32_t*)(base + w.gate_ws), s) == hipSuccess
               ? MOE_OK : MOE_HIP_ERROR;
  }
  if (st != MOE_OK) return st;
  if (launch_dynamic_capacity(d_counts, E, bound, d_C, s, fixed, d_fills) != hipSuccess) return MOE_HIP_ERROR;
  // every buffer keeps the layout the caller's bound gives ([E, C_max, ...]); the chosen capacity only narrows which
  // choices are kept (loc < C, read from device memory) and how many rows of a slab are filled
  if (launch_slot_sources(d_idx, d_loc, T, E, k, C_max, d_src, s, d_C) != hipSuccess) return MOE_HIP_ERROR;
  if (launch_encode(x, dtype, d_idx, d_loc, d_src, T, M, E, k, C_max, base + w.Z, s, false, d_C) != hipSuccess) return MOE_HIP_ERROR;
  if (launch_grouped_gemm(base + w.Z, W1, b1, act, dtype, d_fills, E, C_max, M, H, base + w.hidden, s) != hipSuccess) return MOE_HIP_ERROR;
  if (launch_grouped_gemm(base + w.hidden, W2, b2, -1, dtype, d_fills, E, C_max, H, M, base + w.Y, s) != hipSuccess) return MOE_HIP_ERROR;
  if (launch_decode(base + w.Y, dtype, d_idx, d_loc, d_gw, T, M, E, k, C_max, out, s, d_C) != hipSuccess) return MOE_HIP_ERROR;
  return MOE_OK;
}

size_t moe_layer_train_state_bytes(int64_t T, int64_t M, int64_t H, int64_t E, int k, int64_t C, int dtype) {
  if (!dtype_ok(dtype) || gate_shape_status(T, E, k) || row_shape_status(M) || row_shape_status(H) || C < 1 || C > kMaxDim)
    return 0;
  return train_layout(T, M, H, E, k, C, dtype).total;
}

int moe_layer_forward_train(const void* x, const void* Wg, const float* gate_bias, const void* W1, const void* b1,
                            const void* W2, const void* b2, int64_t T, int64_t M, int64_t H, int64_t E, int k, double f,
                            int normalize, int act, int dtype, void* out, void* state, size_t state_bytes, void* stream) {
  if (!x || !Wg || !W1 || !W2 || !out || !state || !dtype_ok(dtype) || !act_ok(act) || !(f > 0.0)) return MOE_INVALID_ARG;
  if (int st = gate_shape_status(T, E, k)) return st;
  if (int st = row_shape_status(M)) return st;
  if (int st = row_shape_status(H)) return st;
  const int64_t C = moe_capacity(T, E, k, f);
  if (C < 1 || C > kMaxDim) return MOE_INVALID_ARG;
  if (!aligned(x, 16) || !aligned(W1, 16) || !aligned(W2, 16) || !aligned(out, 16) || !aligned(state, 256)) return MOE_UNSUPPORTED;
  const TrainState w = train_layout(T, M, H, E, k, C, dtype);
  if (state_bytes < w.total) return MOE_WORKSPACE_TOO_SMALL;
  char* base = (char*)state;
  float* logits = (float*)(base + w.logits);
  int32_t* idx = (int32_t*)(base + w.idx);
  int32_t* loc = (int32_t*)(base + w.loc);
  float* gw = (float*)(base + w.gate_w);
  int32_t* counts = (int32_t*)(base + w.counts);
  int32_t* src = (int32_t*)(base + w.slot_src);
  hipStream_t s = (hipStream_t)stream;
  if (run_gate(x, Wg, gate_bias, dtype, T, M, E, k, C, normalize, logits, idx, gw, loc, counts, src, base + w.gate_ws, s,
               [] { return true; }) != hipSuccess)
    return MOE_HIP_ERROR;
  if (w.fused) {
    if (launch_grouped_gemm_mfma(x, W1, b1, act, counts, E, C, M, H, base + w.hidden, s, src, T, base + w.pre) != hipSuccess)
      return MOE_HIP_ERROR;
  } else {
    // the slabs are internal and every later stage stops at an expert's fill: no zero rows needed
    if (launch_encode(x, dtype, idx, loc, src, T, M, E, k, C, base + w.Z, s, false) != hipSuccess) return MOE_HIP_ERROR;
    if (launch_grouped_gemm(base + w.Z, W1, b1, act, dtype, counts, E, C, M, H, base + w.hidden, s, base + w.pre) != hipSuccess)
      return MOE_HIP_ERROR;
  }
  if (launch_grouped_gemm(base + w.hidden, W2, b2, -1, dtype, counts, E, C, H, M, base + w.Y, s) != hipSuccess) return MOE_HIP_ERROR;
  if (launch_decode(base + w.Y, dtype, idx, loc, gw, T, M, E, k, C, out, s) != hipSuccess) return MOE_HIP_ERROR;
  return MOE_OK;
}

int moe_layer_backward(const void* x, const void* Wg, const void* W1, const void* b1, const void* W2, int64_t T, int64_t M,
                       int64_t H, int64_t E, int k, double f, int normalize, int act, int dtype, const void* d_out, void* state,
                       size_t state_bytes, void* dx, void* dWg, float* dgate_bias, void* dW1, void* db1, void* dW2, void* db2,
                       void* stream) {
  if (!x || !Wg || !W1 || !W2 || !d_out || !state || !dx || !dtype_ok(dtype) || !act_ok(act) || !(f > 0.0)) return MOE_INVALID_ARG;
  if (int st = gate_shape_status(T, E, k)) return st;
  if (int st = row_shape_status(M)) return st;
  if (int st = row_shape_status(H)) return st;
  const int64_t C = moe_capacity(T, E, k, f);
  if (C < 1 || C > kMaxDim) return MOE_INVALID_ARG;
  for (const void* p : {x, W1, W2, d_out, (const void*)dx, (const void*)dW1, (const void*)dW2})
    if (p && !aligned(p, 16)) return MOE_UNSUPPORTED;
  if (!aligned(state, 256)) return MOE_UNSUPPORTED;
  const TrainState w = train_layout(T, M, H, E, k, C, dtype);
  if (state_bytes < w.total) return MOE_WORKSPACE_TOO_SMALL;
  char* base = (char*)state;
  const float* logits = (const float*)(base + w.logits);
  const int32_t* idx = (const int32_t*)(base + w.idx);
  const int32_t* loc = (const int32_t*)(base + w.loc);
  const float* gw = (const float*)(base + w.gate_w);
  const int32_t* counts = (const int32_t*)(base + w.counts);
  const int32_t* src = (const int32_t*)(base + w.slot_src);
  float* dgw = (float*)(base + w.dgate_w);
  hipStream_t s = (hipStream_t)stream;
  // decode: dY over the filled slots (the expert backward stops at an expert's fill) and the gate weights' gradient
  if (launch_decode_backward(d_out, base + w.Y, dtype, idx, loc, gw, src, T, M, E, k, C, base + w.dY, dgw, s, false) != hipSuccess)
    return MOE_HIP_ERROR;
  // experts: dZ over the filled slots, parameter gradients
  if (launch_expert_ffn_backward(w.fused ? x : base + w.Z, W1, b1, W2, base + w.pre, base + w.hidden, base + w.dY, act, dtype,
                                 counts, E, C, M, H, base + w.ffn_ws, base + w.dZ, dW1, db1, dW2, db2, s, w.fused ? src : nullptr,
                                 w.fused ? T : 0) != hipSuccess)
    return MOE_HIP_ERROR;
  // encode: dx = sum of a token's kept slot rows of dZ (decode with unit weights)
  if (launch_decode(base + w.dZ, dtype, idx, loc, nullptr, T, M, E, k, C, dx, s) != hipSuccess) return MOE_HIP_ERROR;
  // gate: dx += dlogits Wg^T, dWg, dbias
  if (launch_gate_backward(x, Wg, logits, idx, dgw, normalize, dtype, T, M, E, k, base + w.gate_bwd_ws, dx, 1, dWg, dgate_bias,
                           nullptr, s) != hipSuccess)
    return MOE_HIP_ERROR;
  return MOE_OK;
}

int moe_event_create(void** event) {
  if (!event) return MOE_INVALID_ARG;
  hipEvent_t ev;
  if (hipEventCreate(&ev) != hipSuccess) return MOE_HIP_ERROR;
  *event = (void*)ev;
  return MOE_OK;
}
int moe_event_destroy(void* event) {
  if (!event) return MOE_INVALID_ARG;
  return hipEventDestroy((hipEvent_t)event) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
}
int moe_event_record(void* event, void* stream) {
  if (!event) return MOE_INVALID_ARG;
  return hipEventRecord((hipEvent_t)event, (hipStream_t)stream) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
}
int moe_event_synchronize(void* event) {
  if (!event) return MOE_INVALID_ARG;
  return hipEventSynchronize((hipEvent_t)event) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
}
int moe_event_elapsed_ms(void* start, void* stop, float* ms) {
  if (!start || !stop || !ms) return MOE_INVALID_ARG;
  return hipEventElapsedTime(ms, (hipEvent_t)start, (hipEvent_t)stop) == hipSuccess ? MOE_OK : MOE_HIP_ERROR;
}

}  // extern "C"
