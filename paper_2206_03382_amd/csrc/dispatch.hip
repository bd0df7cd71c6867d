// Fast encode / decode (arXiv 2206.03382 Sec. 4.2 and Appendix B): the sparse O(T*k*M) form of the one-hot-mask
// dispatch and combine contractions.  Pure data movement, bound by HBM: every lane moves 16-byte pieces, a wave
// moves whole rows, rows of one wave are adjacent in the destination so stores are fully coalesced.
#include "common.h"

namespace moe {

// --- encode, gather form: one pass over the [E*C] slots; slot_src says which token row (or none) lands there -----
// FILL: unfilled slots are written as zero rows (the operator's contract); without it they are left untouched, which is
// all the layer needs for its internal buffer (the expert GEMM never uses rows past an expert's fill).
template <int ROWS, bool FILL>
__global__ __launch_bounds__(256) void encode_gather_kernel(const uint4* __restrict__ x, const int32_t* __restrict__ slot_src,
                                                            int64_t nrows, int64_t T, int cpr, uint4* __restrict__ Z) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  int nxt[ROWS];                                                      // slot sources of the next iteration, fetched one ahead
#pragma unroll
  for (int i = 0; i < ROWS; ++i) nxt[i] = (wave * ROWS + i < nrows) ? slot_src[wave * ROWS + i] : -2;
  for (int64_t r0 = wave * ROWS; r0 < nrows; r0 += nwaves * ROWS) {
    int src[ROWS];
#pragma unroll
    for (int i = 0; i < ROWS; ++i) src[i] = nxt[i];
    const int64_t r1 = r0 + nwaves * ROWS;
#pragma unroll
    for (int i = 0; i < ROWS; ++i) nxt[i] = (r1 + i < nrows) ? slot_src[r1 + i] : -2;
    if (!FILL) {
      bool any = false;
#pragma unroll
      for (int i = 0; i < ROWS; ++i) {
        if (src[i] < 0 || src[i] >= T) src[i] = -2;                 // nothing to do for this slot
        any = any || src[i] != -2;
      }
      if (!any) continue;
    }
    for (int c = lane; c < cpr; c += 64) {
      uint4 v[ROWS];
#pragma unroll
      for (int i = 0; i < ROWS; ++i) v[i] = (src[i] >= 0 && src[i] < T) ? x[(int64_t)src[i] * cpr + c] : make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < ROWS; ++i)
        if (src[i] != -2) Z[(r0 + i) * cpr + c] = v[i];
    }
  }
}

// --- encode, scatter form (no slot_src): zero-fill, then every token row goes to its kept slots ------------------
__global__ __launch_bounds__(256) void zero_fill_kernel(uint4* __restrict__ p, int64_t n16) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256) p[i] = make_uint4(0, 0, 0, 0);
}

// One wave per token: the row is read once and written to each of its kept slots (every slot row is written whole, so the
// stores are as coalesced as the gather form's).  With k choices per token this moves (1 + k) rows per token where the
// gather form moves 2 k (it re-reads the token once per slot, far apart in time).
template <bool STREAM>
__global__ __launch_bounds__(256) void encode_scatter_kernel(const uint4* __restrict__ x, const int32_t* __restrict__ idx,
                                                             const int32_t* __restrict__ loc, int64_t T, int E, int k,
                                                             int64_t C, int cpr, uint4* __restrict__ Z,
                                                             const int64_t* __restrict__ C_dev) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  int64_t Ck = C;                                                    // kept <=> loc < Ck; the slabs keep their stride C
  if (C_dev) { const int64_t c = *C_dev; Ck = c < C ? c : C; }
  for (int64_t t = wave; t < T; t += nwaves) {
    for (int j0 = 0; j0 < k; j0 += 8) {                              // eight choices at a time share one read of the row
      int64_t row[8];
      bool any = false;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        row[u] = -1;
        if (j0 + u < k) {
          const int e = idx[t * k + j0 + u], l = loc[t * k + j0 + u];
          if (l >= 0 && l < Ck && (unsigned)e < (unsigned)E) { row[u] = (int64_t)e * C + l; any = true; }  // kept choice
        }
      }
      if (!any) continue;
      for (int c = lane; c < cpr; c += 64) {
        const uint4 v = STREAM ? load_stream(x + t * cpr + c) : x[t * cpr + c];
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (row[u] >= 0) Z[row[u] * cpr + c] = v;
      }
    }
  }
}

hipError_t launch_encode(const void* x, int dtype, const int32_t* idx, const int32_t* loc, const int32_t* slot_src,
                         int64_t T, int64_t M, int64_t E, int k, int64_t C, void* Z, hipStream_t s, bool fill_unfilled,
                         const int64_t* C_dev) {
  const int es = (dtype == MOE_F32) ? 4 : 2;
  const int cpr = (int)(M * es / 16);
  const int64_t nrows = E * C;
  const int64_t sb = ceil_div(T, 4);
  // Unfilled slots may stay untouched and a token feeds several slots: reading every token once and writing its kept slots
  // moves 1 + k rows per token where the slot-major form moves 2 k.  That pays when most choices are kept (many choices
  // per token, or slots to spare); where capacity is tight and many choices are dropped the slot-major form wins, because
  // it never looks at a dropped token.
  const bool token_major = k >= 4 || (k >= 2 && 4 * E * C >= 5 * T * k);
  if (slot_src && !fill_unfilled && token_major) {
    if ((double)T * M * es >= 536870912.0)                           // token matrix beyond the caches: rows are streamed
      encode_scatter_kernel<true><<<dim3((unsigned)(sb < 16384 ? sb : 16384)), dim3(256), 0, s>>>((const uint4*)x, idx, loc, T, (int)E, k, C, cpr, (uint4*)Z, C_dev);
    else
      encode_scatter_kernel<false><<<dim3((unsigned)(sb < 16384 ? sb : 16384)), dim3(256), 0, s>>>((const uint4*)x, idx, loc, T, (int)E, k, C, cpr, (uint4*)Z, C_dev);
    return hipGetLastError();
  }
  if (slot_src) {
    constexpr int ROWS = 4;
    const int64_t blocks = ceil_div(nrows, 4 * ROWS);
    const unsigned grid = (unsigned)(blocks < 8192 ? blocks : 8192);
    if (fill_unfilled) encode_gather_kernel<ROWS, true><<<dim3(grid), dim3(256), 0, s>>>((const uint4*)x, slot_src, nrows, T, cpr, (uint4*)Z);
    else encode_gather_kernel<ROWS, false><<<dim3(grid), dim3(256), 0, s>>>((const uint4*)x, slot_src, nrows, T, cpr, (uint4*)Z);
    return hipGetLastError();
  }
  const int64_t n16 = nrows * cpr;
  const int64_t zb = ceil_div(n16, 256 * 8);
  zero_fill_kernel<<<dim3((unsigned)(zb < 16384 ? (zb > 0 ? zb : 1) : 16384)), dim3(256), 0, s>>>((uint4*)Z, n16);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  encode_scatter_kernel<false><<<dim3((unsigned)(sb < 16384 ? sb : 16384)), dim3(256), 0, s>>>((const uint4*)x, idx, loc, T, (int)E, k, C, cpr, (uint4*)Z, nullptr);
  return hipGetLastError();
}

// --- decode: out[t,:] = sum_j kept gate_w[t,j] * Y[idx[t,j], loc[t,j], :], fp32 accumulation in rank order -------
template <typename ET> struct Pack16;
template <> struct Pack16<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[4]) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
  static __device__ __forceinline__ uint4 pack(const float (&f)[4]) {
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
  }
};
template <> struct Pack16<uint16_t> {
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

// STREAM: the slabs are far larger than the caches, so their rows are loaded as streamed data (each is read exactly once).
template <typename ET, bool STREAM>
__global__ __launch_bounds__(256) void decode_kernel(const uint4* __restrict__ Y, const int32_t* __restrict__ idx,
                                                     const int32_t* __restrict__ loc, const float* __restrict__ gate_w,
                                                     int64_t T, int E, int k, int64_t C, int cpr, uint4* __restrict__ out,
                                                     const int64_t* __restrict__ C_dev) {
  constexpr int N = Pack16<ET>::N;
  const int lane = threadIdx.x & 63;
  const int64_t wave = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  const int64_t stride = C;                                          // slabs are [E, C, M]; a capacity chosen on the device only
  if (C_dev) { const int64_t c = *C_dev; C = c < C ? c : C; }        // narrows the kept test
  for (int64_t t = wave; t < T; t += nwaves) {
    for (int c = lane; c < cpr; c += 64) {
      float acc[N];
#pragma unroll
      for (int i = 0; i < N; ++i) acc[i] = 0.f;
      for (int j0 = 0; j0 < k; j0 += 4) {
        uint4 v[4];
        float w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int j = j0 + u;
          w[u] = 0.f;
          v[u] = make_uint4(0, 0, 0, 0);
          if (j < k) {
            const int l = loc[t * k + j], e = idx[t * k + j];
            if (l >= 0 && l < C && (unsigned)e < (unsigned)E) {           // kept choice
              w[u] = gate_w ? gate_w[t * k + j] : 1.0f;               // no weights: backward of encode
              const uint4* src = Y + ((int64_t)e * stride + l) * cpr + c;
              v[u] = STREAM ? load_stream(src) : *src;
            }
          }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          float f[N];
          Pack16<ET>::unpack(v[u], f);
#pragma unroll
          for (int i = 0; i < N; ++i) acc[i] = fmaf(w[u], f[i], acc[i]);
        }
      }
      out[t * cpr + c] = Pack16<ET>::pack(acc);
    }
  }
}

// Up to eight choices per token (the usual case): a token's slots and weights are looked up once, then every 16-byte
// piece of the output row has all its source rows in flight at the same time.  Missing and dropped choices enter the sum
// as 0 * 0 in their rank's place.
template <typename ET, bool STREAM>
__global__ __launch_bounds__(256) void decode_k8_kernel(const uint4* __restrict__ Y, const int32_t* __restrict__ idx,
                                                        const int32_t* __restrict__ loc, const float* __restrict__ gate_w,
                                                        int64_t T, int E, int k, int64_t C, int cpr, uint4* __restrict__ out,
                                                        const int64_t* __restrict__ C_dev) {
  constexpr int N = Pack16<ET>::N;
  const int lane = threadIdx.x & 63;
  const int64_t wave = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  const int64_t stride = C;
  if (C_dev) { const int64_t c = *C_dev; C = c < C ? c : C; }
  for (int64_t t = wave; t < T; t += nwaves) {
    int64_t row[8];
    float w[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      row[u] = -1;
      w[u] = 0.f;
      if (u < k) {
        const int l = loc[t * k + u], e = idx[t * k + u];
        if (l >= 0 && l < C && (unsigned)e < (unsigned)E) {           // kept choice
          w[u] = gate_w ? gate_w[t * k + u] : 1.0f;
          row[u] = ((int64_t)e * stride + l) * cpr;
        }
      }
    }
    for (int c = lane; c < cpr; c += 64) {
      uint4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = row[u] >= 0 ? (STREAM ? load_stream(Y + row[u] + c) : Y[row[u] + c]) : make_uint4(0, 0, 0, 0);
      float acc[N];
#pragma unroll
      for (int i = 0; i < N; ++i) acc[i] = 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        float f[N];
        Pack16<ET>::unpack(v[u], f);
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] = fmaf(w[u], f[i], acc[i]);
      }
      out[t * cpr + c] = Pack16<ET>::pack(acc);
    }
  }
}

hipError_t launch_decode(const void* Y, int dtype, const int32_t* idx, const int32_t* loc, const float* gate_w,
                         int64_t T, int64_t M, int64_t E, int k, int64_t C, void* out, hipStream_t s,
                         const int64_t* C_dev) {
  const int es = (dtype == MOE_F32) ? 4 : 2;
  const int cpr = (int)(M * es / 16);
  const int64_t blocks = ceil_div(T, 4);
  const dim3 grid((unsigned)(blocks < 16384 ? blocks : 16384)), block(256);
  // wide choice lists with slabs beyond the caches: all of a token's rows in flight, loaded as streamed data
  const bool wide = k >= 3 && k <= 8, stream = (double)E * C * M * es >= 1073741824.0;
#define MOE_LAUNCH_DECODE(KERNEL, ET, STREAM) KERNEL<ET, STREAM><<<grid, block, 0, s>>>((const uint4*)Y, idx, loc, gate_w, T, (int)E, k, C, cpr, (uint4*)out, C_dev)
#define MOE_LAUNCH_DECODE_ET(KERNEL, STREAM) do { if (dtype == MOE_F32) MOE_LAUNCH_DECODE(KERNEL, float, STREAM); else MOE_LAUNCH_DECODE(KERNEL, uint16_t, STREAM); } while (0)
  if (wide && stream) MOE_LAUNCH_DECODE_ET(decode_k8_kernel, true);
  else if (wide) MOE_LAUNCH_DECODE_ET(decode_k8_kernel, false);
  else if (stream) MOE_LAUNCH_DECODE_ET(decode_kernel, true);
  else MOE_LAUNCH_DECODE_ET(decode_kernel, false);
#undef MOE_LAUNCH_DECODE_ET
#undef MOE_LAUNCH_DECODE
  return hipGetLastError();
}

// --- backward of decode (Appendix B, differentiable fast decode) ---------------------------------------------------
// dY[e,c,:] = gate_w[t,j] * d_out[t,:] for the kept choice (t,j) that owns slot (e,c), zero for an unfilled slot.
// Gather form over the slots, like encode: a wave moves ROWS adjacent slots; the owner's choice j is found by
// comparing the token's k (expert, location) pairs with the slot.
template <typename ET, int ROWS, bool FILL>
__global__ __launch_bounds__(256) void decode_backward_rows_kernel(const uint4* __restrict__ d_out,
                                                                   const int32_t* __restrict__ slot_src,
                                                                   const int32_t* __restrict__ idx,
                                                                   const int32_t* __restrict__ loc,
                                                                   const float* __restrict__ gate_w, int64_t nrows, int64_t T,
                                                                   int k, int64_t C, int cpr, uint4* __restrict__ dY) {
  constexpr int N = Pack16<ET>::N;
  const int lane = threadIdx.x & 63;
  const int64_t wave = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  for (int64_t r0 = wave * ROWS; r0 < nrows; r0 += nwaves * ROWS) {
    int src[ROWS];
    float w[ROWS];
#pragma unroll
    for (int i = 0; i < ROWS; ++i) {
      const int64_t slot = r0 + i;
      src[i] = slot < nrows ? slot_src[slot] : -2;
      w[i] = 0.f;
      if (!FILL && !(src[i] >= 0 && src[i] < T)) src[i] = -2;          // unfilled slot: its row is left untouched
      if (src[i] >= 0 && src[i] < T) {
        const int e = (int)(slot / C), c = (int)(slot % C);
        for (int j = 0; j < k; ++j) {                               // wave-uniform: the same slot in every lane
          const int64_t p = (int64_t)src[i] * k + j;
          if (idx[p] == e && loc[p] == c) w[i] = gate_w[p];
        }
      }
    }
    for (int ch = lane; ch < cpr; ch += 64) {
      uint4 v[ROWS];
#pragma unroll
      for (int i = 0; i < ROWS; ++i) v[i] = (src[i] >= 0 && src[i] < T) ? d_out[(int64_t)src[i] * cpr + ch] : make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < ROWS; ++i) {
        if (src[i] == -2) continue;
        float f[N];
        Pack16<ET>::unpack(v[i], f);
#pragma unroll
        for (int u = 0; u < N; ++u) f[u] = w[i] * f[u];
        dY[(r0 + i) * cpr + ch] = (src[i] >= 0 && src[i] < T) ? Pack16<ET>::pack(f) : make_uint4(0, 0, 0, 0);
      }
    }
  }
}

// dgate_w[t,j] = <d_out[t,:], Y[idx[t,j], loc[t,j], :]> for a kept choice, 0 for a dropped one.  One wave per token:
// every lane sums its 16-byte pieces in fp32, then a fixed butterfly adds the 64 partial sums (deterministic).
template <typename ET>
__global__ __launch_bounds__(256) void gate_weight_grad_kernel(const uint4* __restrict__ d_out, const uint4* __restrict__ Y,
                                                               const int32_t* __restrict__ idx,
                                                               const int32_t* __restrict__ loc, int64_t T, int E, int k,
                                                               int64_t C, int cpr, float* __restrict__ dgate_w) {
  constexpr int N = Pack16<ET>::N;
  const int lane = threadIdx.x & 63;
  const int64_t wave = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  for (int64_t t = wave; t < T; t += nwaves) {
    for (int j = 0; j < k; ++j) {
      const int l = loc[t * k + j], e = idx[t * k + j];
      float acc = 0.f;
      if (l >= 0 && l < C && (unsigned)e < (unsigned)E) {           // kept choice (wave-uniform)
        const int64_t row = (int64_t)e * C + l;
        for (int ch = lane; ch < cpr; ch += 64) {
          float a[N], b[N];
          Pack16<ET>::unpack(d_out[t * cpr + ch], a);
          Pack16<ET>::unpack(Y[row * cpr + ch], b);
#pragma unroll
          for (int u = 0; u < N; ++u) acc = fmaf(a[u], b[u], acc);
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, 64);
      }
      if (lane == 0) dgate_w[t * k + j] = acc;
    }
  }
}

// Both results in one pass over the tokens, for callers that leave unfilled slots alone (the layer's backward): a wave
// reads its token's d_out row once and, for up to eight kept choices at a time, reads the choice's row of Y (for the
// dot product) and writes its row of dY.  d_out [T,M] is read once instead of once per slot and once per choice.  The
// arithmetic and its order are those of the two kernels above, so the results are bit-identical to theirs.
template <typename ET, bool STREAM>
__global__ __launch_bounds__(256) void decode_backward_token_kernel(const uint4* __restrict__ d_out, const uint4* __restrict__ Y,
                                                                    const int32_t* __restrict__ idx,
                                                                    const int32_t* __restrict__ loc,
                                                                    const float* __restrict__ gate_w, int64_t T, int E, int k,
                                                                    int64_t C, int cpr, uint4* __restrict__ dY,
                                                                    float* __restrict__ dgate_w) {
  constexpr int N = Pack16<ET>::N;
  const int lane = threadIdx.x & 63;
  const int64_t wave = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  for (int64_t t = wave; t < T; t += nwaves) {
    for (int j0 = 0; j0 < k; j0 += 8) {
      int64_t row[8];
      float w[8], acc[8];
      bool any = false;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        row[u] = -1;
        w[u] = 0.f;
        acc[u] = 0.f;
        if (j0 + u < k) {
          const int e = idx[t * k + j0 + u], l = loc[t * k + j0 + u];
          if (l >= 0 && l < C && (unsigned)e < (unsigned)E) {       // kept choice (wave-uniform)
            row[u] = (int64_t)e * C + l;
            w[u] = gate_w[t * k + j0 + u];
            any = true;
          }
        }
      }
      if (any) {
        for (int ch = lane; ch < cpr; ch += 64) {
          float a[N];
          Pack16<ET>::unpack(d_out[t * cpr + ch], a);
          uint4 yv[8];
#pragma unroll
          for (int u = 0; u < 8; ++u)
            if (row[u] >= 0) yv[u] = STREAM ? load_stream(Y + row[u] * cpr + ch) : Y[row[u] * cpr + ch];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            if (row[u] < 0) continue;
            float b[N], f[N];
            Pack16<ET>::unpack(yv[u], b);
#pragma unroll
            for (int v = 0; v < N; ++v) acc[u] = fmaf(a[v], b[v], acc[u]);
#pragma unroll
            for (int v = 0; v < N; ++v) f[v] = w[u] * a[v];
            dY[row[u] * cpr + ch] = Pack16<ET>::pack(f);
          }
        }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (j0 + u >= k) break;
        float sum = acc[u];
        if (row[u] >= 0) {
#pragma unroll
          for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d, 64);
        }
        if (lane == 0) dgate_w[t * k + j0 + u] = sum;
      }
    }
  }
}

hipError_t launch_decode_backward(const void* d_out, const void* Y, int dtype, const int32_t* idx, const int32_t* loc,
                                  const float* gate_w, const int32_t* slot_src, int64_t T, int64_t M, int64_t E, int k,
                                  int64_t C, void* dY, float* dgate_w, hipStream_t s, bool fill_unfilled) {
  const int es = (dtype == MOE_F32) ? 4 : 2;
  const int cpr = (int)(M * es / 16);
  const dim3 block(256);
  if (dY && dgate_w && !fill_unfilled) {
    const int64_t blocks = ceil_div(T, 4);
    const dim3 grid((unsigned)(blocks < 16384 ? blocks : 16384));
    const bool stream = (double)E * C * M * es >= 1073741824.0;
#define MOE_LAUNCH_DBT(ET, STREAM) decode_backward_token_kernel<ET, STREAM><<<grid, block, 0, s>>>((const uint4*)d_out, (const uint4*)Y, idx, loc, gate_w, T, (int)E, k, C, cpr, (uint4*)dY, dgate_w)
    if (dtype == MOE_F32) { if (stream) MOE_LAUNCH_DBT(float, true); else MOE_LAUNCH_DBT(float, false); }
    else { if (stream) MOE_LAUNCH_DBT(uint16_t, true); else MOE_LAUNCH_DBT(uint16_t, false); }
#undef MOE_LAUNCH_DBT
    return hipGetLastError();
  }
  if (dY) {
    constexpr int ROWS = 4;
    const int64_t nrows = E * C, blocks = ceil_div(nrows, 4 * ROWS);
    const dim3 grid((unsigned)(blocks < 8192 ? blocks : 8192));
#define MOE_LAUNCH_DBR(ET, FILL) decode_backward_rows_kernel<ET, ROWS, FILL><<<grid, block, 0, s>>>((const uint4*)d_out, slot_src, idx, loc, gate_w, nrows, T, k, C, cpr, (uint4*)dY)
    if (dtype == MOE_F32) { if (fill_unfilled) MOE_LAUNCH_DBR(float, true); else MOE_LAUNCH_DBR(float, false); }
    else { if (fill_unfilled) MOE_LAUNCH_DBR(uint16_t, true); else MOE_LAUNCH_DBR(uint16_t, false); }
#undef MOE_LAUNCH_DBR
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
  }
  if (dgate_w) {
    const int64_t blocks = ceil_div(T, 4);
    const dim3 grid((unsigned)(blocks < 16384 ? blocks : 16384));
    if (dtype == MOE_F32)
      gate_weight_grad_kernel<float><<<grid, block, 0, s>>>((const uint4*)d_out, (const uint4*)Y, idx, loc, T, (int)E, k, C, cpr, dgate_w);
    else
      gate_weight_grad_kernel<uint16_t><<<grid, block, 0, s>>>((const uint4*)d_out, (const uint4*)Y, idx, loc, T, (int)E, k, C, cpr, dgate_w);
  }
  return hipGetLastError();
}

}  // namespace moe
