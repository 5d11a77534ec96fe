// Memory-bound fused kernels between the GEMMs (paper sec. 2.1): token embedding + position,
// and split-K reduction + bias + residual add + LayerNorm in one launch with no intermediate.
#include "lsq_internal.h"

namespace lsq {

// ---------------------------------------------------------------------------------------------
// Token embedding + position: embed_row (lsq_internal.h) over the rows of a launch.
template <typename T>
__global__ void __launch_bounds__(256) embed_rows_kernel(const T* __restrict__ E, const float* __restrict__ pe,
                                                         const int32_t* __restrict__ ids,
                                                         const int32_t* __restrict__ pos, T* __restrict__ x,
                                                         int rows, int d, float scale) {
  int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  embed_row<T>(E + (size_t)ids[r] * d, pe + (size_t)pos[r] * d, x + (size_t)r * d, d, scale,
               threadIdx.x & 63, 64);
}

// Decoder input of step t: the last token of every hypothesis row.
template <typename T>
__global__ void __launch_bounds__(256) embed_last_kernel(const T* __restrict__ E, const float* __restrict__ pe,
                                                         const int32_t* __restrict__ tokens,
                                                         const int32_t* __restrict__ len, T* __restrict__ x,
                                                         int rows, int d, int T1, const int32_t* __restrict__ tp,
                                                         float scale) {
  int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  const int t = *tp;   // decode-step counter, kept on the device
  int id = tokens[(size_t)r * T1 + len[r]];
  embed_row<T>(E + (size_t)id * d, pe + (size_t)t * d, x + (size_t)r * d, d, scale, threadIdx.x & 63, 64);
}

hipError_t launch_embed_rows(int dtype, const void* E, const float* pe, const int32_t* ids,
                             const int32_t* pos, void* x, int rows, int d, float scale, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  dim3 g((rows + 3) / 4), b(256);
  if (dtype == DT_F16)
    embed_rows_kernel<half_t><<<g, b, 0, s>>>((const half_t*)E, pe, ids, pos, (half_t*)x, rows, d, scale);
  else
    embed_rows_kernel<float><<<g, b, 0, s>>>((const float*)E, pe, ids, pos, (float*)x, rows, d, scale);
  return hipGetLastError();
}

hipError_t launch_embed_last(int dtype, const void* E, const float* pe, const int32_t* tokens,
                             const int32_t* len, void* x, int rows, int d, int T, const int32_t* tp, float scale,
                             hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  dim3 g((rows + 3) / 4), b(256);
  if (dtype == DT_F16)
    embed_last_kernel<half_t><<<g, b, 0, s>>>((const half_t*)E, pe, tokens, len, (half_t*)x, rows, d, T + 1, tp, scale);
  else
    embed_last_kernel<float><<<g, b, 0, s>>>((const float*)E, pe, tokens, len, (float*)x, rows, d, T + 1, tp, scale);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Residual + LayerNorm in one launch with no intermediate (paper sec. 2.1): one wavefront per row,
// the row held in registers (NV vectors of 8 per lane), mean then centred variance (biased), both
// by reductions over the wavefront.  The sublayer output arrives as `splits` fp32 partial-sum slabs
// P[s][rows][d] (the split-K GEMM's output, still without its bias):
//   x <- store(LN(x + (sum_s P[s] + bias)) * g + b).
// The slabs are added in index order, so the result is independent of how the GEMM was scheduled.
// PRE (pre-LN blocks): the residual stream itself is updated, x <- store(x + sum_s P[s] + bias), and
// the normalised copy y <- store(LN(x) * g + b) goes to a second buffer for the next sublayer's GEMM;
// S = 0 means "no sublayer output to add", i.e. y <- LN(x).
template <typename T, int NV, int S, bool PRE>
__global__ void __launch_bounds__(256) add_layernorm_partials_kernel(T* __restrict__ x, T* __restrict__ y,
                                                                     const float* __restrict__ P,
                                                                     const T* __restrict__ bias,
                                                                     const T* __restrict__ g, const T* __restrict__ b,
                                                                     int rows, int d, float eps,
                                                                     const T* __restrict__ x_in) {
  int r = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);   // one wavefront per row, 1..4 rows per workgroup
  if (r >= rows) return;
  int lane = threadIdx.x & 63;
  T* xr = x + (size_t)r * d;
  const T* xi = x_in ? x_in + (size_t)r * d : xr;   // the residual may come from another buffer (x is then only written)
  const size_t slab = (size_t)rows * d;
  float v[NV][8], gv[NV][8], bv[NV][8];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    int c = (j * 64 + lane) * 8;
    if (c < d) {
      float t[8], part[S > 0 ? S : 1][8];
#pragma unroll
      for (int s = 0; s < S; ++s) Vec8<float>::load(P + s * slab + (size_t)r * d + c, part[s]);   // all in flight
      if (S > 0) Vec8<T>::load(bias + c, t);
      Vec8<T>::load(xi + c, v[j]);
      Vec8<T>::load(g + c, gv[j]);      // gain and shift too: one round trip to memory in all
      Vec8<T>::load(b + c, bv[j]);
      if (S > 0) {
        add_partials<(S > 0 ? S : 1)>(v[j], part, S, t);
        if (PRE) {   // the residual stream is stored here; LayerNorm sees the stored values
#pragma unroll
          for (int i = 0; i < 8; ++i) v[j][i] = (float)(T)v[j][i];
          Vec8<T>::store(xr + c, v[j]);
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) { v[j][i] = 0.f; gv[j][i] = 0.f; bv[j][i] = 0.f; }
    }
  }
  float o[NV][8];
  layernorm_row<NV>(v, gv, bv, d, eps, lane, o);
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    int c = (j * 64 + lane) * 8;
    if (c < d) Vec8<T>::store((PRE ? y + (size_t)r * d : xr) + c, o[j]);
  }
}

template <typename T>
__global__ void __launch_bounds__(256) add_layernorm_partials_generic_kernel(T* __restrict__ x,
                                                                             const float* __restrict__ P, int splits,
                                                                             const T* __restrict__ bias,
                                                                             const T* __restrict__ g,
                                                                             const T* __restrict__ b, int rows, int d,
                                                                             float eps, const T* __restrict__ x_in) {
  int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  int lane = threadIdx.x & 63;
  T* xr = x + (size_t)r * d;
  const T* xi = x_in ? x_in + (size_t)r * d : xr;
  const size_t slab = (size_t)rows * d;
  auto val = [&](int c) {
    float a = P[(size_t)r * d + c];
    for (int s = 1; s < splits; ++s) a += P[s * slab + (size_t)r * d + c];
    return (float)xi[c] + (a + (float)bias[c]);
  };
  float sum = 0.f;
  for (int c = lane; c < d; c += 64) sum += val(c);
  float mean = wave_sum(sum) / (float)d;
  float sq = 0.f;
  for (int c = lane; c < d; c += 64) { float t = val(c) - mean; sq += t * t; }
  float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)d + eps);
  for (int c = lane; c < d; c += 64) {
    float t = val(c) - mean;
    xr[c] = (T)((float)g[c] * (t * rstd) + (float)b[c]);
  }
}

template <typename T, int S, bool PRE>
static hipError_t add_layernorm_partials_s(T* x, T* y, const float* P, const T* bias, const T* g, const T* b,
                                           int rows, int d, float eps, hipStream_t s, const T* x_in) {
  // Decoding sizes: a workgroup per row, so that the rows spread over as many CUs as there are rows
  // (a CU takes in its rows' slabs at a fixed rate; measured on whole steps against four rows per
  // workgroup: 0.461 -> 0.449 ms with 8 slabs of 32 rows, 0.492 -> 0.490 with 2 slabs of 512 rows).
  // Thousands of rows (encoder, prefill) fill the chip either way and keep four per workgroup.
  const int rpw = rows <= 2048 ? 1 : 4;
  dim3 grid((rows + rpw - 1) / rpw), blk(64 * rpw);
  if (d <= 512)
    add_layernorm_partials_kernel<T, 1, S, PRE><<<grid, blk, 0, s>>>(x, y, P, bias, g, b, rows, d, eps, x_in);
  else if (d <= 1024)
    add_layernorm_partials_kernel<T, 2, S, PRE><<<grid, blk, 0, s>>>(x, y, P, bias, g, b, rows, d, eps, x_in);
  else if (d <= 2048)
    add_layernorm_partials_kernel<T, 4, S, PRE><<<grid, blk, 0, s>>>(x, y, P, bias, g, b, rows, d, eps, x_in);
  else
    add_layernorm_partials_kernel<T, 8, S, PRE><<<grid, blk, 0, s>>>(x, y, P, bias, g, b, rows, d, eps, x_in);
  return hipGetLastError();
}

template <typename T>
static hipError_t add_layernorm_partials_t(T* x, T* y, const float* P, int splits, const T* bias, const T* g,
                                           const T* b, int rows, int d, float eps, hipStream_t s, const T* x_in) {
  const bool pre = y != nullptr;
  if ((d & 7) != 0 || d > 4096 || (splits != 0 && splits != 1 && splits != 2 && splits != 4 && splits != 8 && !(splits == 16 && y == nullptr)) ||
      (splits == 0 && !pre)) {
    if (pre) return hipErrorInvalidValue;   // pre-LN models need d % 8 == 0, d <= 4096, 0/1/2/4/8 slabs
    dim3 grid((rows + 3) / 4), blk(256);
    add_layernorm_partials_generic_kernel<T><<<grid, blk, 0, s>>>(x, P, splits, bias, g, b, rows, d, eps, x_in);
    return hipGetLastError();
  }
  if (pre) {
    switch (splits) {
      case 0: return add_layernorm_partials_s<T, 0, true>(x, y, P, bias, g, b, rows, d, eps, s, x_in);
      case 1: return add_layernorm_partials_s<T, 1, true>(x, y, P, bias, g, b, rows, d, eps, s, x_in);
      case 2: return add_layernorm_partials_s<T, 2, true>(x, y, P, bias, g, b, rows, d, eps, s, x_in);
      case 4: return add_layernorm_partials_s<T, 4, true>(x, y, P, bias, g, b, rows, d, eps, s, x_in);
      default: return add_layernorm_partials_s<T, 8, true>(x, y, P, bias, g, b, rows, d, eps, s, x_in);
    }
  }
  switch (splits) {
    case 1: return add_layernorm_partials_s<T, 1, false>(x, y, P, bias, g, b, rows, d, eps, s, x_in);
    case 2: return add_layernorm_partials_s<T, 2, false>(x, y, P, bias, g, b, rows, d, eps, s, x_in);
    case 4: return add_layernorm_partials_s<T, 4, false>(x, y, P, bias, g, b, rows, d, eps, s, x_in);
    case 16: return add_layernorm_partials_s<T, 16, false>(x, y, P, bias, g, b, rows, d, eps, s, x_in);   // one slab per head
    default: return add_layernorm_partials_s<T, 8, false>(x, y, P, bias, g, b, rows, d, eps, s, x_in);
  }
}

// Decoder-only models, first kernel of a step: x[r] = store(E[last token of r] * scale + pe[position]) and
// y[r] = store(LN(x[r]) * g + b) in one launch (embed_last_kernel followed by the pre-LN kernel with no slabs: the same
// arithmetic, LayerNorm sees the stored row).  One wavefront per row; d a multiple of 8, at most 64 * 8 * NV.
template <typename T, int NV>
__global__ void __launch_bounds__(64) embed_layernorm_kernel(const T* __restrict__ E, const float* __restrict__ pe,
                                                             const int32_t* __restrict__ tokens,
                                                             const int32_t* __restrict__ len, T* __restrict__ x,
                                                             T* __restrict__ y, const T* __restrict__ g,
                                                             const T* __restrict__ b, int rows, int d, int T1,
                                                             const int32_t* __restrict__ tp, float scale, float eps) {
  const int r = blockIdx.x, lane = threadIdx.x;
  if (r >= rows) return;
  const int t = *tp;
  const int id = tokens[(size_t)r * T1 + len[r]];
  const T* e = E + (size_t)id * d;
  const float* per = pe + (size_t)t * d;
  float v[NV][8], gv[NV][8], bv[NV][8];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int c = (j * 64 + lane) * 8;
    if (c < d) {
      Vec8<T>::load(e + c, v[j]);
      Vec8<T>::load(g + c, gv[j]);
      Vec8<T>::load(b + c, bv[j]);
#pragma unroll
      for (int i = 0; i < 8; ++i) v[j][i] = (float)(T)__fadd_rn(__fmul_rn(v[j][i], scale), per[c + i]);   // as embed_row stores it
      Vec8<T>::store(x + (size_t)r * d + c, v[j]);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) { v[j][i] = 0.f; gv[j][i] = 0.f; bv[j][i] = 0.f; }
    }
  }
  float o[NV][8];
  layernorm_row<NV>(v, gv, bv, d, eps, lane, o);
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int c = (j * 64 + lane) * 8;
    if (c < d) Vec8<T>::store(y + (size_t)r * d + c, o[j]);
  }
}

bool embed_layernorm_supported(int d) { return d % 8 == 0 && d <= 4096; }

hipError_t launch_embed_layernorm(int dtype, const void* E, const float* pe, const int32_t* tokens, const int32_t* len,
                                  void* x, void* y, const void* g, const void* b, int rows, int d, int T,
                                  const int32_t* tp, float scale, float eps, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (!embed_layernorm_supported(d)) return hipErrorInvalidValue;
#define LSQ_EL(T_, NV_)                                                                                                   \
  embed_layernorm_kernel<T_, NV_><<<rows, 64, 0, s>>>((const T_*)E, pe, tokens, len, (T_*)x, (T_*)y, (const T_*)g, (const T_*)b, \
                                                      rows, d, T + 1, tp, scale, eps)
  if (dtype == DT_F16) {
    if (d <= 512) LSQ_EL(half_t, 1); else if (d <= 1024) LSQ_EL(half_t, 2); else if (d <= 2048) LSQ_EL(half_t, 4); else LSQ_EL(half_t, 8);
  } else {
    if (d <= 512) LSQ_EL(float, 1); else if (d <= 1024) LSQ_EL(float, 2); else if (d <= 2048) LSQ_EL(float, 4); else LSQ_EL(float, 8);
  }
#undef LSQ_EL
  return hipGetLastError();
}

// y == nullptr: post-LN (x <- LN(x + sublayer)); y != nullptr: pre-LN (x <- x + sublayer, y <- LN(x)).
hipError_t launch_add_layernorm_partials(int dtype, void* x, void* y, const float* P, int splits, const void* bias,
                                         const void* g, const void* b, int rows, int d, float eps, hipStream_t s,
                                         const void* x_in) {
  if (rows <= 0) return hipSuccess;
  if (splits < 0 || (x_in && (y || x_in == x))) return hipErrorInvalidValue;   // a separate residual input: post-LN only
  if (dtype == DT_F16)
    return add_layernorm_partials_t<half_t>((half_t*)x, (half_t*)y, P, splits, (const half_t*)bias,
                                            (const half_t*)g, (const half_t*)b, rows, d, eps, s, (const half_t*)x_in);
  return add_layernorm_partials_t<float>((float*)x, (float*)y, P, splits, (const float*)bias, (const float*)g,
                                         (const float*)b, rows, d, eps, s, (const float*)x_in);
}

// Prefill of a decoder-only model: copies the K and V thirds of packed [rows, 3d] projections into
// the cache rows [sentence][position] (cache row stride = T * d elements).
template <typename T>
__global__ void __launch_bounds__(256) scatter_kv_kernel(const T* __restrict__ qkv, const int32_t* __restrict__ sent,
                                                         const int32_t* __restrict__ pos, T* __restrict__ Kc,
                                                         T* __restrict__ Vc, int rows, int d, int T_) {
  int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  const size_t dst = ((size_t)sent[r] * T_ + pos[r]) * d;
  for (int c = (threadIdx.x & 63) * 8; c < d; c += 64 * 8) {
    float t[8];
    Vec8<T>::load(qkv + (size_t)r * 3 * d + d + c, t);
    Vec8<T>::store(Kc + dst + c, t);
    Vec8<T>::load(qkv + (size_t)r * 3 * d + 2 * d + c, t);
    Vec8<T>::store(Vc + dst + c, t);
  }
}

hipError_t launch_scatter_kv(int dtype, const void* qkv, const int32_t* sent, const int32_t* pos, void* Kc, void* Vc,
                             int rows, int d, int T, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  dim3 grid((rows + 3) / 4), blk(256);
  if (dtype == DT_F16)
    scatter_kv_kernel<half_t><<<grid, blk, 0, s>>>((const half_t*)qkv, sent, pos, (half_t*)Kc, (half_t*)Vc, rows, d, T);
  else
    scatter_kv_kernel<float><<<grid, blk, 0, s>>>((const float*)qkv, sent, pos, (float*)Kc, (float*)Vc, rows, d, T);
  return hipGetLastError();
}

}  // namespace lsq
