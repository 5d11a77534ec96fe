// Scaled, masked softmax over keys fused with the value sum (paper sec. 2.1 fusion rule applied
// to attention): one wavefront per (key/value stream, head).  HBM-bound: every key and value is
// read exactly once per wavefront, 16 bytes per lane.
//
// Lane layout: a head row of DH elements is split over LPK = DH/8 lanes (8 elements each), so a
// wavefront covers KPI = 64/LPK keys per iteration.  Each lane group runs its own online softmax
// (running max, running sum, running value accumulator) over the keys it sees; the groups are
// merged by shuffles at the end.  Masking is by key count: keys beyond it are never read.
#include "lsq_internal.h"

namespace lsq {

// Keys j0, j0 + jstep, j0 + 2*jstep, ... (< nkeys) are visited, each lane group taking every
// KPI-th of them.  On return every lane holds, for its 8 elements of the head row, the merged
// (running max m, running sum l, un-normalised accumulator acc) of all keys this wavefront saw.
template <typename T, int DH, int NQ>
__device__ __forceinline__ void attend_partial(const T* const (&qp)[NQ], const T* __restrict__ K,
                                               const T* __restrict__ V, long stride, int nkeys, float scale,
                                               int j0, int jstep, int lane, float (&m)[NQ], float (&l)[NQ],
                                               float (&acc)[NQ][8]) {
  constexpr int LPK = DH / 8;
  constexpr int KPI = 64 / LPK;
  const int g = lane / LPK, c = lane % LPK;
  float q[NQ][8];
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    Vec8<T>::load(qp[n] + c * 8, q[n]);
    m[n] = -INFINITY;
    l[n] = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[n][i] = 0.f;
  }
  for (int j = j0 + g * jstep; j < nkeys; j += KPI * jstep) {
    float kv[8], vv[8];
    Vec8<T>::load(K + (long)j * stride + c * 8, kv);
    Vec8<T>::load(V + (long)j * stride + c * 8, vv);
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) s += q[n][i] * kv[i];
#pragma unroll
      for (int o = 1; o < LPK; o <<= 1) s += __shfl_xor(s, o, kWave);
      s *= scale;
      float mn = fmaxf(m[n], s);
      float corr = __expf(m[n] - mn);   // m = -inf on the first key: exp(-inf) = 0
      float p = __expf(s - mn);
      l[n] = l[n] * corr + p;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[n][i] = acc[n][i] * corr + p * vv[i];
      m[n] = mn;
    }
  }
  // merge the KPI lane groups (butterfly: every group ends with the total)
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
#pragma unroll
    for (int o = LPK; o < 64; o <<= 1) {
      float m2 = __shfl_xor(m[n], o, kWave);
      float l2 = __shfl_xor(l[n], o, kWave);
      float mn = fmaxf(m[n], m2);
      float c1 = (m[n] == -INFINITY) ? 0.f : __expf(m[n] - mn);
      float c2 = (m2 == -INFINITY) ? 0.f : __expf(m2 - mn);
      l[n] = l[n] * c1 + l2 * c2;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float a2 = __shfl_xor(acc[n][i], o, kWave);
        acc[n][i] = acc[n][i] * c1 + a2 * c2;
      }
      m[n] = mn;
    }
  }
}

template <typename T, int DH, int NQ>
__device__ __forceinline__ void attend(const T* const (&qp)[NQ], const T* __restrict__ K,
                                       const T* __restrict__ V, long stride, int nkeys, float scale,
                                       T* const (&op)[NQ], int lane) {
  constexpr int LPK = DH / 8;
  float m[NQ], l[NQ], acc[NQ][8];
  attend_partial<T, DH, NQ>(qp, K, V, stride, nkeys, scale, 0, 1, lane, m, l, acc);
  if (lane < LPK) {
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
      float o8[8];
      float inv = 1.0f / l[n];
#pragma unroll
      for (int i = 0; i < 8; ++i) o8[i] = acc[n][i] * inv;
      Vec8<T>::store(op[n] + lane * 8, o8);
    }
  }
}

// Decoder self-attention: row r, head h over cache positions 0..nkeys-1 of Kc/Vc [rows, T, d].
template <typename T, int DH>
__global__ void __launch_bounds__(256) self_attention_kernel(const T* __restrict__ q, const T* __restrict__ Kc,
                                                             const T* __restrict__ Vc, T* __restrict__ out,
                                                             int rows, int H, int d, int T_, int nkeys_base,
                                                             const int32_t* __restrict__ tp, float scale) {
  int w = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (w >= rows * H) return;
  const int nkeys = nkeys_base + (tp ? *tp : 0);
  int r = w / H, h = w % H;
  const T* qp[1] = {q + (size_t)r * d + h * DH};
  T* op[1] = {out + (size_t)r * d + h * DH};
  size_t base = (size_t)r * T_ * d + h * DH;
  attend<T, DH, 1>(qp, Kc + base, Vc + base, d, nkeys, scale, op, threadIdx.x & 63);
}

// Cross-attention: the NQ beams of one sentence share each key/value load.  kv rows are [K | V].
// One workgroup of 4 wavefronts per (sentence, head): wavefront w takes keys w, w+4, w+8, ...
// (source sentences have very different lengths and a workgroup's time is set by its key loop,
// so the loop is cut four ways); the four partial softmax states are merged through LDS.
template <typename T, int DH, int NQ>
__global__ void __launch_bounds__(256) cross_attention_kernel(const T* __restrict__ q, const T* __restrict__ kv,
                                                              const int32_t* __restrict__ off,
                                                              const int32_t* __restrict__ len,
                                                              T* __restrict__ out, int batch, int beam,
                                                              int first, int H, int d, float scale) {
  constexpr int LPK = DH / 8;
  __shared__ float sm[4][NQ], sl[4][NQ], sacc[4][NQ][DH];
  const int b = blockIdx.x / H, h = blockIdx.x % H;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const T* qp[NQ];
#pragma unroll
  for (int n = 0; n < NQ; ++n) qp[n] = q + ((size_t)b * beam + first + n) * d + h * DH;
  const T* K = kv + (size_t)off[b] * 2 * d + h * DH;
  float m[NQ], l[NQ], acc[NQ][8];
  attend_partial<T, DH, NQ>(qp, K, K + d, 2 * d, len[b], scale, wave, 4, lane, m, l, acc);
  if (lane < LPK) {
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
      if (lane == 0) { sm[wave][n] = m[n]; sl[wave][n] = l[n]; }
#pragma unroll
      for (int i = 0; i < 8; ++i) sacc[wave][n][lane * 8 + i] = acc[n][i];
    }
  }
  __syncthreads();
  // thread (n, e) finishes element e of beam n
  for (int idx = threadIdx.x; idx < NQ * DH; idx += 256) {
    const int n = idx / DH, e = idx % DH;
    float mm = fmaxf(fmaxf(sm[0][n], sm[1][n]), fmaxf(sm[2][n], sm[3][n]));
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      float c = (sm[w][n] == -INFINITY) ? 0.f : __expf(sm[w][n] - mm);
      num += sacc[w][n][e] * c;
      den += sl[w][n] * c;
    }
    out[((size_t)b * beam + first + n) * d + h * DH + e] = (T)(num / den);
  }
}

// Encoder self-attention over packed sentences: qkv rows are [Q | K | V]; row i belongs to
// sentence row_sent[i] whose rows start at off[.] and number len[.].
template <typename T, int DH>
__global__ void __launch_bounds__(256) encoder_attention_kernel(const T* __restrict__ qkv,
                                                                const int32_t* __restrict__ row_sent,
                                                                const int32_t* __restrict__ off,
                                                                const int32_t* __restrict__ len,
                                                                T* __restrict__ out, int rows, int H, int d,
                                                                float scale) {
  int w = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (w >= rows * H) return;
  int r = w / H, h = w % H;
  int b = row_sent[r];
  const T* qp[1] = {qkv + (size_t)r * 3 * d + h * DH};
  T* op[1] = {out + (size_t)r * d + h * DH};
  const T* K = qkv + (size_t)off[b] * 3 * d + d + h * DH;
  attend<T, DH, 1>(qp, K, K + d, 3 * d, len[b], scale, op, threadIdx.x & 63);
}

bool head_dim_supported(int dh) { return dh == 16 || dh == 32 || dh == 64 || dh == 128; }

#define LSQ_DISPATCH_DH(DHV, ...)                 \
  switch (DHV) {                                  \
    case 16: { constexpr int DH = 16; __VA_ARGS__; break; }   \
    case 32: { constexpr int DH = 32; __VA_ARGS__; break; }   \
    case 64: { constexpr int DH = 64; __VA_ARGS__; break; }   \
    case 128: { constexpr int DH = 128; __VA_ARGS__; break; } \
    default: return hipErrorInvalidValue;         \
  }

template <typename T>
static hipError_t self_t(const T* q, const T* Kc, const T* Vc, T* out, int rows, int H, int d, int T_,
                         int nkeys, const int32_t* tp, hipStream_t s) {
  int dh = d / H;
  float scale = 1.0f / sqrtf((float)dh);
  dim3 g((rows * H + 3) / 4), b(256);
  LSQ_DISPATCH_DH(dh, (self_attention_kernel<T, DH><<<g, b, 0, s>>>(q, Kc, Vc, out, rows, H, d, T_, nkeys, tp, scale)));
  return hipGetLastError();
}

hipError_t launch_self_attention(int dtype, const void* q, const void* Kc, const void* Vc, void* out,
                                 int rows, int H, int d, int T, int nkeys, const int32_t* tp, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (dtype == DT_F16)
    return self_t<half_t>((const half_t*)q, (const half_t*)Kc, (const half_t*)Vc, (half_t*)out, rows, H, d, T, nkeys, tp, s);
  return self_t<float>((const float*)q, (const float*)Kc, (const float*)Vc, (float*)out, rows, H, d, T, nkeys, tp, s);
}

template <typename T, int NQ>
static hipError_t cross_nq(const T* q, const T* kv, const int32_t* off, const int32_t* len, T* out,
                           int batch, int beam, int first, int H, int d, hipStream_t s) {
  int dh = d / H;
  float scale = 1.0f / sqrtf((float)dh);
  dim3 g(batch * H), b(256);
  LSQ_DISPATCH_DH(dh, (cross_attention_kernel<T, DH, NQ><<<g, b, 0, s>>>(q, kv, off, len, out, batch, beam, first, H, d, scale)));
  return hipGetLastError();
}

template <typename T>
static hipError_t cross_t(const T* q, const T* kv, const int32_t* off, const int32_t* len, T* out, int batch,
                          int beam, int H, int d, hipStream_t s) {
  // beams are handled in groups of 4, 2 or 1 queries per wavefront
  int first = 0;
  while (first < beam) {
    int left = beam - first;
    hipError_t e;
    if (left >= 4) { e = cross_nq<T, 4>(q, kv, off, len, out, batch, beam, first, H, d, s); first += 4; }
    else if (left >= 2) { e = cross_nq<T, 2>(q, kv, off, len, out, batch, beam, first, H, d, s); first += 2; }
    else { e = cross_nq<T, 1>(q, kv, off, len, out, batch, beam, first, H, d, s); first += 1; }
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_cross_attention(int dtype, const void* q, const void* kv, const int32_t* off,
                                  const int32_t* len, void* out, int batch, int beam, int H, int d,
                                  hipStream_t s) {
  if (batch <= 0) return hipSuccess;
  if (dtype == DT_F16)
    return cross_t<half_t>((const half_t*)q, (const half_t*)kv, off, len, (half_t*)out, batch, beam, H, d, s);
  return cross_t<float>((const float*)q, (const float*)kv, off, len, (float*)out, batch, beam, H, d, s);
}

template <typename T>
static hipError_t enc_t(const T* qkv, const int32_t* row_sent, const int32_t* off, const int32_t* len, T* out,
                        int rows, int H, int d, hipStream_t s) {
  int dh = d / H;
  float scale = 1.0f / sqrtf((float)dh);
  dim3 g((rows * H + 3) / 4), b(256);
  LSQ_DISPATCH_DH(dh, (encoder_attention_kernel<T, DH><<<g, b, 0, s>>>(qkv, row_sent, off, len, out, rows, H, d, scale)));
  return hipGetLastError();
}

hipError_t launch_encoder_attention(int dtype, const void* qkv, const int32_t* row_sent, const int32_t* off,
                                    const int32_t* len, void* out, int rows, int H, int d, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (dtype == DT_F16)
    return enc_t<half_t>((const half_t*)qkv, row_sent, off, len, (half_t*)out, rows, H, d, s);
  return enc_t<float>((const float*)qkv, row_sent, off, len, (float*)out, rows, H, d, s);
}

}  // namespace lsq
