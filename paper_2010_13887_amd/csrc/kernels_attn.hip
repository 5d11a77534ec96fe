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
// slot != nullptr: position j is not in this row's own slab but in slab slot[j] of its sentence
// (K + slot[j] * slot_stride); the slot numbers of the next pass are requested together with the
// rows of the current one, so the extra indirection is off the critical path after the first pass.
template <typename T, int DH, int NQ>
__device__ __forceinline__ void attend_partial(const T* const (&qp)[NQ], const T* __restrict__ K,
                                               const T* __restrict__ V, long stride, int nkeys, float scale,
                                               int j0, int jstep, int lane, float (&m)[NQ], float (&l)[NQ],
                                               float (&acc)[NQ][8], const int32_t* __restrict__ slot = nullptr,
                                               long slot_stride = 0) {
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
  // U keys per lane group are requested (K and V rows) before any is used, so a cache of n
  // positions costs n / (KPI * U) round trips to memory instead of n / KPI.
  constexpr int U = 4;
  const int step = KPI * jstep;
  int sl[U];
#pragma unroll
  for (int u = 0; u < U; ++u) sl[u] = slot ? slot[min(j0 + g * jstep + u * step, nkeys - 1)] : 0;
  for (int jb = j0 + g * jstep; jb < nkeys; jb += U * step) {
    float kv[U][8], vv[U][8];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = min(jb + u * step, nkeys - 1);   // past the end: a repeated row, not used
      const long at = (long)sl[u] * slot_stride + (long)j * stride + c * 8;
      Vec8<T>::load(K + at, kv[u]);
      Vec8<T>::load(V + at, vv[u]);
    }
    if (slot) {
#pragma unroll
      for (int u = 0; u < U; ++u) sl[u] = slot[min(jb + (U + u) * step, nkeys - 1)];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (jb + u * step < nkeys) {
#pragma unroll
        for (int n = 0; n < NQ; ++n) {
          float s = 0.f;
#pragma unroll
          for (int i = 0; i < 8; ++i) s += q[n][i] * kv[u][i];
          s = group_sum<LPK>(s) * scale;   // the lanes of a group are active together
          float mn = fmaxf(m[n], s);
          float corr = __expf(m[n] - mn);   // m = -inf on the first key: exp(-inf) = 0
          float p = __expf(s - mn);
          l[n] = l[n] * corr + p;
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[n][i] = acc[n][i] * corr + p * vv[u][i];
          m[n] = mn;
        }
      }
    }
  }
  // merge the KPI lane groups (butterfly: every group ends with the total)
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    for_lane_bits<LPK>([&](auto bit) {
      constexpr int O = decltype(bit)::value;
      float m2 = lane_xor<O>(m[n]);
      float l2 = lane_xor<O>(l[n]);
      float mn = fmaxf(m[n], m2);
      float c1 = (m[n] == -INFINITY) ? 0.f : __expf(m[n] - mn);
      float c2 = (m2 == -INFINITY) ? 0.f : __expf(m2 - mn);
      l[n] = l[n] * c1 + l2 * c2;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float a2 = lane_xor<O>(acc[n][i]);
        acc[n][i] = acc[n][i] * c1 + a2 * c2;
      }
      m[n] = mn;
    });
  }
}

template <typename T, int DH, int NQ>
__device__ __forceinline__ void attend(const T* const (&qp)[NQ], const T* __restrict__ K,
                                       const T* __restrict__ V, long stride, int nkeys, float scale,
                                       T* const (&op)[NQ], int lane, const int32_t* __restrict__ slot = nullptr,
                                       long slot_stride = 0) {
  constexpr int LPK = DH / 8;
  float m[NQ], l[NQ], acc[NQ][8];
  attend_partial<T, DH, NQ>(qp, K, V, stride, nkeys, scale, 0, 1, lane, m, l, acc, slot, slot_stride);
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
// anc == nullptr: the history of row r is slab r.  Otherwise (cache refreshing without moving the
// cache, paper sec. 3.2 turned around): position j of row r's history lives in slab
// (r / beam) * beam + anc[r * anc_ld + j], the slab of the hypothesis that wrote it.
template <typename T, int DH>
__global__ void __launch_bounds__(256) self_attention_kernel(const T* __restrict__ q, const T* __restrict__ Kc,
                                                             const T* __restrict__ Vc, T* __restrict__ out,
                                                             int rows, int H, int d, int T_, int nkeys_base,
                                                             const int32_t* __restrict__ tp, float scale,
                                                             const int32_t* __restrict__ anc, int beam, int anc_ld) {
  int w = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (w >= rows * H) return;
  const int nkeys = nkeys_base + (tp ? *tp : 0);
  int r = w / H, h = w % H;
  if (anc) {
    // the beams of a sentence mostly read the same slabs (shared ancestors): put them, for one
    // head, into neighbouring wavefronts of one workgroup so that those rows are fetched once
    const int bm = w % beam, rest = w / beam;
    h = rest % H;
    r = (rest / H) * beam + bm;
  }
  const T* qp[1] = {q + (size_t)r * d + h * DH};
  T* op[1] = {out + (size_t)r * d + h * DH};
  const int home = anc ? r - r % beam : r;
  size_t base = (size_t)home * T_ * d + h * DH;
  attend<T, DH, 1>(qp, Kc + base, Vc + base, d, nkeys, scale, op, threadIdx.x & 63,
                   anc ? anc + (size_t)r * anc_ld : nullptr, (long)T_ * d);
}

// The same for few rows (rows * heads too small to fill the chip with one wavefront each): one
// workgroup per (row, head), its four wavefronts take every fourth cached position and their
// partial (max, sum, accumulator) are merged through LDS, so a cache of n positions costs
// n / 128 round trips to memory per wavefront instead of n / 32.
template <typename T, int DH>
__global__ void __launch_bounds__(256) self_attention_split_kernel(const T* __restrict__ q,
                                                                   const T* __restrict__ Kc,
                                                                   const T* __restrict__ Vc, T* __restrict__ out,
                                                                   int rows, int H, int d, int T_, int nkeys_base,
                                                                   const int32_t* __restrict__ tp, float scale,
                                                                   const int32_t* __restrict__ anc, int beam,
                                                                   int anc_ld) {
  constexpr int LPK = DH / 8;
  __shared__ float part[4][LPK][10];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nkeys = nkeys_base + (tp ? *tp : 0);
  const int r = blockIdx.x / H, h = blockIdx.x % H;
  const T* qp[1] = {q + (size_t)r * d + h * DH};
  const int home = anc ? r - r % beam : r;
  const size_t base = (size_t)home * T_ * d + h * DH;
  float m[1], l[1], acc[1][8];
  attend_partial<T, DH, 1>(qp, Kc + base, Vc + base, d, nkeys, scale, wave, 4, lane, m, l, acc,
                           anc ? anc + (size_t)r * anc_ld : nullptr, (long)T_ * d);
  if (lane < LPK) {
    part[wave][lane][0] = m[0];
    part[wave][lane][1] = l[0];
#pragma unroll
    for (int i = 0; i < 8; ++i) part[wave][lane][2 + i] = acc[0][i];
  }
  __syncthreads();
  if (wave == 0 && lane < LPK) {
    float mx = fmaxf(fmaxf(part[0][lane][0], part[1][lane][0]), fmaxf(part[2][lane][0], part[3][lane][0]));
    float sum = 0.f, o8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float mw = part[w][lane][0];
      const float c = (mw == -INFINITY) ? 0.f : __expf(mw - mx);   // a wavefront that saw no key
      sum += part[w][lane][1] * c;
#pragma unroll
      for (int i = 0; i < 8; ++i) o8[i] += part[w][lane][2 + i] * c;
    }
    const float inv = 1.0f / sum;
#pragma unroll
    for (int i = 0; i < 8; ++i) o8[i] *= inv;
    Vec8<T>::store(out + (size_t)r * d + h * DH + lane * 8, o8);
  }
}

// Cross-attention: the NQ beams of one sentence share every key/value load.  kv rows are [K | V].
// One wavefront per (sentence, head): no LDS, no barrier.  Source sentences are short (tens of
// keys), so the work is organised to keep the fixed cost small rather than to stream.  Lane = (key
// slot, 8-element chunk): DH/8 lanes share a key, 64/(DH/8) keys per pass.  A lane requests the key
// and the value chunks of its keys of G passes at once (32 keys at head size 64: one round trip
// for the usual sentence), dots the key chunks with the NQ query chunks (summed over the chunk
// lanes by shuffles) and updates a running maximum, a running sum and an unnormalised weighted
// value sum per query (the usual streaming softmax); the key slots add theirs up by shuffles at
// the end.  Measured against a workgroup per (sentence, head) with the scores in LDS (two barriers,
// values fetched after the softmax): 7.9 instead of 13.3 us for 128 sentences of 28 keys, 17.8
// instead of 26.7 us at 128 keys; more passes in flight per wavefront were slower, not faster.
template <typename T, int DH, int NQ, bool SPLIT>
__global__ void __launch_bounds__(256) cross_attention_kernel(const T* __restrict__ q, const T* __restrict__ kv,
                                                              const int32_t* __restrict__ off,
                                                              const int32_t* __restrict__ len,
                                                              T* __restrict__ out, int batch, int beam,
                                                              int first, int H, int d, float scale) {
  using raw_t = typename Vec8<T>::raw_t;
  constexpr int LPK = DH / 8;        // lanes per key
  constexpr int KPW = 64 / LPK;      // keys per pass
  constexpr int G = 4;               // passes per round trip
  constexpr int NW = SPLIT ? 4 : 1;  // wavefronts that share a (sentence, head)
  __shared__ float part[SPLIT ? 4 : 1][NQ][DH + 2];   // SPLIT: per wavefront and query the sums, then max and sum
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int w = SPLIT ? blockIdx.x : blockIdx.x * 4 + wave;
  if (w >= batch * H) return;
  const int b = w / H, h = w % H;
  const int n_keys = len[b];
  const int c = lane % LPK, slot = lane / LPK;
  const T* K = kv + (size_t)off[b] * 2 * d + h * DH + c * 8;
  const T* V = K + d;
  const long stride = 2 * d;
  float qv[NQ][8];
#pragma unroll
  for (int n = 0; n < NQ; ++n) Vec8<T>::load(q + ((size_t)b * beam + first + n) * d + h * DH + c * 8, qv[n]);
  float m[NQ], l[NQ], acc[NQ][8];
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    m[n] = -INFINITY;
    l[n] = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[n][i] = 0.f;
  }
  for (int j0 = SPLIT ? wave * G * KPW : 0; j0 < n_keys; j0 += NW * G * KPW) {
    raw_t kk[G], vv[G];
#pragma unroll
    for (int u = 0; u < G; ++u) {
      const int j = min(j0 + u * KPW + slot, n_keys - 1);
      kk[u] = Vec8<T>::load_raw(K + (long)j * stride);
      vv[u] = Vec8<T>::load_raw(V + (long)j * stride);
    }
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
      float sc[G], mx = m[n];
#pragma unroll
      for (int u = 0; u < G; ++u) {
        float kf[8], sdot = 0.f;
        Vec8<T>::unpack(kk[u], kf);
#pragma unroll
        for (int i = 0; i < 8; ++i) sdot += qv[n][i] * kf[i];
        sdot = group_sum<LPK>(sdot);
        sc[u] = (j0 + u * KPW + slot < n_keys) ? sdot * scale : -INFINITY;
        mx = fmaxf(mx, sc[u]);
      }
      for_lane_bits<LPK>([&](auto bit) { mx = max_lane_xor<decltype(bit)::value>(mx); });   // over the key slots
      // mx is finite: key j0 exists
      const float corr = __expf(m[n] - mx);   // 0 the first time (m = -inf)
      m[n] = mx;
      l[n] *= corr;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[n][i] *= corr;
#pragma unroll
      for (int u = 0; u < G; ++u) {
        float vf[8];
        Vec8<T>::unpack(vv[u], vf);
        const float pj = __expf(sc[u] - mx);   // masked keys: exp(-inf) = 0
        l[n] += pj;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[n][i] += pj * vf[i];
      }
    }
  }
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    for_lane_bits<LPK>([&](auto bit) {
      constexpr int O = decltype(bit)::value;
      l[n] = add_lane_xor<O>(l[n]);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[n][i] = add_lane_xor<O>(acc[n][i]);
    });
    if (slot == 0) {
      if constexpr (SPLIT) {
#pragma unroll
        for (int i = 0; i < 8; ++i) part[wave][n][c * 8 + i] = acc[n][i];
        if (c == 0) { part[wave][n][DH] = m[n]; part[wave][n][DH + 1] = l[n]; }
      } else {
        const float r = 1.0f / l[n];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[n][i] *= r;
        Vec8<T>::store(out + ((size_t)b * beam + first + n) * d + h * DH + c * 8, acc[n]);
      }
    }
  }
  if constexpr (SPLIT) {
    __syncthreads();   // every wavefront of the workgroup gets here: none left early
    // wavefront n (and n + 4, ...) finishes query n; a wavefront that had no keys left m = -inf, l = 0
    for (int n = wave; n < NQ; n += 4) {
      float mx = -INFINITY;
#pragma unroll
      for (int w2 = 0; w2 < 4; ++w2) mx = fmaxf(mx, part[w2][n][DH]);
      float sum = 0.f;
#pragma unroll
      for (int w2 = 0; w2 < 4; ++w2) sum += part[w2][n][DH + 1] * __expf(part[w2][n][DH] - mx);
      for (int x = lane; x < DH; x += 64) {
        float v = 0.f;
#pragma unroll
        for (int w2 = 0; w2 < 4; ++w2) v += part[w2][n][x] * __expf(part[w2][n][DH] - mx);
        out[((size_t)b * beam + first + n) * d + h * DH + x] = (T)(v / sum);
      }
    }
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
                                                                int causal, float scale) {
  int w = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (w >= rows * H) return;
  int r = w / H, h = w % H;
  int b = row_sent[r];
  // causal (decoder-only prefill): row r sits at position r - off[b] and sees keys up to itself
  const int nk = causal ? r - off[b] + 1 : len[b];
  const T* qp[1] = {qkv + (size_t)r * 3 * d + h * DH};
  T* op[1] = {out + (size_t)r * d + h * DH};
  const T* K = qkv + (size_t)off[b] * 3 * d + d + h * DH;
  attend<T, DH, 1>(qp, K, K + d, 3 * d, nk, scale, op, threadIdx.x & 63);
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

// up to this many (row, head) pairs a workgroup, not a wavefront, takes each pair
constexpr int kSplitAttentionUnits = 2048;

template <typename T>
static hipError_t self_t(const T* q, const T* Kc, const T* Vc, T* out, int rows, int H, int d, int T_,
                         int nkeys, const int32_t* tp, const int32_t* anc, int beam, int anc_ld, hipStream_t s) {
  int dh = d / H;
  float scale = 1.0f / sqrtf((float)dh);
  dim3 b(256);
  if (rows * H <= kSplitAttentionUnits) {
    dim3 g(rows * H);
    LSQ_DISPATCH_DH(dh, (self_attention_split_kernel<T, DH><<<g, b, 0, s>>>(q, Kc, Vc, out, rows, H, d, T_, nkeys, tp, scale, anc, beam, anc_ld)));
  } else {
    dim3 g((rows * H + 3) / 4);
    LSQ_DISPATCH_DH(dh, (self_attention_kernel<T, DH><<<g, b, 0, s>>>(q, Kc, Vc, out, rows, H, d, T_, nkeys, tp, scale, anc, beam, anc_ld)));
  }
  return hipGetLastError();
}

hipError_t launch_self_attention(int dtype, const void* q, const void* Kc, const void* Vc, void* out,
                                 int rows, int H, int d, int T, int nkeys, const int32_t* tp, const int32_t* anc,
                                 int beam, int anc_ld, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (anc && (beam < 1 || rows % beam != 0)) return hipErrorInvalidValue;
  if (dtype == DT_F16)
    return self_t<half_t>((const half_t*)q, (const half_t*)Kc, (const half_t*)Vc, (half_t*)out, rows, H, d, T, nkeys, tp, anc, beam, anc_ld, s);
  return self_t<float>((const float*)q, (const float*)Kc, (const float*)Vc, (float*)out, rows, H, d, T, nkeys, tp, anc, beam, anc_ld, s);
}

// Four wavefronts per (sentence, head) instead of one: only when the launch is small enough to
// leave most of the chip idle otherwise (few sentences alive) and the longest sentence is long
// enough for the split to pay for its barrier (measured at 16 heads of 64: 128 keys, 8 sentences:
// 6.4 against 10.2 us; 32 sentences: 8.4 against 10.5; 128 sentences: 24.9 against 18.1).
bool cross_attention_splits(int units, int longest) { return units <= 512 && longest > 48; }

template <typename T, int NQ>
static hipError_t cross_nq(const T* q, const T* kv, const int32_t* off, const int32_t* len, T* out,
                           int batch, int beam, int first, int H, int d, int smax, hipStream_t s) {
  int dh = d / H;
  float scale = 1.0f / sqrtf((float)dh);
  if (cross_attention_splits(batch * H, smax)) {
    dim3 g(batch * H), b(256);
    LSQ_DISPATCH_DH(dh, (cross_attention_kernel<T, DH, NQ, true><<<g, b, 0, s>>>(q, kv, off, len, out, batch, beam, first, H, d, scale)));
    return hipGetLastError();
  }
  dim3 g((batch * H + 3) / 4), b(256);
  LSQ_DISPATCH_DH(dh, (cross_attention_kernel<T, DH, NQ, false><<<g, b, 0, s>>>(q, kv, off, len, out, batch, beam, first, H, d, scale)));
  return hipGetLastError();
}

template <typename T>
static hipError_t cross_t(const T* q, const T* kv, const int32_t* off, const int32_t* len, T* out, int batch,
                          int beam, int H, int d, int smax, hipStream_t s) {
  // beams are handled in groups of 4, 2 or 1 queries per wavefront
  int first = 0;
  while (first < beam) {
    int left = beam - first;
    hipError_t e;
    if (left >= 4) { e = cross_nq<T, 4>(q, kv, off, len, out, batch, beam, first, H, d, smax, s); first += 4; }
    else if (left >= 2) { e = cross_nq<T, 2>(q, kv, off, len, out, batch, beam, first, H, d, smax, s); first += 2; }
    else { e = cross_nq<T, 1>(q, kv, off, len, out, batch, beam, first, H, d, smax, s); first += 1; }
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_cross_attention(int dtype, const void* q, const void* kv, const int32_t* off,
                                  const int32_t* len, void* out, int batch, int beam, int H, int d, int smax,
                                  hipStream_t s) {
  if (batch <= 0) return hipSuccess;
  if (smax < 1) return hipErrorInvalidValue;
  if (dtype == DT_F16)
    return cross_t<half_t>((const half_t*)q, (const half_t*)kv, off, len, (half_t*)out, batch, beam, H, d, smax, s);
  return cross_t<float>((const float*)q, (const float*)kv, off, len, (float*)out, batch, beam, H, d, smax, s);
}

template <typename T>
static hipError_t enc_t(const T* qkv, const int32_t* row_sent, const int32_t* off, const int32_t* len, T* out,
                        int rows, int H, int d, int causal, hipStream_t s) {
  int dh = d / H;
  float scale = 1.0f / sqrtf((float)dh);
  dim3 g((rows * H + 3) / 4), b(256);
  LSQ_DISPATCH_DH(dh, (encoder_attention_kernel<T, DH><<<g, b, 0, s>>>(qkv, row_sent, off, len, out, rows, H, d, causal, scale)));
  return hipGetLastError();
}

hipError_t launch_encoder_attention(int dtype, const void* qkv, const int32_t* row_sent, const int32_t* off,
                                    const int32_t* len, void* out, int rows, int H, int d, int causal,
                                    hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (dtype == DT_F16)
    return enc_t<half_t>((const half_t*)qkv, row_sent, off, len, (half_t*)out, rows, H, d, causal, s);
  return enc_t<float>((const float*)qkv, row_sent, off, len, (float*)out, rows, H, d, causal, s);
}

}  // namespace lsq
