// Scaled, masked softmax over keys fused with the value sum (paper sec. 2.1 fusion rule applied
// to attention): one wavefront per (key/value stream, head).  HBM-bound: every key and value is
// read exactly once per wavefront, 16 bytes per lane.
//
// Lane layout: a head row of DH elements is split over LPK = DH/8 lanes (8 elements each), so a
// wavefront covers KPI = 64/LPK keys per iteration.  Each lane group runs its own online softmax
// (running max, running sum, running value accumulator) over the keys it sees; the groups are
// merged across lanes at the end.  Masking is by key count: what lies beyond it never reaches a sum.
#include "lsq_internal.h"

namespace lsq {

// Keys j0, j0 + jstep, j0 + 2*jstep, ... (< nkeys) are visited, each lane group taking every
// KPI-th of them.  On return every lane holds, for its 8 elements of the head row, the merged
// (running max m, in units of log 2: the sums are of 2^(score - m); running sum l; un-normalised
// accumulator acc) of all keys this wavefront saw.
// TABLE: position j is not in this row's own slab but in slab slot[j] of its sentence
// (K + slot[j] * slot_stride, slot numbers 0..slot_max).
//
// Trips to memory are what this costs at decoding sizes, so as few as possible depend on each
// other.  nkeys usually comes from a counter in memory: nothing that forms an address uses it
// before the first keys and values have been requested.  That first request is speculative: it
// reads positions up to jcap (the last one that exists in memory, nkeys - 1 <= jcap) and slot
// numbers forced into 0..slot_max, so whatever the table and the cache hold beyond nkeys the
// addresses stay inside them; what was read from beyond nkeys is discarded by selection (not by a
// zero weight: it may be anything) once nkeys has arrived.  After that each trip's rows, and the
// slot numbers of the trip after it, are requested before the current trip is worked on.
template <typename T, int DH, int NQ, bool TABLE = false>
__device__ __forceinline__ void attend_partial(const T* const (&qp)[NQ], const T* __restrict__ K,
                                               const T* __restrict__ V, int stride, int nkeys, int jcap,
                                               float scale, int j0, int jstep, int lane, float (&m)[NQ],
                                               float (&l)[NQ], float (&acc)[NQ][8],
                                               const int32_t* __restrict__ slot = nullptr, int slot_stride = 0,
                                               int slot_max = 0) {
  using raw_t = typename Vec8<T>::raw_t;
  constexpr int LPK = DH / 8;
  constexpr int KPI = 64 / LPK;
  constexpr int U = 4;   // keys per lane group and trip
  const int g = lane / LPK, c = lane % LPK;
  const int step = KPI * jstep;
  const int jfirst = j0 + g * jstep;
  int sl[U];
  raw_t kn[U], vn[U];   // the trip that is on its way
  auto request_slots = [&](int jb, int last) {
#pragma unroll
    for (int u = 0; u < U; ++u) sl[u] = TABLE ? slot[min(jb + u * step, last)] : 0;   // as stored: forced into range when used
  };
  auto request = [&](int jb, int last) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      // K, V and the strides are the same in every lane (the caller's part of the address sits in
      // scalar registers); a lane's own part fits 32 bits: an element offset inside one sentence's slabs
      // (in bytes, so that the instruction takes it as it is next to the scalar base)
      const unsigned at = ((TABLE ? min(max(sl[u], 0), slot_max) * slot_stride : 0) + min(jb + u * step, last) * stride + c * 8) *
                          (unsigned)sizeof(T);
      kn[u] = Vec8<T>::load_raw(reinterpret_cast<const T*>(reinterpret_cast<const char*>(K) + at));
      vn[u] = Vec8<T>::load_raw(reinterpret_cast<const T*>(reinterpret_cast<const char*>(V) + at));
    }
  };
  jcap = max(jcap, 0);   // position 0 exists whenever the kernel runs
  request_slots(jfirst, jcap);
  raw_t qr[NQ];
#pragma unroll
  for (int n = 0; n < NQ; ++n) qr[n] = Vec8<T>::load_raw(qp[n] + c * 8);
  request(jfirst, jcap);
  request_slots(jfirst + U * step, jcap);
  // scores are kept in units of log 2 (multiplied by scale * log2 e), so every exponential below is
  // the bare hardware instruction
  const float qscale = scale * 1.44269504088896340736f;
  float q[NQ][8];
#pragma unroll
  for (int n = 0; n < NQ; ++n) Vec8<T>::unpack(qr[n], q[n]);
  float kv[U][8], vv[U][8];
  auto scores = [&](int jb, int n, float (&sc)[U]) {   // of query n against the U keys in kv; -inf beyond nkeys
    float mx = -INFINITY;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) s += q[n][i] * kv[u][i];
      s = group_sum<LPK>(s) * qscale;   // the lanes of a group are active together
      sc[u] = (jb + u * step < nkeys) ? s : -INFINITY;
      mx = fmaxf(mx, sc[u]);
    }
    return mx;
  };
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    m[n] = -INFINITY;
    l[n] = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[n][i] = 0.f;
  }
  // The loop body runs at least once, whether or not this lane group has a key at all (a test of
  // nkeys in front of it would draw the requests above down behind the test): in the first trip
  // nkeys only selects.  The U scores of a trip share one update of the running maximum (one
  // rescaling of the sums per U keys, not per key).
  int jb = jfirst;
  bool speculative = true;
  do {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      Vec8<T>::unpack(kn[u], kv[u]);
      Vec8<T>::unpack(vn[u], vv[u]);
    }
    if (speculative) {
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (jb + u * step >= nkeys) {   // read from beyond the end: may be anything, and 0 * anything is not 0
#pragma unroll
          for (int i = 0; i < 8; ++i) vv[u][i] = 0.f;
        }
    }
    // from here on no position beyond nkeys - 1 is read: a lane past the end repeats the last row, weighted 0
    const int jn = jb + U * step;
    if (jn < nkeys) {   // requested before this trip's arithmetic
      request(jn, nkeys - 1);
      request_slots(jn + U * step, nkeys - 1);
    }
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
      float sc[U];
      const float mn = fmaxf(m[n], scores(jb, n, sc));   // -inf: no key for this group so far
      const float corr = m[n] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m[n] - mn);
      m[n] = mn;
      l[n] *= corr;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[n][i] *= corr;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float p = sc[u] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(sc[u] - mn);
        l[n] += p;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[n][i] += p * vv[u][i];
      }
    }
    jb = jn;
    speculative = false;
  } while (jb < nkeys);
  // merge the KPI lane groups: every group rescales its sums to the maximum over all groups once,
  // then the sums are added (every group ends with the totals)
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    float mx = m[n];
    for_lane_bits<LPK>([&](auto bit) { mx = max_lane_xor<decltype(bit)::value>(mx); });
    const float c1 = (m[n] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m[n] - mx);   // a group that saw no key
    m[n] = mx;
    l[n] *= c1;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[n][i] *= c1;
    for_lane_bits<LPK>([&](auto bit) {
      constexpr int O = decltype(bit)::value;
      l[n] = add_lane_xor<O>(l[n]);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[n][i] = add_lane_xor<O>(acc[n][i]);
    });
  }
}

template <typename T, int DH, int NQ, bool TABLE = false>
__device__ __forceinline__ void attend(const T* const (&qp)[NQ], const T* __restrict__ K,
                                       const T* __restrict__ V, int stride, int nkeys, int jcap, float scale,
                                       T* const (&op)[NQ], int lane,
                                       const int32_t* __restrict__ slot = nullptr, int slot_stride = 0,
                                       int slot_max = 0) {
  constexpr int LPK = DH / 8;
  float m[NQ], l[NQ], acc[NQ][8];
  attend_partial<T, DH, NQ, TABLE>(qp, K, V, stride, nkeys, jcap, scale, 0, 1, lane, m, l, acc, slot, slot_stride, slot_max);
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
// Argument order (here and in the kernels below): what the first addresses are formed from comes
// first, so that it is among the arguments that arrive in registers with the wavefront; the step
// counter and the output pointer, needed later, may take a trip of their own.
template <typename T, int DH, bool TABLE>
__global__ void __launch_bounds__(256) self_attention_kernel(const T* __restrict__ q, const T* __restrict__ Kc,
                                                             const T* __restrict__ Vc,
                                                             const int32_t* __restrict__ anc,
                                                             const int32_t* __restrict__ tp, int H_beam, int d,
                                                             int T_, int rows, int nkeys_base, T* __restrict__ out) {
  const int H = H_beam & 0xffff, beam = H_beam >> 16;
  constexpr float scale = DH == 16 ? 0.25f : DH == 32 ? 0.17677669529663688f : DH == 64 ? 0.125f : 0.08838834764831845f;
  const int anc_ld = T_ + 1;
  // the wavefront's number is the same in all of its lanes: said so, the row, the head and the
  // bases below are computed once, in scalar registers
  const int w = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (threadIdx.x >> 6));
  if (w >= rows * H) return;
  const int nkeys = nkeys_base + (tp ? *tp : 0);
  int r = w / H, h = w % H;
  if constexpr (TABLE) {
    // the beams of a sentence mostly read the same slabs (shared ancestors): put them, for one
    // head, into neighbouring wavefronts of one workgroup so that those rows are fetched once
    const int bm = w % beam, rest = w / beam;
    h = rest % H;
    r = (rest / H) * beam + bm;
  }
  const T* qp[1] = {q + (size_t)r * d + h * DH};
  T* op[1] = {out + (size_t)r * d + h * DH};
  const int home = TABLE ? r - r % beam : r;
  size_t base = (size_t)home * T_ * d + h * DH;
  attend<T, DH, 1, TABLE>(qp, Kc + base, Vc + base, d, nkeys, T_ - 1, scale, op, threadIdx.x & 63,
                          anc + (size_t)r * anc_ld, T_ * d, beam - 1);
}

// The same for few rows (rows * heads too small to fill the chip with one wavefront each): one
// workgroup per (row, head), its four wavefronts take every fourth cached position and their
// partial (max, sum, accumulator) are merged through LDS, so a cache of n positions costs
// n / 128 round trips to memory per wavefront instead of n / 32.
template <typename T, int DH, bool TABLE>
__global__ void __launch_bounds__(256) self_attention_split_kernel(const T* __restrict__ q,
                                                                   const T* __restrict__ Kc,
                                                                   const T* __restrict__ Vc,
                                                                   const int32_t* __restrict__ anc,
                                                                   const int32_t* __restrict__ tp, int H_beam,
                                                                   int d, int T_, int rows, int nkeys_base,
                                                                   T* __restrict__ out) {
  const int H = H_beam & 0xffff, beam = H_beam >> 16;
  constexpr float scale = DH == 16 ? 0.25f : DH == 32 ? 0.17677669529663688f : DH == 64 ? 0.125f : 0.08838834764831845f;
  const int anc_ld = T_ + 1;
  constexpr int LPK = DH / 8;
  __shared__ float part[4][LPK][10];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nkeys = nkeys_base + (tp ? *tp : 0);
  const int r = blockIdx.x / H, h = blockIdx.x % H;
  const T* qp[1] = {q + (size_t)r * d + h * DH};
  const int home = TABLE ? r - r % beam : r;
  const size_t base = (size_t)home * T_ * d + h * DH;
  float m[1], l[1], acc[1][8];
  attend_partial<T, DH, 1, TABLE>(qp, Kc + base, Vc + base, d, nkeys, T_ - 1, scale, wave, 4, lane, m, l, acc,
                                  anc + (size_t)r * anc_ld, T_ * d, beam - 1);
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
      const float c = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - mx);   // a wavefront that saw no key; m is in units of log 2
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

// The key stream of cross-attention, shared by the two kernels below.  A wavefront's lanes are
// (key slot, 8-element chunk): DH/8 lanes share a key, KPW = 64/(DH/8) keys per pass, G passes per
// trip to memory.  K and V are the sentence's first key and value row of this head (the same in
// every lane: scalar registers), a lane adds 32-bit byte offsets.
template <typename T, int DH, int NQ>
struct CrossKeys {
  static constexpr int LPK = DH / 8, KPW = 64 / LPK, G = 4;
  using raw_t = typename Vec8<T>::raw_t;
  const char* K;
  const char* V;
  unsigned stride, lane_at;
  int n_keys, slot;
  raw_t kn[G], vn[G];   // the trip that is on its way

  __device__ __forceinline__ void request(int j0) {
#pragma unroll
    for (int u = 0; u < G; ++u) {
      const unsigned at = (unsigned)min(j0 + u * KPW + slot, n_keys - 1) * stride + lane_at;
      kn[u] = Vec8<T>::load_raw(reinterpret_cast<const T*>(K + at));
      vn[u] = Vec8<T>::load_raw(reinterpret_cast<const T*>(V + at));
    }
  }

  // Trips j0 = jfirst, jfirst + jstep, ... < n_keys; the first one has been requested by the
  // caller (if jfirst < n_keys), each later one is requested before the one before it is worked
  // on.  Streaming softmax per query in units of log 2 (qscale = scale * log2 e): running maximum
  // m, sum l of 2^(score - m), weighted value sum acc; on return the key slots have been added up.
  __device__ __forceinline__ void run(const float (&qv)[NQ][8], float qscale, int jfirst, int jstep, float (&m)[NQ],
                                      float (&l)[NQ], float (&acc)[NQ][8]) {
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
      m[n] = -INFINITY;
      l[n] = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[n][i] = 0.f;
    }
    for (int j0 = jfirst; j0 < n_keys; j0 += jstep) {
      raw_t kk[G], vv[G];
#pragma unroll
      for (int u = 0; u < G; ++u) { kk[u] = kn[u]; vv[u] = vn[u]; }
      if (j0 + jstep < n_keys) request(j0 + jstep);   // travels while this trip is worked on
      asm volatile("" ::: "memory");
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
          sc[u] = (j0 + u * KPW + slot < n_keys) ? sdot * qscale : -INFINITY;
          mx = fmaxf(mx, sc[u]);
        }
        for_lane_bits<LPK>([&](auto bit) { mx = max_lane_xor<decltype(bit)::value>(mx); });   // over the key slots
        // mx is finite: key j0 exists
        const float corr = __builtin_amdgcn_exp2f(m[n] - mx);   // 0 the first time (m = -inf)
        m[n] = mx;
        l[n] *= corr;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[n][i] *= corr;
#pragma unroll
        for (int u = 0; u < G; ++u) {
          float vf[8];
          Vec8<T>::unpack(vv[u], vf);
          const float pj = __builtin_amdgcn_exp2f(sc[u] - mx);   // masked keys: 2^-inf = 0
          l[n] += pj;
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[n][i] += pj * vf[i];
        }
      }
    }
#pragma unroll
    for (int n = 0; n < NQ; ++n)
      for_lane_bits<LPK>([&](auto bit) {
        constexpr int O = decltype(bit)::value;
        l[n] = add_lane_xor<O>(l[n]);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[n][i] = add_lane_xor<O>(acc[n][i]);
      });
  }
};

// Four wavefronts shared a (sentence, head): each leaves its sums, maximum and total in LDS
// (`deposit`, wavefronts 0..3), and after the workgroup's barrier wavefront n finishes query n
// (`finish`): a wavefront that had no keys left m = -inf, l = 0.  out_row0: row of query 0.
template <int DH, int NQ>
__device__ __forceinline__ void cross_deposit(float (&part)[4][NQ][DH + 2], int wave, int lane, const float (&m)[NQ],
                                              const float (&l)[NQ], const float (&acc)[NQ][8]) {
  constexpr int LPK = DH / 8;
  const int c = lane % LPK;
  if (lane / LPK != 0) return;
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
#pragma unroll
    for (int i = 0; i < 8; ++i) part[wave][n][c * 8 + i] = acc[n][i];
    if (c == 0) { part[wave][n][DH] = m[n]; part[wave][n][DH + 1] = l[n]; }
  }
}
template <typename T, int DH, int NQ>
__device__ __forceinline__ void cross_finish(const float (&part)[4][NQ][DH + 2], int wave, int lane, T* __restrict__ out_row0,
                                             int d) {
  for (int n = wave; n < NQ; n += 4) {
    float mx = -INFINITY;
#pragma unroll
    for (int w2 = 0; w2 < 4; ++w2) mx = fmaxf(mx, part[w2][n][DH]);
    float sum = 0.f;
#pragma unroll
    for (int w2 = 0; w2 < 4; ++w2) sum += part[w2][n][DH + 1] * __builtin_amdgcn_exp2f(part[w2][n][DH] - mx);
    for (int x = lane; x < DH; x += 64) {
      float v = 0.f;
#pragma unroll
      for (int w2 = 0; w2 < 4; ++w2) v += part[w2][n][x] * __builtin_amdgcn_exp2f(part[w2][n][DH] - mx);
      out_row0[(size_t)n * d + x] = (T)(v / sum);
    }
  }
}

// Cross-attention: the NQ beams of one sentence share every key/value load.  kv rows are [K | V].
// One wavefront per (sentence, head): no LDS, no barrier.  Source sentences are short (tens of
// keys), so the work is organised to keep the fixed cost small rather than to stream.  Lane = (key
// slot, 8-element chunk): DH/8 lanes share a key, 64/(DH/8) keys per pass.  A lane requests the key
// and the value chunks of its keys of G passes at once (32 keys at head size 64: one round trip
// for the usual sentence), dots the key chunks with the NQ query chunks (summed over the chunk
// lanes) and updates a running maximum, a running sum and an unnormalised weighted
// value sum per query (the usual streaming softmax); the key slots add theirs up across lanes at
// the end.  Measured against a workgroup per (sentence, head) with the scores in LDS (two barriers,
// values fetched after the softmax): 7.9 instead of 13.3 us for 128 sentences of 28 keys, 17.8
// instead of 26.7 us at 128 keys; more passes in flight per wavefront were slower, not faster.
template <typename T, int DH, int NQ, bool SPLIT>
__global__ void __launch_bounds__(256) cross_attention_kernel(const T* __restrict__ q, const T* __restrict__ kv,
                                                              const int32_t* __restrict__ off,
                                                              const int32_t* __restrict__ len, int batch, int beam,
                                                              int first, int H, int d, T* __restrict__ out) {
  constexpr float scale = DH == 16 ? 0.25f : DH == 32 ? 0.17677669529663688f : DH == 64 ? 0.125f : 0.08838834764831845f;
  using raw_t = typename Vec8<T>::raw_t;
  constexpr int LPK = DH / 8;        // lanes per key
  constexpr int KPW = 64 / LPK;      // keys per pass
  constexpr int G = 4;               // passes per round trip
  constexpr int NW = SPLIT ? 4 : 1;  // wavefronts that share a (sentence, head)
  __shared__ float part[SPLIT ? 4 : 1][NQ][DH + 2];   // SPLIT: per wavefront and query the sums, then max and sum
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  // one (sentence, head) per wavefront: its number, and with it the sentence's length, first row
  // and the bases below, live in scalar registers
  const int w = SPLIT ? blockIdx.x : __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + wave);
  if (w >= batch * H) return;
  const int b = w / H, h = w % H;
  const int c = lane % LPK, slot = lane / LPK;
  // Trips to memory before the first score: {length, first row, queries} together, then the keys
  // and values of the first G passes.  Left to itself the compiler fetches the row offset only
  // once the length has arrived (it is used in the loop, which the length may skip) and waits for
  // the queries (to convert them) before the loop requests any key; so the queries are kept as
  // they come from memory until the first keys are on their way, and length and offset are
  // awaited at one point.
  raw_t qr[NQ];
#pragma unroll
  for (int n = 0; n < NQ; ++n) qr[n] = Vec8<T>::load_raw(q + ((size_t)b * beam + first + n) * d + h * DH + c * 8);
  int n_keys = len[b], row0 = off[b];
  asm volatile("" : "+s"(n_keys), "+s"(row0));
  CrossKeys<T, DH, NQ> keys;
  keys.K = reinterpret_cast<const char*>(kv + (size_t)row0 * 2 * d + h * DH);
  keys.V = keys.K + d * sizeof(T);
  keys.stride = 2 * d * sizeof(T);
  keys.lane_at = c * 8 * sizeof(T);
  keys.n_keys = n_keys;
  keys.slot = slot;
  const int jfirst = SPLIT ? wave * G * KPW : 0;
  if (jfirst < n_keys) keys.request(jfirst);
  asm volatile("" ::: "memory");   // keeps the requests above what follows
  float qv[NQ][8];
#pragma unroll
  for (int n = 0; n < NQ; ++n) Vec8<T>::unpack(qr[n], qv[n]);
  float m[NQ], l[NQ], acc[NQ][8];
  keys.run(qv, scale * 1.44269504088896340736f, jfirst, NW * G * KPW, m, l, acc);
  T* out_row0 = out + ((size_t)b * beam + first) * d + h * DH;
  if constexpr (SPLIT) {
    cross_deposit<DH, NQ>(part, wave, lane, m, l, acc);
    __syncthreads();   // every wavefront of the workgroup gets here: none left early
    cross_finish<T, DH, NQ>(part, wave, lane, out_row0, d);
  } else if (slot == 0) {
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
      const float r = 1.0f / l[n];
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[n][i] *= r;
      Vec8<T>::store(out_row0 + (size_t)n * d + c * 8, acc[n]);
    }
  }
}

// Cross-attention that makes its own queries, for the last sentences of a batch (and small batches),
// where a step is a chain of launches that each cost their latency: the LayerNorm of the rows, their
// query product and the attention kernel become one.  One workgroup per (sentence, head):
//   1. requests its 64 x d slice of Wq (fragment order), the sentence's length and first row, then
//      its first keys and values: everything the kernel reads from memory is on its way before
//      anything is computed;
//   2. wavefront w normalises row w of the sentence's NQ rows (the arithmetic of
//      gemm_f16_skinny_ln_kernel, so the rows are the same bits) into LDS, head 0 also to x_new;
//   3. q = rows . slice^T: eight wavefronts, four per 32-column half, each taking every fourth
//      16-wide k-step of its half; partial tiles are added through LDS (in the order of the skinny
//      kernels: the queries are the same bits), bias added, rounded to float16 as the stored q of
//      the separate kernels is;
//   4. the first four wavefronts attend as cross_attention_kernel's four-wavefront variant does.
template <int NQ>
__global__ void __launch_bounds__(512) cross_attention_ln_kernel(const half_t* __restrict__ Wp,
                                                                 const half_t* __restrict__ kv,
                                                                 const int32_t* __restrict__ off,
                                                                 const int32_t* __restrict__ len, int beam, int H,
                                                                 int d, int M, LnInput ln,
                                                                 const half_t* __restrict__ bq,
                                                                 half_t* __restrict__ out) {
  constexpr int DH = 64, LPK = 8, KPW = 8, G = 4, NV = 2, UMAX = 16;
  constexpr float scale = 0.125f;
  __shared__ __attribute__((aligned(16))) half_t a_rows[NQ][1024 + 8];
  __shared__ float red[8][16][64];
  __shared__ float q_s[NQ][DH];
  __shared__ float part[4][NQ][DH + 2];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int b = blockIdx.x / H, h = blockIdx.x % H;
  const int ksteps = d / 16, per_wave = ksteps / 4;   // d is a multiple of 64
  const int fr = lane & 31, fk = (lane >> 5) * 8;
  const int cb = wave >> 2, kw = wave & 3;            // product: column half and k-share of this wavefront
  // 1. requests: this wavefront's share of the slice (16 fragments: all 128 KB of the slice are on
  // their way at once, 16 KB per wavefront), then length and first row, then the first keys
  const half_t* wp = Wp + ((size_t)(h * 2 + cb) * ksteps) * 512 + lane * 8;
  half8_t bf[UMAX];
#pragma unroll
  for (int u = 0; u < UMAX; ++u) bf[u] = *reinterpret_cast<const half8_t*>(wp + (size_t)min(kw + 4 * u, ksteps - 1) * 512);
  int n_keys = len[b], row0 = off[b];
  asm volatile("" : "+s"(n_keys), "+s"(row0));
  const int c = lane % LPK, slot = lane / LPK;
  CrossKeys<half_t, DH, NQ> keys;
  keys.K = reinterpret_cast<const char*>(kv + (size_t)row0 * 2 * d + h * DH);
  keys.V = keys.K + d * sizeof(half_t);
  keys.stride = 2 * d * sizeof(half_t);
  keys.lane_at = c * 8 * sizeof(half_t);
  keys.n_keys = n_keys;
  keys.slot = slot;
  // the first four wavefronts attend (step 4); the others have no keys
  const int jfirst = wave < 4 ? wave * G * KPW : 0x7fffffff;
  if (jfirst < n_keys) keys.request(jfirst);
  // 2. LayerNorm of row (b * beam + wave)
  if (wave < NQ) {
    const int r = b * beam + wave;
    const size_t slab = (size_t)M * d;
    float v[NV][8], gv[NV][8], bv[NV][8];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int cc = (j * 64 + lane) * 8;
      if (cc < d) {
        float t[8], prt[4][8];
#pragma unroll
        for (int sp = 0; sp < 4; ++sp)
          if (sp < ln.splits) Vec8<float>::load(ln.P + sp * slab + (size_t)r * d + cc, prt[sp]);
        Vec8<half_t>::load(ln.bias + cc, t);
        Vec8<half_t>::load(ln.x_old + (size_t)r * d + cc, v[j]);
        Vec8<half_t>::load(ln.g + cc, gv[j]);
        Vec8<half_t>::load(ln.b + cc, bv[j]);
        add_partials<4>(v[j], prt, ln.splits, t);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) { v[j][i] = 0.f; gv[j][i] = 0.f; bv[j][i] = 0.f; }
      }
    }
    float o[NV][8];
    layernorm_row<NV>(v, gv, bv, d, ln.eps, lane, o);
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int cc = (j * 64 + lane) * 8;
      if (cc < d) {
        Vec8<half_t>::store(&a_rows[wave][cc], o[j]);
        if (h == 0) Vec8<half_t>::store(ln.x_new + (size_t)r * d + cc, o[j]);
      }
    }
  }
  __syncthreads();
  // 3. the head's 64 query columns of the NQ rows (rows past NQ repeat the last one; never stored):
  // wavefront (cb, kw) multiplies every fourth k-step of column half cb
  floatx16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  const half_t* ar = &a_rows[min(fr, NQ - 1)][fk];
#pragma unroll
  for (int u = 0; u < UMAX; ++u)
    if (u < per_wave) {
      const half8_t af = *reinterpret_cast<const half8_t*>(ar + (kw + 4 * u) * 16);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[u], af, acc, 0, 0, 0);
    }
#pragma unroll
  for (int e = 0; e < 16; ++e) red[wave][e][lane] = acc[e];
  __syncthreads();
  {
    // accumulator element vg*4 + e of lane (m, half) is column vg*8 + half*4 + e of row m (the
    // layout of the skinny kernels' epilogue); wavefront (cb, vg) finishes those of its half
    const int vg = kw, m = lane & 31;
    if (m < NQ) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int rr = vg * 4 + e, n = cb * 32 + vg * 8 + (lane >> 5) * 4 + e;
        float x = (red[cb * 4 + 0][rr][lane] + red[cb * 4 + 1][rr][lane]) + (red[cb * 4 + 2][rr][lane] + red[cb * 4 + 3][rr][lane]);
        x += (float)bq[h * DH + n];
        q_s[m][n] = (float)(half_t)x;
      }
    }
  }
  __syncthreads();
  // 4. attention, four wavefronts sharing the keys
  float qv[NQ][8];
#pragma unroll
  for (int n = 0; n < NQ; ++n)
#pragma unroll
    for (int i = 0; i < 8; ++i) qv[n][i] = q_s[n][c * 8 + i];
  float mx_[NQ], l_[NQ], acc_[NQ][8];
  keys.run(qv, scale * 1.44269504088896340736f, jfirst, 4 * G * KPW, mx_, l_, acc_);
  if (wave < 4) cross_deposit<DH, NQ>(part, wave, lane, mx_, l_, acc_);
  __syncthreads();
  cross_finish<half_t, DH, NQ>(part, wave, lane, out + (size_t)b * beam * d + h * DH, d);
}

// Every (sentence, head) workgroup streams its own 64 x d slice of Wq, so the weights are read once per
// sentence: measured on whole steps against LayerNorm kernel + query product + attention kernel,
// ahead up to 64 rows (0.262 -> 0.241 ms at 32 rows of the base model, 0.456 -> 0.449 with the
// limit at 64 on the batch-32 workload of the big one), level at 128, far behind at 512.
constexpr int kCrossLnRows = 64;

bool cross_attention_ln_supported(int dtype, int rows, int beam, int H, int d) {
  return dtype == DT_F16 && rows >= 1 && rows <= kCrossLnRows && beam >= 1 && beam <= 4 && rows % beam == 0 && H >= 1 &&
         d == H * 64 && d <= 1024 && d % 64 == 0;
}

hipError_t launch_cross_attention_ln(const LnInput& ln, const void* Wq_packed, const void* bq, const void* kv,
                                     const int32_t* off, const int32_t* len, void* out, int batch, int beam,
                                     int H, int d, hipStream_t s) {
  if (batch <= 0) return hipSuccess;
  if (!cross_attention_ln_supported(DT_F16, batch * beam, beam, H, d) || !Wq_packed || !bq || ln.splits < 1 ||
      ln.splits > 4 || ln.x_old == ln.x_new)
    return hipErrorInvalidValue;
  dim3 g(batch * H), b(512);
  const int M = batch * beam;
#define LSQ_CROSS_LN(NQ_)                                                                                    \
  cross_attention_ln_kernel<NQ_><<<g, b, 0, s>>>((const half_t*)Wq_packed, (const half_t*)kv, off, len, beam, H, d, M, ln, \
                                                  (const half_t*)bq, (half_t*)out)
  switch (beam) {
    case 1: LSQ_CROSS_LN(1); break;
    case 2: LSQ_CROSS_LN(2); break;
    case 3: LSQ_CROSS_LN(3); break;
    default: LSQ_CROSS_LN(4); break;
  }
#undef LSQ_CROSS_LN
  return hipGetLastError();
}

// Cross-attention that makes its own queries from already normalised rows, for MORE than 64 rows alive
// (above, the kernel that also normalises its rows takes one sentence per workgroup): query product and
// attention in one launch instead of two.  One workgroup of eight wavefronts per (GS sentences, head):
//   1. every wavefront requests its share of the head's 64 x d slice of Wq (fragment order) and of the
//      GS * beam <= 32 rows of x, wavefront w < GS also the first keys and values of sentence w of the
//      group: everything the kernel reads is on its way before anything is computed;
//   2. q = rows . slice^T as in cross_attention_ln_kernel (four wavefronts per 32-column half, every
//      fourth 16-wide k-step each, partial tiles added through LDS, bias, rounded to float16);
//   3. wavefront w attends for sentence w of the group, as cross_attention_kernel's one-wavefront variant.
// The weights are read once per group of sentences; GS is chosen so that the launch has about as many
// workgroups as the chip has CUs.  Measured at 512 rows of the big model: query product 8.9 us + attention
// 10.3 us + the boundary between them -> one kernel.
template <int NQ>
__global__ void __launch_bounds__(512) cross_attention_q_kernel(const half_t* __restrict__ x, const half_t* __restrict__ Wp,
                                                                const half_t* __restrict__ kv,
                                                                const int32_t* __restrict__ off,
                                                                const int32_t* __restrict__ len, int batch, int GS,
                                                                int H, int d, const half_t* __restrict__ bq,
                                                                half_t* __restrict__ out) {
  constexpr int DH = 64, LPK = 8, KPW = 8, G = 4, UMAX = 16;
  constexpr float scale = 0.125f;
  __shared__ float red[8][16][64];
  __shared__ float q_s[32][DH];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int grp = blockIdx.x / H, h = blockIdx.x % H;
  const int b0 = grp * GS;
  const int M = batch * NQ;
  const int ksteps = d / 16, per_wave = ksteps / 4;   // d is a multiple of 64, at most 1024
  const int fr = lane & 31, fk = (lane >> 5) * 8;
  const int cb = wave >> 2, kw = wave & 3;
  const half_t* wp = Wp + ((size_t)(h * 2 + cb) * ksteps) * 512 + lane * 8;
  const half_t* ap = x + (size_t)min(b0 * NQ + fr, M - 1) * d + fk;   // tile row fr = row b0 * NQ + fr (past the end: the last row, never used)
  half8_t bf[UMAX], af[UMAX];
#pragma unroll
  for (int u = 0; u < UMAX; ++u) {
    const int ks = min(kw + 4 * u, ksteps - 1);
    bf[u] = *reinterpret_cast<const half8_t*>(wp + (size_t)ks * 512);
    af[u] = *reinterpret_cast<const half8_t*>(ap + ks * 16);
  }
  const int b = min(b0 + wave, batch - 1);
  const bool attends = wave < GS && b0 + wave < batch;
  int n_keys = len[b], row0 = off[b];
  const int c = lane % LPK, slot = lane / LPK;
  CrossKeys<half_t, DH, NQ> keys;
  keys.K = reinterpret_cast<const char*>(kv + (size_t)row0 * 2 * d + h * DH);
  keys.V = keys.K + d * sizeof(half_t);
  keys.stride = 2 * d * sizeof(half_t);
  keys.lane_at = c * 8 * sizeof(half_t);
  keys.n_keys = attends ? n_keys : 0;
  keys.slot = slot;
  if (attends) keys.request(0);
  asm volatile("" ::: "memory");
  floatx16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
  for (int u = 0; u < UMAX; ++u)
    if (u < per_wave) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[u], af[u], acc, 0, 0, 0);
#pragma unroll
  for (int e = 0; e < 16; ++e) red[wave][e][lane] = acc[e];
  __syncthreads();
  {
    const int vg = kw, m = lane & 31;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int rr = vg * 4 + e, n = cb * 32 + vg * 8 + (lane >> 5) * 4 + e;
      float v = (red[cb * 4 + 0][rr][lane] + red[cb * 4 + 1][rr][lane]) + (red[cb * 4 + 2][rr][lane] + red[cb * 4 + 3][rr][lane]);
      v += (float)bq[h * DH + n];
      q_s[m][n] = (float)(half_t)v;
    }
  }
  __syncthreads();
  if (!attends) return;
  float qv[NQ][8];
#pragma unroll
  for (int n = 0; n < NQ; ++n)
#pragma unroll
    for (int i = 0; i < 8; ++i) qv[n][i] = q_s[wave * NQ + n][c * 8 + i];
  float mx_[NQ], l_[NQ], acc_[NQ][8];
  keys.run(qv, scale * 1.44269504088896340736f, 0, G * KPW, mx_, l_, acc_);
  if (slot == 0) {
    half_t* out_row0 = out + (size_t)b * NQ * d + h * DH;
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
      const float r = 1.0f / l_[n];
#pragma unroll
      for (int i = 0; i < 8; ++i) acc_[n][i] *= r;
      Vec8<half_t>::store(out_row0 + (size_t)n * d + c * 8, acc_[n]);
    }
  }
}

// Measured on whole steps of the big model: 0.678 -> 0.671 ms at 512 rows, nothing at 128 (a sentence of 125 keys
// takes four dependent trips for its keys whichever kernel attends, and here they start only after the product).
// sentences per workgroup: 8 (32 rows at beam 4) once that still gives a workgroup per CU, fewer below
static int cross_q_group(int batch, int H) {
  int GS = 8;
  while (GS > 1 && (long)((batch + GS - 1) / GS) * H < 256) GS >>= 1;
  return GS;
}

// Ahead of the two separate launches from 256 rows on, and below that where its workgroups, of at least two sentences
// each, fill the CUs in one round (whole translations, 16 heads of the big model: 32 sentences = 256 workgroups
// 46.2 -> 45.4 ms, 30 and 28 sentences level, 48 sentences = 384 workgroups 51.9 -> 54.4 ms, 20 sentences level;
// 8 heads of d = 512, 32 sentences = 256 workgroups of one sentence: 34.7 -> 34.8 ms).
bool cross_attention_q_worthwhile(int batch, int beam, int H) {
  if (batch * beam >= 256) return true;
  const int GS = cross_q_group(batch, H);
  const long wgs = (long)((batch + GS - 1) / GS) * H;
  return GS >= 2 && wgs >= 240 && wgs <= 256;
}

bool cross_attention_q_supported(int dtype, int rows, int beam, int H, int d) {
  return dtype == DT_F16 && rows > kCrossLnRows && beam >= 1 && beam <= 4 && rows % beam == 0 && H >= 1 && d == H * 64 &&
         d <= 1024;
}

hipError_t launch_cross_attention_q(const void* x, const void* Wq_packed, const void* bq, const void* kv,
                                    const int32_t* off, const int32_t* len, void* out, int batch, int beam, int H,
                                    int d, hipStream_t s) {
  if (batch <= 0) return hipSuccess;
  if (!cross_attention_q_supported(DT_F16, batch * beam, beam, H, d) || !Wq_packed || !bq) return hipErrorInvalidValue;
  const int GS = cross_q_group(batch, H);
  dim3 g(((batch + GS - 1) / GS) * H), b(512);
#define LSQ_CROSS_Q(NQ_)                                                                                      \
  cross_attention_q_kernel<NQ_><<<g, b, 0, s>>>((const half_t*)x, (const half_t*)Wq_packed, (const half_t*)kv, off, len, \
                                                 batch, GS, H, d, (const half_t*)bq, (half_t*)out)
  switch (beam) {
    case 1: LSQ_CROSS_Q(1); break;
    case 2: LSQ_CROSS_Q(2); break;
    case 3: LSQ_CROSS_Q(3); break;
    default: LSQ_CROSS_Q(4); break;
  }
#undef LSQ_CROSS_Q
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Whole attention sublayers in one launch (paper sec. 2.1: fewer kernels between the products, taken
// to the point where the products themselves join in), for the last sentences of a batch and for
// small batches, where a step is a chain of launches that each cost their latency.  A workgroup owns a
// (sentence, head): it streams that head's slices of the weights itself, so nothing it needs comes
// from another workgroup of the same launch, and what it leaves is the head's share of the output
// projection as one float32 slab per head; whoever consumes the sublayer adds the H slabs, the
// projection's bias and the residual, and normalises (the next block below, or the LayerNorm kernel).

// a <- P[0] + P[1] + ... + P[S-1] at one 8-element column, slabs `slab` floats apart, added in index
// order (as add_partials does for up to 4)
template <int CH>
__device__ __forceinline__ void sum_slabs(const float* __restrict__ P, size_t slab, int S, float (&a)[8]) {
  for (int s0 = 0; s0 < S; s0 += CH) {
    float prt[CH][8];
#pragma unroll
    for (int sp = 0; sp < CH; ++sp)
      if (s0 + sp < S) Vec8<float>::load(P + (size_t)(s0 + sp) * slab, prt[sp]);
#pragma unroll
    for (int sp = 0; sp < CH; ++sp)
      if (s0 + sp < S) {
#pragma unroll
        for (int i = 0; i < 8; ++i) a[i] = (s0 + sp == 0) ? prt[sp][i] : __fadd_rn(a[i], prt[sp][i]);
      }
  }
}

// Row `r` of LayerNorm(x_old + (sum of the slabs + bias)) * g + b by one wavefront, into LDS (and to
// x_new when `keep`); ln.splits == 0: the row is x_old as it is.  d <= 1024.  CH: slabs requested together.
// ln.pre (pre-LN models): the sum x_old + (slabs + bias), rounded to float16, is what x_new receives and what is
// normalised, as in the stand-alone kernel; without slabs the row is LayerNorm(x_old) and nothing is kept.
template <int CH>
__device__ __forceinline__ void block_row(const LnInput& ln, int r, int M, int d, int lane, bool keep,
                                          half_t* __restrict__ dst) {
  constexpr int NV = 2;
  const size_t slab = (size_t)M * d;
  if (ln.splits == 0 && !ln.pre) {
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int cc = (j * 64 + lane) * 8;
      if (cc < d) *reinterpret_cast<half8_t*>(dst + cc) = *reinterpret_cast<const half8_t*>(ln.x_old + (size_t)r * d + cc);
    }
    return;
  }
  float v[NV][8], gv[NV][8], bv[NV][8];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int cc = (j * 64 + lane) * 8;
    if (cc < d) {
      float t[8], a[8];
      if (ln.splits > 0) Vec8<half_t>::load(ln.bias + cc, t);
      Vec8<half_t>::load(ln.x_old + (size_t)r * d + cc, v[j]);
      Vec8<half_t>::load(ln.g + cc, gv[j]);
      Vec8<half_t>::load(ln.b + cc, bv[j]);
      if (ln.splits > 0) {
        sum_slabs<CH>(ln.P + (size_t)r * d + cc, slab, ln.splits, a);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[j][i] = __fadd_rn(v[j][i], __fadd_rn(a[i], t[i]));
        if (ln.pre) {
#pragma unroll
          for (int i = 0; i < 8; ++i) v[j][i] = (float)(half_t)v[j][i];
          if (keep) Vec8<half_t>::store(ln.x_new + (size_t)r * d + cc, v[j]);
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) { v[j][i] = 0.f; gv[j][i] = 0.f; bv[j][i] = 0.f; }
    }
  }
  float o[NV][8];
  layernorm_row<NV>(v, gv, bv, d, ln.eps, lane, o);
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int cc = (j * 64 + lane) * 8;
    if (cc < d) {
      Vec8<half_t>::store(dst + cc, o[j]);
      if (keep && !ln.pre) Vec8<half_t>::store(ln.x_new + (size_t)r * d + cc, o[j]);
    }
  }
}

// The head's share of an output projection: P_out[h][r][:] = ctx[r, 0..63] . Wo[:, h*64 .. h*64+63]^T for
// the NQ rows in ctx_s (float16, LDS).  fo holds this wavefront's fragments of the slice: out blocks
// wave*nb + i (i < nb = d/256), k-steps h*4 + kq (kq < 4) at fo[i*4 + kq].
template <int NQ>
__device__ __forceinline__ void block_out_projection(const half8_t (&fo)[16], const half_t (&ctx_s)[NQ][64 + 8], int wave,
                                                     int lane, int nb, int h, int row0, int M, int d,
                                                     float* __restrict__ P_out) {
  const int fr = lane & 31, fk = (lane >> 5) * 8;
  const half_t* cr = &ctx_s[min(fr, NQ - 1)][fk];
  half8_t af[4];
#pragma unroll
  for (int kq = 0; kq < 4; ++kq) af[kq] = *reinterpret_cast<const half8_t*>(cr + kq * 16);
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (i < nb) {
      floatx16 acc;
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
      for (int kq = 0; kq < 4; ++kq) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(fo[i * 4 + kq], af[kq], acc, 0, 0, 0);
      if (fr < NQ) {
        float* dst = P_out + ((size_t)h * M + row0 + fr) * d + (wave * nb + i) * 32 + (lane >> 5) * 4;
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
          floatx4 o = {acc[vg * 4 + 0], acc[vg * 4 + 1], acc[vg * 4 + 2], acc[vg * 4 + 3]};
          *reinterpret_cast<floatx4*>(dst + vg * 8) = o;
        }
      }
    }
}

template <int NQ>
__device__ __forceinline__ void block_request_out_fragments(half8_t (&fo)[16], const half_t* __restrict__ Wo, int wave,
                                                            int lane, int nb, int h, int ksteps) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (i < nb) {
#pragma unroll
      for (int kq = 0; kq < 4; ++kq)
        fo[i * 4 + kq] = *reinterpret_cast<const half8_t*>(Wo + ((size_t)(wave * nb + i) * ksteps + h * 4 + kq) * 512 + lane * 8);
    }
}

// Self-attention sublayer up to the output projection's partial sums.  Workgroup (sentence b, head h),
// eight wavefronts:
//   1. requests before anything is computed: the slab numbers of each attending wavefront's first trip
//      through the history (speculatively, as attend_partial does; its keys and values follow after
//      step 2); the NQ rows' LayerNorm inputs; the first 32 k-steps of the head's 192 x d slice of
//      Wqkv (fragment order; wavefronts 0..5 each own 32 of the 192 columns over all of k);
//   2. wavefronts 6 and 7 normalise the NQ rows into LDS (head 0 also to x_new);
//   3. q, k, v of the new position: bias added, rounded to float16, kept in LDS; k and v also go to
//      position `nkeys` of the rows' slabs.  While the last fragments are multiplied the head's 64
//      k-columns of Wo are requested;
//   4. every row's history (positions 0..nkeys-1, through the slab table when there is one) is shared
//      by NSH wavefronts; the new position's key and value come from LDS; partial softmax sums are
//      merged through LDS and the context rounded to float16;
//   5. the head's share of the output projection (above).
template <int NQ, bool TABLE>
__global__ void __launch_bounds__(512) self_block_kernel(const half_t* __restrict__ Wqkv, const half_t* __restrict__ Wo,
                                                         const int32_t* __restrict__ anc,
                                                         const int32_t* __restrict__ tp, int nkeys_base, int H, int d,
                                                         int T_, int M, half_t* __restrict__ Kc,
                                                         half_t* __restrict__ Vc, const half_t* __restrict__ bqkv,
                                                         LnInput ln, float* __restrict__ P_out) {
  constexpr int DH = 64, LPK = 8, KPI = 8, U = 4;
  constexpr int NSH = NQ <= 2 ? 4 : 2;   // wavefronts that share a row's history
  using raw_t = half8_t;
  __shared__ __attribute__((aligned(16))) half_t a_rows[NQ][1024 + 8];
  __shared__ float qkv_s[3][NQ][DH];
  __shared__ float part[NQ][NSH][LPK][10];
  __shared__ __attribute__((aligned(16))) half_t ctx_s[NQ][DH + 8];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int b = blockIdx.x / H, h = blockIdx.x % H;
  const int ksteps = d / 16, nb = d / 256;
  const int fr = lane & 31, fk = (lane >> 5) * 8;
  const int nkeys = nkeys_base + (tp ? *tp : 0);   // cached positions; the new one gets this index
  // --- 1a. the history stream of this wavefront: row an, every NSH-th position from ash
  const int an = wave % NQ, ash = wave / NQ;
  const bool attends = ash < NSH;
  const int g = lane / LPK, c = lane % LPK;
  const int step = KPI * NSH;
  const int jfirst = ash + g * NSH;
  const int r_att = b * NQ + an;
  const size_t hbase = (size_t)(TABLE ? b * NQ : r_att) * T_ * d + h * DH;
  const char* Kb = reinterpret_cast<const char*>(Kc + hbase);
  const char* Vb = reinterpret_cast<const char*>(Vc + hbase);
  const int32_t* slot = TABLE ? anc + (size_t)r_att * (T_ + 1) : nullptr;
  const int slot_stride = T_ * d, slot_max = NQ - 1;
  int sl[U];
  raw_t kn[U], vn[U];
  auto request_slots = [&](int jb, int last) {
#pragma unroll
    for (int u = 0; u < U; ++u) sl[u] = TABLE ? slot[min(jb + u * step, last)] : 0;
  };
  auto request = [&](int jb, int last) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const unsigned at = ((TABLE ? min(max(sl[u], 0), slot_max) * slot_stride : 0) + min(jb + u * step, last) * d + c * 8) *
                          (unsigned)sizeof(half_t);
      kn[u] = *reinterpret_cast<const raw_t*>(Kb + at);
      vn[u] = *reinterpret_cast<const raw_t*>(Vb + at);
    }
  };
  const int jcap = T_ - 1;
  if (attends) request_slots(jfirst, jcap);
  // --- 1b/2. LayerNorm inputs are requested (and awaited) by the wavefronts that normalise
  // --- 1c. weight fragments: wavefront (part, column half) = (wave >> 1, wave & 1) for wave < 6
  const bool multiplies = wave < 6;
  const int prt_ = wave >> 1, cb = wave & 1;
  const half_t* wp = Wqkv + ((size_t)((prt_ * d) / 32 + h * 2 + cb) * ksteps) * 512 + lane * 8;
  half8_t f0[16], f1[16];
  half4_t bias4[4];
  if (multiplies) {
#pragma unroll
    for (int u = 0; u < 16; ++u) f0[u] = *reinterpret_cast<const half8_t*>(wp + (size_t)min(u, ksteps - 1) * 512);
#pragma unroll
    for (int u = 0; u < 16; ++u) f1[u] = *reinterpret_cast<const half8_t*>(wp + (size_t)min(16 + u, ksteps - 1) * 512);
#pragma unroll
    for (int vg = 0; vg < 4; ++vg)
      bias4[vg] = *reinterpret_cast<const half4_t*>(bqkv + prt_ * d + h * DH + cb * 32 + vg * 8 + (lane >> 5) * 4);
  } else {
    block_request_out_fragments<NQ>(f0, Wo, wave, lane, nb, h, ksteps);
  }
  asm volatile("" ::: "memory");
  // the two wavefronts that multiply nothing normalise
  if (wave >= 6)
    for (int n = wave - 6; n < NQ; n += 2) block_row<4>(ln, b * NQ + n, M, d, lane, h == 0, a_rows[n]);
  __syncthreads();
  // the first trip through the history is not needed before the products are done: requested here,
  // where the registers of the LayerNorm are free again
  if (attends) {
    request(jfirst, jcap);
    request_slots(jfirst + U * step, jcap);
  }
  asm volatile("" ::: "memory");
  // --- 3. the new position's q, k, v
  if (multiplies) {
    floatx16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    const half_t* ar = &a_rows[min(fr, NQ - 1)][fk];
    auto multiply = [&](const half8_t (&f)[16], int ks0) {
#pragma unroll
      for (int u = 0; u < 16; ++u)
        if (ks0 + u < ksteps) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(f[u], *reinterpret_cast<const half8_t*>(ar + (ks0 + u) * 16), acc, 0, 0, 0);
    };
    multiply(f0, 0);
    if (ksteps > 32) {
#pragma unroll
      for (int u = 0; u < 16; ++u) f0[u] = *reinterpret_cast<const half8_t*>(wp + (size_t)min(32 + u, ksteps - 1) * 512);
    } else {
      block_request_out_fragments<NQ>(f0, Wo, wave, lane, nb, h, ksteps);
    }
    multiply(f1, 16);
    if (ksteps > 48) {
#pragma unroll
      for (int u = 0; u < 16; ++u) f1[u] = *reinterpret_cast<const half8_t*>(wp + (size_t)min(48 + u, ksteps - 1) * 512);
    }
    if (ksteps > 32) {
      multiply(f0, 32);
      block_request_out_fragments<NQ>(f0, Wo, wave, lane, nb, h, ksteps);
    }
    if (ksteps > 48) multiply(f1, 48);
    if (fr < NQ) {
      const int r = b * NQ + fr;
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const int col = cb * 32 + vg * 8 + (lane >> 5) * 4;
        half4_t o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          o[e] = (half_t)(acc[vg * 4 + e] + (float)bias4[vg][e]);
          qkv_s[prt_][fr][col + e] = (float)o[e];
        }
        if (prt_ >= 1) *reinterpret_cast<half4_t*>((prt_ == 1 ? Kc : Vc) + ((size_t)r * T_ + nkeys) * d + h * DH + col) = o;
      }
    }
  }
  __syncthreads();
  // --- 4. attention
  if (attends) {
    constexpr float qscale = 0.125f * 1.44269504088896340736f;   // scores in units of log 2
    float q[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) q[i] = qkv_s[0][an][c * 8 + i];
    float m = -INFINITY, l = 0.f, acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    int jb = jfirst;
    bool speculative = true;
    do {
      float kv[U][8], vv[U][8];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        Vec8<half_t>::unpack(kn[u], kv[u]);
        Vec8<half_t>::unpack(vn[u], vv[u]);
      }
      if (speculative) {
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (jb + u * step >= nkeys) {   // read from beyond the history: may be anything
#pragma unroll
            for (int i = 0; i < 8; ++i) vv[u][i] = 0.f;
          }
      }
      const int jn = jb + U * step;
      if (jn < nkeys) {   // the next trip, requested before this one's arithmetic
        request(jn, nkeys - 1);
        request_slots(jn + U * step, nkeys - 1);
      }
      float sc[U], mx = m;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) s += q[i] * kv[u][i];
        s = group_sum<LPK>(s) * qscale;
        sc[u] = (jb + u * step < nkeys) ? s : -INFINITY;
        mx = fmaxf(mx, sc[u]);
      }
      const float corr = m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m - mx);
      m = mx;
      l *= corr;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] *= corr;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float p = sc[u] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(sc[u] - mx);
        l += p;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] += p * vv[u][i];
      }
      jb = jn;
      speculative = false;
    } while (jb < nkeys);
    {
      // the new position: its key and value never left the workgroup; counted once, by the first key
      // slot of the row's first wavefront
      float s = 0.f, vt[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) { s += q[i] * qkv_s[1][an][c * 8 + i]; vt[i] = qkv_s[2][an][c * 8 + i]; }
      s = group_sum<LPK>(s) * qscale;
      const float st = (ash == 0 && g == 0) ? s : -INFINITY;
      const float mx = fmaxf(m, st);
      const float corr = m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m - mx);
      const float p = st == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(st - mx);
      m = mx;
      l = l * corr + p;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = acc[i] * corr + p * vt[i];
    }
    // the key slots of the wavefront, then (through LDS) the wavefronts of the row
    float mx = m;
    for_lane_bits<LPK>([&](auto bit) { mx = max_lane_xor<decltype(bit)::value>(mx); });
    const float c1 = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - mx);
    l *= c1;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] *= c1;
    for_lane_bits<LPK>([&](auto bit) {
      constexpr int O = decltype(bit)::value;
      l = add_lane_xor<O>(l);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = add_lane_xor<O>(acc[i]);
    });
    if (g == 0) {
      part[an][ash][c][0] = mx;
      part[an][ash][c][1] = l;
#pragma unroll
      for (int i = 0; i < 8; ++i) part[an][ash][c][2 + i] = acc[i];
    }
  }
  __syncthreads();
  if (threadIdx.x < NQ * LPK) {
    const int n = threadIdx.x / LPK, cc = threadIdx.x % LPK;
    float mx = -INFINITY;
#pragma unroll
    for (int w = 0; w < NSH; ++w) mx = fmaxf(mx, part[n][w][cc][0]);   // finite: the first wavefront saw the new position
    float sum = 0.f, o8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < NSH; ++w) {
      const float mw = part[n][w][cc][0];
      const float cw = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - mx);
      sum += part[n][w][cc][1] * cw;
#pragma unroll
      for (int i = 0; i < 8; ++i) o8[i] += part[n][w][cc][2 + i] * cw;
    }
    const float inv = 1.0f / sum;
#pragma unroll
    for (int i = 0; i < 8; ++i) o8[i] *= inv;
    Vec8<half_t>::store(&ctx_s[n][cc * 8], o8);
  }
  __syncthreads();
  // --- 5. the head's share of the output projection
  block_out_projection<NQ>(f0, ctx_s, wave, lane, nb, h, b * NQ, M, d, P_out);
}

// Cross-attention sublayer up to the output projection's partial sums: cross_attention_ln_kernel (its
// steps 1-4, with up to 16 slabs behind the LayerNorm: the self-attention block above leaves one per
// head) whose context rows stay in LDS and are multiplied by the head's 64 k-columns of Woc.
template <int NQ>
__global__ void __launch_bounds__(512) cross_block_kernel(const half_t* __restrict__ Wp, const half_t* __restrict__ Wo,
                                                          const half_t* __restrict__ kv,
                                                          const int32_t* __restrict__ off,
                                                          const int32_t* __restrict__ len, int H, int d, int M,
                                                          LnInput ln, const half_t* __restrict__ bq,
                                                          float* __restrict__ P_out) {
  constexpr int DH = 64, LPK = 8, KPW = 8, G = 4, UMAX = 16;
  constexpr float scale = 0.125f;
  __shared__ __attribute__((aligned(16))) half_t a_rows[NQ][1024 + 8];
  __shared__ float red[8][16][64];
  __shared__ float q_s[NQ][DH];
  __shared__ float part[4][NQ][DH + 2];
  __shared__ __attribute__((aligned(16))) half_t ctx_s[NQ][DH + 8];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int b = blockIdx.x / H, h = blockIdx.x % H;
  const int ksteps = d / 16, per_wave = ksteps / 4, nb = d / 256;
  const int fr = lane & 31, fk = (lane >> 5) * 8;
  const int cb = wave >> 2, kw = wave & 3;
  const half_t* wp = Wp + ((size_t)(h * 2 + cb) * ksteps) * 512 + lane * 8;
  half8_t bf[UMAX];
#pragma unroll
  for (int u = 0; u < UMAX; ++u) bf[u] = *reinterpret_cast<const half8_t*>(wp + (size_t)min(kw + 4 * u, ksteps - 1) * 512);
  int n_keys = len[b], row0 = off[b];
  asm volatile("" : "+s"(n_keys), "+s"(row0));
  const int c = lane % LPK, slot = lane / LPK;
  CrossKeys<half_t, DH, NQ> keys;
  keys.K = reinterpret_cast<const char*>(kv + (size_t)row0 * 2 * d + h * DH);
  keys.V = keys.K + d * sizeof(half_t);
  keys.stride = 2 * d * sizeof(half_t);
  keys.lane_at = c * 8 * sizeof(half_t);
  keys.n_keys = n_keys;
  keys.slot = slot;
  const int jfirst = wave < 4 ? wave * G * KPW : 0x7fffffff;
  if (jfirst < n_keys) keys.request(jfirst);
  asm volatile("" ::: "memory");
  if (wave < NQ) block_row<8>(ln, b * NQ + wave, M, d, lane, h == 0, a_rows[wave]);
  __syncthreads();
  floatx16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  const half_t* ar = &a_rows[min(fr, NQ - 1)][fk];
#pragma unroll
  for (int u = 0; u < UMAX; ++u)
    if (u < per_wave) {
      const half8_t af = *reinterpret_cast<const half8_t*>(ar + (kw + 4 * u) * 16);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[u], af, acc, 0, 0, 0);
    }
  block_request_out_fragments<NQ>(bf, Wo, wave, lane, nb, h, ksteps);   // travel while the wavefronts attend
#pragma unroll
  for (int e = 0; e < 16; ++e) red[wave][e][lane] = acc[e];
  __syncthreads();
  {
    const int vg = kw, m = lane & 31;
    if (m < NQ) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int rr = vg * 4 + e, n = cb * 32 + vg * 8 + (lane >> 5) * 4 + e;
        float x = (red[cb * 4 + 0][rr][lane] + red[cb * 4 + 1][rr][lane]) + (red[cb * 4 + 2][rr][lane] + red[cb * 4 + 3][rr][lane]);
        x += (float)bq[h * DH + n];
        q_s[m][n] = (float)(half_t)x;
      }
    }
  }
  __syncthreads();
  float qv[NQ][8];
#pragma unroll
  for (int n = 0; n < NQ; ++n)
#pragma unroll
    for (int i = 0; i < 8; ++i) qv[n][i] = q_s[n][c * 8 + i];
  float mx_[NQ], l_[NQ], acc_[NQ][8];
  keys.run(qv, scale * 1.44269504088896340736f, jfirst, 4 * G * KPW, mx_, l_, acc_);
  if (wave < 4) cross_deposit<DH, NQ>(part, wave, lane, mx_, l_, acc_);
  __syncthreads();
  cross_finish<half_t, DH, NQ>(part, wave, lane, &ctx_s[0][0], DH + 8);
  __syncthreads();
  block_out_projection<NQ>(bf, ctx_s, wave, lane, nb, h, b * NQ, M, d, P_out);
}

constexpr int kBlockRows = 64;

bool attention_blocks_supported(int dtype, int rows, int beam, int H, int d) {
  return dtype == DT_F16 && rows >= 1 && rows <= kBlockRows && beam >= 1 && beam <= 4 && rows % beam == 0 && H >= 1 &&
         d == H * 64 && d % 256 == 0 && d <= 1024;
}

hipError_t launch_self_block(const LnInput& ln, const void* Wqkv_packed, const void* bqkv, const void* Wo_packed,
                             void* Kc, void* Vc, const int32_t* anc, const int32_t* tp, int nkeys_base, float* P_out,
                             int batch, int beam, int H, int d, int T, hipStream_t s) {
  if (batch <= 0) return hipSuccess;
  if (!attention_blocks_supported(DT_F16, batch * beam, beam, H, d) || !Wqkv_packed || !bqkv || !Wo_packed || !Kc || !Vc ||
      !P_out || ln.splits < 0 || ln.splits > 4 || !ln.x_old || (ln.splits > 0 && (ln.x_old == ln.x_new || !ln.x_new)) ||
      ((ln.splits > 0 || ln.pre) && (!ln.g || !ln.b)) || (ln.splits > 0 && (!ln.P || !ln.bias)) ||
      (long)beam * T * d * 2 > 0x7fffffffL)
    return hipErrorInvalidValue;
  dim3 g(batch * H), b(512);
  const int M = batch * beam;
#define LSQ_SELF_BLOCK(NQ_)                                                                                          \
  do {                                                                                                               \
    if (anc)                                                                                                         \
      self_block_kernel<NQ_, true><<<g, b, 0, s>>>((const half_t*)Wqkv_packed, (const half_t*)Wo_packed, anc, tp,    \
                                                   nkeys_base, H, d, T, M, (half_t*)Kc, (half_t*)Vc,                \
                                                   (const half_t*)bqkv, ln, P_out);                                  \
    else                                                                                                             \
      self_block_kernel<NQ_, false><<<g, b, 0, s>>>((const half_t*)Wqkv_packed, (const half_t*)Wo_packed, anc, tp,   \
                                                    nkeys_base, H, d, T, M, (half_t*)Kc, (half_t*)Vc,               \
                                                    (const half_t*)bqkv, ln, P_out);                                 \
  } while (0)
  switch (beam) {
    case 1: LSQ_SELF_BLOCK(1); break;
    case 2: LSQ_SELF_BLOCK(2); break;
    case 3: LSQ_SELF_BLOCK(3); break;
    default: LSQ_SELF_BLOCK(4); break;
  }
#undef LSQ_SELF_BLOCK
  return hipGetLastError();
}

hipError_t launch_cross_block(const LnInput& ln, const void* Wq_packed, const void* bq, const void* Wo_packed,
                              const void* kv, const int32_t* off, const int32_t* len, float* P_out, int batch, int beam,
                              int H, int d, hipStream_t s) {
  if (batch <= 0) return hipSuccess;
  if (!attention_blocks_supported(DT_F16, batch * beam, beam, H, d) || !Wq_packed || !bq || !Wo_packed || !P_out ||
      ln.splits < 1 || ln.splits > 16 || !ln.x_old || !ln.x_new || ln.x_old == ln.x_new)
    return hipErrorInvalidValue;
  dim3 g(batch * H), b(512);
  const int M = batch * beam;
#define LSQ_CROSS_BLOCK(NQ_)                                                                                       \
  cross_block_kernel<NQ_><<<g, b, 0, s>>>((const half_t*)Wq_packed, (const half_t*)Wo_packed, (const half_t*)kv, off, len, \
                                          H, d, M, ln, (const half_t*)bq, P_out)
  switch (beam) {
    case 1: LSQ_CROSS_BLOCK(1); break;
    case 2: LSQ_CROSS_BLOCK(2); break;
    case 3: LSQ_CROSS_BLOCK(3); break;
    default: LSQ_CROSS_BLOCK(4); break;
  }
#undef LSQ_CROSS_BLOCK
  return hipGetLastError();
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
  const int w = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (threadIdx.x >> 6));   // one value per wavefront
  if (w >= rows * H) return;
  int r = w / H, h = w % H;
  int b = row_sent[r];
  // causal (decoder-only prefill): row r sits at position r - off[b] and sees keys up to itself
  const int nk = causal ? r - off[b] + 1 : len[b];
  const T* qp[1] = {qkv + (size_t)r * 3 * d + h * DH};
  T* op[1] = {out + (size_t)r * d + h * DH};
  const T* K = qkv + (size_t)off[b] * 3 * d + d + h * DH;
  attend<T, DH, 1>(qp, K, K + d, 3 * d, nk, nk - 1, scale, op, threadIdx.x & 63);
}

// The same on the matrix cores, float16, heads of 32, 64 or 128: one wavefront per (block of 32 packed
// rows, head).  Packed rows run through the sentences one after the other, so a block's rows belong to a
// few consecutive sentences and the keys any of them may see are one contiguous run of packed rows, taken
// 32 at a time:
//   S = Q K^T      v_mfma_f32_32x32x16_f16 with both operands straight from global memory (a row's 8
//                  consecutive head dimensions per lane, as the skinny products read theirs);
//   mask           key j counts for row i if it lies in i's sentence (and, causal, not behind i);
//   softmax        streaming (running maximum and sum per row; a row's 32 scores sit in the two lanes
//                  l and l + 32, 16 each);
//   O += P V       the contraction runs over keys, and a matrix-core operand wants 8 contraction indices
//                  per lane.  Which key sits at which index is free as long as P and V agree, so P is used
//                  exactly as the first product left it in the lane's registers (index j of step st =
//                  key 16 st + 8 (j >> 2) + 4 (lane >> 5) + (j & 3)) and the V operand is gathered to
//                  match: 8 two-byte loads per lane and step, each a 64-byte run of one key's row across
//                  the lanes.  No LDS, no transposition, no barrier.
// Scores of keys outside a row's sentence are computed and thrown away (with sentences of about 30 tokens a
// block of 32 rows sees two or three key blocks); the kernel is bounded by its handful of trips to
// memory, not by the matrix cores.
template <int DH>
__global__ void __launch_bounds__(256) encoder_attention_mfma_kernel(const half_t* __restrict__ qkv,
                                                                     const int32_t* __restrict__ row_sent,
                                                                     const int32_t* __restrict__ off,
                                                                     const int32_t* __restrict__ len,
                                                                     half_t* __restrict__ out, int rows, int H, int d,
                                                                     int causal, float scale_log2e) {
  constexpr int QS = DH / 16;   // k-steps of the score product
  constexpr int NB = DH / 32;   // 32-wide blocks of output dimensions
  const int w = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (threadIdx.x >> 6));
  const int nblk = (rows + 31) / 32;
  if (w >= nblk * H) return;
  const int blk = w / H, h = w % H;
  const int lane = threadIdx.x & 63, m = lane & 31, hi = lane >> 5;
  const int r = min(blk * 32 + m, rows - 1);             // this lane's row (past the end: the last row, not stored)
  const int b = row_sent[r];
  const int lo = off[b];
  const int hi_key = causal ? r + 1 : lo + len[b];       // keys lo .. hi_key - 1 count for row r
  const int ld = 3 * d;
  // the block's key range: from the first row's sentence start to the last row's limit
  const int k_first = __builtin_amdgcn_readlane(lo, 0);
  const int k_last = __builtin_amdgcn_readlane(hi_key, 31);
  const half_t* qp = qkv + (size_t)r * ld + h * DH + hi * 8;
  half8_t qf[QS];
#pragma unroll
  for (int i = 0; i < QS; ++i) qf[i] = *reinterpret_cast<const half8_t*>(qp + i * 16);
  const half_t* kbase = qkv + d + h * DH + hi * 8;
  const half_t* vbase = qkv + 2 * d + h * DH + m;
  floatx16 o[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[nb][e] = 0.f;
  float mx = -INFINITY, sum = 0.f;
  for (int k0 = k_first; k0 < k_last; k0 += 32) {
    // operands of this key block: K rows (key = k0 + m), V gathered in the order the scores come out
    const int krow = min(k0 + m, k_last - 1);
    half8_t kf[QS];
#pragma unroll
    for (int i = 0; i < QS; ++i) kf[i] = *reinterpret_cast<const half8_t*>(kbase + (size_t)krow * ld + i * 16);
    half8_t vf[NB][2];
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int key = min(k0 + 16 * st + 8 * (j >> 2) + 4 * hi + (j & 3), k_last - 1);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) vf[nb][st][j] = vbase[(size_t)key * ld + nb * 32];
      }
    floatx16 sc;
#pragma unroll
    for (int e = 0; e < 16; ++e) sc[e] = 0.f;
#pragma unroll
    for (int i = 0; i < QS; ++i) sc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[i], qf[i], sc, 0, 0, 0);
    // sc[vg * 4 + e] = q_m . k_key, key = k0 + vg * 8 + hi * 4 + e
    float bm = -INFINITY;
#pragma unroll
    for (int vg = 0; vg < 4; ++vg)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int key = k0 + vg * 8 + hi * 4 + e;
        const float v = (key >= lo && key < hi_key) ? sc[vg * 4 + e] * scale_log2e : -INFINITY;
        sc[vg * 4 + e] = v;
        bm = fmaxf(bm, v);
      }
    bm = max_lane_xor<32>(bm);                            // the row's other 16 keys are in lane ^ 32
    const float mn = fmaxf(mx, bm);
    const float base = mn == -INFINITY ? 0.f : mn;        // no key of this block (or any before) counts for the row
    const float corr = exp2f(mx - base);                  // mx = -inf: 0
    float ps = 0.f;
    half8_t pf[2];
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float pv = exp2f(sc[st * 8 + j] - base);
        const half_t ph = (half_t)pv;
        ps += (float)ph;                                  // the sum of what the second product multiplies
        pf[st][j] = ph;
      }
    ps = add_lane_xor<32>(ps);
    sum = sum * corr + ps;
    mx = mn;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
      for (int e = 0; e < 16; ++e) o[nb][e] *= corr;
#pragma unroll
      for (int st = 0; st < 2; ++st) o[nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf[nb][st], pf[st], o[nb], 0, 0, 0);
    }
  }
  if (blk * 32 + m >= rows) return;
  const float inv = 1.0f / sum;
  half_t* op = out + (size_t)r * d + h * DH;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int vg = 0; vg < 4; ++vg) {
      half4_t hv;
#pragma unroll
      for (int e = 0; e < 4; ++e) hv[e] = (half_t)(o[nb][vg * 4 + e] * inv);
      *reinterpret_cast<half4_t*>(op + nb * 32 + vg * 8 + hi * 4) = hv;
    }
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

// up to this many (row, head) pairs a workgroup, not a wavefront, takes each pair: the launch would leave most of
// the chip idle otherwise.  Beyond, one wavefront per pair with the beams of a sentence in one workgroup, which
// fetches an ancestor they share once (whole translations of the big model, 16 heads: 32 sentences of beam 4 =
// 2048 pairs 49.5 -> 46.3 ms, 16 sentences 41.7 -> 40.5 ms, the batch of 128 level, when the limit went from 2048
// to 512 pairs; with no split at all the last sentences of a batch and 32 rows of 12 heads are 1-2 % slower)
constexpr int kSplitAttentionUnits = 512;

template <typename T>
static hipError_t self_t(const T* q, const T* Kc, const T* Vc, T* out, int rows, int H, int d, int T_,
                         int nkeys, const int32_t* tp, const int32_t* anc, int beam, int anc_ld, hipStream_t s) {
  int dh = d / H;
  if (H > 0xffff || beam < 0 || beam > 0x7fff) return hipErrorInvalidValue;
  const int H_beam = H | beam << 16;   // two small numbers in one argument word
  dim3 b(256);
  if (rows * H <= kSplitAttentionUnits) {
    dim3 g(rows * H);
    if (anc) { LSQ_DISPATCH_DH(dh, (self_attention_split_kernel<T, DH, true><<<g, b, 0, s>>>(q, Kc, Vc, anc, tp, H_beam, d, T_, rows, nkeys, out))); }
    else { LSQ_DISPATCH_DH(dh, (self_attention_split_kernel<T, DH, false><<<g, b, 0, s>>>(q, Kc, Vc, anc, tp, H_beam, d, T_, rows, nkeys, out))); }
  } else {
    dim3 g((rows * H + 3) / 4);
    if (anc) { LSQ_DISPATCH_DH(dh, (self_attention_kernel<T, DH, true><<<g, b, 0, s>>>(q, Kc, Vc, anc, tp, H_beam, d, T_, rows, nkeys, out))); }
    else { LSQ_DISPATCH_DH(dh, (self_attention_kernel<T, DH, false><<<g, b, 0, s>>>(q, Kc, Vc, anc, tp, H_beam, d, T_, rows, nkeys, out))); }
  }
  return hipGetLastError();
}

hipError_t launch_self_attention(int dtype, const void* q, const void* Kc, const void* Vc, void* out,
                                 int rows, int H, int d, int T, int nkeys, const int32_t* tp, const int32_t* anc,
                                 int beam, int anc_ld, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (anc && (beam < 1 || rows % beam != 0 || anc_ld != T + 1)) return hipErrorInvalidValue;   // table rows hold T + 1 entries
  if ((long)(anc ? beam : 1) * T * d * 4 > 0xffffffffL) return hipErrorInvalidValue;   // a lane's byte offset inside a sentence's slabs is 32 bits wide
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
  if (cross_attention_splits(batch * H, smax)) {
    dim3 g(batch * H), b(256);
    LSQ_DISPATCH_DH(dh, (cross_attention_kernel<T, DH, NQ, true><<<g, b, 0, s>>>(q, kv, off, len, batch, beam, first, H, d, out)));
    return hipGetLastError();
  }
  dim3 g((batch * H + 3) / 4), b(256);
  LSQ_DISPATCH_DH(dh, (cross_attention_kernel<T, DH, NQ, false><<<g, b, 0, s>>>(q, kv, off, len, batch, beam, first, H, d, out)));
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
  if constexpr (std::is_same<T, half_t>::value) {
    if ((dh == 32 || dh == 64 || dh == 128) && d % 8 == 0 && (reinterpret_cast<uintptr_t>(qkv) & 15) == 0 &&
        (reinterpret_cast<uintptr_t>(out) & 7) == 0) {
      dim3 g((((rows + 31) / 32) * H + 3) / 4), b(256);
      const float sl = scale * 1.4426950408889634f;
      if (dh == 32) encoder_attention_mfma_kernel<32><<<g, b, 0, s>>>(qkv, row_sent, off, len, out, rows, H, d, causal, sl);
      else if (dh == 64) encoder_attention_mfma_kernel<64><<<g, b, 0, s>>>(qkv, row_sent, off, len, out, rows, H, d, causal, sl);
      else encoder_attention_mfma_kernel<128><<<g, b, 0, s>>>(qkv, row_sent, off, len, out, rows, H, d, causal, sl);
      return hipGetLastError();
    }
  }
  dim3 g((rows * H + 3) / 4), b(256);
  LSQ_DISPATCH_DH(dh, (encoder_attention_kernel<T, DH><<<g, b, 0, s>>>(qkv, row_sent, off, len, out, rows, H, d, causal, scale)));
  return hipGetLastError();
}

hipError_t launch_encoder_attention(int dtype, const void* qkv, const int32_t* row_sent, const int32_t* off,
                                    const int32_t* len, void* out, int rows, int H, int d, int causal,
                                    hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if ((long)rows * 3 * d * 4 > 0xffffffffL) return hipErrorInvalidValue;   // a lane's byte offset inside a sentence is 32 bits wide
  if (dtype == DT_F16)
    return enc_t<half_t>((const half_t*)qkv, row_sent, off, len, (half_t*)out, rows, H, d, causal, s);
  return enc_t<float>((const float*)qkv, row_sent, off, len, (float*)out, rows, H, d, causal, s);
}

}  // namespace lsq
