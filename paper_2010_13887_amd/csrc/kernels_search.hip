// Output layer of the auto-regressive search (paper sec. 2.2) and cache refreshing (sec. 3.2).
//
//  row_topk   -- "retrieve", made exact: one workgroup reads one row of logits ONCE into
//                registers, computes the full-vocabulary max and sum-of-exponentials, forms
//                cand = score + ((x - max) - log sum) for every token, picks a rough top-k
//                threshold from group maxima (the paper's idea, with the lanes as the groups),
//                collects the tokens at or above it in LDS and ranks those exactly by
//                (cand descending, token ascending).  Nothing but k pairs per row is written.
//  beam_refine-- "re-rank": per sentence the k best of the k*k survivors by (cand descending,
//                beam*V + token ascending), then the hypothesis bookkeeping.
//  cache_reorder -- gathers K/V cache rows by parent beam, in place.
#include "lsq_internal.h"

namespace lsq {

// Total order used everywhere: higher score first, lower index first among equal scores.
__device__ __forceinline__ bool precedes(float s1, int i1, float s2, int i2) {
  return s1 > s2 || (s1 == s2 && i1 < i2);
}

// One workgroup of BLOCK threads per row; each thread holds NV*8 tokens in registers.
// Token held in slot (j, e) of thread tid:  vectorised rows (V % 8 == 0): (j*BLOCK + tid)*8 + e;
// otherwise (j*8 + e)*BLOCK + tid.
// Register budget: two workgroups must fit a CU, so that one loads its row while the other reduces.
template <typename T, int BLOCK, int NV>
__global__ void __launch_bounds__(BLOCK) __attribute__((amdgpu_waves_per_eu(BLOCK == 512 ? 4 : 1)))
row_topk_kernel(const T* __restrict__ logits,
                                                         const float* __restrict__ score,
                                                         const int32_t* __restrict__ fin, int V, int k, int eos,
                                                         int raw, float* __restrict__ out_score,
                                                         int32_t* __restrict__ out_idx, SearchGroups gr) {
  __shared__ float reds[BLOCK / 64];
  __shared__ int redi[BLOCK / 64];
  const int tid = threadIdx.x;
  const int sent = blockIdx.x / gr.kg;                                   // one group of every sentence per launch
  const int r = sent * gr.k_all + gr.goff + blockIdx.x % gr.kg;
  const float bs = raw ? 0.f : score[r];
  float* os = out_score + (size_t)r * k;
  int32_t* oi = out_idx + (size_t)r * k;
  float* op = gr.out_plain ? gr.out_plain + (size_t)r * k : nullptr;     // unpenalised values of the kept
  if (!raw && fin[r]) {   // a finished hypothesis offers itself once
    if (tid < k) {
      os[tid] = tid == 0 ? bs : -INFINITY; oi[tid] = tid == 0 ? eos : -1;
      if (op) op[tid] = os[tid];
    }
    return;
  }
  if (bs == -INFINITY) {   // every candidate is -inf: the order is by token alone
    if (tid < k) {
      os[tid] = -INFINITY; oi[tid] = tid < V ? tid : -1;
      if (op) op[tid] = -INFINITY;
    }
    return;
  }
  const T* row = logits + (size_t)r * V;
  const bool vec = (V & 7) == 0;
  float x[NV * 8];
  float mx = -INFINITY;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    if (vec) {
      int base = (j * BLOCK + tid) * 8;
      if (base < V) {
        float t[8];
        Vec8<T>::load(row + base, t);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[j * 8 + e] = t[e];
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) x[j * 8 + e] = -INFINITY;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        int v = (j * 8 + e) * BLOCK + tid;
        x[j * 8 + e] = v < V ? (float)row[v] : -INFINITY;
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) mx = fmaxf(mx, x[j * 8 + e]);
  }
  // One reduction for both softmax statistics: every thread owns (local max, local sum of
  // exp(x - local max)); pairs merge as (max, z1*exp(m1-max) + z2*exp(m2-max)).
  constexpr int NW = BLOCK / 64, CAP = 1024;   // a few k * H_k candidates are expected; k = 32 needs the room
  const int cap = k > LSQ_MAX_BEAM_ ? CAP : 256;   // a beam's list is short: beyond 256 the k-round search is quicker
  __shared__ float red_m[NW], red_z[NW], wave_best[NW * LSQ_MAX_TOPK_];
  __shared__ float cand_s[CAP];
  __shared__ int cand_i[CAP];
  __shared__ int cand_n;
  const int lane = tid & 63, wave = tid >> 6;
  float z = 0.f;
  if (!raw && mx != -INFINITY) {
#pragma unroll
    for (int i = 0; i < NV * 8; ++i) z += __expf(x[i] - mx);   // padding slots: exp(-inf) = 0
  }
  float wm = mx, wz = z;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float m2 = __shfl_xor(wm, o, kWave), z2 = __shfl_xor(wz, o, kWave);
    const float mn = fmaxf(wm, m2);
    if (mn != -INFINITY) wz = wz * __expf(wm - mn) + z2 * __expf(m2 - mn);
    wm = mn;
  }
  if (lane == 0) { red_m[wave] = wm; red_z[wave] = wz; }
  if (tid == 0) cand_n = 0;
  __syncthreads();
  float m = red_m[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) m = fmaxf(m, red_m[w]);
  float zt = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) zt += red_z[w] * __expf(red_m[w] - m);   // a wave of padding has z = 0
  const float logz = logf(zt);
  // candidate scores, rounded exactly as (score + ((x - m) - logz)) with no fused operation;
  // raw mode (sampling) ranks the logits themselves
  float best = -INFINITY;
#pragma unroll
  for (int i = 0; i < NV * 8; ++i) {
    if (!raw) x[i] = __fadd_rn(bs, __fsub_rn(__fsub_rn(x[i], m), logz));
  }
  // diverse beam search: every time an earlier group of this sentence took token v at this step,
  // v's ranking value drops by `strength` (all occurrences counted first, one subtraction)
  auto plain_of = [&](int v) { return __fadd_rn(bs, __fsub_rn(__fsub_rn((float)row[v], m), logz)); };
  if (gr.pen_tok) {
    const int np = gr.pen_n[sent];
    for (int p = 0; p < np; ++p) {
      const int tk = gr.pen_tok[(size_t)sent * gr.pen_ld + p];
      int cnt = 0;
      bool first = true;
      for (int q = 0; q < np; ++q) {
        const bool same = gr.pen_tok[(size_t)sent * gr.pen_ld + q] == tk;
        cnt += same ? 1 : 0;
        if (same && q < p) first = false;
      }
      const int owner = vec ? (tk >> 3) % BLOCK : tk % BLOCK;
      if (first && owner == tid && tk < V) {
        const int slot = vec ? ((tk >> 3) / BLOCK) * 8 + (tk & 7) : tk / BLOCK;
        const float pen = __fmul_rn(gr.strength, (float)cnt);
#pragma unroll
        for (int i = 0; i < NV * 8; ++i)
          if (i == slot) x[i] = __fsub_rn(x[i], pen);
      }
    }
  }
#pragma unroll
  for (int i = 0; i < NV * 8; ++i) best = fmaxf(best, x[i]);     // padding slots stay -inf

  // ---- rough stage (the paper's retrieve, sec. 2.2): split the row into k groups, take each
  // group's maximum, R = the smallest of them.  Each group maximum is the score of a distinct
  // token, so k tokens reach R and every token of the row's top k satisfies score >= R (ties at R
  // included).  Groups here: the wavefronts taken modulo k (blocks of at least k wavefronts) or the
  // lanes taken modulo k (fewer wavefronts than k).  The tokens at or above R -- a dozen or so on average --
  // go to a short list in LDS which is then ranked exactly.  Rows where the list
  // overflows (e.g. thousands of equal logits) take the exact k-round arg-max below instead.
  float R;
  // wavefront groups need every wavefront to hold tokens: with the vectorised layout wavefront w
  // starts at token 512 w, so short rows leave the last wavefronts empty (their maximum would be
  // -inf and every token would pass the threshold)
  if (NW >= k && (long)(NW - 1) * 512 < V) {
    const float wb = wave_max(best);
    if (lane == 0) wave_best[wave] = wb;
    __syncthreads();
    R = INFINITY;
    for (int grp = 0; grp < k; ++grp) {
      float gm = -INFINITY;
      for (int w = grp; w < NW; w += k) gm = fmaxf(gm, wave_best[w]);
      R = fminf(R, gm);
    }
  } else {
    // fewer wavefronts than groups (or empty ones): groups are the lanes modulo k of every
    // wavefront.  Group maxima inside a wavefront: a butterfly over the lanes that share lane % k
    // when k is a power of two, else one wavefront reduction per group; then thread g < k merges
    // group g across the wavefronts and the first wavefront takes the minimum.
    __shared__ float r_sh;
    if ((k & (k - 1)) == 0) {
      float gm = best;
      for (int o = k; o < 64; o <<= 1) gm = fmaxf(gm, __shfl_xor(gm, o, kWave));
      if (lane < k) wave_best[wave * LSQ_MAX_TOPK_ + lane] = gm;
    } else {
      for (int grp = 0; grp < k; ++grp) {
        const float gm = wave_max((lane % k) == grp ? best : -INFINITY);
        if (lane == 0) wave_best[wave * LSQ_MAX_TOPK_ + grp] = gm;
      }
    }
    __syncthreads();
    if (wave == 0) {
      float gm = INFINITY;
      if (lane < k) {
        gm = -INFINITY;
        for (int w = 0; w < NW; ++w) gm = fmaxf(gm, wave_best[w * LSQ_MAX_TOPK_ + lane]);
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) gm = fminf(gm, __shfl_xor(gm, o, kWave));
      if (lane == 0) r_sh = gm;
    }
    __syncthreads();
    R = r_sh;
  }
#pragma unroll
  for (int j = 0; j < NV; ++j)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int v = vec ? (j * BLOCK + tid) * 8 + e : (j * 8 + e) * BLOCK + tid;
      const float sc = x[j * 8 + e];
      if (v < V && sc >= R) {
        const int slot = atomicAdd(&cand_n, 1);
        if (slot < cap) { cand_s[slot] = sc; cand_i[slot] = v; }
      }
    }
  __syncthreads();
  const int n = cand_n;
  if (n <= cap) {
    // ---- exact ranking of the short list: a dozen entries for a beam (first wavefront), up to a
    // few hundred for wide sampling (all wavefronts) ----------------------------------------------
    if (wave == 0 || n > 64) {
      for (int c = (n > 64 ? tid : lane); c < n; c += (n > 64 ? BLOCK : 64)) {
        const float sc = cand_s[c];
        const int v = cand_i[c];
        int rank = 0;
        for (int o = 0; o < n; ++o) rank += precedes(cand_s[o], cand_i[o], sc, v) ? 1 : 0;
        if (rank < k) {
          os[rank] = sc; oi[rank] = v;
          if (op) op[rank] = plain_of(v);
        }
      }
      if (wave == 0 && lane >= n && lane < k) {   // vocabulary smaller than k
        os[lane] = -INFINITY; oi[lane] = -1;
        if (op) op[lane] = -INFINITY;
      }
    }
    return;
  }

  // ---- exact fallback: k rounds, each the best token strictly after the previous winner ----------
  float ps = INFINITY;
  int pi = -1;
  for (int round = 0; round < k; ++round) {
    float cs = -INFINITY;
    int ci = 0x7fffffff;
#pragma unroll
    for (int j = 0; j < NV; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        int v = vec ? (j * BLOCK + tid) * 8 + e : (j * 8 + e) * BLOCK + tid;
        float s = x[j * 8 + e];
        bool ok = v < V && precedes(ps, pi, s, v) && (ci == 0x7fffffff || precedes(s, v, cs, ci));
        if (ok) { cs = s; ci = v; }
      }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      float s2 = __shfl_xor(cs, o, kWave);
      int i2 = __shfl_xor(ci, o, kWave);
      if (i2 != 0x7fffffff && (ci == 0x7fffffff || precedes(s2, i2, cs, ci))) { cs = s2; ci = i2; }
    }
    __syncthreads();
    if ((tid & 63) == 0) { reds[tid >> 6] = cs; redi[tid >> 6] = ci; }
    __syncthreads();
    cs = reds[0];
    ci = redi[0];
#pragma unroll
    for (int w = 1; w < BLOCK / 64; ++w) {
      float s2 = reds[w];
      int i2 = redi[w];
      if (i2 != 0x7fffffff && (ci == 0x7fffffff || precedes(s2, i2, cs, ci))) { cs = s2; ci = i2; }
    }
    if (ci == 0x7fffffff) {   // fewer than k tokens in the vocabulary
      if (tid == 0) { os[round] = -INFINITY; oi[round] = -1; if (op) op[round] = -INFINITY; }
    } else {
      if (tid == 0) { os[round] = cs; oi[round] = ci; if (op) op[round] = plain_of(ci); }
      ps = cs;
      pi = ci;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// The retrieve stage (paper sec. 2.2) from group statistics that the logit product left behind: for every
// row and every group of 32 consecutive tokens the pair (largest logit, sum of exp(logit - largest)).
// One wavefront per row:
//   * softmax normaliser of the row from the G pairs (no pass over the logits);
//   * candidate value of every group's best token, cand = score + ((x - max) - log sum), the same
//     arithmetic as row_topk_kernel token by token (monotone in x, so it is the group's best cand);
//   * R = the k-th largest of the 64 lanes' best group values (each lane holds every 64th group): k distinct
//     tokens reach R, so every token of the row's exact top k has cand >= R, and such tokens only sit
//     in groups whose best reaches R -- the paper's threshold with the product's column groups as
//     the "random" groups;
//   * only those groups' logits are read (k groups of 32 unless values tie), tokens with cand >= R
//     are ranked exactly by (cand descending, token ascending).
// Rows where more than QMAX groups or CMAX tokens reach R (long runs of equal logits) fall back to k
// exact rounds over the whole row.  Same output as row_topk_kernel (no diverse groups); raw: the k largest
// logits themselves (sampling), no score, no normaliser.
constexpr int kTopkGroupsQ = 64, kTopkGroupsC = 128;   // groups / tokens that may reach the threshold before the fallback

// One row by one wavefront; ql, cs, ci: the wavefront's own LDS lists (kTopkGroupsQ, kTopkGroupsC entries); os, oi:
// where the k pairs go (global memory or LDS).
template <int GPL>
__device__ __forceinline__ void topk_groups_row(const float* __restrict__ logits, const float* __restrict__ stats,
                                                const float* __restrict__ score, const int32_t* __restrict__ fin,
                                                int r, int V, int G, int k, int eos, float* os, int32_t* oi, int lane,
                                                int* ql_w, float* cs_w, int* ci_w, int raw = 0) {
  constexpr int QMAX = kTopkGroupsQ, CMAX = kTopkGroupsC;
  // raw (sampling): the k largest logits themselves, no score, no normaliser, no finished rows
  const float bs = raw ? 0.f : score[r];
  const int f = raw ? 0 : fin[r];
  // the row's statistics, requested before anything is decided
  float gm[GPL], gz[GPL];
#pragma unroll
  for (int q = 0; q < GPL; ++q) {
    const int g = q * 64 + lane;
    if (g < G) {
      const float2 t = *reinterpret_cast<const float2*>(stats + ((size_t)r * G + g) * 2);
      gm[q] = t.x; gz[q] = t.y;
    } else {
      gm[q] = -INFINITY; gz[q] = 0.f;
    }
  }
  if (f) {   // a finished hypothesis offers itself once
    if (lane < k) { os[lane] = lane == 0 ? bs : -INFINITY; oi[lane] = lane == 0 ? eos : -1; }
    return;
  }
  if (bs == -INFINITY) {   // every candidate is -inf: the order is by token alone
    if (lane < k) { os[lane] = -INFINITY; oi[lane] = lane < V ? lane : -1; }
    return;
  }
  float m = -INFINITY;
#pragma unroll
  for (int q = 0; q < GPL; ++q) m = fmaxf(m, gm[q]);
  m = wave_max(m);
  float zt = 0.f;
#pragma unroll
  for (int q = 0; q < GPL; ++q) zt += gz[q] * __expf(gm[q] - m);   // a group that does not exist: 0 * exp(-inf) = 0
  zt = wave_sum(zt);
  const float logz = logf(zt);
  auto cand_of = [&](float x) { return raw ? x : __fadd_rn(bs, __fsub_rn(__fsub_rn(x, m), logz)); };
  float cg[GPL];
#pragma unroll
  for (int q = 0; q < GPL; ++q) cg[q] = (q * 64 + lane < G) ? cand_of(gm[q]) : -INFINITY;
  // R: every lane's best group value is the value of a distinct token; the k-th largest of those 64 is
  // reached by k tokens, so it is a valid threshold (at most the k-th largest group value, and close to it
  // when there are many more groups than k).  Ranked by (value, lane): 64 broadcasts, whatever k.
  float lm = -INFINITY;
#pragma unroll
  for (int q = 0; q < GPL; ++q) lm = fmaxf(lm, cg[q]);
  int lrank = 0;
#pragma unroll
  for (int c = 0; c < 64; ++c) {
    const float o = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, lm), c));
    lrank += (o > lm || (o == lm && c < lane)) ? 1 : 0;
  }
  const float R = wave_max(lrank == k - 1 ? lm : -INFINITY);   // fewer than k groups: -inf, every token passes
  // the groups that reach R
  int nq = 0;
#pragma unroll
  for (int q = 0; q < GPL; ++q) {
    const bool in = q * 64 + lane < G && cg[q] >= R;
    const unsigned long long mask = __ballot(in);
    if (in) {
      const int at = nq + __popcll(mask & ((1ull << lane) - 1ull));
      if (at < QMAX) ql_w[at] = q * 64 + lane;
    }
    nq += __popcll(mask);
  }
  __builtin_amdgcn_wave_barrier();   // the list is read by other lanes of this wavefront (LDS keeps a wavefront's order)
  const float* row = logits + (size_t)r * V;
  int nc = 0;
  if (nq <= QMAX) {
    // two groups per pass (lanes 0-31 one, lanes 32-63 the next), the logits of PB passes requested together
    constexpr int PB = 8;
    for (int p0 = 0; p0 < nq && nc <= CMAX; p0 += 2 * PB) {
      float xs[PB];
      int vs[PB];
#pragma unroll
      for (int u = 0; u < PB; ++u) {
        const int gi = p0 + 2 * u + (lane >> 5);
        vs[u] = gi < nq ? ql_w[min(gi, QMAX - 1)] * 32 + (lane & 31) : V;
        xs[u] = row[min(vs[u], V - 1)];
      }
#pragma unroll
      for (int u = 0; u < PB; ++u) {
        const float c = cand_of(xs[u]);
        const bool in = vs[u] < V && c >= R;
        const unsigned long long mask = __ballot(in);
        if (in) {
          const int at = nc + __popcll(mask & ((1ull << lane) - 1ull));
          if (at < CMAX) { cs_w[at] = c; ci_w[at] = vs[u]; }
        }
        nc += __popcll(mask);
      }
    }
  }
  __builtin_amdgcn_wave_barrier();
  if (nq <= QMAX && nc <= CMAX) {
    for (int c = lane; c < nc; c += 64) {
      const float sc = cs_w[c];
      const int v = ci_w[c];
      int rank = 0;
      for (int o = 0; o < nc; ++o) rank += precedes(cs_w[o], ci_w[o], sc, v) ? 1 : 0;
      if (rank < k) { os[rank] = sc; oi[rank] = v; }
    }
    if (lane >= nc && lane < k) { os[lane] = -INFINITY; oi[lane] = -1; }   // vocabulary smaller than k
    return;
  }
  // exact fallback: k rounds over the whole row, each the best token strictly after the previous winner
  float ps = INFINITY;
  int pi = -1;
  for (int round = 0; round < k; ++round) {
    float bsc = -INFINITY;
    int bi = 0x7fffffff;
    for (int v = lane; v < V; v += 64) {
      const float c = cand_of(row[v]);
      if (precedes(ps, pi, c, v) && (bi == 0x7fffffff || precedes(c, v, bsc, bi))) { bsc = c; bi = v; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float s2 = __shfl_xor(bsc, o, kWave);
      const int i2 = __shfl_xor(bi, o, kWave);
      if (i2 != 0x7fffffff && (bi == 0x7fffffff || precedes(s2, i2, bsc, bi))) { bsc = s2; bi = i2; }
    }
    if (bi == 0x7fffffff) {
      if (lane == 0) { os[round] = -INFINITY; oi[round] = -1; }
    } else {
      if (lane == 0) { os[round] = bsc; oi[round] = bi; }
      ps = bsc;
      pi = bi;
    }
  }
}

template <int GPL>
__global__ void __launch_bounds__(256) row_topk_groups_kernel(const float* __restrict__ logits,
                                                              const float* __restrict__ stats,
                                                              const float* __restrict__ score,
                                                              const int32_t* __restrict__ fin, int M, int V, int G,
                                                              int k, int eos, float* __restrict__ out_score,
                                                              int32_t* __restrict__ out_idx, int raw) {
  __shared__ int ql[4][kTopkGroupsQ];
  __shared__ float cs[4][kTopkGroupsC];
  __shared__ int ci[4][kTopkGroupsC];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + wave;
  if (r >= M) return;
  topk_groups_row<GPL>(logits, stats, score, fin, r, V, G, k, eos, out_score + (size_t)r * k, out_idx + (size_t)r * k, lane,
                       ql[wave], cs[wave], ci[wave], raw);
}

// beam search: k up to the beam limit; raw (sampling): up to the top-k limit (k rounds find the threshold)
bool topk_groups_supported(int V, int k, int raw) {
  return V >= 1 && V <= 65536 && k >= 1 && k <= (raw ? LSQ_MAX_TOPK_ : LSQ_MAX_BEAM_) && k <= kTopkGroupsQ;
}

hipError_t launch_row_topk_groups(const float* logits, const float* stats, const float* score, const int32_t* fin, int M,
                                  int V, int k, int eos, int raw, float* out_score, int32_t* out_idx, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  if (!topk_groups_supported(V, k, raw) || !stats || (!raw && (!score || !fin))) return hipErrorInvalidValue;
  const int G = (V + 31) / 32;
  dim3 g((M + 3) / 4), b(256);
  if (G <= 64 * 4) row_topk_groups_kernel<4><<<g, b, 0, s>>>(logits, stats, score, fin, M, V, G, k, eos, out_score, out_idx, raw);
  else if (G <= 64 * 16) row_topk_groups_kernel<16><<<g, b, 0, s>>>(logits, stats, score, fin, M, V, G, k, eos, out_score, out_idx, raw);
  else row_topk_groups_kernel<32><<<g, b, 0, s>>>(logits, stats, score, fin, M, V, G, k, eos, out_score, out_idx, raw);
  return hipGetLastError();
}

bool topk_supported(int V) { return V >= 1 && V <= 65536; }

template <typename T>
static hipError_t row_topk_t(const T* logits, const float* score, const int32_t* fin, int M, int V, int k,
                             int eos, int raw, float* os, int32_t* oi, hipStream_t s, const SearchGroups& gr) {
  if (V <= 2048)
    row_topk_kernel<T, 256, 1><<<M, 256, 0, s>>>(logits, score, fin, V, k, eos, raw, os, oi, gr);
  else if (V <= 8192)
    row_topk_kernel<T, 256, 4><<<M, 256, 0, s>>>(logits, score, fin, V, k, eos, raw, os, oi, gr);
  else if (V <= 32768)   // 512 threads x 64 tokens: two workgroups fit a CU, one loads while the other reduces
    row_topk_kernel<T, 512, 8><<<M, 512, 0, s>>>(logits, score, fin, V, k, eos, raw, os, oi, gr);
  else if (V <= 65536)
    row_topk_kernel<T, 1024, 8><<<M, 1024, 0, s>>>(logits, score, fin, V, k, eos, raw, os, oi, gr);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_row_topk(int dtype, const void* logits, const float* score, const int32_t* fin, int M,
                           int V, int k, int eos, int raw, float* out_score, int32_t* out_idx, hipStream_t s,
                           const SearchGroups& gr) {
  if (M <= 0) return hipSuccess;
  if (k < 1 || k > LSQ_MAX_TOPK_ || gr.kg < 1 || M % gr.kg != 0) return hipErrorInvalidValue;
  if (dtype == DT_F16) return row_topk_t<half_t>((const half_t*)logits, score, fin, M, V, k, eos, raw, out_score, out_idx, s, gr);
  return row_topk_t<float>((const float*)logits, score, fin, M, V, k, eos, raw, out_score, out_idx, s, gr);
}

// x[base + i] = E[tok[i]] * scale + pe[pos] for the k rows of a sentence (tok[i] < 0: row left alone), by one
// wavefront: the rows' 16-byte chunks are dealt out over the lanes and requested eight per lane at a time, so the
// k gathers travel together instead of one row after the other.  The arithmetic is embed_row's.
template <typename T>
__device__ __forceinline__ void next_input_rows(const NextInput& nx, const int* tok, int base, int k, int pos, int lane) {
  const int d = nx.d;
  const T* E = (const T*)nx.E;
  T* x = (T*)nx.x;
  const float* pe = nx.pe + (size_t)pos * d;
  if ((d & 7) != 0) {
    for (int i = 0; i < k; ++i)
      if (tok[i] >= 0) embed_row<T>(E + (size_t)tok[i] * d, pe, x + (size_t)(base + i) * d, d, nx.scale, lane, 64);
    return;
  }
  using raw_t = typename Vec8<T>::raw_t;
  constexpr int U = 8;
  const int cpr = d >> 3, total = k * cpr;
  for (int u0 = 0; u0 < total; u0 += 64 * U) {
    raw_t e[U];
    floatx4 pa[U], pb[U];
    int row[U], col[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = u0 + u * 64 + lane;
      const int i = min(idx, total - 1) / cpr;
      col[u] = (min(idx, total - 1) - i * cpr) * 8;
      row[u] = (idx < total && tok[i] >= 0) ? base + i : -1;
      e[u] = Vec8<T>::load_raw(E + (size_t)max(tok[i], 0) * d + col[u]);
      pa[u] = *reinterpret_cast<const floatx4*>(pe + col[u]);
      pb[u] = *reinterpret_cast<const floatx4*>(pe + col[u] + 4);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float v[8];
      Vec8<T>::unpack(e[u], v);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        v[c] = __fadd_rn(__fmul_rn(v[c], nx.scale), pa[u][c]);
        v[4 + c] = __fadd_rn(__fmul_rn(v[4 + c], nx.scale), pb[u][c]);
      }
      if (row[u] >= 0) Vec8<T>::store(x + (size_t)row[u] * d + col[u], v);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// One wavefront per sentence (per group of a sentence under diverse beam search: k is then the
// group width, the group's rows start at beam slot goff of the sentence's k_all).  Lane c < k*k owns
// survivor (beam c / k of the group, slot c % k).
// ALONE: the wavefront is the whole workgroup (its barriers are the workgroup's); otherwise other wavefronts of the
// workgroup have finished their part and this one orders its own LDS and memory traffic.
template <bool ALONE>
__device__ __forceinline__ void rerank_sync() {
  if constexpr (ALONE) {
    __syncthreads();
  } else {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  }
}

// cand_score / cand_idx: the sentence's k*k survivors at [(row - first row of the launch's unit) ...]: pointers to the
// pairs of row `base` (global memory, or LDS when the retrieve stage ran in the same workgroup).
template <bool ALONE>
__device__ __forceinline__ void rerank_sentence(const float* cand_score_b, const int32_t* cand_idx_b, const float* plain_b,
                                                float* __restrict__ score, int32_t* __restrict__ tokens,
                                                int32_t* __restrict__ len, int32_t* __restrict__ fin,
                                                int32_t* __restrict__ parent, const int32_t* __restrict__ cap,
                                                int32_t* __restrict__ active, int k, int V, int T1, int t_base,
                                                int32_t* __restrict__ step_state, int eos, int32_t* __restrict__ anc,
                                                const SearchGroups& gr, const NextInput& nx, int b, int lane,
                                                int* sh_parent, int* sh_tok, int& sh_unfinished, int& sh_taken) {
  const int t = t_base + (step_state ? step_state[0] : 0);
  const int kk = k * k;
  const int k_all = gr.k_all > 1 ? gr.k_all : k;           // rows of a sentence (k_all == 1: no groups)
  const int base = b * k_all + gr.goff;                    // first row of this group
  if (lane == 0) { sh_unfinished = 0; sh_taken = 0; }
  if (lane < LSQ_MAX_BEAM_) sh_tok[lane] = -1;
  // Everything the kernel reads is requested here, before any of it is used (one trip to memory
  // instead of one per phase): the candidates, the state of the beam a candidate continues (lane
  // c continues beam c / k whatever its rank turns out to be), the sentence's length cap and this
  // lane's first position of the k token histories and slab tables.
  // No request sits behind a test of something that is itself read from memory: lanes past the
  // k*k candidates repeat the last one and positions past the step repeat the last position of the
  // histories (both discarded below), so every load can leave before the step counter has arrived.
  const int cl = min(lane, kk - 1);
  const int j = cl / k;
  float s = cand_score_b[cl];
  float plain = plain_b ? plain_b[cl] : s;
  int tok = cand_idx_b[cl];
  const int plen = len[base + j], pfin = fin[base + j];
  const int cap_b = cap[b];
  int p = lane;
  int h[LSQ_MAX_BEAM_], ha[LSQ_MAX_BEAM_];
  auto fetch = [&]() {
    const int pc = min(p, T1 - 1);
#pragma unroll
    for (int i = 0; i < LSQ_MAX_BEAM_; ++i)
      if (i < k) {
        h[i] = tokens[(size_t)(base + i) * T1 + pc];
        ha[i] = anc ? anc[(size_t)(base + i) * T1 + pc] : 0;
      }
  };
  fetch();
  if (lane >= kk) { s = -INFINITY; plain = -INFINITY; tok = -1; }
  long flat = -1;
  if (tok >= 0) flat = (long)(gr.goff + j) * V + tok;
  // rank among the k*k candidates: lane c's pair is read straight from its registers
  int rank = 0;
  for (int c = 0; c < kk; ++c) {
    const float s2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, s), c));
    const int t2 = __builtin_amdgcn_readlane(tok, c);
    const long f2 = t2 >= 0 ? (long)(gr.goff + c / k) * V + t2 : -1;
    if (f2 >= 0 && (s2 > s || (s2 == s && f2 < flat))) ++rank;
  }
  const bool win = flat >= 0 && rank < k;
  if (win) sh_parent[rank] = j;
  rerank_sync<ALONE>();
  // token histories, positions 0..t, and the table that says which slab holds position p of each
  // history (cache refreshing without moving the cache; position t+1 is written by the row
  // itself): every lane has all k beams of a position, then writes those that change
  for (; p <= t && p < T1;) {
#pragma unroll
    for (int i = 0; i < LSQ_MAX_BEAM_; ++i)
      if (i < k) {
        int src = sh_parent[i], val = 0, vala = 0;
#pragma unroll
        for (int jj = 0; jj < LSQ_MAX_BEAM_; ++jj)
          if (jj == src) { val = h[jj]; vala = ha[jj]; }
        if (src != i) {
          tokens[(size_t)(base + i) * T1 + p] = val;
          if (anc) anc[(size_t)(base + i) * T1 + p] = vala;
        }
      }
    p += 64;
    if (p <= t && p < T1) fetch();   // a history longer than 64 positions: one more trip per 64
  }
  if (anc && lane < k && t + 1 < T1) anc[(size_t)(base + lane) * T1 + t + 1] = gr.goff + lane;
  rerank_sync<ALONE>();
  if (win) {
    const int row = base + rank;
    int nlen = plen, nfin = pfin;
    sh_tok[rank] = pfin ? eos : tok;   // what the row feeds the decoder next (a finished row: anything valid)
    if (!pfin) {
      nlen = plen + 1;
      tokens[(size_t)row * T1 + nlen] = tok;
      nfin = (tok == eos || nlen >= cap_b) ? 1 : 0;
      // a live hypothesis that took a token: later groups of this sentence are steered away from it
      if (gr.pen_tok && !gr.last && plain != -INFINITY) {
        const int at = atomicAdd(&sh_taken, 1);
        gr.pen_tok[(size_t)b * gr.pen_ld + gr.pen_n[b] + at] = tok;
      }
    }
    len[row] = nlen;
    fin[row] = nfin;
    score[row] = plain;
    parent[row] = gr.goff + j;
    if (!nfin) sh_unfinished = 1;
  }
  rerank_sync<ALONE>();
  // The next step's decoder input of these rows (one launch less per step).  A row that no candidate won
  // (fewer live candidates than beams) embeds nothing: it is dead and stays so.
  if (nx.E && t + 1 < T1 - 1) {
    if (nx.dtype == DT_F16) next_input_rows<half_t>(nx, sh_tok, base, k, t + 1, lane);
    else next_input_rows<float>(nx, sh_tok, base, k, t + 1, lane);
  }
  if (gr.pen_n && lane == 0) gr.pen_n[b] = gr.last ? 0 : gr.pen_n[b] + sh_taken;
  if (!gr.last) return;
  // the sentence is still active if any hypothesis of any group is unfinished (the other groups'
  // rows were settled by earlier launches of this step)
  int others = 0;
  if (lane < k_all && (lane < gr.goff || lane >= gr.goff + k)) others = fin[b * k_all + lane] ? 0 : 1;
  others = __any(others) ? 1 : 0;
  if (lane == 0) {
    if (sh_unfinished || others) atomicAdd(step_state ? active + t : active, 1);   // per-step counters, or the caller's one
    if (step_state) {
      // the last sentence to get here advances the step counter: every workgroup read it at its
      // start, before its own increment, and the only other readers are kernels launched later
      if (atomicAdd(&step_state[1], 1) == (int)gridDim.x - 1) {
        step_state[1] = 0;
        step_state[0] = t + 1 - t_base;
      }
    }
  }
}

__global__ void __launch_bounds__(64) beam_refine_kernel(const float* __restrict__ cand_score,
                                                         const int32_t* __restrict__ cand_idx,
                                                         float* __restrict__ score, int32_t* __restrict__ tokens,
                                                         int32_t* __restrict__ len, int32_t* __restrict__ fin,
                                                         int32_t* __restrict__ parent,
                                                         const int32_t* __restrict__ cap,
                                                         int32_t* __restrict__ active, int k, int V, int T1,
                                                         int t_base, int32_t* __restrict__ step_state, int eos,
                                                         int32_t* __restrict__ anc, SearchGroups gr, NextInput nx) {
  __shared__ int sh_parent[LSQ_MAX_BEAM_], sh_tok[LSQ_MAX_BEAM_];
  __shared__ int sh_unfinished, sh_taken;
  const int b = blockIdx.x;
  const int k_all = gr.k_all > 1 ? gr.k_all : k;
  const size_t first = ((size_t)b * k_all + gr.goff) * k;   // the pairs of the unit's first row
  rerank_sentence<true>(cand_score + first, cand_idx + first, gr.out_plain ? gr.out_plain + first : nullptr, score, tokens, len,
                        fin, parent, cap, active, k, V, T1, t_base, step_state, eos, anc, gr, nx, b, (int)threadIdx.x,
                        sh_parent, sh_tok, sh_unfinished, sh_taken);
}

// Retrieve and re-rank in one launch (plain beam search from the logit product's group statistics): a workgroup
// per sentence, wavefront w retrieves row w's k best into LDS, the first wavefront then re-ranks the sentence.
template <int GPL>
__global__ void __launch_bounds__(64 * LSQ_MAX_BEAM_) retrieve_rerank_kernel(
    const float* __restrict__ logits, const float* __restrict__ stats, float* __restrict__ score, int32_t* __restrict__ tokens,
    int32_t* __restrict__ len, int32_t* __restrict__ fin, int32_t* __restrict__ parent, const int32_t* __restrict__ cap,
    int32_t* __restrict__ active, int k, int V, int G, int T1, int32_t* __restrict__ step_state, int eos,
    int32_t* __restrict__ anc, NextInput nx, float* __restrict__ cand_out_s, int32_t* __restrict__ cand_out_i) {
  __shared__ int ql[LSQ_MAX_BEAM_][kTopkGroupsQ];
  __shared__ float cs[LSQ_MAX_BEAM_][kTopkGroupsC];
  __shared__ int ci[LSQ_MAX_BEAM_][kTopkGroupsC];
  __shared__ float cand_s[LSQ_MAX_BEAM_ * LSQ_MAX_BEAM_];
  __shared__ int cand_i[LSQ_MAX_BEAM_ * LSQ_MAX_BEAM_];
  __shared__ int sh_parent[LSQ_MAX_BEAM_], sh_tok[LSQ_MAX_BEAM_];
  __shared__ int sh_unfinished, sh_taken;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int b = blockIdx.x;
  topk_groups_row<GPL>(logits, stats, score, fin, b * k + wave, V, G, k, eos, cand_s + wave * k, cand_i + wave * k, lane,
                       ql[wave], cs[wave], ci[wave]);
  __syncthreads();   // blockDim.x = 64 k: every wavefront has a row
  if (cand_out_s && (int)threadIdx.x < k * k) {   // the survivors, for whoever inspects them afterwards
    cand_out_s[(size_t)b * k * k + threadIdx.x] = cand_s[threadIdx.x];
    cand_out_i[(size_t)b * k * k + threadIdx.x] = cand_i[threadIdx.x];
  }
  if (wave != 0) return;
  rerank_sentence<false>(cand_s, cand_i, nullptr, score, tokens, len, fin, parent, cap, active, k, V, T1, 0, step_state, eos,
                         anc, one_group(), nx, b, lane, sh_parent, sh_tok, sh_unfinished, sh_taken);
}

hipError_t launch_beam_refine(const float* cand_score, const int32_t* cand_idx, float* score, int32_t* tokens,
                              int32_t* len, int32_t* fin, int32_t* parent, const int32_t* cap,
                              int32_t* active, int batch, int k, int V, int T, int t_base, int32_t* step_state,
                              int eos, int32_t* anc, hipStream_t s, const SearchGroups& gr, const NextInput& nx) {
  if (batch <= 0) return hipSuccess;
  if (k < 1 || k > LSQ_MAX_BEAM_) return hipErrorInvalidValue;
  if (gr.k_all > 1 && (gr.kg != k || gr.k_all % k != 0 || gr.k_all > LSQ_MAX_BEAM_ || gr.goff % k != 0 || gr.goff + k > gr.k_all))
    return hipErrorInvalidValue;
  beam_refine_kernel<<<batch, 64, 0, s>>>(cand_score, cand_idx, score, tokens, len, fin, parent, cap, active,
                                          k, V, T + 1, t_base, step_state, eos, anc, gr, nx);
  return hipGetLastError();
}

hipError_t launch_retrieve_rerank(const float* logits, const float* stats, float* score, int32_t* tokens, int32_t* len,
                                  int32_t* fin, int32_t* parent, const int32_t* cap, int32_t* active, int batch, int k,
                                  int V, int T, int32_t* step_state, int eos, int32_t* anc, hipStream_t s,
                                  const NextInput& nx, float* cand_score, int32_t* cand_idx) {
  if (batch <= 0) return hipSuccess;
  if (!topk_groups_supported(V, k, 0) || !stats || !step_state) return hipErrorInvalidValue;
  const int G = (V + 31) / 32;
  dim3 g(batch), b(64 * k);
#define LSQ_RR(GPL_)                                                                                                     \
  retrieve_rerank_kernel<GPL_><<<g, b, 0, s>>>(logits, stats, score, tokens, len, fin, parent, cap, active, k, V, G, T + 1, \
                                               step_state, eos, anc, nx, cand_score, cand_idx)
  if (G <= 64 * 4) LSQ_RR(4);
  else if (G <= 64 * 16) LSQ_RR(16);
  else LSQ_RR(32);
#undef LSQ_RR
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// In-place gather of cache rows by parent.  A thread owns the same 16-byte column of all k rows
// of one sentence: it loads the rows that some other row needs, then overwrites the rows whose
// parent is not themselves.  No other thread touches those bytes, so no double buffer is needed,
// rows that keep their own history cost nothing, and a sentence whose beams did not move is
// skipped outright.  grid = (chunks of the used prefix, sentences, layers).
template <int KB>
__global__ void __launch_bounds__(256) cache_reorder_kernel(uint4* __restrict__ cache,
                                                            const int32_t* __restrict__ parent, int k,
                                                            long row_vecs, long pos_vecs, int npos_base,
                                                            const int32_t* __restrict__ tp, long layer_vecs) {
  const int b = blockIdx.y;
  const long used_vecs = (long)(npos_base + (tp ? *tp : 0)) * pos_vecs;
  if ((long)blockIdx.x * 1024 >= used_vecs) return;
  int par[KB];
  unsigned need = 0, moved = 0;
#pragma unroll
  for (int i = 0; i < KB; ++i) {
    par[i] = i < k ? parent[b * k + i] : i;
    if (par[i] != i) { need |= 1u << par[i]; moved |= 1u << i; }
  }
  if (!moved) return;
  uint4* base = cache + (size_t)blockIdx.z * layer_vecs + (size_t)b * k * row_vecs;
  for (long v = (long)blockIdx.x * 1024 + threadIdx.x; v < used_vecs && v < (long)(blockIdx.x + 1) * 1024;
       v += 256) {
    uint4 val[KB];
#pragma unroll
    for (int i = 0; i < KB; ++i)
      if (need >> i & 1) val[i] = base[i * row_vecs + v];
#pragma unroll
    for (int i = 0; i < KB; ++i)
      if (moved >> i & 1) {
        uint4 o = val[0];
#pragma unroll
        for (int jj = 1; jj < KB; ++jj)
          if (par[i] == jj) o = val[jj];
        base[i * row_vecs + v] = o;
      }
  }
}

hipError_t launch_cache_reorder(int dtype, void* cache, const int32_t* parent, int layers, int batch,
                                int rows_total, int k, int T, int d, int npos_base, const int32_t* tp,
                                int npos_max, hipStream_t s) {
  if (batch <= 0 || layers <= 0 || npos_max <= 0 || k <= 1) return hipSuccess;
  size_t esz = dtype == DT_F16 ? 2 : 4;
  if ((d * esz) % 16 != 0 || k > LSQ_MAX_BEAM_) return hipErrorInvalidValue;
  long pos_vecs = (long)d * esz / 16;
  long row_vecs = (long)T * pos_vecs, used = (long)npos_max * pos_vecs;
  long layer_vecs = (long)rows_total * row_vecs;   // a layer holds rows_total rows; the first batch*k are reordered
  dim3 grid((unsigned)((used + 1023) / 1024), batch, layers), blk(256);
  if (k <= 4)
    cache_reorder_kernel<4><<<grid, blk, 0, s>>>((uint4*)cache, parent, k, row_vecs, pos_vecs, npos_base, tp, layer_vecs);
  else
    cache_reorder_kernel<8><<<grid, blk, 0, s>>>((uint4*)cache, parent, k, row_vecs, pos_vecs, npos_base, tp, layer_vecs);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
__global__ void beam_reset_kernel(float* __restrict__ score, int32_t* __restrict__ tokens, int32_t* __restrict__ len,
                                  int32_t* __restrict__ fin, int32_t* __restrict__ active_counts,
                                  int32_t* __restrict__ step_state, int32_t* __restrict__ anc,
                                  int32_t* __restrict__ pen_n, int M, int k, int kg, int T1, int bos, int pad) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < 3) step_state[i] = 0;   // [0] position counter, [1] arrival counter, [2] position of step 0
  if (i < M * T1) tokens[i] = (i % T1 == 0) ? bos : pad;
  if (i < M) {
    score[i] = (i % kg == 0) ? 0.f : -INFINITY;   // one live hypothesis per search group
    if (pen_n && i % k == 0) pen_n[i / k] = 0;
    len[i] = 0;
    fin[i] = 0;
    if (anc) anc[(size_t)i * T1] = i % k;   // position 0 is written by the row itself
  }
  if (i < T1) active_counts[i] = 0;
}

hipError_t launch_beam_reset(float* score, int32_t* tokens, int32_t* len, int32_t* fin, int32_t* active_counts,
                             int32_t* step_state, int32_t* anc, int32_t* pen_n, int batch, int k, int kg, int T,
                             int bos, int pad, hipStream_t s) {
  int M = batch * k, n = M * (T + 1);
  if (kg < 1 || k % kg != 0) return hipErrorInvalidValue;
  beam_reset_kernel<<<(n + 255) / 256, 256, 0, s>>>(score, tokens, len, fin, active_counts, step_state, anc, pen_n, M,
                                                    k, kg, T + 1, bos, pad);
  return hipGetLastError();
}

// Length-normalised score and best-first order per sentence; one wavefront per sentence.
__global__ void __launch_bounds__(64) finalize_kernel(const float* __restrict__ score,
                                                      const int32_t* __restrict__ tokens,
                                                      const int32_t* __restrict__ len, int32_t* __restrict__ out_ids,
                                                      int32_t* __restrict__ out_lens, float* __restrict__ out_scores,
                                                      const int32_t* __restrict__ sentence_order, int k, int T,
                                                      float alpha, int pad, int first) {
  __shared__ int order[LSQ_MAX_BEAM_];
  const int b = blockIdx.x, lane = threadIdx.x;
  const int ob = sentence_order[b];   // where the caller expects this sentence
  float f = -INFINITY;
  int n = 0;
  if (lane < k) {
    n = len[b * k + lane] - (first - 1);   // len = index of the last token in the history
    float sc = score[b * k + lane];
    float den = n > 0 ? (alpha == 1.0f ? (float)n : powf((float)n, alpha)) : 1.0f;
    f = sc / den;
  }
  int rank = 0;
  for (int c = 0; c < k; ++c) {
    float f2 = __shfl(f, c, kWave);
    if (f2 > f || (f2 == f && c < lane)) ++rank;
  }
  if (lane < k) {
    order[rank] = lane;
    out_lens[ob * k + rank] = n;
    out_scores[ob * k + rank] = f;
  }
  __syncthreads();
  for (int i = 0; i < k; ++i) {
    int src = b * k + order[i];
    int n_i = len[src] - (first - 1);
    for (int p = lane; p < T; p += 64)
      out_ids[(size_t)(ob * k + i) * T + p] = p < n_i ? tokens[(size_t)src * (T + 1) + first + p] : pad;
  }
}

hipError_t launch_finalize(const float* score, const int32_t* tokens, const int32_t* len, int32_t* out_ids,
                           int32_t* out_lens, float* out_scores, const int32_t* sentence_order, int batch, int k,
                           int T, float alpha, int pad, int first, hipStream_t s) {
  finalize_kernel<<<batch, 64, 0, s>>>(score, tokens, len, out_ids, out_lens, out_scores, sentence_order, k, T,
                                       alpha, pad, first);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Top-k sampling (the paper's sampling decoding, sec. 3.4): one thread per row.  The row's k largest
// logits arrive ranked (logit descending, token ascending); p = softmax over those k, cut to the
// shortest prefix whose mass reaches topp when topp < 1;
// u = (philox4x32_10(key = seed, counter = (step, row, 0, 0))[0] >> 8) * 2^-24; the token is the
// first j whose cumulative p exceeds u * (sum of the kept p).  Appends it to the history, adds log p to the
// row's score, and the last thread to finish advances the position counter.
__device__ __forceinline__ unsigned philox4x32_10_first(unsigned c0, unsigned c1, unsigned c2, unsigned c3,
                                                        unsigned k0, unsigned k1) {
  const unsigned M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const unsigned hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    const unsigned hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    c0 = hi1 ^ c1 ^ k0; c1 = lo1;
    c2 = hi0 ^ c3 ^ k1; c3 = lo0;
    k0 += W0; k1 += W1;
  }
  return c0;
}

// Encoder-decoder models (fin given): a finished sentence draws nothing and keeps its state; EOS or
// the sentence's cap finishes one; the uniform number is that of the sentence's place in the
// caller's batch (order[r]); active[t] counts the sentences still unfinished after the step.
// Decoder-only models (fin == nullptr): every row draws at every step, n_new tokens in all.
// One row's draw from its k ranked candidates (global memory or LDS) by one thread; returns whether the row is
// still unfinished (always false for decoder-only models, which count differently) and the token through tok_out.
__device__ __forceinline__ bool sample_row(const float* cl, const int32_t* ci, int r, int32_t* __restrict__ tokens,
                                           int32_t* __restrict__ len, float* __restrict__ logp, int k, float topp, int T1,
                                           unsigned seed_lo, unsigned seed_hi, int pos, int t, int32_t* __restrict__ fin,
                                           const int32_t* __restrict__ cap, const int32_t* __restrict__ order, int eos,
                                           int& tok_out) {
  float e[LSQ_MAX_TOPK_], cum[LSQ_MAX_TOPK_];
  const float l0 = cl[0];
  float run = 0.f;
  for (int j = 0; j < k; ++j) {
    e[j] = expf(cl[j] - l0);
    run += e[j];
    cum[j] = run;
  }
  // nucleus inside the candidates: the shortest ranked prefix whose mass reaches topp of the total
  int n = k;
  if (topp < 1.0f) {
    const float thresh = __fmul_rn(topp, run);
    n = 1;
    while (n < k && !(cum[n - 1] >= thresh)) ++n;
  }
  const float total = cum[n - 1];
  const unsigned word = philox4x32_10_first((unsigned)t, (unsigned)(order ? order[r] : r), 0u, 0u, seed_lo, seed_hi);
  const float u = (float)(word >> 8) * 5.9604644775390625e-08f;   // 2^-24
  const float target = __fmul_rn(u, total);
  int j = 0;
  while (j < n - 1 && !(cum[j] > target)) ++j;
  const int tok = ci[j];
  tokens[(size_t)r * T1 + pos + 1] = tok;
  len[r] = pos + 1;
  logp[r] += logf(e[j] / total);
  tok_out = tok;
  if (!fin) return false;
  const bool unfinished = !(tok == eos || pos + 1 >= cap[r]);
  fin[r] = unfinished ? 0 : 1;
  return unfinished;
}

__global__ void __launch_bounds__(64) sample_kernel(const float* __restrict__ cand_logit,
                                                    const int32_t* __restrict__ cand_idx,
                                                    int32_t* __restrict__ tokens, int32_t* __restrict__ len,
                                                    float* __restrict__ logp, int32_t* __restrict__ active,
                                                    int32_t* __restrict__ step_state, int rows, int k, float topp,
                                                    int T1, unsigned seed_lo, unsigned seed_hi, int n_new,
                                                    int32_t* __restrict__ fin, const int32_t* __restrict__ cap,
                                                    const int32_t* __restrict__ order, int eos) {
  const int r = blockIdx.x * 64 + threadIdx.x;
  const int pos = step_state[0], t = pos - step_state[2];   // position of the token just fed; step index
  bool unfinished = false;
  int tok;
  if (r < rows && !(fin && fin[r]))
    unfinished = sample_row(cand_logit + (size_t)r * k, cand_idx + (size_t)r * k, r, tokens, len, logp, k, topp, T1, seed_lo,
                            seed_hi, pos, t, fin, cap, order, eos, tok);
  const int alive = __popcll(__ballot(unfinished));
  if (threadIdx.x == 0) {
    if (fin && alive) atomicAdd(active + t, alive);
    __threadfence();
    if (atomicAdd(&step_state[1], 1) == (int)gridDim.x - 1) {
      step_state[1] = 0;
      if (!fin) active[t] = (t + 1 < n_new) ? rows : 0;
      step_state[0] = pos + 1;
    }
  }
}

// Retrieve (the k largest logits from the logit product's group statistics) and draw in one launch: a wavefront
// per row, four rows per workgroup; the candidates stay in LDS, the first lane draws.  nx.E given (encoder-decoder
// models): the row's next decoder input is written as well (a finished row: nothing; its logits are not used).
template <int GPL>
__global__ void __launch_bounds__(256) retrieve_sample_kernel(const float* __restrict__ logits, const float* __restrict__ stats,
                                                              int32_t* __restrict__ tokens, int32_t* __restrict__ len,
                                                              float* __restrict__ logp, int32_t* __restrict__ active,
                                                              int32_t* __restrict__ step_state, int rows, int V, int G, int k,
                                                              float topp, int T1, unsigned seed_lo, unsigned seed_hi,
                                                              int n_new, int32_t* __restrict__ fin,
                                                              const int32_t* __restrict__ cap,
                                                              const int32_t* __restrict__ order, int eos, NextInput nx,
                                                              float* __restrict__ cand_out_s, int32_t* __restrict__ cand_out_i) {
  __shared__ int ql[4][kTopkGroupsQ];
  __shared__ float cs[4][kTopkGroupsC];
  __shared__ int ci[4][kTopkGroupsC];
  __shared__ float cand_s[4][LSQ_MAX_TOPK_];
  __shared__ int cand_i[4][LSQ_MAX_TOPK_];
  __shared__ int next_tok[4];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + wave;
  if (r >= rows) return;
  const int pos = step_state[0], t = pos - step_state[2];
  const bool done = fin && fin[r];   // the same in every lane
  if (!done) {
    topk_groups_row<GPL>(logits, stats, nullptr, nullptr, r, V, G, k, eos, cand_s[wave], cand_i[wave], lane, ql[wave], cs[wave],
                         ci[wave], 1);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  }
  if (!done && cand_out_s && lane < k) {   // the candidates, for whoever inspects them afterwards
    cand_out_s[(size_t)r * k + lane] = cand_s[wave][lane];
    cand_out_i[(size_t)r * k + lane] = cand_i[wave][lane];
  }
  bool unfinished = false;
  if (lane == 0) {
    int tok = -1;
    if (!done)
      unfinished = sample_row(cand_s[wave], cand_i[wave], r, tokens, len, logp, k, topp, T1, seed_lo, seed_hi, pos, t, fin, cap,
                              order, eos, tok);
    next_tok[wave] = tok;
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  if (nx.E && pos + 1 < T1 - 1) {
    if (nx.dtype == DT_F16) next_input_rows<half_t>(nx, &next_tok[wave], r, 1, pos + 1, lane);
    else next_input_rows<float>(nx, &next_tok[wave], r, 1, pos + 1, lane);
  }
  if (lane == 0) {
    if (fin && unfinished) atomicAdd(active + t, 1);
    __threadfence();
    if (atomicAdd(&step_state[1], 1) == rows - 1) {   // one count per row: the last row advances the position
      step_state[1] = 0;
      if (!fin) active[t] = (t + 1 < n_new) ? rows : 0;
      step_state[0] = pos + 1;
    }
  }
}

hipError_t launch_sample(const float* cand_logit, const int32_t* cand_idx, int32_t* tokens, int32_t* len,
                         float* logp, int32_t* active, int32_t* step_state, int rows, int k, float topp, int T,
                         unsigned long long seed, int n_new, hipStream_t s, int32_t* fin, const int32_t* cap,
                         const int32_t* order, int eos) {
  if (rows <= 0) return hipSuccess;
  if (k < 1 || k > LSQ_MAX_TOPK_ || !(topp > 0.f) || (fin && !cap)) return hipErrorInvalidValue;
  sample_kernel<<<(rows + 63) / 64, 64, 0, s>>>(cand_logit, cand_idx, tokens, len, logp, active, step_state, rows, k,
                                                topp, T + 1, (unsigned)(seed & 0xFFFFFFFFull), (unsigned)(seed >> 32),
                                                n_new, fin, cap, order, eos);
  return hipGetLastError();
}

hipError_t launch_retrieve_sample(const float* logits, const float* stats, int32_t* tokens, int32_t* len, float* logp,
                                  int32_t* active, int32_t* step_state, int rows, int V, int k, float topp, int T,
                                  unsigned long long seed, int n_new, hipStream_t s, int32_t* fin, const int32_t* cap,
                                  const int32_t* order, int eos, const NextInput& nx, float* cand_score, int32_t* cand_idx) {
  if (rows <= 0) return hipSuccess;
  if (!topk_groups_supported(V, k, 1) || !stats || !(topp > 0.f) || (fin && !cap)) return hipErrorInvalidValue;
  const int G = (V + 31) / 32;
  dim3 g((rows + 3) / 4), b(256);
  const unsigned lo = (unsigned)(seed & 0xFFFFFFFFull), hi = (unsigned)(seed >> 32);
#define LSQ_RS(GPL_)                                                                                                    \
  retrieve_sample_kernel<GPL_><<<g, b, 0, s>>>(logits, stats, tokens, len, logp, active, step_state, rows, V, G, k, topp, \
                                               T + 1, lo, hi, n_new, fin, cap, order, eos, nx, cand_score, cand_idx)
  if (G <= 64 * 4) LSQ_RS(4);
  else if (G <= 64 * 16) LSQ_RS(16);
  else LSQ_RS(32);
#undef LSQ_RS
  return hipGetLastError();
}

}  // namespace lsq
