// Internal declarations shared by the translation units of liblsq.so.
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>
#include <stdint.h>

namespace lsq {

enum { DT_F32 = 0, DT_F16 = 1 };

typedef _Float16 half_t;
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;
constexpr int LSQ_MAX_BEAM_ = 8;   // k*k survivors of one sentence fit one wavefront
constexpr int LSQ_MAX_TOPK_ = 32;  // per-row retrieve width (sampling draws from up to this many candidates)

// Where a GEMM writes: output column n belongs to segment s = n / seg_n and goes to
// ptr[s] + m * ld[s] + (n - s * seg_n).  One segment for an ordinary matrix; three for the
// fused Q | K | V projection whose K and V columns land directly in the caches.
struct GemmOut {
  void* ptr[3];
  long ld[3];
  int seg_n;
  int f32_out;   // fp16 GEMM only: write the fp32 accumulators unrounded (vocabulary logits)
  // Optional step-dependent offset: segment s is shifted by (*tpos) * tmul[s] elements, with *tpos
  // read on the device (the decode-step counter), so the same launch serves every step.
  const int32_t* tpos;
  long tmul[3];
  // Optional, fp32 output of a float16 product only (vocabulary logits): for every row and every group of 32
  // consecutive output columns the pair (largest value, sum of exp(value - largest)) at
  // stats[(m * stats_groups + n / 32) * 2]: the group maxima of the retrieve stage (paper sec. 2.2) and the
  // softmax normaliser, taken where the logits are made.  Every float16 product kernel but the direct-to-LDS one fills it (gemm_writes_stats).
  float* stats;
  int stats_groups;
};

inline GemmOut plain_out(void* c, int N) {
  GemmOut o;
  o.ptr[0] = c; o.ptr[1] = nullptr; o.ptr[2] = nullptr;
  o.ld[0] = N; o.ld[1] = 0; o.ld[2] = 0;
  o.seg_n = N;
  o.f32_out = 0;
  o.tpos = nullptr;
  o.tmul[0] = o.tmul[1] = o.tmul[2] = 0;
  o.stats = nullptr; o.stats_groups = 0;
  return o;
}

// Every launcher enqueues on `s` and returns hipGetLastError().
// act: 0 none, 1 ReLU, 2 tanh-GELU
hipError_t launch_gemm(int dtype, const void* A, const void* B, const void* bias, const GemmOut& out,
                       int M, int N, int K, int act, hipStream_t s, bool b_packed = false);

// whether launch_gemm's kernel for this shape fills out.stats (float16 operands, fp32 output)
bool gemm_writes_stats(int dtype, int M, int N, int K);

int gemm_partial_splits(int dtype, int M, int N, int K);

// float16 weights in fragment order ([column block of 32][k-step of 16][lane][8 halves], rows past N
// zero) for the products of at most 64 rows.  launch_pack_weights makes the copy (gemm_packed_bytes
// of it; K a multiple of 16); after gemm_register_packed every product launched with the row-major
// pointer and the same N, K finds it.  launch_gemm's b_packed says B itself is such a copy.
size_t gemm_packed_bytes(int N, int K);
hipError_t launch_pack_weights(const void* plain, void* packed, int N, int K, hipStream_t s);
void gemm_register_packed(const void* plain, const void* packed, int N, int K);
void gemm_clear_packed();
// the registered fragment-ordered copy of a row-major matrix, or nullptr
const void* gemm_packed_weights(const void* plain, int N, int K);

// A product that makes its own input: A = LayerNorm(x_old + sum of `splits` fp32 slabs P[s][M][K] + bias) * g + b,
// rounded to float16; the rows are also written to x_new (not the same buffer as x_old).  For the few-row end
// of a batch only: see gemm_ln_supported.
struct LnInput {
  const float* P;
  int splits;
  const half_t* bias;
  const half_t* g;
  const half_t* b;
  const half_t* x_old;
  half_t* x_new;
  float eps;
  int pre;   // attention blocks only: pre-LN arithmetic (see block_row); the products take 0
};
bool gemm_ln_supported(int dtype, int M, int K);
hipError_t launch_gemm_ln(const LnInput& ln, const void* B, const void* bias, const GemmOut& out, int M, int N,
                          int K, int act, hipStream_t s);
hipError_t launch_gemm_partials(int dtype, const void* A, const void* B, float* P, int M, int N, int K,
                                int splits, hipStream_t s);

// x = E[id] * scale + pe[position]
hipError_t launch_embed_rows(int dtype, const void* E, const float* pe, const int32_t* ids,
                             const int32_t* pos, void* x, int rows, int d, float scale, hipStream_t s);
hipError_t launch_embed_last(int dtype, const void* E, const float* pe, const int32_t* tokens,
                             const int32_t* len, void* x, int rows, int d, int T, const int32_t* tp,
                             float scale, hipStream_t s);
// launch_embed_last followed by the pre-LN kernel without slabs (y = LN(x) * g + b), in one launch; same bits
bool embed_layernorm_supported(int d);
hipError_t launch_embed_layernorm(int dtype, const void* E, const float* pe, const int32_t* tokens, const int32_t* len,
                                  void* x, void* y, const void* g, const void* b, int rows, int d, int T,
                                  const int32_t* tp, float scale, float eps, hipStream_t s);
hipError_t launch_scatter_kv(int dtype, const void* qkv, const int32_t* sent, const int32_t* pos, void* Kc,
                             void* Vc, int rows, int d, int T, hipStream_t s);
// x_in (post-LN only): the residual is read from there instead of x, which is then only written
hipError_t launch_add_layernorm_partials(int dtype, void* x, void* y, const float* P, int splits,
                                         const void* bias, const void* g, const void* b, int rows, int d,
                                         float eps, hipStream_t s, const void* x_in = nullptr);

// nkeys = nkeys_base + (tp ? *tp : 0), with *tp read on the device.  anc != null: position j of row
// r's history is in slab (r / beam) * beam + anc[r * anc_ld + j] instead of slab r.
hipError_t launch_self_attention(int dtype, const void* q, const void* Kc, const void* Vc, void* out,
                                 int rows, int H, int d, int T, int nkeys_base, const int32_t* tp,
                                 const int32_t* anc, int beam, int anc_ld, hipStream_t s);
// smax: the longest of len[] as known to the host, or an upper bound of it; it only picks the launch geometry:
// cross_attention_splits(batch * H, smax) says whether a (sentence, head) gets four wavefronts instead of one
bool cross_attention_splits(int units, int smax);
hipError_t launch_cross_attention(int dtype, const void* q, const void* kv, const int32_t* off,
                                  const int32_t* len, void* out, int batch, int beam, int H, int d, int smax,
                                  hipStream_t s);
// Few rows alive (at most 64, beams of 4 at most, head size 64, float16): the
// cross-attention kernel makes its own queries, q = LayerNorm(x_old + partial sums + bias) . Wq^T
// + bq for the head it serves, from the fragment-ordered copy of Wq (gemm_packed_weights), instead
// of a product kernel of 32 workgroups followed by an attention kernel.  The workgroups of head 0
// write the normalised rows to ln.x_new.
// Attention sublayers in one launch each, for at most 64 rows (kernels_attn.hip): self_block = [LayerNorm] + QKV slice +
// cache append + self-attention + the head's share of the output projection; cross_block = LayerNorm + query slice +
// cross-attention + the head's share of the output projection.  P_out: [H][batch*beam][d] float partial sums.
bool attention_blocks_supported(int dtype, int rows, int beam, int H, int d);
hipError_t launch_self_block(const LnInput& ln, const void* Wqkv_packed, const void* bqkv, const void* Wo_packed,
                             void* Kc, void* Vc, const int32_t* anc, const int32_t* tp, int nkeys_base, float* P_out,
                             int batch, int beam, int H, int d, int T, hipStream_t s);
hipError_t launch_cross_block(const LnInput& ln, const void* Wq_packed, const void* bq, const void* Wo_packed,
                              const void* kv, const int32_t* off, const int32_t* len, float* P_out, int batch, int beam,
                              int H, int d, hipStream_t s);
bool cross_attention_ln_supported(int dtype, int rows, int beam, int H, int d);
hipError_t launch_cross_attention_ln(const LnInput& ln, const void* Wq_packed, const void* bq, const void* kv,
                                     const int32_t* off, const int32_t* len, void* out, int batch, int beam,
                                     int H, int d, hipStream_t s);
// More than 64 rows alive (beams of 4 at most, head size 64, float16, d <= 1024): query product and cross-attention
// in one launch; x holds the normalised rows.
bool cross_attention_q_supported(int dtype, int rows, int beam, int H, int d);
bool cross_attention_q_worthwhile(int batch, int beam, int H);   // where it is ahead of the two separate launches
hipError_t launch_cross_attention_q(const void* x, const void* Wq_packed, const void* bq, const void* kv,
                                    const int32_t* off, const int32_t* len, void* out, int batch, int beam, int H,
                                    int d, hipStream_t s);
hipError_t launch_encoder_attention(int dtype, const void* qkv, const int32_t* row_sent,
                                    const int32_t* off, const int32_t* len, void* out, int rows, int H,
                                    int d, int causal, hipStream_t s);

// Diverse beam search: the search kernels work on one group of every sentence at a time.  A sentence's
// k_all rows are split into groups of kg; this launch takes group goff / kg (rows goff .. goff+kg-1 of
// each sentence).  pen_tok [sentences, pen_ld] / pen_n [sentences]: tokens taken at this step by the
// groups before it; every occurrence of a token lowers its ranking value by `strength`.
// out_plain [M, k]: the unpenalised values of the kept candidates (what the hypothesis score becomes).
struct SearchGroups {
  int kg, k_all, goff;
  int32_t* pen_tok;
  int32_t* pen_n;
  int pen_ld;
  float strength;
  float* out_plain;
  int last;   // the last group of the step: counts active sentences, advances the step, clears pen_n
};
// no groups: every row is its own unit for the retrieve kernel, a sentence's k rows one unit for the re-rank kernel
__host__ __device__ inline SearchGroups one_group() { return SearchGroups{1, 1, 0, nullptr, nullptr, 0, 0.f, nullptr, 1}; }

// raw != 0: rank the logits themselves (score and fin are ignored, may be null).  M counts the rows
// this launch works on (sentences * groups.kg).
hipError_t launch_row_topk(int dtype, const void* logits, const float* score, const int32_t* fin,
                           int M, int V, int k, int eos, int raw, float* out_score, int32_t* out_idx,
                           hipStream_t s, const SearchGroups& groups = one_group());
// topp < 1: only the shortest prefix of the ranked candidates whose k-way softmax mass reaches topp is drawn from.
// fin != null (encoder-decoder models; cap [rows] then required): finished rows draw nothing, EOS or the cap
// finishes a row, the uniform number is that of row order[r] (r if order is null) and active[step] counts the
// rows left unfinished; fin == null: every row draws, active[step] = rows until n_new tokens are out.
hipError_t launch_sample(const float* cand_logit, const int32_t* cand_idx, int32_t* tokens, int32_t* len,
                         float* logp, int32_t* active, int32_t* step_state, int rows, int k, float topp, int T,
                         unsigned long long seed, int n_new, hipStream_t s, int32_t* fin = nullptr,
                         const int32_t* cap = nullptr, const int32_t* order = nullptr, int eos = -1);
// step = t_base + (step_state ? step_state[0] : 0).  `active` points at the counter array indexed
// by step.  With step_state != null the last workgroup to finish advances step_state[0]
// (step_state[1] is its arrival counter and must be zero at launch).  anc != null: the slab table
// [batch*k, T+1] is gathered by parent like the token histories, and entry t+1 of every row is set
// to the row's own beam index.
// groups given (kg < k_all): k is the group width kg, candidates are [rows, kg]; see SearchGroups.
// row_topk (plain beam search, or raw: the k largest logits for sampling) from the logit product's group
// statistics (GemmOut::stats): same output, the logits of only the groups that can hold a top-k token are read
bool topk_groups_supported(int V, int k, int raw);
hipError_t launch_row_topk_groups(const float* logits, const float* stats, const float* score, const int32_t* fin, int M,
                                  int V, int k, int eos, int raw, float* out_score, int32_t* out_idx, hipStream_t s);
// The next step's decoder input, left behind by the kernel that settles the step's tokens:
// x[row] = E[last token of row] * scale + pe[t + 1] (E == nullptr: not asked for).
struct NextInput {
  const void* E;
  const float* pe;
  void* x;
  int d, dtype;
  float scale;
};
inline NextInput no_next_input() { return NextInput{nullptr, nullptr, nullptr, 0, 0, 0.f}; }
hipError_t launch_beam_refine(const float* cand_score, const int32_t* cand_idx, float* score,
                              int32_t* tokens, int32_t* len, int32_t* fin, int32_t* parent,
                              const int32_t* cap, int32_t* active, int batch, int k, int V, int T,
                              int t_base, int32_t* step_state, int eos, int32_t* anc, hipStream_t s,
                              const SearchGroups& groups = one_group(), const NextInput& next = no_next_input());
// launch_row_topk_groups (raw) and launch_sample in one launch; next.E given: the rows' next decoder input as well
hipError_t launch_retrieve_sample(const float* logits, const float* stats, int32_t* tokens, int32_t* len, float* logp,
                                  int32_t* active, int32_t* step_state, int rows, int V, int k, float topp, int T,
                                  unsigned long long seed, int n_new, hipStream_t s, int32_t* fin = nullptr,
                                  const int32_t* cap = nullptr, const int32_t* order = nullptr, int eos = -1,
                                  const NextInput& next = no_next_input(), float* cand_score = nullptr,
                                  int32_t* cand_idx = nullptr);   // cand_*: the candidates are also left there
// launch_row_topk_groups and launch_beam_refine (no groups, device-side step counter) in one launch
hipError_t launch_retrieve_rerank(const float* logits, const float* stats, float* score, int32_t* tokens, int32_t* len,
                                  int32_t* fin, int32_t* parent, const int32_t* cap, int32_t* active, int batch, int k,
                                  int V, int T, int32_t* step_state, int eos, int32_t* anc, hipStream_t s,
                                  const NextInput& next = no_next_input(), float* cand_score = nullptr,
                                  int32_t* cand_idx = nullptr);   // cand_*: the survivors are also left there
// npos = npos_base + (tp ? *tp : 0); the grid covers npos_max positions
hipError_t launch_cache_reorder(int dtype, void* cache, const int32_t* parent, int layers, int batch,
                                int rows_total, int k, int T, int d, int npos_base, const int32_t* tp,
                                int npos_max, hipStream_t s);
// kg: width of a search group (k without diverse beam search): the first hypothesis of every group starts alive
hipError_t launch_beam_reset(float* score, int32_t* tokens, int32_t* len, int32_t* fin,
                             int32_t* active_counts, int32_t* step_state, int32_t* anc, int32_t* pen_n, int batch,
                             int k, int kg, int T, int bos, int pad, hipStream_t s);
// first: index in the token history of the first token to hand out (1 after BOS; prompt length for
// the decoder-only model)
hipError_t launch_finalize(const float* score, const int32_t* tokens, const int32_t* len, int32_t* out_ids,
                           int32_t* out_lens, float* out_scores, const int32_t* sentence_order, int batch,
                           int k, int T, float alpha, int pad, int first, hipStream_t s);

bool topk_supported(int V);
bool head_dim_supported(int dh);

// ---- device helpers -------------------------------------------------------------------------
// Cross-lane moves inside the vector ALU.  __shfl_xor is an LDS-crossbar instruction (ds_bpermute:
// an address register, the LDS queue and its latency for every step of a reduction); operand
// swizzles (quad permutes, mirrors and rotations inside a row of 16 lanes) are a modifier of the
// add or max itself, and gfx950 swaps rows of 16 and halves of 32 lanes between two registers in
// one instruction.  All of them want every lane they read to be active.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7 - i inside every 8 lanes
constexpr int kDppMirror = 0x140;      // lane i <-> 15 - i inside every 16 lanes
constexpr int kDppRor8 = 0x128;        // rotate every 16 lanes by 8: lane i <-> i ^ 8

// O = 16 or 32: {a, b} = the values of this lane and of lane (lane ^ O), the lower lane's in one and
// the upper lane's in the other, in both lanes alike (swap(x, x) does exactly this).
template <int O>
__device__ __forceinline__ void lane_pair(float v, float& a, float& b) {
  static_assert(O == 16 || O == 32, "rows of 16 or halves of 32 lanes");
  const unsigned x = __builtin_bit_cast(unsigned, v);
  unsigned ra, rb;
  if constexpr (O == 16) {
    const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
    ra = r[0]; rb = r[1];
  } else {
    const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    ra = r[0]; rb = r[1];
  }
  a = __builtin_bit_cast(float, ra);
  b = __builtin_bit_cast(float, rb);
}

// The value that lane (lane ^ O) holds.
template <int O>
__device__ __forceinline__ float lane_xor(float v) {
  static_assert(O == 1 || O == 2 || O == 4 || O == 8 || O == 16 || O == 32, "one bit of the lane number");
  if constexpr (O == 1) return dpp_move<kDppXor1>(v);
  else if constexpr (O == 2) return dpp_move<kDppXor2>(v);
  else if constexpr (O == 8) return dpp_move<kDppRor8>(v);
  else if constexpr (O == 16 || O == 32) {
    float a, b;
    lane_pair<O>(v, a, b);   // whichever is not this lane's own value is the other's (or equal to it)
    return __builtin_bit_cast(unsigned, a) == __builtin_bit_cast(unsigned, v) ? b : a;
  } else {
    return __shfl_xor(v, O, kWave);
  }
}

// v + (value of lane ^ O) and max(v, value of lane ^ O)
template <int O>
__device__ __forceinline__ float add_lane_xor(float v) {
  if constexpr (O == 16 || O == 32) { float a, b; lane_pair<O>(v, a, b); return a + b; }
  else return v + lane_xor<O>(v);
}
template <int O>
__device__ __forceinline__ float max_lane_xor(float v) {
  if constexpr (O == 16 || O == 32) { float a, b; lane_pair<O>(v, a, b); return fmaxf(a, b); }
  else return fmaxf(v, lane_xor<O>(v));
}

// Sum / maximum over every aligned group of W lanes (W a power of two), left in all of its lanes.
// Once the quads hold equal values a mirror is as good as an exchange.
template <int W>
__device__ __forceinline__ float group_sum(float v) {
  static_assert(W >= 1 && W <= 64 && (W & (W - 1)) == 0, "power of two");
  if constexpr (W >= 2) v += dpp_move<kDppXor1>(v);
  if constexpr (W >= 4) v += dpp_move<kDppXor2>(v);
  if constexpr (W >= 8) v += dpp_move<kDppHalfMirror>(v);
  if constexpr (W >= 16) v += dpp_move<kDppMirror>(v);
  if constexpr (W >= 32) v = add_lane_xor<16>(v);
  if constexpr (W >= 64) v = add_lane_xor<32>(v);
  return v;
}
template <int W>
__device__ __forceinline__ float group_max(float v) {
  static_assert(W >= 1 && W <= 64 && (W & (W - 1)) == 0, "power of two");
  if constexpr (W >= 2) v = fmaxf(v, dpp_move<kDppXor1>(v));
  if constexpr (W >= 4) v = fmaxf(v, dpp_move<kDppXor2>(v));
  if constexpr (W >= 8) v = fmaxf(v, dpp_move<kDppHalfMirror>(v));
  if constexpr (W >= 16) v = fmaxf(v, dpp_move<kDppMirror>(v));
  if constexpr (W >= 32) v = max_lane_xor<16>(v);
  if constexpr (W >= 64) v = max_lane_xor<32>(v);
  return v;
}
__device__ __forceinline__ float wave_sum(float v) { return group_sum<64>(v); }
__device__ __forceinline__ float wave_max(float v) { return group_max<64>(v); }

// f(integral constant O) for O = LO, 2 LO, ... < 64: the steps of a butterfly over lane groups
template <int LO, typename F>
__device__ __forceinline__ void for_lane_bits(F&& f) {
  if constexpr (LO < 64) {
    f(std::integral_constant<int, LO>{});
    for_lane_bits<LO * 2>(f);
  }
}

template <typename T> struct Vec8;
template <> struct Vec8<half_t> {
  // the 16 bytes as they are in memory, for data that waits in registers before it is used
  using raw_t = half8_t;
  __device__ static __forceinline__ raw_t load_raw(const half_t* p) { return *reinterpret_cast<const half8_t*>(p); }
  __device__ static __forceinline__ void unpack(const raw_t& h, float (&f)[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = (float)h[i];
  }
  __device__ static __forceinline__ void load(const half_t* p, float (&f)[8]) {
    half8_t h = *reinterpret_cast<const half8_t*>(p);
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = (float)h[i];
  }
  __device__ static __forceinline__ void store(half_t* p, const float (&f)[8]) {
    half8_t h;
#pragma unroll
    for (int i = 0; i < 8; ++i) h[i] = (half_t)f[i];
    *reinterpret_cast<half8_t*>(p) = h;
  }
};
template <> struct Vec8<float> {
  struct raw_t { floatx4 a, b; };
  __device__ static __forceinline__ raw_t load_raw(const float* p) {
    return {*reinterpret_cast<const floatx4*>(p), *reinterpret_cast<const floatx4*>(p + 4)};
  }
  __device__ static __forceinline__ void unpack(const raw_t& r, float (&f)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) { f[i] = r.a[i]; f[4 + i] = r.b[i]; }
  }
  __device__ static __forceinline__ void load(const float* p, float (&f)[8]) {
    floatx4 a = *reinterpret_cast<const floatx4*>(p);
    floatx4 b = *reinterpret_cast<const floatx4*>(p + 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) { f[i] = a[i]; f[4 + i] = b[i]; }
  }
  __device__ static __forceinline__ void store(float* p, const float (&f)[8]) {
    floatx4 a, b;
#pragma unroll
    for (int i = 0; i < 4; ++i) { a[i] = f[i]; b[i] = f[4 + i]; }
    *reinterpret_cast<floatx4*>(p) = a;
    *reinterpret_cast<floatx4*>(p + 4) = b;
  }
};

// x[r,:] = store(E[id_r,:] * sqrt(d) + PE[pos_r,:]).  Product and sum are rounded separately
// (no fused multiply-add) so the fp32 value before storage is the textbook one.
template <typename T>
__device__ __forceinline__ void embed_row(const T* __restrict__ e, const float* __restrict__ pe,
                                          T* __restrict__ x, int d, float scale, int lane, int nl) {
  if ((d & 7) == 0) {
    for (int c = lane * 8; c < d; c += nl * 8) {
      float v[8];
      Vec8<T>::load(e + c, v);
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = __fadd_rn(__fmul_rn(v[i], scale), pe[c + i]);
      Vec8<T>::store(x + c, v);
    }
  } else {
    for (int c = lane; c < d; c += nl) x[c] = (T)__fadd_rn(__fmul_rn((float)e[c], scale), pe[c]);
  }
}

// LayerNorm of one row held by one wavefront: lane l owns elements (j*64 + l)*8 .. +7 of the row for
// j < NV (those at or beyond d are absent).  v comes in as the row, leaves centred; o = g * (v * rstd) + b.
// Shared by the stand-alone kernel and the product kernel that normalises its own input, so that
// both round identically.
template <int NV>
__device__ __forceinline__ void layernorm_row(float (&v)[NV][8], const float (&gv)[NV][8], const float (&bv)[NV][8],
                                              int d, float eps, int lane, float (&o)[NV][8]) {
  // every operation is spelled out (no contraction left to the compiler), so the two kernels that
  // inline this give the same bits
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < NV; ++j)
    if ((j * 64 + lane) * 8 < d) {
#pragma unroll
      for (int i = 0; i < 8; ++i) sum = __fadd_rn(sum, v[j][i]);
    }
  const float mean = __fdiv_rn(wave_sum(sum), (float)d);
  float sq = 0.f;
#pragma unroll
  for (int j = 0; j < NV; ++j)
    if ((j * 64 + lane) * 8 < d) {
#pragma unroll
      for (int i = 0; i < 8; ++i) { v[j][i] = __fsub_rn(v[j][i], mean); sq = __fmaf_rn(v[j][i], v[j][i], sq); }
    }
  const float var = __fdiv_rn(wave_sum(sq), (float)d);
  const float rstd = __fdiv_rn(1.0f, __fsqrt_rn(__fadd_rn(var, eps)));
#pragma unroll
  for (int j = 0; j < NV; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      o[j][i] = __fmaf_rn(gv[j][i], __fmul_rn(v[j][i], rstd), bv[j][i]);
      // keep the float32 result as it is: without this the compiler may merge the multiply-add with
      // the caller's conversion to float16 into one mixed-precision instruction that rounds once
      // instead of twice, in one kernel and not in the other
      asm volatile("" : "+v"(o[j][i]));
    }
}

// Softmax statistics of two sets of values merged: (max, sum of exp(value - max)).  A set without values is (-inf, 0).
__device__ __forceinline__ void merge_stat(float& m, float& z, float m2, float z2) {
  const float mn = fmaxf(m, m2);
  if (mn != -INFINITY) z = z * __expf(m - mn) + z2 * __expf(m2 - mn);
  m = mn;
}

// v <- v + ((p[0] + p[1] + ... + p[S-1]) + t), slabs added in index order, nothing contracted
template <int SMAX>
__device__ __forceinline__ void add_partials(float (&v)[8], const float (&part)[SMAX][8], int S, const float (&t)[8]) {
  float a[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = part[0][i];
#pragma unroll
  for (int sp = 1; sp < SMAX; ++sp)
    if (sp < S) {
#pragma unroll
      for (int i = 0; i < 8; ++i) a[i] = __fadd_rn(a[i], part[sp][i]);
    }
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = __fadd_rn(v[i], __fadd_rn(a[i], t[i]));
}

}  // namespace lsq
