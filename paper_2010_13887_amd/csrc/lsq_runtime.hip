// Host side of liblsq.so: the C ABI, blob parsing, the max-shape memory plan (paper sec. 2.3)
// and the per-call launch sequences.  No device memory is ever allocated here.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <vector>

#include "../../include/lsq.h"
#include "lsq_internal.h"

using namespace lsq;

static_assert(LSQ_MAX_BEAM == LSQ_MAX_BEAM_, "public and internal beam limits differ");
static_assert(LSQ_MAX_SAMPLE_TOPK == LSQ_MAX_TOPK_, "public and internal retrieve widths differ");

namespace {

char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

#define HIPCHK(expr)                                                                     \
  do {                                                                                   \
    hipError_t e_ = (expr);                                                              \
    if (e_ != hipSuccess) return fail(LSQ_E_HIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

// Optional per-launch timing: when enabled, every kernel launched by lsq_decode_step(s) is
// bracketed by two events on the library's stream; lsq_profile_read adds the elapsed times up
// per kernel class.  Events come from a host-side pool that only grows.
enum ProfClass {
  PC_EMBED, PC_GEMM_QKV, PC_ATTN_SELF, PC_GEMM_DD, PC_LAYERNORM, PC_ATTN_CROSS, PC_GEMM_FFN1, PC_GEMM_FFN2,
  PC_GEMM_VOCAB, PC_ROW_TOPK, PC_REFINE, PC_REORDER, PC_GEMM_OUT, PC_ATTN_CROSS_Q, PC_SELF_BLOCK, PC_CROSS_BLOCK, PC_ROW_TOPK_GROUPS, PC_RETRIEVE_RERANK, PC_COUNT
};
const char* const kProfNames[PC_COUNT] = {"embed", "gemm_qkv", "attn_self", "gemm_dxd", "add_layernorm",
                                          "attn_cross", "gemm_ffn1", "gemm_ffn2", "gemm_vocab", "row_topk",
                                          "beam_refine", "cache_reorder", "gemm_out", "attn_cross_q", "self_block",
                                          "cross_block", "row_topk_groups", "retrieve_rerank"};
struct Prof {
  bool on = false;
  std::vector<hipEvent_t> pool;   // pairs: [2i] start, [2i+1] stop
  std::vector<int> cls;           // class of pair i
  size_t used = 0;                // pairs in flight
} g_prof;

hipError_t prof_mark(hipStream_t s, int c, bool start) {
  if (!g_prof.on || c < 0) return hipSuccess;
  if (start) {
    if (g_prof.used * 2 >= g_prof.pool.size()) {
      hipEvent_t a, b;
      hipError_t e = hipEventCreate(&a);
      if (e != hipSuccess) return e;
      e = hipEventCreate(&b);
      if (e != hipSuccess) return e;
      g_prof.pool.push_back(a);
      g_prof.pool.push_back(b);
      g_prof.cls.push_back(c);
    }
    g_prof.cls[g_prof.used] = c;
    return hipEventRecord(g_prof.pool[g_prof.used * 2], s);
  }
  hipError_t e = hipEventRecord(g_prof.pool[g_prof.used * 2 + 1], s);
  ++g_prof.used;
  return e;
}

#define TIMED(cls, expr)                      \
  do {                                        \
    HIPCHK(prof_mark(s, cls, true));          \
    HIPCHK(expr);                             \
    HIPCHK(prof_mark(s, cls, false));         \
  } while (0)

constexpr size_t kAlign = 256;
constexpr size_t kMaxSplits = 8;        // fp32 partial-sum slabs a split-K product may leave
constexpr int kMaxSplitsFusedLn = 4;    // ... when the consuming product adds them itself
constexpr size_t kBlockRowsMax = 64;    // most rows the attention blocks (attention_blocks_supported) take
inline size_t up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct HParams {
  int arch, n_enc, n_dec, d, H, F, V, max_pos, act, norm, dtype, pad, bos, eos, cap_extra, sample_topk;
  float alpha, eps, topp;
  uint64_t seed, total;
};

int parse_header(const void* blob, size_t bytes, HParams* hp) {
  if (!blob) return fail(LSQ_E_ARG, "weights is null");
  if (bytes < 256) return fail(LSQ_E_BLOB, "blob shorter than its header");
  const char* p = (const char*)blob;
  if (memcmp(p, "LSQBLOB1", 8) != 0) return fail(LSQ_E_BLOB, "bad magic");
  int32_t f[17];
  memcpy(f, p + 8, sizeof f);
  if (f[0] != 1) return fail(LSQ_E_BLOB, "unsupported blob version %d", f[0]);
  hp->arch = f[1]; hp->n_enc = f[2]; hp->n_dec = f[3]; hp->d = f[4]; hp->H = f[5]; hp->F = f[6];
  hp->V = f[7]; hp->max_pos = f[8]; hp->act = f[9]; hp->norm = f[10]; hp->dtype = f[11];
  hp->pad = f[12]; hp->bos = f[13]; hp->eos = f[14]; hp->cap_extra = f[15]; hp->sample_topk = f[16];
  memcpy(&hp->alpha, p + 76, 4);
  memcpy(&hp->eps, p + 80, 4);
  memcpy(&hp->topp, p + 84, 4);
  if (!(hp->topp > 0.f && hp->topp < 1.f)) hp->topp = 1.f;   // 0 in the header: no nucleus cut
  memcpy(&hp->seed, p + 88, 8);
  memcpy(&hp->total, p + 96, 8);
  const bool encdec = hp->arch == 0 && hp->norm == 0 && hp->act == 0;
  const bool deconly = hp->arch == 1 && hp->norm == 1 && hp->act == 1;
  if (!encdec && !deconly)
    return fail(LSQ_E_BLOB, "supported: post-LN ReLU encoder-decoder (arch 0) or pre-LN tanh-GELU decoder-only (arch 1)");
  if (hp->dtype != DT_F32 && hp->dtype != DT_F16) return fail(LSQ_E_BLOB, "unknown dtype %d", hp->dtype);
  if (deconly && (hp->n_enc != 0 || hp->sample_topk < 1 || hp->sample_topk > LSQ_MAX_SAMPLE_TOPK || hp->max_pos < 1 ||
                  hp->d > 4096))
    return fail(LSQ_E_BLOB, "decoder-only blob: n_enc must be 0, sample_topk in [1, %d], max_pos >= 1, d <= 4096", LSQ_MAX_SAMPLE_TOPK);
  if (encdec && (hp->sample_topk < 0 || hp->sample_topk > LSQ_MAX_SAMPLE_TOPK))
    return fail(LSQ_E_BLOB, "sample_topk outside [0, %d] (0: beam search)", LSQ_MAX_SAMPLE_TOPK);
  if ((encdec && hp->n_enc < 1) || hp->n_dec < 1 || hp->n_enc > 64 || hp->n_dec > 64 || hp->d < 8 || hp->H < 1 ||
      hp->F < 8 || hp->V < 4 || hp->d % hp->H != 0 || hp->d > 16384 || hp->F > 262144 || hp->max_pos < 0 ||
      hp->max_pos > (1 << 20) || hp->cap_extra > (1 << 20))
    return fail(LSQ_E_BLOB, "implausible model shape");
  if (hp->d % 8 != 0 || hp->F % 8 != 0) return fail(LSQ_E_BLOB, "d_model and d_ffn must be multiples of 8");
  if (!head_dim_supported(hp->d / hp->H)) return fail(LSQ_E_BLOB, "head size %d unsupported (16/32/64/128)", hp->d / hp->H);
  if (!topk_supported(hp->V)) return fail(LSQ_E_BLOB, "vocabulary %d unsupported (<= 65536)", hp->V);
  for (int id : {hp->pad, hp->bos, hp->eos})
    if (id < 0 || id >= hp->V) return fail(LSQ_E_BLOB, "special token id outside the vocabulary");
  if (hp->cap_extra < 0 || !(hp->eps > 0.f)) return fail(LSQ_E_BLOB, "bad cap_extra / ln_eps");
  return LSQ_OK;
}

// One tensor of the blob: `rows` x `cols` as stored ([in, out] for matrices; rows == 1 for vectors).
struct TensorDesc { int rows, cols; bool transpose; bool gemm = false; };   // gemm: the weight matrix of a product

void tensor_walk(const HParams& hp, std::vector<TensorDesc>* out) {
  const int d = hp.d, F = hp.F, V = hp.V;
  auto mat = [&](int r, int c) { out->push_back({r, c, true, true}); };
  auto vec = [&](int n) { out->push_back({1, n, false}); };
  out->push_back({V, d, false, true});   // embedding: already [vocab, d] = [N, K] of the logit GEMM
  if (hp.arch == 1) {
    out->push_back({hp.max_pos, d, false});   // learned positions
    for (int i = 0; i < hp.n_dec; ++i) {
      vec(d); vec(d); mat(d, 3 * d); vec(3 * d); mat(d, d); vec(d);
      vec(d); vec(d); mat(d, F); vec(F); mat(F, d); vec(d);
    }
    vec(d); vec(d);
    return;
  }
  for (int i = 0; i < hp.n_enc; ++i) {
    mat(d, 3 * d); vec(3 * d); mat(d, d); vec(d); vec(d); vec(d);
    mat(d, F); vec(F); mat(F, d); vec(d); vec(d); vec(d);
  }
  for (int i = 0; i < hp.n_dec; ++i) {
    mat(d, 3 * d); vec(3 * d); mat(d, d); vec(d); vec(d); vec(d);
    mat(d, d); vec(d); mat(d, 2 * d); vec(2 * d); mat(d, d); vec(d); vec(d); vec(d);
    mat(d, F); vec(F); mat(F, d); vec(d); vec(d); vec(d);
  }
}

struct GptLayer { char *ln1g, *ln1b, *Wqkv, *bqkv, *Wo, *bo, *ln2g, *ln2b, *W1, *b1, *W2, *b2; };
struct EncLayer { char *Wqkv, *bqkv, *Wo, *bo, *ln1g, *ln1b, *W1, *b1, *W2, *b2, *ln2g, *ln2b; };
struct DecLayer {
  char *Wqkv, *bqkv, *Wo, *bo, *ln1g, *ln1b, *Wq, *bq, *Wkv, *bkv, *Woc, *boc, *ln2g, *ln2b, *W1, *b1, *W2,
      *b2, *ln3g, *ln3b;
};

// Byte offsets into the workspace.  Everything is sized for max_batch / beam / max_len once;
// encoder intermediates and decoder intermediates are never live together and share `scratch`,
// and inside the decoder the FFN activation and the logits share bytes as well.
// Debug aid for the memory plan (sec. 2.3: buffers that share one arena are exactly where an overrun or a wrong
// lifetime would hide): with canaries on, every region of the plan is followed by a 256-byte red zone filled
// with a pattern; lsq_debug_check_canaries says how many have been touched.
bool g_canaries = false;
constexpr size_t kCanaryBytes = 256;
constexpr unsigned char kCanaryByte = 0xA5;

struct Plan {
  std::vector<size_t> canaries;       // red zones behind the regions that live as long as the model
  std::vector<size_t> dec_canaries;   // ... behind the decoder's intermediates (valid from the end of lsq_encode on)
  size_t weights, wpacked, pe, cache, cross, score, tokens, len, fin, parent, anc, pen_tok, pen_n, cand_plain, cap, order, src_off, src_len, active, step_state,
      cand_score, cand_idx, out_ids, out_lens, out_scores, scratch, total;
  // encoder view of scratch
  size_t e_ids, e_pos, e_sent, e_x, e_qkv, e_ctx, e_tmp, e_ffn;
  // decoder view of scratch
  size_t d_x, d_q, d_ctx, d_tmp, d_tmp2, d_ffn, d_logits, d_y, e_y, d_x2, d_x0, d_stats;
};

size_t packed_weight_bytes(const HParams& hp);

Plan make_plan(const HParams& hp, size_t weight_bytes, int B, int k, int T) {
  Plan p;
  const size_t esz = hp.dtype == DT_F16 ? 2 : 4;
  const size_t M = (size_t)B * k, R = (size_t)B * T, d = hp.d, F = hp.F, V = hp.V;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off += up(bytes);
    if (g_canaries) { p.canaries.push_back(off); off += kCanaryBytes; }
    return o;
  };
  p.weights = take(weight_bytes);
  p.wpacked = take(packed_weight_bytes(hp));
  p.pe = take((size_t)T * d * 4);
  p.cache = take((size_t)hp.n_dec * 2 * M * T * d * esz);
  p.cross = take((size_t)hp.n_dec * R * 2 * d * esz);
  p.score = take(M * 4);
  p.tokens = take(M * (T + 1) * 4);
  p.len = take(M * 4);
  p.fin = take(M * 4);
  p.parent = take(M * 4);
  p.anc = take(M * (T + 1) * 4);   // which slab of its sentence holds position j of row r's history
  p.pen_tok = take(M * 4);         // diverse beam search: tokens taken at this step by the earlier groups of a sentence
  p.pen_n = take((size_t)B * 4);
  p.cand_plain = take(M * k * 4);  // ... and the kept candidates' values without the diversity penalty
  p.cap = take((size_t)B * 4);
  p.order = take((size_t)B * 4);
  p.src_off = take((size_t)(B + 1) * 4);
  p.src_len = take((size_t)B * 4);
  p.active = take((size_t)(T + 1) * 4);
  p.step_state = take(4 * 4);   // [0] position counter, [1] arrival counter, [2] position of step 0
  const size_t kk = std::max(k, hp.sample_topk);   // survivors per row
  p.cand_score = take(M * kk * 4);
  p.cand_idx = take(M * kk * 4);
  p.out_ids = take(M * T * 4);
  p.out_lens = take(M * 4);
  p.out_scores = take(M * 4);
  p.scratch = off;
  // encoder phase
  size_t e = p.scratch;
  auto etake = [&](size_t bytes) { size_t o = e; e += up(bytes); return o; };
  p.e_ids = etake(R * 4); p.e_pos = etake(R * 4); p.e_sent = etake(R * 4);
  p.e_x = etake(R * d * esz); p.e_qkv = etake(R * 3 * d * esz); p.e_ctx = etake(R * d * esz);
  p.e_tmp = etake(R * d * 4); p.e_ffn = etake(R * F * esz);
  p.e_y = etake(R * d * esz);     // pre-LN models: normalised copy of the residual stream   // e_tmp: one fp32 slab (no split-K at encoder sizes)
  // decoder phase
  size_t q = p.scratch;
  auto dtake = [&](size_t bytes) {
    size_t o = q;
    q += up(bytes);
    if (g_canaries) { p.dec_canaries.push_back(q); q += kCanaryBytes; }
    return o;
  };
  p.d_x = dtake(M * d * esz); p.d_q = dtake(M * d * esz); p.d_ctx = dtake(M * d * esz);
  // fp32 partial-sum slabs: of the split-K GEMMs, or one per head from the attention blocks (few rows), which
  // read one set while they write the other
  const size_t head_slabs = (size_t)hp.H * std::min<size_t>(M, kBlockRowsMax) * d * 4;
  p.d_tmp = dtake(std::max(kMaxSplits * M * d * 4, head_slabs));
  p.d_tmp2 = dtake(std::max<size_t>(std::min<size_t>(M, kBlockRowsMax) * kMaxSplits * d * 4, head_slabs));
  p.d_y = dtake(M * d * esz);
  p.d_x2 = dtake(M * d * esz);   // second hidden-state buffer for products that normalise their own input
  p.d_x0 = dtake(M * d * esz);   // decoder input of the next step, left by the kernel that settles this step's tokens
  p.d_stats = dtake(M * ((V + 31) / 32) * 2 * 4);   // (largest, sum of exponentials) of every 32 logits of a row
  p.d_ffn = q;
  p.d_logits = q;
  q += up(std::max(M * F * esz, M * V * 4));   // logits stay fp32 whatever the model dtype
  if (g_canaries) { p.dec_canaries.push_back(q); q += kCanaryBytes; }
  p.total = std::max(e, q);
  if (g_canaries) { p.total = up(p.total); p.canaries.push_back(p.total); p.total += kCanaryBytes; }   // the end of the workspace
  return p;
}

// Size of the serialized model these hyper-parameters describe: header, then tensors at 256-byte boundaries.
size_t blob_bytes(const HParams& hp) {
  std::vector<TensorDesc> ts;
  tensor_walk(hp, &ts);
  const size_t es = hp.dtype == DT_F16 ? 2 : 4;
  size_t n = 256;
  for (auto& t : ts) n = up(n) + (size_t)t.rows * t.cols * es;
  return n;
}

// Fragment-ordered second copies of the float16 matrices (products of at most 64 rows read these).
size_t packed_weight_bytes(const HParams& hp) {
  if (hp.dtype != DT_F16) return 0;
  std::vector<TensorDesc> ts;
  tensor_walk(hp, &ts);
  size_t n = 0;
  for (auto& t : ts)
    if (t.gemm) n += up(gemm_packed_bytes(t.transpose ? t.cols : t.rows, t.transpose ? t.rows : t.cols));
  return n;
}

size_t device_weight_bytes(const HParams& hp) {
  std::vector<TensorDesc> ts;
  tensor_walk(hp, &ts);
  const size_t esz = hp.dtype == DT_F16 ? 2 : 4;
  size_t off = 0;
  for (auto& t : ts) off = up(off) + (size_t)t.rows * t.cols * esz;
  return up(off);
}

struct Ctx {
  int state = 0;   // 0 nothing, 1 workspace set, 2 model loaded, 3 sentences encoded
  char* ws = nullptr;
  size_t ws_bytes = 0;
  hipStream_t stream = nullptr;
  HParams hp{};
  Plan plan{};
  int max_batch = 0, beam = 0, max_len = 0;
  int batch = 0, rows_enc = 0, t = 0;
  int src_longest = 1;         // longest source sentence of this translation
  bool done = false;
  std::vector<int> order;      // internal (sorted) sentence index -> caller's index
  bool use_graphs = true;
  int refresh_mode = 1;   // how the next lsq_encode keeps the cache in step with the beams: 0 move rows, 1 slab table
  bool anc_on = false;    // this translation uses the slab table
  bool fuse_ln = true;    // few rows alive: LayerNorm inside the product that consumes it
  int block_rows = 64;    // ... and whole attention sublayers in one launch up to this many rows
  bool topk_stats = true; // beam search: retrieve from the logit product's group statistics
  bool merge_rerank = true;   // ... and in the same launch as the re-rank stage
  bool sample_fold = false;   // this translation (sampling decoding): retrieve, draw and next input in one launch at every step
  int groups_next = 1, groups = 1;          // diverse beam search: groups per sentence (next encode / this translation)
  float strength_next = 0.f, strength = 0.f;
  bool hidden_in_alt = false;   // the last step left its final hidden rows in the second buffer
  std::map<int, hipGraphExec_t> graphs;   // (live sentences, cross-attention geometry) -> captured decode step
  std::map<int, bool> graph_hidden_in_alt; // ... and where that step leaves its final hidden rows
  std::vector<int> alive_at;   // alive_at[t] = sentences whose cap exceeds t: the prefix step t works on
  char* E = nullptr;
  std::vector<GptLayer> gpt;
  char *lnfg = nullptr, *lnfb = nullptr;
  int prompt_len = 0;
  std::vector<EncLayer> enc;
  std::vector<DecLayer> dec;
  int32_t* pinned = nullptr;   // host staging: ids, positions, sentence map, offsets, lengths, caps, 1 count
  size_t pinned_ints = 0;
} g;

template <typename T> T* at(size_t off) { return reinterpret_cast<T*>(g.ws + off); }
inline size_t esz() { return g.hp.dtype == DT_F16 ? 2 : 4; }

void transpose_copy(const char* src, char* dst, int rows, int cols, size_t es) {
  // src [rows, cols] -> dst [cols, rows]
  constexpr int BL = 32;
  for (int r0 = 0; r0 < rows; r0 += BL)
    for (int c0 = 0; c0 < cols; c0 += BL) {
      int r1 = std::min(rows, r0 + BL), c1 = std::min(cols, c0 + BL);
      if (es == 2) {
        const uint16_t* s = (const uint16_t*)src;
        uint16_t* d = (uint16_t*)dst;
        for (int r = r0; r < r1; ++r)
          for (int c = c0; c < c1; ++c) d[(size_t)c * rows + r] = s[(size_t)r * cols + c];
      } else {
        const uint32_t* s = (const uint32_t*)src;
        uint32_t* d = (uint32_t*)dst;
        for (int r = r0; r < r1; ++r)
          for (int c = c0; c < c1; ++c) d[(size_t)c * rows + r] = s[(size_t)r * cols + c];
      }
    }
}

int check_limits(int max_batch, int beam, int max_len, const HParams& hp) {
  if (max_batch < 1 || max_batch > 4096) return fail(LSQ_E_ARG, "max_batch %d outside [1, 4096]", max_batch);
  if (beam < 1 || beam > LSQ_MAX_BEAM) return fail(LSQ_E_ARG, "beam %d outside [1, %d]", beam, LSQ_MAX_BEAM);
  if (beam > hp.V) return fail(LSQ_E_ARG, "beam wider than the vocabulary");
  if (max_len < 1 || max_len > 4096) return fail(LSQ_E_ARG, "max_len %d outside [1, 4096]", max_len);
  if (hp.sample_topk > 0 && beam != 1) return fail(LSQ_E_ARG, "a sampling model (sample_topk > 0) runs with beam 1");
  if (hp.arch == 1 && max_len > hp.max_pos) return fail(LSQ_E_ARG, "max_len %d exceeds the model's %d positions", max_len, hp.max_pos);
  return LSQ_OK;
}

// x <- LN(x + in . W^T + bias): the GEMM leaves fp32 partial sums (split over k when the output has
// too few tiles to fill the chip), the LayerNorm kernel adds them, the bias and the residual.
// Post-LN (y == nullptr): x <- LN(x + in.W^T + bias).  Pre-LN (y given): x <- x + in.W^T + bias and
// y <- LN(x) with the NEXT sublayer's gain and shift.
int sublayer(int cls, const void* in, const void* W, const void* bias, const void* g_, const void* b_, void* x,
             void* y, float* partials, int M, int d, int K, int max_splits, hipStream_t s, const void* x_in = nullptr) {
  const HParams& hp = g.hp;
  int S = std::min(gemm_partial_splits(hp.dtype, M, d, K), max_splits);
  TIMED(cls, launch_gemm_partials(hp.dtype, in, W, partials, M, d, K, S, s));
  TIMED(PC_LAYERNORM, launch_add_layernorm_partials(hp.dtype, x, y, partials, S, bias, g_, b_, M, d, hp.eps, s, x_in));
  return LSQ_OK;
}

// All launches of one decode step for the first B sentences (B*k rows).  Nothing here depends on
// the step index: kernels read it from the device-side counter (step_state[0]), the cache and
// cross-K/V strides are those of the maximum shapes, and grids that depend on the number of cached
// positions cover max_len of them.  The same sequence therefore serves every step with B sentences
// alive, which is what lets it be captured once into a hipGraph and replayed.
int launch_step(int B) {
  const HParams& hp = g.hp;
  const Plan& p = g.plan;
  hipStream_t s = g.stream;
  const int dt = hp.dtype, d = hp.d, F = hp.F, V = hp.V, H = hp.H, k = g.beam, T = g.max_len;
  const int M = B * k, M_max = g.max_batch * k;
  const size_t es = esz();
  char* const x_home = g.ws + p.d_x;
  // Under beam search the step's decoder input waits in a buffer of its own (the re-rank kernel of the step before
  // wrote it while this step's final hidden rows were still to be read); it is only read, by the first sublayer,
  // whose LayerNorm leaves the residual stream in the usual two buffers.  Sampling decoding embeds in place.
  char* const x0 = (hp.sample_topk > 0 && !g.sample_fold) ? x_home : g.ws + p.d_x0;
  char* x = x0; char* q = g.ws + p.d_q; char* ctx = g.ws + p.d_ctx; char* tmp = g.ws + p.d_tmp;
  char* ffn = g.ws + p.d_ffn; char* logits = g.ws + p.d_logits;
  int32_t* step = at<int32_t>(p.step_state);
  int32_t* anc = g.anc_on ? at<int32_t>(p.anc) : nullptr;
  const size_t slab = (size_t)M_max * T * d * es;   // one layer's K (or V) cache
  const size_t cross_l = (size_t)g.max_batch * g.max_len * 2 * d * es;
  // Under beam search the decoder input of this step is already there: the re-rank kernel of the step before
  // (lsq_encode for the first step) wrote it.  Sampling decoding embeds here.
  if (hp.sample_topk > 0 && !g.sample_fold)
    TIMED(PC_EMBED, launch_embed_last(dt, g.E, at<float>(p.pe), at<int32_t>(p.tokens), at<int32_t>(p.len), x, M, d, T, step, sqrtf((float)d), s));
  char* x_alt = g.ws + p.d_x2;
  const NextInput next = {g.E, at<float>(p.pe), g.ws + p.d_x0, d, dt, sqrtf((float)d)};
  // after a swap of the two hidden-state buffers: the input buffer never becomes one of them
  auto swapped = [&]() { if (x_alt == x0 && x0 != x_home) x_alt = x_home; };
  // With very few rows alive a sublayer's "add the partial sums, the bias and the residual, then
  // LayerNorm" is not a kernel of its own: the product that consumes the normalised rows does it
  // on its way in, reading the residual from one hidden-state buffer and leaving the new rows in
  // the other.  `pending` carries what that product needs.
  const bool fuse = g.fuse_ln && gemm_ln_supported(dt, M, d);
  // Few rows alive: each attention sublayer is one launch up to its output projection, which it leaves as one
  // slab of partial sums per head (kernels_attn.hip).  The blocks read their LayerNorm's slabs from one set and
  // write theirs to the other.
  // Measured on whole translations: ahead for d = 512 at every row count up to 64 (Transformer-base, 32 rows:
  // 27.07 -> 25.70 ms under beam search, 27.88 -> 24.97 ms sampled), behind for d = 1024, where a workgroup has
  // to stream 512 KB of weight slices through one CU (batch 32 of the big model: 49.3 -> 49.7..50.4 ms whatever
  // the row limit).
  const bool blocks = g.fuse_ln && d <= 512 && attention_blocks_supported(dt, M, k, H, d) && M <= g.block_rows;
  float* slabs = (float*)tmp;
  float* slabs_alt = (float*)(g.ws + p.d_tmp2);
  struct { bool on; int S; const void* bias; const void* gain; const void* shift; } pending = {false, 0, nullptr, nullptr, nullptr};
  auto close_sublayer = [&](int cls, const void* in, const void* W, const void* bias, const void* gain, const void* shift,
                            int K, bool defer) -> int {
    if (!defer) {
      if (x == x0 && x0 != x_home) {   // the first sublayer of a step: residual from the input buffer, rows to the stream's own
        x = x_home;
        return sublayer(cls, in, W, bias, gain, shift, x, nullptr, slabs, M, d, K, kMaxSplits, s, x0);
      }
      return sublayer(cls, in, W, bias, gain, shift, x, nullptr, slabs, M, d, K, kMaxSplits, s);
    }
    const int S = std::min(gemm_partial_splits(dt, M, d, K), kMaxSplitsFusedLn);
    TIMED(cls, launch_gemm_partials(dt, in, W, slabs, M, d, K, S, s));
    pending = {true, S, bias, gain, shift};
    return LSQ_OK;
  };
  auto product = [&](int cls, const void* W, const void* bias, const GemmOut& o, int N, int act) -> int {
    if (!pending.on) {
      TIMED(cls, launch_gemm(dt, x, W, bias, o, M, N, d, act, s));
      return LSQ_OK;
    }
    LnInput ln = {slabs, pending.S, (const half_t*)pending.bias, (const half_t*)pending.gain,
                  (const half_t*)pending.shift, (const half_t*)x, (half_t*)x_alt, hp.eps};
    TIMED(cls, launch_gemm_ln(ln, W, bias, o, M, N, d, act, s));
    std::swap(x, x_alt); swapped();
    pending.on = false;
    return LSQ_OK;
  };
  for (int l = 0; l < hp.n_dec; ++l) {
    const DecLayer& L = g.dec[l];
    char* Kc = g.ws + p.cache + (size_t)(2 * l) * slab;
    char* Vc = Kc + slab;
    if (blocks) {
      const void *wqkv_p = gemm_packed_weights(L.Wqkv, 3 * d, d), *wo_p = gemm_packed_weights(L.Wo, d, d);
      const void *wq_p = gemm_packed_weights(L.Wq, d, d), *woc_p = gemm_packed_weights(L.Woc, d, d);
      if (!wqkv_p || !wo_p || !wq_p || !woc_p) return fail(LSQ_E_STATE, "fragment-ordered weights missing");
      LnInput ln = {slabs, pending.on ? pending.S : 0, (const half_t*)pending.bias, (const half_t*)pending.gain,
                    (const half_t*)pending.shift, (const half_t*)x, pending.on ? (half_t*)x_alt : nullptr, hp.eps};
      TIMED(PC_SELF_BLOCK, launch_self_block(ln, wqkv_p, L.bqkv, wo_p, Kc, Vc, anc, step, 0, slabs_alt, B, k, H, d, T, s));
      if (pending.on) { std::swap(x, x_alt); swapped(); }
      pending.on = false;
      std::swap(slabs, slabs_alt);
      LnInput ln1 = {slabs, H, (const half_t*)L.bo, (const half_t*)L.ln1g, (const half_t*)L.ln1b, (const half_t*)x,
                     (half_t*)x_alt, hp.eps};
      TIMED(PC_CROSS_BLOCK, launch_cross_block(ln1, wq_p, L.bq, woc_p, g.ws + p.cross + l * cross_l, at<int32_t>(p.src_off),
                                               at<int32_t>(p.src_len), slabs_alt, B, k, H, d, s));
      std::swap(x, x_alt); swapped();
      std::swap(slabs, slabs_alt);
      TIMED(PC_LAYERNORM, launch_add_layernorm_partials(dt, x, nullptr, slabs, H, L.boc, L.ln2g, L.ln2b, M, d, hp.eps, s));
      if (int rc = product(PC_GEMM_FFN1, L.W1, L.b1, plain_out(ffn, F), F, 1)) return rc;
      if (int rc = close_sublayer(PC_GEMM_FFN2, ffn, L.W2, L.b2, L.ln3g, L.ln3b, F, true)) return rc;
      continue;
    }
    GemmOut o = plain_out(q, d);        // Q | K | V: Q to the activation buffer, K and V to cache position t
    o.ptr[1] = Kc; o.ptr[2] = Vc;
    o.ld[1] = (long)T * d; o.ld[2] = (long)T * d;
    o.tpos = step;
    o.tmul[1] = d; o.tmul[2] = d;
    if (int rc = product(PC_GEMM_QKV, L.Wqkv, L.bqkv, o, 3 * d, 0)) return rc;
    TIMED(PC_ATTN_SELF, launch_self_attention(dt, q, Kc, Vc, ctx, M, H, d, T, 1, step, anc, k, T + 1, s));
    // the cross-attention kernel can normalise its own rows with more sentences alive than the products can
    const void* wq_for_ln = g.fuse_ln && cross_attention_ln_supported(dt, M, k, H, d) ? gemm_packed_weights(L.Wq, d, d) : nullptr;
    if (int rc = close_sublayer(PC_GEMM_OUT, ctx, L.Wo, L.bo, L.ln1g, L.ln1b, d, fuse || wq_for_ln != nullptr)) return rc;
    const void* wq_packed = pending.on ? wq_for_ln : nullptr;
    if (wq_packed) {
      // few rows: the attention kernel normalises its rows and makes its queries itself
      LnInput ln = {slabs, pending.S, (const half_t*)pending.bias, (const half_t*)pending.gain,
                    (const half_t*)pending.shift, (const half_t*)x, (half_t*)x_alt, hp.eps};
      TIMED(PC_ATTN_CROSS, launch_cross_attention_ln(ln, wq_packed, L.bq, g.ws + p.cross + l * cross_l, at<int32_t>(p.src_off),
                                                     at<int32_t>(p.src_len), ctx, B, k, H, d, s));
      std::swap(x, x_alt); swapped();
      pending.on = false;
    } else if (const void* wq_p = (g.fuse_ln && !pending.on && cross_attention_q_worthwhile(B, k, H) && cross_attention_q_supported(dt, M, k, H, d))
                                      ? gemm_packed_weights(L.Wq, d, d) : nullptr) {
      // many rows: the attention kernel still makes its own queries (the rows are normalised already)
      TIMED(PC_ATTN_CROSS_Q, launch_cross_attention_q(x, wq_p, L.bq, g.ws + p.cross + l * cross_l, at<int32_t>(p.src_off),
                                                    at<int32_t>(p.src_len), ctx, B, k, H, d, s));
    } else {
      if (int rc = product(PC_GEMM_DD, L.Wq, L.bq, plain_out(q, d), d, 0)) return rc;
      TIMED(PC_ATTN_CROSS, launch_cross_attention(dt, q, g.ws + p.cross + l * cross_l, at<int32_t>(p.src_off),
                                                  at<int32_t>(p.src_len), ctx, B, k, H, d, g.src_longest, s));
    }
    if (int rc = close_sublayer(PC_GEMM_OUT, ctx, L.Woc, L.boc, L.ln2g, L.ln2b, d, fuse)) return rc;
    if (int rc = product(PC_GEMM_FFN1, L.W1, L.b1, plain_out(ffn, F), F, 1)) return rc;
    if (int rc = close_sublayer(PC_GEMM_FFN2, ffn, L.W2, L.b2, L.ln3g, L.ln3b, F, fuse)) return rc;
  }
  GemmOut lo = plain_out(logits, V);
  lo.f32_out = 1;
  if (pending.on) {
    // The vocabulary product does not take the last LayerNorm along: with it the kernel needs 240
    // registers, half of its 1000 workgroups wait for the other half, and the 64 MB of the
    // embedding stream in two rounds (19.4 us against 3 + 13.5 for the two kernels; same bits)
    TIMED(PC_LAYERNORM, launch_add_layernorm_partials(dt, x, nullptr, slabs, pending.S, pending.bias, pending.gain,
                                                      pending.shift, M, d, hp.eps, s));
    pending.on = false;
  }
  g.hidden_in_alt = (x != x_home);   // which of the two hidden-state buffers the last LayerNorm wrote
  // Plain beam search: the logit product also leaves (largest, sum of exponentials) of every 32 logits of a row,
  // and the retrieve kernel works from those instead of reading the rows (sec. 2.2, with the product's column
  // groups as the groups)
  const bool sampling = hp.sample_topk > 0;
  const bool from_stats = (sampling && g.sample_fold) ||
                          (g.topk_stats && g.groups == 1 && gemm_writes_stats(dt, M, V, d) &&
                           topk_groups_supported(V, sampling ? hp.sample_topk : k, sampling ? 1 : 0));
  if (from_stats) { lo.stats = at<float>(p.d_stats); lo.stats_groups = (V + 31) / 32; }
  if (int rc = product(PC_GEMM_VOCAB, g.E, nullptr, lo, V, 0)) return rc;
  if (hp.sample_topk > 0) {
    // sampling decoding (sec. 3.4): one hypothesis per sentence, nothing to re-rank or to refresh
    if (g.sample_fold) {
      // retrieve, draw and the next step's input in one launch
      TIMED(PC_RETRIEVE_RERANK, launch_retrieve_sample((const float*)logits, at<float>(p.d_stats), at<int32_t>(p.tokens),
                                                       at<int32_t>(p.len), at<float>(p.score), at<int32_t>(p.active), step, M, V,
                                                       hp.sample_topk, hp.topp, T, (unsigned long long)hp.seed, 0, s,
                                                       at<int32_t>(p.fin), at<int32_t>(p.cap), at<int32_t>(p.order), hp.eos, next,
                                                       at<float>(p.cand_score), at<int32_t>(p.cand_idx)));
      return LSQ_OK;
    }
    if (from_stats)
      TIMED(PC_ROW_TOPK_GROUPS, launch_row_topk_groups((const float*)logits, at<float>(p.d_stats), nullptr, nullptr, M, V,
                                                       hp.sample_topk, hp.eos, 1, at<float>(p.cand_score),
                                                       at<int32_t>(p.cand_idx), s));
    else
      TIMED(PC_ROW_TOPK, launch_row_topk(DT_F32, logits, nullptr, nullptr, M, V, hp.sample_topk, hp.eos, 1,
                                         at<float>(p.cand_score), at<int32_t>(p.cand_idx), s));
    TIMED(PC_REFINE, launch_sample(at<float>(p.cand_score), at<int32_t>(p.cand_idx), at<int32_t>(p.tokens),
                                   at<int32_t>(p.len), at<float>(p.score), at<int32_t>(p.active), step, M,
                                   hp.sample_topk, hp.topp, T, (unsigned long long)hp.seed, 0, s, at<int32_t>(p.fin),
                                   at<int32_t>(p.cap), at<int32_t>(p.order), hp.eos));
    return LSQ_OK;
  }
  if (g.groups > 1) {
    // diverse beam search: the groups of a sentence choose one after the other, each steered away
    // from the tokens the earlier ones took at this step
    const int kg = k / g.groups;
    for (int gi = 0; gi < g.groups; ++gi) {
      SearchGroups gr{kg, k, gi * kg, at<int32_t>(p.pen_tok), at<int32_t>(p.pen_n), k, g.strength,
                      at<float>(p.cand_plain), gi + 1 == g.groups ? 1 : 0};
      TIMED(PC_ROW_TOPK, launch_row_topk(DT_F32, logits, at<float>(p.score), at<int32_t>(p.fin), B * kg, V, kg, hp.eos,
                                         0, at<float>(p.cand_score), at<int32_t>(p.cand_idx), s, gr));
      TIMED(PC_REFINE, launch_beam_refine(at<float>(p.cand_score), at<int32_t>(p.cand_idx), at<float>(p.score),
                                          at<int32_t>(p.tokens), at<int32_t>(p.len), at<int32_t>(p.fin),
                                          at<int32_t>(p.parent), at<int32_t>(p.cap), at<int32_t>(p.active), B, kg, V,
                                          T, 0, step, hp.eos, anc, s, gr, next));
    }
    if (!anc)
      TIMED(PC_REORDER, launch_cache_reorder(dt, g.ws + p.cache, at<int32_t>(p.parent), 2 * hp.n_dec, B, M_max, k, T, d,
                                             0, step, T, s));
    return LSQ_OK;
  }
  if (from_stats && g.merge_rerank) {
    // retrieve and re-rank in one launch
    TIMED(PC_RETRIEVE_RERANK, launch_retrieve_rerank((const float*)logits, at<float>(p.d_stats), at<float>(p.score),
                                                     at<int32_t>(p.tokens), at<int32_t>(p.len), at<int32_t>(p.fin),
                                                     at<int32_t>(p.parent), at<int32_t>(p.cap), at<int32_t>(p.active), B, k, V, T,
                                                     step, hp.eos, anc, s, next, at<float>(p.cand_score), at<int32_t>(p.cand_idx)));
    if (!anc)
      TIMED(PC_REORDER, launch_cache_reorder(dt, g.ws + p.cache, at<int32_t>(p.parent), 2 * hp.n_dec, B, M_max, k, T, d,
                                             0, step, T, s));
    return LSQ_OK;
  }
  if (from_stats)
    TIMED(PC_ROW_TOPK_GROUPS, launch_row_topk_groups((const float*)logits, at<float>(p.d_stats), at<float>(p.score), at<int32_t>(p.fin),
                                              M, V, k, hp.eos, 0, at<float>(p.cand_score), at<int32_t>(p.cand_idx), s));
  else
    TIMED(PC_ROW_TOPK, launch_row_topk(DT_F32, logits, at<float>(p.score), at<int32_t>(p.fin), M, V, k, hp.eos, 0,
                                       at<float>(p.cand_score), at<int32_t>(p.cand_idx), s));
  // refine gathers the token histories (and the slab table, when the cache is refreshed through
  // it) by parent and advances the device-side step counter when its last workgroup finishes, so a
  // reorder kernel that follows reads t + 1 = the number of cache positions to move
  TIMED(PC_REFINE, launch_beam_refine(at<float>(p.cand_score), at<int32_t>(p.cand_idx), at<float>(p.score),
                            at<int32_t>(p.tokens), at<int32_t>(p.len), at<int32_t>(p.fin),
                            at<int32_t>(p.parent), at<int32_t>(p.cap), at<int32_t>(p.active), B, k, V, T, 0,
                            step, hp.eos, anc, s, one_group(), next));
  if (!anc)
    TIMED(PC_REORDER, launch_cache_reorder(dt, g.ws + p.cache, at<int32_t>(p.parent), 2 * hp.n_dec, B, M_max, k, T, d,
                                           0, step, T, s));
  return LSQ_OK;
}

// Decoder-only model: one sampled token for every row.  Same conventions as launch_step.
int launch_step_gpt(int B) {
  const HParams& hp = g.hp;
  const Plan& p = g.plan;
  hipStream_t s = g.stream;
  const int dt = hp.dtype, d = hp.d, F = hp.F, V = hp.V, H = hp.H, T = g.max_len, ks = hp.sample_topk;
  const int M = B, M_max = g.max_batch;
  const size_t es = esz();
  char* x = g.ws + p.d_x; char* y = g.ws + p.d_y; char* q = g.ws + p.d_q; char* ctx = g.ws + p.d_ctx;
  char* tmp = g.ws + p.d_tmp; char* ffn = g.ws + p.d_ffn; char* logits = g.ws + p.d_logits;
  int32_t* step = at<int32_t>(p.step_state);
  const size_t slab = (size_t)M_max * T * d * es;
  // Few rows, d <= 512: the attention sublayer of every block is one launch up to its output projection
  // (kernels_attn.hip; a workgroup takes nq rows and one head), the LayerNorm kernel adds the per-head slabs, and
  // the block of the next layer adds the FFN's partial sums on its way in.  Rows are independent here, so nq is
  // free: one row per workgroup while that keeps the launch within one workgroup per CU, else two.
  // Measured on whole translations (6 layers, prompt 64, 96 new tokens): d = 512, 8 / 32 / 64 rows: 16.18 -> 15.08,
  // 18.06 -> 16.49, 23.51 -> 21.30 ms; d = 256, 32 rows: 16.59 -> 14.10 ms.  Behind at d = 768, where a workgroup
  // streams 393 KB of weight slices through one CU (12 layers, 8 rows: 33.45 -> 35.03 ms; 32 rows: 0.427 -> 0.464 ms
  // per step, the block at 15.7 us against 18.0 us for the four kernels it replaces, but 6.7 us instead of 3.9 for
  // the LayerNorm over 12 slabs and the second FFN product held to 4 slabs).
  int nq = 0;
  if (g.fuse_ln && dt == DT_F16 && d <= 512 && M <= g.block_rows) {
    if (attention_blocks_supported(dt, M, 1, H, d)) nq = 1;
    if (M * H > 256 && M % 2 == 0 && attention_blocks_supported(dt, M, 2, H, d)) nq = 2;
  }
  if (nq) {
    char* x_alt = g.ws + p.d_x2;
    float* ffn_slabs = (float*)tmp;
    float* head_slabs = (float*)(g.ws + p.d_tmp2);
    TIMED(PC_EMBED, launch_embed_last(dt, g.E, at<float>(p.pe), at<int32_t>(p.tokens), at<int32_t>(p.len), x, M, d, T, step, 1.0f, s));
    int S = 0;                  // partial sums of the block before, still to be added to the residual stream
    const void* pb = nullptr;   // ... and that product's bias
    for (int l = 0; l < hp.n_dec; ++l) {
      const GptLayer& L = g.gpt[l];
      char* Kc = g.ws + p.cache + (size_t)(2 * l) * slab;
      char* Vc = Kc + slab;
      const void *wqkv_p = gemm_packed_weights(L.Wqkv, 3 * d, d), *wo_p = gemm_packed_weights(L.Wo, d, d);
      if (!wqkv_p || !wo_p) return fail(LSQ_E_STATE, "fragment-ordered weights missing");
      LnInput ln = {ffn_slabs, S, (const half_t*)pb, (const half_t*)L.ln1g, (const half_t*)L.ln1b, (const half_t*)x,
                    S ? (half_t*)x_alt : nullptr, hp.eps, 1};
      TIMED(PC_SELF_BLOCK, launch_self_block(ln, wqkv_p, L.bqkv, wo_p, Kc, Vc, nullptr, step, 0, head_slabs, M / nq, nq, H, d, T, s));
      if (S) std::swap(x, x_alt);
      TIMED(PC_LAYERNORM, launch_add_layernorm_partials(dt, x, y, head_slabs, H, L.bo, L.ln2g, L.ln2b, M, d, hp.eps, s));
      TIMED(PC_GEMM_FFN1, launch_gemm(dt, y, L.W1, L.b1, plain_out(ffn, F), M, F, d, 2, s));
      S = std::min(gemm_partial_splits(dt, M, d, F), kMaxSplitsFusedLn);
      TIMED(PC_GEMM_FFN2, launch_gemm_partials(dt, ffn, L.W2, ffn_slabs, M, d, F, S, s));
      pb = L.b2;
    }
    TIMED(PC_LAYERNORM, launch_add_layernorm_partials(dt, x, y, ffn_slabs, S, pb, g.lnfg, g.lnfb, M, d, hp.eps, s));
    g.hidden_in_alt = (x != g.ws + p.d_x);
  } else if (g.fuse_ln && embed_layernorm_supported(d)) {
    // the step's input rows and their first LayerNorm in one launch
    TIMED(PC_EMBED, launch_embed_layernorm(dt, g.E, at<float>(p.pe), at<int32_t>(p.tokens), at<int32_t>(p.len), x, y,
                                           g.gpt[0].ln1g, g.gpt[0].ln1b, M, d, T, step, 1.0f, hp.eps, s));
  } else {
    TIMED(PC_EMBED, launch_embed_last(dt, g.E, at<float>(p.pe), at<int32_t>(p.tokens), at<int32_t>(p.len), x, M, d, T, step, 1.0f, s));
    TIMED(PC_LAYERNORM, launch_add_layernorm_partials(dt, x, y, nullptr, 0, nullptr, g.gpt[0].ln1g, g.gpt[0].ln1b, M, d, hp.eps, s));
  }
  for (int l = 0; l < (nq ? 0 : hp.n_dec); ++l) {
    const GptLayer& L = g.gpt[l];
    char* Kc = g.ws + p.cache + (size_t)(2 * l) * slab;
    char* Vc = Kc + slab;
    GemmOut o = plain_out(q, d);
    o.ptr[1] = Kc; o.ptr[2] = Vc;
    o.ld[1] = (long)T * d; o.ld[2] = (long)T * d;
    o.tpos = step;
    o.tmul[1] = d; o.tmul[2] = d;
    TIMED(PC_GEMM_QKV, launch_gemm(dt, y, L.Wqkv, L.bqkv, o, M, 3 * d, d, 0, s));
    TIMED(PC_ATTN_SELF, launch_self_attention(dt, q, Kc, Vc, ctx, M, H, d, T, 1, step, nullptr, 1, 0, s));
    if (int rc = sublayer(PC_GEMM_OUT, ctx, L.Wo, L.bo, L.ln2g, L.ln2b, x, y, (float*)tmp, M, d, d, kMaxSplits, s)) return rc;
    TIMED(PC_GEMM_FFN1, launch_gemm(dt, y, L.W1, L.b1, plain_out(ffn, F), M, F, d, 2, s));
    const bool last = l + 1 == hp.n_dec;
    if (int rc = sublayer(PC_GEMM_FFN2, ffn, L.W2, L.b2, last ? g.lnfg : g.gpt[l + 1].ln1g, last ? g.lnfb : g.gpt[l + 1].ln1b,
                          x, y, (float*)tmp, M, d, F, kMaxSplits, s)) return rc;
  }
  GemmOut lo = plain_out(logits, V);
  lo.f32_out = 1;
  // the k largest logits of a row from the product's group statistics (as under beam search, without a normaliser)
  const bool from_stats = g.topk_stats && gemm_writes_stats(dt, M, V, d) && topk_groups_supported(V, ks, 1);
  if (from_stats) { lo.stats = at<float>(p.d_stats); lo.stats_groups = (V + 31) / 32; }
  TIMED(PC_GEMM_VOCAB, launch_gemm(dt, y, g.E, nullptr, lo, M, V, d, 0, s));
  if (from_stats && g.merge_rerank) {
    TIMED(PC_RETRIEVE_RERANK, launch_retrieve_sample((const float*)logits, at<float>(p.d_stats), at<int32_t>(p.tokens),
                                                     at<int32_t>(p.len), at<float>(p.score), at<int32_t>(p.active), step, M, V, ks,
                                                     hp.topp, T, (unsigned long long)hp.seed, hp.cap_extra, s, nullptr, nullptr, nullptr,
                                                     -1, no_next_input(), at<float>(p.cand_score), at<int32_t>(p.cand_idx)));
    return LSQ_OK;
  }
  if (from_stats)
    TIMED(PC_ROW_TOPK_GROUPS, launch_row_topk_groups((const float*)logits, at<float>(p.d_stats), nullptr, nullptr, M, V, ks,
                                                     hp.eos, 1, at<float>(p.cand_score), at<int32_t>(p.cand_idx), s));
  else
    TIMED(PC_ROW_TOPK, launch_row_topk(DT_F32, logits, nullptr, nullptr, M, V, ks, hp.eos, 1, at<float>(p.cand_score),
                                       at<int32_t>(p.cand_idx), s));
  TIMED(PC_REFINE, launch_sample(at<float>(p.cand_score), at<int32_t>(p.cand_idx), at<int32_t>(p.tokens),
                                 at<int32_t>(p.len), at<float>(p.score), at<int32_t>(p.active), step, M, ks, hp.topp, T,
                                 (unsigned long long)hp.seed, hp.cap_extra, s));
  return LSQ_OK;
}

// One decode step: replay the captured graph for this number of live sentences, capturing it on
// first use.  Graphs need a capturable (non-default) stream and are bypassed while per-kernel
// timing is on.
int enqueue_step() {
  const int B = g.alive_at[g.t];
  auto launch = [&](int n) { return g.hp.arch == 1 ? launch_step_gpt(n) : launch_step(n); };
  g.hidden_in_alt = false;   // launch_step says otherwise
  if (!g.use_graphs || g.stream == nullptr || g_prof.on) {
    int rc = launch(B);
    if (rc) return rc;
    g.t += 1;
    return LSQ_OK;
  }
  // the captured launches depend on the number of live sentences and, through the geometry of
  // cross-attention, on the longest source sentence
  const int key = B * 2 + (g.hp.arch == 0 && cross_attention_splits(B * g.hp.H, g.src_longest) ? 1 : 0);
  auto it = g.graphs.find(key);
  if (it == g.graphs.end()) {
    hipGraph_t graph = nullptr;
    HIPCHK(hipStreamBeginCapture(g.stream, hipStreamCaptureModeThreadLocal));
    int rc = launch(B);
    hipError_t e = hipStreamEndCapture(g.stream, &graph);
    if (rc) { if (graph) (void)hipGraphDestroy(graph); return rc; }
    if (e != hipSuccess) return fail(LSQ_E_HIP, "hipStreamEndCapture failed: %s", hipGetErrorString(e));
    hipGraphExec_t exec = nullptr;
    e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (e != hipSuccess) return fail(LSQ_E_HIP, "hipGraphInstantiate failed: %s", hipGetErrorString(e));
    it = g.graphs.emplace(key, exec).first;
    g.graph_hidden_in_alt[key] = g.hidden_in_alt;
  }
  g.hidden_in_alt = g.graph_hidden_in_alt[key];
  HIPCHK(hipGraphLaunch(it->second, g.stream));
  g.t += 1;
  return LSQ_OK;
}

int read_active(int step, int* out) {
  int32_t* slot = g.pinned + g.pinned_ints - 1;
  HIPCHK(hipMemcpyAsync(slot, at<int32_t>(g.plan.active) + step, 4, hipMemcpyDeviceToHost, g.stream));
  HIPCHK(hipStreamSynchronize(g.stream));
  *out = *slot;
  return LSQ_OK;
}

// Decoder-only model: "encode" takes the prompts (all of one length P), runs the blocks over their
// first P-1 tokens to fill the K/V cache (causal attention inside the prompt), and leaves the last
// prompt token as the input of decode step 0, so that every sampled token comes from a decode step.
int encode_gpt(const int32_t* ids, const int32_t* lens, int batch, int stride) {
  const HParams& hp = g.hp;
  const Plan& p = g.plan;
  const int P = lens[0], T = g.max_len, n_new = hp.cap_extra;
  for (int b = 0; b < batch; ++b)
    if (lens[b] != P) return fail(LSQ_E_ARG, "decoder-only models need prompts of one length (got %d and %d)", P, lens[b]);
  if (P + n_new > T + 1) return fail(LSQ_E_ARG, "prompt %d + %d new tokens do not fit max_len %d", P, n_new, T);
  hipStream_t s = g.stream;
  const int R = batch * (P - 1);
  const size_t Rmax = (size_t)g.max_batch * g.max_len;
  int32_t* h_ids = g.pinned;
  int32_t* h_pos = h_ids + Rmax;
  int32_t* h_sent = h_pos + Rmax;
  int32_t* h_off = h_sent + Rmax;
  int32_t* h_len = h_off + g.max_batch + 1;
  int32_t* h_order = h_len + 2 * g.max_batch;
  int32_t* h_tok = h_order + g.max_batch + 2;                  // [batch, T+1] token histories
  int32_t* h_row = h_tok + (size_t)g.max_batch * (T + 1);      // [batch] index of the last token
  int32_t* h_step = h_row + g.max_batch;                       // step_state
  g.order.resize(batch);
  for (int b = 0; b < batch; ++b) {
    g.order[b] = b;
    h_order[b] = b;
    h_off[b] = b * (P - 1);
    h_len[b] = P - 1;
    h_row[b] = P - 1;
    for (int j = 0; j <= T; ++j) h_tok[(size_t)b * (T + 1) + j] = j < P ? ids[(size_t)b * stride + j] : hp.pad;
    for (int j = 0; j + 1 < P; ++j) {
      h_ids[b * (P - 1) + j] = ids[(size_t)b * stride + j];
      h_pos[b * (P - 1) + j] = j;
      h_sent[b * (P - 1) + j] = b;
    }
  }
  h_off[batch] = R;
  h_step[0] = P - 1; h_step[1] = 0; h_step[2] = P - 1; h_step[3] = 0;
  g.alive_at.assign(g.max_len + 1, 0);
  for (int t = 0; t < n_new && t <= g.max_len; ++t) g.alive_at[t] = batch;
  if (R > 0) {
    HIPCHK(hipMemcpyAsync(g.ws + p.e_ids, h_ids, (size_t)R * 4, hipMemcpyHostToDevice, s));
    HIPCHK(hipMemcpyAsync(g.ws + p.e_pos, h_pos, (size_t)R * 4, hipMemcpyHostToDevice, s));
    HIPCHK(hipMemcpyAsync(g.ws + p.e_sent, h_sent, (size_t)R * 4, hipMemcpyHostToDevice, s));
  }
  HIPCHK(hipMemcpyAsync(g.ws + p.src_off, h_off, (size_t)(batch + 1) * 4, hipMemcpyHostToDevice, s));
  HIPCHK(hipMemcpyAsync(g.ws + p.src_len, h_len, (size_t)batch * 4, hipMemcpyHostToDevice, s));
  HIPCHK(hipMemcpyAsync(g.ws + p.order, h_order, (size_t)batch * 4, hipMemcpyHostToDevice, s));
  HIPCHK(hipMemcpyAsync(g.ws + p.tokens, h_tok, (size_t)batch * (T + 1) * 4, hipMemcpyHostToDevice, s));
  HIPCHK(hipMemcpyAsync(g.ws + p.len, h_row, (size_t)batch * 4, hipMemcpyHostToDevice, s));
  HIPCHK(hipMemcpyAsync(g.ws + p.step_state, h_step, 16, hipMemcpyHostToDevice, s));
  HIPCHK(hipMemsetAsync(g.ws + p.score, 0, (size_t)batch * 4, s));
  HIPCHK(hipMemsetAsync(g.ws + p.active, 0, (size_t)(T + 1) * 4, s));

  const int dt = hp.dtype, d = hp.d, F = hp.F, H = hp.H;
  const size_t es = esz();
  char* x = g.ws + p.e_x; char* y = g.ws + p.e_y; char* qkv = g.ws + p.e_qkv; char* ctx = g.ws + p.e_ctx;
  char* tmp = g.ws + p.e_tmp; char* ffn = g.ws + p.e_ffn;
  const int32_t* sent = at<int32_t>(p.e_sent);
  const int32_t* pos = at<int32_t>(p.e_pos);
  const size_t slab = (size_t)g.max_batch * T * d * es;
  if (R > 0) {
    HIPCHK(launch_embed_rows(dt, g.E, at<float>(p.pe), at<int32_t>(p.e_ids), pos, x, R, d, 1.0f, s));
    HIPCHK(launch_add_layernorm_partials(dt, x, y, nullptr, 0, nullptr, g.gpt[0].ln1g, g.gpt[0].ln1b, R, d, hp.eps, s));
    for (int l = 0; l < hp.n_dec; ++l) {
      const GptLayer& L = g.gpt[l];
      char* Kc = g.ws + p.cache + (size_t)(2 * l) * slab;
      HIPCHK(launch_gemm(dt, y, L.Wqkv, L.bqkv, plain_out(qkv, 3 * d), R, 3 * d, d, 0, s));
      HIPCHK(launch_scatter_kv(dt, qkv, sent, pos, Kc, Kc + slab, R, d, T, s));
      HIPCHK(launch_encoder_attention(dt, qkv, sent, at<int32_t>(p.src_off), at<int32_t>(p.src_len), ctx, R, H, d, 1, s));
      if (int rc = sublayer(-1, ctx, L.Wo, L.bo, L.ln2g, L.ln2b, x, y, (float*)tmp, R, d, d, 1, s)) return rc;
      HIPCHK(launch_gemm(dt, y, L.W1, L.b1, plain_out(ffn, F), R, F, d, 2, s));
      const bool last = l + 1 == hp.n_dec;
      if (int rc = sublayer(-1, ffn, L.W2, L.b2, last ? g.lnfg : g.gpt[l + 1].ln1g, last ? g.lnfb : g.gpt[l + 1].ln1b,
                            x, y, (float*)tmp, R, d, F, 1, s)) return rc;
    }
  }
  for (size_t c : p.dec_canaries) HIPCHK(hipMemsetAsync(g.ws + c, kCanaryByte, kCanaryBytes, s));
  g.batch = batch;
  g.rows_enc = R;
  g.prompt_len = P;
  g.t = 0;
  g.done = false;
  g.state = 3;
  return LSQ_OK;
}

}  // namespace

extern "C" {

const char* lsq_last_error(void) { return g_err; }

int lsq_workspace_bytes(const void* weights, size_t weights_bytes, int max_batch, int beam, int max_len,
                        size_t* out_bytes) {
  if (!out_bytes) return fail(LSQ_E_ARG, "out_bytes is null");
  HParams hp;
  int rc = parse_header(weights, weights_bytes, &hp);
  if (rc) return rc;
  rc = check_limits(max_batch, beam, max_len, hp);
  if (rc) return rc;
  if (blob_bytes(hp) != hp.total)
    return fail(LSQ_E_BLOB, "header says %llu bytes, its shapes add up to %zu", (unsigned long long)hp.total, blob_bytes(hp));
  *out_bytes = make_plan(hp, device_weight_bytes(hp), max_batch, beam, max_len).total;
  return LSQ_OK;
}

int lsq_set_workspace(void* dev_ptr, size_t bytes, void* hip_stream) {
  if (!dev_ptr || bytes == 0) return fail(LSQ_E_ARG, "workspace is null or empty");
  if (reinterpret_cast<uintptr_t>(dev_ptr) % kAlign) return fail(LSQ_E_ARG, "workspace must be 256-byte aligned");
  if (g.state >= 2) return fail(LSQ_E_STATE, "a model is loaded; call lsq_free first");
  g.ws = (char*)dev_ptr;
  g.ws_bytes = bytes;
  g.stream = (hipStream_t)hip_stream;
  g.state = 1;
  return LSQ_OK;
}

int lsq_init(const void* weights, size_t weights_bytes, int max_batch, int beam, int max_len) {
  if (g.state < 1) return fail(LSQ_E_STATE, "lsq_set_workspace has not been called");
  if (g.state >= 2) return fail(LSQ_E_STATE, "already initialised; call lsq_free first");
  HParams hp;
  int rc = parse_header(weights, weights_bytes, &hp);
  if (rc) return rc;
  rc = check_limits(max_batch, beam, max_len, hp);
  if (rc) return rc;
  if (hp.total != weights_bytes) return fail(LSQ_E_BLOB, "blob is %zu bytes, header says %llu", weights_bytes,
                                             (unsigned long long)hp.total);
  std::vector<TensorDesc> ts;
  tensor_walk(hp, &ts);
  const size_t es = hp.dtype == DT_F16 ? 2 : 4;
  if (blob_bytes(hp) != weights_bytes)
    return fail(LSQ_E_BLOB, "blob size %zu does not match its shape (%zu)", weights_bytes, blob_bytes(hp));
  const size_t wbytes = device_weight_bytes(hp);
  Plan plan = make_plan(hp, wbytes, max_batch, beam, max_len);
  if (plan.total > g.ws_bytes)
    return fail(LSQ_E_NOMEM, "workspace has %zu bytes, %zu needed", g.ws_bytes, plan.total);

  // stage the weights on the host: matrices become [out, in] so every GEMM reads K-contiguous rows
  char* stage = nullptr;
  HIPCHK(hipHostMalloc((void**)&stage, wbytes, hipHostMallocDefault));
  memset(stage, 0, wbytes);
  std::vector<char*> dev;
  size_t so = 256, dof = 0;
  for (auto& t : ts) {
    so = up(so);
    dof = up(dof);
    size_t n = (size_t)t.rows * t.cols * es;
    if (t.transpose) transpose_copy((const char*)weights + so, stage + dof, t.rows, t.cols, es);
    else memcpy(stage + dof, (const char*)weights + so, n);
    dev.push_back(g.ws + plan.weights + dof);
    so += n;
    dof += n;
  }
  hipError_t e = hipMemcpyAsync(g.ws + plan.weights, stage, wbytes, hipMemcpyHostToDevice, g.stream);
  if (e == hipSuccess) e = hipStreamSynchronize(g.stream);
  (void)hipHostFree(stage);
  if (e != hipSuccess) return fail(LSQ_E_HIP, "weight upload failed: %s", hipGetErrorString(e));
  gemm_clear_packed();
  if (hp.dtype == DT_F16) {
    size_t po = 0;
    for (size_t i = 0; i < ts.size(); ++i) {
      if (!ts[i].gemm) continue;
      const int N = ts[i].transpose ? ts[i].cols : ts[i].rows, K = ts[i].transpose ? ts[i].rows : ts[i].cols;
      const size_t nb = gemm_packed_bytes(N, K);
      if (nb == 0) continue;   // K not a multiple of 16: the products read the row-major copy
      char* dst = g.ws + plan.wpacked + po;
      HIPCHK(launch_pack_weights(dev[i], dst, N, K, g.stream));
      gemm_register_packed(dev[i], dst, N, K);
      po += up(nb);
    }
    HIPCHK(hipStreamSynchronize(g.stream));
  }

  // position table in fp32: sinusoidal, evaluated in double precision, or the model's learned one
  {
    const int d = hp.d;
    float* pe = nullptr;
    HIPCHK(hipHostMalloc((void**)&pe, (size_t)max_len * d * 4, hipHostMallocDefault));
    if (hp.arch == 1) {
      const char* P = (const char*)weights + up(256 + (size_t)hp.V * d * es);   // second tensor of the blob
      for (size_t i = 0; i < (size_t)max_len * d; ++i)
        pe[i] = es == 2 ? (float)((const _Float16*)P)[i] : ((const float*)P)[i];
    }
    for (int pos = 0; pos < max_len && hp.arch == 0; ++pos)
      for (int i = 0; i < d; i += 2) {
        double ang = (double)pos / std::pow(10000.0, (double)i / d);
        pe[(size_t)pos * d + i] = (float)std::sin(ang);
        if (i + 1 < d) pe[(size_t)pos * d + i + 1] = (float)std::cos(ang);
      }
    e = hipMemcpyAsync(g.ws + plan.pe, pe, (size_t)max_len * d * 4, hipMemcpyHostToDevice, g.stream);
    if (e == hipSuccess) e = hipStreamSynchronize(g.stream);
    (void)hipHostFree(pe);
    if (e != hipSuccess) return fail(LSQ_E_HIP, "position table upload failed: %s", hipGetErrorString(e));
  }

  for (size_t c : plan.canaries) HIPCHK(hipMemsetAsync(g.ws + c, kCanaryByte, kCanaryBytes, g.stream));
  HIPCHK(hipStreamSynchronize(g.stream));
  g.pinned_ints = (size_t)3 * max_batch * max_len + 4 * (size_t)max_batch + 2 + (size_t)max_batch * (max_len + 2) + 8;
  HIPCHK(hipHostMalloc((void**)&g.pinned, g.pinned_ints * 4, hipHostMallocDefault));

  g.hp = hp;
  g.plan = plan;
  g.max_batch = max_batch; g.beam = beam; g.max_len = max_len;
  size_t i = 0;
  g.E = dev[i++];
  if (hp.arch == 1) {
    ++i;   // learned positions: used through the fp32 table
    g.gpt.assign(hp.n_dec, GptLayer{});
    for (auto& L : g.gpt) {
      L.ln1g = dev[i++]; L.ln1b = dev[i++]; L.Wqkv = dev[i++]; L.bqkv = dev[i++]; L.Wo = dev[i++]; L.bo = dev[i++];
      L.ln2g = dev[i++]; L.ln2b = dev[i++]; L.W1 = dev[i++]; L.b1 = dev[i++]; L.W2 = dev[i++]; L.b2 = dev[i++];
    }
    g.lnfg = dev[i++]; g.lnfb = dev[i++];
    g.state = 2;
    return LSQ_OK;
  }
  g.enc.assign(hp.n_enc, EncLayer{});
  for (auto& L : g.enc) {
    L.Wqkv = dev[i++]; L.bqkv = dev[i++]; L.Wo = dev[i++]; L.bo = dev[i++]; L.ln1g = dev[i++]; L.ln1b = dev[i++];
    L.W1 = dev[i++]; L.b1 = dev[i++]; L.W2 = dev[i++]; L.b2 = dev[i++]; L.ln2g = dev[i++]; L.ln2b = dev[i++];
  }
  g.dec.assign(hp.n_dec, DecLayer{});
  for (auto& L : g.dec) {
    L.Wqkv = dev[i++]; L.bqkv = dev[i++]; L.Wo = dev[i++]; L.bo = dev[i++]; L.ln1g = dev[i++]; L.ln1b = dev[i++];
    L.Wq = dev[i++]; L.bq = dev[i++]; L.Wkv = dev[i++]; L.bkv = dev[i++]; L.Woc = dev[i++]; L.boc = dev[i++];
    L.ln2g = dev[i++]; L.ln2b = dev[i++];
    L.W1 = dev[i++]; L.b1 = dev[i++]; L.W2 = dev[i++]; L.b2 = dev[i++]; L.ln3g = dev[i++]; L.ln3b = dev[i++];
  }
  g.state = 2;
  return LSQ_OK;
}

int lsq_encode(const int32_t* src_ids, const int32_t* src_lens, int batch, int src_stride) {
  if (g.state < 2) return fail(LSQ_E_STATE, "lsq_init has not been called");
  if (!src_ids || !src_lens) return fail(LSQ_E_ARG, "src_ids / src_lens is null");
  if (batch < 1 || batch > g.max_batch) return fail(LSQ_E_ARG, "batch %d outside [1, %d]", batch, g.max_batch);
  if (src_stride < 1 || src_stride > g.max_len)
    return fail(LSQ_E_ARG, "src_stride %d outside [1, max_len = %d]", src_stride, g.max_len);
  const HParams& hp = g.hp;
  long R = 0;
  for (int b = 0; b < batch; ++b) {
    int n = src_lens[b];
    if (n < 1 || n > src_stride) return fail(LSQ_E_ARG, "src_lens[%d] = %d outside [1, %d]", b, n, src_stride);
    for (int j = 0; j < n; ++j) {
      int id = src_ids[(size_t)b * src_stride + j];
      if (id < 0 || id >= hp.V) return fail(LSQ_E_ARG, "src_ids[%d,%d] = %d outside the vocabulary", b, j, id);
    }
    R += n;
  }
  HIPCHK(hipStreamSynchronize(g.stream));   // the staging buffer may still feed an earlier copy
  const int groups = hp.arch == 0 ? g.groups_next : 1;
  if (g.beam % groups != 0) return fail(LSQ_E_ARG, "beam %d is not a multiple of %d groups", g.beam, groups);
  const bool anc_on = hp.arch == 0 && g.beam > 1 && g.refresh_mode == 1;
  if (groups != g.groups || (groups > 1 && g.strength_next != g.strength)) {
    for (auto& kv : g.graphs) (void)hipGraphExecDestroy(kv.second);
    g.graphs.clear();
    g.graph_hidden_in_alt.clear();
  }
  g.groups = groups;
  g.strength = g.strength_next;
  if (anc_on != g.anc_on) {   // captured steps hold the other mode's kernels and arguments
    for (auto& kv : g.graphs) (void)hipGraphExecDestroy(kv.second);
    g.graphs.clear();
    g.graph_hidden_in_alt.clear();
    g.anc_on = anc_on;
  }
  if (hp.arch == 1) return encode_gpt(src_ids, src_lens, batch, src_stride);
  const Plan& p = g.plan;
  const size_t Rmax = (size_t)g.max_batch * g.max_len;
  int32_t* h_ids = g.pinned;
  int32_t* h_pos = h_ids + Rmax;
  int32_t* h_sent = h_pos + Rmax;
  int32_t* h_off = h_sent + Rmax;            // batch + 1
  int32_t* h_len = h_off + g.max_batch + 1;  // batch
  int32_t* h_cap = h_len + g.max_batch;      // batch
  int32_t* h_order = h_cap + g.max_batch;    // batch
  // Internal sentence order: by cap, descending (stable).  A sentence is certainly finished once
  // it has taken cap steps, so the sentences that can still be unfinished at step t are a prefix
  // whose length alive_at[t] the host knows in advance; every kernel of step t is launched on
  // that prefix only.  Results are handed back in the caller's order.
  g.order.resize(batch);
  for (int b = 0; b < batch; ++b) g.order[b] = b;
  auto cap_of = [&](int b) { return std::min(src_lens[b] + hp.cap_extra, g.max_len); };
  std::stable_sort(g.order.begin(), g.order.end(), [&](int a, int b) { return cap_of(a) > cap_of(b); });
  g.alive_at.assign(g.max_len + 1, 0);
  for (int b = 0; b < batch; ++b)
    for (int t = 0; t < cap_of(b); ++t) g.alive_at[t] += 1;
  int r = 0;
  for (int i = 0; i < batch; ++i) {
    const int b = g.order[i];
    h_off[i] = r;
    h_len[i] = src_lens[b];
    h_cap[i] = cap_of(b);
    h_order[i] = b;
    for (int j = 0; j < src_lens[b]; ++j, ++r) {
      h_ids[r] = src_ids[(size_t)b * src_stride + j];
      h_pos[r] = j;
      h_sent[r] = i;
    }
  }
  h_off[batch] = r;
  hipStream_t s = g.stream;
  HIPCHK(hipMemcpyAsync(g.ws + p.e_ids, h_ids, (size_t)R * 4, hipMemcpyHostToDevice, s));
  HIPCHK(hipMemcpyAsync(g.ws + p.e_pos, h_pos, (size_t)R * 4, hipMemcpyHostToDevice, s));
  HIPCHK(hipMemcpyAsync(g.ws + p.e_sent, h_sent, (size_t)R * 4, hipMemcpyHostToDevice, s));
  HIPCHK(hipMemcpyAsync(g.ws + p.src_off, h_off, (size_t)(batch + 1) * 4, hipMemcpyHostToDevice, s));
  HIPCHK(hipMemcpyAsync(g.ws + p.src_len, h_len, (size_t)batch * 4, hipMemcpyHostToDevice, s));
  HIPCHK(hipMemcpyAsync(g.ws + p.cap, h_cap, (size_t)batch * 4, hipMemcpyHostToDevice, s));
  HIPCHK(hipMemcpyAsync(g.ws + p.order, h_order, (size_t)batch * 4, hipMemcpyHostToDevice, s));

  const int dt = hp.dtype, d = hp.d, F = hp.F, H = hp.H;
  const size_t es = esz();
  char* x = g.ws + p.e_x; char* qkv = g.ws + p.e_qkv; char* ctx = g.ws + p.e_ctx; char* tmp = g.ws + p.e_tmp;
  char* ffn = g.ws + p.e_ffn;
  const int32_t* sent = at<int32_t>(p.e_sent);
  const int32_t* off = at<int32_t>(p.src_off);
  const int32_t* len = at<int32_t>(p.src_len);
  HIPCHK(launch_embed_rows(dt, g.E, at<float>(p.pe), at<int32_t>(p.e_ids), at<int32_t>(p.e_pos), x, (int)R, d, sqrtf((float)d), s));
  for (const EncLayer& L : g.enc) {
    HIPCHK(launch_gemm(dt, x, L.Wqkv, L.bqkv, plain_out(qkv, 3 * d), (int)R, 3 * d, d, 0, s));
    HIPCHK(launch_encoder_attention(dt, qkv, sent, off, len, ctx, (int)R, H, d, 0, s));
    if (int rc = sublayer(-1, ctx, L.Wo, L.bo, L.ln1g, L.ln1b, x, nullptr, (float*)tmp, (int)R, d, d, 1, s)) return rc;
    HIPCHK(launch_gemm(dt, x, L.W1, L.b1, plain_out(ffn, F), (int)R, F, d, 1, s));
    if (int rc = sublayer(-1, ffn, L.W2, L.b2, L.ln2g, L.ln2b, x, nullptr, (float*)tmp, (int)R, d, F, 1, s)) return rc;
  }
  const size_t cross_l = (size_t)g.max_batch * g.max_len * 2 * d * es;   // layer stride of the maximum shape
  for (int l = 0; l < hp.n_dec; ++l)
    HIPCHK(launch_gemm(dt, x, g.dec[l].Wkv, g.dec[l].bkv, plain_out(g.ws + p.cross + l * cross_l, 2 * d), (int)R,
                       2 * d, d, 0, s));
  HIPCHK(launch_beam_reset(at<float>(p.score), at<int32_t>(p.tokens), at<int32_t>(p.len), at<int32_t>(p.fin),
                           at<int32_t>(p.active), at<int32_t>(p.step_state), g.anc_on ? at<int32_t>(p.anc) : nullptr,
                           at<int32_t>(p.pen_n), batch, g.beam, g.beam / g.groups, g.max_len, hp.bos,
                           hp.pad, s));
  // the first step's decoder input (BOS at position 0); later ones are left by each step's re-rank kernel
  // sampling decoding: one launch for retrieve + draw + next input when every row count of this translation has a
  // logit product that leaves group statistics (decided here, for the whole translation)
  bool fold = false;
  if (hp.sample_topk > 0 && g.topk_stats && g.merge_rerank && topk_groups_supported(hp.V, hp.sample_topk, 1)) {
    fold = true;
    for (int m = 1; m <= batch * g.beam; ++m) fold = fold && gemm_writes_stats(dt, m, hp.V, d);
  }
  if (fold != g.sample_fold) {   // captured steps hold the other variant's launches
    for (auto& kv : g.graphs) (void)hipGraphExecDestroy(kv.second);
    g.graphs.clear();
    g.graph_hidden_in_alt.clear();
  }
  g.sample_fold = fold;
  if (hp.sample_topk == 0 || g.sample_fold)
    HIPCHK(launch_embed_last(dt, g.E, at<float>(p.pe), at<int32_t>(p.tokens), at<int32_t>(p.len), g.ws + p.d_x0,
                             batch * g.beam, d, g.max_len, at<int32_t>(p.step_state), sqrtf((float)d), s));
  for (size_t c : p.dec_canaries) HIPCHK(hipMemsetAsync(g.ws + c, kCanaryByte, kCanaryBytes, s));
  g.batch = batch;
  g.rows_enc = (int)R;
  g.src_longest = *std::max_element(src_lens, src_lens + batch);
  g.t = 0;
  g.done = false;
  g.state = 3;
  return LSQ_OK;
}

int lsq_decode_step(void) { return lsq_decode_steps(1); }

int lsq_decode_steps(int n) {
  if (g.state < 3) return fail(LSQ_E_STATE, "lsq_encode has not been called");
  if (n < 1) return fail(LSQ_E_ARG, "n must be positive");
  if (g.done || g.t >= g.max_len || g.alive_at[g.t] == 0) return 0;
  int issued = 0;
  while (issued < n && g.t < g.max_len && g.alive_at[g.t] > 0) {
    int rc = enqueue_step();
    if (rc) return rc;
    ++issued;
  }
  int active = 0;
  int rc = read_active(g.t - 1, &active);
  if (rc) return rc;
  if (active == 0) g.done = true;
  return active;
}

int lsq_profile_enable(int on) {
  if (g_prof.used) return fail(LSQ_E_STATE, "read the pending profile first");
  g_prof.on = on != 0;
  return LSQ_OK;
}

int lsq_profile_classes(void) { return PC_COUNT; }

const char* lsq_profile_class_name(int c) { return (c >= 0 && c < PC_COUNT) ? kProfNames[c] : ""; }

int lsq_profile_read(double* ms, int64_t* launches, int n) {
  if (!ms || !launches || n < PC_COUNT) return fail(LSQ_E_ARG, "need %d slots", (int)PC_COUNT);
  for (int i = 0; i < n; ++i) { ms[i] = 0; launches[i] = 0; }
  if (g.state >= 1) HIPCHK(hipStreamSynchronize(g.stream));
  for (size_t i = 0; i < g_prof.used; ++i) {
    float t = 0.f;
    HIPCHK(hipEventElapsedTime(&t, g_prof.pool[2 * i], g_prof.pool[2 * i + 1]));
    ms[g_prof.cls[i]] += t;
    launches[g_prof.cls[i]] += 1;
  }
  g_prof.used = 0;
  return LSQ_OK;
}

int lsq_set_graphs(int on) {
  g.use_graphs = on != 0;
  return LSQ_OK;
}

int lsq_set_layernorm_fusion(int on) {
  if ((on != 0) != g.fuse_ln) {   // captured steps hold the other variant's launches
    if (g.stream) (void)hipStreamSynchronize(g.stream);
    for (auto& kv : g.graphs) (void)hipGraphExecDestroy(kv.second);
    g.graphs.clear();
    g.graph_hidden_in_alt.clear();
  }
  g.fuse_ln = on != 0;
  return LSQ_OK;
}

int lsq_set_topk_statistics(int mode) {
  if (mode < 0 || mode > 2) return fail(LSQ_E_ARG, "mode %d outside [0, 2]", mode);
  const bool stats = mode != 0, merge = mode == 1;
  if (stats != g.topk_stats || merge != g.merge_rerank) {   // captured steps hold the other variant's launches
    if (g.stream) (void)hipStreamSynchronize(g.stream);
    for (auto& kv : g.graphs) (void)hipGraphExecDestroy(kv.second);
    g.graphs.clear();
    g.graph_hidden_in_alt.clear();
  }
  g.topk_stats = stats;
  g.merge_rerank = merge;
  return LSQ_OK;
}

int lsq_set_attention_blocks(int max_rows) {
  if (max_rows < 0 || max_rows > (int)kBlockRowsMax) return fail(LSQ_E_ARG, "max_rows %d outside [0, %d]", max_rows, (int)kBlockRowsMax);
  if (max_rows != g.block_rows) {   // captured steps hold the other variant's launches
    if (g.stream) (void)hipStreamSynchronize(g.stream);
    for (auto& kv : g.graphs) (void)hipGraphExecDestroy(kv.second);
    g.graphs.clear();
    g.graph_hidden_in_alt.clear();
  }
  g.block_rows = max_rows;
  return LSQ_OK;
}

int lsq_set_diversity(int groups, float strength) {
  if (groups < 1 || groups > LSQ_MAX_BEAM) return fail(LSQ_E_ARG, "groups %d outside [1, %d]", groups, LSQ_MAX_BEAM);
  if (!(strength >= 0.f)) return fail(LSQ_E_ARG, "diversity strength must be >= 0");
  g.groups_next = groups;
  g.strength_next = strength;
  return LSQ_OK;
}

int lsq_set_cache_refresh(int mode) {
  if (mode != LSQ_REFRESH_MOVE && mode != LSQ_REFRESH_TABLE) return fail(LSQ_E_ARG, "unknown cache refresh mode %d", mode);
  g.refresh_mode = mode;
  return LSQ_OK;
}

int lsq_step_index(void) { return g.state >= 3 ? g.t : 0; }

int lsq_set_canaries(int on) {
  if (g.state >= 2) return fail(LSQ_E_STATE, "a model is loaded: the memory plan is fixed; call lsq_free first");
  g_canaries = on != 0;
  return LSQ_OK;
}

int lsq_debug_check_canaries(void) {
  if (g.state < 2) return fail(LSQ_E_STATE, "lsq_init has not been called");
  HIPCHK(hipStreamSynchronize(g.stream));
  std::vector<size_t> zones = g.plan.canaries;
  if (g.state >= 3) zones.insert(zones.end(), g.plan.dec_canaries.begin(), g.plan.dec_canaries.end());
  std::vector<unsigned char> host(kCanaryBytes);
  int damaged = 0;
  for (size_t c : zones) {
    HIPCHK(hipMemcpy(host.data(), g.ws + c, kCanaryBytes, hipMemcpyDeviceToHost));
    bool ok = true;
    for (unsigned char v : host) ok = ok && v == kCanaryByte;
    damaged += ok ? 0 : 1;
  }
  return damaged;
}

int lsq_get_beams(int32_t* out_ids, int32_t* out_lens, float* out_scores) {
  if (g.state < 3) return fail(LSQ_E_STATE, "lsq_encode has not been called");
  if (!out_ids || !out_lens || !out_scores) return fail(LSQ_E_ARG, "an output pointer is null");
  const Plan& p = g.plan;
  const int M = g.batch * g.beam, T = g.max_len;
  HIPCHK(launch_finalize(at<float>(p.score), at<int32_t>(p.tokens), at<int32_t>(p.len), at<int32_t>(p.out_ids),
                         at<int32_t>(p.out_lens), at<float>(p.out_scores), at<int32_t>(p.order), g.batch, g.beam,
                         T, g.hp.arch == 1 ? 0.0f : g.hp.alpha, g.hp.pad, g.hp.arch == 1 ? g.prompt_len : 1,
                         g.stream));
  HIPCHK(hipMemcpyAsync(out_ids, g.ws + p.out_ids, (size_t)M * T * 4, hipMemcpyDeviceToHost, g.stream));
  HIPCHK(hipMemcpyAsync(out_lens, g.ws + p.out_lens, (size_t)M * 4, hipMemcpyDeviceToHost, g.stream));
  HIPCHK(hipMemcpyAsync(out_scores, g.ws + p.out_scores, (size_t)M * 4, hipMemcpyDeviceToHost, g.stream));
  HIPCHK(hipStreamSynchronize(g.stream));
  return LSQ_OK;
}

void lsq_free(void) {
  if (!g.graphs.empty()) {
    (void)hipStreamSynchronize(g.stream);
    for (auto& kv : g.graphs) (void)hipGraphExecDestroy(kv.second);
    g.graphs.clear();
    g.graph_hidden_in_alt.clear();
  }
  if (g.pinned) {
    if (g.stream || g.state >= 2) (void)hipStreamSynchronize(g.stream);
    (void)hipHostFree(g.pinned);
  }
  gemm_clear_packed();
  g = Ctx{};
}

int lsq_debug_read(int what, void* host_dst, size_t bytes) {
  if (g.state < 3) return fail(LSQ_E_STATE, "lsq_encode has not been called");
  if (!host_dst) return fail(LSQ_E_ARG, "host_dst is null");
  const Plan& p = g.plan;
  const HParams& hp = g.hp;
  const size_t M = (size_t)g.batch * g.beam, T = g.max_len, d = hp.d, R = g.rows_enc;
  const char* src = nullptr;
  size_t n = 0;
  bool is_float_data = false;   // stored in the model dtype, delivered as float
  bool per_source_row = false;  // leading dimension is packed source rows, not batch*beam rows
  bool cache_item = false;
  switch (what) {
    case LSQ_DBG_LOGITS: src = g.ws + p.d_logits; n = M * hp.V; break;   // always fp32
    case LSQ_DBG_SCORE: src = g.ws + p.score; n = M; break;
    case LSQ_DBG_TOKENS: src = g.ws + p.tokens; n = M * (T + 1); break;
    case LSQ_DBG_LEN: src = g.ws + p.len; n = M; break;
    case LSQ_DBG_FINISHED: src = g.ws + p.fin; n = M; break;
    case LSQ_DBG_PARENT: src = g.ws + p.parent; n = M; break;
    case LSQ_DBG_CAND_SCORE: src = g.ws + p.cand_score; n = M * (hp.sample_topk > 0 ? hp.sample_topk : g.beam); break;
    case LSQ_DBG_CAND_IDX: src = g.ws + p.cand_idx; n = M * (hp.sample_topk > 0 ? hp.sample_topk : g.beam); break;
    case LSQ_DBG_HIDDEN: src = g.ws + (g.hidden_in_alt ? p.d_x2 : p.d_x); n = M * d; is_float_data = true; break;
    case LSQ_DBG_MEMORY:
      if (g.t != 0) return fail(LSQ_E_STATE, "encoder output is overwritten by the first decode step");
      src = g.ws + p.e_x; n = R * d; is_float_data = true; per_source_row = true; break;
    default: {
      int l = what % 100, kind = what - l;
      if (l < 0 || l >= hp.n_dec) return fail(LSQ_E_ARG, "unknown debug item %d", what);
      if (kind == LSQ_DBG_CROSS_KV) { n = R * 2 * d; src = g.ws + p.cross + (size_t)l * g.max_batch * g.max_len * 2 * d * esz(); per_source_row = true; }
      else if (kind == LSQ_DBG_CACHE_K) { cache_item = true; n = M * T * d; src = g.ws + p.cache + (size_t)(2 * l) * g.max_batch * g.beam * T * d * esz(); }
      else if (kind == LSQ_DBG_CACHE_V) { cache_item = true; n = M * T * d; src = g.ws + p.cache + (size_t)(2 * l + 1) * g.max_batch * g.beam * T * d * esz(); }
      else return fail(LSQ_E_ARG, "unknown debug item %d", what);
      is_float_data = true;
    }
  }
  if (bytes != n * 4) return fail(LSQ_E_ARG, "debug item %d has %zu bytes, caller gave %zu", what, n * 4, bytes);
  // download in the internal sentence order, widen, then hand back in the caller's order
  std::vector<float> raw(n);
  if (!is_float_data || hp.dtype == DT_F32) {
    HIPCHK(hipMemcpyAsync(raw.data(), src, n * 4, hipMemcpyDeviceToHost, g.stream));
    HIPCHK(hipStreamSynchronize(g.stream));
  } else {
    std::vector<_Float16> tmp(n);
    HIPCHK(hipMemcpyAsync(tmp.data(), src, n * 2, hipMemcpyDeviceToHost, g.stream));
    HIPCHK(hipStreamSynchronize(g.stream));
    for (size_t i = 0; i < n; ++i) raw[i] = (float)tmp[i];
  }
  if (cache_item && g.anc_on) {
    // hand the cache back as if rows had been moved: position j of row r comes from the slab the table names
    std::vector<int32_t> anc((size_t)M * (T + 1));
    HIPCHK(hipMemcpyAsync(anc.data(), g.ws + p.anc, anc.size() * 4, hipMemcpyDeviceToHost, g.stream));
    HIPCHK(hipStreamSynchronize(g.stream));
    std::vector<float> moved(n);
    const size_t written = std::min((size_t)g.t, T);   // positions 0..t-1 hold keys/values; the rest is stale either way
    for (size_t r = 0; r < M; ++r)
      for (size_t j = 0; j < T; ++j) {
        const size_t from = j < written ? r - r % g.beam + (size_t)anc[r * (T + 1) + j] : r;
        memcpy(&moved[(r * T + j) * d], &raw[(from * T + j) * d], d * 4);
      }
    raw.swap(moved);
  }
  float* dst = (float*)host_dst;
  if (per_source_row) {
    // packed encoder rows: sentence i (internal) holds rows off_i .. off_i + len_i
    const size_t width = n / R;
    std::vector<size_t> start_internal(g.batch + 1, 0), len_by_caller(g.batch, 0), start_caller(g.batch + 1, 0);
    for (int i = 0; i < g.batch; ++i) {
      int32_t li = g.pinned[3 * (size_t)g.max_batch * g.max_len + g.max_batch + 1 + i];   // staged lengths
      start_internal[i + 1] = start_internal[i] + li;
      len_by_caller[g.order[i]] = li;
    }
    for (int b = 0; b < g.batch; ++b) start_caller[b + 1] = start_caller[b] + len_by_caller[b];
    for (int i = 0; i < g.batch; ++i)
      memcpy(dst + start_caller[g.order[i]] * width, raw.data() + start_internal[i] * width,
             (start_internal[i + 1] - start_internal[i]) * width * 4);
  } else {
    const size_t per_sentence = n / g.batch;
    for (int i = 0; i < g.batch; ++i)
      memcpy(dst + (size_t)g.order[i] * per_sentence, raw.data() + (size_t)i * per_sentence, per_sentence * 4);
  }
  return LSQ_OK;
}

// ---- single-kernel entry points ---------------------------------------------------------------
#define KCHK(cond, msg) do { if (!(cond)) return fail(LSQ_E_ARG, msg); } while (0)
#define KRUN(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return fail(LSQ_E_HIP, "%s", hipGetErrorString(e_)); return LSQ_OK; } while (0)

int lsq_k_gemm(int dtype, const void* A, const void* B, const void* bias, void* C, int M, int N, int K, int flags,
               void* stream) {
  KCHK(A && B && C, "null matrix");
  KCHK(dtype == DT_F32 || dtype == DT_F16, "dtype");
  KCHK(M >= 0 && N >= 0 && K >= 1, "shape");
  KCHK(dtype == DT_F32 || K % 8 == 0, "K must be a multiple of 8 for float16");
  GemmOut o = plain_out(C, N);
  o.f32_out = (dtype == DT_F16 && (flags & LSQ_GEMM_F32_OUT)) ? 1 : 0;
  const bool packed = (flags & LSQ_GEMM_PACKED_B) != 0;
  KCHK(!packed || (dtype == DT_F16 && M <= 64 && K % 16 == 0), "fragment-ordered weights: float16, at most 64 rows, K a multiple of 16");
  KRUN(launch_gemm(dtype, A, B, bias, o, M, N, K, (flags & LSQ_GEMM_RELU) ? 1 : ((flags & LSQ_GEMM_GELU) ? 2 : 0),
                   (hipStream_t)stream, packed));
}

size_t lsq_k_packed_weight_bytes(int N, int K) { return gemm_packed_bytes(N, K); }

int lsq_k_pack_weights(const void* W, void* packed, int N, int K, void* stream) {
  KCHK(W && packed, "null pointer");
  KCHK(N >= 1 && K >= 16 && K % 16 == 0, "N >= 1, K a positive multiple of 16");
  KCHK((reinterpret_cast<uintptr_t>(W) & 15) == 0 && (reinterpret_cast<uintptr_t>(packed) & 15) == 0, "16-byte alignment");
  KRUN(launch_pack_weights(W, packed, N, K, (hipStream_t)stream));
}

size_t lsq_k_gemm_add_layernorm_scratch(int dtype, int M, int d, int K) {
  return (size_t)std::max(1, gemm_partial_splits(dtype, M, d, K)) * (size_t)M * d * 4;
}

int lsq_k_gemm_add_layernorm(int dtype, const void* in, const void* W, const void* bias, void* x, const void* gamma,
                             const void* beta, int M, int d, int K, float eps, void* scratch, void* stream) {
  KCHK(in && W && bias && x && gamma && beta && scratch, "null pointer");
  KCHK(dtype == DT_F32 || dtype == DT_F16, "dtype");
  KCHK(M >= 0 && d >= 1 && K >= 1, "shape");
  KCHK(dtype == DT_F32 || K % 8 == 0, "K must be a multiple of 8 for float16");
  KCHK((reinterpret_cast<uintptr_t>(scratch) & 15) == 0, "scratch must be 16-byte aligned");
  const int S = gemm_partial_splits(dtype, M, d, K);
  hipError_t e = launch_gemm_partials(dtype, in, W, (float*)scratch, M, d, K, S, (hipStream_t)stream);
  if (e == hipSuccess)
    e = launch_add_layernorm_partials(dtype, x, nullptr, (const float*)scratch, S, bias, gamma, beta, M, d, eps,
                                      (hipStream_t)stream);
  if (e != hipSuccess) return fail(LSQ_E_HIP, "%s", hipGetErrorString(e));
  return LSQ_OK;
}

// ---- the same sublayer tail for callers that cannot allocate ------------------------------------
// The split-K slabs live in a file-scope device array instead of caller memory.  In host code the
// array's name is only a stand-in for the symbol: its device address is asked for once per device
// (hipGetSymbolAddress with that device current) and kept; kernels, and anything else that touches
// the memory from the host, get that address.
}  // extern "C"

namespace {
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;   // 8 slabs of 512 x 1024 floats
constexpr int kMaxDevices = 64;
void* g_static_scratch_ptr[kMaxDevices] = {};
}  // namespace
static __device__ __align__(256) unsigned char lsq_static_scratch[kStaticScratchBytes];

extern "C" {

size_t lsq_k_gemm_add_layernorm_static_limit(void) { return kStaticScratchBytes; }

int lsq_k_gemm_add_layernorm_static(int dtype, const void* in, const void* W, const void* bias, void* x,
                                    const void* gamma, const void* beta, int M, int d, int K, float eps,
                                    void* stream) {
  KCHK(in && W && bias && x && gamma && beta, "null pointer");
  KCHK(dtype == DT_F32 || dtype == DT_F16, "dtype");
  KCHK(M >= 0 && d >= 1 && K >= 1, "shape");
  KCHK(dtype == DT_F32 || K % 8 == 0, "K must be a multiple of 8 for float16");
  const size_t need = lsq_k_gemm_add_layernorm_scratch(dtype, M, d, K);
  if (need > kStaticScratchBytes)
    return fail(LSQ_E_ARG, "this shape needs %zu bytes of partial sums, the built-in buffer holds %zu", need,
                kStaticScratchBytes);
  int dev = -1;
  HIPCHK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(LSQ_E_ARG, "device %d outside [0, %d)", dev, kMaxDevices);
  if (!g_static_scratch_ptr[dev]) {
    void* p = nullptr;
    HIPCHK(hipGetSymbolAddress(&p, HIP_SYMBOL(lsq_static_scratch)));
    if (!p || (reinterpret_cast<uintptr_t>(p) & 15) != 0) return fail(LSQ_E_HIP, "built-in scratch buffer has no usable address");
    g_static_scratch_ptr[dev] = p;
  }
  return lsq_k_gemm_add_layernorm(dtype, in, W, bias, x, gamma, beta, M, d, K, eps, g_static_scratch_ptr[dev], stream);
}

int lsq_k_layernorm_gemm(int dtype, const float* P, int splits, const void* ln_bias, const void* gamma, const void* beta,
                         const void* x_old, void* x_new, float eps, const void* W, const void* bias, void* C, int M,
                         int N, int K, int flags, void* stream) {
  KCHK(P && ln_bias && gamma && beta && x_old && x_new && W && C, "null pointer");
  KCHK(x_old != x_new, "x_new must not be x_old");
  KCHK(gemm_ln_supported(dtype, M, K), "float16, 1..8 rows, K a multiple of 16 up to 1024");
  KCHK(splits >= 1 && splits <= 4 && N >= 0, "shape");
  GemmOut o = plain_out(C, N);
  o.f32_out = (flags & LSQ_GEMM_F32_OUT) ? 1 : 0;
  LnInput ln = {P, splits, (const half_t*)ln_bias, (const half_t*)gamma, (const half_t*)beta, (const half_t*)x_old,
                (half_t*)x_new, eps};
  KRUN(launch_gemm_ln(ln, W, bias, o, M, N, K, (flags & LSQ_GEMM_RELU) ? 1 : ((flags & LSQ_GEMM_GELU) ? 2 : 0),
                      (hipStream_t)stream));
}

int lsq_k_layernorm_cross_attention(const float* P, int splits, const void* ln_bias, const void* gamma,
                                    const void* beta, const void* x_old, void* x_new, float eps, const void* Wq_packed,
                                    const void* bq, const void* kv, const int32_t* src_off, const int32_t* src_len,
                                    void* out, int batch, int beam, int heads, int d, void* stream) {
  KCHK(P && ln_bias && gamma && beta && x_old && x_new && Wq_packed && bq && kv && src_off && src_len && out, "null pointer");
  KCHK(x_old != x_new, "x_new must not be x_old");
  KCHK(batch >= 0 && splits >= 1 && splits <= 4, "shape");
  KCHK(batch == 0 || cross_attention_ln_supported(DT_F16, batch * beam, beam, heads, d),
       "float16, at most 64 rows, beam 1..4, heads of 64, d a multiple of 64 up to 1024");
  LnInput ln = {P, splits, (const half_t*)ln_bias, (const half_t*)gamma, (const half_t*)beta, (const half_t*)x_old,
                (half_t*)x_new, eps};
  KRUN(launch_cross_attention_ln(ln, Wq_packed, bq, kv, src_off, src_len, out, batch, beam, heads, d, (hipStream_t)stream));
}

int lsq_k_self_attention_block(const float* P, int splits, const void* ln_bias, const void* gamma, const void* beta,
                               const void* x_old, void* x_new, float eps, const void* Wqkv_packed, const void* bqkv,
                               const void* Wo_packed, void* Kc, void* Vc, const int32_t* slab_table, int nkeys,
                               float* P_out, int batch, int beam, int heads, int d, int T, int pre_ln, void* stream) {
  KCHK(x_old && Wqkv_packed && bqkv && Wo_packed && Kc && Vc && P_out, "null pointer");
  KCHK(splits >= 0 && splits <= 4, "0..4 slabs");
  KCHK(pre_ln == 0 || pre_ln == 1, "pre_ln is 0 or 1");
  KCHK(splits == 0 || (P && ln_bias && gamma && beta && x_new && x_new != x_old), "LayerNorm inputs; x_new must not be x_old");
  KCHK(!pre_ln || (gamma && beta), "pre-LN rows need gamma and beta");
  KCHK(batch >= 0 && T >= 1 && nkeys >= 0 && nkeys < T, "nkeys outside [0, T)");
  KCHK(batch == 0 || attention_blocks_supported(DT_F16, batch * beam, beam, heads, d),
       "float16, at most 64 rows, beam 1..4, heads of 64, d = 64 * heads a multiple of 256 up to 1024");
  LnInput ln = {P, splits, (const half_t*)ln_bias, (const half_t*)gamma, (const half_t*)beta, (const half_t*)x_old,
                (half_t*)x_new, eps, pre_ln};
  KRUN(launch_self_block(ln, Wqkv_packed, bqkv, Wo_packed, Kc, Vc, slab_table, nullptr, nkeys, P_out, batch, beam, heads, d,
                         T, (hipStream_t)stream));
}

int lsq_k_cross_attention_block(const float* P, int splits, const void* ln_bias, const void* gamma, const void* beta,
                                const void* x_old, void* x_new, float eps, const void* Wq_packed, const void* bq,
                                const void* Wo_packed, const void* kv, const int32_t* src_off, const int32_t* src_len,
                                float* P_out, int batch, int beam, int heads, int d, void* stream) {
  KCHK(P && ln_bias && gamma && beta && x_old && x_new && Wq_packed && bq && Wo_packed && kv && src_off && src_len && P_out,
       "null pointer");
  KCHK(x_old != x_new, "x_new must not be x_old");
  KCHK(batch >= 0 && splits >= 1 && splits <= 16, "1..16 slabs");
  KCHK(batch == 0 || attention_blocks_supported(DT_F16, batch * beam, beam, heads, d),
       "float16, at most 64 rows, beam 1..4, heads of 64, d = 64 * heads a multiple of 256 up to 1024");
  LnInput ln = {P, splits, (const half_t*)ln_bias, (const half_t*)gamma, (const half_t*)beta, (const half_t*)x_old,
                (half_t*)x_new, eps};
  KRUN(launch_cross_block(ln, Wq_packed, bq, Wo_packed, kv, src_off, src_len, P_out, batch, beam, heads, d,
                          (hipStream_t)stream));
}

int lsq_k_cross_attention_q(const void* x, const void* Wq_packed, const void* bq, const void* kv,
                            const int32_t* src_off, const int32_t* src_len, void* out, int batch, int beam, int heads,
                            int d, void* stream) {
  KCHK(x && Wq_packed && bq && kv && src_off && src_len && out, "null pointer");
  KCHK(batch >= 0, "shape");
  KCHK(batch == 0 || cross_attention_q_supported(DT_F16, batch * beam, beam, heads, d),
       "float16, more than 64 rows, beam 1..4, heads of 64, d = 64 * heads <= 1024");
  KRUN(launch_cross_attention_q(x, Wq_packed, bq, kv, src_off, src_len, out, batch, beam, heads, d, (hipStream_t)stream));
}

int lsq_k_self_attention(int dtype, const void* q, const void* Kc, const void* Vc, void* out, int rows, int heads,
                         int d, int T, int nkeys, void* stream) {
  KCHK(q && Kc && Vc && out, "null pointer");
  KCHK(dtype == DT_F32 || dtype == DT_F16, "dtype");
  KCHK(rows >= 0 && heads >= 1 && d % heads == 0 && head_dim_supported(d / heads), "head size must be 16/32/64/128");
  KCHK(nkeys >= 1 && nkeys <= T, "nkeys outside [1, T]");
  KRUN(launch_self_attention(dtype, q, Kc, Vc, out, rows, heads, d, T, nkeys, nullptr, nullptr, 1, 0, (hipStream_t)stream));
}

int lsq_k_encoder_attention(int dtype, const void* qkv, const int32_t* row_seq, const int32_t* seq_off,
                            const int32_t* seq_len, void* out, int rows, int heads, int d, int causal, void* stream) {
  KCHK(qkv && row_seq && seq_off && seq_len && out, "null pointer");
  KCHK(dtype == DT_F32 || dtype == DT_F16, "dtype");
  KCHK(rows >= 0 && heads >= 1 && d % heads == 0 && head_dim_supported(d / heads), "head size must be 16/32/64/128");
  KRUN(launch_encoder_attention(dtype, qkv, row_seq, seq_off, seq_len, out, rows, heads, d, causal ? 1 : 0,
                                (hipStream_t)stream));
}

int lsq_k_cross_attention(int dtype, const void* q, const void* kv, const int32_t* src_off, const int32_t* src_len,
                          void* out, int batch, int beam, int heads, int d, int max_src_len, void* stream) {
  KCHK(q && kv && src_off && src_len && out, "null pointer");
  KCHK(dtype == DT_F32 || dtype == DT_F16, "dtype");
  KCHK(batch >= 0 && beam >= 1 && heads >= 1 && d % heads == 0 && head_dim_supported(d / heads), "shape");
  KCHK(max_src_len >= 1 && (size_t)std::min(beam, 4) * max_src_len * 4 <= 60 * 1024, "max_src_len");
  KRUN(launch_cross_attention(dtype, q, kv, src_off, src_len, out, batch, beam, heads, d, max_src_len, (hipStream_t)stream));
}

int lsq_k_row_topk(int dtype, const void* logits, const float* score, const int32_t* finished, int M, int V, int k,
                   int eos, float* out_score, int32_t* out_idx, void* stream) {
  KCHK(logits && score && finished && out_score && out_idx, "null pointer");
  KCHK(dtype == DT_F32 || dtype == DT_F16, "dtype");
  KCHK(M >= 0 && topk_supported(V) && k >= 1 && k <= LSQ_MAX_SAMPLE_TOPK && eos >= 0 && eos < V, "shape");
  KRUN(launch_row_topk(dtype, logits, score, finished, M, V, k, eos, 0, out_score, out_idx, (hipStream_t)stream));
}

int lsq_k_beam_refine_table(const float* cand_score, const int32_t* cand_idx, float* score, int32_t* tokens,
                            int32_t* len, int32_t* finished, int32_t* parent, const int32_t* cap, int32_t* active,
                            int32_t* slab, int batch, int k, int V, int T, int t, int eos, void* stream) {
  KCHK(cand_score && cand_idx && score && tokens && len && finished && parent && cap && active, "null pointer");
  KCHK(batch >= 0 && k >= 1 && k <= LSQ_MAX_BEAM && V >= k && T >= 1 && t >= 0 && t < T, "shape");
  KRUN(launch_beam_refine(cand_score, cand_idx, score, tokens, len, finished, parent, cap, active, batch, k, V, T, t,
                          nullptr, eos, slab, (hipStream_t)stream));
}

int lsq_k_gemm_logits(const void* A, const void* B, void* C, float* stats, int M, int N, int K, void* stream) {
  KCHK(A && B && C && stats, "null pointer");
  KCHK(M >= 0 && N >= 1 && K >= 1, "shape");
  KCHK(M == 0 || gemm_writes_stats(DT_F16, M, N, K), "no kernel with group statistics for this shape");
  GemmOut o = plain_out(C, N);
  o.f32_out = 1;
  o.stats = stats;
  o.stats_groups = (N + 31) / 32;
  KRUN(launch_gemm(DT_F16, A, B, nullptr, o, M, N, K, 0, (hipStream_t)stream));
}

int lsq_k_gemm_logits_supported(int M, int N, int K) { return gemm_writes_stats(DT_F16, M, N, K) ? 1 : 0; }

int lsq_k_row_topk_groups(const float* logits, const float* stats, const float* score, const int32_t* finished, int M,
                          int V, int k, int eos, int raw, float* out_score, int32_t* out_idx, void* stream) {
  KCHK(logits && stats && out_score && out_idx && (raw || (score && finished)), "null pointer");
  KCHK(M >= 0 && topk_groups_supported(V, k, raw ? 1 : 0), "V in [1, 65536], k in [1, beam limit] (raw: [1, 32])");
  KRUN(launch_row_topk_groups(logits, stats, score, finished, M, V, k, eos, raw ? 1 : 0, out_score, out_idx, (hipStream_t)stream));
}

int lsq_k_beam_refine(const float* cand_score, const int32_t* cand_idx, float* score, int32_t* tokens, int32_t* len,
                      int32_t* finished, int32_t* parent, const int32_t* cap, int32_t* active, int batch, int k,
                      int V, int T, int t, int eos, void* stream) {
  return lsq_k_beam_refine_table(cand_score, cand_idx, score, tokens, len, finished, parent, cap, active, nullptr,
                                 batch, k, V, T, t, eos, stream);
}

int lsq_k_self_attention_table(int dtype, const void* q, const void* Kc, const void* Vc, const int32_t* slab,
                               void* out, int rows, int beam, int heads, int d, int T, int nkeys, void* stream) {
  KCHK(q && Kc && Vc && slab && out, "null pointer");
  KCHK(dtype == DT_F32 || dtype == DT_F16, "dtype");
  KCHK(rows >= 0 && beam >= 1 && beam <= LSQ_MAX_BEAM && rows % beam == 0, "rows must be a multiple of beam");
  KCHK(heads >= 1 && d % heads == 0 && head_dim_supported(d / heads), "head size must be 16/32/64/128");
  KCHK(T >= 1 && nkeys >= 1 && nkeys <= T, "nkeys outside [1, T]");
  KRUN(launch_self_attention(dtype, q, Kc, Vc, out, rows, heads, d, T, nkeys, nullptr, slab, beam, T + 1,
                             (hipStream_t)stream));
}

int lsq_k_cache_reorder(int dtype, void* cache, const int32_t* parent, int layers, int batch, int k, int T, int d,
                        int npos, void* stream) {
  KCHK(cache && parent, "null pointer");
  KCHK(dtype == DT_F32 || dtype == DT_F16, "dtype");
  KCHK(layers >= 0 && batch >= 0 && k >= 1 && k <= LSQ_MAX_BEAM && npos >= 0 && npos <= T && d % 8 == 0, "shape");
  KRUN(launch_cache_reorder(dtype, cache, parent, layers, batch, batch * k, k, T, d, npos, nullptr, npos, (hipStream_t)stream));
}

}  // extern "C"
