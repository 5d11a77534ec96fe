/*
 * lsq -- beam-search Transformer decoding on one AMD MI355X (gfx950).
 *
 * C ABI of liblsq.so.  Plain pointers and sizes only.  "host" / "device" in a
 * comment says where the pointed-to memory must live.  Every function returns
 * LSQ_OK (0) or a non-negative count on success and a negative lsq_status on
 * failure; nothing aborts or throws.  Argument, state and blob errors are
 * detected before any device work is issued.  lsq_last_error() describes the
 * most recent failure.
 *
 * There is one process-global context (the four principal calls carry no
 * handle).  The library allocates no device memory at all: the caller hands
 * over ONE device workspace (lsq_set_workspace) which lsq_init carves into
 * weights, K/V caches and every intermediate, each at its maximum shape, with
 * intermediates that are never live together sharing bytes -- the paper's
 * dynamic-memory-reuse scheme (sec. 2.3).  Calls are not thread safe and all
 * device work is issued on the one stream given to lsq_set_workspace.
 *
 * Call order:
 *   lsq_workspace_bytes -> lsq_set_workspace -> lsq_init ->
 *   ( lsq_encode -> lsq_decode_step* -> lsq_get_beams )* -> lsq_free
 *
 * Two model kinds are accepted (blob header): the encoder-decoder Transformer
 * decoded with beam search, and a decoder-only model (pre-LN, tanh-GELU,
 * learned positions; the paper's GPT column and sampling decoding, Table 1 and
 * sec. 3.4) decoded with top-k sampling at beam 1.  For the latter lsq_encode
 * takes the prompts (all of one length P), fills the cache from their first
 * P-1 tokens, and each lsq_decode_step samples one token per row from a Philox
 * stream keyed by the blob's seed (counter = step, row) until cap_extra tokens
 * have been produced; lsq_get_beams returns those tokens and the sum of their
 * log-probabilities.  The draw is from the k <= LSQ_MAX_SAMPLE_TOPK largest
 * logits under their k-way softmax, cut -- when the blob sets a nucleus mass
 * p < 1 -- to the shortest ranked prefix whose probability reaches p (top-k
 * and top-p sampling, sec. 3.4).
 * An encoder-decoder blob whose header sets sample_topk >= 1 is decoded with the
 * same sampling instead of beam search (sec. 3.4: the paper's text-generation
 * runs sample from a Transformer): beam must be 1, every sentence carries one
 * hypothesis, an unfinished sentence draws one token per step (counter = step,
 * index of the sentence in the caller's batch), its score adds the log of the
 * token's probability among the kept candidates, and EOS or the length cap
 * finishes it as under beam search.
 */
#ifndef LSQ_H
#define LSQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LSQ_OK = 0,
  LSQ_E_ARG = -1,   /* null pointer, size out of range, id outside the vocabulary ... */
  LSQ_E_STATE = -2, /* call out of order                                            */
  LSQ_E_BLOB = -3,  /* weight blob: magic / version / size / unsupported variant     */
  LSQ_E_NOMEM = -4, /* workspace smaller than lsq_workspace_bytes reports            */
  LSQ_E_HIP = -5    /* a HIP runtime call failed; text in lsq_last_error()           */
} lsq_status;

#define LSQ_MAX_BEAM 8
#define LSQ_MAX_SAMPLE_TOPK 32 /* widest per-row retrieve: candidates a sampling model draws from */

/* Bytes of device workspace that lsq_init will need for this model blob and
 * these maxima (sec. 2.3: every dynamic shape is bounded when the service
 * starts).  weights: host, the serialized model (format: 256-byte header, then
 * tensors, see the blob writer); only its header is read here.
 * max_batch >= 1 sentences, 1 <= beam <= LSQ_MAX_BEAM, max_len >= 1 bounds both
 * the source length and the target length (= K/V cache positions). */
int lsq_workspace_bytes(const void* weights, size_t weights_bytes, int max_batch, int beam,
                        int max_len, size_t* out_bytes);

/* Hands over the workspace (device, 256-byte aligned, `bytes` long) and the HIP
 * stream (a hipStream_t passed as void*, NULL = the default stream).  The
 * caller keeps ownership and must keep both alive until lsq_free. */
int lsq_set_workspace(void* dev_ptr, size_t bytes, void* hip_stream);

/* Parses the blob (host), lays out the workspace, uploads the weights (stored
 * in their compute type already -- the paper folds the cast into weight loading,
 * sec. 3.2) and builds the position table.  The blob may be freed afterwards.
 * Synchronizes the stream before returning. */
int lsq_init(const void* weights, size_t weights_bytes, int max_batch, int beam, int max_len);

/* Runs the encoder over a batch of variable-length sentences and resets the
 * beams (the paper's problem statement: batched sequence-to-sequence generation
 * with variable-length inputs, sec. 1 and Fig. 1).
 * src_ids: host, int32 [batch, src_stride], sentence i uses its first
 * src_lens[i] entries; src_lens: host, int32 [batch].
 * 1 <= batch <= max_batch, 1 <= src_lens[i] <= src_stride <= max_len,
 * 0 <= id < vocab.  Device work is enqueued; the call does not wait for it. */
int lsq_encode(const int32_t* src_ids, const int32_t* src_lens, int batch, int src_stride);

/* One auto-regressive step for every hypothesis of every sentence: decoder
 * layers over the cached keys/values, vocabulary logits, log-softmax plus
 * hypothesis score, the k best (beam, token) pairs per sentence, and the
 * K/V cache made to follow the parent beams (sec. 2.2 and the "cache
 * refreshing" of sec. 3.2; see lsq_set_cache_refresh).
 * Returns the number of sentences that still have an unfinished hypothesis
 * (0 = done); waits for the step to finish to read that count back.
 * A step after every sentence finished, or after max_len steps, changes
 * nothing and returns 0. */
int lsq_decode_step(void);

/* Enqueues up to n steps without waiting between them, then waits once and
 * returns the active count after the last one.  Steps issued after everything
 * finished leave the state unchanged. */
int lsq_decode_steps(int n);

/* Copies the hypotheses out, best first per sentence by length-normalised
 * score = score / len^alpha.  All outputs are host memory:
 * out_ids int32 [batch, beam, max_len] (tokens after BOS, through EOS if one
 * was produced; pad_id beyond), out_lens int32 [batch, beam],
 * out_scores float [batch, beam].  Legal after any number of steps. */
int lsq_get_beams(int32_t* out_ids, int32_t* out_lens, float* out_scores);

/* Forgets the workspace and the model.  Frees only host-side bookkeeping. */
void lsq_free(void);

const char* lsq_last_error(void);

/* Decode steps are replayed from hipGraphs captured on first use, one per number
 * of sentences still alive, when the stream given to lsq_set_workspace is not
 * the default stream (stream capture needs a capturable stream).  on = 0 issues
 * the same kernels one by one instead; results are identical.  Default: on. */
int lsq_set_graphs(int on);

/* Cache refreshing (sec. 3.2): after every beam-search step hypothesis r continues
 * the history of hypothesis parent[r], so its cached keys/values must follow.
 * LSQ_REFRESH_MOVE copies cache rows (what the paper does; lsq_k_cache_reorder).
 * LSQ_REFRESH_TABLE (default) never moves a key or value: a table slab[r, j] names,
 * for every position j of r's history, which of its sentence's beam rows wrote it;
 * the re-rank kernel gathers that small table by parent and self-attention reads
 * through it.  Takes effect at the next lsq_encode; results are bit-identical.
 * Models decoded at beam 1 have nothing to refresh. */
enum { LSQ_REFRESH_MOVE = 0, LSQ_REFRESH_TABLE = 1 };
int lsq_set_cache_refresh(int mode);

/* With at most 8 rows alive (the end of a batch, single sentences) a float16
 * encoder-decoder model folds every sublayer's "partial sums + bias + residual,
 * LayerNorm" into the product that consumes the normalised rows (sec. 2.1 taken
 * one step further: 18 fewer launches per step), and with at most 64 rows (beams
 * of at most 4, heads of 64) the cross-attention kernel normalises its rows and
 * makes its queries itself (12 fewer); with more rows it still makes its queries,
 * from rows the LayerNorm kernel has normalised (6 fewer).  on = 0 keeps the stand-alone LayerNorm
 * kernel at every size.  The row arithmetic is the same either way; the
 * cross-attention kernel that makes its own queries takes its sums in another
 * order (fewer split-K slabs, keys shared by four wavefronts), so results agree
 * to the last bits, not always bit for bit.  Default: on. */
int lsq_set_layernorm_fusion(int on);

/* Few rows alive (float16 models with heads of 64 and d = 256 or 512, beam <= 4: with wider models
 * the separate kernels are faster): each attention sublayer of a decoder layer runs as one launch up to its output
 * projection (sec. 2.1 taken further; lsq_k_self_attention_block, lsq_k_cross_attention_block)
 * while at most max_rows rows are alive.  0 switches this off; default and largest value 64.  Same
 * tokens as the separate kernels; scores equal to float16 rounding (other summation orders).  Also
 * off when lsq_set_layernorm_fusion(0).  May be called at any time. */
int lsq_set_attention_blocks(int max_rows);

/* Plain beam search of float16 models: the logit product also leaves, for every row and every 32
 * consecutive tokens, the largest logit and the sum of exponentials, and the retrieve stage (sec.
 * 2.2) takes its threshold and the softmax normaliser from those and reads only the logits of the
 * groups that reach the threshold (lsq_k_gemm_logits, lsq_k_row_topk_groups).
 * mode 1 (default): so, with retrieve and re-rank in one launch; 2: so, as two launches; 0: the
 * retrieve kernel reads every row in full.  Same tokens in all modes; scores of mode 0 differ
 * from the others by the rounding of the normaliser, modes 1 and 2 are bit-identical.  May be
 * called at any time. */
int lsq_set_topk_statistics(int mode);

/* Diverse beam search (named among the search methods of sec. 3.4; Vijayakumar et
 * al. 2016, Hamming diversity).  The beam is split into `groups` groups of
 * beam / groups hypotheses; at every step the groups of a sentence choose in
 * order, and a candidate token is ranked by score + log p - strength * (number
 * of hypotheses of the earlier groups that took that token at this step).
 * Hypothesis scores stay plain log-probability sums; finished hypotheses are
 * neither penalised nor counted.  groups = 1 (default) is ordinary beam search.
 * groups must divide the beam of lsq_init; takes effect at the next lsq_encode
 * (which fails with LSQ_E_ARG otherwise).  Encoder-decoder models only. */
int lsq_set_diversity(int groups, float strength);

/* Debug aid for the shared memory plan (sec. 2.3): with canaries on, lsq_workspace_bytes / lsq_init put a
 * 256-byte red zone, filled with a pattern, behind every region of the workspace (weights, caches, beam state,
 * each of the decoder's intermediates, the end of the workspace).  Set before lsq_workspace_bytes; LSQ_E_STATE
 * once a model is loaded.  lsq_debug_check_canaries waits for the stream and returns how many zones no longer
 * hold the pattern (0 = no kernel wrote outside its region); the zones behind the decoder's intermediates are
 * checked from the end of lsq_encode on (the encoder's intermediates share those bytes before).  Default: off. */
int lsq_set_canaries(int on);
int lsq_debug_check_canaries(void);

/* Number of decode steps taken since the last lsq_encode. */
int lsq_step_index(void);

/* ------------------------------------------------------------------------- */
/* Per-kernel timing for benchmarks.  While enabled, each kernel that
 * lsq_decode_step(s) launches is bracketed by two HIP events on the library's
 * stream.  lsq_profile_read waits for the stream, then fills ms[c] (summed
 * elapsed milliseconds) and launches[c] for each of lsq_profile_classes()
 * kernel classes (names from lsq_profile_class_name) and clears the record.
 * Enabling costs two event records per launch; leave it off when timing
 * whole steps.  ms, launches: host arrays of at least lsq_profile_classes(). */
int lsq_profile_enable(int on);
int lsq_profile_classes(void);
const char* lsq_profile_class_name(int c);
int lsq_profile_read(double* ms, int64_t* launches, int n);

/* ------------------------------------------------------------------------- */
/* Debug / test hooks: copy library state to host memory.  Floating-point data
 * is always delivered as float32 whatever the model's storage type. `bytes`
 * must equal the size of the item.  M = batch*beam rows, T = max_len.          */
enum {
  LSQ_DBG_LOGITS = 0,     /* float [M, vocab]  logits of the last step (always fp32); rows of sentences past their cap are stale */
  LSQ_DBG_SCORE = 1,      /* float [M]         raw hypothesis scores                   */
  LSQ_DBG_TOKENS = 2,     /* int32 [M, T+1]    token histories, BOS first              */
  LSQ_DBG_LEN = 3,        /* int32 [M]                                                 */
  LSQ_DBG_FINISHED = 4,   /* int32 [M]                                                 */
  LSQ_DBG_PARENT = 5,     /* int32 [M]         parent beam (0..beam-1) chosen in the last step the sentence took part in */
  LSQ_DBG_CAND_SCORE = 6, /* float [M, beam]   per-row top-k scores of the last step ([M, sample_topk] logits for a sampling model) */
  LSQ_DBG_CAND_IDX = 7,   /* int32 [M, beam]   per-row top-k tokens (-1 = none)        */
  LSQ_DBG_HIDDEN = 8,     /* float [M, d]      decoder output of the last step         */
  LSQ_DBG_MEMORY = 9,     /* float [sum(src_lens), d] encoder output, sentences packed */
  LSQ_DBG_CROSS_KV = 100, /* +layer: float [sum(src_lens), 2d]                          */
  LSQ_DBG_CACHE_K = 200,  /* +layer: float [M, T, d]                                    */
  LSQ_DBG_CACHE_V = 300   /* +layer: float [M, T, d]                                    */
};
int lsq_debug_read(int what, void* host_dst, size_t bytes);

/* ------------------------------------------------------------------------- */
/* Single-kernel entry points on caller-provided DEVICE buffers, for kernel-level
 * parity tests and bandwidth / MFMA measurements.  dtype: 0 = float32,
 * 1 = float16 storage (fp32 accumulation in both).  stream: hipStream_t as
 * void*.  They need no context and enqueue without waiting.                    */

/* C[M,N] = act(A[M,K] . B[N,K]^T + bias[N]); bias may be NULL.  The dense
 * contractions of sec. 2.1.  flags: LSQ_GEMM_RELU applies max(.,0);
 * LSQ_GEMM_F32_OUT (float16 inputs only) makes C float32, the accumulators
 * unrounded, as the vocabulary-logit GEMM does.  K % 8 == 0 for float16. */
#define LSQ_GEMM_RELU 1
#define LSQ_GEMM_F32_OUT 2
#define LSQ_GEMM_GELU 4    /* tanh-GELU instead of ReLU */
#define LSQ_GEMM_PACKED_B 16 /* lsq_k_gemm: B is in fragment order (lsq_k_pack_weights); float16, M <= 64, K % 16 == 0 */
int lsq_k_gemm(int dtype, const void* A, const void* B, const void* bias, void* C, int M, int N,
               int K, int flags, void* stream);

/* Weights in fragment order, which the products of at most 64 rows read fastest (one
 * contiguous KB per matrix-core fragment instead of 16 bytes from each of 32 rows):
 * packed [ceil(N/32)][K/16][64 lanes][8 halves], lane l of block b and k-step s holding
 * W[32 b + (l & 31), 16 s + 8 (l >> 5) ... + 7], rows past N zero.  lsq_init packs the
 * model's matrices itself; these two calls exist for lsq_k_gemm with LSQ_GEMM_PACKED_B.
 * W [N,K] float16, device, 16-byte aligned; packed: device, lsq_k_packed_weight_bytes(N, K)
 * bytes (0 if K is not a multiple of 16: unsupported). */
size_t lsq_k_packed_weight_bytes(int N, int K);
int lsq_k_pack_weights(const void* W, void* packed, int N, int K, void* stream);

/* One residual sublayer tail: x[M,d] <- LayerNorm(x + in[M,K] . W[d,K]^T + bias) * gamma + beta,
 * in place on x, biased variance.  The projection's fp32 accumulators are not
 * rounded before the sum.  Two launches: a GEMM that leaves fp32 partial sums in
 * `scratch` (split over K when the output has too few tiles to fill the chip) and
 * one LayerNorm launch with no further intermediate (sec. 2.1).  scratch: device,
 * 16-byte aligned, lsq_k_gemm_add_layernorm_scratch(dtype, M, d, K) bytes. */
size_t lsq_k_gemm_add_layernorm_scratch(int dtype, int M, int d, int K);
int lsq_k_gemm_add_layernorm(int dtype, const void* in, const void* W, const void* bias, void* x,
                             const void* gamma, const void* beta, int M, int d, int K, float eps,
                             void* scratch, void* stream);

/* lsq_k_gemm_add_layernorm for callers that cannot allocate device memory or bring a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * two launches, with the fp32 partial sums in a buffer built into the library (one copy per GPU,
 * held until the process ends) of lsq_k_gemm_add_layernorm_static_limit() = 16 MiB.  Allocates
 * nothing and frees nothing; results are those of lsq_k_gemm_add_layernorm bit for bit.  A shape
 * whose lsq_k_gemm_add_layernorm_scratch() exceeds the limit is refused with LSQ_E_ARG before any
 * device work (M * d * 4 bytes per slab, up to 8 slabs: e.g. 512 rows of 1024 always fit).  Every
 * call on a GPU uses that GPU's one buffer: calls that overlap on one GPU (two streams, two
 * threads) race; calls on one stream are ordered and need nothing cleared in between (every slab
 * element that is read was written by the same call).  The device current at the call is the
 * one whose buffer is used and must be the device of the operands and the stream. */
size_t lsq_k_gemm_add_layernorm_static_limit(void);
int lsq_k_gemm_add_layernorm_static(int dtype, const void* in, const void* W, const void* bias, void* x,
                                    const void* gamma, const void* beta, int M, int d, int K, float eps,
                                    void* stream);

/* C = act(LN(x_old + sum_s P[s] + ln_bias) . W^T + bias) for 1..8 rows, float16:
 * the LayerNorm of lsq_k_gemm_add_layernorm done by the product that consumes it.
 * P float [splits <= 4, M, K]; x_old, x_new [M,K] (different buffers; x_new
 * receives the normalised rows); W [N,K]; K a multiple of 16, at most 1024. */
int lsq_k_layernorm_gemm(int dtype, const float* P, int splits, const void* ln_bias, const void* gamma,
                         const void* beta, const void* x_old, void* x_new, float eps, const void* W,
                         const void* bias, void* C, int M, int N, int K, int flags, void* stream);

/* Cross-attention that normalises its rows and makes its queries itself (few
 * rows alive, where fewer launches matter most;
 * paper sec. 2.1 taken one step further): for every sentence b and head h,
 *   rows  = LN(x_old + sum_s P[s] + ln_bias)            (as lsq_k_layernorm_gemm; written to x_new)
 *   q     = rows . Wq[h*64:(h+1)*64, :]^T + bq[h*64:..]   (rounded to float16)
 *   out   = lsq_k_cross_attention(q, kv, ...)
 * float16 only; batch*beam <= 64 rows, beam <= 4, heads of 64, d = 64*heads <=
 * 1024.  Wq_packed: the fragment-ordered copy of Wq [d, d] made by
 * lsq_k_pack_weights; P float [splits <= 4, batch*beam, d]; x_old and x_new
 * different buffers; everything else as in lsq_k_cross_attention. */
int lsq_k_layernorm_cross_attention(const float* P, int splits, const void* ln_bias, const void* gamma,
                                    const void* beta, const void* x_old, void* x_new, float eps,
                                    const void* Wq_packed, const void* bq, const void* kv,
                                    const int32_t* src_off, const int32_t* src_len, void* out, int batch,
                                    int beam, int heads, int d, void* stream);

/* The self-attention sublayer of a decoder layer up to its output projection in one launch, for
 * at most 64 rows (sec. 2.1 taken further: the products join the fused kernels where a step is a
 * chain of launch latencies).  For every sentence b, head h and row r of b:
 *   rows      = LN(x_old + sum_s P[s] + ln_bias) * gamma + beta   (splits 1..4; written to x_new)
 *               or x_old as it is                                  (splits 0; x_new and P unused)
 *     pre_ln = 1 (pre-LN models): u = x_old + sum_s P[s] + ln_bias rounded to float16 is what x_new
 *               receives, rows = LN(u) * gamma + beta; splits 0: rows = LN(x_old) * gamma + beta
 *   [q|k|v]   = rows . Wqkv[{0,d,2d} + h*64 .. +63, :]^T + bqkv[..]   (rounded to float16)
 *   Kc, Vc[r, nkeys, h*64..] = k, v
 *   ctx       = softmax(q . K^T / 8) V over positions 0..nkeys of r's history, rounded to float16
 *               (position j < nkeys: slab (r - r % beam) + slab_table[r*(T+1) + j], or slab r when
 *               slab_table is NULL; position nkeys: the new k, v)
 *   P_out[h][r][:] = ctx . Wo[:, h*64 .. h*64+63]^T   (float; the sum over h is ctx_all . Wo^T)
 * float16 only; beam 1..4, heads of 64, d = 64*heads a multiple of 256, at most 1024.
 * Wqkv_packed, Wo_packed: lsq_k_pack_weights of Wqkv [3d, d] and Wo [d, d]; Kc, Vc [rows, T, d];
 * P float [splits, rows, d]; P_out float [heads, rows, d]; 0 <= nkeys < T.  All device, 16-byte
 * aligned.  Positions beyond nkeys may be read and are discarded. */
int lsq_k_self_attention_block(const float* P, int splits, const void* ln_bias, const void* gamma,
                               const void* beta, const void* x_old, void* x_new, float eps,
                               const void* Wqkv_packed, const void* bqkv, const void* Wo_packed, void* Kc,
                               void* Vc, const int32_t* slab_table, int nkeys, float* P_out, int batch,
                               int beam, int heads, int d, int T, int pre_ln, void* stream);

/* The cross-attention sublayer up to its output projection in one launch, for at most 64 rows:
 * lsq_k_layernorm_cross_attention with 1..16 slabs behind the LayerNorm (the block above leaves
 * one per head) whose context rows are multiplied by the head's 64 columns of Wo:
 *   P_out[h][r][:] = ctx[r, h*64..+63] . Wo[:, h*64 .. h*64+63]^T   (float [heads, rows, d]).
 * Same limits as lsq_k_self_attention_block. */
int lsq_k_cross_attention_block(const float* P, int splits, const void* ln_bias, const void* gamma,
                                const void* beta, const void* x_old, void* x_new, float eps,
                                const void* Wq_packed, const void* bq, const void* Wo_packed,
                                const void* kv, const int32_t* src_off, const int32_t* src_len,
                                float* P_out, int batch, int beam, int heads, int d, void* stream);

/* Cross-attention that makes its own queries from normalised rows, for more than 64 rows
 * (sec. 2.1: one launch instead of a product and an attention kernel):
 *   q   = x . Wq[h*64:(h+1)*64, :]^T + bq[h*64:..]   (rounded to float16)
 *   out = lsq_k_cross_attention(q, kv, ...)
 * float16 only; 64 < batch*beam rows, beam <= 4, heads of 64, d = 64*heads <= 1024.
 * x [batch*beam, d]; Wq_packed: lsq_k_pack_weights(Wq [d, d]); the rest as in
 * lsq_k_cross_attention. */
int lsq_k_cross_attention_q(const void* x, const void* Wq_packed, const void* bq, const void* kv,
                            const int32_t* src_off, const int32_t* src_len, void* out, int batch, int beam,
                            int heads, int d, void* stream);

/* Decoder self-attention of one new position per row over its cached keys:
 * out[r, h*dh:(h+1)*dh] = softmax(q_h . K_h^T / sqrt(dh)) V_h over positions
 * 0..nkeys-1 of Kc/Vc [rows, T, d].  Positions nkeys..T-1 of a row may be read
 * too (requested before the length is known, then discarded whatever they
 * hold), never anything outside [rows, T, d].  T*d*4 must fit 32 bits. */
int lsq_k_self_attention(int dtype, const void* q, const void* Kc, const void* Vc, void* out,
                         int rows, int heads, int d, int T, int nkeys, void* stream);

/* Cross-attention: the `beam` rows of sentence b attend over that sentence's
 * src_len[b] encoder positions, kv packed as [sum(src_len), 2d] = [K | V] with
 * sentence b starting at row src_off[b] (both int32, device).  max_src_len: a
 * the longest of src_len[] as the host knows it (or an upper bound), at least
 * 1; it only picks the launch geometry: one wavefront per (sentence, head), or
 * four when few sentences are left and the longest one has many keys.  One
 * sentence's keys and values must span less than 4 GiB. */
int lsq_k_cross_attention(int dtype, const void* q, const void* kv, const int32_t* src_off,
                          const int32_t* src_len, void* out, int batch, int beam, int heads, int d,
                          int max_src_len, void* stream);

/* Self-attention inside packed sequences (encoder layers; with causal != 0 the
 * prompt prefill of a decoder-only model): qkv [rows, 3d] = [Q | K | V], row i
 * belongs to sequence row_seq[i], whose rows are seq_off[b] .. seq_off[b] +
 * seq_len[b] - 1 (all int32, device).  Row i attends every row of its sequence,
 * or with causal only those up to itself.  out [rows, d].  rows*3*d*4 must
 * fit 32 bits. */
int lsq_k_encoder_attention(int dtype, const void* qkv, const int32_t* row_seq, const int32_t* seq_off,
                            const int32_t* seq_len, void* out, int rows, int heads, int d, int causal,
                            void* stream);

/* Retrieve stage of the hierarchical search (sec. 2.2) made exact: per row r of
 * logits [M,V], cand = score[r] + log_softmax(logits[r,:]) and the k best
 * (cand descending, token ascending) are written to out_score/out_idx [M,k],
 * 1 <= k <= LSQ_MAX_SAMPLE_TOPK.
 * A finished row yields the single candidate (score[r], eos) and k-1 empty
 * slots (idx -1).  score float32, finished int32. */
int lsq_k_row_topk(int dtype, const void* logits, const float* score, const int32_t* finished,
                   int M, int V, int k, int eos, float* out_score, int32_t* out_idx, void* stream);

/* Vocabulary logits with the retrieve stage's group statistics (paper sec. 2.2, made where the
 * logits are made): C [M,N] float = A [M,K] . B [N,K]^T (float16 operands, float32 accumulators,
 * nothing rounded) and, for every row m and every group g of 32 consecutive columns,
 *   stats[(m * G + g) * 2 + 0] = largest C[m, n] of the group,
 *   stats[(m * G + g) * 2 + 1] = sum over the group of exp(C[m, n] - largest),   G = ceil(N / 32).
 * lsq_k_gemm_logits_supported(M, N, K) != 0 says that the shape is taken (every float16 product
 * kernel writes them: K a multiple of 8), else LSQ_E_ARG.  All device pointers, 16-byte aligned; stats M * G * 2 floats. */
int lsq_k_gemm_logits(const void* A, const void* B, void* C, float* stats, int M, int N, int K, void* stream);
int lsq_k_gemm_logits_supported(int M, int N, int K);

/* lsq_k_row_topk on float32 logits computed from the statistics above: the normaliser from the G
 * pairs, the threshold R = k-th largest group maximum (as a candidate score), and only the
 * logits of groups that reach R are read.  raw == 0: beam search, k at most the beam limit, same
 * outputs as lsq_k_row_topk up to the rounding of the normaliser.  raw != 0 (sampling): the k <=
 * 32 largest logits themselves, score and finished unused (may be NULL). */
int lsq_k_row_topk_groups(const float* logits, const float* stats, const float* score, const int32_t* finished,
                          int M, int V, int k, int eos, int raw, float* out_score, int32_t* out_idx,
                          void* stream);

/* Re-rank stage: per sentence the k best of its k*k row candidates by
 * (score descending, beam*V+token ascending); updates score, tokens [M,T+1],
 * len, finished in place, writes parent [M] and adds the number of still-active
 * sentences to *active (int32, device; caller zeroes it).  cap int32 [batch]. */
int lsq_k_beam_refine(const float* cand_score, const int32_t* cand_idx, float* score,
                      int32_t* tokens, int32_t* len, int32_t* finished, int32_t* parent,
                      const int32_t* cap, int32_t* active, int batch, int k, int V, int T, int t,
                      int eos, void* stream);

/* The same with the slab table of LSQ_REFRESH_TABLE: slab int32 [M, T+1] (device),
 * slab[r, j] in 0..k-1 for j <= t on entry.  On return slab[r, 0..t] =
 * old slab[b*k + parent[r], 0..t] and slab[r, t+1] = r mod k (row r itself will
 * write position t+1). */
int lsq_k_beam_refine_table(const float* cand_score, const int32_t* cand_idx, float* score,
                            int32_t* tokens, int32_t* len, int32_t* finished, int32_t* parent,
                            const int32_t* cap, int32_t* active, int32_t* slab, int batch, int k, int V,
                            int T, int t, int eos, void* stream);

/* Self-attention through the slab table: as lsq_k_self_attention, but position j
 * of row r is read from cache row (r - r mod beam) + slab[r*(T+1) + j].
 * rows must be a multiple of beam; beam*T*d*4 must fit 32 bits.  Table entries
 * at j >= nkeys may hold anything (a value read from there is forced into
 * 0..beam-1 before it forms an address, and what it fetches is discarded). */
int lsq_k_self_attention_table(int dtype, const void* q, const void* Kc, const void* Vc,
                               const int32_t* slab, void* out, int rows, int beam, int heads, int d,
                               int T, int nkeys, void* stream);

/* Cache refreshing (sec. 3.2): cache[l, b*k+i, 0:npos, :] <- cache[l, b*k+parent[b*k+i], 0:npos, :]
 * for all layers, in place.  cache [layers, M, T, d]. */
int lsq_k_cache_reorder(int dtype, void* cache, const int32_t* parent, int layers, int batch, int k,
                        int T, int d, int npos, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LSQ_H */
