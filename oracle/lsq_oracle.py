"""CPU oracle for beam-search Transformer decoding.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this file.  It shares no code with the HIP library and never calls it.

What it computes.  Given the logits, the paper's hierarchical search (sec. 2.2:
retrieve, then re-rank) reaches exactly the result of the plain procedure it
replaces (sec. 2.2, the two enumerated whole-vocabulary calculations): softmax
over the vocabulary, add the hypothesis score, keep the k best (beam, token)
pairs.  Operator fusion (sec. 2.1) and memory reuse (sec. 2.3) change no value.
So this oracle is the plain definition written out: a Transformer
encoder-decoder forward pass (the paper defers the model to Vaswani et al.,
sec. 3.1) and textbook beam search with a full sort.  Plain numpy, one
operation per line, no blocking or fusion; ``@`` (matmul), ``einsum`` and
``lexsort`` are the library primitives used as steps.

Precision.  The arithmetic type is ``ctype``: the pins and the parity runs of fp32
models use fp64; parity runs of fp16 models use fp32 between the storage points
(the type of the accumulators the rounding to fp16 is applied to).  With
``storage='blob'`` and an fp16 blob, every tensor the model *stores* between
operations (embedding sum, the Q/K/V and FFN-hidden projections after their
bias/activation, attention context, LayerNorm output, K/V cache entries) is
rounded to fp16 and widened again, which is what "fp16 weights and activations,
fp32 accumulate" means; a sublayer's output projection is not stored: its fp32
accumulators go straight into the residual sum that LayerNorm consumes; the
vocabulary logits, softmax statistics, probabilities, log-probabilities and
hypothesis scores are never rounded below fp32 (a logit rounded to fp16 moves by
up to 2e-3 near |x| = 2..4, more than the 1e-3 score margin at which token ids
must already agree).  ``storage='wide'`` rounds nothing.

Readings of points the paper leaves open (it gives no model equations):
  * one embedding table shared by source, target and the output projection;
    inputs scaled by sqrt(d); no output bias;
  * sinusoidal positions PE(p,2i)=sin(p/10000^(2i/d)), PE(p,2i+1)=cos(same),
    positions from 0, evaluated in double precision;
  * post-LN residual blocks, ReLU, LayerNorm with biased variance and eps from
    the blob; attention scale 1/sqrt(dh) applied to q.k; masked keys excluded;
  * beam search prunes on the raw cumulative log-probability; candidates are
    ordered by (score descending, flat index beam*V+token ascending); a finished
    hypothesis stays in the beam with a frozen score and offers one candidate
    (its score, token EOS); a hypothesis finishes on EOS or on reaching
    cap = min(src_len + cap_extra, max_len); the returned score is
    score / len^alpha (len counts EOS), beams sorted by (that descending, beam
    index ascending).

Pins (tests/test_oracle_*.py): softmax rows sum to one and are shift invariant;
LayerNorm gives mean 0 / variance 1 and agrees with torch; PE closed forms; one
encoder and one decoder layer agree with torch.nn.TransformerEncoderLayer /
TransformerDecoderLayer loaded with the same weights; cached decoding equals
full recomputation of the prefix; top-k equals a brute-force scan; beam 1 equals
greedy; a beam at least vocab^len wide equals exhaustive enumeration; the
paper's retrieve threshold keeps a superset of the top-k.  The readings listed
above are pinned only by those library routines and invariants, not by the
paper, which prints no worked value: parity unpinned against the paper for them.
"""
from __future__ import annotations

import struct

import numpy as np

_MAGIC = b"LSQBLOB1"


# ----------------------------------------------------------------------------
# blob reader (own statement of the format; the writer lives elsewhere)
# ----------------------------------------------------------------------------
class Model:
    """Hyper-parameters and tensors of one blob, tensors widened to ``ctype``."""

    def __init__(self, blob: bytes, ctype=np.float32, storage: str = "blob"):
        if len(blob) < 256 or blob[:8] != _MAGIC:
            raise ValueError("not a model blob")
        (ver, self.arch, self.n_enc, self.n_dec, self.d, self.H, self.F, self.V, self.max_pos,
         self.act, self.norm, self.dtype, self.pad, self.bos, self.eos, self.cap_extra,
         self.sample_topk) = struct.unpack_from("<17i", blob, 8)
        self.alpha, self.eps, topp = struct.unpack_from("<3f", blob, 76)
        self.sample_topp = float(topp) if 0.0 < topp < 1.0 else 1.0      # 0 in the header: no nucleus cut
        self.seed, total = struct.unpack_from("<2Q", blob, 88)
        if ver != 1 or total != len(blob) or (self.arch, self.norm, self.act) not in ((0, 0, 0), (1, 1, 1)):
            raise ValueError("unsupported blob")
        if self.d % self.H:
            raise ValueError("d_model not divisible by heads")
        self.dh = self.d // self.H
        self.ctype = ctype
        assert storage in ("blob", "wide")
        self.round16 = (storage == "blob" and self.dtype == 1)
        src_dt = np.float16 if self.dtype == 1 else np.float32
        esz = 2 if self.dtype == 1 else 4
        pos = 256
        d, F, V = self.d, self.F, self.V

        def take(*shape):
            nonlocal pos
            pos = (pos + 255) // 256 * 256
            n = int(np.prod(shape))
            a = np.frombuffer(blob, src_dt, n, pos).reshape(shape).astype(ctype)
            pos += n * esz
            return a

        self.E = take(V, d)
        self.enc, self.dec = [], []
        if self.arch == 1:      # decoder-only: learned positions, pre-LN blocks, final LayerNorm
            self.P = take(self.max_pos, d)
            for _ in range(self.n_dec):
                L = {}
                L["ln1_g"], L["ln1_b"] = take(d), take(d)
                L["Wqkv"], L["bqkv"], L["Wo"], L["bo"] = take(d, 3 * d), take(3 * d), take(d, d), take(d)
                L["ln2_g"], L["ln2_b"] = take(d), take(d)
                L["W1"], L["b1"], L["W2"], L["b2"] = take(d, F), take(F), take(F, d), take(d)
                self.dec.append(L)
            self.lnf_g, self.lnf_b = take(d), take(d)
            if pos != len(blob):
                raise ValueError("blob size does not match its header")
            return
        for _ in range(self.n_enc):
            L = {}
            L["Wqkv"], L["bqkv"], L["Wo"], L["bo"] = take(d, 3 * d), take(3 * d), take(d, d), take(d)
            L["ln1_g"], L["ln1_b"] = take(d), take(d)
            L["W1"], L["b1"], L["W2"], L["b2"] = take(d, F), take(F), take(F, d), take(d)
            L["ln2_g"], L["ln2_b"] = take(d), take(d)
            self.enc.append(L)
        for _ in range(self.n_dec):
            L = {}
            L["Wqkv"], L["bqkv"], L["Wo"], L["bo"] = take(d, 3 * d), take(3 * d), take(d, d), take(d)
            L["ln1_g"], L["ln1_b"] = take(d), take(d)
            L["Wq_c"], L["bq_c"] = take(d, d), take(d)
            L["Wkv_c"], L["bkv_c"] = take(d, 2 * d), take(2 * d)
            L["Wo_c"], L["bo_c"] = take(d, d), take(d)
            L["ln2_g"], L["ln2_b"] = take(d), take(d)
            L["W1"], L["b1"], L["W2"], L["b2"] = take(d, F), take(F), take(F, d), take(d)
            L["ln3_g"], L["ln3_b"] = take(d), take(d)
            self.dec.append(L)
        if pos != len(blob):
            raise ValueError("blob size does not match its header")

    def store(self, x):
        """Rounding applied where the model stores a tensor (see module docstring)."""
        x = np.asarray(x, self.ctype)
        if self.round16:
            return x.astype(np.float16).astype(self.ctype)
        return x


# ----------------------------------------------------------------------------
# elementary operations
# ----------------------------------------------------------------------------
def positional_encoding(p, d, ctype=np.float32):
    """Sinusoidal position vector(s) for position(s) p (Vaswani et al. form; the
    paper's configuration only says "sinusoidal")."""
    p = np.atleast_1d(np.asarray(p, np.float64))
    i = np.arange(0, d, 2, dtype=np.float64)
    ang = p[:, None] / np.power(10000.0, i / d)[None, :]
    pe = np.zeros((p.shape[0], d), np.float64)
    pe[:, 0::2] = np.sin(ang)
    pe[:, 1::2] = np.cos(ang)[:, : d // 2]
    return pe.astype(ctype)


def softmax(s):
    """Softmax over the last axis; entries equal to -inf get probability 0."""
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def log_softmax(x):
    """log of the vocabulary softmax (sec. 2.2, calculation 1), last axis."""
    m = np.max(x, axis=-1, keepdims=True)
    z = np.sum(np.exp(x - m), axis=-1, keepdims=True)
    return (x - m) - np.log(z)


def layer_norm(v, g, b, eps):
    """Layer normalisation (the reduce operation of sec. 2.1): biased variance."""
    mean = np.mean(v, axis=-1, keepdims=True)
    c = v - mean
    var = np.mean(c * c, axis=-1, keepdims=True)
    return g * (c / np.sqrt(var + v.dtype.type(eps))) + b


def attention(q, K, V, H, allowed=None):
    """Multi-head scaled dot-product attention of queries q[nq,d] over keys
    K[nk,d] / values V[nk,d]; ``allowed[nq,nk]`` (bool) masks keys out."""
    nq, d = q.shape
    nk = K.shape[0]
    dh = d // H
    qh = q.reshape(nq, H, dh)
    Kh = K.reshape(nk, H, dh)
    Vh = V.reshape(nk, H, dh)
    s = np.einsum("qhd,khd->hqk", qh, Kh) * q.dtype.type(1.0 / np.sqrt(dh))
    if allowed is not None:
        s = np.where(allowed[None, :, :], s, -np.inf).astype(q.dtype)
    p = softmax(s)
    return np.einsum("hqk,khd->qhd", p, Vh).reshape(nq, d)


def topk_by_full_sort(scores, flat, k):
    """Indices (into the candidate arrays) of the k best candidates under the
    total order (score descending, flat index ascending), by sorting them all
    (sec. 2.2, calculation 2)."""
    order = np.lexsort((flat, -scores))
    return order[:k]


def hars_retrieve(logits, k, groups):
    """The paper's retrieve stage (sec. 2.2, the four enumerated steps) for one
    beam: ``groups`` assigns each logit to one of k groups; the threshold R is
    the smallest of the k group maxima; logits not below R survive.  ("Larger
    than R" is read as >= R: R is itself a logit, and with k disjoint groups
    the k-th largest logit is >= R, so the survivors contain the top k.)"""
    m = np.array([logits[groups == g].max() for g in range(k)])
    R = m.min()
    return np.nonzero(logits >= R)[0], R


# ----------------------------------------------------------------------------
# encoder
# ----------------------------------------------------------------------------
def embed(model, ids, positions):
    x = model.E[ids] * model.ctype(np.sqrt(model.d)) + positional_encoding(positions, model.d, model.ctype)
    return model.store(x)


def encoder_layer(model, L, x):
    d = model.d
    qkv = model.store(x @ L["Wqkv"] + L["bqkv"])
    ctx = model.store(attention(qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:], model.H))
    a = ctx @ L["Wo"] + L["bo"]
    x = model.store(layer_norm(x + a, L["ln1_g"], L["ln1_b"], model.eps))
    h = model.store(np.maximum(x @ L["W1"] + L["b1"], 0))
    f = h @ L["W2"] + L["b2"]
    return model.store(layer_norm(x + f, L["ln2_g"], L["ln2_b"], model.eps))


def encode(model, src_ids, src_lens):
    """Encoder memory of every sentence (its real tokens only) and, per decoder
    layer, the cross-attention keys and values projected from it."""
    memory, cross = [], []
    for b, s in enumerate(src_lens):
        s = int(s)
        x = embed(model, np.asarray(src_ids[b][:s]), np.arange(s))
        for L in model.enc:
            x = encoder_layer(model, L, x)
        memory.append(x)
        kv = []
        for L in model.dec:
            t = model.store(x @ L["Wkv_c"] + L["bkv_c"])
            kv.append((t[:, :model.d], t[:, model.d:]))
        cross.append(kv)
    return memory, cross


# ----------------------------------------------------------------------------
# decoder, one position for every hypothesis row, K/V cached
# ----------------------------------------------------------------------------
class DecodeState:
    def __init__(self, model, src_lens, beam, max_len, groups=1):
        B = len(src_lens)
        assert groups >= 1 and beam % groups == 0
        self.B, self.k, self.T, self.groups = B, beam, max_len, groups
        M = B * beam
        self.t = 0
        self.tokens = np.full((M, max_len + 1), model.pad, np.int32)
        self.tokens[:, 0] = model.bos
        self.len = np.zeros(M, np.int32)
        self.finished = np.zeros(M, bool)
        self.score = np.full((B, beam), -np.inf, model.ctype)
        self.score[:, ::beam // groups] = 0          # one live hypothesis per group (one group: per sentence)
        self.cap = np.minimum(np.asarray(src_lens, np.int64) + model.cap_extra, max_len).astype(np.int32)
        self.Kc = [np.zeros((M, max_len, model.d), model.ctype) for _ in model.dec]
        self.Vc = [np.zeros((M, max_len, model.d), model.ctype) for _ in model.dec]


def decoder_logits_cached(model, st, cross):
    """Logits of step st.t for all rows; appends this position's self-attention
    key and value to the cache."""
    d, k, t = model.d, st.k, st.t
    M = st.B * k
    last = st.tokens[np.arange(M), st.len]
    y = embed(model, last, np.full(M, t))
    for l, L in enumerate(model.dec):
        qkv = model.store(y @ L["Wqkv"] + L["bqkv"])
        st.Kc[l][:, t] = qkv[:, d:2 * d]
        st.Vc[l][:, t] = qkv[:, 2 * d:]
        ctx = np.empty((M, d), model.ctype)
        for r in range(M):
            ctx[r] = attention(qkv[r:r + 1, :d], st.Kc[l][r, :t + 1], st.Vc[l][r, :t + 1], model.H)[0]
        a = model.store(ctx) @ L["Wo"] + L["bo"]
        y = model.store(layer_norm(y + a, L["ln1_g"], L["ln1_b"], model.eps))
        q = model.store(y @ L["Wq_c"] + L["bq_c"])
        ctx = np.empty((M, d), model.ctype)
        for b in range(st.B):
            Ke, Ve = cross[b][l]
            ctx[b * k:(b + 1) * k] = attention(q[b * k:(b + 1) * k], Ke, Ve, model.H)
        a = model.store(ctx) @ L["Wo_c"] + L["bo_c"]
        y = model.store(layer_norm(y + a, L["ln2_g"], L["ln2_b"], model.eps))
        h = model.store(np.maximum(y @ L["W1"] + L["b1"], 0))
        f = h @ L["W2"] + L["b2"]
        y = model.store(layer_norm(y + f, L["ln3_g"], L["ln3_b"], model.eps))
    return y @ model.E.T


def decoder_logits_full(model, prefix, Ke_Ve_per_layer):
    """Logits after the last token of ``prefix`` (starting with BOS) for ONE
    hypothesis, recomputing every position with a causal mask and no cache.
    Must agree with the cached path (the K/V-cache invariant)."""
    n = len(prefix)
    d = model.d
    y = embed(model, np.asarray(prefix), np.arange(n))
    causal = np.tril(np.ones((n, n), bool))
    for l, L in enumerate(model.dec):
        qkv = model.store(y @ L["Wqkv"] + L["bqkv"])
        ctx = model.store(attention(qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:], model.H, causal))
        a = ctx @ L["Wo"] + L["bo"]
        y = model.store(layer_norm(y + a, L["ln1_g"], L["ln1_b"], model.eps))
        q = model.store(y @ L["Wq_c"] + L["bq_c"])
        Ke, Ve = Ke_Ve_per_layer[l]
        ctx = model.store(attention(q, Ke, Ve, model.H))
        a = ctx @ L["Wo_c"] + L["bo_c"]
        y = model.store(layer_norm(y + a, L["ln2_g"], L["ln2_b"], model.eps))
        h = model.store(np.maximum(y @ L["W1"] + L["b1"], 0))
        f = h @ L["W2"] + L["b2"]
        y = model.store(layer_norm(y + f, L["ln3_g"], L["ln3_b"], model.eps))
    return y[-1] @ model.E.T


# ----------------------------------------------------------------------------
# beam search
# ----------------------------------------------------------------------------
def beam_select(model, st, logits):
    """One pruning step on given logits [M,V]: per sentence, softmax over the
    vocabulary, add the hypothesis score, keep the k best (beam, token) pairs
    (sec. 2.2).  Returns token, parent, score arrays [B,k] and, per sentence,
    the smallest gap between consecutive candidates among the k kept and the
    first one dropped (inf when nothing was dropped)."""
    B, k, V = st.B, st.k, model.V
    logp = log_softmax(np.asarray(logits, model.ctype))
    token = np.zeros((B, k), np.int32)
    parent = np.zeros((B, k), np.int32)
    score = np.zeros((B, k), model.ctype)
    margin = np.full(B, np.inf)
    for b in range(B):
        cs, cf = [], []
        for j in range(k):
            r = b * k + j
            if st.finished[r]:
                cs.append(np.array([st.score[b, j]], model.ctype))
                cf.append(np.array([j * V + model.eos], np.int64))
            else:
                cs.append(st.score[b, j] + logp[r])
                cf.append(j * V + np.arange(V, dtype=np.int64))
        cs = np.concatenate(cs)
        cf = np.concatenate(cf)
        order = np.lexsort((cf, -cs))
        best = order[:k]
        token[b] = cf[best] % V
        parent[b] = cf[best] // V
        score[b] = cs[best]
        top = cs[order[:k + 1]].astype(np.float64)
        fin = np.isfinite(top)
        gaps = [top[i] - top[i + 1] for i in range(len(top) - 1) if fin[i] and fin[i + 1]]
        if gaps:
            margin[b] = min(gaps)
    return token, parent, score, margin


def group_select(model, st, logp, b, g, strength, counts):
    """Diverse beam search (Vijayakumar et al. 2016, Hamming diversity; named in sec. 3.4's list of
    search methods): group g of sentence b picks its k' = k / groups best (beam, token) pairs among
    its own hypotheses, ranked by score + log p(token) - strength * counts[token], where
    counts[token] says how many hypotheses of the groups before g chose that token at this step.
    A finished hypothesis offers itself once, unpenalised.  Ties: flat index (beam within the
    sentence) * V + token, ascending.  Returns tokens, parents (beam index within the sentence),
    the hypotheses' new scores (log-probability sums, without the penalty), the ranking values and
    the smallest gap between consecutive ranking values among the kept and the first dropped."""
    k, V = st.k, model.V
    kg = k // st.groups
    cs, cp, cf = [], [], []
    for j in range(g * kg, (g + 1) * kg):
        r = b * k + j
        if st.finished[r]:
            plain = np.array([st.score[b, j]], model.ctype)
            cs.append(plain); cp.append(plain)
            cf.append(np.array([j * V + model.eos], np.int64))
        else:
            plain = (st.score[b, j] + logp[r]).astype(model.ctype)
            pen = (np.asarray(strength, model.ctype) * counts.astype(model.ctype)).astype(model.ctype)
            cs.append((plain - pen).astype(model.ctype)); cp.append(plain)
            cf.append(j * V + np.arange(V, dtype=np.int64))
    cs, cp, cf = np.concatenate(cs), np.concatenate(cp), np.concatenate(cf)
    order = np.lexsort((cf, -cs))
    best = order[:kg]
    top = cs[order[:kg + 1]].astype(np.float64)
    fin = np.isfinite(top)
    gaps = [top[i] - top[i + 1] for i in range(len(top) - 1) if fin[i] and fin[i + 1]]
    return (cf[best] % V).astype(np.int32), (cf[best] // V).astype(np.int32), cp[best], cs[best], \
        (min(gaps) if gaps else np.inf)


def beam_select_diverse(model, st, logits, strength):
    """One pruning step of diverse beam search for every sentence: the groups choose in order, each
    seeing the tokens the earlier groups of its sentence took at this step.  Same returns as
    beam_select (margin = the smallest over the groups)."""
    B, k, V, G = st.B, st.k, model.V, st.groups
    kg = k // G
    logp = log_softmax(np.asarray(logits, model.ctype))
    token = np.zeros((B, k), np.int32)
    parent = np.zeros((B, k), np.int32)
    score = np.zeros((B, k), model.ctype)
    margin = np.full(B, np.inf)
    for b in range(B):
        counts = np.zeros(V, np.int64)
        for g in range(G):
            tok, par, sc, _, m = group_select(model, st, logp, b, g, strength, counts)
            sl = slice(g * kg, (g + 1) * kg)
            token[b, sl], parent[b, sl], score[b, sl] = tok, par, sc
            margin[b] = min(margin[b], m)
            for i in range(kg):
                if not st.finished[b * k + par[i]] and np.isfinite(sc[i]):
                    counts[tok[i]] += 1
    return token, parent, score, margin


def beam_advance(model, st, token, parent, score):
    """Adopt the selected candidates: gather histories and caches from the
    parents ("cache refreshing", sec. 3.2), append tokens, update flags."""
    B, k = st.B, st.k
    rows = (np.arange(B)[:, None] * k + parent).reshape(-1)
    st.tokens = st.tokens[rows].copy()
    old_len = st.len[rows].copy()
    old_fin = st.finished[rows].copy()
    for l in range(len(st.Kc)):
        st.Kc[l] = st.Kc[l][rows].copy()
        st.Vc[l] = st.Vc[l][rows].copy()
    tok = token.reshape(-1)
    grow = ~old_fin
    new_len = old_len + grow.astype(np.int32)
    r = np.nonzero(grow)[0]
    st.tokens[r, new_len[r]] = tok[r]
    cap = np.repeat(st.cap, k)
    st.finished = old_fin | (grow & ((tok == model.eos) | (new_len >= cap)))
    st.len = new_len
    st.score = score.copy()
    st.t += 1
    active = (~st.finished).reshape(B, k).any(axis=1)
    return int(active.sum())


def finalize(model, st):
    """Length-normalised scores and best-first hypotheses per sentence."""
    B, k = st.B, st.k
    ln = st.len.reshape(B, k)
    with np.errstate(divide="ignore", invalid="ignore"):
        norm = np.where(ln > 0, np.power(np.maximum(ln, 1).astype(model.ctype), model.ctype(model.alpha)), 1)
        final = (st.score / norm).astype(model.ctype)
    ids = np.full((B, k, st.T), model.pad, np.int32)
    lens = np.zeros((B, k), np.int32)
    scores = np.zeros((B, k), model.ctype)
    for b in range(B):
        order = np.lexsort((np.arange(k), -final[b]))
        for i, j in enumerate(order):
            r = b * k + j
            n = int(st.len[r])
            ids[b, i, :n] = st.tokens[r, 1:n + 1]
            lens[b, i] = n
            scores[b, i] = final[b, j]
    return ids, lens, scores


def translate(model, src_ids, src_lens, beam, max_len, max_steps=None, trace=None, groups=1, strength=0.0):
    """Whole path: encode, then decode steps until every sentence is finished
    (or ``max_steps``).  ``trace``, if a list, receives one dict per step.
    groups > 1: diverse beam search with that many groups and that diversity strength."""
    memory, cross = encode(model, src_ids, src_lens)
    st = DecodeState(model, src_lens, beam, max_len, groups)
    steps = 0
    while True:
        logits = decoder_logits_cached(model, st, cross)
        if groups > 1:
            token, parent, score, margin = beam_select_diverse(model, st, logits, strength)
        else:
            token, parent, score, margin = beam_select(model, st, logits)
        active = beam_advance(model, st, token, parent, score)
        steps += 1
        if trace is not None:
            trace.append(dict(logits=logits, token=token, parent=parent, score=score, margin=margin,
                              active=active, finished=st.finished.copy(), len=st.len.copy()))
        if active == 0 or (max_steps is not None and steps >= max_steps):
            break
    return finalize(model, st), st


# ----------------------------------------------------------------------------
# decoder-only model with top-k sampling (the paper's GPT column of Table 1 and
# the sampling decoding of sec. 3.4; the paper gives no definitions, so: pre-LN
# blocks x += Attn(LN1 x), x += MLP(LN2 x), final LN, tanh-GELU, learned
# positions, tied output embedding; sampling: the k largest logits in the order
# (logit descending, token ascending), p = softmax over those k,
# u = (philox4x32_10(key = seed, counter = (step, row, 0, 0))[0] >> 8) * 2^-24,
# token = the first j whose cumulative p exceeds u * sum(p))
# ----------------------------------------------------------------------------
def gelu_tanh(x):
    c = x.dtype.type(np.sqrt(2.0 / np.pi))
    return x.dtype.type(0.5) * x * (x.dtype.type(1) + np.tanh(c * (x + x.dtype.type(0.044715) * x * x * x)))


def philox4x32_10(counter, key):
    """Philox-4x32 with 10 rounds (Salmon et al., SC'11): counter = 4 and key = 2 uint32 words."""
    M0, M1, W0, W1 = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85
    c = [int(v) & 0xFFFFFFFF for v in counter]
    k = [int(v) & 0xFFFFFFFF for v in key]
    for _ in range(10):
        p0, p1 = M0 * c[0], M1 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & 0xFFFFFFFF, p1 & 0xFFFFFFFF,
             ((p0 >> 32) ^ c[3] ^ k[1]) & 0xFFFFFFFF, p0 & 0xFFFFFFFF]
        k = [(k[0] + W0) & 0xFFFFFFFF, (k[1] + W1) & 0xFFFFFFFF]
    return c


def sample_uniform(seed, step, row):
    """The uniform number in [0, 1) that decides the token of (step, row)."""
    word = philox4x32_10((step, row, 0, 0), (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF))[0]
    return np.float32((word >> 8) * 2.0 ** -24)


def sample_topk(logits, k, u, p=1.0):
    """One draw (sampling decoding, sec. 3.4): the k largest logits, ranked (logit descending, token
    ascending), get the k-way softmax; with p < 1 only the shortest prefix of that ranking whose
    probability mass reaches p stays (nucleus inside the top k); the token is the first of the
    survivors whose cumulative weight exceeds u times the survivors' total.
    Returns (token, log-probability among the survivors, gap).  gap says how far the decision is
    from changing: the smallest of the logit gap between the k-th and (k+1)-th token (the candidate
    set), the logit gaps between the chosen candidate and its neighbours in the ranking (a swap of
    two ranks exchanges their probability segments), the distance of the draw from the nearest
    cumulative-probability boundary, and the distance of the nucleus mass from p at its cut."""
    V = logits.shape[0]
    order = np.lexsort((np.arange(V), -logits))[:k + 1]
    top = order[:k]
    l = logits[top].astype(np.float32)
    e = np.exp(l - l[0])
    cum = np.cumsum(e, dtype=np.float32)
    n = k
    cut_gap = np.inf
    if p < 1.0:
        thresh = np.float32(p) * cum[-1]
        n = min(int(np.searchsorted(cum, thresh, side="left")) + 1, k)     # first prefix with cum >= thresh
        cut_gap = abs(float(cum[n - 1]) / float(cum[-1]) - p)
        if n > 1:
            cut_gap = min(cut_gap, abs(float(cum[n - 2]) / float(cum[-1]) - p))
    target = np.float32(u) * cum[n - 1]
    j = int(np.searchsorted(cum[:n], target, side="right"))
    j = min(j, n - 1)
    edge = float(np.min(np.abs(cum[:n].astype(np.float64) - float(target))) / float(cum[n - 1]))
    gap = float(logits[order[k - 1]] - logits[order[k]]) if len(order) > k else np.inf
    if j > 0:
        gap = min(gap, float(l[j - 1] - l[j]))
    if j < k - 1:
        gap = min(gap, float(l[j] - l[j + 1]))
    return int(top[j]), float(np.log(e[j] / cum[n - 1])), min(gap, edge, cut_gap)


def gpt_forward_full(model, ids):
    """Logits after the last token of ``ids`` for ONE sequence, every position recomputed with a
    causal mask and no cache."""
    n, d = len(ids), model.d
    x = model.store(model.E[np.asarray(ids)] + model.P[:n])
    causal = np.tril(np.ones((n, n), bool))
    for L in model.dec:
        y = model.store(layer_norm(x, L["ln1_g"], L["ln1_b"], model.eps))
        qkv = model.store(y @ L["Wqkv"] + L["bqkv"])
        ctx = model.store(attention(qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:], model.H, causal))
        x = model.store(x + (ctx @ L["Wo"] + L["bo"]))
        y = model.store(layer_norm(x, L["ln2_g"], L["ln2_b"], model.eps))
        h = model.store(gelu_tanh(y @ L["W1"] + L["b1"]))
        x = model.store(x + (h @ L["W2"] + L["b2"]))
    y = model.store(layer_norm(x[-1], model.lnf_g, model.lnf_b, model.eps))
    return y @ model.E.T


class GptState:
    def __init__(self, model, prompts, max_len):
        prompts = np.asarray(prompts, np.int32)
        self.B, self.P = prompts.shape
        self.T = max_len
        self.tokens = np.full((self.B, max_len + 1), model.pad, np.int32)
        self.tokens[:, :self.P] = prompts
        self.pos = self.P - 1            # position of the token fed to the next step
        self.t = 0
        self.logp = np.zeros(self.B, model.ctype)
        self.Kc = [np.zeros((self.B, max_len, model.d), model.ctype) for _ in model.dec]
        self.Vc = [np.zeros((self.B, max_len, model.d), model.ctype) for _ in model.dec]


def gpt_rows(model, st, ids, positions, write_cache=True):
    """Runs the blocks for one position per sequence (ids [B], common position), K/V cached."""
    d, p = model.d, positions
    x = model.store(model.E[ids] + model.P[p])
    for l, L in enumerate(model.dec):
        y = model.store(layer_norm(x, L["ln1_g"], L["ln1_b"], model.eps))
        qkv = model.store(y @ L["Wqkv"] + L["bqkv"])
        st.Kc[l][:, p] = qkv[:, d:2 * d]
        st.Vc[l][:, p] = qkv[:, 2 * d:]
        ctx = np.empty_like(x)
        for r in range(x.shape[0]):
            ctx[r] = attention(qkv[r:r + 1, :d], st.Kc[l][r, :p + 1], st.Vc[l][r, :p + 1], model.H)[0]
        x = model.store(x + (model.store(ctx) @ L["Wo"] + L["bo"]))
        y = model.store(layer_norm(x, L["ln2_g"], L["ln2_b"], model.eps))
        h = model.store(gelu_tanh(y @ L["W1"] + L["b1"]))
        x = model.store(x + (h @ L["W2"] + L["b2"]))
    return x


def gpt_prefill(model, st):
    """Feeds the prompt except its last token, filling the cache for positions 0 .. P-2."""
    for p in range(st.P - 1):
        gpt_rows(model, st, st.tokens[:, p], p)


def gpt_step_logits(model, st):
    x = gpt_rows(model, st, st.tokens[:, st.pos], st.pos)
    y = model.store(layer_norm(x, model.lnf_g, model.lnf_b, model.eps))
    return y @ model.E.T


def gpt_advance(model, st, tokens, logps):
    st.pos += 1
    st.tokens[:, st.pos] = tokens
    st.logp = (st.logp + np.asarray(logps, model.ctype)).astype(model.ctype)
    st.t += 1


def generate(model, prompts, n_new, max_len, trace=None):
    st = GptState(model, prompts, max_len)
    gpt_prefill(model, st)
    for _ in range(n_new):
        logits = gpt_step_logits(model, st)
        picks = [sample_topk(logits[r], model.sample_topk, sample_uniform(model.seed, st.t, r), model.sample_topp)
                 for r in range(st.B)]
        if trace is not None:
            trace.append(dict(logits=logits, picks=picks))
        gpt_advance(model, st, [p[0] for p in picks], [p[1] for p in picks])
    return st.tokens[:, st.P:st.P + n_new].copy(), st.logp.copy(), st


# ----------------------------------------------------------------------------
# sampling decoding for an encoder-decoder model (sec. 3.4: the paper's text-generation runs use a
# Transformer with top-k 32 / top-p 0.75): one hypothesis per sentence; at every step each
# unfinished sentence draws its next token with sample_topk from its own logits, the uniform number
# being that of (step, index of the sentence in the batch); the hypothesis score adds the log of
# the drawn token's probability among the kept candidates; EOS or the length cap finishes a
# sentence, which then stays as it is.  The final score is the same length-normalised one as
# after beam search.
# ----------------------------------------------------------------------------
def sample_select(model, st, logits):
    """The draw of step st.t for every sentence: (token [B,1], parent [B,1] = 0, score [B,1], gaps [B])."""
    assert st.k == 1
    token = np.full((st.B, 1), model.eos, np.int32)
    parent = np.zeros((st.B, 1), np.int32)
    score = st.score.copy()
    gaps = np.full(st.B, np.inf)
    for b in range(st.B):
        if st.finished[b]:
            continue
        tok, lp, gaps[b] = sample_topk(logits[b], model.sample_topk, sample_uniform(model.seed, st.t, b), model.sample_topp)
        token[b, 0] = tok
        score[b, 0] = model.ctype(st.score[b, 0] + model.ctype(lp))
    return token, parent, score, gaps


def translate_sample(model, src_ids, src_lens, max_len, max_steps=None, trace=None):
    """Whole path with sampling instead of beam search; same returns as translate (beam = 1)."""
    assert model.sample_topk >= 1
    memory, cross = encode(model, src_ids, src_lens)
    st = DecodeState(model, src_lens, 1, max_len)
    steps = 0
    while True:
        logits = decoder_logits_cached(model, st, cross)
        token, parent, score, gaps = sample_select(model, st, logits)
        active = beam_advance(model, st, token, parent, score)
        steps += 1
        if trace is not None:
            trace.append(dict(logits=logits, token=token, score=score, gaps=gaps, active=active,
                              finished=st.finished.copy(), len=st.len.copy()))
        if active == 0 or (max_steps is not None and steps >= max_steps):
            break
    return finalize(model, st), st
