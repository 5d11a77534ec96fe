"""Seeded synthetic inputs: weight blobs and translation workloads.

This module is the one thing the CPU oracle and the HIP library have in common:
it draws random numbers and writes them to bytes.  It contains none of the
method's arithmetic (no attention, no normalisation, no search, no positional
table) and imports neither side.

Blob format, version 1 (little endian)
--------------------------------------
A 256-byte header followed by tensors, each starting on a 256-byte boundary,
all in one element type (``dtype``: 0 = IEEE fp32, 1 = IEEE fp16).  Matrices
are row-major ``[in, out]``; the embedding table is ``[vocab, d_model]``.

Header fields (byte offset: type name)::

      0: char[8]  magic "LSQBLOB1"
      8: i32 version (1)        12: i32 arch (0 enc-dec, 1 dec-only)
     16: i32 n_enc              20: i32 n_dec
     24: i32 d_model            28: i32 n_heads
     32: i32 d_ffn              36: i32 vocab
     40: i32 max_pos            44: i32 act (0 relu, 1 gelu-tanh)
     48: i32 norm (0 post-LN, 1 pre-LN)
     52: i32 dtype              56: i32 pad_id   60: i32 bos_id   64: i32 eos_id
     68: i32 cap_extra          72: i32 sample_topk
     76: f32 length_penalty     80: f32 ln_eps   84: f32 sample_topp (0 = off)
     88: u64 seed               96: u64 total_bytes
    104..255: zero

Tensor order for arch 0 (encoder-decoder)::

    E[vocab, d]
    per encoder layer: Wqkv[d,3d] bqkv[3d] Wo[d,d] bo[d] ln1_g[d] ln1_b[d]
                       W1[d,F] b1[F] W2[F,d] b2[d] ln2_g[d] ln2_b[d]
    per decoder layer: Wqkv[d,3d] bqkv[3d] Wo[d,d] bo[d] ln1_g[d] ln1_b[d]
                       Wq_c[d,d] bq_c[d] Wkv_c[d,2d] bkv_c[2d] Wo_c[d,d] bo_c[d]
                       ln2_g[d] ln2_b[d]
                       W1[d,F] b1[F] W2[F,d] b2[d] ln3_g[d] ln3_b[d]

Tensor order for arch 1 (decoder-only, pre-LN, learned positions)::

    E[vocab, d]  P[max_pos, d]
    per layer: ln1_g[d] ln1_b[d] Wqkv[d,3d] bqkv[3d] Wo[d,d] bo[d]
               ln2_g[d] ln2_b[d] W1[d,F] b1[F] W2[F,d] b2[d]
    lnf_g[d] lnf_b[d]

Columns of Wqkv are [Q | K | V]; columns of Wkv_c are [K | V]; head h owns
columns h*dh .. (h+1)*dh of each part.
"""
from __future__ import annotations

import dataclasses
import struct

import numpy as np

MAGIC = b"LSQBLOB1"
HEADER_BYTES = 256
ALIGN = 256

WEIGHT_SEED = 1234
INPUT_SEED = 4321


@dataclasses.dataclass(frozen=True)
class HParams:
    arch: int = 0
    n_enc: int = 1
    n_dec: int = 1
    d_model: int = 64
    n_heads: int = 4
    d_ffn: int = 256
    vocab: int = 1000
    max_pos: int = 256
    act: int = 0
    norm: int = 0
    dtype: int = 0          # 0 fp32, 1 fp16
    pad_id: int = 0
    bos_id: int = 1
    eos_id: int = 2
    cap_extra: int = 50
    sample_topk: int = 0
    sample_topp: float = 1.0   # nucleus mass kept inside the top-k candidates; 1.0 = off
    length_penalty: float = 1.0
    ln_eps: float = 1e-5
    seed: int = WEIGHT_SEED


def tensor_list(hp: HParams):
    """(name, shape) of every tensor in file order."""
    d, F, V = hp.d_model, hp.d_ffn, hp.vocab
    out = [("E", (V, d))]
    if hp.arch == 1:
        out.append(("P", (hp.max_pos, d)))
        for i in range(hp.n_dec):
            p = f"dec{i}."
            out += [(p + "ln1_g", (d,)), (p + "ln1_b", (d,)), (p + "Wqkv", (d, 3 * d)), (p + "bqkv", (3 * d,)),
                    (p + "Wo", (d, d)), (p + "bo", (d,)), (p + "ln2_g", (d,)), (p + "ln2_b", (d,)),
                    (p + "W1", (d, F)), (p + "b1", (F,)), (p + "W2", (F, d)), (p + "b2", (d,))]
        out += [("lnf_g", (d,)), ("lnf_b", (d,))]
        return out
    if hp.arch != 0:
        raise NotImplementedError("unknown architecture")
    for i in range(hp.n_enc):
        p = f"enc{i}."
        out += [(p + "Wqkv", (d, 3 * d)), (p + "bqkv", (3 * d,)), (p + "Wo", (d, d)), (p + "bo", (d,)),
                (p + "ln1_g", (d,)), (p + "ln1_b", (d,)),
                (p + "W1", (d, F)), (p + "b1", (F,)), (p + "W2", (F, d)), (p + "b2", (d,)),
                (p + "ln2_g", (d,)), (p + "ln2_b", (d,))]
    for i in range(hp.n_dec):
        p = f"dec{i}."
        out += [(p + "Wqkv", (d, 3 * d)), (p + "bqkv", (3 * d,)), (p + "Wo", (d, d)), (p + "bo", (d,)),
                (p + "ln1_g", (d,)), (p + "ln1_b", (d,)),
                (p + "Wq_c", (d, d)), (p + "bq_c", (d,)), (p + "Wkv_c", (d, 2 * d)), (p + "bkv_c", (2 * d,)),
                (p + "Wo_c", (d, d)), (p + "bo_c", (d,)), (p + "ln2_g", (d,)), (p + "ln2_b", (d,)),
                (p + "W1", (d, F)), (p + "b1", (F,)), (p + "W2", (F, d)), (p + "b2", (d,)),
                (p + "ln3_g", (d,)), (p + "ln3_b", (d,))]
    return out


def _pack_header(hp: HParams, total: int) -> bytes:
    h = MAGIC + struct.pack(
        "<17i3fQQ", 1, hp.arch, hp.n_enc, hp.n_dec, hp.d_model, hp.n_heads, hp.d_ffn, hp.vocab,
        hp.max_pos, hp.act, hp.norm, hp.dtype, hp.pad_id, hp.bos_id, hp.eos_id, hp.cap_extra,
        hp.sample_topk, hp.length_penalty, hp.ln_eps, hp.sample_topp if hp.sample_topp < 1.0 else 0.0, hp.seed, total)
    return h + b"\0" * (HEADER_BYTES - len(h))


def make_blob(hp: HParams, *, std: float = 0.02, ln_jitter: float = 0.0,
              overrides: dict | None = None) -> bytes:
    """Draw every tensor from N(0, std^2) (LayerNorm gain 1, shift 0) and serialise.

    ``ln_jitter`` > 0 draws gains from N(1, ln_jitter^2) and shifts from
    N(0, ln_jitter^2) instead, so tests can see a swapped or dropped gain/shift.
    ``overrides`` maps a tensor name to an array that replaces the drawn one.
    """
    rng = np.random.Generator(np.random.PCG64(hp.seed))
    np_dt = np.float16 if hp.dtype == 1 else np.float32
    chunks = []
    off = HEADER_BYTES
    for name, shape in tensor_list(hp):
        short = name.split(".")[-1]
        if short.startswith("ln") and short.endswith("_g"):
            a = np.ones(shape, np.float32)
            if ln_jitter > 0:
                a = a + rng.standard_normal(shape, dtype=np.float32) * ln_jitter
        elif short.startswith("ln") and short.endswith("_b"):
            a = np.zeros(shape, np.float32)
            if ln_jitter > 0:
                a = rng.standard_normal(shape, dtype=np.float32) * ln_jitter
        else:
            a = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
        if overrides and name in overrides:
            a = np.asarray(overrides[name], np.float32).reshape(shape)
        raw = np.ascontiguousarray(a.astype(np_dt)).tobytes()
        pad = (-off) % ALIGN
        chunks.append(b"\0" * pad)
        off += pad
        chunks.append(raw)
        off += len(raw)
    body = b"".join(chunks)
    total = HEADER_BYTES + len(body)
    return _pack_header(hp, total) + body


@dataclasses.dataclass
class Workload:
    name: str
    hp: HParams
    batch: int
    beam: int
    max_len: int               # maximum target length == K/V cache length
    src_lens: np.ndarray       # int32 [batch]
    src_ids: np.ndarray        # int32 [batch, src_stride], pad_id beyond each length
    std: float = 0.02

    def blob(self, **kw) -> bytes:
        kw.setdefault("std", self.std)
        return make_blob(self.hp, **kw)


def _ids(rng, lens, vocab, pad):
    stride = int(lens.max())
    ids = np.full((len(lens), stride), pad, np.int32)
    for i, s in enumerate(lens):
        ids[i, :s] = rng.integers(4, vocab, size=int(s), dtype=np.int64).astype(np.int32)
    return ids


def _lognormal_lens(rng, n, mean=28.0, sigma=0.6, lo=1, hi=128):
    mu = np.log(mean) - 0.5 * sigma * sigma
    out = np.empty(n, np.int32)
    i = 0
    while i < n:
        v = int(np.rint(np.exp(rng.normal(mu, sigma))))
        if lo <= v <= hi:
            out[i] = v
            i += 1
    return out


BASE = dict(n_enc=6, n_dec=6, d_model=512, n_heads=8, d_ffn=2048, vocab=32000, dtype=1, max_pos=256)
BIG = dict(n_enc=6, n_dec=6, d_model=1024, n_heads=16, d_ffn=4096, vocab=32000, dtype=1, max_pos=256)


def workload(name: str, *, batch: int | None = None, seed: int = INPUT_SEED) -> Workload:
    """The named synthetic workloads (stand-ins for the paper's WMT14 En-De buckets).

    gpt2s : decoder-only GPT-2-small shape, fp16, top-8 sampling (see below).
    gpt2s_k32p75 : the same with the paper's sampling setting, top-k 32 and top-p 0.75.
    tiny : 1+1 layers, d 64, 4 heads, FFN 256, vocab 1000, fp32; batch 2, lengths 5 and 8,
           beam 4, max target length 8.
    base : Transformer-base shape, fp16; batch 8, lengths U{10..60}, beam 4, cap = len + 50.
    big  : Transformer-big shape, fp16; batch 32, same length law.
    big128 : Transformer-big, batch 128, lengths from a truncated log-normal (mean 28, max 128).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    if name == "tiny":
        hp = HParams(max_pos=64)
        lens = np.array([5, 8], np.int32)
        if batch is not None and batch != 2:
            lens = rng.integers(1, 9, size=batch).astype(np.int32)
        return Workload(name, hp, len(lens), 4, 8, lens, _ids(rng, lens, hp.vocab, hp.pad_id))
    if name in ("base", "big"):
        hp = HParams(**(BASE if name == "base" else BIG))
        b = batch or (8 if name == "base" else 32)
        lens = rng.integers(10, 61, size=b).astype(np.int32)
        return Workload(name, hp, b, 4, int(lens.max()) + hp.cap_extra, lens,
                        _ids(rng, lens, hp.vocab, hp.pad_id))
    if name == "base_k32p75":
        # the paper's text-generation runs (sec. 3.4): randomly initialised Transformer-base, random
        # inputs, sampling decoding with top-k 32 / top-p 0.75; batch 32, one hypothesis per sentence
        hp = HParams(**BASE, sample_topk=32, sample_topp=0.75)
        b = batch or 32
        lens = rng.integers(10, 61, size=b).astype(np.int32)
        return Workload(name, hp, b, 1, int(lens.max()) + hp.cap_extra, lens,
                        _ids(rng, lens, hp.vocab, hp.pad_id))
    if name == "big128":
        hp = HParams(**BIG)
        b = batch or 128
        lens = _lognormal_lens(rng, b)
        return Workload(name, hp, b, 4, int(lens.max()) + hp.cap_extra, lens,
                        _ids(rng, lens, hp.vocab, hp.pad_id))
    if name in ("gpt2s", "gpt2s_k32p75"):
        # decoder-only, GPT-2-small shape: 12 layers, d 768, 12 heads, FFN 3072, tanh-GELU, pre-LN,
        # vocab 50257, learned positions; batch 32 prompts of 64 random ids, 128 sampled tokens (top-8)
        hp = HParams(arch=1, n_enc=0, n_dec=12, d_model=768, n_heads=12, d_ffn=3072, vocab=50257, dtype=1,
                     max_pos=256, act=1, norm=1, cap_extra=128,
                     **(dict(sample_topk=8) if name == "gpt2s" else dict(sample_topk=32, sample_topp=0.75)))
        b = batch or 32
        lens = np.full(b, 64, np.int32)
        return Workload(name, hp, b, 1, 64 + 128, lens, _ids(rng, lens, hp.vocab, hp.pad_id))
    raise KeyError(name)


def custom(hp: HParams, src_lens, beam: int, max_len: int, *, seed: int = INPUT_SEED,
           name: str = "custom", std: float = 0.02) -> Workload:
    """A workload with caller-chosen shapes (tests: ragged sizes, edge cases)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    lens = np.asarray(src_lens, np.int32)
    return Workload(name, hp, len(lens), beam, max_len, lens, _ids(rng, lens, hp.vocab, hp.pad_id), std)
