"""Sampling decoding of encoder-decoder models (paper sec. 3.4): parity of the HIP library against the
oracle (needs an MI355X)."""
import dataclasses

import numpy as np
import pytest

import lsq_synth as S
from oracle import lsq_oracle as O
from tests.parity import lockstep_sample

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lsq():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2010_13887_amd as lib
    lib.load_library()
    yield lib
    lib.lsq_free()


def _final_check(eng, m, res, w):
    ids, lens, scores = eng.get_beams()
    ref_ids, ref_lens, ref_scores = O.finalize(m, res["state"])
    assert np.array_equal(lens, ref_lens) and np.array_equal(ids, ref_ids)
    np.testing.assert_allclose(scores, ref_scores, rtol=2e-5, atol=5e-2 if m.round16 else 1e-3)
    caps = np.minimum(w.src_lens + m.cap_extra, w.max_len)
    assert ((lens[:, 0] >= 1) & (lens[:, 0] <= caps)).all()


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("k,topp", [(4, 1.0), (32, 0.75), (1, 1.0), (8, 0.3)])
def test_small_translation_with_sampling_matches_oracle(lsq, dtype, k, topp):
    hp = S.HParams(n_enc=1, n_dec=2, d_model=128, n_heads=2, d_ffn=264, vocab=503, max_pos=64, dtype=dtype,
                   cap_extra=7, sample_topk=k, sample_topp=topp, seed=77 + k)
    w = S.custom(hp, [5, 11, 2, 8, 8, 3], beam=1, max_len=16, std=0.3 if dtype == 0 else 0.08, seed=5)
    blob = w.blob(ln_jitter=0.1)
    m = O.Model(blob)
    with lsq.Engine(blob, 7, 1, w.max_len) as eng:
        res = lockstep_sample(lsq, eng, blob, w)
        assert res["steps"] == min(max(w.src_lens) + 7, 16)
        assert res["strict"] >= (0.1 if dtype else 0.7) * (res["strict"] + res["loose"]), res
        _final_check(eng, m, res, w)
        assert eng.decode_step() == 0


def test_eos_ends_sentences_early(lsq):
    """A vocabulary barely wider than the candidate set: EOS is drawn often, sentences finish at
    different steps and the live prefix shrinks while others go on."""
    ended_by_eos = 0
    for seed in range(4):
        hp = S.HParams(n_enc=1, n_dec=1, d_model=64, n_heads=4, d_ffn=96, vocab=9, max_pos=32, dtype=0, cap_extra=6,
                       sample_topk=6, seed=seed)
        w = S.custom(hp, [4, 9, 1, 6, 6], beam=1, max_len=12, std=0.5, seed=seed)
        blob = w.blob(ln_jitter=0.1)
        m = O.Model(blob)
        with lsq.Engine(blob, 5, 1, w.max_len) as eng:
            res = lockstep_sample(lsq, eng, blob, w)
            _final_check(eng, m, res, w)
            ids, lens, _ = eng.get_beams()
            ended_by_eos += sum(ids[b, 0, lens[b, 0] - 1] == m.eos for b in range(w.batch))
    assert ended_by_eos >= 5


def test_graph_replay_and_chunking_do_not_change_the_samples(lsq):
    hp = S.HParams(n_enc=2, n_dec=2, d_model=128, n_heads=4, d_ffn=256, vocab=1000, max_pos=64, dtype=1, cap_extra=9,
                   sample_topk=16, sample_topp=0.8, seed=3)
    w = S.custom(hp, [7, 3, 12, 5], beam=1, max_len=21, std=0.08)
    blob = w.blob(ln_jitter=0.1)
    outs = []
    try:
        for graphs, chunk in ((True, 1), (True, 5), (False, 3)):
            lsq.lsq_set_graphs(graphs)
            with lsq.Engine(blob, 4, 1, w.max_len) as eng:
                outs.append(eng.translate(w.src_ids, w.src_lens, sync_every=chunk))
                outs.append(eng.translate(w.src_ids, w.src_lens, sync_every=chunk))     # same seed, same draws
    finally:
        lsq.lsq_set_graphs(True)
    for o in outs[1:]:
        for a, b in zip(outs[0], o):
            assert np.array_equal(a, b)
    # the place in the batch decides the uniform numbers: the same sentences in another order draw differently
    order = [2, 0, 3, 1]
    with lsq.Engine(blob, 4, 1, w.max_len) as eng:
        ids2, lens2, _ = eng.translate(w.src_ids[order], w.src_lens[order], sync_every=4)
    assert not all(np.array_equal(ids2[i], outs[0][0][order[i]]) for i in range(4))


def test_sampling_model_refuses_a_beam(lsq):
    hp = S.HParams(n_enc=1, n_dec=1, d_model=64, n_heads=4, d_ffn=96, vocab=50, max_pos=16, sample_topk=4)
    blob = S.custom(hp, [3], beam=1, max_len=8).blob()
    with pytest.raises(lsq.LsqError, match="beam 1"):
        lsq.Engine(blob, 1, 4, 8)
    bad = S.custom(dataclasses.replace(hp, sample_topk=33), [3], beam=1, max_len=8).blob()
    with pytest.raises(lsq.LsqError, match="sample_topk"):
        lsq.Engine(bad, 1, 1, 8)


def test_transformer_base_top32_nucleus(lsq):
    """The paper's text-generation shape: Transformer-base, top-k 32 / top-p 0.75, batch 32; a few steps in
    lock-step, then the whole generation with properties that hold at any size."""
    w = S.workload("base_k32p75")
    blob = w.blob()
    m = O.Model(blob)
    with lsq.Engine(blob, w.batch, 1, w.max_len) as eng:
        res = lockstep_sample(lsq, eng, blob, w, max_steps=8)
        assert res["steps"] == 8 and res["worst"] <= 1e-2
        ids, lens, scores = eng.translate(w.src_ids, w.src_lens, sync_every=16)
        caps = np.minimum(w.src_lens + m.cap_extra, w.max_len)
        for b in range(w.batch):
            n = lens[b, 0]
            seq = ids[b, 0, :n]
            assert 1 <= n <= caps[b] and m.eos not in seq[:-1] and (seq[-1] == m.eos or n == caps[b])
            assert ((seq >= 0) & (seq < m.V)).all() and (ids[b, 0, n:] == m.pad).all()
        assert np.isfinite(scores).all() and (scores <= 0).all()
        again = eng.translate(w.src_ids, w.src_lens, sync_every=7)
        for a, b_ in zip((ids, lens, scores), again):
            assert np.array_equal(a, b_)
