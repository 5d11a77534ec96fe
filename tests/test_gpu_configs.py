"""Parity on the Transformer-base / -big shaped workloads at their full sizes, in the launch
configuration bench.py times (needs an MI355X).  The oracle is run side by side for a bounded
number of decode steps; beyond that, properties that hold at any size are checked."""
import numpy as np
import pytest

import lsq_synth as S
from tests.parity import lockstep

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lsq():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2010_13887_amd as lib
    lib.load_library()
    yield lib
    lib.lsq_free()


def _properties(w, ids, lens, scores, hp):
    caps = np.minimum(w.src_lens + hp.cap_extra, w.max_len)
    for b in range(w.batch):
        assert (np.diff(scores[b]) <= 0).all()                     # best first
        for i in range(w.beam):
            n = lens[b, i]
            assert 1 <= n <= caps[b]
            seq = ids[b, i, :n]
            assert ((seq >= 0) & (seq < hp.vocab)).all()
            assert hp.eos_id not in seq[:-1]
            assert seq[-1] == hp.eos_id or n == caps[b]
            assert (ids[b, i, n:] == hp.pad_id).all()
    assert np.isfinite(scores).all() and (scores < 0).all()


@pytest.mark.parametrize("name,steps", [("base", 40), ("big", 12), ("big128", 6)])
def test_config_matches_oracle_then_finishes(lsq, name, steps):
    w = S.workload(name)
    blob = w.blob()
    print(f"{name}: batch {w.batch} max_len {w.max_len}", flush=True)
    with lsq.Engine(blob, w.batch, w.beam, w.max_len) as eng:
        res = lockstep(lsq, eng, blob, w, max_steps=steps, verbose=True)
        assert res["steps"] == steps
        assert res["strict"] >= 0.5 * steps * w.batch, res     # most decisions are outside the near-tie band
        assert res["worst_wide"] <= 2e-2 and res["worst_tight"] <= 1e-2
        # run to the end without per-step synchronisation, as bench.py does
        while eng.decode_steps(32) > 0:
            pass
        assert lsq.lsq_step_index() == int((w.src_lens + w.hp.cap_extra).max()) or lsq.lsq_step_index() <= w.max_len
        ids, lens, scores = eng.get_beams()
        _properties(w, ids, lens, scores, w.hp)
        # the same translation again, chunked differently: bit-identical
        ids2, lens2, scores2 = eng.translate(w.src_ids, w.src_lens, sync_every=7)
        assert np.array_equal(ids, ids2) and np.array_equal(lens, lens2) and np.array_equal(scores, scores2)


def test_big_shape_few_sentences_whole_translation(lsq):
    """Transformer-big weights, three sentences, every step to the end in lock-step with the oracle:
    the few-row regime at the real layer sizes (skinny products, LayerNorm inside the consuming
    product once one or two sentences are left, split self-attention, long slab-table histories)."""
    big = S.workload("big")
    w = S.custom(big.hp, [12, 30, 5], beam=4, max_len=30 + big.hp.cap_extra)
    blob = w.blob()
    with lsq.Engine(blob, w.batch, w.beam, w.max_len) as eng:
        res = lockstep(lsq, eng, blob, w, check_wide=False, verbose=True)
        assert res["steps"] == 30 + big.hp.cap_extra
        assert res["strict"] >= 0.5 * (12 + 30 + 5 + 3 * big.hp.cap_extra), res
        assert res["worst_tight"] <= 1e-2
        ids, lens, scores = eng.get_beams()
        _properties(w, ids, lens, scores, w.hp)
