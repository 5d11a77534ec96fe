"""Diverse beam search: the HIP library against the oracle, step by step (needs an MI355X)."""
import numpy as np
import pytest

import lsq_synth as S
from oracle import lsq_oracle as O
from tests.parity import lockstep_diverse

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lsq():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2010_13887_amd as lib
    lib.load_library()
    yield lib
    lib.lsq_set_diversity(1, 0.0)
    lib.lsq_free()


@pytest.mark.parametrize("beam,groups,strength,dtype,vocab", [(4, 2, 0.5, 0, 37), (8, 4, 1.5, 0, 300), (6, 3, 0.3, 0, 1003),
                                                               (4, 4, 0.8, 0, 64), (4, 2, 0.5, 1, 504), (8, 2, 5.0, 1, 1000)])
def test_diverse_beam_search_matches_oracle(lsq, beam, groups, strength, dtype, vocab):
    hp = S.HParams(n_enc=1, n_dec=2, d_model=64, n_heads=4, d_ffn=96, vocab=vocab, max_pos=32, dtype=dtype, cap_extra=6)
    w = S.custom(hp, [5, 2, 9, 1], beam=beam, max_len=15, std=0.08 if dtype else 0.3)
    blob = w.blob(ln_jitter=0.1)
    with lsq.Engine(blob, w.batch, beam, w.max_len) as eng:
        res = lockstep_diverse(lsq, eng, blob, w, groups, strength)
        assert res["steps"] == 15
        assert res["strict"] >= 0.5 * (res["strict"] + res["band"])
        ids, lens, scores = eng.get_beams()
        o_ids, o_lens, o_scores = O.finalize(O.Model(blob), res["state"])
        for b in range(w.batch):
            np.testing.assert_allclose(scores[b], o_scores[b], rtol=2e-5, atol=5e-3)
            if (np.abs(np.diff(o_scores[b])) > 1e-2).all():
                assert np.array_equal(ids[b], o_ids[b]) and np.array_equal(lens[b], o_lens[b])


def test_one_group_and_setting_lifetime(lsq):
    """groups = 1 is ordinary beam search whatever the strength; the setting applies to the next encode only
    through lsq_set_diversity, and a beam the groups do not divide is refused."""
    hp = S.HParams(n_enc=1, n_dec=1, d_model=64, n_heads=4, d_ffn=96, vocab=200, max_pos=32, cap_extra=5)
    w = S.custom(hp, [4, 7, 3], beam=6, max_len=12, std=0.3)
    blob = w.blob()
    with lsq.Engine(blob, 3, 6, 12) as eng:
        plain = eng.translate(w.src_ids, w.src_lens)
        lsq.lsq_set_diversity(1, 3.0)
        same = eng.translate(w.src_ids, w.src_lens)
        lsq.lsq_set_diversity(3, 1.0)
        diverse = eng.translate(w.src_ids, w.src_lens, sync_every=3)
        diverse2 = eng.translate(w.src_ids, w.src_lens, sync_every=5)      # replayed graphs
        lsq.lsq_set_cache_refresh(lsq.REFRESH_MOVE)                         # cache rows moved by (global) parent
        diverse3 = eng.translate(w.src_ids, w.src_lens, sync_every=4)
        lsq.lsq_set_cache_refresh(lsq.REFRESH_TABLE)
        lsq.lsq_set_diversity(4, 1.0)
        with pytest.raises(lsq.LsqError):
            eng.encode(w.src_ids, w.src_lens)
        lsq.lsq_set_diversity(1, 0.0)
        back = eng.translate(w.src_ids, w.src_lens)
    for a, b, c in zip(plain, same, back):
        assert np.array_equal(a, b) and np.array_equal(a, c)
    for a, b, c in zip(diverse, diverse2, diverse3):
        assert np.array_equal(a, b) and np.array_equal(a, c)
    assert not np.array_equal(plain[0], diverse[0])
    with pytest.raises(lsq.LsqError):
        lsq.lsq_set_diversity(0, 1.0)
    with pytest.raises(lsq.LsqError):
        lsq.lsq_set_diversity(2, -1.0)
