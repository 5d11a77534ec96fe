"""Decoder-only model with top-k sampling: parity of the HIP library against the oracle (needs an MI355X)."""
import numpy as np
import pytest

import lsq_synth as S
from tests.parity import lockstep_gpt

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lsq():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2010_13887_amd as lib
    lib.load_library()
    yield lib
    lib.lsq_free()


def _small(dtype, seed):
    hp = S.HParams(arch=1, n_enc=0, n_dec=3, d_model=128, n_heads=2, d_ffn=264, vocab=1003, max_pos=64, act=1, norm=1,
                   dtype=dtype, sample_topk=5, cap_extra=9, seed=seed)
    return S.custom(hp, [6] * 5, beam=1, max_len=6 + 9, std=0.08, seed=seed)


@pytest.mark.parametrize("dtype", [0, 1])
def test_small_gpt_matches_oracle(lsq, dtype):
    w = _small(dtype, 11 + dtype)
    blob = w.blob(ln_jitter=0.1)
    with lsq.Engine(blob, 6, 1, w.max_len) as eng:
        res = lockstep_gpt(lsq, eng, blob, w, verbose=True)
        assert res["strict"] >= (0.5 if dtype else 0.9) * res["steps"] * w.batch, res   # fp16: clear decisions only
        ids, lens, scores = eng.get_beams()
        st = res["state"]
        assert (lens[:, 0] == 9).all()
        assert np.array_equal(ids[:, 0, :9], st.tokens[:, 6:15])
        assert (ids[:, 0, 9:] == 0).all()
        np.testing.assert_allclose(scores[:, 0], st.logp, rtol=2e-5, atol=5e-2 if dtype else 1e-3)
        assert eng.decode_step() == 0                       # nothing left to generate


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("k,topp", [(32, 0.75), (16, 1.0), (32, 0.2), (3, 0.9)])
def test_topk_topp_sampling_matches_oracle(lsq, dtype, k, topp):
    """Wide candidate sets and a nucleus cut inside them (the paper's sampling runs use top-k 32, top-p 0.75)."""
    hp = S.HParams(arch=1, n_enc=0, n_dec=2, d_model=128, n_heads=2, d_ffn=264, vocab=1003, max_pos=64, act=1, norm=1,
                   dtype=dtype, sample_topk=k, sample_topp=topp, cap_extra=8, seed=40 + k)
    w = S.custom(hp, [5] * 6, beam=1, max_len=5 + 8, std=0.3 if dtype == 0 else 0.08, seed=3)
    blob = w.blob(ln_jitter=0.1)
    with lsq.Engine(blob, 6, 1, w.max_len) as eng:
        res = lockstep_gpt(lsq, eng, blob, w)
        # float16 with 32 candidates: the 32nd and 33rd logits are rarely further apart than the fp16 band, so most
        # draws are checked on the library's own logits (exactly) rather than against the oracle's
        assert res["strict"] >= (0.1 if dtype else 0.8) * res["steps"] * w.batch, res
        ids, lens, scores = eng.get_beams()
        st = res["state"]
        assert np.array_equal(ids[:, 0, :8], st.tokens[:, 5:13])
        np.testing.assert_allclose(scores[:, 0], st.logp, rtol=2e-5, atol=5e-2 if dtype else 1e-3)


@pytest.mark.parametrize("d,heads,batch,prompt,rows_per_workgroup", [
    (256, 4, 7, 5, 1),      # one row per workgroup
    (512, 8, 40, 3, 2),     # 40 * 8 workgroups would exceed the CUs: rows in pairs
    (512, 8, 33, 9, 1),     # ... an odd row count cannot pair
    (256, 4, 64, 4, 1),     # the most rows
])
def test_attention_blocks_match_oracle(lsq, d, heads, batch, prompt, rows_per_workgroup):
    """Float16 models with heads of 64 and at most 64 rows run each block's attention sublayer as one launch
    (LayerNorm, QKV, cache append, attention, per-head output projection) with the pre-LN arithmetic; lock-step
    with the oracle, then the same translation with the separate kernels: the logits behind every draw agree to
    float16 rounding, so the scores do wherever the same tokens were drawn."""
    hp = S.HParams(arch=1, n_enc=0, n_dec=3, d_model=d, n_heads=heads, d_ffn=2 * d + 8, vocab=1003, max_pos=64, act=1, norm=1,
                   dtype=1, sample_topk=4, cap_extra=10, seed=d + batch)
    w = S.custom(hp, [prompt] * batch, beam=1, max_len=prompt + 10, std=0.05, seed=batch)
    blob = w.blob(ln_jitter=0.1)
    del rows_per_workgroup   # what the library picks for this shape; documented here, not settable
    with lsq.Engine(blob, batch, 1, w.max_len) as eng:
        res = lockstep_gpt(lsq, eng, blob, w, verbose=True)
        assert res["steps"] == 10
        ids, lens, scores = eng.get_beams()
        st = res["state"]
        assert np.array_equal(ids[:, 0, :10], st.tokens[:, prompt:prompt + 10])
        np.testing.assert_allclose(scores[:, 0], st.logp, rtol=2e-5, atol=5e-2)
        try:
            lsq.lsq_set_attention_blocks(0)
            ids0, lens0, scores0 = eng.translate(w.src_ids, w.src_lens)
        finally:
            lsq.lsq_set_attention_blocks(64)
        same = (ids0[:, 0, :10] == ids[:, 0, :10]).all(axis=1)
        assert same.mean() >= 0.5, same
        np.testing.assert_allclose(scores0[same, 0], scores[same, 0], rtol=0, atol=3e-2)


def test_prompt_of_one_token_and_errors(lsq):
    hp = S.HParams(arch=1, n_enc=0, n_dec=2, d_model=64, n_heads=4, d_ffn=128, vocab=300, max_pos=32, act=1, norm=1,
                   sample_topk=8, cap_extra=4, seed=5)
    w = S.custom(hp, [1, 1, 1], beam=1, max_len=8)
    blob = w.blob()
    with pytest.raises(lsq.LsqError):
        lsq.Engine(blob, 3, 2, 8)                            # sampling models run at beam 1
    with pytest.raises(lsq.LsqError):
        lsq.Engine(blob, 3, 1, 64)                           # more positions than the model has
    with lsq.Engine(blob, 3, 1, 8) as eng:
        res = lockstep_gpt(lsq, eng, blob, w)
        assert res["steps"] == 4
        with pytest.raises(lsq.LsqError):
            eng.encode(np.full((2, 3), 7, np.int32), [3, 2])   # prompts of different lengths
        with pytest.raises(lsq.LsqError):
            eng.encode(np.full((2, 6), 7, np.int32), [6, 6])   # 6 + 4 tokens do not fit 8 positions


@pytest.mark.parametrize("name", ["gpt2s", "gpt2s_k32p75"])
def test_gpt2_small_shape(lsq, name):
    """The GPT-2-small-shaped workload (batch 32, prompt 64, top-8 sampling; or top-32 with a 0.75 nucleus):
    40 steps in lock-step with the oracle, then the remaining steps without per-step waits; a second run is
    bit-identical."""
    w = S.workload(name)
    blob = w.blob()
    with lsq.Engine(blob, w.batch, 1, w.max_len) as eng:
        res = lockstep_gpt(lsq, eng, blob, w, n_steps=40, verbose=True)
        # random weights give nearly flat logits: most draws sit within the fp16 band of a rank swap or an
        # edge and are checked on the library's own logits instead (exactly, inside lockstep_gpt)
        if name == "gpt2s":      # with 32 candidates of a random model no draw is clear of the fp16 band: own-logit checks only
            assert res["strict"] >= 0.25 * 40 * w.batch, res
        while eng.decode_steps(32) > 0:
            pass
        assert lsq.lsq_step_index() == 128
        ids, lens, scores = eng.get_beams()
        assert (lens == 128).all() and ((ids[:, 0, :128] >= 0) & (ids[:, 0, :128] < w.hp.vocab)).all()
        assert np.isfinite(scores).all() and (scores < 0).all()
        ids2, lens2, scores2 = eng.translate(w.src_ids, w.src_lens, sync_every=9)
        assert np.array_equal(ids, ids2) and np.array_equal(scores, scores2)
