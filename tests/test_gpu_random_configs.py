"""Randomised end-to-end parity: seeded draws of model shape (head size 16-128, 1-8 heads, odd FFN
and vocabulary sizes), dtype, depth, batch, source lengths, caps, beam width and search method
(beam search, diverse beam search, sampling), each run in lock-step against the oracle (needs an
MI355X).  Weight scales follow the model width so that activations stay in the range of the other
tests, whose tolerances these runs share."""
import numpy as np
import pytest

import lsq_synth as S
from tests.parity import lockstep, lockstep_diverse, lockstep_gpt, lockstep_sample

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lsq():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2010_13887_amd as lib
    lib.load_library()
    yield lib
    lib.lsq_set_cache_refresh(lib.REFRESH_TABLE)
    lib.lsq_free()


def draw(seed):
    rng = np.random.default_rng(1000 + seed)
    dh = int(rng.choice([16, 32, 64, 128]))
    H = int(rng.choice([1, 2, 3, 4, 8]))
    if dh * H > 512:
        H = 512 // dh
    d = dh * H
    F = int(rng.choice([24, 64, 136, 256, 520]))
    V = int(rng.choice([5, 12, 37, 64, 301, 1000, 1003, 2048, 5000, 9001]))
    dtype = int(rng.integers(0, 2))
    n_enc, n_dec = int(rng.integers(1, 3)), int(rng.integers(1, 4))
    batch = int(rng.integers(1, 10))
    lens = [int(v) for v in rng.integers(1, 40, size=batch)]
    cap_extra = int(rng.integers(0, 8))
    max_len = max(int(min(max(lens) + cap_extra, rng.integers(3, 48))), max(lens))
    mode = str(rng.choice(["beam", "beam", "sample", "diverse"]))
    beam = 1 if mode == "sample" else min(int(rng.integers(1, 9)), V)
    kw = {}
    if mode == "sample":
        kw = dict(sample_topk=int(min(V, rng.choice([1, 3, 8, 32]))), sample_topp=float(rng.choice([1.0, 0.75, 0.3])))
    hp = S.HParams(n_enc=n_enc, n_dec=n_dec, d_model=d, n_heads=H, d_ffn=F, vocab=V, max_pos=64, dtype=dtype,
                   cap_extra=cap_extra, seed=seed, **kw)
    std = min(0.08, 0.9 / d ** 0.5) if dtype else min(0.3, 3.4 / d ** 0.5)
    w = S.custom(hp, lens, beam=beam, max_len=max_len, std=std, seed=seed)
    groups = [g for g in (2, 3, 4) if beam % g == 0] if mode == "diverse" else []
    return dict(w=w, mode=mode, refresh=int(rng.integers(0, 2)), spare=int(rng.integers(0, 3)),
                groups=int(rng.choice(groups)) if groups else 1, strength=float(rng.choice([0.0, 0.5, 2.0])))


F32_STATS = dict(runs=0, steps=0, over=0, over_ceiling=0, worst_bound=0.0, worst_ratio=0.0)


def _collect(res, w):
    if w.hp.dtype != 0:
        return
    F32_STATS["runs"] += 1
    F32_STATS["steps"] += res["steps"]
    F32_STATS["over"] += res["f32_steps_over"]
    F32_STATS["over_ceiling"] += res["f32_steps_over_ceiling"]
    F32_STATS["worst_bound"] = max(F32_STATS["worst_bound"], res["f32_worst_bound"])
    F32_STATS["worst_ratio"] = max(F32_STATS["worst_ratio"], res["f32_worst_ratio"])


# 597: beams of 8 over 37 tokens; a sentence finishes in an order that the comparison took over from the library
# within its band, and must then be left alone by both sides while the other sentences go on
@pytest.mark.parametrize("seed", list(range(48)) + [597])
def test_random_configuration_matches_oracle(lsq, seed):
    c = draw(seed)
    w = c["w"]
    blob = w.blob(ln_jitter=0.1)
    lsq.lsq_set_cache_refresh(c["refresh"])
    with lsq.Engine(blob, w.batch + c["spare"], w.beam, w.max_len) as eng:
        if c["mode"] == "sample":
            res = lockstep_sample(lsq, eng, blob, w)
        elif c["groups"] > 1:
            res = lockstep_diverse(lsq, eng, blob, w, c["groups"], c["strength"])
        else:
            res = lockstep(lsq, eng, blob, w)
        _collect(res, w)
        caps = np.minimum(w.src_lens + w.hp.cap_extra, w.max_len)
        assert res["steps"] <= int(caps.max())
        ids, lens, _ = eng.get_beams()
        assert ((lens >= 0) & (lens <= caps[:, None])).all()
        assert ((ids >= 0) & (ids < w.hp.vocab)).all()


def draw_decoder_only(seed):
    rng = np.random.default_rng(5000 + seed)
    dh = int(rng.choice([16, 32, 64, 128]))
    H = int(rng.choice([1, 2, 3, 4, 6]))
    if dh * H > 768:
        H = 768 // dh
    d = dh * H
    F = int(rng.choice([24, 64, 136, 264, 520]))
    V = int(rng.choice([37, 64, 301, 1003, 2048, 9001]))
    dtype = int(rng.integers(0, 2))
    n_dec = int(rng.integers(1, 5))
    batch = int(rng.integers(1, 12))
    P = int(rng.integers(1, 20))
    n_new = int(rng.integers(1, 12))
    k = int(min(V, rng.choice([1, 2, 5, 8, 16, 32])))
    topp = float(rng.choice([1.0, 0.9, 0.5]))
    hp = S.HParams(arch=1, n_enc=0, n_dec=n_dec, d_model=d, n_heads=H, d_ffn=F, vocab=V, max_pos=64, act=1, norm=1,
                   dtype=dtype, sample_topk=k, sample_topp=topp, cap_extra=n_new, seed=seed)
    std = min(0.08, 0.9 / d ** 0.5) if dtype else min(0.3, 3.4 / d ** 0.5)
    w = S.custom(hp, [P] * batch, beam=1, max_len=P + n_new + int(rng.integers(0, 3)), std=std, seed=seed)
    return w, int(rng.integers(0, 3))


@pytest.mark.parametrize("seed", range(24))
def test_random_decoder_only_configuration_matches_oracle(lsq, seed):
    w, spare = draw_decoder_only(seed)
    blob = w.blob(ln_jitter=0.1)
    with lsq.Engine(blob, w.batch + spare, 1, w.max_len) as eng:
        res = lockstep_gpt(lsq, eng, blob, w)
        _collect(res, w)
        assert res["steps"] == w.hp.cap_extra
        ids, lens, _ = eng.get_beams()
        assert (lens[:, 0] == w.hp.cap_extra).all()
        assert np.array_equal(ids[:, 0, :w.hp.cap_extra], res["state"].tokens[:, int(w.src_lens[0]):int(w.src_lens[0]) + w.hp.cap_extra])


def test_float32_bound_statistics(lsq):
    """How often the float32 models above needed more than the stated 1e-4 (see parity.Float32Shadow), and how far the
    library's worst logit error of a run ever was from plain numpy float32's worst over the same run.  Runs after
    the configurations (same module); the numbers are those quoted in the design notes."""
    print("float32 models of the random configurations:", F32_STATS, flush=True)
    if F32_STATS["runs"] == 0:
        pytest.skip("the random configurations were deselected")
    assert F32_STATS["worst_ratio"] <= 4.0                                     # by construction; measured: see the print
    assert F32_STATS["over_ceiling"] <= 0.25 * F32_STATS["steps"] + 2
    assert F32_STATS["over"] <= 0.6 * F32_STATS["steps"] + 2
