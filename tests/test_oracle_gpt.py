"""Pins for the oracle's decoder-only path: Philox known answers, tanh-GELU and a pre-LN block stack
against torch, cached == full recomputation, and the sampling rule against brute force."""
import numpy as np
import torch

import lsq_synth as S
from oracle import lsq_oracle as O

torch.set_grad_enabled(False)

HP = S.HParams(arch=1, n_enc=0, n_dec=2, d_model=32, n_heads=4, d_ffn=48, vocab=61, max_pos=24, act=1, norm=1,
               sample_topk=5, cap_extra=6, seed=99)


def test_philox_known_answers():
    # Random123 known-answer vectors for philox4x32-10
    assert O.philox4x32_10((0, 0, 0, 0), (0, 0)) == [0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8]
    ones = 0xFFFFFFFF
    assert O.philox4x32_10((ones,) * 4, (ones, ones)) == [0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd]
    assert O.philox4x32_10((0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344), (0xa4093822, 0x299f31d0)) == \
        [0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1]
    u = [float(O.sample_uniform(7, t, r)) for t in range(40) for r in range(25)]
    assert 0 <= min(u) and max(u) < 1 and abs(np.mean(u) - 0.5) < 0.03 and len(set(u)) == len(u)


def test_gelu_tanh_matches_torch():
    x = np.linspace(-6, 6, 1001)
    ref = torch.nn.functional.gelu(torch.from_numpy(x), approximate="tanh").numpy()
    np.testing.assert_allclose(O.gelu_tanh(x), ref, rtol=0, atol=1e-14)


def _t(a):
    return torch.from_numpy(np.ascontiguousarray(a)).double()


def test_block_stack_matches_torch_prenorm_layers():
    m = O.Model(S.make_blob(HP, std=0.3, ln_jitter=0.3), ctype=np.float64)
    rng = np.random.default_rng(0)
    ids = rng.integers(4, m.V, size=9)
    got = O.gpt_forward_full(m, ids)
    x = (_t(m.E[ids]) + _t(m.P[:9]))[None]
    causal = torch.triu(torch.ones(9, 9, dtype=torch.bool), 1)
    for L in m.dec:
        t = torch.nn.TransformerEncoderLayer(m.d, m.H, m.F, dropout=0.0, layer_norm_eps=float(m.eps), batch_first=True,
                                             norm_first=True,
                                             activation=lambda v: torch.nn.functional.gelu(v, approximate="tanh")).double().eval()
        t.self_attn.in_proj_weight.copy_(_t(L["Wqkv"].T)); t.self_attn.in_proj_bias.copy_(_t(L["bqkv"]))
        t.self_attn.out_proj.weight.copy_(_t(L["Wo"].T)); t.self_attn.out_proj.bias.copy_(_t(L["bo"]))
        t.linear1.weight.copy_(_t(L["W1"].T)); t.linear1.bias.copy_(_t(L["b1"]))
        t.linear2.weight.copy_(_t(L["W2"].T)); t.linear2.bias.copy_(_t(L["b2"]))
        t.norm1.weight.copy_(_t(L["ln1_g"])); t.norm1.bias.copy_(_t(L["ln1_b"]))
        t.norm2.weight.copy_(_t(L["ln2_g"])); t.norm2.bias.copy_(_t(L["ln2_b"]))
        x = t(x, src_mask=causal)
    y = torch.nn.functional.layer_norm(x[0, -1], (m.d,), _t(m.lnf_g), _t(m.lnf_b), float(m.eps))
    np.testing.assert_allclose(got, (y @ _t(m.E).T).numpy(), rtol=0, atol=1e-10)


def test_cached_generation_equals_full_recompute():
    m = O.Model(S.make_blob(HP, std=0.3, ln_jitter=0.2), ctype=np.float64)
    rng = np.random.default_rng(1)
    prompts = rng.integers(4, m.V, size=(3, 5))
    trace = []
    toks, logp, st = O.generate(m, prompts, 6, max_len=12, trace=trace)
    for t, rec in enumerate(trace):
        for r in range(3):
            prefix = st.tokens[r, : 5 + t]
            np.testing.assert_allclose(rec["logits"][r], O.gpt_forward_full(m, prefix), rtol=0, atol=1e-10)
    assert toks.shape == (3, 6) and (logp < 0).all()


def test_sampling_rule():
    rng = np.random.default_rng(2)
    logits = rng.standard_normal(50).astype(np.float32)
    k = 6
    top = sorted(range(50), key=lambda v: (-logits[v], v))[:k]
    p = np.exp(logits[top].astype(np.float64)); p /= p.sum()
    cum = np.cumsum(p)
    # the draw u lands in the interval [cum[j-1], cum[j]) of exactly one of the k tokens
    for u in np.linspace(0.001, 0.999, 333):
        tok, lp, gap = O.sample_topk(logits, k, np.float32(u))
        j = int(np.searchsorted(cum, u, side="right"))
        if min(abs(cum - u)) > 1e-5:
            assert tok == top[j] and abs(lp - np.log(p[j])) < 1e-5
    # k = 1 is greedy; ties go to the lower token id
    assert O.sample_topk(logits, 1, np.float32(0.7))[0] == int(np.argmax(logits))
    tie = np.zeros(9, np.float32)
    assert O.sample_topk(tie, 3, np.float32(0.0))[0] == 0 and O.sample_topk(tie, 3, np.float32(0.99))[0] == 2
    # empirical frequencies follow the k-way softmax
    counts = np.zeros(50)
    for i in range(4000):
        counts[O.sample_topk(logits, k, O.sample_uniform(5, i, 3))[0]] += 1
    assert counts[[v for v in range(50) if v not in top]].sum() == 0
    assert np.abs(counts[top] / 4000 - p).max() < 0.03


def test_nucleus_inside_topk():
    """top-p on top of top-k: hand-made probabilities 0.5, 0.25, 0.125, 0.0625, ... among the k candidates."""
    # logits = log2-spaced: softmax over the 5 kept ones is (16, 8, 4, 2, 1) / 31
    logits = np.full(12, -50.0, np.float32)
    kept = [7, 2, 9, 4, 11]
    for r, v in enumerate(kept):
        logits[v] = np.float32(np.log(2.0) * (4 - r))
    w = np.array([16, 8, 4, 2, 1], np.float64) / 31
    # p = 0.75: 16/31 = 0.516 < 0.75 <= 24/31 = 0.774 -> the first two survive, renormalised to 2/3 and 1/3
    seen = {}
    for u in np.linspace(0.0005, 0.9995, 400):
        tok, lp, gap = O.sample_topk(logits, 5, np.float32(u), 0.75)
        seen.setdefault(tok, []).append((u, lp))
    assert set(seen) == {7, 2}
    assert max(u for u, _ in seen[7]) < 2 / 3 < min(u for u, _ in seen[2])
    assert abs(seen[7][0][1] - np.log(2 / 3)) < 1e-6 and abs(seen[2][0][1] - np.log(1 / 3)) < 1e-6
    # p below the first probability: greedy; p = 1: plain top-k; p just above a prefix mass keeps one more
    assert all(O.sample_topk(logits, 5, np.float32(u), 0.3)[0] == 7 for u in (0.0, 0.5, 0.999))
    for u in (0.01, 0.6, 0.8, 0.93, 0.99):
        assert O.sample_topk(logits, 5, np.float32(u), 1.0)[:2] == O.sample_topk(logits, 5, np.float32(u))[:2]
    assert O.sample_topk(logits, 5, np.float32(0.999), float(w[:3].sum()) + 1e-4)[0] == 4     # four survive
    assert O.sample_topk(logits, 5, np.float32(0.999), float(w[:3].sum()) - 1e-4)[0] == 9     # three survive
    # the cut is reported as a near-decision when p sits on a prefix mass
    assert O.sample_topk(logits, 5, np.float32(0.1), float(w[:2].sum()) + 1e-7)[2] < 1e-5
    # k larger than 8 (the paper's sampling runs use 32): survivors and frequencies
    rng = np.random.default_rng(4)
    lg = (rng.standard_normal(500) * 2).astype(np.float32)
    order = sorted(range(500), key=lambda v: (-lg[v], v))[:32]
    pr = np.exp(lg[order].astype(np.float64)); pr /= pr.sum()
    n = int(np.searchsorted(np.cumsum(pr), 0.9)) + 1
    counts = np.zeros(500)
    for i in range(6000):
        counts[O.sample_topk(lg, 32, O.sample_uniform(9, i, 1), 0.9)[0]] += 1
    assert counts[[v for v in range(500) if v not in order[:n]]].sum() == 0
    assert np.abs(counts[order[:n]] / 6000 - pr[:n] / pr[:n].sum()).max() < 0.03


def test_blob_header_carries_nucleus_mass():
    import lsq_synth as S
    hp = S.HParams(arch=1, n_enc=0, n_dec=1, d_model=16, n_heads=1, d_ffn=16, vocab=20, max_pos=8, act=1, norm=1,
                   sample_topk=32, sample_topp=0.75)
    m = O.Model(S.make_blob(hp))
    assert m.sample_topk == 32 and abs(m.sample_topp - 0.75) < 1e-7
    assert O.Model(S.make_blob(S.HParams(arch=1, n_enc=0, n_dec=1, d_model=16, n_heads=1, d_ffn=16, vocab=20, max_pos=8,
                                         act=1, norm=1, sample_topk=4))).sample_topp == 1.0
