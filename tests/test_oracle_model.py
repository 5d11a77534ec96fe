"""Pins for the oracle's model and search: torch.nn library layers loaded with
the same weights, the K/V-cache invariant, greedy and exhaustive search."""
import itertools

import numpy as np
import pytest
import torch

import lsq_synth as S
from oracle import lsq_oracle as O

torch.set_grad_enabled(False)


def _t(a):
    return torch.from_numpy(np.ascontiguousarray(a)).double()


def _load_mha(mha, Win, b_in, Wo, bo):
    mha.in_proj_weight.copy_(_t(Win.T))
    mha.in_proj_bias.copy_(_t(b_in))
    mha.out_proj.weight.copy_(_t(Wo.T))
    mha.out_proj.bias.copy_(_t(bo))


def _torch_encoder_layer(m, L):
    t = torch.nn.TransformerEncoderLayer(m.d, m.H, m.F, dropout=0.0, activation="relu",
                                         layer_norm_eps=float(m.eps), batch_first=True,
                                         norm_first=False).double().eval()
    _load_mha(t.self_attn, L["Wqkv"], L["bqkv"], L["Wo"], L["bo"])
    t.linear1.weight.copy_(_t(L["W1"].T)); t.linear1.bias.copy_(_t(L["b1"]))
    t.linear2.weight.copy_(_t(L["W2"].T)); t.linear2.bias.copy_(_t(L["b2"]))
    t.norm1.weight.copy_(_t(L["ln1_g"])); t.norm1.bias.copy_(_t(L["ln1_b"]))
    t.norm2.weight.copy_(_t(L["ln2_g"])); t.norm2.bias.copy_(_t(L["ln2_b"]))
    return t


def _torch_decoder_layer(m, L):
    t = torch.nn.TransformerDecoderLayer(m.d, m.H, m.F, dropout=0.0, activation="relu",
                                         layer_norm_eps=float(m.eps), batch_first=True,
                                         norm_first=False).double().eval()
    _load_mha(t.self_attn, L["Wqkv"], L["bqkv"], L["Wo"], L["bo"])
    _load_mha(t.multihead_attn, np.concatenate([L["Wq_c"], L["Wkv_c"]], 1),
              np.concatenate([L["bq_c"], L["bkv_c"]]), L["Wo_c"], L["bo_c"])
    t.linear1.weight.copy_(_t(L["W1"].T)); t.linear1.bias.copy_(_t(L["b1"]))
    t.linear2.weight.copy_(_t(L["W2"].T)); t.linear2.bias.copy_(_t(L["b2"]))
    t.norm1.weight.copy_(_t(L["ln1_g"])); t.norm1.bias.copy_(_t(L["ln1_b"]))
    t.norm2.weight.copy_(_t(L["ln2_g"])); t.norm2.bias.copy_(_t(L["ln2_b"]))
    t.norm3.weight.copy_(_t(L["ln3_g"])); t.norm3.bias.copy_(_t(L["ln3_b"]))
    return t


HP = S.HParams(n_enc=2, n_dec=2, d_model=32, n_heads=4, d_ffn=48, vocab=50, max_pos=32)


@pytest.fixture(scope="module")
def model64():
    # std 0.3 so that attention is far from uniform; jittered LayerNorm gains and shifts
    return O.Model(S.make_blob(HP, std=0.3, ln_jitter=0.3), ctype=np.float64)


def test_encoder_stack_matches_torch_with_padding(model64):
    m = model64
    rng = np.random.default_rng(0)
    lens = [5, 9, 1]
    ids = rng.integers(4, m.V, size=(3, 9))
    memory, _ = O.encode(m, ids, lens)
    layers = [_torch_encoder_layer(m, L) for L in m.enc]
    x = torch.zeros(3, 9, m.d, dtype=torch.float64)
    for b, s in enumerate(lens):
        x[b, :s] = _t(O.embed(m, ids[b, :s], np.arange(s)))
    pad = torch.tensor([[j >= s for j in range(9)] for s in lens])
    for t in layers:
        x = t(x, src_key_padding_mask=pad)
    for b, s in enumerate(lens):
        np.testing.assert_allclose(memory[b], x[b, :s].numpy(), rtol=0, atol=1e-11)


def test_decoder_stack_matches_torch(model64):
    m = model64
    rng = np.random.default_rng(1)
    s, n = 7, 6
    src = rng.integers(4, m.V, size=(1, s))
    prefix = np.concatenate([[m.bos], rng.integers(4, m.V, size=n - 1)])
    memory, cross = O.encode(m, src, [s])
    got = O.decoder_logits_full(m, prefix, cross[0])
    y = _t(O.embed(m, prefix, np.arange(n)))[None]
    mem = _t(memory[0])[None]
    causal = torch.triu(torch.ones(n, n, dtype=torch.bool), 1)
    for L in m.dec:
        y = _torch_decoder_layer(m, L)(y, mem, tgt_mask=causal)
    ref = (y[0, -1] @ _t(m.E).T).numpy()
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-10)


def test_embedding_scale_and_position():
    hp = S.HParams(d_model=16, n_heads=2, d_ffn=16, vocab=9, max_pos=8)
    m = O.Model(S.make_blob(hp, std=1.0), ctype=np.float64)
    x = O.embed(m, np.array([4, 4]), np.array([0, 3]))
    # position 0 adds [0,1,0,1,...]; the table row is scaled by sqrt(d) = 4
    np.testing.assert_allclose(x[0] - np.tile([0.0, 1.0], 8), 4.0 * m.E[4], atol=1e-15)
    np.testing.assert_allclose(x[1] - x[0] + np.tile([0.0, 1.0], 8),
                               O.positional_encoding(3, 16, np.float64)[0], atol=1e-12)


def test_padding_and_batch_invariance():
    w = S.workload("tiny")
    m = O.Model(w.blob(std=0.3))
    ids2 = w.src_ids.copy()
    ids2[0, 5:] = 777                        # beyond the first sentence's length
    (a_ids, a_len, a_sc), _ = O.translate(m, w.src_ids, w.src_lens, w.beam, w.max_len)
    (b_ids, b_len, b_sc), _ = O.translate(m, ids2, w.src_lens, w.beam, w.max_len)
    assert np.array_equal(a_ids, b_ids) and np.array_equal(a_sc, b_sc)
    (c_ids, c_len, c_sc), _ = O.translate(m, w.src_ids[1:], w.src_lens[1:], w.beam, w.max_len)
    assert np.array_equal(c_ids[0], a_ids[1]) and np.array_equal(c_len[0], a_len[1])
    np.testing.assert_allclose(c_sc[0], a_sc[1], rtol=1e-5)


@pytest.mark.parametrize("dtype", [0, 1])
def test_cached_decode_equals_full_recompute(dtype):
    hp = S.HParams(n_enc=1, n_dec=2, d_model=32, n_heads=4, d_ffn=64, vocab=40, max_pos=32, dtype=dtype)
    w = S.custom(hp, [3, 6], beam=3, max_len=7, std=0.3)
    m = O.Model(w.blob(std=0.3, ln_jitter=0.2), ctype=np.float64)
    memory, cross = O.encode(m, w.src_ids, w.src_lens)
    st = O.DecodeState(m, w.src_lens, w.beam, w.max_len)
    checked = 0
    for _ in range(w.max_len):
        logits = O.decoder_logits_cached(m, st, cross)
        for r in range(st.B * st.k):
            if st.finished[r]:
                continue
            prefix = st.tokens[r, : st.len[r] + 1]
            full = O.decoder_logits_full(m, prefix, cross[r // st.k])
            if dtype == 0:
                np.testing.assert_allclose(logits[r], full, rtol=0, atol=1e-11)
            else:   # fp16 storage: identical up to rare one-ulp flips of stored halves
                np.testing.assert_allclose(logits[r], full, rtol=0, atol=4e-3)
            checked += 1
        tok, par, sc, _ = O.beam_select(m, st, logits)
        if O.beam_advance(m, st, tok, par, sc) == 0:
            break
    assert checked > 20


def _sequence_logprob(m, cross_b, seq):
    """Sum of log-probabilities of seq (without BOS) under the full-recompute path."""
    total = 0.0
    for i, tok in enumerate(seq):
        prefix = [m.bos] + list(seq[:i])
        lp = O.log_softmax(O.decoder_logits_full(m, np.array(prefix), cross_b).astype(np.float64))
        total += lp[tok]
    return total


def test_wide_beam_equals_exhaustive_search():
    V, cap = 4, 3
    hp = S.HParams(n_enc=1, n_dec=1, d_model=16, n_heads=2, d_ffn=32, vocab=V, max_pos=16, cap_extra=0)
    # ids must lie in [4, V): impossible for V = 4, so build the source by hand
    blob = S.make_blob(hp, std=0.8)
    m = O.Model(blob, ctype=np.float64)
    src = np.array([[3, 0, 3]], np.int32)
    lens = [cap]                                  # cap = min(3 + 0, max_len) = 3
    k = V ** cap
    (ids, ln, sc), st = O.translate(m, src, lens, k, max_len=cap)
    _, cross = O.encode(m, src, lens)
    # enumerate every complete hypothesis: ends with EOS at length <= cap, or has length cap
    best, best_seq, n_hyp = -np.inf, None, 0
    for n in range(1, cap + 1):
        for seq in itertools.product(range(V), repeat=n):
            if m.eos in seq[:-1]:
                continue
            if seq[-1] != m.eos and n < cap:
                continue
            n_hyp += 1
            val = _sequence_logprob(m, cross[0], seq) / (n ** m.alpha)
            if val > best:
                best, best_seq = val, seq
    assert n_hyp <= k
    assert tuple(ids[0, 0, : ln[0, 0]]) == best_seq
    assert abs(sc[0, 0] - best) < 1e-9
    # the beam held every complete hypothesis: all final scores are finite and distinct
    assert np.isfinite(sc[0, :n_hyp]).all() and (sc[0, n_hyp:] == -np.inf).all()


def test_beam_one_is_greedy_and_scores_behave():
    w = S.workload("tiny")
    m = O.Model(w.blob(std=0.3), ctype=np.float64)
    trace = []
    (ids, ln, sc), st = O.translate(m, w.src_ids, w.src_lens, 1, w.max_len, trace=trace)
    _, cross = O.encode(m, w.src_ids, w.src_lens)
    for b in range(w.batch):
        prefix = [m.bos]
        for i in range(ln[b, 0]):
            nxt = int(np.argmax(O.decoder_logits_full(m, np.array(prefix), cross[b])))
            assert nxt == ids[b, 0, i]
            prefix.append(nxt)
    # beam 4: best raw score never increases; finished hypotheses keep their score
    trace = []
    O.translate(m, w.src_ids, w.src_lens, 4, w.max_len, trace=trace)
    for a, b_ in zip(trace[:-1], trace[1:]):
        assert (b_["score"][:, 0] <= a["score"][:, 0] + 1e-12).all()
        for b in range(w.batch):
            for j in range(4):
                p = b_["parent"][b, j]
                if a["finished"][b * 4 + p]:
                    assert b_["score"][b, j] == a["score"][b, p]
                    assert b_["len"][b * 4 + j] == a["len"][b * 4 + p]


def test_eos_and_cap_finish_hypotheses():
    # bias the model towards EOS through the embedding of EOS being large: some hypotheses end early
    hp = S.HParams(n_enc=1, n_dec=1, d_model=16, n_heads=2, d_ffn=32, vocab=12, max_pos=32, cap_extra=2)
    w = S.custom(hp, [2, 4], beam=3, max_len=10, std=0.5)
    m = O.Model(w.blob(std=0.5), ctype=np.float64)
    (ids, ln, sc), st = O.translate(m, w.src_ids, w.src_lens, w.beam, w.max_len)
    caps = np.minimum(w.src_lens + 2, 10)
    for b in range(w.batch):
        for i in range(w.beam):
            n = ln[b, i]
            assert 1 <= n <= caps[b]
            seq = ids[b, i, :n]
            assert m.eos not in seq[:-1]
            assert seq[-1] == m.eos or n == caps[b]
            assert (ids[b, i, n:] == m.pad).all()
        assert (np.diff(sc[b]) <= 0).all()
    assert st.finished.all()


def test_fp16_storage_rounds_and_stays_close_to_wide():
    hp = S.HParams(n_enc=2, n_dec=2, d_model=64, n_heads=4, d_ffn=128, vocab=300, max_pos=32, dtype=1)
    w = S.custom(hp, [4, 9], beam=4, max_len=6)
    blob = w.blob()
    m16, m32 = O.Model(blob), O.Model(blob, storage="wide")
    assert m16.round16 and not m32.round16
    assert np.array_equal(m16.E, m32.E)                    # both read the same fp16-rounded weights
    _, c16 = O.encode(m16, w.src_ids, w.src_lens)
    _, c32 = O.encode(m32, w.src_ids, w.src_lens)
    s16 = O.DecodeState(m16, w.src_lens, w.beam, w.max_len)
    s32 = O.DecodeState(m32, w.src_lens, w.beam, w.max_len)
    l16 = O.decoder_logits_cached(m16, s16, c16)
    l32 = O.decoder_logits_cached(m32, s32, c32)
    # stored tensors are fp16-representable, logits are not rounded
    assert np.array_equal(s16.Kc[0][:, 0], s16.Kc[0][:, 0].astype(np.float16).astype(np.float32))
    assert not np.array_equal(l16, l16.astype(np.float16).astype(np.float32))
    rms = np.sqrt((l32 ** 2).mean(-1, keepdims=True))
    err = np.abs(l16 - l32) / (np.abs(l32) + rms)
    assert err.max() < 2e-2
    assert err.max() > 0


def test_beam_step_hand_worked_example():
    """Two steps worked by hand: V = 4 (EOS = 2), beam 2, one sentence.
    Step 1: p = [.1,.2,.3,.4] from the only live beam -> keep token 3 (log .4) and EOS (log .3).
    Step 2: live beam offers four candidates at log(.4*.25) = log .1; the finished one offers
    (log .3, EOS).  Kept: the finished hypothesis first, then token 0 (lowest flat index of the tie)."""
    hp = S.HParams(n_enc=1, n_dec=1, d_model=8, n_heads=2, d_ffn=8, vocab=4, max_pos=8)
    m = O.Model(S.make_blob(hp), ctype=np.float64)
    st = O.DecodeState(m, [3], 2, 5)
    l1 = np.log(np.array([[.1, .2, .3, .4], [.7, .1, .1, .1]])) + 5.0      # shift must not matter
    tok, par, sc, mar = O.beam_select(m, st, l1)
    assert tok.tolist() == [[3, 2]] and par.tolist() == [[0, 0]]
    np.testing.assert_allclose(sc[0], np.log([.4, .3]), atol=1e-12)
    np.testing.assert_allclose(mar[0], min(np.log(.4 / .3), np.log(.3 / .2)), atol=1e-12)
    assert O.beam_advance(m, st, tok, par, sc) == 1
    assert st.finished.tolist() == [False, True] and st.len.tolist() == [1, 1]
    l2 = np.log(np.array([[.25, .25, .25, .25], [.97, .01, .01, .01]]))
    tok, par, sc, mar = O.beam_select(m, st, l2)
    assert par.tolist() == [[1, 0]] and tok.tolist() == [[2, 0]]
    np.testing.assert_allclose(sc[0], np.log([.3, .1]), atol=1e-12)
    assert mar[0] == 0.0                                    # tie with the first dropped candidate
    assert O.beam_advance(m, st, tok, par, sc) == 1
    assert st.finished.tolist() == [True, False] and st.len.tolist() == [1, 2]
    assert st.tokens[0, :2].tolist() == [m.bos, 2] and st.tokens[1, :3].tolist() == [m.bos, 3, 0]
    (ids, ln, fs), = [O.finalize(m, st)]
    # final = score / len: log(.3)/1 = -1.204 vs log(.1)/2 = -1.151 -> the longer one ranks first
    assert ln.tolist() == [[2, 1]] and ids[0, 0, :2].tolist() == [3, 0] and ids[0, 1, :1].tolist() == [2]
    np.testing.assert_allclose(fs[0], [np.log(.1) / 2, np.log(.3)], atol=1e-12)


def test_length_penalty_hand_worked():
    """score / len^alpha with alpha != 1, worked by hand: raw scores -6, -4, -8, -inf at lengths 4, 1, 16, 0.
    alpha = 0.5: -6/2 = -3, -4/1 = -4, -8/4 = -2, -inf  -> order 2, 0, 1, 3.
    alpha = 2:   -6/16 = -0.375, -4, -8/256 = -0.03125 -> order 2, 0, 1, 3;  alpha = 0: raw order 1, 0, 2, 3.
    A dropped exponent (alpha taken as 1: -1.5, -4, -0.5) gives other values; an inverted one (multiplying
    by len^alpha) reverses the order."""
    for alpha, want_order, want in ((0.5, [2, 0, 1, 3], [-2.0, -3.0, -4.0, -np.inf]),
                                    (2.0, [2, 0, 1, 3], [-0.03125, -0.375, -4.0, -np.inf]),
                                    (0.0, [1, 0, 2, 3], [-4.0, -6.0, -8.0, -np.inf])):
        hp = S.HParams(n_enc=1, n_dec=1, d_model=16, n_heads=2, d_ffn=32, vocab=12, max_pos=32, length_penalty=alpha)
        m = O.Model(S.make_blob(hp), ctype=np.float64)
        assert m.alpha == np.float32(alpha)
        st = O.DecodeState(m, [3], 4, 20)
        st.score[0] = [-6.0, -4.0, -8.0, -np.inf]
        st.len[:] = [4, 1, 16, 0]
        for r, n in enumerate(st.len):
            st.tokens[r, 1:n + 1] = 4 + r
        ids, ln, fs = O.finalize(m, st)
        assert list(ln[0]) == [int(st.len[j]) for j in want_order]
        np.testing.assert_allclose(fs[0], want, rtol=1e-12)
        for i, j in enumerate(want_order):
            assert (ids[0, i, :ln[0, i]] == 4 + j).all() and (ids[0, i, ln[0, i]:] == m.pad).all()


def test_length_penalty_changes_the_winner_of_a_translation():
    """Whole translations with alpha = 0.4 and alpha = 1.6 on the same weights: the search itself (raw
    cumulative log-probabilities) is the same, the final ranking is score / len^alpha recomputed by hand."""
    hp0 = S.HParams(n_enc=1, n_dec=1, d_model=16, n_heads=2, d_ffn=32, vocab=12, max_pos=32, cap_extra=3)
    w = S.custom(hp0, [2, 5, 3], beam=4, max_len=9, std=0.6)
    finals = {}
    for alpha in (0.4, 1.6):
        hp = S.HParams(**{**hp0.__dict__, "length_penalty": alpha})
        m = O.Model(S.make_blob(hp, std=0.6), ctype=np.float64)
        (ids, ln, fs), st = O.translate(m, w.src_ids, w.src_lens, 4, 9)
        finals[alpha] = (st.score.copy(), st.len.copy())
        want = st.score / st.len.reshape(3, 4).astype(np.float64) ** np.float64(np.float32(alpha))
        for b in range(3):
            np.testing.assert_allclose(fs[b], np.sort(want[b])[::-1], rtol=1e-12)
    assert np.array_equal(finals[0.4][0], finals[1.6][0]) and np.array_equal(finals[0.4][1], finals[1.6][1])
