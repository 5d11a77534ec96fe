"""Pins for the oracle's diverse beam search (Hamming diversity between groups): special cases that
reduce to plain beam search, a hand-worked step, and a brute-force restatement of the rule."""
import numpy as np

import lsq_synth as S
from oracle import lsq_oracle as O


def _model(vocab=9, seed=3, dtype=0):
    hp = S.HParams(n_enc=1, n_dec=1, d_model=16, n_heads=2, d_ffn=24, vocab=vocab, max_pos=16, cap_extra=5, seed=seed,
                   dtype=dtype)
    return O.Model(S.make_blob(hp, std=0.6), np.float64)


def test_one_group_is_plain_beam_search():
    m = _model()
    src = np.array([[4, 5, 6, 0], [7, 8, 4, 5]], np.int32)
    lens = np.array([3, 4], np.int32)
    st = O.DecodeState(m, lens, 4, 8)
    _, cross = O.encode(m, src, lens)
    for _ in range(4):
        logits = O.decoder_logits_cached(m, st, cross)
        a = O.beam_select(m, st, logits)
        b = O.beam_select_diverse(m, st, logits, 0.7)          # the strength has nothing to act on
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
        O.beam_advance(m, st, *a[:3])


def test_zero_strength_gives_independent_identical_groups():
    m = _model()
    src = np.array([[4, 5, 6, 7, 8]], np.int32)
    lens = np.array([5], np.int32)
    (ids2, lens2, sc2), _ = O.translate(m, src, lens, 2, 9)                       # beam 2
    (ids6, lens6, sc6), st = O.translate(m, src, lens, 6, 9, groups=3, strength=0.0)
    # three groups of two, no interaction: each group is the beam-2 search; best-first order interleaves them
    for i in range(2):
        for g in range(3):
            assert np.array_equal(ids6[0, 3 * i + g], ids2[0, i]) and lens6[0, 3 * i + g] == lens2[0, i]
    np.testing.assert_allclose(sc6[0].reshape(2, 3), np.repeat(sc2[0][:, None], 3, axis=1), rtol=0, atol=1e-12)


def test_hand_worked_step():
    """Two groups of one hypothesis each, V = 4: the second group avoids the first group's token when
    the penalty outweighs the log-probability gap."""
    m = _model(vocab=4)
    st = O.DecodeState(m, np.array([2], np.int32), 2, 6, groups=2)
    p = np.array([0.5, 0.3, 0.15, 0.05])
    logits = np.log(np.stack([p, p]))                          # both hypotheses see the same distribution
    assert np.array_equal(st.score, [[0.0, 0.0]])
    tok, par, sc, margin = O.beam_select_diverse(m, st, logits, 0.4)
    # group 0 takes token 0 (log 0.5); group 1 ranks token 0 at log 0.5 - 0.4 = -1.093 < log 0.3 = -1.204? no:
    # -1.093 > -1.204, so it still takes token 0
    assert tok.tolist() == [[0, 0]] and par.tolist() == [[0, 1]]
    np.testing.assert_allclose(sc, [[np.log(0.5), np.log(0.5)]])
    tok, par, sc, margin = O.beam_select_diverse(m, st, logits, 0.6)
    # now -0.693 - 0.6 = -1.293 < -1.204: token 1 wins; its stored score is the plain log-probability
    assert tok.tolist() == [[0, 1]] and par.tolist() == [[0, 1]]
    np.testing.assert_allclose(sc, [[np.log(0.5), np.log(0.3)]])
    assert abs(margin[0] - ((np.log(0.3)) - (np.log(0.5) - 0.6))) < 1e-12      # group 1: kept vs the first dropped


def test_rule_restated_by_brute_force():
    rng = np.random.default_rng(5)
    m = _model(vocab=7, seed=9)
    B, k, G, V, lam = 3, 6, 3, 7, 0.35
    kg = k // G
    st = O.DecodeState(m, np.array([2, 3, 2], np.int32), k, 9, groups=G)
    st.score = rng.standard_normal((B, k)) * 2
    st.score[1, 3] = -np.inf                                   # a dead hypothesis
    st.finished[[4, 13]] = True                                # finished ones: (0,4) and (2,1)
    logits = rng.standard_normal((B * k, V))
    logp = O.log_softmax(logits)
    tok, par, sc, _ = O.beam_select_diverse(m, st, logits, lam)
    for b in range(B):
        chosen = []                                            # tokens taken so far at this step
        for g in range(G):
            cands = []
            for j in range(g * kg, (g + 1) * kg):
                r = b * k + j
                if st.finished[r]:
                    cands.append((-st.score[b, j], j * V + m.eos, m.eos, j, st.score[b, j], True))
                else:
                    for v in range(V):
                        plain = st.score[b, j] + logp[r, v]
                        cands.append((-(plain - lam * chosen.count(v)), j * V + v, v, j, plain, False))
            cands.sort(key=lambda c: (c[0], c[1]))
            for i, c in enumerate(cands[:kg]):
                assert tok[b, g * kg + i] == c[2] and par[b, g * kg + i] == c[3]
                assert sc[b, g * kg + i] == c[4] or (np.isinf(sc[b, g * kg + i]) and np.isinf(c[4]))
                if not c[5] and np.isfinite(c[4]):
                    chosen.append(c[2])
