"""Pins for the oracle's sampling decoding of an encoder-decoder model (paper sec. 3.4): top-1
sampling is greedy search, a hand-worked step, the rule restated with explicit loops, the draw's
frequencies against the k-way softmax, the uniform number tied to the sentence's place in the batch,
EOS and cap bookkeeping."""
import dataclasses

import numpy as np

import lsq_synth as S
from oracle import lsq_oracle as O

HP = S.HParams(n_enc=1, n_dec=2, d_model=32, n_heads=4, d_ffn=48, vocab=23, max_pos=32, cap_extra=5, sample_topk=4,
               seed=2024)


def _model(hp, lens, std=0.4, max_len=12):
    w = S.custom(hp, lens, beam=1, max_len=max_len, std=std)
    return w, O.Model(w.blob(std=std, ln_jitter=0.2), ctype=np.float64)


def test_top1_sampling_is_greedy_search():
    hp = dataclasses.replace(HP, sample_topk=1)
    w, m = _model(hp, [3, 7, 5])
    (ids_s, len_s, sc_s), st_s = O.translate_sample(m, w.src_ids, w.src_lens, w.max_len)
    (ids_b, len_b, sc_b), st_b = O.translate(m, w.src_ids, w.src_lens, 1, w.max_len)
    assert np.array_equal(ids_s, ids_b) and np.array_equal(len_s, len_b)
    assert np.all(sc_s == 0)            # the only kept candidate has probability 1 among the kept
    assert np.all(sc_b < 0)


def test_hand_worked_draws():
    """V = 5, top-3 of logits log[.1,.4,.2,.25,.05] is tokens (1, 3, 2) with weights .4, .25, .2 ->
    cumulative shares 8/17, 13/17, 1: u = .3 -> token 1, u = .5 -> token 3, u = .8 -> token 2;
    with nucleus mass .5 of the kept three the prefix (1, 3) stays (8/17 < .5 <= 13/17): shares 8/13, 1."""
    logits = np.log(np.array([.1, .4, .2, .25, .05])) + 3.0
    for u, tok, p in ((.3, 1, .4 / .85), (.5, 3, .25 / .85), (.8, 2, .2 / .85), (0.0, 1, .4 / .85)):
        t, lp, _ = O.sample_topk(logits, 3, np.float32(u))
        assert t == tok and abs(lp - np.log(p)) < 1e-6
    for u, tok, p in ((.3, 1, .4 / .65), (.7, 3, .25 / .65), (.99, 3, .25 / .65)):
        t, lp, _ = O.sample_topk(logits, 3, np.float32(u), p=0.5)
        assert t == tok and abs(lp - np.log(p)) < 1e-6


def test_step_rule_restated_with_loops():
    w, m = _model(HP, [4, 2, 6])
    trace = []
    (ids, lens, scores), st = O.translate_sample(m, w.src_ids, w.src_lens, w.max_len, trace=trace)
    B = w.batch
    caps = np.minimum(w.src_lens + HP.cap_extra, w.max_len)
    done = [False] * B
    hist = [[] for _ in range(B)]
    total = [0.0] * B
    for t, step in enumerate(trace):
        for b in range(B):
            if done[b]:
                continue
            row = step["logits"][b]
            ranked = sorted(range(m.V), key=lambda v: (-row[v], v))[:HP.sample_topk]
            weights = [float(np.exp(np.float32(row[v]) - np.float32(row[ranked[0]]))) for v in ranked]
            u = float(O.sample_uniform(HP.seed, t, b))
            acc, pick = 0.0, ranked[-1]
            for v, wgt in zip(ranked, weights):
                acc += wgt
                if acc > u * sum(weights):
                    pick = v
                    break
            hist[b].append(pick)
            total[b] += np.log(weights[ranked.index(pick)] / sum(weights))
            done[b] = pick == m.eos or len(hist[b]) >= caps[b]
        assert step["active"] == sum(not x for x in done)
    assert all(done)
    for b in range(B):
        assert lens[b, 0] == len(hist[b]) and ids[b, 0, :lens[b, 0]].tolist() == hist[b]
        assert (ids[b, 0, lens[b, 0]:] == m.pad).all()
        np.testing.assert_allclose(scores[b, 0], total[b] / len(hist[b]) ** HP.length_penalty, rtol=1e-5, atol=1e-6)


def test_first_draw_frequencies_follow_the_kept_softmax():
    w, m = _model(HP, [5])
    _, cross = O.encode(m, w.src_ids, w.src_lens)
    st = O.DecodeState(m, w.src_lens, 1, w.max_len)
    logits = O.decoder_logits_cached(m, st, cross)[0]
    ranked = np.lexsort((np.arange(m.V), -logits))[:HP.sample_topk]
    p = np.exp(logits[ranked] - logits[ranked[0]])
    p /= p.sum()
    n = 3000
    counts = np.zeros(m.V)
    for seed in range(n):
        tok, _, _ = O.sample_topk(logits, HP.sample_topk, O.sample_uniform(seed, 0, 0))
        counts[tok] += 1
    assert counts.sum() == counts[ranked].sum()            # nothing outside the k best is ever drawn
    # 4.5 standard deviations of a binomial share
    assert np.all(np.abs(counts[ranked] / n - p) < 4.5 * np.sqrt(p * (1 - p) / n) + 1e-3)


def test_uniform_number_belongs_to_the_place_in_the_batch():
    w, m = _model(HP, [4, 6, 3])
    (ids3, len3, sc3), _ = O.translate_sample(m, w.src_ids, w.src_lens, w.max_len)
    # the first sentence alone draws the same numbers (step, 0) and sees the same logits
    (ids1, len1, sc1), _ = O.translate_sample(m, w.src_ids[:1], w.src_lens[:1], w.max_len)
    assert np.array_equal(ids1[0], ids3[0]) and len1[0, 0] == len3[0, 0]
    np.testing.assert_allclose(sc1[0], sc3[0], rtol=1e-9)
    # the third sentence moved to the front draws other numbers: its first token follows (0, 0), not (0, 2)
    order = [2, 0, 1]
    trace = []
    O.translate_sample(m, w.src_ids[order], w.src_lens[order], w.max_len, trace=trace, max_steps=1)
    row = trace[0]["logits"][0]
    tok_front, _, _ = O.sample_topk(row, HP.sample_topk, O.sample_uniform(HP.seed, 0, 0))
    assert trace[0]["token"][0, 0] == tok_front


def test_eos_and_cap_finish_sentences():
    hp = dataclasses.replace(HP, vocab=6, sample_topk=5, cap_extra=3)     # EOS is drawn often
    ended_by_eos = ended_by_cap = 0
    for seed in range(12):
        w, m = _model(dataclasses.replace(hp, seed=seed), [2, 5, 3, 4], std=0.6, max_len=7)
        trace = []
        (ids, lens, scores), st = O.translate_sample(m, w.src_ids, w.src_lens, w.max_len, trace=trace)
        caps = np.minimum(w.src_lens + 3, 7)
        assert st.finished.all()
        for b in range(w.batch):
            n = lens[b, 0]
            seq = ids[b, 0, :n]
            assert 1 <= n <= caps[b] and m.eos not in seq[:-1]
            assert seq[-1] == m.eos or n == caps[b]
            ended_by_eos += seq[-1] == m.eos
            ended_by_cap += seq[-1] != m.eos
            # once finished, a sentence's length and score no longer move
            fin_at = next(t for t, s in enumerate(trace) if s["finished"][b])
            for s in trace[fin_at:]:
                assert s["len"][b] == n and s["score"][b, 0] == trace[fin_at]["score"][b, 0]
    assert ended_by_eos > 5 and ended_by_cap > 5
