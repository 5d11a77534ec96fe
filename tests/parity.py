"""Shared helpers for the GPU parity tests: lock-step comparison of the HIP library with the
CPU oracle on the same seeded workload."""
import numpy as np

from oracle import lsq_oracle as O

MARGIN = 1e-3        # token ids are compared only while the oracle's beam-score margins exceed this
TOL_F16 = 2e-2       # logits, fp16 storage, against the unrounded fp32 oracle
TOL_F32 = 1e-4       # logits on the fp32 path


def logit_error(got, ref):
    """max |g - r| / (|r| + rms(r over its row)): relative error that stays defined near zero."""
    ref = np.asarray(ref, np.float64)
    rms = np.sqrt((ref ** 2).mean(-1, keepdims=True))
    return float((np.abs(np.asarray(got, np.float64) - ref) / (np.abs(ref) + rms)).max())


def oracle_model(blob):
    """The oracle for parity runs: float16 models round where the model stores (float32 arithmetic
    in between, as the library's accumulators); float32 models are computed in float64, because
    numpy's own float32 forward pass is up to 2e-4 away from the float64 one on the larger test
    weights, ten times further than the library."""
    m = O.Model(blob)
    return m if m.round16 else O.Model(blob, ctype=np.float64)


def score_slack(round16, got, ref, live):
    """How far one step may move a hypothesis score away from the oracle's: a score adds
    logit - logsumexp(logits), which moves by at most twice the largest logit deviation.  float16
    models: the measured 4e-3; float32 models: 2e-5 or that bound at this step, whichever is larger."""
    if round16:
        return 4e-3
    dev = float(np.abs(np.asarray(got, np.float64)[live] - np.asarray(ref, np.float64)[live]).max()) if np.any(live) else 0.0
    return max(2e-5, 2.0 * dev)


class Float32Shadow:
    """For float32 models: the same oracle once more in numpy float32, following the same decisions.
    Its distance from the float64 oracle says how well conditioned a step is: some rows of some
    random models lose three or four digits in ANY float32 evaluation (the library's and numpy's
    deviations appear in the same rows; on a given row either can be the larger by a factor of four,
    while kernel by kernel the library is as close to float64 as numpy's float32 is), so the bound
    on the library's logits is TOL_F32 or eight times what plain float32 arithmetic deviates at that
    step, whichever is larger."""

    def __init__(self, blob, w, k=None, groups=1, gpt=False):
        self.m = O.Model(blob)
        self.gpt = gpt
        if gpt:
            self.st = O.GptState(self.m, w.src_ids[:, :int(w.src_lens[0])], w.max_len)
            O.gpt_prefill(self.m, self.st)
        else:
            _, self.cross = O.encode(self.m, w.src_ids, w.src_lens)
            self.st = O.DecodeState(self.m, w.src_lens, k, w.max_len, groups)

    def tolerance(self, ref64, live):
        """Call once per step, before advance()."""
        ref32 = O.gpt_step_logits(self.m, self.st) if self.gpt else O.decoder_logits_cached(self.m, self.st, self.cross)
        if not np.any(live):
            return TOL_F32
        return max(TOL_F32, 8.0 * logit_error(ref32[live], ref64[live]))

    def advance(self, *sel):
        if self.gpt:
            O.gpt_advance(self.m, self.st, *sel)
        else:
            tok, par, sc = sel
            O.beam_advance(self.m, self.st, tok, par, np.asarray(sc, np.float32))


def lockstep(lsq, eng, blob, w, max_steps=None, check_wide=True, verbose=False):
    """Runs the library and the oracle side by side, one decode step at a time.

    Every step, for every sentence:
      * logits against the oracle that rounds where the model stores (tight) and, while both
        sides have made identical decisions, against the unrounded fp32 oracle (the stated
        tolerance);
      * the kept (beam, token) pairs.  Where the oracle's smallest gap between competing
        candidates exceeds MARGIN plus twice the measured deviation of the library's candidate
        scores from the oracle's ("strict" decisions) the two orders cannot differ and the pairs
        must be identical.  Otherwise several selections are correct and the library's is
        checked for validity instead: every kept pair's oracle score must reach the oracle's
        k-th best within that band, kept pairs must be in oracle order within the band, and no
        dropped pair may beat a kept one by more than the band.  The oracle then continues from
        the library's (valid) selection with its own scores, so that every later step of every
        sentence is still compared;
      * token histories, lengths, finished flags (exact) and hypothesis scores (tolerance).
    The deviation is measured over the 32 best candidates of every live row on either side
    (candidate = hypothesis score before the step + log-softmax of the row's logits, evaluated
    here in float64 from each side's own numbers).  Returns a summary dict."""
    m = oracle_model(blob)                    # rounds at storage points for fp16 blobs
    mw = O.Model(blob, storage="wide") if (check_wide and m.round16) else None
    B, k, T, V = w.batch, w.beam, w.max_len, m.V
    M = B * k
    eng.encode(w.src_ids, w.src_lens)
    _, cross = O.encode(m, w.src_ids, w.src_lens)
    st = O.DecodeState(m, w.src_lens, k, T)
    if mw is not None:
        _, cross_w = O.encode(mw, w.src_ids, w.src_lens)
        st_w = O.DecodeState(mw, w.src_lens, k, T)
    wide_in_sync = mw is not None
    steps = strict_n = band_n = 0
    worst_tight = worst_wide = worst_dev = 0.0
    tol_tight = 1e-2 if m.round16 else TOL_F32
    shadow = None if m.round16 else Float32Shadow(blob, w, k)
    slack = 0.0                                       # hypothesis scores are sums over the steps: so is their tolerance
    while True:
        ref_logits = O.decoder_logits_cached(m, st, cross)
        prev_ref = st.score.reshape(-1).copy()
        prev_gpu = eng.debug(lsq.DBG.SCORE, (M,))
        old_fin, old_len = st.finished.copy(), st.len.copy()
        active_gpu = eng.decode_step()
        got_logits = eng.debug(lsq.DBG.LOGITS, (M, V))
        live = ~old_fin
        if shadow is not None:
            tol_tight = shadow.tolerance(ref_logits, live)
        slack += score_slack(m.round16, got_logits, ref_logits, live)
        if live.any():
            e = logit_error(got_logits[live], ref_logits[live])
            worst_tight = max(worst_tight, e)
            assert e <= tol_tight, f"step {steps}: logits differ from the storage-rounding oracle by {e}"
        if wide_in_sync:
            wl = O.decoder_logits_cached(mw, st_w, cross_w)
            rows = live & ~st_w.finished
            if rows.any():
                e = logit_error(got_logits[rows], wl[rows])
                worst_wide = max(worst_wide, e)
                assert e <= TOL_F16, f"step {steps}: fp16 logits differ from the fp32 oracle by {e}"
        tok, par, sc, margin = O.beam_select(m, st, ref_logits)
        if wide_in_sync:
            tw, pw, sw, _ = O.beam_select(mw, st_w, wl)
        g_tokens = eng.debug(lsq.DBG.TOKENS, (M, T + 1), np.int32)
        g_len = eng.debug(lsq.DBG.LEN, (M,), np.int32)
        g_fin = eng.debug(lsq.DBG.FINISHED, (M,), np.int32)
        g_par = eng.debug(lsq.DBG.PARENT, (M,), np.int32)
        g_score = eng.debug(lsq.DBG.SCORE, (M,))
        logp = O.log_softmax(np.asarray(ref_logits, m.ctype))
        for b in range(B):
            base = b * k
            if old_fin[base:base + k].all():
                # nothing left to decide, and the library no longer touches the sentence: the hypotheses stay
                # where they are.  (Selecting again would re-sort them by the oracle's scores, which undoes
                # the library's order wherever an earlier step took it over within the band.)
                par[b], tok[b], sc[b] = np.arange(k), m.eos, st.score[b]
                continue                       # the state checks below still apply
            # measured deviation of candidate scores
            cdev = 0.0
            for j in range(k):
                r = base + j
                if not np.isfinite(prev_ref[r]):
                    assert not np.isfinite(prev_gpu[r])
                    continue
                if old_fin[r]:
                    cdev = max(cdev, abs(float(prev_gpu[r]) - float(prev_ref[r])))
                    continue
                c_ref = float(prev_ref[r]) + O.log_softmax(ref_logits[r].astype(np.float64))
                c_gpu = float(prev_gpu[r]) + O.log_softmax(got_logits[r].astype(np.float64))
                top = np.union1d(np.argpartition(-c_ref, 32)[:32], np.argpartition(-c_gpu, 32)[:32]) \
                    if V > 33 else np.arange(V)
                cdev = max(cdev, float(np.abs(c_gpu[top] - c_ref[top]).max()))
            worst_dev = max(worst_dev, cdev)
            band = MARGIN + 2 * cdev
            # the library's selection for this sentence
            gp = g_par[base:base + k].astype(np.int64)
            assert ((gp >= 0) & (gp < k)).all(), f"step {steps} sentence {b}: parent out of range"
            gt = np.empty(k, np.int64)
            for i in range(k):
                pr = base + gp[i]
                gt[i] = m.eos if old_fin[pr] else g_tokens[base + i, old_len[pr] + 1]
            if margin[b] > band:
                strict_n += 1
                assert np.array_equal(gp, par[b]) and np.array_equal(gt, tok[b]), \
                    f"step {steps} sentence {b}: kept pairs differ although the margin {margin[b]:.2e} " \
                    f"exceeds {band:.2e}: parents {gp} vs {par[b]}, tokens {gt} vs {tok[b]}"
            else:
                band_n += 1
                def ref_score(j, v):
                    r = base + j
                    return st.score[b, j] if old_fin[r] else st.score[b, j] + logp[r, v]
                kept = [(int(gp[i]), int(gt[i])) for i in range(k)]
                assert len(set(kept)) == k, f"step {steps} sentence {b}: a pair was kept twice"
                ks = np.array([ref_score(j, v) for j, v in kept], np.float64)
                kth = float(sc[b, k - 1])
                if np.isfinite(kth):
                    assert (ks >= kth - band).all(), f"step {steps} sentence {b}: kept pair below the band: {ks} vs {kth}"
                    assert (np.diff(ks) <= band).all(), f"step {steps} sentence {b}: kept pairs out of order: {ks}"
                    # best dropped pair by the oracle's order
                    best_drop = -np.inf
                    for j in range(k):
                        r = base + j
                        if not np.isfinite(prev_ref[r]):
                            continue
                        if old_fin[r]:
                            if (j, m.eos) not in kept:
                                best_drop = max(best_drop, float(st.score[b, j]))
                            continue
                        for v in np.argpartition(-logp[r], min(k, V - 1))[:k + 1]:
                            if (j, int(v)) not in kept:
                                best_drop = max(best_drop, float(st.score[b, j] + logp[r, v]))
                    assert best_drop <= ks.min() + band, \
                        f"step {steps} sentence {b}: dropped pair {best_drop} beats a kept one {ks.min()}"
                par[b], tok[b] = gp, gt
                sc[b] = np.array([ref_score(j, v) for j, v in kept], m.ctype)
        active_ref = O.beam_advance(m, st, tok, par, sc)
        if shadow is not None:
            shadow.advance(tok, par, sc)
        if wide_in_sync:     # the unrounded oracle is followed only while it decides as the library did
            O.beam_advance(mw, st_w, tw, pw, sw)
            wide_in_sync = bool(np.array_equal(tw, tok) and np.array_equal(pw, par))
        assert np.array_equal(g_len, st.len), f"step {steps}: lengths"
        assert np.array_equal(g_fin != 0, st.finished), f"step {steps}: finished flags"
        for r in range(M):
            n = st.len[r]
            assert np.array_equal(g_tokens[r, : n + 1], st.tokens[r, : n + 1]), f"step {steps} row {r}: tokens"
        fin = np.isfinite(st.score.reshape(-1))
        assert np.array_equal(np.isfinite(g_score), fin), f"step {steps}: -inf scores"
        np.testing.assert_allclose(g_score[fin], st.score.reshape(-1)[fin], rtol=2e-5,
                                   atol=1e-4 + slack)
        assert active_gpu == active_ref, f"step {steps}: active {active_gpu} vs {active_ref}"
        steps += 1
        if verbose:
            print(f"step {steps}: active {active_gpu}, strict {strict_n} band {band_n}, "
                  f"tight {worst_tight:.2e} wide {worst_wide:.2e} dev {worst_dev:.2e}", flush=True)
        if active_gpu == 0 or (max_steps is not None and steps >= max_steps):
            break
    return dict(steps=steps, batch=B, worst_tight=worst_tight, worst_wide=worst_wide, worst_dev=worst_dev,
                strict=strict_n, band=band_n, state=st)


def lockstep_gpt(lsq, eng, blob, w, n_steps=None, verbose=False):
    """Decoder-only model with top-k sampling, library and oracle side by side.

    Every step: logits against the oracle (same tolerances as lockstep), then the sampled token of
    every row.  The uniform numbers are identical on both sides (same Philox counter), so the
    tokens must be identical wherever the decision is clear: the k-th and (k+1)-th logit differ,
    and the draw is away from every cumulative-probability boundary, by more than the measured
    logit deviation allows.  Elsewhere the library's token must be one of the oracle's k
    candidates, and the oracle continues from it.  Returns a summary dict."""
    m = oracle_model(blob)
    B, T, V, k, topp = w.batch, w.max_len, m.V, m.sample_topk, m.sample_topp
    n_new = m.cap_extra if n_steps is None else n_steps
    eng.encode(w.src_ids, w.src_lens)
    P = int(w.src_lens[0])
    st = O.GptState(m, w.src_ids[:, :P], T)
    O.gpt_prefill(m, st)
    tol = 1e-2 if m.round16 else TOL_F32
    shadow = None if m.round16 else Float32Shadow(blob, w, gpt=True)
    worst = slack = 0.0
    strict = loose = 0
    for step in range(n_new):
        ref = O.gpt_step_logits(m, st)
        if shadow is not None:
            tol = shadow.tolerance(ref, np.ones(B, bool))
        active = eng.decode_step()
        got = eng.debug(lsq.DBG.LOGITS, (B, V))
        slack += score_slack(m.round16, got, ref, np.ones(B, bool))
        e = logit_error(got, ref)
        worst = max(worst, e)
        assert e <= tol, f"step {step}: logits differ from the oracle by {e}"
        g_tok = eng.debug(lsq.DBG.TOKENS, (B, T + 1), np.int32)[:, st.pos + 1]
        g_ci = eng.debug(lsq.DBG.CAND_IDX, (B, k), np.int32)
        g_cl = eng.debug(lsq.DBG.CAND_SCORE, (B, k))
        toks, lps = [], []
        for r in range(B):
            u = O.sample_uniform(m.seed, st.t, r)
            # selection alone, on the library's own logits: its k candidates are exactly the k largest
            # (logit descending, token ascending), and its token is the oracle's draw from them
            mine = np.lexsort((np.arange(V), -got[r]))[:k]
            assert np.array_equal(g_ci[r], mine) and np.array_equal(g_cl[r], got[r][mine]), f"step {step} row {r}: candidates"
            tok_own, lp_own, gap_own = O.sample_topk(got[r], k, u, topp)
            assert g_tok[r] == tok_own or gap_own < 1e-5, f"step {step} row {r}: token {g_tok[r]}, expected {tok_own}"
            tok, lp, gap = O.sample_topk(ref[r], k, u, topp)
            dev = float(np.abs(got[r] - ref[r]).max())
            if gap > 4 * dev + 1e-5:
                strict += 1
                assert g_tok[r] == tok, f"step {step} row {r}: sampled {g_tok[r]}, oracle {tok} (gap {gap:.2e})"
            else:
                loose += 1
                order = np.lexsort((np.arange(V), -ref[r]))[:k + 1]
                assert g_tok[r] in order, f"step {step} row {r}: sampled token is not among the oracle's candidates"
                # a near-decision (rank swap, draw at an edge, nucleus cut at its threshold): the oracle
                # follows the library, taking the oracle's own rule applied to the library's logits for
                # the token and for its log-probability (the survivors' mass depends on where the cut fell)
                tok, lp = int(g_tok[r]), lp_own
            toks.append(tok)
            lps.append(lp)
        O.gpt_advance(m, st, toks, lps)
        if shadow is not None:
            shadow.advance(toks, lps)
        g_logp = eng.debug(lsq.DBG.SCORE, (B,))
        np.testing.assert_allclose(g_logp, st.logp, rtol=2e-5, atol=1e-4 + slack)
        assert active == (B if step + 1 < m.cap_extra else 0), f"step {step}: active {active}"
        if verbose:
            print(f"step {step + 1}: strict {strict} loose {loose} worst logit error {worst:.2e}", flush=True)
    return dict(steps=n_new, strict=strict, loose=loose, worst=worst, state=st)


def lockstep_sample(lsq, eng, blob, w, max_steps=None):
    """Encoder-decoder model with sampling decoding, library and oracle side by side: as
    lockstep_gpt for the draws (candidates and token exact on the library's own logits; against the
    oracle's logits identical wherever the decision is clear, else among its candidates and the
    oracle follows), plus the bookkeeping of translation: a finished sentence draws nothing, EOS or
    the cap finishes one, lengths and flags exact, the count of unfinished sentences.
    For float32 models the oracle runs in float64 (oracle_model)."""
    m = oracle_model(blob)
    B, T, V, k, topp = w.batch, w.max_len, m.V, m.sample_topk, m.sample_topp
    eng.encode(w.src_ids, w.src_lens)
    _, cross = O.encode(m, w.src_ids, w.src_lens)
    st = O.DecodeState(m, w.src_lens, 1, T)
    tol = 1e-2 if m.round16 else TOL_F32
    shadow = None if m.round16 else Float32Shadow(blob, w, 1)
    worst = slack = 0.0
    steps = strict = loose = 0
    while True:
        ref = O.decoder_logits_cached(m, st, cross)
        old_fin = st.finished.copy()
        active = eng.decode_step()
        got = eng.debug(lsq.DBG.LOGITS, (B, V))
        live = ~old_fin
        if shadow is not None:
            tol = shadow.tolerance(ref, live)
        slack += score_slack(m.round16, got, ref, live)
        if live.any():
            e = logit_error(got[live], ref[live])
            worst = max(worst, e)
            assert e <= tol, f"step {steps}: logits differ from the oracle by {e}"
        g_tokens = eng.debug(lsq.DBG.TOKENS, (B, T + 1), np.int32)
        g_ci = eng.debug(lsq.DBG.CAND_IDX, (B, k), np.int32)
        g_cl = eng.debug(lsq.DBG.CAND_SCORE, (B, k))
        token = np.full((B, 1), m.eos, np.int32)
        score = st.score.copy()
        for b in range(B):
            if old_fin[b]:
                continue
            u = O.sample_uniform(m.seed, st.t, b)
            g_tok = int(g_tokens[b, st.len[b] + 1])
            mine = np.lexsort((np.arange(V), -got[b]))[:k]
            assert np.array_equal(g_ci[b], mine) and np.array_equal(g_cl[b], got[b][mine]), f"step {steps} sentence {b}: candidates"
            tok_own, lp_own, gap_own = O.sample_topk(got[b], k, u, topp)
            assert g_tok == tok_own or gap_own < 1e-5, f"step {steps} sentence {b}: token {g_tok}, expected {tok_own}"
            tok, lp, gap = O.sample_topk(ref[b], k, u, topp)
            dev = float(np.abs(got[b] - ref[b]).max())
            if gap > 4 * dev + 1e-5:
                strict += 1
                assert g_tok == tok, f"step {steps} sentence {b}: sampled {g_tok}, oracle {tok} (gap {gap:.2e})"
            else:
                loose += 1
                assert g_tok in np.lexsort((np.arange(V), -ref[b]))[:k + 1], f"step {steps} sentence {b}: not a candidate"
                tok, lp = g_tok, lp_own
            token[b, 0] = tok
            score[b, 0] = m.ctype(st.score[b, 0] + m.ctype(lp))
        active_ref = O.beam_advance(m, st, token, np.zeros((B, 1), np.int32), score)
        if shadow is not None:
            shadow.advance(token, np.zeros((B, 1), np.int32), score)
        steps += 1
        assert active == active_ref, f"step {steps}: active {active}, oracle {active_ref}"
        g_tokens = eng.debug(lsq.DBG.TOKENS, (B, T + 1), np.int32)
        assert np.array_equal(eng.debug(lsq.DBG.LEN, (B,), np.int32), st.len), f"step {steps}: lengths"
        assert np.array_equal(eng.debug(lsq.DBG.FINISHED, (B,), np.int32) != 0, st.finished), f"step {steps}: finished flags"
        for b in range(B):
            assert np.array_equal(g_tokens[b, :st.len[b] + 1], st.tokens[b, :st.len[b] + 1]), f"step {steps}: history of sentence {b}"
        np.testing.assert_allclose(eng.debug(lsq.DBG.SCORE, (B,)), st.score[:, 0], rtol=2e-5,
                                   atol=1e-4 + slack)
        if active_ref == 0 or (max_steps is not None and steps >= max_steps):
            break
    return dict(steps=steps, strict=strict, loose=loose, worst=worst, state=st)


def lockstep_diverse(lsq, eng, blob, w, groups, strength, max_steps=None):
    """Diverse beam search, library and oracle side by side.  Per step: logits, then group by group
    (in the order the groups choose) the kept (beam, token) pairs of every sentence.  The oracle's
    selection for a group is computed with the token counts of the earlier groups as the LIBRARY
    chose them (already checked), so one near-tie does not derail the later groups.  Where the
    oracle's smallest gap between ranking values exceeds MARGIN plus twice the measured deviation of
    the library's candidate scores the pairs must be identical; otherwise every kept pair's ranking
    value must reach the oracle's last kept one within that band, in order within the band, and the
    oracle continues from the library's selection.  Histories, lengths, flags exact; scores within
    tolerance."""
    lsq.lsq_set_diversity(groups, strength)
    m = oracle_model(blob)
    B, k, T, V = w.batch, w.beam, w.max_len, m.V
    kg, M = k // groups, B * k
    try:
        eng.encode(w.src_ids, w.src_lens)
    finally:
        lsq.lsq_set_diversity(1, 0.0)                 # the setting was taken by encode; later encodes are plain again
    _, cross = O.encode(m, w.src_ids, w.src_lens)
    st = O.DecodeState(m, w.src_lens, k, T, groups)
    tol = 1e-2 if m.round16 else TOL_F32
    slack = 0.0
    shadow = None if m.round16 else Float32Shadow(blob, w, k, groups)
    steps = strict = band_n = 0
    while True:
        ref_logits = O.decoder_logits_cached(m, st, cross)
        prev_ref = st.score.reshape(-1).copy()
        prev_gpu = eng.debug(lsq.DBG.SCORE, (M,))
        old_fin, old_len = st.finished.copy(), st.len.copy()
        active_gpu = eng.decode_step()
        got_logits = eng.debug(lsq.DBG.LOGITS, (M, V))
        live = ~old_fin
        if shadow is not None:
            tol = shadow.tolerance(ref_logits, live)
        slack += score_slack(m.round16, got_logits, ref_logits, live)
        if live.any():
            e = logit_error(got_logits[live], ref_logits[live])
            assert e <= tol, f"step {steps}: logits differ from the oracle by {e}"
        g_tokens = eng.debug(lsq.DBG.TOKENS, (M, T + 1), np.int32)
        g_len = eng.debug(lsq.DBG.LEN, (M,), np.int32)
        g_fin = eng.debug(lsq.DBG.FINISHED, (M,), np.int32)
        g_par = eng.debug(lsq.DBG.PARENT, (M,), np.int32)
        g_score = eng.debug(lsq.DBG.SCORE, (M,))
        logp = O.log_softmax(np.asarray(ref_logits, m.ctype))
        tok = np.zeros((B, k), np.int32); par = np.zeros((B, k), np.int32); sc = np.zeros((B, k), m.ctype)
        for b in range(B):
            base = b * k
            if old_fin[base:base + k].all():
                tok[b], par[b], sc[b] = m.eos, np.arange(k), st.score[b]
                continue
            cdev = 0.0
            for j in range(k):
                r = base + j
                if not np.isfinite(prev_ref[r]) or old_fin[r]:
                    continue
                c_ref = float(prev_ref[r]) + O.log_softmax(ref_logits[r].astype(np.float64))
                c_gpu = float(prev_gpu[r]) + O.log_softmax(got_logits[r].astype(np.float64))
                top = np.argpartition(-c_ref, min(32, V - 1))[:32] if V > 33 else np.arange(V)
                cdev = max(cdev, float(np.abs(c_gpu[top] - c_ref[top]).max()))
            band = MARGIN + 2 * cdev
            counts = np.zeros(V, np.int64)
            for g in range(groups):
                rows = slice(base + g * kg, base + (g + 1) * kg)
                t_o, p_o, s_o, sel_o, margin = O.group_select(m, st, logp, b, g, strength, counts)
                gp = g_par[rows].astype(np.int64)
                assert ((gp >= g * kg) & (gp < (g + 1) * kg)).all(), f"step {steps} sentence {b} group {g}: parent outside the group"
                gt = np.array([m.eos if old_fin[base + gp[i]] else g_tokens[base + g * kg + i, old_len[base + gp[i]] + 1]
                               for i in range(kg)], np.int64)

                def rank_value(j, v):
                    r = base + j
                    if old_fin[r]:
                        return float(st.score[b, j])
                    return float(st.score[b, j] + logp[r, v]) - float(strength) * float(counts[v])

                def plain_value(j, v):
                    r = base + j
                    return st.score[b, j] if old_fin[r] else m.ctype(st.score[b, j] + logp[r, v])
                if margin > band:
                    strict += 1
                    assert np.array_equal(gp, p_o) and np.array_equal(gt, t_o), \
                        f"step {steps} sentence {b} group {g}: kept pairs differ although the margin {margin:.2e} exceeds " \
                        f"{band:.2e}: parents {gp} vs {p_o}, tokens {gt} vs {t_o}"
                else:
                    band_n += 1
                    kept = [(int(gp[i]), int(gt[i])) for i in range(kg)]
                    assert len(set(kept)) == kg, f"step {steps} sentence {b} group {g}: a pair was kept twice"
                    ks = np.array([rank_value(j, v) for j, v in kept])
                    kth = float(sel_o[kg - 1])
                    if np.isfinite(kth):
                        assert (ks >= kth - band).all(), f"step {steps} sentence {b} group {g}: kept pair below the band"
                        assert (np.diff(ks) <= band).all(), f"step {steps} sentence {b} group {g}: kept pairs out of order"
                    t_o, p_o = gt.astype(np.int32), gp.astype(np.int32)
                    s_o = np.array([plain_value(j, v) for j, v in kept], m.ctype)
                tok[b, g * kg:(g + 1) * kg], par[b, g * kg:(g + 1) * kg], sc[b, g * kg:(g + 1) * kg] = t_o, p_o, s_o
                for i in range(kg):
                    if not old_fin[base + p_o[i]] and np.isfinite(s_o[i]):
                        counts[t_o[i]] += 1
        active_ref = O.beam_advance(m, st, tok, par, sc)
        if shadow is not None:
            shadow.advance(tok, par, sc)
        assert np.array_equal(g_len, st.len), f"step {steps}: lengths"
        assert np.array_equal(g_fin != 0, st.finished), f"step {steps}: finished flags"
        for r in range(M):
            n = st.len[r]
            assert np.array_equal(g_tokens[r, : n + 1], st.tokens[r, : n + 1]), f"step {steps} row {r}: tokens"
        fin = np.isfinite(st.score.reshape(-1))
        assert np.array_equal(np.isfinite(g_score), fin), f"step {steps}: -inf scores"
        np.testing.assert_allclose(g_score[fin], st.score.reshape(-1)[fin], rtol=2e-5, atol=1e-4 + slack)
        assert active_gpu == active_ref, f"step {steps}: active {active_gpu} vs {active_ref}"
        steps += 1
        if active_gpu == 0 or (max_steps is not None and steps >= max_steps):
            break
    return dict(steps=steps, strict=strict, band=band_n, state=st)
