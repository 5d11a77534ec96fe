"""Shared helpers for the GPU parity tests: lock-step comparison of the HIP library with the
CPU oracle on the same seeded workload.

Which oracle judges what.  The judge of every stated tolerance is the oracle that rounds nothing
(`storage='wide'`: the blob's weights as they are, every activation in the arithmetic type, float64
unless a full-size run says float32): the library's logits must stay within TOL_F16 / TOL_F32 of
it at every step of every run, and the kept (beam, token) pairs are judged by its scores.  It knows
nothing of where the kernels round.  For float16 models a second oracle that rounds to float16
where the library stores (`storage='blob'`, the kernel-mirroring mode) runs beside it as a tighter
regression detector for the logits only (TOL_MIRROR); it decides nothing.

Near-ties.  With float16 storage two correct evaluations differ by a few 1e-3 in a logit, so a
decision whose margin is smaller than that has several correct outcomes.  Where the judge's margin
exceeds MARGIN + 2 * cdev ("strict") the kept pairs must be identical; inside that band the
library's selection must be valid (see lockstep) and the oracles continue from it, so every later
step of every sentence is still compared against both.  cdev is measured, but it cannot grow
unseen: every one of its parts is asserted against a fixed bound first (unit(TAU_BAND) for one step's
candidate log-probabilities, CDEV_CAP for the whole), and every test pins the share of strict
decisions it measured.
"""
import dataclasses
import struct

import numpy as np

from oracle import lsq_oracle as O

MARGIN = 1e-3        # token ids are compared strictly while the judge's beam-score margins exceed this (plus the band)
TOL_F16 = 2e-2       # logits, fp16 storage, against the unrounded oracle
TOL_F32 = 1e-4       # logits on the fp32 path ...
TOL_F32_CEIL = 1e-3  # ... bounds beyond this are counted (models on which float32 itself loses three digits)
TOL_MIRROR = 1e-2    # fp16 logits against the oracle that rounds where the library stores
# Fixed bounds on what may enter the near-tie band, in units the library has no hand in.  A logit tolerance
# tau (relative to |r| + rms of the row, logit_error) moves a log-probability by at most
# 2 tau (max |r| + rms) =: unit(tau) of that row.  One step's deviation of a candidate's log-probability
# (library vs judge, 32 best candidates of a row on either side) must stay below unit(TAU_BAND) --
# TAU_BAND = 1e-3 for float16 models (measured: at most 0.3 of it), well inside the stated 2e-2; for float32 models the run's
# conditioning-aware bound (Float32Shadow, from oracle runs alone) -- and the whole
# deviation of a sentence's candidate scores, once the drift its hypotheses share is taken out, below
# CDEV_UNITS such units (hypotheses of a sentence share all but their last few steps).
TAU_BAND_F16 = 1e-3
CDEV_UNITS = 3.0


def logit_error(got, ref):
    """max |g - r| / (|r| + rms(r over its row)): relative error that stays defined near zero."""
    ref = np.asarray(ref, np.float64)
    rms = np.sqrt((ref ** 2).mean(-1, keepdims=True))
    return float((np.abs(np.asarray(got, np.float64) - ref) / (np.abs(ref) + rms)).max())


def blob_is_f16(blob):
    return struct.unpack_from("<i", blob, 52)[0] == 1


def judge_model(blob, ctype=np.float64):
    """The oracle that judges: nothing rounded between operations.  float32 models: always float64."""
    if blob_is_f16(blob):
        return O.Model(blob, ctype=ctype, storage="wide")
    return O.Model(blob, ctype=np.float64)


def oracle_model(blob):
    """Judge for the sampling / decoder-only / diverse comparisons below: float16 models round where the
    model stores (float32 arithmetic in between, as the library's accumulators; the kernel-mirroring mode);
    float32 models are computed in float64, because numpy's own float32 forward pass is up to 2e-4 away from
    the float64 one on the larger test weights, ten times further than the library."""
    m = O.Model(blob)
    return m if m.round16 else O.Model(blob, ctype=np.float64)


def score_slack(round16, got, ref, live):
    """How far one step may move a hypothesis score away from the oracle's: a score adds
    logit - logsumexp(logits), which moves by at most twice the largest logit deviation measured at
    this step (both model types; at least 2e-5 for the float32 sums themselves)."""
    dev = float(np.abs(np.asarray(got, np.float64)[live] - np.asarray(ref, np.float64)[live]).max()) if np.any(live) else 0.0
    return max(2e-5, 2.0 * dev)


F32_FACTOR = 4.0     # float32 models: the library may be this many times further from float64 than numpy float32 is, over a run


class Float32Shadow:
    """For float32 models: how well conditioned the model is, from oracle runs alone.  Some random models
    lose three or four digits in ANY float32 evaluation of some rows at some steps (deep LayerNorm / softmax
    chains with large activations); the library's and numpy's deviations from float64 have the same size over
    a translation but land on different steps and rows (measured on ill-conditioned draws: worst library error
    1.2 to 3.0 times numpy's worst over the run, while step by step the ratio swings between 0.1 and 18).  So
    the bound is per run, not per step:
        s_run = the largest distance of the oracle in numpy float32 from the oracle in float64 over the whole
                translation -- a pass of the two oracles alone before the library runs (both following the
                float64 oracle's decisions), kept up to date with the steps of the lock-step run itself (both
                following the library's decisions);
        bound on the library's logits at every step: max(TOL_F32, F32_FACTOR * s_run).
    Wherever plain float32 arithmetic stays within 2.5e-5 of float64 the bound is the stated 1e-4.
    `over` counts the steps whose bound exceeded TOL_F32, `over_ceiling` those beyond TOL_F32_CEIL,
    `worst_bound` is the largest bound used, `worst_ratio` = the library's worst error of the run over
    max(s_run, TOL_F32 / F32_FACTOR)."""

    def __init__(self, blob, w, k=None, groups=1, gpt=False):
        self.m = O.Model(blob)
        self.gpt = gpt
        self.over = self.over_ceiling = 0
        self.worst_bound = TOL_F32
        self.worst_ratio = 0.0
        self.last = 0.0
        self.e_max = 0.0
        self.s_run = self._conditioning(blob, w, k, groups)
        if gpt:
            self.st = O.GptState(self.m, w.src_ids[:, :int(w.src_lens[0])], w.max_len)
            O.gpt_prefill(self.m, self.st)
        else:
            _, self.cross = O.encode(self.m, w.src_ids, w.src_lens)
            self.st = O.DecodeState(self.m, w.src_lens, k, w.max_len, groups)

    def _conditioning(self, blob, w, k, groups):
        """The two oracles side by side over the whole translation, decisions taken by the float64 one."""
        m64, m32 = O.Model(blob, ctype=np.float64), self.m
        worst = 0.0
        if self.gpt:
            P = int(w.src_lens[0])
            a, b = O.GptState(m64, w.src_ids[:, :P], w.max_len), O.GptState(m32, w.src_ids[:, :P], w.max_len)
            O.gpt_prefill(m64, a)
            O.gpt_prefill(m32, b)
            for _ in range(m64.cap_extra):
                l64, l32 = O.gpt_step_logits(m64, a), O.gpt_step_logits(m32, b)
                worst = max(worst, logit_error(l32, l64))
                picks = [O.sample_topk(l64[r], m64.sample_topk, O.sample_uniform(m64.seed, a.t, r), m64.sample_topp)
                         for r in range(a.B)]
                O.gpt_advance(m64, a, [q[0] for q in picks], [q[1] for q in picks])
                O.gpt_advance(m32, b, [q[0] for q in picks], [q[1] for q in picks])
            return worst
        _, c64 = O.encode(m64, w.src_ids, w.src_lens)
        _, c32 = O.encode(m32, w.src_ids, w.src_lens)
        a, b = O.DecodeState(m64, w.src_lens, k, w.max_len, groups), O.DecodeState(m32, w.src_lens, k, w.max_len, groups)
        while True:
            l64, l32 = O.decoder_logits_cached(m64, a, c64), O.decoder_logits_cached(m32, b, c32)
            live = ~a.finished.reshape(-1)
            if live.any():
                worst = max(worst, logit_error(l32[live], l64[live]))
            if m64.sample_topk >= 1:
                tok, par, sc, _ = O.sample_select(m64, a, l64)
            elif groups > 1:
                tok, par, sc, _ = O.beam_select_diverse(m64, a, l64, 0.0)
            else:
                tok, par, sc, _ = O.beam_select(m64, a, l64)
            active = O.beam_advance(m64, a, tok, par, sc)
            O.beam_advance(m32, b, tok, par, np.asarray(sc, np.float32))
            if active == 0:
                return worst

    def tolerance(self, ref64, live):
        """Call once per step, before advance()."""
        ref32 = O.gpt_step_logits(self.m, self.st) if self.gpt else O.decoder_logits_cached(self.m, self.st, self.cross)
        if np.any(live):
            self.last = logit_error(ref32[live], ref64[live])
            self.s_run = max(self.s_run, self.last)
        else:
            self.last = 0.0
        tol = max(TOL_F32, F32_FACTOR * self.s_run)
        if tol > TOL_F32:
            self.over += 1
            self.worst_bound = max(self.worst_bound, tol)
        if tol > TOL_F32_CEIL:
            self.over_ceiling += 1
        return tol

    def note(self, e):
        self.e_max = max(self.e_max, e)
        self.worst_ratio = self.e_max / max(self.s_run, TOL_F32 / F32_FACTOR)

    def advance(self, *sel):
        if self.gpt:
            O.gpt_advance(self.m, self.st, *sel)
        else:
            tok, par, sc = sel
            O.beam_advance(self.m, self.st, tok, par, np.asarray(sc, np.float32))


def _f32_stats(shadow):
    if shadow is None:
        return dict(f32_steps_over=0, f32_steps_over_ceiling=0, f32_worst_bound=0.0, f32_worst_ratio=0.0)
    return dict(f32_steps_over=shadow.over, f32_steps_over_ceiling=shadow.over_ceiling, f32_worst_bound=shadow.worst_bound,
                f32_worst_ratio=shadow.worst_ratio)


def _follow_scores(model, st, logp, tok, par, old_fin):
    """Scores of the hypotheses an oracle gets when it adopts the selection (tok, par) [B,k]: the
    parent's score, plus the token's log-probability unless the parent had finished."""
    B, k = st.B, st.k
    sc = np.empty((B, k), model.ctype)
    for b in range(B):
        for i in range(k):
            j = int(par[b, i])
            r = b * k + j
            sc[b, i] = st.score[b, j] if old_fin[r] else model.ctype(st.score[b, j] + logp[r, int(tok[b, i])])
    return sc


def lockstep(lsq, eng, blob, w, max_steps=None, sentences=None, mirror=True, judge_ctype=np.float64, verbose=False,
             check_wide=None):
    """Runs the library and the oracle side by side, one decode step at a time.

    sentences: None compares every sentence; a list of indices into the batch compares those only
    (the library still translates the whole batch: sentences do not interact, so the oracle can follow
    any subset of a full-size batch through all of its steps at a fraction of the cost).

    Every step, for every compared sentence:
      * logits of every unfinished row against the judge (TOL_F16; float32 models TOL_F32, see
        Float32Shadow) and, float16 models with mirror=True, against the kernel-mirroring oracle
        (TOL_MIRROR);
      * the kept (beam, token) pairs.  cdev = the largest deviation of the library's candidate scores
        (hypothesis score before the step + log-softmax of its own logits, in float64) from the judge's
        over the 32 best candidates of every row on either side, after subtracting the mean drift of the
        sentence's hypotheses (a shift common to all candidates of a sentence changes no decision).
        Where the judge's smallest gap between competing candidates exceeds MARGIN + 2 cdev the pairs
        must be identical ("strict").  Otherwise the library's selection must be valid: every kept
        pair's judge score reaches the judge's k-th best within the band, kept pairs are in judge order
        within the band, no dropped pair beats a kept one by more than the band; the oracles then
        continue from the library's selection with their own scores.  One step's part of cdev must stay
        below SDEV_CAP and cdev below CDEV_CAP, fixed numbers, before it may widen anything;
      * the library's new scores exactly (fp32 rounding) from its own previous scores and logits, and
        against the judge's within the deviations measured along each hypothesis' own history;
      * token histories, lengths, finished flags (exact), the count of unfinished sentences.
    Returns a summary dict."""
    f16 = blob_is_f16(blob)
    mj = judge_model(blob, judge_ctype)
    if check_wide is False:                     # older call sites: "no second oracle"
        mirror = False
    mm = O.Model(blob) if (f16 and mirror) else None
    k, T, V = w.beam, w.max_len, mj.V
    sel = np.arange(w.batch) if sentences is None else np.asarray(sentences, np.int64)
    ws = dataclasses.replace(w, batch=len(sel), src_lens=w.src_lens[sel], src_ids=w.src_ids[sel])
    B = len(sel)
    M_all, Ms = w.batch * k, B * k
    rows = (sel[:, None] * k + np.arange(k)[None, :]).reshape(-1)
    eng.encode(w.src_ids, w.src_lens)
    _, cross = O.encode(mj, ws.src_ids, ws.src_lens)
    st = O.DecodeState(mj, ws.src_lens, k, T)
    if mm is not None:
        _, cross_m = O.encode(mm, ws.src_ids, ws.src_lens)
        st_m = O.DecodeState(mm, ws.src_lens, k, T)
    shadow = None if f16 else Float32Shadow(blob, ws, k)
    steps = strict_n = band_n = 0
    worst_logit = worst_mirror = worst_sdev = worst_cdev = worst_own = 0.0
    bound = np.zeros(Ms)                                     # per hypothesis: deviations measured along its history
    tol = TOL_F16 if f16 else TOL_F32
    while True:
        ref_logits = O.decoder_logits_cached(mj, st, cross)
        prev_ref = st.score.reshape(-1).astype(np.float64)
        prev_gpu = eng.debug(lsq.DBG.SCORE, (M_all,))[rows].astype(np.float64)
        old_fin, old_len = st.finished.copy(), st.len.copy()
        active_gpu = eng.decode_step()
        got_logits = eng.debug(lsq.DBG.LOGITS, (M_all, V))[rows]
        live = ~old_fin
        if shadow is not None:
            tol = shadow.tolerance(ref_logits, live)
        if live.any():
            e = logit_error(got_logits[live], ref_logits[live])
            worst_logit = max(worst_logit, e)
            if shadow is not None:
                shadow.note(e)
            assert e <= tol, f"step {steps}: logits differ from the judge oracle by {e} (bound {tol})"
        if mm is not None:
            ml = O.decoder_logits_cached(mm, st_m, cross_m)
            if live.any():
                e = logit_error(got_logits[live], ml[live])
                worst_mirror = max(worst_mirror, e)
                assert e <= TOL_MIRROR, f"step {steps}: logits differ from the storage-rounding oracle by {e}"
            logp_m = O.log_softmax(np.asarray(ml, mm.ctype))
        if live.any():
            # the hidden rows handed out are the ones the logits were made from (a few rows per step)
            pick = np.nonzero(live)[0][:: max(1, int(live.sum()) // 6)]
            hid = eng.debug(lsq.DBG.HIDDEN, (M_all, mj.d))[rows][pick].astype(np.float64)
            E64 = np.asarray(mj.E, np.float64)
            want, scale = hid @ E64.T, np.abs(hid) @ np.abs(E64).T
            assert (np.abs(got_logits[pick] - want) <= 2e-6 * scale + 1e-7).all(), f"step {steps}: hidden rows and logits disagree"
        tok, par, sc, margin = O.beam_select(mj, st, ref_logits)
        g_tokens = eng.debug(lsq.DBG.TOKENS, (M_all, T + 1), np.int32)[rows]
        g_len = eng.debug(lsq.DBG.LEN, (M_all,), np.int32)[rows]
        g_fin = eng.debug(lsq.DBG.FINISHED, (M_all,), np.int32)[rows]
        g_par = eng.debug(lsq.DBG.PARENT, (M_all,), np.int32)[rows]
        g_score = eng.debug(lsq.DBG.SCORE, (M_all,))[rows]
        logp = O.log_softmax(np.asarray(ref_logits, mj.ctype))
        # deviation of the candidates' log-probabilities at this step, rows x (32 best of either side)
        lsm_ref = O.log_softmax(np.asarray(ref_logits, np.float64))
        lsm_got = O.log_softmax(np.asarray(got_logits, np.float64))
        if V > 33:
            cols = np.concatenate([np.argpartition(-lsm_ref, 32, axis=1)[:, :32], np.argpartition(-lsm_got, 32, axis=1)[:, :32]], axis=1)
        else:
            cols = np.broadcast_to(np.arange(V), (Ms, V))
        e_top = np.take_along_axis(lsm_got, cols, 1) - np.take_along_axis(lsm_ref, cols, 1)      # [Ms, <=64]
        with np.errstate(invalid="ignore"):
            drift = prev_gpu - prev_ref                                                            # [Ms]; nan where both -inf
        ref64 = np.asarray(ref_logits, np.float64)
        unit = 2.0 * (TAU_BAND_F16 if f16 else tol) * (np.abs(ref64).max(-1) + np.sqrt((ref64 ** 2).mean(-1)))   # [Ms]
        for b in range(B):
            base = b * k
            if old_fin[base:base + k].all():
                # nothing left to decide, and the library no longer touches the sentence: the hypotheses stay
                # where they are.  (Selecting again would re-sort them by the oracle's scores, which undoes
                # the library's order wherever an earlier step took it over within the band.)
                par[b], tok[b] = np.arange(k), mj.eos
                continue                       # the state checks below still apply
            alive = [base + j for j in range(k) if np.isfinite(prev_ref[base + j])]
            for r in range(base, base + k):
                assert np.isfinite(prev_ref[r]) == np.isfinite(prev_gpu[r]), f"step {steps} row {r}: -inf scores"
            common = float(np.mean(drift[alive]))
            cdev = unit_b = 0.0
            for r in alive:
                if old_fin[r]:
                    cdev = max(cdev, abs(drift[r] - common))
                else:
                    sdev = float(np.abs(e_top[r]).max())
                    unit_b = max(unit_b, unit[r])
                    worst_sdev = max(worst_sdev, sdev / unit[r])
                    assert sdev <= unit[r], f"step {steps} row {r}: candidate log-probabilities deviate by {sdev} (bound {unit[r]})"
                    cdev = max(cdev, float(np.abs(drift[r] - common + e_top[r]).max()))
            worst_cdev = max(worst_cdev, cdev / unit_b)
            assert cdev <= CDEV_UNITS * unit_b, f"step {steps} sentence {b}: candidate scores deviate by {cdev} (bound {CDEV_UNITS * unit_b})"
            band = MARGIN + 2 * cdev
            # the library's selection for this sentence
            gp = g_par[base:base + k].astype(np.int64)
            assert ((gp >= 0) & (gp < k)).all(), f"step {steps} sentence {b}: parent out of range"
            gt = np.empty(k, np.int64)
            for i in range(k):
                pr = base + gp[i]
                gt[i] = mj.eos if old_fin[pr] else g_tokens[base + i, old_len[pr] + 1]
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
                            if (j, mj.eos) not in kept:
                                best_drop = max(best_drop, float(st.score[b, j]))
                            continue
                        for v in np.argpartition(-logp[r], min(k, V - 1))[:k + 1]:
                            if (j, int(v)) not in kept:
                                best_drop = max(best_drop, float(st.score[b, j] + logp[r, v]))
                    assert best_drop <= ks.min() + band, \
                        f"step {steps} sentence {b}: dropped pair {best_drop} beats a kept one {ks.min()}"
                par[b], tok[b] = gp, gt
        # every oracle adopts the (checked) selection with its own scores
        prow = (np.arange(B)[:, None] * k + par).reshape(-1)          # parent row of every new hypothesis
        grew = ~old_fin[prow]
        sc = _follow_scores(mj, st, logp, tok, par, old_fin)
        # the library's own arithmetic: new score = parent's score + log-softmax of its own logits at the token
        step_dev = np.where(grew, np.abs((lsm_got - lsm_ref)[prow, tok.reshape(-1)]), 0.0)
        expect = np.where(grew, prev_gpu[prow] + lsm_got[prow, tok.reshape(-1)], prev_gpu[prow])
        fin = np.isfinite(sc.reshape(-1).astype(np.float64))
        assert np.array_equal(np.isfinite(g_score), fin), f"step {steps}: -inf scores"
        own = np.abs(g_score[fin] - expect[fin])
        worst_own = max(worst_own, float(own.max()) if own.size else 0.0)
        assert (own <= 5e-5 + 2e-6 * np.abs(expect[fin])).all(), \
            f"step {steps}: scores do not follow from the library's own logits (off by {own.max()})"
        bound = bound[prow] + step_dev + 1e-5
        active_ref = O.beam_advance(mj, st, tok, par, sc)
        if shadow is not None:
            shadow.advance(tok, par, sc)
        if mm is not None:
            O.beam_advance(mm, st_m, tok, par, _follow_scores(mm, st_m, logp_m, tok, par, old_fin))
        assert np.array_equal(g_len, st.len), f"step {steps}: lengths"
        assert np.array_equal(g_fin != 0, st.finished), f"step {steps}: finished flags"
        for r in range(Ms):
            n = st.len[r]
            assert np.array_equal(g_tokens[r, : n + 1], st.tokens[r, : n + 1]), f"step {steps} row {r}: tokens"
        ref_sc = st.score.reshape(-1).astype(np.float64)
        assert (np.abs(g_score[fin] - ref_sc[fin]) <= bound[fin] + 2e-5 * np.abs(ref_sc[fin])).all(), \
            f"step {steps}: scores drift from the judge's beyond the measured deviations"
        if sentences is None:
            assert active_gpu == active_ref, f"step {steps}: active {active_gpu} vs {active_ref}"
        else:
            assert active_gpu >= active_ref, f"step {steps}: active {active_gpu}, the compared subset alone has {active_ref}"
        steps += 1
        if verbose:
            print(f"step {steps}: active {active_gpu}, strict {strict_n} band {band_n}, judge {worst_logit:.2e} "
                  f"mirror {worst_mirror:.2e} sdev {worst_sdev:.2f} cdev {worst_cdev:.2f} units", flush=True)
        done = active_gpu == 0 if sentences is None else active_ref == 0
        if done or (max_steps is not None and steps >= max_steps):
            break
    return dict(steps=steps, batch=B, worst_logit=worst_logit, worst_mirror=worst_mirror, worst_sdev=worst_sdev,
                worst_cdev=worst_cdev, worst_own=worst_own, strict=strict_n, band=band_n,
                strict_share=strict_n / max(1, strict_n + band_n), state=st, judge=mj, bound=bound,
                **_f32_stats(shadow))


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
    worst = 0.0
    slack = np.zeros(B)                               # per row: the deviations of its own draws' log-probabilities
    strict = loose = 0
    for step in range(n_new):
        ref = O.gpt_step_logits(m, st)
        if shadow is not None:
            tol = shadow.tolerance(ref, np.ones(B, bool))
        prev_logp = eng.debug(lsq.DBG.SCORE, (B,)).astype(np.float64)
        active = eng.decode_step()
        got = eng.debug(lsq.DBG.LOGITS, (B, V))
        e = logit_error(got, ref)
        worst = max(worst, e)
        if shadow is not None:
            shadow.note(e)
        assert e <= tol, f"step {step}: logits differ from the oracle by {e} (bound {tol})"
        g_tok = eng.debug(lsq.DBG.TOKENS, (B, T + 1), np.int32)[:, st.pos + 1]
        g_ci = eng.debug(lsq.DBG.CAND_IDX, (B, k), np.int32)
        g_cl = eng.debug(lsq.DBG.CAND_SCORE, (B, k))
        toks, lps, own = [], [], np.zeros(B)
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
            own[r] = lp_own if g_tok[r] == tok_own else np.nan
            slack[r] += abs(lp_own - lp) + 1e-5
        O.gpt_advance(m, st, toks, lps)
        if shadow is not None:
            shadow.advance(toks, lps)
        g_logp = eng.debug(lsq.DBG.SCORE, (B,))
        ok = np.isfinite(own)       # the library's own arithmetic: the sum grows by the log-probability its logits give
        assert (np.abs(g_logp[ok] - (prev_logp[ok] + own[ok])) <= 5e-5 + 2e-6 * np.abs(g_logp[ok])).all(), f"step {step}: log-probability sums"
        assert (np.abs(g_logp - st.logp) <= slack + 2e-5 * np.abs(st.logp)).all(), f"step {step}: sums drift beyond the measured deviations"
        assert active == (B if step + 1 < m.cap_extra else 0), f"step {step}: active {active}"
        if verbose:
            print(f"step {step + 1}: strict {strict} loose {loose} worst logit error {worst:.2e}", flush=True)
    return dict(steps=n_new, strict=strict, loose=loose, worst=worst, state=st, **_f32_stats(shadow))


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
    worst = 0.0
    slack = np.zeros(B)                               # per sentence: the deviations of its own draws' log-probabilities
    steps = strict = loose = 0
    while True:
        ref = O.decoder_logits_cached(m, st, cross)
        old_fin = st.finished.copy()
        prev_score = eng.debug(lsq.DBG.SCORE, (B,)).astype(np.float64)
        active = eng.decode_step()
        got = eng.debug(lsq.DBG.LOGITS, (B, V))
        live = ~old_fin
        if shadow is not None:
            tol = shadow.tolerance(ref, live)
        own = np.full(B, np.nan)
        if live.any():
            e = logit_error(got[live], ref[live])
            worst = max(worst, e)
            if shadow is not None:
                shadow.note(e)
            assert e <= tol, f"step {steps}: logits differ from the oracle by {e} (bound {tol}, numpy float32 itself {shadow.last if shadow else 0})"
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
            if g_tok == tok_own:
                own[b] = lp_own
            slack[b] += abs(lp_own - lp) + 1e-5
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
        g_score = eng.debug(lsq.DBG.SCORE, (B,))
        ok = np.isfinite(own)       # the library's own arithmetic: the score grows by the log-probability its logits give
        assert (np.abs(g_score[ok] - (prev_score[ok] + own[ok])) <= 5e-5 + 2e-6 * np.abs(g_score[ok])).all(), f"step {steps}: scores"
        assert (np.abs(g_score - st.score[:, 0]) <= slack + 2e-5 * np.abs(st.score[:, 0])).all(), \
            f"step {steps}: scores drift beyond the measured deviations"
        if active_ref == 0 or (max_steps is not None and steps >= max_steps):
            break
    return dict(steps=steps, strict=strict, loose=loose, worst=worst, state=st, **_f32_stats(shadow))


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
            if shadow is not None:
                shadow.note(e)
            assert e <= tol, f"step {steps}: logits differ from the oracle by {e} (bound {tol})"
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
            scale = max(float(np.abs(ref_logits[base + j]).max() + np.sqrt((np.asarray(ref_logits[base + j], np.float64) ** 2).mean())) for j in range(k))
            assert cdev <= 2.0 * (TAU_BAND_F16 if m.round16 else tol) * scale * (steps + 1), \
                f"step {steps} sentence {b}: candidate scores deviate by {cdev}"
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
    return dict(steps=steps, strict=strict, band=band_n, state=st, **_f32_stats(shadow))
