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


def lockstep(lsq, eng, blob, w, max_steps=None, check_wide=True, verbose=False):
    """Runs the library and the oracle side by side, one decode step at a time.

    Every step: logits against the oracle that rounds where the model stores (tight) and, while
    both sides have made identical decisions, against the unrounded fp32 oracle (the stated
    tolerance); then tokens, parents, lengths, finished flags and scores of every sentence that is
    still comparable.  A sentence stays comparable while, at every step so far, the oracle's
    smallest gap between competing candidates exceeded MARGIN plus twice the deviation the
    library's candidate scores can have from the oracle's: (deviation of the hypothesis scores
    before the step) + 2 * (largest logit difference of the step, which also bounds the
    difference of the log-normaliser).  Above that bound the two orders cannot differ, so any
    difference in tokens or parents is an error.  Returns a summary dict."""
    m = O.Model(blob)                         # rounds at storage points for fp16 blobs
    mw = O.Model(blob, storage="wide") if (check_wide and m.round16) else None
    B, k, T, V = w.batch, w.beam, w.max_len, m.V
    M = B * k
    eng.encode(w.src_ids, w.src_lens)
    _, cross = O.encode(m, w.src_ids, w.src_lens)
    st = O.DecodeState(m, w.src_lens, k, T)
    if mw is not None:
        _, cross_w = O.encode(mw, w.src_ids, w.src_lens)
        st_w = O.DecodeState(mw, w.src_lens, k, T)
    comparable = np.ones(B, bool)
    dev = np.zeros(B)                          # |library score - oracle score|, per sentence
    wide_in_sync = mw is not None
    steps = 0
    worst_tight = worst_wide = 0.0
    compared_sentence_steps = 0
    tol_tight = 2e-3 if m.round16 else TOL_F32
    score_atol = 5e-3 if m.round16 else 2e-4
    while True:
        ref_logits = O.decoder_logits_cached(m, st, cross)
        active_gpu = eng.decode_step()
        got_logits = eng.debug(lsq.DBG.LOGITS, (M, V))
        live_rows = np.repeat(comparable, k) & ~st.finished
        if live_rows.any():
            e = logit_error(got_logits[live_rows], ref_logits[live_rows])
            worst_tight = max(worst_tight, e)
            assert e <= tol_tight, f"step {steps}: logits differ from the storage-rounding oracle by {e}"
        if wide_in_sync:
            wl = O.decoder_logits_cached(mw, st_w, cross_w)
            rows = live_rows & ~st_w.finished
            if rows.any():
                e = logit_error(got_logits[rows], wl[rows])
                worst_wide = max(worst_wide, e)
                assert e <= TOL_F16, f"step {steps}: fp16 logits differ from the fp32 oracle by {e}"
        tok, par, sc, margin = O.beam_select(m, st, ref_logits)
        active_ref = O.beam_advance(m, st, tok, par, sc)
        if wide_in_sync:
            tw, pw, sw, _ = O.beam_select(mw, st_w, wl)
            O.beam_advance(mw, st_w, tw, pw, sw)
            wide_in_sync = bool(np.array_equal(tw, tok) and np.array_equal(pw, par))
        ldiff = np.zeros(B)
        for b in range(B):
            rows = np.arange(b * k, (b + 1) * k)[live_rows[b * k:(b + 1) * k]]
            if len(rows):
                ldiff[b] = np.abs(got_logits[rows] - ref_logits[rows]).max()
        comparable &= margin > MARGIN + 2 * (dev + 2 * ldiff)
        g_tokens = eng.debug(lsq.DBG.TOKENS, (M, T + 1), np.int32)
        g_len = eng.debug(lsq.DBG.LEN, (M,), np.int32)
        g_fin = eng.debug(lsq.DBG.FINISHED, (M,), np.int32)
        g_par = eng.debug(lsq.DBG.PARENT, (M,), np.int32)
        g_score = eng.debug(lsq.DBG.SCORE, (M,))
        for b in np.nonzero(comparable)[0]:
            r = slice(b * k, (b + 1) * k)
            assert np.array_equal(g_par[r], par[b]), f"step {steps} sentence {b}: parents {g_par[r]} vs {par[b]}"
            assert np.array_equal(g_len[r], st.len[r]), f"step {steps} sentence {b}: lengths"
            assert np.array_equal(g_fin[r] != 0, st.finished[r]), f"step {steps} sentence {b}: finished flags"
            for j in range(k):
                n = st.len[b * k + j]
                assert np.array_equal(g_tokens[b * k + j, : n + 1], st.tokens[b * k + j, : n + 1]), \
                    f"step {steps} sentence {b} beam {j}: tokens"
            fin = np.isfinite(sc[b])
            assert np.array_equal(np.isfinite(g_score[r]), fin)
            np.testing.assert_allclose(g_score[r][fin], sc[b][fin], rtol=2e-5, atol=score_atol)
            dev[b] = np.abs(g_score[r][fin].astype(np.float64) - sc[b][fin]).max() if fin.any() else 0.0
            compared_sentence_steps += 1
        if comparable.all():
            assert active_gpu == active_ref, f"step {steps}: active {active_gpu} vs {active_ref}"
        steps += 1
        if verbose:
            print(f"step {steps}: active {active_gpu}, comparable {int(comparable.sum())}/{B}, "
                  f"tight {worst_tight:.2e} wide {worst_wide:.2e}", flush=True)
        if active_gpu == 0 or (max_steps is not None and steps >= max_steps):
            break
        if active_ref == 0 and comparable.all():
            raise AssertionError("oracle finished but the library did not")
    return dict(steps=steps, comparable=int(comparable.sum()), batch=B, worst_tight=worst_tight,
                worst_wide=worst_wide, compared=compared_sentence_steps, state=st, comparable_mask=comparable)
