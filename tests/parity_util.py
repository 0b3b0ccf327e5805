"""Comparison rules between the HIP path and the oracle (test infrastructure).

Floating-point bars
  attention  bf16: |out - ref| <= 2e-2 absolute, and relative RMS error <= 1e-2
             fp32: |out - ref| <= 1e-5 * max|ref row| (relative to the largest entry of the
                   output row: an element that happens to be ~0 has no meaningful relative error)
  logits     bf16 inputs / fp32 accumulate: |d| <= 1e-3;  fp32: |d| <= 1e-5 * max|logit|
  row_lse    |d| <= 1e-4;   p_at_draft: relative 1e-3 (bf16 path), 1e-5 * max (fp32 path), 2e-2 absolute
Integer outputs are bit-exact, except that
  - a request whose oracle walk evaluated an accept test with |p/q - u| < 1e-4 is exempt from
    that test on (it is compared up to that test, reported, and not counted);
  - a next_token mismatch is excused when the uniform lies within 1e-6 of the oracle's normalised
    CDF interval of the GPU's token (the draw sat on a knot of the CDF);
  - a greedy request is exempt when a row on the oracle's accepted path has a top-1/top-2 logit gap below 1e-4.
Exempt requests are printed and counted: at most 5 % of a batch of 20 or more requests, none of a smaller one.
"""
import numpy as np

ACCEPT_TIE = 1e-4
CDF_TIE = 1e-6
GREEDY_TIE = 1e-4


def check_attention(out, ref, dtype):
    out = np.asarray(out, dtype=np.float64)
    assert out.shape == ref.shape
    assert np.isfinite(out).all()
    err = np.abs(out - ref)
    if dtype == "bf16":
        assert err.max() <= 2e-2, f"attention abs err {err.max()}"
        rel_rms = np.sqrt((err ** 2).mean()) / max(np.sqrt((ref ** 2).mean()), 1e-30)
        assert rel_rms <= 1e-2, f"attention relative rms {rel_rms}"
    else:
        scale = np.abs(ref).max(axis=-1, keepdims=True)
        # the elementwise relative error, for the record: it is unbounded in principle (an entry that cancels to
        # ~0 has no meaningful relative error in any fp32 summation order), so the bar is relative to the row
        big = np.abs(ref) > 1e-3 * scale
        print(f"[fp32 attention] max |d|/max|row| = {(err / scale).max():.2e}; elementwise max |d|/|ref| = "
              f"{(err / np.maximum(np.abs(ref), 1e-300)).max():.2e} (over entries above 1e-3 of their row: "
              f"{(err[big] / np.abs(ref[big])).max():.2e})", flush=True)
        assert (err <= 1e-5 * scale + 1e-30).all(), f"attention rel err {(err / scale).max()}"
    return float(err.max())


def check_logits(got, ref, dtype):
    err = np.abs(np.asarray(got, np.float64) - ref)
    bar = 1e-3 if dtype == "bf16" else 1e-5 * np.abs(ref).max()
    if dtype != "bf16":
        print(f"[fp32 logits] max |d| = {err.max():.2e} (bar {bar:.2e}); elementwise max |d|/|ref| = "
              f"{(err / np.maximum(np.abs(ref), 1e-300)).max():.2e}", flush=True)
    assert err.max() <= bar, f"logits err {err.max()} > {bar}"
    return float(err.max())


def _ancestors_in_eval_order(orc, b, parents, Nq):
    """Nodes whose accept test the oracle evaluated, in evaluation order (ascending node id is the
    evaluation order of the walk for both chain and tree)."""
    return [n for n in range(1, Nq) if not np.isnan(orc.test_margin[b, n])]


def check_accept(res, orc, w, max_exempt_frac=0.05, small_batch_exempt=0):
    """res: dict of host arrays from the HIP path; orc: oracle.AcceptResult (with final_cdf when T > 0).
    At most int(max_exempt_frac * B) requests may be exempt when B >= 20; smaller batches get none unless the
    caller passes small_batch_exempt and says why where it does."""
    B, Nq = w.batch, w.num_q
    temps = getattr(w, "temperatures", None)   # one temperature per request, or None
    greedy_b = np.full(B, not (w.temperature > 0)) if temps is None else (np.asarray(temps) == 0)
    exempt, mism = [], []
    for b in range(B):
        same_walk = (res["accept_len"][b] == orc.accept_len[b] and
                     np.array_equal(res["accept_mask"][b], orc.accept_mask[b]))
        same_tok = res["next_token"][b] == orc.next_token[b]
        if same_walk and same_tok:
            continue
        if greedy_b[b]:
            # only the rows the oracle's walk consulted (the nodes on its accepted path) can excuse a difference
            on_path = orc.accept_mask[b].astype(bool)
            if (orc.top_gap[b][on_path] < GREEDY_TIE).any():
                exempt.append((b, "greedy near-tie"))
                continue
            mism.append((b, "greedy"))
            continue
        evald = _ancestors_in_eval_order(orc, b, w.parents, Nq)
        tie = [n for n in evald if orc.test_margin[b, n] < ACCEPT_TIE]
        if not same_walk:
            if tie:
                first = tie[0]
                before = [n for n in evald if n < first]
                if all(res["accept_mask"][b, n] == orc.accept_mask[b, n] for n in before):
                    exempt.append((b, f"accept near-tie at node {first}"))
                    continue
            mism.append((b, "walk"))
            continue
        # same walk, different token: excused only on a CDF knot
        vg = int(res["next_token"][b])
        cdf = orc.final_cdf[b]
        stop = int(orc.stop_node[b])
        u = float(w.uniforms[b, stop, 1])
        lo = cdf[vg - 1] if vg > 0 else 0.0
        hi = cdf[vg]
        if 0 <= vg < w.vocab and lo - CDF_TIE <= u <= hi + CDF_TIE:
            exempt.append((b, "draw on a CDF knot"))
        else:
            mism.append((b, f"token {vg} vs {int(orc.next_token[b])}, u={u}, interval=({lo},{hi})"))
    assert not mism, f"{len(mism)} mismatching requests: {mism[:5]}"
    budget = int(max_exempt_frac * B) if B >= 20 else small_batch_exempt
    assert len(exempt) <= budget, f"too many exempt requests ({len(exempt)} > {budget} of {B}): {exempt}"

    # per-node outputs
    lse_err = np.abs(res["row_lse"].astype(np.float64) - orc.row_lse).max()
    assert lse_err <= 1e-4, f"row_lse err {lse_err}"
    pa, pr = res["p_at_draft"].astype(np.float64), orc.p_at_draft
    assert (pa[:, 0] == 0).all()
    perr = np.abs(pa - pr)
    assert perr.max() <= 2e-2
    tie_rows = orc.top_gap < GREEDY_TIE
    par = w.parents if w.parents is not None else np.broadcast_to(np.arange(-1, Nq - 1), (B, Nq))
    for b in np.nonzero(greedy_b)[0]:
        for n in range(1, Nq):
            if not tie_rows[b, par[b, n]]:
                assert pa[b, n] == pr[b, n]
    sm = ~greedy_b
    if sm.any() and w.dtype == "bf16":
        assert (perr[sm] <= 1e-3 * pr[sm] + 1e-12).all(), \
            f"p_at_draft rel err {(perr[sm] / np.maximum(pr[sm], 1e-300)).max()}"
    elif sm.any():
        assert (perr[sm] <= 1e-5 * np.maximum(pr[sm], pr[sm].max() * 1e-3)).all(), \
            f"p_at_draft rel err {(perr[sm] / np.maximum(pr[sm], 1e-300)).max()}"
    return exempt
