"""Shared helpers of the GPU-vs-oracle parity tests: run the CPU oracle over a batch (split
over host threads by session; each session is still computed by the single-threaded oracle
code) and compare it with what the HIP library wrote, under the near-tie rule.

Near-tie rule: a decision is a near-tie when the oracle's uniform lies within 1e-5 of the
decision boundary (|r - p/q| < 1e-5 for an accept test, distance to a CDF boundary below
1e-5 of the total mass for an inverse-CDF draw).  Near-ties are counted, reported and bounded
in number.  Outside near-ties everything is compared exactly.  Inside one, an answer that
differs from the oracle's must still be a legal one: a different stopping position only
through positions that are themselves near-ties, and a token that is a valid draw at the
position where that side stopped.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from oracle import oracle as O

TIE = 1e-5


def to_numpy_inputs(inputs):
    """Host copies of a synth batch, logits as the oracle wants them (fp32 or bf16 bits)."""
    import torch
    lg = inputs["logits"]
    if lg.dtype == torch.bfloat16:
        logits = lg.view(torch.int16).cpu().numpy().view(np.uint16)
        dtype = O.BF16
    else:
        logits = lg.cpu().numpy()
        dtype = O.F32
    off = inputs.get("draft_offsets")
    it = inputs.get("inv_temperature")
    return dict(logits=logits, dtype=dtype, draft_probs=inputs["draft_probs"].cpu().numpy(),
                draft_tokens=inputs["draft_tokens"].cpu().numpy(),
                draft_offsets=None if off is None else off.cpu().numpy(),
                inv_temperature=None if it is None else it.cpu().numpy(),
                B=inputs["B"], V=inputs["V"], gamma=inputs["gamma"])


def run_oracle(h, seed, step, session_base=0, workers=8, sessions=None):
    """Oracle results for sessions `sessions` (default: all) of host batch `h`.
    Returns dict of arrays indexed like the full batch (untouched entries are NaN / -9)."""
    B, V, gamma = h["B"], h["V"], h["gamma"]
    off = h["draft_offsets"]
    if off is None:
        off = (np.arange(B + 1, dtype=np.int64) * gamma).astype(np.int32)
    R_Q = int(off[-1]); R_L = R_Q + B
    res = np.zeros(B, dtype=O.RESULT_DTYPE); res["n"] = -9
    p_tok = np.full(R_Q, np.nan); q_tok = np.full(R_Q, np.nan); r_acc = np.full(R_Q, np.nan)
    row_m = np.full(R_L, np.nan); row_Z = np.full(R_L, np.nan)
    todo = np.arange(B) if sessions is None else np.asarray(sessions)

    def one(b):
        q0, q1 = int(off[b]), int(off[b + 1])
        l0, l1 = q0 + b, q1 + b + 1
        it = None if h["inv_temperature"] is None else h["inv_temperature"][b:b + 1]
        o = O.verify_batch(h["logits"][l0:l1], h["dtype"], h["draft_probs"][q0:q1],
                           h["draft_tokens"][q0:q1], V, gamma=q1 - q0,
                           draft_offsets=np.array([0, q1 - q0], np.int32),
                           inv_temperature=it, seed=seed, step=step, session_base=session_base + b)
        res[b] = o["res"][0]
        p_tok[q0:q1] = o["p_tok"]; q_tok[q0:q1] = o["q_tok"]; r_acc[q0:q1] = o["r_acc"]
        row_m[l0:l1] = o["row_m"]; row_Z[l0:l1] = o["row_Z"]

    if workers > 1 and len(todo) > 1:
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(one, todo))
    else:
        for b in todo:
            one(b)
    return dict(res=res, p_tok=p_tok, q_tok=q_tok, r_acc=r_acc, row_m=row_m, row_Z=row_Z,
                offsets=off, sessions=todo)


def _weights_at(h, orc, b, n, rejected, seed, step, session_base):
    """Weights and uniform of session b's draw if it stops at position n: the residual
    max(0, P_n - Q_n) with word 1 of the position-n block after a rejection (P_n itself when
    that residual has no mass), P_gamma with word 2 of the position-gamma block otherwise."""
    off = orc["offsets"]
    lrow = int(off[b]) + b + n
    tau = 1.0 if h["inv_temperature"] is None else float(h["inv_temperature"][b])
    P = O.softmax_row(h["logits"][lrow], h["dtype"], tau)[0]
    words = O.random_block(seed, step, session_base + b, n)
    if rejected:
        w, R = O.residual(P, h["draft_probs"][int(off[b]) + n])
        return (w if R > 0.0 else P), O.u01(words[1])
    return P, O.u01(words[2])


def _draw_is_valid(h, orc, b, token, seed, step, session_base, n=None, rejected=None):
    """Is `token` a correct draw for session b stopping at position n (default: where the
    oracle stopped) once the target r * total may move by 1e-5 of the total mass?
    Recomputed from the oracle's pieces."""
    r = orc["res"][b]
    n = int(r["n"]) if n is None else n
    rejected = bool(r["rejected"]) if rejected is None else rejected
    w, u = _weights_at(h, orc, b, n, rejected, seed, step, session_base)
    c = np.cumsum(w)
    t, R = u * c[-1], c[-1]
    lo = c[token - 1] if token > 0 else 0.0
    return w[token] > 0 and lo - TIE * R <= t < c[token] + TIE * R


def draw_tie_probability(h, orc, b, seed, step, session_base=0):
    """Probability, over the uniform of the draw, that session b's draw is flagged a near-tie:
    the share of [0, total) within 1e-5 * total of a CDF boundary, which is the sum over tokens
    of min(w_k / total, 2e-5) (each token's own interval is covered from both ends)."""
    r = orc["res"][b]
    w, _ = _weights_at(h, orc, b, int(r["n"]), bool(r["rejected"]), seed, step, session_base)
    return float(np.minimum(w / w.sum(), 2 * TIE).sum())


def position_margins(orc, q0, q1):
    """|r - p/q| at every draft position of a session, from the oracle's per-position scalars,
    with the same conventions for q = 0 as the oracle's flag (recomputed here, in the division
    form, so that the harness does not lean on that flag alone)."""
    p, q, r = orc["p_tok"][q0:q1], orc["q_tok"][q0:q1], orc["r_acc"][q0:q1]
    with np.errstate(divide="ignore", invalid="ignore"):
        m = np.abs(r - p / q)
    m[q == 0] = np.where(p[q == 0] > 1e-30, np.inf, 0.0)
    accept = r * q < p
    return m, accept


def _tied_path_is_valid(h, orc, b, q0, q1, g_n, g_rej, g_tok, seed, step, session_base):
    """Inside an accept near-tie the other side may stop elsewhere than the oracle.  Its path is
    legal iff every position it accepted is one the oracle accepts or a near-tie, the position
    it rejected (if any) is one the oracle rejects or a near-tie, and its token is a valid draw
    at ITS stopping position with that position's random word."""
    margins, accept = position_margins(orc, q0, q1)
    tie = margins < TIE
    if not (accept[:g_n] | tie[:g_n]).all():
        return False
    if g_rej and not (~accept[g_n] or tie[g_n]):
        return False
    if seed is None:
        return True
    return bool(_draw_is_valid(h, orc, b, g_tok, seed, step, session_base, n=g_n, rejected=bool(g_rej)))


def compare(h, gpu, orc, p_rtol, seed=None, step=None, session_base=0):
    """gpu: dict of numpy arrays (accepted_len, rejected, out_token, row_stats, p_tok, q_tok,
    status).  Returns a report dict; raises AssertionError on a mismatch outside near-ties.
    Where the two sides differ inside a near-tie the GPU's answer must still be a valid one
    (its own path re-derived from the oracle's pieces; the draw checked when seed and step are
    given).  The number of near-ties is itself bounded: an accept test is one with probability
    at most 2e-5, a draw with the probability draw_tie_probability gives, estimated on a sample
    of the sessions, so a flag that excused too much would fail here."""
    off = orc["offsets"]
    res = orc["res"]
    rep = dict(sessions=0, positions=0, rejected=0, accept_ties=0, draw_ties=0,
               accept_tie_differs=0, draw_tie_differs=0, max_p_rel=0.0, max_lse_abs=0.0)
    bad = []
    tested = 0   # accept tests the oracle's loop really made
    for b in orc["sessions"]:
        b = int(b)
        q0, q1 = int(off[b]), int(off[b + 1])
        l0, l1 = q0 + b, q1 + b + 1
        r = res[b]
        rep["sessions"] += 1
        rep["positions"] += q1 - q0
        # input-fault bits must agree; the zero-residual bit (2) can only differ in a near-tie
        assert (int(gpu["status"][b]) & ~2) == (int(r["status"]) & ~2), (b, gpu["status"][b], r["status"])
        if r["status"] & 1:
            assert gpu["accepted_len"][b] == 0 and gpu["rejected"][b] == 1 and gpu["out_token"][b] == -1
            continue
        # probabilities at every draft position, statistics of every row
        po, pg = orc["p_tok"][q0:q1], gpu["p_tok"][q0:q1].astype(np.float64)
        big = po > 1e-30
        if big.any():
            rel = np.abs(pg[big] - po[big]) / po[big]
            rep["max_p_rel"] = max(rep["max_p_rel"], float(rel.max()))
        assert (np.abs(pg[~big]) <= 1e-30 * (1 + p_rtol)).all()
        assert (gpu["q_tok"][q0:q1].astype(np.float64) == orc["q_tok"][q0:q1]).all(), b
        lse_o = orc["row_m"][l0:l1] + np.log(orc["row_Z"][l0:l1])
        rs = gpu["row_stats"][l0:l1].astype(np.float64)
        lse_g = rs[:, 0] + np.log(rs[:, 1])
        rep["max_lse_abs"] = max(rep["max_lse_abs"], float(np.abs(lse_g - lse_o).max()))
        # decisions
        rep["rejected"] += int(r["rejected"])
        tested += min(int(r["n"]) + 1, q1 - q0)
        margins, _ = position_margins(orc, q0, q1)
        examined = margins[:min(int(r["n"]) + 1, q1 - q0)]
        accept_tie = bool((examined < TIE).any())
        # the oracle's own flag must say the same as the margins recomputed here
        assert accept_tie == bool(r["accept_margin"] < TIE), (b, float(r["accept_margin"]), examined.min(initial=np.inf))
        draw_tie = r["cdf_margin"] < TIE
        rep["accept_ties"] += int(accept_tie)
        rep["draw_ties"] += int(draw_tie)
        g_n, g_rej, g_tok = int(gpu["accepted_len"][b]), int(gpu["rejected"][b]), int(gpu["out_token"][b])
        assert 0 <= g_n <= q1 - q0 and g_rej == int(g_n < q1 - q0) and 0 <= g_tok < h["V"], (b, g_n, g_rej, g_tok)
        if g_n != r["n"] or g_rej != r["rejected"]:
            if accept_tie and _tied_path_is_valid(h, orc, b, q0, q1, g_n, g_rej, g_tok, seed, step, session_base):
                rep["accept_tie_differs"] += 1
            else:
                bad.append((b, "n", g_n, int(r["n"]), float(r["accept_margin"])))
            continue
        if g_tok != r["token"]:
            if draw_tie and (seed is None or _draw_is_valid(h, orc, b, g_tok, seed, step, session_base)):
                rep["draw_tie_differs"] += 1
            else:
                bad.append((b, "token", g_tok, int(r["token"]), float(r["cdf_margin"])))
    assert not bad, f"{len(bad)} mismatches outside near-ties, first: {bad[:5]}"
    assert rep["max_p_rel"] <= p_rtol, rep
    assert rep["max_lse_abs"] <= p_rtol, rep
    differs = rep["accept_tie_differs"] + rep["draw_tie_differs"]
    assert differs <= max(2, 1e-3 * (rep["positions"] + rep["sessions"])), rep
    # How many near-ties there may be.  Accept tests: each is one with probability <= 2e-5.
    assert rep["accept_ties"] <= 2 + 10 * 2 * TIE * tested, rep
    # Draws: expected count from the tie probability of a sample of the sessions (at most 48,
    # evenly spread), allowed twice that plus five standard deviations of a count plus slack.
    if seed is not None:
        done = [int(b) for b in orc["sessions"] if not (res[int(b)]["status"] & 1)]
        sample = done[::max(1, len(done) // 48)][:48]
        if sample:
            mean_p = float(np.mean([draw_tie_probability(h, orc, b, seed, step, session_base) for b in sample]))
            expected = mean_p * len(done)
            rep["expected_draw_ties"] = expected
            assert rep["draw_ties"] <= 2 * expected + 5 * np.sqrt(expected) + 3, rep
    return rep
