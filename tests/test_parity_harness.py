"""The comparison harness itself, on the CPU: fed with the oracle's own answers it passes,
fed with a planted mistake (planted in a copy of the oracle's answers) it fails."""
import numpy as np
import pytest
import torch

import parity
from paper_2507_12000_amd import synth


def _as_gpu(orc, B):
    res = orc["res"]
    return dict(accepted_len=res["n"].copy(), rejected=res["rejected"].copy(), out_token=res["token"].copy(),
                status=res["status"].copy(), p_tok=orc["p_tok"].astype(np.float32),
                q_tok=orc["q_tok"].astype(np.float32),
                row_stats=np.stack([orc["row_m"], orc["row_Z"]], 1).astype(np.float32))


@pytest.fixture(scope="module")
def case():
    w = synth.Workload("h", B=12, V=2500, gamma=0, dtype="bf16", gamma_range=(1, 6), sigmas=(1.0,))
    inputs = synth.generate(w, seed=2, device="cpu")
    h = parity.to_numpy_inputs(inputs)
    orc = parity.run_oracle(h, 3, 4, workers=2)
    return h, orc


def test_oracle_against_itself_passes(case):
    h, orc = case
    rep = parity.compare(h, _as_gpu(orc, h["B"]), orc, 1e-5, seed=3, step=4)
    assert rep["sessions"] == h["B"] and rep["accept_tie_differs"] == 0 and rep["draw_tie_differs"] == 0


@pytest.mark.parametrize("field,delta", [("out_token", 1), ("accepted_len", 1), ("p_tok", 1e-3)])
def test_planted_mistake_is_caught(case, field, delta):
    h, orc = case
    g = _as_gpu(orc, h["B"])
    if field == "p_tok":
        g["p_tok"] = g["p_tok"] * np.float32(1 + delta)
    elif field == "accepted_len":
        b = int(np.argmax(orc["res"]["rejected"] == 1))
        g["accepted_len"][b] += 1
        gam = np.diff(orc["offsets"])
        g["rejected"][b] = int(g["accepted_len"][b] < gam[b])
    else:
        b = int(np.argmax(orc["res"]["cdf_margin"] > 1e-3))
        g[field][b] = (g[field][b] + delta) % h["V"]
    with pytest.raises(AssertionError):
        parity.compare(h, g, orc, 1e-5, seed=3, step=4)


def test_sessions_subset_and_threads_agree(case):
    h, orc = case
    sub = parity.run_oracle(h, 3, 4, workers=1, sessions=[1, 5, 7])
    for b in (1, 5, 7):
        assert sub["res"][b] == orc["res"][b]


def _plant_accept_tie(h, orc, b):
    """A copy of the oracle's answers in which session b's rejection (at n) is a near-tie:
    its uniform sits 1e-7 above the boundary p/q, and the flag says so."""
    o = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in orc.items()}
    q0 = int(o["offsets"][b])
    n = int(o["res"][b]["n"])
    o["r_acc"][q0 + n] = o["p_tok"][q0 + n] / o["q_tok"][q0 + n] + 1e-7
    o["res"]["accept_margin"][b] = 1e-7
    return o, q0, n


def _other_side_accepts_the_tie(h, o, b, q0, n, seed, step):
    """What an implementation that accepted the tied position legally answers: it goes on to the
    oracle's next rejection (or the bonus row) and draws there with that position's words."""
    q1 = int(o["offsets"][b + 1])
    _, accept = parity.position_margins(o, q0, q1)
    later = [i for i in range(n + 1, q1 - q0) if not accept[i]]
    g_n = later[0] if later else q1 - q0
    g_rej = int(g_n < q1 - q0)
    w, u = parity._weights_at(h, o, b, g_n, bool(g_rej), seed, step, 0)
    tok, _ = parity.O.inverse_cdf(w, u)
    return g_n, g_rej, int(tok)


def test_accept_tie_other_stop_is_excused_only_when_its_own_path_is_legal(case):
    h, orc = case
    gam = np.diff(orc["offsets"])
    b = int(np.argmax((orc["res"]["rejected"] == 1) & (orc["res"]["n"] < gam - 1)))
    assert orc["res"]["rejected"][b] == 1 and orc["res"]["n"][b] < gam[b] - 1
    o, q0, n = _plant_accept_tie(h, orc, b)
    g_n, g_rej, tok = _other_side_accepts_the_tie(h, o, b, q0, n, 3, 4)
    g = _as_gpu(o, h["B"])
    g["accepted_len"][b], g["rejected"][b], g["out_token"][b] = g_n, g_rej, tok
    rep = parity.compare(h, g, o, 1e-5, seed=3, step=4)
    assert rep["accept_ties"] == 1 and rep["accept_tie_differs"] == 1
    # the same answer without the tie is a mismatch
    with pytest.raises(AssertionError):
        parity.compare(h, g, orc, 1e-5, seed=3, step=4)
    # inside the tie: a token that is not a draw at the position where that side stopped
    g2 = {k: v.copy() for k, v in g.items()}
    g2["out_token"][b] = (tok + 1) % h["V"]
    with pytest.raises(AssertionError):
        parity.compare(h, g2, o, 1e-5, seed=3, step=4)
    # inside the tie: stopping before the tied position, at a draft the oracle clearly accepts
    if n > 0:
        g3 = {k: v.copy() for k, v in g.items()}
        g3["accepted_len"][b], g3["rejected"][b] = n - 1, 1
        w, u = parity._weights_at(h, o, b, n - 1, True, 3, 4, 0)
        g3["out_token"][b] = parity.O.inverse_cdf(w, u)[0]
        with pytest.raises(AssertionError):
            parity.compare(h, g3, o, 1e-5, seed=3, step=4)
    # inside the tie: running past the oracle's next clear rejection
    if g_rej:
        g4 = {k: v.copy() for k, v in g.items()}
        g4["accepted_len"][b] = g_n + 1
        g4["rejected"][b] = int(g_n + 1 < gam[b])
        w, u = parity._weights_at(h, o, b, g_n + 1, bool(g4["rejected"][b]), 3, 4, 0)
        g4["out_token"][b] = parity.O.inverse_cdf(w, u)[0]
        with pytest.raises(AssertionError):
            parity.compare(h, g4, o, 1e-5, seed=3, step=4)


def test_a_flag_that_disagrees_with_the_margins_is_caught(case):
    h, orc = case
    o = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in orc.items()}
    o["res"]["accept_margin"][:] = 0.0          # an oracle that called every session a tie
    with pytest.raises(AssertionError):
        parity.compare(h, _as_gpu(o, h["B"]), o, 1e-5, seed=3, step=4)


def test_too_many_draw_ties_are_caught(case):
    h, orc = case
    o = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in orc.items()}
    o["res"]["cdf_margin"][:] = 0.0             # an oracle that called every draw a tie
    with pytest.raises(AssertionError):
        parity.compare(h, _as_gpu(o, h["B"]), o, 1e-5, seed=3, step=4)


def test_draw_tie_probability_matches_the_flag_rate(case):
    """The closed form sum min(w/R, 2e-5) against the share of uniforms the oracle's inverse
    CDF flags, on a small weight vector scanned densely."""
    w = np.array([0.5, 1e-6, 3e-6, 0.2, 0.0, 0.3 - 4e-6])
    us = (np.arange(400000) + 0.5) / 400000
    flagged = np.mean([parity.O.inverse_cdf(w, u)[1] < parity.TIE for u in us])
    want = np.minimum(w / w.sum(), 2 * parity.TIE).sum()
    assert abs(flagged - want) < 1e-5
