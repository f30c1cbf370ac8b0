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
