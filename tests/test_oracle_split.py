"""Pins for the oracle's edge / device split (Sec. 3, Algorithm 2).

* With an exact (fp64) downlink the split reproduces the unsplit step bit for bit: the cut
  moves work, not arithmetic.
* binary16 rounding against numpy's converter (an independent implementation), exhaustively
  over all 65 536 half values' neighbourhoods and on random floats.
* With a 16-bit or 32-bit downlink the device's law is that of norm(max(0, P~ - Q)) with the
  rounded P~: checked against a numpy restatement, and the induced emitted-token law stays
  within a small total-variation distance of P (the paper's "maintaining inference quality"
  is exact only for an exact downlink; the distance is what 16 bits cost).
"""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2507_12000_amd import synth


def _batch(B=30, V=700, seed=3, dtype="bf16", ragged=True):
    import torch
    w = synth.Workload("s", B=B, V=V, gamma=4, dtype=dtype, gamma_range=(1, 6) if ragged else None,
                       sigmas=(1.5,), temperature_range=(0.7, 1.3))
    d = synth.generate(w, seed=seed, device="cpu")
    if dtype == "bf16":
        lg = d["logits"].view(torch.int16).numpy().view(np.uint16); dt = O.BF16
    else:
        lg = d["logits"].numpy(); dt = O.F32
    off = d["draft_offsets"].numpy() if ragged else None
    return dict(lg=lg, dt=dt, Q=d["draft_probs"].numpy(), tok=d["draft_tokens"].numpy(), off=off,
                it=d["inv_temperature"].numpy(), V=V, B=B, gamma=0 if ragged else 4)


def _q_scalars(b):
    return b["Q"][np.arange(b["tok"].size), b["tok"]]


@pytest.mark.parametrize("ragged", [True, False])
def test_split_with_exact_downlink_equals_unsplit(ragged):
    b = _batch(ragged=ragged)
    full = O.verify_batch(b["lg"], b["dt"], b["Q"], b["tok"], b["V"], gamma=b["gamma"], draft_offsets=b["off"],
                          inv_temperature=b["it"], seed=9, step=4, session_base=100)
    edge = O.edge_batch(b["lg"], b["dt"], _q_scalars(b), b["tok"], b["V"], O.P_F64, gamma=b["gamma"],
                        draft_offsets=b["off"], inv_temperature=b["it"], seed=9, step=4, session_base=100, B=b["B"])
    assert (edge["res"]["n"] == full["res"]["n"]).all() and (edge["res"]["rejected"] == full["res"]["rejected"]).all()
    rej = full["res"]["rejected"] == 1
    assert rej.any() and (~rej).any()
    assert (edge["res"]["token"][~rej] == full["res"]["token"][~rej]).all()       # bonus tokens
    assert (edge["res"]["token"][rej] == -1).all()                                # the edge does not redraw
    dev = O.device_batch(b["Q"], edge["p_rows"], O.P_F64, edge["res"]["n"], edge["res"]["rejected"], b["V"],
                         gamma=b["gamma"], draft_offsets=b["off"], seed=9, step=4, session_base=100)
    assert (dev["token"][rej] == full["res"]["token"][rej]).all()
    assert (dev["token"][~rej] == -1).all()
    np.testing.assert_array_equal(dev["resid_mass"][rej], full["res"]["resid_mass"][rej])
    np.testing.assert_array_equal(np.nan_to_num(edge["p_tok"], nan=-1), np.where(np.isnan(edge["p_tok"]), -1, full["p_tok"]))


def test_binary16_rounding_matches_numpy():
    # every half value, the midpoints between neighbours, and one fp32 ulp either side of them
    halves = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float32)
    mids = ((halves[:-1].astype(np.float64) + halves[1:].astype(np.float64)) / 2).astype(np.float32)
    cands = np.concatenate([halves, mids, np.nextafter(mids, np.float32(0)), np.nextafter(mids, np.float32(1e9)),
                            np.random.default_rng(0).random(200000).astype(np.float32),
                            (np.random.default_rng(1).random(50000) * 1e-6).astype(np.float32),
                            np.array([0.0, 1.0, 65504.0, 65519.9, 65520.0, 1e-8, 2.0 ** -25, 2.0 ** -24], np.float32)])
    with np.errstate(over="ignore"):
        want = cands.astype(np.float16).view(np.uint16)
    got = np.array([O.f32_to_f16(x) for x in cands.tolist()], dtype=np.uint16)
    assert (got == want).all()
    neg = np.array([O.f32_to_f16(-x) for x in cands[:2000].tolist()], dtype=np.uint16)
    assert (neg == (want[:2000] | 0x8000)).all()
    back = np.array([O.f16_to_f64(h) for h in range(0, 0x7C00, 7)])
    assert (back == np.arange(0, 0x7C00, 7, dtype=np.uint16).view(np.float16).astype(np.float64)).all()


@pytest.mark.parametrize("p_dtype", [O.P_F32, O.P_F16])
def test_device_draw_matches_numpy_restatement(p_dtype):
    b = _batch(B=40, V=900, seed=5)
    edge = O.edge_batch(b["lg"], b["dt"], _q_scalars(b), b["tok"], b["V"], p_dtype, draft_offsets=b["off"],
                        inv_temperature=b["it"], seed=2, step=1)
    res = edge["res"]
    dev = O.device_batch(b["Q"], edge["p_rows"], p_dtype, res["n"], res["rejected"], b["V"], draft_offsets=b["off"],
                         seed=2, step=1)
    checked = 0
    for s in range(b["B"]):
        if not res["rejected"][s]:
            continue
        n = int(res["n"][s]); lrow = b["off"][s] + s + n
        P = O.softmax_row(b["lg"][lrow], b["dt"], float(b["it"][s]))[0]
        Pq = P.astype(np.float32)
        Pq = Pq.astype(np.float16).astype(np.float64) if p_dtype == O.P_F16 else Pq.astype(np.float64)
        stored = edge["p_rows"][s].view(np.float16).astype(np.float64) if p_dtype == O.P_F16 else edge["p_rows"][s].astype(np.float64)
        assert (stored == Pq).all()
        w = np.maximum(0.0, Pq - b["Q"][b["off"][s] + n].astype(np.float64))
        c = np.cumsum(w)
        r = (int(O.random_block(2, 1, s, n)[1]) >> 8) / 2 ** 24
        assert dev["token"][s] == np.searchsorted(c, r * c[-1], side="right")
        assert dev["resid_mass"][s] == c[-1]
        checked += 1
    assert checked > 5


def test_total_variation_cost_of_a_rounded_downlink():
    """Emitted-token law at one position when the device redraws from a rounded P~:
    law(y) = min(p, q)(y) + (1 - beta) * max(0, P~ - Q)(y) / sum(max(0, P~ - Q)).
    With an exact downlink this is P; with fp32 / fp16 it is close."""
    import torch
    w = synth.Workload("tv", B=4, V=32000, gamma=1, dtype="bf16", sigmas=(1.0,))
    d = synth.generate(w, seed=1, device="cpu")
    lg = d["logits"].view(torch.int16).numpy().view(np.uint16)
    for s in range(4):
        P = O.softmax_row(lg[2 * s], O.BF16)[0]
        Q = d["draft_probs"][s].numpy()
        Qd = Q.astype(np.float64)
        beta = np.minimum(P, Qd).sum()
        tv = {}
        for name, p_dtype in (("f64", O.P_F64), ("f32", O.P_F32), ("f16", O.P_F16)):
            row = O.quantize_p_row(P, p_dtype)
            Pq = row.view(np.float16).astype(np.float64) if p_dtype == O.P_F16 else row.astype(np.float64)
            wq, R = O.residual(Pq, Q)
            law = np.minimum(P, Qd) + (1.0 - beta) * wq / R
            tv[name] = 0.5 * np.abs(law - P).sum()
        assert tv["f64"] < 1e-12 + abs(1 - Qd.sum())     # exact up to sum(Q) != 1 in fp32
        assert tv["f32"] < 1e-6
        assert tv["f16"] < 2e-3
        assert tv["f16"] > tv["f32"]
