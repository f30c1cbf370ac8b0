"""GPU test of dssd_step_static, the whole-step entry point that allocates nothing (its
workspace is a static device array inside the library): through the C ABI, every output must
equal dssd_step_fused's bit for bit, on calls in a row that carve the shared array differently
(the second batch is smaller than the first), and a batch beyond the array is refused."""
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2507_12000_amd import binding as D   # noqa: E402
from paper_2507_12000_amd import synth          # noqa: E402

DEV = "cuda:0"

FIRST = synth.Workload("static_first", B=48, V=4096 * 5 + 24, gamma=0, dtype="bf16", gamma_range=(1, 9),
                       temperature_range=(0.6, 1.4), sigmas=(0.5, 2.0), frac_q_equals_p=0.2, frac_q_uniform=0.2)
SECOND = synth.Workload("static_second_smaller", B=5, V=9000, gamma=3, dtype="f32", sigmas=(1.0,))
THIRD = synth.Workload("static_single_launch", B=2, V=32000, gamma=4, dtype="f32")


def _outputs(run, inputs, seed, step):
    t, out = D.alloc_out(inputs, DEV)
    batch = D.make_batch(inputs, seed=seed, step=step)
    run(batch, out)
    torch.cuda.synchronize()
    return t


def test_static_step_equals_the_context_step_on_calls_in_a_row():
    stream = torch.cuda.current_stream(DEV).cuda_stream
    cases = [(FIRST, 11, 0), (SECOND, 12, 5), (THIRD, 13, 1), (FIRST, 11, 2)]
    batches = {w.name: synth.generate(w, seed=3, device=DEV) for w in (FIRST, SECOND, THIRD)}
    # what the context-based call gives, each on a context of its own
    want = []
    for w, seed, step in cases:
        inputs = batches[w.name]
        ctx = D.Context(DEV, max_rows=inputs["R_L"], max_V=w.V)
        want.append(_outputs(lambda b, o: D.dssd_step_fused(ctx.handle, b, o, stream), inputs, seed, step))
        ctx.close()
    # the static call, back to back on the one shared array: larger batch, smaller, tiny, larger again
    got = [_outputs(lambda b, o: D.dssd_step_static(b, o, stream), batches[w.name], seed, step)
           for w, seed, step in cases]
    for (w, seed, step), g, e in zip(cases, got, want):
        print(f"[static] {w.name} seed={seed} step={step}: rejected {int(e['rejected'].sum())} of {w.B}", flush=True)
        assert int(e["status"].abs().sum()) == 0
        assert ((e["out_token"] >= 0) & (e["out_token"] < w.V)).all()
        for k in e:
            assert torch.equal(g[k], e[k]), (w.name, k)


def test_static_step_refuses_what_does_not_fit_or_needs_lists():
    inputs = synth.generate(SECOND, seed=3, device=DEV)
    t, out = D.alloc_out(inputs, DEV)
    batch = D.make_batch(inputs, seed=1, step=0)
    # more chunk statistics than the array holds: refused, outputs untouched
    big = D.make_batch(inputs, seed=1, step=0)
    big.B, big.gamma, big.V = 4096, 15, 256000
    big.total_drafts = big.B * big.gamma
    big.logits_dtype = D.DSSD_BF16
    assert 8 * (big.total_drafts + big.B) * 63 > D.STATIC_SCRATCH_BYTES
    assert D.dssd_step_static(big, out, 0, check=False) == D.DSSD_ENOMEM
    for flag in (D.FLAG_SPARSE_SUPPORT, D.FLAG_EARLY_EXIT):
        batch.flags = flag
        assert D.dssd_step_static(batch, out, 0, check=False) == D.DSSD_EUNSUPPORTED
    torch.cuda.synchronize()
    assert (t["accepted_len"] == -7).all() and (t["out_token"] == -7).all()
    assert D.dssd_step_static(None, out, 0, check=False) == D.DSSD_EINVAL


def test_static_step_inside_a_hip_graph():
    """The callers the entry point is for include code under graph capture: the call (a fill
    kernel for its counters, then the step's kernels; no allocation, no memset node) is recorded
    once and replayed, with other calls on the shared array and synchronisations between the
    replays, and every replay reproduces the eager result."""
    w = synth.Workload("static_graph", B=24, V=4096 * 3 + 8, gamma=5, dtype="bf16", sigmas=(0.5, 1.5))
    inputs = synth.generate(w, seed=7, device=DEV)
    other_inputs = synth.generate(SECOND, seed=3, device=DEV)
    stream = torch.cuda.current_stream(DEV).cuda_stream
    eager = _outputs(lambda b, o: D.dssd_step_static(b, o, stream), inputs, 31, 2)
    batch = D.make_batch(inputs, seed=31, step=2)
    t, out = D.alloc_out(inputs, DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        D.dssd_step_static(batch, out, side.cuda_stream)          # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            D.dssd_step_static(batch, out, side.cuda_stream)
    torch.cuda.synchronize()
    for rep in range(4):
        for v in t.values():
            v.fill_(-3)
        _outputs(lambda b, o: D.dssd_step_static(b, o, stream), other_inputs, 5, rep)   # re-carves the array
        graph.replay()
        torch.cuda.synchronize()
        for k in eager:
            assert torch.equal(t[k], eager[k]), (k, rep)
