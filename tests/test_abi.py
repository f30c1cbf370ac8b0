"""CPU-side checks of the boundary: the library loads, exports what include/dssd.h declares,
its structs have the layout the binding assumes, and host-checkable errors come back as codes."""
import ctypes as C
import os
import re
import subprocess
import sys

import pytest

from paper_2507_12000_amd import binding as D

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "dssd.h")
AUX_HEADER = os.path.join(ROOT, "include", "dssd_aux.h")


def _built():
    if not os.path.exists(D.LIB_PATH):
        pytest.skip("libdssd.so not built (run __graft_entry__.build())")


def test_library_exports_every_declared_symbol():
    _built()
    text = open(HEADER).read() + open(AUX_HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(dssd_[a-z_0-9]+)\s*\(", text))
    assert declared == set(D.EXPORTS), declared ^ set(D.EXPORTS)
    lib = D.load()
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_layout_matches_the_header(tmp_path):
    src = tmp_path / "layout.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "dssd.h"\nint main(void){\n'
                   'printf("%zu %zu %zu %zu %zu %zu %zu %zu\\n", sizeof(dssd_batch), offsetof(dssd_batch, total_drafts),'
                   ' offsetof(dssd_batch, logits), offsetof(dssd_batch, seed), offsetof(dssd_batch, session_base),'
                   ' sizeof(dssd_out), offsetof(dssd_out, row_stats), offsetof(dssd_out, status));'
                   'printf("%zu %zu %zu %zu %zu %zu\\n", offsetof(dssd_batch, draft_q_tok), sizeof(dssd_device_batch),'
                   ' offsetof(dssd_device_batch, p_rows), offsetof(dssd_device_batch, seed),'
                   ' offsetof(dssd_device_batch, out_token), offsetof(dssd_device_batch, status));'
                   'printf("%zu %zu\\n", offsetof(dssd_batch, step_counter), offsetof(dssd_device_batch, step_counter));'
                   'printf("%zu %zu %zu %zu %zu\\n", sizeof(dssd_topk_batch), offsetof(dssd_topk_batch, total_drafts),'
                   ' offsetof(dssd_topk_batch, q_prob), offsetof(dssd_topk_batch, seed), offsetof(dssd_topk_batch, step_counter));'
                   'return 0;}\n')
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)],
                   check=True)
    got = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    want = [C.sizeof(D.dssd_batch), D.dssd_batch.total_drafts.offset, D.dssd_batch.logits.offset,
            D.dssd_batch.seed.offset, D.dssd_batch.session_base.offset, C.sizeof(D.dssd_out),
            D.dssd_out.row_stats.offset, D.dssd_out.status.offset,
            D.dssd_batch.draft_q_tok.offset, C.sizeof(D.dssd_device_batch), D.dssd_device_batch.p_rows.offset,
            D.dssd_device_batch.seed.offset, D.dssd_device_batch.out_token.offset,
            D.dssd_device_batch.status.offset,
            D.dssd_batch.step_counter.offset, D.dssd_device_batch.step_counter.offset,
            C.sizeof(D.dssd_topk_batch), D.dssd_topk_batch.total_drafts.offset, D.dssd_topk_batch.q_prob.offset,
            D.dssd_topk_batch.seed.offset, D.dssd_topk_batch.step_counter.offset]
    assert got == want


def test_null_arguments_are_rejected_before_any_launch():
    _built()
    batch, out = D.dssd_batch(), D.dssd_out()
    for f in (D.dssd_verify_batch, D.dssd_residual_sample, D.dssd_bonus_sample):
        assert f(None, batch, out, 0, check=False) == D.DSSD_EINVAL
    assert D.load().dssd_verify_batch(None, None, None, None) == D.DSSD_EINVAL
    assert D.load().dssd_profile_enable(None, 1) == D.DSSD_EINVAL
    assert D.load().dssd_set_fused_limit(None, 1) == D.DSSD_EINVAL
    assert D.load().dssd_set_fused_pair_limit(None, 1) == D.DSSD_EINVAL
    assert D.load().dssd_set_early_exit_schedule(None, None, 0) == D.DSSD_EINVAL
    assert D.load().dssd_random_words(None, 0, 0, 0, 0, 1, 1, None, None) == D.DSSD_EINVAL
    assert D.load().dssd_step_topk(None, None, None, None) == D.DSSD_EINVAL
    assert D.status_str(D.DSSD_EALIGN) == "misaligned pointer"
    assert D.kernel_name(D.K_ROW_STATS) == "row_chunk_stats"
    assert D.dssd_workspace_bytes(0, 10) == 0 and D.dssd_workspace_bytes(100, 32000) > 100 * 16 * 8
    h = C.c_void_p()
    assert D.load().dssd_create(C.byref(h), 0, 0, 10) == D.DSSD_EINVAL
    assert D.load().dssd_create(None, 0, 10, 10) == D.DSSD_EINVAL


def test_static_step_checks_its_size_limit_on_the_host():
    """dssd_step_static refuses a batch beyond its static array before it touches a device."""
    _built()
    fake = 0x1000   # never dereferenced: the refusal comes first
    out = D.dssd_out(accepted_len=fake, rejected=fake, out_token=fake)
    big = D.dssd_batch(B=4096, V=256000, gamma=15, logits_dtype=D.DSSD_BF16, total_drafts=4096 * 15,
                       logits=fake, draft_probs=fake, draft_tokens=fake)
    assert D.dssd_step_static(big, out, 0, check=False) == D.DSSD_ENOMEM
    big.flags = D.FLAG_EARLY_EXIT
    assert D.dssd_step_static(big, out, 0, check=False) == D.DSSD_EUNSUPPORTED
    assert D.dssd_step_static(None, out, 0, check=False) == D.DSSD_EINVAL
    assert D.dssd_step_static(big, None, 0, check=False) == D.DSSD_EINVAL


def test_no_cpu_fallback_without_a_gpu():
    _built()
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(D.DssdError) as e:
        D.dssd_create(0, 16, 1000)
    assert e.value.code == D.DSSD_EHIP


def test_product_code_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2507_12000_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in text.lower() or fn == "synth.py", fn
    assert "oracle" not in open(HEADER).read().lower() and "oracle" not in open(AUX_HEADER).read().lower()
    code = "import sys; import paper_2507_12000_amd.binding, paper_2507_12000_amd.synth; " \
           "assert not [m for m in sys.modules if m.startswith('oracle')]"
    subprocess.run([sys.executable, "-c", code], check=True, cwd=ROOT)
