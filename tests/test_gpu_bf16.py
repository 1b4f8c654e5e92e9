"""GPU parity for bf16 models with the 8B-class layer shape (d=4096, 32x128 heads,
FFN 12288, vocab 126464): MFMA kernels against the fp32 CPU oracle (teacher forced),
against the plain FMA kernels, and GPU SSD == GPU stepwise bit for bit."""
import numpy as np
import pytest
import torch

import parity_util
from paper_2510_04147_amd import synth
from parity_util import bits

pytestmark = pytest.mark.gpu

# bf16 GEMM operands, fp32 accumulation and residual, against the fp32 oracle
TOL = dict(maxlogit_tol=2e-2, margin_tol=1e-2, conf_tol=5e-2, conf_rtol=5e-2)


@pytest.fixture(scope="module")
def shallow8b():
    """Two layers of the 8B shape, full vocabulary."""
    from paper_2510_04147_amd import binding
    cfg = synth.model_config("8b", n_layers=2)
    wg = synth.gen_weights(cfg, 0, device="cuda")
    w = synth.weights_to(wg, "cpu")
    eng = binding.SSD(cfg, wg, max_seqs=2, max_seq_len=512, block=32, max_draft=4, max_rows=320)
    yield cfg, w, wg, eng
    eng.close()


def test_mfma_path_teacher_forced_against_oracle(shallow8b):
    cfg, w, wg, eng = shallow8b
    prompt = synth.gen_prompt(cfg, 1002, 100)          # prefix length not a multiple of any tile
    eng.set_kernel_path(1)
    ref, st, tot = parity_util.teacher_forced(eng, cfg, w, prompt, 32, 32, 4, torch.float32, **TOL)
    print("mfma totals:", tot)
    assert tot["forwards"] == st["forwards"] and tot["rows"] > 200
    assert tot["tok_exempt"] <= 0.05 * tot["rows"]


def test_plain_path_teacher_forced_against_oracle(shallow8b):
    cfg, w, wg, eng = shallow8b
    prompt = synth.gen_prompt(cfg, 1002, 100)
    eng.set_kernel_path(0)
    try:
        ref, st, tot = parity_util.teacher_forced(eng, cfg, w, prompt, 32, 32, 4, torch.float32, max_blocks=1, **TOL)
    finally:
        eng.set_kernel_path(1)
    print("plain totals:", tot)
    assert tot["forwards"] == st["forwards"]


def test_gpu_ssd_equals_gpu_stepwise_bf16(shallow8b):
    cfg, w, wg, eng = shallow8b
    prompt = synth.gen_prompt(cfg, 1002, 100)
    base, s0 = eng.generate([prompt], 64, 32, 0)
    assert s0["forwards"] == 64
    for N in (1, 4):
        out, st = eng.generate([prompt], 64, 32, N)
        assert np.array_equal(out, base), f"N={N}"
        print(f"N={N}: forwards {st['forwards']} accept_hist {st['accept_hist'][:N + 2]}")
    # two sequences at once, different prompt lengths
    p2 = synth.gen_prompt(cfg, 77, 61)
    solo, _ = eng.generate([p2], 64, 32, 0)
    both, _ = eng.generate([prompt, p2], 64, 32, 4)
    assert np.array_equal(both[0], base[0]) and np.array_equal(both[1], solo[0])


def test_node_rows_independent_of_batch_shape(shallow8b):
    """A node's rows are bit-identical alone (M=32) and inside a 5-node forward (M=160)."""
    cfg, w, wg, eng = shallow8b
    prompt = synth.gen_prompt(cfg, 5, 75)
    eng.reset(0)
    eng.prefill_kv(0, prompt, 0)
    tok = [cfg["mask_id"]] * 32
    masked = [True] * 32
    drafts = [(5, 11), (0, 12), (30, 13), (7, 99)]
    o1, o3 = eng.new_out(1), eng.new_out(1)
    eng.verify_tree([0], [tok], [bits(masked)], [75], [drafts], 4, o1)
    a = o1.host()
    for j in (0, 3, 4):
        t2, m2 = list(tok), list(masked)
        for q, d in drafts[:j]:
            t2[q], m2[q] = d, False
        eng.draft([0], [t2], [bits(m2)], [75], 4, o3)
        c = o3.host()
        sel = np.array(m2)
        for k in ("row_maxlogit", "row_argmax", "row_conf"):
            assert np.array_equal(a[k][0, j][sel], c[k][0, 0][sel]), (k, j)
