"""GPU parity for bf16 models of the 8B-class layer shape (d=4096, 32x128 heads, FFN 12288,
vocab 126464), two layers deep so the CPU oracle finishes in seconds:

  * every linear step (QKV, O, gate/up+SwiGLU, down, LM-head reduction) on its own, MFMA kernels
    against an fp64 product of the same bf16 operands: tight, nothing upstream to blur it;
  * whole forwards, teacher forced from the oracle's state, against the exact fp32 oracle with
    tolerances derived from the operand noise floor (parity_util.operand_noise_floor);
  * GPU SSD == GPU stepwise bit for bit, one- and multi-sequence, and a node's rows bit-identical
    whether computed alone or inside a 5-node forward.
"""
import math

import numpy as np
import pytest
import torch

import parity_util
from paper_2510_04147_amd import synth
from parity_util import bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def shallow8b():
    """Two layers of the 8B shape, full vocabulary."""
    from paper_2510_04147_amd import binding
    cfg = synth.model_config("8b", n_layers=2)
    wg = synth.gen_weights(cfg, 0, device="cuda")
    w = synth.weights_to(wg, "cpu")
    eng = binding.SSD(cfg, wg, max_seqs=2, max_seq_len=512, block=32, max_draft=4, max_rows=320)
    prompt = synth.gen_prompt(cfg, 1002, 100)          # prefix length not a multiple of any tile
    sigma = parity_util.operand_noise_floor(cfg, w, prompt, 32, torch.float32)
    print(f"operand noise floor sigma = {sigma:.4f}")
    yield cfg, w, wg, eng, prompt, sigma
    eng.close()


@pytest.mark.parametrize("M", [160, 32, 45, 96, 128])
def test_linear_steps_against_fp64_products(shallow8b, M):
    """Each GEMM kernel alone: bf16 operands, fp32 accumulation, against fp64 on the same operands."""
    from paper_2510_04147_amd import binding as B
    cfg, w, wg, eng, _, _ = shallow8b
    d, F, V = cfg["d_model"], cfg["d_ffn"], cfg["vocab"]
    g = torch.Generator(device="cuda").manual_seed(5 + M)
    lw, lwc = wg["layers"][1], w["layers"][1]
    for path in (1, 0):
        eng.set_kernel_path(path)
        for which, W, K, N in ((B.LIN_QKV, lwc["wqkv"], d, 3 * d), (B.LIN_O, lwc["wo"], d, d), (B.LIN_DOWN, lwc["wdown"], F, d)):
            x = torch.randn(M, K, generator=g, device="cuda").to(torch.bfloat16)
            out = torch.empty(M, N, dtype=torch.float32, device="cuda")
            eng.k_linear(which, 1, x, out)
            want = x.cpu().double() @ W.double().T
            err = (out.cpu().double() - want).abs().max().item()
            assert err < 2e-4 * max(1.0, (K / 4096) ** 0.5), (path, which, err)
        x = torch.randn(M, d, generator=g, device="cuda").to(torch.bfloat16)
        out = torch.empty(M, F, dtype=torch.bfloat16, device="cuda")
        eng.k_linear(B.LIN_GU, 1, x, out)
        gu = x.cpu().double() @ lwc["wgu"].double().T
        want = gu[:, :F] / (1 + torch.exp(-gu[:, :F])) * gu[:, F:]
        diff = (out.cpu().double() - want).abs()
        assert bool((diff <= 2.0 ** -8 * want.abs() + 1e-4).all()), (path, diff.max())     # one bf16 rounding
        # LM head: max logit, arg-max and confidence without ever writing the logits
        x = torch.randn(M, d, generator=g, device="cuda").to(torch.bfloat16)
        out = torch.empty(3, M, dtype=torch.float32, device="cuda")
        eng.k_linear(B.LIN_LM, 0, x, out)
        lg = x.cpu().double() @ w["lm_head"].double().T
        lg[:, cfg["mask_id"]] = float("-inf")
        m, t = lg.max(dim=-1)
        c = 1.0 / torch.exp(lg - m[:, None]).sum(-1)
        o = out.cpu().double()
        assert (o[0] - m).abs().max() < 2e-4
        assert torch.equal(o[1].long(), t)
        assert ((o[2] - c).abs() <= 1e-4 * c).all()
    eng.set_kernel_path(1)


def test_mfma_path_teacher_forced_against_oracle(shallow8b):
    cfg, w, wg, eng, prompt, sigma = shallow8b
    eng.set_kernel_path(1)
    tol = parity_util.bf16_tolerances(sigma)
    ref, st, tot = parity_util.teacher_forced(eng, cfg, w, prompt, 32, 32, 4, torch.float32, literal=True, sigma=sigma, **tol)
    print("mfma totals:", tot, "sigma", sigma)
    assert tot["forwards"] == st["forwards"] and tot["rows"] > 200
    # as accurate as the ideal bf16-operand pipeline evaluated on the same rows
    assert tot["rms_dlogit"] <= 1.25 * tot["literal"]["rms_twin"] + 2e-3
    assert tot["rms_dlogit"] <= 1.5 * sigma + 2e-3, "GPU deviates from the exact oracle by more than bf16 operands explain"
    assert tot["tok_exempt"] <= 0.10 * tot["rows"]


def test_mfma_path_ragged_block_and_separate_rotary_kernel(shallow8b):
    """Blocks that fill a 32-row tile only partly (block 24, last block 8), once with the rotary stage
    inside the attention kernel (path 1) and once as a kernel of its own (path 2): both against the
    oracle, and bit-identical to each other."""
    cfg, w, wg, eng, prompt, sigma = shallow8b
    tol = parity_util.bf16_tolerances(sigma)
    outs = {}
    try:
        for path in (1, 2):
            eng.set_kernel_path(path)
            ref, st, tot = parity_util.teacher_forced(eng, cfg, w, prompt, 32, 24, 3, torch.float32, max_forwards=6, **tol)
            print(f"path {path}, block 24:", tot)
            assert tot["rms_dlogit"] <= 1.5 * sigma + 2e-3
            outs[path], _ = eng.generate([prompt], 56, 24, 3)
    finally:
        eng.set_kernel_path(1)
    assert np.array_equal(outs[1], outs[2])
    base, _ = eng.generate([prompt], 56, 24, 0)
    assert np.array_equal(outs[1], base)


def test_plain_path_teacher_forced_against_oracle(shallow8b):
    cfg, w, wg, eng, prompt, sigma = shallow8b
    eng.set_kernel_path(0)
    try:
        tol = parity_util.bf16_tolerances(sigma)
        ref, st, tot = parity_util.teacher_forced(eng, cfg, w, prompt, 32, 32, 4, torch.float32, max_forwards=4, **tol)
    finally:
        eng.set_kernel_path(1)
    print("plain totals:", tot)
    assert tot["rms_dlogit"] <= 1.5 * sigma + 2e-3


def test_gpu_ssd_equals_gpu_stepwise_bf16(shallow8b):
    cfg, w, wg, eng, prompt, _ = shallow8b
    base, s0 = eng.generate([prompt], 64, 32, 0)
    assert s0["forwards"] == 64
    for N in (1, 4):
        out, st = eng.generate([prompt], 64, 32, N)
        assert np.array_equal(out, base), f"N={N}"
        print(f"N={N}: forwards {st['forwards']} accept_hist {st['accept_hist'][:N + 2]}")
    # the mix-order tree (8 nodes for N = 4, MFMA path) changes the rounds, not the tokens
    eng.set_tree_mode(1)
    try:
        out, st = eng.generate([prompt], 64, 32, 4)
    finally:
        eng.set_tree_mode(0)
    assert np.array_equal(out, base), "mix order"
    print(f"mix order N=4: forwards {st['forwards']} accept_hist {st['accept_hist'][:6]}")
    # a round across the block boundary (MFMA path, leaf writes KV, next block behind it): same tokens
    eng.set_cross_block(1)
    try:
        out, st = eng.generate([prompt], 64, 32, 4)
        out8, st8 = eng.generate([prompt], 64, 8, 4)
    finally:
        eng.set_cross_block(0)
    assert np.array_equal(out, base), "cross block"
    base8, s8 = eng.generate([prompt], 64, 8, 4)
    assert np.array_equal(out8, base8) and st8["forwards"] <= s8["forwards"]
    print(f"cross block: block 32 forwards {st['forwards']}; block 8 forwards {st8['forwards']} vs {s8['forwards']}")
    # two sequences at once, different prompt lengths
    p2 = synth.gen_prompt(cfg, 77, 61)
    solo, _ = eng.generate([p2], 64, 32, 0)
    both, _ = eng.generate([prompt, p2], 64, 32, 4)
    assert np.array_equal(both[0], base[0]) and np.array_equal(both[1], solo[0])


def test_dual_cache_with_periodic_refresh_bf16(shallow8b):
    """Section 4.1's cache on the MFMA path: refresh forwards (the whole sequence in three segments that
    write and read the cache in the same layer) and block forwards against prefix + suffix, teacher
    forced against the oracle; free running, SSD equals stepwise decoding bit for bit."""
    cfg, w, wg, eng, prompt, sigma = shallow8b
    tol = parity_util.bf16_tolerances(sigma)
    try:
        for (blk, N, R, mf) in ((32, 4, 4, 8), (8, 3, 8, 10)):
            ref, st, tot = parity_util.teacher_forced_dual(eng, cfg, w, prompt, 48, blk, N, R, torch.float32,
                                                           max_forwards=mf, **tol)
            print(f"dual cache, block {blk}:", tot)
            assert tot["refreshes"] >= 2 and tot["rms_dlogit"] <= 1.5 * sigma + 2e-3
            assert tot["tok_exempt"] <= 0.10 * tot["rows"]
        for (blk, R) in ((8, 8), (32, 8), (24, 0)):
            eng.set_cache_mode(1, R)
            base, s0 = eng.generate([prompt], 56, blk, 0)
            assert s0["forwards"] == 56
            out, st = eng.generate([prompt], 56, blk, 4)
            assert np.array_equal(out, base), (blk, R)
            assert st["kv_passes"] == s0["kv_passes"] and st["forwards"] <= s0["forwards"]
            # spill-over (Section 3.2.2): the chain continues into the next block; same tokens, no more forwards
            eng.set_spill_over(1)
            try:
                out_s, st_s = eng.generate([prompt], 56, blk, 4)
            finally:
                eng.set_spill_over(0)
            assert np.array_equal(out_s, base), ("spill-over", blk, R)
            assert st_s["kv_passes"] == s0["kv_passes"] and st_s["forwards"] <= st["forwards"]
            print(f"dual cache block {blk} refresh {R}: forwards {st['forwards']} (stepwise 56, with spill-over "
                  f"{st_s['forwards']}), refreshes {st['kv_passes']}")
    finally:
        eng.set_cache_mode(0)
    plain, _ = eng.generate([prompt], 56, 8, 4)
    again, _ = eng.generate([prompt], 56, 8, 0)
    assert np.array_equal(plain, again)


def test_acceptance_limit_probe_bf16(shallow8b):
    """Section 5.1 / Table 2 on the 8B layer shape: the probe decodes the tokens stepwise decoding does,
    more candidates never match fewer tokens, and forwards and matches add up per round."""
    cfg, w, wg, eng, prompt, _ = shallow8b
    base, _ = eng.generate([prompt], 48, 8, 0)
    for N in (3, 5):
        toks, pr = eng.acceptance_limit(prompt, 48, 8, N, 5)
        assert np.array_equal(toks, base[0])
        assert pr["rounds"] == 6 * math.ceil(8 / (N + 1))
        assert all(a <= b for a, b in zip(pr["matched"], pr["matched"][1:])) and pr["matched"][-1] <= 48
        assert all(f == 48 - m + pr["rounds"] for f, m in zip(pr["forwards"], pr["matched"]))
        # the logits kept for ranking come from the plain GEMM, the decoded arg-max from the MFMA reduction:
        # they may disagree on a near-tie, so a round's first token is rank 0 in all but a few rounds
        assert pr["matched"][0] >= pr["rounds"] - 2
        print(f"N={N}: reduction per k {[round(x, 3) for x in pr['reduction']]}")


def test_graph_replay_of_the_mfma_forward(shallow8b):
    """HIP-graph replay (off by default) of the bf16 forward with its MFMA kernels: a context on a side
    stream, graphs on, must generate the same tokens and run the same number of forwards."""
    from paper_2510_04147_amd import binding
    cfg, w, wg, eng, prompt, _ = shallow8b
    base, st0 = eng.generate([prompt], 64, 32, 4)
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        g = binding.SSD(cfg, wg, max_seqs=1, max_seq_len=512, block=32, max_draft=4, max_rows=320)
        try:
            g.set_graphs(1)
            for rep in range(3):                       # first run captures, later runs replay every shape
                out, st = g.generate([prompt], 64, 32, 4)
                assert np.array_equal(out, base), rep
                assert st["forwards"] == st0["forwards"] and st["accept_hist"] == st0["accept_hist"]
        finally:
            g.close()


def test_node_rows_independent_of_batch_shape(shallow8b):
    """A node's rows are bit-identical alone (M=32) and inside a 5-node forward (M=160)."""
    cfg, w, wg, eng, _, _ = shallow8b
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
