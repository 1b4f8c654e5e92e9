"""The other workload shapes as GPU parity cases (two layers deep so the oracle stays fast):
  cfg3  8B layer shape, block 64, draft depth 8 (9 nodes, M = 576 rows in one forward)
  cfg4  8B layer shape, batch 4, prompts of 1024 tokens (long shared prefix per sequence)
  cfg5  7B-class GQA shape (28 query / 4 KV heads, d=3584, FFN 18944, vocab 152064), batch 8, depth 8
"""
import numpy as np
import pytest
import torch

import parity_util
from paper_2510_04147_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def w8b():
    cfg = synth.model_config("8b", n_layers=2)
    wg = synth.gen_weights(cfg, 0, device="cuda")
    return cfg, synth.weights_to(wg, "cpu"), wg


def test_cfg3_block64_depth8(w8b):
    from paper_2510_04147_amd import binding
    cfg, w, wg = w8b
    eng = binding.SSD(cfg, wg, max_seqs=1, max_seq_len=512 + 128, block=64, max_draft=8, max_rows=9 * 64)
    prompt = synth.gen_prompt(cfg, 1003, 512)
    base, s0 = eng.generate([prompt], 128, 64, 0)
    out, s8 = eng.generate([prompt], 128, 64, 8)
    assert np.array_equal(out, base) and s0["forwards"] == 128 and s8["forwards"] < 128
    print("cfg3 accept_hist", s8["accept_hist"][:10])
    sigma = parity_util.operand_noise_floor(cfg, w, prompt, 64, torch.float32)
    tol = parity_util.bf16_tolerances(sigma)
    _, _, tot = parity_util.teacher_forced(eng, cfg, w, prompt, 64, 64, 8, torch.float32, max_forwards=4,
                                           verbose=False, literal=True, sigma=sigma, **tol)
    print("cfg3 totals", tot, "sigma", sigma)
    assert tot["rms_dlogit"] <= 1.5 * sigma + 2e-3
    eng.close()


@pytest.mark.parametrize("M", [576, 200, 401])
def test_many_row_gemm_gives_the_bits_of_the_few_row_gemm(w8b, M):
    """Forwards with more than 192 rows run the GEMMs in several row chunks (work-groups of neighbouring
    chunks share an n-block's weights).  Every linear step at M rows: against an fp64 product of the same
    operands, and bit for bit against the same rows sent through in passes of at most 160 rows."""
    from paper_2510_04147_amd import binding as B
    cfg, w, wg = w8b
    eng = B.SSD(cfg, wg, max_seqs=1, max_seq_len=256, block=64, max_draft=8, max_rows=640)
    d, F = cfg["d_model"], cfg["d_ffn"]
    g = torch.Generator(device="cuda").manual_seed(M)
    lw = w["layers"][1]
    try:
        for which, W, K, N in ((B.LIN_QKV, lw["wqkv"], d, 3 * d), (B.LIN_O, lw["wo"], d, d), (B.LIN_DOWN, lw["wdown"], F, d)):
            x = torch.randn(M, K, generator=g, device="cuda").to(torch.bfloat16)
            out = torch.empty(M, N, dtype=torch.float32, device="cuda")
            eng.k_linear(which, 1, x, out)
            err = (out.cpu().double() - x.cpu().double() @ W.double().T).abs().max().item()
            assert err < 2e-4 * max(1.0, (K / 4096) ** 0.5), (which, err)
            for lo in range(0, M, 160):
                part = torch.empty(min(160, M - lo), N, dtype=torch.float32, device="cuda")
                eng.k_linear(which, 1, x[lo:lo + 160].contiguous(), part)
                assert torch.equal(part, out[lo:lo + 160]), (which, lo)
        x = torch.randn(M, d, generator=g, device="cuda").to(torch.bfloat16)
        out = torch.empty(M, F, dtype=torch.bfloat16, device="cuda")
        eng.k_linear(B.LIN_GU, 1, x, out)
        gu = x.cpu().double() @ lw["wgu"].double().T
        want = gu[:, :F] / (1 + torch.exp(-gu[:, :F])) * gu[:, F:]
        assert bool(((out.cpu().double() - want).abs() <= 2.0 ** -8 * want.abs() + 1e-4).all())
        lm = torch.empty(3, M, dtype=torch.float32, device="cuda")
        eng.k_linear(B.LIN_LM, 0, x, lm)
        for lo in range(0, M, 160):
            n = min(160, M - lo)
            part = torch.empty(n, F, dtype=torch.bfloat16, device="cuda")
            eng.k_linear(B.LIN_GU, 1, x[lo:lo + 160].contiguous(), part)
            assert torch.equal(part, out[lo:lo + n]), ("gate/up", lo)
            lmp = torch.empty(3, n, dtype=torch.float32, device="cuda")
            eng.k_linear(B.LIN_LM, 0, x[lo:lo + 160].contiguous(), lmp)
            assert torch.equal(lmp, lm[:, lo:lo + n]), ("lm head", lo)
    finally:
        eng.close()


def test_cfg4_batch4_long_prefix(w8b):
    from paper_2510_04147_amd import binding
    cfg, w, wg = w8b
    eng = binding.SSD(cfg, wg, max_seqs=4, max_seq_len=1024 + 64, block=32, max_draft=4, max_rows=1024)
    prompts = [synth.gen_prompt(cfg, 1004 + i, 1024) for i in range(4)]
    both, st = eng.generate(prompts, 64, 32, 4)
    assert st["tokens"] == 4 * 64
    for i in (0, 3):
        solo, _ = eng.generate([prompts[i]], 64, 32, 0)
        assert np.array_equal(both[i], solo[0]), f"sequence {i} of the batch differs from its solo stepwise run"
    # the batch against the oracle: the first forwards of every sequence (the block-start draft, then 5-node
    # verification forwards), all four sequences in ONE forward each, each sequence compared with its own oracle run
    sigma = parity_util.operand_noise_floor(cfg, w, prompts[0], 32, torch.float32)
    tol = parity_util.bf16_tolerances(sigma)
    tot = parity_util.teacher_forced_batch(eng, cfg, w, prompts, 32, 32, 4, torch.float32, max_forwards=3, sigma=sigma, **tol)
    print("cfg4 totals", tot, "sigma", sigma)
    assert tot["forwards"] == 3 and tot["rows"] >= 4 * 3 * 28
    assert tot["rms_dlogit"] <= 1.5 * sigma + 2e-3
    eng.close()


def test_cfg5_gqa_batch8_depth8():
    from paper_2510_04147_amd import binding
    from paper_2510_04147_amd import binding as B
    cfg = synth.model_config("7b_gqa", n_layers=2)
    wg = synth.gen_weights(cfg, 0, device="cuda")
    w = synth.weights_to(wg, "cpu")
    eng = binding.SSD(cfg, wg, max_seqs=8, max_seq_len=512 + 64, block=32, max_draft=8, max_rows=8 * 9 * 32)
    # linear steps at this shape (K = 3584 and 18944 take the looped kernel)
    d, F = cfg["d_model"], cfg["d_ffn"]
    g = torch.Generator(device="cuda").manual_seed(9)
    for which, W, K, N in ((B.LIN_QKV, w["layers"][0]["wqkv"], d, (28 + 8) * 128), (B.LIN_DOWN, w["layers"][0]["wdown"], F, d)):
        x = torch.randn(160, K, generator=g, device="cuda").to(torch.bfloat16)
        out = torch.empty(160, N, dtype=torch.float32, device="cuda")
        eng.k_linear(which, 0, x, out)
        err = (out.cpu().double() - x.cpu().double() @ W.double().T).abs().max().item()
        assert err < 5e-4, (which, err)
    prompts = [synth.gen_prompt(cfg, 1005 + i, 512) for i in range(8)]
    both, st = eng.generate(prompts, 32, 32, 8)
    assert st["tokens"] == 8 * 32
    for i in (0, 7):
        solo, _ = eng.generate([prompts[i]], 32, 32, 0)
        assert np.array_equal(both[i], solo[0]), f"sequence {i}"
    sigma = parity_util.operand_noise_floor(cfg, w, prompts[0], 32, torch.float32)
    tol = parity_util.bf16_tolerances(sigma)
    _, _, tot = parity_util.teacher_forced(eng, cfg, w, prompts[0], 32, 32, 8, torch.float32, max_forwards=3,
                                           verbose=False, literal=True, sigma=sigma, **tol)
    print("cfg5 totals", tot, "sigma", sigma)
    assert tot["rms_dlogit"] <= 1.5 * sigma + 2e-3
    eng.close()
