"""The benchmark configuration at full size (32 layers of the 8B shape, prompt 256, block 32,
draft depth 4) in the launch configuration bench.py times: GPU SSD == GPU stepwise bit for bit
over two blocks, and every forward of the first block (the block-start draft and all its
verification forwards), teacher forced against the exact fp32 oracle, which computes them one by one
(the oracle receives the weights already widened to fp32, the same values, so that it does not widen
15 GB per forward)."""
import time
import numpy as np
import pytest
import torch

import parity_util
from paper_2510_04147_amd import synth

pytestmark = pytest.mark.gpu


def test_cfg2_full_depth():
    from paper_2510_04147_amd import binding
    wl = synth.WORKLOADS["cfg2_8b_b32_n4"]
    cfg = synth.model_config(wl["model"])
    wg = synth.gen_weights(cfg, 0, device="cuda")
    B, N, P = wl["block"], wl["draft"], wl["prompt_len"]
    eng = binding.SSD(cfg, wg, max_seqs=1, max_seq_len=P + 256, block=B, max_draft=N, max_rows=max(P + 2 * B, (N + 2) * B))
    prompt = synth.gen_prompt(cfg, wl["seed"], P)
    print("generate: stepwise and SSD, two blocks", flush=True)
    base, s0 = eng.generate([prompt], 2 * B, B, 0)
    out, s4 = eng.generate([prompt], 2 * B, B, N)
    assert np.array_equal(out, base), "GPU SSD differs from GPU stepwise at full depth"
    assert s0["forwards"] == 2 * B and s4["forwards"] <= 2 * B
    print("accept_hist", s4["accept_hist"][:N + 2], flush=True)
    # the variants of the decoding loop at full depth: same tokens
    eng.set_cross_block(1)
    out_x, sx = eng.generate([prompt], 2 * B, B, N)
    eng.set_cross_block(0)
    assert np.array_equal(out_x, base) and sx["forwards"] <= s4["forwards"], "round across the block boundary"
    eng.set_tree_mode(1)
    out_m, _ = eng.generate([prompt], 2 * B, B, N)
    eng.set_tree_mode(0)
    assert np.array_equal(out_m, base), "mix-order tree"
    # the dual cache is another model function: SSD against its own stepwise run (320-row refresh forwards)
    eng.set_cache_mode(1, 8)
    base_d, sd0 = eng.generate([prompt], 2 * B, B, 0)
    out_d, sd4 = eng.generate([prompt], 2 * B, B, N)
    eng.set_spill_over(1)
    out_s, sds = eng.generate([prompt], 2 * B, B, N)
    eng.set_spill_over(0)
    eng.set_cache_mode(0)
    assert np.array_equal(out_s, base_d) and sds["forwards"] <= sd4["forwards"], "spill-over with the dual cache"
    assert np.array_equal(out_d, base_d) and sd0["kv_passes"] == sd4["kv_passes"] == 2 * B // 8
    print("dual cache forwards", sd4["forwards"], "of", sd0["forwards"], flush=True)
    print("copying weights to the host for the oracle", flush=True)
    w = synth.weights_to(wg, "cpu")
    w = {k: (v.float() if k != "layers" else [{n: t.float() for n, t in lw.items()} for lw in v]) for k, v in w.items()}
    print("oracle: operand noise floor (4 layer-stack passes)", flush=True)
    t0 = time.time()
    sigma = parity_util.operand_noise_floor(cfg, w, prompt, B, torch.float32)
    tol = parity_util.bf16_tolerances(sigma)
    print(f"sigma = {sigma:.4f} ({time.time() - t0:.0f} s); oracle SSD for the whole first block", flush=True)
    t0 = time.time()
    _, st, tot = parity_util.teacher_forced(eng, cfg, w, prompt, B, B, N, torch.float32, max_blocks=1, sigma=sigma, **tol)
    print(f"full-size totals ({time.time() - t0:.0f} s)", tot, flush=True)
    assert tot["forwards"] == st["forwards"] >= B // (N + 1) and tot["rows"] >= 10 * B
    assert tot["rms_dlogit"] <= 1.5 * sigma + 2e-3
    eng.close()
