"""A small bf16 model with head size 64 and grouped-query attention (8 query / 2 KV heads, d = 512,
FFN 1536, vocabulary 2080 = 65 tiles of 32, 3 layers): the MFMA attention kernel's 64-channel instantiation, the
KV-head placement for head counts that are no multiple of 8, GEMMs with short K (8 and 24 chunks)
and a narrow LM head, none of which the 8B / 7B shapes reach.  Teacher forced against the oracle
with the bf16 tolerances, and every decoding variant against its stepwise run, bit for bit."""
import numpy as np
import pytest
import torch

import parity_util
from paper_2510_04147_amd import synth

pytestmark = pytest.mark.gpu


def test_head_size_64_gqa_bf16():
    from paper_2510_04147_amd import binding
    cfg = synth.model_config("tiny", dtype="bf16", n_layers=3, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=64,
                             d_ffn=1536, vocab=2080)     # 65 vocabulary tiles: the last LM-head work-group is partly empty
    wg = synth.gen_weights(cfg, 11, device="cuda", std=0.05)
    w = synth.weights_to(wg, "cpu")
    eng = binding.SSD(cfg, wg, max_seqs=2, max_seq_len=256, block=32, max_draft=4, max_rows=2 * 8 * 32)
    try:
        prompt = synth.gen_prompt(cfg, 21, 45)
        sigma = parity_util.operand_noise_floor(cfg, w, prompt, 32, torch.float32)
        tol = parity_util.bf16_tolerances(sigma)
        for path in (1, 0):                                  # MFMA kernels, then the plain kernels on the same model
            eng.set_kernel_path(path)
            ref, st, tot = parity_util.teacher_forced(eng, cfg, w, prompt, 64, 32, 4, torch.float32, verbose=False,
                                                      literal=path == 1, sigma=sigma, **tol)
            print(f"path {path}: sigma {sigma:.4f}", tot)
            assert tot["forwards"] == st["forwards"] and tot["rms_dlogit"] <= 1.5 * sigma + 2e-3
            assert tot["tok_exempt"] <= 0.10 * tot["rows"]
        eng.set_kernel_path(1)
        ref, st, tot = parity_util.teacher_forced_dual(eng, cfg, w, prompt, 48, 8, 3, 8, torch.float32, verbose=False, **tol)
        assert tot["rms_dlogit"] <= 1.5 * sigma + 2e-3 and tot["refreshes"] >= 6
        p2 = synth.gen_prompt(cfg, 22, 70)
        for blk in (8, 32, 20):
            base = np.stack([eng.generate([p], 60, blk, 0)[0][0] for p in (prompt, p2)])
            for tree, cross in ((0, 0), (1, 0), (0, 1)):
                eng.set_tree_mode(tree)
                eng.set_cross_block(cross)
                out, _ = eng.generate([prompt, p2], 60, blk, 4)
                assert np.array_equal(out, base), (blk, tree, cross)
            eng.set_tree_mode(0)
            eng.set_cross_block(0)
            eng.set_cache_mode(1, 8)
            base_d = np.stack([eng.generate([p], 60, blk, 0)[0][0] for p in (prompt, p2)])
            out, _ = eng.generate([prompt, p2], 60, blk, 4)
            eng.set_cache_mode(0)
            assert np.array_equal(out, base_d), ("dual", blk)
    finally:
        eng.close()


def test_shapes_that_do_not_tile_fall_back_per_projection():
    """FFN width 1544 and vocabulary 2075 fit no MFMA tile: the gate/up, down and LM-head projections of this
    bf16 model take the plain kernels while QKV and the attention output stay on the matrix cores, inside one
    forward.  Same checks: the oracle teacher forced, and SSD against stepwise bit for bit."""
    from paper_2510_04147_amd import binding
    cfg = synth.model_config("tiny", dtype="bf16", n_layers=2, d_model=512, n_q_heads=8, n_kv_heads=4, head_dim=64,
                             d_ffn=1544, vocab=2075)
    wg = synth.gen_weights(cfg, 12, device="cuda", std=0.05)
    w = synth.weights_to(wg, "cpu")
    eng = binding.SSD(cfg, wg, max_seqs=1, max_seq_len=256, block=16, max_draft=3, max_rows=6 * 16 + 64)
    try:
        prompt = synth.gen_prompt(cfg, 23, 37)
        sigma = parity_util.operand_noise_floor(cfg, w, prompt, 16, torch.float32)
        tol = parity_util.bf16_tolerances(sigma)
        ref, st, tot = parity_util.teacher_forced(eng, cfg, w, prompt, 40, 16, 3, torch.float32, verbose=False, **tol)
        print(f"sigma {sigma:.4f}", tot)
        assert tot["forwards"] == st["forwards"] and tot["rms_dlogit"] <= 1.5 * sigma + 2e-3
        base, _ = eng.generate([prompt], 40, 16, 0)
        for cross, dual in ((0, 0), (1, 0)):
            eng.set_cross_block(cross)
            out, _ = eng.generate([prompt], 40, 16, 3)
            assert np.array_equal(out, base), cross
        eng.set_cross_block(0)
        eng.set_cache_mode(1, 8)
        base_d, _ = eng.generate([prompt], 40, 16, 0)
        out, _ = eng.generate([prompt], 40, 16, 3)
        assert np.array_equal(out, base_d)
    finally:
        eng.close()
