"""Randomised shapes on the tiny fp32 model: sequences per batch, block length (4 .. 64, including
lengths that are no power of two), draft length, generation length with a ragged last block, prompt
lengths from 1 token up, refresh intervals.  Whatever the shape, every decoding variant of the library
(greedy chain, mix-order tree, round across the block boundary, separate KV append, dual cache) must
generate exactly the tokens of its own stepwise run on the GPU, sequence by sequence."""
import random

import numpy as np
import pytest

from paper_2510_04147_amd import synth

pytestmark = pytest.mark.gpu


def test_every_variant_equals_stepwise_on_random_shapes():
    from paper_2510_04147_amd import binding
    cfg = synth.model_config("tiny")
    wg = synth.gen_weights(cfg, 0, device="cuda")
    rng = random.Random(7)
    for it in range(30):
        nseq = rng.choice([1, 1, 2, 3])
        block = rng.choice([4, 8, 13, 16, 32, 64])
        maxd = rng.choice([1, 3, 4, 8])
        gen = min(rng.randrange(1, 4 * block + 1), 150)
        plens = [rng.randrange(1, 90) for _ in range(nseq)]
        N = rng.randrange(0, maxd + 1)
        R = rng.choice([0, 1, 3, 8, 11, 40])
        case = dict(it=it, nseq=nseq, block=block, max_draft=maxd, gen=gen, prompts=plens, N=N, refresh=R)
        max_rows = max(nseq * max(maxd + 2, 2 * maxd) * block, sum(p + gen for p in plens))
        # every other case: a context exactly as long as its longest sequence (the cache ends inside a tile)
        eng = binding.SSD(cfg, wg, max_seqs=nseq, max_seq_len=max(plens) + gen + (8 if it % 2 else 0), block=block,
                          max_draft=maxd, max_rows=max_rows)
        try:
            prompts = [synth.gen_prompt(cfg, 1000 * it + i, p) for i, p in enumerate(plens)]
            base = np.stack([eng.generate([p], gen, block, 0)[0][0] for p in prompts])
            for name, tree, cross, fuse in (("chain", 0, 0, 1), ("mix-order", 1, 0, 1), ("cross-block", 0, 1, 1),
                                            ("separate append", 0, 0, 0)):
                eng.set_tree_mode(tree)
                eng.set_cross_block(cross)
                eng.set_boundary_fusion(fuse)
                out, st = eng.generate(prompts, gen, block, N)
                assert np.array_equal(out, base) and st["tokens"] == gen * nseq, (name, case)
            eng.set_tree_mode(0)
            eng.set_cross_block(0)
            eng.set_boundary_fusion(1)
            eng.set_cache_mode(1, R)
            base_d = np.stack([eng.generate([p], gen, block, 0)[0][0] for p in prompts])
            out, st = eng.generate(prompts, gen, block, N)
            assert np.array_equal(out, base_d) and st["tokens"] == gen * nseq, ("dual cache", case)
        finally:
            eng.close()


def test_sixteen_sequences_at_once():
    """The largest batch a context holds (16 slots): block boundaries, rounds across them and cache refreshes
    of many sequences share forwards (up to three descriptor groups per sequence), and every sequence still
    gets the tokens of its solo stepwise run."""
    from paper_2510_04147_amd import binding
    cfg = synth.model_config("tiny")
    wg = synth.gen_weights(cfg, 0, device="cuda")
    nseq, block, N, gen = 16, 8, 3, 24
    plens = [5 + 3 * i for i in range(nseq)]
    prompts = [synth.gen_prompt(cfg, 4000 + i, p) for i, p in enumerate(plens)]
    eng = binding.SSD(cfg, wg, max_seqs=nseq, max_seq_len=max(plens) + gen + 8, block=block, max_draft=N,
                      max_rows=max(nseq * (N + 2) * block, sum(p + gen for p in plens)))
    try:
        base = np.stack([eng.generate([p], gen, block, 0)[0][0] for p in prompts])
        for cross in (0, 1):
            eng.set_cross_block(cross)
            out, st = eng.generate(prompts, gen, block, N)
            assert np.array_equal(out, base) and st["tokens"] == nseq * gen, cross
        eng.set_cross_block(0)
        eng.set_cache_mode(1, 8)
        base_d = np.stack([eng.generate([p], gen, block, 0)[0][0] for p in prompts])
        out, st = eng.generate(prompts, gen, block, N)
        assert np.array_equal(out, base_d) and st["kv_passes"] == nseq * gen // 8
    finally:
        eng.close()
