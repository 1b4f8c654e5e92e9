"""The acceptance kernel alone (a11) against the oracle's tree walks, through the kernel-level entry
point ssd_k_accept: hand-steered and random confidences / arg-maxes with many ties, every match
length, out-of-order drafts, short blocks, both tree shapes, two sequences per call.  Integer work:
every output must be bit-exact."""
import numpy as np
import pytest
import torch

from oracle import decode
from paper_2510_04147_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def eng():
    from paper_2510_04147_amd import binding
    cfg = synth.model_config("tiny")
    wg = synth.gen_weights(cfg, 0, device="cuda")
    e = binding.SSD(cfg, wg, max_seqs=2, max_seq_len=256, block=64, max_draft=8, max_rows=2 * 16 * 64)
    yield e
    e.close()


def make_case(rng, bl, N, mode, steer):
    """One sequence: block state, drafts and per-node (conf, arg) rows in the forward's node order."""
    V = 50
    n_masked = int(rng.integers(1, bl + 1))
    mpos = sorted(rng.permutation(bl)[:n_masked].tolist())
    masked = [p in mpos for p in range(bl)]
    tok = [int(rng.integers(0, V)) for _ in range(bl)]
    nd = int(min(N, n_masked - 1, rng.integers(0, N + 1)))
    drafts = [(int(p), int(rng.integers(0, V))) for p in rng.permutation(mpos)[:nd]]
    build = decode.build_mix_order if mode == 1 else decode.build_chain
    nodes = build(tok, masked, drafts)
    conf = rng.integers(0, 6, size=(len(nodes), bl)).astype(np.float32) / 8.0          # few levels: many ties
    arg = rng.integers(0, V, size=(len(nodes), bl)).astype(np.int32)
    if steer and nd > 0:
        stop = int(rng.integers(0, nd + 1))                     # the chain verifies `stop` drafts
        for m in range(min(stop, nd)):
            q, t = drafts[m]
            conf[m, q], arg[m, q] = 0.95, t
        if stop < nd:
            kind = int(rng.integers(0, 3))
            if kind == 0 and stop + 1 < nd:                     # out of order: the next-but-one draft wins
                q, t = drafts[stop + 1]
                conf[stop, q], arg[stop, q] = 0.97, t
            elif kind == 1:                                      # right position, wrong token
                q, t = drafts[stop]
                conf[stop, q], arg[stop, q] = 0.97, (t + 1) % V
    return dict(tok=tok, masked=masked, drafts=drafts, nodes=nodes, conf=conf, arg=arg)


def expected(case, mode, n_next):
    t = [torch.from_numpy(r) for r in case["arg"]]
    c = [torch.from_numpy(r.astype(np.float64)) for r in case["conf"]]
    mk = [m for _, m in case["nodes"]]
    walk = decode.accept_mix_order if mode == 1 else decode.accept_chain
    acc, nxt, _ = walk(t, c, mk, case["drafts"], n_next)
    return acc, nxt


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("bl", [64, 32, 17, 1])
def test_acceptance_kernel_matches_the_oracle_walk(eng, mode, bl):
    rng = np.random.default_rng(1000 * mode + bl)
    eng.set_tree_mode(mode)
    try:
        rescued = 0
        for it in range(60):
            N = int(rng.integers(0, 9))
            n_next = int(rng.integers(0, 9))
            cases = [make_case(rng, bl, N, mode, steer=it % 3 != 0) for _ in range(1 + it % 2)]
            conf = torch.from_numpy(np.concatenate([c["conf"].reshape(-1) for c in cases])).cuda()
            arg = torch.from_numpy(np.concatenate([c["arg"].reshape(-1) for c in cases])).cuda()
            out = eng.new_out(len(cases))
            masks = [sum(1 << p for p, m in enumerate(c["masked"]) if m) for c in cases]
            eng.k_accept(list(range(len(cases))), [c["tok"] for c in cases], masks, [c["drafts"] for c in cases],
                         n_next, conf, arg, out, block_len=[bl] * len(cases))
            got = out.host()
            for i, c in enumerate(cases):
                acc, nxt = expected(c, mode, n_next)
                n = int(got["n_accept"][i])
                assert list(zip(got["acc_pos"][i][:n].tolist(), got["acc_tok"][i][:n].tolist())) == acc, (it, i)
                k = int(got["n_next"][i])
                assert list(zip(got["next_pos"][i][:k].tolist(), got["next_tok"][i][:k].tolist())) == nxt, (it, i)
                chain_len = len(decode.accept_chain([torch.from_numpy(r) for r in c["arg"]][:len(c["drafts"]) + 1],
                                                    [torch.from_numpy(r.astype(np.float64)) for r in c["conf"]][:len(c["drafts"]) + 1],
                                                    [m for _, m in c["nodes"]][:len(c["drafts"]) + 1], c["drafts"], n_next)[0])
                rescued += len(acc) > chain_len
        if mode == 1 and bl >= 17:
            assert rescued > 0, "no out-of-order case was exercised"
    finally:
        eng.set_tree_mode(0)
