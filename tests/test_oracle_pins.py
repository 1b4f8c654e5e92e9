"""Pins for the CPU oracle: what the paper and the mathematics fix, none of it
computed by the HIP path.  Runs without a GPU."""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import decode, model
from paper_2510_04147_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))


def small_cfg(**kw):
    base = dict(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=97)
    base.update(kw)
    return synth.model_config("tiny", **base)


@pytest.fixture(scope="module")
def tiny():
    cfg = synth.model_config("tiny")
    return cfg, synth.gen_weights(cfg, 0)


# ---------------------------------------------------------------- losslessness
@pytest.mark.parametrize("seed,gen_len,block", [(1001, 64, 32), (7, 50, 32), (8, 40, 8)])
def test_ssd_is_token_identical_to_stepwise(tiny, seed, gen_len, block):
    """Abstract / Section 4.2: SSD output is identical to stepwise decoding."""
    cfg, w = tiny
    prompt = synth.gen_prompt(cfg, seed, 48)
    ref, sref = decode.stepwise(w, cfg, prompt, gen_len, block)
    assert sref["forwards"] == gen_len            # one token per forward
    for N in range(0, 9):
        out, st = decode.ssd(w, cfg, prompt, gen_len, block, N)
        assert out == ref, f"N={N}"
        hist = st["accept_hist"]
        assert hist[0] == 0 and sum(a * h for a, h in enumerate(hist)) == gen_len
        assert all(h == 0 for a, h in enumerate(hist) if a > N + 1)   # at most N+1 per forward
        if N == 0:
            assert st["forwards"] == sref["forwards"]
        # Section 5.1: step reduction can never exceed N/(N+1)
        assert 1.0 - st["forwards"] / gen_len <= N / (N + 1) + 1e-12


def test_gqa_and_odd_shapes_lossless():
    cfg = small_cfg()
    w = synth.gen_weights(cfg, 3, std=0.2)
    prompt = synth.gen_prompt(cfg, 5, 11)
    ref, _ = decode.stepwise(w, cfg, prompt, 21, 8)
    for N in (1, 3, 5):
        out, _ = decode.ssd(w, cfg, prompt, 21, 8, N)
        assert out == ref


def test_bruteforce_without_cache_matches_cached_stepwise():
    """The exact prefix cache changes nothing: recomputing the whole sequence
    under the block-causal mask for every token gives the same tokens."""
    cfg = small_cfg()
    w = synth.gen_weights(cfg, 11, std=0.2)
    prompt = synth.gen_prompt(cfg, 12, 9)
    a, sa = decode.stepwise(w, cfg, prompt, 20, 8)
    b, sb = decode.bruteforce(w, cfg, prompt, 20, 8)
    assert a == b and sa["forwards"] == sb["forwards"] == 20


def test_bruteforce_tiny_config_first_block(tiny):
    cfg, w = tiny
    prompt = synth.gen_prompt(cfg, 1001, 64)
    a, _ = decode.stepwise(w, cfg, prompt, 16, 8)
    b, _ = decode.bruteforce(w, cfg, prompt, 16, 8)
    assert a == b


# ------------------------------------------------- zero-attention closed form
def _golden_upper_bounds():
    rows = {}
    with open(os.path.join(HERE, "golden", "upper_bound.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                n, pct = line.split()
                rows[int(n)] = float(pct)
    return rows


@pytest.mark.parametrize("N", [0, 1, 3, 4, 5, 8])
def test_zero_attention_model_reaches_upper_bound(tiny, N):
    """With every attention output projection zero a position's logits depend on
    its own token only: all masked positions tie, decoding runs left to right,
    every draft is verified.  Each verification then accepts N_eff+1 tokens and a
    block of B tokens costs 1 + ceil((B-1)/(N+1)) forwards."""
    cfg, w0 = tiny
    w = dict(w0)
    w["layers"] = [dict(lw, wo=torch.zeros_like(lw["wo"])) for lw in w0["layers"]]
    prompt = synth.gen_prompt(cfg, 3, 20)
    B, gen = 32, 64
    trace = []
    out, st = decode.ssd(w, cfg, prompt, gen, B, N, trace=trace)
    assert len(set(out)) == 1                        # same token everywhere
    assert st["forwards"] == (gen // B) * (1 + math.ceil((B - 1) / (N + 1)))
    ref, _ = decode.stepwise(w, cfg, prompt, gen, B)
    assert out == ref
    for rec in trace:
        assert len(rec["accepted"]) == len(rec["drafts"]) + 1      # everything verified
        pos = [p for p, _ in rec["accepted"]]
        assert pos == sorted(pos) and pos[0] == rec["masked"].index(True)   # left to right
    # full-depth verification rounds sit exactly on the paper's bound N/(N+1)
    full = [rec for rec in trace if len(rec["drafts"]) == N]
    if N in _golden_upper_bounds():
        toks = sum(len(r["accepted"]) for r in full)
        assert round(100.0 * (1 - len(full) / toks), 1) == _golden_upper_bounds()[N]


# ------------------------------------------------------ transformer arithmetic
def _library_forward(w, cfg, tokens, seg):
    """The same network written with torch's own routines (rms_norm, linear,
    scaled_dot_product_attention, silu) and complex-number rotary embedding."""
    dt = torch.float64
    Hq, Hkv, dh, Fd = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"], cfg["d_ffn"]
    tokens = torch.as_tensor(tokens, dtype=torch.long)
    seg = torch.as_tensor(seg)
    n = len(tokens)
    allowed = seg[None, :] <= seg[:, None]
    freqs = 1.0 / (cfg["rope_theta"] ** (torch.arange(0, dh, 2, dtype=dt) / dh))
    rot = torch.polar(torch.ones(n, dh // 2, dtype=dt), torch.arange(n, dtype=dt)[:, None] * freqs)

    def rotary(x):                      # x [n, H, dh]; pairs (i, i+dh/2)
        z = torch.complex(x[..., : dh // 2], x[..., dh // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], -1)

    h = F.embedding(tokens, w["embed"].to(dt))
    for lw in w["layers"]:
        x = F.rms_norm(h, (h.shape[-1],), lw["norm1"].to(dt), cfg["rms_eps"])
        qkv = F.linear(x, lw["wqkv"].to(dt))
        q, k, v = qkv.split([Hq * dh, Hkv * dh, Hkv * dh], dim=-1)
        q = rotary(q.view(n, Hq, dh)).transpose(0, 1)
        k = rotary(k.view(n, Hkv, dh)).transpose(0, 1).repeat_interleave(Hq // Hkv, dim=0)
        v = v.view(n, Hkv, dh).transpose(0, 1).repeat_interleave(Hq // Hkv, dim=0)
        a = F.scaled_dot_product_attention(q, k, v, attn_mask=allowed)
        h = h + F.linear(a.transpose(0, 1).reshape(n, Hq * dh), lw["wo"].to(dt))
        x = F.rms_norm(h, (h.shape[-1],), lw["norm2"].to(dt), cfg["rms_eps"])
        g, u = F.linear(x, lw["wgu"].to(dt)).split([Fd, Fd], dim=-1)
        h = h + F.linear(F.silu(g) * u, lw["wdown"].to(dt))
    h = F.rms_norm(h, (h.shape[-1],), w["final_norm"].to(dt), cfg["rms_eps"])
    return F.linear(h, w["lm_head"].to(dt))


def test_forward_matches_torch_library_routines():
    cfg = small_cfg()
    w = synth.gen_weights(cfg, 21, std=0.3)
    for lw in w["layers"]:                     # non-trivial gains so a dropped gain shows
        lw["norm1"] = 0.5 + torch.rand(cfg["d_model"])
        lw["norm2"] = 0.5 + torch.rand(cfg["d_model"])
    w["final_norm"] = 0.5 + torch.rand(cfg["d_model"])
    toks = synth.gen_prompt(cfg, 22, 19)
    seg = [0] * 7 + [1] * 6 + [2] * 6
    want = _library_forward(w, cfg, toks, seg)
    # (a) cache-free masked evaluation
    got = model.forward_full_blockcausal(w, cfg, toks, seg)
    assert torch.allclose(got, want, rtol=1e-10, atol=1e-10)
    # (b) segment-by-segment with the prefix cache
    cache = model.KVCache(cfg["n_layers"])
    pos = 0
    for s in (0, 1, 2):
        rows = [i for i, x in enumerate(seg) if x == s]
        lg, kv = model.forward_segment(w, cfg, toks[rows], pos, cache)
        assert torch.allclose(lg, want[rows], rtol=1e-10, atol=1e-10)
        cache.append(kv)
        pos += len(rows)


def test_attention_against_python_loops():
    torch.manual_seed(0)
    n, m, Hq, Hkv, dh = 3, 5, 4, 2, 4
    q, k, v = torch.randn(n, Hq, dh, dtype=torch.float64), torch.randn(m, Hkv, dh, dtype=torch.float64), \
        torch.randn(m, Hkv, dh, dtype=torch.float64)
    got = model.attention(q, k, v)
    for h in range(Hq):
        g = h // (Hq // Hkv)
        for i in range(n):
            s = [sum(float(q[i, h, x]) * float(k[j, g, x]) for x in range(dh)) / math.sqrt(dh) for j in range(m)]
            z = sum(math.exp(x) for x in s)
            for x in range(dh):
                want = sum(math.exp(s[j]) / z * float(v[j, g, x]) for j in range(m))
                assert abs(float(got[i, h, x]) - want) < 1e-12


def test_rope_identity_norm_and_shift_invariance():
    torch.manual_seed(1)
    q = torch.randn(6, 2, 16, dtype=torch.float64)
    k = torch.randn(6, 2, 16, dtype=torch.float64)
    zero = torch.zeros(6, dtype=torch.long)
    assert torch.equal(model.rope(q, zero, 10000.0), q)                 # position 0 = identity
    pos = torch.tensor([0, 1, 5, 17, 100, 1000])
    rq = model.rope(q, pos, 10000.0)
    assert torch.allclose(rq.norm(dim=-1), q.norm(dim=-1), rtol=1e-12)  # a rotation
    # <rope(q,a), rope(k,b)> depends on a-b only
    d1 = (model.rope(q, pos, 1e4) * model.rope(k, pos + 3, 1e4)).sum(-1)
    d2 = (model.rope(q, pos + 40, 1e4) * model.rope(k, pos + 43, 1e4)).sum(-1)
    assert torch.allclose(d1, d2, rtol=1e-9, atol=1e-9)
    # first pair rotates by exactly `pos` radians (frequency theta^0 = 1), counter-clockwise
    e = torch.zeros(1, 1, 16, dtype=torch.float64)
    e[0, 0, 0] = 1.0
    r = model.rope(e, torch.tensor([2]), 1e4)
    assert abs(float(r[0, 0, 0]) - math.cos(2.0)) < 1e-15 and abs(float(r[0, 0, 8]) - math.sin(2.0)) < 1e-15


def test_rms_norm_and_silu_closed_forms():
    x = torch.tensor([[3.0, -4.0, 0.0, 0.0]], dtype=torch.float64)      # mean square = 25/4
    y = model.rms_norm(x, torch.tensor([1.0, 2.0, 1.0, 1.0]), 0.0)
    assert torch.allclose(y, torch.tensor([[1.2, -3.2, 0.0, 0.0]], dtype=torch.float64))
    assert abs(float(model.silu(torch.tensor(0.0, dtype=torch.float64)))) == 0.0
    z = torch.tensor(1.5, dtype=torch.float64)
    assert abs(float(model.silu(z)) - 1.5 / (1 + math.exp(-1.5))) < 1e-15


# ------------------------------------------------------------ confidence, ties
def test_predict_matches_softmax_and_excludes_mask_token():
    torch.manual_seed(2)
    V, mask_id = 50, 49
    lg = torch.randn(7, V, dtype=torch.float64)
    lg[3, mask_id] = 100.0                       # the mask token would win: must be ignored
    lg[5, 10] = lg[5, 20] = 9.0                  # exact tie -> lowest id
    t, m, c, margin = decode.predict(lg, mask_id)
    sm = torch.softmax(lg[:, :mask_id], dim=-1)
    assert torch.equal(t, sm.argmax(-1)) or int(t[5]) == 10
    assert int(t[5]) == 10 and float(margin[5]) == 0.0
    assert int(t[3]) != mask_id
    assert torch.allclose(c, sm.max(-1).values, rtol=1e-12)
    assert torch.allclose(m, lg[:, :mask_id].max(-1).values)
    assert bool(((c > 1.0 / V) & (c <= 1.0)).all())


def test_zero_lm_head_gives_uniform_confidence_and_left_to_right(tiny):
    cfg, w0 = tiny
    w = dict(w0, lm_head=torch.zeros_like(w0["lm_head"]))
    prompt = synth.gen_prompt(cfg, 9, 8)
    trace = []
    out, _ = decode.ssd(w, cfg, prompt, 8, 8, 3, trace=trace)
    assert out == [0] * 8                         # all logits equal -> lowest token id
    for rec in trace:
        for c, mk in zip(rec["c"], [rec["masked"]]):
            assert torch.allclose(c, torch.full_like(c, 1.0 / (cfg["vocab"] - 1)))


# ---------------------------------------------------- acceptance on hand-made data
def _mk(nodes_conf, nodes_tok):
    return [torch.tensor(x, dtype=torch.float64) for x in nodes_conf], [torch.tensor(x) for x in nodes_tok]


def test_accept_chain_every_match_length():
    # block of 5, position 4 already decoded; drafts in priority order: (2,'7'), (0,'8'), (3,'9')
    drafts = [(2, 7), (0, 8), (3, 9)]
    root_masked = [True, True, True, True, False]
    masked = [root_masked]
    for q, _ in drafts:
        mk = list(masked[-1]); mk[q] = False; masked.append(mk)
    good_c = [[.1, .2, .9, .3, 0], [.8, .2, 0, .3, 0], [0, .2, 0, .7, 0], [0, .6, 0, 0, 0]]
    good_t = [[8, 5, 7, 9, 0], [8, 5, 0, 9, 0], [0, 5, 0, 9, 0], [0, 6, 0, 0, 0]]
    for stop in range(4):                          # break the chain at node `stop`
        c = [list(r) for r in good_c]; t = [list(r) for r in good_t]
        if stop < 3:
            t[stop][drafts[stop][0]] = 99          # right position, wrong token
        cc, tt = _mk(c, t)
        acc, nxt, m = decode.accept_chain(tt, cc, masked, drafts, 3)
        assert m == stop and len(acc) == stop + 1
        assert acc[:stop] == drafts[:stop]
        assert acc[-1] == ((drafts[stop][0], 99) if stop < 3 else (1, 6))
        left = [p for p, mk in enumerate(masked[stop]) if mk and p != acc[-1][0]]
        assert [q for q, _ in nxt] == sorted(left, key=lambda p: (-c[stop][p], p))[:max(len(left) - 1, 0)]
    # right token at the wrong position (generation order differs): no match either
    c = [list(r) for r in good_c]; t = [list(r) for r in good_t]
    c[0][3] = .95; t[0][3] = 7
    cc, tt = _mk(c, t)
    acc, nxt, m = decode.accept_chain(tt, cc, masked, drafts, 3)
    assert m == 0 and acc == [(3, 7)]


def test_accept_chain_ties_and_last_token_of_block():
    # equal confidences: the lowest position wins
    cc, tt = _mk([[.5, .5, .5]], [[4, 5, 6]])
    acc, nxt, m = decode.accept_chain(tt, cc, [[True, True, True]], [], 4)
    assert acc == [(0, 4)] and nxt == [(1, 5)]     # 2 left -> only 1 draft (leaf keeps one)
    # one masked position left: a single node, no drafts, nothing to draft next
    cc, tt = _mk([[0, .3, 0]], [[0, 8, 0]])
    acc, nxt, m = decode.accept_chain(tt, cc, [[False, True, False]], [], 4)
    assert acc == [(1, 8)] and nxt == [] and m == 0
    # fewer drafts than the draft length: the chain is just shorter
    cc, tt = _mk([[.9, .1, 0], [0, .4, 0]], [[3, 2, 0], [0, 2, 0]])
    acc, nxt, m = decode.accept_chain(tt, cc, [[True, True, False], [False, True, False]], [(0, 3)], 8)
    assert m == 1 and acc == [(0, 3), (1, 2)] and nxt == []


# --------------------------------------------------------------- mix-order tree
def test_mix_order_tree_shape():
    """Section 5.2 / Table 3: the N+1 chain nodes plus one node per non-leaf chain node that skips
    the next draft: 2N nodes (6 / 8 / 10 for N = 3 / 4 / 5); the extra node of m holds drafts
    1..m and m+2."""
    tok, masked = [9] * 8, [True] * 8
    for N, size in ((1, 2), (2, 4), (3, 6), (4, 8), (5, 10)):
        drafts = [(p, 20 + p) for p in range(N)]
        nodes = decode.build_mix_order(tok, masked, drafts)
        assert len(nodes) == size == max(2 * N, N + 1)
        assert nodes[:N + 1] == decode.build_chain(tok, masked, drafts)
        for m in range(N - 1):
            t, mk = nodes[N + 1 + m]
            placed = [p for p in range(8) if not mk[p]]
            assert placed == sorted([q for q, _ in drafts[:m]] + [drafts[m + 1][0]])
            assert all(t[q] == 20 + q for q in placed) and t[drafts[m][0]] == 9
    assert decode.build_mix_order(tok, masked, []) == decode.build_chain(tok, masked, [])


def test_accept_mix_order_by_hand():
    """Drafts (2,'7'), (0,'8'), (3,'9') on a block of 5 (position 4 decoded).  Node 0 prefers
    position 0 with token 8 = the second draft: greedy accepts one token, mix order accepts the
    second draft and the choice of the node that holds it."""
    drafts = [(2, 7), (0, 8), (3, 9)]
    root = [True, True, True, True, False]
    chain = [root]
    for q, _ in drafts:
        mk = list(chain[-1]); mk[q] = False; chain.append(mk)
    extra0 = [False, True, True, True, False]              # draft 2 only
    extra1 = [True, True, False, False, False]             # draft 1 and draft 3
    masked = chain + [extra0, extra1]
    c = [[.9, .2, .8, .3, 0], [.8, .2, 0, .3, 0], [0, .2, 0, .7, 0], [0, .6, 0, 0, 0],
         [0, .1, .4, .5, 0], [.2, .3, 0, 0, 0]]
    t = [[8, 5, 7, 9, 0], [8, 5, 0, 9, 0], [0, 5, 0, 9, 0], [0, 6, 0, 0, 0],
         [0, 5, 7, 4, 0], [1, 2, 0, 0, 0]]
    cc, tt = _mk(c, t)
    acc, nxt, last = decode.accept_mix_order(tt, cc, masked, drafts, 3)
    assert acc == [(0, 8), (3, 4)] and last == 4            # out-of-order draft + its node's choice
    assert nxt == [(2, 7)]                                  # masked {1, 2} left, the leaf keeps one
    g_acc, _, g_m = decode.accept_chain(tt[:4], cc[:4], masked[:4], drafts, 3)
    assert g_acc == [(0, 8)] and g_m == 0                   # the greedy chain stops at the root
    # in-order drafts: identical to the chain walk
    c[0] = [.1, .2, .9, .3, 0]
    cc, tt = _mk(c, t)
    assert decode.accept_mix_order(tt, cc, masked, drafts, 3)[0] == decode.accept_chain(tt[:4], cc[:4], masked[:4], drafts, 3)[0]
    # the skipped draft matches after one verified draft: node 1 prefers draft 3
    c[1] = [.3, .2, 0, .9, 0]
    cc, tt = _mk(c, t)
    acc, nxt, last = decode.accept_mix_order(tt, cc, masked, drafts, 3)
    assert acc == [(2, 7), (3, 9), (1, 2)] and last == 5
    # right token at a position that is no draft: no rescue
    c[0] = [.1, .95, .9, .3, 0]
    cc, tt = _mk(c, t)
    assert decode.accept_mix_order(tt, cc, masked, drafts, 3)[0] == [(1, 5)]


@pytest.mark.parametrize("seed,gen_len,block", [(1001, 64, 32), (8, 40, 8)])
def test_mix_order_is_lossless_and_never_accepts_less_per_round(tiny, seed, gen_len, block):
    """The mix-order tree keeps the output identical to stepwise decoding, accepts at most N+1
    tokens per forward, and from any state accepts at least what the chain accepts."""
    cfg, w = tiny
    prompt = synth.gen_prompt(cfg, seed, 48)
    ref, _ = decode.stepwise(w, cfg, prompt, gen_len, block)
    for N in (1, 2, 3, 5):
        trace = []
        out, st = decode.ssd(w, cfg, prompt, gen_len, block, N, mix_order=True, trace=trace)
        assert out == ref, f"N={N}"
        hist = st["accept_hist"]
        assert hist[0] == 0 and sum(a * h for a, h in enumerate(hist)) == gen_len
        assert all(h == 0 for a, h in enumerate(hist) if a > N + 1)
        for rec in trace:
            n = len(rec["drafts"])
            assert len(rec["t"]) == max(2 * n, n + 1)
            chain_acc, _, _ = decode.accept_chain(rec["t"][:n + 1], rec["c"][:n + 1],
                                                  [mk for _, mk in decode.build_chain(rec["tok"], rec["masked"], rec["drafts"])],
                                                  rec["drafts"], N)
            assert rec["accepted"][:len(chain_acc) - 1] == chain_acc[:-1] and len(rec["accepted"]) >= len(chain_acc)


def test_mix_order_equals_chain_when_every_draft_verifies(tiny):
    """Zero attention output projections: decoding runs left to right and every draft is verified,
    so the extra nodes never fire and the forward count is the chain's closed form."""
    cfg, w0 = tiny
    w = dict(w0)
    w["layers"] = [dict(lw, wo=torch.zeros_like(lw["wo"])) for lw in w0["layers"]]
    prompt = synth.gen_prompt(cfg, 3, 20)
    for N in (3, 4):
        out, st = decode.ssd(w, cfg, prompt, 64, 32, N, mix_order=True)
        assert st["forwards"] == 2 * (1 + math.ceil(31 / (N + 1)))


# ----------------------------------------------------------- across the block boundary
@pytest.mark.parametrize("seed,gen_len,block", [(1001, 64, 32), (8, 40, 8), (7, 50, 16)])
def test_cross_block_round_is_lossless_and_saves_forwards(tiny, seed, gen_len, block):
    """Section 3.2.2: once fewer than N positions remain, candidates come from the next block.  The
    oracle's restricted form (the leaf holds the finished block and predicts the next one) keeps the
    output identical to stepwise decoding and never needs more forwards than the in-block chain."""
    cfg, w = tiny
    prompt = synth.gen_prompt(cfg, seed, 48)
    ref, _ = decode.stepwise(w, cfg, prompt, gen_len, block)
    for N in (1, 2, 4, 8):
        out, st = decode.ssd_cross_block(w, cfg, prompt, gen_len, block, N)
        _, sr = decode.ssd(w, cfg, prompt, gen_len, block, N)
        assert out == ref, f"N={N}"
        hist = st["accept_hist"]
        assert hist[0] == 0 and sum(a * h for a, h in enumerate(hist)) == gen_len
        assert all(h == 0 for a, h in enumerate(hist) if a > N + 1)
        assert st["forwards"] <= sr["forwards"]
        assert 1.0 - st["forwards"] / gen_len <= N / (N + 1) + 1e-12          # Section 5.1's bound still holds
    out0, st0 = decode.ssd_cross_block(w, cfg, prompt, gen_len, block, 0)
    assert out0 == ref and st0["forwards"] == gen_len                          # no drafts: stepwise


@pytest.mark.parametrize("N", [3, 4])
def test_cross_block_closed_form_with_zero_attention(tiny, N):
    """Every draft verifies (zero attention output projections, left-to-right order): each block
    boundary that has a next block costs no forward of its own, so B = 32 takes
    1 + n_blocks * ceil((B - 1) / (N + 1)) forwards instead of n_blocks * (1 + ceil((B - 1) / (N + 1)))."""
    cfg, w0 = tiny
    w = dict(w0)
    w["layers"] = [dict(lw, wo=torch.zeros_like(lw["wo"])) for lw in w0["layers"]]
    prompt = synth.gen_prompt(cfg, 3, 20)
    trace = []
    out, st = decode.ssd_cross_block(w, cfg, prompt, 96, 32, N, trace=trace)
    per_block = math.ceil(31 / (N + 1))
    assert st["forwards"] == 1 + 3 * per_block
    assert decode.ssd(w, cfg, prompt, 96, 32, N)[1]["forwards"] == 3 * (1 + per_block)
    assert out == decode.stepwise(w, cfg, prompt, 96, 32)[0]
    assert st["kv_passes"] == 2              # the prompt and the last block: the others keep their leaf's KV
    assert sum(r["complete"] for r in trace) == 2


def test_build_chain_nodes():
    """Section 3.2.3: exactly N+1 nodes; node i holds the first i drafts."""
    nodes = decode.build_chain([9, 9, 9, 1], [True, True, True, False], [(2, 5), (0, 6)])
    assert len(nodes) == 3
    assert nodes[0] == ([9, 9, 9, 1], [True, True, True, False])
    assert nodes[1] == ([9, 9, 5, 1], [True, True, False, False])
    assert nodes[2] == ([6, 9, 5, 1], [False, True, False, False])


def test_semi_autoregressive_order(tiny):
    """Section 3.1: a block is completed before the next one starts."""
    cfg, w = tiny
    prompt = synth.gen_prompt(cfg, 4, 16)
    trace = []
    decode.ssd(w, cfg, prompt, 24, 8, 4, trace=trace)
    starts = [rec["S"] for rec in trace]
    assert starts == sorted(starts)
    for rec in trace:
        assert all(0 <= p < 8 for p, _ in rec["accepted"])
        assert 1 <= len(rec["accepted"]) <= len(rec["drafts"]) + 1
        assert len(rec["t"]) == len(rec["drafts"]) + 1      # N_eff + 1 nodes


# ------------------------------------------------- dual cache with periodic refresh (Section 4.1)
def test_dual_cache_refreshed_every_token_is_cache_free_decoding():
    """With a refresh before every token nothing cached is ever used: decoding must equal the
    cache-free run that recomputes the whole sequence, future masked blocks included, with full
    bidirectional attention for every token (a separate evaluation path: explicit all-true mask)."""
    cfg = small_cfg()
    w = synth.gen_weights(cfg, 3, std=0.2)
    prompt = synth.gen_prompt(cfg, 5, 11)
    out, st = decode.stepwise_dual(w, cfg, prompt, 20, 8, refresh=1)
    assert st["refreshes"] == st["forwards"] == 20
    assert out == decode.bruteforce_full(w, cfg, prompt, 20, 8)
    # ... and the future blocks do matter: the block-causal decoding of the same model differs
    assert out != decode.stepwise(w, cfg, prompt, 20, 8)[0]


def test_dual_cache_block_forward_right_after_a_refresh_reproduces_it():
    """The keys and values a refresh caches are those of the state it ran on, so computing any block
    of that state against the cache (prefix before it, suffix behind it) must give the refresh's own
    logits for that block.  A suffix or prefix taken at the wrong positions fails this."""
    cfg = small_cfg()
    w = synth.gen_weights(cfg, 4, std=0.2)
    x = list(synth.gen_prompt(cfg, 6, 13)) + [cfg["mask_id"]] * 7 + list(synth.gen_prompt(cfg, 7, 5)) + [cfg["mask_id"]] * 9
    logits, K, V = decode._refresh(w, cfg, x, torch.float64)
    for (pos0, n) in ((13, 7), (0, 13), (20, 5), (25, 9), (3, 30)):
        got = model.forward_block_dual(w, cfg, x[pos0:pos0 + n], pos0, K, V)
        assert torch.allclose(got, logits[pos0:pos0 + n], rtol=0, atol=1e-10), (pos0, n)
    # the suffix is really read: without it the logits change
    Kc = [k[:20] for k in K]
    Vc = [v[:20] for v in V]
    cut = model.forward_block_dual(w, cfg, x[13:20], 13, Kc, Vc)
    assert (cut - logits[13:20]).abs().max() > 1e-6


@pytest.mark.parametrize("refresh", [1, 3, 8, 11, 1000])
def test_ssd_with_dual_cache_is_token_identical_to_stepwise(tiny, refresh):
    """Losslessness does not depend on the cache: with the refresh schedule of Section 4.1 (every
    `refresh` decoded tokens) SSD refreshes at the same states as stepwise decoding."""
    cfg, w = tiny
    prompt = synth.gen_prompt(cfg, 21, 30)
    gen_len, block = 40, 8
    ref, sref = decode.stepwise_dual(w, cfg, prompt, gen_len, block, refresh)
    assert sref["forwards"] == gen_len and sref["refreshes"] == math.ceil(gen_len / min(refresh, gen_len))
    for N in (0, 1, 3, 5):
        out, st = decode.ssd_dual(w, cfg, prompt, gen_len, block, N, refresh)
        assert out == ref, (N, refresh)
        assert st["refreshes"] == sref["refreshes"]
        hist = st["accept_hist"]
        assert hist[0] == 0 and sum(a * h for a, h in enumerate(hist)) == gen_len
        assert st["forwards"] <= gen_len and (N > 0 or st["forwards"] == gen_len)


def test_dual_cache_gqa_ragged_blocks_lossless():
    """Grouped-query attention, a prompt and a generation length that fit no tile, a last block of 5."""
    cfg = small_cfg()
    w = synth.gen_weights(cfg, 3, std=0.2)
    prompt = synth.gen_prompt(cfg, 5, 11)
    for refresh in (3, 8):
        ref, _ = decode.stepwise_dual(w, cfg, prompt, 21, 8, refresh)
        for N in (1, 3, 5):
            out, st = decode.ssd_dual(w, cfg, prompt, 21, 8, N, refresh)
            assert out == ref, (refresh, N)


@pytest.mark.parametrize("N,refresh,block", [(3, 8, 8), (4, 8, 8), (3, 4, 8), (4, 32, 32), (2, 16, 8)])
def test_dual_cache_closed_form_with_zero_attention(tiny, N, refresh, block):
    """Zero attention output projections: no position sees any other, cached or not, every draft
    verifies in left-to-right order.  Between two refreshes (or up to the end of the block, whichever
    comes first) e tokens cost 1 + ceil((e - 1) / (N + 1)) forwards; the paper's setting (refresh =
    block = 8) gives n_blocks * (1 + ceil(7 / (N + 1)))."""
    cfg, w0 = tiny
    w = dict(w0)
    w["layers"] = [dict(lw, wo=torch.zeros_like(lw["wo"])) for lw in w0["layers"]]
    prompt = synth.gen_prompt(cfg, 3, 20)
    gen_len = 64
    out, st = decode.ssd_dual(w, cfg, prompt, gen_len, block, N, refresh)
    assert out == decode.stepwise(w, cfg, prompt, gen_len, block)[0]       # the cache plays no part here
    # the bookkeeping alone, every draft accepted: a block's first forward has no drafts and decodes
    # one token; a chain decodes min(N + 1, tokens left in the block, tokens left until the refresh)
    want, since = 0, refresh
    for _ in range(gen_len // block):
        left, first = block, True
        while left:
            if since >= refresh:
                since, e = 0, 1
            else:
                e = 1 if first else min(N + 1, left, refresh - since)
            want, since, left, first = want + 1, since + e, left - e, False
    assert st["forwards"] == want, (st, want)
    if refresh == block:
        assert want == (gen_len // block) * (1 + math.ceil((block - 1) / (N + 1)))


# ------------------------------------------------- acceptance-rate limit probe (Section 5.1, Table 2)
def test_token_rank_against_a_sort():
    g = torch.Generator().manual_seed(3)
    row = torch.randint(0, 6, (40,), generator=g).double()          # many ties
    mask_id = 17
    order = sorted((v for v in range(40) if v != mask_id), key=lambda v: (-float(row[v]), v))
    for t in (0, 5, 16, 18, 39):
        assert decode.token_rank(row, t, mask_id) == order.index(t)


def test_limit_from_ranks_hand_made():
    """Two rounds of four steps (N = 3) and a last round of two: ranks of the decoded tokens in the
    round's first logits.  k = 1 matches ranks 0 only, k = 2 ranks 0 and 1, ..."""
    rounds = [[0, 0, 1, 3], [0, 2, 0, 0], [0, 0]]
    matched, forwards = decode.limit_from_ranks(rounds, 4)
    assert matched == [2 + 3 + 2, 3 + 3 + 2, 3 + 4 + 2, 4 + 4 + 2]
    assert forwards == [(4 - 2 + 1) + (4 - 3 + 1) + (2 - 2 + 1), 2 + 2 + 1, 2 + 1 + 1, 1 + 1 + 1]


@pytest.mark.parametrize("N", [3, 4, 5])
def test_acceptance_limit_probe_invariants_and_upper_bound(tiny, N):
    """Table 2: more candidates per position can only match more; k = V - 1 (every token) matches all
    steps and gives the table's upper bound, N/(N+1) when the rounds are full; with zero attention
    the first logits already predict every later step, so k = 1 reaches the bound (the self-draft is
    perfect there), which is what SSD itself achieves on that model."""
    cfg, w0 = tiny
    prompt = synth.gen_prompt(cfg, 9, 24)
    gen_len, block = 2 * 6 * (N + 1), 6 * (N + 1)                     # whole rounds only
    ref, _ = decode.stepwise(w0, cfg, prompt, gen_len, block)
    out, pr = decode.acceptance_limit_probe(w0, cfg, prompt, gen_len, block, N, cfg["vocab"] - 1)
    assert out == ref and pr["steps"] == gen_len and pr["rounds"] == gen_len // (N + 1)
    assert all(r[0] == 0 for r in pr["ranks"])                          # a round's first token is the arg-max of its logits
    assert all(a <= b for a, b in zip(pr["matched"], pr["matched"][1:]))
    assert pr["matched"][-1] == gen_len and abs(pr["reduction"][-1] - N / (N + 1)) < 1e-12
    w = dict(w0)
    w["layers"] = [dict(lw, wo=torch.zeros_like(lw["wo"])) for lw in w0["layers"]]
    _, pz = decode.acceptance_limit_probe(w, cfg, prompt, gen_len, block, N, 3)
    assert pz["matched"] == [gen_len] * 3 and abs(pz["reduction"][0] - N / (N + 1)) < 1e-12


# --------------------------------------------------------------------------
# cfg["operand_dtype"]: where the oracle rounds matrix-product operands.  The bf16 GPU tolerances are
# multiples of the noise this rounding causes, so its placement is pinned: every operand of every
# matrix product is representable in the operand type, nothing else changes, and the resulting noise
# floor equals a stored value.
# --------------------------------------------------------------------------
class _MatmulSpy:
    """Records both operands of every `a @ b` evaluated while active."""

    def __enter__(self):
        self.calls = []
        self._orig = torch.Tensor.__matmul__
        spy = self

        def patched(a, b):
            spy.calls.append((a.detach().clone(), b.detach().clone()))
            return spy._orig(a, b)

        torch.Tensor.__matmul__ = patched
        return self

    def __exit__(self, *exc):
        torch.Tensor.__matmul__ = self._orig


def _representable(x, dt):
    return bool((x.to(dt).to(x.dtype) == x).all())


def test_operand_dtype_rounds_every_matmul_operand_and_nothing_else():
    cfg = synth.model_config("tiny", dtype="bf16", n_layers=2, d_model=128, n_q_heads=4, n_kv_heads=2, head_dim=32,
                             d_ffn=256, vocab=96)
    w = synth.gen_weights(cfg, 41, std=0.08)
    prompt = synth.gen_prompt(cfg, 42, 12)
    block = [cfg["mask_id"]] * 8

    def run(c):
        cache = model.KVCache(c["n_layers"])
        _, kv = model.forward_segment(w, c, prompt, 0, cache, torch.float64, need_logits=False)
        cache.append(kv)
        with _MatmulSpy() as spy:
            logits, _ = model.forward_segment(w, c, block, len(prompt), cache, torch.float64)
        return logits, spy.calls

    exact, calls_exact = run(dict(cfg))                               # key absent
    none, calls_none = run(dict(cfg, operand_dtype=None))
    rounded, calls_bf16 = run(dict(cfg, operand_dtype=torch.bfloat16))
    # per layer: QKV, (scores, weighted values) per query head, output, gate/up, down; then the LM head
    per_layer = 1 + 2 * cfg["n_q_heads"] + 1 + 1 + 1
    assert len(calls_exact) == len(calls_none) == len(calls_bf16) == cfg["n_layers"] * per_layer + 1
    assert torch.equal(exact, none), "operand_dtype=None must leave the evaluation untouched"
    for (a0, b0), (a1, b1) in zip(calls_exact, calls_none):
        assert torch.equal(a0, a1) and torch.equal(b0, b1)
    # rounded mode: both operands of every product are exactly representable in bf16 ...
    for i, (a, b) in enumerate(calls_bf16):
        assert _representable(a, torch.bfloat16) and _representable(b, torch.bfloat16), f"matmul {i} has an unrounded operand"
    # ... whereas in exact mode every activation operand is not (the check has teeth), and the weights are
    act_unrounded = sum(not _representable(a, torch.bfloat16) for a, _ in calls_exact)
    assert act_unrounded == len(calls_exact)
    # the rounding is a perturbation, not another function: logits move by a small fraction of their spread
    dev = (rounded - exact).abs().max().item()
    assert 0 < dev < 0.05 * exact.std().item()
    # the residual stream, the norms' statistics and the softmax stay in the compute type: with an operand type that
    # holds every fp64 value the rounded mode is the exact mode
    same, _ = run(dict(cfg, operand_dtype=torch.float64))
    assert torch.equal(same, exact)


def test_operand_noise_floor_equals_the_stored_value():
    """sigma of the small bf16 model, recomputed, against tests/golden/operand_sigma.txt (written by
    tests/golden/make_operand_sigma.py from the oracle alone)."""
    import importlib.util
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_operand_sigma", os.path.join(here, "golden", "make_operand_sigma.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = [float(l) for l in open(os.path.join(here, "golden", "operand_sigma.txt")) if not l.startswith("#")]
    assert len(stored) == 1
    assert mod.sigma() == pytest.approx(stored[0], rel=1e-6)
    # dropping one rounding point (here: the softmax weights) must move sigma by far more than that tolerance
    orig = model.attention
    try:
        model.attention = lambda q, k, v, allowed=None, cfg=None: orig(q, k, v, allowed, None)
        assert abs(mod.sigma() - stored[0]) > 1e-3 * stored[0]
    finally:
        model.attention = orig


# --------------------------------------------------------------------------
# spill-over selection with the dual cache (Section 3.2.2 + Section 4.1): ssd_dual_spill
# --------------------------------------------------------------------------
@pytest.mark.parametrize("refresh", [1, 3, 8, 16, 100])
@pytest.mark.parametrize("block,N", [(8, 4), (5, 3), (32, 4), (8, 6)])
def test_spill_over_is_token_identical_to_stepwise_dual(tiny, refresh, block, N):
    """Lossless for every refresh interval and block size, never more forwards than the in-block chain,
    every round accepts between 1 and N + 1 tokens, refreshes at the same moments as stepwise decoding."""
    cfg, w = tiny
    prompt = synth.gen_prompt(cfg, 300 + refresh, 21)
    gen = 40 if block != 32 else 64
    base, s0 = decode.stepwise_dual(w, cfg, prompt, gen, block, refresh)
    inb, s1 = decode.ssd_dual(w, cfg, prompt, gen, block, N, refresh)
    trace = []
    out, s2 = decode.ssd_dual_spill(w, cfg, prompt, gen, block, N, refresh, trace=trace)
    assert out == base == inb
    assert s2["refreshes"] == s0["refreshes"]
    assert s2["forwards"] <= s1["forwards"] <= s0["forwards"] == gen
    assert s2["accept_hist"][0] == 0 and sum(a * n for a, n in enumerate(s2["accept_hist"])) == gen
    assert all(1 <= len(r["accepted"]) <= N + 1 and r["nodes"] <= N + 1 for r in trace)
    assert all(len(r["accepted"]) == 1 and r["nodes"] == 1 for r in trace if r["refresh"])


def test_spill_over_crosses_block_boundaries_and_saves_forwards(tiny):
    """On a model whose drafts mostly verify (attention scaled down, not zeroed: positions still interact)
    rounds do cross the boundary, and fewer forwards are needed than with the in-block chain."""
    cfg, w = tiny
    w2 = {k: v for k, v in w.items() if k != "layers"}
    w2["layers"] = [dict(lw, wo=lw["wo"] * 0.02) for lw in w["layers"]]
    prompt = synth.gen_prompt(cfg, 77, 16)
    base, _ = decode.stepwise_dual(w2, cfg, prompt, 48, 8, 16)
    inb, s1 = decode.ssd_dual(w2, cfg, prompt, 48, 8, 4, 16)
    trace = []
    out, s2 = decode.ssd_dual_spill(w2, cfg, prompt, 48, 8, 4, 16, trace=trace)
    assert out == base == inb
    assert any(r["crossed"] for r in trace)
    assert s2["forwards"] < s1["forwards"]


@pytest.mark.parametrize("N,refresh,block,gen", [(4, 8, 8, 48), (3, 8, 8, 40), (4, 16, 8, 48), (5, 12, 6, 48), (4, 8, 32, 64),
                                                 (2, 5, 8, 43)])
def test_spill_over_closed_form_with_zero_attention(tiny, N, refresh, block, gen):
    """All wo = 0: every position ties, the order is left to right, every draft verifies, also those read off
    the refresh.  Block boundaries then cost nothing: every refresh period of R tokens takes the refresh
    forward (one token) plus ceil((R - 1) / (N + 1)) rounds, whatever the block length."""
    cfg, w = tiny
    w0 = {k: v for k, v in w.items() if k != "layers"}
    w0["layers"] = [dict(lw, wo=torch.zeros_like(lw["wo"])) for lw in w["layers"]]
    prompt = synth.gen_prompt(cfg, 5, 10)
    base, _ = decode.stepwise_dual(w0, cfg, prompt, gen, block, refresh)
    out, st = decode.ssd_dual_spill(w0, cfg, prompt, gen, block, N, refresh)
    assert out == base and len(set(out)) == 1
    full, rem = divmod(gen, refresh)
    want = full * (1 + math.ceil((refresh - 1) / (N + 1))) + ((1 + math.ceil((rem - 1) / (N + 1))) if rem else 0)
    assert st["forwards"] == want and st["refreshes"] == full + (1 if rem else 0)
