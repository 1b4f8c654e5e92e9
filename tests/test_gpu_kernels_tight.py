"""The non-GEMM bf16 kernels alone, on caller-supplied operands, against the oracle's definitions in fp64
on the IDENTICAL operands, with nothing upstream to blur the comparison:

  * the rotary stage (k_rope): fp32 projection -> bf16 q / k / v, one bf16 rounding of the fp64 result;
  * the attention kernel in every variant the forward selects (head size 128 and 64; rotary stage fused
    or separate; with and without a cached suffix; a ragged 24-row block; prefixes that end inside a
    32-position tile; grouped-query heads; several nodes and sequences), against oracle.model.attention
    on the bf16 q / k / v the kernel itself consumed.  Tolerance, derived from the kernel's arithmetic:
    one bf16 rounding of the output (2^-8 relative) plus the rounding of the softmax weights to bf16
    before the second product (2^-9 of the softmax-weighted mean of |v|) plus fp32 accumulation;
  * residual + RMSNorm (k_norm): fp64 sum and norm of the same inputs, one bf16 rounding.

The fp32 kernels (the tiny configuration's path) get the same checks at fp32 tolerances.
"""
import zlib

import pytest
import torch

from oracle import model
from paper_2510_04147_amd import synth

pytestmark = pytest.mark.gpu


def _engine(cfg, seed, max_rows=640, max_seqs=2):
    from paper_2510_04147_amd import binding
    wg = synth.gen_weights(cfg, seed, device="cuda")
    return binding.SSD(cfg, wg, max_seqs=max_seqs, max_seq_len=512, block=64, max_draft=4, max_rows=max_rows)


def _bf16_round_ok(got, want, extra=0.0):
    """|got - want| within one bf16 rounding of want (plus `extra`, elementwise or scalar)."""
    diff = (got.double() - want).abs()
    return diff <= 2.0 ** -8 * want.abs() + 1e-6 + extra, diff


CFG128 = dict(name="8b", over=dict(n_layers=1, vocab=1024))                       # 32 x 128 heads, MHA
CFG128_GQA = dict(name="7b_gqa", over=dict(n_layers=1, vocab=1024))               # 28 q / 4 kv heads x 128
CFG64 = dict(name="tiny", over=dict(dtype="bf16", n_layers=1, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=64,
                                    d_ffn=1536, vocab=1024))
CFG_F32 = dict(name="tiny", over=dict(n_layers=1))

# (config, nodes [(seq, S, blen, T)], variants): variant = (kernel path, fused)
CASES = [
    ("dh128_5_nodes", CFG128, [(0, 100, 32, 0)] * 5, [(1, 1), (1, 0), (0, 0)]),
    ("dh128_ragged24", CFG128, [(0, 75, 24, 0)] * 3, [(1, 1), (1, 0), (0, 0)]),
    ("dh128_block64", CFG128, [(0, 130, 64, 0)] * 2, [(1, 0), (0, 0)]),
    ("dh128_suffix", CFG128, [(0, 70, 24, 250)] * 3 + [(1, 33, 32, 97)], [(1, 1), (1, 0), (0, 0)]),
    ("dh128_two_seqs", CFG128, [(0, 96, 32, 0), (0, 96, 32, 0), (1, 7, 8, 0)], [(1, 1), (1, 0)]),
    ("dh128_gqa", CFG128_GQA, [(0, 90, 32, 0)] * 4 + [(1, 161, 20, 0)], [(1, 1), (1, 0), (0, 0)]),
    ("dh64_gqa", CFG64, [(0, 45, 32, 0)] * 3 + [(1, 64, 24, 0)], [(1, 0), (0, 0)]),
    ("dh64_suffix", CFG64, [(0, 45, 24, 200), (1, 0, 32, 64)], [(1, 0), (0, 0)]),
    ("f32_tiny", CFG_F32, [(0, 64, 32, 0)] * 5 + [(1, 50, 20, 150)], [(0, 0)]),
]


@pytest.mark.parametrize("name,cfgspec,nodes,variants", CASES, ids=[c[0] for c in CASES])
def test_rotary_stage_and_attention_kernels_alone(name, cfgspec, nodes, variants):
    cfg = synth.model_config(cfgspec["name"], **cfgspec["over"])
    eng = _engine(cfg, 5)
    f32 = cfg["dtype"] == "fp32"
    dt = torch.float32 if f32 else torch.bfloat16
    Hq, Hkv, dh = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    nq, nkv = Hq * dh, Hkv * dh
    g = torch.Generator(device="cuda").manual_seed(zlib.crc32(name.encode()) % 1000)
    M = sum(nd[2] for nd in nodes)
    try:
        # ---- cached keys and values, per sequence up to the furthest position any node reads
        cache = {}
        for (seq, S, blen, T) in nodes:
            cache[seq] = max(cache.get(seq, 0), S, T)
        kc, vc = {}, {}
        for seq, n in cache.items():
            if n == 0:
                continue
            kc[seq] = (torch.randn(n, Hkv, dh, generator=g, device="cuda") * 0.7).to(dt)
            vc[seq] = torch.randn(n, Hkv, dh, generator=g, device="cuda").to(dt)
            eng.k_write_cache(seq, 0, 0, kc[seq], vc[seq])
        # ---- the QKV projection as two split-K partial sums (the forward's case) of a typical scale
        qkv = torch.randn(2, M, nq + 2 * nkv, generator=g, device="cuda") * 0.8
        total = (qkv[0].double() + qkv[1].double()).cpu()                # fp64 of the fp32 sum order s = 0, 1
        total32 = (qkv[0] + qkv[1]).cpu().double()                       # what an fp32 adder gives
        outs = {}
        for (path, fused) in variants:
            eng.set_kernel_path(path)
            attn = torch.zeros(M, nq, dtype=dt, device="cuda")
            if fused:
                eng.k_attention(0, nodes, qkv, 1, attn)
                outs[(path, fused)] = (attn.cpu(), None)
                continue
            q = torch.zeros(M, nq, dtype=dt, device="cuda")
            k = torch.zeros(M, Hkv, dh, dtype=dt, device="cuda")
            v = torch.zeros(M, Hkv, dh, dtype=dt, device="cuda")
            eng.k_attention(0, nodes, qkv, 0, attn, q, k, v)
            outs[(path, fused)] = (attn.cpu(), (q.cpu(), k.cpu(), v.cpu()))
        eng.set_kernel_path(1)
        torch.cuda.synchronize()

        # ---- rotary stage against the oracle's rope() in fp64 on the same projection
        pos = torch.cat([S + torch.arange(blen) for (_, S, blen, _) in nodes])
        q_want = model.rope(total32[:, :nq].reshape(M, Hq, dh), pos, cfg["rope_theta"]).reshape(M, nq)
        k_want = model.rope(total32[:, nq:nq + nkv].reshape(M, Hkv, dh), pos, cfg["rope_theta"])
        v_want = total32[:, nq + nkv:].reshape(M, Hkv, dh)
        assert (total - total32).abs().max() < 1e-6
        for key, (attn, qkv_out) in outs.items():
            if qkv_out is None:
                continue
            q, k, v = qkv_out
            for nm, got, want in (("q", q, q_want), ("k", k, k_want), ("v", v, v_want)):
                if f32:
                    assert (got.double() - want).abs().max() < 2e-6, (key, nm)
                else:
                    ok, diff = _bf16_round_ok(got, want)
                    assert bool(ok.all()), (key, nm, float(diff.max()))

        # ---- attention against the oracle's attention() in fp64 on the kernel's own operands
        for key, (attn, qkv_out) in outs.items():
            if qkv_out is None:
                continue
            q, k, v = [t.double() for t in qkv_out]
            row = 0
            worst = 0.0
            for (seq, S, blen, T) in nodes:
                ks = [kc[seq][:S].cpu().double()] if S > 0 else []
                vs = [vc[seq][:S].cpu().double()] if S > 0 else []
                if T > S + blen:
                    ks.append(kc[seq][S + blen:T].cpu().double())
                    vs.append(vc[seq][S + blen:T].cpu().double())
                ks.append(k[row:row + blen])
                vs.append(v[row:row + blen])
                k_all, v_all = torch.cat(ks, 0), torch.cat(vs, 0)
                qn = q[row:row + blen].reshape(blen, Hq, dh)
                want = model.attention(qn, k_all, v_all).reshape(blen, nq)
                got = attn[row:row + blen]
                if f32:
                    assert (got.double() - want).abs().max() < 5e-6, (key, row)
                else:
                    absv = model.attention(qn, k_all, v_all.abs()).reshape(blen, nq)      # softmax-weighted mean |v|
                    ok, diff = _bf16_round_ok(got, want, extra=2.0 ** -9 * absv + 2e-5)
                    assert bool(ok.all()), (key, row, float(diff.max()), float((diff / (want.abs() + 1e-3)).max()))
                    worst = max(worst, float((diff / (2.0 ** -8 * want.abs() + 2.0 ** -9 * absv + 2e-5)).max()))
                row += blen
            if not f32:
                print(f"{name} path/fused {key}: worst error / tolerance = {worst:.3f}")

        # ---- the fused kernel (sums, rotates and converts on chip) gives the bits of the separate kernels,
        # and the MFMA kernel agrees with the plain kernel to the rounding of the softmax weights
        if (1, 1) in outs and (1, 0) in outs:
            assert torch.equal(outs[(1, 1)][0], outs[(1, 0)][0]), "fused rotary stage changes the result"
        if (1, 0) in outs and (0, 0) in outs:
            a, b = outs[(1, 0)][0].double(), outs[(0, 0)][0].double()
            assert (a - b).abs().max() <= 2.0 ** -6 * max(1.0, float(b.abs().max()))
            for i in range(3):
                assert torch.equal(outs[(1, 0)][1][i], outs[(0, 0)][1][i]), "rotary stage differs between kernel paths"
    finally:
        eng.close()


@pytest.mark.parametrize("cfgspec,M,n_part", [(CFG128, 160, 8), (CFG128, 45, 4), (CFG128_GQA, 33, 0), (CFG64, 32, 3),
                                              (CFG_F32, 37, 2)])
def test_residual_rmsnorm_kernel_alone(cfgspec, M, n_part):
    cfg = synth.model_config(cfgspec["name"], **cfgspec["over"])
    eng = _engine(cfg, 6)
    f32 = cfg["dtype"] == "fp32"
    dt = torch.float32 if f32 else torch.bfloat16
    d = cfg["d_model"]
    g = torch.Generator(device="cuda").manual_seed(100 + M)
    try:
        h = torch.randn(M, d, generator=g, device="cuda") * 3.0
        parts = torch.randn(n_part, M, d, generator=g, device="cuda") if n_part else None
        gain = 1.0 + 0.3 * torch.randn(d, generator=g, device="cuda")
        h_in = h.clone()
        out = torch.zeros(M, d, dtype=dt, device="cuda")
        eng.k_norm(h, parts, gain, out)
        torch.cuda.synchronize()
        want_h = h_in.cpu().double()
        for s in range(n_part):
            want_h = want_h + parts[s].cpu().double()
        assert (h.cpu().double() - want_h).abs().max() < 1e-5          # fp32 adds in split order
        # the norm of the residual the kernel itself stored
        want = model.rms_norm(h.cpu().double(), gain.cpu().double(), cfg["rms_eps"])
        if f32:
            assert (out.cpu().double() - want).abs().max() < 5e-6
        else:
            ok, diff = _bf16_round_ok(out.cpu(), want)
            assert bool(ok.all()), float(diff.max())
    finally:
        eng.close()
