"""The allocation-free entry point (ssd_k_lm_head_static): the LM-head reduction with its partial
results in the library's static device array instead of the caller's workspace.  Checked through the
C ABI against the existing entry point (ssd_k_linear, SSD_LIN_LM) on two calls in a row, the second
with fewer rows, and against the definition (fp64 logits of the same operands)."""
import pytest
import torch

from paper_2510_04147_amd import synth

pytestmark = pytest.mark.gpu


def _definition(x, lm_head, mask_id):
    lg = x.cpu().double() @ lm_head.cpu().double().T
    lg[:, mask_id] = float("-inf")
    m, t = lg.max(dim=-1)
    c = 1.0 / torch.exp(lg - m[:, None]).sum(-1)
    return m, t, c


@pytest.mark.parametrize("model,rows", [("8b", (160, 45)), ("tiny", (96, 7))])
def test_static_scratch_lm_head_equals_workspace_lm_head(model, rows):
    from paper_2510_04147_amd import binding as B
    cfg = synth.model_config(model, n_layers=1)
    wg = synth.gen_weights(cfg, 3, device="cuda")
    eng = B.SSD(cfg, wg, max_seqs=1, max_seq_len=256, block=32, max_draft=4, max_rows=192)
    dt = torch.float32 if cfg["dtype"] == "fp32" else torch.bfloat16
    g = torch.Generator(device="cuda").manual_seed(17)
    try:
        for M in rows:                                   # two calls in a row, the second smaller
            x = torch.randn(M, cfg["d_model"], generator=g, device="cuda").to(dt)
            want = torch.empty(3, M, dtype=torch.float32, device="cuda")
            got = torch.full((3, M), -7.0, dtype=torch.float32, device="cuda")
            eng.k_linear(B.LIN_LM, 0, x, want)
            eng.k_lm_head_static(x, got)
            torch.cuda.synchronize()
            assert torch.equal(got, want), f"M={M}: static-scratch result differs from the workspace result"
            m, t, c = _definition(x, wg["lm_head"], cfg["mask_id"])
            o = got.cpu().double()
            assert (o[0] - m).abs().max() < 2e-4
            assert torch.equal(o[1].long(), t)
            assert ((o[2] - c).abs() <= 1e-4 * c).all()
        # more rows than the static array holds: rejected on the host, nothing launched
        if model == "8b":
            big = torch.zeros(192, cfg["d_model"], dtype=dt, device="cuda")
            out = torch.empty(3, 192, dtype=torch.float32, device="cuda")
            with pytest.raises(B.SsdError) as ei:
                eng.k_lm_head_static(big, out)
            assert ei.value.code == -2 and "static array" in str(ei.value)
    finally:
        eng.close()
