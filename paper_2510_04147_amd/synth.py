"""Seeded synthetic inputs: model shapes, random-init weights and random prompts.

This module holds none of the method's arithmetic.  It only names the workload
shapes and draws the random numbers that both the HIP path and the CPU oracle
consume (each side receives the same bytes).  It imports neither of them.

Recipe (stands in for the trained LLaDA / Dream checkpoints and the benchmark
prompts of the paper's Section 4.1, which are not available offline):
  * every projection / embedding / LM-head weight ~ N(0, 0.02), RMSNorm gains 1;
  * prompts uniform over [0, V-1); the mask token is id V-1 and never appears
    in a prompt;
  * one independent counter-based stream per (seed, tensor id).
"""
from __future__ import annotations

import copy

import numpy as np
import torch

# ---------------------------------------------------------------------------
# Workload shapes.  "tiny" is the fp32 parity case; the others are the 8B-class
# (MHA) and 7B-class (GQA) masked-diffusion LLM shapes with block-wise
# generation (Section 3.1, Eq. 3) and small draft depth (Section 4.1).
# ---------------------------------------------------------------------------
_MODELS = {
    "tiny": dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64,
                 d_ffn=768, vocab=1024, dtype="fp32"),
    "8b": dict(n_layers=32, d_model=4096, n_q_heads=32, n_kv_heads=32, head_dim=128,
               d_ffn=12288, vocab=126464, dtype="bf16"),
    "7b_gqa": dict(n_layers=28, d_model=3584, n_q_heads=28, n_kv_heads=4, head_dim=128,
                   d_ffn=18944, vocab=152064, dtype="bf16"),
}

WORKLOADS = {
    # name: (model, batch, prompt_len, gen_len, block, draft_depth, prompt_seed)
    "cfg1_tiny": dict(model="tiny", batch=1, prompt_len=64, gen_len=64, block=32, draft=4, seed=1001),
    "cfg2_8b_b32_n4": dict(model="8b", batch=1, prompt_len=256, gen_len=256, block=32, draft=4, seed=1002),
    "cfg3_8b_b64_n8": dict(model="8b", batch=1, prompt_len=512, gen_len=512, block=64, draft=8, seed=1003),
    "cfg4_8b_batch4": dict(model="8b", batch=4, prompt_len=1024, gen_len=256, block=32, draft=4, seed=1004),
    "cfg5_7b_gqa_batch8": dict(model="7b_gqa", batch=8, prompt_len=512, gen_len=256, block=32, draft=8, seed=1005),
    # the paper's own decoding shape (Section 4.1: block 8, draft length 3 to 5), reported for context
    "ctx_8b_b8_n3": dict(model="8b", batch=1, prompt_len=256, gen_len=256, block=8, draft=3, seed=1006),
    "ctx_8b_b8_n4": dict(model="8b", batch=1, prompt_len=256, gen_len=256, block=8, draft=4, seed=1006),
    "ctx_8b_b8_n5": dict(model="8b", batch=1, prompt_len=256, gen_len=256, block=8, draft=5, seed=1006),
}


def model_config(name: str, **overrides) -> dict:
    """Return a fresh config dict for a named model shape (overrides allowed,
    e.g. n_layers=2 to get a shallow model of the 8B layer shape)."""
    cfg = copy.deepcopy(_MODELS[name])
    cfg.update(rope_theta=10000.0, rms_eps=1e-5)
    cfg.update(overrides)
    cfg["mask_id"] = cfg["vocab"] - 1
    return cfg


def _torch_dtype(cfg) -> torch.dtype:
    return torch.float32 if cfg["dtype"] == "fp32" else torch.bfloat16


def _normal(shape, std, seed, tensor_id, device, dtype):
    """One N(0, std) tensor from the stream keyed by (seed, tensor_id)."""
    dev = torch.device(device)
    if dev.type == "cpu":
        # numpy Philox: counter-based, identical on every machine.
        rng = np.random.Generator(np.random.Philox(key=[seed, tensor_id]))
        a = rng.standard_normal(size=shape, dtype=np.float32)
        return (torch.from_numpy(a) * std).to(dtype)
    g = torch.Generator(device=dev)
    g.manual_seed((int(seed) << 24) + int(tensor_id))
    t = torch.randn(shape, generator=g, device=dev, dtype=torch.float32)
    return (t * std).to(dtype)


def gen_weights(cfg: dict, seed: int = 0, device="cpu", std: float = 0.02) -> dict:
    """Random-init weights.  Linear weights are stored [out_features, in_features]
    (row-major, the contraction dimension contiguous).

    Returns a dict with
      embed [V, d], lm_head [V, d], final_norm [d] (fp32), and per layer
      wqkv [(Hq+2Hkv)*dh, d]  rows = all Q heads, then all K heads, then all V heads
      wo   [d, Hq*dh]
      wgu  [2F, d]            rows [0,F) gate, rows [F,2F) up
      wdown[d, F]
      norm1, norm2 [d] (fp32)
    """
    dt = _torch_dtype(cfg)
    d, F, V = cfg["d_model"], cfg["d_ffn"], cfg["vocab"]
    Hq, Hkv, dh = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    w = {
        "embed": _normal((V, d), std, seed, 1, device, dt),
        "lm_head": _normal((V, d), std, seed, 2, device, dt),
        "final_norm": torch.ones(d, dtype=torch.float32, device=device),
        "layers": [],
    }
    for l in range(cfg["n_layers"]):
        base = 16 * (l + 1)
        w["layers"].append({
            "wqkv": _normal(((Hq + 2 * Hkv) * dh, d), std, seed, base + 0, device, dt),
            "wo": _normal((d, Hq * dh), std, seed, base + 1, device, dt),
            "wgu": _normal((2 * F, d), std, seed, base + 2, device, dt),
            "wdown": _normal((d, F), std, seed, base + 3, device, dt),
            "norm1": torch.ones(d, dtype=torch.float32, device=device),
            "norm2": torch.ones(d, dtype=torch.float32, device=device),
        })
    return w


def weights_to(w: dict, device) -> dict:
    """Copy a weight dict to another device (same bytes)."""
    out = {k: v.to(device) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: v.to(device) for k, v in lw.items()} for lw in w["layers"]]
    return out


def gen_prompt(cfg: dict, seed: int, n: int) -> np.ndarray:
    """n token ids uniform over [0, V-1) (the mask id V-1 excluded), int32."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0]))
    return rng.integers(0, cfg["vocab"] - 1, size=n, dtype=np.int32)


def streamed_param_count(cfg: dict) -> int:
    """Weights one forward streams from HBM: all layer projections + LM head
    (the embedding table is only gathered, so it is not counted)."""
    d, F, V = cfg["d_model"], cfg["d_ffn"], cfg["vocab"]
    Hq, Hkv, dh = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    layer = (Hq + 2 * Hkv) * dh * d + d * Hq * dh + 2 * F * d + d * F
    return layer * cfg["n_layers"] + V * d


def kv_bytes_per_token(cfg: dict) -> int:
    esz = 4 if cfg["dtype"] == "fp32" else 2
    return 2 * cfg["n_kv_heads"] * cfg["head_dim"] * cfg["n_layers"] * esz
