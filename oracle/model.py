"""Oracle transformer f_theta (Section 3.1, Eq. 2): pre-norm bidirectional
transformer with RMSNorm, rotary position embedding, (grouped-query) attention
and a SwiGLU feed-forward, evaluated on a *segment* of tokens against an exact
prefix KV cache.  TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Segments (Section 3.1, Eq. 3): segment 0 is the prompt, segment j+1 is block
B_j.  A position attends to every position of its own segment and of all
earlier segments and to nothing later, so the keys/values of a finished
segment never change and can be cached exactly.

Every formula is written out; torch is used for matmul, exp, sqrt, cos, sin.
Weights arrive as [out_features, in_features] tensors (fp32 or bf16) and are
upcast to the compute dtype at the point of use.

Operand precision.  cfg["operand_dtype"] (absent/None = exact) names the
storage type of matrix-multiply operands in the bf16 configurations: every
activation that enters a matrix product (normed rows, rotated q and k, v,
softmax probabilities, attention output, SwiGLU output) is rounded to that
type first, then the product, the softmax, the norms and the residual stream
are evaluated in the compute dtype.  With operand_dtype=None nothing is
rounded: that is the reference the deviation of a bf16 pipeline is reported
against.
"""
from __future__ import annotations

import math

import torch


def _operand(x, cfg):
    """Round an activation to the operand storage type of the configuration."""
    od = cfg.get("operand_dtype")
    return x if od is None else x.to(od).to(x.dtype)


def rms_norm(x, g, eps):
    """y_i = x_i / sqrt(mean_j x_j^2 + eps) * g_i   (per row)."""
    ms = (x * x).sum(dim=-1, keepdim=True) / x.shape[-1]
    return x / torch.sqrt(ms + eps) * g.to(x.dtype)


def rope(x, pos, theta):
    """Rotary embedding, rotate-half pairing: for i < dh/2 the pair (x_i, x_{i+dh/2})
    is rotated by the angle pos * theta^(-2i/dh).  x: [n, H, dh], pos: [n] ints."""
    n, H, dh = x.shape
    half = dh // 2
    i = torch.arange(half, dtype=torch.float64)
    inv_freq = theta ** (-2.0 * i / dh)
    ang = pos.to(torch.float64)[:, None] * inv_freq[None, :]          # [n, half]
    cos = torch.cos(ang).to(x.dtype)[:, None, :]
    sin = torch.sin(ang).to(x.dtype)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return torch.cat([x1 * cos - x2 * sin, x2 * cos + x1 * sin], dim=-1)


def silu(x):
    return x / (1.0 + torch.exp(-x))


def attention(q, k, v, allowed=None, cfg=None):
    """softmax(q k^T / sqrt(dh)) v per head.
    q: [n, Hq, dh]; k, v: [m, Hkv, dh]; query head h reads kv head h // (Hq/Hkv).
    allowed: optional [n, m] bool (True = may attend).  Returns [n, Hq, dh]."""
    n, Hq, dh = q.shape
    m, Hkv, _ = k.shape
    group = Hq // Hkv
    out = torch.empty_like(q)
    for h in range(Hq):
        kh, vh = k[:, h // group, :], v[:, h // group, :]
        s = (q[:, h, :] @ kh.T) / math.sqrt(dh)                        # [n, m]
        if allowed is not None:
            s = torch.where(allowed, s, torch.full_like(s, float("-inf")))
        s = s - s.max(dim=-1, keepdim=True).values
        p = torch.exp(s)
        p = p / p.sum(dim=-1, keepdim=True)
        if cfg is not None:
            p = _operand(p, cfg)
        out[:, h, :] = p @ vh
    return out


class KVCache:
    """Exact prefix cache: per layer, keys (after RoPE) and values of every
    finished segment, in position order."""

    def __init__(self, n_layers):
        self.k = [None] * n_layers
        self.v = [None] * n_layers

    def length(self):
        return 0 if self.k[0] is None else self.k[0].shape[0]

    def append(self, new_kv):
        for l, (k, v) in enumerate(new_kv):
            self.k[l] = k if self.k[l] is None else torch.cat([self.k[l], k], 0)
            self.v[l] = v if self.v[l] is None else torch.cat([self.v[l], v], 0)


def _layer(h, lw, cfg, pos, k_prefix, v_prefix, allowed, dtype):
    Hq, Hkv, dh = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    F = cfg["d_ffn"]
    n = h.shape[0]
    x = _operand(rms_norm(h, lw["norm1"], cfg["rms_eps"]), cfg)
    qkv = x @ lw["wqkv"].to(dtype).T
    q = qkv[:, : Hq * dh].reshape(n, Hq, dh)
    k = qkv[:, Hq * dh: (Hq + Hkv) * dh].reshape(n, Hkv, dh)
    v = qkv[:, (Hq + Hkv) * dh:].reshape(n, Hkv, dh)
    q = _operand(rope(q, pos, cfg["rope_theta"]), cfg)
    k = _operand(rope(k, pos, cfg["rope_theta"]), cfg)
    v = _operand(v, cfg)
    k_all = k if k_prefix is None else torch.cat([k_prefix, k], 0)
    v_all = v if v_prefix is None else torch.cat([v_prefix, v], 0)
    a = _operand(attention(q, k_all, v_all, allowed, cfg).reshape(n, Hq * dh), cfg)
    h = h + a @ lw["wo"].to(dtype).T
    x = _operand(rms_norm(h, lw["norm2"], cfg["rms_eps"]), cfg)
    gu = x @ lw["wgu"].to(dtype).T
    h = h + _operand(silu(gu[:, :F]) * gu[:, F:], cfg) @ lw["wdown"].to(dtype).T
    return h, k, v


def forward_segment(w, cfg, tokens, pos0, cache, dtype=torch.float64, need_logits=True):
    """Run one segment (len(tokens) rows at absolute positions pos0..) against
    the cached prefix.  Every row attends to the whole prefix and to all rows
    of the segment (bidirectional).  Returns (logits [n, V] or None,
    [(k_l, v_l)] per layer for these rows)."""
    tokens = torch.as_tensor(tokens, dtype=torch.long)
    n = tokens.shape[0]
    assert cache.length() == pos0, "segment must start right after the cached prefix"
    pos = pos0 + torch.arange(n)
    h = w["embed"][tokens].to(dtype)
    new_kv = []
    for l, lw in enumerate(w["layers"]):
        h, k, v = _layer(h, lw, cfg, pos, cache.k[l], cache.v[l], None, dtype)
        new_kv.append((k, v))
    if not need_logits:
        return None, new_kv
    hn = _operand(rms_norm(h, w["final_norm"], cfg["rms_eps"]), cfg)
    return hn @ w["lm_head"].to(dtype).T, new_kv


def forward_block_dual(w, cfg, tokens, pos0, k_all, v_all, dtype=torch.float64):
    """Dual (prefix + suffix) cache of the paper's experimental setup (Section 4.1): the rows of the
    current block, at positions pos0.., attend to their own freshly computed keys and values and to
    the CACHED keys and values of every other position of the sequence, before the block and after
    it.  k_all[l], v_all[l]: [T, Hkv, dh] of the last refresh.  Returns logits [n, V]."""
    tokens = torch.as_tensor(tokens, dtype=torch.long)
    n = tokens.shape[0]
    pos = pos0 + torch.arange(n)
    h = w["embed"][tokens].to(dtype)
    for l, lw in enumerate(w["layers"]):
        k_other = torch.cat([k_all[l][:pos0], k_all[l][pos0 + n:]], 0)
        v_other = torch.cat([v_all[l][:pos0], v_all[l][pos0 + n:]], 0)
        h, _, _ = _layer(h, lw, cfg, pos, k_other, v_other, None, dtype)
    hn = _operand(rms_norm(h, w["final_norm"], cfg["rms_eps"]), cfg)
    return hn @ w["lm_head"].to(dtype).T


def forward_full_blockcausal(w, cfg, tokens, seg, dtype=torch.float64):
    """Cache-free evaluation of a whole sequence: position i may attend to
    position j iff seg[j] <= seg[i].  Returns logits [len, V]."""
    tokens = torch.as_tensor(tokens, dtype=torch.long)
    seg = torch.as_tensor(seg, dtype=torch.long)
    n = tokens.shape[0]
    allowed = seg[None, :] <= seg[:, None]
    pos = torch.arange(n)
    h = w["embed"][tokens].to(dtype)
    for lw in w["layers"]:
        h, _, _ = _layer(h, lw, cfg, pos, None, None, allowed, dtype)
    hn = _operand(rms_norm(h, w["final_norm"], cfg["rms_eps"]), cfg)
    return hn @ w["lm_head"].to(dtype).T
