"""ctypes binding of libssd_mi355x.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch provides
device memory and the stream.  Importing this module fails loudly if the
library has not been built (python -m paper_2510_04147_amd.build).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libssd_mi355x.so")
MEASURE_LIB_PATH = os.path.join(_HERE, "libssd_measure.so")

SSD_MAX_DRAFT = 15
SSD_F32, SSD_BF16 = 0, 1

EXPORTS = ["ssd_workspace_bytes", "ssd_create", "ssd_destroy", "ssd_reset", "ssd_cached_len", "ssd_prefill_kv",
           "ssd_draft", "ssd_verify_tree", "ssd_generate", "ssd_set_kernel_path", "ssd_set_boundary_fusion", "ssd_set_graphs", "ssd_set_tree_mode", "ssd_set_cross_block",
           "ssd_set_cache_mode", "ssd_set_spill_over", "ssd_refresh_kv", "ssd_acceptance_limit",
           "ssd_profile_begin",
           "ssd_profile_read", "ssd_profile_end", "ssd_strerror", "ssd_last_error", "ssd_k_linear", "ssd_k_accept", "ssd_k_lm_head_static",
           "ssd_k_write_cache", "ssd_k_attention", "ssd_k_norm"]
MEASURE_EXPORTS = ["ssd_measure_stream_read", "ssd_measure_mixed_read"]
LIN_QKV, LIN_O, LIN_GU, LIN_DOWN, LIN_LM = range(5)


class SsdConfig(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn",
                                        "vocab", "mask_id", "dtype")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float)] + \
               [(n, C.c_int) for n in ("max_seqs", "max_seq_len", "block", "max_draft", "max_rows")]


class SsdWeights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("wqkv", C.POINTER(C.c_void_p)), ("wo", C.POINTER(C.c_void_p)), ("wgu", C.POINTER(C.c_void_p)),
                ("wdown", C.POINTER(C.c_void_p)), ("norm1", C.POINTER(C.c_void_p)), ("norm2", C.POINTER(C.c_void_p))]


class SsdStepOut(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("n_accept", "acc_pos", "acc_tok", "n_next", "next_pos", "next_tok",
                                           "row_maxlogit", "row_argmax", "row_conf")]


class SsdKNode(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("seq", "S", "blen", "T")]


class SsdStats(C.Structure):
    _fields_ = [("forwards", C.c_int64), ("kv_passes", C.c_int64), ("tokens", C.c_int64),
                ("accept_hist", C.c_int64 * (SSD_MAX_DRAFT + 2)),
                ("decode_ms", C.c_double), ("kv_ms", C.c_double), ("total_ms", C.c_double)]


class SsdError(RuntimeError):
    def __init__(self, code, name, detail):
        super().__init__(f"{name} ({code}): {detail}")
        self.code = code


def load_library() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2510_04147_amd.build`")
    lib = C.CDLL(LIB_PATH)
    lib.ssd_workspace_bytes.restype = C.c_size_t
    lib.ssd_workspace_bytes.argtypes = [C.POINTER(SsdConfig)]
    lib.ssd_create.argtypes = [C.POINTER(SsdConfig), C.POINTER(SsdWeights), C.c_void_p, C.c_size_t, C.c_void_p,
                               C.POINTER(C.c_void_p)]
    lib.ssd_destroy.argtypes = [C.c_void_p]
    lib.ssd_reset.argtypes = [C.c_void_p, C.c_int]
    lib.ssd_cached_len.argtypes = [C.c_void_p, C.c_int]
    lib.ssd_prefill_kv.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int]
    lib.ssd_draft.argtypes = [C.c_void_p, C.c_int] + [C.c_void_p] * 5 + [C.c_int, C.POINTER(SsdStepOut)]
    lib.ssd_verify_tree.argtypes = [C.c_void_p, C.c_int] + [C.c_void_p] * 8 + [C.c_int, C.POINTER(SsdStepOut)]
    lib.ssd_generate.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_void_p), C.c_void_p, C.c_int, C.c_int, C.c_int,
                                 C.c_void_p, C.POINTER(SsdStats)]
    lib.ssd_set_kernel_path.argtypes = [C.c_void_p, C.c_int]
    lib.ssd_k_accept.argtypes = [C.c_void_p, C.c_int] + [C.c_void_p] * 7 + [C.c_int, C.c_void_p, C.c_void_p,
                                                                              C.POINTER(SsdStepOut)]
    lib.ssd_set_boundary_fusion.argtypes = [C.c_void_p, C.c_int]
    lib.ssd_set_graphs.argtypes = [C.c_void_p, C.c_int]
    lib.ssd_set_tree_mode.argtypes = [C.c_void_p, C.c_int]
    lib.ssd_set_cross_block.argtypes = [C.c_void_p, C.c_int]
    lib.ssd_set_cache_mode.argtypes = [C.c_void_p, C.c_int, C.c_int]
    lib.ssd_set_spill_over.argtypes = [C.c_void_p, C.c_int]
    lib.ssd_acceptance_limit.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.ssd_refresh_kv.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int,
                                   C.POINTER(SsdStepOut)]
    for n in ("ssd_profile_begin", "ssd_profile_end"):
        getattr(lib, n).argtypes = [C.c_void_p]
    lib.ssd_profile_read.argtypes = [C.c_void_p, C.POINTER(C.c_int), C.POINTER(C.c_char_p), C.POINTER(C.c_int64),
                                     C.POINTER(C.c_double)]
    lib.ssd_k_linear.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_void_p]
    lib.ssd_k_write_cache.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    lib.ssd_k_attention.argtypes = [C.c_void_p, C.c_int, C.c_int, C.POINTER(SsdKNode), C.c_void_p, C.c_int, C.c_int,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.ssd_k_norm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p]
    lib.ssd_k_lm_head_static.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
    lib.ssd_strerror.restype = C.c_char_p
    lib.ssd_strerror.argtypes = [C.c_int]
    lib.ssd_last_error.restype = C.c_char_p
    lib.ssd_last_error.argtypes = [C.c_void_p]
    return lib


def load_measure_library() -> C.CDLL:
    """The measurement kernels (streaming-read ceiling, a GEMM's loads alone): a library of their own."""
    if not os.path.exists(MEASURE_LIB_PATH):
        raise ImportError(f"{MEASURE_LIB_PATH} is missing: build it with `python -m paper_2510_04147_amd.build`")
    lib = C.CDLL(MEASURE_LIB_PATH)
    lib.ssd_measure_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    lib.ssd_measure_mixed_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_int,
                                           C.c_void_p, C.c_void_p]
    return lib


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = load_library()
    return _lib


def make_config(cfg: dict, max_seqs: int, max_seq_len: int, block: int, max_draft: int, max_rows: int = 0) -> SsdConfig:
    c = SsdConfig()
    for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab", "mask_id"):
        setattr(c, n, int(cfg[n]))
    c.dtype = SSD_F32 if cfg["dtype"] == "fp32" else SSD_BF16
    c.rope_theta, c.rms_eps = float(cfg["rope_theta"]), float(cfg["rms_eps"])
    c.max_seqs, c.max_seq_len, c.block, c.max_draft = max_seqs, max_seq_len, block, max_draft
    c.max_rows = max(max_rows, max_seqs * (max_draft + 1) * block)
    return c


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


class StepOut:
    """Device buffers for one decode forward's outputs, plus host views."""

    def __init__(self, n, block, max_draft, device):
        z = lambda *s, dt=torch.int32: torch.zeros(*s, dtype=dt, device=device)
        self.n_accept, self.n_next = z(n), z(n)
        self.acc_pos, self.acc_tok = z(n, max_draft + 1), z(n, max_draft + 1)
        self.next_pos, self.next_tok = z(n, max(max_draft, 1)), z(n, max(max_draft, 1))
        self.row_maxlogit = z(n, max_draft + 1, block, dt=torch.float32)
        self.row_argmax = z(n, max_draft + 1, block)
        self.row_conf = z(n, max_draft + 1, block, dt=torch.float32)
        self.c = SsdStepOut(*[t.data_ptr() for t in (self.n_accept, self.acc_pos, self.acc_tok, self.n_next,
                                                     self.next_pos, self.next_tok, self.row_maxlogit,
                                                     self.row_argmax, self.row_conf)])

    def host(self):
        torch.cuda.synchronize()
        return {k: getattr(self, k).cpu().numpy() for k in ("n_accept", "acc_pos", "acc_tok", "n_next", "next_pos",
                                                             "next_tok", "row_maxlogit", "row_argmax", "row_conf")}


class SSD:
    """A context of the library on the current CUDA/HIP device and stream."""

    def __init__(self, cfg: dict, weights: dict, max_seqs=1, max_seq_len=2048, block=32, max_draft=4, max_rows=0):
        self.lib = lib()
        self.cfg = cfg
        self.ccfg = make_config(cfg, max_seqs, max_seq_len, block, max_draft, max_rows)
        self.block, self.max_draft, self.max_seqs = block, max_draft, max_seqs
        self.weights = weights                    # keep the tensors alive
        dev = weights["embed"].device
        assert dev.type == "cuda", "weights must live on the GPU"
        self.device = dev
        want = torch.float32 if cfg["dtype"] == "fp32" else torch.bfloat16
        L = cfg["n_layers"]

        def ptrs(name, dt):
            arr = (C.c_void_p * L)()
            for l, lw in enumerate(weights["layers"]):
                t = lw[name]
                assert t.dtype == dt and t.is_contiguous() and t.device == dev, name
                arr[l] = t.data_ptr()
            return arr

        self._arrs = [ptrs(n, want) for n in ("wqkv", "wo", "wgu", "wdown")] + \
                     [ptrs(n, torch.float32) for n in ("norm1", "norm2")]
        for n in ("embed", "lm_head"):
            assert weights[n].dtype == want and weights[n].is_contiguous()
        assert weights["final_norm"].dtype == torch.float32
        w = SsdWeights(weights["embed"].data_ptr(), weights["lm_head"].data_ptr(), weights["final_norm"].data_ptr(),
                       *[C.cast(a, C.POINTER(C.c_void_p)) for a in self._arrs])
        nbytes = self.lib.ssd_workspace_bytes(C.byref(self.ccfg))
        if nbytes == 0:
            raise SsdError(-1, "ssd_workspace_bytes", "config rejected")
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
        base = (self.workspace.data_ptr() + 255) & ~255
        self.stream = torch.cuda.current_stream(dev)
        h = C.c_void_p()
        rc = self.lib.ssd_create(C.byref(self.ccfg), C.byref(w), C.c_void_p(base), C.c_size_t(nbytes),
                                 C.c_void_p(self.stream.cuda_stream), C.byref(h))
        if rc != 0:
            raise SsdError(rc, self.lib.ssd_strerror(rc).decode(), self.lib.ssd_last_error(None).decode())
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.ssd_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _chk(self, rc):
        if rc < 0:
            raise SsdError(rc, self.lib.ssd_strerror(rc).decode(), self.lib.ssd_last_error(self.h).decode())
        return rc

    # ---- thin wrappers, same names as the C entry points
    def reset(self, seq):
        self._chk(self.lib.ssd_reset(self.h, seq))

    def cached_len(self, seq):
        return self._chk(self.lib.ssd_cached_len(self.h, seq))

    def set_kernel_path(self, path):
        return self._chk(self.lib.ssd_set_kernel_path(self.h, path))

    def set_boundary_fusion(self, on):
        return self._chk(self.lib.ssd_set_boundary_fusion(self.h, int(on)))

    def set_tree_mode(self, mode):
        return self._chk(self.lib.ssd_set_tree_mode(self.h, int(mode)))

    def set_cross_block(self, on):
        return self._chk(self.lib.ssd_set_cross_block(self.h, int(on)))

    def set_cache_mode(self, mode, refresh_interval=0):
        return self._chk(self.lib.ssd_set_cache_mode(self.h, int(mode), int(refresh_interval)))

    def set_spill_over(self, on):
        return self._chk(self.lib.ssd_set_spill_over(self.h, int(on)))

    def refresh_kv(self, seq, tokens, pos0, block_len, n_draft_next, out):
        t = _i32(tokens)
        self._chk(self.lib.ssd_refresh_kv(self.h, seq, t.ctypes.data, len(t), pos0, block_len, n_draft_next,
                                          C.byref(out.c)))

    def acceptance_limit(self, prompt, gen_len, block, n_draft, k_max):
        p = _i32(prompt)
        toks = np.zeros(gen_len, dtype=np.int32)
        matched, forwards = np.zeros(k_max, dtype=np.int64), np.zeros(k_max, dtype=np.int64)
        rounds = np.zeros(1, dtype=np.int64)
        reduction = np.zeros(k_max, dtype=np.float64)
        self._chk(self.lib.ssd_acceptance_limit(self.h, p.ctypes.data, len(p), gen_len, block, n_draft, k_max,
                                                toks.ctypes.data, matched.ctypes.data, forwards.ctypes.data,
                                                rounds.ctypes.data, reduction.ctypes.data))
        return toks, dict(steps=gen_len, rounds=int(rounds[0]), matched=[int(v) for v in matched],
                          forwards=[int(v) for v in forwards], reduction=[float(v) for v in reduction])

    def set_graphs(self, on):
        return self._chk(self.lib.ssd_set_graphs(self.h, int(on)))

    def prefill_kv(self, seq, tokens, pos0):
        t = _i32(tokens)
        self._chk(self.lib.ssd_prefill_kv(self.h, seq, t.ctypes.data, len(t), pos0))

    def new_out(self, n=1):
        return StepOut(n, self.block, self.max_draft, self.device)

    def _block_args(self, seqs, block_tok, masked, pos0, block_len):
        n = len(seqs)
        bt = np.zeros((n, self.block), dtype=np.int32)
        for i, row in enumerate(block_tok):
            bt[i, :len(row)] = row
        mk = np.ascontiguousarray(np.asarray(masked, dtype=np.uint64))
        bl = _i32(block_len) if block_len is not None else None
        return n, _i32(seqs), bt, mk, _i32(pos0), bl

    def draft(self, seqs, block_tok, masked, pos0, n_draft_next, out, block_len=None):
        n, sq, bt, mk, p0, bl = self._block_args(seqs, block_tok, masked, pos0, block_len)
        self._chk(self.lib.ssd_draft(self.h, n, sq.ctypes.data, bt.ctypes.data, mk.ctypes.data, p0.ctypes.data,
                                     bl.ctypes.data if bl is not None else None, n_draft_next, C.byref(out.c)))

    def verify_tree(self, seqs, block_tok, masked, pos0, drafts, n_draft_next, out, block_len=None):
        """drafts: per sequence a list of (pos, tok) in priority order."""
        n, sq, bt, mk, p0, bl = self._block_args(seqs, block_tok, masked, pos0, block_len)
        md = max(self.max_draft, 1)
        dp, dtk = np.zeros((n, md), dtype=np.int32), np.zeros((n, md), dtype=np.int32)
        nd = np.zeros(n, dtype=np.int32)
        for i, dr in enumerate(drafts):
            nd[i] = len(dr)
            for j, (q, t) in enumerate(dr[:md]):
                dp[i, j], dtk[i, j] = q, t
        if self.max_draft == 0:
            dp = dp[:, :0].copy()
            dtk = dtk[:, :0].copy()
        self._chk(self.lib.ssd_verify_tree(self.h, n, sq.ctypes.data, bt.ctypes.data, mk.ctypes.data, p0.ctypes.data,
                                           bl.ctypes.data if bl is not None else None, dp.ctypes.data,
                                           dtk.ctypes.data, nd.ctypes.data, n_draft_next, C.byref(out.c)))

    def generate(self, prompts, gen_len, block, draft_depth):
        n = len(prompts)
        ps = [_i32(p) for p in prompts]
        arr = (C.c_void_p * n)(*[p.ctypes.data for p in ps])
        plen = _i32([len(p) for p in ps])
        out = np.zeros((n, gen_len), dtype=np.int32)
        st = SsdStats()
        self._chk(self.lib.ssd_generate(self.h, n, C.cast(arr, C.POINTER(C.c_void_p)), plen.ctypes.data, gen_len,
                                        block, draft_depth, out.ctypes.data, C.byref(st)))
        stats = dict(forwards=st.forwards, kv_passes=st.kv_passes, tokens=st.tokens,
                     accept_hist=list(st.accept_hist), decode_ms=st.decode_ms, kv_ms=st.kv_ms,
                     total_ms=st.total_ms)
        return out, stats

    def k_accept(self, seqs, block_tok, masked, drafts, n_draft_next, row_conf, row_argmax, out, block_len=None):
        """The acceptance step alone on device arrays row_conf (float32) / row_argmax (int32), one entry per row."""
        n, sq, bt, mk, _, bl = self._block_args(seqs, block_tok, masked, [0] * len(seqs), block_len)
        md = max(self.max_draft, 1)
        dp, dtk = np.zeros((n, md), dtype=np.int32), np.zeros((n, md), dtype=np.int32)
        nd = np.zeros(n, dtype=np.int32)
        for i, dr in enumerate(drafts):
            nd[i] = len(dr)
            for j, (q, t) in enumerate(dr[:md]):
                dp[i, j], dtk[i, j] = q, t
        assert row_conf.dtype == torch.float32 and row_argmax.dtype == torch.int32
        assert row_conf.is_contiguous() and row_argmax.is_contiguous() and row_conf.device == self.device
        self._chk(self.lib.ssd_k_accept(self.h, n, sq.ctypes.data, bt.ctypes.data, mk.ctypes.data,
                                        bl.ctypes.data if bl is not None else None, dp.ctypes.data, dtk.ctypes.data,
                                        nd.ctypes.data, n_draft_next, row_conf.data_ptr(), row_argmax.data_ptr(),
                                        C.byref(out.c)))

    def k_linear(self, which, layer, x, out):
        """One linear step on caller-supplied rows x [M, K] (device tensor of the model dtype)."""
        assert x.is_contiguous() and out.is_contiguous() and x.device == self.device
        self._chk(self.lib.ssd_k_linear(self.h, which, layer, x.data_ptr(), x.shape[0], out.data_ptr()))

    def k_write_cache(self, seq, layer, pos0, k, v):
        """k, v: device tensors [n, Hkv, dh] of the model dtype (keys already rotated) into the cache."""
        assert k.is_contiguous() and v.is_contiguous() and k.shape == v.shape and k.device == self.device
        self._chk(self.lib.ssd_k_write_cache(self.h, seq, layer, pos0, k.shape[0], k.data_ptr(), v.data_ptr()))

    def k_attention(self, layer, nodes, qkv, fused, out_attn, out_q=None, out_k=None, out_v=None):
        """nodes: list of (seq, S, blen, T); qkv: device fp32 [n_part, M, (Hq+2Hkv)*dh]."""
        arr = (SsdKNode * len(nodes))(*[SsdKNode(*nd) for nd in nodes])
        assert qkv.dtype == torch.float32 and qkv.is_contiguous() and qkv.dim() == 3 and out_attn.is_contiguous()
        ptr = lambda t: t.data_ptr() if t is not None else None
        self._chk(self.lib.ssd_k_attention(self.h, layer, len(nodes), arr, qkv.data_ptr(), qkv.shape[0], int(fused),
                                           out_attn.data_ptr(), ptr(out_q), ptr(out_k), ptr(out_v)))

    def k_norm(self, h, partials, gain, out):
        """h: device fp32 [M, d] (updated in place); partials: device fp32 [n_part, M, d] or None."""
        assert h.dtype == torch.float32 and h.is_contiguous() and gain.dtype == torch.float32 and out.is_contiguous()
        n_part = 0 if partials is None else partials.shape[0]
        assert partials is None or (partials.dtype == torch.float32 and partials.is_contiguous())
        self._chk(self.lib.ssd_k_norm(self.h, h.data_ptr(), partials.data_ptr() if n_part else None, n_part,
                                      gain.data_ptr(), h.shape[0], out.data_ptr()))

    def k_lm_head_static(self, x, out):
        """The LM-head reduction of k_linear(LIN_LM, ...) with its partial results in the library's static array."""
        assert x.is_contiguous() and out.is_contiguous() and x.device == self.device
        self._chk(self.lib.ssd_k_lm_head_static(self.h, x.data_ptr(), x.shape[0], out.data_ptr()))

    def profile_begin(self):
        self._chk(self.lib.ssd_profile_begin(self.h))

    def profile_read(self):
        n = C.c_int(32)
        names = (C.c_char_p * 32)()
        cnt = (C.c_int64 * 32)()
        ms = (C.c_double * 32)()
        self._chk(self.lib.ssd_profile_read(self.h, C.byref(n), names, cnt, ms))
        return {names[i].decode(): dict(launches=cnt[i], ms=ms[i]) for i in range(n.value)}

    def profile_end(self):
        self._chk(self.lib.ssd_profile_end(self.h))
