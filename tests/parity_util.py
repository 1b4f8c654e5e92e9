"""Helpers for the GPU-vs-oracle comparison protocol (teacher forced per forward).

The oracle's trace gives, per forward: the block state, the drafts, and per node
the predictions (t, m, c) and the top-2 logit margin.  The same state is fed to
the HIP entry points and the outputs are compared row by row.

Exemptions (counted and reported, never silent):
  * token id: only where the oracle's top-2 logit margin is below `margin_tol`;
  * acceptance decision: only where a compared token is exempt, or where the two
    best position confidences of a walked node differ by less than `conf_tol`
    in log space (a legitimate reordering of near-equal confidences).
"""
import math

import numpy as np

from oracle import decode


def bits(masked):
    return sum(1 << p for p, mk in enumerate(masked) if mk)


def node_masks(masked, drafts):
    out, mk = [list(masked)], list(masked)
    for (q, _) in drafts:
        mk[q] = False
        out.append(list(mk))
    return out


def compare_record(rec, gpu, maxlogit_tol, margin_tol, conf_tol, conf_rtol):
    """rec: oracle trace record; gpu: dict of host arrays for ONE sequence
    (row_* of shape [max_draft+1, block], n_accept, acc_*, n_next, next_*).
    Returns counters; raises AssertionError on a real mismatch."""
    stats = dict(rows=0, tok_exempt=0, decision_exempt=0, max_dlogit=0.0, sq_dlogit=0.0, sum_dlogit=0.0, positions=0)
    masks = node_masks(rec["masked"], rec["drafts"])
    n_nodes = len(masks)
    B = len(rec["masked"])
    tok_exempt_rows = set()
    for j in range(n_nodes):
        for p in range(B):
            if not masks[j][p]:
                continue
            stats["rows"] += 1
            stats["positions"] += j == 0
            signed = float(gpu["row_maxlogit"][j, p]) - float(rec["m"][j][p])
            dm = abs(signed)
            stats["max_dlogit"] = max(stats["max_dlogit"], dm)
            stats["sq_dlogit"] += dm * dm
            stats["sum_dlogit"] += signed
            assert dm <= maxlogit_tol, f"max-logit differs by {dm} at node {j} pos {p}"
            if int(gpu["row_argmax"][j, p]) != int(rec["t"][j][p]):
                assert float(rec["margin"][j][p]) < margin_tol, \
                    f"arg-max differs at node {j} pos {p} with oracle margin {float(rec['margin'][j][p])}"
                stats["tok_exempt"] += 1
                tok_exempt_rows.add((j, p))
            else:
                co, cg = float(rec["c"][j][p]), float(gpu["row_conf"][j, p])
                assert abs(cg - co) <= conf_rtol * co, f"confidence {cg} vs {co} at node {j} pos {p}"

    return stats, tok_exempt_rows, masks


def expected_from_gpu_rows(rec, gpu, masks, n_draft_next):
    """Chain walk (oracle's routine) applied to the GPU's own per-row outputs."""
    import torch
    n_nodes = len(masks)
    t = [torch.tensor(gpu["row_argmax"][j]) for j in range(n_nodes)]
    c = [torch.tensor(gpu["row_conf"][j]) for j in range(n_nodes)]
    return decode.accept_chain(t, c, masks, rec["drafts"], n_draft_next)


def decision_near_tie(rec, masks, conf_tol):
    """True if any node the oracle walked has its two best masked confidences
    within conf_tol in log space."""
    m = len(rec["accepted"]) - 1
    for j in range(m + 1):
        cs = sorted((float(rec["c"][j][p]) for p, mk in enumerate(masks[j]) if mk), reverse=True)
        if len(cs) >= 2 and math.log(cs[0]) - math.log(cs[1]) < conf_tol:
            return True
    # the ranking of the next drafts
    cs = sorted((float(rec["c"][m][p]) for p, mk in enumerate(masks[m]) if mk), reverse=True)
    return any(math.log(a) - math.log(b) < conf_tol for a, b in zip(cs, cs[1:]))


def check_forward(rec, gpu, n_draft_next, maxlogit_tol, margin_tol, conf_tol, conf_rtol):
    stats, tok_exempt_rows, masks = compare_record(rec, gpu, maxlogit_tol, margin_tol, conf_tol, conf_rtol)
    acc, nxt, m = expected_from_gpu_rows(rec, gpu, masks, n_draft_next)
    got_acc = [(int(gpu["acc_pos"][i]), int(gpu["acc_tok"][i])) for i in range(int(gpu["n_accept"]))]
    got_nxt = [(int(gpu["next_pos"][i]), int(gpu["next_tok"][i])) for i in range(int(gpu["n_next"]))]
    assert got_acc == acc, f"acceptance kernel {got_acc} != chain walk on its own rows {acc}"
    assert got_nxt == nxt, f"next drafts {got_nxt} != ranking of its own rows {nxt}"
    assert 1 <= len(got_acc) <= len(rec["drafts"]) + 1
    # (2) against the oracle's decision
    if got_acc != rec["accepted"] or got_nxt != rec["next_drafts"]:
        assert tok_exempt_rows or decision_near_tie(rec, masks, conf_tol), \
            f"decision differs from the oracle with no near-tie: {got_acc}/{got_nxt} vs {rec['accepted']}/{rec['next_drafts']}"
        stats["decision_exempt"] += 1
    return stats


def operand_noise_floor(cfg, w, prompt, block, dtype):
    """sigma = rms over the rows of the first forward (all-masked block after the prompt) of the
    difference in max logit between two CPU oracles that differ only in the storage type of the
    matrix-product operands: exact, and rounded to bf16 at every product input.  It is the
    intrinsic deviation of ANY bf16-operand evaluation of this model from the exact one, and it
    is computed from the oracle alone."""
    import torch
    from oracle import model
    ms = []
    for od in (None, torch.bfloat16):
        c2 = dict(cfg, operand_dtype=od)
        cache = model.KVCache(cfg["n_layers"])
        _, kv = model.forward_segment(w, c2, prompt, 0, cache, dtype, need_logits=False)
        cache.append(kv)
        lg, _ = model.forward_segment(w, c2, [cfg["mask_id"]] * block, len(prompt), cache, dtype)
        ms.append(decode.predict(lg, cfg["mask_id"])[1].double())
    return float(((ms[0] - ms[1]) ** 2).mean().sqrt())


def bf16_tolerances(sigma):
    """Tolerances of the bf16 configurations, derived from the operand noise floor sigma:
    a bf16-operand pipeline is an independent draw of that noise, so |m_gpu - m_exact| has
    standard deviation about sigma per row; 6 sigma bounds the maximum over thousands of rows.
    A token may flip only where the oracle's top-2 margin is within the noise of two logits;
    two position confidences may swap only where their log-gap is."""
    return dict(maxlogit_tol=6.0 * sigma, margin_tol=6.0 * sigma, conf_tol=6.0 * sigma, conf_rtol=8.0 * sigma)


LITERAL_MAXLOGIT, LITERAL_MARGIN = 2e-2, 1e-2     # the literal bf16 limits: max logit, top-2 margin below which a token may differ


class OperandTwin:
    """The oracle with every matrix-product operand rounded to bf16 (cfg["operand_dtype"]), evaluated on
    the states the exact oracle recorded: an ideal bf16-operand pipeline to hold the GPU's deviations
    from the exact oracle against, row by row."""

    def __init__(self, w, cfg, prompt, dtype):
        import torch
        self.w, self.dtype = w, dtype
        self.cfg = dict(cfg, operand_dtype=torch.bfloat16)
        self.cache = decode._prefill(w, self.cfg, prompt, dtype)

    def append(self, tokens, S):
        from oracle import model
        _, kv = model.forward_segment(self.w, self.cfg, tokens, S, self.cache, self.dtype, need_logits=False)
        self.cache.append(kv)

    def count_literal(self, rec, gpu, counts):
        """Adds to counts: rows beyond the literal limits, for the GPU and for the twin, both against the exact oracle."""
        nodes = decode.build_chain(rec["tok"], rec["masked"], rec["drafts"])
        for j, (nt, mk) in enumerate(nodes):
            t2, m2, _, _ = decode._node_forward(self.w, self.cfg, nt, rec["S"], self.cache, self.dtype)
            for p, is_masked in enumerate(mk):
                if not is_masked:
                    continue
                me, te, mg = float(rec["m"][j][p]), int(rec["t"][j][p]), float(rec["margin"][j][p])
                counts["rows"] += 1
                counts["gpu_maxlogit"] += abs(float(gpu["row_maxlogit"][j, p]) - me) > LITERAL_MAXLOGIT
                counts["twin_maxlogit"] += abs(float(m2[p]) - me) > LITERAL_MAXLOGIT
                counts["gpu_token"] += int(gpu["row_argmax"][j, p]) != te and mg >= LITERAL_MARGIN
                counts["twin_token"] += int(t2[p]) != te and mg >= LITERAL_MARGIN
                counts["sq_twin"] += (float(m2[p]) - me) ** 2
                counts["sum_twin"] += float(m2[p]) - me


def literal_counts_ok(counts):
    """The GPU may exceed the literal limits no more often than an ideal bf16-operand pipeline does on the
    same rows (both are draws of the same rounding noise: the allowance is that count's own scatter)."""
    def allowed(n):
        return 1.25 * n + 3.0 * math.sqrt(n) + 3.0
    return (counts["gpu_maxlogit"] <= allowed(counts["twin_maxlogit"]) and
            counts["gpu_token"] <= allowed(counts["twin_token"]))


def bias_ok(totals, sigma):
    """Signed mean of (GPU - oracle) max logits: a systematic error shows here long before it moves the rms.
    Rows of one forward that share a block position are nearly the same computation (the nodes differ in
    a few tokens), so the independent samples are the (forward, position) pairs."""
    n = max(totals["positions"], 1)
    return abs(totals["sum_dlogit"] / max(totals["rows"], 1)) <= 4.0 * sigma / math.sqrt(n) + 1e-4


def teacher_forced(eng, cfg, w, prompt, gen_len, block, N, dtype, max_blocks=None, seq=0, verbose=True,
                   max_forwards=None, literal=False, sigma=None, **tol):
    """Runs the oracle's SSD (recording every forward), then replays every
    recorded forward through the HIP entry points from the oracle's state and
    compares.  Returns (oracle tokens, oracle stats, totals).  literal: also count, for the GPU and for the
    bf16-operand oracle, the rows beyond the literal limits (totals["literal"]).  sigma: assert the signed
    mean deviation (bias_ok)."""
    trace = []
    ref, st = decode.ssd(w, cfg, prompt, gen_len, block, N, dtype=dtype, trace=trace, max_blocks=max_blocks,
                         max_forwards=max_forwards)
    eng.reset(seq)
    eng.prefill_kv(seq, prompt, 0)
    out = eng.new_out(1)
    totals = dict(rows=0, tok_exempt=0, decision_exempt=0, max_dlogit=0.0, forwards=0, sum_dlogit=0.0, positions=0)
    P = len(prompt)
    totals["sq_dlogit"] = 0.0
    twin = OperandTwin(w, cfg, prompt, dtype) if literal else None
    counts = dict(rows=0, gpu_maxlogit=0, twin_maxlogit=0, gpu_token=0, twin_token=0, sq_twin=0.0, sum_twin=0.0)
    for i, rec in enumerate(trace):
        if max_forwards is not None and i >= max_forwards:
            break
        if verbose:
            print(f"forward {i}: S={rec['S']} drafts={len(rec['drafts'])}", flush=True)
        if eng.cached_len(seq) < rec["S"]:          # previous block finished: append its (oracle) tokens
            lo = eng.cached_len(seq) - P
            if twin:
                twin.append(ref[lo:rec["S"] - P], eng.cached_len(seq))
            eng.prefill_kv(seq, ref[lo:rec["S"] - P], eng.cached_len(seq))
        bl = len(rec["tok"])
        eng.verify_tree([seq], [rec["tok"]], [bits(rec["masked"])], [rec["S"]], [rec["drafts"]], N, out,
                        block_len=[bl])
        g = {k: v[0] for k, v in out.host().items()}
        s = check_forward(rec, g, N, **tol)
        if twin:
            twin.count_literal(rec, g, counts)
        for k in ("rows", "tok_exempt", "decision_exempt", "sum_dlogit", "positions"):
            totals[k] += s[k]
        totals["max_dlogit"] = max(totals["max_dlogit"], s["max_dlogit"])
        totals["sq_dlogit"] += s["sq_dlogit"]
        totals["forwards"] += 1
    totals["rms_dlogit"] = math.sqrt(totals["sq_dlogit"] / max(totals["rows"], 1))
    totals["mean_dlogit"] = totals["sum_dlogit"] / max(totals["rows"], 1)
    if twin:
        counts["rms_twin"] = math.sqrt(counts["sq_twin"] / max(counts["rows"], 1))
        counts["mean_twin"] = counts["sum_twin"] / max(counts["rows"], 1)
        totals["literal"] = counts
        assert literal_counts_ok(counts), f"the GPU exceeds the literal limits more often than bf16 operands explain: {counts}"
    if sigma is not None:
        assert bias_ok(totals, sigma), f"signed mean deviation {totals['mean_dlogit']:.5f} over {totals['positions']} positions, sigma {sigma:.4f}"
    return ref, st, totals


def teacher_forced_batch(eng, cfg, w, prompts, gen_len, block, N, dtype, max_forwards, sigma=None, **tol):
    """Several sequences decoded together: the oracle runs each sequence on its own (recording max_forwards
    forwards, all inside the first block); forward i of every sequence is then replayed in ONE HIP forward
    that holds all sequences, and each sequence's rows are compared with its own oracle record."""
    n = len(prompts)
    traces = []
    for pr in prompts:
        tr = []
        decode.ssd(w, cfg, pr, gen_len, block, N, dtype=dtype, trace=tr, max_forwards=max_forwards)
        traces.append(tr)
    n_fw = min(len(t) for t in traces)
    for i, pr in enumerate(prompts):
        eng.reset(i)
        eng.prefill_kv(i, pr, 0)
    out = eng.new_out(n)
    totals = dict(rows=0, tok_exempt=0, decision_exempt=0, max_dlogit=0.0, forwards=0, sum_dlogit=0.0, positions=0, sq_dlogit=0.0)
    for f in range(n_fw):
        recs = [t[f] for t in traces]
        assert all(r["S"] == len(pr) for r, pr in zip(recs, prompts)), "the sampled forwards must stay in the first block"
        eng.verify_tree(list(range(n)), [r["tok"] for r in recs], [bits(r["masked"]) for r in recs], [r["S"] for r in recs],
                        [r["drafts"] for r in recs], N, out, block_len=[len(r["tok"]) for r in recs])
        host = out.host()
        for i, rec in enumerate(recs):
            s = check_forward(rec, {k: v[i] for k, v in host.items()}, N, **tol)
            for k in ("rows", "tok_exempt", "decision_exempt", "sum_dlogit", "positions"):
                totals[k] += s[k]
            totals["max_dlogit"] = max(totals["max_dlogit"], s["max_dlogit"])
            totals["sq_dlogit"] += s["sq_dlogit"]
        totals["forwards"] += 1
    totals["rms_dlogit"] = math.sqrt(totals["sq_dlogit"] / max(totals["rows"], 1))
    totals["mean_dlogit"] = totals["sum_dlogit"] / max(totals["rows"], 1)
    if sigma is not None:
        assert bias_ok(totals, sigma), f"signed mean deviation {totals['mean_dlogit']:.5f} over {totals['positions']} positions"
    return totals


def teacher_forced_dual(eng, cfg, w, prompt, gen_len, block, N, refresh, dtype, seq=0, verbose=True, max_forwards=None,
                        **tol):
    """As teacher_forced, for the dual cache with periodic refresh (Section 4.1): a recorded refresh is
    replayed through ssd_refresh_kv with the oracle's whole sequence, every other forward through
    ssd_verify_tree against the prefix and suffix that refresh cached."""
    trace = []
    ref, st = decode.ssd_dual(w, cfg, prompt, gen_len, block, N, refresh, dtype=dtype, trace=trace,
                              max_forwards=max_forwards)
    eng.reset(seq)
    out = eng.new_out(1)
    totals = dict(rows=0, tok_exempt=0, decision_exempt=0, max_dlogit=0.0, forwards=0, refreshes=0, sq_dlogit=0.0)
    last_x = None
    for i, rec in enumerate(trace):
        bl = len(rec["tok"])
        if verbose:
            print(f"forward {i}: S={rec['S']} drafts={len(rec['drafts'])} refresh={rec['refresh']}", flush=True)
        if rec["refresh"]:
            eng.refresh_kv(seq, rec["x"], rec["S"], bl, N, out)
            last_x = rec["x"]
            totals["refreshes"] += 1
        else:
            if eng.cached_len(seq) != rec["S"]:
                # a block that starts between two refreshes: the cache keeps the last refresh's keys and
                # values, which the library can only be given by repeating that refresh for the new block
                eng.refresh_kv(seq, last_x, rec["S"], bl, N, out)
            eng.verify_tree([seq], [rec["tok"]], [bits(rec["masked"])], [rec["S"]], [rec["drafts"]], N, out,
                            block_len=[bl])
        g = {k: v[0] for k, v in out.host().items()}
        s = check_forward(rec, g, N, **tol)
        for k in ("rows", "tok_exempt", "decision_exempt"):
            totals[k] += s[k]
        totals["max_dlogit"] = max(totals["max_dlogit"], s["max_dlogit"])
        totals["sq_dlogit"] += s["sq_dlogit"]
        totals["forwards"] += 1
    totals["rms_dlogit"] = math.sqrt(totals["sq_dlogit"] / max(totals["rows"], 1))
    return ref, st, totals
