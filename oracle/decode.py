"""Oracle decoding loops.  TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

  stepwise     greedy stepwise decoding in semi-autoregressive block order: one
               token per model forward, the most confident masked position of
               the current block (Section 3.1; Figure 2 caption).  This is the
               result every other routine must reproduce.
  ssd          Self Speculative Decoding, greedy chain tree (Section 3.2,
               Algorithm 1): self-draft, select, build N+1 nodes, verify them
               in one batched forward, accept the longest matching prefix plus
               the last valid node's own prediction, reuse that node's
               predictions as the next drafts.
  bruteforce   stepwise decoding with no cache: the whole sequence is
               recomputed under the block-causal mask for every token.
  cross block  ssd_cross_block: drafts may cover every remaining position of the
               current block; the leaf then holds the finished block and the
               same forward also predicts the next block from it (Section 3.2.2:
               once fewer than N positions remain, candidates come from the next
               block).  Restricted to that one step across the boundary.
  mix order    ssd(..., mix_order=True): the greedy chain plus one extra node per
               non-leaf chain node that skips the next draft (Section 5.2,
               Table 3): when node m's stepwise choice is draft m+2 instead of
               draft m+1 (same candidates, different order), that draft is
               accepted and the extra node, which holds drafts 1..m and m+2,
               supplies one more token.  Extra nodes have no children: 2N nodes
               for N drafts (the table's batch sizes 6 / 8 / 10).

  dual cache   stepwise_dual / ssd_dual / bruteforce_full: the cache of the paper's
               experiments (Section 4.1: prefix and suffix cache, refreshed every
               fixed number of decoded tokens).  A refresh is one forward over the
               whole sequence, prompt, decoded tokens and every still masked
               position, with full bidirectional attention; it renews the keys and
               values of all positions and is itself the decoding step of that
               moment.  Between refreshes only the current block is computed, against
               the cached keys and values of all other positions.  A chain never
               reaches past the next refresh, so SSD and stepwise decoding refresh
               at the same states and stay identical.

  spill-over   ssd_dual_spill: SSD with the dual cache whose chain continues into the next block
               (Section 3.2.2: only when the current block has fewer than N positions left are
               further positions taken from the next block).  Drafts for a block nobody has
               predicted yet are read off the last refresh, whose forward covers every masked
               position of the sequence.  Between refreshes a block is computed against the
               cached keys and values of all other positions, so the next block's candidate
               states can be evaluated in the same forward as the current block's.

  limit probe  acceptance_limit_probe: the procedure behind Table 2 (Section 5.1).
               Stepwise decoding is cut into rounds of N+1 steps (a new round at every
               block start); the logits of a round's first forward are what a draft
               made at that moment would know.  A token decoded in the round counts
               as matched for k if it is among the k highest-ranked tokens of those
               logits at its position.  A round of n steps with m matched tokens would
               have cost n - m + 1 forwards (one verification pass for the matched
               ones, a step of its own for every other), which gives the reduction in
               forwards an ideal verification tree could reach; m = n = N+1 in every
               round is the table's upper bound N/(N+1).

Readings where the paper is silent (all also applied by the HIP path):
  * confidence c = softmax probability of the arg-max token (Section 3.2.2);
  * the mask token can never be predicted (excluded from max / arg-max / sum);
  * ties: lowest token id; lowest position;
  * a draft matches only if position AND token equal the stepwise choice
    (Section 5.1: a different generation order is a failure);
  * drafts come from the current block only, and at most (#masked - 1) of them,
    so the leaf node always has a position left to predict; with zero drafts the
    verification forward is a plain stepwise step (Algorithm 1's fallback);
  * next drafts are read off the last valid node's own outputs, no extra
    forward (Section 3.2.4: the verification pass already holds that node's outputs).
"""
from __future__ import annotations

import math

import torch

from .model import KVCache, forward_block_dual, forward_full_blockcausal, forward_segment


# --------------------------------------------------------------------------
# per-node prediction and the two selection rules
# --------------------------------------------------------------------------
def predict(logits, mask_id):
    """Per row: arg-max token t (mask id excluded, ties -> lowest id), max
    logit m, confidence c = exp(m) / sum_v exp(logit_v) = 1 / sum_v exp(logit_v - m),
    and the top-1 minus top-2 logit margin (used only by the parity protocol)."""
    l = logits.clone()
    l[:, mask_id] = float("-inf")
    V = l.shape[1]
    m = l.max(dim=-1).values
    ids = torch.arange(V)
    t = torch.where(l == m[:, None], ids[None, :], torch.full((1, V), V)).min(dim=-1).values
    c = 1.0 / torch.exp(l - m[:, None]).sum(dim=-1)
    l2 = l.clone()
    l2[torch.arange(l.shape[0]), t] = float("-inf")
    margin = m - l2.max(dim=-1).values
    return t, m, c, margin


def stepwise_choice(c, masked):
    """Position of the highest confidence among masked positions (ties -> lowest)."""
    best = None
    for p, is_masked in enumerate(masked):
        if is_masked and (best is None or c[p] > c[best]):
            best = p
    return best


def rank_positions(c, masked, exclude=None):
    """Masked positions ordered by confidence, high to low (ties -> lowest position)."""
    ps = [p for p, mk in enumerate(masked) if mk and p != exclude]
    return sorted(ps, key=lambda p: (-float(c[p]), p))


def build_chain(tok, masked, drafts):
    """Greedy chain of len(drafts)+1 nodes (Section 3.2.3): node i is the current
    block state with drafts 1..i written in."""
    nodes = []
    t, mk = list(tok), list(masked)
    nodes.append((list(t), list(mk)))
    for (q, d) in drafts:
        assert mk[q], "a draft position must still be masked"
        t[q], mk[q] = d, False
        nodes.append((list(t), list(mk)))
    return nodes


def build_mix_order(tok, masked, drafts):
    """Nodes of the mix-order tree (Section 5.2): the len(drafts)+1 chain nodes, then for
    m = 0 .. len(drafts)-2 the node with drafts 1..m and draft m+2 written in."""
    nodes = build_chain(tok, masked, drafts)
    for m in range(len(drafts) - 1):
        t, mk = list(tok), list(masked)
        for (q, d) in list(drafts[:m]) + [drafts[m + 1]]:
            assert mk[q], "a draft position must still be masked"
            t[q], mk[q] = d, False
        nodes.append((t, mk))
    return nodes


def accept_mix_order(node_t, node_c, node_masked, drafts, n_draft_next):
    """Traversal of the mix-order tree.  Nodes are ordered as build_mix_order returns them.
    As accept_chain, except that a mismatch at chain node m whose stepwise choice equals draft
    m+2 accepts that draft and continues at the extra node of m, whose own choice is accepted
    as the last token.  Returns (accepted, next_drafts, index of the node the walk ended at)."""
    n = len(drafts)
    m = 0
    while True:
        p = stepwise_choice(node_c[m], node_masked[m])
        t = int(node_t[m][p])
        if m < n and (p, t) == (drafts[m][0], int(drafts[m][1])):
            m += 1
            continue
        break
    accepted = [(q, int(d)) for (q, d) in drafts[:m]]
    last = m
    if m + 1 < n and (p, t) == (drafts[m + 1][0], int(drafts[m + 1][1])):
        accepted.append((p, t))                      # the out-of-order draft
        last = n + 1 + m                             # its extra node
        p = stepwise_choice(node_c[last], node_masked[last])
        t = int(node_t[last][p])
    accepted.append((p, t))
    rest = rank_positions(node_c[last], node_masked[last], exclude=p)
    n_next = min(n_draft_next, max(len(rest) - 1, 0))
    next_drafts = [(q, int(node_t[last][q])) for q in rest[:n_next]]
    return accepted, next_drafts, last


def accept_chain(node_t, node_c, node_masked, drafts, n_draft_next):
    """Chain traversal (Section 3.2.4).  node_t[i][p], node_c[i][p]: prediction and
    confidence of node i at position p; node_masked[i][p]: masked in node i.
    Returns (accepted [(pos, tok)], next_drafts [(pos, tok)], m = #matched drafts).

    Node m's stepwise choice is compared with draft m+1; the walk stops at the
    first mismatch; the accepted tokens are the m matched drafts plus node m's
    own choice, so between 1 and len(drafts)+1 tokens."""
    m = 0
    while True:
        p = stepwise_choice(node_c[m], node_masked[m])
        t = int(node_t[m][p])
        if m < len(drafts) and (p, t) == (drafts[m][0], int(drafts[m][1])):
            m += 1
            continue
        break
    accepted = [(q, int(d)) for (q, d) in drafts[:m]] + [(p, t)]
    rest = rank_positions(node_c[m], node_masked[m], exclude=p)
    n_next = min(n_draft_next, max(len(rest) - 1, 0))
    next_drafts = [(q, int(node_t[m][q])) for q in rest[:n_next]]
    return accepted, next_drafts, m


# --------------------------------------------------------------------------
# decoding loops
# --------------------------------------------------------------------------
def _blocks(gen_len, block):
    return [(j * block, min(block, gen_len - j * block)) for j in range(math.ceil(gen_len / block))]


def _prefill(w, cfg, prompt, dtype):
    cache = KVCache(cfg["n_layers"])
    _, kv = forward_segment(w, cfg, prompt, 0, cache, dtype, need_logits=False)
    cache.append(kv)
    return cache


def _cache_with(cache, kv):
    """A copy of the cache with one more segment appended (the original is left alone)."""
    c = KVCache(len(cache.k))
    c.k, c.v = list(cache.k), list(cache.v)
    c.append(kv)
    return c


def _node_forward(w, cfg, tok, S, cache, dtype):
    logits, _ = forward_segment(w, cfg, tok, S, cache, dtype)
    return predict(logits, cfg["mask_id"])


def stepwise(w, cfg, prompt, gen_len, block, dtype=torch.float64, trace=None, max_blocks=None):
    """Greedy stepwise decoding.  Returns (tokens, stats)."""
    P = len(prompt)
    cache = _prefill(w, cfg, prompt, dtype)
    out, forwards, kv_passes = [], 0, 1
    for bi, (off, Bj) in enumerate(_blocks(gen_len, block)):
        if max_blocks is not None and bi >= max_blocks:
            break
        S = P + off
        tok, masked = [cfg["mask_id"]] * Bj, [True] * Bj
        while any(masked):
            t, m, c, margin = _node_forward(w, cfg, tok, S, cache, dtype)
            forwards += 1
            p = stepwise_choice(c, masked)
            if trace is not None:
                trace.append(dict(S=S, tok=list(tok), masked=list(masked), drafts=[],
                                  t=[t], m=[m], c=[c], margin=[margin],
                                  accepted=[(p, int(t[p]))], next_drafts=[]))
            tok[p], masked[p] = int(t[p]), False
        _, kv = forward_segment(w, cfg, tok, S, cache, dtype, need_logits=False)
        cache.append(kv)
        kv_passes += 1
        out += tok
    return out, dict(forwards=forwards, kv_passes=kv_passes)


def ssd(w, cfg, prompt, gen_len, block, n_draft, dtype=torch.float64, trace=None, max_blocks=None,
        max_forwards=None, mix_order=False):
    """Self Speculative Decoding with draft length n_draft (Algorithm 1).
    Returns (tokens, stats) with stats['accept_hist'][a] = number of forwards
    that accepted a tokens.  max_blocks / max_forwards stop early (the tokens
    returned are then a prefix; used to sample forwards of large models).
    mix_order: verify the mix-order tree instead of the greedy chain (Section 5.2)."""
    P = len(prompt)
    cache = _prefill(w, cfg, prompt, dtype)
    out, forwards, kv_passes = [], 0, 1
    hist = [0] * (n_draft + 2)
    for bi, (off, Bj) in enumerate(_blocks(gen_len, block)):
        if max_blocks is not None and bi >= max_blocks:
            break
        S = P + off
        tok, masked = [cfg["mask_id"]] * Bj, [True] * Bj
        drafts = []            # the block-start self-draft is a chain with no drafts
        while any(masked):
            if max_forwards is not None and forwards >= max_forwards:
                return out, dict(forwards=forwards, kv_passes=kv_passes, accept_hist=hist)
            nodes = build_mix_order(tok, masked, drafts) if mix_order else build_chain(tok, masked, drafts)
            # one batched forward over all nodes (Eq. 5); nodes do not see each other
            preds = [_node_forward(w, cfg, nt, S, cache, dtype) for (nt, _) in nodes]
            forwards += 1
            accepted, next_drafts, m = (accept_mix_order if mix_order else accept_chain)(
                [p[0] for p in preds], [p[2] for p in preds], [nm for (_, nm) in nodes],
                drafts, n_draft)
            if trace is not None:
                trace.append(dict(S=S, tok=list(tok), masked=list(masked), drafts=list(drafts),
                                  t=[p[0] for p in preds], m=[p[1] for p in preds],
                                  c=[p[2] for p in preds], margin=[p[3] for p in preds],
                                  accepted=list(accepted), next_drafts=list(next_drafts)))
            hist[len(accepted)] += 1
            for (q, d) in accepted:
                assert masked[q]
                tok[q], masked[q] = d, False
            drafts = next_drafts
        _, kv = forward_segment(w, cfg, tok, S, cache, dtype, need_logits=False)
        cache.append(kv)
        kv_passes += 1
        out += tok
    return out, dict(forwards=forwards, kv_passes=kv_passes, accept_hist=hist)


def ssd_cross_block(w, cfg, prompt, gen_len, block, n_draft, dtype=torch.float64, trace=None):
    """SSD whose last round of a block reaches into the next block (Section 3.2.2).

    As ssd(), except that while a next block exists the drafts may cover ALL remaining masked
    positions of the current block (up to n_draft).  The chain's leaf then holds the finished
    block.  The same forward evaluates the next block, all masked, behind that leaf (its keys and
    values are those of the finished block: exactly the block-start forward stepwise decoding
    would run next).  If every draft verifies, the block is finished, its KV is kept, and the
    next block starts with the stepwise choice and the drafts read off that evaluation: the
    boundary costs no forward of its own.  Otherwise the round ends like any other and the
    speculative evaluation is dropped.  Returns (tokens, stats) as ssd()."""
    P = len(prompt)
    cache = _prefill(w, cfg, prompt, dtype)
    blocks = _blocks(gen_len, block)
    out, forwards, kv_passes = [], 0, 1
    hist = [0] * (n_draft + 2)
    mask_id = cfg["mask_id"]

    def n_next_for(rest, has_next):
        return min(n_draft, len(rest) if has_next else max(len(rest) - 1, 0))

    bi = 0
    tok, masked, drafts = [mask_id] * blocks[0][1], [True] * blocks[0][1], []
    while bi < len(blocks):
        off, Bj = blocks[bi]
        S = P + off
        has_next = bi + 1 < len(blocks)
        nodes = build_chain(tok, masked, drafts)
        leaf_t, leaf_mk = nodes[-1]
        leaf_complete = not any(leaf_mk)
        preds = [_node_forward(w, cfg, nt, S, cache, dtype) if any(mk) else None for (nt, mk) in nodes]
        leaf_kv = leaf_next = None
        if leaf_complete:
            _, leaf_kv = forward_segment(w, cfg, leaf_t, S, cache, dtype, need_logits=False)
            if has_next:
                spec = _cache_with(cache, leaf_kv)
                leaf_next = _node_forward(w, cfg, [mask_id] * blocks[bi + 1][1], S + Bj, spec, dtype)
        forwards += 1
        m = 0
        complete = False
        while True:
            if not any(nodes[m][1]):
                complete = True
                break
            p = stepwise_choice(preds[m][2], nodes[m][1])
            t = int(preds[m][0][p])
            if m < len(drafts) and (p, t) == (drafts[m][0], int(drafts[m][1])):
                m += 1
                continue
            break
        if not complete:
            accepted = [(q, int(d)) for (q, d) in drafts[:m]] + [(p, t)]
            for (q, d) in accepted:
                assert masked[q]
                tok[q], masked[q] = d, False
            rest = rank_positions(preds[m][2], nodes[m][1], exclude=p)
            drafts = [(q, int(preds[m][0][q])) for q in rest[:n_next_for(rest, has_next)]]
            hist[len(accepted)] += 1
            if trace is not None:
                trace.append(dict(S=S, accepted=list(accepted), complete=False))
            if not any(masked):                          # finished the ordinary way
                _, kv = forward_segment(w, cfg, tok, S, cache, dtype, need_logits=False)
                cache.append(kv)
                kv_passes += 1
                out += tok
                bi += 1
                if bi < len(blocks):
                    tok, masked, drafts = [mask_id] * blocks[bi][1], [True] * blocks[bi][1], []
            continue
        # every draft verified and the leaf holds the finished block
        n_acc = len(drafts)
        out += leaf_t
        cache.append(leaf_kv)
        bi += 1
        if leaf_next is None:
            hist[n_acc] += 1
            if trace is not None:
                trace.append(dict(S=S, accepted=list(drafts), complete=True))
            continue
        Bn = blocks[bi][1]
        t2, _, c2, _ = leaf_next
        tok, masked = [mask_id] * Bn, [True] * Bn
        p2 = stepwise_choice(c2, masked)
        tok[p2], masked[p2] = int(t2[p2]), False
        hist[n_acc + 1] += 1
        if trace is not None:
            trace.append(dict(S=S, accepted=list(drafts) + [(p2, int(t2[p2]))], complete=True))
        rest = rank_positions(c2, [True] * Bn, exclude=p2)
        drafts = [(q, int(t2[q])) for q in rest[:n_next_for(rest, bi + 1 < len(blocks))]]
        if not any(masked):                              # a one-position block
            _, kv = forward_segment(w, cfg, tok, P + blocks[bi][0], cache, dtype, need_logits=False)
            cache.append(kv)
            kv_passes += 1
            out += tok
            bi += 1
            if bi < len(blocks):
                tok, masked, drafts = [mask_id] * blocks[bi][1], [True] * blocks[bi][1], []
    return out, dict(forwards=forwards, kv_passes=kv_passes, accept_hist=hist)


# --------------------------------------------------------------------------
# the dual cache with periodic refresh (Section 4.1)
# --------------------------------------------------------------------------
def _refresh(w, cfg, x, dtype):
    """One forward over the whole sequence x, every position attending to every position.
    Returns (logits [T, V], keys per layer, values per layer)."""
    logits, kv = forward_segment(w, cfg, x, 0, KVCache(cfg["n_layers"]), dtype)
    return logits, [k for (k, _) in kv], [v for (_, v) in kv]


def stepwise_dual(w, cfg, prompt, gen_len, block, refresh, dtype=torch.float64):
    """Greedy stepwise decoding with the dual cache: the cache is refreshed at the start and
    whenever `refresh` tokens have been decoded since the last refresh.  Returns (tokens, stats)."""
    P = len(prompt)
    x = list(prompt) + [cfg["mask_id"]] * gen_len
    forwards = refreshes = 0
    since = None
    K = V = None
    for (off, Bj) in _blocks(gen_len, block):
        S = P + off
        masked = [True] * Bj
        while any(masked):
            if since is None or since >= refresh:
                logits, K, V = _refresh(w, cfg, x, dtype)
                logits = logits[S:S + Bj]
                refreshes += 1
                since = 0
            else:
                logits = forward_block_dual(w, cfg, x[S:S + Bj], S, K, V, dtype)
            forwards += 1
            t, _, c, _ = predict(logits, cfg["mask_id"])
            p = stepwise_choice(c, masked)
            x[S + p], masked[p] = int(t[p]), False
            since += 1
    return x[P:], dict(forwards=forwards, refreshes=refreshes)


def ssd_dual(w, cfg, prompt, gen_len, block, n_draft, refresh, dtype=torch.float64, trace=None, max_forwards=None):
    """SSD (greedy chain) with the dual cache.  A refresh forward holds the one current state (no
    chain) and supplies the next round's drafts, as a block's first forward does; a chain carries
    at most refresh - since - 1 drafts, so that no round decodes past the next refresh."""
    P = len(prompt)
    x = list(prompt) + [cfg["mask_id"]] * gen_len
    forwards = refreshes = 0
    hist = [0] * (n_draft + 2)
    since = None
    K = V = None
    for (off, Bj) in _blocks(gen_len, block):
        S = P + off
        tok, masked = [cfg["mask_id"]] * Bj, [True] * Bj
        drafts = []
        while any(masked):
            if max_forwards is not None and forwards >= max_forwards:
                return x[P:], dict(forwards=forwards, refreshes=refreshes, accept_hist=hist)
            is_refresh = since is None or since >= refresh
            if is_refresh:
                drafts = []
                logits, K, V = _refresh(w, cfg, x, dtype)
                preds = [predict(logits[S:S + Bj], cfg["mask_id"])]
                nodes = [(list(tok), list(masked))]
                refreshes += 1
                since = 0
            else:
                drafts = drafts[:max(0, min(len(drafts), sum(masked) - 1, refresh - since - 1))]
                nodes = build_chain(tok, masked, drafts)
                preds = [predict(forward_block_dual(w, cfg, nt, S, K, V, dtype), cfg["mask_id"]) for (nt, _) in nodes]
            forwards += 1
            accepted, next_drafts, m = accept_chain([p[0] for p in preds], [p[2] for p in preds],
                                                    [nm for (_, nm) in nodes], drafts, n_draft)
            if trace is not None:
                trace.append(dict(S=S, tok=list(tok), masked=list(masked), drafts=list(drafts), refresh=is_refresh,
                                  x=list(x), t=[p[0] for p in preds], m=[p[1] for p in preds],
                                  c=[p[2] for p in preds], margin=[p[3] for p in preds],
                                  accepted=list(accepted), next_drafts=list(next_drafts)))
            hist[len(accepted)] += 1
            for (q, d) in accepted:
                assert masked[q]
                tok[q], masked[q] = d, False
                x[S + q] = d
            since += len(accepted)
            drafts = next_drafts
    return x[P:], dict(forwards=forwards, refreshes=refreshes, accept_hist=hist)


def ssd_dual_spill(w, cfg, prompt, gen_len, block, n_draft, refresh, dtype=torch.float64, trace=None):
    """SSD with the dual cache and spill-over selection (Section 3.2.2; Section 4.1 for the cache).

    As ssd_dual, with two differences.
    (1) While a next block exists the chain may hold drafts for ALL remaining positions of the current
        block; if draft slots are left (at most n_draft drafts per round, and no round decodes past the
        next refresh) the chain goes on in the next block: its first node there is the next block all
        masked, the following ones have the next block's drafts written in.  Between refreshes a block's
        forward sees every other position through the cache of the last refresh, so those nodes are
        exactly the states stepwise decoding reaches once the current block is complete, and they run in
        the same forward.  The walk crosses the boundary only if every draft of the current block
        verified; at most one boundary per round; the leaf always keeps a position to predict.
    (2) A block that no verification node has predicted yet takes its drafts from the last refresh,
        whose forward covers every masked position of the sequence: all its positions by descending
        confidence.  A block therefore starts with a full chain instead of a one-node forward.
    Returns (tokens, stats) as ssd_dual."""
    P, mask_id = len(prompt), cfg["mask_id"]
    x = list(prompt) + [mask_id] * gen_len
    blocks = _blocks(gen_len, block)
    forwards = refreshes = 0
    hist = [0] * (n_draft + 2)
    since = None
    K = V = refresh_logits = None

    def from_refresh(bj):
        """Drafts for block bj (all masked at the last refresh) read off that refresh's logits."""
        off, Bn = blocks[bj]
        t, _, c, _ = predict(refresh_logits[P + off:P + off + Bn], mask_id)
        return [(q, int(t[q])) for q in rank_positions(c, [True] * Bn)]

    def walk(nodes, preds, drafts):
        """Chain walk: node m's stepwise choice must equal draft m+1.  Returns (m, p, t): m drafts matched and the
        choice (p, t) of node m, or (m, None, None) if the chain has no node m (it ends with its last draft)."""
        m = 0
        while m < len(nodes):
            p = stepwise_choice(preds[m][2], nodes[m][1])
            t = int(preds[m][0][p])
            if m < len(drafts) and (p, t) == (drafts[m][0], int(drafts[m][1])):
                m += 1
                continue
            return m, p, t
        return m, None, None

    bi, drafts, predicted = 0, [], False       # predicted: the drafts come from a node of the current block
    while bi < len(blocks):
        off, Bj = blocks[bi]
        S = P + off
        tok = x[S:S + Bj]
        masked = [t == mask_id for t in tok]
        has_next = bi + 1 < len(blocks)
        r = sum(masked)
        is_refresh = since is None or since >= refresh
        crossing, nodes_n, preds_n, nd = False, [], [], []
        if is_refresh:
            refresh_logits, K, V = _refresh(w, cfg, x, dtype)
            nodes, preds, used = [(list(tok), list(masked))], [predict(refresh_logits[S:S + Bj], mask_id)], []
            refreshes += 1
            since = 0
        else:
            if not predicted:
                drafts = from_refresh(bi) if all(masked) else []
            budget = min(n_draft, refresh - since - 1)
            a = max(0, min(len(drafts), budget, r if has_next else r - 1))
            used = drafts[:a]
            crossing = has_next and a == r
            nodes = build_chain(tok, masked, used)
            if crossing:
                nodes = nodes[:-1]                                  # the complete block has nothing left to predict
                Bn = blocks[bi + 1][1]
                nd = from_refresh(bi + 1)[:max(0, min(budget - a, Bn - 1))]
                nodes_n = build_chain([mask_id] * Bn, [True] * Bn, nd)
                preds_n = [predict(forward_block_dual(w, cfg, nt, S + Bj, K, V, dtype), mask_id) for (nt, _) in nodes_n]
            preds = [predict(forward_block_dual(w, cfg, nt, S, K, V, dtype), mask_id) for (nt, _) in nodes]
        forwards += 1
        # ---- the walk: the current block's nodes, then (if all of its drafts verified) the next block's
        m, p, t = walk(nodes, preds, used)
        crossed = p is None                     # only a chain that ends with its last draft (crossing) can run off its end
        assert crossed <= crossing
        if not crossed:
            accepted = [(q, int(d)) for (q, d) in used[:m]] + [(p, t)]
            for (q, d) in accepted:
                assert x[S + q] == mask_id
                x[S + q] = d
            rest_mask = [x[S + q] == mask_id for q in range(Bj)]
            rest = rank_positions(preds[m][2], rest_mask)
            n_next = min(n_draft, len(rest) if has_next else max(len(rest) - 1, 0))
            drafts, predicted = [(q, int(preds[m][0][q])) for q in rest[:n_next]], True
            if not any(rest_mask):
                bi += 1
                drafts, predicted = [], False
        else:
            for (q, d) in used:
                assert x[S + q] == mask_id
                x[S + q] = d
            k, p2, t2 = walk(nodes_n, preds_n, nd)
            S2, Bn = S + Bj, blocks[bi + 1][1]
            acc_n = [(q, int(d)) for (q, d) in nd[:k]] + [(p2, t2)]
            for (q, d) in acc_n:
                assert x[S2 + q] == mask_id
                x[S2 + q] = d
            accepted = [(q, int(d)) for (q, d) in used] + [(Bj + q, d) for (q, d) in acc_n]   # positions from the current block's start
            bi += 1
            rest_mask = [x[S2 + q] == mask_id for q in range(Bn)]
            rest = rank_positions(preds_n[k][2], rest_mask)
            n_next = min(n_draft, len(rest) if bi + 1 < len(blocks) else max(len(rest) - 1, 0))
            drafts, predicted = [(q, int(preds_n[k][0][q])) for q in rest[:n_next]], True
            if not any(rest_mask):
                bi += 1
                drafts, predicted = [], False
        if trace is not None:
            trace.append(dict(S=S, refresh=is_refresh, used=list(used), next_used=list(nd), crossed=crossed,
                              accepted=list(accepted), nodes=len(nodes) + len(nodes_n)))
        hist[len(accepted)] += 1
        since += len(accepted)
    return x[P:], dict(forwards=forwards, refreshes=refreshes, accept_hist=hist)


def bruteforce_full(w, cfg, prompt, gen_len, block, dtype=torch.float64):
    """Stepwise decoding in block order with no cache at all and full bidirectional attention: every
    step recomputes the whole sequence, masked future blocks included."""
    P = len(prompt)
    x = list(prompt) + [cfg["mask_id"]] * gen_len
    everyone = [0] * len(x)
    for (off, Bj) in _blocks(gen_len, block):
        masked = [True] * Bj
        while any(masked):
            logits = forward_full_blockcausal(w, cfg, x, everyone, dtype)
            t, _, c, _ = predict(logits[P + off: P + off + Bj], cfg["mask_id"])
            p = stepwise_choice(c, masked)
            x[P + off + p], masked[p] = int(t[p]), False
    return x[P:]


# --------------------------------------------------------------------------
# acceptance-rate limit of self-drafting (Section 5.1, Table 2)
# --------------------------------------------------------------------------
def token_rank(logits_row, t, mask_id):
    """Number of tokens ranked ahead of t in one row of logits: higher logit, or equal logit and lower
    id; the mask token is never a candidate."""
    ids = torch.arange(logits_row.shape[0])
    ahead = ((logits_row > logits_row[t]) | ((logits_row == logits_row[t]) & (ids < t))) & (ids != mask_id)
    return int(ahead.sum())


def limit_from_ranks(rounds, k_max):
    """rounds: per round the ranks (token_rank against the round's first logits) of the tokens its steps
    decoded.  Returns per k = 1..k_max (matched tokens, forwards an ideal tree would need)."""
    matched, forwards = [0] * k_max, [0] * k_max
    for ranks in rounds:
        for k in range(1, k_max + 1):
            m = sum(1 for r in ranks if r < k)
            matched[k - 1] += m
            forwards[k - 1] += len(ranks) - m + 1        # m >= 1: a round's first token is its logits' arg-max
    return matched, forwards


def acceptance_limit_probe(w, cfg, prompt, gen_len, block, n_draft, k_max, dtype=torch.float64):
    """Runs stepwise decoding (exact prefix cache) and records, per round of n_draft + 1 steps, how the
    decoded tokens rank in the round's first logits.  Returns (tokens, dict(steps, rounds, ranks,
    matched[k-1], forwards[k-1], reduction[k-1]))."""
    P = len(prompt)
    cache = _prefill(w, cfg, prompt, dtype)
    out, rounds = [], []
    for (off, Bj) in _blocks(gen_len, block):
        S = P + off
        tok, masked = [cfg["mask_id"]] * Bj, [True] * Bj
        step_in_round, first_logits = 0, None
        while any(masked):
            logits, _ = forward_segment(w, cfg, tok, S, cache, dtype)
            if step_in_round == 0:
                first_logits = logits
                rounds.append([])
            t, _, c, _ = predict(logits, cfg["mask_id"])
            p = stepwise_choice(c, masked)
            rounds[-1].append(token_rank(first_logits[p], int(t[p]), cfg["mask_id"]))
            tok[p], masked[p] = int(t[p]), False
            step_in_round = (step_in_round + 1) % (n_draft + 1)
        _, kv = forward_segment(w, cfg, tok, S, cache, dtype, need_logits=False)
        cache.append(kv)
        out += tok
    matched, forwards = limit_from_ranks(rounds, k_max)
    return out, dict(steps=gen_len, rounds=len(rounds), ranks=rounds, matched=matched, forwards=forwards,
                     reduction=[1.0 - f / gen_len for f in forwards])


def bruteforce(w, cfg, prompt, gen_len, block, dtype=torch.float64):
    """Stepwise decoding with no cache: one token per forward, every forward
    recomputes the whole sequence (prompt + all blocks) under the block-causal
    mask."""
    P = len(prompt)
    x = list(prompt) + [cfg["mask_id"]] * gen_len
    seg = [0] * P + [1 + i // block for i in range(gen_len)]
    forwards = 0
    for (off, Bj) in _blocks(gen_len, block):
        masked = [True] * Bj
        while any(masked):
            logits = forward_full_blockcausal(w, cfg, x, seg, dtype)
            forwards += 1
            t, m, c, _ = predict(logits[P + off: P + off + Bj], cfg["mask_id"])
            p = stepwise_choice(c, masked)
            x[P + off + p], masked[p] = int(t[p]), False
    return x[P:], dict(forwards=forwards)
