"""CPU oracle for one EAGLE-3 speculative step.  TEST INFRASTRUCTURE ONLY.

A plain, slow NumPy fp64 statement of what the paper's inference pipeline computes
(Section 3.1 "Inference Pipeline", Section 2.1 "Speculative Sampling", Section 2.2
"EAGLE and EAGLE-2", Appendix A "Implementation Details").  It exists so that tests,
the smoke check and the benchmark's CPU-baseline leg can compare the GPU library
against an independent definition.  The product path never imports it, and it shares
no code with the HIP sources.

Precision: all arithmetic is fp64.  `rounding="bf16"` additionally rounds (to nearest
even) every value that the bf16 configurations store or feed to a matrix product as a
bf16 number: weights and KV arrive already in bf16; activations entering a projection,
rotated q/k, v, the attention output and the SwiGLU product are rounded.  The residual
stream, norms, softmax, scores and logits are never rounded.

Readings of the paper used here (each is a choice where the text is silent):
  * decoder layer = LLaMA style: RMSNorm, rotate-half RoPE, grouped-query attention,
    SwiGLU MLP, no biases (the paper's targets are LLaMA/Vicuna checkpoints, Section 4
    "Models"; Appendix A "Vanilla").
  * feature of layer i = residual-stream OUTPUT of 0-based layer i, un-normed.
  * the draft layer takes the 2k-wide concatenation [RMSNorm(e(token)); RMSNorm(feature)]
    directly into its q/k/v projections (the "FC that reduces 2k to k" of Section 3.1 is
    folded into them); its residual stream carries the feature.
  * tree nodes are in creation order (parent[i] < i), node 0 is the root = last sampled token.
  * depth D = number of draft forwards = levels of drafted tokens below the root.
  * stochastic acceptance on a deterministically drafted tree treats each proposed child
    as a point-mass proposal: Section 2.1's min(1, p/p_hat) with p_hat = delta_child applied
    to the running residual distribution, child after child.

Pins (tests/, `-m "not gpu"`): the target stack against the `transformers` LLaMA
implementation incl. its 4-D mask path for tree attention; chain tree == causal decoding;
mask form == explicit-ancestor-path brute force; fusion == a matmul with block-identity
cases; draft layer against composed library modules and the one-at-a-time == sequence
invariant; expansion against brute-force enumeration of the full K-ary tree; greedy walk
against autoregressive argmax decoding; stochastic walk by chi-square on a tiny vocabulary
and the closed form P(emit x) = p(x).  The bf16 rounding points (operands of every weight
product, rotated queries / keys and values; nothing else) are pinned against the library model
with torch's bfloat16 cast hooked onto exactly those operands, with a leave-one-out control.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------- helpers

def as_f64(x) -> np.ndarray:
    """Torch (any float dtype, CPU) or NumPy array -> float64 NumPy array, value-exact."""
    if hasattr(x, "detach"):
        x = x.detach().cpu()
        if x.dtype.is_floating_point:
            return x.to(dtype=__import__("torch").float64).numpy()
        return x.numpy()
    return np.asarray(x, dtype=np.float64)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even to bfloat16 precision (via fp32), returned as float64."""
    f = np.ascontiguousarray(np.asarray(x, dtype=np.float32))
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(f.shape)


def _rounder(rounding):
    """"none" / "bf16", or a callable applied at the same places (e.g. a test's noisy variant of bf16_round)."""
    if callable(rounding):
        return rounding
    if rounding in (None, "none", "fp64", "fp32"):
        return lambda a: a
    if rounding == "bf16":
        return bf16_round
    raise ValueError(rounding)


def rmsnorm(x, w, eps):
    """RMSNorm(x; w) = w * x / sqrt(mean(x^2) + eps), over the last axis."""
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * w


def rope(x, pos, theta):
    """Rotary embedding, rotate-half pairing (i, i + d/2).  x [..., M, heads, d], pos [M]."""
    d = x.shape[-1]
    half = d // 2
    inv = theta ** (-np.arange(half, dtype=np.float64) * 2.0 / d)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv[None, :]      # [M, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def log_softmax(z):
    m = np.max(z, axis=-1, keepdims=True)
    return z - m - np.log(np.sum(np.exp(z - m), axis=-1, keepdims=True))


def softmax(z):
    e = np.exp(z - np.max(z, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def tree_depth(parent):
    parent = np.asarray(parent)
    depth = np.zeros(len(parent), dtype=np.int64)
    for i in range(1, len(parent)):
        assert 0 <= parent[i] < i, "nodes must be in creation order"
        depth[i] = depth[parent[i]] + 1
    return depth


def ancestor_paths(parent):
    """paths[i] = [root, ..., i]: the explicit ancestor chain of every node."""
    paths = []
    for i in range(len(parent)):
        p, cur = [], i
        while cur >= 0:
            p.append(cur)
            cur = int(parent[cur])
        paths.append(p[::-1])
    return paths


def ancestor_mask(parent):
    """visible[i, j] = node j is node i or one of its ancestors (Section 2.2, tree attention)."""
    n = len(parent)
    vis = np.zeros((n, n), dtype=bool)
    for i, p in enumerate(ancestor_paths(parent)):
        vis[i, p] = True
    return vis


# ----------------------------------------------------------------------------- attention

def attention_prefix_tail(q, K, V, n_prefix, tail_vis):
    """Mask form.  q [M,H,d]; K,V [n_prefix+T,Hkv,d]; row i sees every slot < n_prefix and tail
    slot n_prefix+j iff tail_vis[i,j].  Query head h reads KV head h*Hkv//H.  Returns [M,H,d]."""
    M, H, d = q.shape
    Hkv = K.shape[1]
    T = K.shape[0] - n_prefix
    assert tail_vis.shape == (M, T)
    out = np.empty_like(q)
    scale = 1.0 / np.sqrt(d)
    bias = np.concatenate([np.zeros((M, n_prefix)), np.where(tail_vis, 0.0, -np.inf)], axis=1)
    for h in range(H):
        g = h * Hkv // H
        s = q[:, h, :] @ K[:, g, :].T * scale + bias
        out[:, h, :] = softmax(s) @ V[:, g, :]
    return out


def attention_explicit_sets(q, K, V, visible_slots):
    """Brute-force form: row i runs ordinary softmax attention over exactly the listed slots."""
    M, H, d = q.shape
    Hkv = K.shape[1]
    out = np.empty_like(q)
    for i in range(M):
        idx = np.asarray(visible_slots[i], dtype=np.int64)
        for h in range(H):
            g = h * Hkv // H
            s = K[idx, g, :] @ q[i, h, :] / np.sqrt(d)
            out[i, h, :] = softmax(s) @ V[idx, g, :]
    return out


def ttt_visible_sets(T, s):
    """Training-time test, simulated step s (Section 3.2, Figure 6; s = 0 is the native step): query i of step s sees
    the ORIGINAL training positions 0..i (ordinary causal context) and, of every simulated step t = 1..s, only
    position i itself (those masks are diagonal).  Keys are numbered t * T + j.  Returns the list of visible key
    numbers per query."""
    return [list(range(i + 1)) + [t * T + i for t in range(1, s + 1)] for i in range(T)]


def ttt_attention(q, K_steps, V_steps, form="sets"):
    """Self-attention of the draft layer during a training-time-test step (Section 3.2).  q [T,H,d] = the queries of
    step s; K_steps, V_steps [s+1, T, Hkv, d] = keys / values of the original inputs (index 0) and of the simulated
    steps 1..s (index s = this step's own).  form "sets": every query runs plain softmax attention over exactly its
    visible keys; form "mask": one dense masked attention over all (s+1) T keys.  Returns [T,H,d]."""
    n_steps, T = K_steps.shape[0], K_steps.shape[1]
    s = n_steps - 1
    K = K_steps.reshape(n_steps * T, *K_steps.shape[2:])
    V = V_steps.reshape(n_steps * T, *V_steps.shape[2:])
    sets = ttt_visible_sets(T, s)
    if form == "sets":
        return attention_explicit_sets(q, K, V, sets)
    vis = np.zeros((T, n_steps * T), dtype=bool)
    for i, idx in enumerate(sets):
        vis[i, idx] = True
    return attention_prefix_tail(q, K, V, 0, vis)


# ----------------------------------------------------------------------------- target model

def _mlp(n2, W, rd):
    return rd(silu(n2 @ W["w_gate"].T) * (n2 @ W["w_up"].T)) @ W["w_down"].T


def decoder_layer(x, W, pos, K_ctx, V_ctx, tail_vis, shape, rd, attention="mask", parent=None):
    """One LLaMA-style layer over M new rows against a cached context.
    Returns (x_out [M,k], k_new [M,Hkv,d], v_new)."""
    M = x.shape[0]
    H, Hkv, d = shape.n_heads, shape.n_kv_heads, shape.head_dim
    n1 = rd(rmsnorm(x, W["norm_attn"], shape.rms_eps))
    q = (n1 @ W["wq"].T).reshape(M, H, d)
    k = (n1 @ W["wk"].T).reshape(M, Hkv, d)
    v = (n1 @ W["wv"].T).reshape(M, Hkv, d)
    q, k, v = rd(rope(q, pos, shape.rope_theta)), rd(rope(k, pos, shape.rope_theta)), rd(v)
    P = K_ctx.shape[0]
    K = np.concatenate([K_ctx, k], axis=0)
    V = np.concatenate([V_ctx, v], axis=0)
    if attention == "mask":
        att = attention_prefix_tail(q, K, V, P, tail_vis)
    else:   # explicit ancestor paths, brute force
        paths = ancestor_paths(parent)
        att = attention_explicit_sets(q, K, V, [list(range(P)) + [P + j for j in paths[i]] for i in range(M)])
    x1 = x + rd(att.reshape(M, H * d)) @ W["wo"].T
    n2 = rd(rmsnorm(x1, W["norm_mlp"], shape.rms_eps))
    return x1 + _mlp(n2, W, rd), k, v


def tree_verify(shape, get_layer, tg, tree_tok, parent, get_kv, rounding="none",
                attention="mask", keep_hidden=False, x0=None, layers=None):
    """Target forward over all tree nodes of ONE sequence under the ancestor-only mask.

    get_layer(l) -> dict of float64 arrays; tg = {"embed","final_norm","lm_head"};
    get_kv(l) -> (K_ctx, V_ctx) [P,Hkv,d] float64 (the prefix cache of layer l).
    Node i sits at position P + depth(i).  Returns dict(logits [N,V], taps [3,N,k],
    k_new/v_new [L,N,Hkv,d], hidden [L+1,N,k] if keep_hidden).
    `x0`/`layers` allow teacher-forced checks of a sub-range of layers."""
    rd = _rounder(rounding)
    parent = np.asarray(parent)
    depth = tree_depth(parent)
    vis = ancestor_mask(parent)
    x = as_f64(tg["embed"])[np.asarray(tree_tok)] if x0 is None else np.array(x0, dtype=np.float64)
    taps = np.zeros((3,) + x.shape)
    hidden = [x.copy()]
    ks, vs = [], []
    for l in (range(shape.n_layers) if layers is None else layers):
        K_ctx, V_ctx = get_kv(l)
        x, k, v = decoder_layer(x, get_layer(l), K_ctx.shape[0] + depth, K_ctx, V_ctx, vis, shape, rd,
                                attention=attention, parent=parent)
        ks.append(k); vs.append(v)
        for t in range(3):
            if shape.taps[t] == l:
                taps[t] = x
        if keep_hidden:
            hidden.append(x.copy())
    out = {"taps": taps, "k_new": np.stack(ks), "v_new": np.stack(vs), "x_final": x}
    if tg.get("lm_head") is not None:
        nf = rd(rmsnorm(x, as_f64(tg["final_norm"]), shape.rms_eps))
        out["logits"] = nf @ as_f64(tg["lm_head"]).T
    if keep_hidden:
        out["hidden"] = np.stack(hidden)
    return out


# ----------------------------------------------------------------------------- draft model

def fuse_features(w_fc, low, mid, high, rounding="none"):
    """g = W_fc [l; m; h]  (Section 3.1: concatenate the three k-vectors, one FC back to k)."""
    rd = _rounder(rounding)
    return rd(np.concatenate([low, mid, high], axis=-1)) @ w_fc.T


def draft_forward(shape, dw, embed, f, tok, pos, K, V, n_prefix, slot0, tail_vis, rd):
    """One forward of the draft layer over M rows (feature f[i], target-vocab token tok[i]).
    K, V are the draft cache [cap,Hkv,d]; this call writes slots slot0..slot0+M-1 (all inside the
    tail region, which starts at n_prefix and has tail_vis.shape[1] slots) and reads slots
    < n_prefix plus the visible tail slots.  Returns (a [M,k], z [M,Vd])."""
    M = f.shape[0]
    H, Hkv, d = shape.n_heads, shape.n_kv_heads, shape.head_dim
    W = dw["layer"]
    e = embed[np.asarray(tok)]
    u = rd(np.concatenate([rmsnorm(e, dw["norm_embed"], shape.rms_eps),
                           rmsnorm(f, dw["norm_feat"], shape.rms_eps)], axis=-1))
    q = rd(rope((u @ W["wq"].T).reshape(M, H, d), pos, shape.rope_theta))
    k = rd(rope((u @ W["wk"].T).reshape(M, Hkv, d), pos, shape.rope_theta))
    v = rd((u @ W["wv"].T).reshape(M, Hkv, d))
    K[slot0:slot0 + M] = k
    V[slot0:slot0 + M] = v
    T = tail_vis.shape[1]
    att = attention_prefix_tail(q, K[:n_prefix + T], V[:n_prefix + T], n_prefix, tail_vis)
    y1 = f + rd(att.reshape(M, H * d)) @ W["wo"].T
    a = y1 + _mlp(rd(rmsnorm(y1, W["norm_mlp"], shape.rms_eps)), W, rd)
    z = rd(rmsnorm(a, dw["final_norm"], shape.rms_eps)) @ dw["lm_head"].T
    return a, z


def topk_desc(val, ids, K):
    """Positions of the K best entries: larger value first, ties -> smaller id."""
    order = np.lexsort((ids, -val))
    return order[:K]


def _check_pick(val, ids, picks, K, tol, what):
    """Is `picks` (positions, ordered) an admissible top-K of `val` up to near-ties <= tol?"""
    picks = np.asarray(picks, dtype=np.int64)
    exact = topk_desc(val, ids, K)
    if np.array_equal(picks, exact):
        return False
    assert len(set(picks.tolist())) == K, f"{what}: duplicate picks"
    kth = val[exact[-1]]
    assert np.all(val[picks] >= kth - tol), f"{what}: picked an entry more than tol below the K-th best"
    must = np.nonzero(val > kth + tol)[0]
    assert set(must.tolist()) <= set(picks.tolist()), f"{what}: missed an entry more than tol above the K-th best"
    assert np.all(val[picks][:-1] >= val[picks][1:] - tol), f"{what}: picks out of order beyond tol"
    return True


def draft_expand(shape, dw, embed, g_new, tok_new, K_cache, V_cache, n_ctx, depth, topk, n_nodes,
                 rounding="none", follow=None, tol=1e-2):
    """Draft-tree expansion with per-level top-K frontier and final global rerank
    (Section 2.2: confidence-driven dynamic tree, pruned at the end of drafting; Appendix A:
    total draft tokens, depth, nodes selected per expansion).

    dw: float64 draft weights (incl. "d2t" int map draft id -> target id); embed: target embedding
    [V,k] float64.  g_new [n_new,k], tok_new [n_new] (target ids; tok_new[j] FOLLOWS the position
    whose features gave g_new[j]; the last one is the tree root).  K_cache/V_cache: draft cache
    arrays [>= n_ctx + n_new + (depth-1)*topk, Hkv, d] whose first n_ctx slots hold the draft
    context; they are extended in place.

    Pool ids: 0 = root; level 1 -> 1..K in rank order; level l>=2 -> base_l + r*K + c for the c-th
    best token of the r-th frontier node.  Ordering everywhere: larger score first, ties -> smaller
    id.  `follow` (optional) = {"pool_tok","frontier","chosen"} as emitted by another
    implementation: wherever its pick differs from this one's, it is accepted iff admissible within
    `tol` (see _check_pick), adopted, and counted in "n_followed"; anything else raises.
    """
    rd = _rounder(rounding)
    D, Kk = depth, topk
    n_new = g_new.shape[0]
    d2t = np.asarray(dw["d2t"], dtype=np.int64)
    Vd = dw["lm_head"].shape[0]
    all_ids = np.arange(Vd)
    pool_size = 1 + Kk + (D - 1) * Kk * Kk
    p_tok = np.zeros(pool_size, dtype=np.int64)        # draft-vocab ids (root: unused)
    p_par = np.full(pool_size, -1, dtype=np.int64)
    p_dep = np.zeros(pool_size, dtype=np.int64)
    p_score = np.zeros(pool_size)
    n_followed, min_gap = 0, np.inf

    def row_topk(logp, base, what):
        nonlocal n_followed, min_gap
        pick = topk_desc(logp, all_ids, Kk + 1)
        min_gap = min(min_gap, float(np.min(-np.diff(logp[pick]))))
        pick = pick[:Kk]
        if follow is not None:
            theirs = np.asarray(follow["pool_tok"][base:base + Kk], dtype=np.int64)
            if _check_pick(logp, all_ids, theirs, Kk, tol, what):
                n_followed += 1
                pick = theirs
        return pick

    # forward 1: the n_new freshly verified positions, causal among themselves
    pos1 = n_ctx + np.arange(n_new)
    a, z = draft_forward(shape, dw, embed, np.asarray(g_new, dtype=np.float64), tok_new, pos1,
                         K_cache, V_cache, n_ctx, n_ctx, np.tril(np.ones((n_new, n_new), dtype=bool)), rd)
    logp = log_softmax(z[-1])
    pick = row_topk(logp, 1, "level 1 top-k")
    p_tok[1:1 + Kk] = pick
    p_par[1:1 + Kk] = 0
    p_dep[1:1 + Kk] = 1
    p_score[1:1 + Kk] = logp[pick]
    feat = {int(i): a[-1] for i in range(1, 1 + Kk)}       # feature fed with a candidate = its parent's output
    frontier = np.arange(1, 1 + Kk)
    frontiers = [frontier.copy()]
    slot_of = {}                                           # pool id -> tail slot (once it has been run)
    n_vis = n_ctx + n_new
    for lvl in range(2, D + 1):
        base = 1 + Kk + (lvl - 2) * Kk * Kk
        T = (lvl - 1) * Kk
        tail_vis = np.zeros((Kk, T), dtype=bool)
        for r, c in enumerate(frontier):
            slot_of[int(c)] = (lvl - 2) * Kk + r
            cur = int(c)
            while cur > 0:                                 # itself and every drafted ancestor
                tail_vis[r, slot_of[cur]] = True
                cur = int(p_par[cur])
        f_rows = np.stack([feat[int(c)] for c in frontier])
        toks = d2t[p_tok[frontier]]
        pos = np.full(Kk, n_ctx + n_new - 1 + (lvl - 1))
        a, z = draft_forward(shape, dw, embed, f_rows, toks, pos, K_cache, V_cache, n_vis,
                             n_vis + (lvl - 2) * Kk, tail_vis, rd)
        lp = log_softmax(z)
        for r, c in enumerate(frontier):
            b = base + r * Kk
            pick = row_topk(lp[r], b, f"level {lvl} row {r} top-k")
            p_tok[b:b + Kk] = pick
            p_par[b:b + Kk] = c
            p_dep[b:b + Kk] = lvl
            p_score[b:b + Kk] = p_score[c] + lp[r][pick]
            for i in range(b, b + Kk):
                feat[i] = a[r]
        if lvl < D:
            ids = np.arange(base, base + Kk * Kk)
            sc = p_score[ids]
            sel = topk_desc(sc, ids, Kk + 1)
            if len(sel) > Kk:
                min_gap = min(min_gap, float(sc[sel[Kk - 1]] - sc[sel[Kk]]))
            sel = sel[:Kk]
            if follow is not None:
                theirs = np.asarray(follow["frontier"][lvl - 1], dtype=np.int64) - base
                if _check_pick(sc, ids, theirs, Kk, tol, f"level {lvl} frontier"):
                    n_followed += 1
                    sel = theirs
            frontier = ids[sel]
            frontiers.append(frontier.copy())
    # global rerank over every drafted candidate
    n_keep = n_nodes - 1
    ids = np.arange(1, pool_size)
    sc = p_score[1:]
    sel = topk_desc(sc, ids, min(n_keep + 1, len(ids)))
    if len(sel) > n_keep:
        min_gap = min(min_gap, float(sc[sel[n_keep - 1]] - sc[sel[n_keep]]))
    sel = sel[:n_keep]
    if follow is not None:
        theirs_sorted = np.asarray(follow["chosen"], dtype=np.int64) - 1     # ascending pool id
        theirs = theirs_sorted[np.lexsort((theirs_sorted, -sc[theirs_sorted]))]
        mine_set, theirs_set = set(sel.tolist()), set(theirs.tolist())
        if mine_set != theirs_set:
            _check_pick(sc, ids, theirs, n_keep, tol, "global rerank")
            n_followed += 1
            sel = theirs
    chosen = np.sort(ids[sel])
    node_of = {0: 0}
    for n, pid in enumerate(chosen, start=1):
        node_of[int(pid)] = n
    tree_tok = np.concatenate([[int(tok_new[-1])], d2t[p_tok[chosen]]]).astype(np.int64)
    parent = np.array([-1] + [node_of[int(p_par[pid])] for pid in chosen], dtype=np.int64)
    return {
        "tree_tok": tree_tok, "parent": parent, "depth": np.concatenate([[0], p_dep[chosen]]),
        "score": np.concatenate([[0.0], p_score[chosen]]),
        "pool_tok": p_tok, "pool_parent": p_par, "pool_depth": p_dep, "pool_score": p_score,
        "frontier": frontiers, "chosen": chosen, "n_followed": n_followed, "min_gap": min_gap,
    }


def draft_chains(shape, dw, embed, g_new, tok_new, caches, n_ctx, length, rounding="none"):
    """Chain drafting for a batch (Section 4.3 / 4.4: chains of 2-3 draft tokens, no tree, at large batch sizes):
    every sequence independently runs the draft steps of Section 3.1 with ONE proposal per step, i.e. the
    expansion above with top-k 1.  g_new[b] [n_b, k], tok_new[b] [n_b], caches[b] = (K, V) draft cache arrays
    (extended in place), n_ctx[b] valid entries.  Returns (chain_tok [B, length+1] with the root first,
    chain_logp [B, length+1] cumulative)."""
    toks, logps = [], []
    for b in range(len(g_new)):
        t = draft_expand(shape, dw, embed, np.asarray(g_new[b], dtype=np.float64), np.asarray(tok_new[b]),
                         caches[b][0], caches[b][1], int(n_ctx[b]), length, 1, length + 1, rounding=rounding)
        assert np.array_equal(t["parent"], np.arange(-1, length))
        toks.append(t["tree_tok"]); logps.append(t["score"])
    return np.stack(toks), np.stack(logps)


# ----------------------------------------------------------------------------- acceptance

def _children(parent, node):
    return [c for c in range(len(parent)) if parent[c] == node]


def accept_greedy(logits, tree_tok, parent):
    """Temperature 0 (Section 2.1 with a deterministic target): follow the child whose token is the
    target's argmax (ties -> smaller id); stop at the first node where no child matches; the argmax
    there is the bonus token.  Returns (accept_len, path node ids, bonus token)."""
    cur, path = 0, [0]
    while True:
        x = int(np.argmax(logits[cur]))          # first maximal index
        nxt = [c for c in _children(parent, cur) if int(tree_tok[c]) == x]
        if not nxt:
            return len(path) - 1, path, x
        cur = nxt[0]
        path.append(cur)


def accept_stochastic(logits, tree_tok, parent, temperature, U, return_info=False):
    """Temperature > 0.  At node `cur` with target distribution p = softmax(logits/T): test its
    children in ascending node id; child c (token t) is accepted with probability
    p[t] / (1 - rejected mass) using U[2c]; a rejected child's token is struck from the residual.
    When no child is accepted the bonus token is drawn by inverse CDF (vocabulary order) from the
    renormalised residual using U[2*cur+1].  Returns (accept_len, path, bonus, margin) where margin is
    the smallest distance of any uniform used from its decision threshold (in probability units).
    With return_info a fifth value describes the final draw: the residual CDF (un-normalised, vocabulary
    order), the target it was searched for, and the margin of the child tests alone, so that a checker can
    decide whether another implementation's bonus token is admissible within its rounding error."""
    cur, path, margin, margin_children = 0, [0], np.inf, np.inf
    while True:
        p = softmax(np.asarray(logits[cur], dtype=np.float64) / temperature)
        rej, struck, accepted = 0.0, [], None
        for c in _children(parent, cur):
            t = int(tree_tok[c])
            thr = p[t] / (1.0 - rej) if t not in struck else 0.0
            r = float(U[2 * c])
            margin = min(margin, abs(r - thr) * (1.0 - rej))
            margin_children = margin
            if r < thr:
                accepted = c
                break
            if t not in struck:
                rej += p[t]
                struck.append(t)
        if accepted is not None:
            cur = accepted
            path.append(cur)
            continue
        res = p.copy()
        res[struck] = 0.0
        cdf = np.cumsum(res)
        target = float(U[2 * cur + 1]) * (1.0 - rej)
        hit = np.nonzero((cdf >= target) & (res > 0.0))[0]
        if len(hit):
            bonus = int(hit[0])
        else:                                    # rounding left the running sum short of the target
            bonus = int(np.nonzero(res > 0.0)[0][-1])
        margin = min(margin, float(np.min(np.abs(cdf - target))))
        if return_info:
            return len(path) - 1, path, bonus, margin, {"cdf": cdf, "target": target, "residual": res,
                                                        "margin_children": margin_children}
        return len(path) - 1, path, bonus, margin


def bonus_admissible(info, bonus, eps):
    """True iff `bonus` is a token the inverse-CDF draw could return when every partial sum carries an
    absolute error of at most eps: it has residual mass and its CDF interval, widened by eps, holds the target."""
    cdf, target, res = info["cdf"], info["target"], info["residual"]
    if not (0 <= bonus < len(cdf)) or res[bonus] <= 0.0:
        return False
    lo = cdf[bonus] - res[bonus]
    return lo - eps <= target <= cdf[bonus] + eps


# ----------------------------------------------------------------------------- across steps

def commit_path(tree_tok, path, bonus, taps, k_new, v_new):
    """What one step hands to the next (Section 2.1: the accepted draft tokens are kept, everything after the first
    rejection is discarded; Section 3.1: the features recorded during this verification feed the next draft).
    path = accepted node ids from the root (accept_len + 1 of them).  Returns
      k_keep, v_keep [L, n, Hkv, d]  cache rows of the accepted nodes, in path order (they extend the prefix)
      taps_new [3, n, k]             low / mid / high features of the accepted positions
      tok_new [n]                    the token FOLLOWING each accepted position: the next node on the path, and the
                                     bonus token after the last one (the next step's root)
    with n = accept_len + 1."""
    path = np.asarray(path, dtype=np.int64)
    tok_new = np.concatenate([np.asarray(tree_tok, dtype=np.int64)[path[1:]], [int(bonus)]])
    return k_new[:, path], v_new[:, path], taps[:, path], tok_new


def greedy_decode(shape, get_layer, tg, prompt, n_tokens):
    """Ordinary autoregressive arg-max decoding of the target (Appendix A "Vanilla"), the reference that greedy
    speculative decoding must reproduce token for token.  Plain and slow: one full causal forward per token."""
    toks = [int(t) for t in prompt]
    for _ in range(n_tokens):
        out = prefill(shape, get_layer, tg, np.asarray(toks))
        toks.append(int(np.argmax(out["logits"][-1])))
    return toks[len(prompt):]


def speculative_decode(shape, get_layer, tg, dw, prompt, n_steps, depth, topk, n_nodes, temperature=0.0,
                       uniforms=None, tree_hook=None, rounding="none"):
    """The whole pipeline of Section 3.1 over several draft-verify cycles, one sequence.

    Prefill: target forward over the prompt (its taps are the features g of every prompt position, its last arg-max
    is the first root), draft cache = the draft layer's keys/values over (g_i, token_{i+1}).  Each cycle: draft tree
    from the features of the positions accepted last cycle, tree verification, acceptance walk, commit.
    tree_hook(step, tree_tok, parent, depth) -> tree_tok lets a test replace drafted tokens (the tree's SHAPE stays the
    draft's).  Returns dict(tokens = everything emitted after the prompt, accept_lens, trees, per-step records)."""
    rd = _rounder(rounding)
    embed = tg["embed"]
    prompt = np.asarray(prompt, dtype=np.int64)
    P = len(prompt)
    pre = prefill(shape, get_layer, tg, prompt, rounding=rounding)
    K_t = [pre["k_new"][l] for l in range(shape.n_layers)]          # target cache per layer [P, Hkv, d]
    V_t = [pre["v_new"][l] for l in range(shape.n_layers)]
    g_all = fuse_features(dw["w_fc"], pre["taps"][0], pre["taps"][1], pre["taps"][2], rounding=rounding)
    cap = P + n_steps * (depth + 1) + (depth - 1) * topk + 8
    Kd = np.zeros((cap, shape.n_kv_heads, shape.head_dim))
    Vd = np.zeros_like(Kd)
    if P > 1:                                                        # draft rows (g_i, token_{i+1}), i < P-1
        draft_forward(shape, dw, embed, g_all[:P - 1], prompt[1:], np.arange(P - 1), Kd, Vd, 0, 0,
                      np.tril(np.ones((P - 1, P - 1), dtype=bool)), rd)
    n_d = P - 1                                                      # valid draft cache entries
    root = int(np.argmax(pre["logits"][-1])) if temperature == 0 else None
    assert root is not None, "the first token is taken greedily by the caller; pass temperature 0 or extend here"
    g_new, tok_new = g_all[P - 1:P], np.array([root], dtype=np.int64)
    emitted, accept_lens, records = [root], [], []
    for step in range(n_steps):
        tree = draft_expand(shape, dw, embed, g_new, tok_new, Kd, Vd, n_d, depth, topk, n_nodes, rounding=rounding)
        n_d += len(tok_new)                                          # forward 1's rows stay in the draft cache
        tree_tok = tree["tree_tok"] if tree_hook is None else np.asarray(
            tree_hook(step, tree["tree_tok"].copy(), tree["parent"], tree["depth"], emitted))
        ver = tree_verify(shape, get_layer, tg, tree_tok, tree["parent"], lambda l: (K_t[l], V_t[l]), rounding=rounding)
        if temperature == 0:
            n_acc, path, bonus = accept_greedy(ver["logits"], tree_tok, tree["parent"])
        else:
            n_acc, path, bonus, _ = accept_stochastic(ver["logits"], tree_tok, tree["parent"], temperature, uniforms[step])
        k_keep, v_keep, taps_new, tok_new = commit_path(tree_tok, path, bonus, ver["taps"], ver["k_new"], ver["v_new"])
        for l in range(shape.n_layers):
            K_t[l] = np.concatenate([K_t[l], k_keep[l]], axis=0)
            V_t[l] = np.concatenate([V_t[l], v_keep[l]], axis=0)
        g_new = fuse_features(dw["w_fc"], taps_new[0], taps_new[1], taps_new[2], rounding=rounding)
        emitted += [int(t) for t in tok_new]
        accept_lens.append(n_acc)
        records.append({"tree_tok": tree_tok, "parent": tree["parent"], "path": path, "bonus": bonus, "tok_new": tok_new})
    return {"tokens": emitted, "accept_lens": accept_lens, "records": records,
            "tau": float(np.mean(np.asarray(accept_lens) + 1.0))}


# ----------------------------------------------------------------------------- plumbing for whole-step use

def weights_f64(d):
    """Recursively convert a dict of torch/NumPy float tensors to float64 NumPy (ints kept)."""
    out = {}
    for k, v in d.items():
        if isinstance(v, dict):
            out[k] = weights_f64(v)
        elif hasattr(v, "dtype") and not str(v.dtype).startswith(("torch.int", "int")):
            out[k] = as_f64(v)
        else:
            out[k] = np.asarray(v.cpu() if hasattr(v, "cpu") else v)
    return out


def prefill(shape, get_layer, tg, tokens, rounding="none"):
    """Ordinary causal forward of the target over `tokens` (a chain tree on an empty cache).
    Returns the same dict as tree_verify plus per-layer K/V of every position."""
    parent = np.arange(-1, len(tokens) - 1)
    empty = np.zeros((0, shape.n_kv_heads, shape.head_dim))
    return tree_verify(shape, get_layer, tg, tokens, parent, lambda l: (empty, empty), rounding=rounding)
