"""Counter-based synthetic tensors, bit-identical on CPU and GPU.

Every value is a pure function of (seed, tensor id, flat index): a splitmix64-style
integer hash gives four 16-bit fields per 64-bit word, each field indexes a
65 536-entry table of standard-normal quantiles computed once on the host in fp64.
Only integer arithmetic and a table gather run on the device, so the CPU oracle's
tests and the GPU tests see exactly the same bits without shipping gigabytes.

Distributions (the paper evaluates trained checkpoints on public prompt sets; neither
is available here, so only the SHAPES of LLaMA-3.1-8B / 3.3-70B and the tree
hyper-parameters of the paper's Appendix A are kept):
  weights     N(0, 0.02)            norm gains  1 + N(0, 0.02)
  KV caches   N(0, 1)               features    N(0, 1)
  token ids   uniform in the vocabulary
"""
from functools import lru_cache

import numpy as np
import torch

SEED = 20250301

_MASK64 = (1 << 64) - 1
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_G = 0x9E3779B97F4A7C15


def _s64(v: int) -> int:
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


def _mix_py(x: int) -> int:
    x &= _MASK64
    x = ((x ^ (x >> 30)) * _M1) & _MASK64
    x = ((x ^ (x >> 27)) * _M2) & _MASK64
    return x ^ (x >> 31)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(x: torch.Tensor) -> torch.Tensor:
    x = (x ^ _lsr(x, 30)) * _s64(_M1)
    x = (x ^ _lsr(x, 27)) * _s64(_M2)
    return x ^ _lsr(x, 31)


def _key(seed: int, tid: int) -> int:
    return _mix_py(_mix_py(seed) + tid * _G)


def _hashes(seed: int, tid: int, start: int, count: int, device) -> torch.Tensor:
    j = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _mix(j * _s64(_G) + _s64(_key(seed, tid)))


@lru_cache(maxsize=None)
def _quantiles() -> torch.Tensor:
    from scipy.special import ndtri
    p = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
    return torch.from_numpy(ndtri(p))


@lru_cache(maxsize=None)
def _table(std: float, mean: float, dtype: torch.dtype, device: str) -> torch.Tensor:
    return (_quantiles() * std + mean).to(dtype).to(device)


_CHUNK = 1 << 23   # hashes per chunk (4 values each)


def normal(seed, tid, shape, std=1.0, mean=0.0, dtype=torch.float32, device="cpu", start=0):
    """Tensor of `shape` whose flat element i is table[field((start+i)%4) of hash((start+i)//4)]*std+mean, in
    `dtype`.  `start` (a multiple of 4) selects a window of the tensor's stream, e.g. some rows of a cache."""
    shape = tuple(int(s) for s in shape)
    numel = int(np.prod(shape)) if shape else 1
    assert start % 4 == 0
    table = _table(float(std), float(mean), dtype, str(device))
    out = torch.empty(numel, dtype=dtype, device=device)
    n_hash = (numel + 3) // 4
    for h0 in range(0, n_hash, _CHUNK):
        cnt = min(_CHUNK, n_hash - h0)
        h = _hashes(seed, tid, start // 4 + h0, cnt, device)
        idx = torch.stack([(h >> (16 * f)) & 0xFFFF for f in range(4)], dim=1).reshape(-1)
        lo = 4 * h0
        hi = min(numel, lo + 4 * cnt)
        out[lo:hi] = table[idx[: hi - lo]]
        del h, idx
    return out.reshape(shape)


def uniform01(seed, tid, shape, device="cpu"):
    """fp32 uniforms in [0,1) with 24 random bits each."""
    numel = int(np.prod(shape))
    h = _hashes(seed, tid, 0, numel, device)
    return (_lsr(h, 40).to(torch.float32) / float(1 << 24)).reshape(tuple(shape))


def uniform_ints(seed, tid, shape, lo, hi, device="cpu"):
    """int32 values uniform in [lo, hi)."""
    numel = int(np.prod(shape))
    h = _hashes(seed, tid, 0, numel, device)
    return (_lsr(h, 33) % (hi - lo) + lo).to(torch.int32).reshape(tuple(shape))


def make_d2t(seed, vocab, draft_vocab, device="cpu"):
    """Strictly increasing int32 map draft id -> target id (identity when the vocabularies match)."""
    i = torch.arange(draft_vocab, dtype=torch.int64, device=device)
    if draft_vocab == vocab:
        return i.to(torch.int32)
    lo = (i * vocab) // draft_vocab
    gap = ((i + 1) * vocab) // draft_vocab - lo
    r = _lsr(_hashes(seed, TensorIds.D2T, 0, draft_vocab, device), 33) % gap
    return (lo + r).to(torch.int32)


class TensorIds:
    EMBED, FINAL_NORM, LM_HEAD = 1, 2, 3
    D2T = 9
    LAYER0 = 1000          # + 16*layer + slot
    WQ, WK, WV, WO, WGATE, WUP, WDOWN, NORM_ATTN, NORM_MLP = range(9)
    DRAFT0 = 100           # draft layer slots use the same offsets
    D_FC, D_NORM_EMBED, D_NORM_FEAT, D_FINAL_NORM, D_LM_HEAD = 120, 121, 122, 123, 124
    KV0 = 100000           # + 2*layer (+1 for V)
    DRAFT_KV = 90000
    TAPS, G_NEW, TOK_NEW, PREFIX_TOK, UNIFORMS, TREE, TREE_TOK, PREFIX_LEN, LOGITS = range(200, 209)


def _tdtype(shape):
    return torch.float32 if shape.dtype == "fp32" else torch.bfloat16


def _layer(shape, base, in_dim, seed, device):
    k, I, dt = shape.hidden, shape.intermediate, _tdtype(shape)
    T = TensorIds
    w = lambda slot, dims: normal(seed, base + slot, dims, 0.02, 0.0, dt, device)
    g = lambda slot: normal(seed, base + slot, (k,), 0.02, 1.0, dt, device)
    return {
        "wq": w(T.WQ, (shape.q_dim, in_dim)), "wk": w(T.WK, (shape.kv_dim, in_dim)),
        "wv": w(T.WV, (shape.kv_dim, in_dim)), "wo": w(T.WO, (k, shape.q_dim)),
        "w_gate": w(T.WGATE, (I, k)), "w_up": w(T.WUP, (I, k)), "w_down": w(T.WDOWN, (k, I)),
        "norm_attn": g(T.NORM_ATTN), "norm_mlp": g(T.NORM_MLP),
    }


def layer_weights(shape, layer, seed=SEED, device="cpu"):
    """Weights of target decoder layer `layer`: [out, in] row-major, storage dtype of the shape."""
    return _layer(shape, TensorIds.LAYER0 + 16 * layer, shape.hidden, seed, device)


def target_globals(shape, seed=SEED, device="cpu"):
    dt, T = _tdtype(shape), TensorIds
    return {
        "embed": normal(seed, T.EMBED, (shape.vocab, shape.hidden), 0.02, 0.0, dt, device),
        "final_norm": normal(seed, T.FINAL_NORM, (shape.hidden,), 0.02, 1.0, dt, device),
        "lm_head": normal(seed, T.LM_HEAD, (shape.vocab, shape.hidden), 0.02, 0.0, dt, device),
    }


def draft_weights(shape, seed=SEED, device="cpu"):
    """Draft model: fusion FC [k,3k]; one decoder layer whose q/k/v take 2k inputs; two input
    norms, a final norm, the draft LM head [Vd,k] and the draft->target id map."""
    dt, T, k = _tdtype(shape), TensorIds, shape.hidden
    d = {
        "w_fc": normal(seed, T.D_FC, (k, 3 * k), 0.02, 0.0, dt, device),
        "layer": _layer(shape, T.DRAFT0, 2 * k, seed, device),
        "norm_embed": normal(seed, T.D_NORM_EMBED, (k,), 0.02, 1.0, dt, device),
        "norm_feat": normal(seed, T.D_NORM_FEAT, (k,), 0.02, 1.0, dt, device),
        "final_norm": normal(seed, T.D_FINAL_NORM, (k,), 0.02, 1.0, dt, device),
        "lm_head": normal(seed, T.D_LM_HEAD, (shape.draft_vocab, k), 0.02, 0.0, dt, device),
        "d2t": make_d2t(seed, shape.vocab, shape.draft_vocab, device),
    }
    del d["layer"]["norm_attn"]      # the draft layer's attention input norms are norm_embed / norm_feat
    return d


def kv_layer(shape, layer, n_tokens, seed=SEED, device="cpu", draft=False, first_slot=0):
    """(K, V) of cache slots [first_slot, first_slot + n_tokens), [n_tokens, Hkv, d], N(0,1) in the storage
    dtype.  K is taken as already rotated (as a cache stores it)."""
    base = TensorIds.DRAFT_KV if draft else TensorIds.KV0 + 2 * layer
    dims = (n_tokens, shape.n_kv_heads, shape.head_dim)
    dt = _tdtype(shape)
    start = first_slot * shape.n_kv_heads * shape.head_dim
    return (normal(seed, base, dims, 1.0, 0.0, dt, device, start=start),
            normal(seed, base + 1, dims, 1.0, 0.0, dt, device, start=start))


def ragged_batch(shape, seed=SEED):
    """Seeded batch layout of the ragged-cache configuration: prefix_len[b] uniform in
    [prefix_lo, prefix_hi], kv_indptr with room for the tree nodes after every prefix, one random tree
    (at most `topk` children per node, depth <= `depth`) and uniform token ids per sequence."""
    B, N = shape.batch, shape.n_nodes
    plen = uniform_ints(seed, TensorIds.PREFIX_LEN, (B,), shape.prefix_lo, shape.prefix_hi + 1).numpy().astype(np.int64)
    indptr = np.zeros(B + 1, dtype=np.int64)
    indptr[1:] = np.cumsum(plen + N)
    parents = np.stack([random_tree(seed, 1000 + b, N, shape.depth, shape.topk)[0] for b in range(B)])
    toks = uniform_ints(seed, TensorIds.TREE_TOK, (B, N), 0, shape.vocab).numpy()
    return {"prefix_len": plen.astype(np.int32), "kv_indptr": indptr.astype(np.int32), "parent": parents.astype(np.int32),
            "tree_tok": toks.astype(np.int32)}


def random_tree(seed, salt, n_nodes, max_depth, max_children):
    """Seeded random rooted tree as (parent[int32, N], depth[int32, N]); parent[0] = -1, parent[i] < i,
    every node at depth <= max_depth, at most `max_children` children per node, and siblings /
    levels are laid out in non-decreasing depth order (as a level-by-level drafter emits them)."""
    rs = np.random.RandomState((seed * 1000003 + salt) % (2 ** 31 - 1))
    while True:
        par, dep, nch = [-1], [0], [0]
        ok = True
        for i in range(1, n_nodes):
            cand = [j for j in range(i) if nch[j] < max_children and dep[j] < max_depth]
            if not cand:
                ok = False
                break
            p = cand[rs.randint(len(cand))]
            par.append(p); dep.append(dep[p] + 1); nch.append(0); nch[p] += 1
        if ok:
            break
    order = sorted(range(n_nodes), key=lambda i: (dep[i], i))
    new_id = {old: new for new, old in enumerate(order)}
    parent = np.array([-1 if par[o] < 0 else new_id[par[o]] for o in order], dtype=np.int32)
    depth = np.array([dep[o] for o in order], dtype=np.int32)
    return parent, depth


def reorder_tree(parent, order="dfs", seed=SEED):
    """The same rooted tree with its nodes renumbered: "dfs" = depth-first pre-order (a child directly follows
    its parent's earlier subtrees, depths go up and down along the node ids), "mixed" = a seeded random order
    that only keeps every parent before its children.  Returns (parent[int32, N], old id of every new node)."""
    parent = np.asarray(parent)
    n = len(parent)
    kids = [[] for _ in range(n)]
    for i in range(1, n):
        kids[int(parent[i])].append(i)
    if order == "dfs":
        seq, stack = [], [0]
        while stack:
            u = stack.pop()
            seq.append(u)
            stack.extend(reversed(kids[u]))
    else:
        rs = np.random.RandomState(seed % (2 ** 31 - 1))
        seq, ready = [], [0]
        while ready:
            u = ready.pop(rs.randint(len(ready)))
            seq.append(u)
            ready.extend(kids[u])
    new_id = {old: new for new, old in enumerate(seq)}
    new_parent = np.array([-1 if parent[o] < 0 else new_id[int(parent[o])] for o in seq], dtype=np.int32)
    return new_parent, np.array(seq, dtype=np.int32)


def chain_tree(n_nodes):
    parent = np.arange(-1, n_nodes - 1, dtype=np.int32)
    return parent, np.arange(n_nodes, dtype=np.int32)
