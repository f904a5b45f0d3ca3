"""Test infrastructure shared by the GPU parity tests, the smoke check and the benchmark's CPU leg:
builds one workload's inputs from the seeded generators, runs the ORACLE over it (CPU), and mirrors the
same inputs onto the device for the library.  No expected value comes from the GPU side."""
import numpy as np
import torch

import eagle3_synth as S
from oracle import eagle3_oracle as O


class LazyEmbedRows:
    """Rows of the seeded embedding table, generated when indexed (the full 128256 x 8192 table is never built)."""

    def __init__(self, shape, seed=S.SEED):
        self.shape, self.seed = shape, seed

    def __getitem__(self, idx):
        k = self.shape.hidden
        dt = torch.float32 if self.shape.dtype == "fp32" else torch.bfloat16
        rows = [O.as_f64(S.normal(self.seed, S.TensorIds.EMBED, (k,), 0.02, 0.0, dt, start=int(t) * k))
                for t in np.asarray(idx).reshape(-1)]
        return np.stack(rows).reshape(tuple(np.shape(idx)) + (k,))


class OracleModel:
    """Float64 weights of a shape; target layers are generated on demand (and cached when small)."""

    def __init__(self, shape, seed=S.SEED, cache_layers=None, lazy_embed=False):
        self.shape, self.seed = shape, seed
        self.lazy_embed = lazy_embed
        self.rounding = "bf16" if shape.dtype == "bf16" else "none"
        self._cache = {} if (cache_layers if cache_layers is not None else shape.layer_params() * shape.n_layers < 3e8) else None
        self.tg = None
        self.dw = None

    def layer(self, l):
        if self._cache is not None and l in self._cache:
            return self._cache[l]
        W = O.weights_f64(S.layer_weights(self.shape, l, self.seed))
        if self._cache is not None:
            self._cache[l] = W
        return W

    def globals(self):
        if self.tg is None:
            self.tg = O.weights_f64(S.target_globals(self.shape, self.seed))
        return self.tg

    def embed(self):
        return LazyEmbedRows(self.shape, self.seed) if self.lazy_embed else self.globals()["embed"]

    def draft(self):
        if self.dw is None:
            self.dw = O.weights_f64(S.draft_weights(self.shape, self.seed))
        return self.dw


def synthetic_step_inputs(shape, seed=S.SEED, n_new=None, prefix=None):
    """bf16-style workloads: random caches, features and tokens (NumPy / torch CPU, storage dtype kept)."""
    n_new = shape.n_new if n_new is None else n_new
    P = shape.prefix_lo if prefix is None else prefix
    T = S.TensorIds
    inp = {
        "P": P, "n_new": n_new,
        "g_new": S.normal(seed, T.G_NEW, (n_new, shape.hidden)),
        "tok_new": S.uniform_ints(seed, T.TOK_NEW, (n_new,), 0, shape.vocab),
        "taps": S.normal(seed, T.TAPS, (3, max(n_new, 1), shape.hidden)),
        "draft_kv": S.kv_layer(shape, 0, P, seed, draft=True),
    }
    return inp


def real_prefill_inputs(shape, model, seed=S.SEED):
    """Tiny fp32 workload: a real oracle prefill of random token ids gives the target cache, the taps,
    the root token, and (by running the draft layer over the prefix) the draft cache."""
    P = shape.prefix_lo
    toks = S.uniform_ints(seed, S.TensorIds.PREFIX_TOK, (P,), 0, shape.vocab).numpy()
    pre = O.prefill(shape, model.layer, model.globals(), toks)
    dw, emb = model.draft(), model.globals()["embed"]
    g_all = O.fuse_features(dw["w_fc"], pre["taps"][0], pre["taps"][1], pre["taps"][2])
    Kd = np.zeros((P - 1, shape.n_kv_heads, shape.head_dim)); Vd = np.zeros_like(Kd)
    if P > 1:                                            # a one-token prompt has no position whose next token is known
        O.draft_forward(shape, dw, emb, g_all[:P - 1], toks[1:], np.arange(P - 1), Kd, Vd, 0, 0,
                        np.tril(np.ones((P - 1, P - 1), dtype=bool)), lambda a: a)
    root = int(np.argmax(pre["logits"][-1]))
    return {
        "P": P, "n_new": 1, "prefix_tok": toks, "prefill": pre,
        "taps": torch.from_numpy(pre["taps"][:, -4:, :].copy()).float(),
        "g_new": torch.from_numpy(g_all[P - 1:P].copy()).float(),
        "tok_new": torch.tensor([root], dtype=torch.int32),
        "draft_kv": (torch.from_numpy(Kd).float(), torch.from_numpy(Vd).float()),
        "target_kv": [(torch.from_numpy(pre["k_new"][l]).float(), torch.from_numpy(pre["v_new"][l]).float())
                      for l in range(shape.n_layers)],
    }


def oracle_draft(shape, model, inp, depth, topk, n_nodes, follow=None, tol=1e-2):
    Kd, Vd = inp["draft_kv"]
    n_ctx = Kd.shape[0]
    cap = n_ctx + inp["n_new"] + (depth - 1) * topk
    Kc = np.zeros((cap, shape.n_kv_heads, shape.head_dim)); Vc = np.zeros_like(Kc)
    Kc[:n_ctx], Vc[:n_ctx] = O.as_f64(Kd), O.as_f64(Vd)
    out = O.draft_expand(shape, model.draft(), model.embed(), O.as_f64(inp["g_new"]),
                         inp["tok_new"].numpy().astype(np.int64), Kc, Vc, n_ctx, depth, topk, n_nodes,
                         rounding=model.rounding, follow=follow, tol=tol)
    out["K_cache"], out["V_cache"] = Kc, Vc
    return out


def target_kv_cpu(shape, inp, layer, seed=S.SEED):
    if "target_kv" in inp:
        return inp["target_kv"][layer]
    return S.kv_layer(shape, layer, inp["P"], seed)


def oracle_verify(shape, model, inp, tree_tok, parent, keep_hidden=False, seed=S.SEED, with_logits=True):
    tg = model.globals() if with_logits else {"embed": model.globals()["embed"], "lm_head": None}
    return O.tree_verify(shape, model.layer, tg, np.asarray(tree_tok), np.asarray(parent),
                         lambda l: tuple(O.as_f64(t) for t in target_kv_cpu(shape, inp, l, seed)),
                         rounding=model.rounding, keep_hidden=keep_hidden)


# ------------------------------------------------------------------------------------------ device side

def device_weights(shape, seed=S.SEED, device="cuda:0", target=True, draft=True):
    out = {}
    if target:
        tg = S.target_globals(shape, seed, device)
        out["target"] = {"layers": [S.layer_weights(shape, l, seed, device) for l in range(shape.n_layers)], **tg}
    if draft:
        out["draft"] = S.draft_weights(shape, seed, device)
    return out


def device_kv(pairs, extra_slots, device="cuda:0"):
    """pairs: per layer (K, V) [P,Hkv,d] CPU tensors of ONE sequence -> KVCache args with room for `extra_slots`."""
    ks, vs = [], []
    for K, V in pairs:
        P = K.shape[0]
        kd = torch.zeros((P + extra_slots,) + tuple(K.shape[1:]), dtype=K.dtype, device=device)
        vd = torch.zeros_like(kd)
        kd[:P], vd[:P] = K.to(device), V.to(device)
        ks.append(kd); vs.append(vd)
    P = pairs[0][0].shape[0]
    indptr = torch.tensor([0, P + extra_slots], dtype=torch.int32, device=device)
    plen = torch.tensor([P], dtype=torch.int32, device=device)
    return ks, vs, indptr, plen, P
