"""ctypes binding of libeagle3.so: argument marshalling only.

Every step of the speculative path runs in the HIP kernels behind the C ABI declared in
include/eagle3.h; this module turns torch tensors into pointers and sizes, allocates output
tensors and the workspace through torch, and passes torch's current stream.  There is no CPU or
torch fallback: a missing library raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libeagle3.so")
EAGLE3_FP32, EAGLE3_BF16 = 0, 1

EXPORTS = ["eagle3_create", "eagle3_destroy", "eagle3_workspace_bytes", "eagle3_set_workspace", "eagle3_set_weights",
           "eagle3_strerror", "eagle3_last_error", "eagle3_profile_begin", "eagle3_profile_read", "eagle3_profile_end",
           "eagle3_fuse_features", "eagle3_draft_expand",
           "eagle3_tree_verify", "eagle3_tree_verify_layers", "eagle3_accept", "eagle3_accept_static", "eagle3_commit", "eagle3_prefill", "eagle3_draft_chain", "eagle3_ttt_attention"]


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("hidden", "n_heads", "n_kv_heads", "head_dim", "intermediate", "vocab",
                                         "draft_vocab", "n_layers")] + \
               [("tap_layers", C.c_int32 * 3), ("dtype", C.c_int32), ("rope_theta", C.c_float), ("rms_eps", C.c_float)] + \
               [(n, C.c_int32) for n in ("max_batch", "max_nodes", "max_depth", "max_topk", "max_new")]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_mlp")]


class TargetWeights(C.Structure):
    _fields_ = [("layers", C.POINTER(LayerWeights)), ("embed", C.c_void_p), ("final_norm", C.c_void_p),
                ("lm_head", C.c_void_p)]


class DraftWeights(C.Structure):
    _fields_ = [("w_fc", C.c_void_p), ("layer", LayerWeights), ("norm_embed", C.c_void_p), ("norm_feat", C.c_void_p),
                ("final_norm", C.c_void_p), ("lm_head", C.c_void_p), ("d2t", C.c_void_p)]


class KV(C.Structure):
    _fields_ = [("k", C.POINTER(C.c_void_p)), ("v", C.POINTER(C.c_void_p)), ("kv_indptr", C.c_void_p),
                ("prefix_len", C.c_void_p), ("max_prefix_len", C.c_int32)]


class DraftDebug(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("pool_tok", "pool_parent", "pool_score", "frontier", "chosen")]


_lib = None


def lib():
    """Loads libeagle3.so (built in-tree by paper_2503_01840_amd.build); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2503_01840_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        L.eagle3_strerror.restype = C.c_char_p
        L.eagle3_last_error.restype = C.c_char_p
        L.eagle3_strerror.argtypes = [C.c_int]
        L.eagle3_create.argtypes = [C.POINTER(Config), C.POINTER(C.c_void_p)]
        L.eagle3_destroy.argtypes = [C.c_void_p]
        L.eagle3_workspace_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_size_t)]
        L.eagle3_set_workspace.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
        L.eagle3_set_weights.argtypes = [C.c_void_p, C.POINTER(TargetWeights), C.POINTER(DraftWeights)]
        L.eagle3_profile_begin.argtypes = [C.c_void_p]
        L.eagle3_profile_end.argtypes = [C.c_void_p]
        L.eagle3_profile_read.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64),
                                          C.POINTER(C.c_double)]
        L.eagle3_fuse_features.argtypes = [C.c_void_p] + [C.c_void_p] * 3 + [C.c_int32, C.c_void_p, C.c_void_p]
        L.eagle3_draft_expand.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(KV), C.c_int32,
                                          C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.POINTER(DraftDebug), C.c_void_p]
        L.eagle3_tree_verify.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.POINTER(KV),
                                         C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.eagle3_tree_verify_layers.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.POINTER(KV),
                                                C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.eagle3_accept.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_float,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.eagle3_accept_static.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_float,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.eagle3_commit.argtypes = [C.c_void_p, C.c_int32, C.c_int32] + [C.c_void_p] * 4 + [C.POINTER(KV), C.c_void_p,
                                    C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                    C.c_void_p]
        L.eagle3_prefill.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(KV), C.POINTER(KV), C.c_void_p, C.c_void_p,
                                     C.c_void_p]
        L.eagle3_draft_chain.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(KV),
                                         C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.eagle3_ttt_attention.argtypes = [C.c_int32] * 6 + [C.c_void_p] * 5
        _lib = L
    return _lib


class Eagle3Error(RuntimeError):
    def __init__(self, code):
        L = lib()
        msg = L.eagle3_strerror(code).decode()
        if code == -4:
            msg += ": " + L.eagle3_last_error().decode()
        super().__init__(f"eagle3 error {code}: {msg}")
        self.code = code


def _check(code):
    if code != 0:
        raise Eagle3Error(code)


def _ptr(t, dtype=None):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device, contiguous tensors only"
    if dtype is not None:
        assert t.dtype == dtype, (t.dtype, dtype)
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _layer_struct(W, keep):
    s = LayerWeights()
    for n, _ in LayerWeights._fields_:
        t = W.get(n)
        if t is not None:
            keep.append(t)
            setattr(s, n, _ptr(t))
    return s


class KVCache:
    """Per-layer cache tensors [slots, Hkv, d] plus device kv_indptr [B+1] / prefix_len [B] (int32)."""

    def __init__(self, k_layers, v_layers, kv_indptr, prefix_len, max_prefix_len):
        self.k_layers, self.v_layers = list(k_layers), list(v_layers)
        self.kv_indptr, self.prefix_len, self.max_prefix_len = kv_indptr, prefix_len, int(max_prefix_len)
        self._build()

    def set_max_prefix_len(self, n):
        """The host-side bound on prefix_len (sizes launches); to be kept ahead of the device values."""
        self.max_prefix_len = int(n)
        self.c.max_prefix_len = int(n)

    def _build(self):
        n = len(self.k_layers)
        self._k = (C.c_void_p * n)(*[_ptr(t) for t in self.k_layers])
        self._v = (C.c_void_p * n)(*[_ptr(t) for t in self.v_layers])
        self.c = KV(C.cast(self._k, C.POINTER(C.c_void_p)), C.cast(self._v, C.POINTER(C.c_void_p)),
                    _ptr(self.kv_indptr, torch.int32), _ptr(self.prefix_len, torch.int32), self.max_prefix_len)


class Eagle3Context:
    """Owns the library context and its torch-allocated workspace."""

    def __init__(self, shape=None, *, max_batch=1, max_nodes=64, max_depth=8, max_topk=10, max_new=8, device="cuda:0",
                 **dims):
        """`shape`: an object with the model fields of eagle3_config (e.g. eagle3_synth.Eagle3Shape) or None with
        the fields given as keyword arguments."""
        g = (lambda n: dims[n]) if shape is None else (lambda n: dims.get(n, getattr(shape, n, None)))
        cfg = Config()
        for n in ("hidden", "n_heads", "n_kv_heads", "head_dim", "intermediate", "vocab", "draft_vocab", "n_layers"):
            setattr(cfg, n, int(g(n)))
        taps = dims.get("tap_layers", getattr(shape, "taps", None))
        cfg.tap_layers = (C.c_int32 * 3)(*[int(t) for t in taps])
        dt = g("dtype")
        cfg.dtype = EAGLE3_BF16 if dt in ("bf16", EAGLE3_BF16, torch.bfloat16) else EAGLE3_FP32
        cfg.rope_theta, cfg.rms_eps = float(g("rope_theta")), float(g("rms_eps"))
        cfg.max_batch, cfg.max_nodes, cfg.max_depth, cfg.max_topk, cfg.max_new = (int(max_batch), int(max_nodes),
                                                                                  int(max_depth), int(max_topk), int(max_new))
        self.cfg, self.device = cfg, torch.device(device)
        self.storage_dtype = torch.bfloat16 if cfg.dtype == EAGLE3_BF16 else torch.float32
        self._h = C.c_void_p()
        _check(lib().eagle3_create(C.byref(cfg), C.byref(self._h)))
        need = C.c_size_t()
        _check(lib().eagle3_workspace_bytes(self._h, C.byref(need)))
        self.workspace_bytes = need.value
        self._ws = torch.empty(need.value + 256, dtype=torch.uint8, device=self.device)
        off = (-self._ws.data_ptr()) % 256
        _check(lib().eagle3_set_workspace(self._h, self._ws.data_ptr() + off, need.value))
        self._keep = []

    def close(self):
        if self._h:
            lib().eagle3_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def profile_begin(self):
        _check(lib().eagle3_profile_begin(self._h))

    def profile_read(self, kind):
        """(total ms, launches, weight bytes) of the GEMM launches of one kind since profile_begin: 0 = at most 32
        rows, 1 = 33..64 rows with 64-weight-row workgroups, 2 = 33..64 rows with 128-weight-row workgroups,
        3 = more than 64 rows (see include/eagle3_measure.h)."""
        ms, n, by = C.c_double(), C.c_int64(), C.c_double()
        _check(lib().eagle3_profile_read(self._h, int(kind), C.byref(ms), C.byref(n), C.byref(by)))
        return ms.value, n.value, by.value

    def profile_end(self):
        _check(lib().eagle3_profile_end(self._h))

    def set_weights(self, target=None, draft=None):
        """target: {"layers": [layer dicts], "embed", "final_norm", "lm_head"}; draft: {"w_fc", "layer": {...},
        "norm_embed", "norm_feat", "final_norm", "lm_head", "d2t"}; tensors on the device in the storage dtype."""
        keep = []
        tw = dw = None
        if target is not None:
            arr = (LayerWeights * len(target["layers"]))(*[_layer_struct(W, keep) for W in target["layers"]])
            assert len(target["layers"]) == self.cfg.n_layers
            tw = TargetWeights(C.cast(arr, C.POINTER(LayerWeights)), _ptr(target["embed"]), _ptr(target["final_norm"]),
                               _ptr(target["lm_head"]))
            keep += [arr, target["embed"], target["final_norm"], target["lm_head"]]
        if draft is not None:
            dw = DraftWeights(_ptr(draft["w_fc"]), _layer_struct(draft["layer"], keep), _ptr(draft["norm_embed"]),
                              _ptr(draft["norm_feat"]), _ptr(draft["final_norm"]), _ptr(draft["lm_head"]),
                              _ptr(draft["d2t"], torch.int32))
            keep += [draft[n] for n in ("w_fc", "norm_embed", "norm_feat", "final_norm", "lm_head", "d2t")]
        _check(lib().eagle3_set_weights(self._h, C.byref(tw) if tw else None, C.byref(dw) if dw else None))
        self._keep += keep


def eagle3_fuse_features(ctx, low, mid, high):
    M, k = low.shape
    g = torch.empty(M, k, dtype=torch.float32, device=low.device)
    _check(lib().eagle3_fuse_features(ctx._h, _ptr(low, torch.float32), _ptr(mid, torch.float32),
                                      _ptr(high, torch.float32), M, _ptr(g), _stream()))
    return g


def eagle3_draft_expand(ctx, g_new, tok_new, draft_kv, depth, topk, n_nodes, debug=False):
    dev = g_new.device
    n_new = g_new.shape[0]
    out = {"tree_tok": torch.empty(n_nodes, dtype=torch.int32, device=dev),
           "parent": torch.empty(n_nodes, dtype=torch.int32, device=dev),
           "depth": torch.empty(n_nodes, dtype=torch.int32, device=dev),
           "score": torch.empty(n_nodes, dtype=torch.float32, device=dev)}
    dbg = None
    if debug:
        pool = 1 + topk + (depth - 1) * topk * topk
        out.update(pool_tok=torch.zeros(pool, dtype=torch.int32, device=dev),
                   pool_parent=torch.zeros(pool, dtype=torch.int32, device=dev),
                   pool_score=torch.zeros(pool, dtype=torch.float32, device=dev),
                   frontier=torch.zeros(max(depth - 1, 1), topk, dtype=torch.int32, device=dev),
                   chosen=torch.zeros(n_nodes - 1, dtype=torch.int32, device=dev))
        dbg = DraftDebug(*[_ptr(out[n]) for n in ("pool_tok", "pool_parent", "pool_score", "frontier", "chosen")])
    _check(lib().eagle3_draft_expand(ctx._h, _ptr(g_new, torch.float32), _ptr(tok_new, torch.int32), n_new,
                                     C.byref(draft_kv.c), depth, topk, n_nodes, _ptr(out["tree_tok"]),
                                     _ptr(out["parent"]), _ptr(out["depth"]), _ptr(out["score"]),
                                     C.byref(dbg) if dbg else None, _stream()))
    return out


def eagle3_tree_verify(ctx, tree_tok, parent, kv, want_hidden=False, logits=None, taps=None):
    B, N = tree_tok.shape
    dev = tree_tok.device
    k, V, L = ctx.cfg.hidden, ctx.cfg.vocab, ctx.cfg.n_layers
    if logits is None:
        logits = torch.empty(B, N, V, dtype=torch.float32, device=dev)
    if taps is None:
        taps = torch.empty(3, B, N, k, dtype=torch.float32, device=dev)
    hidden = torch.empty(L + 1, B, N, k, dtype=torch.float32, device=dev) if want_hidden else None
    _check(lib().eagle3_tree_verify(ctx._h, B, N, _ptr(tree_tok, torch.int32), _ptr(parent, torch.int32),
                                    C.byref(kv.c), _ptr(logits), _ptr(taps), _ptr(hidden), _stream()))
    return (logits, taps, hidden) if want_hidden else (logits, taps)


def eagle3_tree_verify_layers(ctx, tree_tok, parent, kv, x_in, layer_begin, layer_end, want_logits=False):
    """Layers [layer_begin, layer_end) from the residual stream x_in [B,N,k] (None = embeddings).
    Returns (x_out, logits or None)."""
    B, N = tree_tok.shape
    dev = tree_tok.device
    x_out = torch.empty(B, N, ctx.cfg.hidden, dtype=torch.float32, device=dev)
    logits = torch.empty(B, N, ctx.cfg.vocab, dtype=torch.float32, device=dev) if want_logits else None
    _check(lib().eagle3_tree_verify_layers(ctx._h, B, N, _ptr(tree_tok, torch.int32), _ptr(parent, torch.int32),
                                           C.byref(kv.c), _ptr(x_in, torch.float32) if x_in is not None else None,
                                           int(layer_begin), int(layer_end), _ptr(x_out), _ptr(logits), _stream()))
    return x_out, logits


def eagle3_accept(ctx, logits, tree_tok, parent, temperature=0.0, uniforms=None):
    B, N = tree_tok.shape
    dev = tree_tok.device
    accept_len = torch.empty(B, dtype=torch.int32, device=dev)
    path = torch.empty(B, N, dtype=torch.int32, device=dev)
    bonus = torch.empty(B, dtype=torch.int32, device=dev)
    _check(lib().eagle3_accept(ctx._h, B, N, _ptr(logits, torch.float32), _ptr(tree_tok, torch.int32),
                               _ptr(parent, torch.int32), float(temperature),
                               _ptr(uniforms, torch.float32) if uniforms is not None else None, _ptr(accept_len),
                               _ptr(path), _ptr(bonus), _stream()))
    return accept_len, path, bonus


def eagle3_accept_static(logits, tree_tok, parent, temperature=0.0, uniforms=None, out=None):
    """eagle3_accept without a context or workspace (fixed scratch inside the library).  `out` = preallocated
    (accept_len, path, bonus) to make the call allocation-free on the torch side as well."""
    B, N = tree_tok.shape
    dev = tree_tok.device
    if out is None:
        out = (torch.empty(B, dtype=torch.int32, device=dev), torch.empty(B, N, dtype=torch.int32, device=dev),
               torch.empty(B, dtype=torch.int32, device=dev))
    accept_len, path, bonus = out
    _check(lib().eagle3_accept_static(B, N, logits.shape[-1], _ptr(logits, torch.float32), _ptr(tree_tok, torch.int32),
                                      _ptr(parent, torch.int32), float(temperature),
                                      _ptr(uniforms, torch.float32) if uniforms is not None else None, _ptr(accept_len),
                                      _ptr(path), _ptr(bonus), _stream()))
    return accept_len, path, bonus


def eagle3_commit(ctx, tree_tok, path, accept_len, bonus, kv, taps, rows, draft_kv=None, draft_rows=0):
    """Commits the accepted paths: cache rows compacted in place, kv.prefix_len advanced (and draft_kv.prefix_len by
    draft_rows).  Returns (taps_new [3,B,rows,k], tok_new [B,rows], n_new [B])."""
    B, N = tree_tok.shape
    dev = tree_tok.device
    taps_new = torch.zeros(3, B, rows, ctx.cfg.hidden, dtype=torch.float32, device=dev)
    tok_new = torch.zeros(B, rows, dtype=torch.int32, device=dev)
    n_new = torch.zeros(B, dtype=torch.int32, device=dev)
    _check(lib().eagle3_commit(ctx._h, B, N, _ptr(tree_tok, torch.int32), _ptr(path, torch.int32),
                               _ptr(accept_len, torch.int32), _ptr(bonus, torch.int32), C.byref(kv.c),
                               _ptr(kv.prefix_len, torch.int32), _ptr(taps, torch.float32), int(rows), _ptr(taps_new),
                               _ptr(tok_new), _ptr(n_new),
                               _ptr(draft_kv.prefix_len, torch.int32) if draft_kv is not None else None, int(draft_rows),
                               _stream()))
    return taps_new, tok_new, n_new


def eagle3_prefill(ctx, tokens, kv, draft_kv):
    """Runs the prompt through the target (cache, features) and builds the draft cache; advances both prefix_len
    arrays on the device and the host bounds.  Returns (g_last [hidden], logits_last [vocab])."""
    T = tokens.shape[0]
    g_last = torch.empty(ctx.cfg.hidden, dtype=torch.float32, device=tokens.device)
    logits = torch.empty(ctx.cfg.vocab, dtype=torch.float32, device=tokens.device)
    _check(lib().eagle3_prefill(ctx._h, _ptr(tokens, torch.int32), T, C.byref(kv.c), C.byref(draft_kv.c), _ptr(g_last),
                                _ptr(logits), _stream()))
    kv.set_max_prefix_len(kv.max_prefix_len + T)
    draft_kv.set_max_prefix_len(draft_kv.max_prefix_len + T - 1)
    return g_last, logits


def eagle3_draft_chain(ctx, g_new, tok_new, n_new, draft_kv, length):
    """Batched chain drafting.  g_new [B, rows1, k], tok_new [B, rows1], n_new [B].  Returns (chain_tok [B, length+1],
    chain_logp [B, length+1])."""
    B, rows1 = tok_new.shape
    dev = tok_new.device
    chain_tok = torch.empty(B, length + 1, dtype=torch.int32, device=dev)
    chain_logp = torch.empty(B, length + 1, dtype=torch.float32, device=dev)
    _check(lib().eagle3_draft_chain(ctx._h, B, _ptr(g_new, torch.float32), _ptr(tok_new, torch.int32),
                                    _ptr(n_new, torch.int32), rows1, C.byref(draft_kv.c), int(length), _ptr(chain_tok),
                                    _ptr(chain_logp), _stream()))
    return chain_tok, chain_logp


def eagle3_ttt_attention(q, k_steps, v_steps):
    """Training-time-test attention forward.  q [T,H,d], k_steps / v_steps [s+1,T,Hkv,d] (bf16 or fp32) -> fp32 [T,H,d]."""
    T, H, d = q.shape
    s, Hkv = k_steps.shape[0] - 1, k_steps.shape[2]
    dt = EAGLE3_BF16 if q.dtype == torch.bfloat16 else EAGLE3_FP32
    out = torch.empty(T, H, d, dtype=torch.float32, device=q.device)
    _check(lib().eagle3_ttt_attention(dt, T, H, Hkv, d, s, _ptr(q), _ptr(k_steps, q.dtype), _ptr(v_steps, q.dtype), _ptr(out),
                                      _stream()))
    return out
