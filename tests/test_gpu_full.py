"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

Tolerances (bf16 configurations).  A SINGLE layer given the same input on both sides holds logits to 2e-2 max-abs
and the residual stream / taps to 2e-2 in units of the stream's RMS (teacher-forced tests below and in
test_gpu_shapes.py, full 8B / 70B shapes, every element).  Through a deep stack two correct implementations that
round to bf16 at the same places still drift apart: a last-bit difference before a rounding flips that rounding now
and then, and the synthetic random-weight stack amplifies every flip.  The ORACLE measures that drift on itself:
tests/golden stores, beside its bf16-mode result, statistics of two more oracle runs: "drift_in" (rows entering
layer 0 perturbed by 1e-7 relative) and "drift_all" (relative noise of 2^-20, the size of fp32 accumulation error,
on every value right before each bf16 rounding).  The end-to-end tests require, per checked layer, for the taps and
for the logits,
    RMS(GPU - oracle) <= 1.5 * RMS drift_all      and      max|GPU - oracle| <= 2 * max drift_all
(never tighter than the single-layer tolerance), identical arg-max wherever the oracle's top-1 margin exceeds the max
bound, and they print the measured figures (collected in profiles/parity_errors.txt).  The draft's cumulative scores
and near-tie margin are bounded the same way by the stored per-level score drift (maxima: factor 2).

c2 (one 8B-shaped layer + LM head, draft depth 6) runs the oracle online.  c3 / c4 / c5 compare with the stored
oracle outputs: residual stream after selected layers and the taps in full (every row and column), logits at 2048
seeded vocabulary entries per row plus the 64 largest and the log-sum-exp.
"""
import os

import numpy as np
import pytest
import torch

import eagle3_synth as S
from oracle import eagle3_oracle as O
import pipeline as PL

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
from parity import (MAX_FACTOR, RMS_FACTOR, TOL, bounded as _bounded, check_scores as _check_scores,
                    draft_tolerances as _draft_tolerances, golden as _golden, report as _report, rms as _rms)
def _E():
    import paper_2503_01840_amd as E
    return E


def _ctx(shape, target=True, draft=True, **kw):
    E = _E()
    args = dict(max_batch=1, max_nodes=64, max_depth=shape.depth, max_topk=shape.topk, max_new=8)
    args.update(kw)
    ctx = E.Eagle3Context(shape, device=DEV, **args)
    W = PL.device_weights(shape, device=DEV, target=target, draft=draft)
    ctx.set_weights(W.get("target"), W.get("draft"))
    return ctx


def _stream_close(got, ref, what=""):
    """2e-2 max-abs in units of the reference stream's RMS (never tighter than 2e-2 absolute)."""
    scale = max(1.0, float(np.sqrt(np.mean(ref * ref))))
    err = float(np.max(np.abs(got - ref)))
    assert err < TOL * scale, f"{what}: max err {err:.4f} > {TOL * scale:.4f}"


def _check_stored(tag, g, prefix, logits, taps, hidden):
    """End-to-end comparison through a deep stack against the stored oracle outputs (see the module docstring)."""
    hl = g["hidden_layers"]
    for i, l in enumerate(hl):
        ref = g[prefix + "hidden"][i].astype(np.float64)
        _bounded(f"{tag} residual stream after layer {int(l) - 1}", hidden[l], ref, g[prefix + "drift_all_hidden"][i],
                 max(1.0, _rms(ref)))
    for t in range(3):
        ref = g[prefix + "taps"][t].astype(np.float64)
        _bounded(f"{tag} tap {t}", taps[t], ref, g[prefix + "drift_all_taps"][t], max(1.0, _rms(ref)))
    vsel = g[prefix + "vsel"].astype(np.int64)
    drift = g[prefix + "drift_all_logits"]
    lbound = _bounded(f"{tag} logits ({vsel.shape[1]} sampled entries per row)", np.take_along_axis(logits, vsel, 1),
                      g[prefix + "logits_at"].astype(np.float64), drift)
    top_idx, top_val = g[prefix + "top_idx"].astype(np.int64), g[prefix + "top_val"].astype(np.float64)
    _bounded(f"{tag} logits ({top_idx.shape[1]} largest per row)", np.take_along_axis(logits, top_idx, 1), top_val, drift)
    clear = (top_val[:, 0] - top_val[:, 1]) > 2 * lbound
    assert np.array_equal(np.argmax(logits, 1)[clear], top_idx[clear, 0])
    lse = np.log(np.sum(np.exp(logits - logits.max(1, keepdims=True)), 1)) + logits.max(1)
    assert np.max(np.abs(lse - g[prefix + "logsumexp"])) <= lbound
    _report(f"{tag}: arg-max compared on {int(clear.sum())} of {len(clear)} rows (top-1 margin > {2 * lbound:.3f})")


def test_c2_draft_and_verify_online_oracle():
    E = _E()
    shape = S.get_shape("c2")
    D, K, N = shape.depth, shape.topk, shape.n_nodes
    model = PL.OracleModel(shape, cache_layers=True)
    inp = PL.synthetic_step_inputs(shape)
    ctx = _ctx(shape)
    ks, vs, indptr, plen, P = PL.device_kv([inp["draft_kv"]], 1 + (D - 1) * K, DEV)
    got = E.eagle3_draft_expand(ctx, inp["g_new"].to(DEV), inp["tok_new"].to(DEV), E.KVCache(ks, vs, indptr, plen, P),
                                D, K, N, debug=True)
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in got.items()}
    g = _golden("c2")
    tie_tol, level_tol = _draft_tolerances(g, D)
    ref = PL.oracle_draft(shape, model, inp, D, K, N, tol=tie_tol,
                          follow={"pool_tok": got["pool_tok"], "frontier": got["frontier"], "chosen": got["chosen"]})
    if ref["min_gap"] > tie_tol:
        assert ref["n_followed"] == 0
    for key in ("tree_tok", "parent", "depth", "chosen"):
        assert np.array_equal(got[key], ref[key]), key
    _check_scores("c2", got, ref, level_tol)
    # verification of the oracle's tree: one layer + LM head against a 2048-token cache
    vref = PL.oracle_verify(shape, model, inp, ref["tree_tok"], ref["parent"], keep_hidden=True)
    pairs = [PL.target_kv_cpu(shape, inp, 0)]
    ks, vs, indptr, plen, P = PL.device_kv(pairs, N, DEV)
    tt = torch.as_tensor(ref["tree_tok"], dtype=torch.int32, device=DEV)[None]
    pp = torch.as_tensor(ref["parent"], dtype=torch.int32, device=DEV)[None]
    logits, taps, hidden = E.eagle3_tree_verify(ctx, tt, pp, E.KVCache(ks, vs, indptr, plen, P), want_hidden=True)
    torch.cuda.synchronize()
    for l in range(shape.n_layers + 1):
        _stream_close(hidden[l, 0].cpu().numpy(), vref["hidden"][l], f"residual stream after layer {l - 1}")
    for t in range(3):
        _stream_close(taps[t, 0].cpu().numpy(), vref["taps"][t], f"tap {t}")
    lg = logits[0].cpu().numpy()
    # one layer + LM head: the plain 2e-2 is where the oracle's own self-drift already sits (stored: max 0.03 over the
    # 7.7 M logits for fp32-sized noise, 0.025 for a 1e-7 input perturbation), so the bound is the drift multiple
    _bounded("c2 logits (every entry)", lg, vref["logits"], g["drift_all_logits"])
    srt = np.sort(vref["logits"], 1)
    clear = (srt[:, -1] - srt[:, -2]) > 1e-2
    assert np.array_equal(np.argmax(lg, 1)[clear], np.argmax(vref["logits"], 1)[clear])


def test_c3_draft_online_oracle_follows_near_ties():
    E = _E()
    shape = S.get_shape("c3")
    D, K, N = shape.depth, shape.topk, shape.n_nodes
    model = PL.OracleModel(shape, cache_layers=False)
    inp = PL.synthetic_step_inputs(shape)
    ctx = E.Eagle3Context(shape.with_(n_layers=1, taps=(0, 0, 0)), max_depth=D, max_topk=K, max_new=8, device=DEV)
    tg = S.target_globals(shape, device=DEV)
    ctx.set_weights({"layers": [S.layer_weights(shape, 0, device=DEV)], **tg}, S.draft_weights(shape, device=DEV))
    ks, vs, indptr, plen, P = PL.device_kv([inp["draft_kv"]], 1 + (D - 1) * K, DEV)
    got = E.eagle3_draft_expand(ctx, inp["g_new"].to(DEV), inp["tok_new"].to(DEV), E.KVCache(ks, vs, indptr, plen, P),
                                D, K, N, debug=True)
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in got.items()}
    tie_tol, level_tol = _draft_tolerances(_golden("c3"), D)
    ref = PL.oracle_draft(shape, model, inp, D, K, N, tol=tie_tol,
                          follow={"pool_tok": got["pool_tok"], "frontier": got["frontier"], "chosen": got["chosen"]})
    for key in ("tree_tok", "parent", "depth", "chosen"):
        assert np.array_equal(got[key], ref[key]), key
    _check_scores("c3", got, ref, level_tol)


@pytest.mark.parametrize("name", ["c3", "c5"])
def test_full_depth_verify_against_stored_oracle_samples(name):
    E = _E()
    g = _golden(name)
    shape = S.get_shape(name)
    N, P = shape.n_nodes, shape.prefix_lo
    ctx = _ctx(shape, draft=False)
    ks, vs = zip(*[S.kv_layer(shape, l, P + N, device=DEV) for l in range(shape.n_layers)])
    kv = E.KVCache(ks, vs, torch.tensor([0, P + N], dtype=torch.int32, device=DEV),
                   torch.tensor([P], dtype=torch.int32, device=DEV), P)
    tt = torch.as_tensor(g["tree_tok"], dtype=torch.int32, device=DEV)[None]
    pp = torch.as_tensor(g["parent"], dtype=torch.int32, device=DEV)[None]
    logits, taps, hidden = E.eagle3_tree_verify(ctx, tt, pp, kv, want_hidden=True)
    torch.cuda.synchronize()
    _check_stored(name, g, "", logits[0].cpu().numpy(), taps[:, 0].cpu().numpy(), hidden[:, 0].cpu().numpy())


def test_c4_ragged_batch64_verify_against_stored_oracle_samples():
    E = _E()
    g = _golden("c4")
    shape = S.get_shape("c4")
    rb = S.ragged_batch(shape)
    B, N = shape.batch, shape.n_nodes
    ctx = _ctx(shape, draft=False, max_batch=B, max_nodes=N)
    total = int(rb["kv_indptr"][-1])
    ks, vs = zip(*[S.kv_layer(shape, l, total, device=DEV) for l in range(shape.n_layers)])
    kv = E.KVCache(ks, vs, torch.as_tensor(rb["kv_indptr"], device=DEV), torch.as_tensor(rb["prefix_len"], device=DEV),
                   int(rb["prefix_len"].max()))
    logits, taps, hidden = E.eagle3_tree_verify(ctx, torch.as_tensor(rb["tree_tok"], device=DEV),
                                                torch.as_tensor(rb["parent"], device=DEV), kv, want_hidden=True)
    torch.cuda.synchronize()
    for b in g["seqs"]:
        _check_stored(f"c4 sequence {b}", g, f"s{b}_", logits[b].cpu().numpy(), taps[:, b].cpu().numpy(), hidden[:, b].cpu().numpy())
    # per-sequence independence: every sequence of the batch gives finite logits, and a second run is bit-identical
    assert torch.isfinite(logits).all()
    logits2, _ = E.eagle3_tree_verify(ctx, torch.as_tensor(rb["tree_tok"], device=DEV), torch.as_tensor(rb["parent"], device=DEV), kv)
    assert torch.equal(logits, logits2)


@pytest.mark.parametrize("name,layers", [("c3", (0, 16, 31)), ("c5", (0, 40, 79))])
def test_single_layers_teacher_forced_at_full_shape(name, layers):
    """Every checked layer gets the SAME synthetic residual stream on both sides (N(0, 8^2) rows), so the
    comparison is not blurred by drift from earlier layers: the stated tolerances must hold as such."""
    E = _E()
    full = S.get_shape(name)
    N, P = full.n_nodes, full.prefix_lo
    shape = full.with_(n_layers=1, taps=(0, 0, 0))
    parent, _ = S.random_tree(S.SEED, 3, N, full.depth, full.topk)
    tok = S.uniform_ints(S.SEED, S.TensorIds.TREE_TOK, (N,), 0, full.vocab).numpy()
    tt = torch.as_tensor(tok, dtype=torch.int32, device=DEV)[None]
    pp = torch.as_tensor(parent, dtype=torch.int32, device=DEV)[None]
    tg = S.target_globals(full)
    tg64 = O.weights_f64(tg)
    tg_dev = {k: v.to(DEV) for k, v in tg.items()}
    ctx = E.Eagle3Context(shape, max_depth=full.depth, max_topk=full.topk, max_new=8, device=DEV)
    for l in layers:
        x_in = S.normal(S.SEED + l, S.TensorIds.TAPS, (N, full.hidden), 8.0)
        W = S.layer_weights(full, l)
        pair = S.kv_layer(full, l, P)
        W64 = O.weights_f64(W)
        ref = O.tree_verify(shape, lambda _l: W64, tg64, tok, parent, lambda _l: tuple(O.as_f64(t) for t in pair),
                            rounding="bf16", x0=O.as_f64(x_in), keep_hidden=True)
        ctx.set_weights({"layers": [{k: v.to(DEV) for k, v in W.items()}], **tg_dev}, None)
        ks, vs, indptr, plen, _ = PL.device_kv([pair], N, DEV)
        x_out, logits = E.eagle3_tree_verify_layers(ctx, tt, pp, E.KVCache(ks, vs, indptr, plen, P),
                                                    x_in.to(DEV)[None].contiguous(), 0, 1, want_logits=True)
        torch.cuda.synchronize()
        _stream_close(x_out[0].cpu().numpy(), ref["hidden"][1], f"{name} layer {l}")
        err = np.max(np.abs(logits[0].cpu().numpy() - ref["logits"]))
        assert err < TOL, f"{name} layer {l} + LM head: logits err {err:.4f}"
        assert np.max(np.abs(ks[0][P:].float().cpu().numpy() - ref["k_new"][0])) < 4e-2      # one bf16 ulp at |k| < 8
        del W64, ref
