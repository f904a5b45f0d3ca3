"""GPU parity at shapes and orderings the other files do not reach: feature fusion and drafting at the 8B / 70B
shapes, node orders other than level order, one teacher-forced layer of the batched configuration at 384 and 512
rows (every row and column), and a whole step chained on the library's own outputs."""
import numpy as np
import pytest
import torch

import eagle3_synth as S
from oracle import eagle3_oracle as O
import parity
import pipeline as PL

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 2e-2


def _E():
    import paper_2503_01840_amd as E
    return E


def _rms(a):
    return float(np.sqrt(np.mean(np.square(a))))


@pytest.mark.parametrize("name", ["c3", "c5"])
def test_feature_fusion_at_full_shape(name):
    """g = W_fc [low; mid; high] with the 8B (12288 -> 4096) and 70B (24576 -> 8192) matrices, 1 and 7 rows."""
    E = _E()
    full = S.get_shape(name)
    shape = full.with_(n_layers=1, taps=(0, 0, 0))
    ctx = E.Eagle3Context(shape, max_depth=full.depth, max_topk=full.topk, max_new=8, device=DEV)
    ctx.set_weights(None, S.draft_weights(full, device=DEV))
    w_fc = O.as_f64(S.normal(S.SEED, S.TensorIds.D_FC, (full.hidden, 3 * full.hidden), 0.02, 0.0, torch.bfloat16))
    for M in (1, 7):
        taps = S.normal(S.SEED + M, S.TensorIds.TAPS, (3, M, full.hidden))
        ref = O.fuse_features(w_fc, *[O.as_f64(taps[i]) for i in range(3)], rounding="bf16")
        got = E.eagle3_fuse_features(ctx, *[taps[i].contiguous().to(DEV) for i in range(3)]).cpu().numpy()
        err = float(np.max(np.abs(got - ref)))
        print(f"{name} fuse M={M}: max err {err:.5f}, rms err {_rms(got - ref):.5f}, g rms {_rms(ref):.3f}")
        assert err < TOL


def test_c5_draft_online_oracle():
    """Draft expansion at the 70B shape (FC-free path: 16384-wide draft input, 8192 hidden, 32000 draft ids)."""
    E = _E()
    shape = S.get_shape("c5")
    D, K, N = shape.depth, shape.topk, shape.n_nodes
    model = PL.OracleModel(shape, cache_layers=False, lazy_embed=True)
    inp = PL.synthetic_step_inputs(shape)
    sub = shape.with_(n_layers=1, taps=(0, 0, 0))
    ctx = E.Eagle3Context(sub, max_depth=D, max_topk=K, max_new=8, device=DEV)
    T = S.TensorIds
    tg = {"embed": S.normal(S.SEED, T.EMBED, (shape.vocab, shape.hidden), 0.02, 0.0, torch.bfloat16, DEV),
          "final_norm": S.normal(S.SEED, T.FINAL_NORM, (shape.hidden,), 0.02, 1.0, torch.bfloat16, DEV)}
    tg["lm_head"] = tg["embed"]                     # never read by the draft call
    ctx.set_weights({"layers": [S.layer_weights(sub, 0, device=DEV)], **tg},
                    S.draft_weights(shape, device=DEV))
    ks, vs, indptr, plen, P = PL.device_kv([inp["draft_kv"]], 1 + (D - 1) * K, DEV)
    got = E.eagle3_draft_expand(ctx, inp["g_new"].to(DEV), inp["tok_new"].to(DEV), E.KVCache(ks, vs, indptr, plen, P),
                                D, K, N, debug=True)
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in got.items()}
    print("c5 draft: GPU side done, running the oracle", flush=True)
    tie_tol, level_tol = parity.draft_tolerances(parity.golden("c5"), D)     # from the oracle's stored score drift
    ref = PL.oracle_draft(shape, model, inp, D, K, N, tol=tie_tol,
                          follow={"pool_tok": got["pool_tok"], "frontier": got["frontier"], "chosen": got["chosen"]})
    for key in ("tree_tok", "parent", "depth", "chosen"):
        assert np.array_equal(got[key], ref[key]), key
    parity.check_scores("c5", got, ref, level_tol)


@pytest.mark.parametrize("order", ["dfs", "mixed"])
def test_verify_trees_in_other_node_orders(order):
    """The ABI promises only parent[i] < i.  A 60-node tree renumbered depth-first and in a random parent-first
    order: the renumbered tree against the oracle, and node for node equal to the level-ordered run."""
    E = _E()
    shape = S.get_shape("c2").with_(name="mid", hidden=512, n_heads=8, n_kv_heads=2, intermediate=1024, vocab=4096,
                                    draft_vocab=2048, n_layers=2, taps=(0, 1, 1), prefix_lo=203, prefix_hi=203)
    model = PL.OracleModel(shape)
    N, P = 60, shape.prefix_lo
    ctx = E.Eagle3Context(shape, max_nodes=64, max_depth=8, max_topk=10, max_new=8, device=DEV)
    W = PL.device_weights(shape, device=DEV)
    ctx.set_weights(W["target"], W["draft"])
    base_parent, _ = S.random_tree(S.SEED, 21, N, 8, 10)
    parent, old = S.reorder_tree(base_parent, order, seed=S.SEED + 5)
    depth = O.tree_depth(parent)
    assert np.any(np.diff(depth) < 0), "the order must not be level order"
    tok_level = S.uniform_ints(S.SEED, S.TensorIds.TREE_TOK, (N,), 0, shape.vocab).numpy()
    tok = tok_level[old]
    pairs = [S.kv_layer(shape, l, P) for l in range(shape.n_layers)]
    ref = O.tree_verify(shape, model.layer, model.globals(), tok, parent, lambda l: tuple(O.as_f64(t) for t in pairs[l]),
                        rounding="bf16")

    def run(tk, pr):
        ks, vs, indptr, plen, _ = PL.device_kv(pairs, N, DEV)
        lg, tp = E.eagle3_tree_verify(ctx, torch.as_tensor(tk, dtype=torch.int32, device=DEV)[None],
                                      torch.as_tensor(pr, dtype=torch.int32, device=DEV)[None], E.KVCache(ks, vs, indptr, plen, P))
        torch.cuda.synchronize()
        return lg[0].cpu().numpy(), tp[:, 0].cpu().numpy(), [k[P:].float().cpu().numpy() for k in ks]

    lg, tp, kn = run(tok, parent)
    assert np.max(np.abs(lg - ref["logits"])) < TOL
    assert np.max(np.abs(tp - ref["taps"])) < TOL
    for l in range(shape.n_layers):
        assert np.max(np.abs(kn[l] - ref["k_new"][l])) < TOL
    lg0, tp0, _ = run(tok_level, base_parent)              # the same tree in level order: node old[i] <-> node i
    assert np.max(np.abs(lg - lg0[old])) < TOL
    assert np.max(np.abs(tp - tp0[:, old])) < TOL


@pytest.mark.parametrize("n_seq,n_nodes", [(48, 8), (64, 8), (64, 4)])
def test_batched_layer_teacher_forced_every_row_and_column(n_seq, n_nodes):
    """One decoder layer + LM head at the 8B shape over n_seq x 8 = 384 / 512 node rows with ragged caches of
    512..2048 tokens (the batched-verification launch shapes: every projection takes the many-row GEMM), and over
    64 four-node chains = 256 rows (the verification launch of batched chain decoding); the same N(0, 8^2) residual
    rows on both sides, every output element compared."""
    E = _E()
    full = S.get_shape("c4")
    rb = S.ragged_batch(full)
    B, N = n_seq, n_nodes
    if N != full.n_nodes:                                  # chains instead of the stored trees
        rb = dict(rb, parent=np.tile(np.arange(-1, N - 1, dtype=np.int32), (full.batch, 1)),
                  tree_tok=np.ascontiguousarray(rb["tree_tok"][:, :N]))
    shape = full.with_(n_layers=1, taps=(0, 0, 0), batch=B)
    layer_id = 5
    W = S.layer_weights(full, layer_id)
    tg = S.target_globals(full)
    ctx = E.Eagle3Context(shape, max_batch=B, max_nodes=N, max_depth=full.depth, max_topk=full.topk, max_new=8, device=DEV)
    ctx.set_weights({"layers": [{k: v.to(DEV) for k, v in W.items()}], **{k: v.to(DEV) for k, v in tg.items()}}, None)
    plen = rb["prefix_len"][:B].astype(np.int64)
    indptr = np.zeros(B + 1, dtype=np.int64)
    indptr[1:] = np.cumsum(plen + N)
    total = int(indptr[-1])
    K_all, V_all = S.kv_layer(full, layer_id, total, device=DEV)
    kv = E.KVCache([K_all], [V_all], torch.as_tensor(indptr, dtype=torch.int32, device=DEV),
                   torch.as_tensor(plen, dtype=torch.int32, device=DEV), int(plen.max()))
    x_in = S.normal(S.SEED + 11, S.TensorIds.TAPS, (B, N, full.hidden), 8.0)
    tt = torch.as_tensor(rb["tree_tok"][:B], dtype=torch.int32, device=DEV)
    pp = torch.as_tensor(rb["parent"][:B], dtype=torch.int32, device=DEV)
    x_out, logits = E.eagle3_tree_verify_layers(ctx, tt, pp, kv, x_in.to(DEV), 0, 1, want_logits=True)
    torch.cuda.synchronize()
    x_out, logits = x_out.cpu().numpy(), logits.cpu().numpy()
    K_new = K_all.float().cpu().numpy()
    print(f"{B} x {N} rows: GPU side done, running the oracle per sequence", flush=True)
    W64, tg64 = O.weights_f64(W), O.weights_f64(tg)
    worst_x = worst_l = 0.0
    se_x = se_l = 0.0
    for b in range(B):
        P, base = int(plen[b]), int(indptr[b])
        pair = tuple(O.as_f64(t) for t in S.kv_layer(full, layer_id, P, first_slot=base))
        ref = O.tree_verify(shape, lambda _l: W64, tg64, rb["tree_tok"][b], rb["parent"][b], lambda _l: pair,
                            rounding="bf16", x0=O.as_f64(x_in[b]), keep_hidden=True)
        scale = max(1.0, _rms(ref["hidden"][1]))
        ex = np.abs(x_out[b] - ref["hidden"][1])
        el = np.abs(logits[b] - ref["logits"])
        worst_x, worst_l = max(worst_x, float(ex.max()) / scale), max(worst_l, float(el.max()))
        se_x += float(np.mean(ex * ex)); se_l += float(np.mean(el * el))
        assert ex.max() < TOL * scale, f"sequence {b}: residual stream err {ex.max():.4f} (rms {scale:.2f})"
        assert el.max() < TOL, f"sequence {b}: logits err {el.max():.4f}"
        assert np.max(np.abs(K_new[base + P:base + P + N] - ref["k_new"][0])) < 4e-2, b     # one bf16 ulp at |k| < 8
        if b % 16 == 0:
            print(f"  sequence {b} checked", flush=True)
    print(f"{B} x {N} rows: stream max err / rms {worst_x:.5f} (rms err {np.sqrt(se_x / B):.5f}), "
          f"logits max err {worst_l:.5f} (rms err {np.sqrt(se_l / B):.5f})")


def test_whole_step_chained_on_the_librarys_own_outputs():
    """fuse -> draft_expand -> tree_verify -> accept, every stage fed by the previous stage's GPU output (tiny fp32
    configuration), against the oracle's own chain: tree, accepted length, path and bonus token must be identical."""
    E = _E()
    shape = S.get_shape("c1")
    D, K, N = shape.depth, shape.topk, shape.n_nodes
    model = PL.OracleModel(shape)
    inp = PL.real_prefill_inputs(shape, model)
    ctx = E.Eagle3Context(shape, max_batch=1, max_nodes=N, max_depth=D, max_topk=K, max_new=4, device=DEV)
    W = PL.device_weights(shape, device=DEV)
    ctx.set_weights(W["target"], W["draft"])
    pre = inp["prefill"]
    # GPU chain
    taps_last = [torch.from_numpy(pre["taps"][t, -1:, :].copy()).float().to(DEV) for t in range(3)]
    g = E.eagle3_fuse_features(ctx, *taps_last)
    ks, vs, indptr, plen, P = PL.device_kv([inp["draft_kv"]], 1 + (D - 1) * K, DEV)
    tree = E.eagle3_draft_expand(ctx, g, inp["tok_new"].to(DEV), E.KVCache(ks, vs, indptr, plen, P), D, K, N, debug=True)
    tt, pp = tree["tree_tok"][None].contiguous(), tree["parent"][None].contiguous()
    ks, vs, indptr, plen, P = PL.device_kv(inp["target_kv"], N, DEV)
    logits, taps = E.eagle3_tree_verify(ctx, tt, pp, E.KVCache(ks, vs, indptr, plen, P))
    U = S.uniform01(S.SEED + 6, S.TensorIds.UNIFORMS, (1, 2 * N)).to(DEV)
    al0, path0, bonus0 = E.eagle3_accept(ctx, logits, tt, pp, 0.0)
    al1, path1, bonus1 = E.eagle3_accept(ctx, logits, tt, pp, 1.0, U)
    torch.cuda.synchronize()
    # oracle chain
    g_ref = O.fuse_features(model.draft()["w_fc"], *[pre["taps"][t, -1:, :] for t in range(3)])
    inp_ref = dict(inp, g_new=torch.from_numpy(g_ref))
    got = {k: v.cpu().numpy() for k, v in tree.items()}
    ref = PL.oracle_draft(shape, model, inp_ref, D, K, N, tol=1e-4,
                          follow={"pool_tok": got["pool_tok"], "frontier": got["frontier"], "chosen": got["chosen"]})
    assert ref["n_followed"] == 0 or ref["min_gap"] <= 1e-4
    for key in ("tree_tok", "parent", "depth"):
        assert np.array_equal(got[key], ref[key]), key
    vref = PL.oracle_verify(shape, model, inp, ref["tree_tok"], ref["parent"])
    assert np.max(np.abs(logits[0].cpu().numpy() - vref["logits"])) < 1e-4
    assert np.max(np.abs(taps[:, 0].cpu().numpy() - vref["taps"])) < 1e-4
    n_acc, rpath, rbonus = O.accept_greedy(vref["logits"], ref["tree_tok"], ref["parent"])
    srt = np.sort(vref["logits"][rpath], axis=1)
    assert (srt[:, -1] - srt[:, -2]).min() > 1e-3, "the seeded case must have clear arg-max margins on the walk"
    assert (int(al0[0]), int(bonus0[0])) == (n_acc, rbonus)
    assert path0[0].cpu().numpy().tolist() == rpath + [-1] * (N - len(rpath))
    n_acc, rpath, rbonus, margin = O.accept_stochastic(vref["logits"], ref["tree_tok"], ref["parent"], 1.0,
                                                        U[0].double().cpu().numpy())
    assert margin > 1e-4, "the seeded uniforms must not sit on a decision threshold"
    assert (int(al1[0]), int(bonus1[0])) == (n_acc, rbonus)
    assert path1[0].cpu().numpy().tolist() == rpath + [-1] * (N - len(rpath))


def test_chain_drafting_at_the_batch_64_serving_shape():
    """Batched chain drafting exactly as `bench.py --config chain` launches it: the 8B-shaped draft layer, 64 sequences
    with ragged draft caches of 549..2029 tokens, one new position each, chains of 3 tokens.  Ten of the sequences
    (shortest and longest context included) are run through the oracle one by one: the chain tokens must be the
    oracle's wherever its arg-max margins exceed the stored score drift, cumulative log-probabilities and the cached
    rows agree within the stored drift; the other sequences must be finite and identical run to run."""
    E = _E()
    shape = S.get_shape("c4")
    L = 3
    rb = S.ragged_batch(shape)
    B = shape.batch
    plen = rb["prefix_len"].astype(np.int64)
    indptr = np.zeros(B + 1, dtype=np.int64)
    indptr[1:] = np.cumsum(plen + 8)
    total = int(indptr[-1])
    sub = shape.with_(n_layers=1, taps=(0, 0, 0))
    ctx = E.Eagle3Context(sub, max_batch=B, max_nodes=8, max_depth=4, max_topk=2, max_new=8, device=DEV)
    T = S.TensorIds
    tg = {"embed": S.normal(S.SEED, T.EMBED, (shape.vocab, shape.hidden), 0.02, 0.0, torch.bfloat16, DEV),
          "final_norm": S.normal(S.SEED, T.FINAL_NORM, (shape.hidden,), 0.02, 1.0, torch.bfloat16, DEV)}
    tg["lm_head"] = tg["embed"]                     # never read by the draft call
    ctx.set_weights({"layers": [S.layer_weights(sub, 0, device=DEV)], **tg}, S.draft_weights(shape, device=DEV))
    K_all, V_all = S.kv_layer(shape, 0, total, draft=True)
    i32 = lambda a: torch.as_tensor(np.asarray(a), dtype=torch.int32, device=DEV)
    g = S.normal(S.SEED, T.G_NEW, (B, 1, shape.hidden))
    tok = S.uniform_ints(S.SEED, T.TOK_NEW, (B, 1), 0, shape.vocab)
    n_new = torch.ones(B, dtype=torch.int32, device=DEV)
    runs = []
    for _ in range(2):
        Kd, Vd = K_all.to(DEV), V_all.to(DEV)
        dkv = E.KVCache([Kd], [Vd], i32(indptr), i32(plen), int(plen.max()))
        chain_tok, chain_logp = E.eagle3_draft_chain(ctx, g.to(DEV), tok.to(DEV), n_new, dkv, L)
        torch.cuda.synchronize()
        runs.append((chain_tok.cpu().numpy(), chain_logp.cpu().numpy(), Kd, Vd))
    got_tok, got_logp, Kd, Vd = runs[0]
    assert np.array_equal(got_tok, runs[1][0]) and np.array_equal(got_logp, runs[1][1])
    assert torch.equal(Kd, runs[1][2]) and torch.equal(Vd, runs[1][3])
    assert np.all(np.isfinite(got_logp)) and np.all(got_logp[:, 1:] < 0) and np.all(np.diff(got_logp, axis=1) <= 0)
    assert np.array_equal(got_tok[:, 0], tok[:, 0].numpy())
    print("chain bs64: GPU side done, running the oracle", flush=True)
    model = PL.OracleModel(shape, cache_layers=False, lazy_embed=True)
    dw, emb = model.draft(), model.embed()
    _, level_tol = parity.draft_tolerances(parity.golden("c3"), S.get_shape("c3").depth)         # same draft shape
    tie_tol = float(np.max(level_tol[:L]) / parity.MAX_FACTOR)   # the stored score drift of the three levels in use
    sample = sorted({0, 9, 17, 26, 35, 44, 53, 63, int(np.argmin(plen)), int(np.argmax(plen))})
    checked_tokens = 0
    worst = np.zeros(L)
    for b in sample:
        lo, c = int(indptr[b]), int(plen[b])
        Kc = np.zeros((c + L + 1, shape.n_kv_heads, shape.head_dim)); Vc = np.zeros_like(Kc)
        Kc[:c], Vc[:c] = O.as_f64(K_all[lo:lo + c]), O.as_f64(V_all[lo:lo + c])
        ref = O.draft_expand(shape, dw, emb, O.as_f64(g[b]), tok[b].numpy().astype(np.int64), Kc, Vc, c, L, 1, L + 1,
                             rounding=model.rounding)
        assert np.array_equal(ref["parent"], np.arange(-1, L))
        if ref["min_gap"] > tie_tol:                 # every arg-max of this chain is clear of the score drift
            assert np.array_equal(got_tok[b], ref["tree_tok"]), b
            checked_tokens += 1
            err = np.abs(got_logp[b, 1:] - ref["score"][1:])
            worst = np.maximum(worst, err)
            assert np.all(err <= level_tol[:L]), (b, err)
            rows = slice(lo + c, lo + c + L)             # the root's row and the two drafted rows that were fed back
            for cur, want in ((Kd, Kc), (Vd, Vc)):       # bf16 values on both sides: equal, or one unit in the last
                d = cur[rows].float().cpu().numpy() - want[c:c + L]   # place apart (2^-4 at |x| in [8, 16)) where the input drifted
                assert np.max(np.abs(d)) <= 0.125 and parity.rms(d) < parity.TOL, (b, np.max(np.abs(d)), parity.rms(d))
        print(f"chain bs64: sequence {b} (context {c}) min arg-max gap {ref['min_gap']:.3f}", flush=True)
    parity.report(f"chain bs64 draft: {checked_tokens} of {len(sample)} sampled chains clear of near-ties and identical; "
                  f"log-prob error per level {np.round(worst, 5).tolist()}, allowed {np.round(level_tol[:L], 5).tolist()}")
    assert checked_tokens >= len(sample) * 3 // 4


@pytest.mark.parametrize("name", ["c3", "c4"])
def test_commit_at_full_shape(name):
    """eagle3_commit over all 32 layers of the 8B-shaped caches: one sequence with a 60-node tree behind 4096 cached
    tokens, and the ragged batch of 64 eight-node trees; random root paths; every moved row is an exact copy."""
    E = _E()
    shape = S.get_shape(name)
    rs = np.random.RandomState(21)
    if name == "c3":
        B, N = 1, shape.n_nodes
        plen = np.array([shape.prefix_lo], dtype=np.int64)
        parents = [S.random_tree(S.SEED, 31, N, shape.depth, shape.topk)[0]]
    else:
        rb = S.ragged_batch(shape)
        B, N = shape.batch, shape.n_nodes
        plen = rb["prefix_len"].astype(np.int64)
        parents = [rb["parent"][b] for b in range(B)]
    ctx = E.Eagle3Context(shape, max_batch=B, max_nodes=N, max_depth=shape.depth, max_topk=shape.topk, max_new=8, device=DEV)
    indptr = np.zeros(B + 1, dtype=np.int64)
    indptr[1:] = np.cumsum(plen + N)
    total = int(indptr[-1])
    paths = []
    for b in range(B):
        all_paths = O.ancestor_paths(parents[b])
        deepest = max(all_paths, key=len)
        paths.append([int(x) for x in (deepest if b % 4 == 0 else all_paths[int(rs.randint(N))])])
    path = np.full((B, N), -1, dtype=np.int32)
    for b, p in enumerate(paths):
        path[b, :len(p)] = p
    i32 = lambda a: torch.as_tensor(np.asarray(a), dtype=torch.int32, device=DEV)
    ks, vs = zip(*[S.kv_layer(shape, l, total, device=DEV) for l in range(shape.n_layers)])
    tails = [(torch.cat([k[int(indptr[b] + plen[b]):int(indptr[b + 1])] for b in range(B)]).clone(),
              torch.cat([v[int(indptr[b] + plen[b]):int(indptr[b + 1])] for b in range(B)]).clone()) for k, v in zip(ks, vs)]
    heads = [k[:int(plen[0])].clone() for k in ks[:2]]
    plen_d = i32(plen)
    kv = E.KVCache(ks, vs, i32(indptr), plen_d, int(plen.max()))
    tok = S.uniform_ints(S.SEED, S.TensorIds.TREE_TOK, (B, N), 0, shape.vocab).to(DEV)
    bonus = i32(rs.randint(0, shape.vocab, size=B))
    taps = S.normal(S.SEED, S.TensorIds.TAPS, (3, B, N, shape.hidden), device=DEV)
    rows = max(len(p) for p in paths)
    taps_new, tok_new, n_new = E.eagle3_commit(ctx, tok, i32(path), i32([len(p) - 1 for p in paths]), bonus, kv, taps, rows)
    torch.cuda.synchronize()
    assert n_new.cpu().tolist() == [len(p) for p in paths]
    assert plen_d.cpu().tolist() == (plen + np.array([len(p) for p in paths])).tolist()
    for b, p in enumerate(paths):
        first = int(indptr[b] + plen[b])
        idx = torch.as_tensor(p, device=DEV) + b * N
        assert tok_new[b, :len(p)].cpu().tolist() == [int(tok[b, q]) for q in p[1:]] + [int(bonus[b])], b
        assert torch.equal(taps_new[:, b, :len(p)], taps[:, b, p]), b
        for l in range(shape.n_layers):
            assert torch.equal(ks[l][first:first + len(p)], tails[l][0][idx]), (b, l)
            assert torch.equal(vs[l][first:first + len(p)], tails[l][1][idx]), (b, l)
    for l in range(2):                                     # cached context untouched
        assert torch.equal(ks[l][:int(plen[0])], heads[l])
