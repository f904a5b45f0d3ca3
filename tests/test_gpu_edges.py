"""GPU parity on edge and degenerate cases, and acceptance at full vocabulary size."""
import numpy as np
import pytest
import torch

import eagle3_synth as S
from oracle import eagle3_oracle as O
import pipeline as PL

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

SMALL = S.get_shape("c2").with_(name="small", hidden=256, n_heads=4, n_kv_heads=2, intermediate=512, vocab=1024,
                                draft_vocab=512, n_layers=2, taps=(0, 1, 1), prefix_lo=70, prefix_hi=70, depth=3,
                                topk=3, n_nodes=10)


def _E():
    import paper_2503_01840_amd as E
    return E


def _ctx(shape, weights=True, **kw):
    E = _E()
    args = dict(max_batch=1, max_nodes=64, max_depth=8, max_topk=16, max_new=8)
    args.update(kw)
    ctx = E.Eagle3Context(shape, device=DEV, **args)
    if weights:
        W = PL.device_weights(shape, device=DEV)
        ctx.set_weights(W["target"], W["draft"])
    return ctx


def _verify_case(ctx, shape, model, parent, P, seed_salt=0, tol=2e-2):
    """One sequence: random cache of P slots, given tree; GPU vs oracle on logits, taps, written cache rows."""
    E = _E()
    N = len(parent)
    toks = S.uniform_ints(S.SEED + seed_salt, S.TensorIds.TREE_TOK, (N,), 0, shape.vocab).numpy()
    pairs = [S.kv_layer(shape, l, P, seed=S.SEED + seed_salt) for l in range(shape.n_layers)]
    ref = O.tree_verify(shape, model.layer, model.globals(), toks, parent,
                        lambda l: tuple(O.as_f64(t) for t in pairs[l]), rounding=model.rounding)
    ks, vs, indptr, plen, _ = PL.device_kv(pairs, N, DEV)
    kv = E.KVCache(ks, vs, indptr, plen, P)
    tt = torch.as_tensor(toks, dtype=torch.int32, device=DEV)[None]
    pp = torch.as_tensor(np.asarray(parent), dtype=torch.int32, device=DEV)[None]
    logits, taps = E.eagle3_tree_verify(ctx, tt, pp, kv)
    torch.cuda.synchronize()
    assert np.max(np.abs(logits[0].cpu().numpy() - ref["logits"])) < tol
    assert np.max(np.abs(taps[:, 0].cpu().numpy() - ref["taps"])) < tol
    for l in range(shape.n_layers):
        assert np.max(np.abs(ks[l][P:].float().cpu().numpy() - ref["k_new"][l])) < tol
    return ref


@pytest.mark.parametrize("shape", [S.get_shape("c1").with_(prefix_lo=40, prefix_hi=40), SMALL], ids=["fp32", "bf16"])
def test_verify_degenerate_trees_and_prefixes(shape):
    model = PL.OracleModel(shape)
    ctx = _ctx(shape)
    tol = 1e-4 if shape.dtype == "fp32" else 2e-2
    star = np.array([-1] + [0] * 15, dtype=np.int32)
    cases = [
        (np.array([-1], dtype=np.int32), 33),                 # root only
        (S.chain_tree(16)[0], 0),                             # empty prefix: the tree is the whole context
        (np.array([-1], dtype=np.int32), 0),                  # one token, nothing cached
        (star, 31),                                           # star: every node sees only the root and itself
        (np.array([-1] + [0] * 39, dtype=np.int32), 0),       # star of 40 without a prefix: for the first 32 rows the
                                                              # second 32-key block of the only tile is wholly invisible
        (S.chain_tree(64)[0], 65),                            # maximum node count as one deep chain
        (S.random_tree(S.SEED, 9, 64, 6, 10)[0], 97),         # maximum node count, bushy; prefix not a tile multiple
        (S.random_tree(S.SEED, 10, 33, 5, 4)[0], 1),          # one cached token; node count just past a 32-tile
    ]
    for i, (parent, P) in enumerate(cases):
        _verify_case(ctx, shape, model, parent, P, seed_salt=i, tol=tol)


def test_verify_ragged_batch_matches_per_sequence_oracle():
    E = _E()
    shape = SMALL
    model = PL.OracleModel(shape)
    B, N = 5, 9
    ctx = _ctx(shape, max_batch=B)
    plens = [0, 37, 64, 129, 5]
    parents = np.stack([S.random_tree(S.SEED, 50 + b, N, 4, 3)[0] for b in range(B)])
    toks = S.uniform_ints(S.SEED, S.TensorIds.TREE_TOK, (B, N), 0, shape.vocab).numpy()
    indptr = np.zeros(B + 1, dtype=np.int64)
    indptr[1:] = np.cumsum(np.array(plens) + N + 3)           # spare slots after every sequence
    total = int(indptr[-1])
    ks, vs = [], []
    for l in range(shape.n_layers):
        K, V = S.kv_layer(shape, l, total)
        ks.append(K.to(DEV)); vs.append(V.to(DEV))
    kv = E.KVCache(ks, vs, torch.as_tensor(indptr, dtype=torch.int32, device=DEV),
                   torch.tensor(plens, dtype=torch.int32, device=DEV), max(plens))
    logits, taps = E.eagle3_tree_verify(ctx, torch.as_tensor(toks, dtype=torch.int32, device=DEV),
                                        torch.as_tensor(parents, dtype=torch.int32, device=DEV), kv)
    torch.cuda.synchronize()
    for b in range(B):
        base, P = int(indptr[b]), plens[b]
        ref = O.tree_verify(shape, model.layer, model.globals(), toks[b], parents[b],
                            lambda l: tuple(O.as_f64(t) for t in S.kv_layer(shape, l, P, first_slot=base)),
                            rounding="bf16")
        assert np.max(np.abs(logits[b].cpu().numpy() - ref["logits"])) < 2e-2, b
        assert np.max(np.abs(taps[:, b].cpu().numpy() - ref["taps"])) < 2e-2, b


def test_verify_more_than_64_rows_uses_the_wide_gemm_path():
    """12 sequences x 8 nodes = 96 rows (the batched-verification GEMM tiling), 16 x 16 = 256 rows with a ragged tail;
    176 and 225 rows take the one-row-block tiling of 129..256 rows with a partly empty block; 768 and 1024 rows span
    three and four 256-row blocks."""
    E = _E()
    shape = SMALL
    model = PL.OracleModel(shape)
    for B, N in ((12, 8), (16, 16), (5, 13), (11, 16), (15, 15), (24, 32), (64, 16)):
        ctx = _ctx(shape, max_batch=B, max_nodes=N)
        plens = [(37 * b + 11) % 150 for b in range(B)]
        parents = np.stack([S.random_tree(S.SEED, 80 + b, N, 4, 3)[0] for b in range(B)])
        toks = S.uniform_ints(S.SEED + B, S.TensorIds.TREE_TOK, (B, N), 0, shape.vocab).numpy()
        indptr = np.zeros(B + 1, dtype=np.int64)
        indptr[1:] = np.cumsum(np.array(plens) + N)
        total = int(indptr[-1])
        ks, vs = zip(*[tuple(t.to(DEV) for t in S.kv_layer(shape, l, total)) for l in range(shape.n_layers)])
        kv = E.KVCache(ks, vs, torch.as_tensor(indptr, dtype=torch.int32, device=DEV),
                       torch.tensor(plens, dtype=torch.int32, device=DEV), max(plens))
        logits, taps = E.eagle3_tree_verify(ctx, torch.as_tensor(toks, dtype=torch.int32, device=DEV),
                                            torch.as_tensor(parents, dtype=torch.int32, device=DEV), kv)
        torch.cuda.synchronize()
        for b in (0, B // 2, B - 1):
            base, P = int(indptr[b]), plens[b]
            ref = O.tree_verify(shape, model.layer, model.globals(), toks[b], parents[b],
                                lambda l: tuple(O.as_f64(t) for t in S.kv_layer(shape, l, P, first_slot=base)),
                                rounding="bf16")
            assert np.max(np.abs(logits[b].cpu().numpy() - ref["logits"])) < 2e-2, (B, N, b)
            assert np.max(np.abs(taps[:, b].cpu().numpy() - ref["taps"])) < 2e-2, (B, N, b)


def test_verify_33_to_64_rows_on_large_ragged_matrices():
    """33, 48 and 64 tree nodes against an LM head of 24613 rows (192 tiles of 128 weight rows and a ragged one) and a
    12416-wide gate/up pair: the launches that take the 128-weight-row workgroups, with a K of only two stages."""
    shape = SMALL.with_(name="small-wide", n_layers=1, taps=(0, 0, 0), intermediate=12416, vocab=24613)
    model = PL.OracleModel(shape)
    ctx = _ctx(shape)
    for i, N in enumerate((33, 48, 64)):
        _verify_case(ctx, shape, model, S.random_tree(S.SEED, 40 + i, N, 6, 8)[0], 70 + i, seed_salt=20 + i)


@pytest.mark.parametrize("n_new,D,K,N", [(8, 3, 3, 10), (1, 4, 1, 5), (2, 1, 4, 5), (1, 2, 16, 40), (3, 8, 2, 30),
                                          (2, 8, 16, 64)])          # the largest pool: 1809 candidates, 114 draft rows
def test_draft_expand_shapes(n_new, D, K, N):
    E = _E()
    shape = SMALL
    model = PL.OracleModel(shape)
    ctx = _ctx(shape)
    inp = PL.synthetic_step_inputs(shape, n_new=n_new, prefix=shape.prefix_lo + n_new)
    ks, vs, indptr, plen, P = PL.device_kv([inp["draft_kv"]], n_new + (D - 1) * K, DEV)
    got = E.eagle3_draft_expand(ctx, inp["g_new"].to(DEV), inp["tok_new"].to(DEV), E.KVCache(ks, vs, indptr, plen, P),
                                D, K, N, debug=True)
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in got.items()}
    ref = PL.oracle_draft(shape, model, inp, D, K, N,
                          follow={"pool_tok": got["pool_tok"], "frontier": got["frontier"], "chosen": got["chosen"]})
    if ref["min_gap"] > 1e-2:
        assert ref["n_followed"] == 0
    for key in ("tree_tok", "parent", "depth", "chosen"):
        assert np.array_equal(got[key], ref[key]), key
    assert np.max(np.abs(got["score"] - ref["score"])) < 2e-2
    assert all(got["parent"][i] < i for i in range(1, N)) and got["parent"][0] == -1


def _planted_logits(rs, parent, tok, V, target_node, B=1):
    N = len(parent)
    logits = rs.randn(N, V).astype(np.float32)
    path = O.ancestor_paths(parent)[target_node]
    for u, c in zip(path[:-1], path[1:]):
        logits[u, tok[c]] += 25.0
    kids = {int(tok[c]) for c in range(N) if parent[c] == target_node}
    stop = next(t for t in range(V) if t not in kids)
    logits[target_node, stop] += 25.0
    return logits, path, stop


def test_accept_full_vocabulary_planted_paths_and_stochastic():
    E = _E()
    shape = S.get_shape("c2")
    ctx = _ctx(shape, weights=False, max_batch=64)
    V = shape.vocab
    rs = np.random.RandomState(3)
    parent, depth = S.random_tree(S.SEED, 77, 60, 8, 10)
    tok = S.uniform_ints(S.SEED, S.TensorIds.TREE_TOK, (60,), 0, V).numpy()
    tt = torch.as_tensor(tok, dtype=torch.int32, device=DEV)[None]
    pp = torch.as_tensor(parent, dtype=torch.int32, device=DEV)[None]
    # greedy: a planted path to every node of the tree (every depth 0..8 occurs)
    for target in range(0, 60, 3):
        logits, path, stop = _planted_logits(rs, parent, tok, V, target)
        al, gp, bonus = E.eagle3_accept(ctx, torch.from_numpy(logits).to(DEV)[None], tt, pp, 0.0)
        assert int(al[0]) == len(path) - 1 and int(bonus[0]) == stop
        assert gp[0].cpu().numpy().tolist() == path + [-1] * (60 - len(path))
    # all logits equal: the argmax tie goes to token 0, no child has it
    al, gp, bonus = E.eagle3_accept(ctx, torch.zeros(1, 60, V, device=DEV), tt, pp, 0.0)
    assert (int(al[0]), int(bonus[0])) == (0, 0)
    # stochastic: peaked distributions so that children carry real mass; compare with the oracle given the same uniforms
    agree = 0
    for trial in range(24):
        logits = (rs.randn(60, V) * 1.0).astype(np.float32)
        for u in range(60):
            for c in [c for c in range(60) if parent[c] == u][:3]:
                logits[u, tok[c]] += rs.uniform(6.0, 12.0)
        U = S.uniform01(S.SEED + trial, S.TensorIds.UNIFORMS, (1, 120))
        temp = [1.0, 0.7, 1.5][trial % 3]
        al, gp, bonus = E.eagle3_accept(ctx, torch.from_numpy(logits).to(DEV)[None], tt, pp, temp, U.to(DEV))
        n_acc, rpath, rbonus, margin, info = O.accept_stochastic(logits.astype(np.float64), tok, parent, temp,
                                                                 U[0].double().numpy(), return_info=True)
        if info["margin_children"] > 1e-5:              # every accept/reject decision is clear: the walk is unique
            agree += 1
            assert int(al[0]) == n_acc, trial
            assert gp[0].cpu().numpy().tolist() == rpath + [-1] * (60 - len(rpath))
            # the bonus draw: over 128k entries fp32 partial sums may legitimately land one token away
            assert O.bonus_admissible(info, int(bonus[0]), 2e-5), trial
            if margin > 2e-5:
                assert int(bonus[0]) == rbonus
    assert agree >= 12


def test_accept_batch_of_64_small_trees():
    E = _E()
    shape = S.get_shape("c4")
    ctx = _ctx(shape, weights=False, max_batch=64, max_nodes=8)
    rb = S.ragged_batch(shape)
    B, N, V = 64, 8, shape.vocab
    rs = np.random.RandomState(5)
    logits = np.zeros((B, N, V), dtype=np.float32)
    expect = []
    for b in range(B):
        lg, path, stop = _planted_logits(rs, rb["parent"][b], rb["tree_tok"][b], V, b % N)
        logits[b] = lg
        expect.append((len(path) - 1, path, stop))
    tt = torch.as_tensor(rb["tree_tok"], device=DEV)
    pp = torch.as_tensor(rb["parent"], device=DEV)
    lg_d = torch.from_numpy(logits).to(DEV)
    al, gp, bonus = E.eagle3_accept(ctx, lg_d, tt, pp, 0.0)
    for b in range(B):
        assert (int(al[b]), int(bonus[b])) == (expect[b][0], expect[b][2]), b
        assert gp[b].cpu().numpy().tolist() == expect[b][1] + [-1] * (N - len(expect[b][1]))
    U = S.uniform01(S.SEED, S.TensorIds.UNIFORMS, (B, 2 * N))
    al, gp, bonus = E.eagle3_accept(ctx, lg_d, tt, pp, 1.0, U.to(DEV))
    checked = 0
    for b in range(B):
        n_acc, rpath, rbonus, margin, info = O.accept_stochastic(logits[b].astype(np.float64), rb["tree_tok"][b],
                                                                 rb["parent"][b], 1.0, U[b].double().numpy(), return_info=True)
        if info["margin_children"] > 1e-5:
            checked += 1
            assert int(al[b]) == n_acc, b
            assert O.bonus_admissible(info, int(bonus[b]), 2e-5), b
            if margin > 2e-5:
                assert int(bonus[b]) == rbonus
    assert checked >= 48


def test_argument_checks_on_a_live_context():
    E = _E()
    shape = SMALL
    ctx = _ctx(shape, max_nodes=16, max_depth=3, max_topk=3, max_new=2)
    pairs = [S.kv_layer(shape, l, 10) for l in range(shape.n_layers)]
    ks, vs, indptr, plen, P = PL.device_kv(pairs, 32, DEV)
    kv = E.KVCache(ks, vs, indptr, plen, P)
    tt = torch.zeros(1, 17, dtype=torch.int32, device=DEV)
    with pytest.raises(E.Eagle3Error) as e:
        E.eagle3_tree_verify(ctx, tt, tt, kv)                 # 17 nodes > max_nodes
    assert e.value.code == -2
    inp = PL.synthetic_step_inputs(shape, n_new=3)
    dks, dvs, di, dp, dP = PL.device_kv([inp["draft_kv"]], 32, DEV)
    for bad in (dict(n=3, D=3, K=3, N=10), dict(n=1, D=4, K=3, N=10), dict(n=1, D=3, K=4, N=10), dict(n=1, D=1, K=3, N=5)):
        with pytest.raises(E.Eagle3Error) as e:
            E.eagle3_draft_expand(ctx, inp["g_new"][:bad["n"]].contiguous().to(DEV), inp["tok_new"][:bad["n"]].contiguous().to(DEV),
                                  E.KVCache(dks, dvs, di, dp, dP), bad["D"], bad["K"], bad["N"])
        assert e.value.code == -2, bad
    with pytest.raises(E.Eagle3Error) as e:
        E.eagle3_accept(ctx, torch.zeros(1, 4, shape.vocab, device=DEV), tt[:, :4].contiguous(), tt[:, :4].contiguous(), 1.0, None)
    assert e.value.code == -1


def test_verify_against_a_long_context():
    """20 003 cached tokens under a 60-node tree on the small bf16 model: 313 key tiles cut into dozens of key splits
    (the split merge runs several rounds), prefix not a multiple of the tile; and 9 000 tokens under a 3-node tree."""
    shape = SMALL
    model = PL.OracleModel(shape)
    ctx = _ctx(shape)
    _verify_case(ctx, shape, model, S.random_tree(S.SEED, 61, 60, 8, 10)[0], 20003, seed_salt=31)
    _verify_case(ctx, shape, model, S.random_tree(S.SEED, 62, 3, 2, 2)[0], 9000, seed_salt=32)
