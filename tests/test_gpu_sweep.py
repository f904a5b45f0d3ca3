"""Seeded sweeps over shapes the hand-picked edge cases do not enumerate: node counts, prefix lengths, node orders
and ragged batches drawn at random (fixed seed), every case compared with the oracle element by element."""
import numpy as np
import pytest
import torch

import eagle3_synth as S
from oracle import eagle3_oracle as O
import pipeline as PL
from test_gpu_edges import SMALL, _ctx, _E

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
import os
SALT = int(os.environ.get("SWEEP_SALT", "0"))                # other draws of the same sweeps: SWEEP_SALT=1, 2, ...


def _random_case(rs, salt, n_max):
    N = int(rs.choice([1, 2, 3, 5, 8, 17, 31, 32, 33, 47, 63, 64])) if rs.rand() < 0.5 else int(rs.randint(1, n_max + 1))
    N = min(N, n_max)
    while True:                                               # a depth / fan-out limit the node count fits under
        max_depth, max_children = int(rs.randint(1, 9)), int(rs.randint(1, 11))
        if sum(max_children ** j for j in range(max_depth + 1)) >= 2 * N:
            break
    parent = S.random_tree(S.SEED, 300 + salt, N, max_depth, max_children)[0]
    order = rs.choice(["level", "dfs", "mixed"])
    if order != "level" and N > 2:
        parent = S.reorder_tree(parent, order)[0]
    return np.asarray(parent, dtype=np.int32)


@pytest.mark.parametrize("shape", [S.get_shape("c1"), SMALL], ids=["fp32", "bf16"])
def test_single_sequence_verify_and_accept_sweep(shape):
    """24 random (tree, node order, prefix length) cases: logits, taps, written cache rows, then both acceptance walks
    on the library's own logits against the oracle's walks on the same logits."""
    E = _E()
    rs = np.random.RandomState(11 + 100 * SALT)
    model = PL.OracleModel(shape)
    ctx = _ctx(shape)
    tol = 1e-4 if shape.dtype == "fp32" else 2e-2
    for i in range(24):
        parent = _random_case(rs, i, 64)
        N = len(parent)
        P = int(rs.choice([0, 1, 63, 64, 65, 127, 128, 129])) if rs.rand() < 0.4 else int(rs.randint(0, 400))
        toks = S.uniform_ints(S.SEED + 500 + i, S.TensorIds.TREE_TOK, (N,), 0, shape.vocab).numpy()
        pairs = [S.kv_layer(shape, l, P, seed=S.SEED + 500 + i) for l in range(shape.n_layers)]
        ref = O.tree_verify(shape, model.layer, model.globals(), toks, parent,
                            lambda l: tuple(O.as_f64(t) for t in pairs[l]), rounding=model.rounding)
        ks, vs, indptr, plen, _ = PL.device_kv(pairs, N, DEV)
        kv = E.KVCache(ks, vs, indptr, plen, P)
        tt = torch.as_tensor(toks, dtype=torch.int32, device=DEV)[None]
        pp = torch.as_tensor(parent, dtype=torch.int32, device=DEV)[None]
        logits, taps = E.eagle3_tree_verify(ctx, tt, pp, kv)
        torch.cuda.synchronize()
        case = (i, N, P)
        assert np.max(np.abs(logits[0].cpu().numpy() - ref["logits"])) < tol, case
        assert np.max(np.abs(taps[:, 0].cpu().numpy() - ref["taps"])) < tol, case
        for l in range(shape.n_layers):
            assert np.max(np.abs(ks[l][P:].float().cpu().numpy() - ref["k_new"][l])) < tol, case
            assert np.max(np.abs(vs[l][P:].float().cpu().numpy() - ref["v_new"][l])) < tol, case
        lg = logits[0].cpu().numpy()
        al, gp, bonus = E.eagle3_accept(ctx, logits, tt, pp, 0.0)
        n_acc, rpath, rbonus = O.accept_greedy(lg.astype(np.float64), toks, parent)   # same fp32 values: no tolerance
        assert int(al[0]) == n_acc and int(bonus[0]) == rbonus, case
        assert gp[0].cpu().numpy().tolist() == rpath + [-1] * (N - len(rpath)), case
        U = S.uniform01(S.SEED + i, S.TensorIds.UNIFORMS, (1, 2 * N))
        al, gp, bonus = E.eagle3_accept(ctx, logits, tt, pp, 1.0, U.to(DEV))
        n_acc, rpath, rbonus, margin, info = O.accept_stochastic(lg.astype(np.float64), toks, parent, 1.0,
                                                                 U[0].double().numpy(), return_info=True)
        if info["margin_children"] > 1e-5:
            assert int(al[0]) == n_acc, case
            assert gp[0].cpu().numpy().tolist()[:len(rpath)] == rpath, case
            assert O.bonus_admissible(info, int(bonus[0]), 2e-5), case


def test_ragged_batch_verify_sweep():
    """8 random batches (2..12 sequences, 1..16 nodes, prefix lengths 0..300 with spare slots between the sequences),
    every sequence compared with the single-sequence oracle."""
    E = _E()
    shape = SMALL
    rs = np.random.RandomState(12 + 100 * SALT)
    model = PL.OracleModel(shape)
    for i in range(8):
        B, N = int(rs.randint(2, 13)), int(rs.randint(1, 17))
        ctx = _ctx(shape, max_batch=B, max_nodes=N)
        plens = [int(x) for x in rs.randint(0, 301, size=B)]
        spare = [int(x) for x in rs.randint(0, 5, size=B)]
        parents = np.stack([S.random_tree(S.SEED, 700 + 16 * i + b, N, 5, 4)[0] for b in range(B)]).astype(np.int32)
        toks = S.uniform_ints(S.SEED + 40 + i, S.TensorIds.TREE_TOK, (B, N), 0, shape.vocab).numpy()
        indptr = np.zeros(B + 1, dtype=np.int64)
        indptr[1:] = np.cumsum(np.array(plens) + N + np.array(spare))
        total = int(indptr[-1])
        ks, vs = zip(*[tuple(t.to(DEV) for t in S.kv_layer(shape, l, total)) for l in range(shape.n_layers)])
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
            case = (i, B, N, b, P)
            assert np.max(np.abs(logits[b].cpu().numpy() - ref["logits"])) < 2e-2, case
            assert np.max(np.abs(taps[:, b].cpu().numpy() - ref["taps"])) < 2e-2, case
            for l in range(shape.n_layers):
                got_k = ks[l][base + P:base + P + N].float().cpu().numpy()
                assert np.max(np.abs(got_k - ref["k_new"][l])) < 2e-2, case


def test_commit_sweep_random_paths():
    """10 random batches: every sequence commits a random root path of a random tree (accept lengths 0 .. depth);
    rows of every layer, gathered features, following tokens and advanced lengths are all exact copies."""
    E = _E()
    shape = SMALL.with_(name="small3", n_layers=3, taps=(0, 1, 2))
    rs = np.random.RandomState(13 + 100 * SALT)
    for i in range(10):
        B, N = int(rs.randint(1, 9)), int(rs.choice([1, 2, 7, 16, 33, 64]))
        ctx = _ctx(shape, weights=False, max_batch=B, max_nodes=N)
        plens = rs.randint(0, 200, size=B)
        indptr = np.zeros(B + 1, dtype=np.int64)
        indptr[1:] = np.cumsum(plens + N + rs.randint(0, 4, size=B))
        total = int(indptr[-1])
        ks, vs = zip(*[tuple(t.to(DEV) for t in S.kv_layer(shape, l, total, seed=S.SEED + i)) for l in range(shape.n_layers)])
        k0 = [k.clone() for k in ks]; v0 = [v.clone() for v in vs]
        plen_d = torch.as_tensor(plens, dtype=torch.int32, device=DEV)
        kv = E.KVCache(ks, vs, torch.as_tensor(indptr, dtype=torch.int32, device=DEV), plen_d, int(plens.max()))
        paths, parents = [], []
        for b in range(B):
            depth_cap = max(1, min(8, N - 1))
            parent = S.random_tree(S.SEED, 900 + 16 * i + b, N, depth_cap, 10)[0] if N > 1 else np.array([-1], dtype=np.int32)
            if N > 2 and rs.rand() < 0.5:
                parent = S.reorder_tree(parent, "mixed")[0]
            all_paths = O.ancestor_paths(parent)
            paths.append([int(x) for x in all_paths[int(rs.randint(N))]])
            parents.append(parent)
        path = np.full((B, N), -1, dtype=np.int32)
        for b, p in enumerate(paths):
            path[b, :len(p)] = p
        al = torch.tensor([len(p) - 1 for p in paths], dtype=torch.int32, device=DEV)
        tok = S.uniform_ints(S.SEED + i, S.TensorIds.TREE_TOK, (B, N), 0, shape.vocab).to(DEV)
        bonus = torch.as_tensor(rs.randint(0, shape.vocab, size=B), dtype=torch.int32, device=DEV)
        taps = S.normal(S.SEED + i, S.TensorIds.TAPS, (3, B, N, shape.hidden)).to(DEV)
        rows = max(len(p) for p in paths)
        dpl0 = rs.randint(0, 50, size=B)
        dpl = torch.as_tensor(dpl0, dtype=torch.int32, device=DEV)

        class _D:                                   # only the draft prefix lengths are touched
            prefix_len = dpl
        taps_new, tok_new, n_new = E.eagle3_commit(ctx, tok, torch.as_tensor(path, device=DEV), al, bonus, kv, taps, rows,
                                                   draft_kv=_D, draft_rows=2)
        torch.cuda.synchronize()
        assert n_new.cpu().tolist() == [len(p) for p in paths], i
        assert plen_d.cpu().tolist() == (plens + np.array([len(p) for p in paths])).tolist(), i
        assert dpl.cpu().tolist() == (dpl0 + 2).tolist(), i
        for b, p in enumerate(paths):
            first = int(indptr[b] + plens[b])
            assert tok_new[b, :len(p)].cpu().tolist() == [int(tok[b, q]) for q in p[1:]] + [int(bonus[b])], (i, b)
            assert torch.equal(taps_new[:, b, :len(p)], taps[:, b, p]), (i, b)
            for l in range(shape.n_layers):
                for cur, old in ((ks[l], k0[l]), (vs[l], v0[l])):
                    assert torch.equal(cur[first:first + len(p)], old[first + torch.as_tensor(p, device=DEV)]), (i, b, l)
                    assert torch.equal(cur[int(indptr[b]):first], old[int(indptr[b]):first]), (i, b, l)


@pytest.mark.parametrize("shape", [S.get_shape("c1"), SMALL], ids=["fp32", "bf16"])
def test_draft_expand_sweep(shape):
    """12 random (new rows, depth, top-k, tree size, context length) draws: the tree is bit-compared with the oracle
    (which follows the library's choice only where two candidates are closer than the tolerance), scores by value."""
    E = _E()
    rs = np.random.RandomState(14 + 100 * SALT)
    model = PL.OracleModel(shape)
    ctx = _ctx(shape)
    tol = 1e-4 if shape.dtype == "fp32" else 2e-2
    for i in range(12):
        n_new, D, K = int(rs.randint(1, 9)), int(rs.randint(1, 9)), int(rs.randint(1, 9))
        pool = 1 + K + (D - 1) * K * K
        N = int(rs.randint(2, min(64, pool) + 1))
        inp = PL.synthetic_step_inputs(shape, seed=S.SEED + 60 + i, n_new=n_new, prefix=int(rs.randint(0, 200)) + n_new)
        ks, vs, indptr, plen, P = PL.device_kv([inp["draft_kv"]], n_new + (D - 1) * K, DEV)
        got = E.eagle3_draft_expand(ctx, inp["g_new"].to(DEV), inp["tok_new"].to(DEV), E.KVCache(ks, vs, indptr, plen, P),
                                    D, K, N, debug=True)
        torch.cuda.synchronize()
        got = {k: v.cpu().numpy() for k, v in got.items()}
        ref = PL.oracle_draft(shape, model, inp, D, K, N, tol=tol / 2,
                              follow={"pool_tok": got["pool_tok"], "frontier": got["frontier"], "chosen": got["chosen"]})
        case = (i, n_new, D, K, N)
        if ref["min_gap"] > tol / 2:
            assert ref["n_followed"] == 0, case
        for key in ("tree_tok", "parent", "depth", "chosen"):
            assert np.array_equal(got[key], ref[key]), (case, key)
        assert np.max(np.abs(got["score"] - ref["score"])) < tol, case
        assert all(got["parent"][j] < j for j in range(1, N)) and got["parent"][0] == -1, case


def test_chain_drafting_sweep():
    """8 random batched chain drafts on the exact fp32 model (batch 1..12, 1..6 new rows per sequence with ragged
    counts, chains of 1..4 tokens, ragged draft contexts of 0..89 tokens): tokens, cumulative log-probabilities and
    the cache rows against the per-sequence oracle."""
    from test_gpu_decode import _chain_case
    E = _E()
    rs = np.random.RandomState(15 + 100 * SALT)
    for i in range(8):
        B, rows1, L = int(rs.randint(1, 13)), int(rs.randint(1, 7)), int(rs.randint(1, 5))
        _chain_case(E, S.get_shape("c1"), B, rows1, L, 200 + 10 * SALT + i, 1e-4)


def test_ttt_attention_sweep():
    """10 random training-time-test attention shapes (1..400 positions, grouped heads, simulated steps 0..4) in bf16
    storage, and 4 in fp32, every output element against the oracle's dense-mask form."""
    import torch
    from test_gpu_ttt import _case
    E = _E()
    rs = np.random.RandomState(16 + 100 * SALT)
    for i in range(10):
        T = int(rs.choice([1, 31, 32, 33, 63, 64, 65, 127, 128, 129])) if rs.rand() < 0.5 else int(rs.randint(1, 401))
        H, Hkv = [(2, 1), (4, 2), (4, 4), (8, 2), (2, 2)][int(rs.randint(5))]
        s = int(rs.randint(0, 5))
        err = _case(E, T, H, Hkv, 128, s, torch.bfloat16, 300 + 20 * SALT + i)
        assert err < 2e-3, (T, H, Hkv, s, err)
    for i in range(4):
        T, s = int(rs.randint(1, 120)), int(rs.randint(0, 4))
        H, Hkv = [(2, 1), (4, 2), (4, 4)][int(rs.randint(3))]
        assert _case(E, T, H, Hkv, 64, s, torch.float32, 340 + 20 * SALT + i) < 1e-5, (T, H, Hkv, s)


def test_prefill_sweep():
    """6 random prompts (1..90 tokens) prefilled in chunks of 1..64 positions on the exact fp32 model: the target cache
    of every layer, the draft cache, the last position's logits and fused feature against the oracle's prefill."""
    E = _E()
    rs = np.random.RandomState(17 + 100 * SALT)
    base = S.get_shape("c1")
    model = PL.OracleModel(base)
    W = PL.device_weights(base, device=DEV)
    for i in range(6):
        T = int(rs.choice([1, 2, 63, 64, 65])) if rs.rand() < 0.4 else int(rs.randint(1, 91))
        chunk = int(rs.choice([1, 7, 16, 33, 64]))
        shape = base.with_(prefix_lo=T, prefix_hi=T)
        inp = PL.real_prefill_inputs(shape, model, seed=S.SEED + 400 + 10 * SALT + i)
        prompt, pre = inp["prefix_tok"], inp["prefill"]
        ctx = E.Eagle3Context(shape, max_batch=1, max_nodes=chunk, max_depth=2, max_topk=2, max_new=chunk, device=DEV)
        ctx.set_weights(W["target"], W["draft"])
        cap = T + 8
        z = lambda: torch.zeros(cap, shape.n_kv_heads, shape.head_dim, dtype=torch.float32, device=DEV)
        ks, vs = [z() for _ in range(shape.n_layers)], [z() for _ in range(shape.n_layers)]
        i32 = lambda v: torch.tensor(v, dtype=torch.int32, device=DEV)
        kv = E.KVCache(ks, vs, i32([0, cap]), i32([0]), 0)
        dkv = E.KVCache([z()], [z()], i32([0, cap]), i32([0]), 0)
        g_last, logits = E.eagle3_prefill(ctx, torch.as_tensor(prompt, dtype=torch.int32, device=DEV), kv, dkv)
        torch.cuda.synchronize()
        case = (i, T, chunk)
        assert int(kv.prefix_len[0]) == T and int(dkv.prefix_len[0]) == T - 1, case
        for l in range(shape.n_layers):
            assert np.max(np.abs(ks[l][:T].cpu().numpy() - pre["k_new"][l])) < 1e-4, case
            assert np.max(np.abs(vs[l][:T].cpu().numpy() - pre["v_new"][l])) < 1e-4, case
        assert np.max(np.abs(logits.cpu().numpy() - pre["logits"][-1])) < 1e-4, case
        assert np.max(np.abs(g_last.cpu().numpy() - inp["g_new"][0].numpy())) < 1e-4, case
        if T > 1:
            Kd, Vd = inp["draft_kv"]
            assert np.max(np.abs(dkv.k_layers[0][:T - 1].cpu().numpy() - Kd.numpy())) < 1e-4, case
            assert np.max(np.abs(dkv.v_layers[0][:T - 1].cpu().numpy() - Vd.numpy())) < 1e-4, case


def test_multi_step_decode_sweep():
    """4 random prompts (2..40 tokens) taken through eagle3_prefill and 8 draft-verify-commit cycles with random
    planted acceptance lengths and random tree sizes, entirely on the library's own state: the emitted tokens must be
    the oracle target's plain greedy decoding."""
    from test_gpu_decode import gpu_decode
    from test_oracle_decode import planted_hook
    E = _E()
    rs = np.random.RandomState(18 + 100 * SALT)
    shape = S.get_shape("c1")
    D, K = shape.depth, shape.topk
    model = PL.OracleModel(shape)
    W = PL.device_weights(shape, device=DEV)
    n_steps = 8
    for i in range(4):
        T = int(rs.randint(2, 41))
        N = int(rs.randint(D + 2, 31))
        prompt = S.uniform_ints(S.SEED + 500 + 10 * SALT + i, S.TensorIds.PREFIX_TOK, (T,), 0, shape.vocab).numpy()
        ref = O.greedy_decode(shape, model.layer, model.globals(), prompt, n_steps * (D + 1) + 2)
        ctx = E.Eagle3Context(shape, max_batch=1, max_nodes=32, max_depth=D, max_topk=K, max_new=32, device=DEV)
        ctx.set_weights(W["target"], W["draft"])
        cap = T + n_steps * (D + 1) + N + (D - 1) * K + 8
        z = lambda: torch.zeros(cap, shape.n_kv_heads, shape.head_dim, dtype=torch.float32, device=DEV)
        i32 = lambda v: torch.tensor(v, dtype=torch.int32, device=DEV)
        kv = E.KVCache([z() for _ in range(shape.n_layers)], [z() for _ in range(shape.n_layers)], i32([0, cap]), i32([0]), 0)
        dkv = E.KVCache([z()], [z()], i32([0, cap]), i32([0]), 0)
        g_last, logits = E.eagle3_prefill(ctx, torch.as_tensor(prompt, dtype=torch.int32, device=DEV), kv, dkv)
        root = int(torch.argmax(logits))
        assert root == ref[0], (i, T)
        kv.set_max_prefix_len(T)
        dkv.set_max_prefix_len(T - 1)
        wanted = [int(x) for x in rs.randint(0, D + 1, size=n_steps)]
        state = {"kv": kv, "dkv": dkv, "g_new": g_last[None].contiguous(), "tok_new": i32([root]), "P": T, "Pd": T - 1}
        emitted, accept_lens, trees = gpu_decode(E, ctx, shape, state, n_steps, D, K, N, planted_hook(ref, wanted))
        assert emitted == ref[:len(emitted)], (i, T, N, wanted, accept_lens)
        reach = [int(O.tree_depth(pp).max()) for _, pp, _ in trees]      # a small tree may be shallower than the plant
        assert all(a >= min(w, r) for a, w, r in zip(accept_lens, wanted, reach)), (wanted, reach, accept_lens)


@pytest.mark.parametrize("hidden,inter", [(1024, 1408), (1152, 2816), (1280, 1536), (1408, 1664)])
def test_gemm_stage_count_sweep(hidden, inter):
    """bf16 models whose projections have 8, 9, 10 and 11 (hidden) and 11, 22, 12 and 13 (intermediate) K stages: every
    remainder of the GEMM kernels' unrolled stage loops and of their split-K choices, through one verification
    (17, 60 rows: the few-row and the 64-row kernels; 96 rows in a batch: the many-row kernel) and one draft expansion."""
    E = _E()
    shape = S.get_shape("c2").with_(name=f"h{hidden}", hidden=hidden, n_heads=hidden // 128, n_kv_heads=2 if hidden % 256 == 0 else 1,
                                    intermediate=inter, vocab=2048 + 64, draft_vocab=1024, n_layers=1, taps=(0, 0, 0),
                                    prefix_lo=70, prefix_hi=70, depth=3, topk=4, n_nodes=17)
    model = PL.OracleModel(shape)
    ctx = _ctx(shape, max_batch=6, max_nodes=64)
    rs = np.random.RandomState(hidden + 100 * SALT)
    for N in (17, 60):
        parent = S.random_tree(S.SEED, 800 + N, N, 6, 8)[0]
        P = int(rs.randint(1, 200))
        toks = S.uniform_ints(S.SEED + N, S.TensorIds.TREE_TOK, (N,), 0, shape.vocab).numpy()
        pairs = [S.kv_layer(shape, 0, P, seed=S.SEED + N)]
        ref = O.tree_verify(shape, model.layer, model.globals(), toks, parent, lambda l: tuple(O.as_f64(t) for t in pairs[l]),
                            rounding="bf16")
        ks, vs, indptr, plen, _ = PL.device_kv(pairs, N, DEV)
        logits, taps = E.eagle3_tree_verify(ctx, torch.as_tensor(toks, dtype=torch.int32, device=DEV)[None],
                                            torch.as_tensor(parent, dtype=torch.int32, device=DEV)[None],
                                            E.KVCache(ks, vs, indptr, plen, P))
        torch.cuda.synchronize()
        assert np.max(np.abs(logits[0].cpu().numpy() - ref["logits"])) < 2e-2, (hidden, N)
        assert np.max(np.abs(taps[:, 0].cpu().numpy() - ref["taps"])) < 2e-2 * max(1.0, float(np.sqrt(np.mean(ref["taps"] ** 2)))), (hidden, N)
    # a batch of 6 x 16 = 96 rows
    B, N = 6, 16
    plens = [int(x) for x in rs.randint(0, 150, size=B)]
    parents = np.stack([S.random_tree(S.SEED, 820 + b, N, 4, 3)[0] for b in range(B)]).astype(np.int32)
    toks = S.uniform_ints(S.SEED + 7, S.TensorIds.TREE_TOK, (B, N), 0, shape.vocab).numpy()
    indptr = np.zeros(B + 1, dtype=np.int64)
    indptr[1:] = np.cumsum(np.array(plens) + N)
    K_all, V_all = S.kv_layer(shape, 0, int(indptr[-1]))
    kv = E.KVCache([K_all.to(DEV)], [V_all.to(DEV)], torch.as_tensor(indptr, dtype=torch.int32, device=DEV),
                   torch.tensor(plens, dtype=torch.int32, device=DEV), max(plens))
    logits, taps = E.eagle3_tree_verify(ctx, torch.as_tensor(toks, dtype=torch.int32, device=DEV),
                                        torch.as_tensor(parents, dtype=torch.int32, device=DEV), kv)
    torch.cuda.synchronize()
    for b in range(B):
        base, P = int(indptr[b]), plens[b]
        ref = O.tree_verify(shape, model.layer, model.globals(), toks[b], parents[b],
                            lambda l: tuple(O.as_f64(t) for t in S.kv_layer(shape, l, P, first_slot=base)), rounding="bf16")
        assert np.max(np.abs(logits[b].cpu().numpy() - ref["logits"])) < 2e-2, (hidden, "batch", b)
    # one draft expansion (2k-wide draft input: twice as many stages)
    D, K, N = 3, 4, 17
    inp = PL.synthetic_step_inputs(shape, n_new=2, prefix=72)
    ks, vs, indptr, plen, P = PL.device_kv([inp["draft_kv"]], 2 + (D - 1) * K, DEV)
    got = E.eagle3_draft_expand(ctx, inp["g_new"].to(DEV), inp["tok_new"].to(DEV), E.KVCache(ks, vs, indptr, plen, P), D, K, N, debug=True)
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in got.items()}
    ref = PL.oracle_draft(shape, model, inp, D, K, N, follow={"pool_tok": got["pool_tok"], "frontier": got["frontier"], "chosen": got["chosen"]})
    for key in ("tree_tok", "parent", "depth", "chosen"):
        assert np.array_equal(got[key], ref[key]), (hidden, key)
    assert np.max(np.abs(got["score"] - ref["score"])) < 2e-2, hidden
