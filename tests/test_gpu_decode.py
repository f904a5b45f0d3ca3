"""Several draft-verify cycles on the GPU, each fed by the previous one through eagle3_commit: the emitted tokens
must be the target's plain greedy decoding (Section 2.1: lossless), and the per-cycle accepted lengths give tau
(Section 4 "Metrics") mechanically."""
import numpy as np
import pytest
import torch

import eagle3_synth as S
from oracle import eagle3_oracle as O
import pipeline as PL
from test_oracle_decode import planted_hook

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def gpu_decode(E, ctx, shape, state, n_steps, D, K, N, hook=None):
    """state: dict(kv, dkv, g_new [n,k] device, tok_new [n] device, P (target prefix), Pd (draft prefix)).
    Returns (emitted tokens after the first root, accept_lens, per-step trees)."""
    kv, dkv = state["kv"], state["dkv"]
    g_new, tok_new = state["g_new"], state["tok_new"]
    P, Pd = state["P"], state["Pd"]
    emitted, accept_lens, trees = [int(tok_new[-1])], [], []
    for step in range(n_steps):
        n_prev = g_new.shape[0]
        tree = E.eagle3_draft_expand(ctx, g_new, tok_new, dkv, D, K, N)
        tt, pp = tree["tree_tok"][None].contiguous(), tree["parent"][None].contiguous()
        if hook is not None:
            new_tok = hook(step, tt[0].cpu().numpy().copy(), pp[0].cpu().numpy(), tree["depth"].cpu().numpy(), emitted)
            tt = torch.as_tensor(new_tok, dtype=torch.int32, device=DEV)[None].contiguous()
        logits, taps = E.eagle3_tree_verify(ctx, tt, pp, kv)
        al, path, bonus = E.eagle3_accept(ctx, logits, tt, pp, 0.0)
        taps_new, tok_rows, n_new = E.eagle3_commit(ctx, tt, path, al, bonus, kv, taps, D + 1, draft_kv=dkv, draft_rows=n_prev)
        n = int(n_new[0])                                            # the host needs the tokens anyway
        assert n == int(al[0]) + 1
        P, Pd = P + n, Pd + n_prev
        assert int(kv.prefix_len[0]) == P and int(dkv.prefix_len[0]) == Pd
        kv.set_max_prefix_len(P)
        dkv.set_max_prefix_len(Pd)
        g_new = E.eagle3_fuse_features(ctx, *[taps_new[t, 0, :n].contiguous() for t in range(3)])
        tok_new = tok_rows[0, :n].contiguous()
        emitted += tok_new.cpu().numpy().tolist()
        accept_lens.append(n - 1)
        trees.append((tt[0].cpu().numpy(), pp[0].cpu().numpy(), path[0].cpu().numpy()))
    return emitted, accept_lens, trees


def oracle_prefill_state(E, shape, model, prompt, extra_slots):
    """Caches, features and the first root from the ORACLE's prefill, mirrored onto the device."""
    P = len(prompt)
    pre = O.prefill(shape, model.layer, model.globals(), prompt)
    dw, emb = model.draft(), model.globals()["embed"]
    g_all = O.fuse_features(dw["w_fc"], pre["taps"][0], pre["taps"][1], pre["taps"][2])
    Kd = np.zeros((P - 1, shape.n_kv_heads, shape.head_dim)); Vd = np.zeros_like(Kd)
    O.draft_forward(shape, dw, emb, g_all[:P - 1], prompt[1:], np.arange(P - 1), Kd, Vd, 0, 0,
                    np.tril(np.ones((P - 1, P - 1), dtype=bool)), lambda a: a)
    pairs = [(torch.from_numpy(pre["k_new"][l]).float(), torch.from_numpy(pre["v_new"][l]).float()) for l in range(shape.n_layers)]
    ks, vs, indptr, plen, _ = PL.device_kv(pairs, extra_slots, DEV)
    dks, dvs, dindptr, dplen, _ = PL.device_kv([(torch.from_numpy(Kd).float(), torch.from_numpy(Vd).float())], extra_slots, DEV)
    root = int(np.argmax(pre["logits"][-1]))
    return {"kv": E.KVCache(ks, vs, indptr, plen, P), "dkv": E.KVCache(dks, dvs, dindptr, dplen, P - 1),
            "g_new": torch.from_numpy(g_all[P - 1:P].copy()).float().to(DEV),
            "tok_new": torch.tensor([root], dtype=torch.int32, device=DEV), "P": P, "Pd": P - 1}


def test_multi_step_greedy_decode_equals_plain_greedy_decoding():
    import paper_2503_01840_amd as E
    shape = S.get_shape("c1")
    D, K, N = shape.depth, shape.topk, 30
    model = PL.OracleModel(shape)
    prompt = S.uniform_ints(S.SEED, S.TensorIds.PREFIX_TOK, (12,), 0, shape.vocab).numpy()
    ref = O.greedy_decode(shape, model.layer, model.globals(), prompt, 48)
    ctx = E.Eagle3Context(shape, max_batch=1, max_nodes=32, max_depth=D, max_topk=K, max_new=D + 1, device=DEV)
    W = PL.device_weights(shape, device=DEV)
    ctx.set_weights(W["target"], W["draft"])
    wanted = [3, 0, 1, 2, 3, 1, 2, 3, 0, 3, 2, 1]
    n_steps = 14
    hook = planted_hook(ref, wanted)
    state = oracle_prefill_state(E, shape, model, prompt, n_steps * (D + 1) + N + (D - 1) * K + 8)
    emitted, accept_lens, trees = gpu_decode(E, ctx, shape, state, n_steps, D, K, N, hook)
    assert len(emitted) >= 32
    assert emitted == ref[:len(emitted)], "greedy speculative decoding must reproduce plain greedy decoding"
    want = (wanted * 2)[:n_steps]
    assert all(a >= w for a, w in zip(accept_lens, want))
    assert max(accept_lens) == D and min(accept_lens) == 0          # every compaction distance occurs
    # the oracle's own multi-step run with the same planted continuations: same accepted lengths, same paths
    out = O.speculative_decode(shape, model.layer, model.globals(), model.draft(), prompt, n_steps, D, K, N, tree_hook=hook)
    assert out["tokens"] == emitted
    assert out["accept_lens"] == accept_lens
    for rec, (tt, pp, path) in zip(out["records"], trees):
        assert np.array_equal(rec["parent"], pp) and np.array_equal(rec["tree_tok"], tt)
        assert path[:len(rec["path"])].tolist() == list(rec["path"])
    tau = float(np.mean(np.asarray(accept_lens) + 1))
    print(f"{len(emitted)} tokens in {n_steps} cycles: tau = {tau:.2f} (planted), accepted lengths {accept_lens}")
    # without planted tokens the random-weight draft almost never guesses right: still lossless
    state = oracle_prefill_state(E, shape, model, prompt, n_steps * (D + 1) + N + (D - 1) * K + 8)
    emitted2, accept2, _ = gpu_decode(E, ctx, shape, state, 6, D, K, N, None)
    assert emitted2 == ref[:len(emitted2)]


def test_commit_moves_rows_in_every_layer_for_a_ragged_batch():
    """bf16 storage, 3 sequences with different prefixes and paths (including a path whose sources and destinations
    overlap: 0, 2, 5, 6, 9 ... and the longest possible chain), every layer's keys and values checked."""
    import paper_2503_01840_amd as E
    shape = S.get_shape("c2").with_(name="small", hidden=256, n_heads=4, n_kv_heads=2, intermediate=512, vocab=1024,
                                    draft_vocab=512, n_layers=3, taps=(0, 1, 2))
    B, N = 3, 24
    ctx = E.Eagle3Context(shape, max_batch=B, max_nodes=N, max_depth=8, max_topk=4, max_new=8, device=DEV)
    plens = np.array([5, 0, 130])
    indptr = np.zeros(B + 1, dtype=np.int64)
    indptr[1:] = np.cumsum(plens + N + 2)
    total = int(indptr[-1])
    ks, vs = zip(*[tuple(t.to(DEV) for t in S.kv_layer(shape, l, total)) for l in range(shape.n_layers)])
    k0 = [k.clone() for k in ks]; v0 = [v.clone() for v in vs]
    plen_d = torch.as_tensor(plens, dtype=torch.int32, device=DEV)
    kv = E.KVCache(ks, vs, torch.as_tensor(indptr, dtype=torch.int32, device=DEV), plen_d, int(plens.max()))
    paths = [[0, 2, 5, 6, 9, 10, 17, 20, 23], [0], list(range(0, 24))[:12]]
    paths[2] = [0, 1, 2, 3, 5, 6, 7, 8, 10, 12, 13, 23]
    path = np.full((B, N), -1, dtype=np.int32)
    for b, p in enumerate(paths):
        path[b, :len(p)] = p
    al = torch.tensor([len(p) - 1 for p in paths], dtype=torch.int32, device=DEV)
    tok = S.uniform_ints(S.SEED, S.TensorIds.TREE_TOK, (B, N), 0, shape.vocab).to(DEV)
    bonus = torch.tensor([7, 8, 9], dtype=torch.int32, device=DEV)
    taps = S.normal(S.SEED, S.TensorIds.TAPS, (3, B, N, shape.hidden)).to(DEV)
    rows = 12
    dpl = torch.tensor([4, 4, 4], dtype=torch.int32, device=DEV)

    class _D:                                   # only the draft prefix lengths are touched
        prefix_len = dpl
    taps_new, tok_new, n_new = E.eagle3_commit(ctx, tok, torch.as_tensor(path, device=DEV), al, bonus, kv, taps, rows,
                                               draft_kv=_D, draft_rows=3)
    torch.cuda.synchronize()
    assert n_new.cpu().tolist() == [len(p) for p in paths]
    assert plen_d.cpu().tolist() == (plens + np.array([len(p) for p in paths])).tolist()
    assert dpl.cpu().tolist() == [7, 7, 7]
    for b, p in enumerate(paths):
        first = int(indptr[b] + plens[b])
        want_tok = [int(tok[b, q]) for q in p[1:]] + [int(bonus[b])]
        assert tok_new[b, :len(p)].cpu().tolist() == want_tok
        assert torch.equal(taps_new[:, b, :len(p)], taps[:, b, p])
        for l in range(shape.n_layers):
            for cur, old in ((ks[l], k0[l]), (vs[l], v0[l])):
                assert torch.equal(cur[first:first + len(p)], old[first + torch.as_tensor(p, device=DEV)]), (b, l)
                assert torch.equal(cur[int(indptr[b]):first], old[int(indptr[b]):first])   # the context did not move


@pytest.mark.parametrize("chunk", [64, 24])
def test_prefill_builds_caches_features_and_the_draft_context(chunk):
    """eagle3_prefill against the oracle's prefill (tiny fp32 model, 64-token prompt; one chunk of 64, and chunks of
    24 + 24 + 16): target cache of every layer, draft cache, fused feature and logits of the last position; then
    decoding continues from the GPU-built state and still equals plain greedy decoding."""
    import paper_2503_01840_amd as E
    shape = S.get_shape("c1")
    D, K, N = shape.depth, shape.topk, min(chunk, 30)
    model = PL.OracleModel(shape)
    inp = PL.real_prefill_inputs(shape, model)
    prompt, pre, P = inp["prefix_tok"], inp["prefill"], inp["P"]
    ctx = E.Eagle3Context(shape, max_batch=1, max_nodes=chunk, max_depth=D, max_topk=K, max_new=chunk, device=DEV)
    W = PL.device_weights(shape, device=DEV)
    ctx.set_weights(W["target"], W["draft"])
    cap = P + 8 * (D + 1) + 64
    z = lambda: torch.zeros(cap, shape.n_kv_heads, shape.head_dim, dtype=torch.float32, device=DEV)
    ks, vs = [z() for _ in range(shape.n_layers)], [z() for _ in range(shape.n_layers)]
    i32 = lambda v: torch.tensor(v, dtype=torch.int32, device=DEV)
    kv = E.KVCache(ks, vs, i32([0, cap]), i32([0]), 0)
    dkv = E.KVCache([z()], [z()], i32([0, cap]), i32([0]), 0)
    g_last, logits = E.eagle3_prefill(ctx, torch.as_tensor(prompt, dtype=torch.int32, device=DEV), kv, dkv)
    torch.cuda.synchronize()
    assert int(kv.prefix_len[0]) == P and int(dkv.prefix_len[0]) == P - 1
    for l in range(shape.n_layers):
        assert np.max(np.abs(ks[l][:P].cpu().numpy() - pre["k_new"][l])) < 1e-4, l
        assert np.max(np.abs(vs[l][:P].cpu().numpy() - pre["v_new"][l])) < 1e-4, l
    assert np.max(np.abs(logits.cpu().numpy() - pre["logits"][-1])) < 1e-4
    assert np.max(np.abs(g_last.cpu().numpy() - inp["g_new"][0].numpy())) < 1e-4
    Kd, Vd = inp["draft_kv"]
    assert np.max(np.abs(dkv.k_layers[0][:P - 1].cpu().numpy() - Kd.numpy())) < 1e-4
    assert np.max(np.abs(dkv.v_layers[0][:P - 1].cpu().numpy() - Vd.numpy())) < 1e-4
    # go on decoding from this state
    root = int(torch.argmax(logits))
    assert root == int(inp["tok_new"][0])
    ref = O.greedy_decode(shape, model.layer, model.globals(), prompt, 24)
    state = {"kv": kv, "dkv": dkv, "g_new": g_last[None].contiguous(), "tok_new": i32([root]), "P": P, "Pd": P - 1}
    emitted, accept_lens, _ = gpu_decode(E, ctx, shape, state, 5, D, K, N, planted_hook(ref, [2, 1, 0, 2]))
    assert emitted == ref[:len(emitted)] and max(accept_lens) >= 2


def _chain_case(E, shape, B, rows1, L, seed, tol):
    model = PL.OracleModel(shape)
    dw, emb = model.draft(), model.globals()["embed"]
    rs = np.random.RandomState(seed)
    n_ctx = rs.randint(0, 90, B)
    n_ctx[0] = 0                                         # one sequence with an empty draft context
    n_new = rs.randint(1, rows1 + 1, B)
    n_new[-1] = rows1
    dt = torch.float32 if shape.dtype == "fp32" else torch.bfloat16
    g = S.normal(S.SEED + seed, S.TensorIds.G_NEW, (B, rows1, shape.hidden))
    tok = S.uniform_ints(S.SEED + seed, S.TensorIds.TOK_NEW, (B, rows1), 0, shape.vocab)
    cap = rows1 + L + 2
    indptr = np.zeros(B + 1, dtype=np.int64)
    indptr[1:] = np.cumsum(n_ctx + cap)
    total = int(indptr[-1])
    K_all, V_all = S.kv_layer(shape, 0, total, seed=S.SEED + seed, draft=True)
    ctx = E.Eagle3Context(shape, max_batch=B, max_nodes=max(rows1, L + 1, 8), max_depth=max(L, 2), max_topk=4, max_new=max(rows1, 2),
                          device=DEV)
    W = PL.device_weights(shape, device=DEV)
    ctx.set_weights(W["target"], W["draft"])
    Kd, Vd = K_all.to(DEV), V_all.to(DEV)
    dkv = E.KVCache([Kd], [Vd], torch.as_tensor(indptr, dtype=torch.int32, device=DEV),
                    torch.as_tensor(n_ctx, dtype=torch.int32, device=DEV), int(n_ctx.max()))
    chain_tok, chain_logp = E.eagle3_draft_chain(ctx, g.to(DEV), tok.to(DEV), torch.as_tensor(n_new, dtype=torch.int32, device=DEV),
                                                 dkv, L)
    torch.cuda.synchronize()
    caches = []
    for b in range(B):
        lo = int(indptr[b])
        Kc = np.zeros((int(n_ctx[b]) + cap, shape.n_kv_heads, shape.head_dim)); Vc = np.zeros_like(Kc)
        Kc[:n_ctx[b]] = O.as_f64(K_all[lo:lo + n_ctx[b]]); Vc[:n_ctx[b]] = O.as_f64(V_all[lo:lo + n_ctx[b]])
        caches.append((Kc, Vc))
    ref_tok, ref_logp = O.draft_chains(shape, dw, emb, [O.as_f64(g[b, :n_new[b]]) for b in range(B)],
                                       [tok[b, :n_new[b]].numpy().astype(np.int64) for b in range(B)], caches, n_ctx, L,
                                       rounding=model.rounding)
    got_tok, got_logp = chain_tok.cpu().numpy(), chain_logp.cpu().numpy()
    # arg-max margins of the oracle decide whether a differing token is a near-tie; none is expected at these sizes
    assert np.array_equal(got_tok, ref_tok), (got_tok, ref_tok)
    assert np.max(np.abs(got_logp - ref_logp)) < tol * L
    for b in range(B):                                   # the cache rows of the real positions and of the chain
        lo, c, n = int(indptr[b]), int(n_ctx[b]), int(n_new[b])
        rows = slice(lo + c, lo + c + n + L - 1)
        assert np.max(np.abs(Kd[rows].float().cpu().numpy() - caches[b][0][c:c + n + L - 1])) < tol, b
        assert np.max(np.abs(Vd[rows].float().cpu().numpy() - caches[b][1][c:c + n + L - 1])) < tol, b


def test_batched_chain_drafting_matches_the_per_sequence_oracle():
    import paper_2503_01840_amd as E
    _chain_case(E, S.get_shape("c1"), 3, 3, 3, 1, 1e-4)                     # fp32, exact
    small = S.get_shape("c2").with_(name="small", hidden=256, n_heads=4, n_kv_heads=2, intermediate=512, vocab=1024,
                                    draft_vocab=512, n_layers=1, taps=(0, 0, 0))
    _chain_case(E, small, 5, 1, 2, 2, 2e-2)                                 # one new position per sequence
    _chain_case(E, small, 7, 4, 3, 3, 2e-2)                                 # ragged n_new, 28 rows in forward 1
    _chain_case(E, small, 24, 3, 2, 4, 2e-2)                                # 72 rows: the many-row GEMM path


def test_batched_chain_decoding_equals_plain_greedy_decoding_per_sequence():
    """The serving regime of Sections 4.3 / 4.4 end to end on the tiny model: three sequences with different prompts
    share one ragged cache; per cycle one batched chain draft (3 tokens), one batched verification of the 4-node chains,
    acceptance and commit for the whole batch; the next cycle's rows per sequence are ragged (accept_len + 1).  Every
    sequence must reproduce its own plain greedy decoding; planted continuations exercise every accepted length."""
    import paper_2503_01840_amd as E
    shape = S.get_shape("c1")
    model = PL.OracleModel(shape)
    B, L, n_steps = 3, 3, 8
    N = L + 1
    lens = [9, 17, 12]
    prompts = [S.uniform_ints(S.SEED + 40 + b, S.TensorIds.PREFIX_TOK, (lens[b],), 0, shape.vocab).numpy() for b in range(B)]
    refs = [O.greedy_decode(shape, model.layer, model.globals(), prompts[b], 40) for b in range(B)]
    ctx = E.Eagle3Context(shape, max_batch=B, max_nodes=32, max_depth=4, max_topk=4, max_new=32, device=DEV)
    W = PL.device_weights(shape, device=DEV)
    ctx.set_weights(W["target"], W["draft"])
    cap = max(lens) + n_steps * N + 16
    i32 = lambda v: torch.tensor(v, dtype=torch.int32, device=DEV)
    z = lambda: torch.zeros(B * cap, shape.n_kv_heads, shape.head_dim, dtype=torch.float32, device=DEV)
    ks, vs = [z() for _ in range(shape.n_layers)], [z() for _ in range(shape.n_layers)]
    dk, dv = z(), z()
    indptr = i32([b * cap for b in range(B + 1)])
    plen, dplen = i32([0] * B), i32([0] * B)
    kv = E.KVCache(ks, vs, indptr, plen, 0)
    dkv = E.KVCache([dk], [dv], indptr, dplen, 0)
    g_rows = torch.zeros(B, N, shape.hidden, dtype=torch.float32, device=DEV)
    tok_rows = torch.zeros(B, N, dtype=torch.int32, device=DEV)
    emitted = []
    for b in range(B):                                   # prefill one sequence at a time into its slice of the caches
        kvb = E.KVCache(ks, vs, indptr[b:b + 2], plen[b:b + 1], 0)
        dkvb = E.KVCache([dk], [dv], indptr[b:b + 2], dplen[b:b + 1], 0)
        g_last, logits = E.eagle3_prefill(ctx, torch.as_tensor(prompts[b], dtype=torch.int32, device=DEV), kvb, dkvb)
        root = int(torch.argmax(logits))
        assert root == refs[b][0]
        g_rows[b, 0], tok_rows[b, 0] = g_last, root
        emitted.append([root])
    n_new = i32([1] * B)
    parent = i32(np.tile(np.arange(-1, L), (B, 1)))
    wanted = [[3, 0, 2, 1], [1, 3, 0, 2], [0, 2, 3, 3]]
    accepted = [[] for _ in range(B)]
    for step in range(n_steps):
        rows1 = int(n_new.max())
        kv.set_max_prefix_len(int(plen.max()))
        dkv.set_max_prefix_len(int(dplen.max()))
        chain_tok, chain_logp = E.eagle3_draft_chain(ctx, g_rows[:, :rows1].contiguous(), tok_rows[:, :rows1].contiguous(), n_new,
                                                     dkv, L)
        ct = chain_tok.cpu().numpy().copy()
        for b in range(B):                               # plant the true continuation to the wanted depth
            pos = len(emitted[b])
            for lvl in range(wanted[b][step % 4]):
                ct[b, 1 + lvl] = refs[b][pos + lvl]
        tt = torch.as_tensor(ct, dtype=torch.int32, device=DEV)
        logits, taps = E.eagle3_tree_verify(ctx, tt, parent, kv)
        al, path, bonus = E.eagle3_accept(ctx, logits, tt, parent, 0.0)
        prev = n_new.clone()
        taps_new, tok_new, n_new = E.eagle3_commit(ctx, tt, path, al, bonus, kv, taps, N)
        dplen += prev                                    # forward 1's real rows of every sequence stay in the draft cache
        for b in range(B):
            n = int(n_new[b])
            assert n - 1 >= wanted[b][step % 4]
            accepted[b].append(n - 1)
            emitted[b] += tok_new[b, :n].cpu().numpy().tolist()
            g_rows[b, :n] = E.eagle3_fuse_features(ctx, *[taps_new[t, b, :n].contiguous() for t in range(3)])
        tok_rows = tok_new
    for b in range(B):
        assert emitted[b] == refs[b][:len(emitted[b])], b
        assert max(accepted[b]) == L and min(accepted[b]) == 0
    print("batched chain decoding: accepted lengths per sequence", accepted)


def test_prefill_bf16_two_chunks_matches_the_oracle():
    """bf16 storage: a 70-token prompt in chunks of 64 + 6 against the oracle's prefill in bf16 mode (2-layer model, so
    the single-layer tolerances apply): target cache, draft cache, fused feature and logits of the last position."""
    import paper_2503_01840_amd as E
    shape = S.get_shape("c2").with_(name="small", hidden=256, n_heads=4, n_kv_heads=2, intermediate=512, vocab=1024,
                                    draft_vocab=512, n_layers=2, taps=(0, 1, 1))
    model = PL.OracleModel(shape)
    T = 70
    prompt = S.uniform_ints(S.SEED + 3, S.TensorIds.PREFIX_TOK, (T,), 0, shape.vocab).numpy()
    pre = O.prefill(shape, model.layer, model.globals(), prompt, rounding="bf16")
    dw, emb = model.draft(), model.globals()["embed"]
    g_all = O.fuse_features(dw["w_fc"], pre["taps"][0], pre["taps"][1], pre["taps"][2], rounding="bf16")
    Kd = np.zeros((T - 1, shape.n_kv_heads, shape.head_dim)); Vd = np.zeros_like(Kd)
    O.draft_forward(shape, dw, emb, g_all[:T - 1], prompt[1:], np.arange(T - 1), Kd, Vd, 0, 0,
                    np.tril(np.ones((T - 1, T - 1), dtype=bool)), O.bf16_round)
    ctx = E.Eagle3Context(shape, max_batch=1, max_nodes=64, max_depth=4, max_topk=4, max_new=64, device=DEV)
    W = PL.device_weights(shape, device=DEV)
    ctx.set_weights(W["target"], W["draft"])
    cap = T + 16
    z = lambda: torch.zeros(cap, shape.n_kv_heads, shape.head_dim, dtype=torch.bfloat16, device=DEV)
    ks, vs = [z() for _ in range(shape.n_layers)], [z() for _ in range(shape.n_layers)]
    i32 = lambda v: torch.tensor(v, dtype=torch.int32, device=DEV)
    kv = E.KVCache(ks, vs, i32([0, cap]), i32([0]), 0)
    dkv = E.KVCache([z()], [z()], i32([0, cap]), i32([0]), 0)
    g_last, logits = E.eagle3_prefill(ctx, torch.as_tensor(prompt, dtype=torch.int32, device=DEV), kv, dkv)
    torch.cuda.synchronize()
    assert int(kv.prefix_len[0]) == T and int(dkv.prefix_len[0]) == T - 1
    for l in range(shape.n_layers):
        assert np.max(np.abs(ks[l][:T].float().cpu().numpy() - pre["k_new"][l])) < 4e-2, l      # one bf16 ulp at |k| < 8
        assert np.max(np.abs(vs[l][:T].float().cpu().numpy() - pre["v_new"][l])) < 2e-2, l
    assert np.max(np.abs(logits.cpu().numpy() - pre["logits"][-1])) < 2e-2
    assert np.max(np.abs(g_last.cpu().numpy() - g_all[-1])) < 2e-2
    assert np.max(np.abs(dkv.k_layers[0][:T - 1].float().cpu().numpy() - Kd)) < 4e-2
    assert np.max(np.abs(dkv.v_layers[0][:T - 1].float().cpu().numpy() - Vd)) < 2e-2
