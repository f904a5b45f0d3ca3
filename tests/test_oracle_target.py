"""Pins for the oracle's target stack and tree attention (CPU only).

The pins are things the oracle does not define itself: the `transformers` LLaMA
implementation (also through its 4-D mask path, which makes it a tree-attention
implementation), closed forms of the rotary embedding, torch's bfloat16 cast, and the
two invariants the benchmark definition names: chain tree == causal decoding and
mask form == explicit-ancestor-path brute force.
"""
import numpy as np
import pytest
import torch

import eagle3_synth as S
from oracle import eagle3_oracle as O
from hf_llama import hf_forward, hf_model

TINY = S.get_shape("c1")
# The library computes its rotary cos/sin tables in fp32 whatever the model dtype, so agreement with
# the fp64 oracle stops at ~1e-7; a dropped term, wrong sign, index or transposition is >= 1e-3.
HF_ATOL = 2e-6
GQA = TINY.with_(name="gqa", n_kv_heads=2, hidden=128, intermediate=176, n_layers=3, taps=(0, 1, 2), vocab=512,
                 draft_vocab=512)


def _weights(shape, seed=S.SEED):
    layers = [S.layer_weights(shape, l, seed) for l in range(shape.n_layers)]
    tg = S.target_globals(shape, seed)
    return layers, tg, [O.weights_f64(W) for W in layers], O.weights_f64(tg)


def _prefill_and_tree(shape, parent, n_prefix, seed_salt=0):
    layers, tg, L64, tg64 = _weights(shape)
    toks = S.uniform_ints(S.SEED + seed_salt, S.TensorIds.PREFIX_TOK, (n_prefix + len(parent),), 0, shape.vocab).numpy()
    pre = O.prefill(shape, lambda l: L64[l], tg64, toks[:n_prefix])
    out = O.tree_verify(shape, lambda l: L64[l], tg64, toks[n_prefix:], parent,
                        lambda l: (pre["k_new"][l], pre["v_new"][l]), keep_hidden=True)
    return layers, tg, L64, tg64, toks, pre, out


@pytest.mark.parametrize("shape", [TINY, GQA], ids=lambda s: s.name)
def test_chain_tree_equals_causal_decoding_of_library_llama(shape):
    """A single-chain tree verified against a KV cache == the library's causal forward over prefix++chain."""
    n_prefix, n_chain = 24, 8
    parent, _ = S.chain_tree(n_chain)
    layers, tg, L64, tg64, toks, pre, out = _prefill_and_tree(shape, parent, n_prefix)
    logits, hid = hf_forward(hf_model(shape, layers, tg), toks)
    np.testing.assert_allclose(out["logits"], logits[n_prefix:], atol=HF_ATOL, rtol=0)
    np.testing.assert_allclose(pre["logits"], logits[:n_prefix], atol=HF_ATOL, rtol=0)
    for t, l in enumerate(shape.taps):       # feature of layer l = that layer's residual-stream output
        np.testing.assert_allclose(out["taps"][t], hid[l][n_prefix:], atol=HF_ATOL, rtol=0)
    for l in range(shape.n_layers):
        np.testing.assert_allclose(out["hidden"][l + 1], hid[l][n_prefix:], atol=HF_ATOL, rtol=0)


@pytest.mark.parametrize("shape", [TINY, GQA], ids=lambda s: s.name)
@pytest.mark.parametrize("salt", [0, 1])
def test_tree_attention_equals_library_4d_mask(shape, salt):
    """Random 16-node tree: node i at position P+depth(i) seeing prefix + ancestors + itself,
    against the library run with an explicit [T,T] mask and position ids."""
    n_prefix = 20
    parent, depth = S.random_tree(S.SEED, salt, 16, 3, 4)
    layers, tg, L64, tg64, toks, pre, out = _prefill_and_tree(shape, parent, n_prefix, salt)
    N, T = len(parent), n_prefix + len(parent)
    mask = np.zeros((T, T), dtype=bool)
    mask[:n_prefix, :n_prefix] = np.tril(np.ones((n_prefix, n_prefix), dtype=bool))
    mask[n_prefix:, :n_prefix] = True
    for i in range(N):
        cur = i
        while cur >= 0:
            mask[n_prefix + i, n_prefix + cur] = True
            cur = parent[cur]
    pos = np.concatenate([np.arange(n_prefix), n_prefix + depth])
    logits, hid = hf_forward(hf_model(shape, layers, tg), toks, mask, pos)
    np.testing.assert_allclose(out["logits"], logits[n_prefix:], atol=HF_ATOL, rtol=0)
    np.testing.assert_allclose(out["taps"][2], hid[shape.taps[2]][n_prefix:], atol=HF_ATOL, rtol=0)


def _trees_under_test():
    trees = [S.random_tree(S.SEED, s, n, d, c) for s, (n, d, c) in
             enumerate([(16, 3, 4), (16, 3, 4), (12, 5, 2), (16, 15, 1), (9, 2, 8), (2, 1, 1), (1, 0, 1)])]
    trees.append(S.chain_tree(16))
    trees.append((np.array([-1] + [0] * 15, dtype=np.int32), np.array([0] + [1] * 15, dtype=np.int32)))   # star
    return trees


def test_mask_form_equals_explicit_ancestor_paths_every_node():
    """Every node's attention == plain attention over prefix ++ its explicit root->node path."""
    shape = GQA
    rs = np.random.RandomState(7)
    P, H, Hkv, d = 11, shape.n_heads, shape.n_kv_heads, shape.head_dim
    for parent, _ in _trees_under_test():
        N = len(parent)
        q = rs.randn(N, H, d)
        K, V = rs.randn(P + N, Hkv, d), rs.randn(P + N, Hkv, d)
        a = O.attention_prefix_tail(q, K, V, P, O.ancestor_mask(parent))
        paths = O.ancestor_paths(parent)
        b = O.attention_explicit_sets(q, K, V, [list(range(P)) + [P + j for j in paths[i]] for i in range(N)])
        np.testing.assert_allclose(a, b, atol=1e-12, rtol=0)
        # and against torch's library attention, one node at a time
        for i in range(N):
            idx = list(range(P)) + [P + j for j in paths[i]]
            for h in range(H):
                g = h * Hkv // H
                ref = torch.nn.functional.scaled_dot_product_attention(
                    torch.from_numpy(q[i, h])[None, None], torch.from_numpy(K[idx, g])[None],
                    torch.from_numpy(V[idx, g])[None])[0, 0].numpy()
                np.testing.assert_allclose(a[i, h], ref, atol=1e-12, rtol=0)


def test_whole_layer_stack_mask_equals_paths():
    shape = GQA
    parent, _ = S.random_tree(S.SEED, 3, 12, 4, 3)
    layers, tg, L64, tg64, toks, pre, out = _prefill_and_tree(shape, parent, 9)
    out2 = O.tree_verify(shape, lambda l: L64[l], tg64, toks[9:], parent,
                         lambda l: (pre["k_new"][l], pre["v_new"][l]), attention="paths")
    np.testing.assert_allclose(out["logits"], out2["logits"], atol=1e-10, rtol=0)


def test_node_output_equals_verifying_its_own_root_path_as_a_chain():
    """Per-node invariant at the model level: logits of node i == last logits of the chain root..i."""
    shape = GQA
    parent, _ = S.random_tree(S.SEED, 5, 10, 4, 3)
    layers, tg, L64, tg64, toks, pre, out = _prefill_and_tree(shape, parent, 9)
    kv = lambda l: (pre["k_new"][l], pre["v_new"][l])
    for i, path in enumerate(O.ancestor_paths(parent)):
        cp, _ = S.chain_tree(len(path))
        oc = O.tree_verify(shape, lambda l: L64[l], tg64, toks[9:][path], cp, kv)
        np.testing.assert_allclose(out["logits"][i], oc["logits"][-1], atol=1e-10, rtol=0)


def test_sibling_order_does_not_change_any_node():
    shape = GQA
    parent = np.array([-1, 0, 0, 0, 1, 1, 2, 3], dtype=np.int32)
    perm = np.array([0, 3, 1, 2, 7, 5, 4, 6])          # new order -> old node id (still creation order)
    inv = np.argsort(perm)
    parent2 = np.array([-1 if parent[o] < 0 else inv[parent[o]] for o in perm], dtype=np.int32)
    assert all(parent2[i] < i for i in range(1, 8))
    layers, tg, L64, tg64, toks, pre, out = _prefill_and_tree(shape, parent, 9)
    out2 = O.tree_verify(shape, lambda l: L64[l], tg64, toks[9:][perm], parent2,
                         lambda l: (pre["k_new"][l], pre["v_new"][l]))
    np.testing.assert_allclose(out2["logits"], out["logits"][perm], atol=1e-10, rtol=0)


def test_rope_closed_forms():
    rs = np.random.RandomState(0)
    # d = 2: one complex pair rotating by `pos` radians (frequency theta^0 = 1)
    got = O.rope(np.array([[[1.0, 0.0]], [[0.0, 1.0]]]), np.array([0.5, 0.5]), 1e4)
    np.testing.assert_allclose(got[0, 0], [np.cos(0.5), np.sin(0.5)], atol=1e-15)
    np.testing.assert_allclose(got[1, 0], [-np.sin(0.5), np.cos(0.5)], atol=1e-15)
    x = rs.randn(5, 3, 64)
    np.testing.assert_allclose(O.rope(x, np.zeros(5), 1e4), x, atol=0)                 # position 0 is identity
    pos = np.array([3, 17, 100, 4096, 16390])
    np.testing.assert_allclose(np.linalg.norm(O.rope(x, pos, 5e5), axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)
    # complex form: pair (x_i, x_{i+d/2}) times exp(j * pos * theta^(-2i/d))
    z = (x[..., :32] + 1j * x[..., 32:]) * np.exp(1j * pos[:, None, None] * (5e5 ** (-np.arange(32) / 32.0)))
    np.testing.assert_allclose(O.rope(x, pos, 5e5), np.concatenate([z.real, z.imag], -1), atol=1e-9)
    # scores depend only on the position difference
    q, k = rs.randn(1, 1, 64), rs.randn(1, 1, 64)
    s = lambda m, n: float(np.sum(O.rope(q, [m], 1e4) * O.rope(k, [n], 1e4)))
    assert abs(s(10, 3) - s(107, 100)) < 1e-9 and abs(s(10, 3) - s(11, 3)) > 1e-6


def test_rmsnorm_softmax_silu_against_torch():
    rs = np.random.RandomState(1)
    x, w = rs.randn(4, 32) * 3, 1 + 0.1 * rs.randn(32)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (32,), torch.from_numpy(w), 1e-5).numpy()
    np.testing.assert_allclose(O.rmsnorm(x, w, 1e-5), ref, rtol=1e-12)
    np.testing.assert_allclose(O.softmax(x), torch.softmax(torch.from_numpy(x), -1).numpy(), rtol=1e-12)
    np.testing.assert_allclose(O.log_softmax(x), torch.log_softmax(torch.from_numpy(x), -1).numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(O.silu(x), torch.nn.functional.silu(torch.from_numpy(x)).numpy(), rtol=1e-12)


def test_bf16_rounding_is_torch_bfloat16_cast():
    rs = np.random.RandomState(2)
    x = np.concatenate([rs.randn(4096) * 10.0 ** rs.randint(-6, 6, 4096), [0.0, 1.0, -1.0, 1.00390625, 1.01171875]])
    ref = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).double().numpy()
    np.testing.assert_array_equal(O.bf16_round(x), ref)


def test_bf16_mode_stays_within_the_stated_budget_of_fp64_on_tiny_bf16_model():
    """Quantifies the rounding budget: bf16-boundary mode vs exact, same bf16 weights."""
    shape = GQA.with_(dtype="bf16")
    parent, _ = S.random_tree(S.SEED, 1, 16, 3, 4)
    layers = [O.weights_f64(S.layer_weights(shape, l)) for l in range(shape.n_layers)]
    tg = O.weights_f64(S.target_globals(shape))
    K, V = S.kv_layer(shape, 0, 40)
    kv = lambda l: (O.as_f64(K), O.as_f64(V))
    toks = S.uniform_ints(S.SEED, S.TensorIds.TREE_TOK, (16,), 0, shape.vocab).numpy()
    a = O.tree_verify(shape, lambda l: layers[l], tg, toks, parent, kv, rounding="none")
    b = O.tree_verify(shape, lambda l: layers[l], tg, toks, parent, kv, rounding="bf16")
    assert 0 < np.max(np.abs(a["logits"] - b["logits"])) < 2e-2


def _library_forward_rounding_operands(shape, layers, tg, toks, mask=None, pos=None):
    """The library model with torch's bfloat16 cast applied to every operand of a weight product (the input of every
    Linear) and to the three attention operands (rotated queries and keys, values): built from hooks on the library's
    own modules, it shares nothing with the oracle's layer code."""
    import transformers.models.llama.modeling_llama as ML
    cast = lambda t: t.float().bfloat16().double()
    model = hf_model(shape, layers, tg)
    hooks = []
    for mod in model.modules():
        if isinstance(mod, torch.nn.Linear):
            hooks.append(mod.register_forward_pre_hook(lambda m, args: (cast(args[0]),) + tuple(args[1:])))
    for lyr in model.model.layers:
        hooks.append(lyr.self_attn.v_proj.register_forward_hook(lambda m, a, out: cast(out)))
    rotary = ML.apply_rotary_pos_emb

    def rounded_rotary(*a, **kw):
        q, k = rotary(*a, **kw)
        return cast(q), cast(k)
    ML.apply_rotary_pos_emb = rounded_rotary
    try:
        return hf_forward(model, toks, mask, pos)
    finally:
        ML.apply_rotary_pos_emb = rotary
        for h in hooks:
            h.remove()


def test_bf16_rounding_points_are_the_operands_of_every_product():
    """Pins WHERE the oracle's bf16 mode rounds: at the operands of every weight product and of attention (queries
    and keys after the rotation, values), nowhere else: residual stream, norm arithmetic, scores and softmax weights
    stay unrounded.  Reference: the library model with torch's cast hooked onto exactly those operands.  Both sides
    are fp64 except the library's fp32 softmax and rotary tables (1e-7), which can move a value across a bf16 rounding
    boundary now and then; such a flip changes one operand entry by one unit in the last place, while a rounding
    point that is missing, extra or misplaced changes every entry of a tensor: the control below shows the gap."""
    shape = GQA.with_(dtype="bf16")
    layers = [S.layer_weights(shape, l) for l in range(shape.n_layers)]
    tg = S.target_globals(shape)
    L64, tg64 = [O.weights_f64(W) for W in layers], O.weights_f64(tg)
    empty = np.zeros((0, shape.n_kv_heads, shape.head_dim))
    n_prefix = 12
    parent, depth = S.random_tree(S.SEED, 5, 20, 4, 3)
    N, T = len(parent), n_prefix + len(parent)
    # the prefix as a chain in front of the tree: one tree of T nodes over an empty cache
    full_parent = np.concatenate([np.arange(-1, n_prefix - 1), [n_prefix - 1 if p < 0 else n_prefix + p for p in parent]])
    toks = S.uniform_ints(S.SEED + 9, S.TensorIds.PREFIX_TOK, (T,), 0, shape.vocab).numpy()
    mask = O.ancestor_mask(full_parent)
    pos = O.tree_depth(full_parent)
    logits, hid = _library_forward_rounding_operands(shape, layers, tg, toks, mask, pos)

    def run(rounding):
        return O.tree_verify(shape, lambda l: L64[l], tg64, toks, full_parent, lambda l: (empty, empty),
                             rounding=rounding, keep_hidden=True)
    out = run("bf16")
    scale = np.sqrt(np.mean(logits ** 2))
    err = np.max(np.abs(out["logits"] - logits))
    assert err < 2e-4 * scale, (err, scale)
    for l in range(shape.n_layers):
        s = np.sqrt(np.mean(hid[l] ** 2))
        assert np.max(np.abs(out["hidden"][l + 1] - hid[l])) < 2e-4 * s, l
    # control: the same oracle with any ONE of its rounding points left out is off by far more than that
    n_calls = [0]

    def counting(a):
        n_calls[0] += 1
        return O.bf16_round(a)
    run(counting)
    total = n_calls[0]
    assert total == 7 * shape.n_layers + 1                     # per layer: n1, q, k, v, attention output, n2, gate * up; final norm
    worst = np.inf
    for skip in range(total):
        i = [0]

        def leave_one_out(a):
            i[0] += 1
            return a if i[0] - 1 == skip else O.bf16_round(a)
        worst = min(worst, np.max(np.abs(run(leave_one_out)["logits"] - logits)))
    assert worst > 10 * max(err, 1e-6), (worst, err)
    print(f"rounding-point pin: max logit error {err:.2e} (logit RMS {scale:.2f}), smallest leave-one-out error {worst:.2e}")
