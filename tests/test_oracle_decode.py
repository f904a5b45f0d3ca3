"""Pins of the multi-step pipeline of the oracle: greedy speculative decoding must reproduce ordinary greedy
decoding of the target token for token (Section 2.1: the method is lossless; Section 4 "Metrics": tau = tokens per
draft-verify cycle), whatever the draft proposes."""
import numpy as np
import pytest

import eagle3_synth as S
from oracle import eagle3_oracle as O
import pipeline as PL

SHAPE = S.get_shape("c1")


def planted_hook(reference, wanted):
    """Overwrites drafted tokens along one root-to-leaf chain of the draft's tree with the target's TRUE greedy
    continuation, to depth wanted[step] (the tree shape stays the draft's): the walk must then accept at least that
    many tokens.  `reference` = the target's greedy tokens after the prompt."""
    def hook(step, tree_tok, parent, depth, emitted):
        pos = len(emitted)                       # emitted[-1] is the root; reference[pos] is what follows it
        n = len(parent)
        height = [0] * n                         # longest chain below every node
        for c in range(n - 1, 0, -1):
            height[parent[c]] = max(height[parent[c]], height[c] + 1)
        cur = 0
        for lvl in range(wanted[step % len(wanted)]):
            kids = [c for c in range(n) if parent[c] == cur]
            if not kids or pos + lvl >= len(reference):
                break
            nxt = max(kids, key=lambda c: (height[c], -c))
            true_tok = reference[pos + lvl]
            for c in kids:                       # siblings must stay distinct
                if c != nxt and tree_tok[c] == true_tok:
                    tree_tok[c] = tree_tok[nxt]
            tree_tok[nxt] = true_tok
            cur = nxt
        return tree_tok
    return hook


@pytest.fixture(scope="module")
def setup():
    model = PL.OracleModel(SHAPE)
    prompt = S.uniform_ints(S.SEED, S.TensorIds.PREFIX_TOK, (12,), 0, SHAPE.vocab).numpy()
    ref = O.greedy_decode(SHAPE, model.layer, model.globals(), prompt, 40)
    return model, prompt, ref


def test_commit_path_orders_rows_and_tokens():
    tree_tok = np.array([10, 11, 12, 13, 14])
    parent = np.array([-1, 0, 0, 2, 3])
    taps = np.arange(3 * 5 * 2, dtype=np.float64).reshape(3, 5, 2)
    k_new = np.arange(2 * 5 * 1 * 2, dtype=np.float64).reshape(2, 5, 1, 2)
    k_keep, v_keep, taps_new, tok_new = O.commit_path(tree_tok, [0, 2, 3], 99, taps, k_new, -k_new)
    assert tok_new.tolist() == [12, 13, 99]
    assert np.array_equal(taps_new, taps[:, [0, 2, 3]])
    assert np.array_equal(k_keep, k_new[:, [0, 2, 3]]) and np.array_equal(v_keep, -k_new[:, [0, 2, 3]])


def test_greedy_speculative_decoding_equals_plain_greedy_decoding(setup):
    model, prompt, ref = setup
    D, K, N = SHAPE.depth, SHAPE.topk, SHAPE.n_nodes
    # (i) the draft's own trees (random weights: it almost never guesses right, tau ~ 1)
    out = O.speculative_decode(SHAPE, model.layer, model.globals(), model.draft(), prompt, 10, D, K, N)
    assert out["tokens"] == ref[:len(out["tokens"])]
    assert len(out["tokens"]) == 1 + sum(a + 1 for a in out["accept_lens"])
    # (ii) trees that contain the true continuation to depth 0..D, cycling: every depth of acceptance is exercised
    # (30 of the 36 drafted candidates are kept, so that the tree reaches depth D)
    wanted = [3, 0, 1, 2, 3, 1]
    out = O.speculative_decode(SHAPE, model.layer, model.globals(), model.draft(), prompt, 9, D, K, 30,
                               tree_hook=planted_hook(ref, wanted))
    assert out["tokens"] == ref[:len(out["tokens"])]
    assert all(a >= w for a, w in zip(out["accept_lens"], (wanted * 2)[:9]))
    assert max(out["accept_lens"]) == D and min(out["accept_lens"]) == 0
    assert out["tau"] == pytest.approx(np.mean(np.asarray(out["accept_lens"]) + 1))
    assert 1.0 <= out["tau"] <= D + 1


def test_a_wrong_commit_breaks_the_equality(setup):
    """Control: keeping the cache rows of the wrong nodes (node order instead of path order) must show up."""
    model, prompt, ref = setup
    D, K, N = SHAPE.depth, SHAPE.topk, SHAPE.n_nodes
    real = O.commit_path

    def wrong(tree_tok, path, bonus, taps, k_new, v_new):
        k_keep, v_keep, taps_new, tok_new = real(tree_tok, path, bonus, taps, k_new, v_new)
        idx = np.arange(len(path))                       # rows 0..n-1 instead of the path's rows
        return k_new[:, idx], v_new[:, idx], taps_new, tok_new
    O.commit_path = wrong
    try:
        out = O.speculative_decode(SHAPE, model.layer, model.globals(), model.draft(), prompt, 9, D, K, 30,
                                   tree_hook=planted_hook(ref, [3, 2, 3, 1]))
    finally:
        O.commit_path = real
    assert out["tokens"] != ref[:len(out["tokens"])]
