"""Pins for the oracle's acceptance walks (CPU only): greedy never departs from target argmax
decoding; the stochastic walk preserves the target distribution (Section 2.1; Section 4 "Metrics":
strict speculative sampling, no loss)."""
import numpy as np
import pytest
from scipy import stats

import eagle3_synth as S
from oracle import eagle3_oracle as O
from hf_llama import hf_forward, hf_model

TINY = S.get_shape("c1")


def _target(shape):
    layers = [S.layer_weights(shape, l) for l in range(shape.n_layers)]
    tg = S.target_globals(shape)
    return layers, tg, [O.weights_f64(W) for W in layers], O.weights_f64(tg)


def test_greedy_walk_reproduces_target_argmax_decoding():
    """Trees that contain the true greedy continuation down to depth a are accepted to exactly depth a,
    and the emitted tokens are the autoregressive argmax tokens of the library model."""
    shape = TINY
    D, P = 3, 24
    layers, tg, L64, tg64 = _target(shape)
    prefix = S.uniform_ints(S.SEED, S.TensorIds.PREFIX_TOK, (P,), 0, shape.vocab).numpy()
    model = hf_model(shape, layers, tg)
    seq = list(prefix)
    for _ in range(D + 2):                       # library autoregressive greedy decoding
        logits, _ = hf_forward(model, np.array(seq))
        seq.append(int(np.argmax(logits[-1])))
    greedy = seq[P:]                             # greedy[0] is the root token, greedy[1:] its continuation
    pre = O.prefill(shape, lambda l: L64[l], tg64, prefix)
    kv = lambda l: (pre["k_new"][l], pre["v_new"][l])
    rs = np.random.RandomState(0)
    for a in range(D + 1):
        # chain of true tokens to depth a, then a wrong token; plus wrong siblings everywhere
        tok, par = [greedy[0]], [-1]
        cur = 0
        for lvl in range(1, D + 1):
            right = greedy[lvl] if lvl <= a else (greedy[lvl] + 1) % shape.vocab
            sibs = [(greedy[lvl] + 7 + s) % shape.vocab for s in range(2)]
            first = len(tok)
            for t in ([sibs[0], right, sibs[1]]):
                tok.append(t); par.append(cur)
            cur = first + 1
        # children must be in creation order by level: they are (each level appended after its parent)
        out = O.tree_verify(shape, lambda l: L64[l], tg64, np.array(tok), np.array(par), kv)
        n_acc, path, bonus = O.accept_greedy(out["logits"], tok, par)
        assert n_acc == a
        emitted = [tok[i] for i in path[1:]] + [bonus]
        assert emitted == greedy[1:a + 2]
        assert path[0] == 0 and all(par[path[i + 1]] == path[i] for i in range(n_acc))


def test_greedy_walk_planted_paths_and_tie_break():
    rs = np.random.RandomState(1)
    parent, depth = S.random_tree(S.SEED, 4, 16, 3, 4)
    N, V = len(parent), 50
    tok = np.arange(100, 100 + N) % V
    for target_node in range(N):
        logits = rs.randn(N, V)
        path = O.ancestor_paths(parent)[target_node]
        for u, c in zip(path[:-1], path[1:]):
            logits[u, tok[c]] += 20.0
        stop_tok = next(t for t in range(V) if t not in {tok[c] for c in range(N) if parent[c] == target_node})
        logits[target_node, stop_tok] += 20.0
        n_acc, p, bonus = O.accept_greedy(logits, tok, parent)
        assert (n_acc, p, bonus) == (len(path) - 1, path, stop_tok)
    logits = np.zeros((N, V))                    # all equal: argmax is the smallest token id, 0
    n_acc, p, bonus = O.accept_greedy(logits, np.arange(1, N + 1), parent)
    assert (n_acc, bonus) == (0, 0)


def _hand_tree():
    #        0
    #      / | \
    #     1  2  3        tokens 5, 2, 6
    #    / \    |
    #   4   5   6        tokens 1, 7 | 3
    parent = np.array([-1, 0, 0, 0, 1, 1, 3])
    tok = np.array([0, 5, 2, 6, 1, 7, 3])
    return parent, tok


def test_stochastic_walk_preserves_target_distribution_chi_square():
    parent, tok = _hand_tree()
    V, N, trials = 8, 7, 60000
    rs = np.random.RandomState(11)
    logits = rs.randn(N, V) * 1.5
    T = 1.0
    p = O.softmax(logits / T)
    U = S.uniform01(S.SEED, S.TensorIds.UNIFORMS, (trials, 2 * N)).numpy().astype(np.float64)
    first = np.zeros(V)
    second = {1: np.zeros(V), 3: np.zeros(V)}
    lens = np.zeros(4)
    for t in range(trials):
        n_acc, path, bonus, _ = O.accept_stochastic(logits, tok, parent, T, U[t])
        emitted = [tok[i] for i in path[1:]] + [bonus]
        first[emitted[0]] += 1
        lens[n_acc] += 1
        if len(path) > 1 and path[1] in second:
            second[path[1]][emitted[1]] += 1
    # first emitted token ~ p_root exactly (closed form: accept child c w.p. p[t_c]; residual otherwise)
    assert stats.chisquare(first, p[0] * trials).pvalue > 1e-3
    # conditional on having descended into an inner node, the next token ~ that node's distribution
    for node, cnt in second.items():
        assert cnt.sum() > 1000
        assert stats.chisquare(cnt, p[node] * cnt.sum()).pvalue > 1e-3
    # P(accept_len >= 1) = total target mass on the root's children
    exp_len0 = 1.0 - p[0, tok[[1, 2, 3]]].sum()
    assert abs(lens[0] / trials - exp_len0) < 4 * np.sqrt(exp_len0 * (1 - exp_len0) / trials)


def test_stochastic_walk_with_a_wrong_rule_fails_the_same_chi_square():
    """The test above has teeth: accepting with the draft-style ratio min(1, p/p_hat) for a
    deterministically proposed child (p_hat = 0.5, say) distorts the distribution and is caught."""
    parent, tok = np.array([-1, 0]), np.array([0, 3])
    V, trials = 8, 40000
    logits = np.log(np.array([0.05, 0.05, 0.1, 0.2, 0.1, 0.2, 0.2, 0.1]))[None].repeat(2, 0)
    p = O.softmax(logits)
    rs = np.random.RandomState(3)
    cnt = np.zeros(V)
    for _ in range(trials):
        r1, r2 = rs.rand(2)
        if r1 < min(1.0, p[0, 3] / 0.5):
            cnt[3] += 1
        else:
            res = np.maximum(p[0] - np.eye(V)[3] * 0.5, 0); res /= res.sum()
            cnt[np.searchsorted(np.cumsum(res), r2)] += 1
    assert stats.chisquare(cnt, p[0] * trials).pvalue < 1e-6
    U = rs.rand(trials, 4)
    good = np.zeros(V)
    for t in range(trials):
        n_acc, path, bonus, _ = O.accept_stochastic(logits, tok, parent, 1.0, U[t])
        good[([tok[i] for i in path[1:]] + [bonus])[0]] += 1
    assert stats.chisquare(good, p[0] * trials).pvalue > 1e-3


def test_stochastic_walk_low_temperature_is_the_greedy_walk_and_bonus_is_inverse_cdf():
    parent, tok = _hand_tree()
    rs = np.random.RandomState(5)
    logits = rs.randn(7, 8) * 2
    logits[0, 5] += 10; logits[1, 7] += 10; logits[5, 4] += 10
    g = O.accept_greedy(logits, tok, parent)
    for t in range(20):
        s = O.accept_stochastic(logits, tok, parent, 1e-3, rs.rand(14))
        assert s[:3] == g
    # leaf / no child accepted: the bonus is the inverse CDF of the residual in vocabulary order
    p = O.softmax(logits[4])
    for r in (0.0, 0.3, 0.77, 0.999999):
        U = np.zeros(14); U[2 * 1] = 0.0; U[2 * 4] = 0.0; U[2 * 4 + 1] = r
        lg = logits.copy(); lg[0, 5] += 50; lg[1, 1] += 50          # force the walk 0 -> 1 -> 4 (a leaf)
        n_acc, path, bonus, _ = O.accept_stochastic(lg, tok, parent, 1.0, U)
        assert path == [0, 1, 4] and bonus == int(np.searchsorted(np.cumsum(p), r, side="left"))


def test_rejected_sibling_mass_is_removed_from_later_tests_and_from_the_bonus():
    parent, tok = np.array([-1, 0, 0]), np.array([0, 1, 2])
    logits = np.log(np.array([[0.1, 0.5, 0.2, 0.2]] * 3))
    # child 1 (p=.5) rejected with r=.6; child 2 then has threshold .2/(1-.5)=.4
    U = np.array([0, 0.5, 0.6, 0, 0.39, 0])
    assert O.accept_stochastic(logits, tok, parent, 1.0, U)[1] == [0, 2]
    U[4] = 0.41           # both rejected: residual = {0: .1, 3: .2} / .3 ; r=.5 -> target .15 -> token 3
    n_acc, path, bonus, _ = O.accept_stochastic(logits, tok, parent, 1.0, U)
    assert (n_acc, path, bonus) == (0, [0], 3)
    U[1] = 0.3            # target .09 <= .1 -> token 0
    assert O.accept_stochastic(logits, tok, parent, 1.0, U)[2] == 0


def test_bonus_admissibility_window():
    parent, tok = np.array([-1, 0]), np.array([0, 2])
    logits = np.log(np.array([[0.1, 0.2, 0.3, 0.4]] * 2))
    U = np.array([0, 0.5, 0.99, 0])          # child (p=.3) rejected; residual {.1,.2,0,.4}/.7 ; target = .5*.7 = .35
    n_acc, path, bonus, margin, info = O.accept_stochastic(logits, tok, parent, 1.0, U, return_info=True)
    assert (n_acc, bonus) == (0, 3) and abs(info["target"] - 0.35) < 1e-12
    assert O.bonus_admissible(info, 3, 0.0) and not O.bonus_admissible(info, 1, 0.0)
    assert O.bonus_admissible(info, 1, 0.06) and not O.bonus_admissible(info, 0, 0.06)    # .30 + .06 >= .35 ; .10 + .06 < .35
    assert not O.bonus_admissible(info, 2, 1.0)                                           # a struck token never is
