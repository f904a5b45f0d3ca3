"""Pins of the training-time-test attention of the oracle (Section 3.2, Figure 6)."""
import numpy as np
import torch

from oracle import eagle3_oracle as O


def _rand(rs, *shape):
    return rs.standard_normal(shape)


def test_native_step_is_ordinary_causal_attention():
    rs = np.random.RandomState(0)
    T, H, Hkv, d = 37, 4, 2, 16
    q, K, V = _rand(rs, T, H, d), _rand(rs, 1, T, Hkv, d), _rand(rs, 1, T, Hkv, d)
    got = O.ttt_attention(q, K, V)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(K[0]).permute(1, 0, 2).repeat_interleave(H // Hkv, 0)[None]
    tv = torch.from_numpy(V[0]).permute(1, 0, 2).repeat_interleave(H // Hkv, 0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.max(np.abs(got - ref)) < 1e-12


def test_mask_form_equals_explicit_sets_and_the_masks_are_diagonal():
    rs = np.random.RandomState(1)
    T, H, Hkv, d, s = 19, 4, 4, 8, 3
    q, K, V = _rand(rs, T, H, d), _rand(rs, s + 1, T, Hkv, d), _rand(rs, s + 1, T, Hkv, d)
    assert np.max(np.abs(O.ttt_attention(q, K, V, "sets") - O.ttt_attention(q, K, V, "mask"))) < 1e-12
    sets = O.ttt_visible_sets(T, s)
    for i in range(T):
        assert sets[i][:i + 1] == list(range(i + 1))                       # lower triangular over the original data
        assert sets[i][i + 1:] == [t * T + i for t in range(1, s + 1)]     # one key per simulated step: the diagonal
    # a key of a simulated step never reaches another position: perturbing K^2 at position 5 moves only row 5
    K2 = K.copy(); K2[2, 5] += 1.0
    diff = np.abs(O.ttt_attention(q, K2, V) - O.ttt_attention(q, K, V)).max(axis=(1, 2))
    assert diff[5] > 1e-6 and np.all(np.delete(diff, 5) == 0)


def test_a_training_time_test_row_sees_what_the_draft_sees_at_inference():
    """Row i of simulated step s must see exactly what the draft's forward s + 1 sees at inference for the prefix
    0..i: the context and its own chain of s drafted positions (the training step simulates the testing process)."""
    rs = np.random.RandomState(2)
    T, H, Hkv, d, s = 11, 2, 1, 8, 2
    q, K, V = _rand(rs, T, H, d), _rand(rs, s + 1, T, Hkv, d), _rand(rs, s + 1, T, Hkv, d)
    got = O.ttt_attention(q, K, V)
    for i in range(T):
        Kc = np.concatenate([K[0, :i + 1], K[1:, i]], axis=0)               # context, then the chain's own keys
        Vc = np.concatenate([V[0, :i + 1], V[1:, i]], axis=0)
        ref = O.attention_prefix_tail(q[i:i + 1], Kc, Vc, i + 1, np.ones((1, s), dtype=bool))
        assert np.max(np.abs(got[i] - ref[0])) < 1e-12
