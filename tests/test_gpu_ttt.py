"""Training-time-test attention forward (Section 3.2) on the GPU against the oracle."""
import numpy as np
import pytest
import torch

import eagle3_synth as S
from oracle import eagle3_oracle as O

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(E, T, H, Hkv, d, s, dtype, seed):
    q = S.normal(S.SEED + seed, 1, (T, H, d), dtype=dtype)
    k = S.normal(S.SEED + seed, 2, (s + 1, T, Hkv, d), dtype=dtype)
    v = S.normal(S.SEED + seed, 3, (s + 1, T, Hkv, d), dtype=dtype)
    got = E.eagle3_ttt_attention(q.to(DEV), k.to(DEV), v.to(DEV)).cpu().numpy()
    ref = O.ttt_attention(O.as_f64(q), O.as_f64(k), O.as_f64(v), "mask")
    return float(np.max(np.abs(got - ref)))


def test_ttt_attention_matches_the_oracle():
    import paper_2503_01840_amd as E
    # fp32, exact kernels: native step, two simulated steps, one position only
    for i, (T, H, Hkv, d, s) in enumerate([(37, 4, 4, 64, 0), (50, 4, 2, 64, 2), (1, 2, 1, 32, 3)]):
        assert _case(E, T, H, Hkv, d, s, torch.float32, i) < 1e-5
    # bf16 storage, matrix-core kernel: sizes around the 64-query blocks and 32-key halves, grouped heads
    for i, (T, H, Hkv, s) in enumerate([(1, 2, 2, 0), (31, 2, 1, 1), (64, 4, 2, 0), (65, 4, 2, 2), (97, 4, 4, 3),
                                        (300, 8, 2, 2)]):
        err = _case(E, T, H, Hkv, 128, s, torch.bfloat16, 10 + i)
        assert err < 2e-3, (T, H, Hkv, s, err)       # inputs are exact on both sides; only fp32 vs fp64 arithmetic differs


def test_ttt_attention_at_a_training_shape():
    """2048 positions, 32 heads over 8 KV heads, third step: sampled rows against the oracle's explicit form."""
    import paper_2503_01840_amd as E
    T, H, Hkv, d, s = 2048, 32, 8, 128, 2
    q = S.normal(S.SEED, 1, (T, H, d), dtype=torch.bfloat16)
    k = S.normal(S.SEED, 2, (s + 1, T, Hkv, d), dtype=torch.bfloat16)
    v = S.normal(S.SEED, 3, (s + 1, T, Hkv, d), dtype=torch.bfloat16)
    got = E.eagle3_ttt_attention(q.to(DEV), k.to(DEV), v.to(DEV)).cpu().numpy()
    q64, K = O.as_f64(q), O.as_f64(k).reshape((s + 1) * T, Hkv, d)
    V = O.as_f64(v).reshape((s + 1) * T, Hkv, d)
    sets = O.ttt_visible_sets(T, s)
    for i in (0, 1, 63, 64, 1000, 2047):
        ref = O.attention_explicit_sets(q64[i:i + 1], K, V, [sets[i]])
        assert np.max(np.abs(got[i] - ref[0])) < 2e-3, i
    assert np.isfinite(got).all()
