"""The allocation-free acceptance entry point (fixed scratch inside the library) against eagle3_accept, through the
C ABI: two calls in a row, the second with a smaller input, greedy and stochastic."""
import numpy as np
import pytest
import torch

import eagle3_synth as S

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(E, ctx, B, N, V, seed):
    rs = np.random.RandomState(seed)
    parents = np.stack([S.random_tree(S.SEED, seed * 100 + b, N, 6, 4)[0] for b in range(B)])
    toks = S.uniform_ints(S.SEED + seed, S.TensorIds.TREE_TOK, (B, N), 0, V).numpy()
    logits = rs.randn(B, N, V).astype(np.float32)
    for b in range(B):                          # children carry real mass, so walks go several levels deep
        for c in range(1, N):
            logits[b, parents[b, c], toks[b, c]] += rs.uniform(5.0, 11.0)
    lg = torch.from_numpy(logits).to(DEV)
    tt = torch.as_tensor(toks, dtype=torch.int32, device=DEV)
    pp = torch.as_tensor(parents, dtype=torch.int32, device=DEV)
    U = S.uniform01(S.SEED + seed, S.TensorIds.UNIFORMS, (B, 2 * N)).to(DEV)
    depths = []
    for temp, u in ((0.0, None), (1.0, U), (0.6, U)):
        want = E.eagle3_accept(ctx, lg, tt, pp, temp, u)
        got = E.eagle3_accept_static(lg, tt, pp, temp, u)
        torch.cuda.synchronize()
        for w, g in zip(want, got):
            assert torch.equal(w, g), (B, N, V, temp)
        depths.append(int(want[0].max()))
    return depths


def test_accept_static_matches_accept_on_two_calls_in_a_row():
    import paper_2503_01840_amd as E
    shape = S.get_shape("c2")
    ctx = E.Eagle3Context(shape, max_batch=8, max_nodes=64, max_depth=8, max_topk=10, max_new=8, device=DEV)
    d1 = _case(E, ctx, 8, 60, shape.vocab, 1)          # 480 rows x 63 chunks
    d2 = _case(E, ctx, 2, 9, shape.vocab, 2)           # smaller: stale statistics of the first call stay in the array
    assert max(d1) >= 1 and max(d2) >= 1
    small = shape.with_(vocab=1000)                     # one ragged chunk
    ctx2 = E.Eagle3Context(small, max_batch=1, max_nodes=64, max_depth=8, max_topk=10, max_new=8, device=DEV)
    _case(E, ctx2, 1, 5, 1000, 3)


def test_accept_static_rejects_sizes_beyond_its_scratch():
    import paper_2503_01840_amd as E
    z = torch.zeros(1, dtype=torch.int32, device=DEV)
    f = torch.zeros(1, dtype=torch.float32, device=DEV)
    L = E.lib()
    args = (f.data_ptr(), z.data_ptr(), z.data_ptr(), 0.0, None, z.data_ptr(), z.data_ptr(), z.data_ptr(), None)
    assert L.eagle3_accept_static(64, 64, 128256, *args) == -2        # 4096 rows x 63 chunks > 65536
    assert L.eagle3_accept_static(1, 65, 1024, *args) == -2
    assert L.eagle3_accept_static(1, 4, 1024, None, *args[1:]) == -1
