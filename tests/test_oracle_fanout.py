"""Pins for oracle.fanout (the Fig. 4 graph as arithmetic): torch CPU re-assembly, element-wise definition on a tiny
case, and the identities that tie the three consumers together."""
import numpy as np
import torch
from oracle import fanout


def test_fanout_graph_definition_and_identities():
    rng = np.random.default_rng(0)
    D1, D2, D3, K, Co = 5, 3, 4, 7, 2
    a, w, wc = rng.standard_normal((D2 * D3, K)), rng.standard_normal((D1, K)), rng.standard_normal((Co, D3))
    r = fanout.fanout_graph(a, w, wc, D2, D3)
    for i in range(D1):                       # u[i, j, l] = sum_k a[j * D3 + l, k] w[i, k]
        for j in range(D2):
            for l in range(D3):
                assert abs(r["u"][i, j, l] - sum(a[j * D3 + l, k] * w[i, k] for k in range(K))) < 1e-12
    t = torch.from_numpy(a) @ torch.from_numpy(w).T
    u = t.T.reshape(D1, D2, D3)
    assert np.allclose(r["reduce"], u.sum(2).numpy()) and np.allclose(r["reduce_p"], u.sum(0).numpy())
    assert np.allclose(r["conv"], torch.nn.functional.linear(u, torch.from_numpy(wc)).numpy())
    # both reductions sum to the same total; a conv kernel of ones is the Reduce
    assert abs(r["reduce"].sum() - r["reduce_p"].sum()) < 1e-9
    ones = fanout.fanout_graph(a, w, np.ones((1, D3)), D2, D3)
    assert np.allclose(ones["conv"][..., 0], r["reduce"])
