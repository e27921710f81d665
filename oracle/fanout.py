"""The multi-consumer example of the paper's layout selection (Sec. 3.2.2, Fig. 4), as arithmetic.  TEST
INFRASTRUCTURE ONLY.

    T = A . W^T                    [D0, D1],  D0 = D2 * D3          (MatMul)
    U = reshape(transpose(T))      [D1, D2, D3]                      (Transpose, Reshape: the operators that get eliminated)
    reduce   = sum over D3 of U    [D1, D2]                          (Reduce,  reduction dimension D3)
    reduce_p = sum over D1 of U    [D2, D3]                          (Reduce', reduction dimension D1)
    conv     = U . Wc^T over D3    [D1, D2, Cout]                    (Conv with a full-width kernel along D3 = a contraction over D3)

Reading: the figure names the operators but not their arithmetic; Reduce is taken as a sum and the Conv as the
contraction over its reduction dimension, which is all the layout argument uses.  Every transformation is materialised.
"""
import numpy as np
from . import views as V
from . import ops as O


def fanout_graph(a, w, wc, D2, D3):
    D0, D1 = a.shape[0], w.shape[0]
    assert D0 == D2 * D3
    t = O.linear(a, w)                                              # [D0, D1]
    u = V.apply_chain(t, [("permute", (1, 0)), ("reshape", (D1, D2, D3))])
    return {"u": u, "reduce": u.sum(axis=2), "reduce_p": u.sum(axis=0), "conv": O.linear(u, wc)}
