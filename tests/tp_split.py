"""Test helper: cut an unsharded (t = 1) canonical parameter list into rank r of t.

Column-parallel tensors (q, k, v, fc1 and their biases) are cut along the
output dimension, row-parallel weights (o, fc2) along the input dimension,
the token embedding along the vocabulary; everything else is replicated.
Heads stay whole: rank r owns heads [r*H/t, (r+1)*H/t).
"""
import numpy as np


def split(full, layers, t, r):
    def rows(w):
        n = w.shape[0] // t
        return np.ascontiguousarray(w[r * n:(r + 1) * n])

    def cols(w):
        n = w.shape[1] // t
        return np.ascontiguousarray(w[:, r * n:(r + 1) * n])

    out = [rows(full[0]), full[1].copy()]
    for l in range(layers):
        (g1, b1, wq, bq, wk, bk, wv, bv, wo, bo, g2, b2, w1, c1, w2, c2) = full[2 + 16 * l: 18 + 16 * l]
        out += [g1.copy(), b1.copy(), rows(wq), rows(bq), rows(wk), rows(bk), rows(wv), rows(bv),
                cols(wo), bo.copy(), g2.copy(), b2.copy(), rows(w1), rows(c1), cols(w2), c2.copy()]
    out += [full[-2].copy(), full[-1].copy()]
    return out
