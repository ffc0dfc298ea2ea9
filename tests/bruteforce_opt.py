"""Index-by-index float64 evaluation of one OPT tensor-parallel rank.

Pure Python lists and loops: no numpy arithmetic, no BLAS, no code shared with
the oracle.  Only usable at toy sizes.  Every sum is written over its indices
exactly as the definition reads.
"""
import math


def _ln(row, g, b):
    n = len(row)
    mu = sum(row) / n
    var = sum((v - mu) ** 2 for v in row) / n
    inv = 1.0 / math.sqrt(var + 1e-5)
    return [(row[i] - mu) * inv * g[i] + b[i] for i in range(n)]


def _linear(row, w, bias):
    # w is [out][in]
    return [sum(row[j] * w[o][j] for j in range(len(row))) + (bias[o] if bias is not None else 0.0)
            for o in range(len(w))]


def forward(params, ids, layers, heads, tp, rank, allreduce=None):
    """params: list of nested float lists in canonical order; ids: [b][s] ints.

    Returns logits [b][s][V/t].  `allreduce`, if given, maps a per-token vector
    (list of floats) to the hooked vector; identity when None.
    """
    hook = allreduce or (lambda v: v)
    tok, pos = params[0], params[1]
    vl, h = len(tok), len(tok[0])
    lo = rank * vl
    lh = heads // tp
    b, s = len(ids), len(ids[0])
    out = []
    for bi in range(b):
        x = []
        for p in range(s):
            t = ids[bi][p]
            row = list(tok[t - lo]) if lo <= t < lo + vl else [0.0] * h
            row = hook(row)
            x.append([row[c] + pos[p + 2][c] for c in range(h)])
        for l in range(layers):
            (g1, b1, wq, bq, wk, bk, wv, bv, wo, bo, g2, b2, w1, c1, w2, c2) = \
                params[2 + 16 * l: 2 + 16 * (l + 1)]
            a = [_ln(x[p], g1, b1) for p in range(s)]
            q = [_linear(a[p], wq, bq) for p in range(s)]
            k = [_linear(a[p], wk, bk) for p in range(s)]
            v = [_linear(a[p], wv, bv) for p in range(s)]
            hl = len(wq)
            d = hl // lh
            o = [[0.0] * hl for _ in range(s)]
            for hd in range(lh):
                c0 = hd * d
                for i in range(s):
                    sc = [sum(q[i][c0 + c] * d ** -0.5 * k[j][c0 + c] for c in range(d))
                          for j in range(i + 1)]
                    mx = max(sc)
                    e = [math.exp(z - mx) for z in sc]
                    den = sum(e)
                    for c in range(d):
                        o[i][c0 + c] = sum(e[j] / den * v[j][c0 + c] for j in range(i + 1))
            for p in range(s):
                part = hook(_linear(o[p], wo, None))
                x[p] = [x[p][c] + part[c] + bo[c] for c in range(h)]
            for p in range(s):
                a2 = _ln(x[p], g2, b2)
                u = [max(0.0, z) for z in _linear(a2, w1, c1)]
                part = hook(_linear(u, w2, None))
                x[p] = [x[p][c] + part[c] + c2[c] for c in range(h)]
        gf, bf = params[-2], params[-1]
        rows = []
        for p in range(s):
            y = _ln(x[p], gf, bf)
            rows.append([sum(y[c] * tok[r][c] for c in range(h)) for r in range(vl)])
        out.append(rows)
    return out
