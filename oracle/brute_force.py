"""Pure-Python enumeration of the attention contractions, for tiny shapes.

TEST INFRASTRUCTURE ONLY (see mqa_oracle.py).  The paper (Section 2.1) defines
an einsum as: broadcast every input over the union of the index names,
multiply component-wise, sum over the names missing from the output.  This
file does exactly that with nested loops, `math.exp` and `math.fsum`, and is
used only to pin the numpy oracle.  It imports nothing from the numpy oracle.
"""
import math


def softmax_list(z):
    """Section 2.1 softmax over a list of logits."""
    mx = max(z)
    e = [math.exp(t - mx) for t in z]
    s = math.fsum(e)
    return [t / s for t in e]


def mqa_decode_bf(q, K, V, lens, scale=1.0, window=None):
    """Section 3 step: q[b][h][k], K[b][m][k], V[b][m][v] nested lists ->
    o[b][h][v]; sequence i uses its first lens[i] positions, or only the last
    `window` of them (the local variant of Section 4.1)."""
    b, h = len(q), len(q[0])
    kdim, vdim = len(q[0][0]), len(V[0][0])
    out = []
    for i in range(b):
        rows = []
        for j in range(h):
            L = lens[i]
            if L == 0:
                rows.append([0.0] * vdim)
                continue
            lo = 0 if window is None else max(0, L - window)
            logits = [scale * math.fsum(q[i][j][c] * K[i][p][c] for c in range(kdim)) for p in range(lo, L)]
            w = softmax_list(logits)
            rows.append([math.fsum(w[p - lo] * V[i][p][c] for p in range(lo, L)) for c in range(vdim)])
        out.append(rows)
    return out


def mha_decode_bf(q, K, V, lens, scale=1.0):
    """Section 2.4 step: K[b][h][m][k], V[b][h][m][v] carry a heads index."""
    b, h = len(q), len(q[0])
    kdim, vdim = len(q[0][0]), len(V[0][0][0])
    out = []
    for i in range(b):
        rows = []
        for j in range(h):
            L = lens[i]
            if L == 0:
                rows.append([0.0] * vdim)
                continue
            logits = [scale * math.fsum(q[i][j][c] * K[i][j][p][c] for c in range(kdim)) for p in range(L)]
            w = softmax_list(logits)
            rows.append([math.fsum(w[p] * V[i][j][p][c] for p in range(L)) for c in range(vdim)])
        out.append(rows)
    return out


def project_q_bf(x, P_q):
    """einsum('bd,hdk->bhk')."""
    b, d, h, k = len(x), len(x[0]), len(P_q), len(P_q[0][0])
    return [[[math.fsum(x[i][t] * P_q[j][t][c] for t in range(d)) for c in range(k)]
             for j in range(h)] for i in range(b)]


def project_kv_bf(x, P):
    """einsum('bd,dk->bk')."""
    b, d, k = len(x), len(x[0]), len(P[0])
    return [[math.fsum(x[i][t] * P[t][c] for t in range(d)) for c in range(k)] for i in range(b)]


def project_o_bf(o, P_o):
    """einsum('bhv,hdv->bd')."""
    b, h, v, d = len(o), len(o[0]), len(o[0][0]), len(P_o[0])
    return [[math.fsum(o[i][j][c] * P_o[j][t][c] for j in range(h) for c in range(v))
             for t in range(d)] for i in range(b)]
