"""fp64 walk through the streaming algorithm (paper Alg. 2), one head at a time.

TEST INFRASTRUCTURE, not a product path.  This is the paper's tiled procedure
taken step by step in its own notation (m, l, O, r, A, B per query block; a loop
over key/value blocks; the epilogue that divides by l), in float64 and with no
fusion or reordering.  Its purpose is to show, on the CPU, that the streaming
recurrences and the epilogue reproduce the explicit definition in
`attn_jvp_ref` for any block sizes, ragged last blocks included.

Readings: `scale` multiplies S and tS as in the explicit oracle; the last block
of either sequence may be short (the paper assumes exact splits) and is simply a
shorter slice; the epilogue's C = diag(r) O uses the O that was just divided by l,
exactly as printed, which makes tO = (A + B - r O_unnormalised / l) / l.
"""
import numpy as np


def alg2_head(q, k, v, tq, tk, tv, scale, Br, Bc):
    """q, tq: [N1, d]; k, v, tk, tv: [N2, d]; float64.  Returns (o, to, L)."""
    N1, d = q.shape
    N2 = k.shape[0]
    o_out = np.empty((N1, d))
    to_out = np.empty((N1, d))
    L_out = np.empty(N1)
    for i0 in range(0, N1, Br):                       # for i = 1..T_r
        Qi, tQi = q[i0:i0 + Br], tq[i0:i0 + Br]
        n = Qi.shape[0]
        m = np.full(n, -np.inf)
        l = np.zeros(n)
        O = np.zeros((n, d))
        r = np.zeros(n)
        A = np.zeros((n, d))
        Bm = np.zeros((n, d))
        for j0 in range(0, N2, Bc):                   # for j = 1..T_c
            Kj, tKj = k[j0:j0 + Bc], tk[j0:j0 + Bc]
            Vj, tVj = v[j0:j0 + Bc], tv[j0:j0 + Bc]
            S = scale * (Qi @ Kj.T)
            tS = scale * (tQi @ Kj.T + Qi @ tKj.T)
            m_new = np.maximum(m, S.max(axis=1))
            Pt = np.exp(S - m_new[:, None])
            alpha = np.exp(m - m_new)
            l_new = alpha * l + Pt.sum(axis=1)
            O_new = alpha[:, None] * O + Pt @ Vj
            A_new = alpha[:, None] * A + Pt @ tVj
            Ht = Pt * tS
            r_new = alpha * r + Ht.sum(axis=1)
            B_new = alpha[:, None] * Bm + Ht @ Vj
            m, l, O, A, r, Bm = m_new, l_new, O_new, A_new, r_new, B_new
        O = O / l[:, None]
        L = m + np.log(l)
        C = r[:, None] * O
        tO = (A + Bm - C) / l[:, None]
        o_out[i0:i0 + n], to_out[i0:i0 + n], L_out[i0:i0 + n] = O, tO, L
    return o_out, to_out, L_out
