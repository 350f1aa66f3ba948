"""fp64 check of the streaming algebra behind paper Alg. 2, one head at a time.

TEST INFRASTRUCTURE, not a product path.  Alg. 2 never forms the N1 x N2 matrices: it visits the key/value
sequence block by block and keeps, per query row, a running maximum m, the sums l and r, and the accumulators
O, A, B, all expressed relative to exp(m); whenever m grows, everything accumulated so far is multiplied by
exp(m_old - m_new).  That update is one instance of a general fact, which is what this file states and what the
tests check against the explicit definition in `attn_jvp_ref`:

  * a key/value block j alone gives a *partial state* (m, l, O~, r, G) of a query block, with
      m = rowmax S_j,  P~ = exp(S_j - m),  l = rowsum P~,  O~ = P~ V_j,
      H~ = P~ o tS_j,  r = rowsum H~,       G = P~ tV_j + H~ V_j          (G is Alg. 2's A + B);
  * two partial states over disjoint key sets merge into the state of their union by bringing both to the
    larger m and adding: an associative and commutative operation, so the blocks may be folded left to right
    (Alg. 2's loop), right to left, or as a tree (key-sharded execution);
  * the state over all keys gives the outputs: O = O~ / l, L = m + log l, tO = (G - (r / l) O~) / l, which is
    Alg. 2's epilogue with its C = diag(r) O written out (its O is already divided by l at that point).

Readings: `scale` multiplies S and tS as in the explicit oracle; the last block of either sequence may be short
(the paper assumes exact splits) and is simply a shorter slice.
"""
from functools import reduce

import numpy as np


def block_state(Qi, tQi, Kj, Vj, tKj, tVj, scale):
    """Partial state of the query rows Qi over the keys of one block: (m, l, O~, r, G)."""
    S = scale * (Qi @ Kj.T)
    tS = scale * (tQi @ Kj.T + Qi @ tKj.T)
    m = S.max(axis=1)
    Pt = np.exp(S - m[:, None])
    Ht = Pt * tS
    return m, Pt.sum(axis=1), Pt @ Vj, Ht.sum(axis=1), Pt @ tVj + Ht @ Vj


def merge(a, b):
    """State over the union of two disjoint key sets: both sides rescaled to the larger maximum, then added."""
    m = np.maximum(a[0], b[0])
    wa, wb = np.exp(a[0] - m), np.exp(b[0] - m)
    return (m, wa * a[1] + wb * b[1], wa[:, None] * a[2] + wb[:, None] * b[2], wa * a[3] + wb * b[3],
            wa[:, None] * a[4] + wb[:, None] * b[4])


def finish(state):
    """Outputs from the state over all keys: (O, tO, L)."""
    m, l, Ot, r, G = state
    return Ot / l[:, None], (G - (r / l)[:, None] * Ot) / l[:, None], m + np.log(l)


def _fold(states, order):
    if order == "forward":            # Alg. 2's loop: state <- merge(state, next block)
        return reduce(merge, states)
    if order == "backward":
        return reduce(merge, reversed(states))
    if order == "tree":               # pairwise, as shards of the key sequence would be combined
        while len(states) > 1:
            states = [merge(states[i], states[i + 1]) if i + 1 < len(states) else states[i]
                      for i in range(0, len(states), 2)]
        return states[0]
    raise ValueError(order)


def alg2_head(q, k, v, tq, tk, tv, scale, Br, Bc, order="forward"):
    """q, tq: [N1, d]; k, v, tk, tv: [N2, d]; float64.  Query blocks of Br rows, key blocks of Bc rows, the key
    blocks folded in the given order.  Returns (o, to, L)."""
    N1, d = q.shape
    N2 = k.shape[0]
    o_out, to_out, L_out = np.empty((N1, d)), np.empty((N1, d)), np.empty(N1)
    for i0 in range(0, N1, Br):
        Qi, tQi = q[i0:i0 + Br], tq[i0:i0 + Br]
        states = [block_state(Qi, tQi, k[j0:j0 + Bc], v[j0:j0 + Bc], tk[j0:j0 + Bc], tv[j0:j0 + Bc], scale)
                  for j0 in range(0, N2, Bc)]
        n = Qi.shape[0]
        o_out[i0:i0 + n], to_out[i0:i0 + n], L_out[i0:i0 + n] = finish(_fold(states, order))
    return o_out, to_out, L_out
