"""Explicit fp64 definition of attention and its Jacobian-vector product.

TEST INFRASTRUCTURE, not a product path: a plain, slow, obviously-correct CPU
implementation used to judge the HIP kernels.  It shares no code with them.

What it computes (paper App. C.1, the unnumbered equations that define
S, P, O and then tS, tP, tO), per (batch, head), everything in float64:

    S   = scale * Q K^T                       scores           [Lq, Lkv]
    P   = softmax_rows(S)                     probabilities
    lse = log sum_j exp(S_ij)                 the L of Alg. 2's epilogue
    O   = P V
    tS  = scale * (tQ K^T + Q tK^T)           tangent of S
    tP  = P o tS - P o rowsum(P o tS)         tangent of the row softmax
    tO  = tP V + P tV

Readings of points the paper leaves open:
  * the paper writes S = Q K^T with no softmax scale; here the caller's constant
    `scale` multiplies both S and tS (it is not differentiated);
  * in the tP equation the paper writes (P o tS) 1 1^T; that is the row sum of
    P o tS broadcast back over the row, which is what differentiating a row
    softmax gives;
  * inputs are taken at whatever values they hold (bf16 or fp32 values are
    upcast exactly), so input rounding is not part of the error budget.

The full Lq x Lkv matrices are materialised on purpose.  For long sequences the
caller passes `rows`, a list of query indices: query rows are independent of one
another, so evaluating a subset is exact for that subset.
"""
import numpy as np


def _as_f64(x):
    """Exact upcast of a numpy array or a CPU torch tensor (any float dtype) to float64."""
    if hasattr(x, "detach"):  # torch tensor, possibly bf16 which numpy cannot hold
        x = x.detach().cpu().double().numpy()
    return np.asarray(x, dtype=np.float64)


def attn_jvp_ref_head(q, k, v, tq, tk, tv, scale):
    """One head.  q, tq: [Lq, d]; k, v, tk, tv: [Lkv, d]; float64.  Returns (o, to, lse)."""
    s = scale * (q @ k.T)                                  # S
    row_max = s.max(axis=1, keepdims=True)
    e = np.exp(s - row_max)
    z = e.sum(axis=1, keepdims=True)
    p = e / z                                              # P = softmax(S)
    lse = (row_max + np.log(z))[:, 0]
    o = p @ v                                              # O = P V
    ts = scale * (tq @ k.T + q @ tk.T)                     # tS
    h = p * ts
    tp = h - p * h.sum(axis=1, keepdims=True)              # tP
    to = tp @ v + p @ tv                                   # tO
    return o, to, lse


def attn_jvp_ref(q, k, v, tq, tk, tv, scale, rows=None):
    """All heads.  q, tq: [B, H, Lq, d]; k, v, tk, tv: [B, H, Lkv, d].

    rows: optional 1-D integer array of query indices; the same subset is taken in
    every (batch, head).  Returns o, to: [B, H, R, d] and lse: [B, H, R] in float64,
    R = len(rows) or Lq.
    """
    q, k, v, tq, tk, tv = (_as_f64(x) for x in (q, k, v, tq, tk, tv))
    B, H, Lq, d = q.shape
    if rows is not None:
        rows = np.asarray(rows, dtype=np.int64)
        q, tq = q[:, :, rows, :], tq[:, :, rows, :]
    R = q.shape[2]
    o = np.empty((B, H, R, d))
    to = np.empty((B, H, R, d))
    lse = np.empty((B, H, R))
    for b in range(B):
        for h in range(H):
            o[b, h], to[b, h], lse[b, h] = attn_jvp_ref_head(
                q[b, h], k[b, h], v[b, h], tq[b, h], tk[b, h], tv[b, h], float(scale))
    return o, to, lse
