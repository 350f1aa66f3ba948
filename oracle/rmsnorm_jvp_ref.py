"""Explicit fp64 definition of RMS normalisation with a learnable gain and of its Jacobian-vector product.

TEST INFRASTRUCTURE, not a product path: a plain CPU implementation used to judge the HIP kernel.  It shares no
code with it.

What it computes (paper App. C.2, the figure that restructures the RMSNorm layer for JVP mode; Sec. 3.1 names QK
normalisation as part of the networks): for every row x of length d, with gain w and constant eps,

    r  = 1 / sqrt(mean_k(x_k^2) + eps)
    y  = x r w
    ty = d/de [ y(x + e tx) ]_{e=0} = (tx r - x r^3 mean_k(x_k tx_k)) w

(the derivative of r is -r^3 mean(x tx)).  The paper obtains ty by applying forward-mode differentiation to the
layer's forward function; this file writes the derivative out.

Reading of a point the paper leaves to the framework: the layer normalises in float32, casts the result to the
input dtype and then multiplies by the gain.  Those casts are roundings, not part of the function: the oracle
evaluates the real-valued function in float64 on the values the inputs hold, and the comparison tolerance
accounts for the two roundings of a bf16 implementation.
"""
import numpy as np


def _as_f64(x):
    if hasattr(x, "detach"):
        x = x.detach().cpu().double().numpy()
    return np.asarray(x, dtype=np.float64)


def rmsnorm_jvp_ref(x, tx, w, eps):
    """x, tx: [..., d]; w: [d].  Returns (y, ty) in float64 with the shape of x."""
    x, tx, w = _as_f64(x), _as_f64(tx), _as_f64(w)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    r = 1.0 / np.sqrt(ms + eps)
    y = x * r * w
    xt = np.mean(x * tx, axis=-1, keepdims=True)
    ty = (tx * r - x * (r ** 3) * xt) * w
    return y, ty
