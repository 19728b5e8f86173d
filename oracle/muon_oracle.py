"""Plain fp64 CPU oracle for one scaled-Muon optimizer step on one 2-D matrix.

TEST INFRASTRUCTURE ONLY: this module exists to check the HIP library and to be
timed as the CPU baseline.  The product package never imports it, and it shares
no code, tables or helpers with the HIP path.

The method is an iteration (a fixed number of Newton-Schulz steps, not the exact
polar factor), so the oracle is the algorithm itself, step by step, in the
paper's order and notation, in IEEE double precision.  numpy's ``@`` (a library
matmul) is the only primitive used; there is no blocking, fusion or reordering.

Every function is pinned by tests that do not call it to produce the expected
value (SVD closed form, exact rational scalar orbits, hand-worked 2x2 cases,
pure-Python brute force, symmetries, the singular-value band, Lemma 1).
Nothing here is "parity unpinned".

Notation (paper section 2.1 and 2.2): W weight [A, B]; G gradient; M momentum;
mu momentum coefficient; eta learning rate; lambda weight-decay ratio; N number
of Newton-Schulz iterations; (a, b, c) the quintic's coefficients; O the
orthogonalised update.
"""
from __future__ import annotations

import numpy as np

# Coefficients and defaults stated in section 2.1 (coefficients) and
# section 2.2 "Other Hyper-parameters" / "Matching update RMS of AdamW".
NS_A, NS_B, NS_C = 3.4445, -4.7750, 2.0315
DEFAULT_MU = 0.95
DEFAULT_NS_STEPS = 5
DEFAULT_RMS_SCALE = 0.2


def _f64(x) -> np.ndarray:
    """Widen an array exactly to float64 (every fp32/bf16 value is a double)."""
    return np.asarray(x, dtype=np.float64)


def momentum_update(M_prev, G, mu: float) -> np.ndarray:
    """M_t = mu * M_{t-1} + grad   (first line of the update rule, section 2.1)."""
    return float(mu) * _f64(M_prev) + _f64(G)


def ns_input(M_t, G, mu: float, nesterov: bool) -> np.ndarray:
    """Matrix handed to Newton-Schulz.

    Plain momentum feeds M_t (Eq. 1).  The Nesterov-style variant the paper says
    it uses in practice (footnote 1 of section 2.1) feeds mu * M_t + grad.
    """
    if nesterov:
        return float(mu) * _f64(M_t) + _f64(G)
    return _f64(M_t).copy()


def frobenius_normalize(U, eps: float = 0.0) -> np.ndarray:
    """X_0 = U / ||U||_F  (section 2.1, "Newton-Schulz Iterations ...").

    The paper has no epsilon; ``eps`` is added to the norm so that an all-zero
    input gives X_0 = 0 instead of 0/0.  With eps = 0 this is the paper's formula.
    """
    U = _f64(U)
    norm = np.sqrt(np.sum(U * U))
    return U / (norm + float(eps))


def newton_schulz_iterate(X0, steps: int = DEFAULT_NS_STEPS,
                          a: float = NS_A, b: float = NS_B, c: float = NS_C, schedule=None) -> np.ndarray:
    """N applications of Eq. 2:  X_k = a X + b (X X^T) X + c (X X^T)^2 X.

    Written exactly as printed: the Gram matrix X X^T, its square, and the three
    terms summed.  Works for any shape (the formula never transposes).

    ``schedule`` (an extension; the paper uses one triple throughout): a sequence of
    ``steps`` triples (a_k, b_k, c_k), iteration k using the k-th one instead of (a, b, c).
    """
    X = _f64(X0).copy()
    if schedule is not None and len(schedule) != int(steps):
        raise ValueError("schedule needs one (a, b, c) triple per iteration")
    for k in range(int(steps)):
        ak, bk, ck = (a, b, c) if schedule is None else (float(v) for v in schedule[k])
        XXt = X @ X.T
        X = ak * X + bk * (XXt @ X) + ck * ((XXt @ XXt) @ X)
    return X


def newton_schulz(U, steps: int = DEFAULT_NS_STEPS, a: float = NS_A, b: float = NS_B,
                  c: float = NS_C, eps: float = 0.0, orient: bool = True, schedule=None) -> np.ndarray:
    """O = Newton-Schulz(U): normalise, orient so rows <= cols, iterate, orient back.

    The paper never transposes; because the quintic is odd, iterating on U^T and
    transposing the result is the same map in exact arithmetic (only the size of
    the Gram matrix changes).  ``orient=False`` runs the formula as printed.
    """
    U = _f64(U)
    X0 = frobenius_normalize(U, eps)
    transposed = orient and U.shape[0] > U.shape[1]
    if transposed:
        X0 = X0.T
    X = newton_schulz_iterate(X0, steps, a, b, c, schedule)
    return X.T.copy() if transposed else X


def update_factor(O, shape, rms_scale: float = DEFAULT_RMS_SCALE, scale_mode: str = "adjusted_lr",
                  hidden_size=None) -> float:
    """The factor that multiplies O in the update, for the three variants of section 3.1.

    "adjusted_lr" (Eq. 7, identical to Eq. 4): rms_scale * sqrt(max(A, B));
    "baseline"    (Eq. 5):                     rms_scale * sqrt(H), H the model's hidden size;
    "update_norm" (Eq. 6):                     rms_scale / RMS(O)   (0 for O = 0).
    """
    A, B = shape
    if scale_mode == "adjusted_lr":
        return float(rms_scale) * float(np.sqrt(float(max(A, B))))
    if scale_mode == "baseline":
        return float(rms_scale) * float(np.sqrt(float(hidden_size)))
    if scale_mode == "update_norm":
        r = update_rms(O)
        return float(rms_scale) / r if r > 0.0 else 0.0
    raise ValueError(scale_mode)


def apply_update(W_prev, O, lr: float, weight_decay: float, rms_scale: float = DEFAULT_RMS_SCALE,
                 scale_mode: str = "adjusted_lr", hidden_size=None) -> np.ndarray:
    """W_t = W_{t-1} - eta * (factor * O + lambda * W_{t-1}).

    With the default mode this is Eq. 4 (which contains the decoupled weight decay of
    Eq. 3): factor = rms_scale * sqrt(max(A, B)), rms_scale the paper's 0.2, [A, B] the
    shape of the matrix as passed.  The other modes are Eq. 5 and Eq. 6.
    """
    W_prev = _f64(W_prev)
    O = _f64(O)
    factor = update_factor(O, W_prev.shape, rms_scale, scale_mode, hidden_size)
    return W_prev - float(lr) * (factor * O + float(weight_decay) * W_prev)


def update_rms(O) -> float:
    """sqrt(mean(u^2)) of the orthogonalised update (return value of Algorithm 1)."""
    O = _f64(O)
    return float(np.sqrt(np.mean(O * O)))


def muon_step(W_prev, G, M_prev, *, lr: float, weight_decay: float, mu: float = DEFAULT_MU,
              ns_steps: int = DEFAULT_NS_STEPS, a: float = NS_A, b: float = NS_B, c: float = NS_C,
              rms_scale: float = DEFAULT_RMS_SCALE, eps: float = 0.0, nesterov: bool = True,
              scale_mode: str = "adjusted_lr", hidden_size=None, schedule=None):
    """One whole step on one matrix.  Returns (W_t, M_t, O_t) in float64."""
    M = momentum_update(M_prev, G, mu)
    U = ns_input(M, G, mu, nesterov)
    O = newton_schulz(U, ns_steps, a, b, c, eps, schedule=schedule)
    W = apply_update(W_prev, O, lr, weight_decay, rms_scale, scale_mode, hidden_size)
    return W, M, O
