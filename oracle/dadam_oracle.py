"""CPU oracle for the decentralized (accumulated) Adam step.  TEST INFRASTRUCTURE ONLY.

This module is the plain, slow, double-precision statement of what the hot path
computes.  It exists so that the HIP kernels can be checked against something that
can be compared with the paper by eye.  It is imported by the tests, by the
smoke check and by the benchmark's CPU-baseline leg, and by nothing else: the
product path never routes through it and it imports nothing from the package
that holds the kernels.

What it follows
---------------
* the decentralized update template, eq. (2) of section 2: the new model of
  worker i is its search direction scaled by the step size plus the weighted sum
  of the *previous* models of its neighbours (the worker itself included);
* Algorithm 1 (section 4), decentralized Adam;
* Algorithm 3 (appendix "Decentralized accumulated Adam"), which contains
  Algorithm 1 as the case s = 1;
* Algorithm 2 (appendix, "All-Reduce Adam") only as a comparison target for one
  of the pins (see allreduce_adam()).

Every array is float64.  Two state conventions share one code path:

* ``O64``  - nothing is rounded; this is "the exact iteration".
* ``O32m`` - after each iteration the stored quantities are rounded to the dtype
  they are stored in on the device (float32 for m_hat, v_hat, b; float32 or
  bfloat16 for x).  The arithmetic inside an iteration stays double.  This is the
  variant a float32 implementation is compared with, because it does not let
  rounding differences of earlier iterations pile up in the comparison.

Readings of the paper taken here (each is also listed in the design document):

* line 12 of Algorithm 3 prints beta_1 for the decay of v_hat; the oracle takes
  that as a misprint for beta_2 (line 7 and the bias correction of line 8 use
  beta_2, and only then does s = 1 give back Algorithm 1).  The literal reading is
  available through ``beta_vhat``.
* epsilon is added outside the square root, after bias correction (Algorithms 1
  and 3), not inside as in the analysis section.
* [b]^2 in the fold is the square of the averaged gradient.
* the bias-correction exponent is t_hat = ceil(t/s); the moments of lines 6-7 are
  temporaries rebuilt from the persistent m_hat, v_hat at every iteration.
* all rows are updated from the previous iterate at once (Jacobi), which is what
  "x_j^(t-1)" in eq. (2) says.

* the AdamW-style variant (weight_decay argument) is not written out in the paper; the
  reading taken is stated at dadam_step.

Pins: tests/test_oracle_pins.py checks every function below against closed forms,
library routines (torch.optim.Adam), brute force with a dense mixing matrix, and
the invariants the paper states; the two error scales at the end (not part of the
method, but every relative tolerance of the parity tests is relative to them) are
pinned to hand values on the hand-worked trace and to what a float32 evaluation of
an iteration actually commits.  No function here is "parity unpinned".
"""

from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np


# --------------------------------------------------------------------------------------
# storage rounding (only used by the O32m convention)
# --------------------------------------------------------------------------------------

def round_to_f32(a: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest float32 (ties to even), returned as float64."""
    return np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round to bfloat16 (1 sign, 8 exponent, 7 fraction bits), ties to even.

    The value is first rounded to float32, the precision the bf16 variant computes
    in, and that float32 is then rounded to its upper 16 bits.  NaN stays NaN.
    Returned as float64.
    """
    f = np.asarray(a, dtype=np.float64).astype(np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    rounded = (bits + np.uint64(0x7FFF) + lsb) >> np.uint64(16)
    out_bits = (rounded.astype(np.uint32) << np.uint32(16))
    out = out_bits.view(np.float32).astype(np.float64)
    nan = np.isnan(f)
    if np.any(nan):
        out = np.where(nan, np.nan, out)
    return out.reshape(np.shape(a))


def _store_x(a: np.ndarray, mode: str, param_dtype: str) -> np.ndarray:
    if mode == "O64":
        return a
    if param_dtype == "bf16":
        return round_to_bf16(a)
    return round_to_f32(a)


def _store_state(a: np.ndarray, mode: str) -> np.ndarray:
    return a if mode == "O64" else round_to_f32(a)


# --------------------------------------------------------------------------------------
# hyper-parameters and topology
# --------------------------------------------------------------------------------------

@dataclass
class Hyper:
    """Hyper-parameters of Algorithms 1 and 3.  ``s`` is the length of an
    accumulation loop (line 1 of Algorithm 3); s = 1 is Algorithm 1."""
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    s: int = 1
    beta_vhat: Optional[float] = None   # decay of v_hat in the fold; None = beta2

    def bv(self) -> float:
        return self.beta2 if self.beta_vhat is None else self.beta_vhat


@dataclass
class Csr:
    """Rows of the mixing matrix W restricted to the rows being updated.

    Row i lists its neighbourhood N_i (the worker itself is an ordinary entry) as
    column numbers into the list of source buffers, with the weights w_ij
    (eq. (2); Assumption 3 for the properties the analysis wants of W)."""
    row_ptr: np.ndarray
    col: np.ndarray
    w: np.ndarray

    @property
    def n_rows(self) -> int:
        return len(self.row_ptr) - 1

    def dense(self, n_cols: int) -> np.ndarray:
        W = np.zeros((self.n_rows, n_cols), dtype=np.float64)
        for i in range(self.n_rows):
            for k in range(int(self.row_ptr[i]), int(self.row_ptr[i + 1])):
                W[i, int(self.col[k])] += float(self.w[k])
        return W


def t_hat(t: int, s: int) -> int:
    """Group index of iteration t (1-based): ceil(t / s).  Algorithm 3, line 4."""
    return -(-int(t) // int(s))


# --------------------------------------------------------------------------------------
# the pieces of one iteration
# --------------------------------------------------------------------------------------

def mix_rows(x_src: Sequence[np.ndarray], csr: Csr) -> List[np.ndarray]:
    """Neighbour mixing, the sum term of eq. (2) / Algorithm 1 line 6 / Algorithm 3
    line 8:  mix_i = sum over j in N_i of w_ij * x_j^(t-1), entries taken in the
    order the row lists them."""
    out = []
    for i in range(csr.n_rows):
        acc = np.zeros_like(np.asarray(x_src[0], dtype=np.float64))
        for k in range(int(csr.row_ptr[i]), int(csr.row_ptr[i + 1])):
            acc = acc + float(csr.w[k]) * np.asarray(x_src[int(csr.col[k])], dtype=np.float64)
        out.append(acc)
    return out


def temporary_moments(m_hat: np.ndarray, v_hat: np.ndarray, g: np.ndarray, hp: Hyper):
    """Algorithm 3 lines 6-7 (Algorithm 1 lines 4-5 when s = 1): the first and
    second moment used by this iteration, built from the persistent moments of the
    previous group and the fresh gradient."""
    m = hp.beta1 * m_hat + (1.0 - hp.beta1) * g
    v = hp.beta2 * v_hat + (1.0 - hp.beta2) * (g * g)
    return m, v


def search_direction(m: np.ndarray, v: np.ndarray, th: int, hp: Hyper) -> np.ndarray:
    """The fraction of Algorithm 3 line 8 (Algorithm 1 line 6): bias-corrected first
    moment over (square root of bias-corrected second moment, plus epsilon).  The
    exponent of the bias correction is the group index."""
    c1 = 1.0 - hp.beta1 ** th
    c2 = 1.0 - hp.beta2 ** th
    return (m / c1) / (np.sqrt(v / c2) + hp.eps)


def accumulate_and_fold(m_hat, v_hat, b, g, t: int, hp: Hyper):
    """Algorithm 3 lines 9-13: add g/s to the accumulator; at the end of a loop
    (t mod s == 0) fold the averaged gradient into the persistent moments and clear
    the accumulator."""
    b = b + g / float(hp.s)
    if t % hp.s == 0:
        bv = hp.bv()
        m_hat = hp.beta1 * m_hat + (1.0 - hp.beta1) * b
        v_hat = bv * v_hat + (1.0 - bv) * (b * b)
        b = np.zeros_like(b)
    return m_hat, v_hat, b


# --------------------------------------------------------------------------------------
# one iteration for all rows
# --------------------------------------------------------------------------------------

@dataclass
class State:
    """Everything one iteration reads and writes.  x_src holds x^(t-1) of every
    source buffer (own replicas and/or neighbours' receive buffers); the other three
    lists have one entry per updated row."""
    x_src: List[np.ndarray]
    m_hat: List[np.ndarray]
    v_hat: List[np.ndarray]
    b: List[np.ndarray]


def dadam_step(state: State, grads: Sequence[np.ndarray], csr: Csr, t: int, hp: Hyper,
               mode: str = "O32m", param_dtype: str = "f32",
               do_update: bool = True, do_accumulate: bool = True,
               weight_decay=None) -> List[np.ndarray]:
    """Iteration t (1-based) of Algorithm 3 for every row; returns x^(t) per row and
    updates m_hat, v_hat, b in ``state`` (x_src is left alone: all rows read the
    previous iterate, the caller decides what the next iteration's sources are).

    do_update=False skips lines 6-8 (returns None), do_accumulate=False skips lines
    9-13: the two halves of the unfused call sequence.

    weight_decay (None, a number, or an array with one entry per coordinate) selects the
    AdamW-style variant the appendix mentions without writing it out.  Reading taken:
    decoupled weight decay is part of the search direction of eq. (2), which by the
    paper's construction depends on worker i's own quantities only, so the direction
    becomes  u_i + lambda * x_i^(t-1)  with x_i^(t-1) the worker's OWN previous model
    (source buffer i), applied at every model update:
        x_i^(t) = sum_j w_ij x_j^(t-1) - lr * (u_i + lambda * x_i^(t-1)).
    With W = I and s = 1 this is the library's AdamW.
    """
    assert t >= 1 and hp.s >= 1
    th = t_hat(t, hp.s)
    x_new = None
    if do_update:
        mixes = mix_rows(state.x_src, csr)
        x_new = []
        for i in range(csr.n_rows):
            g = np.asarray(grads[i], dtype=np.float64)
            m, v = temporary_moments(state.m_hat[i], state.v_hat[i], g, hp)
            u = search_direction(m, v, th, hp)
            if weight_decay is not None:
                u = u + np.asarray(weight_decay, dtype=np.float64) * np.asarray(state.x_src[i], dtype=np.float64)
            x_new.append(_store_x(mixes[i] - hp.lr * u, mode, param_dtype))
    if do_accumulate:
        for i in range(csr.n_rows):
            g = np.asarray(grads[i], dtype=np.float64)
            mh, vh, b = accumulate_and_fold(state.m_hat[i], state.v_hat[i], state.b[i], g, t, hp)
            state.m_hat[i] = _store_state(mh, mode)
            state.v_hat[i] = _store_state(vh, mode)
            state.b[i] = _store_state(b, mode)
    return x_new


def mix_only(x_src: Sequence[np.ndarray], csr: Csr, mode: str = "O32m",
             param_dtype: str = "f32") -> List[np.ndarray]:
    """x_dst = W x_src: eq. (2) with a zero search direction."""
    return [_store_x(m, mode, param_dtype) for m in mix_rows(x_src, csr)]


def consensus_error(x: Sequence[np.ndarray]) -> float:
    """Squared distance of the replicas from their average, sum_i ||x_i - x_bar||^2 with
    x_bar = (1/N) sum_i x_i: the quantity whose decay per communication round the paper plots
    to compare topologies (section on heterogeneous communication), and the left-hand side of
    the consensus lemma."""
    X = np.stack([np.asarray(a, dtype=np.float64) for a in x])
    xbar = X.mean(axis=0)
    return float(np.sum((X - xbar) ** 2))


def run_simulation(x0: Sequence[np.ndarray], grads_of_t, csr_of_t, T: int, hp: Hyper,
                   mode: str = "O32m", param_dtype: str = "f32", t_start: int = 1,
                   state: Optional[State] = None, weight_decay=None) -> State:
    """All n replicas of a decentralized run held side by side (rows = sources):
    iterations t_start..T.  grads_of_t(t) -> list of n gradient arrays,
    csr_of_t(t) -> Csr for that iteration (time-varying topologies)."""
    n = len(x0)
    if state is None:
        z = lambda: [np.zeros_like(np.asarray(x0[0], dtype=np.float64)) for _ in range(n)]
        state = State([np.asarray(x, dtype=np.float64).copy() for x in x0], z(), z(), z())
    for t in range(t_start, T + 1):
        x_new = dadam_step(state, grads_of_t(t), csr_of_t(t), t, hp, mode, param_dtype, weight_decay=weight_decay)
        state.x_src = x_new
    return state


# --------------------------------------------------------------------------------------
# Algorithm 2 - only a comparison target for the complete-topology pin
# --------------------------------------------------------------------------------------

def allreduce_adam(x0: np.ndarray, grads_of_t, n: int, T: int, hp: Hyper) -> np.ndarray:
    """All-Reduce Adam (appendix, Algorithm 2): average the n gradients, then one
    ordinary Adam update of the single shared model.  Returns x after T iterations
    (float64, nothing rounded)."""
    x = np.asarray(x0, dtype=np.float64).copy()
    m = np.zeros_like(x)
    v = np.zeros_like(x)
    for t in range(1, T + 1):
        gs = grads_of_t(t)
        gbar = sum(np.asarray(g, dtype=np.float64) for g in gs) / float(n)
        m = hp.beta1 * m + (1.0 - hp.beta1) * gbar
        v = hp.beta2 * v + (1.0 - hp.beta2) * gbar * gbar
        x = x - hp.lr * (m / (1.0 - hp.beta1 ** t)) / (np.sqrt(v / (1.0 - hp.beta2 ** t)) + hp.eps)
    return x


# --------------------------------------------------------------------------------------
# error scale used by the parity tests (not part of the method)
# --------------------------------------------------------------------------------------

def magnitude_scale(state: State, grads: Sequence[np.ndarray], csr: Csr, t: int, hp: Hyper, weight_decay=None):
    """Per row, the sum of the magnitudes of the terms that make up x^(t):
    sum_j |w_ij x_j| + lr * (beta1 |m_hat| + (1-beta1)|g|) / c1 / (sqrt(v/c2) + eps).
    A float32 evaluation of the iteration is off by a small multiple of 2^-24 times
    this quantity; relative tolerances in the parity tests are taken against it, so
    that elements where mixing and update cancel do not get a meaningless bound."""
    th = t_hat(t, hp.s)
    c1 = 1.0 - hp.beta1 ** th
    c2 = 1.0 - hp.beta2 ** th
    out = []
    for i in range(csr.n_rows):
        acc = np.zeros_like(np.asarray(state.x_src[0], dtype=np.float64))
        for k in range(int(csr.row_ptr[i]), int(csr.row_ptr[i + 1])):
            acc = acc + abs(float(csr.w[k])) * np.abs(state.x_src[int(csr.col[k])])
        g = np.asarray(grads[i], dtype=np.float64)
        v = hp.beta2 * state.v_hat[i] + (1.0 - hp.beta2) * g * g
        mag_m = hp.beta1 * np.abs(state.m_hat[i]) + (1.0 - hp.beta1) * np.abs(g)
        scale = acc + hp.lr * (mag_m / c1) / (np.sqrt(v / c2) + hp.eps)
        if weight_decay is not None:
            scale = scale + hp.lr * np.abs(np.asarray(weight_decay, dtype=np.float64) * state.x_src[i])
        out.append(scale)
    return out


def state_magnitude_scales(state: State, grads: Sequence[np.ndarray], t: int, hp: Hyper):
    """Per row, the sums of the magnitudes of the terms that make up b, m_hat and v_hat after
    iteration t (state = what the iteration starts from):
        b:      |b| + |g|/s
        m_hat:  beta1 |m_hat| + (1-beta1) (|b| + |g|/s)      on a fold iteration, |m_hat| otherwise
        v_hat:  betav |v_hat| + (1-betav) (|b| + |g|/s)^2    on a fold iteration, |v_hat| otherwise
    Returns (scale_b, scale_m, scale_v), each a list with one array per row."""
    sb, sm, sv = [], [], []
    fold = (t % hp.s == 0)
    for i in range(len(grads)):
        g = np.abs(np.asarray(grads[i], dtype=np.float64))
        bmag = np.abs(state.b[i]) + g / hp.s
        sb.append(bmag)
        if fold:
            sm.append(hp.beta1 * np.abs(state.m_hat[i]) + (1 - hp.beta1) * bmag)
            sv.append(hp.bv() * np.abs(state.v_hat[i]) + (1 - hp.bv()) * bmag * bmag)
        else:
            sm.append(np.abs(state.m_hat[i]))
            sv.append(np.abs(state.v_hat[i]))
    return sb, sm, sv
