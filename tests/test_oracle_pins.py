"""Pins for the CPU oracle: each test fixes some part of oracle/dadam_oracle.py to
something that is not the oracle itself - a library routine, a closed form, brute force
with a dense matrix, an invariant the paper states, or the hand-worked trace under
tests/golden/.  The last group plants plausible mistakes in the oracle and checks that
the pins notice them."""

import copy
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import dadam_oracle as O
from paper_2410_11998_amd import workloads as WL

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def csr_of(t3, w64=False):
    rp, col, w = t3
    return O.Csr(rp, col, w.astype(np.float64) if not w64 else
                 np.asarray([1.0 / (rp[i + 1] - rp[i]) for i in range(len(rp) - 1) for _ in range(rp[i + 1] - rp[i])]))


def rand_grads(seed, n, d, T, std=1e-2):
    rng = np.random.default_rng(seed)
    return [[rng.standard_normal(d) * std for _ in range(n)] for _ in range(T + 1)]


def zeros_state(x0):
    n = len(x0)
    z = lambda: [np.zeros_like(x0[0]) for _ in range(n)]
    return O.State([x.copy() for x in x0], z(), z(), z())


# ---------------------------------------------------------------------------------------
# storage rounding against the library's conversions
# ---------------------------------------------------------------------------------------

def test_rounding_matches_torch_casts():
    rng = np.random.default_rng(1)
    a = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-30, 30, 20000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895313892515355e38, 1e-45, np.inf, -np.inf]])
    t = torch.from_numpy(a)
    assert np.array_equal(O.round_to_f32(a), t.to(torch.float32).to(torch.float64).numpy())
    want = t.to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.round_to_bf16(a), want)
    # ties go to the even neighbour: 1 + 2^-8 is half way between 1 and 1 + 2^-7
    assert O.round_to_bf16(np.array([1.00390625]))[0] == 1.0
    assert O.round_to_bf16(np.array([1.01171875]))[0] == 1.015625
    assert np.isnan(O.round_to_bf16(np.array([np.nan]))[0])


def test_t_hat_is_ceiling():
    assert [O.t_hat(t, 4) for t in range(1, 10)] == [1, 1, 1, 1, 2, 2, 2, 2, 3]
    assert [O.t_hat(t, 1) for t in range(1, 5)] == [1, 2, 3, 4]
    assert [O.t_hat(t, 3) for t in (3, 4, 6, 7)] == [1, 2, 2, 3]


# ---------------------------------------------------------------------------------------
# Adam arithmetic: W = I, s = 1 is n independent runs of the library's Adam
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("betas", [(0.9, 0.999), (0.974, 0.999), (0.5, 0.75)])
def test_identity_topology_s1_equals_torch_adam(betas):
    n, d, T = 3, 257, 9
    hp = O.Hyper(lr=2e-3, beta1=betas[0], beta2=betas[1], eps=1e-8, s=1)
    rng = np.random.default_rng(7)
    x0 = [rng.standard_normal(d) * 0.02 for _ in range(n)]
    G = rand_grads(11, n, d, T)
    st = O.run_simulation(x0, lambda t: G[t], lambda t: csr_of(WL.identity(n)), T, hp, mode="O64")
    for i in range(n):
        p = torch.tensor(x0[i], dtype=torch.float64, requires_grad=True)
        opt = torch.optim.Adam([p], lr=hp.lr, betas=betas, eps=hp.eps, weight_decay=0.0, amsgrad=False)
        for t in range(1, T + 1):
            p.grad = torch.tensor(G[t][i], dtype=torch.float64)
            opt.step()
        np.testing.assert_allclose(st.x_src[i], p.detach().numpy(), rtol=1e-12, atol=1e-15)
        sd = opt.state[p]
        np.testing.assert_allclose(st.m_hat[i], sd["exp_avg"].numpy(), rtol=1e-12, atol=1e-18)
        np.testing.assert_allclose(st.v_hat[i], sd["exp_avg_sq"].numpy(), rtol=1e-12, atol=1e-22)
        assert np.all(st.b[i] == 0.0)


@pytest.mark.parametrize("s", [1, 2, 3, 4, 8])
def test_constant_gradient_closed_form(s):
    """g = c forever  =>  m/c1 = c and v/c2 = c^2 at every iteration, for every s, so
    x^(t) = x^(0) - t * lr * c / (|c| + eps) when W = I."""
    d, T = 6, 13
    hp = O.Hyper(lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-3, s=s)
    c = np.array([0.5, -0.25, 1e-3, -3.0, 0.0, 2.0])
    x0 = [np.linspace(-1, 1, d)]
    st = zeros_state(x0)
    for t in range(1, T + 1):
        st.x_src = O.dadam_step(st, [c], csr_of(WL.identity(1)), t, hp, mode="O64")
        want = x0[0] - t * hp.lr * c / (np.abs(c) + hp.eps)
        np.testing.assert_allclose(st.x_src[0], want, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------------------------------
# mixing: dense matrix brute force, permutations, Jacobi order
# ---------------------------------------------------------------------------------------

def random_stochastic_csr(rng, n_rows, n_cols, shuffle=True):
    row_ptr, col, w = [0], [], []
    for i in range(n_rows):
        deg = int(rng.integers(1, n_cols + 1))
        cols = rng.choice(n_cols, size=deg, replace=False)
        if not shuffle:
            cols = np.sort(cols)
        ww = rng.random(deg) + 0.1
        ww /= ww.sum()
        col += list(cols)
        w += list(ww)
        row_ptr.append(len(col))
    return O.Csr(np.asarray(row_ptr, np.int32), np.asarray(col, np.int32), np.asarray(w, np.float64))


def test_mixing_equals_dense_matrix_per_coordinate():
    """Per coordinate the iteration is x_d^(t) = W x_d^(t-1) + e_d^(t) (matrix form in
    the proof of the consensus lemma): compare with a dense matmul over several steps.
    The direction e comes from search_direction, pinned separately above."""
    rng = np.random.default_rng(3)
    n, d, T = 5, 7, 6
    hp = O.Hyper(lr=1e-2, s=2)
    csr = random_stochastic_csr(rng, n, n)
    W = csr.dense(n)
    x0 = [rng.standard_normal(d) for _ in range(n)]
    G = rand_grads(5, n, d, T, std=1.0)
    st = zeros_state(x0)
    X = np.stack(x0)                      # [n, d]
    for t in range(1, T + 1):
        E = np.stack([-hp.lr * O.search_direction(*O.temporary_moments(st.m_hat[i], st.v_hat[i], G[t][i], hp),
                                                  O.t_hat(t, hp.s), hp) for i in range(n)])
        X = W @ X + E
        st.x_src = O.dadam_step(st, G[t], csr, t, hp, mode="O64")
        np.testing.assert_allclose(np.stack(st.x_src), X, rtol=1e-12, atol=1e-14)


def test_mixing_rectangular_sources_tiny_loops():
    """Rows and source buffers need not coincide (a node's own parameters plus its
    neighbours' receive buffers): scalar loops on a tiny case."""
    rng = np.random.default_rng(4)
    csr = random_stochastic_csr(rng, 2, 5)
    xs = [rng.standard_normal(3) for _ in range(5)]
    got = O.mix_rows(xs, csr)
    for i in range(2):
        for e in range(3):
            s = 0.0
            for k in range(csr.row_ptr[i], csr.row_ptr[i + 1]):
                s += csr.w[k] * xs[csr.col[k]][e]
            assert abs(got[i][e] - s) < 1e-15


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_permutation_matrix_copies_bit_exact_and_is_jacobi(dtype):
    """One weight 1.0 per row: the output is an exact copy of the selected source.  A
    cyclic shift also shows that every row reads the previous iterate (an in-place
    sweep would smear one replica over the others)."""
    n, d = 6, 33
    perm = [(i + 1) % n for i in range(n)]
    xs = [O.round_to_bf16(np.arange(d) * 0.5 + 100.0 * c) if dtype == "bf16"
          else O.round_to_f32(np.arange(d) * 0.001 + c) for c in range(n)]
    out = O.mix_only(xs, csr_of(WL.permutation(perm)), mode="O32m", param_dtype=dtype)
    for i in range(n):
        assert np.array_equal(out[i], xs[perm[i]])


# ---------------------------------------------------------------------------------------
# invariants of doubly stochastic mixing
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("topo", ["ring", "static_exp", "one_peer", "complete"])
def test_replica_mean_recursion(topo):
    """Averaging the update over workers with a doubly stochastic W gives
    mean x^(t) = mean x^(t-1) - (lr/N) sum_i direction_i (the averaged-model recursion
    used throughout the convergence analysis)."""
    n, d, T = 8, 19, 5
    t3 = {"ring": WL.ring(n), "static_exp": WL.static_exponential(n),
          "one_peer": WL.one_peer_exponential(n, 1), "complete": WL.complete(n)}[topo]
    csr = csr_of(t3, w64=True)
    W = csr.dense(n)
    np.testing.assert_allclose(W.sum(0), 1.0, atol=1e-15)
    np.testing.assert_allclose(W.sum(1), 1.0, atol=1e-15)
    hp = O.Hyper(lr=3e-3, s=2)
    rng = np.random.default_rng(9)
    x0 = [rng.standard_normal(d) for _ in range(n)]
    G = rand_grads(2, n, d, T, std=1.0)
    st = zeros_state(x0)
    for t in range(1, T + 1):
        mean_prev = np.mean(st.x_src, axis=0)
        U = [O.search_direction(*O.temporary_moments(st.m_hat[i], st.v_hat[i], G[t][i], hp), O.t_hat(t, hp.s), hp)
             for i in range(n)]
        st.x_src = O.dadam_step(st, G[t], csr, t, hp, mode="O64")
        np.testing.assert_allclose(np.mean(st.x_src, axis=0), mean_prev - hp.lr * np.mean(U, axis=0),
                                   rtol=0, atol=1e-14)


def test_zero_direction_ring4_contracts_by_one_third():
    """With zero gradients and zero moments the direction vanishes and x^(t) = W^t x^(0).
    The 4-ring with weights 1/3 has eigenvalues 1, 1/3, -1/3, 1/3, so the distance to
    consensus shrinks by exactly 1/3 per iteration (lambda of Assumption 3)."""
    n, d = 4, 11
    csr = csr_of(WL.ring(n), w64=True)
    ev = np.sort(np.abs(np.linalg.eigvalsh(csr.dense(n))))
    np.testing.assert_allclose(ev, [1 / 3, 1 / 3, 1 / 3, 1.0], atol=1e-15)
    rng = np.random.default_rng(12)
    x0 = [rng.standard_normal(d) for _ in range(n)]
    st = zeros_state(x0)
    zero = [np.zeros(d)] * n
    hp = O.Hyper(s=2)
    mean0 = np.mean(x0, axis=0)
    err_prev = np.linalg.norm(np.stack(x0) - mean0)
    for t in range(1, 8):
        st.x_src = O.dadam_step(st, zero, csr, t, hp, mode="O64")
        assert all(np.all(np.isfinite(x)) for x in st.x_src)
        np.testing.assert_allclose(np.mean(st.x_src, axis=0), mean0, atol=1e-15)
        err = np.linalg.norm(np.stack(st.x_src) - mean0)
        np.testing.assert_allclose(err, err_prev / 3.0, rtol=1e-12)
        err_prev = err
        np.testing.assert_allclose(np.stack(st.x_src), np.linalg.matrix_power(csr.dense(n), t) @ np.stack(x0), atol=1e-14)


@pytest.mark.parametrize("n", [2, 8, 16, 64])
def test_one_peer_exponential_reaches_exact_mean_after_log2n_slots(n):
    """Pins the slot schedule of the time-varying workload: pairing with hops
    1, 2, 4, ... (weights 1/2) averages all 2^tau replicas exactly after tau slots."""
    d = 5
    tau = WL.one_peer_slots(n)
    assert 2 ** tau == n
    rng = np.random.default_rng(n)
    x0 = [rng.standard_normal(d) for _ in range(n)]
    xs = [x.copy() for x in x0]
    prod = np.eye(n)
    for slot in range(tau):
        csr = csr_of(WL.one_peer_exponential(n, slot))
        prod = csr.dense(n) @ prod
        xs = O.mix_only(xs, csr, mode="O64")
        if slot < tau - 1:
            assert np.max(np.abs(np.stack(xs) - np.mean(x0, axis=0))) > 1e-3
    np.testing.assert_allclose(prod, np.full((n, n), 1.0 / n), atol=1e-15)
    np.testing.assert_allclose(np.stack(xs), np.tile(np.mean(x0, axis=0), (n, 1)), atol=1e-14)


def test_workload_slot_schedule():
    wl = WL.workload(4)
    assert wl.n_slots() == 6
    assert [wl.slot_of_step(t) for t in (1, 2, 5, 6, 7, 30)] == [1, 2, 5, 0, 1, 0]       # hop 2^(t mod 6) at step t
    assert sorted(wl.slot_of_step(t) for t in range(11, 17)) == list(range(6))             # any 6 in a row: every hop once
    rp, col, w = wl.csr(3)
    assert list(col[:2]) == [0, 8] and np.all(w == np.float32(0.5))
    rp, col, w = WL.workload(2).csr()
    assert list(col[:5]) == [0, 1, 2, 4, 8] and list(col[5 * 15:5 * 16]) == [15, 0, 1, 3, 7]
    assert np.all(w == np.float32(1.0) / np.float32(5.0))


# ---------------------------------------------------------------------------------------
# complete topology and All-Reduce Adam
# ---------------------------------------------------------------------------------------

def test_allreduce_adam_equals_torch_adam_on_mean_gradient():
    n, d, T = 4, 31, 6
    hp = O.Hyper(lr=1e-3, s=1)
    G = rand_grads(21, n, d, T)
    x0 = np.random.default_rng(0).standard_normal(d) * 0.02
    got = O.allreduce_adam(x0, lambda t: G[t], n, T, hp)
    p = torch.tensor(x0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([p], lr=hp.lr, betas=(hp.beta1, hp.beta2), eps=hp.eps)
    for t in range(1, T + 1):
        p.grad = torch.tensor(np.mean(G[t], axis=0), dtype=torch.float64)
        opt.step()
    np.testing.assert_allclose(got, p.detach().numpy(), rtol=1e-12, atol=1e-16)


def test_complete_topology_identical_gradients_follows_allreduce_adam():
    """w_ij = 1/N for all i, j, the same start and the same gradient on every worker:
    every replica follows All-Reduce Adam (Algorithm 2)."""
    n, d, T = 4, 31, 7
    hp = O.Hyper(lr=1e-3, s=1)
    rng = np.random.default_rng(5)
    x0 = rng.standard_normal(d) * 0.02
    g1 = rand_grads(22, 1, d, T)
    G = [[g1[t][0]] * n for t in range(T + 1)]
    st = O.run_simulation([x0] * n, lambda t: G[t], lambda t: csr_of(WL.complete(n), w64=True), T, hp, mode="O64")
    want = O.allreduce_adam(x0, lambda t: G[t], n, T, hp)
    for i in range(n):
        np.testing.assert_allclose(st.x_src[i], want, rtol=1e-12, atol=1e-15)


def test_complete_topology_different_gradients_disagree_by_one_direction():
    """With different gradients the replicas are not the All-Reduce result; what does
    hold is x_i - x_k = -lr (direction_i - direction_k) after every iteration."""
    n, d, T = 4, 9, 4
    hp = O.Hyper(lr=1e-2, s=1)
    rng = np.random.default_rng(6)
    x0 = rng.standard_normal(d)
    G = rand_grads(23, n, d, T, std=1.0)
    st = zeros_state([x0] * n)
    csr = csr_of(WL.complete(n), w64=True)
    for t in range(1, T + 1):
        U = [O.search_direction(*O.temporary_moments(st.m_hat[i], st.v_hat[i], G[t][i], hp), t, hp) for i in range(n)]
        st.x_src = O.dadam_step(st, G[t], csr, t, hp, mode="O64")
        np.testing.assert_allclose(st.x_src[0] - st.x_src[2], -hp.lr * (U[0] - U[2]), atol=1e-14)
    assert np.max(np.abs(st.x_src[0] - O.allreduce_adam(x0, lambda t: G[t], n, T, hp))) > 1e-4


# ---------------------------------------------------------------------------------------
# accumulation
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("s,T", [(4, 11), (2, 8), (3, 7)])
def test_accumulated_moments_closed_form(s, T):
    """m^(t) = (1-beta1)(g^(t) + beta1 G^(t_hat-1) + ... + beta1^(t_hat-1) G^(1)) with G the
    mean gradient of a finished loop (the closed form after Algorithm 3), and the same
    for v with beta2 and squares of the G's; b holds (1/s) * sum of the open loop."""
    d = 13
    hp = O.Hyper(lr=1e-3, beta1=0.9, beta2=0.99, eps=1e-8, s=s)
    G = rand_grads(31, 1, d, T, std=1.0)
    rng = np.random.default_rng(8)
    st = zeros_state([rng.standard_normal(d)])
    csr = csr_of(WL.identity(1))
    for t in range(1, T + 1):
        th = O.t_hat(t, s)
        Gbar = [np.mean([G[q][0] for q in range((k - 1) * s + 1, k * s + 1)], axis=0) for k in range(1, th)]
        m_want = (1 - hp.beta1) * (G[t][0] + sum(hp.beta1 ** q * Gbar[th - 1 - q] for q in range(1, th)))
        v_want = (1 - hp.beta2) * (G[t][0] ** 2 + sum(hp.beta2 ** q * Gbar[th - 1 - q] ** 2 for q in range(1, th)))
        x_prev = st.x_src[0]
        x_want = x_prev - hp.lr * (m_want / (1 - hp.beta1 ** th)) / (np.sqrt(v_want / (1 - hp.beta2 ** th)) + hp.eps)
        st.x_src = O.dadam_step(st, G[t], csr, t, hp, mode="O64")
        np.testing.assert_allclose(st.x_src[0], x_want, rtol=1e-11, atol=1e-14)
        r = t % s
        if r == 0:
            assert np.all(st.b[0] == 0.0)
        else:
            np.testing.assert_allclose(st.b[0], sum(G[q][0] for q in range(t - r + 1, t + 1)) / s, rtol=1e-13, atol=1e-16)


def test_hand_worked_trace():
    """tests/golden/hand_worked_accumadam.txt: three iterations of Algorithm 3 on two
    workers, derived by hand in exact fractions."""
    rows = {}
    with open(os.path.join(GOLDEN, "hand_worked_accumadam.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            t, q, a, b = line.split()
            rows[(int(t), q)] = (float(Fraction(a)), float(Fraction(b)))
    hp = O.Hyper(lr=1.0, beta1=0.5, beta2=0.75, eps=1.0, s=2)
    csr = O.Csr(np.array([0, 2, 4]), np.array([0, 1, 0, 1]), np.array([0.5, 0.5, 0.5, 0.5]))
    st = zeros_state([np.array([1.0]), np.array([3.0])])
    G = {1: (2.0, -2.0), 2: (4.0, 1.0), 3: (3.0, -0.5)}
    for t in (1, 2, 3):
        st.x_src = O.dadam_step(st, [np.array([G[t][0]]), np.array([G[t][1]])], csr, t, hp, mode="O64")
        for q, arr in (("x", st.x_src), ("b", st.b), ("m_hat", st.m_hat), ("v_hat", st.v_hat)):
            np.testing.assert_allclose([arr[0][0], arr[1][0]], rows[(t, q)], rtol=1e-15, atol=1e-16)


def test_unfused_halves_equal_fused_iteration():
    n, d, T = 3, 10, 5
    hp = O.Hyper(s=2)
    rng = np.random.default_rng(2)
    x0 = [rng.standard_normal(d) for _ in range(n)]
    G = rand_grads(41, n, d, T)
    csr = csr_of(WL.ring(n))
    a, b = zeros_state(x0), zeros_state(x0)
    for t in range(1, T + 1):
        a.x_src = O.dadam_step(a, G[t], csr, t, hp)
        xb = O.dadam_step(b, G[t], csr, t, hp, do_accumulate=False)
        assert O.dadam_step(b, G[t], csr, t, hp, do_update=False) is None
        b.x_src = xb
        for i in range(n):
            assert np.array_equal(a.x_src[i], b.x_src[i]) and np.array_equal(a.m_hat[i], b.m_hat[i])
            assert np.array_equal(a.v_hat[i], b.v_hat[i]) and np.array_equal(a.b[i], b.b[i])


def test_resume_from_saved_state_is_bit_identical():
    n, d, T, T1 = 4, 21, 9, 5
    hp = O.Hyper(s=4)
    rng = np.random.default_rng(13)
    x0 = [O.round_to_f32(rng.standard_normal(d) * 0.02) for _ in range(n)]
    G = rand_grads(42, n, d, T)
    csr = csr_of(WL.ring(n))
    full = O.run_simulation(x0, lambda t: G[t], lambda t: csr, T, hp)
    part = O.run_simulation(x0, lambda t: G[t], lambda t: csr, T1, hp)
    saved = copy.deepcopy(part)
    rest = O.run_simulation(x0, lambda t: G[t], lambda t: csr, T, hp, t_start=T1 + 1, state=saved)
    for i in range(n):
        for a, b in ((full.x_src, rest.x_src), (full.m_hat, rest.m_hat), (full.v_hat, rest.v_hat), (full.b, rest.b)):
            assert np.array_equal(a[i], b[i])


def test_zero_gradient_zero_state_gives_pure_mixing_without_nan():
    n, d = 4, 8
    rng = np.random.default_rng(14)
    x0 = [rng.standard_normal(d) for _ in range(n)]
    st = zeros_state(x0)
    csr = csr_of(WL.ring(n))
    out = O.dadam_step(st, [np.zeros(d)] * n, csr, 1, O.Hyper(s=2), mode="O64")
    want = O.mix_only(x0, csr, mode="O64")
    for i in range(n):
        assert np.all(np.isfinite(out[i])) and np.array_equal(out[i], want[i])


def test_o32m_rounds_state_to_storage_precision():
    n, d = 2, 50
    rng = np.random.default_rng(15)
    x0 = [rng.standard_normal(d) for _ in range(n)]
    G = rand_grads(43, n, d, 2)
    for dtype, rnd in (("f32", O.round_to_f32), ("bf16", O.round_to_bf16)):
        a, b = zeros_state(x0), zeros_state(x0)
        xa = O.dadam_step(a, G[1], csr_of(WL.ring(n)), 1, O.Hyper(s=1), mode="O64")
        xb = O.dadam_step(b, G[1], csr_of(WL.ring(n)), 1, O.Hyper(s=1), mode="O32m", param_dtype=dtype)
        for i in range(n):
            assert np.array_equal(xb[i], rnd(xa[i]))
            assert np.array_equal(b.m_hat[i], O.round_to_f32(a.m_hat[i]))
            assert np.array_equal(b.v_hat[i], O.round_to_f32(a.v_hat[i]))


def test_literal_beta1_in_fold_is_available_and_differs():
    """The printed line 12 decays v_hat with beta_1.  With that reading s = 1 does not
    give back Algorithm 1 (= the library's Adam), which is the evidence for taking it as a
    misprint; the literal form stays selectable."""
    d, T = 9, 4
    G = rand_grads(44, 1, d, T)
    x0 = [np.zeros(d)]
    csr = csr_of(WL.identity(1))
    a = O.run_simulation(x0, lambda t: G[t], lambda t: csr, T, O.Hyper(s=1), mode="O64")
    b = O.run_simulation(x0, lambda t: G[t], lambda t: csr, T, O.Hyper(s=1, beta_vhat=0.9), mode="O64")
    assert np.max(np.abs(a.v_hat[0] - b.v_hat[0]) / a.v_hat[0]) > 0.5
    # literal fold: v_hat = beta1 v_hat + (1-beta1) b^2
    np.testing.assert_allclose(b.v_hat[0], sum(0.9 ** (T - t) * 0.1 * G[t][0] ** 2 for t in range(1, T + 1)), rtol=1e-12)


# ---------------------------------------------------------------------------------------
# planted mistakes: the pins above must notice each of them
# ---------------------------------------------------------------------------------------

def _adam_pin_holds():
    try:
        test_identity_topology_s1_equals_torch_adam((0.9, 0.999))
        test_constant_gradient_closed_form(4)
        test_hand_worked_trace()
        test_accumulated_moments_closed_form(4, 11)
        return True
    except AssertionError:
        return False


def test_pins_catch_planted_mistakes(monkeypatch):
    assert _adam_pin_holds()

    def eps_inside(m, v, th, hp):
        return (m / (1 - hp.beta1 ** th)) / np.sqrt(v / (1 - hp.beta2 ** th) + hp.eps)
    def no_bias(m, v, th, hp):
        return m / (np.sqrt(v) + hp.eps)
    def swapped_betas(m_hat, v_hat, g, hp):
        return hp.beta2 * m_hat + (1 - hp.beta2) * g, hp.beta1 * v_hat + (1 - hp.beta1) * g * g
    def fold_mean_of_squares(m_hat, v_hat, b, g, t, hp):
        b = b + g / hp.s
        if t % hp.s == 0:
            m_hat = hp.beta1 * m_hat + (1 - hp.beta1) * b
            v_hat = hp.beta2 * v_hat + (1 - hp.beta2) * np.abs(b)   # dropped square
            b = np.zeros_like(b)
        return m_hat, v_hat, b
    def fold_never_clears(m_hat, v_hat, b, g, t, hp):
        b = b + g / hp.s
        if t % hp.s == 0:
            m_hat = hp.beta1 * m_hat + (1 - hp.beta1) * b
            v_hat = hp.beta2 * v_hat + (1 - hp.beta2) * b * b
        return m_hat, v_hat, b
    def t_instead_of_t_hat(t, s):
        return t
    for name, fn in (("search_direction", eps_inside), ("search_direction", no_bias),
                     ("temporary_moments", swapped_betas), ("accumulate_and_fold", fold_mean_of_squares),
                     ("accumulate_and_fold", fold_never_clears), ("t_hat", t_instead_of_t_hat)):
        with monkeypatch.context() as mp:
            mp.setattr(O, name, fn)
            assert not _adam_pin_holds(), f"planted mistake in {name} ({fn.__name__}) went unnoticed"


def test_mixing_pins_catch_planted_mistakes(monkeypatch):
    def transposed(x_src, csr):
        W = csr.dense(len(x_src)).T
        return [sum(W[i, j] * x_src[j] for j in range(len(x_src))) for i in range(csr.n_rows)]
    def first_weight_only(x_src, csr):
        return [sum(float(csr.w[csr.row_ptr[i]]) * x_src[int(csr.col[k])]
                    for k in range(csr.row_ptr[i], csr.row_ptr[i + 1])) for i in range(csr.n_rows)]
    for fn in (transposed, first_weight_only):
        with monkeypatch.context() as mp:
            mp.setattr(O, "mix_rows", fn)
            caught = 0
            for check in (test_mixing_equals_dense_matrix_per_coordinate,
                          lambda: test_permutation_matrix_copies_bit_exact_and_is_jacobi("f32")):
                try:
                    check()
                except AssertionError:
                    caught += 1
            assert caught >= 1, f"planted mistake {fn.__name__} went unnoticed"


# ---------------------------------------------------------------------------------------
# the other topologies the paper draws
# ---------------------------------------------------------------------------------------

def test_one_peer_ring_matchings():
    n = 16
    a, b = csr_of(WL.one_peer_ring(n, 0)).dense(n), csr_of(WL.one_peer_ring(n, 1)).dense(n)
    for W in (a, b):
        assert np.array_equal(W, W.T) and np.all(W.sum(0) == 1) and np.all(W.sum(1) == 1)
        assert np.all((W == 0) | (W == 0.5))
    assert a[0, 1] == 0.5 and a[14, 15] == 0.5 and a[1, 2] == 0       # (0,1), ..., (14,15)
    assert b[1, 2] == 0.5 and b[15, 0] == 0.5 and b[0, 1] == 0        # (1,2), ..., (15,0)
    # the union of the two matchings is the ring: every replica reaches every other one
    reach = np.linalg.matrix_power(((a + b) > 0).astype(float), n)
    assert np.all(reach > 0)


def test_alternating_exponential_ring_phases_and_exact_averaging():
    """Loops as drawn for 16 workers on four nodes; the four phases in a row average all
    replicas exactly (each phase is a group average; pairs (2,3), (0,1), (0,2), (1,3))."""
    m, n = 4, 16
    want_big = [set(range(8, 16)), set(range(0, 8)), {0, 1, 2, 3, 8, 9, 10, 11}, {4, 5, 6, 7, 12, 13, 14, 15}]
    prod = np.eye(n)
    rng = np.random.default_rng(17)
    x0 = [rng.standard_normal(6) for _ in range(n)]
    xs = [x.copy() for x in x0]
    for ph in range(4):
        groups = WL.aer_groups(m, ph)
        assert set(groups[0]) == want_big[ph] and sorted(len(g) for g in groups) == [4, 4, 8]
        assert sorted(i for g in groups for i in g) == list(range(n))
        csr = csr_of(WL.aer(m, ph), w64=True)
        W = csr.dense(n)
        assert np.allclose(W, W.T) and np.allclose(W.sum(0), 1) and np.allclose(W.sum(1), 1)
        for g in groups:
            for i in g:
                assert np.allclose(W[i, g], 1.0 / len(g)) and np.isclose(W[i].sum(), 1.0)
        prod = W @ prod
        xs = O.mix_only(xs, csr, mode="O64")
    np.testing.assert_allclose(prod, np.full((n, n), 1.0 / n), atol=1e-15)
    np.testing.assert_allclose(np.stack(xs), np.tile(np.mean(x0, axis=0), (n, 1)), atol=1e-14)


# ---------------------------------------------------------------------------------------
# decoupled weight decay (the AdamW-style variant)
# ---------------------------------------------------------------------------------------

def test_weight_decay_identity_s1_equals_torch_adamw():
    n, d, T, lam = 2, 101, 8, 3e-2
    hp = O.Hyper(lr=2e-3, s=1)
    rng = np.random.default_rng(71)
    x0 = [rng.standard_normal(d) for _ in range(n)]
    G = rand_grads(72, n, d, T)
    st = O.run_simulation(x0, lambda t: G[t], lambda t: csr_of(WL.identity(n)), T, hp, mode="O64", weight_decay=lam)
    for i in range(n):
        p = torch.tensor(x0[i], dtype=torch.float64, requires_grad=True)
        opt = torch.optim.AdamW([p], lr=hp.lr, betas=(hp.beta1, hp.beta2), eps=hp.eps, weight_decay=lam)
        for t in range(1, T + 1):
            p.grad = torch.tensor(G[t][i], dtype=torch.float64)
            opt.step()
        np.testing.assert_allclose(st.x_src[i], p.detach().numpy(), rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("s", [1, 4])
def test_weight_decay_constant_gradient_closed_form(s):
    """W = I, g = c: x_t = q^t x_0 - lr * c/(|c|+eps) * (1 - q^t)/(1 - q) with q = 1 - lr*lambda,
    for every accumulation length (the decay acts at every model update)."""
    hp = O.Hyper(lr=1e-2, eps=1e-3, s=s)
    lam = 0.5
    c = np.array([0.5, -0.25, 2.0, 0.0])
    x0 = [np.array([1.0, -2.0, 0.5, 3.0])]
    st = zeros_state(x0)
    q = 1.0 - hp.lr * lam
    for t in range(1, 10):
        st.x_src = O.dadam_step(st, [c], csr_of(WL.identity(1)), t, hp, mode="O64", weight_decay=lam)
        want = q ** t * x0[0] - hp.lr * c / (np.abs(c) + hp.eps) * (1 - q ** t) / (1 - q)
        np.testing.assert_allclose(st.x_src[0], want, rtol=1e-12, atol=1e-15)


def test_weight_decay_acts_on_own_previous_model_per_coordinate():
    """Ring, different replicas: x_new - mix + lr*u = -lr * lambda * x_own, coordinate by coordinate,
    with lambda zero on some coordinates (the recipe that exempts normalisation parameters)."""
    n, d = 4, 12
    hp = O.Hyper(lr=1e-2, s=2)
    rng = np.random.default_rng(73)
    x0 = [rng.standard_normal(d) for _ in range(n)]
    lam = np.where(np.arange(d) % 3 == 0, 0.0, 0.1)
    G = rand_grads(74, n, d, 3, std=1.0)
    csr = csr_of(WL.ring(n), w64=True)
    st = zeros_state(x0)
    for t in (1, 2, 3):
        prev = [x.copy() for x in st.x_src]
        mixes = O.mix_rows(prev, csr)
        U = [O.search_direction(*O.temporary_moments(st.m_hat[i], st.v_hat[i], G[t][i], hp), O.t_hat(t, hp.s), hp) for i in range(n)]
        st.x_src = O.dadam_step(st, G[t], csr, t, hp, mode="O64", weight_decay=lam)
        for i in range(n):
            np.testing.assert_allclose(st.x_src[i] - mixes[i] + hp.lr * U[i], -hp.lr * lam * prev[i], atol=1e-15)
        # averaged over workers the decay pulls the mean model (doubly stochastic W)
        np.testing.assert_allclose(np.mean(st.x_src, axis=0),
                                   np.mean(prev, axis=0) - hp.lr * np.mean([U[i] + lam * prev[i] for i in range(n)], axis=0), atol=1e-14)


# ---------------------------------------------------------------------------------------
# consensus error
# ---------------------------------------------------------------------------------------

def test_consensus_error_definition_and_decay():
    """Brute-force double loop on a tiny case; zero for equal replicas; invariant under a common
    shift; and with pure gossip on the 4-ring (all non-consensus eigenvalues +-1/3) it shrinks by
    exactly 1/9 per round, the lambda^2 rate of the consensus lemma."""
    rng = np.random.default_rng(91)
    n, d = 4, 7
    x = [rng.standard_normal(d) for _ in range(n)]
    want = 0.0
    for e in range(d):
        mean = sum(x[i][e] for i in range(n)) / n
        for i in range(n):
            want += (x[i][e] - mean) ** 2
    assert abs(O.consensus_error(x) - want) < 1e-13
    assert O.consensus_error([x[0]] * n) == 0.0
    assert abs(O.consensus_error([a + 5.0 for a in x]) - want) < 1e-12
    csr = csr_of(WL.ring(n), w64=True)
    err = O.consensus_error(x)
    for _ in range(6):
        x = O.mix_only(x, csr, mode="O64")
        new = O.consensus_error(x)
        np.testing.assert_allclose(new, err / 9.0, rtol=1e-12)
        err = new


def test_random_doubly_stochastic_matrices_properties():
    """Random doubly stochastic W (convex combinations of permutation matrices), random s, random
    degree: the replica mean follows the averaged-direction recursion, pure mixing never increases
    the consensus error, and s = 1 with any W leaves the accumulator empty."""
    from hypothesis import given, settings, strategies as st

    @settings(max_examples=40, deadline=None)
    @given(st.integers(2, 9), st.integers(1, 4), st.integers(1, 5), st.integers(0, 10 ** 6))
    def check(n, n_perm, s, seed):
        rng = np.random.default_rng(seed)
        W = np.zeros((n, n))
        coef = rng.random(n_perm) + 0.05
        coef /= coef.sum()
        for c in coef:
            W[np.arange(n), rng.permutation(n)] += c
        row_ptr, col, w = [0], [], []
        for i in range(n):
            nz = np.nonzero(W[i])[0]
            nz = rng.permutation(nz)                       # rows list their entries in any order
            col += list(nz); w += list(W[i, nz]); row_ptr.append(len(col))
        csr = O.Csr(np.array(row_ptr), np.array(col), np.array(w))
        d, T = 5, 2 * s + 1
        hp = O.Hyper(lr=1e-2, s=s)
        x = [rng.standard_normal(d) for _ in range(n)]
        st_ = zeros_state(x)
        G = [[rng.standard_normal(d) for _ in range(n)] for _ in range(T + 1)]
        e0 = O.consensus_error(x)
        assert O.consensus_error(O.mix_only(x, csr, mode="O64")) <= e0 * (1 + 1e-12)
        for t in range(1, T + 1):
            mean_prev = np.mean(st_.x_src, axis=0)
            U = [O.search_direction(*O.temporary_moments(st_.m_hat[i], st_.v_hat[i], G[t][i], hp), O.t_hat(t, s), hp) for i in range(n)]
            st_.x_src = O.dadam_step(st_, G[t], csr, t, hp, mode="O64")
            np.testing.assert_allclose(np.mean(st_.x_src, axis=0), mean_prev - hp.lr * np.mean(U, axis=0), atol=1e-13)
            if s == 1 or t % s == 0:
                assert all(np.all(b == 0) for b in st_.b)

    check()


# ---------------------------------------------------------------------------------------
# the error scales every relative tolerance of the parity tests is relative to
# ---------------------------------------------------------------------------------------

def test_error_scales_on_the_hand_worked_trace():
    """tests/golden/hand_worked_error_scales.txt: the scales of x, b, m_hat, v_hat on the hand-worked
    trace, in exact fractions (the scale of b and m_hat at t = 2 does not cancel where b itself does)."""
    rows = {}
    with open(os.path.join(GOLDEN, "hand_worked_error_scales.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            t, q, a, b = line.split()
            rows[(int(t), q)] = (float(Fraction(a)), float(Fraction(b)))
    hp = O.Hyper(lr=1.0, beta1=0.5, beta2=0.75, eps=1.0, s=2)
    csr = O.Csr(np.array([0, 2, 4]), np.array([0, 1, 0, 1]), np.array([0.5, 0.5, 0.5, 0.5]))
    st = zeros_state([np.array([1.0]), np.array([3.0])])
    G = {1: (2.0, -2.0), 2: (4.0, 1.0), 3: (3.0, -0.5)}
    for t in (1, 2, 3):
        g = [np.array([G[t][0]]), np.array([G[t][1]])]
        sx = O.magnitude_scale(st, g, csr, t, hp)
        sb, sm, sv = O.state_magnitude_scales(st, g, t, hp)
        for q, arr in (("S_x", sx), ("S_b", sb), ("S_m", sm), ("S_v", sv)):
            np.testing.assert_allclose([arr[0][0], arr[1][0]], rows[(t, q)], rtol=1e-15, atol=1e-16, err_msg=f"t={t} {q}")
        st.x_src = O.dadam_step(st, g, csr, t, hp, mode="O64")
    # weight decay adds lr * |lambda x_own| to the scale of x
    st = zeros_state([np.array([1.0]), np.array([3.0])])
    g = [np.array([2.0]), np.array([-2.0])]
    with_decay = O.magnitude_scale(st, g, csr, 1, hp, weight_decay=0.25)
    np.testing.assert_allclose([with_decay[0][0], with_decay[1][0]], [8 / 3 + 0.25, 8 / 3 + 0.75], rtol=1e-15)


def _float32_iteration(x_src, m_hat, v_hat, b, g, csr, t, hp):
    """One iteration evaluated the way a float32 implementation does: every operation rounded to
    float32 (NumPy float32 arithmetic, no fused operations), neighbour sum in list order."""
    f = np.float32
    th = O.t_hat(t, hp.s)
    inv_c1, inv_c2 = f(1.0 / (1.0 - hp.beta1 ** th)), f(1.0 / (1.0 - hp.beta2 ** th))
    b1, b2, bv, eps, lr, inv_s = f(hp.beta1), f(hp.beta2), f(hp.bv()), f(hp.eps), f(hp.lr), f(1.0 / hp.s)
    omb1, omb2, ombv = f(1.0 - hp.beta1), f(1.0 - hp.beta2), f(1.0 - hp.bv())
    xs, ms, vs, bs = [], [], [], []
    for i in range(csr.n_rows):
        mix = None
        for k in range(int(csr.row_ptr[i]), int(csr.row_ptr[i + 1])):
            term = f(csr.w[k]) * x_src[int(csr.col[k])].astype(f)
            mix = term if mix is None else mix + term
        gi, mh, vh, bi = g[i].astype(f), m_hat[i].astype(f), v_hat[i].astype(f), b[i].astype(f)
        m = b1 * mh + omb1 * gi
        v = b2 * vh + omb2 * (gi * gi)
        xs.append(mix - lr * ((m * inv_c1) / (np.sqrt(v * inv_c2) + eps)))
        bi = bi + gi * inv_s
        if t % hp.s == 0:
            mh = b1 * mh + omb1 * bi
            vh = bv * vh + ombv * (bi * bi)
            bi = np.zeros_like(bi)
        ms.append(mh); vs.append(vh); bs.append(bi)
    return xs, ms, vs, bs


@pytest.mark.parametrize("shared_init", [True, False])
def test_error_scales_bound_a_float32_evaluation_but_not_a_planted_error(shared_init):
    """What the tolerance 1e-6 x scale has to do: a float32 evaluation of an iteration (about a dozen
    roundings of 2^-24) stays inside it at every element of every iteration of two accumulation loops,
    with room to spare but not more than a factor of ten; a relative error of 2^-18 (3.8e-6) planted in
    x falls outside almost everywhere and one of 2^-19 (1.9e-6) still at nine elements in ten when the
    replicas are close together (as they are in a real run; elements whose terms cancel have a scale
    above their value, which is the point of the scale); in the moments and the accumulator, where
    the terms of a fold cancel more often, at six in ten at least.  A scale too small by a factor of
    five fails the first half, one too large by a factor of two the second."""
    n, d, s, T = 8, 4096, 4, 9
    hp = O.Hyper(lr=float(np.float32(1e-3)), beta1=float(np.float32(0.9)), beta2=float(np.float32(0.999)),
                 eps=float(np.float32(1e-8)), s=s)
    csr = csr_of(WL.ring(n))
    rng = np.random.default_rng(2410)
    common = rng.standard_normal(d) * 0.02
    x0 = [O.round_to_f32(common + (0.0 if not shared_init else 1e-4) * rng.standard_normal(d)) if shared_init
          else O.round_to_f32(rng.standard_normal(d) * 0.02) for _ in range(n)]
    st = zeros_state(x0)
    worst = {"x": 0.0, "m": 0.0, "v": 0.0, "b": 0.0}
    outside18 = {k: 1.0 for k in worst}
    outside19_x = 1.0
    for t in range(1, T + 1):
        g = [O.round_to_f32(rng.standard_normal(d) * 1e-2) for _ in range(n)]
        sx = O.magnitude_scale(st, g, csr, t, hp)
        sb, sm, sv = O.state_magnitude_scales(st, g, t, hp)
        f32 = _float32_iteration(st.x_src, st.m_hat, st.v_hat, st.b, g, csr, t, hp)
        ref_x = O.dadam_step(st, g, csr, t, hp, mode="O32m")          # advances st's moments and accumulator
        refs = {"x": ref_x, "m": st.m_hat, "v": st.v_hat, "b": st.b}
        for key, got, scale in (("x", f32[0], sx), ("m", f32[1], sm), ("v", f32[2], sv), ("b", f32[3], sb)):
            for i in range(n):
                ref, sc = refs[key][i], scale[i]
                live = sc > 0
                ratio = np.abs(got[i].astype(np.float64) - ref)[live] / (1e-6 * sc[live])
                worst[key] = max(worst[key], float(ratio.max(initial=0.0)))
                assert np.all(got[i][~live] == ref[~live])             # a zero scale means an exact zero
                if live.any():
                    planted = np.abs(ref * 2.0 ** -18)[live] / (1e-6 * sc[live])
                    changed = ref[live] != 0
                    outside18[key] = min(outside18[key], float(np.mean(planted[changed] > 1.0))) if changed.any() else outside18[key]
                    if key == "x":
                        outside19_x = min(outside19_x, float(np.mean(np.abs(ref * 2.0 ** -19)[live] / (1e-6 * sc[live]) > 1.0)))
        st.x_src = ref_x
    print("float32 evaluation, worst error / (1e-6 x scale):", worst, "planted 2^-18 outside:", outside18, "2^-19 (x):", outside19_x)
    for key, v in worst.items():
        assert v <= 1.0, f"{key}: a float32 evaluation is {v:.2f} x the tolerance away: the scale is too small"
        assert v >= 0.1 or key == "b", f"{key}: the worst float32 error is only {v:.3f} of the tolerance: the scale is too large"
    assert min(outside18["m"], outside18["v"], outside18["b"]) > 0.6, outside18
    if shared_init:
        # replicas close together: nothing cancels in the mixing sum, the scale of x is |x| plus the update
        assert outside18["x"] > 0.95 and outside19_x > 0.9, (outside18, outside19_x)
    else:
        # independent replicas: the mixing sum cancels in part, the scale is larger than |x| there
        assert outside18["x"] > 0.5, outside18
