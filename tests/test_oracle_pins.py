"""Pins for the CPU oracle: it is checked against what the paper and the mathematics fix,
never against itself.  Each test names the passage or fact it rests on.
"""
import os

import numpy as np
import pytest
import scipy.linalg

import oracle
from oracle import dense

TINY_SQUARE = [2, 3, 4, 5]
TINY_RECT = [(2, 3, 4, 2), (2, 4, 4, 4), (3, 2, 6, 5), (4, 3, 8, 2), (1, 5, 3, 4), (3, 4, 5, 2), (4, 2, 6, 3)]
READINGS = [oracle.READING_A, oracle.READING_B]


def _rand(rng, k, p, q, s, B=3):
    return (rng.standard_normal((B, k * p)), rng.standard_normal((k, q, p)),
            rng.standard_normal((k, s, q)), rng.standard_normal((B, k * s)))


# ---------------------------------------------------------------- forward ----

@pytest.mark.parametrize("reading", READINGS)
@pytest.mark.parametrize("shape", [(m, m, m, m) for m in TINY_SQUARE] + TINY_RECT)
def test_fwd_equals_literal_dense_product(shape, reading):
    """Def. 3.1: y = (P L P^T R) x with every factor materialised (brute force)."""
    k, p, q, s = shape
    rng = np.random.default_rng(hash(shape) % 1000 + reading)
    x, R, L, _ = _rand(rng, k, p, q, s)
    M = dense.monarch_dense(R, L, reading)
    assert M.shape == (k * s, k * p)
    assert oracle.rel_fro(oracle.fwd(x, R, L, reading), x @ M.T) < 1e-13


@pytest.mark.parametrize("m", TINY_SQUARE)
def test_square_dense_entries_match_equation_1(m):
    """Eq. (1): M[l*m+j, k*m+i] = L[j,l,k] R[k,j,i]; both readings coincide for k == q."""
    rng = np.random.default_rng(m)
    x, R, L, _ = _rand(rng, m, m, m, m, B=m * m)
    M = dense.eq1_dense_square(R, L)
    assert np.allclose(dense.monarch_dense(R, L, 0), M, rtol=0, atol=1e-14)
    assert np.allclose(dense.monarch_dense(R, L, 1), M, rtol=0, atol=1e-14)
    # columns of M through the oracle: fwd(I) = M^T
    eye = np.eye(m * m)
    for reading in READINGS:
        assert np.allclose(oracle.fwd(eye, R, L, reading), M.T, rtol=0, atol=1e-13)


def test_hand_fixture_square_m2(golden):
    g = golden("square_m2.txt")
    R = g["R"].reshape(2, 2, 2)
    L = g["L"].reshape(2, 2, 2)
    x = g["x"].reshape(1, 4)
    for reading in READINGS:
        assert np.array_equal(oracle.fwd(x, R, L, reading)[0], g["y"])
        assert np.array_equal(oracle.fwd(np.eye(4), R, L, reading).T, g["M"].reshape(4, 4))
    assert np.array_equal(dense.monarch_dense(R, L), g["M"].reshape(4, 4))


def test_hand_fixture_rectangular(golden):
    g = golden("rect_k2_p3_q4_s2.txt")
    R = g["R"].reshape(2, 4, 3)
    L = g["L"].reshape(2, 2, 4)
    x = g["x"].reshape(1, 6)
    assert np.array_equal(oracle.fwd(x, R, L, oracle.READING_A)[0], g["y_A"])
    assert np.array_equal(oracle.fwd(x, R, L, oracle.READING_B)[0], g["y_B"])
    # the permutation alone: identity L blocks are impossible here (s != q), so check pi directly
    UA = np.array([g["Y1"][oracle.pi(f, 2, 4, oracle.READING_A)] for f in range(8)])
    UB = np.array([g["Y1"][oracle.pi(f, 2, 4, oracle.READING_B)] for f in range(8)])
    assert np.array_equal(UA, g["U_A"]) and np.array_equal(UB, g["U_B"])


@pytest.mark.parametrize("m", [2, 3, 4, 7])
def test_identity_blocks_square_give_identity(m):
    """P = P^T is an involution (Section 3.1), so identity blocks give M = P P^T = I."""
    eye_blocks = np.broadcast_to(np.eye(m), (m, m, m)).copy()
    x = np.random.default_rng(m).standard_normal((4, m * m))
    for reading in READINGS:
        assert np.array_equal(oracle.fwd(x, eye_blocks, eye_blocks, reading), x)


def test_identity_blocks_rectangular_grid_give_pure_permutation():
    """k != q with identity blocks: reading A composes the same 'transpose a (k, .) grid' twice,
    reading B composes it with its inverse."""
    k, q = 2, 4
    eye_blocks = np.broadcast_to(np.eye(q), (k, q, q)).copy()
    x = np.arange(8, dtype=np.float64).reshape(1, 8)
    assert np.array_equal(oracle.fwd(x, eye_blocks, eye_blocks, oracle.READING_A)[0],
                          np.array([0, 2, 4, 6, 1, 3, 5, 7], dtype=np.float64))
    assert np.array_equal(oracle.fwd(x, eye_blocks, eye_blocks, oracle.READING_B)[0], x[0])
    # general (k, q): reading A == x.reshape(k,q).T.reshape(k,q).T (two grid transposes)
    for (k, q) in [(3, 6), (4, 8), (2, 5)]:
        eb = np.broadcast_to(np.eye(q), (k, q, q)).copy()
        x = np.random.default_rng(k * q).standard_normal((2, k * q))
        want = np.stack([row.reshape(k, q).T.ravel().reshape(k, q).T.ravel() for row in x])
        assert np.array_equal(oracle.fwd(x, eb, eb, oracle.READING_A), want)
        assert np.array_equal(oracle.fwd(x, eb, eb, oracle.READING_B), x)


@pytest.mark.parametrize("m", [2, 3, 4, 8])
def test_kronecker_special_case(m):
    """All R blocks = Bm, all L blocks = A  =>  M = A (x) Bm   (from Eq. 1:
    M[(l,j),(k,i)] = A[l,k] Bm[j,i]); numpy.kron is the independent routine."""
    rng = np.random.default_rng(10 + m)
    A = rng.standard_normal((m, m))
    Bm = rng.standard_normal((m, m))
    R = np.broadcast_to(Bm, (m, m, m)).copy()
    L = np.broadcast_to(A, (m, m, m)).copy()
    x = rng.standard_normal((5, m * m))
    assert oracle.rel_fro(oracle.fwd(x, R, L), x @ np.kron(A, Bm).T) < 1e-13


@pytest.mark.parametrize("m", [2, 4, 8, 16])
def test_hadamard_is_monarch(m):
    """Hadamard matrices are Monarch (Prop. 3.2 / butterfly containment): Sylvester
    H_n = H_m (x) H_m.  Checked against scipy's Hadamard matrix and a textbook fast
    Walsh-Hadamard transform; all values are small integers, so equality is exact."""
    H = scipy.linalg.hadamard(m).astype(np.float64)
    R = np.broadcast_to(H, (m, m, m)).copy()
    L = np.broadcast_to(H, (m, m, m)).copy()
    n = m * m
    rng = np.random.default_rng(m)
    x = rng.integers(-1, 2, size=(6, n)).astype(np.float64)
    y = oracle.fwd(x, R, L)
    assert np.array_equal(y, x @ scipy.linalg.hadamard(n).astype(np.float64).T)

    def fwht(v):
        v = v.copy()
        h = 1
        while h < len(v):
            for i in range(0, len(v), 2 * h):
                for j in range(i, i + h):
                    a, b = v[j], v[j + h]
                    v[j], v[j + h] = a + b, a - b
            h *= 2
        return v

    assert np.array_equal(y, np.stack([fwht(r) for r in x]))
    # H_n H_n = n I
    assert np.array_equal(oracle.fwd(y, R, L), n * x)


def test_single_block_is_two_dense_products():
    """k = 1: both permutations are trivial, y = L0 (R0 x)."""
    rng = np.random.default_rng(5)
    x, R, L, _ = _rand(rng, 1, 5, 3, 4, B=6)
    for reading in READINGS:
        assert oracle.rel_fro(oracle.fwd(x, R, L, reading), x @ R[0].T @ L[0].T) < 1e-14


@pytest.mark.parametrize("m", [3, 4])
def test_rank_one_slices_of_square_monarch(m):
    """Section 3.3: viewed as an m x m x m x m tensor, every slice M[:, j, k, :] has rank 1."""
    rng = np.random.default_rng(m)
    _, R, L, _ = _rand(rng, m, m, m, m)
    M = oracle.fwd(np.eye(m * m), R, L).T.reshape(m, m, m, m)  # [l, j, k, i]
    for j in range(m):
        for k in range(m):
            sv = np.linalg.svd(M[:, j, k, :], compute_uv=False)
            assert sv[1] < 1e-12 * sv[0]


def test_parameter_and_sparsity_count():
    """Section 3.2.2: a square Monarch matrix has 2 n sqrt(n) parameters; with generic
    factors every entry of M is a single product (Eq. 1) and therefore non-zero."""
    m = 4
    rng = np.random.default_rng(0)
    _, R, L, _ = _rand(rng, m, m, m, m)
    assert R.size + L.size == 2 * (m * m) * m
    assert np.count_nonzero(oracle.fwd(np.eye(m * m), R, L)) == (m * m) ** 2


@pytest.mark.parametrize("reading", READINGS)
def test_forward_is_linear_in_each_argument(reading):
    rng = np.random.default_rng(3)
    k, p, q, s = 3, 4, 6, 5
    x, R, L, _ = _rand(rng, k, p, q, s)
    x2, R2, L2, _ = _rand(rng, k, p, q, s)
    a, b = 0.7, -1.3
    f = lambda x_, R_, L_: oracle.fwd(x_, R_, L_, reading)
    assert oracle.rel_fro(f(a * x + b * x2, R, L), a * f(x, R, L) + b * f(x2, R, L)) < 1e-13
    assert oracle.rel_fro(f(x, a * R + b * R2, L), a * f(x, R, L) + b * f(x, R2, L)) < 1e-13
    assert oracle.rel_fro(f(x, R, a * L + b * L2), a * f(x, R, L) + b * f(x, R, L2)) < 1e-13


def test_readings_are_inverse_permutations():
    for (k, q) in [(2, 4), (3, 6), (4, 48), (5, 3), (4, 4)]:
        A = [oracle.pi(f, k, q, 0) for f in range(k * q)]
        Bp = [oracle.pi(f, k, q, 1) for f in range(k * q)]
        assert sorted(A) == list(range(k * q))
        assert all(Bp[A[f]] == f for f in range(k * q))
        if k == q:
            assert A == Bp


# --------------------------------------------------------------- backward ----

@pytest.mark.parametrize("reading", READINGS)
@pytest.mark.parametrize("shape", [(2, 2, 2, 2), (3, 3, 3, 3)] + TINY_RECT)
def test_bwd_matches_unit_step_finite_differences(shape, reading):
    """loss = <dy, fwd(x; R, L)> is linear in each argument, so a one-sided difference
    with step 1 in a single coordinate is the exact partial derivative."""
    k, p, q, s = shape
    rng = np.random.default_rng(sum(shape) + reading)
    x, R, L, dy = _rand(rng, k, p, q, s, B=2)
    dx, dR, dL = oracle.bwd(dy, x, R, L, reading)
    base = float(np.sum(dy * oracle.fwd(x, R, L, reading)))

    def loss(x_, R_, L_):
        return float(np.sum(dy * oracle.fwd(x_, R_, L_, reading)))

    for arr, grad, which in ((x, dx, 0), (R, dR, 1), (L, dL, 2)):
        flat = arr.reshape(-1)
        g = grad.reshape(-1)
        for e in range(flat.size):
            old = flat[e]
            flat[e] = old + 1.0
            fd = loss(x, R, L) - base
            flat[e] = old
            assert abs(fd - g[e]) <= 1e-10 * max(1.0, abs(g[e])), (which, e, fd, g[e])


@pytest.mark.parametrize("reading", READINGS)
@pytest.mark.parametrize("shape", [(3, 3, 3, 3)] + TINY_RECT)
def test_bwd_matches_autograd_through_literal_definition(shape, reading):
    """Independent derivation: torch autograd (float64, CPU) through the explicit dense
    product Pout BD(L) Pmid BD(R) of Def. 3.1."""
    torch = pytest.importorskip("torch")
    k, p, q, s = shape
    rng = np.random.default_rng(7 * sum(shape) + reading)
    x, R, L, dy = _rand(rng, k, p, q, s, B=4)
    xt, Rt, Lt = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (x, R, L))
    Pmid = torch.tensor(dense.mid_perm(k, q, reading))
    Pout = torch.tensor(dense.out_perm(k, s))
    M = Pout @ torch.block_diag(*Lt) @ Pmid @ torch.block_diag(*Rt)
    y = xt @ M.T
    y.backward(torch.tensor(dy))
    dx, dR, dL = oracle.bwd(dy, x, R, L, reading)
    assert oracle.rel_fro(dx, xt.grad.numpy()) < 1e-13
    assert oracle.rel_fro(dR, Rt.grad.numpy()) < 1e-13
    assert oracle.rel_fro(dL, Lt.grad.numpy()) < 1e-13


@pytest.mark.parametrize("reading", READINGS)
def test_dx_is_the_transposed_dense_matrix(reading):
    rng = np.random.default_rng(11)
    k, p, q, s = 4, 3, 8, 2
    x, R, L, dy = _rand(rng, k, p, q, s, B=5)
    dx, _, _ = oracle.bwd(dy, x, R, L, reading)
    assert oracle.rel_fro(dx, dy @ dense.monarch_dense(R, L, reading)) < 1e-13


@pytest.mark.parametrize("shape", [(4, 4, 4, 4), (4, 12, 8, 20), (2, 6, 10, 4)])
def test_adjoint_and_euler_identities(shape):
    """<dy, y> = <dx, x> = <dR, R> = <dL, L> for the form that is linear in x, R and L."""
    k, p, q, s = shape
    rng = np.random.default_rng(sum(shape))
    x, R, L, dy = _rand(rng, k, p, q, s, B=9)
    for reading in READINGS:
        y = oracle.fwd(x, R, L, reading)
        dx, dR, dL = oracle.bwd(dy, x, R, L, reading)
        ref = np.sum(dy * y)
        for v in (np.sum(dx * x), np.sum(dR * R), np.sum(dL * L)):
            assert abs(v - ref) < 1e-11 * abs(ref)


def test_bwd_square_matches_einsum_of_section_3_3():
    """Square case: z[l,j] = sum_{k,i} L[j,l,k] R[k,j,i] x[k,i]  (Section 3.3) differentiated
    by hand: dR[k,j,i] = sum_b x[b,k,i] sum_l L[j,l,k] dz[b,l,j], etc., written as einsums."""
    m = 4
    rng = np.random.default_rng(2)
    x, R, L, dy = _rand(rng, m, m, m, m, B=6)
    X = x.reshape(-1, m, m)
    dZ = dy.reshape(-1, m, m)
    y = np.einsum("jlk,kji,bki->blj", L, R, X).reshape(-1, m * m)
    assert oracle.rel_fro(oracle.fwd(x, R, L), y) < 1e-13
    dx, dR, dL = oracle.bwd(dy, x, R, L)
    assert oracle.rel_fro(dx, np.einsum("jlk,kji,blj->bki", L, R, dZ).reshape(-1, m * m)) < 1e-13
    assert oracle.rel_fro(dR, np.einsum("jlk,bki,blj->kji", L, X, dZ)) < 1e-13
    assert oracle.rel_fro(dL, np.einsum("kji,bki,blj->jlk", R, X, dZ)) < 1e-13


def test_empty_batch_and_bad_shapes():
    R = np.zeros((2, 4, 3))
    L = np.zeros((2, 2, 4))
    assert oracle.fwd(np.zeros((0, 6)), R, L).shape == (0, 4)
    dx, dR, dL = oracle.bwd(np.zeros((0, 4)), np.zeros((0, 6)), R, L)
    assert dx.shape == (0, 6) and not dR.any() and not dL.any()
    with pytest.raises(ValueError):
        oracle.fwd(np.zeros((1, 5)), R, L)
    with pytest.raises(ValueError):
        oracle.fwd(np.zeros((1, 6)), R, np.zeros((2, 2, 5)))


def test_thread_count_changes_only_the_summation_order(tmp_path):
    """The OpenMP split is over rows only.  Run the same backward in fresh processes with 1, 3 and 8
    threads: y and dx are row-local and must agree bit for bit; dR and dL are sums of per-thread
    partials, so they may differ in the order of fp64 additions only (<= 1e-13 relative), and two
    runs at the same thread count must agree bit for bit."""
    import subprocess
    import sys
    script = (
        "import sys, numpy as np\n"
        "sys.path.insert(0, %r)\n"
        "import oracle\n"
        "rng = np.random.default_rng(9)\n"
        "k, p, q, s, B = 4, 8, 8, 8, 37\n"
        "x = rng.standard_normal((B, k * p)); R = rng.standard_normal((k, q, p))\n"
        "L = rng.standard_normal((k, s, q)); dy = rng.standard_normal((B, k * s))\n"
        "y = oracle.fwd(x, R, L); dx, dR, dL = oracle.bwd(dy, x, R, L)\n"
        "np.savez(sys.argv[1], y=y, dx=dx, dR=dR, dL=dL, threads=oracle.num_threads())\n"
    ) % os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    runs = {}
    for tag, threads in (("t1", 1), ("t3", 3), ("t8", 8), ("t3_again", 3)):
        out = str(tmp_path / (tag + ".npz"))
        env = dict(os.environ, OMP_NUM_THREADS=str(threads))
        subprocess.check_call([sys.executable, "-c", script, out], env=env)
        runs[tag] = np.load(out)
        assert int(runs[tag]["threads"]) == threads
    base = runs["t1"]
    for tag in ("t3", "t8"):
        assert np.array_equal(runs[tag]["y"], base["y"]) and np.array_equal(runs[tag]["dx"], base["dx"]), tag
        for name in ("dR", "dL"):
            assert oracle.rel_fro(runs[tag][name], base[name]) < 1e-13, (tag, name)
    for name in ("y", "dx", "dR", "dL"):
        assert np.array_equal(runs["t3"][name], runs["t3_again"][name]), name


# ------------------------------------------------------------ affine layer ----

@pytest.mark.parametrize("reading", READINGS)
@pytest.mark.parametrize("shape", [(3, 3, 3, 3)] + TINY_RECT[:4])
def test_bias_forward_is_the_dense_affine_map(shape, reading):
    """y = x M^T + 1 bias^T with M the literal dense product of Definition 3.1; a zero input returns
    the bias itself and a zero bias returns the plain multiply."""
    k, p, q, s = shape
    rng = np.random.default_rng(31)
    x, R, L, _ = _rand(rng, k, p, q, s, B=4)
    bias = rng.standard_normal(k * s)
    M = dense.monarch_dense(R, L, reading)
    want = x @ M.T + np.ones((4, 1)) @ bias[None, :]
    assert np.allclose(oracle.fwd_bias(x, R, L, bias, reading), want, rtol=0, atol=1e-12)
    assert np.array_equal(oracle.fwd_bias(np.zeros_like(x), R, L, bias, reading), np.tile(bias, (4, 1)))
    assert np.array_equal(oracle.fwd_bias(x, R, L, np.zeros(k * s), reading), oracle.fwd(x, R, L, reading))


@pytest.mark.parametrize("shape", [(2, 2, 2, 2), (3, 2, 6, 5)])
def test_bias_gradient_matches_unit_step_differences(shape):
    """The loss <dy, y> is linear in the bias, so a unit step in coordinate o changes it by exactly
    dbias[o] (up to rounding); the other gradients are those of the plain multiply."""
    k, p, q, s = shape
    rng = np.random.default_rng(32)
    x, R, L, dy = _rand(rng, k, p, q, s, B=5)
    bias = rng.standard_normal(k * s)
    dx, dR, dL, db = oracle.bwd_bias(dy, x, R, L)
    base = np.sum(dy * oracle.fwd_bias(x, R, L, bias))
    for o in range(k * s):
        step = bias.copy()
        step[o] += 1.0
        assert abs(np.sum(dy * oracle.fwd_bias(x, R, L, step)) - base - db[o]) < 1e-11
    for got, want in zip((dx, dR, dL), oracle.bwd(dy, x, R, L)):
        assert np.array_equal(got, want)
    # brute force, and the all-ones upstream gradient counts the rows
    assert np.allclose(db, [sum(dy[b, o] for b in range(5)) for o in range(k * s)], rtol=0, atol=1e-14)
    assert np.array_equal(oracle.bwd_bias(np.ones_like(dy), x, R, L)[3], np.full(k * s, 5.0))


# -------------------------------------------------- projection (Algorithm 1) ----

from oracle import project  # noqa: E402


@pytest.mark.parametrize("m", [1, 2, 3, 4, 6])
def test_projection_recovers_a_monarch_matrix(m):
    """If A is itself Monarch the projection returns factors with P L P^T R = A (remark after
    Theorem 1); A is built by the literal dense product, which shares nothing with the projection."""
    rng = np.random.default_rng(40 + m)
    R0, L0 = rng.standard_normal((m, m, m)), rng.standard_normal((m, m, m))
    A = dense.monarch_dense(R0, L0)
    L, R = project.project_square(A)
    assert np.allclose(dense.monarch_dense(R, L), A, rtol=0, atol=1e-12)
    assert np.allclose(project.monarch_square(L, R), A, rtol=0, atol=1e-12)  # the einsum helper agrees with Eq. (1)
    assert np.allclose(project.monarch_square(L0, R0), dense.eq1_dense_square(R0, L0), rtol=0, atol=1e-14)


def test_projection_of_a_hand_made_matrix():
    """m = 2, slices with known singular triples: slice (j, k) = a_jk * e_(j) e_(k)^T + small second
    term orthogonal to it, so the best rank-1 part can be read off."""
    m = 2
    At = np.zeros((m, m, m, m))
    big = {(0, 0): 3.0, (0, 1): -2.0, (1, 0): 5.0, (1, 1): 0.5}
    for (j, k), a in big.items():
        # singular triples: sigma_1 = |a| on (e_j, e_k), sigma_2 = 0.25 on the other basis vectors
        At[j, j, k, k] = a
        At[1 - j, j, k, 1 - k] = 0.25
    A = At.reshape(4, 4)
    L, R = project.project_square(A)
    M = project.monarch_square(L, R).reshape(m, m, m, m)
    want = np.zeros_like(At)
    for (j, k), a in big.items():
        want[j, j, k, k] = a
    assert np.allclose(M, want, rtol=0, atol=1e-14)
    assert abs(np.sum((A - M.reshape(4, 4)) ** 2) - 4 * 0.25 ** 2) < 1e-14


def test_projection_residual_for_two_by_two_slices_has_the_closed_form():
    """m = 2: a 2 x 2 matrix with Frobenius norm^2 T and determinant D has sigma_2^2 =
    (T - sqrt(T^2 - 4 D^2)) / 2, so the optimal objective of Equation (2)'s problem is the sum of that
    over the four slices."""
    rng = np.random.default_rng(77)
    A = rng.standard_normal((4, 4))
    L, R = project.project_square(A)
    At = A.reshape(2, 2, 2, 2)
    want = 0.0
    for j in range(2):
        for k in range(2):
            S = At[:, j, k, :]
            T, D = np.sum(S * S), S[0, 0] * S[1, 1] - S[0, 1] * S[1, 0]
            want += (T - np.sqrt(T * T - 4 * D * D)) / 2
    got = np.sum((A - project.monarch_square(L, R)) ** 2)
    assert abs(got - want) < 1e-12


@pytest.mark.parametrize("m", [2, 3, 5])
def test_projection_is_stationary_and_not_beaten_by_perturbations(m):
    """Optimality (Theorem 1): at the returned factors every slice's residual E satisfies E v = 0 and
    E^T u = 0 (the normal equations of the rank-1 problem), and no perturbed pair of factors, small or
    large, comes closer to A."""
    rng = np.random.default_rng(90 + m)
    n = m * m
    A = rng.standard_normal((n, n))
    L, R = project.project_square(A)
    E = (A - project.monarch_square(L, R)).reshape(m, m, m, m)
    for j in range(m):
        for k in range(m):
            assert np.allclose(E[:, j, k, :] @ R[k, j, :], 0, atol=1e-12)
            assert np.allclose(E[:, j, k, :].T @ L[j, :, k], 0, atol=1e-12)
    best = np.sum(E ** 2)
    for scale in (1e-4, 1e-2, 0.3, 1.0):
        for _ in range(20):
            Lp = L + scale * rng.standard_normal(L.shape)
            Rp = R + scale * rng.standard_normal(R.shape)
            assert np.sum((A - project.monarch_square(Lp, Rp)) ** 2) >= best - 1e-12


# ------------------------------------------------- transposed multiply (M*) ----

@pytest.mark.parametrize("reading", READINGS)
@pytest.mark.parametrize("shape", [(3, 3, 3, 3)] + TINY_RECT)
def test_transposed_multiply_is_the_dense_transpose(shape, reading):
    """fwd_t(x) = x M with M the literal dense product of Definition 3.1, and it is the adjoint of the
    multiply: <fwd_t(x), z> = <x, fwd(z)>."""
    k, p, q, s = shape
    rng = np.random.default_rng(55)
    z, R, L, x = _rand(rng, k, p, q, s, B=4)   # z (4, k*p), x (4, k*s)
    M = dense.monarch_dense(R, L, reading)
    got = oracle.fwd_t(x, R, L, reading)
    assert np.allclose(got, x @ M, rtol=0, atol=1e-12)
    assert abs(np.sum(got * z) - np.sum(x * oracle.fwd(z, R, L, reading))) < 1e-10


def test_hadamard_monarch_times_its_transpose_is_n_times_identity():
    """M = H_n (all blocks H_m, Sylvester) is in the class M, and M M* = n I (the Hadamard transform
    is in MM*, Proposition 3.2): applying M* and then M multiplies every vector by n, exactly."""
    m = 8
    H = scipy.linalg.hadamard(m).astype(np.float64)
    blocks = np.broadcast_to(H, (m, m, m)).copy()
    rng = np.random.default_rng(56)
    x = rng.integers(-3, 4, size=(5, m * m)).astype(np.float64)
    assert np.array_equal(oracle.fwd(oracle.fwd_t(x, blocks, blocks), blocks, blocks), m * m * x)


# ------------------------------------------------------- complex-valued Monarch ----

from oracle import complex_ref  # noqa: E402


def _crand(rng, *shape):
    return rng.standard_normal(shape) + 1j * rng.standard_normal(shape)


@pytest.mark.parametrize("reading", READINGS)
@pytest.mark.parametrize("shape", [(3, 3, 3, 3)] + TINY_RECT[:4])
def test_complex_forward_is_the_literal_dense_product(shape, reading):
    """Definition 3.1 with complex blocks: M = Pout BD(L) Pmid BD(R) from explicit permutation matrices
    and scipy's block_diag; real inputs reduce to the real oracle."""
    k, p, q, s = shape
    rng = np.random.default_rng(61)
    x, R, L = _crand(rng, 4, k * p), _crand(rng, k, q, p), _crand(rng, k, s, q)
    M = dense.out_perm(k, s) @ scipy.linalg.block_diag(*L) @ dense.mid_perm(k, q, reading) @ scipy.linalg.block_diag(*R)
    assert np.allclose(complex_ref.fwd(x, R, L, reading), x @ M.T, rtol=0, atol=1e-12)
    got = complex_ref.fwd(x.real, R.real, L.real, reading)
    assert np.allclose(got.imag, 0) and np.allclose(got.real, oracle.fwd(x.real, R.real, L.real, reading), rtol=0, atol=1e-12)


@pytest.mark.parametrize("reading", READINGS)
@pytest.mark.parametrize("shape", [(3, 3, 3, 3)] + TINY_RECT[:4])
def test_conjugate_transpose_apply_is_the_dense_adjoint(shape, reading):
    """M* of Section 3.1 (conjugate transpose): against x conj(M) with the literal dense M; the adjoint identity
    <M a, b> = <a, M* b> of the Hermitian inner product; real factors reduce to the real transposed multiply."""
    k, p, q, s = shape
    rng = np.random.default_rng(63)
    a, b = _crand(rng, 4, k * p), _crand(rng, 4, k * s)
    R, L = _crand(rng, k, q, p), _crand(rng, k, s, q)
    M = dense.out_perm(k, s) @ scipy.linalg.block_diag(*L) @ dense.mid_perm(k, q, reading) @ scipy.linalg.block_diag(*R)
    assert np.allclose(complex_ref.fwd_h(b, R, L, reading), b @ np.conj(M), rtol=0, atol=1e-12)
    lhs = np.sum(complex_ref.fwd(a, R, L, reading) * np.conj(b), axis=1)          # <M a, b>, conjugate-linear in b
    rhs = np.sum(a * np.conj(complex_ref.fwd_h(b, R, L, reading)), axis=1)        # <a, M* b>
    assert np.allclose(lhs, rhs, rtol=0, atol=1e-11)
    got = complex_ref.fwd_h(b.real, R.real, L.real, reading)
    assert np.allclose(got.imag, 0) and np.allclose(got.real, oracle.fwd_t(b.real, R.real, L.real, reading), rtol=0, atol=1e-12)


@pytest.mark.parametrize("m", [2, 3, 4, 8])
def test_unitary_dft_monarch_times_its_conjugate_transpose_is_n(m):
    """F F* = n I: the DFT factors applied, then their conjugate transpose, return n times the input (the grid
    transposition inside the Monarch form is a permutation and cancels with its own transpose)."""
    n = m * m
    rng = np.random.default_rng(64)
    x = _crand(rng, 3, n)
    R, L = complex_ref.dft_factors(m)
    assert np.allclose(complex_ref.fwd_h(complex_ref.fwd(x, R, L), R, L), n * x, rtol=0, atol=1e-9 * n)


@pytest.mark.parametrize("m", [2, 3, 4, 8])
def test_dft_is_a_monarch_matrix(m):
    """The 4-step splitting: Monarch(dft_factors) applied to x equals the library FFT of the grid-
    transposed input, and the inverse factors undo it."""
    n = m * m
    rng = np.random.default_rng(62)
    x = _crand(rng, 5, n)
    xt = x.reshape(5, m, m).transpose(0, 2, 1).reshape(5, n)
    R, L = complex_ref.dft_factors(m)
    assert np.allclose(complex_ref.fwd(x, R, L), np.fft.fft(xt, axis=1), rtol=0, atol=1e-10)
    Ri, Li = complex_ref.dft_factors(m, inverse=True)
    assert np.allclose(complex_ref.fwd(x, Ri, Li), np.fft.ifft(xt, axis=1), rtol=0, atol=1e-12)


@pytest.mark.parametrize("reading", READINGS)
@pytest.mark.parametrize("shape", [(2, 2, 2, 2), (3, 2, 4, 2)])
def test_complex_gradients_match_unit_step_differences(shape, reading):
    """Loss = Re <dy, y> = sum Re(conj(dy) y) is real and linear in each of x, R, L: a unit step in the
    real (imaginary) part of a coordinate changes it by the real (imaginary) part of the gradient."""
    k, p, q, s = shape
    rng = np.random.default_rng(63)
    x, R, L, dy = _crand(rng, 3, k * p), _crand(rng, k, q, p), _crand(rng, k, s, q), _crand(rng, 3, k * s)
    loss = lambda x_, R_, L_: float(np.sum((np.conj(dy) * complex_ref.fwd(x_, R_, L_, reading)).real))
    base = loss(x, R, L)
    grads = complex_ref.bwd(dy, x, R, L, reading)
    for which, (arr, g) in enumerate(zip((x, R, L), grads)):
        for idx in np.ndindex(arr.shape):
            for step, part in ((1.0, g[idx].real), (1j, g[idx].imag)):
                moved = arr.copy()
                moved[idx] += step
                args = [x, R, L]
                args[which] = moved
                assert abs(loss(*args) - base - part) < 1e-10, (which, idx, step)


# ----------------------------------------------------- the block's nonlinearity ----

def test_gelu_tanh_form_against_the_exact_form_and_the_library():
    """gelu(v) = v Phi(v) (Hendrycks & Gimpel) with Phi from scipy's erf; the tanh form stays within 1e-3
    of it; torch's own tanh-form routine (float64, CPU) agrees to rounding."""
    import scipy.special
    torch = pytest.importorskip("torch")
    from oracle import activation
    v = np.linspace(-12.0, 12.0, 4801)
    exact = 0.5 * v * (1.0 + scipy.special.erf(v / np.sqrt(2.0)))
    got = activation.gelu(v)
    assert np.max(np.abs(got - exact)) < 1e-3
    assert np.max(np.abs(got - exact)) > 1e-5  # it is the approximation, not the exact form
    lib = torch.nn.functional.gelu(torch.tensor(v, dtype=torch.float64), approximate="tanh").numpy()
    assert np.max(np.abs(got - lib)) < 1e-14


def test_gelu_special_values_and_reflection_identity():
    """gelu(0) = 0, gelu(v) -> v and gelu(-v) -> 0 for large v; tanh is odd, so
    gelu(v) - gelu(-v) = v exactly, and differentiating that, gelu'(v) + gelu'(-v) = 1; gelu'(0) = 1/2."""
    from oracle import activation
    assert activation.gelu(0.0) == 0.0
    assert abs(activation.gelu(20.0) - 20.0) < 1e-12 and abs(activation.gelu(-20.0)) < 1e-12
    v = np.linspace(0.0, 9.0, 901)
    assert np.max(np.abs(activation.gelu(v) - activation.gelu(-v) - v)) < 1e-14
    assert np.max(np.abs(activation.gelu_grad(v) + activation.gelu_grad(-v) - 1.0)) < 1e-14
    assert activation.gelu_grad(0.0) == 0.5
    # the minimum of gelu sits where its derivative changes sign, near v = -0.75 (value about -0.17)
    vv = np.linspace(-2.0, 0.0, 20001)
    i = int(np.argmin(activation.gelu(vv)))
    assert abs(vv[i] + 0.7525) < 2e-3 and abs(activation.gelu(vv[i]) + 0.17) < 1e-3
    assert abs(activation.gelu_grad(vv[i])) < 1e-3


def test_gelu_grad_matches_central_differences():
    from oracle import activation
    v = np.linspace(-6.0, 6.0, 241)
    h = 1e-5
    fd = (activation.gelu(v + h) - activation.gelu(v - h)) / (2 * h)
    assert np.max(np.abs(activation.gelu_grad(v) - fd)) < 1e-9


@pytest.mark.parametrize("reading", READINGS)
@pytest.mark.parametrize("shape", [(3, 3, 3, 3)] + TINY_RECT[:4])
def test_layer_with_gelu_matches_autograd_through_the_dense_matrix(shape, reading):
    """Both layers of a feed-forward block in one graph, float64 torch on the CPU, with the explicit dense
    matrices: h = x M1^T + b1, g = gelu(h), y = g M2^T + b2.  The first layer's forward gives (h, g); the
    second layer's backward at input g = gelu(h) gives d/dh, dR2, dL2, db2."""
    torch = pytest.importorskip("torch")
    from oracle import activation
    k, p, q, s = shape
    rng = np.random.default_rng(101 + 13 * sum(shape) + reading)
    B = 4
    x, R1, L1, _ = _rand(rng, k, p, q, s, B=B)
    b1 = rng.standard_normal(k * s)
    # second layer: n_in = k*s -> blocks of p2 = s inputs, q outputs, then p outputs per block
    R2, L2 = rng.standard_normal((k, q, s)), rng.standard_normal((k, p, q))
    b2 = rng.standard_normal(k * p)
    dy = rng.standard_normal((B, k * p))

    h, g = activation.fwd_bias_gelu(x, R1, L1, b1, reading)
    M1 = torch.tensor(dense.monarch_dense(R1, L1, reading))
    ht = torch.tensor(x) @ M1.T + torch.tensor(b1)
    assert oracle.rel_fro(h, ht.numpy()) < 1e-13
    assert oracle.rel_fro(g, torch.nn.functional.gelu(ht, approximate="tanh").numpy()) < 1e-13

    hl = torch.tensor(h, requires_grad=True)
    R2t, L2t, b2t = (torch.tensor(a, requires_grad=True) for a in (R2, L2, b2))
    Pmid = torch.tensor(dense.mid_perm(k, q, reading))
    Pout = torch.tensor(dense.out_perm(k, p))
    M2 = Pout @ torch.block_diag(*L2t) @ Pmid @ torch.block_diag(*R2t)
    y = torch.nn.functional.gelu(hl, approximate="tanh") @ M2.T + b2t
    y.backward(torch.tensor(dy))
    dh, dR2, dL2, db2 = activation.bwd_bias_gelu_in(dy, h, R2, L2, reading)
    assert oracle.rel_fro(dh, hl.grad.numpy()) < 1e-13
    assert oracle.rel_fro(dR2, R2t.grad.numpy()) < 1e-13
    assert oracle.rel_fro(dL2, L2t.grad.numpy()) < 1e-13
    assert oracle.rel_fro(db2, b2t.grad.numpy()) < 1e-13
