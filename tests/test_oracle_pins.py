"""Pins for the CPU oracle: each checks oracle/powersgd_oracle.py against
something other than itself (a library routine on a different algorithm,
a closed form, an invariant of the method, values derived by hand, numbers the
paper prints).  None of these needs a GPU.
"""
import os

import numpy as np
import pytest

from oracle import powersgd_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def planted(n, m, s, seed):
    g = rng(seed)
    k = len(s)
    U, _ = np.linalg.qr(g.standard_normal((n, k)))
    V, _ = np.linalg.qr(g.standard_normal((m, k)))
    return (U * np.asarray(s)[None, :]) @ V.T


def one_step(M, Q, r=None, E=None):
    """W = 1 step on a single matrix through the public step function."""
    r = Q.shape[1] if r is None else r
    E = np.zeros_like(M) if E is None else E
    res = O.powersgd_step([[M]], [[E]], [Q], r)
    return res["P_hat"][0], res["Q"][0], res["out"][0], res["err"][0][0]


# -- (i) library-routine reduction: Householder QR + least-squares projection --

@pytest.mark.parametrize("n,m,r,seed", [(64, 27, 2, 0), (37, 91, 4, 1), (128, 16, 3, 2), (10, 512, 7, 3)])
def test_against_numpy_qr_and_projection(n, m, r, seed):
    g = rng(seed)
    G = g.standard_normal((n, m))
    E = 0.3 * g.standard_normal((n, m))
    Q0 = g.standard_normal((m, r))
    P_hat, Q, D, E1 = one_step(G, Q0, E=E)
    M = G + E
    A = M @ Q0
    Qh, R = np.linalg.qr(A)                     # Householder, not Gram-Schmidt
    s = np.sign(np.diag(R))
    Qh = Qh * s[None, :]                        # unique factor with diag(R) > 0
    assert np.allclose(P_hat, Qh, atol=1e-11, rtol=0)
    assert np.allclose(Q, M.T @ Qh, atol=1e-11, rtol=0)
    # decompressed result = orthogonal projection of M onto range(M Q0)
    coef, *_ = np.linalg.lstsq(A, M, rcond=None)
    assert np.allclose(D, A @ coef, atol=1e-10, rtol=0)
    assert np.allclose(E1, M - A @ coef, atol=1e-10, rtol=0)


# -- (ii) invariant: orthonormal columns --------------------------------------

@pytest.mark.parametrize("n,r", [(5, 1), (64, 2), (512, 4), (2600, 4), (300, 32)])
def test_orthonormal_columns(n, r):
    P = rng(n + r).standard_normal((n, r)) * np.logspace(0, -3, r)[None, :]
    Ph = O.orthogonalize(P)
    assert np.abs(Ph.T @ Ph - np.eye(r)).max() < 1e-12
    # triangular relation of the Remark: P = P_hat R with R upper triangular, positive diagonal
    R = Ph.T @ P
    assert np.abs(np.tril(R, -1)).max() < 1e-10
    assert (np.diag(R) > 0).all()
    assert np.allclose(Ph @ R, P, atol=1e-12)


# -- (iii) invariant: decompressed + new error = gradient + old error ---------

def test_error_feedback_conservation():
    g = rng(7)
    W, n, m, r = 3, 40, 33, 2
    grads = [[g.standard_normal((n, m))] for _ in range(W)]
    errs = [[g.standard_normal((n, m))] for _ in range(W)]
    Q0 = g.standard_normal((m, r))
    res = O.powersgd_step(grads, errs, [Q0], r)
    for w in range(W):
        lhs = res["out"][0] + res["err"][w][0]
        assert np.allclose(lhs, grads[w][0] + errs[w][0], atol=1e-13, rtol=0)


# -- (iv) special case: r = min(n, m), or rank(M) = r, reconstructs exactly ----

@pytest.mark.parametrize("n,m", [(6, 4), (4, 6), (5, 5)])
def test_full_rank_is_exact(n, m):
    g = rng(n * 10 + m)
    M = g.standard_normal((n, m))
    r = min(n, m)
    Q0 = g.standard_normal((m, r))
    _, _, D, E1 = one_step(M, Q0)
    assert np.allclose(D, M, atol=1e-11)
    assert np.abs(E1).max() < 1e-11


def test_exact_low_rank_is_exact_after_one_step():
    M = planted(64, 576, [1.0, 0.5, 0.25, 0.125], 3)
    Q0 = rng(4).standard_normal((576, 4))
    _, _, D, E1 = one_step(M, Q0)
    assert np.abs(D - M).max() < 1e-12
    # requested rank above min(n, m) is clipped
    M2 = rng(5).standard_normal((3, 50))
    res = O.powersgd_step([[M2]], [[np.zeros_like(M2)]], [rng(6).standard_normal((50, 3))], 8)
    assert res["P_hat"][0].shape == (3, 3) and res["Q"][0].shape == (50, 3)
    assert np.allclose(res["out"][0], M2, atol=1e-12)


# -- (v) theorem: on a fixed matrix warm start converges to the best rank-r ----

@pytest.mark.parametrize("r,limit", [(1, 0.328125), (2, 0.078125), (3, 0.015625)])
def test_subspace_iteration_limit(r, limit):
    s = [1.0, 0.5, 0.25, 0.125]
    M = planted(64, 576, s, 11)
    Q = rng(12).standard_normal((576, r))
    prev = None
    for _ in range(60):
        P_hat, Q, D, _ = one_step(M, Q)         # error memory reset to zero every step
        res2 = np.linalg.norm(M - D) ** 2
        if prev is not None:
            assert res2 <= prev + 1e-12          # monotone
        prev = res2
    # Remark 'Best rank-r approximation': residual = sum_{i>r} sigma_i^2
    assert abs(res2 - limit) < 1e-9
    # and the factors span the top singular subspaces
    U, sv, Vt = np.linalg.svd(M)
    assert np.allclose(P_hat @ (P_hat.T @ U[:, :r]), U[:, :r], atol=1e-6)


# -- (vi) lemma: W workers == one worker on the mean ---------------------------

def test_single_multi_worker_equivalence():
    g = rng(21)
    W, r = 5, 3
    shapes = [(32, 48), (17,), (20, 9)]
    grads = [[g.standard_normal(s) for s in shapes] for _ in range(W)]
    errs = [[g.standard_normal(s) if len(s) == 2 else None for s in shapes] for _ in range(W)]
    Qs = [g.standard_normal((s[1], r)) if len(s) == 2 else None for s in shapes]
    multi = O.powersgd_step(grads, errs, Qs, r)
    gm = [[sum(grads[w][t] for w in range(W)) / W for t in range(len(shapes))]]
    em = [[sum(errs[w][t] for w in range(W)) / W if len(shapes[t]) == 2 else None
           for t in range(len(shapes))]]
    single = O.powersgd_step(gm, em, Qs, r)
    for t, s in enumerate(shapes):
        assert np.allclose(multi["out"][t], single["out"][t], atol=1e-12)
        if len(s) == 2:
            assert np.allclose(multi["P_hat"][t], single["P_hat"][t], atol=1e-12)
            assert np.allclose(multi["Q"][t], single["Q"][t], atol=1e-12)
            mean_err = sum(multi["err"][w][t] for w in range(W)) / W
            assert np.allclose(mean_err, single["err"][0][t], atol=1e-12)


# -- (vii) invariances ----------------------------------------------------------

def test_triangular_and_scale_invariance():
    g = rng(31)
    n, m, r = 50, 70, 4
    M = g.standard_normal((n, m))
    Q0 = g.standard_normal((m, r))
    T = np.triu(g.standard_normal((r, r)))
    T[np.diag_indices(r)] = np.abs(np.diag(T)) + 0.5
    P1, Q1, D1, _ = one_step(M, Q0)
    P2, Q2, D2, _ = one_step(M, Q0 @ T)
    assert np.allclose(P1, P2, atol=1e-10) and np.allclose(Q1, Q2, atol=1e-10)
    P3, Q3, _, _ = one_step(3.5 * M, Q0)
    assert np.allclose(P1, P3, atol=1e-12) and np.allclose(3.5 * Q1, Q3, atol=1e-11)
    # a generic (non-triangular) mixing changes P_hat but not the projection
    P4, _, D4, _ = one_step(M, Q0 @ g.standard_normal((r, r)))
    assert not np.allclose(P1, P4, atol=1e-3)
    assert np.allclose(D1, D4, atol=1e-10)


# -- (viii) r = 1 is textbook power iteration -----------------------------------

def test_rank_one_power_iteration():
    g = rng(41)
    M = planted(30, 40, [3.0, 1.0, 0.5], 42) + 1e-3 * g.standard_normal((30, 40))
    q = g.standard_normal((40, 1))
    P_hat, Q, _, _ = one_step(M, q)
    p = M @ q
    assert np.allclose(P_hat, p / np.linalg.norm(p), atol=1e-13)
    assert np.allclose(Q, M.T @ (p / np.linalg.norm(p)), atol=1e-13)
    for _ in range(80):
        _, q, _, _ = one_step(M, q)
    assert abs(np.linalg.norm(q) - np.linalg.svd(M, compute_uv=False)[0]) < 1e-9


# -- (ix) brute force, derived by hand (not printed in the paper) ----------------

def test_hand_derived_cases():
    M = np.array([[2.0, 0.0], [0.0, 1.0]])
    Q0 = np.array([[1.0], [1.0]])
    P_hat, Q, D, E1 = one_step(M, Q0)
    s5 = np.sqrt(5.0)
    assert np.allclose(P_hat, np.array([[2.0], [1.0]]) / s5, atol=1e-15)
    assert np.allclose(Q, np.array([[4.0], [1.0]]) / s5, atol=1e-15)
    assert np.allclose(D, [[1.6, 0.4], [0.8, 0.2]], atol=1e-15)
    assert np.allclose(E1, [[0.4, -0.4], [-0.8, 0.8]], atol=1e-15)

    M = np.array([[1.0, 2.0], [0.0, 1.0], [1.0, 0.0]])
    P_hat, Q, D, E1 = one_step(M, np.eye(2))
    s2, s3 = np.sqrt(2.0), np.sqrt(3.0)
    assert np.allclose(P_hat, [[1 / s2, 1 / s3], [0.0, 1 / s3], [1 / s2, -1 / s3]], atol=1e-15)
    assert np.allclose(Q, [[s2, 0.0], [s2, s3]], atol=1e-15)
    assert np.allclose(D, M, atol=1e-15) and np.abs(E1).max() < 1e-15


def test_error_feedback_carries_over_two_steps_by_hand():
    # step 1 leaves E = [[.4,-.4],[-.8,.8]] and Q = [4,1]/sqrt5 (case above); step 2 with G = 0
    # works on M = E: E q = [1.2,-2.4]/sqrt5 -> P_hat = [1,-2]/sqrt5, Q = E^T P_hat = [2,-2]/sqrt5,
    # Delta' = P_hat Q^T = E (rank one), so the memory is flushed completely.
    E = np.array([[0.4, -0.4], [-0.8, 0.8]])
    Q1 = np.array([[4.0], [1.0]]) / np.sqrt(5.0)
    P_hat, Q, D, E2 = one_step(np.zeros((2, 2)), Q1, E=E)
    assert np.allclose(P_hat, np.array([[1.0], [-2.0]]) / np.sqrt(5.0), atol=1e-15)
    assert np.allclose(Q, np.array([[2.0], [-2.0]]) / np.sqrt(5.0), atol=1e-15)
    assert np.allclose(D, E, atol=1e-15) and np.abs(E2).max() < 1e-15


# -- degenerate inputs -----------------------------------------------------------

def test_zero_gradient_gives_zero_everything():
    M = np.zeros((8, 6))
    P_hat, Q, D, E1 = one_step(M, rng(1).standard_normal((6, 2)))
    assert not np.isnan(P_hat).any()
    assert np.abs(P_hat).max() == 0 and np.abs(Q).max() == 0 and np.abs(D).max() == 0 and np.abs(E1).max() == 0


def test_vectors_are_averaged_uncompressed():
    g = rng(51)
    grads = [[g.standard_normal(13)] for _ in range(4)]
    res = O.powersgd_step(grads, [[None]] * 4, [None], 2)
    assert np.allclose(res["out"][0], np.mean([x[0] for x in grads], axis=0), atol=1e-15)
    assert res["P_hat"][0] is None and res["err"][0][0] is None


def test_conv_kernels_are_flattened():
    assert O.matrix_view((512, 256, 3, 3)) == (512, 2304)
    assert O.matrix_view((64, 3, 3, 3)) == (64, 27)
    assert O.matrix_view((10, 512)) == (10, 512)
    assert O.matrix_view((128,)) is None
    g = rng(61)
    G4 = g.standard_normal((8, 3, 3, 3))
    Q0 = g.standard_normal((27, 2))
    a = O.powersgd_step([[G4]], [[np.zeros((8, 27))]], [Q0], 2)
    b = O.powersgd_step([[G4.reshape(8, 27)]], [[np.zeros((8, 27))]], [Q0], 2)
    assert np.array_equal(a["out"][0], b["out"][0])


# -- (x) numbers the paper prints -------------------------------------------------

def _golden():
    tensors, totals = [], []
    with open(os.path.join(GOLDEN, "compression_ratios.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            p = line.split()
            if p[0] == "tensor":
                tensors.append((int(p[1]), int(p[2]), int(p[3])))
            else:
                totals.append((p[1], int(p[2]), int(p[3])))
    return tensors, totals


def test_per_tensor_compression_ratios_printed_in_the_paper():
    tensors, _ = _golden()
    assert len(tensors) == 14
    for n, m, ratio in tensors:
        for r in (1, 2, 4):
            got = O.compression_ratio([(n, m)], r)
            # the table prints ratio/r with the ratio rounded to an integer
            assert abs(got * r - ratio) <= 0.5 + 1e-9, (n, m, r, got)


def test_total_compression_ratios_printed_in_the_paper():
    from paper_1905_13727_amd import workloads as WL
    _, totals = _golden()
    shapes = {"resnet18": WL.resnet18_shapes(), "lstm": WL.lstm_shapes(vocab=28869)}
    assert O.uncompressed_floats(shapes["resnet18"]) == 11164352 + 9610
    assert sum(s[0] for s in shapes["resnet18"] if len(s) == 1) == 9610
    assert sum(s[0] for s in shapes["lstm"] if len(s) == 1) == 44469
    for model, r, ratio in totals:
        got = O.compression_ratio(shapes[model], r)
        assert abs(got - ratio) <= 0.5, (model, r, got)


# -- next-row functions ------------------------------------------------------------

def test_momentum_update_by_hand():
    x, m = O.momentum_update(np.array([1.0, 2.0]), np.array([0.5, -1.0]), np.array([0.2, 0.4]), 0.1, 0.9)
    # m' = .9*[.5,-1] + [.2,.4] = [.65,-.5];  x' = x - .1*([.2,.4] + m') = [1-.085, 2+.01]
    assert np.allclose(m, [0.65, -0.5], atol=1e-15)
    assert np.allclose(x, [0.915, 2.01], atol=1e-15)


def test_best_approximation_matches_truncated_svd():
    M = planted(40, 60, [1.0, 0.3, 0.09, 0.027, 0.0081], 71)
    Q0 = rng(72).standard_normal((60, 2))
    P_hat, Q = O.best_approx_compress([M], Q0, 4)
    U, s, Vt = np.linalg.svd(M)
    best = (U[:, :2] * s[:2]) @ Vt[:2]
    # four iterations on a spectrum with ratio 0.3 between kept and dropped directions
    assert np.linalg.norm(O.decompress(P_hat, Q) - best) < 2e-3 * np.linalg.norm(best)
    P1, Q1 = O.best_approx_compress([M], Q0, 1)
    assert np.linalg.norm(O.decompress(P1, Q1) - best) > np.linalg.norm(O.decompress(P_hat, Q) - best)


# -- Appendix G baselines: Random Block and Random K -------------------------------------

def _brute_sparse(Ms, keep, W):
    """Per-element loops: what 'keep these positions, average them, zero the rest' means."""
    n, m = Ms[0].shape
    M_hat = [[0.0] * m for _ in range(n)]
    for pos in keep:
        i, j = divmod(int(pos), m)
        acc = 0.0
        for w in range(W):
            acc += float(Ms[w][i, j])
        M_hat[i][j] = acc / W
    errs = [[[float(Ms[w][i, j]) - M_hat[i][j] for j in range(m)] for i in range(n)] for w in range(W)]
    return np.array(M_hat), [np.array(e) for e in errs]


def test_random_block_by_hand():
    # Appendix G, "Random Block compression": n = 2, m = 3, r = 1 -> b = (3 + 2) * 1 = 5
    G = np.array([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]])
    Z = np.zeros((2, 3))
    assert O.kept_count(2, 3, 1) == 5
    r = O.random_block_step([[G]], [[Z]], [1], 1)       # slice M(1:6) = [2,3,4,5,6]
    assert np.array_equal(r["values"][0], [2, 3, 4, 5, 6])
    assert np.array_equal(r["out"][0], [[0, 2, 3], [4, 5, 6]])
    assert np.array_equal(r["err"][0][0], [[1, 0, 0], [0, 0, 0]])
    # the carried error comes back in the next step (Algorithm 2): M = G + e = [[2,2,3],[4,5,6]], block at 0
    r2 = O.random_block_step([[G]], [r["err"][0]], [0], 1)
    assert np.array_equal(r2["out"][0], [[2, 2, 3], [4, 5, 0]])
    assert np.array_equal(r2["err"][0][0], [[0, 0, 0], [0, 0, 6]])
    # a block that starts near the end stops at the end (no wrap-around): M(4:9) -> [5, 6]
    r3 = O.random_block_step([[G]], [[Z]], [4], 1)
    assert np.array_equal(r3["values"][0], [5, 6, 0, 0, 0])
    assert np.array_equal(r3["out"][0], [[0, 0, 0], [0, 5, 6]])
    # two workers: the kept entries are the mean, each worker keeps its own deviation
    G2 = np.array([[3.0, 0.0, 1.0], [0.0, 1.0, 2.0]])
    r4 = O.random_block_step([[G], [G2]], [[Z], [Z]], [1], 1)
    assert np.array_equal(r4["out"][0], [[0, 1, 2], [2, 3, 4]])
    assert np.array_equal(r4["err"][0][0], [[1, 1, 1], [2, 2, 2]])
    assert np.array_equal(r4["err"][1][0], [[3, -1, -1], [-2, -2, -2]])


def test_random_k_by_hand():
    # Appendix G, "Random K compression": the same 2 x 3 case, I = (5, 0, 3, 2, 1) -> all but position 4
    G = np.array([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]])
    Z = np.zeros((2, 3))
    r = O.random_k_step([[G]], [[Z]], [np.array([5, 0, 3, 2, 1])], 1)
    assert np.array_equal(r["values"][0], [6, 1, 4, 3, 2])          # in the order of I
    assert np.array_equal(r["out"][0], [[1, 2, 3], [4, 0, 6]])
    assert np.array_equal(r["err"][0][0], [[0, 0, 0], [0, 5, 0]])


@pytest.mark.parametrize("W", [1, 3])
def test_baselines_against_per_element_brute_force(W):
    g = rng(200 + W)
    shapes = [(7, 5), (4,), (3, 11)]
    rank = 2
    grads = [[g.standard_normal(s) for s in shapes] for _ in range(W)]
    errs = [[None if len(s) == 1 else g.standard_normal(s) for s in shapes] for _ in range(W)]
    starts = [9, None, 30]                                      # the second block runs past the end (3*11 = 33)
    idx = [g.permutation(35)[: O.kept_count(7, 5, rank)], None, g.permutation(33)[: O.kept_count(3, 11, rank)]]
    rb = O.random_block_step(grads, errs, starts, rank)
    rk = O.random_k_step(grads, errs, idx, rank)
    for t, s in enumerate(shapes):
        if len(s) == 1:
            mean = sum(grads[w][t] for w in range(W)) / W
            assert np.allclose(rb["out"][t], mean, atol=1e-15) and np.allclose(rk["out"][t], mean, atol=1e-15)
            assert rb["err"][0][t] is None and rb["values"][t] is None
            continue
        n, m = s
        b = O.kept_count(n, m, rank)
        Ms = [grads[w][t] + errs[w][t] for w in range(W)]
        for res, keep in ((rb, range(starts[t], min(starts[t] + b, n * m))), (rk, idx[t])):
            M_hat, e = _brute_sparse(Ms, keep, W)
            assert np.allclose(res["out"][t], M_hat, atol=1e-14)
            for w in range(W):
                assert np.allclose(res["err"][w][t], e[w], atol=1e-14)
                # Algorithm 2: what is not sent stays in the memory, exactly
                assert np.allclose(res["out"][t] + res["err"][w][t], Ms[w], atol=1e-14)
            assert np.count_nonzero(res["out"][t]) == len(list(keep))


def test_random_k_on_a_contiguous_range_is_random_block():
    g = rng(210)
    G, E = g.standard_normal((6, 9)), g.standard_normal((6, 9))
    b = O.kept_count(6, 9, 2)
    rb = O.random_block_step([[G]], [[E]], [7], 2)
    rk = O.random_k_step([[G]], [[E]], [np.arange(7, 7 + b)], 2)
    for key in ("values", "out"):
        assert np.array_equal(rb[key][0], rk[key][0])
    assert np.array_equal(rb["err"][0][0], rk["err"][0][0])
    # keeping every position sends the whole update: nothing is left in the memory (W = 1)
    full = O.random_k_step([[G]], [[E]], [g.permutation(54)], 99)
    assert O.kept_count(6, 9, 99) == 54
    assert np.array_equal(full["out"][0], G + E) and not full["err"][0][0].any()


def test_baselines_single_multi_worker_equivalence():
    """Appendix A.3: for a linear compressor W workers equal one worker on the mean update."""
    g = rng(220)
    W, s, rank = 4, (8, 6), 1
    grads = [[g.standard_normal(s)] for _ in range(W)]
    errs = [[g.standard_normal(s)] for _ in range(W)]
    gm = [sum(grads[w][0] for w in range(W)) / W]
    em = [sum(errs[w][0] for w in range(W)) / W]
    idx = [g.permutation(48)[: O.kept_count(8, 6, rank)]]
    for many, one in ((O.random_block_step(grads, errs, [20], rank), O.random_block_step([gm], [em], [20], rank)),
                      (O.random_k_step(grads, errs, idx, rank), O.random_k_step([gm], [em], idx, rank))):
        assert np.allclose(many["out"][0], one["out"][0], atol=1e-14)
        assert np.allclose(many["values"][0], one["values"][0], atol=1e-14)
        assert np.allclose(sum(many["err"][w][0] for w in range(W)) / W, one["err"][0][0], atol=1e-14)


def test_baseline_budget_is_the_papers_compression_ratio():
    """b = (n + m) r "to match rank-r PowerSGD": with the vectors sent whole, the two baselines exchange exactly
    what the paper's tables count for PowerSGD (243x / 136x / 72x, 310x / 203x / 120x)."""
    from paper_1905_13727_amd import workloads as WL
    _, totals = _golden()
    shapes = {"resnet18": WL.resnet18_shapes(), "lstm": WL.lstm_shapes(vocab=28869)}
    for model, r, ratio in totals:
        sent = sum(int(np.prod(s)) if len(s) == 1 else O.kept_count(s[0], int(np.prod(s[1:])), r) for s in shapes[model])
        assert abs(O.uncompressed_floats(shapes[model]) / sent - ratio) <= 0.5, (model, r)
    assert O.kept_count(10, 3, 4) == 30          # capped at n m
