"""CPU oracle for one PowerSGD step (rank-r compression with error feedback).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, fp64 numpy
implementation of what the GPU path computes, written from the paper
(Vogels, Karimireddy, Jaggi: "PowerSGD", arXiv 1905.13727) and nothing else.
Only the tests, the smoke check and the benchmark's `cpu_baseline` leg may
import it; the HIP library never does, and the two share no code.

Every function follows the paper's steps in the paper's order and notation:

  Algorithm 1  ("Rank-r PowerSGD compression"): compress+aggregate, decompress
  Algorithm 2  ("Distributed error-feedback SGD with momentum"): the
               error-feedback add and the error memory update
  Section 3    matrix view of tensors, Gram-Schmidt, warm start
  Appendix A.3 (single/multi worker equivalence): the error is taken against
               the decompressed *aggregate*, eq. (ef-sgd) last line
  Appendix G.7 ("Best-approximation PowerSGD"): several subspace iterations,
               no reuse of the previous step
  Appendix G   ("Random Block compression", "Random K compression"): the two
               linear baselines that run inside the same error-feedback loop

Readings taken where the paper is silent (listed again in the design notes):
  * Gram-Schmidt is the modified variant, columns left to right, one pass.
  * A column whose squared norm is <= ZERO_NORM2 at the moment it is
    normalised is set to zero (rank-deficient input, all-zero gradient);
    otherwise it is divided by its exact norm, no additive epsilon.
  * Effective rank of a matrix is min(r, n, m).
  * The reductions over workers are means.
  * A worker's new error memory is its own update minus the decompressed
    aggregate:  e_w <- (g_w + e_w) - P_hat Q^T.
  * Vector-shaped tensors carry no error memory; their output is the mean of
    the workers' gradients.

Parity pins (tests/test_oracle_pins.py): numpy's Householder QR and a
least-squares projection for P_hat / Q / decompressed result, hand-derived
2x2 and 3x2 cases, exact reconstruction at full rank, the subspace-iteration
limit sum_{i>r} sigma_i^2, W-worker == 1-worker on the mean, triangular
invariance of the warm start, r = 1 power iteration, the compression ratios
the paper prints for ResNet18 and the LSTM; for the Appendix G baselines
hand-worked 2x3 cases, a per-element brute force, conservation, the
W-worker == 1-worker lemma, Random K on a contiguous index range == Random
Block, and the paper's ratios again (their budget is PowerSGD's).  No
function here is unpinned.
"""
from __future__ import annotations

import numpy as np

# Squared-norm threshold under which a column counts as zero (reading of a
# point the paper does not address; 1e-30 is far below anything fp32 data of
# sane scale produces and far above fp64 underflow).
ZERO_NORM2 = 1e-30


def matrix_view(shape):
    """Section 3 / Algorithm 1 line 1: a tensor with >= 2 dims is seen as a
    matrix (d0, prod(d1..)); 4-D conv kernels o*i*k*k become o x (i*k*k).
    1-D tensors are not compressed: returns None for them."""
    shape = tuple(int(s) for s in shape)
    if len(shape) < 2:
        return None
    n = shape[0]
    m = 1
    for s in shape[1:]:
        m *= s
    return (n, m)


def effective_rank(r, n, m):
    return min(int(r), int(n), int(m))


def orthogonalize(P):
    """Algorithm 1 'orthogonalize' by the Gram-Schmidt procedure (Section 3;
    Remark 'Orthogonalization is a linear operation': the result is P R^-1
    with R upper triangular, positive diagonal).  Modified Gram-Schmidt."""
    P = np.array(P, dtype=np.float64, copy=True)
    r = P.shape[1]
    for j in range(r):
        nrm2 = float(np.dot(P[:, j], P[:, j]))
        if nrm2 <= ZERO_NORM2:
            P[:, j] = 0.0
        else:
            P[:, j] = P[:, j] / np.sqrt(nrm2)
        for k in range(j + 1, r):
            P[:, k] = P[:, k] - np.dot(P[:, j], P[:, k]) * P[:, j]
    return P


def compress_aggregate(Ms, Q_prev):
    """Algorithm 1, function compress+aggregate, for one matrix and W workers.

    Ms      list of W update matrices M_w (n x m)
    Q_prev  previous Q (m x r), the warm start
    returns (P_hat n x r, Q m x r)
    """
    W = len(Ms)
    Q_prev = np.asarray(Q_prev, dtype=np.float64)
    # P <- M Q ; P <- all-reduce-mean(P)
    P = np.zeros((Ms[0].shape[0], Q_prev.shape[1]), dtype=np.float64)
    for w in range(W):
        P = P + np.asarray(Ms[w], dtype=np.float64) @ Q_prev
    P = P / W
    # P_hat <- orthogonalize(P)
    P_hat = orthogonalize(P)
    # Q <- M^T P_hat ; Q <- all-reduce-mean(Q)
    Q = np.zeros_like(Q_prev)
    for w in range(W):
        Q = Q + np.asarray(Ms[w], dtype=np.float64).T @ P_hat
    Q = Q / W
    return P_hat, Q


def decompress(P_hat, Q):
    """Algorithm 1, function decompress: P_hat Q^T."""
    return np.asarray(P_hat, dtype=np.float64) @ np.asarray(Q, dtype=np.float64).T


def powersgd_step(grads, errs, Qs, rank):
    """One iterate of Algorithm 2 up to (not including) the momentum update,
    with Algorithm 1 as the compressor, for W workers and a list of tensors.

    grads[w][t]  gradient tensor t of worker w (any shape; >=2-D ones are
                 compressed through their matrix view, 1-D ones are averaged)
    errs[w][t]   error memory e_w of tensor t as an (n x m) array, or None
                 for 1-D tensors
    Qs[t]        warm-start Q (m x r_t) for matrix tensors, None for 1-D
    rank         r

    Returns a dict with, per tensor t:
      'P_hat'[t], 'Q'[t]   compressed representation (None for 1-D)
      'out'[t]             Delta' (decompressed aggregate, matrix view shape;
                           for 1-D tensors the mean gradient)
      'err'[w][t]          new error memory per worker (None for 1-D)
    Nothing is modified in place.
    """
    W = len(grads)
    T = len(grads[0])
    out = {"P_hat": [None] * T, "Q": [None] * T, "out": [None] * T,
           "err": [[None] * T for _ in range(W)]}
    for t in range(T):
        view = matrix_view(np.shape(grads[0][t]))
        if view is None:
            # vector-shaped parameters are aggregated uncompressed
            acc = np.zeros(np.shape(grads[0][t]), dtype=np.float64)
            for w in range(W):
                acc = acc + np.asarray(grads[w][t], dtype=np.float64)
            out["out"][t] = acc / W
            continue
        n, m = view
        r_t = effective_rank(rank, n, m)
        assert Qs[t].shape == (m, r_t)
        # Delta_w <- g_w + e_w      (error feedback)
        Ms = []
        for w in range(W):
            g = np.asarray(grads[w][t], dtype=np.float64).reshape(n, m)
            e = np.asarray(errs[w][t], dtype=np.float64).reshape(n, m)
            Ms.append(g + e)
        # C(Delta) <- compress+aggregate
        P_hat, Q = compress_aggregate(Ms, Qs[t])
        # Delta' <- decompress(C(Delta))
        D = decompress(P_hat, Q)
        # e_w <- Delta_w - Delta'
        for w in range(W):
            out["err"][w][t] = Ms[w] - D
        out["P_hat"][t] = P_hat
        out["Q"][t] = Q
        out["out"][t] = D
    return out


def momentum_update(x, m, delta, lr, lam):
    """Algorithm 2, last two lines: m <- lam*m + Delta' ; x <- x - lr*(Delta' + m).
    Returns (x_new, m_new)."""
    x = np.asarray(x, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    delta = np.asarray(delta, dtype=np.float64)
    m_new = lam * m + delta
    x_new = x - lr * (delta + m_new)
    return x_new, m_new


def best_approx_compress(Ms, Q0, iterations):
    """Appendix G.7: the same compressor with `iterations` subspace-iteration
    steps (2*iterations matrix products) started from a fresh Q0 and no reuse
    across optimisation steps.  Returns (P_hat, Q)."""
    Q = np.asarray(Q0, dtype=np.float64)
    P_hat = None
    for _ in range(int(iterations)):
        P_hat, Q = compress_aggregate(Ms, Q)
    return P_hat, Q


# --- plan-level arithmetic the paper prints (Appendix F tables) -------------

def compressed_floats(shapes, rank):
    """Number of floats exchanged per step: r*(n+m) per matrix plus every
    element of the uncompressed 1-D tensors."""
    total = 0
    for s in shapes:
        v = matrix_view(s)
        if v is None:
            total += int(np.prod(s))
        else:
            n, m = v
            total += effective_rank(rank, n, m) * (n + m)
    return total


def uncompressed_floats(shapes):
    return int(sum(int(np.prod(s)) for s in shapes))


def compression_ratio(shapes, rank):
    return uncompressed_floats(shapes) / compressed_floats(shapes, rank)


# --- Appendix G: the two linear baseline compressors that share the error-feedback loop -----------------
#
# "Random Block" and "Random K" (Appendix G, first two algorithms) plug into Algorithm 2 in the place
# of Algorithm 1: the update matrix M_w = g_w + e_w is seen as a vector of length n*m, every worker keeps
# the same b = (n + m) r entries of it (the budget of rank-r PowerSGD), the kept values are averaged over
# the workers, the decompressed matrix is zero elsewhere, and e_w <- M_w - decompressed.  The random draws
# (the block's start s, the index set I) are the same on all workers; here they are arguments.
#
# Readings where the appendix is silent:
#   * b is capped at n*m (tiny matrices);
#   * a block that would run past the end of the vector stops there (no wrap-around): the slice
#     M(s : s+b) holds min(b, n*m - s) entries; the packed values are zero beyond them;
#   * vector-shaped tensors are averaged uncompressed, as in Algorithm 1.

def kept_count(n, m, rank):
    """Entries a matrix keeps: b = (m + n) r, "to match rank-r PowerSGD", at most n*m."""
    return min((int(n) + int(m)) * int(rank), int(n) * int(m))


def _sparse_step(grads, errs, rank, positions_of):
    """Algorithm 2 up to the momentum update with a keep-these-positions compressor.
    positions_of(t, n, m, b) -> integer array of the kept positions of tensor t (length <= b)."""
    W = len(grads)
    T = len(grads[0])
    out = {"values": [None] * T, "out": [None] * T, "err": [[None] * T for _ in range(W)]}
    for t in range(T):
        view = matrix_view(np.shape(grads[0][t]))
        if view is None:
            acc = np.zeros(np.shape(grads[0][t]), dtype=np.float64)
            for w in range(W):
                acc = acc + np.asarray(grads[w][t], dtype=np.float64)
            out["out"][t] = acc / W
            continue
        n, m = view
        b = kept_count(n, m, rank)
        pos = np.asarray(positions_of(t, n, m, b), dtype=np.int64)
        # Delta_w <- g_w + e_w, treated as a vector of length n m
        Ms = []
        for w in range(W):
            g = np.asarray(grads[w][t], dtype=np.float64).reshape(n * m)
            e = np.asarray(errs[w][t], dtype=np.float64).reshape(n * m)
            Ms.append(g + e)
        # compress: S_w = M_w(positions) ; aggregate: mean over the workers
        S = np.zeros(len(pos), dtype=np.float64)
        for w in range(W):
            S = S + Ms[w][pos]
        S = S / W
        # decompress: zero matrix with the averaged values put back
        M_hat = np.zeros(n * m, dtype=np.float64)
        M_hat[pos] = S
        vals = np.zeros(b, dtype=np.float64)
        vals[: len(pos)] = S
        out["values"][t] = vals
        out["out"][t] = M_hat.reshape(n, m)
        # e_w <- Delta_w - Delta'
        for w in range(W):
            out["err"][w][t] = (Ms[w] - M_hat).reshape(n, m)
    return out


def random_block_step(grads, errs, starts, rank):
    """Appendix G, "Random Block compression", inside Algorithm 2.

    starts[t]  the sampled index s in [0, n m) of matrix tensor t (same on all workers); ignored for 1-D
    Returns 'values'[t] (the b averaged slice entries, zero past the end of the vector), 'out'[t]
    (Delta'), 'err'[w][t]."""
    def positions(t, n, m, b):
        s = int(starts[t])
        assert 0 <= s < n * m
        return np.arange(s, min(s + b, n * m))
    return _sparse_step(grads, errs, rank, positions)


def random_k_step(grads, errs, indices, rank):
    """Appendix G, "Random K compression", inside Algorithm 2.

    indices[t]  the b sampled positions of matrix tensor t, without repetition (same on all workers)
    Returns 'values'[t] (the averaged looked-up values, in the order of indices[t]), 'out'[t], 'err'[w][t]."""
    def positions(t, n, m, b):
        idx = np.asarray(indices[t], dtype=np.int64)
        assert idx.shape == (b,) and len(np.unique(idx)) == b and idx.min() >= 0 and idx.max() < n * m
        return idx
    return _sparse_step(grads, errs, rank, positions)
