"""Pins for the oracle's merge weights, merge and unmerge (paper Sec. 4.2, Alg. 3 steps 2-3)."""
import numpy as np
import pytest
from scipy.special import softmax


def _setup(oracle, rng, B=2, H=8, W=8, C=6, th=4, tw=4, k=5, R=1, tau=0.5):
    X = rng.standard_normal((B, H * W, C))
    d = oracle.make_desc(B, H, W, C, th, tw, k, R, tau)
    idx, _, _ = oracle.select(d, X)
    return d, X, idx


@pytest.mark.parametrize("tile_local", [False, True])
def test_weights_match_library_softmax(oracle, tile_local):
    # Sec. 4.2.1: A = softmax(D X^T / tau) taken over destinations for each source token
    rng = np.random.default_rng(20)
    P = 4
    d, X, idx = _setup(oracle, rng, R=P if tile_local else 1, tau=0.7)
    A, Z, clamps = oracle.merge_weights(d, X, idx)
    _, _, token_of = oracle.region_map(8, 8, 4, 4)
    for b in range(2):
        if tile_local:
            for p in range(P):
                Dm, Xs = X[b, idx[b, p]], X[b, token_of[p]]
                ref = softmax(Dm @ Xs.T / 0.7, axis=0)
                assert np.allclose(A[b, p], ref, atol=1e-13)
                assert np.allclose(Z[b, p * 5:(p + 1) * 5], ref.sum(axis=1), atol=1e-12)
        else:
            Dm = X[b, idx[b].reshape(-1)]
            ref = softmax(Dm @ X[b].T / 0.7, axis=0)
            assert np.allclose(A[b, 0], ref, atol=1e-13)
            assert np.allclose(Z[b], ref.sum(axis=1), atol=1e-12)
    assert clamps == 0


def test_each_source_token_is_split_into_shares_summing_to_one(oracle):
    rng = np.random.default_rng(21)
    for R in (1, 4):
        d, X, idx = _setup(oracle, rng, R=R, tau=0.1)
        A, Z, _ = oracle.merge_weights(d, X, idx)
        assert np.all(A >= 0) and np.all(A <= 1)
        assert np.allclose(A.sum(axis=2), 1.0, atol=1e-12)          # over destinations
        assert np.allclose(Z.sum(axis=1), 64.0, atol=1e-10)          # all mass accounted for


def test_merged_rows_are_convex_combinations(oracle):
    rng = np.random.default_rng(22)
    d, X, idx = _setup(oracle, rng, R=4, tau=0.3)
    A, Z, _ = oracle.merge_weights(d, X, idx)
    At = A / Z.reshape(2, 4, 5, 1)
    assert np.allclose(At.sum(axis=3), 1.0, atol=1e-12)             # rows of A~ sum to one
    Xm = oracle.merge(d, X, A, Z)
    _, _, token_of = oracle.region_map(8, 8, 4, 4)
    for b in range(2):
        for p in range(4):
            src = X[b, token_of[p]]
            blk = Xm[b, p * 5:(p + 1) * 5]
            assert np.all(blk <= src.max(axis=0) + 1e-12) and np.all(blk >= src.min(axis=0) - 1e-12)
            assert np.allclose(blk, At[b, p] @ src, atol=1e-12)      # X_merged = A~ X with numpy


def test_infinite_temperature_gives_uniform_average(oracle):
    rng = np.random.default_rng(23)
    d, X, idx = _setup(oracle, rng, R=4, tau=1e12)
    A, Z, _ = oracle.merge_weights(d, X, idx)
    assert np.allclose(A, 1.0 / 5, atol=1e-9)
    Xm = oracle.merge(d, X, A, Z)
    _, _, token_of = oracle.region_map(8, 8, 4, 4)
    for p in range(4):
        assert np.allclose(Xm[0, p * 5:(p + 1) * 5], X[0, token_of[p]].mean(axis=0), atol=1e-9)


def test_single_destination_per_region_is_the_region_mean(oracle):
    rng = np.random.default_rng(24)
    d, X, idx = _setup(oracle, rng, k=1, R=4, tau=0.05)
    A, Z, _ = oracle.merge_weights(d, X, idx)
    Xm = oracle.merge(d, X, A, Z)
    _, _, token_of = oracle.region_map(8, 8, 4, 4)
    for p in range(4):
        assert np.allclose(Xm[1, p], X[1, token_of[p]].mean(axis=0), atol=1e-12)


@pytest.mark.parametrize("R", [1, 4])
def test_all_destinations_low_temperature_is_identity(oracle, R):
    # every token a destination, equal norms, tau -> 0: A = A~ = permutation, merge and unmerge
    # undo each other (Sec. 4.2.2: A~ A~^T = I makes the transpose the exact inverse)
    rng = np.random.default_rng(25)
    B, H, W, C = 1, 8, 8, 12
    X = rng.standard_normal((B, H * W, C))
    X /= np.linalg.norm(X, axis=2, keepdims=True)
    d = oracle.make_desc(B, H, W, C, 4, 4, 16, R, 1e-4)
    idx, _, _ = oracle.select(d, X)
    A, Z, _ = oracle.merge_weights(d, X, idx)
    Xm = oracle.merge(d, X, A, Z)
    flat = idx.reshape(B, -1)
    assert np.allclose(Xm[0], X[0, flat[0]], atol=1e-12)
    assert np.allclose(Z, 1.0, atol=1e-12)
    O = rng.standard_normal((B, 64, C))
    Y = oracle.unmerge(d, A, Z, O)
    assert np.allclose(Y[0, flat[0]], O[0], atol=1e-12)
    # A~ A~^T = I
    At = (A / Z.reshape(B, R, -1, 1))
    for r in range(R):
        assert np.allclose(At[0, r] @ At[0, r].T, np.eye(At.shape[2]), atol=1e-12)


def test_hard_assignment_limit(oracle):
    # tau -> 0 with fewer destinations: every source goes to the destination with the largest
    # dot product; merge = group mean (Sec. 4.2 uniform averaging), transpose unmerge copies the
    # destination's output back divided by its group size
    rng = np.random.default_rng(26)
    d, X, idx = _setup(oracle, rng, B=1, R=1, k=3, tau=1e-6)
    A, Z, _ = oracle.merge_weights(d, X, idx)
    flat = idx.reshape(-1)
    assign = np.argmax(X[0, flat] @ X[0].T, axis=0)
    Xm = oracle.merge(d, X, A, Z)
    O = rng.standard_normal((1, len(flat), 6))
    Y = oracle.unmerge(d, A, Z, O)
    for j in range(len(flat)):
        grp = np.nonzero(assign == j)[0]
        assert Z[0, j] == pytest.approx(len(grp), abs=1e-9)
        if len(grp):
            assert np.allclose(Xm[0, j], X[0, grp].mean(axis=0), atol=1e-9)
            assert np.allclose(Y[0, grp], O[0, j] / len(grp), atol=1e-9)


def test_unmerge_is_transpose_product(oracle):
    rng = np.random.default_rng(27)
    for R in (1, 4):
        d, X, idx = _setup(oracle, rng, R=R, tau=0.4)
        A, Z, _ = oracle.merge_weights(d, X, idx)
        O = rng.standard_normal((2, 20 + 3, 6))         # extra rows beyond D are not read
        Y = oracle.unmerge(d, A, Z, O)
        _, _, token_of = oracle.region_map(8, 8, 4, 4)
        At = A / Z.reshape(2, R, -1, 1)
        for b in range(2):
            if R == 1:
                assert np.allclose(Y[b], At[b, 0].T @ O[b, :20], atol=1e-12)
            else:
                for p in range(4):
                    assert np.allclose(Y[b, token_of[p]], At[b, p].T @ O[b, p * 5:(p + 1) * 5], atol=1e-12)


def test_single_region_global_equals_tile(oracle):
    rng = np.random.default_rng(28)
    X = rng.standard_normal((1, 36, 5))
    d1 = oracle.make_desc(1, 6, 6, 5, 6, 6, 9, 1, 0.3)
    idx, _, _ = oracle.select(d1, X)
    A1, Z1, _ = oracle.merge_weights(d1, X, idx)
    # with P = 1, merge_regions = 1 and = P are the same computation
    assert oracle.n_regions(d1) == 1
    assert np.allclose(oracle.merge(d1, X, A1, Z1), (A1[0, 0] / Z1[0][:, None]) @ X[0], atol=1e-12)


def test_unchosen_destination_is_clamped_and_counted(oracle):
    # two destinations, the second hugely dominated: its row sum underflows to 0
    X = np.zeros((1, 4, 2))
    X[0, :, 0] = [1000.0, 1e-3, 1000.0, 1000.0]
    d = oracle.make_desc(1, 2, 2, 2, 2, 2, 2, 1, 0.01)
    idx = np.array([[[0, 1]]], np.int32)
    A, Z, clamps = oracle.merge_weights(d, X, idx)
    assert clamps == 1 and Z[0, 1] < 1e-20
    Xm = oracle.merge(d, X, A, Z)
    assert np.all(np.isfinite(Xm))
