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


def _random_weights(rng, B, R, Dr, Nr, density=0.2):
    A = rng.uniform(0.1, 1.0, (B, R, Dr, Nr)) * (rng.uniform(size=(B, R, Dr, Nr)) < density)
    A[..., 0] += 0.05          # no empty rows
    return A, A.sum(axis=3).reshape(B, R * Dr)


def test_pinv_unmerge_is_the_moore_penrose_solution(oracle):
    """Sec. 4.2.2: X' -> A~^+ X'.  Pinned by what defines the pseudo-inverse rather than by the routine
    that computes it: for rows of full rank it is the paper's closed form A~^T (A~ A~^T)^-1 X' (solved
    here as a linear system); A~ Y reproduces X' exactly then; Y lies in the row space of A~ (minimum
    norm); and tokens land at their grid positions in both merge modes."""
    rng = np.random.default_rng(51)
    B, H, W, C, th, tw, k = 2, 8, 8, 5, 4, 4, 6
    for R in (1, 4):
        d = oracle.make_desc(B, H, W, C, th, tw, k, R, 0.1)
        Dr, Nr = 4 * k // R, H * W // R
        A, Z = _random_weights(rng, B, R, Dr, Nr)
        O = rng.standard_normal((B, 4 * k + 3, C))            # three extra rows that must be ignored
        Y = oracle.unmerge_pinv(d, A, Z, O, rcond=1e-12)
        _, _, token_of = oracle.region_map(H, W, th, tw)
        for b in range(B):
            for rho in range(R):
                At = A[b, rho] / Z[b, rho * Dr:(rho + 1) * Dr, None]
                Xp = O[b, rho * Dr:(rho + 1) * Dr]
                toks = np.arange(H * W) if R == 1 else token_of[rho]
                closed = At.T @ np.linalg.solve(At @ At.T, Xp)
                assert np.allclose(Y[b, toks], closed, atol=1e-10)
                assert np.allclose(At @ Y[b, toks], Xp, atol=1e-10)
                # minimum norm: nothing outside the row space of A~
                null = np.eye(Nr) - At.T @ np.linalg.solve(At @ At.T, At)
                assert np.abs(null @ Y[b, toks]).max() < 1e-10


def test_pinv_unmerge_equals_transpose_unmerge_for_orthonormal_rows(oracle):
    """The paper's argument for the transpose: when A~ A~^T = I the two unmerges coincide.  Rows that
    are one-hot on distinct sources (hard assignment of one source per destination) are orthonormal."""
    rng = np.random.default_rng(52)
    B, H, W, C = 1, 4, 8, 3
    d = oracle.make_desc(B, H, W, C, 4, 8, 10, 1, 0.1)
    A = np.zeros((B, 1, 10, 32))
    A[0, 0, np.arange(10), rng.choice(32, 10, replace=False)] = 1.0
    Z = A.sum(axis=3).reshape(B, 10)
    O = rng.standard_normal((B, 10, C))
    assert np.allclose(oracle.unmerge_pinv(d, A, Z, O, rcond=1e-12), oracle.unmerge(d, A, Z, O), atol=1e-13)
    sv, dev = oracle.merge_matrix_spectrum(d, A, Z)
    assert np.allclose(sv, 1.0) and dev.max() < 1e-14


def test_pinv_unmerge_with_deficient_rank_and_the_cut_off(oracle):
    """Rank-deficient merge matrices (the closed form does not exist): a destination that received no
    weight (zero row) is ignored; two destinations with identical rows share their inputs' mean (least
    squares), which keeping only one of them would not give; and a singular value below rcond * largest
    counts as zero while one above is inverted."""
    rng = np.random.default_rng(53)
    B, H, W, C = 1, 4, 8, 4
    d = oracle.make_desc(B, H, W, C, 4, 8, 6, 1, 0.1)
    A, Z = _random_weights(rng, B, 1, 6, 32, density=0.4)
    A[0, 0, 2] = 0.0                       # nobody chose destination 2
    A[0, 0, 5] = A[0, 0, 4]                # destinations 4 and 5 weigh the same sources equally
    Z = A.sum(axis=3).reshape(B, 6)
    O = rng.standard_normal((B, 6, C))
    Y = oracle.unmerge_pinv(d, A, Z, O, rcond=1e-9)
    keep = [0, 1, 3, 4]
    At = A[0, 0, keep] / Z[0, keep, None]
    Xp = O[0, keep].copy()
    Xp[3] = 0.5 * (O[0, 4] + O[0, 5])
    assert np.allclose(Y[0], At.T @ np.linalg.solve(At @ At.T, Xp), atol=1e-9)
    Xp[3] = O[0, 4]
    assert not np.allclose(Y[0], At.T @ np.linalg.solve(At @ At.T, Xp), atol=1e-3)
    # the cut-off: two orthogonal rows with norms 1 and 1e-3 (before normalisation they are rows of A~
    # already: Z = 1 is passed)
    d2 = oracle.make_desc(1, 2, 4, 2, 2, 4, 2, 1, 0.1)
    A2 = np.zeros((1, 1, 2, 8)); A2[0, 0, 0, 0] = 1.0; A2[0, 0, 1, 1] = 1e-3
    O2 = np.array([[[1.0, 2.0], [3.0, 4.0]]])
    kept = oracle.unmerge_pinv(d2, A2, np.ones((1, 2)), O2, rcond=1e-4)
    cut = oracle.unmerge_pinv(d2, A2, np.ones((1, 2)), O2, rcond=1e-2)
    assert np.allclose(kept[0, 1], [3000.0, 4000.0]) and np.allclose(cut[0, 1], 0.0) and np.allclose(cut[0, 0], [1.0, 2.0])
