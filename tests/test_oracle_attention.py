"""Pins for the oracle's attention on merged tokens (Eq. 1) and for the whole layer (Alg. 3)."""
import numpy as np
import pytest
import torch


def _mha_torch(U, Wq, Wk, Wv, heads):
    """Plain multi-head attention with the library's SDPA in float64."""
    U = torch.from_numpy(U)
    B, L, C = U.shape
    dh = C // heads
    q, k, v = (U @ torch.from_numpy(W) for W in (Wq, Wk, Wv))
    sp = lambda t: t.reshape(B, L, heads, dh).transpose(1, 2)
    o = torch.nn.functional.scaled_dot_product_attention(sp(q), sp(k), sp(v))
    return o.transpose(1, 2).reshape(B, L, C).numpy()


def _weights(rng, C):
    return [rng.standard_normal((C, C)) / np.sqrt(C) for _ in range(3)]


def test_attention_matches_library_sdpa(oracle):
    rng = np.random.default_rng(30)
    B, D, C, heads = 2, 37, 24, 3
    Xm = rng.standard_normal((B, D, C))
    W = _weights(rng, C)
    O = oracle.attend(Xm, None, *W, heads=heads)
    assert np.allclose(O, _mha_torch(Xm, *W, heads), atol=1e-12)


def test_extra_tokens_join_after_the_merged_ones(oracle):
    rng = np.random.default_rng(31)
    B, D, T, C, heads = 1, 10, 7, 16, 2
    Xm, Xe = rng.standard_normal((B, D, C)), rng.standard_normal((B, T, C))
    W = _weights(rng, C)
    O = oracle.attend(Xm, Xe, *W, heads=heads)
    assert O.shape == (B, D + T, C)
    assert np.allclose(O, _mha_torch(np.concatenate([Xm, Xe], axis=1), *W, heads), atol=1e-12)


def test_sampled_rows_equal_the_full_attention(oracle):
    rng = np.random.default_rng(37)
    B, D, T, C, heads = 2, 21, 4, 16, 4
    Xm, Xe = rng.standard_normal((B, D, C)), rng.standard_normal((B, T, C))
    W = _weights(rng, C)
    full = oracle.attend(Xm, Xe, *W, heads=heads).reshape(B * (D + T), C)
    rows = np.array([0, 7, 24, 25, 49, 30], np.int32)
    part = oracle.attend_rows(Xm, Xe, *W, heads=heads, rows=rows)
    assert np.allclose(part, full[rows], atol=1e-13)
    assert np.allclose(part, _mha_torch(np.concatenate([Xm, Xe], axis=1), *W, heads).reshape(-1, C)[rows], atol=1e-12)


def test_output_projection_and_constant_values(oracle):
    rng = np.random.default_rng(32)
    B, D, C, heads = 1, 9, 8, 2
    Xm = rng.standard_normal((B, D, C))
    W = _weights(rng, C)
    Wo = rng.standard_normal((C, C))
    O = oracle.attend(Xm, None, *W, heads=heads)
    assert np.allclose(oracle.attend(Xm, None, *W, heads=heads, Wo=Wo), O @ Wo, atol=1e-12)
    # identical tokens -> identical values -> every output row equals that value row
    Xc = np.repeat(rng.standard_normal((B, 1, C)), D, axis=1)
    Oc = oracle.attend(Xc, None, *W, heads=heads)
    assert np.allclose(Oc, Xc @ W[2], atol=1e-12)


def test_keep_everything_layer_is_plain_attention(oracle):
    # all tokens destinations, unit norms, tau -> 0: merge and unmerge are permutations, so the
    # layer output is multi-head attention on X itself (attention has no positional term)
    rng = np.random.default_rng(33)
    B, H, W, C, heads = 2, 8, 8, 16, 4
    X = rng.standard_normal((B, H * W, C))
    X /= np.linalg.norm(X, axis=2, keepdims=True)
    Wt = _weights(rng, C)
    for R in (1, 4):
        d = oracle.make_desc(B, H, W, C, 4, 4, 16, R, 1e-4)
        out = oracle.layer(d, X, *Wt, heads=heads)
        assert np.allclose(out["Y"], _mha_torch(X, *Wt, heads), atol=1e-10)


def test_layer_is_invariant_to_pick_order_and_batch_independent(oracle):
    rng = np.random.default_rng(34)
    B, H, W, C, heads = 2, 8, 8, 8, 2
    X = rng.standard_normal((B, H * W, C))
    Wt = _weights(rng, C)
    for R in (1, 4):
        d = oracle.make_desc(B, H, W, C, 4, 4, 6, R, 0.2)
        base = oracle.layer(d, X, *Wt, heads=heads)
        perm_idx = base["idx"][:, :, ::-1].copy()        # same sets, reversed order inside regions
        again = oracle.layer(d, X, *Wt, heads=heads, idx=perm_idx)
        assert np.allclose(again["Y"], base["Y"], atol=1e-11)
        d1 = oracle.make_desc(1, H, W, C, 4, 4, 6, R, 0.2)
        solo = oracle.layer(d1, X[1:2], *Wt, heads=heads)
        assert np.array_equal(solo["idx"][0], base["idx"][1])
        assert np.allclose(solo["Y"][0], base["Y"][1], atol=1e-12)


def test_pattern_reuse_uses_old_pattern_on_new_tokens(oracle):
    # Sec. 4.3.2: cached destinations skip the selection, cached (A, Z) also skip the weights
    rng = np.random.default_rng(35)
    B, H, W, C, heads = 1, 8, 8, 8, 2
    X0 = rng.standard_normal((B, H * W, C))
    X1 = X0 + 0.05 * rng.standard_normal(X0.shape)
    Wt = _weights(rng, C)
    d = oracle.make_desc(B, H, W, C, 4, 4, 6, 1, 0.2)
    s0 = oracle.layer(d, X0, *Wt, heads=heads)
    r_idx = oracle.layer(d, X1, *Wt, heads=heads, idx=s0["idx"])
    A1, Z1, _ = oracle.merge_weights(d, X1, s0["idx"])
    assert np.array_equal(r_idx["A"], A1) and np.array_equal(r_idx["idx"], s0["idx"])
    r_a = oracle.layer(d, X1, *Wt, heads=heads, idx=s0["idx"], AZ=(s0["A"], s0["Z"]))
    Xm = (s0["A"][0, 0] / s0["Z"][0][:, None]) @ X1[0]
    assert np.allclose(r_a["Xm"][0], Xm, atol=1e-12)
    assert np.allclose(r_a["Y"][0], (s0["A"][0, 0] / s0["Z"][0][:, None]).T @ r_a["O"][0], atol=1e-12)


def test_text_rows_pass_through(oracle):
    rng = np.random.default_rng(36)
    B, H, W, C, heads, T = 1, 8, 8, 8, 2, 5
    X = rng.standard_normal((B, H * W, C))
    Xe = rng.standard_normal((B, T, C))
    Wt = _weights(rng, C)
    d = oracle.make_desc(B, H, W, C, 4, 4, 4, 4, 0.2)
    out = oracle.layer(d, X, *Wt, heads=heads, Xe=Xe)
    assert out["O"].shape == (B, 16 + T, C) and np.array_equal(out["Y_extra"], out["O"][:, 16:])
    assert out["Y"].shape == (B, 64, C)


def test_mlp_matches_numpy_and_scipy_erf(oracle):
    """The feed-forward module against numpy products and scipy's erf (an independent library),
    plus two closed forms: zero input gives zero, and a large positive pre-activation passes
    through unchanged (gelu(x) -> x)."""
    from scipy.special import erf
    rng = np.random.default_rng(31)
    X = rng.standard_normal((3, 7, 16))
    W1 = rng.standard_normal((16, 40)) / 4.0
    W2 = rng.standard_normal((40, 16)) / 6.0
    H = X @ W1
    ref = (0.5 * H * (1.0 + erf(H / np.sqrt(2.0)))) @ W2
    assert np.allclose(oracle.mlp(X, W1, W2), ref, rtol=1e-12, atol=1e-12)
    assert np.array_equal(oracle.mlp(np.zeros((2, 16)), W1, W2), np.zeros((2, 16)))
    big = np.full((1, 16), 50.0)
    eye = np.eye(16)
    assert np.allclose(oracle.mlp(big, eye, eye), big, rtol=1e-12)
    assert np.allclose(oracle.mlp(-big, eye, eye), 0.0, atol=1e-12)


def test_cross_attention_matches_library_sdpa(oracle):
    """Queries from one token set, keys / values from another of a different width and length, against
    torch's SDPA in float64; with the context equal to the queries it is the self-attention above; a
    single context token makes every output row that token's value (softmax over one key)."""
    rng = np.random.default_rng(41)
    B, Lq, Tc, C, Cc, heads = 2, 19, 7, 24, 40, 3
    U, Ctx = rng.standard_normal((B, Lq, C)), rng.standard_normal((B, Tc, Cc))
    Wq = rng.standard_normal((C, C)) / np.sqrt(C)
    Wk, Wv = (rng.standard_normal((Cc, C)) / np.sqrt(Cc) for _ in range(2))
    Wo = rng.standard_normal((C, C)) / np.sqrt(C)
    O = oracle.cross_attend(U, Ctx, Wq, Wk, Wv, heads)
    dh = C // heads
    q, k, v = torch.from_numpy(U @ Wq), torch.from_numpy(Ctx @ Wk), torch.from_numpy(Ctx @ Wv)
    sp = lambda t: t.reshape(B, -1, heads, dh).transpose(1, 2)
    ref = torch.nn.functional.scaled_dot_product_attention(sp(q), sp(k), sp(v)).transpose(1, 2).reshape(B, Lq, C).numpy()
    assert np.allclose(O, ref, atol=1e-12)
    assert np.allclose(oracle.cross_attend(U, Ctx, Wq, Wk, Wv, heads, Wo=Wo), ref @ Wo, atol=1e-12)
    W = _weights(rng, C)
    assert np.allclose(oracle.cross_attend(U, U, *W, heads=heads), oracle.attend(U, None, *W, heads=heads), atol=1e-12)
    one = oracle.cross_attend(U, Ctx[:, :1], Wq, Wk, Wv, heads)
    assert np.allclose(one, np.repeat(Ctx[:, :1] @ Wv, Lq, axis=1), atol=1e-12)
    # a transposed weight or a softmax over the wrong axis does not survive these
    assert not np.allclose(oracle.cross_attend(U, Ctx, Wq.T.copy(), Wk, Wv, heads), ref, atol=1e-3)
