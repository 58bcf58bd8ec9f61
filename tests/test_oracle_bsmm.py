"""Pins of the general block-sparse oracle (oracle/bsmm_oracle.py) against scipy.sparse block-CSR matrices, dense
special cases and adjoint identities.  No GPU."""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle import bsmm_oracle as bo

B = 8      # the definitions do not depend on the block size; small blocks keep these tests instant


def _case(seed, R, C, D, density):
    rng = np.random.default_rng(seed)
    mask = (rng.random((R, C)) < density).astype(np.uint8)
    r, c = bo.block_order(mask)
    vals = rng.standard_normal((len(r), B, B))
    x = rng.standard_normal((R * B, D))
    return mask, vals, x, rng


def _bsr(mask, vals):
    """The same matrix as a scipy block-CSR matrix, built from (data, indices, indptr) in scipy's own convention."""
    R, C = mask.shape
    indptr = np.concatenate([[0], np.cumsum(mask.astype(bool).sum(axis=1))])
    indices = np.nonzero(mask)[1]
    return sp.bsr_matrix((vals, indices, indptr), shape=(R * B, C * B), blocksize=(B, B))


@pytest.mark.parametrize("seed,R,C,density", [(1, 5, 7, 0.4), (2, 3, 3, 1.0), (3, 6, 2, 0.2), (4, 1, 9, 0.5)])
def test_densify_matches_scipy_block_csr(seed, R, C, density):
    mask, vals, _, _ = _case(seed, R, C, 16, density)
    np.testing.assert_array_equal(bo.densify(vals, mask, B), _bsr(mask, vals).toarray())


@pytest.mark.parametrize("seed,R,C,density", [(11, 5, 7, 0.4), (12, 4, 4, 0.7), (13, 6, 2, 0.3)])
def test_dense_output_products_match_scipy(seed, R, C, density):
    mask, vals, x, rng = _case(seed, R, C, 24, density)
    S = _bsr(mask, vals)
    w_nd = rng.standard_normal((C * B, 24))
    w_dn = rng.standard_normal((24, C * B))
    # the oracle's own functions take block = 128 by default; rebuild them on the small block through densify
    dense = bo.densify(vals, mask, B)
    np.testing.assert_allclose(dense @ w_nd, S @ w_nd, rtol=1e-12, atol=1e-12)                 # DSD
    np.testing.assert_allclose(dense @ w_dn.T, S @ w_dn.T, rtol=1e-12, atol=1e-12)             # DSD^T
    np.testing.assert_allclose(dense.T @ x, S.T.tocsr() @ x, rtol=1e-12, atol=1e-12)           # DS^TD
    np.testing.assert_allclose(x.T @ dense, (S.T.tocsr() @ x).T, rtol=1e-12, atol=1e-12)       # DD^TS
    xt = rng.standard_normal((24, R * B))
    np.testing.assert_allclose(xt @ dense, (S.T.tocsr() @ xt.T).T, rtol=1e-12, atol=1e-12)     # DDS


def test_sample_is_the_inverse_of_densify_on_the_mask():
    mask, vals, _, _ = _case(21, 4, 6, 8, 0.5)
    np.testing.assert_array_equal(bo.sample(bo.densify(vals, mask, B), mask, B), vals)
    # and what the mask drops is dropped: a dense matrix sampled and densified again is the masked matrix
    rng = np.random.default_rng(22)
    full = rng.standard_normal((4 * B, 6 * B))
    keep = np.kron(mask, np.ones((B, B)))
    np.testing.assert_array_equal(bo.densify(bo.sample(full, mask, B), mask, B), full * keep)


def test_full_block_size_functions_on_all_ones_and_empty_masks():
    rng = np.random.default_rng(31)
    R, C, D = 2, 3, 128
    x = rng.standard_normal((R * 128, D))
    w = rng.standard_normal((D, C * 128))
    ones = np.ones((R, C), dtype=np.uint8)
    s = bo.sdd(x, w, ones)
    np.testing.assert_allclose(bo.densify(s, ones), x @ w, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(bo.densify(bo.sddt(x, w.T.copy(), ones), ones), x @ w, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(bo.dsd(s, w.T.copy(), ones), (x @ w) @ w.T, rtol=1e-10, atol=1e-9)
    np.testing.assert_allclose(bo.dsdt(s, w, ones), (x @ w) @ w.T, rtol=1e-10, atol=1e-9)
    np.testing.assert_allclose(bo.dstd(s, x, ones), (x @ w).T @ x, rtol=1e-10, atol=1e-9)
    np.testing.assert_allclose(bo.ddts(x, s, ones), x.T @ (x @ w), rtol=1e-10, atol=1e-9)
    np.testing.assert_allclose(bo.dds(x.T.copy(), s, ones), x.T @ (x @ w), rtol=1e-10, atol=1e-9)
    zero = np.zeros((R, C), dtype=np.uint8)
    assert bo.sdd(x, w, zero).shape == (0, 128, 128)
    assert not bo.dsd(np.zeros((0, 128, 128)), w.T.copy(), zero).any()
    assert not bo.dstd(np.zeros((0, 128, 128)), x, zero).any()


def test_adjoint_identities_between_the_products():
    """<SDD(X, W), S> = <X, DSD^T(S, W)> = <W, DD^TS(X, S)> and the same for the transposed pair: each backward
    product is the adjoint of the forward one, which is how Section 5.1 arrives at the list."""
    rng = np.random.default_rng(41)
    R, C, D = 3, 2, 128
    mask = np.array([[1, 0], [1, 1], [0, 1]], dtype=np.uint8)
    x = rng.standard_normal((R * 128, D))
    w = rng.standard_normal((D, C * 128))
    s = rng.standard_normal((int(mask.sum()), 128, 128))
    lhs = float((bo.sdd(x, w, mask) * s).sum())
    np.testing.assert_allclose(lhs, float((x * bo.dsdt(s, w, mask)).sum()), rtol=1e-10)
    np.testing.assert_allclose(lhs, float((w * bo.ddts(x, s, mask)).sum()), rtol=1e-10)
    w2 = rng.standard_normal((C * 128, D))
    lhs = float((bo.sddt(x, w2, mask) * s).sum())
    np.testing.assert_allclose(lhs, float((x * bo.dsd(s, w2, mask)).sum()), rtol=1e-10)
    np.testing.assert_allclose(lhs, float((w2 * bo.dstd(s, x, mask)).sum()), rtol=1e-10)


def test_dds_is_the_transpose_of_a_sparse_times_dense_product_and_the_adjoint_of_sdd():
    """Y = X S has two independent characterisations: Y^T = S^T X^T (the DS^TD product of the transposed input), and
    <X S, G> = <S, X^T G restricted to the mask> (DDS is what the backward pass of an SDD with a transposed left
    input would need)."""
    rng = np.random.default_rng(51)
    mask = np.array([[1, 0, 1], [0, 0, 1], [1, 1, 0], [0, 0, 0]], dtype=np.uint8)
    R, C, D = mask.shape[0], mask.shape[1], 128
    x = rng.standard_normal((D, R * 128))
    s = rng.standard_normal((int(mask.sum()), 128, 128))
    y = bo.dds(x, s, mask)
    np.testing.assert_allclose(y, bo.dstd(s, x.T.copy(), mask).T, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(y, bo.ddts(x.T.copy(), s, mask), rtol=1e-12, atol=1e-12)
    g = rng.standard_normal((D, C * 128))
    np.testing.assert_allclose(float((y * g).sum()), float((s * bo.sdd(x.T.copy(), g, mask)).sum()), rtol=1e-10)
    assert y.shape == (D, C * 128)


def test_remaining_transposition_combinations_against_scipy_and_the_pinned_products():
    """The five products beyond the layer's seven (Section 5.1.1: every combination of transposed inputs), each pinned
    three ways: a scipy block-CSR product at the full block size, the already pinned product of the explicitly
    transposed input, and an adjoint identity."""
    rng = np.random.default_rng(61)
    mask = np.array([[1, 0, 1], [0, 0, 1], [1, 1, 0], [0, 0, 0]], dtype=np.uint8)
    R, C, D = mask.shape[0], mask.shape[1], 256
    M, N = R * 128, C * 128
    s = rng.standard_normal((int(mask.sum()), 128, 128))
    indptr = np.concatenate([[0], np.cumsum(mask.astype(bool).sum(axis=1))])
    S = sp.bsr_matrix((s, np.nonzero(mask)[1], indptr), shape=(M, N), blocksize=(128, 128))
    x_dm, x_dn, x_nd = rng.standard_normal((D, M)), rng.standard_normal((D, N)), rng.standard_normal((N, D))
    w_dn, w_nd = rng.standard_normal((D, N)), rng.standard_normal((N, D))

    # sparse outputs: the masked blocks of the dense product
    full = x_dm.T @ w_dn
    keep = np.kron(mask, np.ones((128, 128)))
    np.testing.assert_allclose(bo.densify(bo.sdtd(x_dm, w_dn, mask), mask), full * keep, rtol=1e-12, atol=1e-12)
    np.testing.assert_array_equal(bo.sdtd(x_dm, w_dn, mask), bo.sdd(x_dm.T.copy(), w_dn, mask))
    np.testing.assert_allclose(bo.densify(bo.sdtdt(x_dm, w_nd, mask), mask), (x_dm.T @ w_nd.T) * keep, rtol=1e-12, atol=1e-12)
    np.testing.assert_array_equal(bo.sdtdt(x_dm, w_nd, mask), bo.sddt(x_dm.T.copy(), w_nd, mask))

    # dense outputs: scipy's own sparse products
    np.testing.assert_allclose(bo.dstdt(s, x_dm, mask), S.T.tocsr() @ x_dm.T, rtol=1e-12, atol=1e-10)
    np.testing.assert_array_equal(bo.dstdt(s, x_dm, mask), bo.dstd(s, x_dm.T.copy(), mask))
    np.testing.assert_allclose(bo.ddst(x_dn, s, mask), (S @ x_dn.T).T, rtol=1e-12, atol=1e-10)
    np.testing.assert_allclose(bo.ddst(x_dn, s, mask), bo.dsd(s, x_dn.T.copy(), mask).T, rtol=1e-12, atol=1e-10)
    np.testing.assert_allclose(bo.ddtst(x_nd, s, mask), (S @ x_nd).T, rtol=1e-12, atol=1e-10)
    np.testing.assert_allclose(bo.ddtst(x_nd, s, mask), bo.dsd(s, x_nd, mask).T, rtol=1e-12, atol=1e-10)
    assert bo.ddst(x_dn, s, mask).shape == (D, M) and bo.dstdt(s, x_dm, mask).shape == (N, D)
    # a row of S without blocks is a zero COLUMN of X S^T
    assert not bo.ddst(x_dn, s, mask)[:, 3 * 128:].any()

    # adjoints: <X S^T, G> = <S, G^T X on the mask>,  <S^T X^T, G> = <S, X^T G^T on the mask>
    g = rng.standard_normal((D, M))
    np.testing.assert_allclose(float((bo.ddst(x_dn, s, mask) * g).sum()), float((s * bo.sdtd(g, x_dn, mask)).sum()), rtol=1e-10)
    g2 = rng.standard_normal((N, D))
    np.testing.assert_allclose(float((bo.dstdt(s, x_dm, mask) * g2).sum()), float((s * bo.sdtdt(x_dm, g2, mask)).sum()), rtol=1e-10)
