"""Parity of the general block-sparse products (dmoe_bsmm) with their CPU oracle on arbitrary block masks:
element by element, same seeded bf16 inputs, through the C-ABI.  Tolerance as for the layer: the outputs are
rounded to bf16 once (2^-9 relative) after an fp32 accumulation, so max|G - O| <= 1e-2 * max|O| with room to spare."""
import zlib

import numpy as np
import pytest

from dmoe_inputs import f32_to_bf16_bits, bf16_bits_to_f32
from oracle import bsmm_oracle as bo

pytestmark = pytest.mark.gpu


def _bf16(rng, shape, scale=1.0):
    bits = f32_to_bf16_bits((scale * rng.standard_normal(shape)).astype(np.float32))
    return bits, bf16_bits_to_f32(bits).astype(np.float64)


def _dev(bits):
    import torch
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def _host(t):
    return bf16_bits_to_f32(t.view(__import__("torch").int16).cpu().numpy().view(np.uint16)).astype(np.float64)


def _close(got, want, what):
    """The layer's own check: tensor-wide maximum <= 1e-2, and every 128x128 tile against its own maximum (a misplaced
    or missing block cannot hide behind the tensor-wide figure).  Block values [nnz, 128, 128] are checked block by
    block as a [nnz*128, 128] matrix."""
    from tests._harness import check_values
    got, want = np.asarray(got), np.asarray(want)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if got.ndim == 3:
        got, want = got.reshape(-1, got.shape[-1]), want.reshape(-1, want.shape[-1])
    if want.size == 0:
        return
    check_values(what, got, want)


MASKS = {
    "random_40pct": lambda rng: (rng.random((7, 9)) < 0.4).astype(np.uint8),
    "dense": lambda rng: np.ones((3, 4), dtype=np.uint8),
    "diagonal": lambda rng: np.eye(5, dtype=np.uint8),
    "empty_rows_and_columns": lambda rng: np.array([[0, 1, 0, 1], [0, 0, 0, 0], [1, 1, 0, 0]], dtype=np.uint8),
    "single_block": lambda rng: np.array([[1]], dtype=np.uint8),
    "tall_column": lambda rng: np.ones((70, 1), dtype=np.uint8),     # a column of more than 64 blocks
    "wide_row": lambda rng: np.ones((1, 70), dtype=np.uint8),        # a row of more than 64 blocks
    "banded": lambda rng: np.triu(np.tril(np.ones((12, 12), dtype=np.uint8), 1), -1),
}


@pytest.mark.parametrize("name", list(MASKS))
@pytest.mark.parametrize("dense", [128, 384])
def test_all_products_on_a_mask(name, dense):
    import paper_2211_15841_amd as dm
    rng = np.random.default_rng(zlib.crc32(("%s/%d" % (name, dense)).encode()))
    mask = MASKS[name](rng)
    if not mask.any():
        mask[0, 0] = 1
    R, C = mask.shape
    M, N, D = R * 128, C * 128, dense
    nnz = int(mask.sum())
    xb, x = _bf16(rng, (M, D))
    wdn_b, wdn = _bf16(rng, (D, N), 0.05)
    wnd_b, wnd = _bf16(rng, (N, D), 0.05)
    sb, s = _bf16(rng, (nnz, 128, 128))
    bs = dm.BlockSparse(mask)
    assert bs.nnz == nnz
    xd, wdn_d, wnd_d, sd = _dev(xb), _dev(wdn_b), _dev(wnd_b), _dev(sb)

    _close(_host(bs.sdd(xd, wdn_d)), bo.sdd(x, wdn, mask), "SDD")
    _close(_host(bs.sddt(xd, wnd_d)), bo.sddt(x, wnd, mask), "SDD^T")
    _close(_host(bs.dsd(sd, wnd_d)), bo.dsd(s, wnd, mask), "DSD")
    _close(_host(bs.dsdt(sd, wdn_d)), bo.dsdt(s, wdn, mask), "DSD^T")
    _close(_host(bs.dstd(sd, xd)), bo.dstd(s, x, mask), "DS^TD")
    _close(_host(bs.ddts(xd, sd)), bo.ddts(x, s, mask), "DD^TS")
    xtb, xt = _bf16(rng, (D, M))
    _close(_host(bs.dds(_dev(xtb), sd)), bo.dds(xt, s, mask), "DDS")

    # the remaining combinations of transposed inputs (Section 5.1.1)
    xdm_b, xdm = xtb, xt                                   # [D, M]
    xdn_b, xdn = _bf16(rng, (D, N))
    xnd_b, xnd = _bf16(rng, (N, D))
    _close(_host(bs.sdtd(_dev(xdm_b), wdn_d)), bo.sdtd(xdm, wdn, mask), "SD^TD")
    _close(_host(bs.sdtdt(_dev(xdm_b), wnd_d)), bo.sdtdt(xdm, wnd, mask), "SD^TD^T")
    _close(_host(bs.dstdt(sd, _dev(xdm_b))), bo.dstdt(s, xdm, mask), "DS^TD^T")
    u = _host(bs.ddst(_dev(xdn_b), sd))
    _close(u, bo.ddst(xdn, s, mask), "DDS^T")
    _close(_host(bs.ddtst(_dev(xnd_b), sd)), bo.ddtst(xnd, s, mask), "DD^TS^T")
    for r in np.nonzero(~mask.any(axis=1))[0]:            # a block row of S without blocks: zero columns of X S^T
        assert not u[:, r * 128:(r + 1) * 128].any()

    # rows / columns without blocks must come out as exact zeros
    y = _host(bs.dsd(sd, wnd_d))
    for r in np.nonzero(~mask.any(axis=1))[0]:
        assert not y[r * 128:(r + 1) * 128].any()
    z = _host(bs.dstd(sd, xd))
    for c in np.nonzero(~mask.any(axis=0))[0]:
        assert not z[c * 128:(c + 1) * 128].any()
    v = _host(bs.dds(_dev(xtb), sd))
    for c in np.nonzero(~mask.any(axis=0))[0]:
        assert not v[:, c * 128:(c + 1) * 128].any()


def test_topology_of_a_mask_is_bit_exact():
    """The uploaded encoding equals the oracle's generic encoder (oracle.dmoe_oracle.encode_mask) on the same mask."""
    import torch
    import paper_2211_15841_amd as dm
    from oracle import dmoe_oracle as orc
    rng = np.random.default_rng(77)
    mask = (rng.random((9, 11)) < 0.35).astype(np.uint8)
    bs = dm.BlockSparse(mask)
    enc = orc.encode_mask(mask.astype(bool))
    raw = bs.topology_mem.cpu().numpy()

    def arr(ptr_field, n):
        off = getattr(bs.topo, ptr_field) - bs.topology_mem.data_ptr()
        return raw[off:off + 4 * n].view(np.int32)
    nnz = bs.nnz
    np.testing.assert_array_equal(arr("row_offsets", mask.shape[0] + 1), enc["row_offsets"])
    np.testing.assert_array_equal(arr("column_indices", nnz), enc["column_indices"])
    np.testing.assert_array_equal(arr("row_indices", nnz), enc["row_indices"])
    np.testing.assert_array_equal(arr("column_offsets_t", mask.shape[1] + 1), enc["column_offsets_t"])
    np.testing.assert_array_equal(arr("row_indices_t", nnz), enc["row_indices_t"])
    np.testing.assert_array_equal(arr("block_offsets_t", nnz), enc["block_offsets_t"])


def test_variable_width_experts_through_the_general_products():
    """Figure 3C draws a block-diagonal matrix whose blocks differ in rows AND columns; Section 4.1 notes that the column
    count could vary per expert (experts of different hidden sizes) and leaves it unexplored.  The general products
    take any mask, so such a layer is a mask away: three experts with 1, 3 and 2 block-columns and 2, 1 and 3
    block-rows of tokens, SDD for the first layer and DSD for the second, against one dense product pair per expert."""
    import paper_2211_15841_amd as dm
    rng = np.random.default_rng(91)
    rows, widths, D = [2, 1, 3], [1, 3, 2], 256
    R, C = sum(rows), sum(widths)
    mask = np.zeros((R, C), dtype=np.uint8)
    r0 = c0 = 0
    spans = []
    for nr, nc in zip(rows, widths):
        mask[r0:r0 + nr, c0:c0 + nc] = 1
        spans.append((r0 * 128, (r0 + nr) * 128, c0 * 128, (c0 + nc) * 128))
        r0, c0 = r0 + nr, c0 + nc
    xb, x = _bf16(rng, (R * 128, D))
    w1b, w1 = _bf16(rng, (D, C * 128), 0.05)
    w2b, w2 = _bf16(rng, (C * 128, D), 0.05)
    bs = dm.BlockSparse(mask)
    h_blocks = bs.sdd(_dev(xb), _dev(w1b))
    y = _host(bs.dsd(h_blocks, _dev(w2b)))
    h_ref = np.zeros((R * 128, C * 128))
    y_ref = np.zeros((R * 128, D))
    hb = _host(h_blocks)
    for (ra, rb, ca, cb) in spans:                        # per expert: two dense products on its own tokens and width
        h_e = x[ra:rb] @ w1[:, ca:cb]
        h_ref[ra:rb, ca:cb] = h_e
        # the second layer consumes what the first one stored (bf16), as the GPU path does
        y_ref[ra:rb] = bo.densify(hb, mask)[ra:rb, ca:cb] @ w2[ca:cb]
    _close(hb, bo.sample(h_ref, mask), "variable-width SDD")
    _close(y, y_ref, "variable-width DSD")
