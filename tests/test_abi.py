"""Host-side checks of the C-ABI library (no GPU): it loads, exports every symbol the header declares, sizes
buffers as documented, and turns invalid arguments into error codes before anything could be launched."""
import ctypes
import os
import re

import pytest

import paper_2211_15841_amd as dm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _cfg(T=1024, d=256, h=1024, E=4, k=1, block=128, act=0, norm=0):
    return dm.DMoEConfig(T, d, h, E, k, block, act, norm)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "dmoe.h")).read()
    declared = re.findall(r"^DMOE_API\s+(?:const\s+)?\w+\s*\*?\s*(dmoe_\w+)\s*\(", header, flags=re.M)
    assert set(declared) >= {"dmoe_sizes", "dmoe_topology_bind", "dmoe_topology", "dmoe_forward", "dmoe_backward",
                             "dmoe_last_error"}
    lib = dm.load_library()
    for name in declared:
        assert hasattr(lib, name), name


def test_sizes_follow_the_documented_bounds():
    s = dm.dmoe_sizes(_cfg(T=8192, d=512, h=2048, E=64))
    assert s["P_max"] == 128 * ((8192 + 127 * 64) // 128)
    assert s["nnz_max"] == s["P_max"] // 128 * 16
    assert s["saved_bytes"] >= 2 * s["P_max"] * 512 * 2 + 2 * s["nnz_max"] * 128 * 128 * 2
    for key in ("topology_bytes", "saved_bytes", "scratch_bytes"):
        assert s[key] % 256 == 0
    # fewer assignments than experts: at most one block-row per assignment
    s2 = dm.dmoe_sizes(_cfg(T=3, d=128, h=128, E=64))
    assert s2["P_max"] == 3 * 128


@pytest.mark.parametrize("kw,frag", [
    (dict(block=64), "block"), (dict(d=200), "d_model"), (dict(h=100), "ffn_hidden"), (dict(E=0), "num_experts"),
    (dict(E=257), "num_experts"), (dict(k=0), "top_k"), (dict(k=5, E=4), "top_k"), (dict(k=9, E=16), "top_k"),
    (dict(T=0), "num_tokens"), (dict(act=2), "activation"), (dict(norm=2), "normalize_topk"),
])
def test_invalid_configurations_are_rejected(kw, frag):
    with pytest.raises(dm.DMoEError) as ei:
        dm.dmoe_sizes(_cfg(**kw))
    assert "dmoe error -1" in str(ei.value) and frag in str(ei.value)


def test_bind_and_calls_validate_pointers_without_launching():
    cfg = _cfg()
    s = dm.dmoe_sizes(cfg)
    fake = 0x7f0000000000                      # never dereferenced on the host: validation only
    topo = dm.dmoe_topology_bind(cfg, fake, s["topology_bytes"])
    assert topo.expert_idx == fake and topo.counts > fake
    with pytest.raises(dm.DMoEError, match="-2"):
        dm.dmoe_topology_bind(cfg, fake, s["topology_bytes"] - 1)
    with pytest.raises(dm.DMoEError, match="aligned"):
        dm.dmoe_topology_bind(cfg, fake + 8, s["topology_bytes"])
    lib = dm.load_library()
    rc = lib.dmoe_topology(ctypes.byref(cfg), None, fake, None, ctypes.byref(topo), fake, s["scratch_bytes"], None)
    assert rc == -1 and "x is NULL" in dm.dmoe_last_error()
    rc = lib.dmoe_topology(ctypes.byref(cfg), fake, fake, None, ctypes.byref(topo), fake, 16, None)
    assert rc == -2
    empty = dm.DMoETopology()
    rc = lib.dmoe_forward(ctypes.byref(cfg), fake, fake, fake, ctypes.byref(empty), fake, fake, s["saved_bytes"],
                          fake, s["scratch_bytes"], None)
    assert rc == -1 and "bind" in dm.dmoe_last_error()
    rc = lib.dmoe_backward(ctypes.byref(cfg), fake, fake, fake, fake, ctypes.byref(topo), fake, 8, fake, fake, fake,
                           fake, fake, fake, s["scratch_bytes"], None)
    assert rc == -2
    rc = lib.dmoe_backward_accumulate(ctypes.byref(cfg), fake, fake, fake, fake, ctypes.byref(topo), fake,
                                      s["saved_bytes"], fake, fake, fake, None, fake, fake, s["scratch_bytes"], None)
    assert rc == -1 and "dw1 is NULL" in dm.dmoe_last_error()
    rc = lib.dmoe_backward_accumulate(ctypes.byref(cfg), fake, fake, fake, fake, ctypes.byref(topo), fake, 8, fake,
                                      fake, fake, fake, fake, fake, s["scratch_bytes"], None)
    assert rc == -2


def test_tile_mode_is_validated():
    dm.dmoe_set_tile_mode(1)
    dm.dmoe_set_tile_mode(2)
    dm.dmoe_set_tile_mode(0)
    with pytest.raises(dm.DMoEError, match="tile mode"):
        dm.dmoe_set_tile_mode(3)


def test_general_products_validate_their_arguments():
    """dmoe_bsmm_sizes / dmoe_bsmm_topology / dmoe_bsmm reject bad dimensions and pointers before touching the GPU."""
    assert dm.dmoe_bsmm_sizes(4, 5, 7) % 256 == 0
    assert dm.dmoe_bsmm_sizes(40, 50, 2000) >= 4 * 4 * 2000 + 4 * (40 + 1) + 4 * (50 + 1)   # four arrays per block
    for rows, cols, nnz, frag in [(0, 3, 0, "block_rows"), (3, 0, 0, "block_cols"), (2, 2, 5, "nnz"),
                                  (2, 2, -1, "nnz"), (1 << 17, 1, 0, "2^24")]:
        with pytest.raises(dm.DMoEError) as e:
            dm.dmoe_bsmm_sizes(rows, cols, nnz)
        assert frag in str(e.value)
    lib = dm.load_library()
    topo = dm.DMoETopology()
    mask = (ctypes.c_uint8 * 4)(1, 0, 0, 1)
    assert lib.dmoe_bsmm_topology(None, 2, 2, 256, 4096, ctypes.byref(topo), None) != 0          # NULL mask
    assert lib.dmoe_bsmm_topology(mask, 2, 2, None, 4096, ctypes.byref(topo), None) != 0          # NULL device buffer
    assert lib.dmoe_bsmm_topology(mask, 2, 2, 256 + 8, 4096, ctypes.byref(topo), None) != 0       # misaligned
    assert lib.dmoe_bsmm_topology(mask, 2, 2, 256, 16, ctypes.byref(topo), None) != 0             # too small
    assert "needs" in dm.dmoe_last_error()
    assert lib.dmoe_bsmm(9, ctypes.byref(topo), 2, 2, 2, 128, 256, 256, 256, None) != 0              # unknown product
    assert lib.dmoe_bsmm(dm.OP_DSD, ctypes.byref(topo), 2, 2, 2, 128, 256, 256, 256, None) != 0   # topology not built
    topo.row_offsets = 256
    topo.counts = 256
    assert lib.dmoe_bsmm(dm.OP_DSD, ctypes.byref(topo), 2, 2, 2, 100, 256, 256, 256, None) != 0   # dense not a multiple
    assert "multiple of 128" in dm.dmoe_last_error()
    assert lib.dmoe_bsmm(dm.OP_SDD, ctypes.byref(topo), 2, 2, 5, 128, 256, 256, 256, None) != 0    # more blocks than the mask has room for
    assert "nnz" in dm.dmoe_last_error()
    assert lib.dmoe_bsmm(dm.OP_SDD, ctypes.byref(topo), 2, 2, 0, 128, 256, 256, None, None) == 0    # empty mask: nothing to write
    assert lib.dmoe_bsmm(dm.OP_DSD, ctypes.byref(topo), 2, 2, 2, 128, None, 256, 256, None) != 0  # NULL operand


def test_a_missing_library_fails_loudly(monkeypatch, tmp_path):
    """There is no CPU or eager fallback: without the built library the binding raises and says how to build it."""
    from paper_2211_15841_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libdmoe.so"))
    with pytest.raises(dm.DMoEError, match="not built"):
        binding.load_library()
    with pytest.raises(dm.DMoEError, match="not built"):
        dm.dmoe_sizes(_cfg())
