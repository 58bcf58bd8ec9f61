"""Host-side checks of the C-ABI library (no GPU): it loads, exports every symbol the header declares, sizes
buffers as documented, and turns invalid arguments into error codes before anything could be launched."""
import ctypes
import os
import re
import subprocess
import sys

import pytest

import paper_2211_15841_amd as dm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _cfg(T=1024, d=256, h=1024, E=4, k=1, block=128, act=0, norm=0, cap=0, pad=0):
    return dm.DMoEConfig(T, d, h, E, k, block, act, norm, cap, pad)


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


def test_sizes_with_an_expert_capacity():
    """Token dropping (Section 2.2): no expert owns more rows than its capacity rounded up to whole blocks; with padding
    to capacity every expert owns exactly that many."""
    free = dm.dmoe_sizes(_cfg(T=8192, d=512, h=2048, E=64))
    assert free["P_max"] == (8192 + 127 * 64) // 128 * 128
    assert dm.dmoe_sizes(_cfg(T=8192, d=512, h=2048, E=64, cap=128))["P_max"] == 64 * 128
    assert dm.dmoe_sizes(_cfg(T=8192, d=512, h=2048, E=64, cap=128, pad=1))["P_max"] == 64 * 128
    assert dm.dmoe_sizes(_cfg(T=8192, d=512, h=2048, E=64, cap=192, pad=1))["P_max"] == 64 * 256
    assert dm.dmoe_sizes(_cfg(T=8192, d=512, h=2048, E=64, cap=100000))["P_max"] == free["P_max"]
    assert dm.dmoe_sizes(_cfg(T=8192, d=512, h=2048, E=64, cap=100))["nnz_max"] == 64 * 16


@pytest.mark.parametrize("kw,frag", [
    (dict(block=64), "block"), (dict(d=200), "d_model"), (dict(h=100), "ffn_hidden"), (dict(E=0), "num_experts"),
    (dict(E=257), "num_experts"), (dict(k=0), "top_k"), (dict(k=5, E=4), "top_k"), (dict(k=9, E=16), "top_k"),
    (dict(T=0), "num_tokens"), (dict(act=2), "activation"), (dict(norm=2), "normalize_topk"),
    (dict(cap=-1), "expert_capacity"), (dict(pad=2, cap=4), "pad_to_capacity"), (dict(pad=1), "pad_to_capacity"),
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
    dm.dmoe_set_tile_mode(3)
    dm.dmoe_set_tile_mode(0)
    with pytest.raises(dm.DMoEError, match="tile mode"):
        dm.dmoe_set_tile_mode(4)


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


# ---- buffer extents at the shape of the Figure-9 problems (65 536 tokens, 8 experts, hidden 512, ffn 2 048) ---------
FIG9_XS = dict(T=65536, d=512, h=2048, E=8, k=1)


@pytest.mark.parametrize("shape", [FIG9_XS, dict(T=8192, d=1536, h=6144, E=8, k=1), dict(T=1000, d=256, h=384, E=7, k=3)],
                         ids=["fig9_xs", "fig9_medium", "ragged"])
def test_topology_arrays_are_disjoint_and_inside_the_buffer(shape):
    """Every array that dmoe_topology_bind carves lies inside the buffer, is 256-byte aligned, and is long enough for
    the upper bounds of dmoe_sizes -- checked from the pointers the library hands back, for the shape whose run once
    preceded an unexplained GPU fault."""
    cfg = _cfg(**shape)
    s = dm.dmoe_sizes(cfg)
    fake = 0x7f0000000000
    topo = dm.dmoe_topology_bind(cfg, fake, s["topology_bytes"])
    T, E, k, hb = shape["T"], shape["E"], shape["k"], shape["h"] // 128
    F, P, R, nnz = T * k, s["P_max"], s["P_max"] // 128, s["nnz_max"]
    g_max = (R + min(E, F) + 1) // 2
    need = {"expert_idx": F, "weights": F, "logits": T * E, "tokens_per_expert": E, "padded_offsets": E + 1,
            "row_of": F, "token_of": P, "row_offsets": R + 1, "column_indices": nnz, "row_indices": nnz,
            "column_offsets_t": E * hb + 1, "row_indices_t": nnz, "block_offsets_t": nnz, "counts": 4,
            "expert_order": E, "group_offsets": E + 1, "row_group": g_max + 1, "sched": 4}
    spans = sorted((getattr(topo, n), getattr(topo, n) + 4 * cnt, n) for n, cnt in need.items())
    assert spans[0][0] == fake and spans[-1][1] <= fake + s["topology_bytes"]
    for (a0, a1, an), (b0, b1, bn) in zip(spans, spans[1:]):
        assert a0 % 256 == 0 and a1 <= b0, "%s overlaps %s" % (an, bn)


@pytest.mark.parametrize("shape", [FIG9_XS, dict(T=8192, d=512, h=2048, E=64, k=1), dict(T=300, d=128, h=256, E=64, k=2),
                                   dict(T=40, d=128, h=128, E=64, k=1)], ids=["fig9_xs", "xs", "ragged", "few_tokens"])
def test_sizes_cover_the_worst_routing(shape):
    """The padded row count, block-row count, row-group count and block count of ANY routing stay within what
    dmoe_sizes reports.  Worst cases are built by hand (every expert one row past a multiple of 128, all rows on one
    expert, perfectly even) and pushed through the oracle's own grouping, which is pinned elsewhere."""
    import numpy as np
    from oracle import dmoe_oracle as orc
    cfg = _cfg(**shape)
    s = dm.dmoe_sizes(cfg)
    T, E, k, hb = shape["T"], shape["E"], shape["k"], shape["h"] // 128
    F = T * k
    loads = []
    n = np.zeros(E, dtype=np.int64)                       # as many experts as possible hold 1 (mod 128) rows
    m = min(E, F)
    n[:m] = 1
    rest = F - m
    n[:m] += (rest // (128 * m)) * 128
    n[0] += F - n.sum()
    loads.append(n)
    one = np.zeros(E, dtype=np.int64); one[E - 1] = F
    loads.append(one)
    loads.append(np.full(E, F // E, dtype=np.int64) + (np.arange(E) < F % E))
    for n in loads:
        assert n.sum() == F
        idx = np.repeat(np.arange(E), n).astype(np.int32).reshape(-1, 1)      # one assignment per row, grouped
        cnt, off, row_of, token_of = orc.permutation(idx, E)
        P = int(off[-1]); R = P // 128
        groups = int(sum((int(off[e + 1] - off[e]) // 128 + 1) // 2 for e in range(E)))
        assert P <= s["P_max"] and R * hb <= s["nnz_max"]
        assert groups <= (s["P_max"] // 128 + min(E, F) + 1) // 2
        assert len(token_of) == P and row_of.max() < P


def test_extreme_sizes_give_an_error_or_a_size_never_a_crash():
    """The size arithmetic with every dimension at its extremes: each call returns sizes or a clean DMOE_EINVAL."""
    big = 2 ** 31 - 1
    seen_ok = seen_err = 0
    for T in (1, 127, 2 ** 23, 2 ** 24 - 1, 2 ** 24, big):
        for d, h in ((128, 128), (128, big // 128 * 128), (big // 128 * 128, 128), (2 ** 20, 2 ** 20), (16384, 65536)):
            for E, k in ((1, 1), (256, 1), (256, 8), (64, 4)):
                for cap, pad in ((0, 0), (1, 1), (big, 0), (big, 1)):
                    try:
                        s = dm.dmoe_sizes(_cfg(T=T, d=d, h=h, E=E, k=k, cap=cap, pad=pad))
                    except dm.DMoEError as e:
                        assert "dmoe error -1" in str(e)
                        seen_err += 1
                        continue
                    seen_ok += 1
                    assert s["P_max"] % 128 == 0 and 0 < s["P_max"] < 2 ** 31 and 0 < s["nnz_max"] < 2 ** 31
                    assert all(s[key] % 256 == 0 and s[key] > 0 for key in ("topology_bytes", "saved_bytes", "scratch_bytes"))
    assert seen_ok and seen_err
    for rows, cols, nnz in ((1, 1, 0), (big, 1, 1), (1, big, big), (big, big, big), (46340, 46341, 1)):
        try:
            assert dm.dmoe_bsmm_sizes(rows, cols, nnz) % 256 == 0
        except dm.DMoEError as e:
            assert "dmoe error" in str(e)


@pytest.mark.skipif(os.environ.get("DMOE_LIBRARY") is not None, reason="already running against another build")
def test_host_code_under_the_undefined_behaviour_sanitizer():
    """The ABI tests once more, in a child process, against a build whose host code traps on undefined behaviour (signed
    overflow, out-of-bounds array index, misaligned access, bad shift) in the size, layout and validation code."""
    from paper_2211_15841_amd import build
    lib = build.build_host_checked()
    env = dict(os.environ, DMOE_LIBRARY=lib)
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.abspath(__file__), "-q", "-x", "-m", "not gpu", "-p",
                        "no:cacheprovider", "-k", "not missing_library"], env=env, cwd=ROOT, capture_output=True, text=True)
    assert r.returncode == 0, (r.returncode, r.stdout[-2000:], r.stderr[-2000:])
    assert " passed" in r.stdout
