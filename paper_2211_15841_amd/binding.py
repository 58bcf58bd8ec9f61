"""ctypes binding of include/dmoe.h.  Same names as the C entry points; argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from ctypes import c_int32, c_size_t, c_void_p, c_char_p, POINTER, byref

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# DMOE_LIBRARY names another build of the same library (the host-sanitized one that the ABI tests load in a child process)
LIB_PATH = os.environ.get("DMOE_LIBRARY") or os.path.join(_HERE, "libdmoe.so")

STAGE_NAMES = ["router", "sort", "topology", "gather", "sdd", "dsd", "scatter", "bwd_gather", "sddt", "dstd",
               "dsdt", "ddts", "router_bwd"]


class DMoEError(RuntimeError):
    pass


class DMoEConfig(ctypes.Structure):
    _fields_ = [("num_tokens", c_int32), ("d_model", c_int32), ("ffn_hidden", c_int32), ("num_experts", c_int32),
                ("top_k", c_int32), ("block", c_int32), ("activation", c_int32), ("normalize_topk", c_int32),
                ("expert_capacity", c_int32), ("pad_to_capacity", c_int32)]


_TOPO_FIELDS = ["expert_idx", "weights", "logits", "tokens_per_expert", "padded_offsets", "row_of", "token_of",
                "row_offsets", "column_indices", "row_indices", "column_offsets_t", "row_indices_t",
                "block_offsets_t", "counts", "expert_order", "group_offsets", "row_group", "sched"]


class DMoETopology(ctypes.Structure):
    _fields_ = [(n, c_void_p) for n in _TOPO_FIELDS]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libdmoe.so (built in-tree by paper_2211_15841_amd.build); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise DMoEError("libdmoe.so is not built: run `python -m paper_2211_15841_amd.build` "
                        "(or __graft_entry__.build()); there is no fallback path")
    # torch ships its own HIP runtime; make sure that one is the copy already resident so that stream handles
    # and device pointers created by torch are valid inside the library.
    hip_rt = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
    if os.path.exists(hip_rt):
        ctypes.CDLL(hip_rt, mode=ctypes.RTLD_GLOBAL)
    lib = ctypes.CDLL(LIB_PATH)
    lib.dmoe_sizes.argtypes = [POINTER(DMoEConfig), POINTER(c_size_t), POINTER(c_size_t), POINTER(c_size_t),
                               POINTER(c_int32), POINTER(c_int32)]
    lib.dmoe_topology_bind.argtypes = [POINTER(DMoEConfig), c_void_p, c_size_t, POINTER(DMoETopology)]
    lib.dmoe_topology.argtypes = [POINTER(DMoEConfig), c_void_p, c_void_p, c_void_p, POINTER(DMoETopology), c_void_p,
                                  c_size_t, c_void_p]
    lib.dmoe_topology_static.argtypes = [POINTER(DMoEConfig), c_void_p, c_void_p, c_void_p, POINTER(DMoETopology),
                                         c_void_p]
    lib.dmoe_forward.argtypes = [POINTER(DMoEConfig), c_void_p, c_void_p, c_void_p, POINTER(DMoETopology), c_void_p,
                                 c_void_p, c_size_t, c_void_p, c_size_t, c_void_p]
    lib.dmoe_backward.argtypes = [POINTER(DMoEConfig), c_void_p, c_void_p, c_void_p, c_void_p, POINTER(DMoETopology),
                                  c_void_p, c_size_t, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                  c_size_t, c_void_p]
    lib.dmoe_backward_accumulate.argtypes = lib.dmoe_backward.argtypes
    lib.dmoe_topology_counts_host.argtypes = [POINTER(DMoETopology), POINTER(c_int32), c_void_p]
    lib.dmoe_set_stage_events.argtypes = [c_void_p]
    lib.dmoe_debug_scratch_offset.argtypes = [POINTER(DMoEConfig), c_char_p, POINTER(c_size_t)]
    lib.dmoe_debug_scratch_offset.restype = ctypes.c_int
    lib.dmoe_debug_trace.argtypes = [c_void_p, c_size_t, ctypes.c_int]
    lib.dmoe_debug_trace.restype = ctypes.c_int
    lib.dmoe_set_tile_mode.argtypes = [ctypes.c_int]
    lib.dmoe_bsmm_sizes.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, POINTER(c_size_t)]
    lib.dmoe_bsmm_topology.argtypes = [c_void_p, ctypes.c_int, ctypes.c_int, c_void_p, c_size_t,
                                       POINTER(DMoETopology), POINTER(c_int32)]
    lib.dmoe_bsmm.argtypes = [ctypes.c_int, POINTER(DMoETopology), ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                              c_void_p, c_void_p, c_void_p, c_void_p]
    lib.dmoe_probe_mfma_tflops.argtypes = [POINTER(ctypes.c_float), c_void_p, c_void_p]
    lib.dmoe_probe_mfma_sustained.argtypes = [POINTER(ctypes.c_float), POINTER(ctypes.c_float), ctypes.c_float, c_void_p,
                                              c_void_p]
    lib.dmoe_last_error.restype = c_char_p
    for name in ("dmoe_sizes", "dmoe_topology_bind", "dmoe_topology", "dmoe_topology_static", "dmoe_forward", "dmoe_backward",
                 "dmoe_backward_accumulate", "dmoe_topology_counts_host", "dmoe_set_stage_events", "dmoe_set_tile_mode", "dmoe_bsmm_sizes",
                 "dmoe_bsmm_topology", "dmoe_bsmm", "dmoe_probe_mfma_tflops", "dmoe_probe_mfma_sustained"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def dmoe_last_error() -> str:
    return load_library().dmoe_last_error().decode()


def _check(rc: int):
    if rc != 0:
        raise DMoEError("dmoe error %d: %s" % (rc, dmoe_last_error()))


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def dmoe_sizes(cfg: DMoEConfig) -> dict:
    tb, sb, wb = c_size_t(), c_size_t(), c_size_t()
    pm, nm = c_int32(), c_int32()
    _check(load_library().dmoe_sizes(byref(cfg), byref(tb), byref(sb), byref(wb), byref(pm), byref(nm)))
    return {"topology_bytes": tb.value, "saved_bytes": sb.value, "scratch_bytes": wb.value, "P_max": pm.value,
            "nnz_max": nm.value}


def dmoe_topology_bind(cfg: DMoEConfig, topology_mem, nbytes: int) -> DMoETopology:
    topo = DMoETopology()
    _check(load_library().dmoe_topology_bind(byref(cfg), _ptr(topology_mem), nbytes, byref(topo)))
    return topo


def dmoe_topology(cfg, x, w_router, router_bias, topo, scratch, scratch_bytes, stream=None):
    _check(load_library().dmoe_topology(byref(cfg), _ptr(x), _ptr(w_router), _ptr(router_bias), byref(topo),
                                        _ptr(scratch), scratch_bytes, _stream(stream)))


def dmoe_topology_static(cfg, x, w_router, router_bias, topo, stream=None):
    _check(load_library().dmoe_topology_static(byref(cfg), _ptr(x), _ptr(w_router), _ptr(router_bias), byref(topo),
                                               _stream(stream)))


def dmoe_forward(cfg, x, w1, w2, topo, y, saved, saved_bytes, scratch, scratch_bytes, stream=None):
    _check(load_library().dmoe_forward(byref(cfg), _ptr(x), _ptr(w1), _ptr(w2), byref(topo), _ptr(y), _ptr(saved),
                                       saved_bytes, _ptr(scratch), scratch_bytes, _stream(stream)))


def dmoe_backward(cfg, x, w_router, w1, w2, topo, saved, saved_bytes, dy, dx, dw_router, dw1, dw2, scratch,
                  scratch_bytes, stream=None):
    _check(load_library().dmoe_backward(byref(cfg), _ptr(x), _ptr(w_router), _ptr(w1), _ptr(w2), byref(topo),
                                        _ptr(saved), saved_bytes, _ptr(dy), _ptr(dx), _ptr(dw_router), _ptr(dw1),
                                        _ptr(dw2), _ptr(scratch), scratch_bytes, _stream(stream)))


def dmoe_backward_accumulate(cfg, x, w_router, w1, w2, topo, saved, saved_bytes, dy, dx, dw_router_acc, dw1_acc,
                             dw2_acc, scratch, scratch_bytes, stream=None):
    for name, t in (("dw_router_acc", dw_router_acc), ("dw1_acc", dw1_acc), ("dw2_acc", dw2_acc)):
        if t.dtype != torch.float32:
            raise TypeError("%s must be float32 (got %s)" % (name, t.dtype))
    _check(load_library().dmoe_backward_accumulate(byref(cfg), _ptr(x), _ptr(w_router), _ptr(w1), _ptr(w2),
                                                   byref(topo), _ptr(saved), saved_bytes, _ptr(dy), _ptr(dx),
                                                   _ptr(dw_router_acc), _ptr(dw1_acc), _ptr(dw2_acc), _ptr(scratch),
                                                   scratch_bytes, _stream(stream)))


def dmoe_topology_counts_host(topo, stream=None):
    out = (c_int32 * 4)()
    _check(load_library().dmoe_topology_counts_host(byref(topo), out, _stream(stream)))
    return list(out)


OP_SDD, OP_DSD, OP_SDDT, OP_DSTD, OP_DSDT, OP_DDTS, OP_DDS, OP_SDTD, OP_SDTDT, OP_DSTDT, OP_DDST, OP_DDTST = range(12)


def dmoe_bsmm_sizes(block_rows: int, block_cols: int, nnz: int) -> int:
    nbytes = c_size_t()
    _check(load_library().dmoe_bsmm_sizes(block_rows, block_cols, nnz, byref(nbytes)))
    return nbytes.value


def dmoe_bsmm_topology(mask, topology_mem, nbytes: int):
    """mask: host uint8 array [block_rows, block_cols] (numpy, C-contiguous).  Returns (topology struct, nnz)."""
    rows, cols = mask.shape
    topo, nnz = DMoETopology(), c_int32()
    _check(load_library().dmoe_bsmm_topology(mask.ctypes.data, rows, cols, _ptr(topology_mem), nbytes, byref(topo),
                                             byref(nnz)))
    return topo, nnz.value


def dmoe_bsmm(op: int, topo, block_rows: int, block_cols: int, nnz: int, dense: int, a, b, out, stream=None):
    _check(load_library().dmoe_bsmm(op, byref(topo), block_rows, block_cols, nnz, dense, _ptr(a), _ptr(b), _ptr(out),
                                    _stream(stream)))


class BlockSparse:
    """A 128x128 block mask on the device plus the six products on it (argument marshalling only)."""

    def __init__(self, mask, device="cuda:0"):
        import numpy as np
        self.mask = np.ascontiguousarray(mask, dtype=np.uint8)
        self.rows, self.cols = self.mask.shape
        nbytes = dmoe_bsmm_sizes(self.rows, self.cols, int((self.mask != 0).sum()))
        self.topology_mem = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.topo, self.nnz = dmoe_bsmm_topology(self.mask, self.topology_mem, nbytes)
        self.device = device

    def _out(self, *shape):
        return torch.empty(*shape, dtype=torch.bfloat16, device=self.device)

    def sdd(self, x, w, stream=None):        # x [M, D], w [D, N] -> S [nnz, 128, 128]
        out = self._out(max(self.nnz, 1), 128, 128)
        dmoe_bsmm(OP_SDD, self.topo, self.rows, self.cols, self.nnz, x.shape[1], x, w, out, stream)
        return out[:self.nnz]

    def sddt(self, x, w, stream=None):       # x [M, D], w [N, D] -> S
        out = self._out(max(self.nnz, 1), 128, 128)
        dmoe_bsmm(OP_SDDT, self.topo, self.rows, self.cols, self.nnz, x.shape[1], x, w, out, stream)
        return out[:self.nnz]

    def dsd(self, s, w, stream=None):        # s [nnz, 128, 128], w [N, D] -> [M, D]
        out = self._out(self.rows * 128, w.shape[1])
        dmoe_bsmm(OP_DSD, self.topo, self.rows, self.cols, self.nnz, w.shape[1], s, w, out, stream)
        return out

    def dsdt(self, s, w, stream=None):       # w [D, N] -> [M, D]
        out = self._out(self.rows * 128, w.shape[0])
        dmoe_bsmm(OP_DSDT, self.topo, self.rows, self.cols, self.nnz, w.shape[0], s, w, out, stream)
        return out

    def dstd(self, s, x, stream=None):       # x [M, D] -> [N, D]
        out = self._out(self.cols * 128, x.shape[1])
        dmoe_bsmm(OP_DSTD, self.topo, self.rows, self.cols, self.nnz, x.shape[1], s, x, out, stream)
        return out

    def ddts(self, x, s, stream=None):       # x [M, D] -> [D, N]
        out = self._out(x.shape[1], self.cols * 128)
        dmoe_bsmm(OP_DDTS, self.topo, self.rows, self.cols, self.nnz, x.shape[1], x, s, out, stream)
        return out

    def dds(self, x, s, stream=None):        # x [D, M] -> [D, N]
        if x.shape[1] != self.rows * 128:
            raise ValueError("x must have %d columns (got %d)" % (self.rows * 128, x.shape[1]))
        out = self._out(x.shape[0], self.cols * 128)
        dmoe_bsmm(OP_DDS, self.topo, self.rows, self.cols, self.nnz, x.shape[0], x, s, out, stream)
        return out

    # the remaining combinations of transposed inputs (a T after the operand's letter)
    def sdtd(self, x, w, stream=None):       # x [D, M], w [D, N] -> S = X^T W on the mask
        out = self._out(max(self.nnz, 1), 128, 128)
        dmoe_bsmm(OP_SDTD, self.topo, self.rows, self.cols, self.nnz, x.shape[0], x, w, out, stream)
        return out[:self.nnz]

    def sdtdt(self, x, w, stream=None):      # x [D, M], w [N, D] -> S = X^T W^T on the mask
        out = self._out(max(self.nnz, 1), 128, 128)
        dmoe_bsmm(OP_SDTDT, self.topo, self.rows, self.cols, self.nnz, x.shape[0], x, w, out, stream)
        return out[:self.nnz]

    def dstdt(self, s, x, stream=None):      # x [D, M] -> S^T X^T [N, D]
        out = self._out(self.cols * 128, x.shape[0])
        dmoe_bsmm(OP_DSTDT, self.topo, self.rows, self.cols, self.nnz, x.shape[0], s, x, out, stream)
        return out

    def ddst(self, x, s, stream=None):       # x [D, N] -> X S^T [D, M]
        out = self._out(x.shape[0], self.rows * 128)
        dmoe_bsmm(OP_DDST, self.topo, self.rows, self.cols, self.nnz, x.shape[0], x, s, out, stream)
        return out

    def ddtst(self, x, s, stream=None):      # x [N, D] -> X^T S^T [D, M]
        out = self._out(x.shape[1], self.rows * 128)
        dmoe_bsmm(OP_DDTST, self.topo, self.rows, self.cols, self.nnz, x.shape[1], x, s, out, stream)
        return out


def dmoe_probe_mfma_tflops(stream=None) -> float:
    """bf16 MFMA rate of a register-only loop on this device, TFLOP/s (synchronises)."""
    out = ctypes.c_float()
    scratch = torch.zeros(64, dtype=torch.float32, device="cuda")
    _check(load_library().dmoe_probe_mfma_tflops(byref(out), _ptr(scratch), _stream(stream)))
    return out.value


def dmoe_probe_mfma_sustained(seconds: float = 0.3, stream=None):
    """(TFLOP/s, shader GHz) of the register-only bf16 MFMA loop after about `seconds` of sustained load (synchronises)."""
    tf, ghz = ctypes.c_float(), ctypes.c_float()
    scratch = torch.zeros(64, dtype=torch.float32, device="cuda")
    _check(load_library().dmoe_probe_mfma_sustained(byref(tf), byref(ghz), float(seconds), _ptr(scratch),
                                                    _stream(stream)))
    return tf.value, ghz.value


def dmoe_set_tile_mode(mode: int):
    """0: tile shape chosen from the configuration, 1: 128x128 blocks, 2: 256x256 macro tiles."""
    _check(load_library().dmoe_set_tile_mode(mode))


def dmoe_set_stage_events(events_array):
    """events_array: ctypes array of 2*len(STAGE_NAMES) hipEvent_t handles (0 = skip), or None."""
    load_library().dmoe_set_stage_events(events_array)


class Workspace:
    """Caller-side buffers for one layer configuration, allocated once with torch (device memory only)."""

    GUARD_BYTE = 0xA5

    def __init__(self, num_tokens, d_model, ffn_hidden, num_experts, top_k, normalize_topk=0, device="cuda:0",
                 activation=0, guard_bytes=0, expert_capacity=0, pad_to_capacity=0):
        """guard_bytes > 0 (tests): every buffer the library writes sits between two guard zones of that many bytes
        holding a fixed pattern; check_guards() then tells whether any kernel wrote outside its buffer."""
        self.cfg = DMoEConfig(num_tokens, d_model, ffn_hidden, num_experts, top_k, 128, activation, normalize_topk,
                              expert_capacity, pad_to_capacity)
        self.device = torch.device(device)
        self.sizes = dmoe_sizes(self.cfg)
        self.guard_bytes = (int(guard_bytes) + 255) // 256 * 256
        self._guarded = []
        self.topology_mem = self._alloc(self.sizes["topology_bytes"], "topology")
        self.saved = self._alloc(self.sizes["saved_bytes"], "saved")
        self.scratch = self._alloc(self.sizes["scratch_bytes"], "scratch")
        self.topo = dmoe_topology_bind(self.cfg, self.topology_mem, self.sizes["topology_bytes"])
        T, d, h, E = num_tokens, d_model, ffn_hidden, num_experts
        bf = torch.bfloat16
        self.y = self._alloc(T * d * 2, "y").view(bf).view(T, d)
        self.dx = self._alloc(T * d * 2, "dx").view(bf).view(T, d)
        self.dw1 = self._alloc(d * E * h * 2, "dw1").view(bf).view(d, E * h)
        self.dw2 = self._alloc(E * h * d * 2, "dw2").view(bf).view(E * h, d)
        self.dw_router = self._alloc(d * E * 4, "dw_router").view(torch.float32).view(d, E)

    def _alloc(self, nbytes, name):
        g = self.guard_bytes
        if not g:
            return torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        body = (nbytes + 255) // 256 * 256
        whole = torch.full((body + 2 * g,), self.GUARD_BYTE, dtype=torch.uint8, device=self.device)
        self._guarded.append((name, whole, g, nbytes))
        return whole[g:g + nbytes]

    def check_guards(self):
        """Raises if any byte of a guard zone (or of the alignment tail behind a buffer) has changed."""
        torch.cuda.synchronize(self.device)
        for name, whole, g, nbytes in self._guarded:
            lo, hi = whole[:g], whole[g + nbytes:]
            for side, z in (("below", lo), ("above", hi)):
                bad = (z != self.GUARD_BYTE).nonzero()
                if bad.numel():
                    first = int(bad[0]) - (g if side == "below" else 0)
                    raise DMoEError("%d bytes written %s buffer '%s' (first at offset %+d from its %s)"
                                    % (bad.numel(), side, name, first, "start" if side == "below" else "end"))

    # -- the three calls of the layer ---------------------------------------------------------------------
    def topology(self, x, w_router, router_bias=None, stream=None):
        dmoe_topology(self.cfg, x, w_router, router_bias, self.topo, self.scratch, self.sizes["scratch_bytes"], stream)

    def topology_static(self, x, w_router, router_bias=None, stream=None):
        """dmoe_topology with the library's built-in scratch instead of this workspace's."""
        dmoe_topology_static(self.cfg, x, w_router, router_bias, self.topo, stream)

    def forward(self, x, w1, w2, stream=None):
        dmoe_forward(self.cfg, x, w1, w2, self.topo, self.y, self.saved, self.sizes["saved_bytes"], self.scratch,
                     self.sizes["scratch_bytes"], stream)
        return self.y

    def backward(self, x, w_router, w1, w2, dy, stream=None):
        dmoe_backward(self.cfg, x, w_router, w1, w2, self.topo, self.saved, self.sizes["saved_bytes"], dy, self.dx,
                      self.dw_router, self.dw1, self.dw2, self.scratch, self.sizes["scratch_bytes"], stream)
        return self.dx, self.dw_router, self.dw1, self.dw2

    def backward_accumulate(self, x, w_router, w1, w2, dy, dw_router_acc, dw1_acc, dw2_acc, stream=None):
        """Backward pass that adds the weight gradients to the caller's fp32 accumulators; returns dx."""
        dmoe_backward_accumulate(self.cfg, x, w_router, w1, w2, self.topo, self.saved, self.sizes["saved_bytes"], dy,
                                 self.dx, dw_router_acc, dw1_acc, dw2_acc, self.scratch, self.sizes["scratch_bytes"],
                                 stream)
        return self.dx

    # -- read-back of the topology arrays (tests) ----------------------------------------------------------
    def topology_arrays(self) -> dict:
        """Copies of the routing/topology arrays as CPU torch tensors, trimmed to their valid lengths."""
        torch.cuda.synchronize(self.device)
        c = self.cfg
        F, E, hb = c.num_tokens * c.top_k, c.num_experts, c.ffn_hidden // 128
        P, R, nnz, _ = dmoe_topology_counts_host(self.topo)
        base = self.topology_mem.data_ptr()

        def view(name, n, dtype):
            off = getattr(self.topo, name) - base
            return self.topology_mem[off:off + 4 * n].view(dtype).cpu()

        i32, f32 = torch.int32, torch.float32
        groups = int(view("group_offsets", E + 1, i32)[E])
        return {
            "expert_idx": view("expert_idx", F, i32).reshape(c.num_tokens, c.top_k),
            "weights": view("weights", F, f32).reshape(c.num_tokens, c.top_k),
            "logits": view("logits", c.num_tokens * E, f32).reshape(c.num_tokens, E),
            "tokens_per_expert": view("tokens_per_expert", E, i32),
            "padded_offsets": view("padded_offsets", E + 1, i32),
            "row_of": view("row_of", F, i32),
            "token_of": view("token_of", P, i32),
            "row_offsets": view("row_offsets", R + 1, i32),
            "column_indices": view("column_indices", nnz, i32),
            "row_indices": view("row_indices", nnz, i32),
            "column_offsets_t": view("column_offsets_t", E * hb + 1, i32),
            "row_indices_t": view("row_indices_t", nnz, i32),
            "block_offsets_t": view("block_offsets_t", nnz, i32),
            "counts": torch.tensor([P, R, nnz, 0], dtype=i32),
            "expert_order": view("expert_order", E, i32),
            "group_offsets": view("group_offsets", E + 1, i32),
            "row_group": view("row_group", groups, i32),
            "sched": view("sched", 4, i32),
        }
