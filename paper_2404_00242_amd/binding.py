"""ctypes binding over libdeft's C ABI (see include/deft.h).

Argument marshalling only: the plan is built by the library's host code, every
step of the attention path runs in the library's HIP kernels.  PyTorch supplies
device memory and the stream.  There is no fallback: if libdeft.so is missing or
a call fails, an exception is raised.
"""

from __future__ import annotations

import ctypes
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
# DEFT_LIB lets a developer point the binding at another build of the same library (A/B timing runs)
LIB_PATH = os.environ.get("DEFT_LIB") or os.path.join(_PKG, "libdeft.so")

DEFT_OUT_BF16 = 0
DEFT_OUT_F32 = 1
# deft_plan flags: how the tree's KV is partitioned and grouped with queries
DEFT_SPLIT_FLATTEN = 0
DEFT_SPLIT_NODE = 1
DEFT_SPLIT_NODE_CHUNK = 2
DEFT_GROUP_QUERY = 3
DEFT_SPLIT_BALANCED = 4  # or rows_per_query(Hq // Hkv) to it
DEFT_PRECISE_WEIGHTS = 0x100  # or-ed to a mode: two-term softmax weights in every group
SPLIT_MODES = {"flatten": DEFT_SPLIT_FLATTEN, "node": DEFT_SPLIT_NODE, "node_chunk": DEFT_SPLIT_NODE_CHUNK,
               "query": DEFT_GROUP_QUERY, "balanced": DEFT_SPLIT_BALANCED}


def rows_per_query(g: int) -> int:
    """DEFT_ROWS_PER_QUERY(g): the flag bits that tell DEFT_SPLIT_BALANCED how many query heads share a KV head"""
    return (int(g) & 0xFFF) << 16

EXPORTS = (
    "deft_plan", "deft_plan_paged", "deft_plan_update", "deft_plan_paged_update", "deft_suggest_chunk_size", "deft_plan_view", "deft_plan_device_bytes", "deft_plan_upload", "deft_workspace_bytes",
    "deft_tree_attn_decode", "deft_tree_attn_decode_static", "deft_stage1_partial_attention", "deft_stage2_global_reduction",
    "deft_hbm_read_probe", "deft_plan_destroy", "deft_strerror", "deft_last_hip_error",
)

_i32p = ctypes.POINTER(ctypes.c_int32)
_u64p = ctypes.POINTER(ctypes.c_uint64)

_VIEW_SCALARS = ("chunk_size", "n_nodes", "nq", "n_flat", "n_chunks", "n_segs", "n_slots", "n_mask_words")
# name -> (ctype pointer, length as a function of the scalars)
_VIEW_ARRAYS = (
    ("q_order", _i32p, lambda s: s["nq"]),
    ("node_q_lo", _i32p, lambda s: s["n_nodes"]),
    ("node_q_hi", _i32p, lambda s: s["n_nodes"]),
    ("chunk_seg_ptr", _i32p, lambda s: s["n_chunks"] + 1),
    ("seg_tok_begin", _i32p, lambda s: s["n_segs"]),
    ("seg_len", _i32p, lambda s: s["n_segs"]),
    ("seg_qlo", _i32p, lambda s: s["n_segs"]),
    ("seg_qhi", _i32p, lambda s: s["n_segs"]),
    ("seg_node", _i32p, lambda s: s["n_segs"]),
    ("chunk_qlo", _i32p, lambda s: s["n_chunks"]),
    ("chunk_qhi", _i32p, lambda s: s["n_chunks"]),
    ("chunk_slot_base", _i32p, lambda s: s["n_chunks"] + 1),
    ("seg_mask_ptr", _i32p, lambda s: s["n_segs"] + 1),
    ("seg_mask", _u64p, lambda s: s["n_mask_words"]),
    ("q_part_ptr", _i32p, lambda s: s["nq"] + 1),
    ("q_part_chunk", _i32p, lambda s: s["n_slots"]),
    ("q_part_slot", _i32p, lambda s: s["n_slots"]),
)


class _PlanView(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in _VIEW_SCALARS] + [(n, t) for n, t, _ in _VIEW_ARRAYS]


class DeftError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(what)


_lib = None


def load_library():
    """Loads libdeft.so (built by paper_2404_00242_amd.build); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2404_00242_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, c32, csz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    lib.deft_plan.restype = ctypes.c_int
    lib.deft_plan.argtypes = [_i32p, _i32p, _i32p, c32, _i32p, c32, c32, c32, ctypes.c_uint32, ctypes.POINTER(vp)]
    lib.deft_plan_paged.restype = ctypes.c_int
    lib.deft_plan_paged.argtypes = [_i32p, _i32p, c32, c32, _i32p, _i32p, c32, _i32p, c32, c32, ctypes.c_uint32,
                                    ctypes.POINTER(vp)]
    lib.deft_plan_update.restype = ctypes.c_int
    lib.deft_plan_update.argtypes = [vp] + lib.deft_plan.argtypes
    lib.deft_plan_paged_update.restype = ctypes.c_int
    lib.deft_plan_paged_update.argtypes = [vp] + lib.deft_plan_paged.argtypes
    lib.deft_suggest_chunk_size.restype = ctypes.c_int32
    lib.deft_suggest_chunk_size.argtypes = [_i32p, _i32p, c32, _i32p, c32, c32, c32, ctypes.c_uint32]
    lib.deft_plan_view.restype = ctypes.c_int
    lib.deft_plan_view.argtypes = [vp, ctypes.POINTER(_PlanView)]
    lib.deft_plan_device_bytes.restype = csz
    lib.deft_plan_device_bytes.argtypes = [vp, c32, c32]
    lib.deft_plan_upload.restype = ctypes.c_int
    lib.deft_plan_upload.argtypes = [vp, c32, c32, vp, csz, vp]
    lib.deft_workspace_bytes.restype = csz
    lib.deft_workspace_bytes.argtypes = [vp, c32, c32, c32]
    lib.deft_tree_attn_decode.restype = ctypes.c_int
    lib.deft_tree_attn_decode.argtypes = [vp, vp, vp, vp, vp, vp, c32, c32, c32, ctypes.c_float, ctypes.c_uint32,
                                          vp, csz, vp]
    lib.deft_tree_attn_decode_static.restype = ctypes.c_int
    lib.deft_tree_attn_decode_static.argtypes = [vp, vp, vp, vp, vp, vp, c32, c32, c32, ctypes.c_float, ctypes.c_uint32,
                                                 vp]
    lib.deft_stage1_partial_attention.restype = ctypes.c_int
    lib.deft_stage1_partial_attention.argtypes = [vp, vp, vp, vp, vp, c32, c32, c32, ctypes.c_float, vp, csz, vp]
    lib.deft_stage2_global_reduction.restype = ctypes.c_int
    lib.deft_stage2_global_reduction.argtypes = [vp, vp, vp, c32, c32, c32, ctypes.c_float, ctypes.c_uint32, vp, csz,
                                                 vp]
    lib.deft_hbm_read_probe.restype = ctypes.c_int
    lib.deft_hbm_read_probe.argtypes = [vp, csz, vp, vp]
    lib.deft_plan_destroy.restype = None
    lib.deft_plan_destroy.argtypes = [vp]
    lib.deft_strerror.restype = ctypes.c_char_p
    lib.deft_strerror.argtypes = [ctypes.c_int]
    lib.deft_last_hip_error.restype = ctypes.c_char_p
    lib.deft_last_hip_error.argtypes = []
    _lib = lib
    return lib


def _check(status: int, what: str):
    if status != 0:
        lib = load_library()
        msg = lib.deft_strerror(status).decode()
        if status == -4:
            msg += " (" + lib.deft_last_hip_error().decode() + ")"
        raise DeftError(status, f"{what}: {msg} [{status}]")


def _i32(x):
    return np.ascontiguousarray(np.asarray(x), dtype=np.int32).reshape(-1)


class Plan:
    """Owns a deft_plan_t handle and, per Hq/Hkv ratio, the device image uploaded for it."""

    def __init__(self, handle):
        self._h = handle
        self._images = {}      # (G, device index) -> torch uint8 tensor holding the device image
        self._workspaces = {}  # (Hq, Hkv, d, device index) -> torch uint8 tensor
        self._view = None

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.deft_plan_destroy(h)

    @property
    def handle(self):
        return self._h

    def view(self) -> dict:
        """The canonical plan as numpy arrays (copies), keyed like include/deft.h's deft_plan_view_t."""
        if self._view is None:
            v = _PlanView()
            _check(load_library().deft_plan_view(self._h, ctypes.byref(v)), "deft_plan_view")
            out = {n: int(getattr(v, n)) for n in _VIEW_SCALARS}
            for name, ctype, length in _VIEW_ARRAYS:
                n = length(out)
                ptr = getattr(v, name)
                dt = np.uint64 if ctype is _u64p else np.int32
                out[name] = np.ctypeslib.as_array(ptr, shape=(n,)).copy() if n > 0 else np.zeros(0, dtype=dt)
            self._view = out
        return self._view

    def device_bytes(self, Hq: int, Hkv: int) -> int:
        return int(load_library().deft_plan_device_bytes(self._h, Hq, Hkv))

    def workspace_bytes(self, Hq: int, Hkv: int, d: int) -> int:
        return int(load_library().deft_workspace_bytes(self._h, Hq, Hkv, d))

    def image(self, Hq: int, Hkv: int, device, stream=None):
        """Device image for this Hq/Hkv ratio, uploaded on first use (memory comes from torch).

        deft_plan_upload only enqueues the copy on the stream of that first call.  An event recorded behind it
        is kept with the image, and a later call on another stream makes that stream wait for the event, so
        that no kernel can read the image before the copy has landed."""
        import torch

        device = torch.device(device)
        if stream is None:
            stream = torch.cuda.current_stream(device)
        key = (Hq // Hkv, device.index)
        entry = self._images.get(key)
        if entry is None:
            nbytes = self.device_bytes(Hq, Hkv)
            if nbytes == 0:
                raise DeftError(-1, "deft_plan_device_bytes: invalid Hq/Hkv")
            img = torch.empty(nbytes, dtype=torch.uint8, device=device)
            st = _stream_ptr(stream, device)
            _check(load_library().deft_plan_upload(self._h, Hq, Hkv, img.data_ptr(), nbytes, st), "deft_plan_upload")
            uploaded = None
            if hasattr(stream, "record_event"):
                uploaded = torch.cuda.Event()
                stream.record_event(uploaded)
            entry = (img, uploaded, getattr(stream, "cuda_stream", stream))
            self._images[key] = entry
        img, uploaded, on = entry
        if uploaded is not None:
            if uploaded.query():  # the copy has landed: nothing to order any more
                self._images[key] = (img, None, on)
            elif getattr(stream, "cuda_stream", stream) != on and hasattr(stream, "wait_event"):
                stream.wait_event(uploaded)
        return img

    def workspace(self, Hq: int, Hkv: int, d: int, device):
        import torch

        device = torch.device(device)
        key = (Hq, Hkv, d, device.index)
        ws = self._workspaces.get(key)
        if ws is None:
            nbytes = self.workspace_bytes(Hq, Hkv, d)
            if nbytes == 0:
                raise DeftError(-1, "deft_workspace_bytes: invalid head shape")
            ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
            self._workspaces[key] = ws
        return ws


def _stream_ptr(stream, device):
    import torch

    if stream is None:
        stream = torch.cuda.current_stream(device)
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def deft_suggest_chunk_size(node_tok_len, node_parent, query_node, Hq: int, Hkv: int, flags: int = 0) -> int:
    """Chunk size S_t suited to this tree for the split named by flags (about two equal stage-1 tasks per
    compute unit)."""
    nl, par, qn = _i32(node_tok_len), _i32(node_parent), _i32(query_node)
    qptr = qn.ctypes.data_as(_i32p) if qn.size else None
    rc = load_library().deft_suggest_chunk_size(nl.ctypes.data_as(_i32p), par.ctypes.data_as(_i32p), nl.size, qptr,
                                                qn.size, int(Hq), int(Hkv), int(flags))
    if rc < 0:
        _check(rc, "deft_suggest_chunk_size")
    return int(rc)


def deft_plan(node_tok_begin, node_tok_len, node_parent, query_node, ntok: int, chunk_size: int = 0,
              flags: int = 0, prev: "Plan | None" = None) -> Plan:
    """QKV Preparation Phase (Algorithm 3): builds the flattened chunk / bit-mask plan on the host.
    prev: the plan of an earlier version of the tree (deft_plan_update: same result, less work)."""
    lib = load_library()
    nb, nl, par, qn = _i32(node_tok_begin), _i32(node_tok_len), _i32(node_parent), _i32(query_node)
    if not (nb.size == nl.size == par.size):
        raise DeftError(-1, "deft_plan: node table columns differ in length")
    out = ctypes.c_void_p()
    qptr = qn.ctypes.data_as(_i32p) if qn.size else None
    args = (nb.ctypes.data_as(_i32p), nl.ctypes.data_as(_i32p), par.ctypes.data_as(_i32p), nb.size,
            qptr, qn.size, int(ntok), int(chunk_size), int(flags), ctypes.byref(out))
    if prev is None:
        _check(lib.deft_plan(*args), "deft_plan")
    else:
        _check(lib.deft_plan_update(prev.handle, *args), "deft_plan_update")
    return Plan(out)


def deft_plan_paged(node_page_ptr, page_ids, page_size: int, n_pool_pages: int, node_tok_len, node_parent,
                    query_node, chunk_size: int = 0, flags: int = 0, prev: "Plan | None" = None) -> Plan:
    """QKV Preparation Phase over a paged KV pool (K/V are [n_pool_pages * page_size, Hkv, d]).
    prev: the plan of an earlier version of the tree (deft_plan_paged_update: same result, less work)."""
    lib = load_library()
    pp, pg, nl, par, qn = (_i32(x) for x in (node_page_ptr, page_ids, node_tok_len, node_parent, query_node))
    if not (nl.size == par.size == pp.size - 1):
        raise DeftError(-1, "deft_plan_paged: node table columns differ in length")
    out = ctypes.c_void_p()
    args = (pp.ctypes.data_as(_i32p), pg.ctypes.data_as(_i32p) if pg.size else None, int(page_size),
            int(n_pool_pages), nl.ctypes.data_as(_i32p), par.ctypes.data_as(_i32p), nl.size,
            qn.ctypes.data_as(_i32p) if qn.size else None, qn.size, int(chunk_size), int(flags), ctypes.byref(out))
    if prev is None:
        _check(lib.deft_plan_paged(*args), "deft_plan_paged")
    else:
        _check(lib.deft_plan_paged_update(prev.handle, *args), "deft_plan_paged_update")
    return Plan(out)


KV_STAGGER_BYTES = 512  # V pool's base relative to the K pool's, modulo 1 KiB


def alloc_kv_cache(n_rows: int, Hkv: int, d: int, device="cuda"):
    """Uninitialised K and V pools [n_rows, Hkv, d] (bf16), carved from one allocation so that the V pool
    starts KV_STAGGER_BYTES past a 1 KiB boundary and the K pool on one.

    Placement only, no arithmetic: on MI355X a compute unit reads fastest when the rows it has in flight
    differ in address bits 7..9.  K and V rows of one head sit at the same offset of their pools, so with
    both pools on the same alignment every row a workgroup streams shares those bits; half a KiB between
    the pools' alignments spreads them (measured on the few-shot benchmark: stage 1 30.5 -> 29.4 us).
    Any 16-byte aligned K and V are accepted by the kernels; this is merely the fast layout."""
    import torch

    pool = n_rows * Hkv * d * 2
    k_span = -(-pool // 1024) * 1024
    buf = torch.empty(1024 + k_span + KV_STAGGER_BYTES + pool, dtype=torch.uint8, device=device)
    k_off = (-buf.data_ptr()) % 1024
    v_off = k_off + k_span + KV_STAGGER_BYTES
    k = buf[k_off:k_off + pool].view(torch.bfloat16).view(n_rows, Hkv, d)
    v = buf[v_off:v_off + pool].view(torch.bfloat16).view(n_rows, Hkv, d)
    return k, v


def deft_tree_attn_decode(plan: Plan, q, k, v, out=None, scale: float = 0.0, out_dtype=None, workspace=None,
                          stream=None):
    """Attention Calculation Phase (Algorithm 4) on the GPU.

    q [nq,Hq,d], k/v [ntok,Hkv,d]: contiguous bf16 CUDA(HIP) tensors.  Returns o [nq,Hq,d] (bf16, or
    float32 when out_dtype / out says so), in the caller's query order.  Asynchronous on `stream`
    (default: torch's current stream).
    """
    import torch

    if not (q.is_cuda and k.is_cuda and v.is_cuda):
        raise DeftError(-1, "deft_tree_attn_decode: q, k, v must be device tensors (there is no CPU path)")
    for name, t in (("q", q), ("k", k), ("v", v)):
        if t.dtype != torch.bfloat16 or not t.is_contiguous() or t.dim() != 3:
            raise DeftError(-1, f"deft_tree_attn_decode: {name} must be a contiguous 3-d bf16 tensor")
    nq, Hq, d = q.shape
    ntok, Hkv, d2 = k.shape
    if v.shape != k.shape or d2 != d:
        raise DeftError(-1, "deft_tree_attn_decode: k and v must both be [ntok, Hkv, d]")
    view = plan.view()
    if nq != view["nq"]:
        raise DeftError(-1, "deft_tree_attn_decode: q has a different number of queries than the plan")
    if view["n_segs"] and int((view["seg_tok_begin"] + view["seg_len"]).max()) > ntok:
        raise DeftError(-1, "deft_tree_attn_decode: the plan addresses rows beyond the KV cache")
    dev = q.device
    if out is None:
        out = torch.empty((nq, Hq, d), dtype=out_dtype or torch.bfloat16, device=dev)
    if out.shape != (nq, Hq, d) or not out.is_contiguous() or out.device != dev:
        raise DeftError(-1, "deft_tree_attn_decode: out must be a contiguous [nq, Hq, d] tensor on q's device")
    if out.dtype == torch.bfloat16:
        flags = DEFT_OUT_BF16
    elif out.dtype == torch.float32:
        flags = DEFT_OUT_F32
    else:
        raise DeftError(-1, "deft_tree_attn_decode: out must be bf16 or float32")
    img = plan.image(Hq, Hkv, dev, stream)
    ws = workspace if workspace is not None else plan.workspace(Hq, Hkv, d, dev)
    rc = load_library().deft_tree_attn_decode(
        plan.handle, img.data_ptr(), q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), Hq, Hkv, d,
        float(scale), flags, ws.data_ptr(), ws.numel() * ws.element_size(), _stream_ptr(stream, dev))
    _check(rc, "deft_tree_attn_decode")
    return out
