"""ctypes binding over libdbsa.so: argument marshalling only.

Function names mirror the C ABI (include/dbsa.h).  torch is used for device
memory and the current stream; every step of the attention path runs inside
the library's kernels.  Loading fails loudly when the library has not been
built (``python -m paper_2503_08640_amd.build``); there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdbsa.so")

# Q-tile heights the benchmark launches with for grouped-query models (4 query heads per KV head):
# 64 tokens x 4 heads = four waves of 64 rows per workgroup, one workgroup per compute unit: every
# K/V tile a compute unit fetches serves 256 rows, and each wave issues a quarter of its loads
# (measured against 32-token tiles, two workgroups of two waves per compute unit: pre-encode of
# the 90k pool 8 % faster, prefill of 64-token queries 20 %).  Queries shorter than 64 tokens keep
# 32-token tiles (half the rows of a 64-token tile would be padding).  The full-size GPU tests use
# the same values.
BENCH_BLOCK_M_PREENCODE = 64
BENCH_BLOCK_M_QUERY = 64
BENCH_BLOCK_M_SHORT_QUERY = 32

DBSA_OK = 0
DBSA_ERR_INVALID_ARG = -1
DBSA_ERR_BAD_BOUNDS = -2
DBSA_ERR_BAD_SELECTION = -3
DBSA_ERR_UNSUPPORTED = -4
DBSA_ERR_WORKSPACE = -5
DBSA_ERR_HIP = -6
DBSA_BF16 = 0
DBSA_F32 = 1
DBSA_LAYOUT_HOST_ONLY = 1

EXPORTED_SYMBOLS = (
    "dbsa_strerror", "dbsa_layout_build", "dbsa_layout_build_append", "dbsa_layout_export", "dbsa_layout_export_decode",
    "dbsa_layout_export_decode_groups", "dbsa_layout_export_order", "dbsa_layout_export_positions", "dbsa_layout_destroy", "dbsa_workspace_bytes", "dbsa_preencode_attn",
    "dbsa_query_attn", "dbsa_decode_attn", "dbsa_rope_table", "dbsa_rope_apply", "dbsa_query_attn_rope",
    "dbsa_decode_attn_rope", "dbsa_decode_attn_kv8", "dbsa_decode_attn_kv8_rope", "dbsa_decode_attn_static", "dbsa_pooled_list_blocks", "dbsa_layout_export_matrix_records",
    "dbsa_layout_export_matrix_plan",
    "dbsa_layout_export_schedule",
)
DBSA_STATIC_SCRATCH_BYTES = 32 << 20


class DbsaError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


class PoolDesc(C.Structure):
    _fields_ = [("sink_len", C.c_int32), ("n_demos", C.c_int32), ("demo_offsets", C.POINTER(C.c_int32)),
                ("n_groups", C.c_int32), ("group_demo_offsets", C.POINTER(C.c_int32)), ("prev_window", C.c_int32)]


class SelectDesc(C.Structure):
    _fields_ = [("n_queries", C.c_int32), ("cu_qlens", C.POINTER(C.c_int32)), ("sel_ptr", C.POINTER(C.c_int32)),
                ("sel_idx", C.POINTER(C.c_int32)), ("n_split", C.c_int32), ("page_start", C.POINTER(C.c_int32))]


class Tensor(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("stride_tok", C.c_int64), ("stride_head", C.c_int64)]


_lib = None


def lib() -> C.CDLL:
    """Load libdbsa.so (once).  Raises if it is missing: nothing stands in for it."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_2503_08640_amd.build`")
    L = C.CDLL(LIB_PATH)
    L.dbsa_strerror.restype = C.c_char_p
    L.dbsa_strerror.argtypes = [C.c_int]
    L.dbsa_layout_build.restype = C.c_int
    L.dbsa_layout_build.argtypes = [C.POINTER(PoolDesc), C.POINTER(SelectDesc), C.c_int32, C.c_int32, C.c_int32,
                                    C.c_void_p, C.POINTER(C.c_void_p)]
    L.dbsa_layout_build_append.restype = C.c_int
    L.dbsa_layout_build_append.argtypes = [C.POINTER(PoolDesc), C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                           C.POINTER(C.c_void_p)]
    L.dbsa_layout_export.restype = C.c_int
    L.dbsa_layout_export.argtypes = [C.c_void_p, C.POINTER(C.POINTER(C.c_int32)), C.POINTER(C.c_int64),
                                     C.POINTER(C.POINTER(C.c_int64)), C.POINTER(C.POINTER(C.c_int32)),
                                     C.POINTER(C.c_int64)]
    L.dbsa_layout_export_decode.restype = C.c_int
    L.dbsa_layout_export_decode.argtypes = [C.c_void_p, C.POINTER(C.POINTER(C.c_int64)),
                                            C.POINTER(C.POINTER(C.c_int32)), C.POINTER(C.c_int64),
                                            C.POINTER(C.POINTER(C.c_int64)), C.POINTER(C.c_int32)]
    L.dbsa_layout_export_decode_groups.restype = C.c_int
    L.dbsa_layout_export_decode_groups.argtypes = [
        C.c_void_p, C.POINTER(C.POINTER(C.c_int64)), C.POINTER(C.POINTER(C.c_int32)), C.POINTER(C.c_int64),
        C.POINTER(C.POINTER(C.c_int32)), C.POINTER(C.c_int64), C.POINTER(C.POINTER(C.c_int32)),
        C.POINTER(C.c_int64), C.POINTER(C.POINTER(C.c_int64)), C.POINTER(C.c_int32)]
    L.dbsa_layout_export_positions.restype = C.c_int
    L.dbsa_layout_export_positions.argtypes = [C.c_void_p] + [C.POINTER(C.POINTER(C.c_int32))] * 3
    L.dbsa_layout_export_order.restype = C.c_int
    L.dbsa_layout_export_order.argtypes = [C.c_void_p, C.POINTER(C.POINTER(C.c_int32)), C.POINTER(C.c_int64)]
    L.dbsa_layout_export_schedule.restype = C.c_int
    L.dbsa_layout_export_schedule.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.POINTER(C.c_int32)),
                                              C.POINTER(C.POINTER(C.c_int32))]
    L.dbsa_layout_export_matrix_records.restype = C.c_int
    L.dbsa_layout_export_matrix_records.argtypes = [C.c_void_p, C.POINTER(C.POINTER(C.c_int32)), C.POINTER(C.c_int64),
                                                    C.POINTER(C.c_float)]
    L.dbsa_layout_export_matrix_plan.restype = C.c_int
    L.dbsa_layout_export_matrix_plan.argtypes = [C.c_void_p, C.POINTER(C.POINTER(C.c_int32)), C.POINTER(C.c_int32),
                                                 C.POINTER(C.c_int32), C.POINTER(C.POINTER(C.c_int32)), C.POINTER(C.c_int64),
                                                 C.POINTER(C.POINTER(C.c_int64))]
    L.dbsa_pooled_list_blocks.restype = C.c_int32
    L.dbsa_pooled_list_blocks.argtypes = []
    L.dbsa_layout_destroy.restype = None
    L.dbsa_layout_destroy.argtypes = [C.c_void_p]
    L.dbsa_workspace_bytes.restype = C.c_size_t
    L.dbsa_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
    tail = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_size_t, C.c_void_p]
    L.dbsa_preencode_attn.restype = C.c_int
    L.dbsa_preencode_attn.argtypes = [C.c_void_p, Tensor, Tensor, Tensor, Tensor, C.c_void_p] + tail
    L.dbsa_query_attn.restype = C.c_int
    L.dbsa_query_attn.argtypes = [C.c_void_p, Tensor, Tensor, Tensor, Tensor, Tensor, Tensor, C.c_void_p] + tail
    L.dbsa_rope_table.restype = C.c_int
    L.dbsa_rope_table.argtypes = [C.POINTER(C.c_double), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    L.dbsa_rope_apply.restype = C.c_int
    L.dbsa_rope_apply.argtypes = [Tensor, Tensor, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int32,
                                  C.c_void_p, C.c_int32, C.c_void_p]
    L.dbsa_query_attn_rope.restype = C.c_int
    L.dbsa_query_attn_rope.argtypes = [C.c_void_p, Tensor, Tensor, Tensor, Tensor, Tensor, Tensor, C.c_void_p,
                                       C.c_void_p, C.c_int32] + tail
    L.dbsa_decode_attn_rope.restype = C.c_int
    L.dbsa_decode_attn_rope.argtypes = [C.c_void_p, Tensor, Tensor, Tensor, C.c_void_p, C.c_int64, Tensor, Tensor,
                                        Tensor, C.c_void_p, C.c_int32] + tail
    L.dbsa_decode_attn_kv8.restype = C.c_int
    L.dbsa_decode_attn_kv8.argtypes = [C.c_void_p, Tensor, Tensor, Tensor, C.c_void_p, C.c_int64, Tensor, Tensor,
                                       C.c_void_p, C.c_void_p, Tensor, C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                       C.c_void_p, C.c_size_t, C.c_void_p]
    L.dbsa_decode_attn.restype = C.c_int
    L.dbsa_decode_attn.argtypes = [C.c_void_p, Tensor, Tensor, Tensor, C.c_void_p, C.c_int64, Tensor, Tensor,
                                   Tensor] + tail
    L.dbsa_decode_attn_static.restype = C.c_int
    L.dbsa_decode_attn_static.argtypes = [C.c_void_p, Tensor, Tensor, Tensor, C.c_void_p, C.c_int64, Tensor, Tensor,
                                          Tensor, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_float, C.c_void_p]
    L.dbsa_decode_attn_kv8_rope.restype = C.c_int
    L.dbsa_decode_attn_kv8_rope.argtypes = [C.c_void_p, Tensor, Tensor, Tensor, C.c_void_p, C.c_int64, Tensor, Tensor,
                                            C.c_void_p, C.c_void_p, Tensor, C.c_void_p, C.c_int32, C.c_int32,
                                            C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_size_t, C.c_void_p]
    _lib = L
    return L


def strerror(code: int) -> str:
    return lib().dbsa_strerror(int(code)).decode()


def _check(rc: int, where: str) -> None:
    if rc != DBSA_OK:
        raise DbsaError(rc, where)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p32(a: Optional[np.ndarray]):
    return a.ctypes.data_as(C.POINTER(C.c_int32)) if a is not None and a.size else C.POINTER(C.c_int32)()


class Layout:
    """Owner of one ``dbsa_layout*`` handle."""

    def __init__(self, handle: int, query_stage: bool, block_m: int, block_n: int):
        self.handle = C.c_void_p(handle)
        self.query_stage = query_stage
        self.block_m, self.block_n = block_m, block_n

    def destroy(self) -> None:
        if self.handle:
            lib().dbsa_layout_destroy(self.handle)
            self.handle = C.c_void_p(None)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def export(self):
        """-> (qtile_tab [n,4] int32, list_ptr [n+1] int64, list_ent [E,2] int32) copies."""
        qt, lp, le = C.POINTER(C.c_int32)(), C.POINTER(C.c_int64)(), C.POINTER(C.c_int32)()
        nq, ne = C.c_int64(), C.c_int64()
        _check(lib().dbsa_layout_export(self.handle, C.byref(qt), C.byref(nq), C.byref(lp), C.byref(le),
                                        C.byref(ne)), "dbsa_layout_export")
        n, e = nq.value, ne.value
        tab = np.ctypeslib.as_array(qt, shape=(n, 4)).copy() if n else np.zeros((0, 4), np.int32)
        ptr = np.ctypeslib.as_array(lp, shape=(n + 1,)).copy()
        ent = np.ctypeslib.as_array(le, shape=(e, 2)).copy() if e else np.zeros((0, 2), np.int32)
        return tab, ptr, ent

    def export_decode(self, n_queries: int):
        """-> (dec_ptr [B+1] int64, dec_ent [E,2] int32, split_ptr [B, n_split+1] int64) copies."""
        dp, de, sp = C.POINTER(C.c_int64)(), C.POINTER(C.c_int32)(), C.POINTER(C.c_int64)()
        ne, ns = C.c_int64(), C.c_int32()
        _check(lib().dbsa_layout_export_decode(self.handle, C.byref(dp), C.byref(de), C.byref(ne), C.byref(sp),
                                               C.byref(ns)), "dbsa_layout_export_decode")
        dec_ptr = np.ctypeslib.as_array(dp, shape=(n_queries + 1,)).copy()
        dec_ent = np.ctypeslib.as_array(de, shape=(ne.value, 2)).copy() if ne.value else np.zeros((0, 2), np.int32)
        split = np.ctypeslib.as_array(sp, shape=(n_queries, ns.value + 1)).copy()
        return dec_ptr, dec_ent, split

    def export_decode_groups(self, n_groups: int, n_queries: int):
        """-> dict(seg_ptr [G+2], seg_ent [E,2], items [I,4], qrefs [R,2], slot_ptr [B+1], chunk_tiles) copies."""
        sp, se, it, qr, sl = (C.POINTER(C.c_int64)(), C.POINTER(C.c_int32)(), C.POINTER(C.c_int32)(),
                              C.POINTER(C.c_int32)(), C.POINTER(C.c_int64)())
        ne, ni, nr, ct = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int32()
        _check(lib().dbsa_layout_export_decode_groups(self.handle, C.byref(sp), C.byref(se), C.byref(ne),
                                                      C.byref(it), C.byref(ni), C.byref(qr), C.byref(nr),
                                                      C.byref(sl), C.byref(ct)), "dbsa_layout_export_decode_groups")

        def arr(ptr, shape, dt):
            return np.ctypeslib.as_array(ptr, shape=shape).copy() if shape[0] else np.zeros(shape, dt)

        return dict(seg_ptr=arr(sp, (n_groups + 2,), np.int64), seg_ent=arr(se, (ne.value, 2), np.int32),
                    items=arr(it, (ni.value, 4), np.int32), qrefs=arr(qr, (nr.value, 2), np.int32),
                    slot_ptr=arr(sl, (n_queries + 1,), np.int64), chunk_tiles=int(ct.value))

    def export_order(self) -> np.ndarray:
        op, n = C.POINTER(C.c_int32)(), C.c_int64()
        _check(lib().dbsa_layout_export_order(self.handle, C.byref(op), C.byref(n)), "dbsa_layout_export_order")
        return np.ctypeslib.as_array(op, shape=(n.value,)).copy() if n.value else np.zeros(0, np.int32)

    def export_positions(self, n_queries: int):
        """-> (list_shift [n_ent], qref_shift [n_qrefs], cache_len [B]) int32 copies."""
        ls, qs, cl = (C.POINTER(C.c_int32)() for _ in range(3))
        _check(lib().dbsa_layout_export_positions(self.handle, C.byref(ls), C.byref(qs), C.byref(cl)),
               "dbsa_layout_export_positions")
        n_ent = self.export()[2].shape[0]
        it, ni, qr, nr = C.POINTER(C.c_int32)(), C.c_int64(), C.POINTER(C.c_int32)(), C.c_int64()
        _check(lib().dbsa_layout_export_decode_groups(self.handle, None, None, None, C.byref(it), C.byref(ni),
                                                      C.byref(qr), C.byref(nr), None, None),
               "dbsa_layout_export_decode_groups")

        def arr(p, n):
            return np.ctypeslib.as_array(p, shape=(n,)).copy() if n else np.zeros(0, np.int32)
        return arr(ls, n_ent), arr(qs, nr.value), arr(cl, n_queries)

    def export_matrix_records(self):
        """-> (records [n, 4] int32 copies: (first reference, references, first tile, tiles), row_fill)."""
        rp, n, fill = C.POINTER(C.c_int32)(), C.c_int64(), C.c_float()
        _check(lib().dbsa_layout_export_matrix_records(self.handle, C.byref(rp), C.byref(n), C.byref(fill)),
               "dbsa_layout_export_matrix_records")
        rec = np.ctypeslib.as_array(rp, shape=(n.value, 4)).copy() if n.value else np.zeros((0, 4), np.int32)
        return rec, float(fill.value)

    def export_matrix_plan(self, n_queries: int = None):
        """-> (plan_ptr [n_workers + 1] int32 copy, or an empty array when records are dealt at launch; nominal workers)
        [, qrefs [n, 2], slot_ptr [n_queries + 1]: the references and slots of the plan's records, when n_queries is given]."""
        pp, n, nominal = C.POINTER(C.c_int32)(), C.c_int32(), C.c_int32()
        qp, nq, sp = C.POINTER(C.c_int32)(), C.c_int64(), C.POINTER(C.c_int64)()
        _check(lib().dbsa_layout_export_matrix_plan(self.handle, C.byref(pp), C.byref(n), C.byref(nominal), C.byref(qp),
                                                    C.byref(nq), C.byref(sp)), "dbsa_layout_export_matrix_plan")
        ptr = np.ctypeslib.as_array(pp, shape=(n.value + 1,)).copy() if n.value else np.zeros(0, np.int32)
        if n_queries is None:
            return ptr, int(nominal.value)
        qrefs = np.ctypeslib.as_array(qp, shape=(nq.value, 2)).copy() if nq.value else np.zeros((0, 2), np.int32)
        slots = np.ctypeslib.as_array(sp, shape=(n_queries + 1,)).copy() if nq.value else np.zeros(0, np.int64)
        return ptr, int(nominal.value), qrefs, slots

    def export_schedule(self, n_classes: int):
        """-> (class_ptr [n_classes+1], records [n_qtiles, 4]) int32 copies."""
        cp, rc = C.POINTER(C.c_int32)(), C.POINTER(C.c_int32)()
        _check(lib().dbsa_layout_export_schedule(self.handle, int(n_classes), C.byref(cp), C.byref(rc)),
               "dbsa_layout_export_schedule")
        ptr = np.ctypeslib.as_array(cp, shape=(n_classes + 1,)).copy()
        n = int(ptr[-1])
        rec = np.ctypeslib.as_array(rc, shape=(n, 4)).copy() if n else np.zeros((0, 4), np.int32)
        return ptr, rec

    def workspace_bytes(self, n_q_heads: int, head_dim: int) -> int:
        return int(lib().dbsa_workspace_bytes(self.handle, n_q_heads, head_dim))


def dbsa_layout_build(sink_len: int, demo_offsets, group_demo_offsets, prev_window: int = 0, *, cu_qlens=None,
                      sel_ptr=None, sel_idx=None, n_split: int = 0, block_m: int = 64, block_n: int = 64,
                      host_only: bool = False, stream: int = 0, page_start=None) -> Layout:
    do, gdo = _i32(demo_offsets), _i32(group_demo_offsets)
    pool = PoolDesc(int(sink_len), len(do) - 1, _p32(do), len(gdo) - 1, _p32(gdo), int(prev_window))
    sel_ref = None
    keep = [do, gdo]
    if cu_qlens is not None:
        cu, sp = _i32(cu_qlens), _i32(sel_ptr)
        si = _i32(sel_idx if sel_idx is not None else [])
        keep += [cu, sp, si]
        ps = _i32(page_start) if page_start is not None else None
        keep.append(ps)
        sel = SelectDesc(len(cu) - 1, _p32(cu), _p32(sp), _p32(si), int(n_split), _p32(ps))
        sel_ref = C.byref(sel)
    out = C.c_void_p()
    rc = lib().dbsa_layout_build(C.byref(pool), sel_ref, int(block_m), int(block_n),
                                 DBSA_LAYOUT_HOST_ONLY if host_only else 0, C.c_void_p(stream), C.byref(out))
    _check(rc, "dbsa_layout_build")
    return Layout(out.value, cu_qlens is not None, int(block_m), int(block_n))


def dbsa_layout_build_append(sink_len: int, demo_offsets, group_demo_offsets, prev_window: int, first_group: int, *,
                             block_m: int = 64, block_n: int = 64, host_only: bool = False,
                             stream: int = 0) -> Layout:
    """Pre-encode layout holding only the Q tiles of groups first_group.. of the described pool."""
    do, gdo = _i32(demo_offsets), _i32(group_demo_offsets)
    pool = PoolDesc(int(sink_len), len(do) - 1, _p32(do), len(gdo) - 1, _p32(gdo), int(prev_window))
    out = C.c_void_p()
    rc = lib().dbsa_layout_build_append(C.byref(pool), int(first_group), int(block_m), int(block_n),
                                        DBSA_LAYOUT_HOST_ONLY if host_only else 0, C.c_void_p(stream), C.byref(out))
    _check(rc, "dbsa_layout_build_append")
    return Layout(out.value, False, int(block_m), int(block_n))


# ---------------------------------------------------------------------------
# attention calls on torch device tensors
# ---------------------------------------------------------------------------

def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return DBSA_BF16
    if t.dtype == torch.float32:
        return DBSA_F32
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _tensor(t) -> Tensor:
    """[tokens, heads, D] device tensor, D contiguous."""
    assert t.is_cuda and t.dim() == 3 and t.stride(2) == 1, "expected a device tensor [tokens, heads, D]"
    return Tensor(t.data_ptr(), t.stride(0), t.stride(1))


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def dbsa_preencode_attn(layout: Layout, q, k, v, scale: float, out=None, lse=None):
    """Stage-1 attention over the whole pool; returns O [N, Hq, D] (same dtype as q)."""
    import torch
    o = torch.empty_like(q) if out is None else out
    rc = lib().dbsa_preencode_attn(layout.handle, _tensor(q), _tensor(k), _tensor(v), _tensor(o),
                                   C.c_void_p(lse.data_ptr() if lse is not None else None), _dtype_code(q),
                                   q.shape[1], k.shape[1], q.shape[2], float(scale), None, 0,
                                   C.c_void_p(_stream()))
    _check(rc, "dbsa_preencode_attn")
    return o


def _workspace(layout: Layout, q, workspace):
    """(pointer, bytes) of the caller's workspace, or of a fresh one of dbsa_workspace_bytes()."""
    import torch
    if workspace is None:
        workspace = torch.empty(max(layout.workspace_bytes(q.shape[1], q.shape[2]), 16), dtype=torch.uint8,
                                device=q.device)
    return workspace, C.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def dbsa_query_attn(layout: Layout, q_self, k_self, v_self, k_pool, v_pool, scale: float, out=None, lse=None,
                    workspace=None):
    """Stage-2 prefill of the packed queries; returns O [sum T, Hq, D].  ``workspace`` (uint8 device
    tensor of dbsa_workspace_bytes(), allocated here when omitted; False = none) lets launches with few
    Q tiles split their KV lists."""
    import torch
    o = torch.empty_like(q_self) if out is None else out
    ws, ws_ptr, ws_bytes = (None, None, 0) if workspace is False else _workspace(layout, q_self, workspace)
    rc = lib().dbsa_query_attn(layout.handle, _tensor(q_self), _tensor(k_self), _tensor(v_self), _tensor(k_pool),
                               _tensor(v_pool), _tensor(o), C.c_void_p(lse.data_ptr() if lse is not None else None),
                               _dtype_code(q_self), q_self.shape[1], k_pool.shape[1], q_self.shape[2], float(scale),
                               ws_ptr, ws_bytes, C.c_void_p(_stream()))
    _check(rc, "dbsa_query_attn")
    return o


def dbsa_decode_attn(layout: Layout, q_step, k_cache, v_cache, self_len, k_pool, v_pool, scale: float, out=None,
                     workspace=None):
    """One decode step.  q_step [B, Hq, D]; caches [B, Tmax, Hkv, D]; self_len int32 [B] on device."""
    import torch
    assert k_cache.dim() == 4 and k_cache.stride(3) == 1 and v_cache.stride() == k_cache.stride()
    o = torch.empty_like(q_step) if out is None else out
    need = layout.workspace_bytes(q_step.shape[1], q_step.shape[2])
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q_step.device)
    kc = Tensor(k_cache.data_ptr(), k_cache.stride(1), k_cache.stride(2))
    vc = Tensor(v_cache.data_ptr(), v_cache.stride(1), v_cache.stride(2))
    rc = lib().dbsa_decode_attn(layout.handle, _tensor(q_step), kc, vc, C.c_void_p(self_len.data_ptr()),
                                k_cache.stride(0), _tensor(k_pool), _tensor(v_pool), _tensor(o), _dtype_code(q_step),
                                q_step.shape[1], k_pool.shape[1], q_step.shape[2], float(scale),
                                C.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                                C.c_void_p(_stream()))
    _check(rc, "dbsa_decode_attn")
    return o


def dbsa_decode_attn_static(layout: Layout, q_step, k_cache, v_cache, self_len, k_pool, v_pool, scale: float, out):
    """dbsa_decode_attn with the partial states in the library's fixed buffer: no workspace argument,
    and ``out`` is required so that nothing is allocated on the way."""
    assert k_cache.dim() == 4 and k_cache.stride(3) == 1 and v_cache.stride() == k_cache.stride()
    kc = Tensor(k_cache.data_ptr(), k_cache.stride(1), k_cache.stride(2))
    vc = Tensor(v_cache.data_ptr(), v_cache.stride(1), v_cache.stride(2))
    rc = lib().dbsa_decode_attn_static(layout.handle, _tensor(q_step), kc, vc, C.c_void_p(self_len.data_ptr()),
                                       k_cache.stride(0), _tensor(k_pool), _tensor(v_pool), _tensor(out),
                                       _dtype_code(q_step), q_step.shape[1], k_pool.shape[1], q_step.shape[2],
                                       float(scale), C.c_void_p(_stream()))
    _check(rc, "dbsa_decode_attn_static")
    return out


# ---------------------------------------------------------------------------
# query stage with re-positioning
# ---------------------------------------------------------------------------

def dbsa_rope_table(inv_freq, n_pos: int, device="cuda"):
    """-> fp32 device tensor [n_pos, D/2, 2] of (cos, sin)(id * inv_freq[i])."""
    import torch
    f = np.ascontiguousarray(inv_freq, dtype=np.float64)
    table = torch.empty((int(n_pos), len(f), 2), dtype=torch.float32, device=device)
    rc = lib().dbsa_rope_table(f.ctypes.data_as(C.POINTER(C.c_double)), 2 * len(f), int(n_pos),
                               C.c_void_p(table.data_ptr()), C.c_void_p(_stream()))
    _check(rc, "dbsa_rope_table")
    return table


def dbsa_rope_apply(x, table, positions=None, first_id: int = 0, out=None):
    """x [T, H, D] rotated at ``positions`` (int32 device tensor [T]) or at first_id + t."""
    import torch
    o = torch.empty_like(x) if out is None else out
    rc = lib().dbsa_rope_apply(_tensor(x), _tensor(o), x.shape[0], x.shape[1], x.shape[2], _dtype_code(x),
                               C.c_void_p(positions.data_ptr() if positions is not None else None), int(first_id),
                               C.c_void_p(table.data_ptr()), table.shape[0], C.c_void_p(_stream()))
    _check(rc, "dbsa_rope_apply")
    return o


def dbsa_query_attn_rope(layout: Layout, q_self, k_self, v_self, k_pool, v_pool, table, scale: float, out=None,
                         workspace=None):
    """Stage-2 prefill with re-positioning: q_self un-rotated, keys rotated at their encoding ids."""
    import torch
    o = torch.empty_like(q_self) if out is None else out
    ws, ws_ptr, ws_bytes = (None, None, 0) if workspace is False else _workspace(layout, q_self, workspace)
    rc = lib().dbsa_query_attn_rope(layout.handle, _tensor(q_self), _tensor(k_self), _tensor(v_self), _tensor(k_pool),
                                    _tensor(v_pool), _tensor(o), None, C.c_void_p(table.data_ptr()), table.shape[0],
                                    _dtype_code(q_self), q_self.shape[1], k_pool.shape[1], q_self.shape[2],
                                    float(scale), ws_ptr, ws_bytes, C.c_void_p(_stream()))
    _check(rc, "dbsa_query_attn_rope")
    return o


def dbsa_decode_attn_rope(layout: Layout, q_step, k_cache, v_cache, self_len, k_pool, v_pool, table, scale: float,
                          out=None, workspace=None):
    """One decode step with re-positioning (see dbsa_decode_attn for the shapes)."""
    import torch
    assert k_cache.dim() == 4 and k_cache.stride(3) == 1 and v_cache.stride() == k_cache.stride()
    o = torch.empty_like(q_step) if out is None else out
    need = layout.workspace_bytes(q_step.shape[1], q_step.shape[2])
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q_step.device)
    kc = Tensor(k_cache.data_ptr(), k_cache.stride(1), k_cache.stride(2))
    vc = Tensor(v_cache.data_ptr(), v_cache.stride(1), v_cache.stride(2))
    rc = lib().dbsa_decode_attn_rope(layout.handle, _tensor(q_step), kc, vc, C.c_void_p(self_len.data_ptr()),
                                     k_cache.stride(0), _tensor(k_pool), _tensor(v_pool), _tensor(o),
                                     C.c_void_p(table.data_ptr()), table.shape[0], _dtype_code(q_step),
                                     q_step.shape[1], k_pool.shape[1], q_step.shape[2], float(scale),
                                     C.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                                     C.c_void_p(_stream()))
    _check(rc, "dbsa_decode_attn_rope")
    return o


def dbsa_decode_attn_kv8(layout: Layout, q_step, k_cache, v_cache, self_len, k_pool8, v_pool8, k_scale, v_scale,
                         scale: float, out=None, workspace=None, rope_table=None):
    """One decode step over an fp8 (e4m3) pool: k_pool8 / v_pool8 are [N, Hkv, D] float8_e4m3fn (or uint8)
    device tensors, k_scale / v_scale float32 [Hkv] on the device; everything else as dbsa_decode_attn.
    With ``rope_table`` the step re-positions (dbsa_decode_attn_kv8_rope): q_step un-rotated, pool keys
    rotated at their encoding ids before quantisation."""
    import torch
    assert k_cache.dim() == 4 and k_cache.stride(3) == 1 and v_cache.stride() == k_cache.stride()
    assert k_pool8.element_size() == 1 and k_pool8.dim() == 3 and k_pool8.stride(2) == 1
    o = torch.empty_like(q_step) if out is None else out
    ws, ws_ptr, ws_bytes = _workspace(layout, q_step, workspace)
    kc = Tensor(k_cache.data_ptr(), k_cache.stride(1), k_cache.stride(2))
    vc = Tensor(v_cache.data_ptr(), v_cache.stride(1), v_cache.stride(2))
    if rope_table is not None:
        rc = lib().dbsa_decode_attn_kv8_rope(layout.handle, _tensor(q_step), kc, vc, C.c_void_p(self_len.data_ptr()),
                                             k_cache.stride(0), _tensor(k_pool8), _tensor(v_pool8),
                                             C.c_void_p(k_scale.data_ptr()), C.c_void_p(v_scale.data_ptr()),
                                             _tensor(o), C.c_void_p(rope_table.data_ptr()), rope_table.shape[0],
                                             q_step.shape[1], k_pool8.shape[1], q_step.shape[2], float(scale),
                                             ws_ptr, ws_bytes, C.c_void_p(_stream()))
        _check(rc, "dbsa_decode_attn_kv8_rope")
        return o
    rc = lib().dbsa_decode_attn_kv8(layout.handle, _tensor(q_step), kc, vc, C.c_void_p(self_len.data_ptr()),
                                    k_cache.stride(0), _tensor(k_pool8), _tensor(v_pool8),
                                    C.c_void_p(k_scale.data_ptr()), C.c_void_p(v_scale.data_ptr()), _tensor(o),
                                    q_step.shape[1], k_pool8.shape[1], q_step.shape[2], float(scale), ws_ptr,
                                    ws_bytes, C.c_void_p(_stream()))
    _check(rc, "dbsa_decode_attn_kv8")
    return o

