"""ctypes binding of libs2attn.so: argument marshalling only.

Every function here has the name of the C entry point it calls (see
``include/s2attn.h``) and does nothing but turn torch tensors into pointers,
sizes and strides.  torch is used for device memory and streams; all of the
attention arithmetic runs inside the HIP library.  There is no fallback: if
the shared library is missing, importing this module raises.
"""

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libs2attn.so")

S2_OK = 0
STATUS_NAMES = {
    0: "S2_OK", -1: "S2_ERR_NULL", -2: "S2_ERR_BAD_PARAM", -3: "S2_ERR_SHAPE", -4: "S2_ERR_ALIGN",
    -5: "S2_ERR_WORKSPACE", -6: "S2_ERR_HIP", -7: "S2_ERR_NO_DEVICE", -8: "S2_ERR_OVERFLOW",
}


class S2Error(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = "%s failed: %s (%s)" % (where, STATUS_NAMES.get(status, status),
                                      lib().s2_status_string(status).decode())
        if status == -6:
            msg += " hipError=%d" % lib().s2_last_hip_error()
        super().__init__(msg)


class LayoutParams(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "num_heads", "head_index_base", "num_blocks", "block_size", "local_blocks", "stride",
        "window_blocks", "dense")]


class LayoutView(C.Structure):
    _fields_ = [("row_ptr", C.POINTER(C.c_int32)), ("col_idx", C.POINTER(C.c_int32)),
                ("col_ptr", C.POINTER(C.c_int32)), ("row_idx", C.POINTER(C.c_int32)),
                ("nnz", C.c_int64), ("num_heads", C.c_int32), ("num_blocks", C.c_int32),
                ("block_size", C.c_int32), ("max_row_blocks", C.c_int32), ("covers_all", C.c_int32),
                ("on_device", C.c_int32)]


class TileView(C.Structure):
    _fields_ = [("ptr", C.POINTER(C.c_int32)), ("ent", C.POINTER(C.c_int32)), ("order", C.POINTER(C.c_int32)),
                ("members", C.POINTER(C.c_int32)), ("tiles_per_head", C.c_int32), ("group", C.c_int32),
                ("blocks_per_unit", C.c_int32)]


class DsUnitsView(C.Structure):
    _fields_ = [("dq_units", C.POINTER(C.c_int32)), ("count", C.c_int64), ("ds_units", C.c_int64)]


class Tensors(C.Structure):
    _fields_ = [("q", C.c_void_p), ("k", C.c_void_p), ("v", C.c_void_p), ("o", C.c_void_p),
                ("lse", C.c_void_p), ("d_o", C.c_void_p), ("dq", C.c_void_p), ("dk", C.c_void_p),
                ("dv", C.c_void_p),
                ("batch", C.c_int32), ("heads", C.c_int32), ("seqlen", C.c_int32), ("head_dim", C.c_int32),
                ("q_stride_b", C.c_int64), ("q_stride_h", C.c_int64), ("q_stride_t", C.c_int64),
                ("kv_stride_b", C.c_int64), ("kv_stride_h", C.c_int64), ("kv_stride_t", C.c_int64)]


class DecodeArgs(C.Structure):
    _fields_ = [("q", C.c_void_p), ("k_cache", C.c_void_p), ("v_cache", C.c_void_p),
                ("seq_lens", C.c_void_p), ("o", C.c_void_p), ("lse", C.c_void_p),
                ("nseq", C.c_int32), ("heads", C.c_int32), ("head_dim", C.c_int32),
                ("max_len", C.c_int32), ("num_splits", C.c_int32),
                ("kv_stride_seq", C.c_int64), ("kv_stride_head", C.c_int64), ("kv_stride_tok", C.c_int64)]


class PagedDecodeArgs(C.Structure):
    _fields_ = [("q", C.c_void_p), ("k_pages", C.c_void_p), ("v_pages", C.c_void_p),
                ("block_table", C.c_void_p), ("seq_lens", C.c_void_p), ("o", C.c_void_p),
                ("lse", C.c_void_p), ("missing", C.c_void_p),
                ("nseq", C.c_int32), ("heads", C.c_int32), ("head_dim", C.c_int32),
                ("max_blocks", C.c_int32), ("num_pages", C.c_int32), ("num_splits", C.c_int32),
                ("page_stride", C.c_int64), ("tok_stride", C.c_int64)]


EXPORTS = (
    "s2_layout_build", "s2_layout_from_csr", "s2_layout_destroy", "s2_layout_get", "s2_layout_get_tiles", "s2_layout_get_ds_units", "s2_attn_fwd", "s2_attn_fwd_rows", "s2_attn_fwd_varlen", "s2_attn_bwd_varlen",
    "s2_attn_bwd_varlen_workspace_bytes", "s2_attn_bwd",
    "s2_attn_bwd_workspace_bytes", "s2_attn_bwd_layout_workspace_bytes", "s2_attn_bwd_stages", "s2_dense_causal_fwd", "s2_dense_causal_bwd", "s2_attn_decode",
    "s2_attn_decode_workspace_bytes", "s2_attn_decode_default_splits", "s2_attn_decode_static", "s2_attn_decode_paged",
    "s2_kv_resident_blocks", "s2_attn_decode_layout", "s2_attn_decode_paged_layout",
    "s2_layout_resident_blocks", "s2_probe_scratch_bytes", "s2_probe_mfma", "s2_probe_read", "s2_probe_atomic_add", "s2_status_string",
    "s2_last_hip_error", "s2_version",
)

_lib = None


def lib():
    """The loaded shared library (loads it on first use; raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libs2attn.so is not built: run `python -m paper_2407_17678_amd.build`")
    L = C.CDLL(LIB_PATH)
    L.s2_layout_build.argtypes = [C.POINTER(LayoutParams), C.POINTER(C.c_void_p)]
    L.s2_layout_from_csr.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32),
                                     C.POINTER(C.c_int32), C.POINTER(C.c_void_p)]
    L.s2_layout_destroy.argtypes = [C.c_void_p]
    L.s2_layout_get.argtypes = [C.c_void_p, C.POINTER(LayoutView)]
    L.s2_layout_get_tiles.argtypes = [C.c_void_p, C.c_int, C.POINTER(TileView)]
    L.s2_layout_get_ds_units.argtypes = [C.c_void_p, C.POINTER(DsUnitsView)]
    L.s2_attn_fwd.argtypes = [C.c_void_p, C.POINTER(Tensors), C.c_float, C.c_void_p]
    L.s2_attn_fwd_rows.argtypes = [C.c_void_p, C.POINTER(Tensors), C.c_int32, C.c_int32, C.c_float, C.c_void_p]
    L.s2_attn_fwd_varlen.argtypes = [C.c_void_p, C.POINTER(Tensors), C.c_void_p, C.c_int32, C.c_int32, C.c_float,
                                     C.c_void_p]
    L.s2_attn_bwd_varlen.argtypes = [C.c_void_p, C.POINTER(Tensors), C.c_void_p, C.c_int32, C.c_int32, C.c_float,
                                     C.c_void_p, C.c_size_t, C.c_void_p]
    L.s2_attn_bwd_varlen_workspace_bytes.argtypes = [C.c_int32] * 3
    L.s2_attn_bwd_varlen_workspace_bytes.restype = C.c_size_t
    L.s2_attn_bwd.argtypes = [C.c_void_p, C.POINTER(Tensors), C.c_float, C.c_void_p, C.c_size_t, C.c_void_p]
    L.s2_attn_bwd_stages.argtypes = [C.c_void_p, C.POINTER(Tensors), C.c_float, C.c_void_p, C.c_size_t,
                                     C.c_int, C.c_void_p]
    L.s2_attn_bwd_workspace_bytes.argtypes = [C.c_int32] * 4
    L.s2_attn_bwd_workspace_bytes.restype = C.c_size_t
    L.s2_attn_bwd_layout_workspace_bytes.argtypes = [C.c_void_p] + [C.c_int32] * 4
    L.s2_attn_bwd_layout_workspace_bytes.restype = C.c_size_t
    L.s2_dense_causal_fwd.argtypes = [C.POINTER(Tensors), C.c_float, C.c_void_p]
    L.s2_dense_causal_bwd.argtypes = [C.POINTER(Tensors), C.c_float, C.c_void_p, C.c_size_t, C.c_void_p]
    L.s2_attn_decode.argtypes = [C.POINTER(LayoutParams), C.POINTER(DecodeArgs), C.c_float, C.c_void_p,
                                 C.c_size_t, C.c_void_p]
    L.s2_attn_decode_static.argtypes = [C.POINTER(LayoutParams), C.POINTER(DecodeArgs), C.c_float, C.c_void_p]
    L.s2_attn_decode_workspace_bytes.argtypes = [C.c_int32] * 5
    L.s2_attn_decode_workspace_bytes.restype = C.c_size_t
    L.s2_attn_decode_default_splits.argtypes = [C.c_int32] * 3
    L.s2_attn_decode_default_splits.restype = C.c_int32
    L.s2_attn_decode_paged.argtypes = [C.POINTER(LayoutParams), C.POINTER(PagedDecodeArgs), C.c_float,
                                       C.c_void_p, C.c_size_t, C.c_void_p]
    L.s2_kv_resident_blocks.argtypes = [C.POINTER(LayoutParams), C.c_int32, C.c_int32,
                                        C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_int32)]
    L.s2_attn_decode_layout.argtypes = [C.c_void_p, C.POINTER(DecodeArgs), C.c_float, C.c_void_p,
                                        C.c_size_t, C.c_void_p]
    L.s2_attn_decode_paged_layout.argtypes = [C.c_void_p, C.POINTER(PagedDecodeArgs), C.c_float,
                                              C.c_void_p, C.c_size_t, C.c_void_p]
    L.s2_layout_resident_blocks.argtypes = [C.c_void_p, C.c_int32, C.c_int32,
                                            C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_int32)]
    L.s2_probe_scratch_bytes.restype = C.c_size_t
    L.s2_probe_mfma.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.POINTER(C.c_double)]
    L.s2_probe_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    L.s2_probe_atomic_add.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_double)]
    L.s2_status_string.argtypes = [C.c_int]
    L.s2_status_string.restype = C.c_char_p
    L.s2_last_hip_error.restype = C.c_int
    L.s2_version.restype = C.c_int
    for name in EXPORTS:
        getattr(L, name)
    _lib = L
    return L


def _check(status, where):
    if status != S2_OK:
        raise S2Error(status, where)


def _stream_ptr(stream):
    """torch stream (or None = torch's current stream) -> hipStream_t as an integer."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def layout_params(num_heads, num_blocks, block_size, local_blocks, stride, head_index_base=0,
                  window_blocks=0, dense=0):
    return LayoutParams(num_heads, head_index_base, num_blocks, block_size, local_blocks, stride,
                        window_blocks, dense)


class Layout:
    """Owner of an s2_layout handle."""

    def __init__(self, handle, params):
        self.handle = handle
        self.params = params

    def __del__(self):
        h, self.handle = getattr(self, "handle", None), None
        if h and _lib is not None:
            _lib.s2_layout_destroy(h)


def s2_layout_build(params):
    out = C.c_void_p()
    _check(lib().s2_layout_build(C.byref(params), C.byref(out)), "s2_layout_build")
    return Layout(out, params)


def s2_layout_from_csr(num_heads, num_blocks, block_size, row_ptr, col_idx):
    """row_ptr, col_idx: host int32 arrays (numpy) in the order s2_layout_get returns them."""
    import numpy as np
    rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
    ci = np.ascontiguousarray(col_idx, dtype=np.int32)
    assert rp.shape == (num_heads * num_blocks + 1,) and ci.shape == (int(rp[-1]),)
    out = C.c_void_p()
    as_p = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    _check(lib().s2_layout_from_csr(num_heads, num_blocks, block_size, as_p(rp), as_p(ci), C.byref(out)),
           "s2_layout_from_csr")
    return Layout(out, None)


def s2_layout_destroy(layout):
    h, layout.handle = layout.handle, None
    if h:
        _check(lib().s2_layout_destroy(h), "s2_layout_destroy")


def s2_layout_get(layout):
    """Host copies of the canonical arrays as numpy int32, plus the scalar fields."""
    v = LayoutView()
    _check(lib().s2_layout_get(layout.handle, C.byref(v)), "s2_layout_get")
    n = v.num_heads * v.num_blocks + 1
    as_np = lambda p, k: np.ctypeslib.as_array(p, shape=(k,)).copy() if k else np.zeros(0, np.int32)
    return {
        "row_ptr": as_np(v.row_ptr, n), "col_idx": as_np(v.col_idx, v.nnz),
        "col_ptr": as_np(v.col_ptr, n), "row_idx": as_np(v.row_idx, v.nnz),
        "nnz": v.nnz, "num_heads": v.num_heads, "num_blocks": v.num_blocks,
        "block_size": v.block_size, "max_row_blocks": v.max_row_blocks,
        "covers_all": v.covers_all, "on_device": v.on_device,
    }


TILES_FWD, TILES_DQ, TILES_DKDV = 0, 1, 2


def s2_layout_get_tiles(layout, which):
    """Host copies of one of the layout's work lists (see s2_tile_view in the header)."""
    v = TileView()
    _check(lib().s2_layout_get_tiles(layout.handle, which, C.byref(v)), "s2_layout_get_tiles")
    heads = s2_layout_get(layout)["num_heads"]
    n = heads * v.tiles_per_head
    as_np = lambda p, k: np.ctypeslib.as_array(p, shape=(k,)).copy() if k else np.zeros(0, np.int32)
    ptr = as_np(v.ptr, n + 1)
    return {"ptr": ptr, "ent": as_np(v.ent, int(ptr[-1])), "order": as_np(v.order, n),
            "members": as_np(v.members, n * v.group), "tiles_per_head": v.tiles_per_head, "group": v.group,
            "blocks_per_unit": v.blocks_per_unit}


def s2_layout_get_ds_units(layout):
    """Host copy of the unit table of the backward that keeps dS (see s2_ds_units_view in the header)."""
    v = DsUnitsView()
    _check(lib().s2_layout_get_ds_units(layout.handle, C.byref(v)), "s2_layout_get_ds_units")
    units = np.ctypeslib.as_array(v.dq_units, shape=(v.count,)).copy() if v.count else np.zeros(0, np.int32)
    return {"dq_units": units, "ds_units": int(v.ds_units)}


def bf16_bits_to_device(bits, device="cuda"):
    """uint16 bf16 bit patterns (numpy) -> torch.bfloat16 tensor on the GPU holding the same bits."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device)
    return t.view(torch.bfloat16)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(None)


def _tensors(q, k, v, o, lse, d_o=None, dq=None, dk=None, dv=None):
    Bt, H, N, D = q.shape
    assert q.stride(3) == 1 and k.stride(3) == 1 and v.stride(3) == 1 and o.stride(3) == 1
    assert k.stride() == v.stride() and q.stride() == o.stride()
    for g, ref in ((d_o, q), (dq, q), (dk, k), (dv, k)):
        assert g is None or g.stride() == ref.stride()
    assert lse.is_contiguous()
    return Tensors(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(dq), _ptr(dk), _ptr(dv),
                   Bt, H, N, D, q.stride(0), q.stride(1), q.stride(2), k.stride(0), k.stride(1), k.stride(2))


def s2_attn_fwd(layout, q, k, v, o, lse, scale, stream=None):
    t = _tensors(q, k, v, o, lse)
    _check(lib().s2_attn_fwd(layout.handle, C.byref(t), scale, _stream_ptr(stream)), "s2_attn_fwd")


def s2_attn_fwd_rows(layout, q, k, v, o, lse, q_row_start, scale, stream=None):
    """q, o: [Bt, H, q_rows, D] (the tokens at positions q_row_start ...); k, v: [Bt, H, N_k, D]."""
    t = _tensors(q, k, v, o, lse)
    t.seqlen = k.shape[2]
    _check(lib().s2_attn_fwd_rows(layout.handle, C.byref(t), q_row_start, q.shape[2], scale,
                                  _stream_ptr(stream)), "s2_attn_fwd_rows")


def s2_attn_fwd_varlen(layout, q, k, v, o, lse, cu_seqlens, max_seqlen, scale, stream=None):
    """q, k, v, o: [1, H, total_rows, D] packed sequences; lse: [H, total_rows]; cu_seqlens: device int32 [n+1]."""
    t = _tensors(q, k, v, o, lse)
    assert q.shape[0] == 1 and cu_seqlens.is_contiguous() and cu_seqlens.numel() >= 2
    _check(lib().s2_attn_fwd_varlen(layout.handle, C.byref(t), _ptr(cu_seqlens), cu_seqlens.numel() - 1,
                                    max_seqlen, scale, _stream_ptr(stream)), "s2_attn_fwd_varlen")


def s2_attn_bwd_varlen_workspace_bytes(heads, rows, head_dim):
    return lib().s2_attn_bwd_varlen_workspace_bytes(heads, rows, head_dim)


def s2_attn_bwd_varlen(layout, q, k, v, o, lse, d_o, dq, dk, dv, cu_seqlens, max_seqlen, scale, workspace, stream=None):
    """Gradient of s2_attn_fwd_varlen; d_o, dq, dk, dv packed like q."""
    t = _tensors(q, k, v, o, lse, d_o, dq, dk, dv)
    assert q.shape[0] == 1 and cu_seqlens.is_contiguous() and cu_seqlens.numel() >= 2
    _check(lib().s2_attn_bwd_varlen(layout.handle, C.byref(t), _ptr(cu_seqlens), cu_seqlens.numel() - 1, max_seqlen,
                                    scale, _ptr(workspace), workspace.numel() * workspace.element_size(),
                                    _stream_ptr(stream)), "s2_attn_bwd_varlen")


def s2_attn_bwd_workspace_bytes(batch, heads, seqlen, head_dim):
    return lib().s2_attn_bwd_workspace_bytes(batch, heads, seqlen, head_dim)


def s2_attn_bwd_layout_workspace_bytes(layout, batch, heads, seqlen, head_dim):
    return lib().s2_attn_bwd_layout_workspace_bytes(layout.handle, batch, heads, seqlen, head_dim)


def s2_attn_bwd(layout, q, k, v, o, lse, d_o, dq, dk, dv, scale, workspace, stream=None):
    t = _tensors(q, k, v, o, lse, d_o, dq, dk, dv)
    _check(lib().s2_attn_bwd(layout.handle, C.byref(t), scale, _ptr(workspace),
                             workspace.numel() * workspace.element_size(), _stream_ptr(stream)),
           "s2_attn_bwd")


BWD_DELTA, BWD_DKDV, BWD_DQ, BWD_ALL = 1, 2, 4, 7


def s2_attn_bwd_stages(layout, q, k, v, o, lse, d_o, dq, dk, dv, scale, workspace, stages, stream=None):
    t = _tensors(q, k, v, o, lse, d_o, dq, dk, dv)
    _check(lib().s2_attn_bwd_stages(layout.handle, C.byref(t), scale, _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), stages,
                                    _stream_ptr(stream)), "s2_attn_bwd_stages")


def s2_dense_causal_fwd(q, k, v, o, lse, scale, stream=None):
    t = _tensors(q, k, v, o, lse)
    _check(lib().s2_dense_causal_fwd(C.byref(t), scale, _stream_ptr(stream)), "s2_dense_causal_fwd")


def s2_dense_causal_bwd(q, k, v, o, lse, d_o, dq, dk, dv, scale, workspace, stream=None):
    t = _tensors(q, k, v, o, lse, d_o, dq, dk, dv)
    _check(lib().s2_dense_causal_bwd(C.byref(t), scale, _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream_ptr(stream)),
           "s2_dense_causal_bwd")


def s2_attn_decode_workspace_bytes(nseq, heads, head_dim, max_len, num_splits=0):
    return lib().s2_attn_decode_workspace_bytes(nseq, heads, head_dim, max_len, num_splits)


def s2_attn_decode_default_splits(nseq, heads, max_len):
    return lib().s2_attn_decode_default_splits(nseq, heads, max_len)


def s2_attn_decode(params, q, k_cache, v_cache, seq_lens, o, lse, scale, workspace, max_len,
                   num_splits=0, stream=None):
    nseq, H, D = q.shape
    assert q.is_contiguous() and o.is_contiguous() and k_cache.stride() == v_cache.stride()
    assert k_cache.stride(3) == 1
    a = DecodeArgs(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens), _ptr(o), _ptr(lse),
                   nseq, H, D, max_len, num_splits,
                   k_cache.stride(0), k_cache.stride(1), k_cache.stride(2))
    _check(lib().s2_attn_decode(C.byref(params), C.byref(a), scale, _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream_ptr(stream)),
           "s2_attn_decode")


def s2_attn_decode_static(params, q, k_cache, v_cache, seq_lens, o, lse, scale, max_len, num_splits=0,
                          stream=None):
    """s2_attn_decode with the split partials in the library's own static device buffer."""
    nseq, H, D = q.shape
    assert q.is_contiguous() and o.is_contiguous() and k_cache.stride() == v_cache.stride()
    assert k_cache.stride(3) == 1
    a = DecodeArgs(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens), _ptr(o), _ptr(lse),
                   nseq, H, D, max_len, num_splits,
                   k_cache.stride(0), k_cache.stride(1), k_cache.stride(2))
    _check(lib().s2_attn_decode_static(C.byref(params), C.byref(a), scale, _stream_ptr(stream)),
           "s2_attn_decode_static")


def s2_attn_decode_layout(layout, q, k_cache, v_cache, seq_lens, o, lse, scale, workspace, max_len,
                          num_splits=0, stream=None):
    """s2_attn_decode following the rows of a Layout (any pattern) instead of the closed form."""
    nseq, H, D = q.shape
    assert q.is_contiguous() and o.is_contiguous() and k_cache.stride() == v_cache.stride()
    assert k_cache.stride(3) == 1
    a = DecodeArgs(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens), _ptr(o), _ptr(lse),
                   nseq, H, D, max_len, num_splits,
                   k_cache.stride(0), k_cache.stride(1), k_cache.stride(2))
    _check(lib().s2_attn_decode_layout(layout.handle, C.byref(a), scale, _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream_ptr(stream)),
           "s2_attn_decode_layout")


def s2_attn_decode_paged(params, q, k_pages, v_pages, block_table, seq_lens, o, lse, scale, workspace,
                         missing=None, num_splits=0, stream=None):
    """k_pages, v_pages: [num_pages, block_size, head_dim]; block_table: int32 [nseq, heads, max_blocks]."""
    nseq, H, D = q.shape
    assert q.is_contiguous() and o.is_contiguous() and block_table.is_contiguous()
    assert k_pages.stride() == v_pages.stride() and k_pages.stride(2) == 1
    assert tuple(block_table.shape[:2]) == (nseq, H)
    a = PagedDecodeArgs(_ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table), _ptr(seq_lens), _ptr(o),
                        _ptr(lse), _ptr(missing), nseq, H, D, block_table.shape[2], k_pages.shape[0],
                        num_splits, k_pages.stride(0), k_pages.stride(1))
    _check(lib().s2_attn_decode_paged(C.byref(params), C.byref(a), scale, _ptr(workspace),
                                      workspace.numel() * workspace.element_size(), _stream_ptr(stream)),
           "s2_attn_decode_paged")


def s2_attn_decode_paged_layout(layout, q, k_pages, v_pages, block_table, seq_lens, o, lse, scale, workspace,
                                missing=None, num_splits=0, stream=None):
    """s2_attn_decode_paged following the rows of a Layout (any pattern) instead of the closed form."""
    nseq, H, D = q.shape
    assert q.is_contiguous() and o.is_contiguous() and block_table.is_contiguous()
    assert k_pages.stride() == v_pages.stride() and k_pages.stride(2) == 1
    assert tuple(block_table.shape[:2]) == (nseq, H)
    a = PagedDecodeArgs(_ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table), _ptr(seq_lens), _ptr(o),
                        _ptr(lse), _ptr(missing), nseq, H, D, block_table.shape[2], k_pages.shape[0],
                        num_splits, k_pages.stride(0), k_pages.stride(1))
    _check(lib().s2_attn_decode_paged_layout(layout.handle, C.byref(a), scale, _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _stream_ptr(stream)),
           "s2_attn_decode_paged_layout")


def s2_kv_resident_blocks(params, head, length):
    """Ascending list of the logical KV blocks local head `head` still needs with `length` tokens cached."""
    n = C.c_int32(0)
    st = lib().s2_kv_resident_blocks(C.byref(params), head, length, None, 0, C.byref(n))
    if st not in (0, -8):
        _check(st, "s2_kv_resident_blocks")
    buf = (C.c_int32 * max(1, n.value))()
    _check(lib().s2_kv_resident_blocks(C.byref(params), head, length, buf, n.value, C.byref(n)),
           "s2_kv_resident_blocks")
    return list(buf[:n.value])


def s2_layout_resident_blocks(layout, head, length):
    """The same from the rows of a Layout: blocks that its row (length-1) div S or a later row keeps."""
    n = C.c_int32(0)
    st = lib().s2_layout_resident_blocks(layout.handle, head, length, None, 0, C.byref(n))
    if st not in (0, -8):
        _check(st, "s2_layout_resident_blocks")
    buf = (C.c_int32 * max(1, n.value))()
    _check(lib().s2_layout_resident_blocks(layout.handle, head, length, buf, n.value, C.byref(n)),
           "s2_layout_resident_blocks")
    return list(buf[:n.value])


def s2_probe_scratch_bytes():
    return int(lib().s2_probe_scratch_bytes())


def s2_probe_mfma(with_vector_work, iters, scratch, stream=None):
    """Enqueues the MFMA ceiling probe; returns the flops of the launch."""
    flops = C.c_double(0.0)
    _check(lib().s2_probe_mfma(int(bool(with_vector_work)), iters, _ptr(scratch), _stream_ptr(stream),
                               C.byref(flops)), "s2_probe_mfma")
    return flops.value


def s2_probe_read(src, scratch, stream=None):
    """Enqueues the read-bandwidth probe over the whole of `src`; returns the bytes read."""
    nbytes = src.numel() * src.element_size()
    _check(lib().s2_probe_read(_ptr(src), nbytes, _ptr(scratch), _stream_ptr(stream)), "s2_probe_read")
    return nbytes


def s2_probe_atomic_add(buf, stream=None):
    """Enqueues the fp32 atomic-add probe on `buf` (a float32 device tensor); returns the bytes added."""
    added = C.c_double(0.0)
    _check(lib().s2_probe_atomic_add(_ptr(buf), buf.numel() * buf.element_size(), _stream_ptr(stream),
                                     C.byref(added)), "s2_probe_atomic_add")
    return added.value
