"""ctypes binding of the C-ABI library (argument marshalling only).

Every function here has the name of the C entry point it calls (see
include/sparse_vdit.h); all arithmetic of the attention path runs in the HIP
kernels and the host pattern compiler inside the shared library.  PyTorch
supplies device memory and streams.  There is no fallback: if the library is
missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsparse_vdit.so")

SVD_OK = 0
STATUS_NAMES = {0: "SVD_OK", 1: "SVD_ERR_NULL", 2: "SVD_ERR_SHAPE", 3: "SVD_ERR_DTYPE", 4: "SVD_ERR_ALIGN",
                5: "SVD_ERR_MODE", 6: "SVD_ERR_PARAMS", 7: "SVD_ERR_EMPTY_PATTERN", 8: "SVD_ERR_WORKSPACE",
                9: "SVD_ERR_UNSUPPORTED", 10: "SVD_ERR_HIP", 11: "SVD_ERR_STATIC_LIMIT"}
SVD_DENSE, SVD_SKIP, SVD_DIAG, SVD_MULTIDIAG, SVD_VSTRIPE = range(5)

EXPORTS = ["svd_default_blocks", "svd_plan_workspace_bytes", "svd_plan_create", "svd_plan_destroy",
           "svd_plan_dense_split", "svd_plan_single_launch", "svd_plan_num_groups", "svd_plan_group_info", "svd_plan_group_rearranged", "svd_plan_group_blocks", "svd_plan_row_map", "svd_plan_band_list", "svd_plan_column_list",
           "svd_plan_work", "svd_plan_group_work", "svd_plan_group_work_fp8", "svd_attn_forward_planned", "svd_attn_forward_group", "sparse_vdit_attn_forward", "sparse_vdit_attn_forward_static",
           "svd_dense_attn_forward", "svd_status_string",
           "svd_head_mse_workspace_bytes", "svd_head_mse", "svd_plan_head_sparsity", "svd_plan_head_block_sparsity", "svd_search_select",
           "svd_select_heads", "svd_search_layer_workspace_bytes", "svd_search_layer",
           "svd_fp8_workspace_bytes", "svd_attn_forward_fp8", "svd_attn_forward_fp8_group", "svd_rearrange_tokens", "svd_probe_mfma", "svd_probe_copy"]


class SvdError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__(f"{where}: {STATUS_NAMES.get(self.status, self.status)} ({status_string(self.status)})")


class TensorDesc(C.Structure):
    _fields_ = [("B", C.c_int32), ("H", C.c_int32), ("L", C.c_int32), ("D", C.c_int32),
                ("stride_b", C.c_int64), ("stride_h", C.c_int64), ("stride_l", C.c_int64)]


class HeadParams(C.Structure):
    _fields_ = [("half_width", C.c_int32), ("n_offsets", C.c_int32), ("offsets", C.POINTER(C.c_int32)),
                ("n_cols", C.c_int32), ("cols", C.POINTER(C.c_int32)),
                ("rearr_first", C.c_int32), ("rearr_frame_tokens", C.c_int32), ("rearr_frames", C.c_int32)]


class PlanOptions(C.Structure):
    _fields_ = [("block_q", C.c_int32), ("block_k", C.c_int32), ("dense_split", C.c_int32),
                ("text_tokens", C.c_int32), ("single_launch", C.c_int32), ("no_fork", C.c_int32)]


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2506_03065_amd.build` "
                               "(there is no fallback path)")
        _lib = C.CDLL(LIB_PATH)
        i32p, vp = C.POINTER(C.c_int32), C.c_void_p
        i32pp = C.POINTER(i32p)
        descp, hpp, optp = C.POINTER(TensorDesc), C.POINTER(HeadParams), C.POINTER(PlanOptions)
        sig = {
            "svd_default_blocks": [C.c_int32, i32p, i32p],
            "svd_plan_workspace_bytes": [descp, i32p, hpp, optp, C.POINTER(C.c_size_t)],
            "svd_plan_create": [C.POINTER(vp), descp, i32p, hpp, optp, vp, C.c_size_t, vp],
            "svd_plan_destroy": [vp],
            "svd_plan_dense_split": [vp, i32p],
            "svd_plan_single_launch": [vp, i32p],
            "svd_plan_num_groups": [vp, i32p],
            "svd_plan_group_info": [vp, C.c_int32, i32p, i32p, i32pp, i32pp, i32p],
            "svd_plan_group_rearranged": [vp, C.c_int32, i32p],
            "svd_plan_group_blocks": [vp, C.c_int32, i32p, i32p],
            "svd_plan_row_map": [vp, C.c_int32, C.c_int32, i32p, i32pp],
            "svd_plan_band_list": [vp, C.c_int32, C.c_int32, i32p, i32pp, i32pp, i32pp, i32pp, i32pp, i32p, i32pp],
            "svd_plan_column_list": [vp, C.c_int32, C.c_int32, i32p, i32p, i32pp],
            "svd_plan_work": [vp, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_double)],
            "svd_plan_group_work": [vp, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_double)],
            "svd_plan_group_work_fp8": [vp, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_double)],
            "svd_attn_forward_planned": [vp, vp, vp, vp, vp, vp],
            "svd_attn_forward_group": [vp, C.c_int32, vp, vp, vp, vp, vp],
            "sparse_vdit_attn_forward": [vp, vp, vp, i32p, hpp, vp, descp, vp, C.c_size_t, vp],
            "sparse_vdit_attn_forward_static": [vp, vp, vp, i32p, hpp, vp, descp, vp],
            "svd_dense_attn_forward": [vp, vp, vp, vp, descp, vp],
            "svd_head_mse_workspace_bytes": [descp, C.POINTER(C.c_size_t)],
            "svd_head_mse": [vp, vp, descp, vp, vp, C.c_size_t, vp],
            "svd_plan_head_sparsity": [vp, C.POINTER(C.c_double)],
            "svd_plan_head_block_sparsity": [vp, C.POINTER(C.c_double)],
            "svd_search_select": [C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_double), C.c_double, C.c_double,
                                  i32p, C.POINTER(C.c_double)],
            "svd_select_heads": [C.POINTER(vp), descp, i32p, vp, descp, vp],
            "svd_search_layer_workspace_bytes": [descp, C.POINTER(hpp), C.POINTER(C.c_size_t)],
            "svd_search_layer": [vp, vp, vp, descp, C.POINTER(hpp), C.c_double, C.c_double, i32p,
                                 C.POINTER(C.c_double), vp, vp, C.c_size_t, vp],
            "svd_rearrange_tokens": [vp, vp, descp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp],
            "svd_probe_mfma": [vp, C.c_size_t, C.c_int32, C.c_int32, C.POINTER(C.c_double), vp],
            "svd_probe_copy": [vp, vp, C.c_size_t, vp],
            "svd_fp8_workspace_bytes": [descp, C.POINTER(C.c_size_t)],
            "svd_attn_forward_fp8": [vp, vp, vp, vp, vp, vp, C.c_size_t, vp],
            "svd_attn_forward_fp8_group": [vp, C.c_int32, vp, vp, vp, vp, vp, C.c_size_t, vp],
        }
        for name, args in sig.items():
            fn = getattr(_lib, name)
            fn.argtypes = args
            fn.restype = C.c_int32
        _lib.svd_status_string.argtypes = [C.c_int32]
        _lib.svd_status_string.restype = C.c_char_p
    return _lib


def status_string(status: int) -> str:
    return lib().svd_status_string(int(status)).decode()


def _check(status, where):
    if status != SVD_OK:
        raise SvdError(status, where)


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _ptr(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def tensor_desc(B, H, L, D, stride_b=None, stride_h=None, stride_l=None) -> TensorDesc:
    stride_l = D if stride_l is None else stride_l
    stride_h = L * stride_l if stride_h is None else stride_h
    stride_b = H * stride_h if stride_b is None else stride_b
    return TensorDesc(B, H, L, D, stride_b, stride_h, stride_l)


def desc_of(t) -> TensorDesc:
    """Descriptor of a [B, H, L, D] torch tensor whose last axis is contiguous."""
    if t.dim() != 4 or t.stride(3) != 1:
        raise ValueError("expected a [B, H, L, D] tensor with a contiguous last axis")
    B, H, L, D = t.shape
    return TensorDesc(B, H, L, D, t.stride(0), t.stride(1), t.stride(2))


class _Marshalled:
    """Host arrays behind an svd_head_params[H]; keeps them alive."""

    def __init__(self, strategy_table, pattern_params):
        self.table = _i32(strategy_table)
        H = self.table.size
        if len(pattern_params) != H:
            raise ValueError("pattern_params must have one entry per head")
        self.keep = []
        self.params = (HeadParams * H)()
        for h, p in enumerate(pattern_params):
            p = p or {}
            offs = _i32(p.get("offsets", ()))
            cols = _i32(p.get("cols", ()))
            self.keep += [offs, cols]
            self.params[h].half_width = int(p.get("half_width", 0))
            self.params[h].n_offsets = offs.size
            self.params[h].offsets = _ptr(offs) if offs.size else None
            self.params[h].n_cols = cols.size
            self.params[h].cols = _ptr(cols) if cols.size else None
            first, n, f = p.get("rearranged") or (0, 0, 0)
            self.params[h].rearr_first, self.params[h].rearr_frame_tokens, self.params[h].rearr_frames = int(first), int(n), int(f)


def _text_tokens(strategy_table, pattern_params, text_tokens):
    """The plan option text_tokens: given explicitly, or read from the parameter
    dicts of the heads in a sparse mode (key "text_tokens"; they must agree)."""
    if text_tokens is not None:
        return int(text_tokens)
    found = {int((p or {}).get("text_tokens", 0)) for m, p in zip(strategy_table, pattern_params) if int(m) >= 2}
    if len(found) > 1:
        raise ValueError("the sparse heads of a layer must share one text prefix")
    return found.pop() if found else 0


def svd_default_blocks(D: int):
    bq, bk = C.c_int32(), C.c_int32()
    _check(lib().svd_default_blocks(D, C.byref(bq), C.byref(bk)), "svd_default_blocks")
    return bq.value, bk.value


def svd_plan_workspace_bytes(desc, strategy_table, pattern_params, block_q=0, block_k=0, dense_split=0,
                             text_tokens=None, single_launch=0, no_fork=0) -> int:
    m = _Marshalled(strategy_table, pattern_params)
    opt = PlanOptions(block_q, block_k, dense_split, _text_tokens(strategy_table, pattern_params, text_tokens),
                      single_launch, no_fork)
    n = C.c_size_t()
    _check(lib().svd_plan_workspace_bytes(C.byref(desc), _ptr(m.table), m.params, C.byref(opt), C.byref(n)),
           "svd_plan_workspace_bytes")
    return n.value


def _copy(ptr, n):
    return np.ctypeslib.as_array(ptr, shape=(n,)).copy() if n else np.zeros(0, dtype=np.int32)


class Plan:
    """Owner of an svd_plan* (and of the torch workspace tensor, if given)."""

    def __init__(self, handle, desc, workspace):
        self.handle, self.desc, self.workspace = handle, desc, workspace

    def close(self):
        if self.handle:
            lib().svd_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- inspection ----
    def head_sparsity(self):
        out = np.zeros(self.desc.H, dtype=np.float64)
        _check(lib().svd_plan_head_sparsity(self.handle, out.ctypes.data_as(C.POINTER(C.c_double))),
               "svd_plan_head_sparsity")
        return out

    def head_block_sparsity(self):
        out = np.zeros(self.desc.H, dtype=np.float64)
        _check(lib().svd_plan_head_block_sparsity(self.handle, out.ctypes.data_as(C.POINTER(C.c_double))),
               "svd_plan_head_block_sparsity")
        return out

    def dense_split(self) -> int:
        n = C.c_int32()
        _check(lib().svd_plan_dense_split(self.handle, C.byref(n)), "svd_plan_dense_split")
        return n.value

    def launch_form(self) -> int:
        """0 = a launch per group, 1 = the layer kernel alone, 3 = the layer kernel after the dense head start."""
        n = C.c_int32()
        _check(lib().svd_plan_single_launch(self.handle, C.byref(n)), "svd_plan_single_launch")
        return n.value

    def single_launch(self) -> bool:
        return self.launch_form() != 0

    def groups(self):
        L_ = lib()
        n = C.c_int32()
        _check(L_.svd_plan_num_groups(self.handle, C.byref(n)), "svd_plan_num_groups")
        out = []
        for g in range(n.value):
            mode, nh, nl = C.c_int32(), C.c_int32(), C.c_int32()
            heads, lid = C.POINTER(C.c_int32)(), C.POINTER(C.c_int32)()
            _check(L_.svd_plan_group_info(self.handle, g, C.byref(mode), C.byref(nh), C.byref(heads),
                                          C.byref(lid), C.byref(nl)), "svd_plan_group_info")
            rearranged = C.c_int32()
            _check(L_.svd_plan_group_rearranged(self.handle, g, C.byref(rearranged)), "svd_plan_group_rearranged")
            gbq, gbk = C.c_int32(), C.c_int32()
            _check(L_.svd_plan_group_blocks(self.handle, g, C.byref(gbq), C.byref(gbk)), "svd_plan_group_blocks")
            out.append({"mode": mode.value, "heads": _copy(heads, nh.value).tolist(),
                        "list_id": _copy(lid, nh.value).tolist(), "n_lists": nl.value,
                        "rearranged": bool(rearranged.value), "block_q": gbq.value, "block_k": gbk.value})
        return out

    def row_map(self, group, lst):
        padded = C.c_int32()
        rm = C.POINTER(C.c_int32)()
        _check(lib().svd_plan_row_map(self.handle, group, lst, C.byref(padded), C.byref(rm)), "svd_plan_row_map")
        return _copy(rm, padded.value)

    def band_list(self, group, lst):
        nqb, nruns = C.c_int32(), C.c_int32()
        ptrs = [C.POINTER(C.c_int32)() for _ in range(6)]
        _check(lib().svd_plan_band_list(self.handle, group, lst, C.byref(nqb), C.byref(ptrs[0]), C.byref(ptrs[1]),
                                        C.byref(ptrs[2]), C.byref(ptrs[3]), C.byref(ptrs[4]), C.byref(nruns),
                                        C.byref(ptrs[5])), "svd_plan_band_list")
        row_ptr = _copy(ptrs[0], nqb.value + 1)
        nnz = int(row_ptr[-1])
        return {"row_ptr": row_ptr, "kv_block_idx": _copy(ptrs[1], nnz), "flags": _copy(ptrs[2], nnz),
                "run_first": _copy(ptrs[3], nnz), "run_count": _copy(ptrs[4], nnz),
                "runs": _copy(ptrs[5], 2 * nruns.value).reshape(-1, 2)}

    def column_list(self, group, lst):
        n, padded = C.c_int32(), C.c_int32()
        cols = C.POINTER(C.c_int32)()
        _check(lib().svd_plan_column_list(self.handle, group, lst, C.byref(n), C.byref(padded), C.byref(cols)),
               "svd_plan_column_list")
        return {"n_cols": n.value, "cols": _copy(cols, padded.value)}

    def work_fp8(self, group=None):
        """Tiles and FLOPs the FP8 forward pass computes (band groups always on the small query tile)."""
        tiles, flops = C.c_int64(), C.c_double()
        _check(lib().svd_plan_group_work_fp8(self.handle, -1 if group is None else group, C.byref(tiles), C.byref(flops)),
               "svd_plan_group_work_fp8")
        return {"computed_tiles": tiles.value, "computed_flops": flops.value}

    def work(self, group=None):
        tiles, flops, pairs = C.c_int64(), C.c_double(), C.c_double()
        if group is None:
            _check(lib().svd_plan_work(self.handle, C.byref(tiles), C.byref(flops), C.byref(pairs)), "svd_plan_work")
        else:
            _check(lib().svd_plan_group_work(self.handle, group, C.byref(tiles), C.byref(flops), C.byref(pairs)),
                   "svd_plan_group_work")
        return {"computed_tiles": tiles.value, "computed_flops": flops.value, "kept_pairs": pairs.value}


def svd_plan_create(desc, strategy_table, pattern_params, block_q=0, block_k=0, workspace=None, stream=None,
                    dense_split=0, text_tokens=None, single_launch=0, no_fork=0) -> Plan:
    """workspace: a torch uint8/int32 CUDA tensor of at least svd_plan_workspace_bytes
    bytes, or None for a host-only plan (inspection, no launches).  text_tokens:
    the plan option; None reads it from the "text_tokens" key of the sparse
    heads' parameter dicts."""
    m = _Marshalled(strategy_table, pattern_params)
    opt = PlanOptions(block_q, block_k, dense_split, _text_tokens(strategy_table, pattern_params, text_tokens),
                      single_launch, no_fork)
    handle = C.c_void_p()
    ws_ptr = C.c_void_p(workspace.data_ptr()) if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().svd_plan_create(C.byref(handle), C.byref(desc), _ptr(m.table), m.params, C.byref(opt),
                                 ws_ptr, ws_bytes, _stream_ptr(stream)), "svd_plan_create")
    return Plan(handle, desc, workspace)


def _stream_ptr(stream):
    if stream is None:
        import torch
        if torch.cuda.is_available():
            return C.c_void_p(torch.cuda.current_stream().cuda_stream)
        return None
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dev(t):
    return C.c_void_p(t.data_ptr())


def svd_attn_forward_planned(plan: Plan, q, k, v, out, stream=None):
    _check(lib().svd_attn_forward_planned(plan.handle, _dev(q), _dev(k), _dev(v), _dev(out), _stream_ptr(stream)),
           "svd_attn_forward_planned")
    return out


def svd_rearrange_tokens(src, dst, first_video_token, frame_tokens, frames, inverse=False, stream=None):
    """src, dst: distinct CUDA bf16 tensors of one [B, H, L, D] layout."""
    if dst.shape != src.shape or dst.stride() != src.stride():
        raise ValueError("src and dst must share shape and strides")
    desc = desc_of(src)
    _check(lib().svd_rearrange_tokens(_dev(src), _dev(dst), C.byref(desc), int(first_video_token), int(frame_tokens),
                                      int(frames), 1 if inverse else 0, _stream_ptr(stream)), "svd_rearrange_tokens")
    return dst


def svd_fp8_workspace_bytes(desc) -> int:
    n = C.c_size_t(0)
    _check(lib().svd_fp8_workspace_bytes(C.byref(desc), C.byref(n)), "svd_fp8_workspace_bytes")
    return int(n.value)


def svd_attn_forward_fp8(plan: Plan, q, k, v, out, fp8_workspace, stream=None):
    """fp8_workspace: uint8 CUDA tensor of svd_fp8_workspace_bytes(desc) bytes."""
    _check(lib().svd_attn_forward_fp8(plan.handle, _dev(q), _dev(k), _dev(v), _dev(out), _dev(fp8_workspace),
                                      fp8_workspace.numel() * fp8_workspace.element_size(), _stream_ptr(stream)),
           "svd_attn_forward_fp8")
    return out


def svd_attn_forward_fp8_group(plan: Plan, group: int, q, k, v, out, fp8_workspace, stream=None):
    _check(lib().svd_attn_forward_fp8_group(plan.handle, int(group), _dev(q), _dev(k), _dev(v), _dev(out),
                                            _dev(fp8_workspace), fp8_workspace.numel() * fp8_workspace.element_size(),
                                            _stream_ptr(stream)), "svd_attn_forward_fp8_group")
    return out


def svd_attn_forward_group(plan: Plan, group: int, q, k, v, out, stream=None):
    _check(lib().svd_attn_forward_group(plan.handle, group, _dev(q), _dev(k), _dev(v), _dev(out),
                                        _stream_ptr(stream)), "svd_attn_forward_group")
    return out


def sparse_vdit_attn_forward(q, k, v, strategy_table, pattern_params, out, workspace, stream=None):
    desc = desc_of(q)
    m = _Marshalled(strategy_table, pattern_params)
    _check(lib().sparse_vdit_attn_forward(_dev(q), _dev(k), _dev(v), _ptr(m.table), m.params, _dev(out),
                                          C.byref(desc), _dev(workspace),
                                          workspace.numel() * workspace.element_size(), _stream_ptr(stream)),
           "sparse_vdit_attn_forward")
    return out


def sparse_vdit_attn_forward_static(q, k, v, strategy_table, pattern_params, out, stream=None):
    desc = desc_of(q)
    m = _Marshalled(strategy_table, pattern_params)
    _check(lib().sparse_vdit_attn_forward_static(_dev(q), _dev(k), _dev(v), _ptr(m.table), m.params, _dev(out),
                                                 C.byref(desc), _stream_ptr(stream)),
           "sparse_vdit_attn_forward_static")
    return out


def svd_dense_attn_forward(q, k, v, out, stream=None):
    desc = desc_of(q)
    _check(lib().svd_dense_attn_forward(_dev(q), _dev(k), _dev(v), _dev(out), C.byref(desc), _stream_ptr(stream)),
           "svd_dense_attn_forward")
    return out


# ---- calibration probes of the benchmark ----

def svd_probe_mfma(scratch, iters, work_groups, stream=None) -> float:
    """Launches the matrix-instruction loop; returns the FLOPs of the launch.  scratch: CUDA float32, work_groups * 512 elements."""
    flops = C.c_double()
    _check(lib().svd_probe_mfma(_dev(scratch), scratch.numel() * scratch.element_size(), int(iters), int(work_groups),
                                C.byref(flops), _stream_ptr(stream)), "svd_probe_mfma")
    return flops.value


def svd_probe_copy(src, dst, stream=None):
    nbytes = src.numel() * src.element_size()
    _check(lib().svd_probe_copy(_dev(src), _dev(dst), nbytes, _stream_ptr(stream)), "svd_probe_copy")
    return dst


# ---- offline search step (Section 4.2, Eq. 2-3, Algorithm 1) ----

def svd_head_mse_workspace_bytes(desc) -> int:
    n = C.c_size_t()
    _check(lib().svd_head_mse_workspace_bytes(C.byref(desc), C.byref(n)), "svd_head_mse_workspace_bytes")
    return n.value


def svd_head_mse(o, o_ref, mse, workspace, stream=None):
    """o, o_ref: CUDA bf16 [B, H, L, D]; mse: CUDA float32 [H] (written); workspace: CUDA scratch."""
    desc = desc_of(o)
    _check(lib().svd_head_mse(_dev(o), _dev(o_ref), C.byref(desc), _dev(mse), _dev(workspace),
                              workspace.numel() * workspace.element_size(), _stream_ptr(stream)), "svd_head_mse")
    return mse


def svd_search_select(mse, sparsity, lam, eps):
    """mse, sparsity: [4, H] (row i - 1 = mode i).  Returns (table int32 [H], loss float64 [4, H])."""
    mse = np.ascontiguousarray(np.asarray(mse, dtype=np.float32))
    sparsity = np.ascontiguousarray(np.asarray(sparsity, dtype=np.float64))
    H = mse.shape[1]
    table = np.zeros(H, dtype=np.int32)
    loss = np.zeros((4, H), dtype=np.float64)
    _check(lib().svd_search_select(H, mse.ctypes.data_as(C.POINTER(C.c_float)),
                                   sparsity.ctypes.data_as(C.POINTER(C.c_double)), float(lam), float(eps),
                                   _ptr(table), loss.ctypes.data_as(C.POINTER(C.c_double))), "svd_search_select")
    return table, loss


def svd_select_heads(o_modes, table, out, stream=None):
    """o_modes: five CUDA tensors (None where the table does not use the mode); out[:, h] = o_modes[table[h]][:, h]."""
    first = next(t for t in o_modes if t is not None)
    src_desc, out_desc = desc_of(first), desc_of(out)
    ptrs = (C.c_void_p * 5)(*[C.c_void_p(t.data_ptr()) if t is not None else None for t in o_modes])
    table = _i32(table)
    _check(lib().svd_select_heads(ptrs, C.byref(src_desc), _ptr(table), _dev(out), C.byref(out_desc),
                                  _stream_ptr(stream)), "svd_select_heads")
    return out


def _params_by_mode(params_by_mode, H):
    """dict mode id (2, 3, 4) -> H parameter dicts  ->  (array of five HeadParams pointers, keep-alive list)."""
    keep, arr = [], (C.POINTER(HeadParams) * 5)()
    for mode in (2, 3, 4):
        m = _Marshalled(np.full(H, mode, dtype=np.int32), params_by_mode[mode])
        keep.append(m)
        arr[mode] = C.cast(m.params, C.POINTER(HeadParams))
    return arr, keep


def svd_search_layer_workspace_bytes(desc, params_by_mode) -> int:
    arr, keep = _params_by_mode(params_by_mode, desc.H)
    n = C.c_size_t()
    _check(lib().svd_search_layer_workspace_bytes(C.byref(desc), arr, C.byref(n)), "svd_search_layer_workspace_bytes")
    return n.value


def svd_search_layer(q, k, v, params_by_mode, lam, eps, out, workspace, stream=None):
    """Returns (table int32 [H], loss float64 [4, H]); out receives the chosen outputs.  Synchronises."""
    desc = desc_of(q)
    arr, keep = _params_by_mode(params_by_mode, desc.H)
    table = np.zeros(desc.H, dtype=np.int32)
    loss = np.zeros((4, desc.H), dtype=np.float64)
    _check(lib().svd_search_layer(_dev(q), _dev(k), _dev(v), C.byref(desc), arr, float(lam), float(eps), _ptr(table),
                                  loss.ctypes.data_as(C.POINTER(C.c_double)), _dev(out), _dev(workspace),
                                  workspace.numel() * workspace.element_size(), _stream_ptr(stream)),
           "svd_search_layer")
    return table, loss
