"""ctypes binding of include/vnm.h.  PyTorch is used for device memory and streams only."""

from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

PATH_AUTO, PATH_GENERIC, PATH_SMFMAC = 0, 1, 2

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class VnmError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(what)


class VnmSizes(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in (
        "out_pad", "in_pad", "row_blocks", "col_blocks", "kc", "values_elems", "meta_bytes",
        "colidx_bytes", "packed_bytes", "workspace_bytes")]


def lib_path() -> str:
    """The in-tree library."""
    return os.path.join(_PKG_DIR, "libvnm.so")


def load_library():
    """Load libvnm.so.  The library carries a hash of the sources it was built from; when it is
    missing, or the sources have changed since, it is rebuilt first (hipcc needed), so results never
    come from kernels that are no longer in the tree.  Raises if neither works."""
    global _LIB
    if _LIB is not None:
        return _LIB
    from .build import build_library, built_hash, source_hash
    path = lib_path()
    want = source_hash()
    if built_hash(path) != want:
        import sys
        print("libvnm.so is missing or older than its sources: rebuilding", file=sys.stderr, flush=True)
        build_library()
        if built_hash(path) != want:
            raise VnmError(-1, "libvnm.so does not match its sources even after a rebuild")
    lib = ctypes.CDLL(path)
    lib.vnm_source_hash.restype = ctypes.c_char_p
    if lib.vnm_source_hash().decode() != want:
        raise VnmError(-1, "the loaded libvnm.so reports a different source hash than its file")
    vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    lib.vnm_query_sizes.argtypes = [i64, i64, ci, ci, ci, ctypes.POINTER(VnmSizes)]
    lib.vnm_prune_compress.argtypes = [vp, i64, i64, i64, ci, ci, ci, vp, vp, vp, vp, vp, vp, i64, vp]
    lib.vnm_pack.argtypes = [vp, vp, vp, i64, i64, ci, ci, ci, vp, vp]
    lib.vnm_spmm.argtypes = [vp, i64, i64, vp, vp, vp, vp, i64, i64, ci, ci, ci, vp, i64, ci, ci, vp, i64, vp]
    lib.vnm_spmm_noalloc.argtypes = [vp, i64, i64, vp, vp, vp, vp, i64, i64, ci, ci, ci, vp, i64, ci, ci, vp]
    lib.vnm_spmm_noalloc.restype = ci
    lib.vnm_spmm_fused.argtypes = [vp, i64, i64, vp, vp, vp, vp, i64, i64, ci, ci, ci, vp, vp, vp, vp, i64, ci, ci,
                                   vp, i64, vp]
    lib.vnm_spmm_fused.restype = ci
    lib.vnm_spmm_fused_workspace_bytes.argtypes = [i64, i64, i64, ci, ci, ci, ci, ctypes.POINTER(i64)]
    lib.vnm_spmm_fused_workspace_bytes.restype = ci
    cd = ctypes.c_double
    lib.vnm_permutation_search_workspace_bytes.argtypes = [i64, i64, ci, ci, ci, ctypes.POINTER(i64)]
    lib.vnm_permutation_search_workspace_bytes.restype = ci
    lib.vnm_permutation_search.argtypes = [vp, i64, i64, i64, ci, ci, ci, cd, ci, vp, vp, vp, vp, i64, vp]
    lib.vnm_permutation_search.restype = ci
    lib.vnm_permutation_gain.argtypes = [vp, i64, i64, i64, ci, ci, ci, cd, ci, ci, vp, vp, vp, vp, i64, vp]
    lib.vnm_permutation_gain.restype = ci
    lib.vnm_retained_score.argtypes = [vp, i64, i64, i64, ci, ci, ci, cd, vp, vp, ctypes.POINTER(i64), vp, i64, vp]
    lib.vnm_retained_score.restype = ci
    lib.vnm_lora_merge.argtypes = [vp, i64, i64, i64, vp, i64, vp, i64, ci, ctypes.c_float, vp, i64, vp]
    lib.vnm_lora_merge.restype = ci
    lib.vnm_lsa_max.argtypes = [vp, ci, vp, ctypes.POINTER(i64)]
    lib.vnm_lsa_max.restype = ci
    lib.vnm_lsa_max_method.argtypes = [vp, ci, ci, vp, ctypes.POINTER(i64)]
    lib.vnm_lsa_max_method.restype = ci
    lib.vnm_fold_permutations.argtypes = [vp, vp, i64, vp]
    lib.vnm_fold_permutations.restype = ci
    lib.vnm_decompress.argtypes = [vp, vp, vp, i64, i64, ci, ci, ci, vp, i64, vp]
    lib.vnm_stage_x.argtypes = [vp, i64, i64, i64, ci, vp, i64, vp]
    lib.vnm_spmm_staged.argtypes = [vp, i64, i64, vp, i64, i64, ci, ci, ci, vp, i64, ci, vp, i64, vp]
    lib.vnm_stage_x.restype = ci
    lib.vnm_spmm_staged.restype = ci
    lib.vnm_spmm_kernel_choice.argtypes = [i64, i64, i64, ci, ci, ci, i64, ctypes.POINTER(ci)]
    lib.vnm_spmm_kernel_choice.restype = ci
    lib.vnm_spmm_workspace_bytes.argtypes = [i64, i64, i64, ci, ci, ci, ctypes.POINTER(i64)]
    lib.vnm_spmm_workspace_bytes.restype = ci
    lib.vnm_ria_scores.argtypes = [vp, i64, i64, i64, vp, vp, i64, vp, i64, vp]
    lib.vnm_ria_scores.restype = ci
    lib.vnm_prune_compress_scored.argtypes = [vp, vp, i64, i64, i64, i64, ci, ci, ci, vp, vp, vp, vp, vp, vp]
    lib.vnm_prune_compress_scored.restype = ci
    lib.vnm_mask_diversity_log.argtypes = [ci, ci, ci, ctypes.POINTER(ctypes.c_double)]
    lib.vnm_mask_diversity_log.restype = ci
    lib.vnm_select_vm.argtypes = [ctypes.POINTER(ci), ctypes.POINTER(ci), ctypes.POINTER(ctypes.c_double), ci,
                                  ctypes.c_double, ctypes.POINTER(ci)]
    lib.vnm_select_vm.restype = ci
    lib.vnm_stage_x_bytes.argtypes = [i64, i64, ci, ctypes.POINTER(i64)]
    lib.vnm_stage_x_bytes.restype = ci
    lib.vnm_spmm_scratch_bytes.argtypes = [i64, i64, ctypes.POINTER(i64)]
    lib.vnm_spmm_scratch_bytes.restype = ci
    for f in (lib.vnm_query_sizes, lib.vnm_prune_compress, lib.vnm_pack, lib.vnm_spmm, lib.vnm_decompress,
              lib.vnm_format_version):
        f.restype = ci
    lib.vnm_status_string.argtypes = [ci]
    lib.vnm_status_string.restype = ctypes.c_char_p
    lib.vnm_last_hip_error.restype = ctypes.c_char_p
    _LIB = lib
    return lib


def _check(status: int, what: str):
    if status != 0:
        lib = load_library()
        msg = lib.vnm_status_string(status).decode()
        detail = lib.vnm_last_hip_error().decode()
        if status == 6 or (status == 5 and what == "vnm_spmm_noalloc" and detail):
            msg += " (" + detail + ")"
        raise VnmError(status, f"{what}: {msg}")


def _ptr(t):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _stream(t):
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def vnm_query_sizes(out: int, inn: int, V: int, M: int, N: int = 2) -> VnmSizes:
    s = VnmSizes()
    _check(load_library().vnm_query_sizes(out, inn, V, N, M, ctypes.byref(s)), "vnm_query_sizes")
    return s


@dataclass
class Compressed:
    """The compressed triple of one layer plus the opaque matrix-core copy (device tensors)."""
    values: object
    meta: object
    colidx: object
    packed: object
    out: int
    inn: int
    V: int
    M: int
    mask: object = None


def _alloc(sizes: VnmSizes, device, want_packed=True):
    import torch
    values = torch.empty(sizes.values_elems, dtype=torch.float16, device=device)
    meta = torch.empty(sizes.meta_bytes, dtype=torch.uint8, device=device)
    colidx = torch.empty(sizes.colidx_bytes, dtype=torch.uint8, device=device)
    packed = None
    if want_packed and sizes.packed_bytes > 0:
        packed = torch.empty(sizes.packed_bytes, dtype=torch.uint8, device=device)
    return values, meta, colidx, packed


def vnm_prune_compress(W, V: int, M: int, N: int = 2, want_mask: bool = False, want_packed: bool = True,
                       out=None) -> Compressed:
    """W: fp16 CUDA tensor [out x in] (row stride may exceed `in`).  Allocates the outputs (or
    reuses `out`, a Compressed of the same layer) and enqueues the kernel on the current stream."""
    import torch
    assert W.is_cuda and W.dtype == torch.float16 and W.dim() == 2 and W.stride(1) == 1
    o, i = W.shape
    sizes = vnm_query_sizes(o, i, V, M, N)
    if out is None:
        values, meta, colidx, packed = _alloc(sizes, W.device, want_packed)
        mask = torch.empty((o, i), dtype=torch.uint8, device=W.device) if want_mask else None
        out = Compressed(values, meta, colidx, packed, o, i, V, M, mask)
    _check(load_library().vnm_prune_compress(
        _ptr(W), o, i, W.stride(0), V, N, M, _ptr(out.values), _ptr(out.meta), _ptr(out.colidx),
        _ptr(out.mask), _ptr(out.packed), None, 0, _stream(W)), "vnm_prune_compress")
    return out


def vnm_ria_scores(W, act, S=None):
    """fp32 RIA scores [out x in] of W (fp16 CUDA) for the activation factors act (fp32 CUDA [in])."""
    import torch
    assert W.is_cuda and W.dtype == torch.float16 and W.dim() == 2 and W.stride(1) == 1
    assert act.is_cuda and act.dtype == torch.float32 and act.shape == (W.shape[1],) and act.is_contiguous()
    o, i = W.shape
    if S is None:
        S = torch.empty((o, i), dtype=torch.float32, device=W.device)
    ws = torch.empty((o + i) * 8, dtype=torch.uint8, device=W.device)
    _check(load_library().vnm_ria_scores(_ptr(W), o, i, W.stride(0), _ptr(act), _ptr(S), S.stride(0), _ptr(ws),
                                         ws.numel(), _stream(W)), "vnm_ria_scores")
    return S


def vnm_prune_compress_scored(W, S, V: int, M: int, N: int = 2, want_mask: bool = False,
                              want_packed: bool = True, out=None) -> Compressed:
    """vnm_prune_compress driven by the fp32 score matrix S [out x in] instead of |W|."""
    import torch
    assert W.is_cuda and W.dtype == torch.float16 and W.dim() == 2 and W.stride(1) == 1
    assert S.is_cuda and S.dtype == torch.float32 and S.shape == W.shape and S.stride(1) == 1
    o, i = W.shape
    sizes = vnm_query_sizes(o, i, V, M, N)
    if out is None:
        values, meta, colidx, packed = _alloc(sizes, W.device, want_packed)
        mask = torch.empty((o, i), dtype=torch.uint8, device=W.device) if want_mask else None
        out = Compressed(values, meta, colidx, packed, o, i, V, M, mask)
    _check(load_library().vnm_prune_compress_scored(
        _ptr(W), _ptr(S), o, i, W.stride(0), S.stride(0), V, N, M, _ptr(out.values), _ptr(out.meta),
        _ptr(out.colidx), _ptr(out.mask), _ptr(out.packed), _stream(W)), "vnm_prune_compress_scored")
    return out


def vnm_pack(c: Compressed, N: int = 2) -> Compressed:
    import torch
    sizes = vnm_query_sizes(c.out, c.inn, c.V, c.M, N)
    if c.packed is None:
        c.packed = torch.empty(sizes.packed_bytes, dtype=torch.uint8, device=c.values.device)
    _check(load_library().vnm_pack(_ptr(c.values), _ptr(c.meta), _ptr(c.colidx), c.out, c.inn, c.V, N, c.M,
                                   _ptr(c.packed), _stream(c.values)), "vnm_pack")
    return c


def vnm_spmm_workspace_bytes(T: int, c: Compressed, N: int = 2) -> int:
    b = ctypes.c_int64(0)
    _check(load_library().vnm_spmm_workspace_bytes(T, c.out, c.inn, c.V, N, c.M, ctypes.byref(b)),
           "vnm_spmm_workspace_bytes")
    return b.value


_WORKSPACES = {}


def _workspace(device, nbytes: int):
    """One grow-only scratch tensor per device, shared by all vnm_spmm calls of this process.
    Its reuse is ordered by the stream the calls run on: callers that use several streams at once
    must hand every call a `workspace` of its own."""
    import torch
    ws = _WORKSPACES.get(device)
    if ws is None or ws.numel() < nbytes:
        dev = device[0] if isinstance(device, tuple) else device
        ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=dev)
        _WORKSPACES[device] = ws
    return ws


def vnm_spmm(X, c: Compressed, N: int = 2, out_dtype=None, path: int = PATH_AUTO, Y=None, workspace=None):
    """Y [T x out] = X [T x in] . W'^T on the compressed weight; fp16 in, fp32 accumulate.
    `workspace`: optional uint8 CUDA tensor of at least vnm_spmm_workspace_bytes(T, c) bytes;
    by default a process-wide grow-only scratch tensor is used."""
    import torch
    assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.stride(1) == 1
    T = X.shape[0]
    assert X.shape[1] == c.inn
    if Y is None:
        Y = torch.empty((T, c.out), dtype=out_dtype or torch.float16, device=X.device)
    y_dtype = {torch.float16: 0, torch.float32: 1}[Y.dtype]
    ws, ws_bytes = None, 0
    if path != PATH_GENERIC and c.packed is not None and T > 0:
        ws_bytes = vnm_spmm_workspace_bytes(T, c, N)
        ws = workspace if workspace is not None else _workspace(X.device, ws_bytes)
        ws_bytes = ws.numel()
    _check(load_library().vnm_spmm(
        _ptr(X), T, X.stride(0) if T > 0 else c.inn, _ptr(c.values), _ptr(c.meta), _ptr(c.colidx),
        _ptr(c.packed), c.out, c.inn, c.V, N, c.M, _ptr(Y), Y.stride(0) if T > 0 else c.out, y_dtype, path,
        _ptr(ws), ws_bytes, _stream(X)), "vnm_spmm")
    return Y


def vnm_spmm_bind(X, c: Compressed, Y, workspace, N: int = 2, path: int = PATH_AUTO):
    """The vnm_spmm call on these buffers with its arguments marshalled once: returns a function of
    no arguments that issues the call on torch's current stream (a loop that serves the same layer
    again and again -- decoding -- pays the argument conversion once, not per call).  The tensors
    must stay alive and in place while the function is used."""
    import torch
    assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.stride(1) == 1
    T = X.shape[0]
    assert T > 0 and X.shape[1] == c.inn and Y.shape == (T, c.out) and Y.stride(1) == 1
    y_dtype = {torch.float16: 0, torch.float32: 1}[Y.dtype]
    fn = load_library().vnm_spmm
    args = (_ptr(X), ctypes.c_int64(T), ctypes.c_int64(X.stride(0)), _ptr(c.values), _ptr(c.meta), _ptr(c.colidx),
            _ptr(c.packed), ctypes.c_int64(c.out), ctypes.c_int64(c.inn), ctypes.c_int(c.V), ctypes.c_int(N),
            ctypes.c_int(c.M), _ptr(Y), ctypes.c_int64(Y.stride(0)), ctypes.c_int(y_dtype), ctypes.c_int(path),
            _ptr(workspace), ctypes.c_int64(0 if workspace is None else workspace.numel()))
    dev = X.device
    keep = (X, c, Y, workspace)

    def call():
        rc = fn(*args, torch.cuda.current_stream(dev).cuda_stream)
        if rc:
            _check(rc, "vnm_spmm")
        return keep[2]
    return call


NOALLOC_SCRATCH_BYTES = 32 << 20


def vnm_spmm_noalloc(X, c: Compressed, Y, N: int = 2, path: int = PATH_AUTO):
    """vnm_spmm into a caller-supplied Y with the library's built-in scratch instead of a workspace:
    the call allocates nothing (for callers that cannot: graph capture, serving loops)."""
    import torch
    assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.stride(1) == 1
    T = X.shape[0]
    assert X.shape[1] == c.inn and Y.shape == (T, c.out) and Y.stride(1) == 1
    y_dtype = {torch.float16: 0, torch.float32: 1}[Y.dtype]
    _check(load_library().vnm_spmm_noalloc(
        _ptr(X), T, X.stride(0) if T > 0 else c.inn, _ptr(c.values), _ptr(c.meta), _ptr(c.colidx),
        _ptr(c.packed), c.out, c.inn, c.V, N, c.M, _ptr(Y), Y.stride(0) if T > 0 else c.out, y_dtype, path,
        _stream(X)), "vnm_spmm_noalloc")
    return Y


def vnm_spmm_fused(X, c: Compressed, bias=None, perm_in=None, perm_out=None, N: int = 2, out_dtype=None,
                   path: int = PATH_AUTO, Y=None, workspace=None):
    """vnm_spmm with an optional bias (fp16 [out], row order of the compressed weight) and the two
    channel permutations of Eq. 6 (int32 CUDA tensors): Y[t, perm_out[o]] = bias[o] + sum_i W'[o, i]
    X[t, perm_in[i]].  If perm_out is not a permutation, untouched columns of a fresh Y are undefined."""
    import torch
    assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.stride(1) == 1
    T = X.shape[0]
    assert X.shape[1] == c.inn
    for name, p, n, dt in (("bias", bias, c.out, torch.float16), ("perm_in", perm_in, c.inn, torch.int32),
                           ("perm_out", perm_out, c.out, torch.int32)):
        assert p is None or (p.is_cuda and p.dtype == dt and p.is_contiguous() and p.numel() == n), name
    if Y is None:
        Y = torch.empty((T, c.out), dtype=out_dtype or torch.float16, device=X.device)
    y_dtype = {torch.float16: 0, torch.float32: 1}[Y.dtype]
    ws, ws_bytes = None, 0
    if path != PATH_GENERIC and c.packed is not None and T > 0:
        b = ctypes.c_int64(0)
        _check(load_library().vnm_spmm_fused_workspace_bytes(T, c.out, c.inn, c.V, N, c.M, int(perm_in is not None),
                                                             ctypes.byref(b)), "vnm_spmm_fused_workspace_bytes")
        ws = workspace if workspace is not None else _workspace(X.device, b.value)
        ws_bytes = ws.numel()
    _check(load_library().vnm_spmm_fused(
        _ptr(X), T, X.stride(0) if T > 0 else c.inn, _ptr(c.values), _ptr(c.meta), _ptr(c.colidx),
        _ptr(c.packed), c.out, c.inn, c.V, N, c.M, _ptr(bias), _ptr(perm_in), _ptr(perm_out), _ptr(Y),
        Y.stride(0) if T > 0 else c.out, y_dtype, path, _ptr(ws), ws_bytes, _stream(X)), "vnm_spmm_fused")
    return Y


def vnm_fold_permutations(perm_out_prev, perm_in_next):
    """Host: input permutation of the next layer when the previous one leaves its output in the
    row order of its (permuted) weight; int32 numpy arrays in, int32 numpy array out."""
    import numpy as np
    po = np.ascontiguousarray(perm_out_prev, dtype=np.int32)
    pi = np.ascontiguousarray(perm_in_next, dtype=np.int32)
    assert po.ndim == 1 and po.shape == pi.shape
    res = np.empty_like(po)
    _check(load_library().vnm_fold_permutations(po.ctypes.data, pi.ctypes.data, po.size, res.ctypes.data),
           "vnm_fold_permutations")
    return res


def _ps_workspace(S, V, M, N):
    import torch
    b = ctypes.c_int64(0)
    _check(load_library().vnm_permutation_search_workspace_bytes(S.shape[0], S.shape[1], V, N, M, ctypes.byref(b)),
           "vnm_permutation_search_workspace_bytes")
    return _workspace((S.device, "permsearch"), b.value)


def _host_perm(p, n):
    import numpy as np
    if p is None:
        return None, None
    a = np.ascontiguousarray(p, dtype=np.int32)
    assert a.shape == (n,)
    return a, a.ctypes.data


def vnm_permutation_search(S, V: int, M: int, scale: float, iterations: int = 2, N: int = 2):
    """Channel-permutation search of Eqs. 7-9 on the fp32 CUDA score matrix S.  Returns
    (perm_out, perm_in, history) as numpy arrays (int32, int32, int64)."""
    import numpy as np
    import torch
    assert S.is_cuda and S.dtype == torch.float32 and S.dim() == 2 and S.stride(1) == 1
    out, inn = S.shape
    ws = _ps_workspace(S, V, M, N)
    po, pi = np.empty(out, dtype=np.int32), np.empty(inn, dtype=np.int32)
    hist = np.zeros(1 + 2 * iterations, dtype=np.int64)
    _check(load_library().vnm_permutation_search(_ptr(S), out, inn, S.stride(0), V, N, M, float(scale), iterations,
                                                 po.ctypes.data, pi.ctypes.data, hist.ctypes.data, _ptr(ws),
                                                 ws.numel(), _stream(S)), "vnm_permutation_search")
    return po, pi, hist


def vnm_permutation_gain(S, V: int, M: int, scale: float, which: int, slot: int, perm_out=None, perm_in=None,
                         N: int = 2):
    """One gain matrix of the search (which: 0 input half-step, 1 output half-step); int64 numpy."""
    import numpy as np
    out, inn = S.shape
    ws = _ps_workspace(S, V, M, N)
    n = inn // M if which == 0 else out // V
    gain = np.zeros((n, n), dtype=np.int64)
    po, po_p = _host_perm(perm_out, out)
    pi, pi_p = _host_perm(perm_in, inn)
    _check(load_library().vnm_permutation_gain(_ptr(S), out, inn, S.stride(0), V, N, M, float(scale), which, slot,
                                               po_p, pi_p, gain.ctypes.data, _ptr(ws), ws.numel(), _stream(S)),
           "vnm_permutation_gain")
    return gain


def vnm_retained_score(S, V: int, M: int, scale: float, perm_out=None, perm_in=None, N: int = 2) -> int:
    """Objective of Eq. 7 at the given permutations (host int arrays or None)."""
    out, inn = S.shape
    ws = _ps_workspace(S, V, M, N)
    po, po_p = _host_perm(perm_out, out)
    pi, pi_p = _host_perm(perm_in, inn)
    tot = ctypes.c_int64(0)
    _check(load_library().vnm_retained_score(_ptr(S), out, inn, S.stride(0), V, N, M, float(scale), po_p, pi_p,
                                             ctypes.byref(tot), _ptr(ws), ws.numel(), _stream(S)),
           "vnm_retained_score")
    return tot.value


def vnm_lora_merge(W, B, A, scale: float, W_merged=None):
    """fp16(W + scale * B A) in the library's fixed fp32 order; W fp16 [out x in], B fp32 [out x r],
    A fp32 [r x in] (CUDA tensors)."""
    import torch
    assert W.is_cuda and W.dtype == torch.float16 and W.dim() == 2 and W.stride(1) == 1
    out, inn = W.shape
    r = B.shape[1]
    assert B.dtype == torch.float32 and A.dtype == torch.float32 and B.shape == (out, r) and A.shape == (r, inn)
    assert (r == 0) or (B.stride(1) == 1 and A.stride(1) == 1)
    if W_merged is None:
        W_merged = torch.empty_like(W)
    _check(load_library().vnm_lora_merge(_ptr(W), out, inn, W.stride(0), _ptr(B), B.stride(0) if r else 0, _ptr(A),
                                         A.stride(0) if r else inn, r, float(scale), _ptr(W_merged),
                                         W_merged.stride(0), _stream(W)), "vnm_lora_merge")
    return W_merged


def vnm_refresh_mask(W, B, A, scale: float, V: int, M: int, act=None, N: int = 2) -> Compressed:
    """Mask update of the LoRA stage with dynamic masks (Section 4.3): merge, score (RIA when `act`
    is given, else |w|), prune.  Returns the Compressed of the merged weight with its mask."""
    merged = vnm_lora_merge(W, B, A, scale)
    if act is None:
        return vnm_prune_compress(merged, V, M, N, want_mask=True)
    return vnm_prune_compress_scored(merged, vnm_ria_scores(merged, act), V, M, N, want_mask=True)


def vnm_stage_x(X, M: int, staged=None):
    """Re-lay X [T x in] for the matrix-core kernel; returns the staged uint8 tensor (reusable by
    every layer with the same `in` and M)."""
    import torch
    assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.stride(1) == 1
    T, inn = X.shape
    b = ctypes.c_int64(0)
    _check(load_library().vnm_stage_x_bytes(T, inn, M, ctypes.byref(b)), "vnm_stage_x_bytes")
    if staged is None:
        staged = torch.empty(max(b.value, 1), dtype=torch.uint8, device=X.device)
    _check(load_library().vnm_stage_x(_ptr(X), T, X.stride(0) if T > 0 else inn, inn, M, _ptr(staged),
                                      staged.numel(), _stream(X)), "vnm_stage_x")
    return staged


KERNEL_GENERIC, KERNEL_FEW_TOKENS, KERNEL_RESIDENT, KERNEL_STAGED = 0, 1, 2, 3


def vnm_spmm_kernel_choice(T: int, c: Compressed, workspace_bytes: int, N: int = 2) -> int:
    """Which kernel vnm_spmm runs for T tokens of this layer with a workspace of that size."""
    ch = ctypes.c_int(-1)
    _check(load_library().vnm_spmm_kernel_choice(T, c.out, c.inn, c.V, N, c.M, workspace_bytes, ctypes.byref(ch)),
           "vnm_spmm_kernel_choice")
    return ch.value


def vnm_spmm_scratch_bytes(T: int, out: int) -> int:
    b = ctypes.c_int64(0)
    _check(load_library().vnm_spmm_scratch_bytes(T, out, ctypes.byref(b)), "vnm_spmm_scratch_bytes")
    return b.value


def vnm_spmm_staged(staged, T: int, c: Compressed, N: int = 2, out_dtype=None, Y=None, scratch=None):
    """Y [T x out] from activations staged by vnm_stage_x and the packed weight of `c`.
    `scratch`: optional uint8 CUDA tensor for the split-K partial products (small T); by default
    the process-wide scratch tensor is used when vnm_spmm_scratch_bytes(T, out) > 0."""
    import torch
    if Y is None:
        Y = torch.empty((T, c.out), dtype=out_dtype or torch.float16, device=staged.device)
    y_dtype = {torch.float16: 0, torch.float32: 1}[Y.dtype]
    if scratch is None:
        nb = vnm_spmm_scratch_bytes(T, c.out)
        if nb > 0:
            scratch = _workspace((staged.device, "splitk"), nb)
    _check(load_library().vnm_spmm_staged(_ptr(staged), staged.numel(), T, _ptr(c.packed), c.out, c.inn, c.V, N, c.M, _ptr(Y),
                                          Y.stride(0) if T > 0 else c.out, y_dtype, _ptr(scratch),
                                          scratch.numel() if scratch is not None else 0, _stream(staged)),
           "vnm_spmm_staged")
    return Y


def vnm_decompress(c: Compressed, N: int = 2, W_out=None):
    import torch
    if W_out is None:
        W_out = torch.empty((c.out, c.inn), dtype=torch.float16, device=c.values.device)
    _check(load_library().vnm_decompress(_ptr(c.values), _ptr(c.meta), _ptr(c.colidx), c.out, c.inn, c.V, N,
                                         c.M, _ptr(W_out), W_out.stride(0), _stream(c.values)),
           "vnm_decompress")
    return W_out


def vnm_mask_diversity_log(V: int, M: int, N: int = 2) -> float:
    k = ctypes.c_double(0.0)
    _check(load_library().vnm_mask_diversity_log(V, N, M, ctypes.byref(k)), "vnm_mask_diversity_log")
    return k.value


def vnm_select_vm(candidates, threshold: float) -> int:
    """candidates: sequence of (V, M, speedup); returns the index of the selected one or -1."""
    n = len(candidates)
    V = (ctypes.c_int * max(n, 1))(*[int(c[0]) for c in candidates])
    M = (ctypes.c_int * max(n, 1))(*[int(c[1]) for c in candidates])
    sp = (ctypes.c_double * max(n, 1))(*[float(c[2]) for c in candidates])
    sel = ctypes.c_int(-1)
    _check(load_library().vnm_select_vm(V, M, sp, n, float(threshold), ctypes.byref(sel)), "vnm_select_vm")
    return sel.value
