"""ctypes binding of libvenom.so: argument marshalling only.

Every step of the path (compression, packing, the product) runs in the library's HIP kernels;
PyTorch supplies device memory and streams.  There is no CPU fallback: if the shared library has
not been built, `lib()` raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_int, c_int64, c_size_t, c_void_p

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libvenom.so")

VENOM_OK = 0
STATUS_NAMES = {
    0: "VENOM_OK", 1: "VENOM_ERR_INVALID_ARG", 2: "VENOM_ERR_SHAPE", 3: "VENOM_ERR_UNSUPPORTED",
    4: "VENOM_ERR_MASK_COLS", 5: "VENOM_ERR_MASK_ROW", 6: "VENOM_ERR_WORKSPACE", 7: "VENOM_ERR_HIP",
}
(VENOM_ERR_INVALID_ARG, VENOM_ERR_SHAPE, VENOM_ERR_UNSUPPORTED, VENOM_ERR_MASK_COLS, VENOM_ERR_MASK_ROW,
 VENOM_ERR_WORKSPACE, VENOM_ERR_HIP) = range(1, 8)

# every symbol include/venom.h declares
EXPORTS = ("venom_workspace_bytes", "venom_prune", "venom_compress", "venom_import", "venom_export", "venom_decompress",
           "venom_spmm", "venom_spmm_variant", "venom_spmm_bias_act", "venom_linear_scratch_bytes", "venom_linear",
           "venom_linear_static_max_bytes", "venom_linear_static", "venom_energy", "venom_probe_smfmac_rate",
           "venom_spmm_variant_count", "venom_spmm_variant_name",
           "venom_get_info", "venom_destroy", "venom_status_string")


class Violation(ctypes.Structure):
    _fields_ = [("block_row", c_int64), ("group", c_int64), ("row", c_int64)]


class VenomError(RuntimeError):
    def __init__(self, status, where, violation=None):
        self.status = status
        self.violation = violation
        msg = f"{where}: {STATUS_NAMES.get(status, status)}"
        if violation is not None:
            msg += f" at (block_row, group, row)={violation}"
        super().__init__(msg)


_lib = None


def lib() -> ctypes.CDLL:
    """Loads the HIP library; raises if it is missing (there is no other implementation)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: build it first (python -m paper_2310_02065_amd.build)")
    L = ctypes.CDLL(LIB_PATH)
    L.venom_workspace_bytes.argtypes = [c_int64, c_int64, c_int, c_int, c_int, POINTER(c_size_t)]
    L.venom_compress.argtypes = [c_void_p, c_int64, c_void_p, c_int64, c_int64, c_int64, c_int, c_int, c_int,
                                 c_void_p, c_size_t, c_void_p, POINTER(c_void_p), POINTER(Violation)]
    L.venom_prune.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_int, c_int, c_int, c_void_p, c_int64, c_void_p,
                              c_void_p, c_void_p]
    L.venom_import.argtypes = [c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int, c_int, c_int, c_void_p,
                               c_size_t, c_void_p, POINTER(c_void_p)]
    L.venom_export.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    L.venom_decompress.argtypes = [c_void_p, c_void_p, c_int64, c_void_p]
    L.venom_spmm.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_void_p, c_int64, c_int, c_void_p]
    L.venom_spmm_variant.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_void_p, c_int64, c_int, c_int, c_void_p]
    L.venom_spmm_bias_act.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_void_p, c_int, c_void_p, c_int64, c_int,
                                      c_int, c_void_p]
    L.venom_linear_scratch_bytes.argtypes = [c_void_p, c_int64, POINTER(c_size_t)]
    L.venom_linear.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_void_p, c_int, c_void_p, c_int64, c_int, c_void_p,
                               c_size_t, c_void_p]
    L.venom_linear_static_max_bytes.argtypes = []
    L.venom_linear_static_max_bytes.restype = c_size_t
    L.venom_linear_static.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_void_p, c_int, c_void_p, c_int64, c_int,
                                      c_void_p]
    L.venom_energy.argtypes = [c_void_p, c_void_p, c_int64, POINTER(ctypes.c_double), c_void_p]
    L.venom_probe_smfmac_rate.argtypes = [c_int, c_void_p, c_void_p]
    L.venom_spmm_variant_count.argtypes = []
    L.venom_spmm_variant_name.argtypes = [c_int]
    L.venom_spmm_variant_name.restype = c_char_p
    L.venom_get_info.argtypes = [c_void_p, POINTER(c_int64), POINTER(c_int64), POINTER(c_int), POINTER(c_int),
                                 POINTER(c_int)]
    L.venom_destroy.argtypes = [c_void_p]
    L.venom_destroy.restype = None
    L.venom_status_string.argtypes = [c_int]
    L.venom_status_string.restype = c_char_p
    for name in ("venom_workspace_bytes", "venom_prune", "venom_compress", "venom_import", "venom_export", "venom_decompress",
                 "venom_spmm", "venom_spmm_variant", "venom_spmm_bias_act", "venom_linear_scratch_bytes", "venom_linear",
                 "venom_linear_static", "venom_energy", "venom_probe_smfmac_rate", "venom_spmm_variant_count", "venom_get_info"):
        getattr(L, name).restype = c_int
    _lib = L
    return L


def _stream_ptr(stream=None):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return c_void_p(s.cuda_stream)


def _ptr(t):
    return c_void_p(t.data_ptr()) if t is not None else c_void_p(0)


def venom_workspace_bytes(R, K, V, N, M) -> int:
    n = c_size_t(0)
    st = lib().venom_workspace_bytes(R, K, V, N, M, byref(n))
    if st != VENOM_OK:
        raise VenomError(st, "venom_workspace_bytes")
    return n.value


class Handle:
    """Owns the workspace tensor and the host-side handle of one compressed matrix."""

    def __init__(self, ptr, workspace, R, K, V, N, M):
        self.ptr, self.workspace = ptr, workspace
        self.R, self.K, self.V, self.N, self.M = R, K, V, N, M

    @property
    def G(self):
        return self.K // self.M

    def close(self):
        if self.ptr:
            lib().venom_destroy(self.ptr)
            self.ptr = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _workspace(R, K, V, N, M, device):
    import torch
    nbytes = venom_workspace_bytes(R, K, V, N, M)
    ws = torch.empty(max(nbytes, 256) + 256, dtype=torch.uint8, device=device)
    off = (-ws.data_ptr()) % 256
    return ws, ws[off:off + max(nbytes, 256)], nbytes


def venom_compress(A, mask, V, N, M, stream=None) -> Handle:
    """A: R x K float16 CUDA tensor (row stride lda), mask: R x K uint8 CUDA tensor."""
    import torch
    assert A.is_cuda and mask.is_cuda and A.dtype == torch.float16 and mask.dtype in (torch.uint8, torch.bool)
    assert A.dim() == 2 and mask.shape == A.shape and A.stride(1) == 1 and mask.stride(1) == 1
    R, K = A.shape
    ws_owner, ws, nbytes = _workspace(R, K, V, N, M, A.device)
    out = c_void_p(0)
    viol = Violation(-1, -1, -1)
    st = lib().venom_compress(_ptr(A), A.stride(0) if R > 1 else max(K, A.stride(0)), _ptr(mask),
                              mask.stride(0) if R > 1 else max(K, mask.stride(0)), R, K, V, N, M, _ptr(ws), nbytes,
                              _stream_ptr(stream), byref(out), byref(viol))
    if st != VENOM_OK:
        v = (viol.block_row, viol.group, viol.row) if st in (VENOM_ERR_MASK_COLS, VENOM_ERR_MASK_ROW) else None
        raise VenomError(st, "venom_compress", v)
    h = Handle(out, ws, R, K, V, N, M)
    h._owner = ws_owner
    return h


def venom_prune(A, V, N, M, stream=None):
    """Magnitude pruning of A (R x K float16 CUDA tensor) to V:N:M.  Returns (mask uint8 R x K,
    kept_mass int64 [R/V], total_mass int64 [R/V]); the masses are exact integers in units of 2^-24."""
    import torch
    assert A.is_cuda and A.dtype == torch.float16 and A.dim() == 2 and A.stride(1) == 1
    R, K = A.shape
    mask = torch.empty((R, K), dtype=torch.uint8, device=A.device)
    nb = max(R // V, 1) if V > 0 else 1
    kept = torch.empty(nb, dtype=torch.int64, device=A.device)
    total = torch.empty(nb, dtype=torch.int64, device=A.device)
    st = lib().venom_prune(_ptr(A), A.stride(0) if R > 1 else max(K, A.stride(0)), R, K, V, N, M, _ptr(mask), K,
                           _ptr(kept), _ptr(total), _stream_ptr(stream))
    if st != VENOM_OK:
        raise VenomError(st, "venom_prune")
    return mask, kept, total


def venom_energy(kept_mass, total_mass, stream=None) -> float:
    """The energy metric from the per-block-row masses venom_prune returns."""
    e = ctypes.c_double(0.0)
    st = lib().venom_energy(_ptr(kept_mass), _ptr(total_mass), kept_mass.numel(), byref(e), _stream_ptr(stream))
    if st != VENOM_OK:
        raise VenomError(st, "venom_energy")
    return e.value


def venom_probe_smfmac_rate(iterations, sink, stream=None):
    """Launches the register-only matrix-instruction loop (the caller times it)."""
    st = lib().venom_probe_smfmac_rate(iterations, _ptr(sink), _stream_ptr(stream))
    if st != VENOM_OK:
        raise VenomError(st, "venom_probe_smfmac_rate")


def venom_import(values, columns, meta, R, K, V, N, M, stream=None) -> Handle:
    ws_owner, ws, nbytes = _workspace(R, K, V, N, M, values.device)
    out = c_void_p(0)
    st = lib().venom_import(_ptr(values), _ptr(columns), _ptr(meta), R, K, V, N, M, _ptr(ws), nbytes,
                            _stream_ptr(stream), byref(out))
    if st != VENOM_OK:
        raise VenomError(st, "venom_import")
    h = Handle(out, ws, R, K, V, N, M)
    h._owner = ws_owner
    return h


def venom_export(h: Handle, stream=None):
    """Returns (values int16 [R,G,2], columns int16 [R/V,G,4], meta int32 [R,ceil(G/8)]) CUDA tensors
    holding the canonical uint16 / uint32 bit patterns."""
    import torch
    G = h.G
    dev = h.workspace.device
    values = torch.empty((h.R, G, 2), dtype=torch.int16, device=dev)
    columns = torch.empty((h.R // h.V, G, 4), dtype=torch.int16, device=dev)
    meta = torch.empty((h.R, (G + 7) // 8), dtype=torch.int32, device=dev)
    st = lib().venom_export(h.ptr, _ptr(values), _ptr(columns), _ptr(meta), _stream_ptr(stream))
    if st != VENOM_OK:
        raise VenomError(st, "venom_export")
    return values, columns, meta


def venom_decompress(h: Handle, out=None, stream=None):
    import torch
    if out is None:
        out = torch.empty((h.R, h.K), dtype=torch.float16, device=h.workspace.device)
    st = lib().venom_decompress(h.ptr, _ptr(out), out.stride(0) if h.R > 1 else max(h.K, out.stride(0)),
                                _stream_ptr(stream))
    if st != VENOM_OK:
        raise VenomError(st, "venom_decompress")
    return out


ACTIVATIONS = {"none": 0, "gelu": 1, "gelu_tanh": 2}


def venom_spmm(h: Handle, B, out=None, out_dtype=None, variant=-1, stream=None, bias=None, activation="none"):
    """C = act(A . B + bias[:, None]).  B: K x C float16 CUDA tensor (unit column stride);
    bias: float16 CUDA vector of R entries or None; returns/fills C (R x C)."""
    import torch
    assert B.is_cuda and B.dtype == torch.float16 and B.dim() == 2 and B.stride(1) == 1
    Ccols = B.shape[1]
    if out is None:
        out = torch.empty((h.R, Ccols), dtype=out_dtype or torch.float16, device=B.device)
    assert out.dtype in (torch.float16, torch.float32) and out.stride(1) == 1
    c_dtype = 1 if out.dtype == torch.float32 else 0
    ldb = B.stride(0) if B.shape[0] > 1 else max(Ccols, B.stride(0))
    ldc = out.stride(0) if out.shape[0] > 1 else max(Ccols, out.stride(0))
    if bias is not None:
        assert bias.is_cuda and bias.dtype == torch.float16 and bias.dim() == 1 and bias.shape[0] == h.R
        assert bias.stride(0) == 1
    st = lib().venom_spmm_bias_act(h.ptr, _ptr(B), ldb, Ccols, _ptr(bias), ACTIVATIONS[activation], _ptr(out), ldc,
                                   c_dtype, variant, _stream_ptr(stream))
    if st != VENOM_OK:
        raise VenomError(st, "venom_spmm")
    return out


def venom_linear(h: Handle, X, bias=None, activation="none", out=None, out_dtype=None, scratch=None, stream=None):
    """Y = act(X . A^T + bias): X tokens x K float16 CUDA tensor, Y tokens x R (token-major in and out).
    `scratch` (uint8 CUDA tensor) receives X transposed; allocated here when not given."""
    import torch
    assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.stride(1) == 1 and X.shape[1] == h.K
    tokens = X.shape[0]
    if out is None:
        out = torch.empty((tokens, h.R), dtype=out_dtype or torch.float16, device=X.device)
    assert out.dtype in (torch.float16, torch.float32) and out.stride(1) == 1 and out.shape == (tokens, h.R)
    need = c_size_t(0)
    st = lib().venom_linear_scratch_bytes(h.ptr, tokens, byref(need))
    if st != VENOM_OK:
        raise VenomError(st, "venom_linear_scratch_bytes")
    if scratch is None:
        scratch = torch.empty(max(need.value, 16), dtype=torch.uint8, device=X.device)
    if bias is not None:
        assert bias.is_cuda and bias.dtype == torch.float16 and bias.dim() == 1 and bias.shape[0] == h.R
    ldx = X.stride(0) if tokens > 1 else max(h.K, X.stride(0))
    ldy = out.stride(0) if tokens > 1 else max(h.R, out.stride(0))
    st = lib().venom_linear(h.ptr, _ptr(X), ldx, tokens, _ptr(bias), ACTIVATIONS[activation], _ptr(out), ldy,
                            1 if out.dtype == torch.float32 else 0, _ptr(scratch), scratch.numel(), _stream_ptr(stream))
    if st != VENOM_OK:
        raise VenomError(st, "venom_linear")
    return out


def venom_linear_static_max_bytes() -> int:
    return lib().venom_linear_static_max_bytes()


def venom_linear_static(h: Handle, X, out, bias=None, activation="none", stream=None):
    """venom_linear with the library's own static scratch: the caller passes the input and the output,
    nothing is allocated here or in the library."""
    import torch
    assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.stride(1) == 1 and X.shape[1] == h.K
    tokens = X.shape[0]
    assert out.dtype in (torch.float16, torch.float32) and out.stride(1) == 1 and out.shape == (tokens, h.R)
    ldx = X.stride(0) if tokens > 1 else max(h.K, X.stride(0))
    ldy = out.stride(0) if tokens > 1 else max(h.R, out.stride(0))
    st = lib().venom_linear_static(h.ptr, _ptr(X), ldx, tokens, _ptr(bias), ACTIVATIONS[activation], _ptr(out), ldy,
                                   1 if out.dtype == torch.float32 else 0, _stream_ptr(stream))
    if st != VENOM_OK:
        raise VenomError(st, "venom_linear_static")
    return out


class Spmm:
    """The layer object of the paper's end-to-end section (its module listing): built once from a
    dense weight, a mask and a bias, it holds the compressed handle and is called like the linear
    layer it replaces, `y = layer(x)` with x tokens x K and y tokens x R.  Holds state only; every
    call is one venom_linear (the scratch for the transposed activations is kept between calls)."""

    def __init__(self, weight, mask, bias=None, V=128, N=2, M=8, activation="none"):
        self.handle = venom_compress(weight, mask, V, N, M)
        self.bias = bias
        self.activation = activation
        self._scratch = None

    @classmethod
    def from_dense(cls, weight, bias=None, V=128, N=2, M=8, activation="none"):
        """Magnitude-prunes `weight` to V:N:M on the GPU (venom_prune), then compresses it."""
        mask, _, _ = venom_prune(weight, V, N, M)
        return cls(weight, mask, bias, V, N, M, activation)

    def __call__(self, x, out=None, out_dtype=None, stream=None):
        import torch
        need = c_size_t(0)
        st = lib().venom_linear_scratch_bytes(self.handle.ptr, x.shape[0], byref(need))
        if st != VENOM_OK:
            raise VenomError(st, "venom_linear_scratch_bytes")
        if self._scratch is None or self._scratch.numel() < need.value or self._scratch.device != x.device:
            self._scratch = torch.empty(max(need.value, 16), dtype=torch.uint8, device=x.device)
        return venom_linear(self.handle, x, self.bias, self.activation, out, out_dtype, self._scratch, stream)


def venom_get_info(h: Handle):
    R, K = c_int64(), c_int64()
    V, N, M = c_int(), c_int(), c_int()
    st = lib().venom_get_info(h.ptr, byref(R), byref(K), byref(V), byref(N), byref(M))
    if st != VENOM_OK:
        raise VenomError(st, "venom_get_info")
    return R.value, K.value, V.value, N.value, M.value


def venom_spmm_variants():
    L = lib()
    return [L.venom_spmm_variant_name(i).decode() for i in range(L.venom_spmm_variant_count())]


def venom_status_string(status: int) -> str:
    return lib().venom_status_string(status).decode()
