"""ctypes binding of the C-ABI library (include/he.h; the test hooks of include/he_test.h).  Argument marshalling only: every step
runs in the library's kernels.  Device tensors are torch int64 tensors whose bit patterns are the
uint64 residues; torch supplies memory and the current stream, nothing else.

The library is loaded from paper_1908_04172_amd/libhe_mi355x.so (built by build.py); if it is
missing or fails to load, importing the symbols raises -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

RATE_MAD32, RATE_MAC_TERM, RATE_SHOUP_EXACT, RATE_SHOUP_CHEAP = 0, 1, 2, 3
RATE_BUTTERFLY_MODE0, RATE_BUTTERFLY_MODE1, RATE_BUTTERFLY_MODE2, RATE_BUTTERFLY_INV = 4, 5, 6, 7
RATE_MAC_TERM3 = 8
RATE_BUTTERFLY_FP64, RATE_BUTTERFLY_FP64_INV = 9, 10
PT_SCALAR = 0
PT_POLY = 1
RESCALE = 1
ACCUMULATE = 2
STATIC_SCRATCH_BYTES = 32 << 20

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhe_mi355x.so")

EXPORTS = [
    "he_strerror", "he_ctx_create", "he_ctx_destroy", "he_ctx_info", "he_encode_scalar", "he_encode_scalar_host",
    "he_encode_vector", "he_decode_vector",
    "he_plan_create", "he_plan_destroy", "he_plan_workspace_bytes", "he_ct_pt_mac", "he_ct_pt_mac_static", "he_ct_pt_add", "he_rescale",
    "he_ntt_fwd", "he_ntt_inv", "he_check_reduced", "he_host_mulmod", "he_host_reduce128", "he_host_shoup_mulmod", "he_host_shoup_lazy",
    "he_host_mac_accumulate", "he_host_mac_accumulate_add", "he_host_mac_accumulate_lazy", "he_test_mac_for_rescale", "he_measure_rate",
    "he_host_barrett64", "he_host_shoup32", "he_host_mac_three_product_terms", "he_host_mac_accumulate_three_products", "he_host_ntt_forward_fp64", "he_host_ntt_inverse_fp64", "he_test_integer_transforms", "he_square_relin_workspace_bytes", "he_ct_square_relin", "he_pack32", "he_unpack32", "he_ct_pt_mac32", "he_ct_pt_add32", "he_rescale32", "he_ntt_fwd32", "he_ntt_inv32",
]

_lib = None


class HeError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {lib().he_strerror(status).decode()} ({status})")


def lib():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_1908_04172_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    vp, u32, u64, i32, dbl, sz = (ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int, ctypes.c_double,
                                  ctypes.c_size_t)
    pp = ctypes.POINTER(vp)
    sigs = {
        "he_strerror": (ctypes.c_char_p, [i32]),
        "he_ctx_create": (i32, [pp, u32, u32, vp, i32]),
        "he_ctx_destroy": (i32, [vp]),
        "he_ctx_info": (i32, [vp, vp, vp, vp, vp]),
        "he_encode_scalar": (i32, [vp, vp, sz, dbl, u32, vp, vp]),
        "he_encode_scalar_host": (i32, [vp, vp, sz, dbl, u32, vp]),
        "he_encode_vector": (i32, [vp, vp, sz, dbl, u32, vp, vp]),
        "he_decode_vector": (i32, [vp, vp, sz, dbl, u32, vp, vp, sz, vp]),
        "he_plan_create": (i32, [vp, u32, u32, u32, vp, vp, vp, pp]),
        "he_plan_destroy": (i32, [vp]),
        "he_plan_workspace_bytes": (i32, [vp, u32, i32, u32, ctypes.POINTER(sz)]),
        "he_ct_pt_mac": (i32, [vp, vp, u32, vp, vp, i32, vp, vp, u32, vp, sz, vp]),
        "he_ct_pt_mac_static": (i32, [vp, vp, u32, vp, vp, i32, vp, vp, u32, vp]),
        "he_ct_pt_add": (i32, [vp, u32, vp, u32, vp, i32, vp]),
        "he_rescale": (i32, [vp, u32, vp, vp, u32, vp]),
        "he_ntt_fwd": (i32, [vp, u32, vp, u32, vp]),
        "he_ntt_inv": (i32, [vp, u32, vp, u32, vp]),
        "he_check_reduced": (i32, [vp, u32, vp, sz, u32, ctypes.POINTER(u64), vp]),
        "he_host_mulmod": (u64, [u64, u64, u64]),
        "he_host_reduce128": (u64, [u64, u64, u64]),
        "he_host_shoup_mulmod": (u64, [u64, u64, u64]),
        "he_host_shoup_lazy": (u64, [u64, u64, u64, ctypes.c_int]),
        "he_host_mac_accumulate_add": (u64, [vp, vp, sz, u64, u64]),
        "he_measure_rate": (i32, [vp, i32, u32, u32, ctypes.POINTER(ctypes.c_double)]),
        "he_host_mac_accumulate_lazy": (u64, [vp, vp, sz, u64, u64]),
        "he_test_mac_for_rescale": (i32, [vp, vp, u32, vp, vp, i32, vp, vp, vp, sz, vp]),
        "he_host_mac_accumulate": (u64, [vp, vp, sz, u64]),
        "he_square_relin_workspace_bytes": (i32, [vp, u32, u32, ctypes.POINTER(sz)]),
        "he_ct_square_relin": (i32, [vp, u32, vp, u32, vp, vp, vp, sz, vp]),
        "he_host_mac_three_product_terms": (u32, [u64]),
        "he_host_mac_accumulate_three_products": (u64, [vp, vp, sz, u64, u64]),
        "he_host_ntt_forward_fp64": (i32, [vp, u32, vp, vp, ctypes.POINTER(ctypes.c_double)]),
        "he_host_ntt_inverse_fp64": (i32, [vp, u32, vp, vp, ctypes.POINTER(ctypes.c_double)]),
        "he_test_integer_transforms": (i32, [vp, i32]),
        "he_host_barrett64": (u32, [u64, u32]),
        "he_host_shoup32": (u32, [u32, u32, u32]),
        "he_pack32": (i32, [vp, vp, vp, sz, vp]),
        "he_unpack32": (i32, [vp, vp, vp, sz, vp]),
        "he_ct_pt_mac32": (i32, [vp, vp, u32, vp, vp, i32, vp, vp, u32, vp, sz, vp]),
        "he_ct_pt_add32": (i32, [vp, u32, vp, u32, vp, i32, vp]),
        "he_rescale32": (i32, [vp, u32, vp, vp, u32, vp]),
        "he_ntt_fwd32": (i32, [vp, u32, vp, u32, vp]),
        "he_ntt_inv32": (i32, [vp, u32, vp, u32, vp]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


def _check(status: int, what: str):
    if status != 0:
        raise HeError(status, what)


def _np64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint64)


def _np32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint32)


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _dev_ptr(t, name: str) -> Optional[int]:
    if t is None:
        return None
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous CUDA tensor")
    if t.dtype not in (torch.int64, torch.int32, torch.float64, torch.uint8, torch.complex128):
        raise TypeError(f"{name}: unexpected dtype {t.dtype}")
    return t.data_ptr()


class Context:
    """he_ctx: ring degree N = 2**log2N and the modulus chain; device=None makes a host-only context."""

    def __init__(self, log2N: int, moduli: Sequence[int], device: Optional[int] = 0):
        self.log2N, self.N, self.L = int(log2N), 1 << int(log2N), len(moduli)
        self.moduli = [int(q) for q in moduli]
        self.device = device
        q = _np64(self.moduli)
        h = ctypes.c_void_p()
        _check(lib().he_ctx_create(ctypes.byref(h), self.log2N, self.L, q.ctypes.data, -1 if device is None else device),
               "he_ctx_create")
        self._h = h
        psi = np.zeros(self.L, dtype=np.uint64)
        _check(lib().he_ctx_info(self._h, None, None, None, psi.ctypes.data), "he_ctx_info")
        self.psi = [int(x) for x in psi]

    def close(self):
        if getattr(self, "_h", None):
            lib().he_ctx_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def integer_transforms(self, integer_only: bool) -> None:
        """he_test_integer_transforms: integer butterflies for every limb (True), or the default (False)."""
        _check(lib().he_test_integer_transforms(self._h, int(bool(integer_only))), "he_test_integer_transforms")

    def host_ntt_forward_fp64(self, limb: int, values) -> "tuple[np.ndarray, float]":
        """he_host_ntt_forward_fp64: the double-precision forward transform run on the host.  values: N integers of
        magnitude at most q; returns (canonical residues of the transform, largest |intermediate| / q)."""
        v = np.ascontiguousarray(values, dtype=np.int64)
        assert v.shape == (self.N,)
        out = np.zeros(self.N, dtype=np.uint64)
        worst = ctypes.c_double()
        _check(lib().he_host_ntt_forward_fp64(self._h, limb, v.ctypes.data, out.ctypes.data, ctypes.byref(worst)),
               "he_host_ntt_forward_fp64")
        return out, float(worst.value)

    def host_ntt_inverse_fp64(self, limb: int, values) -> "tuple[np.ndarray, float]":
        """he_host_ntt_inverse_fp64: canonical residues in transform order -> (canonical coefficients, largest
        |intermediate| / q)."""
        v = _np64(values)
        assert v.shape == (self.N,)
        out = np.zeros(self.N, dtype=np.uint64)
        worst = ctypes.c_double()
        _check(lib().he_host_ntt_inverse_fp64(self._h, limb, v.ctypes.data, out.ctypes.data, ctypes.byref(worst)),
               "he_host_ntt_inverse_fp64")
        return out, float(worst.value)

    def measure_rate(self, kind: int, limb: int = 0, iters: int = 4096) -> float:
        """Operations per second of one arithmetic primitive on register-resident data (he_measure_rate)."""
        r = ctypes.c_double()
        _check(lib().he_measure_rate(self._h, kind, limb, iters, ctypes.byref(r)), "he_measure_rate")
        return float(r.value)

    # -- Alg. 2
    def encode_scalar_host(self, values, scale: float, limbs: Optional[int] = None) -> np.ndarray:
        limbs = self.L if limbs is None else limbs
        v = np.ascontiguousarray(np.atleast_1d(values), dtype=np.float64)
        out = np.empty((v.size, limbs), dtype=np.uint64)
        _check(lib().he_encode_scalar_host(self._h, v.ctypes.data, v.size, float(scale), limbs, out.ctypes.data),
               "he_encode_scalar_host")
        return out

    def encode_scalar(self, values, scale: float, limbs: Optional[int] = None, out=None):
        """values: CUDA float64 tensor [n] -> CUDA int64 tensor [n][limbs] (he_encode_scalar)."""
        import torch
        limbs = self.L if limbs is None else limbs
        n = values.numel()
        if out is None:
            out = torch.empty((n, limbs), dtype=torch.int64, device=values.device)
        _check(lib().he_encode_scalar(self._h, _dev_ptr(values, "values"), n, float(scale), limbs, _dev_ptr(out, "out"),
                                      _stream()), "he_encode_scalar")
        return out

    # -- Alg. 1
    def encode_vector(self, slots, scale: float, limbs: Optional[int] = None, out=None):
        """slots: CUDA complex128 tensor [n][N/2] -> CUDA int64 tensor [n][limbs][N], NTT form (he_encode_vector)."""
        import torch
        limbs = self.L if limbs is None else limbs
        assert slots.dtype == torch.complex128 and slots.dim() == 2 and slots.shape[1] == self.N // 2
        n = slots.shape[0]
        if out is None:
            out = torch.empty((n, limbs, self.N), dtype=torch.int64, device=slots.device)
        assert tuple(out.shape) == (n, limbs, self.N)
        _check(lib().he_encode_vector(self._h, _dev_ptr(slots, "slots"), n, float(scale), limbs, _dev_ptr(out, "out"),
                                      _stream()), "he_encode_vector")
        return out

    def decode_vector(self, poly, scale: float, out=None, workspace=None):
        """poly: CUDA int64 tensor [n][limbs][N] (NTT form) -> CUDA complex128 tensor [n][N/2] (he_decode_vector)."""
        import torch
        n, limbs, N = poly.shape
        assert N == self.N
        if out is None:
            out = torch.empty((n, N // 2), dtype=torch.complex128, device=poly.device)
        if workspace is None:
            workspace = torch.empty(max(n * limbs * N * 8, 8), dtype=torch.uint8, device=poly.device)
        _check(lib().he_decode_vector(self._h, _dev_ptr(poly, "poly"), n, float(scale), limbs, _dev_ptr(out, "slots"),
                                      _dev_ptr(workspace, "workspace"), workspace.numel(), _stream()), "he_decode_vector")
        return out

    # -- Alg. 3 / 4
    def ct_pt_add(self, ct, pt, pt_kind: int, limbs: Optional[int] = None):
        limbs = ct.shape[2] if limbs is None else limbs
        n = ct.shape[0]
        assert tuple(ct.shape) == (n, 2, limbs, self.N)
        assert tuple(pt.shape) == ((n, limbs) if pt_kind == PT_SCALAR else (n, limbs, self.N))
        _check(lib().he_ct_pt_add(self._h, limbs, _dev_ptr(ct, "ct"), n, _dev_ptr(pt, "pt"), pt_kind, _stream()),
               "he_ct_pt_add")
        return ct

    # -- Eq. (2)
    def rescale(self, ct, out=None):
        import torch
        n, two, limbs, N = ct.shape
        assert two == 2 and N == self.N
        if out is None:
            out = torch.empty((n, 2, limbs - 1, N), dtype=torch.int64, device=ct.device)
        _check(lib().he_rescale(self._h, limbs, _dev_ptr(ct, "in"), _dev_ptr(out, "out"), n, _stream()), "he_rescale")
        return out

    def check_reduced(self, data, limbs: Optional[int] = None, row_len: Optional[int] = None) -> int:
        """How many residues of data [...][limbs][row_len] are not below their limb's modulus (he_check_reduced;
        waits for the stream).  row_len defaults to N for tensors of rank >= 3, limbs to the size of the limb axis."""
        if row_len is None:
            row_len = self.N if data.dim() >= 3 else 1
        limbs = data.shape[-2 if row_len > 1 else -1] if limbs is None else limbs
        assert data.numel() % (limbs * row_len) == 0
        bad = ctypes.c_uint64()
        _check(lib().he_check_reduced(self._h, limbs, _dev_ptr(data, "data"), data.numel() // (limbs * row_len), row_len,
                                      ctypes.byref(bad), _stream()), "he_check_reduced")
        return int(bad.value)

    # -- NTT
    def ntt_fwd(self, data):
        limbs, N = data.shape[-2:]
        assert N == self.N
        _check(lib().he_ntt_fwd(self._h, limbs, _dev_ptr(data, "data"), data.numel() // (limbs * N), _stream()),
               "he_ntt_fwd")
        return data

    def ntt_inv(self, data):
        limbs, N = data.shape[-2:]
        assert N == self.N
        _check(lib().he_ntt_inv(self._h, limbs, _dev_ptr(data, "data"), data.numel() // (limbs * N), _stream()),
               "he_ntt_inv")
        return data

    # -- Alg. 7 / 8 over a plan
    def plan(self, n_in: int, n_out: int, n_pt: int, off, term_ct, term_pt) -> "Plan":
        return Plan(self, n_in, n_out, n_pt, off, term_ct, term_pt)

    def ct_pt_mac(self, plan: "Plan", ct_in, pt, pt_kind: int, bias=None, flags: int = 0, out=None, workspace=None,
                  limbs: Optional[int] = None):
        import torch
        limbs = ct_in.shape[2] if limbs is None else limbs
        assert tuple(ct_in.shape) == (plan.n_in, 2, limbs, self.N)
        assert tuple(pt.shape) == ((plan.n_pt, limbs) if pt_kind == PT_SCALAR else (plan.n_pt, limbs, self.N))
        if bias is not None:
            assert tuple(bias.shape) == (plan.n_out, limbs)
        out_limbs = limbs - 1 if flags & RESCALE else limbs
        if out is None:
            assert not flags & ACCUMULATE, "HE_ACCUMULATE adds to an output the caller provides"
            out = torch.empty((plan.n_out, 2, out_limbs, self.N), dtype=torch.int64, device=ct_in.device)
        assert tuple(out.shape) == (plan.n_out, 2, out_limbs, self.N)
        need = plan.workspace_bytes(limbs, pt_kind, flags)
        if workspace is None and need:
            workspace = torch.empty(need, dtype=torch.uint8, device=ct_in.device)
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        _check(lib().he_ct_pt_mac(self._h, plan._h, limbs, _dev_ptr(ct_in, "ct_in"), _dev_ptr(pt, "pt"), pt_kind,
                                  _dev_ptr(bias, "bias"), _dev_ptr(out, "ct_out"), flags, _dev_ptr(workspace, "workspace"),
                                  ws_bytes, _stream()), "he_ct_pt_mac")
        return out


    def mac_for_rescale(self, plan: "Plan", ct_in, pt, pt_kind: int, out, bias=None, workspace=None):
        """he_test_mac_for_rescale: the accumulators of a fused layer, as its rescale kernel receives them."""
        import torch
        limbs = ct_in.shape[2]
        assert tuple(out.shape) == (plan.n_out, 2, limbs, self.N)
        need = plan.workspace_bytes(limbs, pt_kind, 0)
        if workspace is None and need:
            workspace = torch.empty(need, dtype=torch.uint8, device=ct_in.device)
        _check(lib().he_test_mac_for_rescale(self._h, plan._h, limbs, _dev_ptr(ct_in, "ct_in"), _dev_ptr(pt, "pt"), pt_kind,
                                             _dev_ptr(bias, "bias"), _dev_ptr(out, "acc_out"), _dev_ptr(workspace, "workspace"),
                                             0 if workspace is None else workspace.numel(), _stream()), "he_test_mac_for_rescale")
        return out

    def ct_pt_mac_static(self, plan: "Plan", ct_in, pt, pt_kind: int, out, bias=None, flags: int = 0):
        """he_ct_pt_mac_static: the same operation on the library's fixed scratch array; the caller brings the output."""
        limbs = ct_in.shape[2]
        assert tuple(ct_in.shape) == (plan.n_in, 2, limbs, self.N)
        assert tuple(pt.shape) == ((plan.n_pt, limbs) if pt_kind == PT_SCALAR else (plan.n_pt, limbs, self.N))
        assert bias is None or tuple(bias.shape) == (plan.n_out, limbs)
        assert tuple(out.shape) == (plan.n_out, 2, limbs - 1 if flags & RESCALE else limbs, self.N)
        _check(lib().he_ct_pt_mac_static(self._h, plan._h, limbs, _dev_ptr(ct_in, "ct_in"), _dev_ptr(pt, "pt"), pt_kind,
                                         _dev_ptr(bias, "bias"), _dev_ptr(out, "ct_out"), flags, _stream()), "he_ct_pt_mac_static")
        return out

    # -- the x^2 activation: square + relinearise, the context's last limb being the special prime
    def square_relin_workspace_bytes(self, limbs: int, n: int) -> int:
        b = ctypes.c_size_t()
        _check(lib().he_square_relin_workspace_bytes(self._h, limbs, n, ctypes.byref(b)), "he_square_relin_workspace_bytes")
        return b.value

    def ct_square_relin(self, ct, evk, out=None, workspace=None):
        """ct [n][2][limbs][N] at any level limbs <= L-1; evk [L-1][2][L][N], the top-level key."""
        import torch
        n, two, l, N = ct.shape
        assert two == 2 and N == self.N
        assert tuple(evk.shape) == (self.L - 1, 2, self.L, N)
        if out is None:
            out = torch.empty_like(ct)
        need = self.square_relin_workspace_bytes(l, n)
        if workspace is None:
            workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=ct.device)
        _check(lib().he_ct_square_relin(self._h, l, _dev_ptr(ct, "ct_in"), n, _dev_ptr(evk, "evk"), _dev_ptr(out, "ct_out"),
                                        _dev_ptr(workspace, "workspace"), workspace.numel(), _stream()), "he_ct_square_relin")
        return out

    # -- packed 32-bit storage (moduli below 2^30): int32 tensors whose bit patterns are the uint32 residues
    def pack32(self, t):
        import torch
        assert t.dtype == torch.int64
        out = torch.empty(t.shape, dtype=torch.int32, device=t.device)
        _check(lib().he_pack32(self._h, _dev_ptr(t, "in"), _dev_ptr(out, "out"), t.numel(), _stream()), "he_pack32")
        return out

    def unpack32(self, t):
        import torch
        assert t.dtype == torch.int32
        out = torch.empty(t.shape, dtype=torch.int64, device=t.device)
        _check(lib().he_unpack32(self._h, _dev_ptr(t, "in"), _dev_ptr(out, "out"), t.numel(), _stream()), "he_unpack32")
        return out

    def ct_pt_mac32(self, plan: "Plan", ct_in, pt, pt_kind: int, bias=None, flags: int = 0, out=None, workspace=None):
        import torch
        limbs = ct_in.shape[2]
        assert ct_in.dtype == torch.int32 and tuple(ct_in.shape) == (plan.n_in, 2, limbs, self.N)
        if pt_kind == PT_SCALAR:
            assert pt.dtype == torch.int64 and tuple(pt.shape) == (plan.n_pt, limbs)
        else:
            assert pt.dtype == torch.int32 and tuple(pt.shape) == (plan.n_pt, limbs, self.N)
        if bias is not None:
            assert bias.dtype == torch.int64 and tuple(bias.shape) == (plan.n_out, limbs)
        out_limbs = limbs - 1 if flags & RESCALE else limbs
        if out is None:
            assert not flags & ACCUMULATE, "HE_ACCUMULATE adds to an output the caller provides"
            out = torch.empty((plan.n_out, 2, out_limbs, self.N), dtype=torch.int32, device=ct_in.device)
        assert out.dtype == torch.int32 and tuple(out.shape) == (plan.n_out, 2, out_limbs, self.N)
        need = plan.workspace_bytes(limbs, pt_kind, flags)
        if workspace is None and need:
            workspace = torch.empty(need, dtype=torch.uint8, device=ct_in.device)
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        _check(lib().he_ct_pt_mac32(self._h, plan._h, limbs, _dev_ptr(ct_in, "ct_in"), _dev_ptr(pt, "pt"), pt_kind,
                                    _dev_ptr(bias, "bias"), _dev_ptr(out, "ct_out"), flags, _dev_ptr(workspace, "workspace"),
                                    ws_bytes, _stream()), "he_ct_pt_mac32")
        return out

    def ct_pt_add32(self, ct, pt, pt_kind: int):
        import torch
        n, two, limbs, N = ct.shape
        assert ct.dtype == torch.int32 and two == 2 and N == self.N
        if pt_kind == PT_SCALAR:
            assert pt.dtype == torch.int64 and tuple(pt.shape) == (n, limbs)
        else:
            assert pt.dtype == torch.int32 and tuple(pt.shape) == (n, limbs, self.N)
        _check(lib().he_ct_pt_add32(self._h, limbs, _dev_ptr(ct, "ct"), n, _dev_ptr(pt, "pt"), pt_kind, _stream()),
               "he_ct_pt_add32")
        return ct

    def rescale32(self, ct, out=None):
        import torch
        n, two, limbs, N = ct.shape
        assert ct.dtype == torch.int32 and two == 2 and N == self.N
        if out is None:
            out = torch.empty((n, 2, limbs - 1, N), dtype=torch.int32, device=ct.device)
        _check(lib().he_rescale32(self._h, limbs, _dev_ptr(ct, "in"), _dev_ptr(out, "out"), n, _stream()), "he_rescale32")
        return out

    def ntt_fwd32(self, data):
        import torch
        limbs, N = data.shape[-2:]
        assert data.dtype == torch.int32 and N == self.N
        _check(lib().he_ntt_fwd32(self._h, limbs, _dev_ptr(data, "data"), data.numel() // (limbs * N), _stream()),
               "he_ntt_fwd32")
        return data

    def ntt_inv32(self, data):
        import torch
        limbs, N = data.shape[-2:]
        assert data.dtype == torch.int32 and N == self.N
        _check(lib().he_ntt_inv32(self._h, limbs, _dev_ptr(data, "data"), data.numel() // (limbs * N), _stream()),
               "he_ntt_inv32")
        return data


class Plan:
    """he_plan: out[o] = sum over t in [off[o], off[o+1]) of ct_in[term_ct[t]] * pt[term_pt[t]]."""

    def __init__(self, ctx: Context, n_in: int, n_out: int, n_pt: int, off, term_ct, term_pt):
        self.ctx, self.n_in, self.n_out, self.n_pt = ctx, int(n_in), int(n_out), int(n_pt)
        off, term_ct, term_pt = _np32(off), _np32(term_ct), _np32(term_pt)
        assert off.size == self.n_out + 1 and term_ct.size == term_pt.size
        h = ctypes.c_void_p()
        _check(lib().he_plan_create(ctx._h, self.n_in, self.n_out, self.n_pt, off.ctypes.data, term_ct.ctypes.data,
                                    term_pt.ctypes.data, ctypes.byref(h)), "he_plan_create")
        self._h = h

    def workspace_bytes(self, limbs: int, pt_kind: int, flags: int) -> int:
        b = ctypes.c_size_t()
        _check(lib().he_plan_workspace_bytes(self._h, limbs, pt_kind, flags, ctypes.byref(b)), "he_plan_workspace_bytes")
        return int(b.value)

    def close(self):
        if getattr(self, "_h", None):
            lib().he_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# -- host-side checks of the device arithmetic

def host_mulmod(a: int, b: int, q: int) -> int:
    return int(lib().he_host_mulmod(a, b, q))


def host_reduce128(hi: int, lo: int, q: int) -> int:
    return int(lib().he_host_reduce128(hi, lo, q))


def host_shoup_mulmod(y: int, w: int, q: int) -> int:
    return int(lib().he_host_shoup_mulmod(y, w, q))


def host_shoup_lazy(y: int, w: int, q: int, cheap_quotient: bool) -> int:
    return int(lib().he_host_shoup_lazy(y, w, q, int(cheap_quotient)))


def host_mac_three_product_terms(q: int) -> int:
    return int(lib().he_host_mac_three_product_terms(q))


def host_mac_accumulate_three_products(x, w, q: int, addend: int = 0) -> int:
    x, w = _np64(x), _np64(w)
    assert x.shape == w.shape and x.ndim == 1
    return int(lib().he_host_mac_accumulate_three_products(x.ctypes.data, w.ctypes.data, x.size, q, addend))


def host_barrett64(z: int, q: int) -> int:
    return int(lib().he_host_barrett64(z, q))


def host_shoup32(y: int, w: int, q: int) -> int:
    return int(lib().he_host_shoup32(y, w, q))


def host_mac_accumulate_lazy(x, w, q: int, addend: int = 0) -> int:
    x, w = _np64(x), _np64(w)
    assert x.size == w.size
    return int(lib().he_host_mac_accumulate_lazy(x.ctypes.data, w.ctypes.data, x.size, q, addend))


def host_mac_accumulate(x, w, q: int, addend: int = 0) -> int:
    x, w = _np64(x), _np64(w)
    assert x.size == w.size
    if addend:
        return int(lib().he_host_mac_accumulate_add(x.ctypes.data, w.ctypes.data, x.size, q, addend))
    return int(lib().he_host_mac_accumulate(x.ctypes.data, w.ctypes.data, x.size, q))
