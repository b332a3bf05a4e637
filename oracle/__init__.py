"""CPU oracle (test infrastructure only) for the RNS-CKKS ct-pt MAC + lazy-rescale path.

NumPy front end of ``he_oracle.c`` (plain C, ``unsigned __int128 %`` arithmetic).  Only tests,
the smoke check and the benchmark's CPU-baseline leg may import this package; the GPU library
never does, and nothing here imports the GPU package.

Tensors are C-contiguous ``numpy.uint64`` arrays shaped ``[ct][2][limbs][N]``; every residue of
limb ``i`` lies in ``[0, q[i])``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

PT_SCALAR = 0
PT_POLY = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "he_oracle.c")
_LIB = os.path.join(_HERE, "libhe_oracle.so")
_lib = None

_u64p = ctypes.POINTER(ctypes.c_uint64)
_u32p = ctypes.POINTER(ctypes.c_uint32)
_dblp = ctypes.POINTER(ctypes.c_double)
_i64p = ctypes.POINTER(ctypes.c_int64)


def build(force: bool = False) -> str:
    """Compile he_oracle.c with gcc -O2 (the optimisation level the paper's evaluation used)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    u64, u32, i32, dbl = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int, ctypes.c_double
    sigs = {
        "orc_mulmod": (u64, [u64, u64, u64]),
        "orc_powmod": (u64, [u64, u64, u64]),
        "orc_invmod": (u64, [u64, u64]),
        "orc_is_prime": (i32, [u64]),
        "orc_find_psi": (u64, [u64, u64]),
        "orc_ntt_fwd_direct": (None, [_u64p, _u64p, u64, u64, u64]),
        "orc_ntt_inv_direct": (None, [_u64p, _u64p, u64, u64, u64]),
        "orc_ntt_fwd_rows": (None, [_u64p, u64, u32, u64, _u64p, _u64p]),
        "orc_ntt_inv_rows": (None, [_u64p, u64, u32, u64, _u64p, _u64p]),
        "orc_encode_scalar": (i32, [dbl, dbl, _u64p, u32, _u64p]),
        "orc_encode_vector_coeffs": (i32, [_dblp, u64, u64, dbl, _i64p]),
        "orc_encode_vector": (i32, [_dblp, u64, u64, dbl, _u64p, _u64p, u32, _u64p]),
        "orc_decode_vector": (None, [_dblp, u64, u64, dbl, _dblp]),
        "orc_add": (None, [_u64p, u64, u32, u64, _u64p, _u64p, i32]),
        "orc_mac": (None, [u64, u32, _u64p, _u64p, _u32p, _u32p, _u32p, u32, _u64p, i32, _u64p, _u64p]),
        "orc_divide_round": (None, [_u64p, _u64p, u64, u32, u64, _u64p]),
        "orc_rescale": (None, [u64, u32, _u64p, _u64p, _u64p, _u64p, u64]),
        "orc_layer": (u32, [u64, u32, _u64p, _u64p, _u64p, _u32p, _u32p, _u32p, u32, _u64p, i32,
                            _u64p, _u64p]),
        "orc_set_threads": (i32, [i32]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _a64(x) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.uint64)


def _a32(x) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.uint32)


def _p64(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_u64p)


def _p32(a: np.ndarray):
    return a.ctypes.data_as(_u32p)


# ----------------------------------------------------------------------------- scalars

def mulmod(a: int, b: int, q: int) -> int:
    return int(_load().orc_mulmod(a, b, q))


def powmod(a: int, e: int, q: int) -> int:
    return int(_load().orc_powmod(a, e, q))


def invmod(a: int, q: int) -> int:
    return int(_load().orc_invmod(a, q))


def is_prime(q: int) -> bool:
    return bool(_load().orc_is_prime(q))


def find_psi(q: int, N: int) -> int:
    """Smallest psi in [2, q) with psi^N = -1 mod q (the root the NTT entry points use)."""
    psi = int(_load().orc_find_psi(q, N))
    if psi == 0:
        raise ValueError(f"no primitive 2N-th root of unity mod {q} for N={N}")
    return psi


def find_psis(q: Sequence[int], N: int) -> list:
    return [find_psi(int(qi), N) for qi in q]


def set_threads(n: int) -> int:
    """Set the OpenMP thread count (0 = leave unchanged); returns the count in effect."""
    return int(_load().orc_set_threads(int(n)))


# ----------------------------------------------------------------------------- NTT

def ntt_fwd_direct(a, q: int, psi: int) -> np.ndarray:
    """O(N^2) definition: out[j] = a(psi^(2*bitrev(j)+1)) mod q."""
    a = _a64(a)
    out = np.empty_like(a)
    _load().orc_ntt_fwd_direct(_p64(a), _p64(out), a.size, q, psi)
    return out


def ntt_inv_direct(x, q: int, psi: int) -> np.ndarray:
    x = _a64(x)
    out = np.empty_like(x)
    _load().orc_ntt_inv_direct(_p64(x), _p64(out), x.size, q, psi)
    return out


def _rows(data, q, psi, fn_name) -> np.ndarray:
    out = _a64(data).copy()
    q = _a64(q)
    psi = _a64(psi)
    limbs = q.size
    N = out.shape[-1]
    rows = out.size // N
    if out.ndim < 2 or out.shape[-2] != limbs or rows % limbs:
        raise ValueError("expected [..., limbs, N]")
    getattr(_load(), fn_name)(_p64(out), rows // limbs, limbs, N, _p64(q), _p64(psi))
    return out


def ntt_fwd(data, q, psi) -> np.ndarray:
    """Forward negacyclic NTT of every row of a [..., limbs, N] array (returns a copy)."""
    return _rows(data, q, psi, "orc_ntt_fwd_rows")


def ntt_inv(data, q, psi) -> np.ndarray:
    return _rows(data, q, psi, "orc_ntt_inv_rows")


# ----------------------------------------------------------------------------- Alg. 2

def encode_scalar(value: float, scale: float, q) -> np.ndarray:
    """Alg. 2: [round(scale*value)]_{q_i} for each limb -> uint64[limbs] (8*limbs bytes)."""
    q = _a64(q)
    out = np.empty(q.size, dtype=np.uint64)
    rc = _load().orc_encode_scalar(float(value), float(scale), _p64(q), q.size, _p64(out))
    if rc != 0:
        raise ValueError("scale*value is not finite")
    return out


def encode_scalars(values, scale: float, q) -> np.ndarray:
    values = np.asarray(values, dtype=np.float64).ravel()
    return np.stack([encode_scalar(v, scale, q) for v in values]) if values.size else \
        np.empty((0, len(q)), dtype=np.uint64)


# ----------------------------------------------------------------------------- Alg. 1

def _slots(z, N: int) -> np.ndarray:
    z = np.ascontiguousarray(np.atleast_2d(np.asarray(z, dtype=np.complex128)))
    assert z.shape[1] == N // 2, "N/2 complex slots per vector"
    return z


def encode_vector_coeffs(z, scale: float, N: int) -> np.ndarray:
    """Alg. 1 before the modular reduction: int64 [n][N] coefficients round(scale * sigma^-1(z))."""
    z = _slots(z, N)
    out = np.empty((z.shape[0], N), dtype=np.int64)
    rc = _load().orc_encode_vector_coeffs(z.view(np.float64).ctypes.data_as(_dblp), z.shape[0], N, float(scale),
                                          out.ctypes.data_as(_i64p))
    if rc != 0:
        raise ValueError("a coefficient is not finite or not below 2^62")
    return out


def encode_vector(z, scale: float, q, psi, N: int) -> np.ndarray:
    """Alg. 1: [n][N/2] complex slots -> uint64 [n][limbs][N] residues in NTT form."""
    z = _slots(z, N)
    q, psi = _a64(q), _a64(psi)
    out = np.empty((z.shape[0], q.size, N), dtype=np.uint64)
    rc = _load().orc_encode_vector(z.view(np.float64).ctypes.data_as(_dblp), z.shape[0], N, float(scale), _p64(q),
                                   _p64(psi), q.size, _p64(out))
    if rc != 0:
        raise ValueError("a coefficient is not finite or not below 2^62")
    return out


def decode_vector(coeffs, scale: float, N: int) -> np.ndarray:
    """Values of the polynomials with the given signed coefficients ([n][N], any numeric type whose
    entries are exactly representable as doubles) at the slot roots, over the scale: complex [n][N/2]."""
    m = np.ascontiguousarray(np.atleast_2d(np.asarray(coeffs, dtype=np.float64)))
    assert m.shape[1] == N
    out = np.empty((m.shape[0], N // 2), dtype=np.complex128)
    _load().orc_decode_vector(m.ctypes.data_as(_dblp), m.shape[0], N, float(scale),
                              out.view(np.float64).ctypes.data_as(_dblp))
    return out


# ----------------------------------------------------------------------------- Alg. 3/4, 7/8

def add(ct, q, pt, pt_kind: int) -> np.ndarray:
    """ct [n][2][limbs][N] + pt ([n][limbs] scalar or [n][limbs][N]) on component 0 (copy)."""
    out = _a64(ct).copy()
    q = _a64(q)
    pt = _a64(pt)
    n, two, limbs, N = out.shape
    assert two == 2 and limbs == q.size
    assert pt.shape == ((n, limbs) if pt_kind == PT_SCALAR else (n, limbs, N))
    _load().orc_add(_p64(out), n, limbs, N, _p64(q), _p64(pt), pt_kind)
    return out


def mac(ct_in, q, off, term_ct, term_pt, pt, pt_kind: int, bias=None) -> np.ndarray:
    """out[o] = sum_t ct_in[term_ct[t]] (*) pt[term_pt[t]] (+ bias[o] on component 0)."""
    ct_in = _a64(ct_in)
    q = _a64(q)
    off, term_ct, term_pt = _a32(off), _a32(term_ct), _a32(term_pt)
    pt = _a64(pt)
    n_in, two, limbs, N = ct_in.shape
    assert two == 2 and limbs == q.size
    n_out = off.size - 1
    assert off[0] == 0 and off[-1] == term_ct.size == term_pt.size
    assert term_ct.size == 0 or int(term_ct.max()) < n_in
    assert term_pt.size == 0 or int(term_pt.max()) < pt.shape[0]
    assert pt.shape[1:] == ((limbs,) if pt_kind == PT_SCALAR else (limbs, N))
    if bias is not None:
        bias = _a64(bias)
        assert bias.shape == (n_out, limbs)
    out = np.empty((n_out, 2, limbs, N), dtype=np.uint64)
    _load().orc_mac(N, limbs, _p64(q), _p64(ct_in), _p32(off), _p32(term_ct), _p32(term_pt), n_out,
                    _p64(pt), pt_kind, _p64(bias), _p64(out))
    return out


# ----------------------------------------------------------------------------- Eq. (2)

def divide_round(coef, q) -> np.ndarray:
    """Coefficient-domain Eq. (2): [..., limbs, N] -> [..., limbs-1, N]."""
    coef = _a64(coef)
    q = _a64(q)
    limbs, N = coef.shape[-2:]
    assert limbs == q.size and limbs >= 2
    n_polys = coef.size // (limbs * N)
    out = np.empty(coef.shape[:-2] + (limbs - 1, N), dtype=np.uint64)
    _load().orc_divide_round(_p64(coef), _p64(out), n_polys, limbs, N, _p64(q))
    return out


def rescale(ct, q, psi) -> np.ndarray:
    """Eq. (2) on NTT-form ciphertexts: [n][2][limbs][N] -> [n][2][limbs-1][N]."""
    ct = _a64(ct)
    q = _a64(q)
    psi = _a64(psi)
    n, two, limbs, N = ct.shape
    assert two == 2 and limbs == q.size == psi.size and limbs >= 2
    out = np.empty((n, 2, limbs - 1, N), dtype=np.uint64)
    _load().orc_rescale(N, limbs, _p64(q), _p64(psi), _p64(ct), _p64(out), n)
    return out


def layer(ct_in, q, psi, off, term_ct, term_pt, pt, pt_kind: int, bias=None):
    """MAC -> bias -> one rescale per output.  Returns (out, number_of_rescales)."""
    ct_in = _a64(ct_in)
    q = _a64(q)
    psi = _a64(psi)
    off, term_ct, term_pt = _a32(off), _a32(term_ct), _a32(term_pt)
    pt = _a64(pt)
    n_in, two, limbs, N = ct_in.shape
    assert two == 2 and limbs == q.size and limbs >= 2
    n_out = off.size - 1
    assert off[0] == 0 and off[-1] == term_ct.size == term_pt.size
    assert term_ct.size == 0 or int(term_ct.max()) < n_in
    assert term_pt.size == 0 or int(term_pt.max()) < pt.shape[0]
    if bias is not None:
        bias = _a64(bias)
        assert bias.shape == (n_out, limbs)
    out = np.empty((n_out, 2, limbs - 1, N), dtype=np.uint64)
    n_rescales = _load().orc_layer(N, limbs, _p64(q), _p64(psi), _p64(ct_in), _p32(off), _p32(term_ct),
                                   _p32(term_pt), n_out, _p64(pt), pt_kind, _p64(bias), _p64(out))
    return out, int(n_rescales)


# ----------------------------------------------------------------------------- ct x ct square, relinearisation
# The x^2 activation (Sec. "CryptoNets"; "Square" and "Relinearize" in the paper's table of operation
# runtimes).  The paper names the method only: relinearisation (key switching) by raising the modulus
# with a special prime (Sec. "Homomorphic Encryption").  Reading taken: the ciphertext lives on limbs
# q_0..q_{l-1}, the special prime P is one more limb; the quadratic component d2 is cut into its l RNS
# digits, digit j = the coefficients of [d2]_{q_j} as integers in [0, q_j), re-reduced modulo every q_i
# and P; the digits are multiplied by the key-switching key (one pair of polynomials modulo Q*P per
# digit) and summed; the sum is divided by P with rounding (Eq. (2) with P as the dropped limb) and added
# to (d0, d1).  Every step below is one of the oracle's own routines or a plain big-integer product.

def _mulmod_rows(a, b, q) -> np.ndarray:
    """Slot-wise product of [..., limbs, N] arrays, limb i modulo q[i] (Python integers)."""
    a, b = _a64(a), _a64(b)
    out = np.empty(a.shape, dtype=np.uint64)
    for i, qi in enumerate(q):
        out[..., i, :] = ((a[..., i, :].astype(object) * b[..., i, :].astype(object)) % int(qi)).astype(np.uint64)
    return out


def square(ct, q) -> np.ndarray:
    """(c0, c1) -> (c0^2, 2 c0 c1, c1^2), NTT form: [n][2][l][N] -> [n][3][l][N]."""
    ct = _a64(ct)
    n, two, l, N = ct.shape
    assert two == 2 and l == len(q)
    out = np.empty((n, 3, l, N), dtype=np.uint64)
    out[:, 0] = _mulmod_rows(ct[:, 0], ct[:, 0], q)
    cross = _mulmod_rows(ct[:, 0], ct[:, 1], q)
    for i, qi in enumerate(q):
        out[:, 1, i] = ((cross[:, i].astype(object) * 2) % int(qi)).astype(np.uint64)
    out[:, 2] = _mulmod_rows(ct[:, 1], ct[:, 1], q)
    return out


def relin_digits(d2, q_all, psi_all) -> np.ndarray:
    """[n][l][N] (NTT form, limbs q_0..q_{l-1}) -> [n][l digits][l+1 limbs][N] (NTT form, limbs q_0..q_{l-1}, P):
    digit j is the polynomial whose coefficients are those of [d2]_{q_j}, taken in [0, q_j)."""
    d2 = _a64(d2)
    n, l, N = d2.shape
    assert len(q_all) == l + 1
    coef = ntt_inv(d2, q_all[:l], psi_all[:l])                  # row j: coefficients modulo q_j
    out = np.empty((n, l, l + 1, N), dtype=np.uint64)
    for j in range(l):
        rows = np.stack([coef[:, j] % np.uint64(qi) for qi in q_all], axis=1)  # [n][l+1][N]
        out[:, j] = ntt_fwd(rows, q_all, psi_all)
    return out


def relinearize(d, q_all, psi_all, evk) -> np.ndarray:
    """(d0, d1, d2) on limbs q_0..q_{l-1} -> (c0', c1') on the same limbs, with the key evk [l][2][l+1][N]
    (NTT form, limbs q_0..q_{l-1}, P)."""
    d = _a64(d)
    evk = _a64(evk)
    n, three, l, N = d.shape
    assert three == 3 and evk.shape == (l, 2, l + 1, N) and len(q_all) == len(psi_all) == l + 1
    digits = relin_digits(d[:, 2], q_all, psi_all)
    off = np.array([0, l], dtype=np.uint32)
    idx = np.arange(l, dtype=np.uint32)
    out = np.empty((n, 2, l, N), dtype=np.uint64)
    for c in range(n):
        # sum over the digits of digit_j * evk_j: the key's pairs play the ciphertexts, the digits the plaintexts
        acc = mac(evk, q_all, off, idx, idx, digits[c], PT_POLY)            # [1][2][l+1][N]
        down = rescale(acc, q_all, psi_all)[0]                               # divide by P, rounding
        for k in range(2):
            for i in range(l):
                out[c, k, i] = (d[c, k, i].astype(object) + down[k, i].astype(object)) % int(q_all[i])
    return out


def square_relin(ct, q_all, psi_all, evk) -> np.ndarray:
    """The x^2 activation on ciphertexts [n][2][l][N] with l = len(q_all) - 1: square, then relinearise."""
    l = len(q_all) - 1
    return relinearize(square(ct, q_all[:l]), q_all, psi_all, evk)
