"""Minimal CKKS scaffold around the oracle: encode/decode, key generation, symmetric encryption
and decryption.  TEST INFRASTRUCTURE ONLY, CPU only; it exists so that tests can say what the
residue tensors MEAN ("Dec(pt * ct) ~ m1 * m2", Sec. "Homomorphic Encryption"), nothing of it is on
the hot path.

Encoding is the canonical embedding (the reading taken for Alg. 1): a plaintext polynomial m is
identified with its values at the N primitive 2N-th complex roots of unity r_k = exp(i*pi*(2k+1)/N);
slots k < N/2 carry the message, slot N-1-k its complex conjugate, so m has real coefficients.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

from . import ntt_fwd, ntt_inv


def _obj(a) -> np.ndarray:
    return np.asarray(a).astype(object)


def _mulmod_vec(a: np.ndarray, b: np.ndarray, q: int) -> np.ndarray:
    return ((_obj(a) * _obj(b)) % q).astype(np.uint64)


def _addmod_vec(a: np.ndarray, b: np.ndarray, q: int) -> np.ndarray:
    return ((_obj(a) + _obj(b)) % q).astype(np.uint64)


def encode_coeffs(slots: Sequence[complex], scale: float, N: int) -> List[int]:
    """round(scale * sigma^-1(slots)): N integer coefficients (Python ints, signed)."""
    z = np.asarray(slots, dtype=np.complex128)
    assert z.size == N // 2
    v = np.concatenate([z, np.conj(z[::-1])])          # v[N-1-k] = conj(v[k])
    n = np.arange(N)
    m = np.exp(-1j * np.pi * n / N) * np.fft.fft(v) / N  # m_n = (1/N) sum_k v_k r_k^-n
    return [int(round(float(c))) for c in (m.real * scale)]


def decode_coeffs(coeffs: Sequence[int], scale: float, N: int) -> np.ndarray:
    """sigma(m) / scale on the first N/2 slots; coefficients are signed Python ints."""
    m = np.array([float(c) for c in coeffs], dtype=np.float64)
    n = np.arange(N)
    v = np.fft.ifft(m * np.exp(1j * np.pi * n / N)) * N  # v_k = sum_n m_n r_k^n
    return v[: N // 2] / scale


def coeffs_to_rns_ntt(coeffs: Sequence[int], q: Sequence[int], psi: Sequence[int]) -> np.ndarray:
    """Signed integer coefficients -> [limbs][N] residues in NTT form."""
    rows = np.array([[c % int(qi) for c in coeffs] for qi in q], dtype=np.uint64)
    return ntt_fwd(rows, q, psi)


def crt_centered(residues: Sequence[int], q: Sequence[int]) -> int:
    """The integer in (-Q/2, Q/2] with the given residues (Python big ints)."""
    Q = 1
    for qi in q:
        Q *= int(qi)
    x = 0
    for r, qi in zip(residues, q):
        Qi = Q // int(qi)
        x += int(r) * Qi * pow(Qi, -1, int(qi))
    x %= Q
    return x - Q if x > Q // 2 else x


class Scaffold:
    def __init__(self, N: int, q: Sequence[int], psi: Sequence[int], seed: int):
        self.N, self.q, self.psi = N, [int(x) for x in q], [int(x) for x in psi]
        self.rng = np.random.default_rng(seed)
        s = self.rng.integers(-1, 2, size=N)            # ternary secret
        self.s_coeffs = [int(x) for x in s]
        self.s_ntt = coeffs_to_rns_ntt(self.s_coeffs, self.q, self.psi)

    def encrypt(self, slots: Sequence[complex], scale: float) -> np.ndarray:
        """Symmetric encryption at full level: ct = (c0, c1) = (-a*s + e + m, a), [2][L][N]."""
        N, q = self.N, self.q
        m = coeffs_to_rns_ntt(encode_coeffs(slots, scale, N), q, self.psi)
        e = [int(round(x)) for x in self.rng.normal(0.0, 3.2, size=N)]
        e_ntt = coeffs_to_rns_ntt(e, q, self.psi)
        ct = np.empty((2, len(q), N), dtype=np.uint64)
        for i, qi in enumerate(q):
            a = self.rng.integers(0, qi, size=N, dtype=np.uint64)
            a_s = _mulmod_vec(a, self.s_ntt[i], qi)
            neg = ((qi - _obj(a_s)) % qi).astype(np.uint64)
            ct[0, i] = _addmod_vec(_addmod_vec(neg, e_ntt[i], qi), m[i], qi)
            ct[1, i] = a
        return ct

    def decrypt_coeffs(self, ct: np.ndarray) -> List[int]:
        """c0 + c1*s on the first `limbs` moduli, as centred integer coefficients."""
        limbs = ct.shape[1]
        q, psi = self.q[:limbs], self.psi[:limbs]
        d = np.empty((limbs, self.N), dtype=np.uint64)
        for i, qi in enumerate(q):
            d[i] = _addmod_vec(ct[0, i], _mulmod_vec(ct[1, i], self.s_ntt[i], qi), qi)
        d = ntt_inv(d, q, psi)
        return [crt_centered([d[i, k] for i in range(limbs)], q) for k in range(self.N)]

    def decrypt(self, ct: np.ndarray, scale: float) -> np.ndarray:
        return decode_coeffs(self.decrypt_coeffs(ct), scale, self.N)

    def relin_key(self) -> np.ndarray:
        """Key-switching key for s^2 -> s with the LAST modulus as the special prime P: for each digit
        j < l = L-1 the pair (-a_j*s + e_j + P*g_j*s^2, a_j) modulo Q*P, where g_j = 1 mod q_j and 0 modulo
        the other q_i; in RNS the last term is (P mod q_j)*s^2 on limb j and nothing elsewhere.
        [l][2][L][N], NTT form."""
        N, q = self.N, self.q
        l, P = len(q) - 1, q[-1]
        evk = np.empty((l, 2, len(q), N), dtype=np.uint64)
        for j in range(l):
            e_ntt = coeffs_to_rns_ntt([int(round(x)) for x in self.rng.normal(0.0, 3.2, size=N)], q, self.psi)
            for i, qi in enumerate(q):
                a = self.rng.integers(0, qi, size=N, dtype=np.uint64)
                b = (qi - _obj(_mulmod_vec(a, self.s_ntt[i], qi))) % qi + _obj(e_ntt[i])
                if i == j:
                    s2 = _mulmod_vec(self.s_ntt[i], self.s_ntt[i], qi)
                    b = b + _obj(s2) * (P % qi)
                evk[j, 0, i] = (b % qi).astype(np.uint64)
                evk[j, 1, i] = a
        return evk

    def decrypt3_coeffs(self, d: np.ndarray) -> List[int]:
        """d0 + d1*s + d2*s^2 for a three-component ciphertext [3][limbs][N], centred coefficients."""
        limbs = d.shape[1]
        q, psi = self.q[:limbs], self.psi[:limbs]
        v = np.empty((limbs, self.N), dtype=np.uint64)
        for i, qi in enumerate(q):
            s2 = _mulmod_vec(self.s_ntt[i], self.s_ntt[i], qi)
            t = _addmod_vec(d[0, i], _mulmod_vec(d[1, i], self.s_ntt[i], qi), qi)
            v[i] = _addmod_vec(t, _mulmod_vec(d[2, i], s2, qi), qi)
        v = ntt_inv(v, q, psi)
        return [crt_centered([v[i, k] for i in range(limbs)], q) for k in range(self.N)]
