"""Pins of the oracle's square + relinearisation (the x^2 activation): none re-types the oracle's RNS steps."""
import numpy as np
import pytest

import oracle
from oracle import ckks_scaffold as sc
from paper_1908_04172_amd import workloads as wl


def negacyclic(a, b, N, mod):
    out = [0] * N
    for i, ai in enumerate(a):
        if ai == 0:
            continue
        for j, bj in enumerate(b):
            k = i + j
            if k < N:
                out[k] = (out[k] + ai * bj) % mod
            else:
                out[k - N] = (out[k - N] - ai * bj) % mod
    return out


def to_coeffs(rows, q, psi):
    """[limbs][N] NTT form -> N integers in [0, prod q) (CRT of the inverse transforms)."""
    c = oracle.ntt_inv(rows[None], q, psi)[0]
    Q = 1
    for qi in q:
        Q *= int(qi)
    out = []
    for k in range(c.shape[1]):
        x = 0
        for r, qi in zip(c[:, k], q):
            Qi = Q // int(qi)
            x += int(r) * Qi * pow(Qi, -1, int(qi))
        out.append(x % Q)
    return out


@pytest.mark.parametrize("N,bits", [(16, [20, 21, 25]), (32, [22, 22, 22, 27])])
def test_relinearisation_equals_the_big_integer_formulation(N, bits):
    """Brute force on tiny rings, in Z_{QP}[X]/(X^N+1) with Python integers and schoolbook products: the sum over
    the digits of digit_j * key_j modulo Q*P, divided by P with rounding, plus (d0, d1): bit for bit."""
    q = wl.modulus_chain(bits, N)
    psi = oracle.find_psis(q, N)
    l, P = len(q) - 1, q[-1]
    Q = int(np.prod([int(x) for x in q[:l]], dtype=object))
    sf = sc.Scaffold(N, q, psi, seed=N)
    evk = sf.relin_key()
    rng = np.random.default_rng(N + 1)
    d = np.stack([np.stack([rng.integers(0, qi, N, dtype=np.uint64) for qi in q[:l]]) for _ in range(3)])[None]
    got = oracle.relinearize(d, q, psi, evk)[0]
    d2_rows = oracle.ntt_inv(d[0, 2][None], q[:l], psi[:l])[0]           # digit j = coefficients modulo q_j
    evk_coef = [[to_coeffs(evk[j, k], q, psi) for k in range(2)] for j in range(l)]
    for k in range(2):
        acc = [0] * N
        for j in range(l):
            prod = negacyclic([int(x) for x in d2_rows[j]], evk_coef[j][k], N, Q * P)
            acc = [(x + y) % (Q * P) for x, y in zip(acc, prod)]
        down = [((x + P // 2) // P) % Q for x in acc]
        dk = to_coeffs(d[0, k], q[:l], psi[:l])
        want = [(x + y) % Q for x, y in zip(dk, down)]
        assert to_coeffs(got[k], q[:l], psi[:l]) == want


def test_relinearised_ciphertext_decrypts_like_the_three_component_one():
    """Dec(c0', c1') = d0 + d1 s + d2 s^2 up to the key-switching noise, which the division by P makes small."""
    N = 64
    q = wl.modulus_chain([30, 30, 36], N)
    psi = oracle.find_psis(q, N)
    sf = sc.Scaffold(N, q, psi, seed=3)
    evk = sf.relin_key()
    z = np.random.default_rng(4).normal(size=N // 2) + 0j
    ct = sf.encrypt(z, 2.0**20)[:, :2]                                   # limbs q_0, q_1: the special prime is not used
    d = oracle.square(ct[None], q[:2])
    out = oracle.relinearize(d, q, psi, evk)[0]
    a, b = sf.decrypt3_coeffs(d[0]), sf.decrypt_coeffs(out)
    assert max(abs(x - y) for x, y in zip(a, b)) < 2 * N * 2 * 8 * 3.2 + N    # l digits * N terms * |e| / (P/q_j) + rounding * |s|
    # and it means z^2 at scale^2
    back = sf.decrypt(out, 2.0**40)
    assert np.abs(back - z * z).max() < 1e-3


def test_square_then_rescale_through_the_scaffold():
    """The activation as a network uses it: square, relinearise, one rescale; Dec ~ z^2 at scale^2 / q_last."""
    N = 256
    q = wl.modulus_chain([40, 30, 30, 45], N)
    psi = oracle.find_psis(q, N)
    sf = sc.Scaffold(N, q, psi, seed=5)
    evk = sf.relin_key()
    z = np.random.default_rng(6).uniform(-1, 1, size=N // 2) + 0j
    ct = sf.encrypt(z, 2.0**30)[:, :3]
    out = oracle.square_relin(ct[None], q, psi, evk)
    down = oracle.rescale(out, q[:3], psi[:3])[0]
    back = sf.decrypt(down, 2.0**60 / q[2])
    assert np.abs(back - z * z).max() < 1e-4
    # the components of a square: symmetric in the two factors (c0*c1 counted twice), checked on one slot by hand
    i, k = 1, 7
    d = oracle.square(ct[None], q[:3])[0]
    assert int(d[1, i, k]) == 2 * int(ct[0, i, k]) * int(ct[1, i, k]) % q[i]
    assert int(d[2, i, k]) == int(ct[1, i, k]) ** 2 % q[i]
