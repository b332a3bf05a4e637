"""Pins of the oracle's general encoding (Alg. 1, read as the canonical embedding) and of complex
packing (Sec. "Complex packing"): none of these checks re-types the oracle's own formula."""
import numpy as np
import pytest

import oracle
from oracle import ckks_scaffold as sc
from paper_1908_04172_amd import workloads as wl


def slot_roots(N):
    k = np.arange(N // 2)
    return np.exp(1j * np.pi * (2 * k + 1) / N)


def rand_slots(rng, n, N, complex_=True):
    z = rng.normal(size=(n, N // 2))
    return z + 1j * rng.normal(size=(n, N // 2)) if complex_ else z + 0j


@pytest.mark.parametrize("N", [4, 8, 32])
def test_coefficients_solve_the_interpolation_system(N):
    """Brute force on tiny rings: the coefficients are the real solution of m(r_k) = scale*z_k,
    m(conj r_k) = scale*conj(z_k), found here with a dense linear solve."""
    rng = np.random.default_rng(N)
    z = rand_slots(rng, 3, N)
    scale = 2.0 ** 20
    r = slot_roots(N)
    roots = np.concatenate([r, np.conj(r)])
    V = roots[:, None] ** np.arange(N)[None, :]
    got = oracle.encode_vector_coeffs(z, scale, N)
    for v in range(3):
        m = np.linalg.solve(V, scale * np.concatenate([z[v], np.conj(z[v])]))
        assert np.abs(m.imag).max() < 1e-6
        assert np.array_equal(got[v], np.round(m.real).astype(np.int64))


def test_paper_example_two_slots():
    """N = 4 as in the paper's illustration of complex packing: CEnc(a, b, c, d) holds a+bi and c+di.
    With r = exp(i*pi/4) the two slot roots are r and r^3, and the interpolation has the closed form
    m_j = (1/2) Re(z_0 r^-j + z_1 r^-3j)."""
    a, b, c, d = 0.75, -0.5, 0.125, 1.5
    scale = 2.0 ** 12
    r = np.exp(1j * np.pi / 4)
    z0, z1 = a + 1j * b, c + 1j * d
    want = [round(scale * 0.5 * (z0 * r ** (-j) + z1 * r ** (-3 * j)).real) for j in range(4)]
    assert oracle.encode_vector_coeffs([[z0, z1]], scale, 4)[0].tolist() == want
    back = oracle.decode_vector(want, scale, 4)[0]
    assert np.abs(back - np.array([z0, z1])).max() < 2e-3


@pytest.mark.parametrize("cfg", [1, 2, 4])
def test_equal_real_slots_give_the_scalar_encoding(cfg):
    """The paper's Lemma (appendix "Scalar Encoding"): N/2 equal real slots encode to a constant
    polynomial, whose NTT form repeats one residue per limb: exactly what Alg. 2 stores once."""
    c = wl.config(cfg)
    psi = oracle.find_psis(c.q, c.N)
    value, scale = -0.3141592653589793, 2.0 ** c.log2_scale
    m = oracle.encode_vector_coeffs(np.full(c.N // 2, value), scale, c.N)[0]
    assert m[0] == int(np.round(value * scale)) and not m[1:].any()
    full = oracle.encode_vector(np.full(c.N // 2, value), scale, c.q, psi, c.N)[0]
    scalar = oracle.encode_scalar(value, scale, c.q)
    assert np.array_equal(full, np.repeat(scalar[:, None], c.N, axis=1))


@pytest.mark.parametrize("N", [16, 256, 4096])
def test_matches_the_fft_route_and_inverts(N):
    """A second route to the same map (numpy's FFT with a twist, as the test scaffold encodes) gives
    the same integers; decoding returns the slots to within the rounding of the coefficients."""
    rng = np.random.default_rng(100 + N)
    z = rand_slots(rng, 2, N)
    for scale in (2.0 ** 20, 2.0 ** 40):
        got = oracle.encode_vector_coeffs(z, scale, N)
        for v in range(2):
            assert np.array_equal(got[v], np.array(sc.encode_coeffs(z[v], scale, N), dtype=np.int64))
        back = oracle.decode_vector(got, scale, N)
        # each coefficient is off by at most 1/2 before scaling; N of them add up at a root
        assert np.abs(back - z).max() <= 0.5 * N / scale
        # evaluation of the polynomial at the roots, the plain way
        r = slot_roots(N)
        if N <= 256:
            for v in range(2):
                direct = np.array([np.sum(got[v] * rk ** np.arange(N)) for rk in r]) / scale
                assert np.abs(direct - back[v]).max() < 1e-6


def test_ring_product_is_the_slotwise_product():
    """The embedding is a ring homomorphism: the negacyclic product of two encodings (slot-wise product
    in NTT form, through the oracle's NTT) decodes to the slot-wise product of the vectors."""
    N = 64
    q = wl.modulus_chain([60, 50], N)
    psi = oracle.find_psis(q, N)
    rng = np.random.default_rng(5)
    z = rand_slots(rng, 2, N)
    scale = 2.0 ** 24
    enc = oracle.encode_vector(z, scale, q, psi, N)                       # [2][limbs][N]
    prod = np.stack([np.array([int(x) * int(y) % qi for x, y in zip(enc[0, i], enc[1, i])], dtype=np.uint64)
                     for i, qi in enumerate(q)])
    coef = oracle.ntt_inv(prod[None], q, psi)[0]
    m = [sc.crt_centered([int(coef[i, j]) for i in range(len(q))], q) for j in range(N)]
    back = oracle.decode_vector(m, scale * scale, N)[0]
    assert np.abs(back - z[0] * z[1]).max() < 1e-4
    # and the full encoding is the coefficients' residues, transformed
    m0 = oracle.encode_vector_coeffs(z[:1], scale, N)[0]
    rows = np.array([[int(x) % qi for x in m0] for qi in q], dtype=np.uint64)
    assert np.array_equal(enc[0], oracle.ntt_fwd(rows[None], q, psi)[0])


def test_complex_packing_identities():
    """Sec. "Complex packing": add/subtract and broadcast-multiply act on real and imaginary parts
    independently; a general multiply does not (cross terms)."""
    N = 32
    rng = np.random.default_rng(6)
    scale = 2.0 ** 30
    x, y = rand_slots(rng, 1, N)[0], rand_slots(rng, 1, N)[0]
    f = rng.normal(size=N // 2)
    ex, ey = oracle.encode_vector_coeffs(x, scale, N)[0], oracle.encode_vector_coeffs(y, scale, N)[0]
    for sign in (1, -1):
        s = oracle.decode_vector(ex + sign * ey, scale, N)[0]
        assert np.abs(s.real - (x.real + sign * y.real)).max() < 1e-6
        assert np.abs(s.imag - (x.imag + sign * y.imag)).max() < 1e-6

    def negacyclic(a, b):
        out = [0] * N
        for i, ai in enumerate(a):
            for j, bj in enumerate(b):
                if i + j < N:
                    out[i + j] += int(ai) * int(bj)
                else:
                    out[i + j - N] -= int(ai) * int(bj)
        return out
    ef = oracle.encode_vector_coeffs(f + 0j, scale, N)[0]                  # CEnc(f, 0, f, 0, ...)
    p = oracle.decode_vector(negacyclic(ex, ef), scale * scale, N)[0]
    assert np.abs(p.real - x.real * f).max() < 1e-6 and np.abs(p.imag - x.imag * f).max() < 1e-6
    p = oracle.decode_vector(negacyclic(ex, ey), scale * scale, N)[0]
    assert np.abs(p - x * y).max() < 1e-6                                    # the complex product ...
    assert np.abs(p.real - x.real * y.real).max() > 1e-2                     # ... not the pairwise one


def test_out_of_range_and_non_finite_inputs_are_refused():
    N = 16
    with pytest.raises(ValueError):
        oracle.encode_vector_coeffs(np.full(N // 2, 1.0), 2.0 ** 63, N)
    z = np.zeros(N // 2, dtype=np.complex128)
    z[3] = np.nan
    with pytest.raises(ValueError):
        oracle.encode_vector_coeffs(z, 2.0 ** 20, N)
