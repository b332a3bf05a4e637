"""GPU parity of the packed 32-bit storage path (moduli below 2^30; Sec. "Ciphertext-plaintext
Multiplication", Alg. 6 and Alg. 8) against the CPU oracle: bit-exact residues, through the C ABI."""
import numpy as np
import pytest

import oracle
from paper_1908_04172_amd import workloads as wl
from test_gpu_parity import irregular_plan

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def he():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1908_04172_amd import he as he_mod
    he_mod.lib()                                                # fails loudly if the library is not built
    return he_mod


def dev32(a: np.ndarray):
    """uint64 residues below 2^32 -> int32 CUDA tensor holding the uint32 bit patterns."""
    assert int(a.max(initial=0)) < 1 << 32
    return torch.from_numpy(np.ascontiguousarray(a).astype(np.uint32).view(np.int32)).cuda()


def dev64(a: np.ndarray):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).cuda()


def host32(t) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32).astype(np.uint64)


SMALL = {10: [30, 29, 30], 11: [30, 30], 12: [30, 30, 28], 13: [30, 27, 30, 30], 14: [30, 30, 30]}


@pytest.mark.parametrize("log2N", [10, 11, 12, 13, 14])
def test_ntt32_matches_oracle(he, log2N):
    N = 1 << log2N
    q = wl.modulus_chain(SMALL[log2N], N)
    ctx = he.Context(log2N, q)
    a = wl.uniform_residues((3,), q, N, 3000 + log2N)
    a[0, :, :] = 0
    a[0, :, 1] = 1                                              # the monomial X: pins root and ordering
    a[1] = np.array(q, dtype=np.uint64)[:, None] - 1            # edge values q-1 everywhere
    d = dev32(a)
    ctx.ntt_fwd32(d)
    assert np.array_equal(host32(d), oracle.ntt_fwd(a, q, ctx.psi))
    ctx.ntt_inv32(d)
    assert np.array_equal(host32(d), a)
    b = wl.uniform_residues((2, 2), q[:2], N, 4000 + log2N)     # lower level
    db = dev32(b)
    ctx.ntt_inv32(db)
    assert np.array_equal(host32(db), oracle.ntt_inv(b, q[:2], ctx.psi[:2]))
    ctx.ntt_fwd32(db[:0])                                       # zero polys: a no-op


def test_pack_unpack_round_trip(he):
    q = wl.modulus_chain([30, 30], 1 << 10)
    ctx = he.Context(10, q)
    a = wl.uniform_residues((5, 2), q, 1 << 10, 7)
    p = ctx.pack32(dev64(a))
    assert np.array_equal(host32(p), a)
    assert np.array_equal(ctx.unpack32(p).cpu().numpy().view(np.uint64), a)
    odd = dev64(a.reshape(-1)[:1001].copy())                    # an odd count: the last thread takes one element
    assert np.array_equal(host32(ctx.pack32(odd)), a.reshape(-1)[:1001])
    assert np.array_equal(ctx.unpack32(ctx.pack32(odd)).cpu().numpy().view(np.uint64), a.reshape(-1)[:1001])


def test_add32_matches_oracle(he):
    c = wl.config(1)
    ctx = he.Context(c.log2N, c.q)
    n = 5
    ct = wl.uniform_residues((n, 2), c.q, c.N, 31)
    ct[0, 0] = np.array(c.q, dtype=np.uint64)[:, None] - 1
    pts = wl.uniform_residues((n,), c.q, 1, 32)[..., 0]
    pts[0] = np.array(c.q, dtype=np.uint64) - 1
    d = dev32(ct)
    ctx.ct_pt_add32(d, dev64(pts), he.PT_SCALAR)
    assert np.array_equal(host32(d), oracle.add(ct, c.q, pts, oracle.PT_SCALAR))
    ptv = wl.uniform_residues((n,), c.q, c.N, 33)
    d = dev32(ct)
    ctx.ct_pt_add32(d, dev32(ptv), he.PT_POLY)
    assert np.array_equal(host32(d), oracle.add(ct, c.q, ptv, oracle.PT_POLY))


@pytest.mark.parametrize("log2N,bits", [(10, [30, 29, 30]), (12, [30, 30])])
def test_mac32_scalar_and_poly_match_oracle_on_irregular_plan(he, log2N, bits):
    N = 1 << log2N
    q = wl.modulus_chain(bits, N)
    ctx = he.Context(log2N, q)
    plan = irregular_plan(11, 5)
    hp = ctx.plan(plan.n_in, plan.n_out, plan.n_pt, plan.off, plan.term_ct, plan.term_pt)
    ct = wl.uniform_residues((plan.n_in, 2), q, N, 41)
    w = wl.uniform_residues((plan.n_pt,), q, 1, 42)[..., 0]
    bias = wl.uniform_residues((plan.n_out,), q, 1, 43)[..., 0]
    got = host32(ctx.ct_pt_mac32(hp, dev32(ct), dev64(w), he.PT_SCALAR, bias=dev64(bias)))
    assert np.array_equal(got, oracle.mac(ct, q, plan.off, plan.term_ct, plan.term_pt, w, oracle.PT_SCALAR, bias))
    got = host32(ctx.ct_pt_mac32(hp, dev32(ct), dev64(w), he.PT_SCALAR))
    assert np.array_equal(got, oracle.mac(ct, q, plan.off, plan.term_ct, plan.term_pt, w, oracle.PT_SCALAR))
    wp = wl.uniform_residues((plan.n_pt,), q, N, 44)
    got = host32(ctx.ct_pt_mac32(hp, dev32(ct), dev32(wp), he.PT_POLY, bias=dev64(bias)))
    assert np.array_equal(got, oracle.mac(ct, q, plan.off, plan.term_ct, plan.term_pt, wp, oracle.PT_POLY, bias))
    # the packed path and the 64-bit path give the same residues
    got64 = ctx.ct_pt_mac(hp, dev64(ct), dev64(w), he.PT_SCALAR, bias=dev64(bias)).cpu().numpy().view(np.uint64)
    assert np.array_equal(got64, host32(ctx.ct_pt_mac32(hp, dev32(ct), dev64(w), he.PT_SCALAR, bias=dev64(bias))))


def test_mac32_long_sums_of_extreme_operands(he):
    # (q-1)*(q-1) summed 100 times: crosses the reduction every 15 terms with the largest sums possible
    N = 1 << 10
    q = wl.modulus_chain([30, 30, 25], N)
    ctx = he.Context(10, q)
    K, M = 100, 18
    plan = wl.dense_plan(K, M)
    hp = ctx.plan(plan.n_in, plan.n_out, plan.n_pt, plan.off, plan.term_ct, plan.term_pt)
    qa = np.array(q, dtype=np.uint64)
    ct = np.broadcast_to((qa - 1)[None, None, :, None], (K, 2, len(q), N)).copy()
    ct[:, :, :, 1::2] = wl.uniform_residues((K, 2), q, N // 2, 51)
    w = np.broadcast_to((qa - 1)[None, :], (K * M, len(q))).copy()
    w[1::3] = wl.uniform_residues((len(w[1::3]),), q, 1, 52)[..., 0]
    want = oracle.mac(ct, q, plan.off, plan.term_ct, plan.term_pt, w, oracle.PT_SCALAR)
    assert np.array_equal(host32(ctx.ct_pt_mac32(hp, dev32(ct), dev64(w), he.PT_SCALAR)), want)
    for l in range(len(q)):
        assert int(want[0, 0, l, 0]) == K * (q[l] - 1) ** 2 % q[l]
    wp = np.broadcast_to((qa - 1)[None, :, None], (K * M, len(q), N)).copy()
    wp[:, :, 1::2] = wl.uniform_residues((K * M,), q, N // 2, 53)
    assert np.array_equal(host32(ctx.ct_pt_mac32(hp, dev32(ct), dev32(wp), he.PT_POLY)),
                          oracle.mac(ct, q, plan.off, plan.term_ct, plan.term_pt, wp, oracle.PT_POLY))


@pytest.mark.parametrize("log2N,bits", [(12, [30, 30]), (13, [30, 27, 30, 30]), (14, [30, 30, 30])])
def test_rescale32_matches_oracle(he, log2N, bits):
    N = 1 << log2N
    q = wl.modulus_chain(bits, N)
    ctx = he.Context(log2N, q)
    ct = wl.uniform_residues((3, 2), q, N, 61)
    ct[0, 0] = 0
    ct[0, 1] = np.array(q, dtype=np.uint64)[:, None] - 1
    got = host32(ctx.rescale32(dev32(ct)))
    assert np.array_equal(got, oracle.rescale(ct, q, ctx.psi))
    if len(q) > 2:                                              # one level down
        ct2 = ct[:, :, :len(q) - 1].copy()
        assert np.array_equal(host32(ctx.rescale32(dev32(ct2))), oracle.rescale(ct2, q[:-1], ctx.psi[:-1]))


def test_config1_layer_through_the_packed_path(he):
    """cfg1 (dense 64 -> 16, N = 2^12, two 30-bit limbs): encode, MAC, bias and one lazy rescale per output in
    one call on 32-bit storage; equal to the oracle's layer and to the 64-bit path."""
    c = wl.config(1)
    ctx = he.Context(c.log2N, c.q)
    plan = c.plan
    hp = ctx.plan(plan.n_in, plan.n_out, plan.n_pt, plan.off, plan.term_ct, plan.term_pt)
    ct = wl.uniform_residues((plan.n_in, 2), c.q, c.N, c.seed)
    w = torch.from_numpy(wl.normal_values(plan.n_pt, c.sigma, c.seed + 100)).cuda()
    b = torch.from_numpy(wl.normal_values(plan.n_out, c.sigma, c.seed + 200)).cuda()
    wenc = ctx.encode_scalar(w, 2.0**c.log2_scale)
    benc = ctx.encode_scalar(b, 2.0**c.log2_scale)
    out32 = ctx.ct_pt_mac32(hp, dev32(ct), wenc, he.PT_SCALAR, bias=benc, flags=he.RESCALE)
    want, n_rescales = oracle.layer(ct, c.q, ctx.psi, plan.off, plan.term_ct, plan.term_pt,
                                    wenc.cpu().numpy().view(np.uint64), oracle.PT_SCALAR, benc.cpu().numpy().view(np.uint64))
    assert n_rescales == plan.n_out
    assert np.array_equal(host32(out32), want)
    out64 = ctx.ct_pt_mac(hp, dev64(ct), wenc, he.PT_SCALAR, bias=benc, flags=he.RESCALE)
    assert np.array_equal(out64.cpu().numpy().view(np.uint64), host32(out32))


def test_packed_calls_refuse_wide_moduli_and_bad_arguments(he):
    N = 1 << 10
    q = wl.modulus_chain([30, 40, 30], N)
    ctx = he.Context(10, q)
    one = torch.zeros((1, 2, 1, N), dtype=torch.int32, device="cuda")
    ctx.ntt_fwd32(one[0])                                       # level 1 uses the 30-bit limb only
    two = torch.zeros((1, 2, 2, N), dtype=torch.int32, device="cuda")
    for call in (lambda: ctx.ntt_fwd32(two[0]), lambda: ctx.rescale32(two),
                 lambda: ctx.ct_pt_add32(two, torch.zeros((1, 2), dtype=torch.int64, device="cuda"), he.PT_SCALAR)):
        with pytest.raises(he.HeError) as e:
            call()
        assert e.value.status == -2                             # HE_ERR_MODULUS: the 40-bit limb has no 32-bit form
    with pytest.raises(he.HeError) as e:
        ctx.rescale32(one)                                      # a rescale needs two limbs
    assert e.value.status == -3
    # a modulus just below 2^30 is accepted, one just above is not
    big = wl.modulus_chain([31], N)
    ctx2 = he.Context(10, big)
    with pytest.raises(he.HeError) as e:
        ctx2.ntt_fwd32(one[0])
    assert e.value.status == -2
