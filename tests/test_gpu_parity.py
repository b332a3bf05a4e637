"""GPU parity: every entry point of the C-ABI library against the CPU oracle, element by element,
on the same seeded inputs.  Residues must match bit-exactly (integer work); the encrypt-compute-
decrypt check uses |err| <= 2^-10 * max(1, |value|)."""
import numpy as np
import pytest

import oracle
from oracle import ckks_scaffold as sc
from paper_1908_04172_amd import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def he():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1908_04172_amd import he as he_mod
    he_mod.lib()  # raises if the HIP library is not built: no fallback
    return he_mod


def dev(a: np.ndarray):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).cuda()


def host(t) -> np.ndarray:
    return t.cpu().numpy().view(np.uint64)


def rows(t, ids):
    """t[ids] for a NumPy index array of any integer type."""
    return t[torch.as_tensor(np.asarray(ids, dtype=np.int64), device=t.device)]


def compact(plan: wl.Plan, outputs):
    """Sub-problem for the listed outputs with ct/pt indices renumbered densely."""
    sub = plan.subset(outputs)
    ct_ids, ct_inv = np.unique(sub.term_ct, return_inverse=True)
    pt_ids, pt_inv = np.unique(sub.term_pt, return_inverse=True)
    return wl.Plan(len(ct_ids), sub.n_out, len(pt_ids), sub.off, ct_inv.astype(np.uint32), pt_inv.astype(np.uint32)), ct_ids, pt_ids


MIXED = {10: [30, 62, 50], 11: [40, 60], 12: [30, 30, 60], 13: [60, 40, 40, 40], 14: [60, 60, 50, 50, 50]}


# ----------------------------------------------------------------------------- NTT

@pytest.mark.parametrize("log2N", [10, 11, 12, 13, 14])
def test_ntt_fwd_inv_match_oracle(he, log2N):
    N = 1 << log2N
    q = wl.modulus_chain(MIXED[log2N], N)
    ctx = he.Context(log2N, q)
    assert ctx.psi == oracle.find_psis(q, N)
    a = wl.uniform_residues((3,), q, N, 1000 + log2N)          # 3 polys x limbs rows, ragged vs 256 CUs
    a[0, :, :] = 0
    a[0, :, 1] = 1                                              # the monomial X: pins root and ordering
    d = dev(a)
    ctx.ntt_fwd(d)
    want = oracle.ntt_fwd(a, q, ctx.psi)
    assert np.array_equal(host(d), want)
    ctx.ntt_inv(d)
    assert np.array_equal(host(d), a)
    # lower level: only the first limbs
    b = wl.uniform_residues((2, 2), q[:2], N, 2000 + log2N)
    db = dev(b)
    ctx.ntt_inv(db)
    assert np.array_equal(host(db), oracle.ntt_inv(b, q[:2], ctx.psi[:2]))
    # edge values q-1 everywhere
    e = np.stack([np.full(N, qi - 1, dtype=np.uint64) for qi in q])[None]
    de = dev(e)
    ctx.ntt_fwd(de)
    assert np.array_equal(host(de), oracle.ntt_fwd(e, q, ctx.psi))
    ctx.ntt_fwd(de[:0])                                         # zero polys: a no-op


@pytest.mark.gpu
@pytest.mark.parametrize("log2N,polys", [(14, 111), (12, 437)])
def test_ntt_with_several_rows_per_workgroup(he, log2N, polys):
    """More rows than resident workgroups (256 at N = 2^14, 1280 at N = 2^12), and not a multiple of
    them: every workgroup loops, some once more than others.  All rows against the oracle."""
    N = 1 << log2N
    q = wl.modulus_chain(MIXED[log2N], N)
    ctx = he.Context(log2N, q)
    a = wl.uniform_residues((polys,), q, N, 3000 + log2N)
    assert polys * len(q) > (256 if log2N == 14 else 1280)
    d = dev(a)
    ctx.ntt_fwd(d)
    assert np.array_equal(host(d), oracle.ntt_fwd(a, q, ctx.psi))
    ctx.ntt_inv(d)
    assert np.array_equal(host(d), a)


# ----------------------------------------------------------------------------- Alg. 1

def crt_centered_rows(coef, q):
    """[n][limbs][N] residues -> [n][N] integers in (-Q/2, Q/2] (Python ints in an object array)."""
    q = [int(x) for x in q]
    Q = 1
    for qi in q:
        Q *= qi
    x = np.zeros((coef.shape[0], coef.shape[2]), dtype=object)
    for i, qi in enumerate(q):
        Qi = Q // qi
        x = (x + coef[:, i, :].astype(object) * (Qi * pow(Qi % qi, -1, qi))) % Q
    return np.where(x > Q // 2, x - Q, x)


def gpu_encode_coeffs(ctx, z, scale, q, limbs=None):
    """he_encode_vector, then back to signed coefficients: the oracle's INTT and a centred lift."""
    d = ctx.encode_vector(torch.from_numpy(z).cuda(), scale, limbs=limbs)
    ntt_form = host(d)
    ql = q[: ntt_form.shape[1]]
    coef = oracle.ntt_inv(ntt_form, ql, ctx.psi[: len(ql)])
    return crt_centered_rows(coef, ql).astype(np.int64), ntt_form


@pytest.mark.parametrize("log2N", [10, 11, 12, 13, 14])
def test_encode_vector_matches_oracle(he, log2N):
    """Alg. 1 on the GPU against the oracle's term-by-term long-double evaluation.  The GPU interpolates
    with a double-precision FFT: a coefficient of magnitude M may differ by 1 + M * 2^-53 * 4 * log2(N)
    (the bound the header states); at a small scale that is at most 1, and only where the exact value
    falls within the FFT's error of a half-integer."""
    N = 1 << log2N
    q = wl.modulus_chain(MIXED[log2N], N)
    ctx = he.Context(log2N, q)
    rng = np.random.default_rng(400 + log2N)
    z = rng.normal(size=(3, N // 2)) + 1j * rng.normal(size=(3, N // 2))
    z[1] = z[1].real                                       # a real vector (real packing)
    z[2] = 0.37                                            # equal real slots: the scalar-encoding Lemma
    for scale in (2.0 ** 20, 2.0 ** 45):
        want = oracle.encode_vector_coeffs(z, scale, N)
        got, ntt_form = gpu_encode_coeffs(ctx, z, scale, q)
        M = float(np.abs(want).max())
        bound = 1 + M * 2.0 ** -53 * 4 * log2N
        diff = np.abs(got - want)
        assert diff.max() <= bound, (log2N, scale, diff.max(), bound)
        if scale == 2.0 ** 20:
            assert (diff != 0).mean() < 1e-3               # off by one only at near-ties
            # the Lemma, through the GPU: N equal residues per limb, the ones Alg. 2 gives
            assert np.array_equal(ntt_form[2], np.repeat(oracle.encode_scalar(0.37, scale, q)[:, None], N, axis=1))
        # decoding what the GPU encoded returns the slots
        back = oracle.decode_vector(got, scale, N)
        assert np.abs(back - z).max() <= (0.5 + bound) * N / scale
    # a lower level writes the first limbs only; no vectors is a no-op
    got2, _ = gpu_encode_coeffs(ctx, z[:1], 2.0 ** 16, q, limbs=1)
    assert np.abs(got2 - oracle.encode_vector_coeffs(z[:1], 2.0 ** 16, N)).max() <= 1
    ctx.encode_vector(torch.zeros((0, N // 2), dtype=torch.complex128, device="cuda"), 2.0 ** 20)
    with pytest.raises(he.HeError):
        ctx.encode_vector(torch.zeros((1, N // 2), dtype=torch.complex128, device="cuda"), float("inf"))


@pytest.mark.parametrize("log2N", [10, 12, 14])
def test_decode_vector_matches_oracle(he, log2N):
    """The inverse map on the GPU: an exact lift of the residues (checked here on coefficients far
    beyond 64 bits and of both signs), then double arithmetic against the oracle's long-double sums."""
    N = 1 << log2N
    q = wl.modulus_chain(MIXED[log2N], N)
    ctx = he.Context(log2N, q)
    rng = np.random.default_rng(500 + log2N)
    Q = 1
    for qi in q:
        Q *= int(qi)
    bits = Q.bit_length() - 2
    # three polynomials: small coefficients, coefficients near +-Q/2, and the extremes themselves
    m = np.zeros((3, N), dtype=object)
    m[0] = [int(x) for x in rng.integers(-2**40, 2**40, size=N)]
    m[1] = [int(rng.integers(-2**62, 2**62)) * (1 << (bits - 62)) + int(rng.integers(-5, 5)) for _ in range(N)]
    m[2] = [0] * N
    m[2, :6] = [Q // 2, -(Q // 2), 1, -1, Q // 2 - 1, 0]
    res = np.stack([np.array([[int(x) % int(qi) for x in m[v]] for qi in q], dtype=np.uint64) for v in range(3)])
    poly = oracle.ntt_fwd(res, q, ctx.psi)
    for scale, vecs in ((2.0 ** 30, [0]), (2.0 ** (bits - 10), [1, 2])):
        got = ctx.decode_vector(dev(poly[vecs]), scale).cpu().numpy()
        want = oracle.decode_vector(np.array([[float(x) for x in m[v]] for v in vecs]), scale, N)
        mag = max(abs(int(x)) for v in vecs for x in m[v])
        tol = N * mag * 2.0 ** -53 * 4 * log2N / scale
        assert np.abs(got - want).max() <= tol, (log2N, scale, np.abs(got - want).max(), tol)
    # encode then decode on the GPU returns the slots (to the rounding of the coefficients)
    z = rng.normal(size=(2, N // 2)) + 1j * rng.normal(size=(2, N // 2))
    enc = ctx.encode_vector(torch.from_numpy(z).cuda(), 2.0 ** 40)
    back = ctx.decode_vector(enc, 2.0 ** 40).cpu().numpy()
    assert np.abs(back - z).max() <= N / 2.0 ** 40
    assert np.array_equal(host(enc), host(enc.clone()))               # the input polynomial is left as it was
    # a lower level, an empty batch, a workspace that is too small
    back1 = ctx.decode_vector(ctx.encode_vector(torch.from_numpy(z).cuda(), 2.0 ** 20, limbs=1), 2.0 ** 20).cpu().numpy()
    assert np.abs(back1 - z).max() <= N / 2.0 ** 20
    ctx.decode_vector(enc[:0], 2.0 ** 40)
    with pytest.raises(he.HeError) as e:
        ctx.decode_vector(enc, 2.0 ** 40, workspace=torch.empty(64, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -6


def test_complex_packed_layer_through_encrypt_compute_decrypt(he):
    """Complex packing end to end: two real batches ride in the real and imaginary parts of the slots;
    a dense layer with scalar weights and a complex-packed bias vector (encoded on the GPU by Alg. 1),
    one lazy rescale, decrypt: both parts carry the float layer's result."""
    c = wl.config(2)
    N, q = c.N, c.q
    ctx = he.Context(c.log2N, q)
    scf = sc.Scaffold(N, q, ctx.psi, seed=77)
    rng = np.random.default_rng(78)
    K, M = 6, 3
    xa, xb = rng.uniform(-1, 1, size=(K, N // 2)), rng.uniform(-1, 1, size=(K, N // 2))
    w = rng.normal(0, 0.5, size=(K, M))
    bias = rng.normal(0, 0.5, size=(M, N // 2)) + 1j * rng.normal(0, 0.5, size=(M, N // 2))
    scale = 2.0 ** 40
    ct = np.stack([scf.encrypt(xa[k] + 1j * xb[k], scale) for k in range(K)])
    plan = wl.dense_plan(K, M)
    hp = ctx.plan(plan.n_in, plan.n_out, plan.n_pt, plan.off, plan.term_ct, plan.term_pt)
    wenc = ctx.encode_scalar(torch.from_numpy(w.reshape(-1).copy()).cuda(), scale)        # plaintext index k*M + o
    acc = ctx.ct_pt_mac(hp, dev(ct), wenc, he.PT_SCALAR)
    benc = ctx.encode_vector(torch.from_numpy(bias).cuda(), scale * scale)                # bias at scale^2
    ctx.ct_pt_add(acc, benc, he.PT_POLY)
    out = host(ctx.rescale(acc))
    new_scale = scale * scale / q[-1]
    for o in range(M):
        got = scf.decrypt(out[o], new_scale)
        want = (xa.T @ w[:, o] + bias[o].real) + 1j * (xb.T @ w[:, o] + bias[o].imag)
        assert np.abs(got - want).max() <= 2.0 ** -10 * max(1.0, np.abs(want).max())


# ----------------------------------------------------------------------------- Alg. 2

def test_encode_scalar_kernel_matches_oracle(he):
    c = wl.config(4)
    ctx = he.Context(c.log2N, c.q)
    rng = np.random.default_rng(7)
    vals = np.concatenate([rng.normal(0, 0.1, 1000), [0.0, -0.0, 0.5, -0.5, 1.5, 2.5, -2.5, 0.49999999999999994, 3.0],
                           rng.integers(-999, 999, 50) + 0.5])
    for scale in (1.0, 2.0**24, 2.0**50, 2.0**63, 2.0**100):
        got = host(ctx.encode_scalar(torch.from_numpy(vals).cuda(), scale))
        want = oracle.encode_scalars(vals, scale, c.q)
        assert np.array_equal(got, want), scale
        assert np.array_equal(got, ctx.encode_scalar_host(vals, scale))
    got = host(ctx.encode_scalar(torch.tensor([float("nan"), 1.0, float("inf")], dtype=torch.float64).cuda(), 2.0**30, limbs=3))
    assert np.all(got[0] == 2**64 - 1) and np.all(got[2] == 2**64 - 1)
    assert got[1].tolist() == [2**30 % qi for qi in c.q[:3]]


# ----------------------------------------------------------------------------- Alg. 3 / 4

@pytest.mark.parametrize("cfg", [1, 4])
def test_ct_pt_add_matches_oracle(he, cfg):
    c = wl.config(cfg)
    ctx = he.Context(c.log2N, c.q)
    n = 5
    ct = wl.uniform_residues((n, 2), c.q, c.N, 31)
    ct[0, 0] = np.array(c.q, dtype=np.uint64)[:, None] - 1      # wrap-around edge
    pts = wl.uniform_residues((n,), c.q, 1, 32)[..., 0]
    pts[0] = np.array(c.q, dtype=np.uint64) - 1
    d = dev(ct)
    ctx.ct_pt_add(d, dev(pts), he.PT_SCALAR)
    assert np.array_equal(host(d), oracle.add(ct, c.q, pts, oracle.PT_SCALAR))
    ptv = wl.uniform_residues((n,), c.q, c.N, 33)
    d = dev(ct)
    ctx.ct_pt_add(d, dev(ptv), he.PT_POLY)
    assert np.array_equal(host(d), oracle.add(ct, c.q, ptv, oracle.PT_POLY))
    # level 2 of a deeper chain
    d = dev(ct[:, :, :2].copy())
    ctx.ct_pt_add(d, dev(pts[:, :2].copy()), he.PT_SCALAR)
    assert np.array_equal(host(d), oracle.add(ct[:, :, :2], c.q[:2], pts[:, :2], oracle.PT_SCALAR))


# ----------------------------------------------------------------------------- Alg. 7 / 8 over plans

def irregular_plan(n_in, seed):
    """Outputs with 0, 1, 2, ... terms, some sharing their inputs (groups of 2..16), some not."""
    rng = np.random.default_rng(seed)
    off, tc, tp = [0], [], []
    n_pt = 0
    def add(cts):
        nonlocal n_pt
        tc.extend(cts)
        tp.extend(range(n_pt, n_pt + len(cts)))
        n_pt += len(cts)
        off.append(len(tc))
    add([])                                                     # empty output
    for k in (1, 2, 3, 9):
        add(rng.integers(0, n_in, k).tolist())
    for group, k in ((2, 5), (4, 7), (5, 3), (16, 6), (19, 4)):  # shared input lists
        cts = rng.integers(0, n_in, k).tolist()
        for _ in range(group):
            add(cts)
    add([])
    return wl.Plan(n_in, len(off) - 1, n_pt, np.asarray(off, np.uint32), np.asarray(tc, np.uint32), np.asarray(tp, np.uint32))


@pytest.mark.parametrize("log2N,bits", [(10, [30, 62, 50]), (12, [60, 60, 50])])
def test_mac_scalar_and_poly_match_oracle_on_irregular_plan(he, log2N, bits):
    N = 1 << log2N
    q = wl.modulus_chain(bits, N)
    ctx = he.Context(log2N, q)
    plan = irregular_plan(11, 5)
    hp = ctx.plan(plan.n_in, plan.n_out, plan.n_pt, plan.off, plan.term_ct, plan.term_pt)
    ct = wl.uniform_residues((plan.n_in, 2), q, N, 41)
    w = wl.uniform_residues((plan.n_pt,), q, 1, 42)[..., 0]
    bias = wl.uniform_residues((plan.n_out,), q, 1, 43)[..., 0]
    got = host(ctx.ct_pt_mac(hp, dev(ct), dev(w), he.PT_SCALAR, bias=dev(bias)))
    want = oracle.mac(ct, q, plan.off, plan.term_ct, plan.term_pt, w, oracle.PT_SCALAR, bias)
    assert np.array_equal(got, want)
    got = host(ctx.ct_pt_mac(hp, dev(ct), dev(w), he.PT_SCALAR))
    assert np.array_equal(got, oracle.mac(ct, q, plan.off, plan.term_ct, plan.term_pt, w, oracle.PT_SCALAR))
    wp = wl.uniform_residues((plan.n_pt,), q, N, 44)
    got = host(ctx.ct_pt_mac(hp, dev(ct), dev(wp), he.PT_POLY, bias=dev(bias)))
    assert np.array_equal(got, oracle.mac(ct, q, plan.off, plan.term_ct, plan.term_pt, wp, oracle.PT_POLY, bias))
    # Alg. 8 == Alg. 7 on replicated plaintexts
    rep = np.repeat(w[:, :, None], N, axis=2)
    assert np.array_equal(host(ctx.ct_pt_mac(hp, dev(ct), dev(rep), he.PT_POLY)),
                          host(ctx.ct_pt_mac(hp, dev(ct), dev(w), he.PT_SCALAR)))


def chained_groups_plan(n_in, seed, shared_weights=False, largest=16):
    """Enough groups of every size class for the kernel to chain several per workgroup, every group
    with more than 4 terms, term counts changing from group to group.  shared_weights: output g of a group
    multiplies by plaintexts 40*g .. 40*g + k - 1, so that groups of equal shape share their weight table (as the
    windows of a convolution do); else every output has plaintexts of its own (as in a dense layer).
    largest: the most outputs a group has (at most 8: the launch takes the kernel for narrow groups)."""
    rng = np.random.default_rng(seed)
    off, tc, tp, first_of_group = [0], [], [], []
    n_pt = 16 * 40 if shared_weights else 0
    for n_groups, lo, hi in ((2100, 5, largest), (1200, 2, 4), (40, 1, 1)):
        for _ in range(n_groups):
            k = int(rng.integers(5, 41))
            cts = rng.integers(0, n_in, k).tolist()
            first_of_group.append(len(off) - 1)
            for g in range(int(rng.integers(lo, hi + 1))):
                tc.extend(cts)
                if shared_weights:
                    tp.extend(range(40 * g, 40 * g + k))
                else:
                    tp.extend(range(n_pt, n_pt + k))
                    n_pt += k
                off.append(len(tc))
    plan = wl.Plan(n_in, len(off) - 1, n_pt, np.asarray(off, np.uint32), np.asarray(tc, np.uint32), np.asarray(tp, np.uint32))
    return plan, first_of_group


@pytest.mark.gpu
@pytest.mark.parametrize("bits,shared,largest", [([50, 58], False, 16), ([59, 61, 30], False, 16), ([50, 57, 40], True, 16),
                                                 ([50, 58], False, 8), ([59, 61, 30], False, 7), ([50, 57, 40], True, 8)])
def test_mac_scalar_chains_groups_with_changing_term_counts(he, bits, shared, largest):
    """Several groups per workgroup (the input ring and the weight pointer run on from one group
    into the next): whole runs of consecutive groups at both ends of every size class, and random
    groups in between, against the oracle on a sub-plan."""
    log2N, N = 11, 1 << 11
    q = wl.modulus_chain(bits, N)
    ctx = he.Context(log2N, q)
    plan, first = chained_groups_plan(37, 77, shared, largest)         # shared tables: the three-product form of the terms
    hp = ctx.plan(plan.n_in, plan.n_out, plan.n_pt, plan.off, plan.term_ct, plan.term_pt)
    ct = wl.uniform_residues((plan.n_in, 2), q, N, 78)
    w = dev(wl.uniform_residues((plan.n_pt,), q, 1, 79)[..., 0])
    bias = wl.uniform_residues((plan.n_out,), q, 1, 80)[..., 0]
    out = ctx.ct_pt_mac(hp, dev(ct), w, he.PT_SCALAR, bias=dev(bias))
    torch.cuda.synchronize()
    rng = np.random.default_rng(81)
    groups = set(rng.integers(0, len(first), 40).tolist())
    for lo, hi in ((0, 2100), (2100, 3300), (3300, 3340)):
        groups |= set(range(lo, min(lo + 20, hi))) | set(range(max(hi - 20, lo), hi))
    bounds = first + [plan.n_out]
    outputs = [o for g in sorted(groups) for o in range(bounds[g], bounds[g + 1])]
    sub, ct_ids, pt_ids = compact(plan, outputs)
    want = oracle.mac(ct[ct_ids], q, sub.off, sub.term_ct, sub.term_pt, host(rows(w, pt_ids)), oracle.PT_SCALAR, bias[outputs])
    assert np.array_equal(host(rows(out, outputs)), want)
    for l in range(len(q)):                                     # every output, any size: canonical residues
        assert int(out[:, :, l].max()) < q[l] and int(out[:, :, l].min()) >= 0


def split_plan(plan, seed):
    """Two plans over the same outputs: each output's terms cut at a place of its own (possibly at an end, so
    that some outputs get no term from one of the two calls); together they are `plan`."""
    rng = np.random.default_rng(seed)
    parts = [([0], [], []), ([0], [], [])]
    cut_of_list = {}
    for o in range(plan.n_out):
        a, b = int(plan.off[o]), int(plan.off[o + 1])
        key = tuple(plan.term_ct[a:b].tolist())                    # outputs of one group keep a common cut: they stay a group
        cut = cut_of_list.setdefault(key, int(rng.integers(0, b - a + 1)))
        for (off, tc, tp), (lo, hi) in zip(parts, ((a, a + cut), (a + cut, b))):
            tc.extend(plan.term_ct[lo:hi].tolist())
            tp.extend(plan.term_pt[lo:hi].tolist())
            off.append(len(tc))
    return [wl.Plan(plan.n_in, plan.n_out, plan.n_pt, np.asarray(off, np.uint32), np.asarray(tc, np.uint32), np.asarray(tp, np.uint32))
            for off, tc, tp in parts]


@pytest.mark.parametrize("log2N,bits", [(10, [30, 62, 50]), (12, [60, 57, 50])])
def test_mac_accumulate_over_two_calls_equals_one_call(he, log2N, bits):
    """HE_ACCUMULATE: a layer whose terms are split over two calls (the second adds into the output of the
    first; the bias goes with either) gives the residues of the one-call oracle layer.  Scalar and polynomial
    plaintexts, groups of every size class, outputs that get no term from one call."""
    N = 1 << log2N
    q = wl.modulus_chain(bits, N)
    ctx = he.Context(log2N, q)
    plans = [irregular_plan(11, 5)]
    chained, _ = chained_groups_plan(37, 91, shared_weights=True, largest=8)
    plans.append(chained.subset(list(range(0, 300)) + list(range(chained.n_out - 200, chained.n_out))))
    for plan in plans:
        first, second = split_plan(plan, 17)
        h1 = ctx.plan(first.n_in, first.n_out, first.n_pt, first.off, first.term_ct, first.term_pt)
        h2 = ctx.plan(second.n_in, second.n_out, second.n_pt, second.off, second.term_ct, second.term_pt)
        ct = wl.uniform_residues((plan.n_in, 2), q, N, 141)
        w = wl.uniform_residues((plan.n_pt,), q, 1, 142)[..., 0]
        bias = wl.uniform_residues((plan.n_out,), q, 1, 143)[..., 0]
        want = oracle.mac(ct, q, plan.off, plan.term_ct, plan.term_pt, w, oracle.PT_SCALAR, bias)
        out = ctx.ct_pt_mac(h1, dev(ct), dev(w), he.PT_SCALAR, bias=dev(bias))
        ctx.ct_pt_mac(h2, dev(ct), dev(w), he.PT_SCALAR, flags=he.ACCUMULATE, out=out)
        assert np.array_equal(host(out), want)
        out = ctx.ct_pt_mac(h1, dev(ct), dev(w), he.PT_SCALAR)                    # the bias with the second call
        ctx.ct_pt_mac(h2, dev(ct), dev(w), he.PT_SCALAR, bias=dev(bias), flags=he.ACCUMULATE, out=out)
        assert np.array_equal(host(out), want)
        assert ctx.check_reduced(out) == 0
        if plan is plans[0]:
            wp = wl.uniform_residues((plan.n_pt,), q, N, 144)
            wantp = oracle.mac(ct, q, plan.off, plan.term_ct, plan.term_pt, wp, oracle.PT_POLY, bias)
            out = ctx.ct_pt_mac(h1, dev(ct), dev(wp), he.PT_POLY, bias=dev(bias))
            ctx.ct_pt_mac(h2, dev(ct), dev(wp), he.PT_POLY, flags=he.ACCUMULATE, out=out)
            assert np.array_equal(host(out), wantp)
    with pytest.raises(he.HeError) as e:                                         # a rescaled output is no partial sum
        ctx.ct_pt_mac(h2, dev(ct), dev(w), he.PT_SCALAR, flags=he.ACCUMULATE | he.RESCALE,
                      out=torch.empty((plan.n_out, 2, len(q) - 1, N), dtype=torch.int64, device="cuda"))
    assert e.value.status == -1


def test_check_reduced_counts_residues_that_are_not_canonical(he):
    c = wl.config(2)
    ctx = he.Context(c.log2N, c.q)
    ct = wl.uniform_residues((3, 2), c.q, c.N, 151)
    assert ctx.check_reduced(dev(ct)) == 0
    assert ctx.check_reduced(dev(ct[:, :, :2].copy())) == 0                       # a lower level
    ct[0, 0, 0, 5] = c.q[0]
    ct[2, 1, 3, c.N - 1] = 2**64 - 1
    ct[1, 0, 1, 0] = c.q[0] - 1                                                   # canonical for limb 0, not for limb 1
    assert ctx.check_reduced(dev(ct)) == 3
    w = wl.uniform_residues((7,), c.q, 1, 152)[..., 0]                            # scalar plaintexts: [n][limbs]
    assert ctx.check_reduced(dev(w)) == 0
    w[6, 3] = c.q[3]
    assert ctx.check_reduced(dev(w)) == 1
    assert ctx.check_reduced(dev(ct[:0])) == 0


def test_mac_long_sums_of_extreme_operands(he):
    # (q-1)*(q-1) summed 700 times: crosses every fold and reduce boundary of the accumulator
    N = 1 << 10
    q = wl.modulus_chain([62, 60, 50, 30], N)
    ctx = he.Context(10, q)
    K, M = 700, 3
    plan = wl.dense_plan(K, M)
    hp = ctx.plan(plan.n_in, plan.n_out, plan.n_pt, plan.off, plan.term_ct, plan.term_pt)
    qa = np.array(q, dtype=np.uint64)
    ct = np.broadcast_to((qa - 1)[None, None, :, None], (K, 2, len(q), N)).copy()
    ct[:, :, :, 1::2] = wl.uniform_residues((K, 2), q, N // 2, 51)
    w = np.broadcast_to((qa - 1)[None, :], (K * M, len(q))).copy()
    w[1::3] = wl.uniform_residues((len(w[1::3]),), q, 1, 52)[..., 0]
    want = oracle.mac(ct, q, plan.off, plan.term_ct, plan.term_pt, w, oracle.PT_SCALAR)
    assert np.array_equal(host(ctx.ct_pt_mac(hp, dev(ct), dev(w), he.PT_SCALAR)), want)
    for l in range(len(q)):
        assert int(want[0, 0, l, 0]) == K * (q[l] - 1) ** 2 % q[l]
    wp = np.broadcast_to((qa - 1)[None, :, None], (K * M, len(q), N)).copy()
    wp[:, :, 1::2] = wl.uniform_residues((K * M,), q, N // 2, 53)
    assert np.array_equal(host(ctx.ct_pt_mac(hp, dev(ct), dev(wp), he.PT_POLY)),
                          oracle.mac(ct, q, plan.off, plan.term_ct, plan.term_pt, wp, oracle.PT_POLY))


def test_mac_argument_errors(he):
    c = wl.config(1)
    ctx = he.Context(c.log2N, c.q)
    p = wl.dense_plan(2, 2)
    with pytest.raises(he.HeError) as e:
        ctx.plan(p.n_in, p.n_out, p.n_pt, p.off, p.term_ct + 2, p.term_pt)       # ct index out of range
    assert e.value.status == -4
    hp = ctx.plan(p.n_in, p.n_out, p.n_pt, p.off, p.term_ct, p.term_pt)
    ct = dev(wl.uniform_residues((2, 2), c.q, c.N, 1))
    w = dev(wl.uniform_residues((4,), c.q, 1, 2)[..., 0])
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(he.HeError) as e:
        ctx.ct_pt_mac(hp, ct, w, he.PT_SCALAR, flags=he.RESCALE, workspace=small)
    assert e.value.status == -6
    with pytest.raises(he.HeError) as e:                                            # rescale needs 2 limbs
        ctx.ct_pt_mac(hp, ct[:, :, :1].contiguous(), w[:, :1].contiguous(), he.PT_SCALAR, flags=he.RESCALE)
    assert e.value.status == -3
    with pytest.raises(he.HeError) as e:                                            # output over the input
        ctx.ct_pt_mac(hp, ct, w, he.PT_SCALAR, out=ct)
    assert e.value.status == -1
    with pytest.raises(he.HeError) as e:
        ctx.rescale(ct, out=ct.view(-1)[c.N: 5 * c.N].view(2, 2, 1, c.N))
    assert e.value.status == -1
    with pytest.raises(he.HeError) as e:                                            # the workspace over the plaintexts
        ctx.ct_pt_mac(hp, ct, w, he.PT_SCALAR, workspace=w.view(torch.uint8))
    assert e.value.status in (-1, -6)
    big = torch.empty(1 << 20, dtype=torch.int64, device="cuda")
    with pytest.raises(he.HeError) as e:                                            # the workspace over the input
        ctx.ct_pt_mac(hp, big[: ct.numel()].view(ct.shape), w, he.PT_SCALAR, workspace=big.view(torch.uint8))
    assert e.value.status == -1
    # a plan outlives its context without harm: its device arrays are freed on their own
    ctx2 = he.Context(c.log2N, c.q)
    hp2 = ctx2.plan(p.n_in, p.n_out, p.n_pt, p.off, p.term_ct, p.term_pt)
    ctx2.close()
    hp2.close()
    assert torch.zeros(4, device="cuda").sum().item() == 0                          # no error left behind


def test_measured_rates_are_plausible(he):
    """he_measure_rate: register-resident ceilings; the butterfly modes get faster as they get lazier."""
    c = wl.config(4)
    ctx = he.Context(c.log2N, c.q)
    mad = ctx.measure_rate(he.RATE_MAD32, 0, 512)
    assert 5e12 < mad < 45e12                                                       # nominal 39.3e12 on 256 CUs
    b0, b1, b2 = (ctx.measure_rate(k, 2, 512) for k in (he.RATE_BUTTERFLY_MODE0, he.RATE_BUTTERFLY_MODE1,
                                                         he.RATE_BUTTERFLY_MODE2))
    assert b0 < b1 < b2 < mad / 4
    t4, t3 = ctx.measure_rate(he.RATE_MAC_TERM, 2, 512), ctx.measure_rate(he.RATE_MAC_TERM3, 2, 512)
    assert mad / 6 < t4 < t3 < mad / 2                                              # four and three multiply-adds per term
    f_fwd, f_inv = ctx.measure_rate(he.RATE_BUTTERFLY_FP64, 2, 512), ctx.measure_rate(he.RATE_BUTTERFLY_FP64_INV, 2, 512)
    assert b2 < f_inv < f_fwd < mad / 4                                             # the double-precision butterflies of a 50-bit limb
    for kind in (he.RATE_BUTTERFLY_MODE2, he.RATE_BUTTERFLY_FP64, he.RATE_BUTTERFLY_FP64_INV):
        with pytest.raises(he.HeError) as e:                                        # a 60-bit limb has no mode 2 and no double form
            ctx.measure_rate(kind, 0, 512)
        assert e.value.status == -2


# ----------------------------------------------------------------------------- Eq. (2)

@pytest.mark.parametrize("cfg", [1, 2, 4])
def test_rescale_matches_oracle(he, cfg):
    c = wl.config(cfg)
    ctx = he.Context(c.log2N, c.q)
    ct = wl.uniform_residues((3, 2), c.q, c.N, 61)
    ct[0, 0] = 0
    ct[0, 1] = np.array(c.q, dtype=np.uint64)[:, None] - 1
    got = host(ctx.rescale(dev(ct)))
    assert np.array_equal(got, oracle.rescale(ct, c.q, ctx.psi))
    if c.L >= 3:                                                # one level down: drops limb L-2
        sub = np.ascontiguousarray(ct[:, :, : c.L - 1])
        assert np.array_equal(host(ctx.rescale(dev(sub))), oracle.rescale(sub, c.q[:-1], ctx.psi[:-1]))


@pytest.mark.parametrize("integer_only", [False, True])
@pytest.mark.parametrize("log2N", [11, 14])
def test_rescale_with_dropped_modulus_above_and_below_the_kept_ones(he, log2N, integer_only):
    """The dropped modulus p against a kept q_i: p < q_i (t needs no reduction), q_i < p < 2 q_i, and p > 2 q_i
    (a full reduction), for kept limbs of every butterfly mode (62-, 60-, 50-, 30-bit), with the limbs below 2^50 on
    the double-precision transforms (the default) and on the integer butterflies."""
    N = 1 << log2N
    p50 = wl.ntt_primes(50, N, 30)
    q = [p50[29], wl.ntt_primes(30, N, 1)[0], wl.ntt_primes(62, N, 1)[0], wl.ntt_primes(60, N, 1)[0], p50[1], p50[0]]
    assert q[0] < q[-1] < 2 * q[0] and q[-1] > 2 * q[1] and q[-1] < q[2]
    ctx = he.Context(log2N, q)
    ctx.integer_transforms(integer_only)
    ct = wl.uniform_residues((3, 2), q, N, 160 + log2N)
    ct[0, 0, -1] = 0
    ct[0, 1, -1] = q[-1] - 1
    assert np.array_equal(host(ctx.rescale(dev(ct))), oracle.rescale(ct, q, ctx.psi))
    # the 62-bit limb dropped (every kept limb far below it), and a 50-bit limb dropped under a 60-bit one
    for chain in ([q[0], q[1], q[3], q[2]], [q[3], q[1], q[4]]):
        ctx2 = he.Context(log2N, chain)
        ctx2.integer_transforms(integer_only)
        ct2 = wl.uniform_residues((2, 2), chain, N, 170 + log2N)
        assert np.array_equal(host(ctx2.rescale(dev(ct2))), oracle.rescale(ct2, chain, ctx2.psi))


@pytest.mark.parametrize("log2N", [10, 12, 13, 14])
def test_integer_and_double_precision_transforms_give_the_same_residues(he, log2N):
    """Limbs below 2^50 are transformed on double-precision FMAs, larger ones on integer butterflies.  With the
    integer butterflies forced for every limb the transforms and the rescale still equal the oracle, so the two
    arithmetics agree bit for bit (and the integer butterflies of small limbs stay tested)."""
    N = 1 << log2N
    q = wl.modulus_chain([60, 50, 49, 40, 31, 30], N)
    ctx = he.Context(log2N, q)
    a = wl.uniform_residues((5, 2), q, N, 3000 + log2N)
    a[0, 0] = np.array(q, dtype=np.uint64)[:, None] - 1
    a[0, 1] = 0
    fwd, inv, res = oracle.ntt_fwd(a, q, ctx.psi), oracle.ntt_inv(a, q, ctx.psi), oracle.rescale(a, q, ctx.psi)
    for integer_only in (True, False, True):
        ctx.integer_transforms(integer_only)
        d = dev(a)
        ctx.ntt_fwd(d)
        assert np.array_equal(host(d), fwd), integer_only
        d = dev(a)
        ctx.ntt_inv(d)
        assert np.array_equal(host(d), inv), integer_only
        assert np.array_equal(host(ctx.rescale(dev(a))), res), integer_only


def test_config4_layer_is_the_same_with_integer_transforms(he):
    """cfg4 at full size as one fused call: the 4096 outputs with the integer butterflies forced for every limb
    equal those of the default (double-precision transforms for the 50-bit limbs), bit for bit."""
    c, ctx, plan, ct, wenc, benc = scalar_layer_inputs(he, 4)
    out = run_layer(he, c, ctx, plan, ct, wenc, he.PT_SCALAR, benc)
    ctx.integer_transforms(True)
    out_int = run_layer(he, c, ctx, plan, ct, wenc, he.PT_SCALAR, benc)
    assert torch.equal(out, out_int)


def test_maximum_sizes_and_degenerate_calls(he):
    # largest ring degree with the largest number of limbs, mixed widths including 61- and 62-bit moduli
    N, L = 1 << 14, 16
    q = wl.modulus_chain([62, 61, 60, 60] + [50] * 6 + [40] * 4 + [30] * 2, N)
    ctx = he.Context(14, q)
    assert ctx.psi == oracle.find_psis(q, N)
    ct = wl.uniform_residues((2, 2), q, N, 71)
    d = dev(ct)
    ctx.ntt_fwd(d)
    assert np.array_equal(host(d), oracle.ntt_fwd(ct, q, ctx.psi))
    assert np.array_equal(host(ctx.rescale(dev(ct))), oracle.rescale(ct, q, ctx.psi))
    plan = wl.dense_plan(20, 17)                                    # one full group of 16 and a ragged one of 1
    hp = ctx.plan(plan.n_in, plan.n_out, plan.n_pt, plan.off, plan.term_ct, plan.term_pt)
    cts = wl.uniform_residues((plan.n_in, 2), q, N, 72)
    w = wl.uniform_residues((plan.n_pt,), q, 1, 73)[..., 0]
    b = wl.uniform_residues((plan.n_out,), q, 1, 74)[..., 0]
    got = host(ctx.ct_pt_mac(hp, dev(cts), dev(w), he.PT_SCALAR, bias=dev(b), flags=he.RESCALE))
    want, n_rescales = oracle.layer(cts, q, ctx.psi, plan.off, plan.term_ct, plan.term_pt, w, oracle.PT_SCALAR, b)
    assert n_rescales == plan.n_out and np.array_equal(got, want)
    # two limbs: the smallest level a rescale accepts; one limb: MAC and add only
    sub = np.ascontiguousarray(ct[:, :, :2])
    assert np.array_equal(host(ctx.rescale(dev(sub))), oracle.rescale(sub, q[:2], ctx.psi[:2]))
    one = np.ascontiguousarray(cts[:, :, :1])
    got = host(ctx.ct_pt_mac(hp, dev(one), dev(np.ascontiguousarray(w[:, :1])), he.PT_SCALAR))
    assert np.array_equal(got, oracle.mac(one, q[:1], plan.off, plan.term_ct, plan.term_pt, w[:, :1], oracle.PT_SCALAR))
    # empty batches are no-ops
    empty = torch.empty((0, 2, L, N), dtype=torch.int64, device="cuda")
    assert ctx.rescale(empty).shape == (0, 2, L - 1, N)
    ctx.ct_pt_add(empty, torch.empty((0, L), dtype=torch.int64, device="cuda"), he.PT_SCALAR)
    hp0 = ctx.plan(3, 0, 2, np.zeros(1, np.uint32), np.zeros(0, np.uint32), np.zeros(0, np.uint32))
    out0 = ctx.ct_pt_mac(hp0, dev(cts[:3]), dev(w[:2]), he.PT_SCALAR)
    assert out0.shape == (0, 2, L, N)
    # a plan whose outputs have no terms at all: zero plus the bias
    hpz = ctx.plan(3, 2, 2, np.zeros(3, np.uint32), np.zeros(0, np.uint32), np.zeros(0, np.uint32))
    z = host(ctx.ct_pt_mac(hpz, dev(cts[:3]), dev(w[:2]), he.PT_SCALAR, bias=dev(b[:2])))
    assert np.all(z[:, 1] == 0) and np.array_equal(z[:, 0], np.broadcast_to(b[:2, :, None], (2, L, N)))


# ----------------------------------------------------------------------------- whole layers, all five configs

def run_layer(he, c, ctx, plan, ct_dev, pt_dev, pt_kind, bias_dev):
    hp = ctx.plan(plan.n_in, plan.n_out, plan.n_pt, plan.off, plan.term_ct, plan.term_pt)
    out = ctx.ct_pt_mac(hp, ct_dev, pt_dev, pt_kind, bias=bias_dev, flags=he.RESCALE)
    torch.cuda.synchronize()
    return out


def check_outputs(c, ctx, plan, outputs, out_dev, ct_rows, pt_rows, pt_kind, bias):
    """Oracle layer for the listed outputs on host copies of just the inputs they touch."""
    sub, ct_ids, pt_ids = compact(plan, outputs)
    ct = host(ct_rows(ct_ids))
    pt = host(pt_rows(pt_ids))
    b = None if bias is None else bias[list(outputs)]
    want, n_rescales = oracle.layer(ct, c.q, ctx.psi, sub.off, sub.term_ct, sub.term_pt, pt, pt_kind, b)
    assert n_rescales == len(outputs)
    got = host(rows(out_dev, list(outputs)))
    assert np.array_equal(got, want)


def test_config1_dense_layer_full_parity(he):
    c = wl.config(1)
    ctx = he.Context(c.log2N, c.q)
    plan = c.plan
    ct = dev(wl.uniform_residues((plan.n_in, 2), c.q, c.N, c.seed))
    w = torch.from_numpy(wl.normal_values(plan.n_pt, c.sigma, c.seed + 100)).cuda()
    b = torch.from_numpy(wl.normal_values(plan.n_out, c.sigma, c.seed + 200)).cuda()
    wenc = ctx.encode_scalar(w, 2.0**c.log2_scale)
    benc = ctx.encode_scalar(b, 2.0**c.log2_scale)
    out = run_layer(he, c, ctx, plan, ct, wenc, he.PT_SCALAR, benc)
    check_outputs(c, ctx, plan, range(plan.n_out), out, lambda i: rows(ct, i), lambda i: rows(wenc, i), oracle.PT_SCALAR, host(benc))


def scalar_layer_inputs(he, cfg):
    c = wl.config(cfg)
    ctx = he.Context(c.log2N, c.q)
    plan = c.plan
    ct = wl.uniform_residues_torch((plan.n_in, 2), c.q, c.N, c.seed, "cuda")
    w = torch.from_numpy(wl.normal_values(plan.n_pt, c.sigma, c.seed + 100)).cuda()
    b = torch.from_numpy(wl.normal_values(plan.n_out, c.sigma, c.seed + 200)).cuda()
    wenc = ctx.encode_scalar(w, 2.0**c.log2_scale)
    benc = ctx.encode_scalar(b, 2.0**c.log2_scale)
    assert np.array_equal(host(wenc[:50]), oracle.encode_scalars(w[:50].cpu().numpy(), 2.0**c.log2_scale, c.q))
    return c, ctx, plan, ct, wenc, benc


def assert_canonical(c, out):
    """Holds for every output at any size: residues in [0, q_i)."""
    for l in range(c.L - 1):
        assert int(out[:, :, l].max()) < c.q[l] and int(out[:, :, l].min()) >= 0


@pytest.mark.parametrize("cfg", [2, 3])
def test_scalar_layers_at_full_size_every_output(he, cfg):
    """cfg2 (convolution, 720 outputs) and cfg3 (dense, 100 outputs of 845 terms) as the one fused call the
    benchmark times; EVERY output ciphertext against the oracle, in batches that bound the host memory."""
    c, ctx, plan, ct, wenc, benc = scalar_layer_inputs(he, cfg)
    out = run_layer(he, c, ctx, plan, ct, wenc, he.PT_SCALAR, benc)
    hb = host(benc)
    step = 180 if cfg == 2 else 50
    for a in range(0, plan.n_out, step):
        check_outputs(c, ctx, plan, range(a, min(a + step, plan.n_out)), out, lambda i: rows(ct, i),
                      lambda i: rows(wenc, i), oracle.PT_SCALAR, hb)
    assert_canonical(c, out)


def test_config4_conv_layer_at_full_size_runs_of_groups(he):
    """cfg4 at full size (4096 outputs = 256 windows x 16 channels; a workgroup of the MAC kernel runs through
    8 consecutive windows = 128 outputs).  Checked against the oracle: the first and the last such run, two
    runs at random places, one stretch of 128 outputs that straddles two runs, and the last window of every
    window size (the padded last row and column have 18 and 12 terms): 640 + 48 outputs of 4096 (> 1/8)."""
    c, ctx, plan, ct, wenc, benc = scalar_layer_inputs(he, 4)
    out = run_layer(he, c, ctx, plan, ct, wenc, he.PT_SCALAR, benc)
    run = 8 * 16
    n_runs = plan.n_out // run
    rng = np.random.default_rng(c.seed)
    picks = sorted(set([0, n_runs - 1] + (1 + rng.permutation(n_runs - 2)[:2]).tolist()))
    assert len(picks) == 4
    chosen = set()
    for r in picks:
        chosen |= set(range(r * run, (r + 1) * run))
    mid = int(rng.integers(2, n_runs - 2)) * run + run // 2            # half of one run, half of the next
    chosen |= set(range(mid, mid + run))
    lens = np.diff(plan.off.astype(np.int64))
    for k in np.unique(lens):
        last = int(np.flatnonzero(lens == k)[-1])
        chosen |= set(range(last // 16 * 16, last // 16 * 16 + 16))      # the whole window
    outputs = sorted(chosen)
    assert len(outputs) >= 256 and {int(lens[o]) for o in outputs} == set(lens.tolist())
    hb = host(benc)
    for a in range(0, len(outputs), 128):
        check_outputs(c, ctx, plan, outputs[a:a + 128], out, lambda i: rows(ct, i),
                      lambda i: rows(wenc, i), oracle.PT_SCALAR, hb)
    assert_canonical(c, out)


def test_config5_full_poly_layer_sampled_outputs(he):
    """cfg5 at full size (16 GiB of plaintext polynomials; the kernel handles 4 outputs per thread): the
    first, the last and two inner groups of four, i.e. 16 of the 64 outputs and all four positions of a group."""
    c = wl.config(5)
    ctx = he.Context(c.log2N, c.q)
    plan = c.plan
    ct = wl.uniform_residues_torch((plan.n_in, 2), c.q, c.N, c.seed, "cuda")
    pt = wl.uniform_residues_torch((plan.n_pt,), c.q, c.N, c.seed + 100, "cuda")     # 16 GiB
    out = run_layer(he, c, ctx, plan, ct, pt, he.PT_POLY, None)
    outputs = [o for g in (0, 5, 10, 15) for o in range(4 * g, 4 * g + 4)]
    assert len(outputs) == 16 and {o % 4 for o in outputs} == {0, 1, 2, 3}
    for a in range(0, len(outputs), 4):                                # 4 outputs = 1024 plaintext polynomials = 1 GiB on the host
        check_outputs(c, ctx, plan, outputs[a:a + 4], out, lambda i: rows(ct, i),
                      lambda i: rows(pt, i), oracle.PT_POLY, None)
    assert_canonical(c, out)
    # the unfused route gives the same residues as the fused call
    hp = ctx.plan(plan.n_in, plan.n_out, plan.n_pt, plan.off, plan.term_ct, plan.term_pt)
    acc = ctx.ct_pt_mac(hp, ct, pt, he.PT_POLY)
    assert torch.equal(ctx.rescale(acc), out)


def test_fused_layer_accumulators_are_congruent_and_rescale_to_the_layer(he):
    """The accumulators a fused layer hands from its MAC to its rescale kernel (kept limbs of scalar-plaintext sums
    are left unreduced): congruent to the oracle's sums modulo every limb, canonical on the dropped limb, below 12q,
    and he_rescale of them is the fused call's output and the oracle's layer.  Chains with 62-, 60-, 57-, 50-, 40- and
    30-bit limbs: every reduction path."""
    for log2N, bits in ((11, [62, 60, 57, 50, 40, 30]), (13, [60, 40, 40, 40])):
        N = 1 << log2N
        q = wl.modulus_chain(bits, N)
        ctx = he.Context(log2N, q)
        plan = wl.conv_plan(7, 7, 3, 3, 3, 16, 2, "same")           # windows of 27, 18 and 12 terms, 16 outputs each
        hp = ctx.plan(plan.n_in, plan.n_out, plan.n_pt, plan.off, plan.term_ct, plan.term_pt)
        ct = wl.uniform_residues((plan.n_in, 2), q, N, 181)
        w = wl.uniform_residues((plan.n_pt,), q, 1, 182)[..., 0]
        b = wl.uniform_residues((plan.n_out,), q, 1, 183)[..., 0]
        w[:16] = np.array(q, dtype=np.uint64) - 1                    # extreme operands in the first window
        ct[:3] = (np.array(q, dtype=np.uint64) - 1)[None, None, :, None]
        acc = torch.empty((plan.n_out, 2, len(q), N), dtype=torch.int64, device="cuda")
        ctx.mac_for_rescale(hp, dev(ct), dev(w), he.PT_SCALAR, acc, bias=dev(b))
        want = oracle.mac(ct, q, plan.off, plan.term_ct, plan.term_pt, w, oracle.PT_SCALAR, b)
        got = host(acc)
        qa = np.array(q, dtype=np.uint64)[None, None, :, None]
        assert np.array_equal(got % qa, want)
        assert np.array_equal(got[:, :, -1], want[:, :, -1])          # the dropped limb is canonical
        assert np.all(got < 12 * qa.astype(object))
        fused = ctx.ct_pt_mac(hp, dev(ct), dev(w), he.PT_SCALAR, bias=dev(b), flags=he.RESCALE)
        assert torch.equal(ctx.rescale(acc), fused)
        layer, _ = oracle.layer(ct, q, ctx.psi, plan.off, plan.term_ct, plan.term_pt, w, oracle.PT_SCALAR, b)
        assert np.array_equal(host(fused), layer)


def test_two_chained_layers_with_depth_aware_encoding(he):
    # Sec. "Depth-aware Encoding": the second layer runs one level down, its weights encoded at that level
    N = 1 << 12
    q = wl.modulus_chain([60, 40, 40], N)
    ctx = he.Context(12, q)
    conv = wl.conv_plan(6, 6, 2, 3, 3, 4, 2, "same")               # 72 cts -> 3x3x4 = 36 cts
    dense = wl.dense_plan(conv.n_out, 5)
    ct = wl.uniform_residues((conv.n_in, 2), q, N, 81)
    w1, b1 = wl.normal_values(conv.n_pt, 0.1, 82), wl.normal_values(conv.n_out, 0.1, 83)
    w2, b2 = wl.normal_values(dense.n_pt, 0.1, 84), wl.normal_values(dense.n_out, 0.1, 85)
    scale = 2.0**40
    h1 = ctx.plan(conv.n_in, conv.n_out, conv.n_pt, conv.off, conv.term_ct, conv.term_pt)
    h2 = ctx.plan(dense.n_in, dense.n_out, dense.n_pt, dense.off, dense.term_ct, dense.term_pt)
    t = lambda a: torch.from_numpy(a).cuda()
    y1 = ctx.ct_pt_mac(h1, dev(ct), ctx.encode_scalar(t(w1), scale), he.PT_SCALAR, bias=ctx.encode_scalar(t(b1), scale),
                       flags=he.RESCALE)
    assert y1.shape == (conv.n_out, 2, 2, N)
    w2e, b2e = ctx.encode_scalar(t(w2), scale, limbs=2), ctx.encode_scalar(t(b2), scale, limbs=2)
    assert w2e.shape == (dense.n_pt, 2)                                          # 8 * 2 bytes per scalar at level 2
    y2 = ctx.ct_pt_mac(h2, y1, w2e, he.PT_SCALAR, bias=b2e, flags=he.RESCALE)
    o1, _ = oracle.layer(ct, q, ctx.psi, conv.off, conv.term_ct, conv.term_pt, oracle.encode_scalars(w1, scale, q),
                         oracle.PT_SCALAR, oracle.encode_scalars(b1, scale, q))
    o2, _ = oracle.layer(o1, q[:2], ctx.psi[:2], dense.off, dense.term_ct, dense.term_pt,
                         oracle.encode_scalars(w2, scale, q[:2]), oracle.PT_SCALAR, oracle.encode_scalars(b2, scale, q[:2]))
    assert np.array_equal(host(y1), o1) and np.array_equal(host(y2), o2)
    assert y2.shape == (dense.n_out, 2, 1, N)


# ----------------------------------------------------------------------------- meaning: encrypt, compute, decrypt

def test_encrypted_dense_layer_decrypts_to_float_layer(he):
    from oracle.ckks_scaffold import Scaffold
    c = wl.config(1)
    ctx = he.Context(c.log2N, c.q)
    K, M = 64, 16
    sc = Scaffold(c.N, c.q, ctx.psi, 300)
    rng = np.random.default_rng(301)
    x = rng.uniform(-1, 1, size=(K, c.N // 2))
    w = rng.normal(0, 0.1, size=(K, M))
    b = rng.normal(0, 0.1, size=M)
    cts = np.stack([sc.encrypt(x[k], 2.0**30) for k in range(K)])
    plan = wl.dense_plan(K, M)
    hp = ctx.plan(plan.n_in, plan.n_out, plan.n_pt, plan.off, plan.term_ct, plan.term_pt)
    wenc = ctx.encode_scalar(torch.from_numpy(w.ravel()).cuda(), 2.0**24)
    benc = ctx.encode_scalar(torch.from_numpy(b).cuda(), 2.0**54)
    out = host(ctx.ct_pt_mac(hp, dev(cts), wenc, he.PT_SCALAR, bias=benc, flags=he.RESCALE))
    want = x.T @ w + b
    scale_out = 2.0**54 / c.q[-1]
    worst = 0.0
    for o in range(M):
        got = sc.decrypt(out[o], scale_out).real
        worst = max(worst, float(np.max(np.abs(got - want[:, o]) / np.maximum(1.0, np.abs(want[:, o])))))
    assert worst <= 2.0**-10, worst


# ----------------------------------------------------------------------------- ring degree 2^15 (rows beyond the LDS)

def test_ring_degree_2_15_transforms_and_rescale(he):
    """log2N = 15: a row is 256 KiB and the transforms run as one stage over global memory plus two half-size
    transforms.  he_ntt_fwd / he_ntt_inv against the oracle (the monomial X pins root and ordering, q-1 everywhere the
    ranges), he_rescale against the oracle at two levels, with the limbs below 2^50 on either arithmetic."""
    log2N, N = 15, 1 << 15
    q = wl.modulus_chain([60, 50, 50, 40, 31], N)
    ctx = he.Context(log2N, q)
    assert ctx.psi == oracle.find_psis(q, N)
    a = wl.uniform_residues((3, 2), q, N, 1500)
    a[0, 0] = 0
    a[0, 0, :, 1] = 1
    a[0, 1] = np.array(q, dtype=np.uint64)[:, None] - 1
    fwd, inv = oracle.ntt_fwd(a, q, ctx.psi), oracle.ntt_inv(a, q, ctx.psi)
    res = oracle.rescale(a, q, ctx.psi)
    sub = np.ascontiguousarray(a[:, :, :3])
    res_sub = oracle.rescale(sub, q[:3], ctx.psi[:3])
    for integer_only in (False, True):
        ctx.integer_transforms(integer_only)
        d = dev(a)
        ctx.ntt_fwd(d)
        assert np.array_equal(host(d), fwd), integer_only
        ctx.ntt_inv(d)
        assert np.array_equal(host(d), a), integer_only
        d = dev(a)
        ctx.ntt_inv(d)
        assert np.array_equal(host(d), inv), integer_only
        assert np.array_equal(host(ctx.rescale(dev(a))), res), integer_only
        assert np.array_equal(host(ctx.rescale(dev(sub))), res_sub), integer_only
    # lower level, one polynomial, one limb
    b = wl.uniform_residues((1, 1), q[:1], N, 1501)
    db = dev(b)
    ctx.ntt_fwd(db)
    assert np.array_equal(host(db), oracle.ntt_fwd(b, q[:1], ctx.psi[:1]))


def test_ring_degree_2_15_layers_match_oracle(he):
    """log2N = 15: the MAC kernels do not depend on the ring degree; a fused layer (scalar and full-polynomial
    plaintexts, bias, one rescale per output) and the plaintext addition against the oracle on the irregular plan."""
    log2N, N = 15, 1 << 15
    q = wl.modulus_chain([60, 50, 50], N)
    ctx = he.Context(log2N, q)
    plan = irregular_plan(7, 15)
    hp = ctx.plan(plan.n_in, plan.n_out, plan.n_pt, plan.off, plan.term_ct, plan.term_pt)
    ct = wl.uniform_residues((plan.n_in, 2), q, N, 1510)
    w = wl.uniform_residues((plan.n_pt,), q, 1, 1511)[..., 0]
    bias = wl.uniform_residues((plan.n_out,), q, 1, 1512)[..., 0]
    got = host(ctx.ct_pt_mac(hp, dev(ct), dev(w), he.PT_SCALAR, bias=dev(bias), flags=he.RESCALE))
    want, n_rescales = oracle.layer(ct, q, ctx.psi, plan.off, plan.term_ct, plan.term_pt, w, oracle.PT_SCALAR, bias)
    assert n_rescales == plan.n_out and np.array_equal(got, want)
    assert np.array_equal(host(ctx.ct_pt_mac(hp, dev(ct), dev(w), he.PT_SCALAR, bias=dev(bias))),
                          oracle.mac(ct, q, plan.off, plan.term_ct, plan.term_pt, w, oracle.PT_SCALAR, bias))
    wp = wl.uniform_residues((plan.n_pt,), q, N, 1513)
    got = host(ctx.ct_pt_mac(hp, dev(ct), dev(wp), he.PT_POLY, flags=he.RESCALE))
    want, _ = oracle.layer(ct, q, ctx.psi, plan.off, plan.term_ct, plan.term_pt, wp, oracle.PT_POLY, None)
    assert np.array_equal(got, want)
    pt = wl.uniform_residues((plan.n_in,), q, 1, 1514)[..., 0]
    d = dev(ct)
    ctx.ct_pt_add(d, dev(pt), he.PT_SCALAR)
    assert np.array_equal(host(d), oracle.add(ct, q, pt, oracle.PT_SCALAR))
    bad = ctx.check_reduced(d)
    assert bad == 0


def test_ring_degree_2_15_calls_built_on_one_row_per_workgroup_are_refused(he):
    """The vector encoder and decoder, square + relinearisation and the packed 32-bit path stop at log2N = 14:
    HE_ERR_ARG at 15, with nothing enqueued."""
    log2N, N = 15, 1 << 15
    q = wl.modulus_chain([30, 30, 30], N)
    ctx = he.Context(log2N, q)
    z = torch.zeros((1, N // 2), dtype=torch.complex128, device="cuda")
    poly = torch.zeros((1, 3, N), dtype=torch.int64, device="cuda")
    ct = torch.zeros((1, 2, 2, N), dtype=torch.int64, device="cuda")
    ct32 = torch.zeros((1, 2, 2, N), dtype=torch.int32, device="cuda")
    evk = torch.zeros((2, 2, 3, N), dtype=torch.int64, device="cuda")
    calls = [lambda: ctx.encode_vector(z, 2.0**20), lambda: ctx.decode_vector(poly, 2.0**20),
             lambda: ctx.ct_square_relin(ct, evk), lambda: ctx.rescale32(ct32), lambda: ctx.ntt_fwd32(ct32)]
    for f in calls:
        with pytest.raises(he.HeError) as e:
            f()
        assert e.value.status == -1
    assert torch.zeros(4, device="cuda").sum().item() == 0
