"""he_ct_pt_mac_static, the allocation-free variant of he_ct_pt_mac (its workspace is a fixed array inside
the library's device code): through the C ABI, against he_ct_pt_mac on the same inputs, bit for bit, on
calls in a row that shrink (the array keeps the last call's contents), and against the oracle."""
import numpy as np
import pytest

import oracle
from paper_1908_04172_amd import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def he():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1908_04172_amd import he as he_mod
    he_mod.lib()
    return he_mod


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).cuda()


def host(t):
    return t.cpu().numpy().view(np.uint64)


def layer_inputs(plan, q, N, seed):
    ct = wl.uniform_residues((plan.n_in, 2), q, N, seed)
    w = wl.uniform_residues((plan.n_pt,), q, 1, seed + 1)[..., 0]
    b = wl.uniform_residues((plan.n_out,), q, 1, seed + 2)[..., 0]
    return ct, w, b


def test_static_scratch_layer_calls_match_the_workspace_entry_point(he):
    c = wl.config(1)                                               # N = 2^12, two 30-bit limbs
    ctx = he.Context(c.log2N, c.q)
    # two fused layers in a row (MAC + bias + one rescale per output), the second smaller than the first
    for k, (K, M) in enumerate(((64, 16), (9, 5))):
        plan = wl.dense_plan(K, M)
        hp = ctx.plan(plan.n_in, plan.n_out, plan.n_pt, plan.off, plan.term_ct, plan.term_pt)
        assert 0 < hp.workspace_bytes(c.L, he.PT_SCALAR, he.RESCALE) <= he.STATIC_SCRATCH_BYTES
        ct, w, b = layer_inputs(plan, c.q, c.N, 900 + 10 * k)
        d_ct, d_w, d_b = dev(ct), dev(w), dev(b)
        out = torch.full((M, 2, c.L - 1, c.N), -1, dtype=torch.int64, device="cuda")
        ctx.ct_pt_mac_static(hp, d_ct, d_w, he.PT_SCALAR, out, bias=d_b, flags=he.RESCALE)
        torch.cuda.synchronize()
        first = out.clone()
        # once the runtime has loaded the kernels (their first launch), a call leaves the device's free memory as it was
        free_before = torch.cuda.mem_get_info()[0]
        out.fill_(-1)
        ctx.ct_pt_mac_static(hp, d_ct, d_w, he.PT_SCALAR, out, bias=d_b, flags=he.RESCALE)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before
        assert torch.equal(out, first)
        ref = ctx.ct_pt_mac(hp, d_ct, d_w, he.PT_SCALAR, bias=d_b, flags=he.RESCALE)
        assert torch.equal(out, ref)
        want, _ = oracle.layer(ct, c.q, ctx.psi, plan.off, plan.term_ct, plan.term_pt, w, oracle.PT_SCALAR, b)
        assert np.array_equal(host(out), want)


def test_static_scratch_on_a_convolution_and_with_accumulate(he):
    c = wl.config(2)                                               # N = 2^13, 60-bit + 3 x 40-bit limbs
    ctx = he.Context(c.log2N, c.q)
    for k, geometry in enumerate(((10, 10, 2, 3, 3, 5, 2, "same"), (6, 6, 1, 3, 3, 3, 1, "valid"))):
        plan = wl.conv_plan(*geometry)
        hp = ctx.plan(plan.n_in, plan.n_out, plan.n_pt, plan.off, plan.term_ct, plan.term_pt)
        ct, w, b = layer_inputs(plan, c.q, c.N, 950 + 10 * k)
        d_ct, d_w, d_b = dev(ct), dev(w), dev(b)
        out = torch.full((plan.n_out, 2, c.L, c.N), -1, dtype=torch.int64, device="cuda")
        ctx.ct_pt_mac_static(hp, d_ct, d_w, he.PT_SCALAR, out, bias=d_b)
        assert torch.equal(out, ctx.ct_pt_mac(hp, d_ct, d_w, he.PT_SCALAR, bias=d_b))
        want = oracle.mac(ct, c.q, plan.off, plan.term_ct, plan.term_pt, w, oracle.PT_SCALAR, b)
        assert np.array_equal(host(out), want)
        # adding the same sums once more (HE_ACCUMULATE), in both entry points
        ref = out.clone()
        ctx.ct_pt_mac_static(hp, d_ct, d_w, he.PT_SCALAR, out, flags=he.ACCUMULATE)
        ctx.ct_pt_mac(hp, d_ct, d_w, he.PT_SCALAR, flags=he.ACCUMULATE, out=ref)
        assert torch.equal(out, ref)
        twice = oracle.mac(ct, c.q, plan.off, plan.term_ct, plan.term_pt, w, oracle.PT_SCALAR)
        qa = np.array(c.q, dtype=object)[None, None, :, None]
        assert np.array_equal(host(out).astype(object), (want.astype(object) + twice.astype(object)) % qa)
    # polynomial plaintexts use no scratch memory at all without a rescale; with one, the accumulators
    plan = wl.dense_plan(5, 3)
    hp = ctx.plan(plan.n_in, plan.n_out, plan.n_pt, plan.off, plan.term_ct, plan.term_pt)
    ct = wl.uniform_residues((plan.n_in, 2), c.q, c.N, 990)
    wp = wl.uniform_residues((plan.n_pt,), c.q, c.N, 991)
    out = torch.empty((plan.n_out, 2, c.L - 1, c.N), dtype=torch.int64, device="cuda")
    ctx.ct_pt_mac_static(hp, dev(ct), dev(wp), he.PT_POLY, out, flags=he.RESCALE)
    want, _ = oracle.layer(ct, c.q, ctx.psi, plan.off, plan.term_ct, plan.term_pt, wp, oracle.PT_POLY, None)
    assert np.array_equal(host(out), want)


def test_static_scratch_refuses_what_does_not_fit(he):
    c = wl.config(2)
    ctx = he.Context(c.log2N, c.q)
    plan = wl.dense_plan(2, 80)                                    # 80 outputs x 512 KiB of accumulators = 40 MiB
    hp = ctx.plan(plan.n_in, plan.n_out, plan.n_pt, plan.off, plan.term_ct, plan.term_pt)
    assert hp.workspace_bytes(c.L, he.PT_SCALAR, he.RESCALE) > he.STATIC_SCRATCH_BYTES
    ct, w, b = layer_inputs(plan, c.q, c.N, 970)
    out = torch.empty((plan.n_out, 2, c.L - 1, c.N), dtype=torch.int64, device="cuda")
    with pytest.raises(he.HeError) as e:
        ctx.ct_pt_mac_static(hp, dev(ct), dev(w), he.PT_SCALAR, out, bias=dev(b), flags=he.RESCALE)
    assert e.value.status == -6
    # without the rescale only the weight table is needed, and the same plan runs
    full = torch.empty((plan.n_out, 2, c.L, c.N), dtype=torch.int64, device="cuda")
    ctx.ct_pt_mac_static(hp, dev(ct), dev(w), he.PT_SCALAR, full, bias=dev(b))
    assert np.array_equal(host(full), oracle.mac(ct, c.q, plan.off, plan.term_ct, plan.term_pt, w, oracle.PT_SCALAR, b))
    with pytest.raises(he.HeError) as e:                           # the usual argument checks still apply
        ctx.ct_pt_mac_static(hp, dev(ct), dev(w), he.PT_SCALAR, out, flags=he.RESCALE | he.ACCUMULATE)
    assert e.value.status == -1
