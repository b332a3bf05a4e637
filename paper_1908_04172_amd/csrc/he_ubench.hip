// Register-resident rates of the library's own arithmetic on this GPU: the vector-ALU ceilings that
// the kernels' throughputs are quoted against.  Each thread runs CHAINS independent dependency chains
// of one primitive with no memory traffic inside the timed loop; the grid fills every SIMD with as
// many waves as the real kernels keep resident.  A measurement aid: nothing on the compute path
// calls this file.
#include "he_internal.h"
#include "../../include/he_test.h"

namespace {

constexpr int CHAINS = 8;
constexpr u32 BLOCKS = 256 * 16, THREADS = 256;

template <int KIND>
__global__ void __launch_bounds__(THREADS) rate_kernel(LimbTable lt, u32 limb, u32 iters, u64 w, u64 w_shoup, u64* sink) {
    const LimbConst& c = lt.c[limb];
    const u32 gid = blockIdx.x * THREADS + threadIdx.x;
    u64 x[CHAINS], y[CHAINS];
    u32 xa[CHAINS], xb[CHAINS];
    MacAcc acc[CHAINS];
#pragma unroll
    for (int i = 0; i < CHAINS; i++) {
        x[i] = ((u64)gid * 0x9E3779B97F4A7C15ull + i) % c.q;
        y[i] = ((u64)gid * 0xC2B2AE3D27D4EB4Full + 7 * i + 1) % c.q;
        acc_clear(acc[i]);
        split_operand(x[i], c, xa[i], xb[i]);
    }
    const Twiddle t{w, w_shoup};
    // operands of the double-precision butterflies
    const double q_f = (double)c.q;
    const TwiddleF tf{fp_centred(w % c.q, c.q)};
    double fx[CHAINS], fy[CHAINS];
#pragma unroll
    for (int i = 0; i < CHAINS; i++) {
        fx[i] = fp_centred(x[i], c.q);
        fy[i] = fp_centred(y[i], c.q);
    }
    const u64 below_q = (1ull << c.mu_shift) - 1;  // mu_shift = bit length of q, minus 1
    u32 wa, wb;
    split_operand(w, c, wa, wb);
    const u32 ws = wa + wb;
    u32 ta = xa[0], tb = xb[0], ts = ta + tb;
    for (u32 it = 0; it < iters; it++) {
        if constexpr (KIND == HE_RATE_MAC_TERM || KIND == HE_RATE_MAC_TERM3) {  // the next term's input residue
            ta = ta * 0x9E3779B1u + 1u;
            tb ^= ta >> 7;
            ts = ta + tb;
        }
#pragma unroll
        for (int i = 0; i < CHAINS; i++) {
            if constexpr (KIND == HE_RATE_MAD32) {
                x[i] = (u64)(u32)x[i] * (u32)w + x[i];
            } else if constexpr (KIND == HE_RATE_MAC_TERM) {
                // the four multiply-adds of one MAC term into the three running sums; the periodic
                // folds and the final reduction are not part of the ceiling (the sums may wrap here,
                // which only changes the discarded values).  As in the kernels, the chains of a thread
                // are outputs that share the input residue of the term (ta, tb: renewed once per
                // iteration, below) and have a plaintext residue each.
                acc_mac(acc[i], ta, tb, wa + i, wb + i);
            } else if constexpr (KIND == HE_RATE_MAC_TERM3) {
                // the three-product form of a term (lo += xa*wa, mid += (xa+xb)*(wa+wb), hi += xb*wb): the sum
                // wa + wb comes with the weights, xa + xb is formed once per term for all outputs
                acc[i].lo += (u64)ta * (wa + i);
                acc[i].mid += (u64)ts * (ws + 2 * i);
                acc[i].hi += (u64)tb * (wb + i);
            } else if constexpr (KIND == HE_RATE_SHOUP_EXACT) {
                x[i] = shoup_mul_lazy(x[i], w, w_shoup, c.q);
            } else if constexpr (KIND == HE_RATE_SHOUP_CHEAP) {
                x[i] = shoup_mul_lazy4(x[i], w, w_shoup, c.q);
            } else if constexpr (KIND == HE_RATE_BUTTERFLY_MODE0) {
                bfly_fwd<0>(x[i], y[i], t, c);
            } else if constexpr (KIND == HE_RATE_BUTTERFLY_MODE1) {
                bfly_fwd<1>(x[i], y[i], t, c);
            } else if constexpr (KIND == HE_RATE_BUTTERFLY_MODE2) {
                // without conditional subtraction the values grow by 4q per butterfly (a transform has
                // at most 14 stages): both are masked back below q every 8 iterations, four 32-bit ANDs
                // per 8 butterflies
                bfly_fwd<2>(x[i], y[i], t, c);
            } else if constexpr (KIND == HE_RATE_BUTTERFLY_INV) {
                bfly_inv<1>(x[i], y[i], t, c);
            } else if constexpr (KIND == HE_RATE_BUTTERFLY_FP64) {
                bfly_fwd_f(fx[i], fy[i], tf, q_f, c.q_inv_f);
            } else if constexpr (KIND == HE_RATE_BUTTERFLY_FP64_INV) {
                bfly_inv_f(fx[i], fy[i], tf, q_f, c.q_inv_f);
            }
        }
        if constexpr (KIND == HE_RATE_BUTTERFLY_FP64 || KIND == HE_RATE_BUTTERFLY_FP64_INV) {
            // the reductions a transform spends on four stages: every value once, in the inverse the sums once more
            if ((it & 3) == 3) {
#pragma unroll
                for (int i = 0; i < CHAINS; i++) {
                    fx[i] = fp_reduce(fx[i], q_f, c.q_inv_f);
                    fy[i] = fp_reduce(fy[i], q_f, c.q_inv_f);
                }
            }
            if constexpr (KIND == HE_RATE_BUTTERFLY_FP64_INV) {
                if ((it & 3) == 1) {
#pragma unroll
                    for (int i = 0; i < CHAINS; i++) fx[i] = fp_reduce(fx[i], q_f, c.q_inv_f);
                }
            }
        }
        if constexpr (KIND == HE_RATE_BUTTERFLY_MODE2) {
            if ((it & 7) == 7) {
#pragma unroll
                for (int i = 0; i < CHAINS; i++) {
                    x[i] &= below_q;
                    y[i] &= below_q;
                }
            }
        }
    }
    u64 s = 0;
#pragma unroll
    for (int i = 0; i < CHAINS; i++)
        s += x[i] + y[i] + acc[i].lo + acc[i].mid + acc[i].hi + __builtin_bit_cast(u64, fx[i]) + __builtin_bit_cast(u64, fy[i]);
    sink[gid] = s;
}

template <int KIND>
int run_rate(he_ctx* ctx, u32 limb, u32 iters, double* ops_per_s) {
    const LimbConst& c = ctx->limbs.c[limb];
    const u64 w = c.n_inv;  // any fixed residue with its Shoup companion at hand
    const u64 w_shoup = c.n_inv_shoup;
    u64* sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = HE_ERR_DEVICE;
    float best = 0.f;
    if (hipMalloc((void**)&sink, (size_t)BLOCKS * THREADS * sizeof(u64)) != hipSuccess) goto done;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) goto done;
    for (int rep = 0; rep < 4; rep++) {  // the first repetition warms up
        if (hipEventRecord(e0, nullptr) != hipSuccess) goto done;
        hipLaunchKernelGGL((rate_kernel<KIND>), dim3(BLOCKS), dim3(THREADS), 0, nullptr, ctx->limbs, limb, iters, w, w_shoup, sink);
        if (hipEventRecord(e1, nullptr) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) goto done;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) goto done;
        if (rep > 0 && (best == 0.f || ms < best)) best = ms;
    }
    if (hipGetLastError() != hipSuccess || best <= 0.f) goto done;
    *ops_per_s = (double)BLOCKS * THREADS * CHAINS * (double)iters / (best * 1e-3);
    rc = HE_OK;
done:
    (void)hipGetLastError();
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (sink) (void)hipFree(sink);
    return rc;
}

}  // namespace

int launch_rate(he_ctx* ctx, int kind, u32 limb, u32 iters, double* ops_per_s) {
    switch (kind) {
        case HE_RATE_MAD32: return run_rate<HE_RATE_MAD32>(ctx, limb, iters, ops_per_s);
        case HE_RATE_MAC_TERM: return run_rate<HE_RATE_MAC_TERM>(ctx, limb, iters, ops_per_s);
        case HE_RATE_SHOUP_EXACT: return run_rate<HE_RATE_SHOUP_EXACT>(ctx, limb, iters, ops_per_s);
        case HE_RATE_SHOUP_CHEAP: return run_rate<HE_RATE_SHOUP_CHEAP>(ctx, limb, iters, ops_per_s);
        case HE_RATE_BUTTERFLY_MODE0: return run_rate<HE_RATE_BUTTERFLY_MODE0>(ctx, limb, iters, ops_per_s);
        case HE_RATE_BUTTERFLY_MODE1: return run_rate<HE_RATE_BUTTERFLY_MODE1>(ctx, limb, iters, ops_per_s);
        case HE_RATE_BUTTERFLY_MODE2: return run_rate<HE_RATE_BUTTERFLY_MODE2>(ctx, limb, iters, ops_per_s);
        case HE_RATE_BUTTERFLY_INV: return run_rate<HE_RATE_BUTTERFLY_INV>(ctx, limb, iters, ops_per_s);
        case HE_RATE_MAC_TERM3: return run_rate<HE_RATE_MAC_TERM3>(ctx, limb, iters, ops_per_s);
        case HE_RATE_BUTTERFLY_FP64: return run_rate<HE_RATE_BUTTERFLY_FP64>(ctx, limb, iters, ops_per_s);
        case HE_RATE_BUTTERFLY_FP64_INV: return run_rate<HE_RATE_BUTTERFLY_FP64_INV>(ctx, limb, iters, ops_per_s);
    }
    return HE_ERR_ARG;
}
