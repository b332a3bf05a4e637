/*
 * he_test.h -- test and measurement hooks of the library, kept apart from the product ABI of he.h:
 * the device arithmetic compiled for the host (for CPU-only tests of Alg. 5 / Alg. 6, the Shoup
 * products and the MAC accumulator), and the register-resident rate probes against which the
 * benchmark quotes the MAC and NTT kernels.  Nothing on the compute path calls these.
 */
#ifndef HE_TEST_H
#define HE_TEST_H

#include "he.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Host-side checks of the device arithmetic (the same inline functions the kernels use, compiled
 * for the host): a*b mod q by 128-bit Barrett reduction (Alg. 5), and the lazy Shoup product used
 * in the NTT butterflies.  For tests; no device needed.
 */
uint64_t he_host_mulmod(uint64_t a, uint64_t b, uint64_t q);
uint64_t he_host_reduce128(uint64_t hi, uint64_t lo, uint64_t q);
uint64_t he_host_shoup_mulmod(uint64_t y, uint64_t w, uint64_t q);
/* The unreduced Shoup product of the butterflies: congruent to y*w mod q for any 64-bit y, in [0, 2q)
 * with the exact quotient estimate (cheap_quotient = 0), in [0, 4q) with the cheap one (= 1). */
uint64_t he_host_shoup_lazy(uint64_t y, uint64_t w, uint64_t q, int cheap_quotient);
/* The accumulator the MAC kernels use, run on the host: sum of x[t]*w[t] (n terms) mod q. */
uint64_t he_host_mac_accumulate(const uint64_t* x, const uint64_t* w, size_t n, uint64_t q);
/* The same with the kernels' final step: (sum + addend) mod q for an addend below q (the bias of Alg. 4). */
uint64_t he_host_mac_accumulate_add(const uint64_t* x, const uint64_t* w, size_t n, uint64_t q, uint64_t addend);
/* The unreduced result that the MAC of a fused layer (he_ct_pt_mac with HE_RESCALE) leaves for the rescale kernel:
 * congruent to (sum of x[t]*w[t] + addend) modulo q and below 12q, for an addend below 2q. */
uint64_t he_host_mac_accumulate_lazy(const uint64_t* x, const uint64_t* w, size_t n, uint64_t q, uint64_t addend);
/* The three-product (Karatsuba) form of the MAC terms that the 16-output kernel uses on limbs that leave room
 * for it: the number of terms such sums can take for modulus q (0: the form is not used for q), and
 * (sum of x[t]*w[t] + addend) mod q computed that way for n terms (UINT64_MAX if n exceeds that number). */
uint32_t he_host_mac_three_product_terms(uint64_t q);
uint64_t he_host_mac_accumulate_three_products(const uint64_t* x, const uint64_t* w, size_t n, uint64_t q, uint64_t addend);
/* The forward negacyclic transform as the kernels run it on double-precision FMAs for moduli below 2^50 (the same
 * inline butterfly and reductions, compiled for the host; works on a host-only context): in host [N], integers of
 * magnitude at most q standing for residues of limb `limb`; out host [N], the canonical residues of the transform
 * (the order of he_ntt).  *max_over_q (may be NULL) receives the largest |value| / q that any butterfly produced.
 * HE_ERR_MODULUS if the limb's modulus is 2^50 or more, HE_ERR_RANGE if an input exceeds q in magnitude or an
 * intermediate value was not an integer below 2^53 (which the bounds the kernels rely on exclude). */
int he_host_ntt_forward_fp64(he_ctx* ctx, uint32_t limb, const int64_t* in, uint64_t* out, double* max_over_q);
/* The inverse transform the same way: in host [N], canonical residues in the order of he_ntt_fwd's output; out host [N],
 * the canonical coefficients (multiplied by N^-1).  *max_over_q: the largest |value| / q among the sums, differences
 * and products.  Errors as above (HE_ERR_RANGE also for an input that is not below q). */
int he_host_ntt_inverse_fp64(he_ctx* ctx, uint32_t limb, const uint64_t* in, uint64_t* out, double* max_over_q);
/* The two primitives of the packed 32-bit path, for q in [2, 2^30): BarrettReduction64 (Alg. 6), z mod q for
 * any 64-bit z; and the lazy 32-bit Shoup product, congruent to y*w mod q and in [0, 2q), for w < q and any
 * 32-bit y. */
uint32_t he_host_barrett64(uint64_t z, uint32_t q);
uint32_t he_host_shoup32(uint32_t y, uint32_t w, uint32_t q);

/*
 * The first kernel launches of he_ct_pt_mac(..., HE_RESCALE) on their own, for timing the two halves of a fused layer
 * separately: acc_out dev [n_out][2][limbs][N] receives the accumulators (sums + bias) as the fused call leaves them in
 * its workspace, where the kept limbs of scalar-plaintext sums are congruent to the result but not reduced below
 * the modulus; he_rescale(limbs, acc_out, ...) then yields what the fused call yields.  workspace: as for
 * he_ct_pt_mac with flags = 0.
 */
int he_test_mac_for_rescale(he_ctx* ctx, const he_plan* plan, uint32_t limbs, const uint64_t* ct_in, const uint64_t* pt, int pt_kind,
                            const uint64_t* bias, uint64_t* acc_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The transforms of limbs below 2^50 run on double-precision FMAs, those of larger limbs on integer butterflies; both
 * produce the same residues.  integer_only = 1 makes every later call on this context use the integer butterflies for
 * all limbs (for tests of those butterflies on such limbs, and for timing one arithmetic against the other);
 * integer_only = 0 restores the state a context is created in.  Not to be called while work of this context is being
 * enqueued from another thread.
 */
int he_test_integer_transforms(he_ctx* ctx, int integer_only);

/*
 * Measurement aid, not part of the compute path: the rate (operations per second, whole GPU) at
 * which this device runs one of the library's arithmetic primitives on register-resident data, with
 * the constants of limb `limb` of the context.  These are the integer-ALU ceilings against which
 * the MAC and NTT kernels' throughputs are quoted.  Allocates a small device buffer, runs on the
 * default stream and synchronises.  iters in [1, 2^20] loop iterations per thread (4096 gives a
 * run of a few milliseconds).
 */
enum {
    HE_RATE_MAD32 = 0,           /* one 32x32+64-bit multiply-add */
    HE_RATE_MAC_TERM = 1,        /* the four multiply-adds of one MAC term (folds and reduction excluded) */
    HE_RATE_SHOUP_EXACT = 2,     /* Shoup product, exact quotient estimate (result below 2q) */
    HE_RATE_SHOUP_CHEAP = 3,     /* Shoup product, cheap quotient estimate (result below 4q) */
    HE_RATE_BUTTERFLY_MODE0 = 4, /* forward butterfly for moduli up to 2^62 */
    HE_RATE_BUTTERFLY_MODE1 = 5, /* forward butterfly for moduli below 2^61 */
    HE_RATE_BUTTERFLY_MODE2 = 6, /* forward butterfly for moduli below 2^58 */
    HE_RATE_BUTTERFLY_INV = 7,   /* inverse butterfly for moduli below 2^61 */
    HE_RATE_MAC_TERM3 = 8,       /* the three multiply-adds of one MAC term in the three-product form */
    HE_RATE_BUTTERFLY_FP64 = 9,  /* forward butterfly on double-precision FMAs for moduli below 2^50, with the transform's
                                    share of reductions (both values once per four butterflies) */
    HE_RATE_BUTTERFLY_FP64_INV = 10 /* inverse butterfly the same way (both values once per four butterflies, the sum
                                    once more) */
};
int he_measure_rate(he_ctx* ctx, int kind, uint32_t limb, uint32_t iters, double* ops_per_s);

#ifdef __cplusplus
}
#endif
#endif /* HE_TEST_H */
