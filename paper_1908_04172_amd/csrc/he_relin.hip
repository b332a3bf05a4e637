// The x^2 activation on ciphertexts (Sec. "CryptoNets"; "Square" and "Relinearize" in the paper's table of
// operation runtimes): square a ciphertext and relinearise the result with a special prime (Sec.
// "Homomorphic Encryption": key switching by raising the modulus).  The ciphertext lives on limbs
// q_0..q_{l-1}, 1 <= l <= L-1; the context's last limb is the special prime P.  Working tensors have l+1
// limb positions: q_0..q_{l-1}, then P.  With (d0, d1, d2) = (c0^2, 2 c0 c1, c1^2) slot-wise, four launches:
//   1. d2 and its inverse NTT in one kernel (the transform kernel squares the rows it loads): row j then holds the
//      coefficients of [d2]_{q_j} in [0, q_j), RNS digit j; the NTT-form d2 goes to its place among the digits;
//   2. every digit re-reduced modulo the other q_i and P and transformed under that limb: the transform kernel in
//      its digit-expansion form, l * l rows written from l rows read;
//   3. acc_k = P * d_k + sum_j digit_j * evk[j][k], k = 0, 1, on all l+1 limbs (d_k formed from c0, c1 on the spot);
//   4. division of acc by P with rounding: Eq. (2) with P as the dropped limb, the rescale kernel as it is.  P * d_k is
//      an exact multiple of P, so round(acc / P) = d_k + round(sum / P): the relinearised ciphertext, with no
//      addition of its own.
#include "he_internal.h"

namespace {

// step 3: one thread = one slot of one limb position of one ciphertext, both components
// (L = l + 1 limb positions; `lt` has the special prime's constants at position l, and `p_mod` its residues modulo
// the other limbs; the key is the top-level one, [..][2][key_limbs][N], in which the special prime is limb
// key_limbs - 1)
struct SpecialPrimeResidues {
    u64 r[HE_MAX_LIMBS];
};
__global__ void __launch_bounds__(256) key_product_kernel(LimbTable lt, SpecialPrimeResidues p_mod, u32 l, u32 L, u32 key_limbs, u32 N,
                                                          const u64* digits, size_t n, const u64* evk, const u64* ct, u64* acc) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n * L * N) return;
    const size_t k = idx % N, row = idx / N;  // row = ct * L + limb position
    const u32 limb = (u32)(row % L);
    const u32 key_limb = limb == l ? key_limbs - 1 : limb;
    const size_t c_idx = row / L;
    const LimbConst& c = lt.c[limb];
    // at most 15 products below 2^124 each: the sums fit 128 bits and are reduced once (Alg. 5)
    u128 a0 = 0, a1 = 0;
    for (u32 j = 0; j < l; ++j) {
        const u64 b = digits[((c_idx * l + j) * L + limb) * N + k];
        a0 += (u128)b * evk[(((size_t)j * 2) * key_limbs + key_limb) * N + k];
        a1 += (u128)b * evk[(((size_t)j * 2 + 1) * key_limbs + key_limb) * N + k];
    }
    u64 r0 = reduce128((u64)(a0 >> 64), (u64)a0, c), r1 = reduce128((u64)(a1 >> 64), (u64)a1, c);
    if (limb < l) {  // + P * (c0^2, 2 c0 c1); modulo P itself that is zero
        const u64 c0 = ct[((c_idx * 2) * l + limb) * N + k], c1 = ct[((c_idx * 2 + 1) * l + limb) * N + k];
        const u64 pc0 = mul_mod(c0, p_mod.r[limb], c);
        const u64 cross = mul_mod(pc0, c1, c);
        r0 = add_mod(r0, mul_mod(pc0, c0, c), c.q);
        r1 = add_mod(r1, add_mod(cross, cross, c.q), c.q);
    }
    acc[((c_idx * 2) * L + limb) * N + k] = r0;
    acc[((c_idx * 2 + 1) * L + limb) * N + k] = r1;
}

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

}  // namespace

size_t square_relin_workspace(const he_ctx* ctx, u32 l, u32 n) {
    const size_t row = (size_t)ctx->N * sizeof(u64), L = (size_t)l + 1;
    return align256(n * l * row) + align256(n * l * L * row) + align256(n * 2 * L * row);
}

int launch_square_relin(he_ctx* ctx, u32 l, const u64* ct_in, u32 n, const u64* evk, u64* ct_out, void* workspace, hipStream_t s) {
    const u32 L = l + 1, N = ctx->N;  // limb positions of the working tensors: q_0..q_{l-1}, P
    const size_t row = (size_t)N * sizeof(u64);
    char* ws = (char*)workspace;
    u64* d2 = (u64*)ws;
    ws += align256((size_t)n * l * row);
    u64* digits = (u64*)ws;
    ws += align256((size_t)n * l * L * row);
    u64* acc = (u64*)ws;
    const size_t b3 = ((size_t)n * L * N + 255) / 256;
    if (b3 > 0x7FFFFFFFull || (u64)n * l > 0x0FFFFFFFull) return HE_ERR_RANGE;
    LimbTable lt = ctx->limbs;
    lt.c[l] = ctx->limbs.c[ctx->L - 1];  // the special prime at the last position
    SpecialPrimeResidues p_mod = {};
    for (u32 i = 0; i < l; ++i) p_mod.r[i] = ctx->q[ctx->L - 1] % ctx->q[i];
    int rc;
    if ((rc = launch_ntt_square(ctx, l, ct_in, d2, digits, n, s)) != HE_OK) return rc;
    if ((rc = launch_ntt_spread(ctx, L, d2, digits, n * l, l, s)) != HE_OK) return rc;
    hipLaunchKernelGGL(key_product_kernel, dim3((u32)b3), dim3(256), 0, s, lt, p_mod, l, L, ctx->L, N, digits, (size_t)n, evk, ct_in, acc);
    HE_HIP(hipGetLastError());
    return launch_rescale_drop(ctx, L, ctx->L - 1, acc, ct_out, n, s);
}
