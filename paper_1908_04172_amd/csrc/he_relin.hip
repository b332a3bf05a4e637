// The x^2 activation on ciphertexts (Sec. "CryptoNets"; "Square" and "Relinearize" in the paper's table of
// operation runtimes): square a ciphertext and relinearise the result with a special prime (Sec.
// "Homomorphic Encryption": key switching by raising the modulus).  The ciphertext lives on limbs
// q_0..q_{l-1}, 1 <= l <= L-1; the context's last limb is the special prime P.  Working tensors have l+1
// limb positions: q_0..q_{l-1}, then P.  Steps, each a launch:
//   1. (d0, d1, d2) = (c0^2, 2 c0 c1, c1^2), slot-wise; d0, d1 go to the output, d2 to the workspace;
//   2. inverse NTT of d2: row j now holds the coefficients of [d2]_{q_j} in [0, q_j): RNS digit j;
//   3+4. every digit re-reduced modulo the other q_i and P and transformed under that limb: one launch of the
//      transform kernel in its digit-expansion form, l * l rows written from l rows read (digit j under limb j
//      is d2's own row, written by step 1);
//   5. acc_k = sum_j digit_j * evk[j][k], k = 0, 1, on all L limbs;
//   6. division of acc by P with rounding: Eq. (2) with P as the dropped limb, the rescale kernel as it is;
//   7. out_k = d_k + that.
// Steps 2, 3+4 and 6 are the library's transforms; this file adds the three slot-wise kernels around them.
#include "he_internal.h"

namespace {

// step 1: one thread = one slot of one limb of one ciphertext
// (d2 goes out twice: to d2 [n][l][N], which the inverse transform then turns into coefficients, and to its place
// among the expanded digits, digit j under limb j, where it needs no transform)
__global__ void __launch_bounds__(256) square_kernel(LimbTable lt, u32 l, u32 N, const u64* ct, size_t n, u64* out, u64* d2,
                                                     u64* digits) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n * l * N) return;
    const size_t k = idx % N, row = idx / N;  // row = ct * l + limb
    const u32 limb = (u32)(row % l);
    const size_t c_idx = row / l;
    const LimbConst& c = lt.c[limb];
    const u64 c0 = ct[((c_idx * 2) * l + limb) * N + k], c1 = ct[((c_idx * 2 + 1) * l + limb) * N + k];
    const u64 cross = mul_mod(c0, c1, c);
    out[((c_idx * 2) * l + limb) * N + k] = mul_mod(c0, c0, c);
    out[((c_idx * 2 + 1) * l + limb) * N + k] = add_mod(cross, cross, c.q);
    const u64 sq = mul_mod(c1, c1, c);
    d2[row * N + k] = sq;
    digits[(row * (l + 1) + limb) * N + k] = sq;
}

// step 5: one thread = one slot of one limb of one ciphertext, both components
// (L = l + 1 limb positions; `lt` has the special prime's constants at position l; the key is the top-level one,
// [..][2][key_limbs][N], in which the special prime is limb key_limbs - 1)
__global__ void __launch_bounds__(256) key_product_kernel(LimbTable lt, u32 l, u32 L, u32 key_limbs, u32 N, const u64* digits,
                                                          size_t n, const u64* evk, u64* acc) {
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
    acc[((c_idx * 2) * L + limb) * N + k] = reduce128((u64)(a0 >> 64), (u64)a0, c);
    acc[((c_idx * 2 + 1) * L + limb) * N + k] = reduce128((u64)(a1 >> 64), (u64)a1, c);
}

// step 7: out += down, both [n][2][l][N]
__global__ void __launch_bounds__(256) add_rows_kernel(LimbTable lt, u32 l, u32 N, u64* out, const u64* down, size_t rows) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= rows * N) return;
    const u32 limb = (u32)((idx / N) % l);
    out[idx] = add_mod(out[idx], down[idx], lt.c[limb].q);
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
    u64* down = digits;  // the digits are dead once the key product is taken
    const size_t per_ct = (size_t)l * N;
    const size_t b1 = ((size_t)n * per_ct + 255) / 256, b5 = ((size_t)n * L * N + 255) / 256, b7 = ((size_t)n * 2 * per_ct + 255) / 256;
    if (b1 > 0x7FFFFFFFull || b5 > 0x7FFFFFFFull || b7 > 0x7FFFFFFFull || (u64)n * l > 0x0FFFFFFFull) return HE_ERR_RANGE;
    LimbTable lt = ctx->limbs;
    lt.c[l] = ctx->limbs.c[ctx->L - 1];  // the special prime at the last position
    int rc;
    hipLaunchKernelGGL(square_kernel, dim3((u32)b1), dim3(256), 0, s, ctx->limbs, l, N, ct_in, (size_t)n, ct_out, d2, digits);
    HE_HIP(hipGetLastError());
    if ((rc = launch_ntt(ctx, l, d2, n, true, s)) != HE_OK) return rc;
    if ((rc = launch_ntt_spread(ctx, L, d2, digits, n * l, l, s)) != HE_OK) return rc;
    hipLaunchKernelGGL(key_product_kernel, dim3((u32)b5), dim3(256), 0, s, lt, l, L, ctx->L, N, digits, (size_t)n, evk, acc);
    HE_HIP(hipGetLastError());
    if ((rc = launch_rescale_drop(ctx, L, ctx->L - 1, acc, down, n, s)) != HE_OK) return rc;
    hipLaunchKernelGGL(add_rows_kernel, dim3((u32)b7), dim3(256), 0, s, ctx->limbs, l, N, ct_out, down, (size_t)n * 2 * l);
    HE_HIP(hipGetLastError());
    return HE_OK;
}
