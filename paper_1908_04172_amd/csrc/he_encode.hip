// General CKKS encoding (Alg. 1) and its inverse for gfx950: N/2 complex slots -> the integer polynomial whose values
// at the roots r_k = exp(i*pi*(2k+1)/N), k < N/2, are scale*z_k (and the conjugates at the conjugate
// roots) -> residues per limb.  The forward NTT of the rows follows as a separate launch.
//
// The interpolation is a complex FFT of half the ring size.  Half of the 2N-th roots of unity, those
// with exponent 1 mod 4, satisfy r^(N/2) = i, so on them m(r) = sum_{j < N/2} (m_j + i*m_{j+N/2}) r^j:
// the N real coefficients are the real and imaginary parts of the N/2 complex numbers
//     w_j = xi^-j * (2/N) * sum_kappa z'_kappa * e^(-2 pi i kappa j / (N/2)),   xi = exp(i*pi/N),
// where z'_kappa is the value wanted at xi^(4 kappa + 1): slot 2*kappa itself while 4 kappa + 1 < N,
// otherwise the conjugate of slot N - 2*kappa - 1 (whose own root is the conjugate of that one).
// One workgroup per vector; the FFT runs in LDS (N/2 complex doubles = 8N bytes, the same footprint
// as a transform of the NTT kernels), radix 2, decimation in frequency, in place.
#include "he_internal.h"

namespace {

struct cplx {
    double re, im;
};

__device__ __forceinline__ cplx cmul(cplx a, cplx b) { return cplx{a.re * b.re - a.im * b.im, a.re * b.im + a.im * b.re}; }

template <int LOGN>
__global__ void __launch_bounds__((1 << LOGN) / 16)
encode_vector_kernel(LimbTable lt, u32 limbs, const cplx* slots, double scale, const cplx* fft_tw, const cplx* twist,
                     u64* out) {
    constexpr u32 N = 1u << LOGN, n = N / 2, T = N / 16, LOGn = LOGN - 1;
    constexpr u32 PER = n / T;  // 8 values per thread
    extern __shared__ cplx buf[];
    const u32 tid = threadIdx.x;
    const cplx* z = slots + (size_t)blockIdx.x * n;
    const double f = scale / (double)n;
    for (u32 kappa = tid; kappa < n; kappa += T) {
        cplx v;
        if (4 * kappa + 1 < N) {
            v = z[2 * kappa];
        } else {
            v = z[N - 2 * kappa - 1];
            v.im = -v.im;
        }
        buf[kappa] = cplx{v.re * f, v.im * f};
    }
    __syncthreads();
    for (u32 s = 0; s < LOGn; s++) {
        const u32 half = n >> (s + 1);
        for (u32 b = tid; b < n / 2; b += T) {
            const u32 r = b & (half - 1);
            const u32 i = ((b >> (LOGn - 1 - s)) << (LOGn - s)) | r;  // block * 2*half + r
            const cplx a = buf[i], c = buf[i + half];
            buf[i] = cplx{a.re + c.re, a.im + c.im};
            buf[i + half] = cmul(cplx{a.re - c.re, a.im - c.im}, fft_tw[r << s]);
        }
        __syncthreads();
    }
    // position pos holds the output of index bitrev(pos): twist it, then put it where it belongs
    cplx w[PER];
    u32 at[PER];
#pragma unroll
    for (u32 k = 0; k < PER; k++) {
        const u32 pos = tid + k * T;
        at[k] = __brev(pos) >> (32 - LOGn);
        w[k] = cmul(buf[pos], twist[at[k]]);
    }
    __syncthreads();
#pragma unroll
    for (u32 k = 0; k < PER; k++) buf[at[k]] = w[k];
    __syncthreads();
    // coefficient j = round(Re w_j), coefficient j + N/2 = round(Im w_j); residues of every limb
    u64* rows = out + (size_t)blockIdx.x * limbs * N;
    for (u32 j = tid; j < n; j += T) {
        const cplx v = buf[j];
        u64 lo[HE_MAX_LIMBS], hi[HE_MAX_LIMBS];
        encode_one(v.re, 1.0, lt.c, limbs, lo);
        encode_one(v.im, 1.0, lt.c, limbs, hi);
        for (u32 i = 0; i < limbs; i++) {
            rows[(size_t)i * N + j] = lo[i];
            rows[(size_t)i * N + n + j] = hi[i];
        }
    }
}

template <int LOGN>
int launch_t(he_ctx* ctx, u32 limbs, const double* slots, u32 n, double scale, u64* out, hipStream_t s) {
    constexpr u32 N = 1u << LOGN;
    const size_t lds = (size_t)N * 8;
    static std::atomic<uint32_t> lds_allowed{0};
    if (int rc = allow_dynamic_lds((const void*)encode_vector_kernel<LOGN>, lds, ctx->device, lds_allowed)) return rc;
    hipLaunchKernelGGL((encode_vector_kernel<LOGN>), dim3(n), dim3(N / 16), lds, s, ctx->limbs, limbs,
                       reinterpret_cast<const cplx*>(slots), scale, reinterpret_cast<const cplx*>(ctx->fft_tw),
                       reinterpret_cast<const cplx*>(ctx->twist), out);
    HE_HIP(hipGetLastError());
    return HE_OK;
}

// ---------------------------------------------------------------------------------------------
// Decoding: the inverse map.  Per coefficient the residues are lifted to the integer of smallest
// magnitude by Garner's mixed-radix form  x = v_0 + v_1 q_0 + v_2 q_0 q_1 + ...  (v_i < q_i, modular
// arithmetic only); x > Q/2 is decided exactly by comparing digits with those of floor(Q/2), and then
// Q - x is formed digit by digit, so the conversion to double (Horner, from the top digit) never
// subtracts large numbers.  The slots are the values of the polynomial at the slot roots: the same
// half-size FFT with the opposite sign, preceded by the twist xi^j.
struct GarnerInv {
    u64 inv, inv_shoup;  // q_k^-1 mod q_i and its Shoup companion, at [i * HE_MAX_LIMBS + k]
};

// (LMAX: a compile-time bound on `limbs`, 8 or HE_MAX_LIMBS: the unrolled loops and the digit registers are that many)
template <int LMAX>
__device__ __forceinline__ double lift_centred(const u64* col, size_t limb_stride, u32 limbs, const LimbTable& lt,
                                               const GarnerInv* g, const u64* half_digits) {
    u64 v[LMAX];
#pragma unroll
    for (u32 i = 0; i < (u32)LMAX; i++) {
        if (i < limbs) {
            const LimbConst& c = lt.c[i];
            u64 t = col[i * limb_stride];
#pragma unroll
            for (u32 k = 0; k < i; k++) {
                const u64 vk = v[k] < c.q ? v[k] : reduce64(v[k], c);
                t = shoup_mul(sub_mod(t, vk, c.q), g[i * HE_MAX_LIMBS + k].inv, g[i * HE_MAX_LIMBS + k].inv_shoup, c.q);
            }
            v[i] = t;
        }
    }
    bool above = false, decided = false;
#pragma unroll
    for (int i = LMAX - 1; i >= 0; i--) {
        if ((u32)i < limbs && !decided && v[i] != half_digits[i]) {
            above = v[i] > half_digits[i];
            decided = true;
        }
    }
    if (above) {  // digits of Q - x = (Q - 1 - x) + 1
        bool carry = true;
#pragma unroll
        for (u32 i = 0; i < (u32)LMAX; i++) {
            if (i < limbs) {
                u64 d = lt.c[i].q - 1 - v[i];
                if (carry) {
                    d += 1;
                    carry = d == lt.c[i].q;
                    if (carry) d = 0;
                }
                v[i] = d;
            }
        }
    }
    double acc = 0.0;
#pragma unroll
    for (int i = LMAX - 1; i >= 0; i--)
        if ((u32)i < limbs) acc = acc * (double)lt.c[i].q + (double)v[i];
    return above ? -acc : acc;
}

template <int LOGN, int LMAX>
__global__ void __launch_bounds__((1 << LOGN) / 16)
decode_vector_kernel(LimbTable lt, u32 limbs, const u64* coef, double inv_scale, const GarnerInv* garner,
                     const u64* half_digits, const cplx* fft_tw, const cplx* twist, cplx* slots) {
    constexpr u32 N = 1u << LOGN, n = N / 2, T = N / 16, LOGn = LOGN - 1;
    constexpr u32 PER = n / T;
    extern __shared__ cplx buf[];
    const u32 tid = threadIdx.x;
    const u64* rows = coef + (size_t)blockIdx.x * limbs * N;
    for (u32 j = tid; j < n; j += T) {
        const double re = lift_centred<LMAX>(rows + j, N, limbs, lt, garner, half_digits) * inv_scale;
        const double im = lift_centred<LMAX>(rows + n + j, N, limbs, lt, garner, half_digits) * inv_scale;
        const cplx tw = twist[j];
        buf[j] = cmul(cplx{re, im}, cplx{tw.re, -tw.im});  // times xi^j
    }
    __syncthreads();
    for (u32 s = 0; s < LOGn; s++) {
        const u32 half = n >> (s + 1);
        for (u32 b = tid; b < n / 2; b += T) {
            const u32 r = b & (half - 1);
            const u32 i = ((b >> (LOGn - 1 - s)) << (LOGn - s)) | r;
            const cplx a = buf[i], c = buf[i + half];
            const cplx tw = fft_tw[r << s];
            buf[i] = cplx{a.re + c.re, a.im + c.im};
            buf[i + half] = cmul(cplx{a.re - c.re, a.im - c.im}, cplx{tw.re, -tw.im});
        }
        __syncthreads();
    }
    cplx w[PER];
    u32 at[PER];
#pragma unroll
    for (u32 k = 0; k < PER; k++) {
        const u32 pos = tid + k * T;
        at[k] = __brev(pos) >> (32 - LOGn);
        w[k] = buf[pos];
    }
    __syncthreads();
#pragma unroll
    for (u32 k = 0; k < PER; k++) buf[at[k]] = w[k];
    __syncthreads();
    // buf[kappa] is the value at xi^(4 kappa + 1): slot 2*kappa, or the conjugate of slot N - 2*kappa - 1
    cplx* z = slots + (size_t)blockIdx.x * n;
    for (u32 k = tid; k < n; k += T) {
        cplx v = (k & 1) ? buf[(N - k - 1) / 2] : buf[k / 2];
        if (k & 1) v.im = -v.im;
        z[k] = v;
    }
}

template <int LOGN>
int launch_decode_t(he_ctx* ctx, u32 limbs, const u64* coef, u32 n, double scale, double* slots, hipStream_t s) {
    constexpr u32 N = 1u << LOGN;
    const size_t lds = (size_t)N * 8;
    auto launch = [&](auto kernel, std::atomic<uint32_t>& lds_allowed) -> int {
        if (int rc = allow_dynamic_lds((const void*)kernel, lds, ctx->device, lds_allowed)) return rc;
        hipLaunchKernelGGL(kernel, dim3(n), dim3(N / 16), lds, s, ctx->limbs, limbs, coef, 1.0 / scale,
                           reinterpret_cast<const GarnerInv*>(ctx->garner), ctx->half_digits + (size_t)limbs * HE_MAX_LIMBS,
                           reinterpret_cast<const cplx*>(ctx->fft_tw), reinterpret_cast<const cplx*>(ctx->twist),
                           reinterpret_cast<cplx*>(slots));
        HE_HIP(hipGetLastError());
        return HE_OK;
    };
    static std::atomic<uint32_t> lds_allowed_8{0}, lds_allowed_all{0};
    if (limbs <= 8) return launch(decode_vector_kernel<LOGN, 8>, lds_allowed_8);
    return launch(decode_vector_kernel<LOGN, HE_MAX_LIMBS>, lds_allowed_all);
}

}  // namespace

int launch_decode_vector(he_ctx* ctx, u32 limbs, const u64* coef, u32 n, double scale, double* slots, hipStream_t s) {
    switch (ctx->log2N) {
        case 10: return launch_decode_t<10>(ctx, limbs, coef, n, scale, slots, s);
        case 11: return launch_decode_t<11>(ctx, limbs, coef, n, scale, slots, s);
        case 12: return launch_decode_t<12>(ctx, limbs, coef, n, scale, slots, s);
        case 13: return launch_decode_t<13>(ctx, limbs, coef, n, scale, slots, s);
        case 14: return launch_decode_t<14>(ctx, limbs, coef, n, scale, slots, s);
    }
    return HE_ERR_ARG;
}

int launch_encode_vector(he_ctx* ctx, u32 limbs, const double* slots, u32 n, double scale, u64* out, hipStream_t s) {
    switch (ctx->log2N) {
        case 10: return launch_t<10>(ctx, limbs, slots, n, scale, out, s);
        case 11: return launch_t<11>(ctx, limbs, slots, n, scale, out, s);
        case 12: return launch_t<12>(ctx, limbs, slots, n, scale, out, s);
        case 13: return launch_t<13>(ctx, limbs, slots, n, scale, out, s);
        case 14: return launch_t<14>(ctx, limbs, slots, n, scale, out, s);
    }
    return HE_ERR_ARG;
}
