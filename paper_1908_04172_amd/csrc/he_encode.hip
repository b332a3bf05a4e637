// General CKKS encoding (Alg. 1) for gfx950: N/2 complex slots -> the integer polynomial whose values
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

}  // namespace

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
