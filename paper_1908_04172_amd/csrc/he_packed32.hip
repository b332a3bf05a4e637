// Packed 32-bit storage for limbs whose moduli are below 2^30: the paper's 32-bit optimisation
// (Sec. "Ciphertext-plaintext Multiplication": BarrettReduction64, Alg. 6, and the scalar multiply of
// Alg. 8) carried through to the memory system.  Residue tensors are uint32 [ct][2][limbs][N], half the
// bytes of the 64-bit form; a product of two residues fits 60 bits, so a MAC term is ONE 32x32+64-bit
// multiply-add into a single 64-bit sum (four into three sums in the 64-bit path), fifteen terms go by
// between two reductions, and a reduction is Alg. 6: one high product with floor(2^64 / q), one low
// product, one conditional subtraction.  The transforms keep a whole row (and, in the rescale, the
// dropped limb's coefficients beside it) in LDS.
#include <algorithm>

#include "he_internal.h"

namespace {

constexpr u32 TERMS_PER_REDUCTION = 15;  // r + 15 * (2^30 - 1)^2 < 2^64 for r < 2^30

__device__ __forceinline__ u32 barrett64(u64 z, const Limb32& c) { return ::barrett64(z, c.q, c.ratio); }

__device__ __forceinline__ u32 add_mod32(u32 a, u32 b, u32 q) {
    const u32 s = a + b;
    return s >= q ? s - q : s;
}

template <typename T>
__device__ __forceinline__ T uniform_load(const T* p) {  // read-only, workgroup-uniform data: a scalar load
    return *(const __attribute__((address_space(4))) T*)(p);
}

// ---------------------------------------------------------------------------------------------
// conversions between the two storage forms

__global__ void __launch_bounds__(256) pack32_kernel(const u64* in, u32* out, size_t count) {
    const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 2;
    if (i + 1 < count) {
        const ulonglong2 v = *reinterpret_cast<const ulonglong2*>(in + i);
        *reinterpret_cast<uint2*>(out + i) = make_uint2((u32)v.x, (u32)v.y);
    } else if (i < count) {
        out[i] = (u32)in[i];
    }
}

__global__ void __launch_bounds__(256) unpack32_kernel(const u32* in, u64* out, size_t count) {
    const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 2;
    if (i + 1 < count) {
        const uint2 v = *reinterpret_cast<const uint2*>(in + i);
        *reinterpret_cast<ulonglong2*>(out + i) = make_ulonglong2(v.x, v.y);
    } else if (i < count) {
        out[i] = in[i];
    }
}

// ---------------------------------------------------------------------------------------------
// Alg. 8 summed over a window, 32-bit moduli

constexpr u32 MAC32_THREADS = 256;
constexpr u32 MAC32_SLICE = 2 * MAC32_THREADS;  // residues of a row one workgroup covers (two per thread)

// wtab32[limb*wtab_elems + wbase + t*G + g] = pt[term_pt[off[out0+g] + t]][limb] for g < count, else 0: the
// scalar plaintexts of a group laid out in the order the MAC loop reads them (the plan's table offsets
// are shared with the 64-bit path; groups with the same plaintext indices share a table).
template <int G>
__global__ void __launch_bounds__(256) gather_weights32_kernel(const Tile* tiles, const u64* wbase, const u32* wowner, u32 n_tiles,
                                                               u32 limbs, const u32* off, const u32* term_pt, const u64* pt,
                                                               u32* wtab, u64 wtab_elems) {
    const u32 tile_i = blockIdx.x;
    if (tile_i >= n_tiles || !wowner[tile_i]) return;
    const Tile tile = tiles[tile_i];
    const u64 per_limb = (u64)tile.n_terms * G;
    u32* dst = wtab + wbase[tile_i];
    for (u64 i = threadIdx.x; i < per_limb * limbs; i += blockDim.x) {
        const u32 limb = (u32)(i / per_limb);
        const u64 rem = i % per_limb;
        const u32 t = (u32)(rem / G), g = (u32)(rem % G);
        dst[(u64)limb * wtab_elems + rem] = g < tile.count ? (u32)pt[(size_t)term_pt[off[tile.out0 + g] + t] * limbs + limb] : 0;
    }
}

// One thread = two adjacent residues of one (component, limb) row x a group of G outputs.
template <int G>
__global__ void __launch_bounds__(MAC32_THREADS)
mac_scalar32_kernel(Limb32Table lt, u32 limbs, u32 N, const Tile* tiles, u32 n_tiles, const u64* wbase, const u32* term_ct,
                    const u32* wtab, u64 wtab_elems, const u32* ct_in, const u64* bias, u32* out, u32 accumulate) {
    const u32 slices = N / MAC32_SLICE;
    u32 b = blockIdx.x;
    const u32 slice = b % slices; b /= slices;
    const u32 tile_i = b % n_tiles; b /= n_tiles;
    const u32 comp = b & 1;
    const u32 limb = b >> 1;
    const Limb32& c = lt.c[limb];
    const u32 K = uniform_load(&tiles[tile_i].n_terms), count = uniform_load(&tiles[tile_i].count);
    const u32 out0 = uniform_load(&tiles[tile_i].out0);
    const u32* tc = term_ct + uniform_load(&tiles[tile_i].term0);
    const u32* w = wtab + (u64)limb * wtab_elems + uniform_load(wbase + tile_i);
    const u32 pair = slice * MAC32_THREADS + threadIdx.x;
    const size_t ct_pairs = (size_t)limbs * N;  // uint2 elements per ciphertext (2 components x limbs x N / 2)
    const uint2* x_base = reinterpret_cast<const uint2*>(ct_in) + ((size_t)comp * limbs + limb) * (N / 2) + pair;
    u64 acc[G][2];
#pragma unroll
    for (int g = 0; g < G; g++) acc[g][0] = acc[g][1] = 0;
    u32 since = 0;
    // the next term's input and weights are requested before this term's multiply-adds, so that the loads
    // (the weights of a dense layer miss the scalar cache) are in flight while those run
    uint2 x_next = make_uint2(0, 0);
    u32 w_next[G];
#pragma unroll
    for (int g = 0; g < G; g++) w_next[g] = 0;
    if (K > 0) {
        x_next = x_base[(size_t)uniform_load(tc) * ct_pairs];
#pragma unroll
        for (int g = 0; g < G; g++) w_next[g] = uniform_load(w + g);
    }
    for (u32 t = 0; t < K; ++t) {
        const uint2 x = x_next;
        u32 wv[G];
#pragma unroll
        for (int g = 0; g < G; g++) wv[g] = w_next[g];
        const u32 tn = min(t + 1, K - 1);  // the last term asks for itself again: a repeat that is never used
        x_next = x_base[(size_t)uniform_load(tc + tn) * ct_pairs];
#pragma unroll
        for (int g = 0; g < G; g++) w_next[g] = uniform_load(w + (size_t)tn * G + g);
#pragma unroll
        for (int g = 0; g < G; g++) {
            acc[g][0] += (u64)x.x * wv[g];
            acc[g][1] += (u64)x.y * wv[g];
        }
        if (++since == TERMS_PER_REDUCTION && t + 1 < K) {
            since = 0;
#pragma unroll
            for (int g = 0; g < G; g++) {
                acc[g][0] = barrett64(acc[g][0], c);
                acc[g][1] = barrett64(acc[g][1], c);
            }
        }
    }
    const bool with_bias = bias != nullptr && comp == 0;  // Alg. 4: the bias goes to component 0 only
#pragma unroll
    for (int g = 0; g < G; g++) {
        if ((u32)g < count) {
            const u32 o = out0 + g;
            u32 r0 = barrett64(acc[g][0], c), r1 = barrett64(acc[g][1], c);
            if (with_bias) {
                const u32 bv = (u32)bias[(size_t)o * limbs + limb];
                r0 = add_mod32(r0, bv, c.q);
                r1 = add_mod32(r1, bv, c.q);
            }
            uint2* dst = reinterpret_cast<uint2*>(out) + (((size_t)o * 2 + comp) * limbs + limb) * (N / 2) + pair;
            if (accumulate) {  // HE_ACCUMULATE: add what the output holds (uniform branch)
                const uint2 old = *dst;
                r0 = add_mod32(r0, old.x, c.q);
                r1 = add_mod32(r1, old.y, c.q);
            }
            *dst = make_uint2(r0, r1);
        }
    }
}

// Alg. 7 summed, 32-bit moduli: one thread = two adjacent residues of one limb x G <= 4 outputs x both
// components; every plaintext residue is read once and used for c0 and c1.
template <int G>
__global__ void __launch_bounds__(MAC32_THREADS)
mac_poly32_kernel(Limb32Table lt, u32 limbs, u32 N, const Tile* tiles, u32 n_tiles, const u32* off, const u32* term_ct,
                  const u32* term_pt, const u32* pt, const u32* ct_in, const u64* bias, u32* out, u32 accumulate) {
    const u32 slices = N / MAC32_SLICE;
    u32 b = blockIdx.x;
    const u32 slice = b % slices; b /= slices;
    const u32 tile_i = b % n_tiles;
    const u32 limb = b / n_tiles;
    const Limb32& c = lt.c[limb];
    const Tile tile = tiles[tile_i];
    const u32 pair = slice * MAC32_THREADS + threadIdx.x;
    const size_t ct_pairs = (size_t)limbs * N;
    const size_t row_pairs = N / 2;
    const uint2* ct2 = reinterpret_cast<const uint2*>(ct_in);
    const uint2* pt2 = reinterpret_cast<const uint2*>(pt);
    u64 acc[G][2][2];
#pragma unroll
    for (int g = 0; g < G; g++) acc[g][0][0] = acc[g][0][1] = acc[g][1][0] = acc[g][1][1] = 0;
    u32 since = 0;
    for (u32 t = 0; t < tile.n_terms; ++t) {
        const size_t ci = term_ct[tile.term0 + t];
        const uint2 x0 = ct2[ci * ct_pairs + (size_t)limb * row_pairs + pair];
        const uint2 x1 = ct2[ci * ct_pairs + ((size_t)limbs + limb) * row_pairs + pair];
#pragma unroll
        for (int g = 0; g < G; g++) {
            if ((u32)g < tile.count) {
                const size_t pi = term_pt[off[tile.out0 + g] + t];
                const uint2 wv = pt2[(pi * limbs + limb) * row_pairs + pair];
                acc[g][0][0] += (u64)x0.x * wv.x;
                acc[g][0][1] += (u64)x0.y * wv.y;
                acc[g][1][0] += (u64)x1.x * wv.x;
                acc[g][1][1] += (u64)x1.y * wv.y;
            }
        }
        if (++since == TERMS_PER_REDUCTION && t + 1 < tile.n_terms) {
            since = 0;
#pragma unroll
            for (int g = 0; g < G; g++)
                for (int k = 0; k < 2; k++) {
                    acc[g][k][0] = barrett64(acc[g][k][0], c);
                    acc[g][k][1] = barrett64(acc[g][k][1], c);
                }
        }
    }
#pragma unroll
    for (int g = 0; g < G; g++) {
        if ((u32)g < tile.count) {
            const u32 o = tile.out0 + g;
            const u32 bv = bias ? (u32)bias[(size_t)o * limbs + limb] : 0;
            for (int k = 0; k < 2; k++) {
                u32 r0 = barrett64(acc[g][k][0], c), r1 = barrett64(acc[g][k][1], c);
                if (k == 0) {
                    r0 = add_mod32(r0, bv, c.q);
                    r1 = add_mod32(r1, bv, c.q);
                }
                uint2* dst = reinterpret_cast<uint2*>(out) + (((size_t)o * 2 + k) * limbs + limb) * row_pairs + pair;
                if (accumulate) {
                    const uint2 old = *dst;
                    r0 = add_mod32(r0, old.x, c.q);
                    r1 = add_mod32(r1, old.y, c.q);
                }
                *dst = make_uint2(r0, r1);
            }
        }
    }
}

// Alg. 3 / Alg. 4: component 0 += plaintext.  pt: u64 [n][limbs] residues (scalar) or u32 [n][limbs][N].
template <bool POLY>
__global__ void __launch_bounds__(256) add32_kernel(Limb32Table lt, u32 limbs, u32 N, u32* ct, size_t n, const void* pt) {
    const size_t quads = N / 4;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n * limbs * quads) return;
    const size_t k4 = i % quads, row = i / quads;  // row = ct * limbs + limb
    const u32 limb = (u32)(row % limbs);
    const size_t c_idx = row / limbs;
    const u32 q = lt.c[limb].q;
    uint4* p = reinterpret_cast<uint4*>(ct + ((c_idx * 2) * limbs + limb) * N) + k4;
    uint4 v = *p, a;
    if constexpr (POLY) {
        a = reinterpret_cast<const uint4*>(static_cast<const u32*>(pt) + row * N)[k4];
    } else {
        a.x = a.y = a.z = a.w = (u32) static_cast<const u64*>(pt)[row];
    }
    v.x = add_mod32(v.x, a.x, q);
    v.y = add_mod32(v.y, a.y, q);
    v.z = add_mod32(v.z, a.z, q);
    v.w = add_mod32(v.w, a.w, q);
    *p = v;
}

// ---------------------------------------------------------------------------------------------
// Negacyclic transforms of a row held in LDS (same root and output order as the 64-bit entry points:
// slot j holds the value at psi^(2*bitrev(j)+1)).  Harvey's lazy butterflies in 32 bits: forward values
// stay in [0, 4q), inverse values in [0, 2q); both need 4q < 2^32.  Two stages are taken per trip
// through LDS (four values per thread in registers), a single one when the number of stages is odd.
// The "lazy" transforms leave the last reduction (and, for the inverse, the factor N^-1) to the caller,
// who applies finish_forward / finish_inverse to each value as it consumes it.  Every thread of the
// workgroup must call; the caller has synchronised after filling `a`, and the transforms end with a
// barrier.

__device__ __forceinline__ void bfly32_fwd(u32& x, u32& y, uint2 w, u32 q, u32 two_q) {  // (X, Y) -> (X + W*Y, X - W*Y)
    const u32 u = x >= two_q ? x - two_q : x;
    const u32 v = shoup32(y, w.x, w.y, q);
    x = u + v;
    y = u - v + two_q;
}

__device__ __forceinline__ void bfly32_inv(u32& x, u32& y, uint2 w, u32 q, u32 two_q) {  // (X, Y) -> (X + Y, (X - Y)*W)
    const u32 s = x + y;
    const u32 d = x - y + two_q;
    x = s >= two_q ? s - two_q : s;
    y = shoup32(d, w.x, w.y, q);
}

__device__ __forceinline__ u32 finish_forward(u32 v, const Limb32& c) {  // [0, 4q) -> [0, q)
    v = v >= c.two_q ? v - c.two_q : v;
    return v >= c.q ? v - c.q : v;
}

__device__ __forceinline__ u32 finish_inverse(u32 v, const Limb32& c) {  // [0, 2q) -> times N^-1, in [0, q)
    v = shoup32(v, c.n_inv, c.n_inv_shoup, c.q);
    return v >= c.q ? v - c.q : v;
}

__device__ void ntt32_forward_lazy(u32* a, const uint2* tw, u32 N, const Limb32& c) {
    const u32 q = c.q, two_q = c.two_q;
    u32 m = 1, t = N >> 1, logt = 31 - __clz(t);
    while (m < N) {
        if (2 * m < N) {  // the stages with distances t and t/2
            const u32 h = t >> 1;
            for (u32 b = threadIdx.x; b < N / 4; b += blockDim.x) {
                const u32 i = b >> (logt - 1), j = b & (h - 1);
                const u32 p = (i << (logt + 1)) + j;
                u32 x0 = a[p], x1 = a[p + h], x2 = a[p + t], x3 = a[p + t + h];
                const uint2 w1 = tw[m + i];
                bfly32_fwd(x0, x2, w1, q, two_q);
                bfly32_fwd(x1, x3, w1, q, two_q);
                bfly32_fwd(x0, x1, tw[2 * m + 2 * i], q, two_q);
                bfly32_fwd(x2, x3, tw[2 * m + 2 * i + 1], q, two_q);
                a[p] = x0;
                a[p + h] = x1;
                a[p + t] = x2;
                a[p + t + h] = x3;
            }
            m <<= 2;
            t >>= 2;
            logt -= 2;
        } else {  // a last single stage (distance 1)
            for (u32 b = threadIdx.x; b < N / 2; b += blockDim.x) {
                u32 x = a[2 * b], y = a[2 * b + 1];
                bfly32_fwd(x, y, tw[m + b], q, two_q);
                a[2 * b] = x;
                a[2 * b + 1] = y;
            }
            m <<= 1;
        }
        __syncthreads();
    }
}

__device__ void ntt32_inverse_lazy(u32* a, const uint2* tw, u32 N, const Limb32& c) {
    const u32 q = c.q, two_q = c.two_q;
    u32 m = N >> 1, t = 1, logt = 0;  // m groups of butterflies at distance t
    while (m >= 1) {
        if (m >= 2) {  // the stages with distances t and 2t
            for (u32 b = threadIdx.x; b < N / 4; b += blockDim.x) {
                const u32 i = b >> logt, j = b & (t - 1);
                const u32 p = (i << (logt + 2)) + j;
                u32 x0 = a[p], x1 = a[p + t], x2 = a[p + 2 * t], x3 = a[p + 3 * t];
                bfly32_inv(x0, x1, tw[m + 2 * i], q, two_q);
                bfly32_inv(x2, x3, tw[m + 2 * i + 1], q, two_q);
                const uint2 w = tw[(m >> 1) + i];
                bfly32_inv(x0, x2, w, q, two_q);
                bfly32_inv(x1, x3, w, q, two_q);
                a[p] = x0;
                a[p + t] = x1;
                a[p + 2 * t] = x2;
                a[p + 3 * t] = x3;
            }
            m >>= 2;
            t <<= 2;
            logt += 2;
        } else {  // a last single stage (one group, distance N/2)
            for (u32 b = threadIdx.x; b < N / 2; b += blockDim.x) {
                u32 x = a[b], y = a[b + t];
                bfly32_inv(x, y, tw[1], q, two_q);
                a[b] = x;
                a[b + t] = y;
            }
            m = 0;
        }
        __syncthreads();
    }
}

template <bool INVERSE>
__global__ void __launch_bounds__(1024) ntt32_rows_kernel(Limb32Table lt, u32 limbs, u32 N, u32* data, const u32* tw_all) {
    extern __shared__ u32 lds32[];
    const size_t row_i = blockIdx.x;
    const u32 limb = (u32)(row_i % limbs);
    const Limb32& c = lt.c[limb];
    u32* row = data + row_i * N;
    const uint2* tw = reinterpret_cast<const uint2*>(tw_all) + (size_t)limb * N;
    for (u32 k = threadIdx.x; k < N; k += blockDim.x) lds32[k] = row[k];
    __syncthreads();
    if (INVERSE) {
        ntt32_inverse_lazy(lds32, tw, N, c);
        for (u32 k = threadIdx.x; k < N; k += blockDim.x) row[k] = finish_inverse(lds32[k], c);
    } else {
        ntt32_forward_lazy(lds32, tw, N, c);
        for (u32 k = threadIdx.x; k < N; k += blockDim.x) row[k] = finish_forward(lds32[k], c);
    }
}

// Rescale, Eq. (2) in RNS form, one workgroup per polynomial (ciphertext, component):
//   t = (INTT(x_last) + floor(p/2)) mod p, kept in LDS for all kept limbs;
//   out_i = (x_i - NTT_i((t mod q_i) - (floor(p/2) mod q_i))) * p^-1 mod q_i.
__global__ void __launch_bounds__(1024) rescale32_kernel(Limb32Table lt, Drop32Row drop, u32 limbs, u32 N, const u32* in, u32* out,
                                                         const u32* tw_fwd, const u32* tw_inv) {
    extern __shared__ u32 lds32[];
    u32* trow = lds32;      // t, coefficient form, in [0, p)
    u32* wrow = lds32 + N;  // the row being transformed
    const size_t poly = blockIdx.x;
    const u32 last = limbs - 1;
    const u32* src = in + poly * limbs * N;
    u32* dst = out + poly * (limbs - 1) * N;
    {
        const Limb32& c = lt.c[last];
        for (u32 k = threadIdx.x; k < N; k += blockDim.x) trow[k] = src[(size_t)last * N + k];
        __syncthreads();
        ntt32_inverse_lazy(trow, reinterpret_cast<const uint2*>(tw_inv) + (size_t)last * N, N, c);
        // (in the loops below every thread touches only the elements k = tid mod blockDim, as here)
        const u32 half = c.q >> 1;
        for (u32 k = threadIdx.x; k < N; k += blockDim.x) trow[k] = add_mod32(finish_inverse(trow[k], c), half, c.q);
    }
    for (u32 i = 0; i < last; i++) {
        const Limb32& c = lt.c[i];
        const Drop32 d = drop.d[i];
        for (u32 k = threadIdx.x; k < N; k += blockDim.x) {
            const u32 r = barrett64(trow[k], c);  // t mod q_i
            wrow[k] = r >= d.half_mod ? r - d.half_mod : r + c.q - d.half_mod;
        }
        __syncthreads();
        ntt32_forward_lazy(wrow, reinterpret_cast<const uint2*>(tw_fwd) + (size_t)i * N, N, c);
        for (u32 k = threadIdx.x; k < N; k += blockDim.x) {
            u32 corr = wrow[k];  // below 4q
            corr = corr >= c.two_q ? corr - c.two_q : corr;
            const u32 v = shoup32(src[(size_t)i * N + k] + c.two_q - corr, d.p_inv, d.p_inv_shoup, c.q);  // argument below 3q < 2^32
            dst[(size_t)i * N + k] = v >= c.q ? v - c.q : v;
        }
        // wrow is refilled by the next limb: each thread rewrites the elements it has just read
    }
}

// workgroup size of the transforms: two radix-4 groups per thread and trip (measured best of N/4, N/8, N/16)
u32 transform_threads(u32 N) { return std::min<u32>(1024, N / 8); }

}  // namespace

// ------------------------------------------------------------------------------------------------
// launchers (arguments are checked by the entry points)

int launch_pack32(he_ctx* ctx, const u64* in, u32* out, size_t count, hipStream_t s) {
    const size_t blocks = (count / 2 + 1 + 255) / 256;
    if (blocks > 0x7FFFFFFFull) return HE_ERR_RANGE;
    hipLaunchKernelGGL(pack32_kernel, dim3((u32)blocks), dim3(256), 0, s, in, out, count);
    HE_HIP(hipGetLastError());
    return HE_OK;
}

int launch_unpack32(he_ctx* ctx, const u32* in, u64* out, size_t count, hipStream_t s) {
    const size_t blocks = (count / 2 + 1 + 255) / 256;
    if (blocks > 0x7FFFFFFFull) return HE_ERR_RANGE;
    hipLaunchKernelGGL(unpack32_kernel, dim3((u32)blocks), dim3(256), 0, s, in, out, count);
    HE_HIP(hipGetLastError());
    return HE_OK;
}

template <int G>
static int launch_scalar32_class(he_ctx* ctx, const he_plan* plan, int cls, u32 limbs, const u32* ct_in, const u64* pt,
                                 const u64* bias, u32* out, u32* wtab, u32 accumulate, hipStream_t s) {
    const u32 begin = plan->class_begin_s[cls], count = plan->class_begin_s[cls + 1] - begin;
    if (count == 0) return HE_OK;
    const Tile* tiles = plan->tiles_s_dev + begin;
    const u64* wbase = plan->wbase_s_dev + begin;
    hipLaunchKernelGGL((gather_weights32_kernel<G>), dim3(count), dim3(256), 0, s, tiles, wbase, plan->wowner_s_dev + begin, count, limbs,
                       plan->off_dev, plan->term_pt_dev, pt, wtab, plan->wtab_elems);
    HE_HIP(hipGetLastError());
    const u64 blocks = (u64)count * limbs * 2 * (ctx->N / MAC32_SLICE);
    if (blocks > 0x7FFFFFFFull) return HE_ERR_RANGE;
    hipLaunchKernelGGL((mac_scalar32_kernel<G>), dim3((u32)blocks), dim3(MAC32_THREADS), 0, s, ctx->limbs32, limbs, ctx->N, tiles, count,
                       wbase, plan->term_ct_dev, wtab, plan->wtab_elems, ct_in, bias, out, accumulate);
    HE_HIP(hipGetLastError());
    return HE_OK;
}

template <int G>
static int launch_poly32_class(he_ctx* ctx, const he_plan* plan, int cls, u32 limbs, const u32* ct_in, const u32* pt, const u64* bias,
                               u32* out, u32 accumulate, hipStream_t s) {
    const u32 begin = plan->class_begin_p[cls], count = plan->class_begin_p[cls + 1] - begin;
    if (count == 0) return HE_OK;
    const u64 blocks = (u64)count * limbs * (ctx->N / MAC32_SLICE);
    if (blocks > 0x7FFFFFFFull) return HE_ERR_RANGE;
    hipLaunchKernelGGL((mac_poly32_kernel<G>), dim3((u32)blocks), dim3(MAC32_THREADS), 0, s, ctx->limbs32, limbs, ctx->N,
                       plan->tiles_p_dev + begin, count, plan->off_dev, plan->term_ct_dev, plan->term_pt_dev, pt, ct_in, bias, out, accumulate);
    HE_HIP(hipGetLastError());
    return HE_OK;
}

// the grid sizes launch_mac32 would use, checked without launching anything
int check_mac32_launch(he_ctx* ctx, const he_plan* plan, u32 limbs, int pt_kind) {
    for (int cls = 0; cls < 3; cls++) {
        const u64 count = pt_kind == HE_PT_SCALAR ? plan->class_begin_s[cls + 1] - plan->class_begin_s[cls]
                                                  : plan->class_begin_p[cls + 1] - plan->class_begin_p[cls];
        if (count * limbs * (pt_kind == HE_PT_SCALAR ? 2 : 1) * (ctx->N / MAC32_SLICE) > 0x7FFFFFFFull) return HE_ERR_RANGE;
    }
    return HE_OK;
}

int launch_mac32(he_ctx* ctx, const he_plan* plan, u32 limbs, const u32* ct_in, const void* pt, int pt_kind, const u64* bias,
                 u32* out, void* workspace, u32 accumulate, hipStream_t s) {
    int rc;
    if (pt_kind == HE_PT_SCALAR) {
        const u64* p = static_cast<const u64*>(pt);
        u32* wtab = static_cast<u32*>(workspace);
        if ((rc = launch_scalar32_class<1>(ctx, plan, 0, limbs, ct_in, p, bias, out, wtab, accumulate, s)) != HE_OK) return rc;
        if ((rc = launch_scalar32_class<4>(ctx, plan, 1, limbs, ct_in, p, bias, out, wtab, accumulate, s)) != HE_OK) return rc;
        if ((rc = launch_scalar32_class<16>(ctx, plan, 2, limbs, ct_in, p, bias, out, wtab, accumulate, s)) != HE_OK) return rc;
    } else {
        const u32* p = static_cast<const u32*>(pt);
        if ((rc = launch_poly32_class<1>(ctx, plan, 0, limbs, ct_in, p, bias, out, accumulate, s)) != HE_OK) return rc;
        if ((rc = launch_poly32_class<2>(ctx, plan, 1, limbs, ct_in, p, bias, out, accumulate, s)) != HE_OK) return rc;
        if ((rc = launch_poly32_class<4>(ctx, plan, 2, limbs, ct_in, p, bias, out, accumulate, s)) != HE_OK) return rc;
    }
    return HE_OK;
}

int launch_add32(he_ctx* ctx, u32 limbs, u32* ct, u32 n, const void* pt, int pt_kind, hipStream_t s) {
    const size_t total = (size_t)n * limbs * (ctx->N / 4);
    const size_t blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFull) return HE_ERR_RANGE;
    if (pt_kind == HE_PT_POLY)
        hipLaunchKernelGGL(add32_kernel<true>, dim3((u32)blocks), dim3(256), 0, s, ctx->limbs32, limbs, ctx->N, ct, (size_t)n, pt);
    else
        hipLaunchKernelGGL(add32_kernel<false>, dim3((u32)blocks), dim3(256), 0, s, ctx->limbs32, limbs, ctx->N, ct, (size_t)n, pt);
    HE_HIP(hipGetLastError());
    return HE_OK;
}

int launch_ntt32(he_ctx* ctx, u32 limbs, u32* data, u32 rows, bool inverse, hipStream_t s) {
    const size_t lds = (size_t)ctx->N * sizeof(u32);  // at most 64 KiB: the default limit
    const u32 threads = transform_threads(ctx->N);
    if (inverse)
        hipLaunchKernelGGL(ntt32_rows_kernel<true>, dim3(rows), dim3(threads), lds, s, ctx->limbs32, limbs, ctx->N, data, ctx->tw32_inv);
    else
        hipLaunchKernelGGL(ntt32_rows_kernel<false>, dim3(rows), dim3(threads), lds, s, ctx->limbs32, limbs, ctx->N, data, ctx->tw32_fwd);
    HE_HIP(hipGetLastError());
    return HE_OK;
}

int launch_rescale32(he_ctx* ctx, u32 limbs, const u32* in, u32* out, u32 n, hipStream_t s) {
    const size_t lds = (size_t)2 * ctx->N * sizeof(u32);  // up to 128 KiB
    static std::atomic<uint32_t> lds_allowed{0};
    if (lds > (64u << 10))
        if (int rc = allow_dynamic_lds((const void*)rescale32_kernel, lds, ctx->device, lds_allowed)) return rc;
    Drop32Row row = {};
    const u32 last = limbs - 1;
    for (u32 i = 0; i < last; ++i) {
        const DropConst& d = ctx->drop[last][i];
        const u64 qi = ctx->q[i];
        row.d[i].p_inv = (u32)d.p_inv;
        row.d[i].p_inv_shoup = (u32)((d.p_inv << 32) / qi);
        row.d[i].half_mod = (u32)d.half_mod;
    }
    hipLaunchKernelGGL(rescale32_kernel, dim3(n * 2), dim3(transform_threads(ctx->N)), lds, s, ctx->limbs32, row, limbs, ctx->N, in, out,
                       ctx->tw32_fwd, ctx->tw32_inv);
    HE_HIP(hipGetLastError());
    return HE_OK;
}
