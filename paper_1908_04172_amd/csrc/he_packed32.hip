// Packed 32-bit storage for limbs whose moduli are below 2^30: the paper's 32-bit optimisation
// (Sec. "Ciphertext-plaintext Multiplication": BarrettReduction64, Alg. 6, and the scalar multiply of
// Alg. 8) carried through to the memory system.  Residue tensors are uint32 [ct][2][limbs][N], half the
// bytes of the 64-bit form; a product of two residues fits 60 bits, so a MAC term is ONE 32x32+64-bit
// multiply-add into a single 64-bit sum (four into three sums in the 64-bit path), fifteen terms go by
// between two reductions, and a reduction is Alg. 6: one high product with floor(2^64 / q), one low
// product, one conditional subtraction.  The transforms are the register-resident ones of the 64-bit path
// with 32-bit butterflies; the rescale keeps the dropped limb's coefficients in registers throughout.
#include <algorithm>

#include "he_internal.h"
#include "he_ntt_core.h"

namespace {

constexpr u32 TERMS_PER_REDUCTION = 15;  // r + 15 * (2^30 - 1)^2 < 2^64 for r < 2^49

// Between two runs of TERMS_PER_REDUCTION terms a sum is not reduced modulo q but folded at bit 48: the part above
// (16 bits) times 2^48 mod q goes back onto the part below, which leaves a congruent value below 2^48 + 2^46 for
// three instructions instead of the dozen of Alg. 6; the one reduction at the end takes any 64-bit value.
__device__ __forceinline__ u64 fold48(u64 z, const Limb32& c) { return (u64)(u32)(z >> 48) * c.pow48 + (z & 0xFFFFFFFFFFFFull); }

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

constexpr u32 GATHER32_BLOCKS = 16;  // workgroups that share the gathering of one group's table
constexpr u32 MAC32_BLOCK = 4;  // terms per unrolled block; an input is requested a block before its use
__host__ __device__ inline u32 padded_terms32(u32 n_terms) { return (n_terms + MAC32_BLOCK - 1) / MAC32_BLOCK * MAC32_BLOCK; }

// wtab32[limb*wtab_elems + wbase + t*G + g] = pt[term_pt[off[out0+g] + t]][limb] for g < count and t < n_terms, else 0,
// for t up to n_terms rounded up to whole blocks: the scalar plaintexts of a group laid out in the order the MAC
// loop reads them (the plan's table offsets are shared with the 64-bit path, whose entries are larger; groups with
// the same plaintext indices share a table).
template <int G>
__global__ void __launch_bounds__(256) gather_weights32_kernel(const Tile* tiles, const u64* wbase, const u32* wowner, u32 n_tiles,
                                                               u32 limbs, const u32* off, const u32* term_pt, const u64* pt,
                                                               u32* wtab, u64 wtab_elems) {
    const u32 tile_i = blockIdx.x / GATHER32_BLOCKS, sub = blockIdx.x % GATHER32_BLOCKS;
    if (tile_i >= n_tiles || !wowner[tile_i]) return;
    const Tile tile = tiles[tile_i];
    const u64 per_limb = (u64)padded_terms32(tile.n_terms) * G;
    u32* dst = wtab + wbase[tile_i];
    for (u64 i = (u64)sub * blockDim.x + threadIdx.x; i < per_limb * limbs; i += (u64)GATHER32_BLOCKS * blockDim.x) {
        const u32 limb = (u32)(i / per_limb);
        const u64 rem = i % per_limb;
        const u32 t = (u32)(rem / G), g = (u32)(rem % G);
        dst[(u64)limb * wtab_elems + rem] =
            g < tile.count && t < tile.n_terms ? (u32)pt[(size_t)term_pt[off[tile.out0 + g] + t] * limbs + limb] : 0;
    }
}

// One thread = two adjacent residues of one (component, limb) row x a group of G outputs.  Terms run in blocks of
// four (the terms that pad a group to whole blocks have zero weights and the last real term's input again); a ring
// of four inputs keeps each request a whole block of multiply-adds ahead of its use, and a term's G weights are
// requested (scalar loads) while the term before is multiplied.
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
    if (K > 0) {
        const u32 Kp = padded_terms32(K), last = K - 1;
        uint2 xq[MAC32_BLOCK];
#pragma unroll
        for (u32 j = 0; j < MAC32_BLOCK; j++) xq[j] = x_base[(size_t)uniform_load(tc + min(j, last)) * ct_pairs];
        u32 w_next[G];
#pragma unroll
        for (int g = 0; g < G; g++) w_next[g] = uniform_load(w + g);
        u32 since = 0;
        for (u32 t = 0; t < Kp; t += MAC32_BLOCK) {
#pragma unroll
            for (u32 j = 0; j < MAC32_BLOCK; j++) {
                const uint2 x = xq[j];
                xq[j] = x_base[(size_t)uniform_load(tc + min(t + MAC32_BLOCK + j, last)) * ct_pairs];
                u32 wv[G];
#pragma unroll
                for (int g = 0; g < G; g++) wv[g] = w_next[g];
                // (after the last term this reads the entry that follows the group's table: another table or the
                // padding at the end of the limb's part; never used)
#pragma unroll
                for (int g = 0; g < G; g++) w_next[g] = uniform_load(w + (size_t)(t + j + 1) * G + g);
#pragma unroll
                for (int g = 0; g < G; g++) {
                    acc[g][0] += (u64)x.x * wv[g];
                    acc[g][1] += (u64)x.y * wv[g];
                }
            }
            since += MAC32_BLOCK;
            if (since + MAC32_BLOCK > TERMS_PER_REDUCTION && t + MAC32_BLOCK < Kp) {
                since = 0;
#pragma unroll
                for (int g = 0; g < G; g++) {
                    acc[g][0] = fold48(acc[g][0], c);
                    acc[g][1] = fold48(acc[g][1], c);
                }
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
                    acc[g][k][0] = fold48(acc[g][k][0], c);
                    acc[g][k][1] = fold48(acc[g][k][1], c);
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
// Negacyclic transforms, register-resident like the 64-bit ones (he_ntt_core.h: sixteen residues per thread,
// four stages per pass, regrouping through the LDS, the same root and output order: slot j holds the value at
// psi^(2*bitrev(j)+1)).  Harvey's lazy butterflies in 32 bits: forward values stay in [0, 4q), inverse values
// in [0, 2q); both need 4q < 2^32, hence moduli below 2^30.  A 32-bit Shoup product is one high product and
// two multiply-adds (y*w, then - qh*q on top of it); as in the 64-bit butterflies the forward X + W*Y comes out
// of that chain itself.

// x - m if that is not negative, else x, for x < 2m < 2^32 (the difference wraps to a larger number exactly when x < m)
__device__ __forceinline__ u32 csub32(u32 x, u32 m) { return min(x, x - m); }

// base + y*w - floor(y*ws / 2^32)*q modulo 2^32: congruent to base + y*w, and below base + 2q
__device__ __forceinline__ u32 shoup32_add(u32 y, Twiddle32 t, u32 q, u32 base) {
    const u32 qh = mul_hi32(y, t.w_shoup);
    const u64 lo = mad_wide(y, t.w, base);
    return (u32)mad_wide(qh, 0u - q, lo);
}

__device__ __forceinline__ void bfly32_fwd(u32& x, u32& y, Twiddle32 t, const Limb32& c) {  // (X, Y) -> (X + W*Y, X - W*Y)
    const u32 u = csub32(x, c.two_q);
    x = shoup32_add(y, t, c.q, u);
    y = (u << 1) + c.two_q - x;  // U + 2q - W*Y
}

__device__ __forceinline__ void bfly32_inv(u32& x, u32& y, Twiddle32 t, const Limb32& c) {  // (X, Y) -> (X + Y, (X - Y)*W)
    const u32 s = x + y;
    const u32 d = x + c.two_q - y;
    x = csub32(s, c.two_q);
    y = shoup32_add(d, t, c.q, 0);
}

template <int LOGN, int P, bool INVERSE>
__device__ __forceinline__ void run_pass32(u32 (&a)[16], const PassTwiddles<LOGN, P, Twiddle32>& pt, const Limb32& c) {
    using S = PassShape<LOGN, P>;
#pragma unroll
    for (int kk = 0; kk < S::NST; kk++) {
        const int k = INVERSE ? S::NST - 1 - kk : kk;
        const int s = 4 * P + k;         // stage
        const int bit = S::NST - 1 - k;  // register-index bit that the stage pairs
#pragma unroll
        for (u32 e = 0; e < 16; e++) {
            if (e & (1u << bit)) continue;
            u32 &x = a[e], &y = a[e | (1u << bit)];
            if constexpr (INVERSE) {
                if (s == 0) {  // the last inverse stage, merged with the multiplication by N^-1
                    const u32 sum = x + y, dif = x + c.two_q - y;
                    x = shoup32_add(sum, Twiddle32{c.n_inv, c.n_inv_shoup}, c.q, 0);
                    y = shoup32_add(dif, Twiddle32{c.w1n_inv, c.w1n_inv_shoup}, c.q, 0);
                } else {
                    bfly32_inv(x, y, pt.t[S::slot(k, e)], c);
                }
            } else {
                bfly32_fwd(x, y, pt.t[S::slot(k, e)], c);
            }
        }
    }
}

// Registers in pass-0 order, below 4q -> registers in last-pass order, below 4q.
template <int LOGN>
__device__ __forceinline__ void ntt32_forward(u32 (&a)[16], const Twiddle32* tw, u32* lds, u32 tid, const Limb32& c) {
    using G = Geo<LOGN>;
    static_assert(G::NPASS >= 2 && G::NPASS <= 4, "two to four passes");
    {
        PassTwiddles<LOGN, 0, Twiddle32> t0;
        load_pass_twiddles<LOGN, 0>(t0, tw, tid);
        run_pass32<LOGN, 0, false>(a, t0, c);
    }
    {
        PassTwiddles<LOGN, 1, Twiddle32> t1;
        load_pass_twiddles<LOGN, 1>(t1, tw, tid);
        regroup<LOGN, 0, 1>(a, lds, tid);
        run_pass32<LOGN, 1, false>(a, t1, c);
    }
    if constexpr (G::NPASS > 2) {
        PassTwiddles<LOGN, 2, Twiddle32> t2;
        load_pass_twiddles<LOGN, 2>(t2, tw, tid);
        regroup<LOGN, 1, 2>(a, lds, tid);
        run_pass32<LOGN, 2, false>(a, t2, c);
    }
    if constexpr (G::NPASS > 3) {
        PassTwiddles<LOGN, 3, Twiddle32> t3;
        load_pass_twiddles<LOGN, 3>(t3, tw, tid);
        regroup<LOGN, 2, 3>(a, lds, tid);
        run_pass32<LOGN, 3, false>(a, t3, c);
    }
}

// Registers in last-pass order, below 2q -> registers in pass-0 order, below 2q, multiplied by N^-1.
template <int LOGN>
__device__ __forceinline__ void ntt32_inverse(u32 (&a)[16], const Twiddle32* tw, u32* lds, u32 tid, const Limb32& c) {
    using G = Geo<LOGN>;
    if constexpr (G::NPASS > 3) {
        PassTwiddles<LOGN, 3, Twiddle32> t3;
        load_pass_twiddles<LOGN, 3>(t3, tw, tid);
        run_pass32<LOGN, 3, true>(a, t3, c);
    }
    if constexpr (G::NPASS > 2) {
        PassTwiddles<LOGN, 2, Twiddle32> t2;
        load_pass_twiddles<LOGN, 2>(t2, tw, tid);
        if constexpr (G::NPASS > 3) regroup<LOGN, 3, 2>(a, lds, tid);
        run_pass32<LOGN, 2, true>(a, t2, c);
    }
    {
        PassTwiddles<LOGN, 1, Twiddle32> t1;
        load_pass_twiddles<LOGN, 1>(t1, tw, tid);
        if constexpr (G::NPASS > 2) regroup<LOGN, 2, 1>(a, lds, tid);
        run_pass32<LOGN, 1, true>(a, t1, c);
    }
    {
        PassTwiddles<LOGN, 0, Twiddle32> t0;
        load_pass_twiddles<LOGN, 0>(t0, tw, tid);
        regroup<LOGN, 1, 0>(a, lds, tid);
        run_pass32<LOGN, 0, true>(a, t0, c);
    }
}

// In-place transforms of `rows` rows of N residues, row r under limb r % limbs; a workgroup takes rows
// blockIdx.x, blockIdx.x + gridDim.x, ... and has its next row in flight while it finishes the current one.
template <int LOGN, bool INVERSE>
__global__ void __launch_bounds__(Geo<LOGN>::T) ntt32_rows_kernel(Limb32Table lt, u32 limbs, u32* data, const u32* tw_all, u32 rows) {
    using G = Geo<LOGN>;
    constexpr int PIN = INVERSE ? G::NPASS - 1 : 0, POUT = INVERSE ? 0 : G::NPASS - 1;
    extern __shared__ u32 lds32[];
    u32 a[16];
    {
        const u32* p = data + (size_t)blockIdx.x * G::N;
#pragma unroll
        for (u32 e = 0; e < 16; e++) a[e] = p[reg_index<LOGN, PIN>(threadIdx.x, e)];
    }
    for (u32 row = blockIdx.x; row < rows; row += gridDim.x) {
        const u32 tid = threadIdx.x;
        const u32 limb = row % limbs;
        const Limb32& c = lt.c[limb];
        const Twiddle32* tw = reinterpret_cast<const Twiddle32*>(tw_all) + (size_t)limb * G::N;
        u32 next[16];
#pragma unroll
        for (u32 e = 0; e < 16; e++) next[e] = 0;
        if (row + gridDim.x < rows) {  // sixteen registers: the next row travels while this one is transformed
            const u32* p = data + (size_t)(row + gridDim.x) * G::N;
#pragma unroll
            for (u32 e = 0; e < 16; e++) next[e] = p[reg_index<LOGN, PIN>(tid, e)];
        }
        if constexpr (INVERSE) {
            ntt32_inverse<LOGN>(a, tw, lds32, tid, c);
#pragma unroll
            for (u32 e = 0; e < 16; e++) a[e] = csub32(a[e], c.q);
        } else {
            ntt32_forward<LOGN>(a, tw, lds32, tid, c);
#pragma unroll
            for (u32 e = 0; e < 16; e++) a[e] = csub32(csub32(a[e], c.two_q), c.q);
        }
        // (the next row is waited for before the stores are issued: see the 64-bit transform kernel)
#pragma unroll
        for (u32 e = 0; e < 16; e++) asm volatile("" : "+v"(next[e])::"memory");
        u32* p = data + (size_t)row * G::N;
#pragma unroll
        for (u32 e = 0; e < 16; e++) p[reg_index<LOGN, POUT>(tid, e)] = a[e];
#pragma unroll
        for (u32 e = 0; e < 16; e++) a[e] = next[e];
    }
}

// Rescale, Eq. (2) in RNS form, one workgroup per polynomial (ciphertext, component):
//   t = (INTT(x_last) + floor(p/2)) mod p, sixteen residues per thread, kept in registers for all kept limbs;
//   out_i = (x_i - NTT_i((t mod q_i) - (floor(p/2) mod q_i))) * p^-1 mod q_i.
// Every input row is read once and every output row written once; the row x_i is requested before the transform
// of its correction and arrives while that runs.
template <int LOGN>
__global__ void __launch_bounds__(Geo<LOGN>::T) rescale32_kernel(Limb32Table lt, Drop32Row drop, u32 limbs, const u32* in, u32* out,
                                                                  const u32* tw_fwd, const u32* tw_inv) {
    using G = Geo<LOGN>;
    constexpr int LAST_PASS = G::NPASS - 1;
    extern __shared__ u32 lds32[];
    const size_t poly = blockIdx.x;
    const u32 tid = threadIdx.x;
    const u32 last = limbs - 1;
    const u32* src = in + poly * limbs * G::N;
    u32* dst = out + poly * (limbs - 1) * G::N;
    u32 t[16];
    {
        const Limb32& c = lt.c[last];
        const u32* row = src + (size_t)last * G::N;
#pragma unroll
        for (u32 e = 0; e < 16; e++) t[e] = row[reg_index<LOGN, LAST_PASS>(tid, e)];
        ntt32_inverse<LOGN>(t, reinterpret_cast<const Twiddle32*>(tw_inv) + (size_t)last * G::N, lds32, tid, c);
        const u32 half = c.q >> 1;
#pragma unroll
        for (u32 e = 0; e < 16; e++) t[e] = add_mod32(csub32(t[e], c.q), half, c.q);
    }
    for (u32 i = 0; i < last; i++) {
        const Limb32& c = lt.c[i];
        const Drop32 d = drop.d[i];
        const u32* xrow = src + (size_t)i * G::N;
        u32 x[16], a[16];
#pragma unroll
        for (u32 e = 0; e < 16; e++) x[e] = xrow[reg_index<LOGN, LAST_PASS>(tid, e)];
        // t < p is below 2*q_i unless p > 2*q_i (then Alg. 6 reduces it first); adding q_i - (h mod q_i) gives a
        // value congruent to t - h and below 3*q_i, which the forward transform takes
        const u32 minus_half = c.q - d.half_mod;
#pragma unroll
        for (u32 e = 0; e < 16; e++) a[e] = (d.reduce ? barrett64(t[e], c) : t[e]) + minus_half;
        ntt32_forward<LOGN>(a, reinterpret_cast<const Twiddle32*>(tw_fwd) + (size_t)i * G::N, lds32, tid, c);
        u32* orow = dst + (size_t)i * G::N;
#pragma unroll
        for (u32 e = 0; e < 16; e++) {
            const u32 corr = csub32(a[e], c.two_q);  // below 2q: x + 2q - corr is positive and below 3q < 2^32
            const u32 v = shoup32_add(x[e] + c.two_q - corr, Twiddle32{d.p_inv, d.p_inv_shoup}, c.q, 0);
            orow[reg_index<LOGN, LAST_PASS>(tid, e)] = csub32(v, c.q);
        }
    }
}

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
    hipLaunchKernelGGL((gather_weights32_kernel<G>), dim3(count * GATHER32_BLOCKS), dim3(256), 0, s, tiles, wbase, plan->wowner_s_dev + begin, count, limbs,
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
        if (pt_kind == HE_PT_SCALAR && count * GATHER32_BLOCKS > 0x7FFFFFFFull) return HE_ERR_RANGE;
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

template <int LOGN>
static int launch_ntt32_t(he_ctx* ctx, u32 limbs, u32* data, u32 rows, bool inverse, hipStream_t s) {
    using G = Geo<LOGN>;
    const size_t lds = (size_t)G::N * sizeof(u32);
    // as many workgroups as stay resident at once, each looping over its share of the rows
    const u32 per_cu = (u32)std::max<size_t>(1, std::min<size_t>((160u << 10) / lds, 2048 / G::T));
    const u32 grid = std::min<u32>(rows, 256 * per_cu);
    if (inverse) {
        static std::atomic<uint32_t> checked{0};
        if (int rc = allow_dynamic_lds((const void*)ntt32_rows_kernel<LOGN, true>, lds, ctx->device, checked, true)) return rc;
        hipLaunchKernelGGL((ntt32_rows_kernel<LOGN, true>), dim3(grid), dim3(G::T), lds, s, ctx->limbs32, limbs, data, ctx->tw32_inv, rows);
    } else {
        static std::atomic<uint32_t> checked{0};
        if (int rc = allow_dynamic_lds((const void*)ntt32_rows_kernel<LOGN, false>, lds, ctx->device, checked, true)) return rc;
        hipLaunchKernelGGL((ntt32_rows_kernel<LOGN, false>), dim3(grid), dim3(G::T), lds, s, ctx->limbs32, limbs, data, ctx->tw32_fwd, rows);
    }
    HE_HIP(hipGetLastError());
    return HE_OK;
}

int launch_ntt32(he_ctx* ctx, u32 limbs, u32* data, u32 rows, bool inverse, hipStream_t s) {
    switch (ctx->log2N) {
        case 10: return launch_ntt32_t<10>(ctx, limbs, data, rows, inverse, s);
        case 11: return launch_ntt32_t<11>(ctx, limbs, data, rows, inverse, s);
        case 12: return launch_ntt32_t<12>(ctx, limbs, data, rows, inverse, s);
        case 13: return launch_ntt32_t<13>(ctx, limbs, data, rows, inverse, s);
        case 14: return launch_ntt32_t<14>(ctx, limbs, data, rows, inverse, s);
    }
    return HE_ERR_ARG;
}

template <int LOGN>
static int launch_rescale32_t(he_ctx* ctx, u32 limbs, const Drop32Row& row, const u32* in, u32* out, u32 n, hipStream_t s) {
    using G = Geo<LOGN>;
    const size_t lds = (size_t)G::N * sizeof(u32);
    static std::atomic<uint32_t> checked{0};
    if (int rc = allow_dynamic_lds((const void*)rescale32_kernel<LOGN>, lds, ctx->device, checked, true)) return rc;
    hipLaunchKernelGGL((rescale32_kernel<LOGN>), dim3(n * 2), dim3(G::T), lds, s, ctx->limbs32, row, limbs, in, out, ctx->tw32_fwd,
                       ctx->tw32_inv);
    HE_HIP(hipGetLastError());
    return HE_OK;
}

int launch_rescale32(he_ctx* ctx, u32 limbs, const u32* in, u32* out, u32 n, hipStream_t s) {
    Drop32Row row = {};
    const u32 last = limbs - 1;
    for (u32 i = 0; i < last; ++i) {
        const DropConst& d = ctx->drop[last][i];
        const u64 qi = ctx->q[i];
        row.d[i].p_inv = (u32)d.p_inv;
        row.d[i].p_inv_shoup = (u32)((d.p_inv << 32) / qi);
        row.d[i].half_mod = (u32)d.half_mod;
        row.d[i].reduce = d.reduce_mode == 2;
    }
    switch (ctx->log2N) {
        case 10: return launch_rescale32_t<10>(ctx, limbs, row, in, out, n, s);
        case 11: return launch_rescale32_t<11>(ctx, limbs, row, in, out, n, s);
        case 12: return launch_rescale32_t<12>(ctx, limbs, row, in, out, n, s);
        case 13: return launch_rescale32_t<13>(ctx, limbs, row, in, out, n, s);
        case 14: return launch_rescale32_t<14>(ctx, limbs, row, in, out, n, s);
    }
    return HE_ERR_ARG;
}
