// Modular arithmetic on 64-bit residues for gfx950's vector ALU: 32-bit integer multiply-adds, and for moduli
// below 2^50 the double-precision FMAs of the transforms (last section).  Every function is
// __host__ __device__ so that the host-side check entry points run exactly the code the
// kernels run.  Moduli are primes below 2^62.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint64_t u64;
typedef uint32_t u32;
typedef unsigned __int128 u128;

#define HE_HD __host__ __device__ __forceinline__

// Per-limb constants, computed once per context on the host.
struct LimbConst {
    u64 q;
    u64 ratio_hi, ratio_lo;  // floor(2^128 / q): the Barrett ratio of Alg. 5
    u64 two_q;
    u64 n_inv, n_inv_shoup;        // N^-1 mod q and its Shoup companion
    u64 w1n_inv, w1n_inv_shoup;    // (psi^-brv(1)) * N^-1: last inverse butterfly merged with N^-1
    u64 split_mask;   // 2^split_bits - 1
    u32 split_bits;   // where MAC operands are cut in two (see MacAcc)
    u32 fold_every;   // MAC terms the partial sums take between two acc_fold calls
    u32 reduce_every; // MAC terms the accumulator takes between two reductions mod q
    u32 narrow;       // 1: accumulated values stay below 2^(63 + bit length of q): one-word Barrett applies
    u64 mu;           // floor(2^(63 + bit length of q) / q), in (2^63, 2^64)
    u32 mu_shift;     // bit length of q, minus 1
    u32 ntt_mode;     // how lazily the butterflies reduce: 0 for q >= 2^61, 1 for q >= 2^58, else 2 (see the butterflies at the end of this file)
    u64 neg_two_q, four_q, neg_four_q;  // 2^64 - 2q, 4q mod 2^64, 2^64 - 4q (4q is used only when it fits)
    u32 kara_terms;   // MAC terms whose three-product sums (see acc_uncross) fit 64 bits and the one-word Barrett; 0: never
    u32 mac_lazy;     // 1: the rescale kernel can combine a MAC result that is only congruent to the sum and below 12q
                      // with its transformed correction without leaving 64 bits (depends on q, the butterfly mode and N)
    u32 fp_ok;        // 1: q < 2^50, the forward transform can run on double-precision FMAs (see bfly_fwd_f)
    u32 pad;
    double q_inv_f;   // 1 / q, rounded to nearest
    u64 pow64, pow64_shoup;  // 2^64 mod q and its Shoup companion (acc_reduce_lazy)
};

HE_HD u64 mul_hi64(u64 a, u64 b) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __umul64hi(a, b);
#else
    return (u64)(((u128)a * b) >> 64);
#endif
}

HE_HD u64 add_mod(u64 a, u64 b, u64 q) {  // a, b < q
    u64 s = a + b;
    return s >= q ? s - q : s;
}

HE_HD u64 sub_mod(u64 a, u64 b, u64 q) {  // a, b < q
    return a >= b ? a - b : a + q - b;
}

// x - m if that is not negative, else x, for x < 2m <= 2^63: the difference wraps past 2^63 exactly
// when x < m.  neg_m = 2^64 - m.
HE_HD u64 sub_if_ge(u64 x, u64 neg_m) {
    const u64 t = x + neg_m;
    return (int32_t)(t >> 32) < 0 ? x : t;
}

// Barrett reduction of a 128-bit value z = hi:lo by a modulus below 2^62 (Alg. 5).  With
// r = floor(2^128/q) = rh:rl, floor(z*r / 2^128) is the true quotient or one less.  The estimate
// used here, hi*rh + floor(lo*rh / 2^64) + floor(hi*rl / 2^64), leaves out the product lo*rl and the
// carry between the two middle products, each worth at most one more, so it is short of the true
// quotient by at most 3 and z - estimate*q lies in [0, 4q), which fits 64 bits; only the low 64 bits
// of the estimate matter for that difference.
HE_HD u64 reduce128(u64 hi, u64 lo, const LimbConst& c) {
    u64 qe = hi * c.ratio_hi + mul_hi64(lo, c.ratio_hi) + mul_hi64(hi, c.ratio_lo);
    u64 r = lo - qe * c.q;
    r = r >= c.two_q ? r - c.two_q : r;
    return r >= c.q ? r - c.q : r;
}

HE_HD u64 reduce64(u64 z, const LimbConst& c) { return reduce128(0, z, c); }

HE_HD u64 mul_mod(u64 a, u64 b, const LimbConst& c) {
    u128 p = (u128)a * b;
    return reduce128((u64)(p >> 64), (u64)p, c);
}

// a*b + c as one 32x32+64-bit multiply-add.  On the device the result is pinned to a 64-bit register
// pair, so that a chain of these whose upper halves are never used still compiles to one instruction
// per link instead of a separate multiply and add.
HE_HD u64 mad_wide(u32 a, u32 b, u64 c) {
    u64 r = (u64)a * b + c;
#if defined(__HIP_DEVICE_COMPILE__)
    asm("" : "+v"(r));
#endif
    return r;
}

HE_HD u32 mul_hi32(u32 a, u32 b) { return (u32)(((u64)a * b) >> 32); }

// base + y*w - qh*q modulo 2^64 on 32-bit pieces, as base + y*w + qh*(2^64 - q): the two products that reach
// the low word chain through one accumulator that starts from `base`, the four that reach only the high
// word through another.  (A butterfly passes its other operand as `base` and so gets X + W*Y out of the
// multiply-add chain itself, with no addition of its own.)
HE_HD u64 shoup_remainder_add(u64 y, u64 w, u64 qh, u64 q, u64 base) {
    const u32 y0 = (u32)y, y1 = (u32)(y >> 32), w0 = (u32)w, w1 = (u32)(w >> 32);
    const u32 h0 = (u32)qh, h1 = (u32)(qh >> 32);
    const u64 nq = 0 - q;
    const u32 n0 = (u32)nq, n1 = (u32)(nq >> 32);
    u64 cross = mad_wide(y0, w1, 0);
    cross = mad_wide(y1, w0, cross);
    cross = mad_wide(h0, n1, cross);
    cross = mad_wide(h1, n0, cross);
    u64 e = (u64)y0 * w0 + base;
    e = (u64)h0 * n0 + e;
    u32 hi = (u32)(e >> 32) + (u32)cross;
#if defined(__HIP_DEVICE_COMPILE__)
    asm("" : "+v"(hi));  // one 32-bit add into the high word, not a 64-bit add of a shifted pair
#endif
    return ((u64)hi << 32) | (u32)e;
}

HE_HD u64 shoup_remainder(u64 y, u64 w, u64 qh, u64 q) { return shoup_remainder_add(y, w, qh, q, 0); }

// The quotient estimates of the Shoup product y*w with w' = floor(w * 2^64 / q): the exact one,
// floor(y*w' / 2^64), and the cheap one, short of it by at most 2 (see shoup_mul_lazy4).
HE_HD u64 shoup_quotient(u64 y, u64 w_shoup) {
    const u32 y0 = (u32)y, y1 = (u32)(y >> 32), p0 = (u32)w_shoup, p1 = (u32)(w_shoup >> 32);
    const u64 b = (u64)y0 * p1 + mul_hi32(y0, p0);
    const u64 c = (u64)y1 * p0 + (u32)b;
    return (u64)y1 * p1 + (b >> 32) + (c >> 32);
}
HE_HD u64 shoup_quotient_cheap(u64 y, u64 w_shoup) {
    const u32 y0 = (u32)y, y1 = (u32)(y >> 32), p0 = (u32)w_shoup, p1 = (u32)(w_shoup >> 32);
    return (u64)y1 * p1 + mul_hi32(y0, p1) + mul_hi32(y1, p0);
}

// Shoup product with a fixed operand w < q and w' = floor(w * 2^64 / q): for ANY 64-bit y the
// result is congruent to y*w and lies in [0, 2q) (Harvey's lazy form); needs q < 2^63.  The
// quotient estimate qh = floor(y*w' / 2^64) is exact here.
HE_HD u64 shoup_mul_lazy(u64 y, u64 w, u64 w_shoup, u64 q) { return shoup_remainder(y, w, shoup_quotient(y, w_shoup), q); }

// The same product with a cheaper quotient estimate: y1*p1 + floor(y0*p1 / 2^32) + floor(y1*p0 / 2^32)
// leaves out the product y0*p0 and the fractions of the two middle products, so it is short of
// floor(y*w' / 2^64) by at most 2 and the result lies in [0, 4q).  For ANY 64-bit y; needs q < 2^62.
HE_HD u64 shoup_mul_lazy4(u64 y, u64 w, u64 w_shoup, u64 q) { return shoup_remainder(y, w, shoup_quotient_cheap(y, w_shoup), q); }

HE_HD u64 shoup_mul(u64 y, u64 w, u64 w_shoup, u64 q) {
    u64 r = shoup_mul_lazy(y, w, w_shoup, q);
    return r >= q ? r - q : r;
}

// ---------------------------------------------------------------------------------------------
// Alg. 2 on one value: [round(value * scale)]_{q_i} for the first `limbs` limbs (shared by the
// scalar encoder's kernel and host entry point and by the general encoder, which passes its
// already scaled coefficients with scale 1).  False (and all-ones residues) for a non-finite product.

HE_HD bool encode_one(double value, double scale, const LimbConst* lc, u32 limbs, u64* out) {
    const double v = value * scale;
    const double mag = v < 0 ? -v : v;
    if (!(mag <= 1.7976931348623157e308)) {  // NaN or infinity
        for (u32 i = 0; i < limbs; ++i) out[i] = ~0ull;
        return false;
    }
    const bool negative = v < 0;
    for (u32 i = 0; i < limbs; ++i) {
        const LimbConst& c = lc[i];
        u64 r;
        if (mag < 9223372036854775808.0) {
            const double whole = trunc(mag);
            u64 z = (u64)whole;
            if (mag - whole >= 0.5) z += 1;  // mag - whole is exact; halves go away from zero
            r = reduce64(z, c);
        } else {
            // mag = m * 2^e exactly, m a 53-bit integer, e >= 11
            u64 bits;
            __builtin_memcpy(&bits, &mag, sizeof bits);
            const u64 m = (bits & 0xFFFFFFFFFFFFFull) | (1ull << 52);
            u32 e = (u32)(bits >> 52) - 1075u;
            u64 pow2 = 1, base = 2;
            for (; e; e >>= 1) {
                if (e & 1) pow2 = mul_mod(pow2, base, c);
                base = mul_mod(base, base, c);
            }
            r = mul_mod(reduce64(m, c), pow2, c);
        }
        out[i] = (negative && r) ? c.q - r : r;
    }
    return true;
}

// ---------------------------------------------------------------------------------------------
// MAC accumulator.  Both operands of a product are cut at bit s = LimbConst::split_bits (about half
// the modulus width): x = xa + xb*2^s, w = wa + wb*2^s with all four pieces below 2^32, and
//   value = lo + mid*2^s + hi*2^(2s),   lo += xa*wa,  mid += xa*wb + xb*wa,  hi += xb*wb.
// Each piece product is below 2^(2s) <= 2^62, so a term is four 32x32+64-bit multiply-adds with no
// carries between the three sums.  Every LimbConst::fold_every terms the sums are renormalised
// (acc_fold), every LimbConst::reduce_every terms the value is reduced mod q (acc_restart); both
// periods are derived from q on the host so that no 64-bit sum can wrap.
struct MacAcc {
    u64 lo, mid, hi;
};

HE_HD void acc_clear(MacAcc& a) { a.lo = a.mid = a.hi = 0; }

HE_HD void split_operand(u64 v, const LimbConst& c, u32& va, u32& vb) {
    va = (u32)(v & c.split_mask);
    vb = (u32)(v >> c.split_bits);
}

HE_HD void acc_mac(MacAcc& a, u32 xa, u32 xb, u32 wa, u32 wb) {
    a.lo += (u64)xa * wa;
    a.mid += (u64)xa * wb;
#if defined(__HIP_DEVICE_COMPILE__)
    asm("" : "+v"(a.mid));  // keep the two products as two multiply-adds into `mid`
#endif
    a.mid += (u64)xb * wa;
    a.hi += (u64)xb * wb;
}

// The three-product form of a term (Karatsuba) adds xa*wa to lo, xb*wb to hi and (xa+xb)*(wa+wb) to mid;
// this turns such sums into the plain ones (mid = the cross terms xa*wb + xb*wa), once, when they are read out.
HE_HD void acc_uncross(MacAcc& a) { a.mid -= a.lo + a.hi; }

HE_HD void acc_fold(MacAcc& a, const LimbConst& c) {  // push the high parts of lo and mid upwards
    a.mid += a.lo >> c.split_bits;
    a.lo &= c.split_mask;
    a.hi += a.mid >> c.split_bits;
    a.mid &= c.split_mask;
}

// The accumulated value mod q.  After a fold lo, mid < 2^s, so the value is
// (lo | mid << s | hi << 2s) in its low word and hi >> (64 - 2s) in its high word (2s <= 62).
// Narrow limbs (value < 2^(63+b), b the bit length of q) take a one-word Barrett step: with
// x1 = floor(value / 2^(b-1)) < 2^64 and mu = floor(2^(63+b) / q), floor(x1 * mu / 2^64) is short
// of the true quotient by at most 3, like the estimate in reduce128.
HE_HD u64 acc_reduce(MacAcc a, const LimbConst& c) {
    acc_fold(a, c);
    const u32 s2 = 2 * c.split_bits;
    const u64 lo = a.lo | (a.mid << c.split_bits) | (a.hi << s2);
    const u64 hi = a.hi >> (64 - s2);
    if (c.narrow) {
        const u64 x1 = (hi << (64 - c.mu_shift)) | (lo >> c.mu_shift);
        u64 r = lo - mul_hi64(x1, c.mu) * c.q;
        r = r >= c.two_q ? r - c.two_q : r;
        return r >= c.q ? r - c.q : r;
    }
    return reduce128(hi, lo, c);
}

// (accumulated value + addend) mod q for an addend below q (the bias of Alg. 4, or 0), for limbs with
// LimbConst::narrow set and q < 2^61.  The one-word Barrett step of acc_reduce with the high product
// x1*mu / 2^64 taken from three 32-bit products only (x1h*muh + hi32(x1l*muh) + hi32(x1h*mul)), which
// is short of the full product by at most 2 more: the remainder lies in [0, 6q), the addend brings it
// below 7q, and three conditional subtractions (4q, 2q, q) finish.  8q fits 64 bits and 4q is below
// 2^63, as sub_if_ge needs.
HE_HD u64 acc_reduce_add(MacAcc a, u64 addend, const LimbConst& c) {
    acc_fold(a, c);
    const u32 s2 = 2 * c.split_bits;
    const u64 lo = a.lo | (a.mid << c.split_bits) | (a.hi << s2);
    const u64 hi = a.hi >> (64 - s2);
    const u64 x1 = (hi << (64 - c.mu_shift)) | (lo >> c.mu_shift);
    const u32 xl = (u32)x1, xh = (u32)(x1 >> 32), ml = (u32)c.mu, mh = (u32)(c.mu >> 32);
    const u64 qe = (u64)xh * mh + mul_hi32(xl, mh) + mul_hi32(xh, ml);
    // lo - qe*q modulo 2^64, as lo + qe*(2^64 - q) on 32-bit pieces
    const u64 nq = 0 - c.q;
    const u32 n0 = (u32)nq, n1 = (u32)(nq >> 32), e0 = (u32)qe, e1 = (u32)(qe >> 32);
    u64 cross = mad_wide(e0, n1, 0);
    cross = mad_wide(e1, n0, cross);
    const u64 low = (u64)e0 * n0 + lo;
    u32 top = (u32)(low >> 32) + (u32)cross;
#if defined(__HIP_DEVICE_COMPILE__)
    asm("" : "+v"(top));
#endif
    u64 r = (((u64)top << 32) | (u32)low) + addend;
    r = sub_if_ge(r, c.neg_four_q);
    r = sub_if_ge(r, c.neg_two_q);
    return sub_if_ge(r, 0 - c.q);
}

// The sums taken to a value that is only CONGRUENT to (accumulated value + addend) modulo q and lies below 12q,
// for limbs with LimbConst::narrow set and an addend below 2q: what the MAC leaves for the rescale kernel, which
// takes any representative that small (see LimbConst::mac_lazy).  The sums are used as they are, not folded:
// with b the bit length of q and s the cut, x1 = (hi << (2s-b+1)) + (mid >> (b-1-s)) + (lo >> (b-1)) is
// floor(value / 2^(b-1)) or up to 2 less and fits 64 bits; the one-word Barrett quotient of acc_reduce_add from
// it is short of the true quotient by at most 3 + 3 + 2, so the remainder, taken modulo 2^64 from the low word
// lo + (mid << s) + (hi << 2s) with the addend as the start of the multiply-add chain, is below 9q + 2q.
HE_HD u64 acc_reduce_add_lazy(const MacAcc& a, u64 addend, const LimbConst& c) {
    const u32 s = c.split_bits, sh = c.mu_shift;
    const u64 x1 = (a.hi << (2 * s - sh)) + (a.mid >> (sh - s)) + (a.lo >> sh);
    const u32 xl = (u32)x1, xh = (u32)(x1 >> 32), ml = (u32)c.mu, mh = (u32)(c.mu >> 32);
    const u64 qe = (u64)xh * mh + mul_hi32(xl, mh) + mul_hi32(xh, ml);
    const u64 low_word = a.lo + (a.mid << s) + (a.hi << (2 * s)) + addend;
    const u64 nq = 0 - c.q;
    const u32 n0 = (u32)nq, n1 = (u32)(nq >> 32), e0 = (u32)qe, e1 = (u32)(qe >> 32);
    u64 cross = mad_wide(e0, n1, 0);
    cross = mad_wide(e1, n0, cross);
    const u64 low = (u64)e0 * n0 + low_word;
    u32 top = (u32)(low >> 32) + (u32)cross;
#if defined(__HIP_DEVICE_COMPILE__)
    asm("" : "+v"(top));
#endif
    return ((u64)top << 32) | (u32)low;
}

// The same for the other limbs (moduli below 2^62): two lazy Shoup products, below 4q each, plus the addend
// (below 2q): below 10q.
HE_HD u64 acc_reduce_lazy(const MacAcc& a, u64 addend, const LimbConst& c) {
    // the value lo + mid * 2^s + hi * 2^(2s) as two words (it is below 2^128; the sums are used as they are)
    const u32 s = c.split_bits;
    const u64 mid_lo = a.mid << s, hi_lo = a.hi << (2 * s);
    const u64 t = a.lo + mid_lo;
    const u64 low = t + hi_lo;
    const u64 high = (a.mid >> (64 - s)) + (a.hi >> (64 - 2 * s)) + (u64)(t < mid_lo) + (u64)(low < hi_lo);
    // low + high * 2^64 = low * 1 + high * (2^64 mod q), each as a lazy Shoup product (below 4q; the companion of 1
    // is floor(2^64 / q)), the addend and the first product being the starting values of the multiply-add chains
    const u64 r0 = shoup_remainder_add(low, 1, shoup_quotient_cheap(low, c.ratio_hi), c.q, addend);
    return shoup_remainder_add(high, c.pow64, shoup_quotient_cheap(high, c.pow64_shoup), c.q, r0);
}

HE_HD void acc_restart(MacAcc& a, const LimbConst& c) {  // reduce in place and keep accumulating
    u64 r = acc_reduce(a, c);
    a.lo = r & c.split_mask;
    a.mid = r >> c.split_bits;
    a.hi = 0;
}

// ---------------------------------------------------------------------------------------------
// 32-bit moduli (below 2^30), the primitives of the packed path.

// Alg. 6 (BarrettReduction64): z mod q for a 64-bit z, ratio = floor(2^64 / q).  The estimate
// floor(z * ratio / 2^64) is the quotient or one less, so one conditional subtraction finishes.
HE_HD u32 barrett64(u64 z, u32 q, u64 ratio) {
    const u64 est = mul_hi64(z, ratio);
    const u32 r = (u32)z - (u32)est * q;  // below 2q < 2^31: the low words suffice
    return r >= q ? r - q : r;
}

// y * w mod q up to one q: w < q with ws = floor(w * 2^32 / q), any y below 2^32; the result is in [0, 2q).
HE_HD u32 shoup32(u32 y, u32 w, u32 ws, u32 q) { return y * w - (u32)(((u64)y * ws) >> 32) * q; }

// ---------------------------------------------------------------------------------------------
// NTT butterflies (Harvey's lazy forms with Shoup multiplication by a precomputed twiddle).
struct Twiddle {
    typedef u64 raw __attribute__((ext_vector_type(2)));  // a table entry as one 16-byte load
    u64 w, w_shoup;  // W and floor(W * 2^64 / q)
};
struct Twiddle32 {
    typedef u32 raw __attribute__((ext_vector_type(2)));
    u32 w, w_shoup;  // W and floor(W * 2^32 / q), for the packed 32-bit transforms
};

// How lazily the butterflies reduce depends on the room the modulus leaves in 64 bits
// (LimbConst::ntt_mode):
//   mode 0, q < 2^62: Harvey's butterflies as published: forward values in [0, 4q), inverse in [0, 2q),
//           Shoup products with the exact quotient estimate (result below 2q).
//   mode 1, q < 2^61: the Shoup products take the cheap quotient estimate (result below 4q); forward
//           values in [0, 8q), inverse in [0, 4q), one conditional subtraction of 4q per butterfly.
//   mode 2, q < 2^58: forward butterflies without any conditional subtraction: both outputs exceed
//           the larger input by less than 4q, so canonical inputs stay below (1 + 4*log2N)*q <= 57q
//           through all stages.  (Inverse butterflies add their inputs, which would double the
//           bound per stage, so the inverse transform runs as in mode 1.)

// Forward butterfly: (X, Y) -> (X + W*Y, X - W*Y).  With U the (possibly reduced) X and V the lazy product
// W*Y, the first output U + V comes out of the product's own multiply-add chain (U is its starting value), and
// the second is (2U + m) - (U + V) = U + m - V for the mode's multiple m of q: a shift-and-add and a subtraction,
// all modulo 2^64, the true values being below 2^64.
template <int MODE>
__device__ __forceinline__ void bfly_fwd(u64& x, u64& y, Twiddle t, const LimbConst& c) {
    if constexpr (MODE == 0) {
        const u64 u = sub_if_ge(x, c.neg_two_q);
        x = shoup_remainder_add(y, t.w, shoup_quotient(y, t.w_shoup), c.q, u);
        y = (u << 1) + c.two_q - x;
    } else if constexpr (MODE == 1) {
        const u64 u = sub_if_ge(x, c.neg_four_q);
        x = shoup_remainder_add(y, t.w, shoup_quotient_cheap(y, t.w_shoup), c.q, u);
        y = (u << 1) + c.four_q - x;
    } else {
        const u64 u = x;
        x = shoup_remainder_add(y, t.w, shoup_quotient_cheap(y, t.w_shoup), c.q, u);
        y = (u << 1) + c.four_q - x;
    }
}

// Inverse butterfly: (X, Y) -> (X + Y, (X - Y) * W).
template <int MODE>
__device__ __forceinline__ void bfly_inv(u64& x, u64& y, Twiddle t, const LimbConst& c) {
    const u64 s = x + y;
    if constexpr (MODE == 0) {
        const u64 d = x + c.two_q - y;
        x = sub_if_ge(s, c.neg_two_q);
        y = shoup_mul_lazy(d, t.w, t.w_shoup, c.q);
    } else {
        const u64 d = x + c.four_q - y;
        x = sub_if_ge(s, c.neg_four_q);
        y = shoup_mul_lazy4(d, t.w, t.w_shoup, c.q);
    }
}

// ---------------------------------------------------------------------------------------------
// Forward butterflies on double-precision FMAs, for moduli below 2^50 (LimbConst::fp_ok).
//
// A residue is held as a double whose value is an integer congruent to it, of either sign and of magnitude below
// 2^53, so every value, sum and difference below is exact.  The product W*Y is taken as h + l (the rounded
// product and, by one FMA, its rounding error), the quotient k = rint(h / q) from a rounded multiply by 1/q, and
// h - k*q (one FMA: the true value is an integer below 2^53 in magnitude, hence exact) plus l is congruent to W*Y.
// With |W| <= q/2 (the table holds the centred twiddles) and |Y| <= B*q, the estimate of W*Y/q is off by at most
// 3 roundings of 2^-53 relative to a value below B*q/2 < B*2^49, that is by less than 0.1875*B, so the result r
// has |r| <= (0.5 + 0.1875*B) * q.  A butterfly therefore takes values bounded by B*q to values bounded by
// (0.5 + 1.1875*B) * q: from B = 1, four stages end below 4.63q; from B = 0.5 (after fp_reduce), four stages end
// below 3.64q, six below 6.22q, seven below 7.88q -- all below 2^53 for q < 2^50.  (The bound on r uses exactness,
// not the other way round: h - k*q + l is W*Y - k*q whatever k is, as long as it stays below 2^53.)
struct TwiddleF {
    double w;  // the twiddle's representative in (-q/2, q/2)
};

HE_HD double fp_rint(double v) { return __builtin_rint(v); }
HE_HD double fp_fma(double a, double b, double c) { return __builtin_fma(a, b, c); }

// x - q * rint(x / q): congruent to x, magnitude at most q/2 up to the rounding of x / q (below 0.5001 q)
HE_HD double fp_reduce(double x, double q, double q_inv) { return fp_fma(-fp_rint(x * q_inv), q, x); }

// w * y modulo q as described above: |result| <= (0.5 + 0.1875 * B) * q for |w| <= q/2, |y| <= B * q
HE_HD double fp_mulmod(double w, double y, double q, double q_inv) {
    const double h = w * y;
    const double l = fp_fma(w, y, -h);
    const double k = fp_rint(h * q_inv);
    return fp_fma(-k, q, h) + l;
}

// (X, Y) -> (X + W*Y, X - W*Y), each congruent modulo q to the true value
HE_HD void bfly_fwd_f(double& x, double& y, TwiddleF t, double q, double q_inv) {
    const double r = fp_mulmod(t.w, y, q, q_inv);
    y = x - r;
    x = x + r;
}

// (X, Y) -> (X + Y, (X - Y) * W).  Sums double the bound per stage, products start again below
// (0.5 + 0.1875 * 2B) * q: from values bounded by B = 0.5001 (after fp_reduce), two stages end below 2.0005q and
// three below 4.001q; with the sums of the second stage reduced, the fourth stage ends below 3.501q.
HE_HD void bfly_inv_f(double& x, double& y, TwiddleF t, double q, double q_inv) {
    const double d = x - y;
    x = x + y;
    y = fp_mulmod(t.w, d, q, q_inv);
}

// the representative of v < q in (-q/2, q/2), as a double (q < 2^52)
HE_HD double fp_centred(u64 v, u64 q) { return v > q / 2 ? -(double)(int64_t)(q - v) : (double)(int64_t)v; }

// the canonical residue of an integer-valued double y with |y| below 2^51 that is within q of zero: the integer
// is read off the mantissa of y + 1.5 * 2^52, and q is added to a negative one
HE_HD u64 fp_to_canonical(double y, u64 q) {
    const int64_t v = (int64_t)(__builtin_bit_cast(u64, y + 6755399441055744.0) - 0x4338000000000000ull);
    return (u64)v + ((u64)(v >> 63) & q);
}

// 1.5 * 2^52: adding it to an integer-valued double of magnitude below 2^51 puts that integer, as a two's
// complement offset, into the low mantissa bits
#define HE_FP_MAGIC 6755399441055744.0
// a double holding the integer v < 2^52, from OR-ing it into the mantissa of 2^52
HE_HD double fp_from_u52(u64 v) { return __builtin_bit_cast(double, v | 0x4330000000000000ull) - 4503599627370496.0; }
