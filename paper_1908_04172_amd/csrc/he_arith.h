// Modular arithmetic on 64-bit residues for gfx950 integer ALUs.  Every function is
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
    u32 fold_every;   // MAC terms the middle accumulator word takes before it must be folded
    u32 reduce_every; // MAC terms the whole accumulator takes before it must be reduced mod q
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

// Barrett reduction of a 128-bit value z = hi:lo by a modulus below 2^64 (Alg. 5).  With
// r = floor(2^128/q), Qe = floor(z*r / 2^128) is the true quotient or one less, so z - Qe*q lies in
// [0, 2q); only the low 64 bits of Qe are needed because that difference fits in 64 bits.
HE_HD u64 reduce128(u64 hi, u64 lo, const LimbConst& c) {
    u64 carry = mul_hi64(lo, c.ratio_lo);
    u128 p1 = (u128)lo * c.ratio_hi + carry;                 // < 2^128: no overflow
    u128 p2 = (u128)hi * c.ratio_lo + (u64)p1;
    u64 qe = hi * c.ratio_hi + (u64)(p1 >> 64) + (u64)(p2 >> 64);
    u64 r = lo - qe * c.q;
    return r >= c.q ? r - c.q : r;
}

HE_HD u64 reduce64(u64 z, const LimbConst& c) { return reduce128(0, z, c); }

HE_HD u64 mul_mod(u64 a, u64 b, const LimbConst& c) {
    u128 p = (u128)a * b;
    return reduce128((u64)(p >> 64), (u64)p, c);
}

// Shoup product with a fixed operand w < q and w' = floor(w * 2^64 / q): for ANY 64-bit y the
// result is congruent to y*w and lies in [0, 2q) (Harvey's lazy form); needs q < 2^63.
HE_HD u64 shoup_mul_lazy(u64 y, u64 w, u64 w_shoup, u64 q) {
    u64 qh = mul_hi64(y, w_shoup);
    return y * w - qh * q;
}

HE_HD u64 shoup_mul(u64 y, u64 w, u64 w_shoup, u64 q) {
    u64 r = shoup_mul_lazy(y, w, w_shoup, q);
    return r >= q ? r - q : r;
}

// ---------------------------------------------------------------------------------------------
// MAC accumulator: sum of 64x64-bit products kept as three partial sums so that a term costs four
// 32x32+64 multiply-adds and one carry add, with no carry chain between the partial sums:
//   value = lo + carry*2^64 + mid*2^32 + hi*2^64
//   lo  += x0*w0 (may wrap: the wrap is counted in `carry`)
//   mid += x0*w1 + x1*w0      hi += x1*w1
// `mid` must be folded into `hi` every LimbConst::fold_every terms and the whole accumulator
// reduced every LimbConst::reduce_every terms; both bounds are derived from q on the host.
struct MacAcc {
    u64 lo, mid, hi;
    u32 carry;
};

HE_HD void acc_clear(MacAcc& a) { a.lo = a.mid = a.hi = 0; a.carry = 0; }

// w lives in scalar registers on the device (one plaintext residue for the whole wave).
HE_HD void acc_mac_s(MacAcc& a, u64 x, u64 w) {
    u32 x0 = (u32)x, x1 = (u32)(x >> 32), w0 = (u32)w, w1 = (u32)(w >> 32);
#if defined(__HIP_DEVICE_COMPILE__)
    u64 c;
    asm("v_mad_u64_u32 %0, %1, %2, %3, %0" : "+v"(a.lo), "=s"(c) : "v"(x0), "s"(w0));
    asm("v_addc_co_u32_e64 %0, %1, 0, %0, %1" : "+v"(a.carry), "+s"(c));
    asm("v_mad_u64_u32 %0, %1, %2, %3, %0" : "+v"(a.mid), "=s"(c) : "v"(x0), "s"(w1));
    asm("v_mad_u64_u32 %0, %1, %2, %3, %0" : "+v"(a.mid), "=s"(c) : "v"(x1), "s"(w0));
    asm("v_mad_u64_u32 %0, %1, %2, %3, %0" : "+v"(a.hi), "=s"(c) : "v"(x1), "s"(w1));
#else
    u64 p = (u64)x0 * w0, s = a.lo + p;
    a.carry += s < p;
    a.lo = s;
    a.mid += (u64)x0 * w1;
    a.mid += (u64)x1 * w0;
    a.hi += (u64)x1 * w1;
#endif
}

// w in vector registers (a full-polynomial plaintext: one residue per lane).
HE_HD void acc_mac_v(MacAcc& a, u64 x, u64 w) {
#if defined(__HIP_DEVICE_COMPILE__)
    u32 x0 = (u32)x, x1 = (u32)(x >> 32), w0 = (u32)w, w1 = (u32)(w >> 32);
    u64 c;
    asm("v_mad_u64_u32 %0, %1, %2, %3, %0" : "+v"(a.lo), "=s"(c) : "v"(x0), "v"(w0));
    asm("v_addc_co_u32_e64 %0, %1, 0, %0, %1" : "+v"(a.carry), "+s"(c));
    asm("v_mad_u64_u32 %0, %1, %2, %3, %0" : "+v"(a.mid), "=s"(c) : "v"(x0), "v"(w1));
    asm("v_mad_u64_u32 %0, %1, %2, %3, %0" : "+v"(a.mid), "=s"(c) : "v"(x1), "v"(w0));
    asm("v_mad_u64_u32 %0, %1, %2, %3, %0" : "+v"(a.hi), "=s"(c) : "v"(x1), "v"(w1));
#else
    acc_mac_s(a, x, w);
#endif
}

HE_HD void acc_fold(MacAcc& a) {  // move the upper half of `mid` into `hi`
    a.hi += a.mid >> 32;
    a.mid &= 0xFFFFFFFFull;
}

HE_HD u64 acc_reduce(const MacAcc& a, const LimbConst& c) {  // the accumulated value mod q
    u128 v = (u128)a.lo + ((u128)a.mid << 32) + ((u128)(a.hi + a.carry) << 64);
    return reduce128((u64)(v >> 64), (u64)v, c);
}

HE_HD void acc_restart(MacAcc& a, const LimbConst& c) {  // reduce in place and keep accumulating
    u64 r = acc_reduce(a, c);
    acc_clear(a);
    a.lo = r;
}
