// Negacyclic NTT / INTT and the rescale of Eq. (2) for gfx950, 64-bit residues.
//
// One workgroup transforms one polynomial limb (N residues), sixteen residues per thread in registers, four
// butterfly stages per pass, regrouping through the LDS between passes: geometry, regrouping and twiddle loading
// are in he_ntt_core.h (shared with the packed 32-bit kernels); this file has the 64-bit butterfly passes and the
// kernels built from them.  Butterflies are Harvey's lazy ones with Shoup multiplication by precomputed twiddles
// psi^bitrev(k), in the laziness mode the limb's modulus leaves room for (he_arith.h); moduli are below 2^62.
// A limb below 2^50 is transformed on double-precision FMAs instead (ntt_forward_f, ntt_inverse_f): eight
// operations per butterfly, the same residues.
#include <algorithm>

#include "he_internal.h"
#include "he_ntt_core.h"

namespace {

// The stages of pass P on the 16 registers of one thread.
template <int LOGN, int P, bool INVERSE, int MODE>
__device__ __forceinline__ void run_pass(u64 (&a)[16], const PassTwiddles<LOGN, P>& pt, const LimbConst& c) {
    using S = PassShape<LOGN, P>;
    static_assert(!(INVERSE && MODE == 2), "the inverse transform has modes 0 and 1 only");
#pragma unroll
    for (int kk = 0; kk < S::NST; kk++) {
        const int k = INVERSE ? S::NST - 1 - kk : kk;
        const int s = 4 * P + k;       // stage
        const int bit = S::NST - 1 - k;   // register-index bit that the stage pairs
#pragma unroll
        for (u32 e = 0; e < 16; e++) {
            if (e & (1u << bit)) continue;
            if constexpr (INVERSE) {
                if (s == 0) {  // merged with the multiplication by N^-1 (the table's entry of this stage is the
                               // twiddle times N^-1); the exact products end below 2q
                    const Twiddle w1n = pt.t[S::slot(k, e)];
                    u64 sum = a[e] + a[e | (1u << bit)];
                    u64 dif = a[e] + (MODE == 0 ? c.two_q : c.four_q) - a[e | (1u << bit)];
                    a[e] = shoup_mul_lazy(sum, c.n_inv, c.n_inv_shoup, c.q);
                    a[e | (1u << bit)] = shoup_mul_lazy(dif, w1n.w, w1n.w_shoup, c.q);
                } else {
                    bfly_inv<MODE>(a[e], a[e | (1u << bit)], pt.t[S::slot(k, e)], c);
                }
            } else {
                bfly_fwd<MODE>(a[e], a[e | (1u << bit)], pt.t[S::slot(k, e)], c);
            }
        }
    }
}

// Registers in pass-0 order, canonical -> registers in last-pass order, below 4q (mode 0), 8q
// (mode 1) or (1 + 4*log2N)*q (mode 2).
template <int LOGN, int MODE>
__device__ __forceinline__ void ntt_forward(u64 (&a)[16], const u64* tw, u64* lds, u32 tid, const LimbConst& c) {
    using G = Geo<LOGN>;
    static_assert(G::NPASS >= 2 && G::NPASS <= 4, "two to four passes");
    {
        PassTwiddles<LOGN, 0> t0;
        load_pass_twiddles<LOGN, 0>(t0, reinterpret_cast<const Twiddle*>(tw), tid);
        run_pass<LOGN, 0, false, MODE>(a, t0, c);
    }
    {
        PassTwiddles<LOGN, 1> t1;
        load_pass_twiddles<LOGN, 1>(t1, reinterpret_cast<const Twiddle*>(tw), tid);
        regroup<LOGN, 0, 1>(a, lds, tid);
        run_pass<LOGN, 1, false, MODE>(a, t1, c);
    }
    if constexpr (G::NPASS > 2) {
        PassTwiddles<LOGN, 2> t2;
        load_pass_twiddles<LOGN, 2>(t2, reinterpret_cast<const Twiddle*>(tw), tid);
        regroup<LOGN, 1, 2>(a, lds, tid);
        run_pass<LOGN, 2, false, MODE>(a, t2, c);
    }
    if constexpr (G::NPASS > 3) {
        PassTwiddles<LOGN, 3> t3;
        load_pass_twiddles<LOGN, 3>(t3, reinterpret_cast<const Twiddle*>(tw), tid);
        regroup<LOGN, 2, 3>(a, lds, tid);
        run_pass<LOGN, 3, false, MODE>(a, t3, c);
    }
}

// The forward transform in the limb's mode, of inputs below IN_Q * q (IN_Q <= 3: every mode takes them),
// ending below `cap` (returned): 4q, 4q or (IN_Q + 4*log2N)*q.  In mode 1 the values are brought from below
// 8q to below 4q, so that x + cap - value fits 64 bits for any canonical x.
template <int LOGN, int IN_Q = 1>
__device__ __forceinline__ u64 ntt_forward_any(u64 (&a)[16], const u64* tw, u64* lds, u32 tid, const LimbConst& c) {
    static_assert(IN_Q >= 1 && IN_Q <= 3 && IN_Q + 4 * LOGN + 1 <= 64, "mode 2: (IN_Q + 4*log2N + 1) * q stays below 2^64 for q < 2^58");
    if (c.ntt_mode == 2) {
        ntt_forward<LOGN, 2>(a, tw, lds, tid, c);
        return c.q * (4 * LOGN + IN_Q);
    }
    if (c.ntt_mode == 1) {
        ntt_forward<LOGN, 1>(a, tw, lds, tid, c);
#pragma unroll
        for (u32 e = 0; e < 16; e++) a[e] = sub_if_ge(a[e], c.neg_four_q);
        return c.four_q;
    }
    ntt_forward<LOGN, 0>(a, tw, lds, tid, c);
    return 2 * c.two_q;
}

// The forward transform on double-precision FMAs, for limbs with LimbConst::fp_ok (see bfly_fwd_f): registers in
// pass-0 order holding integers of magnitude at most q -> registers in last-pass order, magnitude below 6.22q
// (3.64q when the last pass has four stages).  The values are brought back to q/2 before every pass but the
// first and, when it has at most two stages and a full pass before it, the last: at most six stages run between
// two reductions.
template <int LOGN, int P>
__device__ __forceinline__ void run_pass_f(double (&a)[16], const PassTwiddles<LOGN, P, TwiddleF>& pt, double q, double q_inv) {
    using S = PassShape<LOGN, P>;
#pragma unroll
    for (int k = 0; k < S::NST; k++) {
        const int bit = S::NST - 1 - k;
#pragma unroll
        for (u32 e = 0; e < 16; e++) {
            if (e & (1u << bit)) continue;
            bfly_fwd_f(a[e], a[e | (1u << bit)], pt.t[S::slot(k, e)], q, q_inv);
        }
    }
}

template <int LOGN, int P>
__device__ __forceinline__ void pass_f(double (&a)[16], const TwiddleF* tw, double* lds, u32 tid, double q, double q_inv) {
    using G = Geo<LOGN>;
    constexpr bool KEEP = P == 0 || (P == G::NPASS - 1 && P >= 2 && G::REM <= 2);  // no reduction before this pass
    PassTwiddles<LOGN, P, TwiddleF> t;
    load_pass_twiddles<LOGN, P, TwiddleF>(t, tw, tid);
    if constexpr (P > 0) regroup<LOGN, P - 1, P>(a, lds, tid);
    if constexpr (!KEEP) {
#pragma unroll
        for (u32 e = 0; e < 16; e++) a[e] = fp_reduce(a[e], q, q_inv);
    }
    run_pass_f<LOGN, P>(a, t, q, q_inv);
}

template <int LOGN>
__device__ __forceinline__ void ntt_forward_f(double (&a)[16], const double* tw, double* lds, u32 tid, const LimbConst& c) {
    using G = Geo<LOGN>;
    static_assert(G::NPASS >= 2 && G::NPASS <= 4, "two to four passes");
    const double q = (double)c.q, q_inv = c.q_inv_f;
    const TwiddleF* t = reinterpret_cast<const TwiddleF*>(tw);
    pass_f<LOGN, 0>(a, t, lds, tid, q, q_inv);
    pass_f<LOGN, 1>(a, t, lds, tid, q, q_inv);
    if constexpr (G::NPASS > 2) pass_f<LOGN, 2>(a, t, lds, tid, q, q_inv);
    if constexpr (G::NPASS > 3) pass_f<LOGN, 3>(a, t, lds, tid, q, q_inv);
}

// Registers in last-pass order, canonical -> registers in pass-0 order, below 2q, multiplied by N^-1.
template <int LOGN, int MODE>
__device__ __forceinline__ void ntt_inverse(u64 (&a)[16], const u64* tw, u64* lds, u32 tid, const LimbConst& c) {
    using G = Geo<LOGN>;
    if constexpr (G::NPASS > 3) {
        PassTwiddles<LOGN, 3> t3;
        load_pass_twiddles<LOGN, 3>(t3, reinterpret_cast<const Twiddle*>(tw), tid);
        run_pass<LOGN, 3, true, MODE>(a, t3, c);
    }
    if constexpr (G::NPASS > 2) {
        PassTwiddles<LOGN, 2> t2;
        load_pass_twiddles<LOGN, 2>(t2, reinterpret_cast<const Twiddle*>(tw), tid);
        if constexpr (G::NPASS > 3) regroup<LOGN, 3, 2>(a, lds, tid);
        run_pass<LOGN, 2, true, MODE>(a, t2, c);
    }
    if constexpr (G::NPASS > 1) {
        PassTwiddles<LOGN, 1> t1;
        load_pass_twiddles<LOGN, 1>(t1, reinterpret_cast<const Twiddle*>(tw), tid);
        if constexpr (G::NPASS > 2) regroup<LOGN, 2, 1>(a, lds, tid);
        run_pass<LOGN, 1, true, MODE>(a, t1, c);
    }
    {
        PassTwiddles<LOGN, 0> t0;
        load_pass_twiddles<LOGN, 0>(t0, reinterpret_cast<const Twiddle*>(tw), tid);
        if constexpr (G::NPASS > 1) regroup<LOGN, 1, 0>(a, lds, tid);
        run_pass<LOGN, 0, true, MODE>(a, t0, c);
    }
}

// The inverse transform on double-precision FMAs (see bfly_inv_f): registers in last-pass order, magnitude at most
// 0.5001q -> registers in pass-0 order, multiplied by N^-1, magnitude below 1.16q (every output of the last stage
// is a product).  The values are reduced before every pass but the first one run, and the sums of the second stage
// of a four-stage pass are reduced again, so that no value exceeds 4.001q.
template <int LOGN, int P>
__device__ __forceinline__ void pass_inv_f(double (&a)[16], const TwiddleF* tw, double* lds, u32 tid, double q, double q_inv,
                                           double n_inv) {
    using G = Geo<LOGN>;
    using S = PassShape<LOGN, P>;
    PassTwiddles<LOGN, P, TwiddleF> t;
    load_pass_twiddles<LOGN, P, TwiddleF>(t, tw, tid);
    if constexpr (P < G::NPASS - 1) {
        regroup<LOGN, P + 1, P>(a, lds, tid);
#pragma unroll
        for (u32 e = 0; e < 16; e++) a[e] = fp_reduce(a[e], q, q_inv);
    }
#pragma unroll
    for (int kk = 0; kk < S::NST; kk++) {
        const int k = S::NST - 1 - kk;
        const int s = 4 * P + k;
        const int bit = S::NST - 1 - k;
#pragma unroll
        for (u32 e = 0; e < 16; e++) {
            if (e & (1u << bit)) continue;
            double& x = a[e];
            double& y = a[e | (1u << bit)];
            if (s == 0) {  // merged with the multiplication by N^-1 (in the table's entry of this stage as well)
                const double sum = x + y, dif = x - y;
                x = fp_mulmod(n_inv, sum, q, q_inv);
                y = fp_mulmod(t.t[S::slot(k, e)].w, dif, q, q_inv);
            } else {
                bfly_inv_f(x, y, t.t[S::slot(k, e)], q, q_inv);
                if (S::NST == 4 && kk == 1) x = fp_reduce(x, q, q_inv);
            }
        }
    }
}

template <int LOGN>
__device__ __forceinline__ void ntt_inverse_f(double (&a)[16], const double* tw, double* lds, u32 tid, const LimbConst& c) {
    using G = Geo<LOGN>;
    const double q = (double)c.q, q_inv = c.q_inv_f;
    const double n_inv = fp_centred(c.n_inv, c.q);
    const TwiddleF* t = reinterpret_cast<const TwiddleF*>(tw);
    if constexpr (G::NPASS > 3) pass_inv_f<LOGN, 3>(a, t, lds, tid, q, q_inv, n_inv);
    if constexpr (G::NPASS > 2) pass_inv_f<LOGN, 2>(a, t, lds, tid, q, q_inv, n_inv);
    pass_inv_f<LOGN, 1>(a, t, lds, tid, q, q_inv, n_inv);
    pass_inv_f<LOGN, 0>(a, t, lds, tid, q, q_inv, n_inv);
}

// The inverse transform of canonical values in the limb's form: on doubles for a limb below 2^50 (canonical
// results), else on the integer butterflies (results below 2q).
template <int LOGN>
__device__ __forceinline__ void ntt_inverse_any(u64 (&a)[16], const u64* tw, const double* tw_f, u64* lds, u32 tid, const LimbConst& c) {
    if (c.fp_ok) {
        const double q_f = (double)c.q;
        double f[16];
#pragma unroll
        for (u32 e = 0; e < 16; e++) f[e] = fp_reduce(fp_from_u52(a[e]), q_f, c.q_inv_f);
        ntt_inverse_f<LOGN>(f, tw_f, reinterpret_cast<double*>(lds), tid, c);
#pragma unroll
        for (u32 e = 0; e < 16; e++) a[e] = fp_to_canonical(fp_reduce(f[e], q_f, c.q_inv_f), c.q);
    } else if (c.ntt_mode != 0) {
        ntt_inverse<LOGN, 1>(a, tw, lds, tid, c);
    } else {
        ntt_inverse<LOGN, 0>(a, tw, lds, tid, c);
    }
}

__device__ __forceinline__ u64 canon4(u64 v, u64 q, u64 two_q) {  // [0,4q) -> [0,q)
    v = v >= two_q ? v - two_q : v;
    return v >= q ? v - q : v;
}

// In-place transforms of `rows` rows of N residues, row r under limb r % limbs.  A workgroup takes one row of every
// slab of gridDim.x rows (a different place in each slab, see the loop) and requests its next row before it stores
// the current one, so that the loads do not queue behind the stores and arrive while those drain.
// KIND = ROWS_SPREAD (forward only): a row is not read from `data` but from a row of `spread_src`, a table of
// coefficient rows [..][digits][N] whose row (.., j) holds integers below q_j; they are reduced
// modulo the target limb first.  This is the digit expansion of a key switch: each
// digit transformed under every limb, written to data [..][digits][limbs][N]; the limbs are
// q_0..q_{limbs-2} and, at the last position, the special prime (limb `last_id` of the context).
// KIND = ROWS_SQUARE (inverse only): row r = (ciphertext, limb j) is the slot-wise square of component 1 of that
// ciphertext, read from spread_src [..][2][limbs][N]: the quadratic component of a squared ciphertext.  The squares
// are stored as they are (NTT form) at row r * (limbs + 1) + j of `aux`, the place of digit j under its own limb
// among the expanded digits, and their inverse transform, digit j as coefficients, goes to row r of `data`.
// KIND = ROWS_HALVES: the rows are the two halves of rows of 2N residues, a ring degree whose rows do not fit the LDS:
// after the first stage of a forward transform of 2N points (before the last stage of an inverse one), which
// split_top_kernel runs, each half is a transform of N points with twiddles of its own, laid out as a table of N
// entries per (limb, half) (see he_ctx_create).  Work item w is half w % 2 of the long row (w / 2) * map.stride +
// map.first, under limb map.limb_fixed if that is set, else under limb (long row) % limbs.
enum { ROWS_PLAIN = 0, ROWS_SPREAD = 1, ROWS_SQUARE = 2, ROWS_HALVES = 3 };
struct RowMap {
    u32 stride, first, limb_fixed;  // limb_fixed = NO_LIMB: none
    u32 rotate = 0;                 // 1: workgroups change their place from slab to slab (see the loop of ntt_rows_kernel)
};
constexpr u32 NO_LIMB = 0xFFFFFFFFu;
template <int LOGN, bool INVERSE, int KIND = ROWS_PLAIN>
__global__ void __launch_bounds__(Geo<LOGN>::T)
ntt_rows_kernel(LimbTable lt, u32 limbs, u64* data, const u64* tw_all, const double* tw_f_all, u32 rows,
                const u64* spread_src = nullptr, u32 digits = 1, u32 last_id = 0, u64* aux = nullptr,
                RowMap map = RowMap{1, 0, NO_LIMB}) {
    using G = Geo<LOGN>;
    constexpr bool SPREAD = KIND == ROWS_SPREAD, SQUARE = KIND == ROWS_SQUARE, HALVES = KIND == ROWS_HALVES;
    static_assert(!(SPREAD && INVERSE), "the digit expansion is a forward transform");
    static_assert(!SQUARE || INVERSE, "the squares are taken back to coefficients");
    constexpr int PIN = INVERSE ? G::NPASS - 1 : 0, POUT = INVERSE ? 0 : G::NPASS - 1;
    extern __shared__ u64 lds[];
    u64 a[16];
    // SPREAD: `rows` counts the rows to transform, limbs - 1 per digit row: digit j under every limb position but
    // j, where the result is the digit's own NTT-form row, which the caller has put there.  Work item w maps to
    // digit row w / (limbs - 1) and limb position (w % (limbs - 1)), stepped over j.
    auto spread_row = [&](u32 w, u32& src_row) -> u32 {
        src_row = w / (limbs - 1);
        u32 pos = w % (limbs - 1);
        pos += pos >= src_row % digits;
        return src_row * limbs + pos;
    };
    // where row w is read from
    auto source = [&](u32 w) -> const u64* {
        if constexpr (SPREAD) {
            u32 src_row = 0;
            (void)spread_row(w, src_row);
            return spread_src + (size_t)src_row * G::N;
        } else if constexpr (SQUARE) {
            return spread_src + ((size_t)(w / limbs) * 2 + 1) * limbs * G::N + (size_t)(w % limbs) * G::N;
        } else if constexpr (HALVES) {
            return data + ((size_t)((w >> 1) * map.stride + map.first) * 2 + (w & 1u)) * G::N;
        } else {
            // (plain rows: from `spread_src` if the caller gave one, the transform then being out of place)
            return (spread_src != nullptr ? spread_src : data) + (size_t)w * G::N;
        }
    };
    {
        const u64* p = source(blockIdx.x);
#pragma unroll
        for (u32 e = 0; e < 16; e++) a[e] = p[reg_index<LOGN, PIN>(threadIdx.x, e)];
    }
    // Work items are taken in slabs of gridDim.x, workgroup b taking item (b + k / hold) % gridDim.x of slab k: with a plain
    // stride a workgroup would meet the same limb in every slab whenever the limb count divides the grid, and the
    // workgroups of the wide limbs (integer butterflies) would finish long after those of the narrow ones.
    // The place moves on every `hold` slabs only: the workgroups of an XCD are at the same limb at any time (they are
    // dispatched round-robin, so they share blockIdx.x % 8), and its L2 keeps that limb's twiddle table for `hold` rows
    // per workgroup instead of fetching another one for every row.
    // The launcher asks for this (map.rotate) only when the limbs differ in cost: with equal limbs the plain stride is a
    // few per cent faster.
    const u32 slabs = (rows + gridDim.x - 1) / gridDim.x;
    const u32 hold = min(8u, max(1u, slabs / (2 * limbs)));  // (once per workgroup)
    // (the place and the slab are stepped, not computed: no division in the loop)
    u32 place = blockIdx.x, held = 0;
    u32 work = blockIdx.x;  // < rows: the grid has at most `rows` workgroups
    while (true) {
        // this workgroup's item of the next slab, or `rows` if there is none
        u32 next_place = place, next_held = held + 1;
        if (map.rotate && next_held == hold) {
            next_held = 0;
            next_place = place + 1 == gridDim.x ? 0 : place + 1;
        }
        const u32 next_base = work - place + gridDim.x;
        const u32 next_work = next_base < rows && next_base + next_place < rows ? next_base + next_place : rows;
        u32 tid_i = threadIdx.x;  // opaque per iteration: addresses are recomputed, not kept live
        asm volatile("" : "+v"(tid_i));
        const u32 tid = tid_i;
        u32 src_row_unused = 0;
        const u32 row = SPREAD ? spread_row(work, src_row_unused) : work;
        const u32 long_row = (work >> 1) * map.stride + map.first;  // HALVES only
        const u32 limb = HALVES ? (map.limb_fixed != NO_LIMB ? map.limb_fixed : long_row % limbs) : row % limbs;
        const LimbConst& c = lt.c[limb];
        // (digit expansion: the last position is the special prime, whose twiddles sit at its own limb's
        // place in the table; `lt` comes with that limb's constants at the last position)
        // (halves: the table has a block of N entries per limb and half)
        const u32 tw_limb = HALVES ? limb * 2 + (work & 1u) : SPREAD && limb == limbs - 1 ? last_id : limb;
        const u64* tw = tw_all + (size_t)tw_limb * G::N * 2;
        const bool fp = !INVERSE && c.fp_ok;  // the forward transform of a limb below 2^50 runs on doubles
        if constexpr (SPREAD) {
#pragma unroll
            for (u32 e = 0; e < 16; e++) a[e] = reduce64(a[e], c);
        }
        if constexpr (SQUARE) {
            u64* own = aux + ((size_t)row * (limbs + 1) + limb) * G::N;
#pragma unroll
            for (u32 e = 0; e < 16; e++) {
                a[e] = mul_mod(a[e], a[e], c);
                own[reg_index<LOGN, PIN>(tid, e)] = a[e];
            }
        }
        if constexpr (!INVERSE) {
            if (fp) {
                double f[16];
#pragma unroll
                for (u32 e = 0; e < 16; e++) f[e] = fp_from_u52(a[e]);
                ntt_forward_f<LOGN>(f, tw_f_all + (size_t)tw_limb * G::N, reinterpret_cast<double*>(lds), tid, c);
#pragma unroll
                for (u32 e = 0; e < 16; e++) a[e] = __builtin_bit_cast(u64, f[e]);
            } else {
                ntt_forward_any<LOGN>(a, tw, lds, tid, c);
            }
        } else {
            ntt_inverse_any<LOGN>(a, tw, tw_f_all + (size_t)tw_limb * G::N, lds, tid, c);
        }
        // The next row is requested first, the last reductions of this row run while it travels, and it is
        // waited for before this row's stores are issued: a wait for loads that have stores behind them would
        // wait for the stores as well (loads and stores complete out of order with respect to each other).
        const u32 tid_s = fresh(tid);
        u64 next[16];
#pragma unroll
        for (u32 e = 0; e < 16; e++) next[e] = 0;
        if (next_work < rows) {
            const u64* p = source(next_work);
#pragma unroll
            for (u32 e = 0; e < 16; e++) next[e] = p[reg_index<LOGN, PIN>(tid_s, e)];
        }
        if constexpr (!INVERSE) {
            if (fp) {
                // reduced to |y| <= q/2 + 1, then the canonical residue
                const double q_f = (double)c.q;
#pragma unroll
                for (u32 e = 0; e < 16; e++) a[e] = fp_to_canonical(fp_reduce(__builtin_bit_cast(double, a[e]), q_f, c.q_inv_f), c.q);
            } else {
                if (c.ntt_mode == 2) {
                    // below 57q: a Shoup product by 1 (whose companion is floor(2^64/q)) brings it below 4q
#pragma unroll
                    for (u32 e = 0; e < 16; e++) a[e] = shoup_mul_lazy4(a[e], 1, c.ratio_hi, c.q);
                }
#pragma unroll
                for (u32 e = 0; e < 16; e++) a[e] = canon4(a[e], c.q, c.two_q);
            }
        } else {
#pragma unroll
            for (u32 e = 0; e < 16; e++) a[e] = a[e] >= c.q ? a[e] - c.q : a[e];
        }
        // (an inverse transform ends with one subtraction per value: too little to cover the loads, and waiting
        // for them behind the stores costs less than waiting for them here)
        if constexpr (!INVERSE) {
#pragma unroll
            for (u32 e = 0; e < 16; e++) asm volatile("" : "+v"(next[e]) :: "memory");
        }
        u64* p = HALVES ? const_cast<u64*>(source(work)) : data + (size_t)row * G::N;
#pragma unroll
        for (u32 e = 0; e < 16; e++) p[reg_index<LOGN, POUT>(tid_s, e)] = a[e];
#pragma unroll
        for (u32 e = 0; e < 16; e++) a[e] = next[e];
        if (next_work >= rows) break;
        work = next_work;
        place = next_place;
        held = next_held;
    }
}

// Rescale of one polynomial (one ciphertext component) per workgroup, Eq. (2) in RNS form.  With
// p the dropped modulus, h = floor(p/2), r the last limb's coefficients and t = (r + h) mod p:
//   out_i = (x_i - NTT_i((t mod q_i) - (h mod q_i))) * p^-1  mod q_i      for every kept limb i,
// which equals round(X / p) mod q_i for the integer X the residues stand for.  The inverse
// transform of the last limb ends in the register order in which a forward transform starts, so
// the first kept limb takes t straight from the registers; for the others t is parked in memory.
//
// The parked t for limb i+1 is requested, and waited for, before the outputs of limb i are stored.
template <int LOGN, bool SPLIT>
__global__ void __launch_bounds__(Geo<LOGN>::T)
rescale_kernel(LimbTable lt, DropRow drop, u32 limbs, u32 parts, const u64* in, u64* out, const u64* tw_fwd,
               const u64* tw_inv, const double* tw_fwd_f, const double* tw_inv_f) {
    using G = Geo<LOGN>;
    extern __shared__ __align__(16) u64 lds[];
    // A polynomial is handled by `parts` workgroups when there are too few polynomials to fill the
    // chip: each repeats the inverse transform of the dropped limb and takes a contiguous share
    // [first, end) of the kept limbs.
    // (SPLIT = false is the plain case, one workgroup per polynomial, with nothing of this computed.)
    const size_t poly = SPLIT ? blockIdx.x / parts : blockIdx.x;  // ct*2 + component
    const u32 part = SPLIT ? blockIdx.x % parts : 0;
    const u32 last = limbs - 1;
    const u32 first = SPLIT ? part * last / parts : 0, end = SPLIT ? (part + 1) * last / parts : last;
    const u64* src = in + poly * limbs * G::N;
    u64* dst = out + poly * (limbs - 1) * G::N;
    // t is parked in the output row of this workgroup's last limb: every thread re-reads only what it
    // wrote itself, and that row is overwritten only in the last iteration, after all its threads have
    // taken their t back (they use it before the first regrouping barrier of that iteration).
    u64* park = dst + (size_t)(end - 1) * G::N;
    u64 a[16];
    {
        const u32 tid = threadIdx.x;
        const LimbConst& c = lt.c[last];
        const u64* row = src + (size_t)last * G::N;
#pragma unroll
        for (u32 e = 0; e < 16; e++) a[e] = row[reg_index<LOGN, G::NPASS - 1>(tid, e)];
        ntt_inverse_any<LOGN>(a, tw_inv + (size_t)last * G::N * 2, tw_inv_f + (size_t)last * G::N, lds, tid, c);
        const u64 half = c.q >> 1;
        const u32 tid_s = fresh(tid);
#pragma unroll
        for (u32 e = 0; e < 16; e++) {
            u64 v = a[e];
            v = v >= c.q ? v - c.q : v;
            a[e] = add_mod(v, half, c.q);
            if (end - first > 1) park[reg_index<LOGN, 0>(tid_s, e)] = a[e];
        }
    }
    for (u32 i = first; i < end; i++) {
        // the thread index is made opaque per iteration so that the many addresses derived from it
        // are recomputed (a few integer operations) instead of being kept live across the loop
        u32 tid_i = threadIdx.x;
        asm volatile("" : "+v"(tid_i));
        const u32 tid = tid_i;
        const LimbConst& c = lt.c[i];
        const DropConst& d = drop.d[i];
        const u64* xrow = src + (size_t)i * G::N;
        u64* orow = dst + (size_t)i * G::N;
        // Vector loads and stores share one in-order counter per kind but complete out of order with respect
        // to each other, so a wait for a load that has stores behind it waits for the stores as well (until they
        // are acknowledged by the L2).  Hence the order below: every load the next iteration needs is issued AND
        // waited for before this iteration's stores are issued, and the transform that follows starts on scalar
        // loads (its first two passes' twiddles), with nothing to wait for behind the stores.
        // The transformed correction stays below `cap` (a multiple of q), so x + cap - correction is
        // positive, congruent to x - correction and fits 64 bits; the Shoup product takes it as it is.
        u64 cap;
        if (d.fp64) {
            // q_i < 2^50 and p <= 2*q_i: the transform runs on doubles.  t - h as an integer lies in [-h, h],
            // within q_i in magnitude; it is formed from t < 2^52 directly as a double.
            const double half_f = (double)(lt.c[last].q >> 1);
            double f[16];
#pragma unroll
            for (u32 e = 0; e < 16; e++) f[e] = fp_from_u52(a[e]) - half_f;
            ntt_forward_f<LOGN>(f, tw_fwd_f + (size_t)i * G::N, reinterpret_cast<double*>(lds), tid, c);
#pragma unroll
            for (u32 e = 0; e < 16; e++) a[e] = __builtin_bit_cast(u64, f[e]);
            cap = c.q + __builtin_bit_cast(u64, HE_FP_MAGIC);
        } else {
            // t < p is below 2*q_i unless p > 2*q_i (then a full reduction comes first); adding q_i - (h mod q_i)
            // gives a value congruent to t - h and below 3*q_i, which the forward transform takes as it is
            if (d.reduce_mode == 2) {
#pragma unroll
                for (u32 e = 0; e < 16; e++) a[e] = reduce64(a[e], c);
            }
            const u64 minus_half = c.q - d.half_mod;
#pragma unroll
            for (u32 e = 0; e < 16; e++) a[e] += minus_half;
            cap = ntt_forward_any<LOGN, 3>(a, tw_fwd + (size_t)i * G::N * 2, lds, tid, c);
            if (c.ntt_mode == 0) {  // 5q need not fit 64 bits, 3q does
#pragma unroll
                for (u32 e = 0; e < 16; e++) a[e] = sub_if_ge(a[e], c.neg_two_q);
                cap = c.two_q;
            }
        }
        const u32 tid_s = fresh(tid);
        u64 x[16], next[16];
#pragma unroll
        for (u32 e = 0; e < 16; e++) x[e] = xrow[reg_index<LOGN, G::NPASS - 1>(tid_s, e)];
#pragma unroll
        for (u32 e = 0; e < 16; e++) next[e] = 0;
        if (i + 1 < end) {
#pragma unroll
            for (u32 e = 0; e < 16; e++) next[e] = park[reg_index<LOGN, 0>(tid_s, e)];
        }
        if (d.fp64) {
            // the transformed correction y, reduced to |y| <= q/2 + 1, as the mantissa offset of y + 1.5 * 2^52:
            // x + (q + bits of 1.5 * 2^52) - bits of (y + 1.5 * 2^52) = x + q - y, positive and below 14q
            const double q_f = (double)c.q;
#pragma unroll
            for (u32 e = 0; e < 16; e++)
                a[e] = __builtin_bit_cast(u64, fp_reduce(__builtin_bit_cast(double, a[e]), q_f, c.q_inv_f) + HE_FP_MAGIC);
        }
#pragma unroll
        for (u32 e = 0; e < 16; e++) x[e] = shoup_mul(x[e] + cap - a[e], d.p_inv, d.p_inv_shoup, c.q);
#pragma unroll
        for (u32 e = 0; e < 16; e++) {
            a[e] = next[e];
            asm volatile("" : "+v"(a[e]) :: "memory");  // t for the next limb has arrived: nothing is left to wait for
        }
#pragma unroll
        for (u32 e = 0; e < 16; e++) orow[reg_index<LOGN, G::NPASS - 1>(tid_s, e)] = x[e];
    }
}

// ---- ring degree 2^15: a row (256 KiB) does not fit the LDS.  A transform of 2N = 2^15 points is its first stage
// (last stage of the inverse), run by split_top_kernel over global memory, and two transforms of N = 2^14 points,
// run by ntt_rows_kernel<14, ., ROWS_HALVES> with the twiddle tables laid out per half (he_ctx_create).

constexpr u32 HALF_N = 1u << 14;

// One butterfly per thread and step over the pairs (j, j + N) of `rows` long rows (mapped as in ROWS_HALVES):
// forward (X, Y) -> (X + W*Y, X - W*Y), inverse (X, Y) -> (X + Y, (X - Y) * W), canonical in and out, W the
// entry 0 of the limb's first table block (the root's power of the stage; N^-1 is applied by the halves).
template <bool INVERSE>
__global__ void __launch_bounds__(256) split_top_kernel(LimbTable lt, u32 limbs, u64* data, const u64* tw_all, u32 rows, RowMap map) {
    const size_t total = (size_t)rows * HALF_N;
    for (size_t k = (size_t)blockIdx.x * 256 + threadIdx.x; k < total; k += (size_t)gridDim.x * 256) {
        const u32 r = (u32)(k / HALF_N), j = (u32)(k % HALF_N);
        const u32 long_row = r * map.stride + map.first;
        const u32 limb = map.limb_fixed != NO_LIMB ? map.limb_fixed : long_row % limbs;
        const LimbConst& c = lt.c[limb];
        const u64* tw = tw_all + (size_t)limb * 2 * HALF_N * 2;
        const u64 w = tw[0], w_shoup = tw[1];
        u64* p = data + (size_t)long_row * 2 * HALF_N;
        const u64 x = p[j], y = p[j + HALF_N];
        if constexpr (INVERSE) {
            p[j] = add_mod(x, y, c.q);
            p[j + HALF_N] = shoup_mul(sub_mod(x, y, c.q), w, w_shoup, c.q);
        } else {
            const u64 v = shoup_mul(y, w, w_shoup, c.q);
            p[j] = add_mod(x, v, c.q);
            p[j + HALF_N] = sub_mod(x, v, c.q);
        }
    }
}

// Whether the first `limbs` limbs of a table differ in the arithmetic their transforms run on (double precision, or
// one of the integer butterflies' modes), i.e. in cost per row.
u32 limbs_differ(const LimbTable& lt, u32 limbs) {
    auto kind = [&](u32 i) { return lt.c[i].fp_ok ? 3u : lt.c[i].ntt_mode; };
    for (u32 i = 1; i < limbs; i++)
        if (kind(i) != kind(0)) return 1;
    return 0;
}

u32 elementwise_grid(size_t total) { return (u32)std::min<size_t>((total + 255) / 256, 256 * 32); }

// Transforms of `rows` long rows of 2^15 residues in place (mapped by `map`; tw / tw_f: the tables of the direction).
// top_done: the stage over global memory has been run by the caller (forward only).
int launch_split_transform(he_ctx* ctx, const LimbTable& lt, u32 limbs, u64* data, u32 rows, bool inverse, const u64* tw,
                           const double* tw_f, RowMap map, hipStream_t s, bool top_done = false) {
    using G = Geo<14>;
    const size_t lds = (size_t)G::N * sizeof(u64);
    const u32 halves = rows * 2;
    const u32 grid = std::min<u32>(halves, 256);
    if (map.limb_fixed == NO_LIMB) map.rotate = limbs_differ(lt, limbs);
    if (inverse) {
        static std::atomic<uint32_t> lds_allowed{0};
        if (int rc = allow_dynamic_lds((const void*)ntt_rows_kernel<14, true, ROWS_HALVES>, lds, ctx->device, lds_allowed, true)) return rc;
        hipLaunchKernelGGL((ntt_rows_kernel<14, true, ROWS_HALVES>), dim3(grid), dim3(G::T), lds, s, lt, limbs, data, tw, tw_f, halves,
                           (const u64*)nullptr, 1u, 0u, (u64*)nullptr, map);
        hipLaunchKernelGGL((split_top_kernel<true>), dim3(elementwise_grid((size_t)rows * HALF_N)), dim3(256), 0, s, lt, limbs, data, tw,
                           rows, map);
    } else {
        static std::atomic<uint32_t> lds_allowed{0};
        if (int rc = allow_dynamic_lds((const void*)ntt_rows_kernel<14, false, ROWS_HALVES>, lds, ctx->device, lds_allowed, true)) return rc;
        if (!top_done)
            hipLaunchKernelGGL((split_top_kernel<false>), dim3(elementwise_grid((size_t)rows * HALF_N)), dim3(256), 0, s, lt, limbs, data,
                               tw, rows, map);
        hipLaunchKernelGGL((ntt_rows_kernel<14, false, ROWS_HALVES>), dim3(grid), dim3(G::T), lds, s, lt, limbs, data, tw, tw_f, halves,
                           (const u64*)nullptr, 1u, 0u, (u64*)nullptr, map);
    }
    HE_HIP(hipGetLastError());
    return HE_OK;
}

// The rescale at ring degree 2^15, in the output tensor itself: the dropped limb's rows are copied into the rows of
// the last kept limb and brought back to coefficients there (t); one pass writes, for every kept limb i, t - h
// reduced modulo q_i into row i, already through the first stage of its forward transform (the last kept row in
// place: a thread reads its two values of t before it writes); the half rows are transformed; the last pass combines
// them with the input rows: out_i = (x_i - correction_i) * p^-1.
__global__ void __launch_bounds__(256) split_copy_last_kernel(u32 limbs, const u64* in, u64* out, u32 polys) {
    const size_t total = (size_t)polys * 2 * HALF_N;
    for (size_t k = (size_t)blockIdx.x * 256 + threadIdx.x; k < total; k += (size_t)gridDim.x * 256) {
        const size_t p = k / (2 * HALF_N), j = k % (2 * HALF_N);
        out[(p * (limbs - 1) + (limbs - 2)) * 2 * HALF_N + j] = in[(p * limbs + (limbs - 1)) * 2 * HALF_N + j];
    }
}

// (with the first stage of the corrections' forward transforms: a thread takes the pair (j, j + N/2) of its polynomial)
__global__ void __launch_bounds__(256) split_corrections_kernel(LimbTable lt, DropRow drop, u32 limbs, u64* out, const u64* tw_fwd, u32 polys) {
    const size_t total = (size_t)polys * HALF_N;
    const u64 p_mod = lt.c[limbs - 1].q, half = p_mod >> 1;
    for (size_t k = (size_t)blockIdx.x * 256 + threadIdx.x; k < total; k += (size_t)gridDim.x * 256) {
        const size_t p = k / HALF_N, j = k % HALF_N;
        u64* rows = out + p * (limbs - 1) * 2 * HALF_N + j;
        const u64* r = rows + (size_t)(limbs - 2) * 2 * HALF_N;
        const u64 t0 = add_mod(r[0], half, p_mod), t1 = add_mod(r[HALF_N], half, p_mod);  // (r + h) mod p
        for (u32 i = 0; i + 1 < limbs; i++) {
            const LimbConst& c = lt.c[i];
            const DropConst& d = drop.d[i];
            const u64 x = sub_mod(d.reduce_mode == 0 ? t0 : reduce64(t0, c), d.half_mod, c.q);
            const u64 y = sub_mod(d.reduce_mode == 0 ? t1 : reduce64(t1, c), d.half_mod, c.q);
            const u64* tw = tw_fwd + (size_t)i * 2 * HALF_N * 2;  // entry 0 of the limb's first block: the stage's twiddle
            const u64 v = shoup_mul(y, tw[0], tw[1], c.q);
            rows[(size_t)i * 2 * HALF_N] = add_mod(x, v, c.q);
            rows[(size_t)i * 2 * HALF_N + HALF_N] = sub_mod(x, v, c.q);
        }
    }
}

__global__ void __launch_bounds__(256) split_combine_kernel(LimbTable lt, DropRow drop, u32 limbs, const u64* in, u64* out, u32 polys) {
    const size_t total = (size_t)polys * (limbs - 1) * 2 * HALF_N;
    for (size_t k = (size_t)blockIdx.x * 256 + threadIdx.x; k < total; k += (size_t)gridDim.x * 256) {
        const size_t row = k / (2 * HALF_N), j = k % (2 * HALF_N);
        const size_t p = row / (limbs - 1);
        const u32 i = (u32)(row % (limbs - 1));
        const LimbConst& c = lt.c[i];
        // x may be the unreduced accumulator of a fused layer (below 12q where LimbConst::mac_lazy allows it)
        const u64 x = in[(p * limbs + i) * 2 * HALF_N + j];
        out[k] = shoup_mul(x + c.q - out[k], drop.d[i].p_inv, drop.d[i].p_inv_shoup, c.q);
    }
}

int launch_rescale_split(he_ctx* ctx, u32 limbs, u32 drop_id, const u64* in, u64* out, u32 n, hipStream_t s) {
    LimbTable lt = ctx->limbs;
    lt.c[limbs - 1] = ctx->limbs.c[drop_id];
    DropRow row;
    for (u32 i = 0; i < HE_MAX_LIMBS; i++) row.d[i] = ctx->drop[drop_id][i];
    const u32 polys = 2 * n;
    const size_t per_limb = (size_t)2 * HALF_N;
    hipLaunchKernelGGL(split_copy_last_kernel, dim3(elementwise_grid((size_t)polys * per_limb)), dim3(256), 0, s, limbs, in, out, polys);
    // the dropped limb's constants sit at position limbs - 1 of `lt`; its tables are found from that position
    const u64* tw_inv = ctx->tw_inv + ((size_t)drop_id - (limbs - 1)) * per_limb * 2;
    const double* tw_inv_f = ctx->tw_inv_f + ((size_t)drop_id - (limbs - 1)) * per_limb;
    if (int rc = launch_split_transform(ctx, lt, limbs, out, polys, true, tw_inv, tw_inv_f, RowMap{limbs - 1, limbs - 2, limbs - 1}, s)) return rc;
    hipLaunchKernelGGL(split_corrections_kernel, dim3(elementwise_grid((size_t)polys * HALF_N)), dim3(256), 0, s, lt, row, limbs, out,
                       ctx->tw_fwd, polys);
    if (int rc = launch_split_transform(ctx, lt, limbs - 1, out, polys * (limbs - 1), false, ctx->tw_fwd, ctx->tw_fwd_f, RowMap{1, 0, NO_LIMB}, s,
                                        /*top_done=*/true))
        return rc;
    hipLaunchKernelGGL(split_combine_kernel, dim3(elementwise_grid((size_t)polys * (limbs - 1) * per_limb)), dim3(256), 0, s, lt, row, limbs, in,
                       out, polys);
    HE_HIP(hipGetLastError());
    return HE_OK;
}

template <int LOGN>
int launch_ntt_t(he_ctx* ctx, u32 limbs, u64* data, u32 rows, bool inverse, const u64* src, hipStream_t s) {
    using G = Geo<LOGN>;
    const RowMap map{1, 0, NO_LIMB, limbs_differ(ctx->limbs, limbs)};
    const size_t lds = (size_t)G::N * sizeof(u64);
    // as many workgroups as stay resident at once (LDS and the 2048 threads of a compute unit bound
    // that), each looping over its share of the rows
    const u32 per_cu = (u32)std::max<size_t>(1, std::min<size_t>((160u << 10) / lds, 2048 / G::T));
    const u32 grid = std::min<u32>(rows, 256 * per_cu);
    if (inverse) {
        static std::atomic<uint32_t> lds_allowed{0};
        if (int rc = allow_dynamic_lds((const void*)ntt_rows_kernel<LOGN, true>, lds, ctx->device, lds_allowed, true)) return rc;
        hipLaunchKernelGGL((ntt_rows_kernel<LOGN, true>), dim3(grid), dim3(G::T), lds, s, ctx->limbs, limbs, data, ctx->tw_inv, ctx->tw_inv_f, rows, src, 1u, 0u, (u64*)nullptr, map);
    } else {
        static std::atomic<uint32_t> lds_allowed{0};
        if (int rc = allow_dynamic_lds((const void*)ntt_rows_kernel<LOGN, false>, lds, ctx->device, lds_allowed, true)) return rc;
        hipLaunchKernelGGL((ntt_rows_kernel<LOGN, false>), dim3(grid), dim3(G::T), lds, s, ctx->limbs, limbs, data, ctx->tw_fwd, ctx->tw_fwd_f, rows, src, 1u, 0u, (u64*)nullptr, map);
    }
    HE_HIP(hipGetLastError());
    return HE_OK;
}

template <int LOGN>
int launch_ntt_spread_t(he_ctx* ctx, u32 limbs, const u64* src, u64* out, u32 rows, u32 digits, hipStream_t s) {
    LimbTable lt = ctx->limbs;
    lt.c[limbs - 1] = ctx->limbs.c[ctx->L - 1];
    using G = Geo<LOGN>;
    const size_t lds = (size_t)G::N * sizeof(u64);
    const u32 per_cu = (u32)std::max<size_t>(1, std::min<size_t>((160u << 10) / lds, 2048 / G::T));
    const u32 grid = std::min<u32>(rows, 256 * per_cu);
    static std::atomic<uint32_t> lds_allowed{0};
    if (int rc = allow_dynamic_lds((const void*)ntt_rows_kernel<LOGN, false, ROWS_SPREAD>, lds, ctx->device, lds_allowed, true)) return rc;
    hipLaunchKernelGGL((ntt_rows_kernel<LOGN, false, ROWS_SPREAD>), dim3(grid), dim3(G::T), lds, s, lt, limbs, out, ctx->tw_fwd, ctx->tw_fwd_f,
                       rows, src, digits, ctx->L - 1);
    HE_HIP(hipGetLastError());
    return HE_OK;
}

// d2 [n_ct][limbs][N] = the coefficients of the square of component 1 of ct [n_ct][2][limbs][N] (slot-wise square, then
// the inverse transform); the squares themselves go to digits [n_ct][limbs][limbs + 1][N] at (.., j, j).
template <int LOGN>
int launch_ntt_square_t(he_ctx* ctx, u32 limbs, const u64* ct, u64* d2, u64* digits, u32 rows, hipStream_t s) {
    using G = Geo<LOGN>;
    const size_t lds = (size_t)G::N * sizeof(u64);
    const u32 per_cu = (u32)std::max<size_t>(1, std::min<size_t>((160u << 10) / lds, 2048 / G::T));
    const u32 grid = std::min<u32>(rows, 256 * per_cu);
    static std::atomic<uint32_t> lds_allowed{0};
    if (int rc = allow_dynamic_lds((const void*)ntt_rows_kernel<LOGN, true, ROWS_SQUARE>, lds, ctx->device, lds_allowed, true)) return rc;
    hipLaunchKernelGGL((ntt_rows_kernel<LOGN, true, ROWS_SQUARE>), dim3(grid), dim3(G::T), lds, s, ctx->limbs, limbs, d2, ctx->tw_inv,
                       ctx->tw_inv_f, rows, ct, 1u, 0u, digits);
    HE_HIP(hipGetLastError());
    return HE_OK;
}

// drop_id: the context's limb that sits at the last position of `in` and is dropped (limbs - 1 for a
// rescale; the special prime for the division that ends a key switch).  The kernel addresses limbs by
// position: it gets a table with drop_id's constants at the last position and the inverse twiddles
// shifted so that the last position finds drop_id's.
template <int LOGN>
int launch_rescale_t(he_ctx* ctx, u32 limbs, u32 drop_id, const u64* in, u64* out, u32 n, hipStream_t s) {
    using G = Geo<LOGN>;
    LimbTable lt = ctx->limbs;
    lt.c[limbs - 1] = ctx->limbs.c[drop_id];
    const u64* tw_inv = ctx->tw_inv + (size_t)(drop_id - (limbs - 1)) * G::N * 2;
    const double* tw_inv_f = ctx->tw_inv_f + (size_t)(drop_id - (limbs - 1)) * G::N;
    const size_t lds = (size_t)G::N * sizeof(u64);
    static std::atomic<uint32_t> lds_allowed{0}, lds_allowed_split{0};
    if (int rc = allow_dynamic_lds((const void*)rescale_kernel<LOGN, false>, lds, ctx->device, lds_allowed, true)) return rc;
    if (int rc = allow_dynamic_lds((const void*)rescale_kernel<LOGN, true>, lds, ctx->device, lds_allowed_split, true)) return rc;
    DropRow row;
    for (u32 i = 0; i < HE_MAX_LIMBS; i++) row.d[i] = ctx->drop[drop_id][i];
    // with fewer polynomials than workgroups the chip holds at once, split each over several workgroups
    // (at most one per kept limb), as far as they still all run at the same time
    const u32 resident = 256 * (u32)std::max<size_t>(1, std::min<size_t>((160u << 10) / lds, 2048 / G::T));
    const u32 parts = std::max(1u, std::min(limbs - 1, resident / (2 * n)));
    if (parts > 1)
        hipLaunchKernelGGL((rescale_kernel<LOGN, true>), dim3(2 * n * parts), dim3(G::T), lds, s, lt, row, limbs, parts,
                           in, out, ctx->tw_fwd, tw_inv, ctx->tw_fwd_f, tw_inv_f);
    else
        hipLaunchKernelGGL((rescale_kernel<LOGN, false>), dim3(2 * n), dim3(G::T), lds, s, lt, row, limbs, 1u, in, out,
                           ctx->tw_fwd, tw_inv, ctx->tw_fwd_f, tw_inv_f);
    HE_HIP(hipGetLastError());
    return HE_OK;
}

}  // namespace

// src: where the rows are read from (nullptr: from `data`, in place); not available at ring degree 2^15
int launch_ntt(he_ctx* ctx, u32 limbs, u64* data, u32 n_polys, bool inverse, hipStream_t s, const u64* src) {
    const u64 rows64 = (u64)n_polys * limbs;
    if (rows64 == 0) return HE_OK;
    if (rows64 > 0x7FFFFFFFull) return HE_ERR_RANGE;
    const u32 rows = (u32)rows64;
    switch (ctx->log2N) {
        case 10: return launch_ntt_t<10>(ctx, limbs, data, rows, inverse, src, s);
        case 11: return launch_ntt_t<11>(ctx, limbs, data, rows, inverse, src, s);
        case 12: return launch_ntt_t<12>(ctx, limbs, data, rows, inverse, src, s);
        case 13: return launch_ntt_t<13>(ctx, limbs, data, rows, inverse, src, s);
        case 14: return launch_ntt_t<14>(ctx, limbs, data, rows, inverse, src, s);
        case 15:
            if (rows > 0x3FFFFFFFu) return HE_ERR_RANGE;  // two halves per row
            if (src != nullptr) return HE_ERR_ARG;
            return launch_split_transform(ctx, ctx->limbs, limbs, data, rows, inverse, inverse ? ctx->tw_inv : ctx->tw_fwd,
                                          inverse ? ctx->tw_inv_f : ctx->tw_fwd_f, RowMap{1, 0, NO_LIMB}, s);
    }
    return HE_ERR_ARG;
}

// out [n_digit_rows][limbs][N] = forward transforms, under the limbs q_0..q_{limbs-2} and the special prime (the
// context's last limb), of the coefficient rows src [n_digit_rows][N] (row r holding integers below the modulus of
// limb r % digits); the row of digit j under limb j itself is not written: it is the NTT-form row the coefficients
// came from, which the caller has
int launch_ntt_spread(he_ctx* ctx, u32 limbs, const u64* src, u64* out, u32 n_digit_rows, u32 digits, hipStream_t s) {
    const u64 rows64 = (u64)n_digit_rows * (limbs - 1);  // digit j under its own limb is left to the caller
    if (rows64 == 0) return HE_OK;
    if (rows64 > 0x7FFFFFFFull) return HE_ERR_RANGE;
    const u32 rows = (u32)rows64;
    switch (ctx->log2N) {
        case 10: return launch_ntt_spread_t<10>(ctx, limbs, src, out, rows, digits, s);
        case 11: return launch_ntt_spread_t<11>(ctx, limbs, src, out, rows, digits, s);
        case 12: return launch_ntt_spread_t<12>(ctx, limbs, src, out, rows, digits, s);
        case 13: return launch_ntt_spread_t<13>(ctx, limbs, src, out, rows, digits, s);
        case 14: return launch_ntt_spread_t<14>(ctx, limbs, src, out, rows, digits, s);
    }
    return HE_ERR_ARG;
}

int launch_ntt_square(he_ctx* ctx, u32 limbs, const u64* ct, u64* d2, u64* digits, u32 n_ct, hipStream_t s) {
    const u64 rows64 = (u64)n_ct * limbs;
    if (rows64 == 0) return HE_OK;
    if (rows64 > 0x0FFFFFFFull) return HE_ERR_RANGE;
    const u32 rows = (u32)rows64;
    switch (ctx->log2N) {
        case 10: return launch_ntt_square_t<10>(ctx, limbs, ct, d2, digits, rows, s);
        case 11: return launch_ntt_square_t<11>(ctx, limbs, ct, d2, digits, rows, s);
        case 12: return launch_ntt_square_t<12>(ctx, limbs, ct, d2, digits, rows, s);
        case 13: return launch_ntt_square_t<13>(ctx, limbs, ct, d2, digits, rows, s);
        case 14: return launch_ntt_square_t<14>(ctx, limbs, ct, d2, digits, rows, s);
    }
    return HE_ERR_ARG;
}

int launch_rescale(he_ctx* ctx, u32 limbs, const u64* in, u64* out, u32 n, hipStream_t s) {
    return launch_rescale_drop(ctx, limbs, limbs - 1, in, out, n, s);
}

// `in` [n][2][limbs][N] holds the context's limbs 0..limbs-2 and, at the last position, limb drop_id >= limbs - 1
int launch_rescale_drop(he_ctx* ctx, u32 limbs, u32 drop_id, const u64* in, u64* out, u32 n, hipStream_t s) {
    if (n == 0) return HE_OK;
    if (n > 0x3FFFFFFFu) return HE_ERR_RANGE;
    switch (ctx->log2N) {
        case 10: return launch_rescale_t<10>(ctx, limbs, drop_id, in, out, n, s);
        case 11: return launch_rescale_t<11>(ctx, limbs, drop_id, in, out, n, s);
        case 12: return launch_rescale_t<12>(ctx, limbs, drop_id, in, out, n, s);
        case 13: return launch_rescale_t<13>(ctx, limbs, drop_id, in, out, n, s);
        case 14: return launch_rescale_t<14>(ctx, limbs, drop_id, in, out, n, s);
        case 15:
            if ((u64)n * 2 * (limbs - 1) > 0x3FFFFFFFull) return HE_ERR_RANGE;
            return launch_rescale_split(ctx, limbs, drop_id, in, out, n, s);
    }
    return HE_ERR_ARG;
}
