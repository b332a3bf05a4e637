/*
 * CPU oracle for the RNS-CKKS ciphertext-plaintext hot path of nGraph-HE2
 * (arXiv 1908.04172).  TEST INFRASTRUCTURE ONLY: plain, slow, written from the
 * paper's definitions.  Every modular product is (unsigned __int128) a * b % q;
 * there is no Barrett, Shoup, Montgomery, lazy reduction, blocking or fusion, and
 * nothing here is shared with (or imported by) the GPU library.
 *
 * Tensor layout everywhere: row-major uint64 [ct][2][limbs][N]; residues of limb i
 * are canonical, in [0, q_i).  Limb `limbs-1` is the one a rescale drops.
 *
 * What each function follows:
 *   orc_encode_scalar  Alg. 2 (scalar encoding), Sec. "Scalar Encoding"
 *   orc_encode_vector  Alg. 1 (general encoding), read as the canonical embedding: the integer
 *                      polynomial whose values at the roots exp(i*pi*(2k+1)/N), k < N/2, are the
 *                      scaled slots (and their conjugates at the conjugate roots), then the
 *                      residues and the NTT.  Complex slots are the paper's complex packing.
 *   orc_decode_vector  the inverse map: values of the polynomial at those roots, over the scale
 *   orc_add            Alg. 3 (vector plaintext) / Alg. 4 (scalar plaintext)
 *   orc_mac            Alg. 7 (64-bit multiply) / Alg. 8 (scalar multiply), summed over the
 *                      inner dimension of a Dot/Convolution (Sec. "Lazy Rescaling")
 *   orc_ntt_*          negacyclic NTT (Sec. "Double-CRT Representation"); the paper leaves root and
 *                      ordering open: psi = smallest 2N-th primitive root, output j is the
 *                      evaluation at psi^(2*bitrev(j)+1)
 *   orc_rescale        Eq. (2) (rescaling), read as  ct' = round(ct / p_last)  on the integer
 *                      coefficient rebuilt by the Chinese remainder theorem; INTT, divide, NTT
 *                      as Sec. "Double-CRT Representation" prescribes
 *   orc_layer          MAC, then bias add, then ONE rescale per output (lazy rescaling)
 *
 * Parallelism: an OpenMP loop over output ciphertexts, the strategy the paper's appendix
 * "Parallel Scaling" describes.  orc_set_threads(1) gives the serial program.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef unsigned __int128 u128;
typedef uint64_t u64;

#define ORC_PT_SCALAR 0
#define ORC_PT_POLY 1
#define ORC_MAX_LIMBS 16

/* ------------------------------------------------------------------ scalars mod q */

u64 orc_addmod(u64 a, u64 b, u64 q) { return (u64)(((u128)a + b) % q); }
u64 orc_submod(u64 a, u64 b, u64 q) { return (u64)(((u128)a + q - b) % q); }
u64 orc_mulmod(u64 a, u64 b, u64 q) { return (u64)((u128)a * b % q); }

u64 orc_powmod(u64 base, u64 exp, u64 q) {
    u64 result = 1 % q;
    base %= q;
    while (exp) {
        if (exp & 1) result = orc_mulmod(result, base, q);
        base = orc_mulmod(base, base, q);
        exp >>= 1;
    }
    return result;
}

/* q prime => a^(q-2) is the inverse of a (Fermat). */
u64 orc_invmod(u64 a, u64 q) { return orc_powmod(a, q - 2, q); }

/* Deterministic Miller-Rabin; the first twelve primes as bases decide every n < 3.3e24. */
int orc_is_prime(u64 n) {
    static const u64 bases[12] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
    if (n < 2) return 0;
    for (int i = 0; i < 12; i++) {
        if (n == bases[i]) return 1;
        if (n % bases[i] == 0) return 0;
    }
    u64 d = n - 1;
    int r = 0;
    while ((d & 1) == 0) { d >>= 1; r++; }
    for (int i = 0; i < 12; i++) {
        u64 x = orc_powmod(bases[i], d, n);
        if (x == 1 || x == n - 1) continue;
        int composite = 1;
        for (int k = 1; k < r; k++) {
            x = orc_mulmod(x, x, n);
            if (x == n - 1) { composite = 0; break; }
        }
        if (composite) return 0;
    }
    return 1;
}

/* Smallest psi in [2, q) with psi^N = -1 (mod q); 0 if none.  N is a power of two, so such a
 * psi has order exactly 2N.  x^N + 1 has exactly N roots mod a prime q = 1 (mod 2N): the odd
 * powers of any one of them.  One root is found as g^((q-1)/2N) for the first g = 2, 3, ... whose
 * power has order 2N; all N are then enumerated and the least is returned. */
u64 orc_find_psi(u64 q, u64 N) {
    if (q < 3 || (q - 1) % (2 * N) != 0) return 0;
    u64 root = 0;
    for (u64 g = 2; g < q && g < 1000; g++) {
        u64 cand = orc_powmod(g, (q - 1) / (2 * N), q);
        if (orc_powmod(cand, N, q) == q - 1) { root = cand; break; }
    }
    if (root == 0) return 0;
    u64 sq = orc_mulmod(root, root, q), best = root, cur = root;
    for (u64 k = 1; k < N; k++) { /* cur = root^(2k+1) */
        cur = orc_mulmod(cur, sq, q);
        if (cur < best) best = cur;
    }
    return best;
}

static u64 bitrev(u64 x, int bits) {
    u64 r = 0;
    for (int b = 0; b < bits; b++)
        if (x & ((u64)1 << b)) r |= (u64)1 << (bits - 1 - b);
    return r;
}

static int ilog2(u64 n) {
    int l = 0;
    while (((u64)1 << l) < n) l++;
    return l;
}

/* ------------------------------------------------------------------ negacyclic NTT */

/* The definition, O(N^2):  out[j] = sum_n a[n] * psi^((2*bitrev(j)+1) * n)  mod q. */
void orc_ntt_fwd_direct(const u64* a, u64* out, u64 N, u64 q, u64 psi) {
    int logN = ilog2(N);
    for (u64 j = 0; j < N; j++) {
        u64 point = orc_powmod(psi, 2 * bitrev(j, logN) + 1, q);
        u64 acc = 0, xn = 1; /* xn = point^n */
        for (u64 n = 0; n < N; n++) {
            acc = orc_addmod(acc, orc_mulmod(a[n], xn, q), q);
            xn = orc_mulmod(xn, point, q);
        }
        out[j] = acc;
    }
}

/* Its inverse, O(N^2):  a[n] = N^-1 * sum_j in[j] * psi^(-(2*bitrev(j)+1) * n)  mod q. */
void orc_ntt_inv_direct(const u64* in, u64* a, u64 N, u64 q, u64 psi) {
    int logN = ilog2(N);
    u64 psi_inv = orc_invmod(psi, q), n_inv = orc_invmod(N % q, q);
    for (u64 n = 0; n < N; n++) {
        u64 acc = 0;
        for (u64 j = 0; j < N; j++) {
            u64 e = ((2 * bitrev(j, logN) + 1) * n) % (2 * N);
            acc = orc_addmod(acc, orc_mulmod(in[j], orc_powmod(psi_inv, e, q), q), q);
        }
        a[n] = orc_mulmod(acc, n_inv, q);
    }
}

/* Textbook even/odd split.  With rho^n = -1 and a(x) = e(x^2) + x*o(x^2):
 *   out[2j]   = E[j] + w_j * O[j],   out[2j+1] = E[j] - w_j * O[j],
 *   w_j = rho^(2*bitrev_{log n - 1}(j) + 1),
 * where E, O are the size-n/2 transforms of the even/odd coefficients with root rho^2.
 * `pw` is the table psi^e, e in [0, 2N); `step` = log2 of how often psi was squared. */
static void ntt_fwd_rec(u64* a, u64 n, u64 q, const u64* pw, int step, u64* tmp) {
    if (n == 1) return;
    u64 h = n / 2;
    u64 *ev = tmp, *od = tmp + h;
    for (u64 k = 0; k < h; k++) { ev[k] = a[2 * k]; od[k] = a[2 * k + 1]; }
    ntt_fwd_rec(ev, h, q, pw, step + 1, tmp + n);
    ntt_fwd_rec(od, h, q, pw, step + 1, tmp + n);
    int hb = ilog2(h);
    for (u64 j = 0; j < h; j++) {
        u64 w = pw[(2 * bitrev(j, hb) + 1) << step];
        u64 t = orc_mulmod(w, od[j], q);
        a[2 * j] = orc_addmod(ev[j], t, q);
        a[2 * j + 1] = orc_submod(ev[j], t, q);
    }
}

/* Exact inverse of ntt_fwd_rec: E[j] = (x0+x1)/2, O[j] = (x0-x1)/(2 w_j), then recurse. */
static void ntt_inv_rec(u64* a, u64 n, u64 q, const u64* pw, u64 twoN, int step, u64* tmp) {
    if (n == 1) return;
    u64 h = n / 2;
    u64 *ev = tmp, *od = tmp + h;
    int hb = ilog2(h);
    u64 inv2 = orc_invmod(2, q);
    for (u64 j = 0; j < h; j++) {
        u64 e = (2 * bitrev(j, hb) + 1) << step;
        u64 w_inv = pw[(twoN - e) % twoN];
        ev[j] = orc_mulmod(orc_addmod(a[2 * j], a[2 * j + 1], q), inv2, q);
        od[j] = orc_mulmod(orc_mulmod(orc_submod(a[2 * j], a[2 * j + 1], q), inv2, q), w_inv, q);
    }
    ntt_inv_rec(ev, h, q, pw, twoN, step + 1, tmp + n);
    ntt_inv_rec(od, h, q, pw, twoN, step + 1, tmp + n);
    for (u64 k = 0; k < h; k++) { a[2 * k] = ev[k]; a[2 * k + 1] = od[k]; }
}

static u64* power_table(u64 N, u64 q, u64 psi) {
    u64* pw = (u64*)malloc(2 * N * sizeof(u64));
    pw[0] = 1;
    for (u64 e = 1; e < 2 * N; e++) pw[e] = orc_mulmod(pw[e - 1], psi, q);
    return pw;
}

/* In-place transforms of one length-N row. */
void orc_ntt_fwd(u64* a, u64 N, u64 q, u64 psi) {
    u64* pw = power_table(N, q, psi);
    u64* tmp = (u64*)malloc(2 * N * sizeof(u64));
    ntt_fwd_rec(a, N, q, pw, 0, tmp);
    free(tmp);
    free(pw);
}

void orc_ntt_inv(u64* a, u64 N, u64 q, u64 psi) {
    u64* pw = power_table(N, q, psi);
    u64* tmp = (u64*)malloc(2 * N * sizeof(u64));
    ntt_inv_rec(a, N, q, pw, 2 * N, 0, tmp);
    free(tmp);
    free(pw);
}

/* rows = n_polys*limbs rows of N; row r uses modulus q[r % limbs]. */
void orc_ntt_fwd_rows(u64* data, u64 n_polys, uint32_t limbs, u64 N, const u64* q, const u64* psi) {
    long rows = (long)(n_polys * limbs);
#pragma omp parallel for schedule(dynamic)
    for (long r = 0; r < rows; r++) orc_ntt_fwd(data + (u64)r * N, N, q[r % limbs], psi[r % limbs]);
}

void orc_ntt_inv_rows(u64* data, u64 n_polys, uint32_t limbs, u64 N, const u64* q, const u64* psi) {
    long rows = (long)(n_polys * limbs);
#pragma omp parallel for schedule(dynamic)
    for (long r = 0; r < rows; r++) orc_ntt_inv(data + (u64)r * N, N, q[r % limbs], psi[r % limbs]);
}

/* ------------------------------------------------------------------ Alg. 2: scalar encoding */

/* y_i = [round(scale*value)]_{q_i}.  Reading of Alg. 2: ONE IEEE double multiply, rounding to
 * the nearest integer with halves away from zero, then the non-negative residue.  A product of
 * magnitude >= 2^63 is already an integer m*2^e (53-bit m); it is reduced as
 * (m mod q)*(2^e mod q).  Returns -1 (and writes nothing) for a non-finite product. */
int orc_encode_scalar(double value, double scale, const u64* q, uint32_t limbs, u64* out) {
    double v = value * scale;
    if (!isfinite(v)) return -1;
    int negative = v < 0;
    double mag = fabs(v);
    for (uint32_t i = 0; i < limbs; i++) {
        u64 r;
        if (mag < 9223372036854775808.0) { /* 2^63 */
            u64 z = (u64)llround(mag);       /* halves away from zero */
            r = z % q[i];
        } else {
            int e;
            double f = frexp(mag, &e);       /* mag = f * 2^e, f in [0.5, 1) */
            u64 m = (u64)ldexp(f, 53);       /* exact 53-bit integer */
            e -= 53;                         /* mag = m * 2^e, e >= 11 */
            r = orc_mulmod(m % q[i], orc_powmod(2, (u64)e, q[i]), q[i]);
        }
        out[i] = (negative && r != 0) ? q[i] - r : r;
    }
    return 0;
}

/* ------------------------------------------------------------------ Alg. 1: general encoding */

/* cos and sin of pi*r/N for r = 0 .. 2N-1, in long double: every angle the embedding needs is
 * one of these after reducing an integer product mod 2N. */
static void root_table(u64 N, long double* c, long double* s) {
    const long double pi = 3.14159265358979323846264338327950288L;
    for (u64 r = 0; r < 2 * N; r++) {
        c[r] = cosl(pi * (long double)r / (long double)N);
        s[r] = sinl(pi * (long double)r / (long double)N);
    }
}

/* Coefficients of Alg. 1 before the modular reduction, for n_vec vectors of N/2 complex slots
 * (slots[v][k][0] real part, [1] imaginary part):
 *     m_j = round( scale * (2/N) * sum_{k < N/2} Re( z_k * r_k^-j ) ),   r_k = exp(i*pi*(2k+1)/N),
 * i.e. the real polynomial with m(r_k) = scale*z_k and m(conj r_k) = scale*conj(z_k), rounded
 * coefficient-wise (halves away from zero).  The sum is taken term by term in long double; the
 * result must stay below 2^62 in magnitude (returns -1 otherwise, or for a non-finite input). */
int orc_encode_vector_coeffs(const double* slots, u64 n_vec, u64 N, double scale, int64_t* coeffs) {
    long double* c = (long double*)malloc(2 * N * sizeof(long double));
    long double* s = (long double*)malloc(2 * N * sizeof(long double));
    root_table(N, c, s);
    int bad = 0;
    for (u64 v = 0; v < n_vec; v++) {
        const double* z = slots + v * N;  /* N/2 complex numbers */
#pragma omp parallel for schedule(static)
        for (u64 j = 0; j < N; j++) {
            long double acc = 0.0L;
            for (u64 k = 0; k < N / 2; k++) {
                u64 r = ((2 * k + 1) * j) % (2 * N);            /* r_k^-j = cos(pi r/N) - i sin(pi r/N) */
                acc += (long double)z[2 * k] * c[r] + (long double)z[2 * k + 1] * s[r];
            }
            long double m = (long double)scale * (2.0L * acc / (long double)N);
            if (!(fabsl(m) < 4611686018427387904.0L)) { /* 2^62; also catches NaN */
#pragma omp atomic write
                bad = 1;
                coeffs[v * N + j] = 0;
            } else {
                coeffs[v * N + j] = (int64_t)roundl(m);         /* halves away from zero */
            }
        }
    }
    free(c);
    free(s);
    return bad ? -1 : 0;
}

/* Alg. 1 complete: coefficients as above, residues [m_j]_{q_i}, forward NTT of every limb.
 * out: [n_vec][limbs][N]. */
int orc_encode_vector(const double* slots, u64 n_vec, u64 N, double scale, const u64* q, const u64* psi,
                      uint32_t limbs, u64* out) {
    int64_t* m = (int64_t*)malloc(n_vec * N * sizeof(int64_t));
    int rc = orc_encode_vector_coeffs(slots, n_vec, N, scale, m);
    if (rc == 0) {
        for (u64 v = 0; v < n_vec; v++)
            for (uint32_t i = 0; i < limbs; i++)
                for (u64 j = 0; j < N; j++) {
                    int64_t x = m[v * N + j];
                    u64 r = (u64)(x < 0 ? -x : x) % q[i];
                    out[(v * limbs + i) * N + j] = (x < 0 && r != 0) ? q[i] - r : r;
                }
        orc_ntt_fwd_rows(out, n_vec, limbs, N, q, psi);
    }
    free(m);
    return rc;
}

/* The inverse map on signed integer coefficients (given as doubles: the caller lifts residues to
 * the centred representative first): z_k = m(r_k) / scale for k < N/2, term by term in long double.
 * out[v][k][0..1] = real and imaginary part. */
void orc_decode_vector(const double* coeffs, u64 n_vec, u64 N, double scale, double* out) {
    long double* c = (long double*)malloc(2 * N * sizeof(long double));
    long double* s = (long double*)malloc(2 * N * sizeof(long double));
    root_table(N, c, s);
    for (u64 v = 0; v < n_vec; v++) {
#pragma omp parallel for schedule(static)
        for (u64 k = 0; k < N / 2; k++) {
            long double re = 0.0L, im = 0.0L;
            for (u64 j = 0; j < N; j++) {
                u64 r = ((2 * k + 1) * j) % (2 * N);
                re += (long double)coeffs[v * N + j] * c[r];
                im += (long double)coeffs[v * N + j] * s[r];
            }
            out[(v * N / 2 + k) * 2] = (double)(re / (long double)scale);
            out[(v * N / 2 + k) * 2 + 1] = (double)(im / (long double)scale);
        }
    }
    free(c);
    free(s);
}

/* ------------------------------------------------------------------ Alg. 3 / 4: ct + pt */

/* Component 0 of each of the n ciphertexts gets the plaintext added; component 1 is untouched.
 * pt: [n][limbs] (scalar, Alg. 4) or [n][limbs][N] (Alg. 3). */
void orc_add(u64* ct, u64 n, uint32_t limbs, u64 N, const u64* q, const u64* pt, int pt_kind) {
    for (u64 c = 0; c < n; c++)
        for (uint32_t l = 0; l < limbs; l++)
            for (u64 k = 0; k < N; k++) {
                u64 p = pt_kind == ORC_PT_SCALAR ? pt[c * limbs + l] : pt[(c * limbs + l) * N + k];
                u64* x = &ct[((c * 2 + 0) * limbs + l) * N + k];
                *x = orc_addmod(*x, p, q[l]);
            }
}

/* ------------------------------------------------------------------ Alg. 7 / 8 summed: MAC */

/* out[o][c][l][k] = sum_{t in [off[o], off[o+1])} ct_in[term_ct[t]][c][l][k] * P(term_pt[t], l, k)
 * with P = pt[j][l] (scalar) or pt[j][l][k] (polynomial, NTT form).  Both components are
 * multiplied.  bias (may be NULL): [n_out][limbs] scalar residues added to component 0. */
void orc_mac(u64 N, uint32_t limbs, const u64* q, const u64* ct_in, const uint32_t* off,
             const uint32_t* term_ct, const uint32_t* term_pt, uint32_t n_out, const u64* pt,
             int pt_kind, const u64* bias, u64* out) {
#pragma omp parallel for schedule(dynamic)
    for (long o = 0; o < (long)n_out; o++)
        for (int c = 0; c < 2; c++)
            for (uint32_t l = 0; l < limbs; l++)
                for (u64 k = 0; k < N; k++) {
                    u64 acc = 0;
                    for (uint32_t t = off[o]; t < off[o + 1]; t++) {
                        u64 x = ct_in[(((u64)term_ct[t] * 2 + c) * limbs + l) * N + k];
                        u64 p = pt_kind == ORC_PT_SCALAR ? pt[(u64)term_pt[t] * limbs + l]
                                                         : pt[((u64)term_pt[t] * limbs + l) * N + k];
                        acc = orc_addmod(acc, orc_mulmod(x, p, q[l]), q[l]);
                    }
                    if (bias && c == 0) acc = orc_addmod(acc, bias[(u64)o * limbs + l], q[l]);
                    out[(((u64)o * 2 + c) * limbs + l) * N + k] = acc;
                }
}

/* ------------------------------------------------------------------ Eq. (2): rescale */

/* Little-endian multiword naturals, W words; only "bignum op word" operations are needed. */
#define BN_WORDS (ORC_MAX_LIMBS + 1)
typedef struct { u64 w[BN_WORDS]; } bn;

static void bn_set(bn* a, u64 v) { memset(a, 0, sizeof *a); a->w[0] = v; }
static void bn_mul_word(bn* a, u64 m) { /* a *= m */
    u64 carry = 0;
    for (int i = 0; i < BN_WORDS; i++) {
        u128 t = (u128)a->w[i] * m + carry;
        a->w[i] = (u64)t;
        carry = (u64)(t >> 64);
    }
}
static void bn_add(bn* a, const bn* b) { /* a += b */
    u64 carry = 0;
    for (int i = 0; i < BN_WORDS; i++) {
        u128 t = (u128)a->w[i] + b->w[i] + carry;
        a->w[i] = (u64)t;
        carry = (u64)(t >> 64);
    }
}
static void bn_sub(bn* a, const bn* b) { /* a -= b, a >= b */
    u64 borrow = 0;
    for (int i = 0; i < BN_WORDS; i++) {
        u128 t = (u128)a->w[i] - b->w[i] - borrow;
        a->w[i] = (u64)t;
        borrow = (u64)(t >> 64) & 1;
    }
}
static int bn_cmp(const bn* a, const bn* b) {
    for (int i = BN_WORDS - 1; i >= 0; i--)
        if (a->w[i] != b->w[i]) return a->w[i] < b->w[i] ? -1 : 1;
    return 0;
}
static u64 bn_divmod_word(bn* a, u64 d) { /* a = floor(a/d), returns a mod d */
    u64 rem = 0;
    for (int i = BN_WORDS - 1; i >= 0; i--) {
        u128 t = ((u128)rem << 64) | a->w[i];
        a->w[i] = (u64)(t / d);
        rem = (u64)(t % d);
    }
    return rem;
}
static u64 bn_mod_word(const bn* a, u64 d) { bn t = *a; return bn_divmod_word(&t, d); }

/* Integer in [0, Q) with the given residues:  X = sum_i [x_i * (Q/q_i)^-1]_{q_i} * (Q/q_i) mod Q. */
static void crt_rebuild(const u64* x, const u64* q, uint32_t limbs, const bn* Q, const bn* Qhat,
                        const u64* Qhat_inv, bn* X) {
    bn_set(X, 0);
    for (uint32_t i = 0; i < limbs; i++) {
        bn term = Qhat[i];
        bn_mul_word(&term, orc_mulmod(x[i], Qhat_inv[i], q[i]));
        bn_add(X, &term);
    }
    while (bn_cmp(X, Q) >= 0) bn_sub(X, Q);
}

/* One polynomial: coefficient-form residues coef[limbs][N] -> res[limbs-1][N],
 * Y = floor((X + floor(p/2)) / p), p = q[limbs-1] (p odd: no ties), res_i = Y mod q_i. */
static void divide_round_poly(const u64* coef, u64* res, uint32_t limbs, u64 N, const u64* q) {
    bn Q, Qhat[ORC_MAX_LIMBS];
    u64 Qhat_inv[ORC_MAX_LIMBS];
    bn_set(&Q, 1);
    for (uint32_t i = 0; i < limbs; i++) bn_mul_word(&Q, q[i]);
    for (uint32_t i = 0; i < limbs; i++) {
        bn_set(&Qhat[i], 1);
        for (uint32_t j = 0; j < limbs; j++)
            if (j != i) bn_mul_word(&Qhat[i], q[j]);
        Qhat_inv[i] = orc_invmod(bn_mod_word(&Qhat[i], q[i]), q[i]);
    }
    u64 p = q[limbs - 1];
    bn half;
    bn_set(&half, p / 2);
    for (u64 k = 0; k < N; k++) {
        u64 x[ORC_MAX_LIMBS];
        for (uint32_t i = 0; i < limbs; i++) x[i] = coef[(u64)i * N + k];
        bn X;
        crt_rebuild(x, q, limbs, &Q, Qhat, Qhat_inv, &X);
        bn_add(&X, &half);
        bn_divmod_word(&X, p); /* X is now Y */
        for (uint32_t i = 0; i + 1 < limbs; i++) res[(u64)i * N + k] = bn_mod_word(&X, q[i]);
    }
}

/* Coefficient-domain Eq. (2) alone, exposed so tests can pin it against big-integer arithmetic:
 * coef [n_polys][limbs][N] -> res [n_polys][limbs-1][N]. */
void orc_divide_round(const u64* coef, u64* res, u64 n_polys, uint32_t limbs, u64 N, const u64* q) {
    for (u64 pidx = 0; pidx < n_polys; pidx++)
        divide_round_poly(coef + pidx * limbs * N, res + pidx * (limbs - 1) * N, limbs, N, q);
}

/* in [n][2][limbs][N] (NTT form) -> out [n][2][limbs-1][N] (NTT form):
 * INTT every limb, divide-and-round, NTT the kept limbs. */
void orc_rescale(u64 N, uint32_t limbs, const u64* q, const u64* psi, const u64* in, u64* out, u64 n) {
#pragma omp parallel for schedule(dynamic)
    for (long pidx = 0; pidx < (long)(2 * n); pidx++) {
        u64* coef = (u64*)malloc((u64)limbs * N * sizeof(u64));
        memcpy(coef, in + (u64)pidx * limbs * N, (u64)limbs * N * sizeof(u64));
        for (uint32_t i = 0; i < limbs; i++) orc_ntt_inv(coef + (u64)i * N, N, q[i], psi[i]);
        u64* res = out + (u64)pidx * (limbs - 1) * N;
        divide_round_poly(coef, res, limbs, N, q);
        for (uint32_t i = 0; i + 1 < limbs; i++) orc_ntt_fwd(res + (u64)i * N, N, q[i], psi[i]);
        free(coef);
    }
}

/* One FC/Conv layer with lazy rescaling: all MACs, the bias, then exactly one rescale per
 * output ciphertext.  out: [n_out][2][limbs-1][N].  Returns the number of rescales done. */
uint32_t orc_layer(u64 N, uint32_t limbs, const u64* q, const u64* psi, const u64* ct_in,
                   const uint32_t* off, const uint32_t* term_ct, const uint32_t* term_pt,
                   uint32_t n_out, const u64* pt, int pt_kind, const u64* bias, u64* out) {
    u64* acc = (u64*)malloc((u64)n_out * 2 * limbs * N * sizeof(u64));
    orc_mac(N, limbs, q, ct_in, off, term_ct, term_pt, n_out, pt, pt_kind, bias, acc);
    orc_rescale(N, limbs, q, psi, acc, out, n_out);
    free(acc);
    return n_out;
}

/* ------------------------------------------------------------------ threads */

int orc_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
    return omp_get_max_threads();
#else
    (void)n;
    return 1;
#endif
}
