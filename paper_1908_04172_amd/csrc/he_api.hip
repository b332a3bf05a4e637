// Context, plans, the C entry points, and the small kernels (scalar encoding, plaintext addition).
#include <math.h>
#include <string.h>

#include <algorithm>
#include <map>
#include <mutex>
#include <new>

#include "he_internal.h"
#include "../../include/he_test.h"

// ---- the scratch memory of he_ct_pt_mac_static: a fixed array in every GPU's copy of the library's code
// object, in place of the caller's workspace.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the device address (one per GPU) is looked up once per device, with that device
// current, when a context is created there, and every later use goes through that address.
static __device__ __align__(256) unsigned char scratch[HE_STATIC_SCRATCH_BYTES];
static constexpr int MAX_DEVICES = 64;
static std::mutex scratch_mutex;
static void* scratch_address[MAX_DEVICES];  // [device], null until looked up

// the caller has made `device` current
static int static_scratch(int device, void** out) {
    *out = nullptr;
    if (device < 0 || device >= MAX_DEVICES) return HE_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_address[device]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return HE_ERR_DEVICE;
        }
        scratch_address[device] = p;
    }
    *out = scratch_address[device];
    return HE_OK;
}

// ------------------------------------------------------------------------------------------------
// host number theory (context set-up only)

namespace {

u64 h_mulmod(u64 a, u64 b, u64 q) { return (u64)((u128)a * b % q); }

u64 h_powmod(u64 b, u64 e, u64 q) {
    u64 r = 1 % q;
    b %= q;
    for (; e; e >>= 1) {
        if (e & 1) r = h_mulmod(r, b, q);
        b = h_mulmod(b, b, q);
    }
    return r;
}

// Miller-Rabin with the first twelve primes as witnesses: exact for every 64-bit input.
bool h_is_prime(u64 n) {
    const u64 wit[12] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
    if (n < 2) return false;
    for (u64 p : wit) {
        if (n == p) return true;
        if (n % p == 0) return false;
    }
    u64 d = n - 1;
    int twos = 0;
    while (!(d & 1)) { d >>= 1; ++twos; }
    for (u64 a : wit) {
        u64 x = h_powmod(a, d, n);
        if (x == 1 || x == n - 1) continue;
        bool witness = true;
        for (int i = 1; i < twos && witness; ++i) {
            x = h_mulmod(x, x, n);
            if (x == n - 1) witness = false;
        }
        if (witness) return false;
    }
    return true;
}

// The least element of order 2N with psi^N = -1: take any root of x^N + 1 (a 2N-th root of a
// non-residue-like generator power), then walk its odd powers, which are all the roots.
u64 h_min_psi(u64 q, u32 N) {
    const u64 cof = (q - 1) / (2ull * N);
    u64 root = 0;
    for (u64 g = 2; g < 4096 && root == 0; ++g) {
        u64 cand = h_powmod(g, cof, q);
        if (h_powmod(cand, N, q) == q - 1) root = cand;
    }
    if (!root) return 0;
    const u64 step = h_mulmod(root, root, q);
    u64 best = root, cur = root;
    for (u32 k = 1; k < N; ++k) {
        cur = h_mulmod(cur, step, q);
        best = std::min(best, cur);
    }
    return best;
}

u64 h_shoup(u64 w, u64 q) { return (u64)(((u128)w << 64) / q); }

u32 h_bitrev(u32 x, u32 bits) {
    u32 r = 0;
    for (u32 i = 0; i < bits; ++i) r |= ((x >> i) & 1u) << (bits - 1 - i);
    return r;
}

void fill_limb_const(LimbConst& c, u64 q, u64 psi, u32 N) {
    c.q = q;
    c.two_q = 2 * q;
    const u128 all_ones = ~(u128)0;  // floor(2^128 / q) = floor((2^128 - 1) / q) because q is odd and > 1
    const u128 ratio = all_ones / q;
    c.ratio_hi = (u64)(ratio >> 64);
    c.ratio_lo = (u64)ratio;
    c.n_inv = h_powmod(N % q, q - 2, q);
    c.n_inv_shoup = h_shoup(c.n_inv, q);
    const u64 psi_inv = h_powmod(psi, q - 2, q);
    const u64 w1_inv = h_powmod(psi_inv, N / 2, q);  // psi^-bitrev(1)
    c.w1n_inv = h_mulmod(w1_inv, c.n_inv, q);
    c.w1n_inv_shoup = h_shoup(c.w1n_inv, q);
    // Accumulator periods (see MacAcc).  Pieces: xa, wa <= A = 2^s - 1; xb, wb <= B = (q-1) >> s.
    // The cut may sit at half the modulus width or one bit higher: a higher cut folds more often
    // but reduces less often; the cheaper of the two (about 6 operations per fold, 40 per reduction)
    // is taken.
    u32 bits = 0;
    while (bits < 64 && ((q - 1) >> bits)) ++bits;
    double best_cost = 1e300;
    for (u32 s = (bits + 1) / 2; s <= std::min<u32>((bits + 1) / 2 + 1, 31); ++s) {
        const u128 A = (1ull << s) - 1, B = (q - 1) >> s, top = (u128)1 << 64;
        // after a fold (or a restart) lo <= A and mid <= A; F more terms must keep
        //   lo <= A + F*A*A  and  mid + (lo >> s) <= A + 2*F*A*B + (lo >> s)  below 2^64
        u64 fold = 0;
        for (u64 f = 1; f <= 0x7FFFFFFFull; f = (f < 64 ? f + 1 : f * 2)) {
            const u128 lo_max = A + (u128)f * A * A;
            const u128 mid_max = A + 2 * (u128)f * A * B + (lo_max >> s);
            if (lo_max >= top || mid_max >= top) break;
            fold = f;
        }
        if (fold == 0) continue;
        // hi <= value >> 2s must stay below 2^64 and the value below 2^128: q + R*(q-1)^2 < 2^min(128, 64+2s)
        const u128 cap = (64 + 2 * s >= 128) ? all_ones : (((u128)1 << (64 + 2 * s)) - 1);
        const u128 sq = (u128)(q - 1) * (q - 1);
        const u128 red = std::min<u128>((cap - q) / sq, 0x7FFFFFFFull);
        if (red == 0) continue;
        const double cost = 6.0 / (double)fold + 40.0 / (double)(u64)red;
        if (cost < best_cost) {
            best_cost = cost;
            c.split_bits = s;
            c.split_mask = (1ull << s) - 1;
            c.fold_every = (u32)fold;
            c.reduce_every = (u32)red;
        }
    }
    // one-word Barrett for the accumulator when every value it can hold stays below 2^(63+bits)
    c.mu_shift = bits - 1;
    c.mu = (u64)((((u128)1) << (63 + bits)) / q);
    {
        const u128 sq = (u128)(q - 1) * (q - 1);
        const u128 lim = ((((u128)1) << (63 + bits)) - 1 - q) / sq;
        c.narrow = lim >= 64;
        if (c.narrow) c.reduce_every = (u32)std::min<u128>(c.reduce_every, lim);
    }
    c.ntt_mode = q < (1ull << 58) ? 2 : q < (1ull << 61) ? 1 : 0;
    c.fp_ok = q < (1ull << 50);
    c.pad = 0;
    c.q_inv_f = 1.0 / (double)q;  // (a double holds q exactly; the division rounds to nearest)
    c.pow64 = (u64)((((u128)1) << 64) % q);
    c.pow64_shoup = h_shoup(c.pow64, q);
    // three products per MAC term: the sum of (xa+xb)*(wa+wb) must fit 64 bits with xa+xb, wa+wb below 2^32,
    // and the total must stay within the one-word Barrett of acc_reduce_add (narrow limbs below 2^61)
    c.kara_terms = 0;
    const u128 all_ones64 = (((u128)1) << 64) - 1;
    if (c.narrow && q < (1ull << 61)) {
        const u128 ab = (u128)c.split_mask + ((q - 1) >> c.split_bits);
        if (ab < ((u128)1 << 32)) {
            const u128 sq = (u128)(q - 1) * (q - 1);
            u128 lim = std::min<u128>(all_ones64 / (ab * ab), ((((u128)1) << (63 + bits)) - 1 - q) / sq);
            // the kernel runs such a group's padded terms (up to 3 more, zero weights) in one go, with no
            // fold or reduction on the way: stay within those periods too
            lim = std::min<u128>(lim, std::min(c.fold_every, c.reduce_every));
            c.kara_terms = lim > 3 ? (u32)std::min<u128>(lim - 3, 0x7FFFFFFFull) : 0;
        }
    }
    c.neg_two_q = 0 - 2 * q;
    c.four_q = 4 * q;
    c.neg_four_q = 0 - 4 * q;
}

int check_level(const he_ctx* ctx, u32 limbs, u32 min_limbs) {
    if (!ctx) return HE_ERR_ARG;
    if (limbs < min_limbs || limbs > ctx->L) return HE_ERR_LEVEL;
    return HE_OK;
}

// Do the byte ranges [a, a + na) and [b, b + nb) share a byte?  (Plain address arithmetic on device
// pointers: nothing is dereferenced.)
bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
    if (!a || !b || !na || !nb) return false;
    const uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
    return x < y + nb && y < x + na;
}

int need_device(const he_ctx* ctx) {
    if (ctx->device < 0) return HE_ERR_DEVICE;
    if (hipSetDevice(ctx->device) != hipSuccess) { (void)hipGetLastError(); return HE_ERR_DEVICE; }
    return HE_OK;
}

template <typename T>
int upload(T** dst, const T* src, size_t n) {
    *dst = nullptr;
    if (n == 0) n = 1;
    HE_HIP(hipMalloc((void**)dst, n * sizeof(T)));
    if (src) HE_HIP(hipMemcpy(*dst, src, n * sizeof(T), hipMemcpyHostToDevice));
    return HE_OK;
}

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

__global__ void __launch_bounds__(256) encode_kernel(LimbTable lt, const double* values, size_t n, double scale, u32 limbs,
                                                     u64* out) {
    const size_t j = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= n) return;
    u64 tmp[HE_MAX_LIMBS];
    encode_one(values[j], scale, lt.c, limbs, tmp);
    for (u32 i = 0; i < limbs; ++i) out[j * limbs + i] = tmp[i];
}

// Alg. 4 / Alg. 3: component 0 of every ciphertext gets the plaintext added.  A thread handles ADD_UNROLL pairs of
// adjacent residues (16-byte accesses, a workgroup's accesses contiguous), all loaded before the first is stored, so
// that a wave has several requests in flight; total = ct * limbs * N/2 pairs.
constexpr u32 ADD_UNROLL = 4;
template <bool POLY>
__global__ void __launch_bounds__(256) add_kernel(LimbTable lt, u32 limbs, u32 N, u64* ct, size_t n_ct, const u64* pt) {
    const size_t half = N / 2;
    const size_t total = n_ct * limbs * half;
    const size_t first = (size_t)blockIdx.x * (256 * ADD_UNROLL) + threadIdx.x;
    ulonglong2* p[ADD_UNROLL];
    ulonglong2 v[ADD_UNROLL], a[ADD_UNROLL];
    u64 q[ADD_UNROLL];
#pragma unroll
    for (u32 u = 0; u < ADD_UNROLL; u++) {
        const size_t i = first + (size_t)u * 256;  // pair index
        p[u] = nullptr;
        if (i >= total) continue;
        const size_t k2 = i % half;
        const size_t row = i / half;  // ct * limbs + limb
        const u32 limb = (u32)(row % limbs);
        const size_t c_idx = row / limbs;
        q[u] = lt.c[limb].q;
        p[u] = reinterpret_cast<ulonglong2*>(ct + ((c_idx * 2) * limbs + limb) * N) + k2;
        v[u] = *p[u];
        if constexpr (POLY) {
            a[u] = reinterpret_cast<const ulonglong2*>(pt + row * N)[k2];
        } else {
            a[u].x = a[u].y = pt[row];
        }
    }
#pragma unroll
    for (u32 u = 0; u < ADD_UNROLL; u++) {
        if (p[u] == nullptr) continue;
        v[u].x = add_mod(v[u].x, a[u].x, q[u]);
        v[u].y = add_mod(v[u].y, a[u].y, q[u]);
        *p[u] = v[u];
    }
}

// he_check_reduced: residues of data [rows][limbs][row_len] that are not below their limb's modulus, counted
// into *bad (one atomic per wave that found any).
__global__ void __launch_bounds__(256) check_reduced_kernel(LimbTable lt, u32 limbs, const u64* data, size_t total, u32 row_len,
                                                            unsigned long long* bad) {
    u32 mine = 0;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const u32 limb = (u32)((i / row_len) % limbs);
        mine += data[i] >= lt.c[limb].q;
    }
    if (mine) atomicAdd(bad, (unsigned long long)mine);
}

// Group consecutive outputs whose term_ct lists are identical, at most `cap` per group.
void build_tiles(const u32* off, const u32* term_ct, u32 n_out, u32 cap, std::vector<Tile>& tiles) {
    u32 o = 0;
    while (o < n_out) {
        const u32 k = off[o + 1] - off[o];
        u32 cnt = 1;
        while (cnt < cap && o + cnt < n_out) {
            const u32 o2 = o + cnt;
            if (off[o2 + 1] - off[o2] != k) break;
            if (k && memcmp(term_ct + off[o], term_ct + off[o2], (size_t)k * sizeof(u32)) != 0) break;
            ++cnt;
        }
        tiles.push_back(Tile{o, cnt, off[o], k});
        o += cnt;
    }
}

// Stable sort of the tiles into capacity classes caps[0] < caps[1] < caps[2].
void classify(std::vector<Tile>& tiles, const u32 caps[3], u32 class_begin[4]) {
    std::vector<Tile> sorted;
    sorted.reserve(tiles.size());
    for (int cls = 0; cls < 3; ++cls) {
        class_begin[cls] = (u32)sorted.size();
        for (const Tile& t : tiles) {
            const u32 lo = cls ? caps[cls - 1] : 0;
            if (t.count > lo && t.count <= caps[cls]) sorted.push_back(t);
        }
    }
    class_begin[3] = (u32)sorted.size();
    tiles.swap(sorted);
}

const u32 CAPS_S[3] = {1, 4, 16};
const u32 CAPS_P[3] = {1, 2, 4};

}  // namespace

// ------------------------------------------------------------------------------------------------
// ABI

extern "C" {

const char* he_strerror(int status) {
    switch (status) {
        case HE_OK: return "ok";
        case HE_ERR_ARG: return "bad argument";
        case HE_ERR_MODULUS: return "modulus is not a distinct prime = 1 (mod 2N) below 2^62";
        case HE_ERR_LEVEL: return "limbs out of range for this context or operation";
        case HE_ERR_RANGE: return "index or size out of range";
        case HE_ERR_DEVICE: return "HIP call failed or context has no device";
        case HE_ERR_WORKSPACE: return "workspace missing or too small";
    }
    return "unknown status";
}

int he_ctx_create(he_ctx** out, uint32_t log2N, uint32_t L, const uint64_t* moduli, int device) {
    if (!out) return HE_ERR_ARG;
    *out = nullptr;
    if (!moduli || log2N < HE_MIN_LOG2N || log2N > HE_MAX_LOG2N || L < 1 || L > HE_MAX_LIMBS || device < -1)
        return HE_ERR_ARG;
    const u32 N = 1u << log2N;
    for (u32 i = 0; i < L; ++i) {
        const u64 q = moduli[i];
        if (q >= (1ull << 62) || q < 2ull * N || (q - 1) % (2ull * N) != 0 || !h_is_prime(q)) return HE_ERR_MODULUS;
        for (u32 j = 0; j < i; ++j)
            if (moduli[j] == q) return HE_ERR_MODULUS;
    }
    he_ctx* ctx = new (std::nothrow) he_ctx();
    if (!ctx) return HE_ERR_ARG;
    memset(ctx, 0, sizeof *ctx);
    ctx->device = device;
    ctx->log2N = log2N;
    ctx->N = N;
    ctx->L = L;
    for (u32 i = 0; i < L; ++i) {
        ctx->q[i] = moduli[i];
        ctx->psi[i] = h_min_psi(moduli[i], N);
        if (!ctx->psi[i]) { delete ctx; return HE_ERR_MODULUS; }
        fill_limb_const(ctx->limbs.c[i], ctx->q[i], ctx->psi[i], N);
        {   // x + cap - correction in the rescale's combine step must fit 64 bits for x below 12q, where cap bounds the
            // transformed correction: (3 + 4 log2 N) q in butterfly mode 2, 4q in mode 1, 2q in mode 0
            LimbConst& c = ctx->limbs.c[i];
            const u128 cap_q = c.ntt_mode == 2 ? 3 + 4 * log2N : c.ntt_mode == 1 ? 4 : 2;
            c.mac_lazy = (12 + cap_q) * (u128)c.q < ((u128)1 << 64);
        }
        if (ctx->q[i] < (1ull << 30)) {  // the limb has a packed 32-bit form
            Limb32& c = ctx->limbs32.c[i];
            const u64 q = ctx->q[i], n_inv = ctx->limbs.c[i].n_inv;
            c.q = (u32)q;
            c.two_q = (u32)(2 * q);
            c.n_inv = (u32)n_inv;
            c.n_inv_shoup = (u32)((n_inv << 32) / q);
            c.w1n_inv = (u32)ctx->limbs.c[i].w1n_inv;
            c.w1n_inv_shoup = (u32)((ctx->limbs.c[i].w1n_inv << 32) / q);
            c.ratio = (u64)((((u128)1) << 64) / q);
            c.pow48 = (u32)((1ull << 48) % q);
            c.ok = 1;
        }
    }
    for (u32 j = 0; j < L; ++j)
        for (u32 i = 0; i < L; ++i) {
            if (i == j) continue;
            DropConst& d = ctx->drop[j][i];
            const u64 qi = ctx->q[i], p = ctx->q[j];
            d.p_inv = h_powmod(p % qi, qi - 2, qi);
            d.p_inv_shoup = h_shoup(d.p_inv, qi);
            d.half_mod = (p >> 1) % qi;
            d.reduce_mode = p <= qi ? 0 : (p <= 2 * qi ? 1 : 2);
            d.fp64 = ctx->limbs.c[i].fp_ok && d.reduce_mode <= 1;
        }
    if (device >= 0) {
        int rc = need_device(ctx);
        if (rc == HE_OK) rc = static_scratch(device, &ctx->static_scratch);
        if (rc != HE_OK) { delete ctx; return rc; }
        std::vector<u64> fwd((size_t)L * N * 2), inv((size_t)L * N * 2);
        for (u32 i = 0; i < L; ++i) {
            const u64 q = ctx->q[i], psi = ctx->psi[i], psi_inv = h_powmod(psi, q - 2, q);
            u64 pw = 1, pwi = 1;
            for (u32 k = 0; k < N; ++k) {
                const size_t slot = ((size_t)i * N + h_bitrev(k, log2N)) * 2;
                fwd[slot] = pw;
                fwd[slot + 1] = h_shoup(pw, q);
                inv[slot] = pwi;
                inv[slot + 1] = h_shoup(pwi, q);
                pw = h_mulmod(pw, psi, q);
                pwi = h_mulmod(pwi, psi_inv, q);
            }
        }
        // the forward twiddles as centred doubles, for the limbs whose transform can run on doubles
        std::vector<double> fwd_f((size_t)L * N, 0.0), inv_f((size_t)L * N, 0.0);
        for (u32 i = 0; i < L; ++i) {
            if (!ctx->limbs.c[i].fp_ok) continue;
            for (size_t k = 0; k < N; ++k) {
                fwd_f[(size_t)i * N + k] = fp_centred(fwd[((size_t)i * N + k) * 2], ctx->q[i]);
                inv_f[(size_t)i * N + k] = fp_centred(inv[((size_t)i * N + k) * 2], ctx->q[i]);
            }
            inv_f[(size_t)i * N + 1] = fp_centred(ctx->limbs.c[i].w1n_inv, ctx->q[i]);  // last inverse stage: times N^-1
        }
        if (upload(&ctx->tw_fwd_f, fwd_f.data(), fwd_f.size()) != HE_OK || upload(&ctx->tw_inv_f, inv_f.data(), inv_f.size()) != HE_OK) {
            he_ctx_destroy(ctx);
            return HE_ERR_DEVICE;
        }
        // 32-bit tables for the limbs that have a packed form (moduli below 2^30), zeros for the others
        std::vector<u32> fwd32((size_t)L * N * 2, 0), inv32((size_t)L * N * 2, 0);
        for (u32 i = 0; i < L; ++i) {
            if (!ctx->limbs32.c[i].ok) continue;
            const u64 q = ctx->q[i];
            for (size_t k = 0; k < N; ++k) {
                const size_t slot = ((size_t)i * N + k) * 2;
                fwd32[slot] = (u32)fwd[slot];
                fwd32[slot + 1] = (u32)((fwd[slot] << 32) / q);
                inv32[slot] = (u32)inv[slot];
                inv32[slot + 1] = (u32)((inv[slot] << 32) / q);
            }
        }
        if (upload(&ctx->tw32_fwd, fwd32.data(), fwd32.size()) != HE_OK || upload(&ctx->tw32_inv, inv32.data(), inv32.size()) != HE_OK) {
            he_ctx_destroy(ctx);
            return HE_ERR_DEVICE;
        }
        // tables of the general encoder: e^(-2 pi i k / (N/2)) for k < N/4, and e^(-i pi j / N) for j < N/2
        std::vector<double> fft_tw((size_t)N / 2), twist((size_t)N);
        const long double pi = 3.14159265358979323846264338327950288L;
        for (u32 k = 0; k < N / 4; ++k) {
            fft_tw[2 * k] = (double)cosl(4.0L * pi * k / N);
            fft_tw[2 * k + 1] = (double)-sinl(4.0L * pi * k / N);
        }
        for (u32 j = 0; j < N / 2; ++j) {
            twist[2 * j] = (double)cosl(pi * j / N);
            twist[2 * j + 1] = (double)-sinl(pi * j / N);
        }
        // tables of the decoder: Garner inverses, and the digits of floor(Q_l / 2) in the mixed radix
        // (q_0, q_1, ...) for every level l.  Q_l - 1 has the digits q_i - 1; halve it from the top digit.
        std::vector<u64> garner((size_t)HE_MAX_LIMBS * HE_MAX_LIMBS * 2, 0), half((size_t)(HE_MAX_LIMBS + 1) * HE_MAX_LIMBS, 0);
        for (u32 i = 0; i < L; ++i)
            for (u32 k = 0; k < i; ++k) {
                garner[((size_t)i * HE_MAX_LIMBS + k) * 2] = ctx->drop[k][i].p_inv;
                garner[((size_t)i * HE_MAX_LIMBS + k) * 2 + 1] = ctx->drop[k][i].p_inv_shoup;
            }
        for (u32 l = 1; l <= L; ++l) {
            u64 rem = 0;
            for (int i = (int)l - 1; i >= 0; --i) {
                const u128 cur = (u128)rem * ctx->q[i] + (ctx->q[i] - 1);
                half[(size_t)l * HE_MAX_LIMBS + i] = (u64)(cur / 2);
                rem = (u64)(cur % 2);
            }
        }
        if (log2N <= 14) {
            // the entry of the last inverse stage carries N^-1 (the butterflies of that stage multiply by it anyway)
            for (u32 i = 0; i < L; ++i) {
                inv[((size_t)i * N + 1) * 2] = ctx->limbs.c[i].w1n_inv;
                inv[((size_t)i * N + 1) * 2 + 1] = ctx->limbs.c[i].w1n_inv_shoup;
            }
        } else {
            // N = 2^15: a transform is one stage over global memory and two transforms of H = N/2 points (he_ntt.hip,
            // ROWS_HALVES).  The tables become [L][2][H]: block (limb, half h) is the table of that half's transform,
            // entry 2^s + r (stage s of the half = stage s + 1 of the whole, r < 2^s) being entry 2^(s+1) + h*2^s + r of
            // the whole table; entry 0, which no half uses, holds the twiddle of the stage over global memory (entry 1 of
            // the whole table); the inverse halves' entry 1 carries N^-1.
            const size_t H = N / 2;
            auto split = [&](auto& table, auto& table_f, bool inverse) {
                auto whole = table;
                for (u32 i = 0; i < L; ++i) {
                    const u64 q = ctx->q[i];
                    for (u32 h = 0; h < 2; ++h)
                        for (size_t k = 0; k < H; ++k) {
                            size_t src = 1;
                            if (k > 0) {
                                u32 st = 0;
                                while ((size_t)2 << st <= k) ++st;  // 2^st <= k < 2^(st+1)
                                src = ((size_t)2 << st) + ((size_t)h << st) + (k - ((size_t)1 << st));
                            }
                            u64 w = whole[((size_t)i * N + src) * 2];
                            if (inverse && k == 1) w = h_mulmod(w, ctx->limbs.c[i].n_inv, q);
                            const size_t dst = ((size_t)i * 2 + h) * H + k;
                            table[dst * 2] = w;
                            table[dst * 2 + 1] = h_shoup(w, q);
                            table_f[dst] = ctx->limbs.c[i].fp_ok ? fp_centred(w, q) : 0.0;
                        }
                }
            };
            split(fwd, fwd_f, false);
            split(inv, inv_f, true);
            // (the double-precision tables were uploaded above in the whole-table layout: replace them)
            if (hipMemcpy(ctx->tw_fwd_f, fwd_f.data(), fwd_f.size() * sizeof(double), hipMemcpyHostToDevice) != hipSuccess ||
                hipMemcpy(ctx->tw_inv_f, inv_f.data(), inv_f.size() * sizeof(double), hipMemcpyHostToDevice) != hipSuccess) {
                (void)hipGetLastError();
                he_ctx_destroy(ctx);
                return HE_ERR_DEVICE;
            }
        }
        if (upload(&ctx->bad_count, (const u64*)nullptr, 1) != HE_OK ||
            upload(&ctx->garner, garner.data(), garner.size()) != HE_OK || upload(&ctx->half_digits, half.data(), half.size()) != HE_OK ||
            upload(&ctx->tw_fwd, fwd.data(), fwd.size()) != HE_OK || upload(&ctx->tw_inv, inv.data(), inv.size()) != HE_OK ||
            upload(&ctx->fft_tw, fft_tw.data(), fft_tw.size()) != HE_OK || upload(&ctx->twist, twist.data(), twist.size()) != HE_OK) {
            he_ctx_destroy(ctx);
            return HE_ERR_DEVICE;
        }
    }
    *out = ctx;
    return HE_OK;
}

int he_ctx_destroy(he_ctx* ctx) {
    if (!ctx) return HE_ERR_ARG;
    if (ctx->device >= 0 && hipSetDevice(ctx->device) == hipSuccess) {
        if (ctx->tw_fwd) (void)hipFree(ctx->tw_fwd);
        if (ctx->tw_inv) (void)hipFree(ctx->tw_inv);
        if (ctx->tw_fwd_f) (void)hipFree(ctx->tw_fwd_f);
        if (ctx->tw_inv_f) (void)hipFree(ctx->tw_inv_f);
        if (ctx->fft_tw) (void)hipFree(ctx->fft_tw);
        if (ctx->twist) (void)hipFree(ctx->twist);
        if (ctx->garner) (void)hipFree(ctx->garner);
        if (ctx->half_digits) (void)hipFree(ctx->half_digits);
        if (ctx->tw32_fwd) (void)hipFree(ctx->tw32_fwd);
        if (ctx->tw32_inv) (void)hipFree(ctx->tw32_inv);
        if (ctx->bad_count) (void)hipFree(ctx->bad_count);
    }
    if (ctx->device >= 0) (void)hipGetLastError();  // a failure here must not surface in the caller's next HIP call
    delete ctx;
    return HE_OK;
}

int he_ctx_info(const he_ctx* ctx, uint32_t* log2N, uint32_t* L, uint64_t* moduli, uint64_t* psi) {
    if (!ctx) return HE_ERR_ARG;
    if (log2N) *log2N = ctx->log2N;
    if (L) *L = ctx->L;
    for (u32 i = 0; i < ctx->L; ++i) {
        if (moduli) moduli[i] = ctx->q[i];
        if (psi) psi[i] = ctx->psi[i];
    }
    return HE_OK;
}

int he_encode_scalar(he_ctx* ctx, const double* values, size_t n, double scale, uint32_t limbs, uint64_t* out,
                     void* stream) {
    int rc = check_level(ctx, limbs, 1);
    if (rc != HE_OK) return rc;
    if (n == 0) return HE_OK;
    if (!values || !out) return HE_ERR_ARG;
    if ((rc = need_device(ctx)) != HE_OK) return rc;
    const size_t blocks = (n + 255) / 256;
    if (blocks > 0x7FFFFFFFull) return HE_ERR_RANGE;
    hipLaunchKernelGGL(encode_kernel, dim3((u32)blocks), dim3(256), 0, (hipStream_t)stream, ctx->limbs, values, n, scale,
                       limbs, out);
    HE_HIP(hipGetLastError());
    return HE_OK;
}

int he_encode_vector(he_ctx* ctx, const double* slots, size_t n, double scale, uint32_t limbs, uint64_t* out,
                     void* stream) {
    int rc = check_level(ctx, limbs, 1);
    if (rc != HE_OK) return rc;
    if (ctx->log2N > HE_MAX_LOG2N_IN_LDS) return HE_ERR_ARG;
    if (!(scale > 0.0) || !(scale <= 1.7976931348623157e308)) return HE_ERR_ARG;
    if (n == 0) return HE_OK;
    if (!slots || !out) return HE_ERR_ARG;
    if (n > 0x7FFFFFFFull / limbs) return HE_ERR_RANGE;
    if ((rc = need_device(ctx)) != HE_OK) return rc;
    if ((rc = launch_encode_vector(ctx, limbs, slots, (u32)n, scale, out, (hipStream_t)stream)) != HE_OK) return rc;
    return launch_ntt(ctx, limbs, out, (u32)n, false, (hipStream_t)stream);
}

int he_decode_vector(he_ctx* ctx, const uint64_t* poly, size_t n, double scale, uint32_t limbs, double* slots,
                     void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_level(ctx, limbs, 1);
    if (rc != HE_OK) return rc;
    if (ctx->log2N > HE_MAX_LOG2N_IN_LDS) return HE_ERR_ARG;
    if (!(scale > 0.0) || !(scale <= 1.7976931348623157e308)) return HE_ERR_ARG;
    if (n == 0) return HE_OK;
    if (!poly || !slots) return HE_ERR_ARG;
    if (n > 0x7FFFFFFFull / limbs) return HE_ERR_RANGE;
    const size_t bytes = n * limbs * ctx->N * sizeof(u64);
    if (!workspace || workspace_bytes < bytes) return HE_ERR_WORKSPACE;
    if (overlaps(workspace, bytes, poly, bytes) || overlaps(workspace, bytes, slots, n * ctx->N * sizeof(double)))
        return HE_ERR_ARG;
    if ((rc = need_device(ctx)) != HE_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    // the inverse transform reads the caller's rows and writes the workspace
    if ((rc = launch_ntt(ctx, limbs, (u64*)workspace, (u32)n, true, s, poly)) != HE_OK) return rc;
    return launch_decode_vector(ctx, limbs, (const u64*)workspace, (u32)n, scale, slots, s);
}

int he_encode_scalar_host(const he_ctx* ctx, const double* values, size_t n, double scale, uint32_t limbs,
                          uint64_t* out) {
    int rc = check_level(ctx, limbs, 1);
    if (rc != HE_OK) return rc;
    if (n == 0) return HE_OK;
    if (!values || !out) return HE_ERR_ARG;
    bool ok = true;
    for (size_t j = 0; j < n; ++j) ok &= encode_one(values[j], scale, ctx->limbs.c, limbs, out + j * limbs);
    return ok ? HE_OK : HE_ERR_ARG;
}

int he_plan_create(he_ctx* ctx, uint32_t n_in, uint32_t n_out, uint32_t n_pt, const uint32_t* off,
                   const uint32_t* term_ct, const uint32_t* term_pt, he_plan** out) {
    if (!out) return HE_ERR_ARG;
    *out = nullptr;
    if (!ctx || !off) return HE_ERR_ARG;
    if (off[0] != 0) return HE_ERR_RANGE;
    for (u32 o = 0; o < n_out; ++o)
        if (off[o + 1] < off[o]) return HE_ERR_RANGE;
    const u32 n_terms = off[n_out];
    if (n_terms && (!term_ct || !term_pt)) return HE_ERR_ARG;
    for (u32 t = 0; t < n_terms; ++t)
        if (term_ct[t] >= n_in || term_pt[t] >= n_pt) return HE_ERR_RANGE;
    int rc = need_device(ctx);
    if (rc != HE_OK) return rc;
    he_plan* p = new (std::nothrow) he_plan();
    if (!p) return HE_ERR_ARG;
    p->ctx = ctx;
    p->device = ctx->device;
    p->n_in = n_in; p->n_out = n_out; p->n_pt = n_pt; p->n_terms = n_terms;
    p->off.assign(off, off + n_out + 1);
    p->tiles_s_dev = p->tiles_p_dev = nullptr;
    p->wbase_s_dev = nullptr;
    p->wowner_s_dev = nullptr;
    p->off_dev = p->term_ct_dev = p->term_pt_dev = nullptr;
    std::vector<Tile> ts, tp;
    build_tiles(off, term_ct, n_out, CAPS_S[2], ts);
    build_tiles(off, term_ct, n_out, CAPS_P[2], tp);
    classify(ts, CAPS_S, p->class_begin_s);
    classify(tp, CAPS_P, p->class_begin_p);
    p->n_tiles_s = (u32)ts.size();
    p->n_tiles_p = (u32)tp.size();
    // Groups of one class that multiply by the same plaintexts in the same arrangement (all windows of a
    // convolution that have the same shape) share one table of gathered weights: the table then stays
    // in the scalar cache instead of being fetched anew by every group.  wowner[i] = 1 for the group
    // that fills the table.
    std::vector<u64> wbase(ts.size() + 1, 0);
    std::vector<u32> wowner(ts.size() + 1, 0);
    u64 elems = 0;
    for (int cls = 0; cls < 3; ++cls) {
        p->min_terms_s[cls] = p->class_begin_s[cls] < p->class_begin_s[cls + 1] ? ~0u : 0;
        p->max_terms_s[cls] = 0;
        p->max_count_s[cls] = 0;
        std::map<std::vector<u32>, u64> tables;
        std::vector<u32> key;
        for (u32 i = p->class_begin_s[cls]; i < p->class_begin_s[cls + 1]; ++i) {
            p->min_terms_s[cls] = std::min(p->min_terms_s[cls], ts[i].n_terms);
            p->max_terms_s[cls] = std::max(p->max_terms_s[cls], ts[i].n_terms);
            p->max_count_s[cls] = std::max(p->max_count_s[cls], ts[i].count);
            key.assign(1, ts[i].n_terms);
            for (u32 g = 0; g < ts[i].count; ++g)
                key.insert(key.end(), term_pt + off[ts[i].out0 + g], term_pt + off[ts[i].out0 + g] + ts[i].n_terms);
            const auto found = tables.find(key);
            if (found != tables.end()) {
                wbase[i] = found->second;
                continue;
            }
            tables.emplace(key, elems);
            wbase[i] = elems;
            wowner[i] = 1;
            elems += (u64)((ts[i].n_terms + 3) / 4 * 4) * (cls == 2 ? 24 : CAPS_S[cls]);  // terms padded to whole blocks of 4; 24 words per term in 16-output tables
        }
    }
    p->wtab_elems = elems + 24;  // padding: the 16-output kernel requests one term's entry past its last
    if (upload(&p->tiles_s_dev, ts.data(), ts.size()) != HE_OK || upload(&p->tiles_p_dev, tp.data(), tp.size()) != HE_OK ||
        upload(&p->wbase_s_dev, wbase.data(), ts.size()) != HE_OK || upload(&p->wowner_s_dev, wowner.data(), ts.size()) != HE_OK || upload(&p->off_dev, off, (size_t)n_out + 1) != HE_OK ||
        upload(&p->term_ct_dev, term_ct, n_terms) != HE_OK || upload(&p->term_pt_dev, term_pt, n_terms) != HE_OK) {
        he_plan_destroy(p);
        return HE_ERR_DEVICE;
    }
    *out = p;
    return HE_OK;
}

int he_plan_destroy(he_plan* p) {
    if (!p) return HE_ERR_ARG;
    if (p->device >= 0 && hipSetDevice(p->device) == hipSuccess) {
        void* bufs[] = {p->tiles_s_dev, p->tiles_p_dev, p->wbase_s_dev, p->wowner_s_dev, p->off_dev, p->term_ct_dev, p->term_pt_dev};
        for (void* b : bufs)
            if (b) (void)hipFree(b);
    }
    (void)hipGetLastError();  // a failure here must not surface in the caller's next HIP call
    delete p;
    return HE_OK;
}

int he_plan_workspace_bytes(const he_plan* plan, uint32_t limbs, int pt_kind, uint32_t flags, size_t* bytes) {
    if (!plan || !bytes) return HE_ERR_ARG;
    if (pt_kind != HE_PT_SCALAR && pt_kind != HE_PT_POLY) return HE_ERR_ARG;
    if (flags & ~(HE_RESCALE | HE_ACCUMULATE)) return HE_ERR_ARG;
    if ((flags & HE_RESCALE) && (flags & HE_ACCUMULATE)) return HE_ERR_ARG;  // a rescaled output is not a partial sum
    int rc = check_level(plan->ctx, limbs, (flags & HE_RESCALE) ? 2 : 1);
    if (rc != HE_OK) return rc;
    size_t b = 0;
    if (pt_kind == HE_PT_SCALAR) b += align256((size_t)plan->wtab_elems * limbs * sizeof(u64));
    if (flags & HE_RESCALE) b += align256((size_t)plan->n_out * 2 * limbs * plan->ctx->N * sizeof(u64));
    *bytes = b;
    return HE_OK;
}

int he_ct_pt_mac(he_ctx* ctx, const he_plan* plan, uint32_t limbs, const uint64_t* ct_in, const uint64_t* pt,
                 int pt_kind, const uint64_t* bias, uint64_t* ct_out, uint32_t flags, void* workspace,
                 size_t workspace_bytes, void* stream) {
    if (!ctx || !plan || plan->ctx != ctx) return HE_ERR_ARG;
    size_t need = 0;
    int rc = he_plan_workspace_bytes(plan, limbs, pt_kind, flags, &need);
    if (rc != HE_OK) return rc;
    if (plan->n_out == 0) return HE_OK;
    if (!ct_out || (plan->n_terms && (!ct_in || !pt))) return HE_ERR_ARG;
    if (need && (!workspace || workspace_bytes < need)) return HE_ERR_WORKSPACE;
    {   // the output and the workspace are written while the inputs are still being read: neither may share
        // memory with them, nor with each other
        const size_t row = (size_t)ctx->N * sizeof(u64);
        const size_t out_bytes = (size_t)plan->n_out * 2 * ((flags & HE_RESCALE) ? limbs - 1 : limbs) * row;
        const size_t in_bytes = (size_t)plan->n_in * 2 * limbs * row;
        const size_t pt_bytes = (size_t)plan->n_pt * limbs * (pt_kind == HE_PT_POLY ? row : sizeof(u64));
        const size_t bias_bytes = (size_t)plan->n_out * limbs * sizeof(u64);
        if (overlaps(ct_out, out_bytes, ct_in, in_bytes) || overlaps(ct_out, out_bytes, pt, pt_bytes) ||
            overlaps(ct_out, out_bytes, bias, bias_bytes) || overlaps(ct_out, out_bytes, workspace, need) ||
            overlaps(workspace, need, ct_in, in_bytes) || overlaps(workspace, need, pt, pt_bytes) ||
            overlaps(workspace, need, bias, bias_bytes))
            return HE_ERR_ARG;
    }
    if ((rc = check_mac_launch(ctx, plan, limbs, pt_kind)) != HE_OK) return rc;
    if ((flags & HE_RESCALE) && plan->n_out > 0x3FFFFFFFu) return HE_ERR_RANGE;
    if ((rc = need_device(ctx)) != HE_OK) return rc;
    char* ws = (char*)workspace;
    u64* wtab = nullptr;
    if (pt_kind == HE_PT_SCALAR) {
        wtab = (u64*)ws;
        ws += align256((size_t)plan->wtab_elems * limbs * sizeof(u64));
    }
    hipStream_t s = (hipStream_t)stream;
    if (flags & HE_RESCALE) {
        u64* acc = (u64*)ws;
        if ((rc = launch_mac(ctx, plan, limbs, ct_in, pt, pt_kind, bias, acc, wtab, MAC_FOR_RESCALE, s)) != HE_OK) return rc;
        return launch_rescale(ctx, limbs, acc, ct_out, plan->n_out, s);
    }
    return launch_mac(ctx, plan, limbs, ct_in, pt, pt_kind, bias, ct_out, wtab, (flags & HE_ACCUMULATE) ? MAC_ACCUMULATE : 0u, s);
}

// The first half of he_ct_pt_mac(HE_RESCALE) on its own (he_test.h): the accumulators as the fused call leaves them for
// the rescale kernel.  Same checks as the fused call, by way of it.
int he_test_mac_for_rescale(he_ctx* ctx, const he_plan* plan, uint32_t limbs, const uint64_t* ct_in, const uint64_t* pt, int pt_kind,
                            const uint64_t* bias, uint64_t* acc_out, void* workspace, size_t workspace_bytes, void* stream) {
    if (!ctx || !plan || plan->ctx != ctx) return HE_ERR_ARG;
    size_t need = 0;
    int rc = he_plan_workspace_bytes(plan, limbs, pt_kind, 0, &need);
    if (rc != HE_OK) return rc;
    if (limbs < 2) return HE_ERR_LEVEL;
    if (plan->n_out == 0) return HE_OK;
    if (!acc_out || (plan->n_terms && (!ct_in || !pt))) return HE_ERR_ARG;
    if (need && (!workspace || workspace_bytes < need)) return HE_ERR_WORKSPACE;
    if ((rc = check_mac_launch(ctx, plan, limbs, pt_kind)) != HE_OK) return rc;
    if ((rc = need_device(ctx)) != HE_OK) return rc;
    return launch_mac(ctx, plan, limbs, ct_in, pt, pt_kind, bias, acc_out, (u64*)workspace, MAC_FOR_RESCALE, (hipStream_t)stream);
}

int he_ct_pt_mac_static(he_ctx* ctx, const he_plan* plan, uint32_t limbs, const uint64_t* ct_in, const uint64_t* pt,
                        int pt_kind, const uint64_t* bias, uint64_t* ct_out, uint32_t flags, void* stream) {
    if (!ctx || !plan || plan->ctx != ctx) return HE_ERR_ARG;
    size_t need = 0;
    int rc = he_plan_workspace_bytes(plan, limbs, pt_kind, flags, &need);
    if (rc != HE_OK) return rc;
    if (need > HE_STATIC_SCRATCH_BYTES) return HE_ERR_WORKSPACE;  // the fixed array is all there is
    if (ctx->device < 0 || !ctx->static_scratch) return HE_ERR_DEVICE;
    // the same path as he_ct_pt_mac (whose host code allocates nothing), on this GPU's fixed array
    return he_ct_pt_mac(ctx, plan, limbs, ct_in, pt, pt_kind, bias, ct_out, flags, ctx->static_scratch, HE_STATIC_SCRATCH_BYTES,
                        stream);
}

int he_ct_pt_add(he_ctx* ctx, uint32_t limbs, uint64_t* ct, uint32_t n, const uint64_t* pt, int pt_kind,
                 void* stream) {
    int rc = check_level(ctx, limbs, 1);
    if (rc != HE_OK) return rc;
    if (pt_kind != HE_PT_SCALAR && pt_kind != HE_PT_POLY) return HE_ERR_ARG;
    if (n == 0) return HE_OK;
    if (!ct || !pt) return HE_ERR_ARG;
    if ((rc = need_device(ctx)) != HE_OK) return rc;
    const size_t total = (size_t)n * limbs * (ctx->N / 2);
    const size_t blocks = (total + 256 * ADD_UNROLL - 1) / (256 * ADD_UNROLL);
    if (blocks > 0x7FFFFFFFull) return HE_ERR_RANGE;
    if (pt_kind == HE_PT_POLY)
        hipLaunchKernelGGL(add_kernel<true>, dim3((u32)blocks), dim3(256), 0, (hipStream_t)stream, ctx->limbs, limbs, ctx->N,
                           ct, (size_t)n, pt);
    else
        hipLaunchKernelGGL(add_kernel<false>, dim3((u32)blocks), dim3(256), 0, (hipStream_t)stream, ctx->limbs, limbs, ctx->N,
                           ct, (size_t)n, pt);
    HE_HIP(hipGetLastError());
    return HE_OK;
}

int he_rescale(he_ctx* ctx, uint32_t limbs, const uint64_t* in, uint64_t* out, uint32_t n, void* stream) {
    int rc = check_level(ctx, limbs, 2);
    if (rc != HE_OK) return rc;
    if (n == 0) return HE_OK;
    if (!in || !out) return HE_ERR_ARG;
    if (overlaps(in, (size_t)n * 2 * limbs * ctx->N * sizeof(u64), out, (size_t)n * 2 * (limbs - 1) * ctx->N * sizeof(u64)))
        return HE_ERR_ARG;
    if ((rc = need_device(ctx)) != HE_OK) return rc;
    return launch_rescale(ctx, limbs, in, out, n, (hipStream_t)stream);
}

int he_check_reduced(he_ctx* ctx, uint32_t limbs, const uint64_t* data, size_t rows, uint32_t row_len, uint64_t* n_bad,
                     void* stream) {
    int rc = check_level(ctx, limbs, 1);
    if (rc != HE_OK) return rc;
    if (!n_bad || row_len == 0) return HE_ERR_ARG;
    *n_bad = 0;
    if (rows == 0) return HE_OK;
    if (!data) return HE_ERR_ARG;
    if (rows > (~(size_t)0) / limbs / row_len) return HE_ERR_RANGE;
    if ((rc = need_device(ctx)) != HE_OK) return rc;
    const size_t total = rows * limbs * row_len;
    const u32 blocks = (u32)std::min<size_t>((total + 255) / 256, 256 * 32);
    hipStream_t s = (hipStream_t)stream;
    // (this call waits for the stream, so it is never part of a captured graph)
    HE_HIP(hipMemsetAsync(ctx->bad_count, 0, sizeof(u64), s));
    hipLaunchKernelGGL(check_reduced_kernel, dim3(blocks), dim3(256), 0, s, ctx->limbs, limbs, data, total, row_len,
                       (unsigned long long*)ctx->bad_count);
    HE_HIP(hipGetLastError());
    u64 bad = 0;
    HE_HIP(hipMemcpyAsync(&bad, ctx->bad_count, sizeof bad, hipMemcpyDeviceToHost, s));
    HE_HIP(hipStreamSynchronize(s));
    *n_bad = bad;
    return HE_OK;
}

int he_ntt_fwd(he_ctx* ctx, uint32_t limbs, uint64_t* data, uint32_t n_polys, void* stream) {
    int rc = check_level(ctx, limbs, 1);
    if (rc != HE_OK) return rc;
    if (n_polys == 0) return HE_OK;
    if (!data) return HE_ERR_ARG;
    if ((rc = need_device(ctx)) != HE_OK) return rc;
    return launch_ntt(ctx, limbs, data, n_polys, false, (hipStream_t)stream);
}

int he_ntt_inv(he_ctx* ctx, uint32_t limbs, uint64_t* data, uint32_t n_polys, void* stream) {
    int rc = check_level(ctx, limbs, 1);
    if (rc != HE_OK) return rc;
    if (n_polys == 0) return HE_OK;
    if (!data) return HE_ERR_ARG;
    if ((rc = need_device(ctx)) != HE_OK) return rc;
    return launch_ntt(ctx, limbs, data, n_polys, true, (hipStream_t)stream);
}

// ---- ciphertext square + relinearisation

int he_square_relin_workspace_bytes(const he_ctx* ctx, uint32_t limbs, uint32_t n, size_t* bytes) {
    if (!ctx || !bytes) return HE_ERR_ARG;
    if (limbs < 1 || limbs + 1 > ctx->L) return HE_ERR_LEVEL;
    *bytes = square_relin_workspace(ctx, limbs, n);
    return HE_OK;
}

int he_ct_square_relin(he_ctx* ctx, uint32_t limbs, const uint64_t* ct_in, uint32_t n, const uint64_t* evk,
                       uint64_t* ct_out, void* workspace, size_t workspace_bytes, void* stream) {
    if (!ctx || ctx->log2N > HE_MAX_LOG2N_IN_LDS) return HE_ERR_ARG;
    if (limbs < 1 || limbs + 1 > ctx->L) return HE_ERR_LEVEL;
    if (n == 0) return HE_OK;
    if (!ct_in || !evk || !ct_out) return HE_ERR_ARG;
    const size_t need = square_relin_workspace(ctx, limbs, n);
    if (!workspace || workspace_bytes < need) return HE_ERR_WORKSPACE;
    const size_t row = (size_t)ctx->N * sizeof(u64);
    const size_t ct_bytes = (size_t)n * 2 * limbs * row, key_bytes = (size_t)(ctx->L - 1) * 2 * ctx->L * row;
    if (overlaps(ct_out, ct_bytes, ct_in, ct_bytes) || overlaps(ct_out, ct_bytes, evk, key_bytes) ||
        overlaps(ct_out, ct_bytes, workspace, need) || overlaps(ct_in, ct_bytes, workspace, need) ||
        overlaps(evk, key_bytes, workspace, need))
        return HE_ERR_ARG;
    int rc = need_device(ctx);
    if (rc != HE_OK) return rc;
    return launch_square_relin(ctx, limbs, ct_in, n, evk, ct_out, workspace, (hipStream_t)stream);
}

// ---- packed 32-bit storage

// every limb of the level must have a 32-bit form
static int check_level32(const he_ctx* ctx, u32 limbs, u32 min_limbs) {
    int rc = check_level(ctx, limbs, min_limbs);
    if (rc != HE_OK) return rc;
    if (ctx->log2N > HE_MAX_LOG2N_IN_LDS) return HE_ERR_ARG;
    for (u32 i = 0; i < limbs; ++i)
        if (!ctx->limbs32.c[i].ok) return HE_ERR_MODULUS;
    return HE_OK;
}

int he_pack32(he_ctx* ctx, const uint64_t* in, uint32_t* out, size_t count, void* stream) {
    if (!ctx) return HE_ERR_ARG;
    if (count == 0) return HE_OK;
    if (!in || !out) return HE_ERR_ARG;
    if (overlaps(in, count * sizeof(u64), out, count * sizeof(u32))) return HE_ERR_ARG;
    int rc = need_device(ctx);
    if (rc != HE_OK) return rc;
    return launch_pack32(ctx, in, out, count, (hipStream_t)stream);
}

int he_unpack32(he_ctx* ctx, const uint32_t* in, uint64_t* out, size_t count, void* stream) {
    if (!ctx) return HE_ERR_ARG;
    if (count == 0) return HE_OK;
    if (!in || !out) return HE_ERR_ARG;
    if (overlaps(in, count * sizeof(u32), out, count * sizeof(u64))) return HE_ERR_ARG;
    int rc = need_device(ctx);
    if (rc != HE_OK) return rc;
    return launch_unpack32(ctx, in, out, count, (hipStream_t)stream);
}

int he_ct_pt_mac32(he_ctx* ctx, const he_plan* plan, uint32_t limbs, const uint32_t* ct_in, const void* pt, int pt_kind,
                   const uint64_t* bias, uint32_t* ct_out, uint32_t flags, void* workspace, size_t workspace_bytes,
                   void* stream) {
    if (!ctx || !plan || plan->ctx != ctx) return HE_ERR_ARG;
    size_t need = 0;
    int rc = he_plan_workspace_bytes(plan, limbs, pt_kind, flags, &need);
    if (rc != HE_OK) return rc;
    if ((rc = check_level32(ctx, limbs, (flags & HE_RESCALE) ? 2 : 1)) != HE_OK) return rc;
    if (plan->n_out == 0) return HE_OK;
    if (!ct_out || (plan->n_terms && (!ct_in || !pt))) return HE_ERR_ARG;
    if (need && (!workspace || workspace_bytes < need)) return HE_ERR_WORKSPACE;
    {
        const size_t row = (size_t)ctx->N * sizeof(u32);
        const size_t out_bytes = (size_t)plan->n_out * 2 * ((flags & HE_RESCALE) ? limbs - 1 : limbs) * row;
        const size_t in_bytes = (size_t)plan->n_in * 2 * limbs * row;
        const size_t pt_bytes = (size_t)plan->n_pt * limbs * (pt_kind == HE_PT_POLY ? row : sizeof(u64));
        const size_t bias_bytes = (size_t)plan->n_out * limbs * sizeof(u64);
        if (overlaps(ct_out, out_bytes, ct_in, in_bytes) || overlaps(ct_out, out_bytes, pt, pt_bytes) ||
            overlaps(ct_out, out_bytes, bias, bias_bytes) || overlaps(ct_out, out_bytes, workspace, need) ||
            overlaps(workspace, need, ct_in, in_bytes) || overlaps(workspace, need, pt, pt_bytes) ||
            overlaps(workspace, need, bias, bias_bytes))
            return HE_ERR_ARG;
    }
    if ((rc = check_mac32_launch(ctx, plan, limbs, pt_kind)) != HE_OK) return rc;
    if ((flags & HE_RESCALE) && plan->n_out > 0x3FFFFFFFu) return HE_ERR_RANGE;
    if ((rc = need_device(ctx)) != HE_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    if (flags & HE_RESCALE) {
        // the workspace is sized for the 64-bit form: the weight table first, the accumulators after it
        char* ws = (char*)workspace;
        if (pt_kind == HE_PT_SCALAR) ws += align256((size_t)plan->wtab_elems * limbs * sizeof(u64));
        u32* acc = (u32*)ws;
        if ((rc = launch_mac32(ctx, plan, limbs, ct_in, pt, pt_kind, bias, acc, workspace, 0, s)) != HE_OK) return rc;
        return launch_rescale32(ctx, limbs, acc, ct_out, plan->n_out, s);
    }
    return launch_mac32(ctx, plan, limbs, ct_in, pt, pt_kind, bias, ct_out, workspace, (flags & HE_ACCUMULATE) ? 1u : 0u, s);
}

int he_ct_pt_add32(he_ctx* ctx, uint32_t limbs, uint32_t* ct, uint32_t n, const void* pt, int pt_kind, void* stream) {
    int rc = check_level32(ctx, limbs, 1);
    if (rc != HE_OK) return rc;
    if (pt_kind != HE_PT_SCALAR && pt_kind != HE_PT_POLY) return HE_ERR_ARG;
    if (n == 0) return HE_OK;
    if (!ct || !pt) return HE_ERR_ARG;
    if ((rc = need_device(ctx)) != HE_OK) return rc;
    return launch_add32(ctx, limbs, ct, n, pt, pt_kind, (hipStream_t)stream);
}

int he_rescale32(he_ctx* ctx, uint32_t limbs, const uint32_t* in, uint32_t* out, uint32_t n, void* stream) {
    int rc = check_level32(ctx, limbs, 2);
    if (rc != HE_OK) return rc;
    if (n == 0) return HE_OK;
    if (!in || !out) return HE_ERR_ARG;
    if (n > 0x3FFFFFFFu) return HE_ERR_RANGE;
    if (overlaps(in, (size_t)n * 2 * limbs * ctx->N * sizeof(u32), out, (size_t)n * 2 * (limbs - 1) * ctx->N * sizeof(u32)))
        return HE_ERR_ARG;
    if ((rc = need_device(ctx)) != HE_OK) return rc;
    return launch_rescale32(ctx, limbs, in, out, n, (hipStream_t)stream);
}

static int ntt32_entry(he_ctx* ctx, uint32_t limbs, uint32_t* data, uint32_t n_polys, bool inverse, void* stream) {
    int rc = check_level32(ctx, limbs, 1);
    if (rc != HE_OK) return rc;
    if (n_polys == 0) return HE_OK;
    if (!data) return HE_ERR_ARG;
    if ((u64)n_polys * limbs > 0x7FFFFFFFull) return HE_ERR_RANGE;
    if ((rc = need_device(ctx)) != HE_OK) return rc;
    return launch_ntt32(ctx, limbs, data, n_polys * limbs, inverse, (hipStream_t)stream);
}

int he_ntt_fwd32(he_ctx* ctx, uint32_t limbs, uint32_t* data, uint32_t n_polys, void* stream) {
    return ntt32_entry(ctx, limbs, data, n_polys, false, stream);
}

int he_ntt_inv32(he_ctx* ctx, uint32_t limbs, uint32_t* data, uint32_t n_polys, void* stream) {
    return ntt32_entry(ctx, limbs, data, n_polys, true, stream);
}

// ---- host-side checks of the device arithmetic

static LimbConst host_const(u64 q) {
    LimbConst c;
    memset(&c, 0, sizeof c);
    fill_limb_const(c, q, 1, 1);
    return c;
}

uint64_t he_host_reduce128(uint64_t hi, uint64_t lo, uint64_t q) { return reduce128(hi, lo, host_const(q)); }

uint64_t he_host_mulmod(uint64_t a, uint64_t b, uint64_t q) { return mul_mod(a, b, host_const(q)); }

uint64_t he_host_shoup_mulmod(uint64_t y, uint64_t w, uint64_t q) { return shoup_mul(y, w, h_shoup(w, q), q); }

uint64_t he_host_shoup_lazy(uint64_t y, uint64_t w, uint64_t q, int cheap_quotient) {
    return cheap_quotient ? shoup_mul_lazy4(y, w, h_shoup(w, q), q) : shoup_mul_lazy(y, w, h_shoup(w, q), q);
}

uint32_t he_host_barrett64(uint64_t z, uint32_t q) { return barrett64(z, q, (u64)((((u128)1) << 64) / q)); }

uint32_t he_host_shoup32(uint32_t y, uint32_t w, uint32_t q) { return shoup32(y, w, (u32)(((u64)w << 32) / q), q); }

int he_measure_rate(he_ctx* ctx, int kind, uint32_t limb, uint32_t iters, double* ops_per_s) {
    if (!ctx || !ops_per_s || limb >= ctx->L || iters == 0 || iters > (1u << 20)) return HE_ERR_ARG;
    if (kind < HE_RATE_MAD32 || kind > HE_RATE_BUTTERFLY_FP64_INV) return HE_ERR_ARG;
    if ((kind == HE_RATE_BUTTERFLY_FP64 || kind == HE_RATE_BUTTERFLY_FP64_INV) && !ctx->limbs.c[limb].fp_ok) return HE_ERR_MODULUS;
    if (kind == HE_RATE_MAC_TERM3 && ctx->limbs.c[limb].kara_terms == 0) return HE_ERR_MODULUS;  // the limb never takes that form
    // the lazier butterflies assume the room their modes are chosen by
    const u32 mode = ctx->limbs.c[limb].ntt_mode;
    if ((kind == HE_RATE_BUTTERFLY_MODE2 && mode < 2) || ((kind == HE_RATE_BUTTERFLY_MODE1 || kind == HE_RATE_BUTTERFLY_INV) && mode < 1))
        return HE_ERR_MODULUS;
    int rc = need_device(ctx);
    if (rc != HE_OK) return rc;
    return launch_rate(ctx, kind, limb, iters, ops_per_s);
}

uint64_t he_host_mac_accumulate(const uint64_t* x, const uint64_t* w, size_t n, uint64_t q) {
    return he_host_mac_accumulate_add(x, w, n, q, 0);
}

// The unreduced result that a fused layer's MAC hands to its rescale kernel: congruent to sum + addend, below 12q.
uint64_t he_host_mac_accumulate_lazy(const uint64_t* x, const uint64_t* w, size_t n, uint64_t q, uint64_t addend) {
    const LimbConst c = host_const(q);
    MacAcc a;
    acc_clear(a);
    u32 f = 0, r = 0;
    for (size_t t = 0; t < n; ++t) {
        u32 xa, xb, wa, wb;
        split_operand(x[t], c, xa, xb);
        split_operand(w[t], c, wa, wb);
        acc_mac(a, xa, xb, wa, wb);
        ++f;
        ++r;
        if (r + 1 > c.reduce_every) { acc_restart(a, c); r = 0; f = 0; }
        else if (f + 1 > c.fold_every) { acc_fold(a, c); f = 0; }
    }
    if (c.narrow && c.ntt_mode >= 1) return acc_reduce_add_lazy(a, addend, c);
    return acc_reduce_lazy(a, addend, c);
}

uint64_t he_host_mac_accumulate_add(const uint64_t* x, const uint64_t* w, size_t n, uint64_t q, uint64_t addend) {
    const LimbConst c = host_const(q);
    MacAcc a;
    acc_clear(a);
    u32 f = 0, r = 0;
    for (size_t t = 0; t < n; ++t) {
        u32 xa, xb, wa, wb;
        split_operand(x[t], c, xa, xb);
        split_operand(w[t], c, wa, wb);
        acc_mac(a, xa, xb, wa, wb);
        ++f;
        ++r;
        if (r + 1 > c.reduce_every) { acc_restart(a, c); r = 0; f = 0; }
        else if (f + 1 > c.fold_every) { acc_fold(a, c); f = 0; }
    }
    // the final step as the kernels take it
    if (c.narrow && c.ntt_mode >= 1) return acc_reduce_add(a, addend, c);
    return add_mod(acc_reduce(a, c), addend, c.q);
}

// The three-product form of the MAC terms, as the 16-output kernel takes it where the limb allows:
// (sum of x[t]*w[t] + addend) mod q for n <= he_host_mac_three_product_terms(q) terms.  Returns UINT64_MAX if
// n exceeds that.
uint64_t he_host_mac_accumulate_three_products(const uint64_t* x, const uint64_t* w, size_t n, uint64_t q, uint64_t addend) {
    const LimbConst c = host_const(q);
    if (n > c.kara_terms) return ~0ull;
    MacAcc a;
    acc_clear(a);
    for (size_t t = 0; t < n; ++t) {
        u32 xa, xb, wa, wb;
        split_operand(x[t], c, xa, xb);
        split_operand(w[t], c, wa, wb);
        a.lo += (u64)xa * wa;
        a.mid += (u64)(xa + xb) * (wa + wb);
        a.hi += (u64)xb * wb;
    }
    acc_uncross(a);
    return acc_reduce_add(a, addend, c);
}

uint32_t he_host_mac_three_product_terms(uint64_t q) { return host_const(q).kara_terms; }

// Which arithmetic the transforms of limbs below 2^50 use from now on: integer butterflies only (1), or the
// double-precision ones (0, the state a context is created in).
int he_test_integer_transforms(he_ctx* ctx, int integer_only) {
    if (!ctx) return HE_ERR_ARG;
    for (u32 i = 0; i < ctx->L; ++i) ctx->limbs.c[i].fp_ok = !integer_only && ctx->q[i] < (1ull << 50);
    for (u32 j = 0; j < ctx->L; ++j)
        for (u32 i = 0; i < ctx->L; ++i)
            if (i != j) ctx->drop[j][i].fp64 = ctx->limbs.c[i].fp_ok && ctx->drop[j][i].reduce_mode <= 1;
    return HE_OK;
}

// The double-precision forward transform (bfly_fwd_f, fp_reduce, the reduction points of ntt_forward_f) run on the
// host, stage by stage in the textbook loop order.
int he_host_ntt_forward_fp64(he_ctx* ctx, uint32_t limb, const int64_t* in, uint64_t* out, double* max_over_q) {
    if (!ctx || !in || !out || limb >= ctx->L || ctx->log2N > 14) return HE_ERR_ARG;
    const LimbConst& c = ctx->limbs.c[limb];
    if (!c.fp_ok) return HE_ERR_MODULUS;
    const u32 N = ctx->N, log2N = ctx->log2N;
    const u64 q = c.q;
    const double qf = (double)q, q_inv = c.q_inv_f;
    std::vector<double> tw(N), a(N);
    {
        u64 pw = 1;
        for (u32 k = 0; k < N; ++k) {
            tw[h_bitrev(k, log2N)] = fp_centred(pw, q);
            pw = h_mulmod(pw, ctx->psi[limb], q);
        }
    }
    double worst = 0.0;
    bool exact = true;
    auto seen = [&](double v) {
        worst = std::max(worst, std::fabs(v) / qf);
        exact = exact && std::fabs(v) < 9007199254740992.0 && v == std::nearbyint(v);
    };
    for (u32 j = 0; j < N; ++j) {
        if ((u64)std::llabs(in[j]) > q) return HE_ERR_RANGE;
        a[j] = (double)in[j];
    }
    const u32 npass = (log2N + 3) / 4, rem = log2N - 4 * (npass - 1);
    for (u32 s = 0; s < log2N; ++s) {
        const u32 pass = s / 4;
        if (s % 4 == 0 && pass > 0 && !(pass == npass - 1 && pass >= 2 && rem <= 2))
            for (u32 j = 0; j < N; ++j) a[j] = fp_reduce(a[j], qf, q_inv);
        const u32 m = 1u << s, t = N >> (s + 1);
        for (u32 i = 0; i < m; ++i)
            for (u32 j = 2 * i * t; j < 2 * i * t + t; ++j) {
                bfly_fwd_f(a[j], a[j + t], TwiddleF{tw[m + i]}, qf, q_inv);
                seen(a[j]);
                seen(a[j + t]);
            }
    }
    for (u32 j = 0; j < N; ++j) out[j] = fp_to_canonical(fp_reduce(a[j], qf, q_inv), q);
    if (max_over_q) *max_over_q = worst;
    return exact ? HE_OK : HE_ERR_RANGE;
}

// The inverse transform the same way (bfly_inv_f, the reduction points of ntt_inverse_f).
int he_host_ntt_inverse_fp64(he_ctx* ctx, uint32_t limb, const uint64_t* in, uint64_t* out, double* max_over_q) {
    if (!ctx || !in || !out || limb >= ctx->L || ctx->log2N > 14) return HE_ERR_ARG;
    const LimbConst& c = ctx->limbs.c[limb];
    if (!c.fp_ok) return HE_ERR_MODULUS;
    const u32 N = ctx->N, log2N = ctx->log2N;
    const u64 q = c.q;
    const double qf = (double)q, q_inv = c.q_inv_f;
    std::vector<double> tw(N), a(N);
    {
        const u64 psi_inv = h_powmod(ctx->psi[limb], q - 2, q);
        u64 pw = 1;
        for (u32 k = 0; k < N; ++k) {
            tw[h_bitrev(k, log2N)] = fp_centred(pw, q);
            pw = h_mulmod(pw, psi_inv, q);
        }
    }
    double worst = 0.0;
    bool exact = true;
    auto seen = [&](double v) {
        worst = std::max(worst, std::fabs(v) / qf);
        exact = exact && std::fabs(v) < 9007199254740992.0 && v == std::nearbyint(v);
    };
    for (u32 j = 0; j < N; ++j) {
        if (in[j] >= q) return HE_ERR_RANGE;
        a[j] = fp_reduce(fp_from_u52(in[j]), qf, q_inv);
    }
    const u32 npass = (log2N + 3) / 4, rem = log2N - 4 * (npass - 1);
    const double n_inv = fp_centred(c.n_inv, q), w1n_inv = fp_centred(c.w1n_inv, q);
    for (int s = (int)log2N - 1; s >= 0; --s) {
        const u32 pass = (u32)s / 4, nst = pass == npass - 1 ? rem : 4, k = (u32)s % 4;
        if (k == nst - 1 && pass < npass - 1)  // the first stage a pass runs
            for (u32 j = 0; j < N; ++j) a[j] = fp_reduce(a[j], qf, q_inv);
        const u32 m = 1u << s, t = N >> (s + 1);
        for (u32 i = 0; i < m; ++i)
            for (u32 j = 2 * i * t; j < 2 * i * t + t; ++j) {
                if (s == 0) {
                    const double sum = a[j] + a[j + t], dif = a[j] - a[j + t];
                    seen(sum);
                    seen(dif);
                    a[j] = fp_mulmod(n_inv, sum, qf, q_inv);
                    a[j + t] = fp_mulmod(w1n_inv, dif, qf, q_inv);
                } else {
                    seen(a[j] - a[j + t]);
                    bfly_inv_f(a[j], a[j + t], TwiddleF{tw[m + i]}, qf, q_inv);
                    seen(a[j]);
                    if (nst == 4 && k == 2) a[j] = fp_reduce(a[j], qf, q_inv);  // the sums of the second stage run
                }
                seen(a[j]);
                seen(a[j + t]);
            }
    }
    for (u32 j = 0; j < N; ++j) out[j] = fp_to_canonical(fp_reduce(a[j], qf, q_inv), q);
    if (max_over_q) *max_over_q = worst;
    return exact ? HE_OK : HE_ERR_RANGE;
}

}  // extern "C"
