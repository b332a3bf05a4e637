// Internal structures shared by the translation units of the library (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <vector>

#include "../../include/he.h"
#include "he_arith.h"

// The largest ring degree whose rows (8 * N bytes) fit the LDS of a compute unit: the transforms of larger rings are
// split (he_ntt.hip), and the vector encoder and decoder, square + relinearisation and the packed 32-bit path, which are
// built on one-row-per-workgroup kernels, stop here (HE_ERR_ARG above).
#define HE_MAX_LOG2N_IN_LDS 14

// Per-limb constants handed to kernels by value (16 x 168 B; with the other arguments of the largest kernel well
// below the 4 KiB that kernel arguments may take).
struct LimbTable {
    LimbConst c[HE_MAX_LIMBS];
};

// Constants for dropping limb j while keeping limb i < j (Eq. (2) in RNS form).
struct DropConst {
    u64 p_inv, p_inv_shoup;  // q_j^-1 mod q_i and its Shoup companion
    u64 half_mod;            // floor(q_j / 2) mod q_i
    u32 reduce_mode;         // a value below q_j is below q_i already (0), after one subtraction (1), or needs a full reduction (2)
    u32 fp64;                // 1: q_i < 2^50 and q_j <= 2*q_i: the correction's transform runs on doubles (ntt_forward_f)
};

// The constants of one dropped limb against every kept limb, passed to the rescale kernel by value
// (kernel arguments are read with scalar loads, whatever else the kernel does to memory).
struct DropRow {
    DropConst d[HE_MAX_LIMBS];
};

// ---- packed 32-bit storage (moduli below 2^30: Sec. "Ciphertext-plaintext Multiplication", Alg. 6 / Alg. 8)
// Per-limb constants of the 32-bit arithmetic.
struct Limb32 {
    u32 q, two_q;
    u32 n_inv, n_inv_shoup;      // N^-1 mod q and floor(N^-1 * 2^32 / q)
    u32 w1n_inv, w1n_inv_shoup;  // (psi^-brv(1)) * N^-1 and its companion: the last inverse butterfly merged with N^-1
    u64 ratio;                   // floor(2^64 / q): the Barrett ratio of Alg. 6
    u32 ok;                      // 1 if this limb's modulus is below 2^30 (else the limb has no 32-bit form)
    u32 pow48;                   // 2^48 mod q: what the part of a MAC sum above bit 48 is folded back with
};
struct Limb32Table {
    Limb32 c[HE_MAX_LIMBS];
};
// Dropping limb j while keeping limb i < j, 32-bit constants.
struct Drop32 {
    u32 p_inv, p_inv_shoup;  // q_j^-1 mod q_i and floor(that * 2^32 / q_i)
    u32 half_mod;            // floor(q_j / 2) mod q_i
    u32 reduce;              // 1 if q_j > 2 * q_i: a value below q_j is reduced modulo q_i first
};
struct Drop32Row {
    Drop32 d[HE_MAX_LIMBS];
};

struct he_ctx {
    int device;  // -1: host-only
    u32 log2N, N, L;
    u64 q[HE_MAX_LIMBS], psi[HE_MAX_LIMBS];
    LimbTable limbs;
    DropConst drop[HE_MAX_LIMBS][HE_MAX_LIMBS];  // [dropped j][kept i]
    // device tables
    u64* tw_fwd;      // [L][N][2]: (psi^brv(k), Shoup companion), k in [0, N)
    u64* tw_inv;      // [L][N][2]: (psi^-brv(k), Shoup companion); entry 1, the last stage's, is psi^-brv(1) * N^-1
    double* tw_fwd_f; // [L][N]: psi^brv(k) as the double in (-q/2, q/2), for limbs below 2^50 (LimbConst::fp_ok), else zeros
    double* tw_inv_f; // [L][N]: the same for psi^-brv(k)
    double* fft_tw;   // [N/4][2]: e^(-2 pi i k / (N/2)), the twiddles of the encoder's complex FFT
    double* twist;    // [N/2][2]: e^(-i pi j / N), the twist that follows it
    u64* garner;      // [L][L][2]: (q_k^-1 mod q_i, Shoup companion) at [i][k], for the decoder's lift
    u64* half_digits; // [L+1][L]: mixed-radix digits of floor(q_0...q_{l-1} / 2) for every level l
    Limb32Table limbs32;
    u32* tw32_fwd;    // [L][N][2]: (psi^brv(k), floor(that * 2^32 / q)) for limbs below 2^30, else zeros
    u32* tw32_inv;    // [L][N][2]: the same for psi^-brv(k)
    u64* bad_count;   // [1]: the counter of he_check_reduced
    void* static_scratch;  // this GPU's address of the library's fixed scratch array (he_ct_pt_mac_static); not owned
};

// One group of outputs that read the same ciphertexts in the same order.
struct Tile {
    u32 out0;    // first output of the group; the group is out0 .. out0+count-1
    u32 count;   // outputs in the group (1 .. 16)
    u32 term0;   // off[out0]: where the shared term_ct list starts
    u32 n_terms; // terms per output of the group
};

struct he_plan {
    he_ctx* ctx;
    int device;            // the context's device, kept so that the plan can be destroyed after its context
    u32 n_in, n_out, n_pt, n_terms;
    std::vector<u32> off;  // host copy, for argument checks
    // tiles sorted by class; a class-k tile is run by the kernel instance with capacity cap[k]
    u32 class_begin_s[4];  // scalar plaintexts: capacities 1, 4, 16 outputs per thread
    u32 class_begin_p[4];  // polynomial plaintexts: capacities 1, 2, 4 outputs per thread
    u32 min_terms_s[3];    // fewest terms of any scalar tile of the class (0 for an empty class)
    u32 max_terms_s[3];    // most terms of any scalar tile of the class
    u32 max_count_s[3];    // most outputs of any scalar tile of the class
    Tile* tiles_s_dev;
    Tile* tiles_p_dev;
    u64* wbase_s_dev;      // per scalar tile: start of its weights in the gathered table, per limb
    u32* wowner_s_dev;     // per scalar tile: 1 if it fills the table at wbase (tiles with equal plaintexts share one)
    u64 wtab_elems;        // residues per limb in the gathered weight table
    u32 n_tiles_s, n_tiles_p;
    u32* off_dev;
    u32* term_ct_dev;
    u32* term_pt_dev;
};

#define HE_HIP(call)                                   \
    do {                                               \
        if ((call) != hipSuccess) {                    \
            (void)hipGetLastError();                   \
            return HE_ERR_DEVICE;                      \
        }                                              \
    } while (0)

// kernels' launchers (defined in he_mac.hip / he_ntt.hip); all return a he_status
// hipFuncSetAttribute(MaxDynamicSharedMemorySize) for a kernel that needs more than the default
// 64 KiB of LDS: once per kernel and device (`done` is a bit mask over device numbers, one static
// per call site), not on every launch.
inline int allow_dynamic_lds(const void* kernel, size_t bytes, int device, std::atomic<uint32_t>& done, bool row_at_zero = false) {
    const uint32_t bit = 1u << (device & 31);
    if (device < 32 && (done.load(std::memory_order_acquire) & bit)) return HE_OK;
    if (row_at_zero) {
        // the transform kernels form LDS addresses on the premise that their dynamic row starts at LDS
        // address 0, i.e. that the kernel has no static LDS in front of it (lds_row_starts_at_zero)
        hipFuncAttributes attr;
        if (hipFuncGetAttributes(&attr, kernel) != hipSuccess || attr.sharedSizeBytes != 0) {
            (void)hipGetLastError();
            return HE_ERR_DEVICE;
        }
    }
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) {
        (void)hipGetLastError();
        return HE_ERR_DEVICE;
    }
    if (device < 32) done.fetch_or(bit, std::memory_order_release);
    return HE_OK;
}

// `accumulate` argument of the MAC launchers and kernels: bits
enum : u32 {
    MAC_ACCUMULATE = 1,   // add the canonical residues that the output holds (HE_ACCUMULATE)
    MAC_FOR_RESCALE = 2   // the output is the accumulator tensor of a fused layer, read next by the rescale kernel: the
                          // kept limbs of scalar-plaintext sums may be left unreduced (LimbConst::mac_lazy)
};
int check_mac_launch(he_ctx* ctx, const he_plan* plan, u32 limbs, int pt_kind);
int launch_mac(he_ctx* ctx, const he_plan* plan, u32 limbs, const u64* ct_in, const u64* pt, int pt_kind,
               const u64* bias, u64* out, u64* wtab, u32 accumulate, hipStream_t s);
int launch_ntt(he_ctx* ctx, u32 limbs, u64* data, u32 n_polys, bool inverse, hipStream_t s, const u64* src = nullptr);
int launch_rescale(he_ctx* ctx, u32 limbs, const u64* in, u64* out, u32 n, hipStream_t s);
int launch_rate(he_ctx* ctx, int kind, u32 limb, u32 iters, double* ops_per_s);
int launch_rescale_drop(he_ctx* ctx, u32 limbs, u32 drop_id, const u64* in, u64* out, u32 n, hipStream_t s);
int launch_ntt_spread(he_ctx* ctx, u32 limbs, const u64* src, u64* out, u32 n_digit_rows, u32 digits, hipStream_t s);
int launch_ntt_square(he_ctx* ctx, u32 limbs, const u64* ct, u64* d2, u64* digits, u32 n_ct, hipStream_t s);
// square + relinearisation (he_relin.hip)
size_t square_relin_workspace(const he_ctx* ctx, u32 limbs, u32 n);
int launch_square_relin(he_ctx* ctx, u32 limbs, const u64* ct_in, u32 n, const u64* evk, u64* ct_out, void* workspace, hipStream_t s);
// packed 32-bit storage (he_packed32.hip)
int launch_pack32(he_ctx* ctx, const u64* in, u32* out, size_t count, hipStream_t s);
int launch_unpack32(he_ctx* ctx, const u32* in, u64* out, size_t count, hipStream_t s);
int check_mac32_launch(he_ctx* ctx, const he_plan* plan, u32 limbs, int pt_kind);
int launch_mac32(he_ctx* ctx, const he_plan* plan, u32 limbs, const u32* ct_in, const void* pt, int pt_kind, const u64* bias,
                 u32* out, void* workspace, u32 accumulate, hipStream_t s);
int launch_add32(he_ctx* ctx, u32 limbs, u32* ct, u32 n, const void* pt, int pt_kind, hipStream_t s);
int launch_ntt32(he_ctx* ctx, u32 limbs, u32* data, u32 rows, bool inverse, hipStream_t s);
int launch_rescale32(he_ctx* ctx, u32 limbs, const u32* in, u32* out, u32 n, hipStream_t s);
int launch_encode_vector(he_ctx* ctx, u32 limbs, const double* slots, u32 n, double scale, u64* out, hipStream_t s);
int launch_decode_vector(he_ctx* ctx, u32 limbs, const u64* coef, u32 n, double scale, double* slots, hipStream_t s);
