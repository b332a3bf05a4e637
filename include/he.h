/*
 * he.h -- C ABI of the MI355X (gfx950) library for the data-parallel hot path of nGraph-HE2
 * (arXiv 1908.04172): RNS-CKKS ciphertext x plaintext multiply-accumulate over tensors of
 * ciphertexts with scalar-encoded plaintexts, plaintext addition, and lazy rescaling.
 *
 * Conventions
 *  - Residue tensors are row-major uint64 [ct][2][limbs][N]: for fixed (ciphertext, component,
 *    limb) the N residues are contiguous.  Limb i holds residues modulo moduli[i], canonical, in
 *    [0, q_i).  Ciphertexts are in NTT ("double-CRT") form unless a call says otherwise.
 *    `limbs` (1..L) is the level: the first `limbs` moduli of the context are in use; a rescale
 *    drops limb limbs-1.  Inputs outside [0, q_i) are not detected and give undefined residues.
 *  - "dev" pointers are device (HBM) addresses on the context's GPU, 8-byte aligned; "host"
 *    pointers are ordinary host memory.  The caller owns every buffer; the library allocates device
 *    memory only in he_ctx_create and he_plan_create.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All device work is
 *    enqueued on it and no call synchronises with the device, except he_ctx_create,
 *    he_plan_create and the two destroy calls.
 *  - Every call returns HE_OK (0) or a negative he_status; nothing aborts or throws.  Arguments,
 *    sizes and launch shapes are all checked before the first launch: on any status other than
 *    HE_ERR_DEVICE no device work has been enqueued by that call.  HE_ERR_DEVICE reports a failed HIP
 *    call; launches that the same call made before it stay on the stream.
 */
#ifndef HE_H
#define HE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum he_status {
    HE_OK = 0,
    HE_ERR_ARG = -1,       /* NULL pointer, size zero where not allowed, bad flag or kind */
    HE_ERR_MODULUS = -2,   /* a modulus is not a prime = 1 (mod 2N) below 2^62, or repeats */
    HE_ERR_LEVEL = -3,     /* limbs outside [1, L] (or < 2 for a rescale) */
    HE_ERR_RANGE = -4,     /* a plan index or a size is out of range */
    HE_ERR_DEVICE = -5,    /* a HIP call failed, or the context has no device */
    HE_ERR_WORKSPACE = -6  /* workspace missing or too small */
} he_status;

#define HE_PT_SCALAR 0 /* plaintext = one residue per limb (Alg. 2 / 4 / 8) */
#define HE_PT_POLY 1   /* plaintext = N residues per limb, NTT form (Alg. 3 / 7) */

#define HE_RESCALE 1u     /* he_ct_pt_mac flag: finish with one lazy rescale per output */
#define HE_ACCUMULATE 2u  /* he_ct_pt_mac flag: add the sums (and the bias) to what ct_out holds */

#define HE_MAX_LIMBS 16
#define HE_MIN_LOG2N 10
#define HE_MAX_LOG2N 15

typedef struct he_ctx he_ctx;   /* moduli, roots, twiddle tables (device), per-limb constants */
typedef struct he_plan he_plan; /* which ciphertext meets which plaintext in a layer */

const char* he_strerror(int status);

/*
 * Context for ring degree N = 2^log2N and the modulus chain moduli[0..L-1] (host).  Each
 * modulus must be a prime = 1 (mod 2N) below 2^62 (the bound on the moduli in Sec.
 * "Ciphertext-plaintext Multiplication"), all distinct.  For limb i the library fixes
 * psi_i = the smallest primitive 2N-th root of unity modulo q_i; the NTT entry points are defined
 * with respect to it.  device >= 0 selects the GPU (tables are uploaded there); device = -1 makes a
 * host-only context on which only the *_host calls, he_ctx_info and the plan calls work.
 * log2N in [HE_MIN_LOG2N, HE_MAX_LOG2N].  At log2N = 15 a row of residues no longer fits the LDS of a compute unit:
 * he_ntt_fwd, he_ntt_inv and he_rescale (also inside he_ct_pt_mac with HE_RESCALE) run one butterfly stage over
 * global memory and two half-size transforms per row, with the same results; he_encode_vector, he_decode_vector,
 * he_ct_square_relin and the he_*32 calls return HE_ERR_ARG there.
 */
int he_ctx_create(he_ctx** out, uint32_t log2N, uint32_t L, const uint64_t* moduli, int device);
int he_ctx_destroy(he_ctx* ctx);
/* Any of the outputs may be NULL.  psi: host [L]. */
int he_ctx_info(const he_ctx* ctx, uint32_t* log2N, uint32_t* L, uint64_t* moduli, uint64_t* psi);

/*
 * Scalar encoding, Alg. 2 (Sec. "Scalar Encoding"): out[j][i] = [round(scale * values[j])]_{q_i},
 * i < limbs.  The product is one IEEE double multiply; rounding is to nearest with halves away
 * from zero; the residue is the non-negative one.  Products of magnitude >= 2^63 (they are exact
 * integers m*2^e) are reduced exactly.  A non-finite product yields UINT64_MAX in every limb of
 * that entry (never a valid residue).  Encoding at a level below L ("Depth-aware Encoding") is
 * `limbs` < L.
 *   he_encode_scalar:      values dev [n] double  ->  out dev [n][limbs]   (a kernel on `stream`)
 *   he_encode_scalar_host: the same arithmetic on the host, values/out host; returns HE_ERR_ARG
 *                          for a non-finite product.
 */
int he_encode_scalar(he_ctx* ctx, const double* values, size_t n, double scale, uint32_t limbs,
                     uint64_t* out, void* stream);
int he_encode_scalar_host(const he_ctx* ctx, const double* values, size_t n, double scale,
                          uint32_t limbs, uint64_t* out);

/*
 * General encoding, Alg. 1 (Sec. "Scalar Encoding", "General CKKS Encoding"), read as the canonical
 * embedding: vector v of N/2 complex slots -> the polynomial with real integer coefficients
 *     m_j = round( scale * (2/N) * sum_{k < N/2} Re( z_k * r_k^-j ) ),   r_k = exp(i*pi*(2k+1)/N),
 * i.e. m(r_k) = scale*z_k and m(conj r_k) = scale*conj(z_k) up to the rounding (halves away from
 * zero), then the residues [m_j]_{q_i} and the forward NTT of each limb: a plaintext for
 * HE_PT_POLY.  Slots with a non-zero imaginary part are the paper's complex packing
 * (Sec. "Complex packing"); N/2 equal real slots give N equal residues per limb, the value Alg. 2
 * stores once.
 *   slots: dev [n][N/2][2] double (real, imaginary), 16-byte aligned   ->   out: dev [n][limbs][N].
 * The interpolation runs in IEEE double arithmetic (an FFT of N/2 points), so a coefficient of
 * magnitude M carries an error of up to about M * 2^-53 * 4 * log2(N) before the rounding: the
 * integers agree with an exact evaluation to within 1 + that bound.  scale must be positive and
 * finite; non-finite slots give unspecified residues.  Two kernels on `stream`.
 */
int he_encode_vector(he_ctx* ctx, const double* slots, size_t n, double scale, uint32_t limbs,
                     uint64_t* out, void* stream);

/*
 * The inverse of he_encode_vector: poly dev [n][limbs][N] (a plaintext polynomial in NTT form, e.g. a
 * decrypted message at the level given by `limbs`)  ->  slots dev [n][N/2][2] double,
 *     z_k = m(r_k) / scale,
 * m being the polynomial whose coefficients are the integers of smallest magnitude with the given
 * residues (an exact lift, then IEEE double arithmetic: a result is accurate to about
 * N * max|m_j| * 2^-53 * 4 * log2(N) / scale).  poly is not modified; workspace: device memory of at
 * least n*limbs*N*8 bytes (HE_ERR_WORKSPACE otherwise) that overlaps neither poly nor slots (it receives the
 * coefficients).  Two kernels on `stream`.
 */
int he_decode_vector(he_ctx* ctx, const uint64_t* poly, size_t n, double scale, uint32_t limbs,
                     double* slots, void* workspace, size_t workspace_bytes, void* stream);

/*
 * A MAC plan (Sec. "Lazy Rescaling": an FC or Convolution output is a sum over the inner
 * dimension / window):  out[o] = sum over t in [off[o], off[o+1]) of
 * ct_in[term_ct[t]] * pt[term_pt[t]].  All three arrays are host memory and are copied;
 * off has n_out+1 entries, off[0] = 0, non-decreasing; term_ct[t] < n_in; term_pt[t] < n_pt.
 * Outputs that read the same ciphertexts in the same order (the output channels of one
 * convolution window, the outputs of a dense layer) are grouped so that each input is loaded once
 * per group.  Needs a device context.
 */
int he_plan_create(he_ctx* ctx, uint32_t n_in, uint32_t n_out, uint32_t n_pt, const uint32_t* off,
                   const uint32_t* term_ct, const uint32_t* term_pt, he_plan** out);
/* Frees the plan's device arrays.  Valid also after the plan's context was destroyed; every other
 * call on a plan needs its context alive. */
int he_plan_destroy(he_plan* plan);
/* Device bytes he_ct_pt_mac needs in `workspace` for this plan, level and flags. */
int he_plan_workspace_bytes(const he_plan* plan, uint32_t limbs, int pt_kind, uint32_t flags,
                            size_t* bytes);

/*
 * Ciphertext x plaintext multiply-accumulate, Alg. 7 (HE_PT_POLY: pt dev [n_pt][limbs][N], NTT
 * form, slot-wise product) and Alg. 8 (HE_PT_SCALAR: pt dev [n_pt][limbs]) summed per the plan;
 * both ciphertext components are multiplied.  bias (dev [n_out][limbs] scalar residues, or NULL)
 * is added to component 0 after the sum (Alg. 4; "addition is allowed post-multiplication,
 * pre-rescaling").
 *   flags = 0:             ct_out dev [n_out][2][limbs][N]
 *   flags = HE_RESCALE:    ct_out dev [n_out][2][limbs-1][N]; each output is rescaled exactly once,
 *                          after its MACs and bias (lazy rescaling); needs limbs >= 2.
 *   flags = HE_ACCUMULATE: ct_out dev [n_out][2][limbs][N] holds canonical residues on entry and
 *                          ct_out[o] += the sum (+ bias[o] on component 0): the accumulate-into-output
 *                          form of Alg. 7 / Alg. 8 inside a Dot or Convolution.  A layer whose terms are
 *                          split over several calls (several plans over the same outputs) gives the
 *                          residues of the one-call layer.  Not together with HE_RESCALE (HE_ERR_ARG):
 *                          the rescale belongs after the last partial sum, as a he_rescale call.
 * ct_in dev [n_in][2][limbs][N].  ct_out and workspace must not overlap each other nor ct_in, pt or bias
 * (checked on the host: HE_ERR_ARG).
 * workspace: dev, at least he_plan_workspace_bytes() bytes (may be NULL if that is 0).
 */
int he_ct_pt_mac(he_ctx* ctx, const he_plan* plan, uint32_t limbs, const uint64_t* ct_in,
                 const uint64_t* pt, int pt_kind, const uint64_t* bias, uint64_t* ct_out,
                 uint32_t flags, void* workspace, size_t workspace_bytes, void* stream);

/*
 * he_ct_pt_mac for callers that cannot allocate device memory or may not call an allocator: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same operation, arguments,
 * flags and errors as he_ct_pt_mac, but the workspace is a fixed array of HE_STATIC_SCRATCH_BYTES inside
 * the library's device code (each GPU a context was created on holds its copy until the process ends),
 * and the call allocates nothing, on the host's HIP side or the device's.  A plan, level and flags whose
 * he_plan_workspace_bytes() exceeds HE_STATIC_SCRATCH_BYTES is refused with HE_ERR_WORKSPACE (with
 * HE_RESCALE the accumulators of all outputs must fit: use he_ct_pt_mac, or flags = 0 followed by
 * he_rescale, for larger layers).  All calls on one GPU share that GPU's array, whatever their context or
 * stream: calls that overlap in time on one GPU race; calls on one stream do not.  Nothing in the array
 * has to be cleared between calls (every word a call reads it has written itself).
 */
#define HE_STATIC_SCRATCH_BYTES (32u << 20)
int he_ct_pt_mac_static(he_ctx* ctx, const he_plan* plan, uint32_t limbs, const uint64_t* ct_in, const uint64_t* pt,
                        int pt_kind, const uint64_t* bias, uint64_t* ct_out, uint32_t flags, void* stream);

/*
 * Ciphertext + plaintext, Alg. 3 (HE_PT_POLY: pt dev [n][limbs][N]) and Alg. 4 (HE_PT_SCALAR:
 * pt dev [n][limbs]), in place on component 0 of each of the n ciphertexts ct dev
 * [n][2][limbs][N]; component 1 is not touched.
 */
int he_ct_pt_add(he_ctx* ctx, uint32_t limbs, uint64_t* ct, uint32_t n, const uint64_t* pt,
                 int pt_kind, void* stream);

/*
 * Rescaling, Eq. (2), read as ct' = round(ct / q_{limbs-1}) on the integer coefficients:
 * in dev [n][2][limbs][N] (NTT form) -> out dev [n][2][limbs-1][N] (NTT form), limbs >= 2.
 * out must not overlap in (checked on the host: HE_ERR_ARG).
 */
int he_rescale(he_ctx* ctx, uint32_t limbs, const uint64_t* in, uint64_t* out, uint32_t n,
               void* stream);

/*
 * Negacyclic NTT (Sec. "Double-CRT Representation") in place over data dev [n_polys][limbs][N]
 * (a [ct][2][limbs][N] tensor is n_polys = 2*ct).  Forward: coefficients in natural order ->
 * slot j = value of the polynomial at psi_i^(2*bitrev(j)+1), bitrev over log2N bits.  Inverse:
 * the exact inverse map (includes N^-1).  Outputs are canonical.
 */
int he_ntt_fwd(he_ctx* ctx, uint32_t limbs, uint64_t* data, uint32_t n_polys, void* stream);
int he_ntt_inv(he_ctx* ctx, uint32_t limbs, uint64_t* data, uint32_t n_polys, void* stream);

/*
 * The x^2 activation (Sec. "CryptoNets"; "Square" and "Relinearize" in the paper's table of operation
 * runtimes): ct_out = relinearise(ct_in squared).  The ciphertexts live on the first `limbs` limbs of the
 * context, 1 <= limbs <= L-1 (HE_ERR_LEVEL otherwise), and the context's LAST limb is the special prime P of
 * the key switching (Sec. "Homomorphic Encryption": relinearisation by raising the modulus with a special
 * prime).  ct_in, ct_out dev [n][2][limbs][N], NTT form.
 * evk dev [L-1][2][L][N], NTT form, the key of the top level (lower levels use its first `limbs` digits and,
 * of each, the limbs in use and P): for digit j the pair (-a_j s + e_j + P g_j s^2, a_j) modulo q_0...q_{L-2} P,
 * where g_j is 1 modulo q_j and 0 modulo the other q_i.  Computes (d0, d1, d2) = (c0^2, 2 c0 c1, c1^2); cuts d2
 * into its RNS digits (digit j = the coefficients of d2 modulo q_j, as integers in [0, q_j)); sums
 * digit_j * evk[j] over j on the limbs in use and P; divides by P with rounding (Eq. (2), P the dropped limb);
 * adds (d0, d1).  The result is at the same level and scale^2: a he_rescale(limbs) usually follows.
 * workspace: dev, at least he_square_relin_workspace_bytes bytes (HE_ERR_WORKSPACE otherwise); ct_out, ct_in,
 * evk and workspace must not overlap one another (HE_ERR_ARG).
 */
int he_square_relin_workspace_bytes(const he_ctx* ctx, uint32_t limbs, uint32_t n, size_t* bytes);
int he_ct_square_relin(he_ctx* ctx, uint32_t limbs, const uint64_t* ct_in, uint32_t n, const uint64_t* evk,
                       uint64_t* ct_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Packed 32-bit storage: the paper's optimisation for moduli of at most 32 bits (Sec.
 * "Ciphertext-plaintext Multiplication": BarrettReduction64, Alg. 6, and Alg. 8) with the residues
 * stored as uint32, half the bytes of the 64-bit form.  The calls below mirror he_ct_pt_mac,
 * he_ct_pt_add, he_rescale, he_ntt_fwd and he_ntt_inv on tensors dev uint32 [ct][2][limbs][N] and
 * compute the same residues.  Every limb of the level must be below 2^30 (the lazy 32-bit butterflies
 * need 4q < 2^32), else HE_ERR_MODULUS.  Scalar plaintexts and biases stay uint64 [n][limbs], as
 * he_encode_scalar writes them; full-polynomial plaintexts are dev uint32 [n_pt][limbs][N].
 *
 * he_pack32 / he_unpack32 convert `count` residues between the two forms (dev pointers, which must
 * not overlap; values of at least 2^32 lose their high word in he_pack32).
 * he_ct_pt_mac32 takes the same plan and the same workspace size (he_plan_workspace_bytes) as
 * he_ct_pt_mac, and the same flags; the no-overlap rule of he_ct_pt_mac applies.
 */
int he_pack32(he_ctx* ctx, const uint64_t* in, uint32_t* out, size_t count, void* stream);
int he_unpack32(he_ctx* ctx, const uint32_t* in, uint64_t* out, size_t count, void* stream);
int he_ct_pt_mac32(he_ctx* ctx, const he_plan* plan, uint32_t limbs, const uint32_t* ct_in, const void* pt,
                   int pt_kind, const uint64_t* bias, uint32_t* ct_out, uint32_t flags, void* workspace,
                   size_t workspace_bytes, void* stream);
int he_ct_pt_add32(he_ctx* ctx, uint32_t limbs, uint32_t* ct, uint32_t n, const void* pt, int pt_kind,
                   void* stream);
int he_rescale32(he_ctx* ctx, uint32_t limbs, const uint32_t* in, uint32_t* out, uint32_t n, void* stream);
int he_ntt_fwd32(he_ctx* ctx, uint32_t limbs, uint32_t* data, uint32_t n_polys, void* stream);
int he_ntt_inv32(he_ctx* ctx, uint32_t limbs, uint32_t* data, uint32_t n_polys, void* stream);

/*
 * Debug aid for the precondition "every residue is canonical" (the un-reduced accumulators of the MAC
 * kernels rely on it): counts the residues of data dev [rows][limbs][row_len] that are not below the
 * modulus of their limb (row_len = N for ciphertext components and polynomial plaintexts, 1 for scalar
 * plaintexts and biases; a [n][2][limbs][N] tensor is rows = 2n).  Writes the count to *n_bad (host),
 * after waiting for `stream`.  One call at a time per context (the counter lives in the context).
 */
int he_check_reduced(he_ctx* ctx, uint32_t limbs, const uint64_t* data, size_t rows, uint32_t row_len,
                     uint64_t* n_bad, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HE_H */
