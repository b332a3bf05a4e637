// Ciphertext x plaintext multiply-accumulate kernels (Alg. 7 / Alg. 8 summed over a plan).
//
// A thread owns one slot n of one (component, limb) row and the accumulators of a whole group of
// outputs that read the same ciphertexts, so each input residue is loaded once per group and used
// for every output of it.  Products are accumulated unreduced (MacAcc) and reduced once at the end
// (or every LimbConst::reduce_every terms), then the bias residue is added on component 0.
#include "he_internal.h"

namespace {

constexpr int MAC_THREADS = 256;
constexpr int GATHER_BLOCKS = 8;
constexpr u32 BLOCK_TERMS = 4;  // terms per unrolled block; an input is loaded one block before its use
constexpr u32 GROUPS_PER_WG = 8;  // groups of outputs a workgroup of the scalar kernel runs through, at most
constexpr u64 MIN_WORKGROUPS = 256 * 32;  // ... while the launch keeps at least this many workgroups

__host__ __device__ inline u32 padded_terms(u32 n_terms) { return (n_terms + BLOCK_TERMS - 1) / BLOCK_TERMS * BLOCK_TERMS; }

// A term's entry in a 16-output weight table: 16 residues as (wa, wb) pairs, then the 16 sums wa + wb
// (used by the three-product form), 24 64-bit words in all; smaller groups have G words per term.
template <int G>
struct TermStride {
    static constexpr u32 WORDS = G == 16 ? 24 : G;
};

// Weight table for scalar plaintexts: the entry of term t (0 <= t < Kp = n_terms rounded up to a
// multiple of BLOCK_TERMS) of a group starts at wtab[limb*wtab_elems + wbase + t*WORDS]; word g holds the
// two pieces (wa | wb << 32, see MacAcc) of pt[term_pt[off[out0+g] + t]][limb], zero for g >= tile.count or
// t >= n_terms, and in 16-output tables the 32-bit sums wa + wb follow in words 16..23.  The MAC loop then
// reads a term's entry with scalar loads, runs whole blocks of terms, and needs neither a per-output
// branch nor a split of the plaintext operand.  Groups with the same plaintext indices share one table
// (same wbase; the group with wowner set fills it), and every limb's part ends with one entry of padding
// that is read ahead but never used.
template <int G>
__global__ void __launch_bounds__(256) gather_weights_kernel(LimbTable lt, const Tile* tiles, const u64* wbase, const u32* wowner, u32 n_tiles,
                                                             u32 limbs, const u32* off, const u32* term_pt, const u64* pt,
                                                             u64* wtab, u64 wtab_elems) {
    constexpr u32 WORDS = TermStride<G>::WORDS;
    const u32 tile_i = blockIdx.x / GATHER_BLOCKS;
    const u32 sub = blockIdx.x % GATHER_BLOCKS;
    if (tile_i >= n_tiles || !wowner[tile_i]) return;  // a shared table is filled by one of its groups
    const Tile tile = tiles[tile_i];
    const u64 per_limb = (u64)padded_terms(tile.n_terms) * G;
    const u64 total = per_limb * limbs;
    u64* dst = wtab + wbase[tile_i];
    for (u64 i = (u64)sub * blockDim.x + threadIdx.x; i < total; i += (u64)GATHER_BLOCKS * blockDim.x) {
        const u32 limb = (u32)(i / per_limb);
        const u64 rem = i % per_limb;
        const u32 t = (u32)(rem / G), g = (u32)(rem % G);
        u32 wa = 0, wb = 0;
        if (g < tile.count && t < tile.n_terms)
            split_operand(pt[(size_t)term_pt[off[tile.out0 + g] + t] * limbs + limb], lt.c[limb], wa, wb);
        u64* entry = dst + (u64)limb * wtab_elems + (u64)t * WORDS;
        entry[g] = (u64)wa | ((u64)wb << 32);
        if constexpr (G == 16) reinterpret_cast<u32*>(entry + 16)[g] = wa + wb;
    }
}

template <int A>
__device__ __forceinline__ void fold_all(MacAcc (&acc)[A], const LimbConst& c) {
#pragma unroll
    for (int g = 0; g < A; g++) acc_fold(acc[g], c);
}

template <int A>
__device__ __forceinline__ void restart_all(MacAcc (&acc)[A], const LimbConst& c) {
#pragma unroll
    for (int g = 0; g < A; g++) {
        acc_restart(acc[g], c);
        __builtin_amdgcn_sched_barrier(0);  // one reduction at a time: keeps its temporaries few
    }
}

// Called between runs of terms: reduce when `reduce_period` terms have gone by since the last
// reduction, else fold when `fold_period` terms have gone by since the last fold.
template <int A>
__device__ __forceinline__ void housekeeping(MacAcc (&acc)[A], u32& f, u32& r, u32 fold_period, u32 reduce_period,
                                             const LimbConst& c) {
    if (r >= reduce_period) {
        restart_all<A>(acc, c);
        r = 0;
        f = 0;
    } else if (f >= fold_period) {
        fold_all<A>(acc, c);
        f = 0;
    }
}

// A load of read-only, workgroup-uniform data (the plan's tables) through the constant address space:
// it becomes a scalar load wherever it sits, also after hand-issued loads that clobber "memory".
template <typename T>
__device__ __forceinline__ T uniform_load(const T* p) {
    return *(const __attribute__((address_space(4))) T*)(p);
}
__device__ __forceinline__ Tile uniform_load(const Tile* p) {
    return Tile{uniform_load(&p->out0), uniform_load(&p->count), uniform_load(&p->term0), uniform_load(&p->n_terms)};
}

// Eight plaintext residues (as 32-bit pieces) in 16 scalar registers, and (SUMS) their eight sums
// wa + wb in 8 more.  The loads are issued by hand so that they are in flight during multiply-adds
// that do not need them: request<HALF>(term) starts the loads of outputs 8*HALF .. 8*HALF+7 of the
// table entry `term`, arrived() waits for them; between the two calls the registers must not be read.
typedef u32 u32x16 __attribute__((ext_vector_type(16)));
typedef u32 u32x8 __attribute__((ext_vector_type(8)));
template <bool SUMS>
struct ScalarWeights8 {
    u32x16 v;  // (wa, wb) pairs
    u32x8 s;   // wa + wb
    template <int HALF>
    __device__ __forceinline__ void request(const u64* term) {
        if constexpr (HALF == 0) asm volatile("s_load_dwordx16 %0, %1, 0x0" : "=&s"(v) : "s"(term) : "memory");
        else asm volatile("s_load_dwordx16 %0, %1, 0x40" : "=&s"(v) : "s"(term) : "memory");
        if constexpr (SUMS) {
            if constexpr (HALF == 0) asm volatile("s_load_dwordx8 %0, %1, 0x80" : "=&s"(s) : "s"(term) : "memory");
            else asm volatile("s_load_dwordx8 %0, %1, 0xa0" : "=&s"(s) : "s"(term) : "memory");
        }
    }
    __device__ __forceinline__ void arrived() {
        if constexpr (SUMS) asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(v), "+s"(s));
        else asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(v));
    }
};

// One term's multiply-adds into eight of the sixteen outputs (acc_mac, spelt out).  A multiply-add
// that reads the sum its predecessor wrote waits for it (the result takes far longer than the issue
// of one instruction), so the two that go into `mid` are kept 16 instructions apart: four passes over
// the eight outputs, pinned in this order.
template <int FIRST, int A>
__device__ __forceinline__ void scalar_half_term(MacAcc (&acc)[A], u32 xa, u32 xb, const ScalarWeights8<false>& w) {
#pragma unroll
    for (int g = 0; g < 8; g++) acc[FIRST + g].lo += (u64)xa * w.v[2 * g];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int g = 0; g < 8; g++) acc[FIRST + g].mid += (u64)xa * w.v[2 * g + 1];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int g = 0; g < 8; g++) acc[FIRST + g].hi += (u64)xb * w.v[2 * g + 1];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int g = 0; g < 8; g++) acc[FIRST + g].mid += (u64)xb * w.v[2 * g];
}

// The three-product form (Karatsuba): lo += xa*wa, hi += xb*wb, mid += (xa+xb)*(wa+wb); the cross
// terms xa*wb + xb*wa are mid - lo - hi, formed once per output when the sums are read out
// (acc_uncross).  Used where LimbConst::kara_terms says that a whole group's terms fit the sums.
template <int FIRST, int A>
__device__ __forceinline__ void scalar_half_term(MacAcc (&acc)[A], u32 xa, u32 xb, const ScalarWeights8<true>& w) {
    const u32 xs = xa + xb;
#pragma unroll
    for (int g = 0; g < 8; g++) acc[FIRST + g].lo += (u64)xa * w.v[2 * g];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int g = 0; g < 8; g++) acc[FIRST + g].mid += (u64)xs * w.s[g];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int g = 0; g < 8; g++) acc[FIRST + g].hi += (u64)xb * w.v[2 * g + 1];
}

template <int G>
__device__ __forceinline__ void load_weights(u64 (&dst)[G], const u64* wt) {
#pragma unroll
    for (int g = 0; g < G; g++) dst[g] = wt[g];
}

template <int G>
__device__ __forceinline__ void scalar_term(MacAcc (&acc)[G], u64 x, const u64 (&wt)[G], const LimbConst& c) {
    u32 xa, xb;
    split_operand(x, c, xa, xb);
#pragma unroll
    for (int g = 0; g < G; g++) acc_mac(acc[g], xa, xb, (u32)wt[g], (u32)(wt[g] >> 32));
}

// Where ciphertext `ct`'s residue of this thread's (component, limb, slot) is: one 32 x 32 -> 64 bit
// multiply-add (a ciphertext has fewer than 2^32 bytes, so the stride needs no 64-bit multiply).
static_assert(((u64)2 * HE_MAX_LIMBS * 8) << HE_MAX_LOG2N < (1ull << 32), "a ciphertext's byte stride fits 32 bits");
__device__ __forceinline__ const u64* input_at(const u64* x_base, u32 ct, u32 ct_stride_bytes) {
    return reinterpret_cast<const u64*>(reinterpret_cast<const char*>(x_base) + (u64)ct * ct_stride_bytes);
}

// Final reduction, bias (Alg. 4, component 0 only) and store of one group of outputs; the cheaper
// reduction where it applies, chosen once so that the per-output code has no branch.  The group's
// bias residues come in with one load (lane g of every wave fetches output g's) and are handed out
// with lane reads, so the outputs do not each wait for a load of their own.  mode & MAC_ACCUMULATE: the canonical
// residue already at the output's place is added as well (HE_ACCUMULATE); the branches on `mode` are uniform.
template <int G>
__device__ __forceinline__ void store_group(MacAcc (&acc)[G], u32 out0, u32 count, const LimbConst& c, const u64* bias, u32 comp,
                                            u32 limb, u32 limbs, u32 N, u32 n, u64* out, u32 mode) {
    const u32 lane = threadIdx.x % 64;
    u64 bias_lane = 0;
    if (bias != nullptr && comp == 0 && lane < count) bias_lane = bias[(size_t)(out0 + lane) * limbs + limb];
    u64* dst = out + (((size_t)out0 * 2 + comp) * limbs + limb) * N + n;
    const size_t out_stride = (size_t)2 * limbs * N;
    const bool add_old = mode & MAC_ACCUMULATE;
    // MAC_FOR_RESCALE: the output is the accumulator tensor that the rescale kernel reads next.  Its kept limbs
    // need not be canonical there (LimbConst::mac_lazy): the final conditional subtractions, the folding of the
    // sums and the exact quotient are left out, which is most of this step (about 20 vector instructions per
    // output instead of about 70; with the short sums of a convolution window that is a third of the kernel).
    const bool lazy = (mode & MAC_FOR_RESCALE) && limb + 1 < limbs && c.mac_lazy;
    auto bias_of = [&](int g) -> u64 {
        return (u64)(u32)__builtin_amdgcn_readlane((int)(u32)bias_lane, g) |
               ((u64)(u32)__builtin_amdgcn_readlane((int)(u32)(bias_lane >> 32), g) << 32);
    };
    if (c.narrow && c.ntt_mode >= 1) {
        // the constants of the reduction, fetched once and held in registers for all the outputs (left
        // to itself the compiler fetches them again for every output, and waits each time)
        LimbConst k = c;
        asm volatile("" : "+s"(k.q), "+s"(k.mu), "+s"(k.neg_four_q), "+s"(k.neg_two_q), "+s"(k.split_mask), "+s"(k.split_bits), "+s"(k.mu_shift));
        if (lazy) {
#pragma unroll
            for (int g = 0; g < G; g++) {
                if ((u32)g < count) {
                    dst[g * out_stride] = acc_reduce_add_lazy(acc[g], bias_of(g), k);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            return;
        }
#pragma unroll
        for (int g = 0; g < G; g++) {
            if ((u32)g < count) {
                u64 b = bias_of(g);
                if (add_old) b = add_mod(b, dst[g * out_stride], k.q);
                dst[g * out_stride] = acc_reduce_add(acc[g], b, k);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    } else if (lazy) {
#pragma unroll
        for (int g = 0; g < G; g++) {
            if ((u32)g < count) {
                dst[g * out_stride] = acc_reduce_lazy(acc[g], bias_of(g), c);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    } else {
#pragma unroll
        for (int g = 0; g < G; g++) {
            if ((u32)g < count) {
                u64 b = bias_of(g);
                if (add_old) b = add_mod(b, dst[g * out_stride], c.q);
                dst[g * out_stride] = add_mod(acc_reduce(acc[g], c), b, c.q);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
}

// The main path of the scalar MAC kernel (see mac_scalar_kernel): groups tile_first .. tile_end-1, chained.
// KARA selects the three-product form of a term (16-output groups only).
template <int G, bool KARA>
__device__ __forceinline__ void scalar_main_path(const LimbConst& c, u32 limbs, u32 N, const Tile* tiles, u32 tile_first, u32 tile_end,
                                                 const u64* wbase, const u32* term_ct, const u64* wtab, u64 wtab_elems,
                                                 const u64* x_base, u32 ct_stride_bytes, const u64* bias, u32 comp, u32 limb, u32 n,
                                                 u64* out, u32 accumulate) {
    constexpr u32 WS = TermStride<G>::WORDS;
    MacAcc acc[G];
    // Terms run in blocks of four (terms K..Kp-1 are padding: zero weights, input K-1 again).
    // Ring of inputs: xq[j] holds the residue of term t+j and is refilled for term t+j+4 as soon
    // as it has been consumed, so a load has a whole block of MACs (256 multiply-adds per lane, 192
    // in the three-product form) to complete.  The ring looks 8 terms ahead; two blocks before the end of a group it moves
    // on to the next group's list (the host runs several groups per workgroup only if every
    // group has at least 8 padded terms, so the ring is never more than one group ahead).
    // Folds and reductions happen between runs of whole blocks only, so inside a run the partial
    // sums are plain loop-carried registers.
    const u32 fold_blocks = c.fold_every / BLOCK_TERMS * BLOCK_TERMS;
    const u32 reduce_blocks = c.reduce_every / BLOCK_TERMS * BLOCK_TERMS;
    const Tile first = uniform_load(tiles + tile_first);
    u32 Kp = padded_terms(first.n_terms);
    // the list the ring is filled from: term u of the current group (u may run past Kp, into the
    // next group) is term_ct[list0 + min(u, u_last)], the sum taken modulo 2^32 (list0 is the
    // next list's start minus Kp, which may be "negative")
    u32 list0 = first.term0;
    u32 u_last = first.n_terms - 1;
    // weights of the term being multiplied
    const u64* w_limb = wtab + (u64)limb * wtab_elems;
    const u64* wp = w_limb + uniform_load(wbase + tile_first);
    u64 xq[BLOCK_TERMS];
    u32 cq[BLOCK_TERMS];  // ciphertext indices of terms t+4 .. t+7, fetched a block before they are needed
#pragma unroll
    for (int j = 0; j < BLOCK_TERMS; j++) {
        xq[j] = *input_at(x_base, term_ct[(u32)(list0 + min((u32)j, u_last))], ct_stride_bytes);
        cq[j] = term_ct[(u32)(list0 + min((u32)(BLOCK_TERMS + j), u_last))];
    }
    // The plaintext residues of a term sit in scalar registers, eight outputs' worth in each of
    // two sets.  While one set's multiply-adds run, the other set's next load is in flight: at
    // the start of a term w_lo holds this term's residues for outputs 0..7 and the load of w_hi
    // (outputs 8..15) has been issued.  After the last term of the last group the requests reach
    // whatever follows its table (another table or the padding).
    ScalarWeights8<KARA> w_lo, w_hi;
    // where the operands are cut, held in registers for the whole loop (left to itself the
    // compiler fetches the two words again in every block, and waits for them)
    u32 split_mask = (u32)c.split_mask, split_bits = c.split_bits;
    asm volatile("" : "+s"(split_mask), "+s"(split_bits));
    // Smaller groups keep their weights in vector registers, in a ring like the inputs': wq[j] holds the
    // residues of term t+j and is refilled for term t+j+4 once they have been multiplied.
    constexpr int WQ = G == 16 ? 1 : G;
    u64 wq[BLOCK_TERMS][WQ];
    if constexpr (G == 16) {
        w_lo.template request<0>(wp);
        w_lo.arrived();
        w_hi.template request<1>(wp);
    } else {
#pragma unroll
        for (int j = 0; j < BLOCK_TERMS; j++) load_weights<G>(wq[j], wp + j * WS);
    }
    for (u32 tile_i = tile_first; tile_i < tile_end; tile_i++) {
        // the group after this one; after the last one the ring stays on this group's last term
        // (loads that hit in the cache and are never used)
        u32 next_list0 = list0 + u_last, next_K = 1;
        const u64* wp_next_group = wp + (size_t)Kp * WS;  // after the last group: whatever follows its table
        if (tile_i + 1 < tile_end) {
            const Tile next = uniform_load(tiles + tile_i + 1);
            next_list0 = next.term0;
            next_K = next.n_terms;
            wp_next_group = w_limb + uniform_load(wbase + tile_i + 1);
        }
        const Tile cur = uniform_load(tiles + tile_i);
        const u32 out0 = cur.out0, count = cur.count;
#pragma unroll
        for (int g = 0; g < G; g++) acc_clear(acc[g]);
        u32 f = 0, r = 0, t = 0;
        while (t < Kp) {
            const u32 run = min(Kp - t, min(fold_blocks - f, reduce_blocks - r));
            const u32 t_end = t + run;
#pragma unroll 1
            for (; t < t_end; t += BLOCK_TERMS) {
                if (t + 2 * BLOCK_TERMS == Kp) {  // from here on the look-ahead is in the next group
                    list0 = next_list0 - Kp;
                    u_last = Kp + next_K - 1;
                }
                // where the weights of the term after this block are
                const u64* wp_after = t + BLOCK_TERMS == Kp ? wp_next_group : wp + BLOCK_TERMS * WS;
#pragma unroll
                for (int j = 0; j < BLOCK_TERMS; j++) {
                    const u64 x = xq[j];
                    xq[j] = *input_at(x_base, cq[j], ct_stride_bytes);
                    cq[j] = term_ct[(u32)(list0 + min(t + 2 * BLOCK_TERMS + j, u_last))];
                    if constexpr (G == 16) {
                        // (the scheduling barriers keep each half's multiply-adds between a
                        // request and the wait for it, where they hide the load's latency)
                        const u32 xa = (u32)x & split_mask, xb = (u32)(x >> split_bits);  // split_operand
                        __builtin_amdgcn_sched_barrier(0);
                        scalar_half_term<0>(acc, xa, xb, w_lo);
                        __builtin_amdgcn_sched_barrier(0);
                        w_hi.arrived();
                        w_lo.template request<0>(j + 1 < (int)BLOCK_TERMS ? wp + (j + 1) * WS : wp_after);
                        __builtin_amdgcn_sched_barrier(0);
                        scalar_half_term<8>(acc, xa, xb, w_hi);
                        __builtin_amdgcn_sched_barrier(0);
                        w_lo.arrived();
                        w_hi.template request<1>(j + 1 < (int)BLOCK_TERMS ? wp + (j + 1) * WS : wp_after);
                    } else {
                        u64 wt[G];
#pragma unroll
                        for (int g = 0; g < G; g++) wt[g] = wq[j][g];
                        load_weights<G>(wq[j], wp_after + j * WS);
                        scalar_term<G>(acc, x, wt, c);
                    }
                    __builtin_amdgcn_sched_barrier(0);  // one term at a time: keeps the live values few
                }
                wp = wp_after;
            }
            if constexpr (G == 16) w_hi.arrived();  // no load in flight outside the block loop
            f += run;
            r += run;
            if (t < Kp) housekeeping<G>(acc, f, r, fold_blocks, reduce_blocks, c);
        }
        if constexpr (KARA) {
#pragma unroll
        for (int g = 0; g < G; g++) acc_uncross(acc[g]);
    }
    store_group<G>(acc, out0, count, c, bias, comp, limb, limbs, N, n, out, accumulate);
        list0 += Kp;
        u_last -= Kp;
        Kp = padded_terms(next_K);
    }
}

// A workgroup owns one 256-residue slice of one (component, limb) row and `per_wg` consecutive groups
// of outputs, which it handles one after the other.  In the main path the input ring and the scalar
// weights run on into the next group while the current one is still being reduced and stored, so the
// chain of dependent loads that opens a group (descriptor -> term list -> inputs) and the stores that
// close it are paid once per workgroup instead of once per group.
// (`b` is the workgroup's index within the launch of this class.)
template <int G>
__device__ __forceinline__ void mac_scalar_body(u32 b, const LimbTable& lt, u32 limbs, u32 N, const Tile* tiles, u32 n_tiles, u32 per_wg,
                                                u32 max_terms, const u64* wbase, const u32* term_ct, const u64* wtab, u64 wtab_elems,
                                                const u64* ct_in, const u64* bias, u64* out, u32 accumulate) {
    const u32 chunks = N / MAC_THREADS;
    const u32 n_wg_tiles = (n_tiles + per_wg - 1) / per_wg;
    // Order: slice of the row fastest, then run of groups, then (component, limb).  Workgroups go
    // to the eight XCDs round-robin and the number of slices is a multiple of eight, so the same
    // slice of neighbouring groups (which read overlapping inputs) runs on the same XCD, close in
    // time, and hits in its L2, while the slices in flight at any moment cover whole rows.
    const u32 chunk = b % chunks; b /= chunks;
    const u32 tile_first = (b % n_wg_tiles) * per_wg; b /= n_wg_tiles;
    const u32 tile_end = min(tile_first + per_wg, n_tiles);
    const u32 comp = b & 1;
    const u32 limb = b >> 1;
    const LimbConst& c = lt.c[limb];
    const u32 n = chunk * MAC_THREADS + threadIdx.x;
    const size_t ct_stride = (size_t)2 * limbs * N;
    const u64* x_base = ct_in + ((size_t)comp * limbs + limb) * N + n;
    MacAcc acc[G];

    if (c.fold_every >= BLOCK_TERMS && uniform_load(&tiles[tile_first].n_terms) > 0) {
        // three products per term where every group of the launch fits the sums (16-output groups only)
        if (G == 16 && max_terms <= c.kara_terms)
            scalar_main_path<G, G == 16>(c, limbs, N, tiles, tile_first, tile_end, wbase, term_ct, wtab, wtab_elems, x_base,
                                         (u32)(ct_stride * 8), bias, comp, limb, n, out, accumulate);
        else
            scalar_main_path<G, false>(c, limbs, N, tiles, tile_first, tile_end, wbase, term_ct, wtab, wtab_elems, x_base,
                                       (u32)(ct_stride * 8), bias, comp, limb, n, out, accumulate);
        return;
    }
    // Every other case, one group at a time: moduli above 2^60 (they fold more often than once per
    // block), groups without terms.
    for (u32 tile_i = tile_first; tile_i < tile_end; tile_i++) {
        const Tile tile = tiles[tile_i];
        const u32 K = tile.n_terms;
        const u64* w = wtab + (u64)limb * wtab_elems + wbase[tile_i];
        const u32* tc = term_ct + tile.term0;
#pragma unroll
        for (int g = 0; g < G; g++) acc_clear(acc[g]);
        u32 f = 0, r = 0;
        for (u32 t = 0; t < K; ++t) {
            u64 wt[G];
            load_weights<G>(wt, w + (size_t)t * TermStride<G>::WORDS);
            scalar_term<G>(acc, x_base[(size_t)tc[t] * ct_stride], wt, c);
            ++f;
            ++r;
            if (t + 1 < K) housekeeping<G>(acc, f, r, c.fold_every, c.reduce_every, c);
        }
        store_group<G>(acc, tile.out0, tile.count, c, bias, comp, limb, limbs, N, n, out, accumulate);
    }
}

template <int G>
__global__ void __launch_bounds__(MAC_THREADS) __attribute__((amdgpu_waves_per_eu(3, 8)))
mac_scalar_kernel(LimbTable lt, u32 limbs, u32 N, const Tile* tiles, u32 n_tiles, u32 per_wg, u32 max_terms, const u64* wbase,
                  const u32* term_ct, const u64* wtab, u64 wtab_elems, const u64* ct_in, const u64* bias, u64* out, u32 accumulate) {
    mac_scalar_body<G>(blockIdx.x, lt, limbs, N, tiles, n_tiles, per_wg, max_terms, wbase, term_ct, wtab, wtab_elems, ct_in, bias, out, accumulate);
}

// A plan's groups of 5..16 outputs and its groups of 2..4 in one launch: the first `blocks16` workgroups
// take the larger class, the others the smaller one (often the ragged end of a layer: too few workgroups
// to fill the chip in a launch of their own), which so fills in while the larger class drains.
struct ScalarClass {
    const Tile* tiles;
    const u64* wbase;
    u32 n_tiles, per_wg, max_terms, blocks;
};
__global__ void __launch_bounds__(MAC_THREADS) __attribute__((amdgpu_waves_per_eu(3, 8)))
mac_scalar_two_class_kernel(LimbTable lt, u32 limbs, u32 N, ScalarClass c16, ScalarClass c4, const u32* term_ct, const u64* wtab,
                            u64 wtab_elems, const u64* ct_in, const u64* bias, u64* out, u32 accumulate) {
    if (blockIdx.x < c16.blocks)
        mac_scalar_body<16>(blockIdx.x, lt, limbs, N, c16.tiles, c16.n_tiles, c16.per_wg, c16.max_terms, c16.wbase, term_ct, wtab,
                            wtab_elems, ct_in, bias, out, accumulate);
    else
        mac_scalar_body<4>(blockIdx.x - c16.blocks, lt, limbs, N, c4.tiles, c4.n_tiles, c4.per_wg, c4.max_terms, c4.wbase, term_ct, wtab,
                           wtab_elems, ct_in, bias, out, accumulate);
}

// The main path for launches whose groups all have at most eight outputs (a convolution with five
// filters, say): the tables are the 16-output ones, of which only outputs 0..7 are read and multiplied,
// so no multiply-add goes to the empty half of a group.  Eight accumulators per thread leave room for
// five waves per SIMD.  A term's eight residues fill one set of scalar registers; the two sets take the
// even and the odd terms, one being loaded while the other is multiplied.
template <bool KARA>
__device__ __forceinline__ void scalar_eight_path(const LimbConst& c, u32 limbs, u32 N, const Tile* tiles, u32 tile_first, u32 tile_end,
                                                  const u64* wbase, const u32* term_ct, const u64* wtab, u64 wtab_elems,
                                                  const u64* x_base, u32 ct_stride_bytes, const u64* bias, u32 comp, u32 limb, u32 n,
                                                  u64* out, u32 accumulate) {
    constexpr u32 WS = TermStride<16>::WORDS;
    static_assert(BLOCK_TERMS % 2 == 0, "the weight sets alternate term by term");
    MacAcc acc[8];
    // (blocks, ring of inputs, switch to the next group's list, folds: as in scalar_main_path)
    const u32 fold_blocks = c.fold_every / BLOCK_TERMS * BLOCK_TERMS;
    const u32 reduce_blocks = c.reduce_every / BLOCK_TERMS * BLOCK_TERMS;
    const Tile first = uniform_load(tiles + tile_first);
    u32 Kp = padded_terms(first.n_terms);
    u32 list0 = first.term0;
    u32 u_last = first.n_terms - 1;
    const u64* w_limb = wtab + (u64)limb * wtab_elems;
    const u64* wp = w_limb + uniform_load(wbase + tile_first);
    u64 xq[BLOCK_TERMS];
    u32 cq[BLOCK_TERMS];
#pragma unroll
    for (int j = 0; j < BLOCK_TERMS; j++) {
        xq[j] = *input_at(x_base, term_ct[(u32)(list0 + min((u32)j, u_last))], ct_stride_bytes);
        cq[j] = term_ct[(u32)(list0 + min((u32)(BLOCK_TERMS + j), u_last))];
    }
    ScalarWeights8<KARA> w_even, w_odd;
    u32 split_mask = (u32)c.split_mask, split_bits = c.split_bits;
    asm volatile("" : "+s"(split_mask), "+s"(split_bits));
    w_even.template request<0>(wp);
    w_even.arrived();
    for (u32 tile_i = tile_first; tile_i < tile_end; tile_i++) {
        u32 next_list0 = list0 + u_last, next_K = 1;
        const u64* wp_next_group = wp + (size_t)Kp * WS;  // after the last group: whatever follows its table
        if (tile_i + 1 < tile_end) {
            const Tile next = uniform_load(tiles + tile_i + 1);
            next_list0 = next.term0;
            next_K = next.n_terms;
            wp_next_group = w_limb + uniform_load(wbase + tile_i + 1);
        }
        const Tile cur = uniform_load(tiles + tile_i);
        const u32 out0 = cur.out0, count = cur.count;
#pragma unroll
        for (int g = 0; g < 8; g++) acc_clear(acc[g]);
        u32 f = 0, r = 0, t = 0;
        while (t < Kp) {
            const u32 run = min(Kp - t, min(fold_blocks - f, reduce_blocks - r));
            const u32 t_end = t + run;
#pragma unroll 1
            for (; t < t_end; t += BLOCK_TERMS) {
                if (t + 2 * BLOCK_TERMS == Kp) {
                    list0 = next_list0 - Kp;
                    u_last = Kp + next_K - 1;
                }
                const u64* wp_after = t + BLOCK_TERMS == Kp ? wp_next_group : wp + BLOCK_TERMS * WS;
#pragma unroll
                for (int j = 0; j < BLOCK_TERMS; j++) {
                    const u64 x = xq[j];
                    xq[j] = *input_at(x_base, cq[j], ct_stride_bytes);
                    cq[j] = term_ct[(u32)(list0 + min(t + 2 * BLOCK_TERMS + j, u_last))];
                    const u32 xa = (u32)x & split_mask, xb = (u32)(x >> split_bits);  // split_operand
                    const u64* wp_term_after = j + 1 < (int)BLOCK_TERMS ? wp + (j + 1) * WS : wp_after;
                    __builtin_amdgcn_sched_barrier(0);
                    if (j % 2 == 0) {
                        w_odd.template request<0>(wp_term_after);
                        __builtin_amdgcn_sched_barrier(0);
                        scalar_half_term<0>(acc, xa, xb, w_even);
                        __builtin_amdgcn_sched_barrier(0);
                        w_odd.arrived();
                    } else {
                        w_even.template request<0>(wp_term_after);
                        __builtin_amdgcn_sched_barrier(0);
                        scalar_half_term<0>(acc, xa, xb, w_odd);
                        __builtin_amdgcn_sched_barrier(0);
                        w_even.arrived();
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                wp = wp_after;
            }
            f += run;
            r += run;
            if (t < Kp) housekeeping<8>(acc, f, r, fold_blocks, reduce_blocks, c);
        }
        if constexpr (KARA) {
#pragma unroll
            for (int g = 0; g < 8; g++) acc_uncross(acc[g]);
        }
        store_group<8>(acc, out0, count, c, bias, comp, limb, limbs, N, n, out, accumulate);
        list0 += Kp;
        u_last -= Kp;
        Kp = padded_terms(next_K);
    }
}

// Launched instead of mac_scalar_kernel<16> where no group of the class has more than eight outputs and
// every limb and every group can take the main path (the host checks: no modulus that folds more often
// than once per block, no group without terms).  Same grid and block order.
__global__ void __launch_bounds__(MAC_THREADS) __attribute__((amdgpu_waves_per_eu(5, 8)))
mac_scalar_eight_kernel(LimbTable lt, u32 limbs, u32 N, const Tile* tiles, u32 n_tiles, u32 per_wg, u32 max_terms, const u64* wbase,
                        const u32* term_ct, const u64* wtab, u64 wtab_elems, const u64* ct_in, const u64* bias, u64* out, u32 accumulate) {
    const u32 chunks = N / MAC_THREADS;
    const u32 n_wg_tiles = (n_tiles + per_wg - 1) / per_wg;
    u32 b = blockIdx.x;
    const u32 chunk = b % chunks; b /= chunks;
    const u32 tile_first = (b % n_wg_tiles) * per_wg; b /= n_wg_tiles;
    const u32 tile_end = min(tile_first + per_wg, n_tiles);
    const u32 comp = b & 1;
    const u32 limb = b >> 1;
    const LimbConst& c = lt.c[limb];
    const u32 n = chunk * MAC_THREADS + threadIdx.x;
    const u32 ct_stride_bytes = 2 * limbs * N * 8;
    const u64* x_base = ct_in + ((size_t)comp * limbs + limb) * N + n;
    if (max_terms <= c.kara_terms)
        scalar_eight_path<true>(c, limbs, N, tiles, tile_first, tile_end, wbase, term_ct, wtab, wtab_elems, x_base, ct_stride_bytes, bias,
                                comp, limb, n, out, accumulate);
    else
        scalar_eight_path<false>(c, limbs, N, tiles, tile_first, tile_end, wbase, term_ct, wtab, wtab_elems, x_base, ct_stride_bytes, bias,
                                 comp, limb, n, out, accumulate);
}

// Outputs that share their inputs with no other output (one multiply per output is the extreme
// case: a plain Alg. 8 call over a tensor).  There is little arithmetic per byte here, so the kernel
// is shaped for the memory system instead: a thread handles SL pairs of adjacent residues (16-byte
// accesses, SL independent loads in flight), a workgroup 512*SL residues of one row.
template <int SL>
__global__ void __launch_bounds__(MAC_THREADS)
mac_scalar_single_kernel(LimbTable lt, u32 limbs, u32 N, const Tile* tiles, u32 n_tiles, const u64* wbase,
                         const u32* term_ct, const u64* wtab, u64 wtab_elems, const u64* ct_in, const u64* bias, u64* out, u32 accumulate) {
    const u32 per_block = MAC_THREADS * 2 * SL;
    const u32 blocks_per_row = N / per_block;
    u32 b = blockIdx.x;
    const u32 part = b % blocks_per_row; b /= blocks_per_row;
    const u32 tile_i = b % n_tiles; b /= n_tiles;
    const u32 comp = b & 1;
    const u32 limb = b >> 1;
    const Tile tile = tiles[tile_i];
    const LimbConst& c = lt.c[limb];
    const size_t ct_stride = (size_t)2 * limbs * N;
    const size_t row_off = ((size_t)comp * limbs + limb) * N + (size_t)part * per_block;
    const u32 K = tile.n_terms;
    const u64* w = wtab + (u64)limb * wtab_elems + wbase[tile_i];
    const u32* tc = term_ct + tile.term0;

    MacAcc acc[SL][2];
#pragma unroll
    for (int s = 0; s < SL; s++) { acc_clear(acc[s][0]); acc_clear(acc[s][1]); }
    u32 f = 0, r = 0;
    for (u32 t = 0; t < K; ++t) {
        const ulonglong2* row = reinterpret_cast<const ulonglong2*>(ct_in + (size_t)tc[t] * ct_stride + row_off);
        const u64 wv = w[t];
        ulonglong2 x[SL];
#pragma unroll
        for (int s = 0; s < SL; s++) x[s] = row[s * MAC_THREADS + threadIdx.x];
#pragma unroll
        for (int s = 0; s < SL; s++) {
            u32 xa, xb;
            split_operand(x[s].x, c, xa, xb);
            acc_mac(acc[s][0], xa, xb, (u32)wv, (u32)(wv >> 32));
            split_operand(x[s].y, c, xa, xb);
            acc_mac(acc[s][1], xa, xb, (u32)wv, (u32)(wv >> 32));
        }
        ++f;
        ++r;
        if (t + 1 < K) {
            if (r >= c.reduce_every) {
#pragma unroll
                for (int s = 0; s < SL; s++) { acc_restart(acc[s][0], c); acc_restart(acc[s][1], c); }
                r = 0;
                f = 0;
            } else if (f >= c.fold_every) {
#pragma unroll
                for (int s = 0; s < SL; s++) { acc_fold(acc[s][0], c); acc_fold(acc[s][1], c); }
                f = 0;
            }
        }
    }
    const u32 o = tile.out0;
    const u64 bv = (bias != nullptr && comp == 0) ? bias[(size_t)o * limbs + limb] : 0;
    ulonglong2* dst = reinterpret_cast<ulonglong2*>(out + (size_t)o * ct_stride + row_off);
#pragma unroll
    for (int s = 0; s < SL; s++) {
        ulonglong2 v;
        v.x = add_mod(acc_reduce(acc[s][0], c), bv, c.q);
        v.y = add_mod(acc_reduce(acc[s][1], c), bv, c.q);
        if (accumulate & MAC_ACCUMULATE) {
            const ulonglong2 old = dst[s * MAC_THREADS + threadIdx.x];
            v.x = add_mod(v.x, old.x, c.q);
            v.y = add_mod(v.y, old.y, c.q);
        }
        dst[s * MAC_THREADS + threadIdx.x] = v;
    }
}

// Full-polynomial plaintexts: the plaintext residue differs per slot, is loaded once and used for
// both ciphertext components.  A thread owns two adjacent slots (16-byte accesses) of one limb, for
// G outputs x 2 components: 4*G accumulators.
template <int G>
__global__ void __launch_bounds__(MAC_THREADS)
mac_poly_kernel(LimbTable lt, u32 limbs, u32 N, const Tile* tiles, u32 n_tiles, const u32* off, const u32* term_ct, const u32* term_pt,
                const u64* pt, const u64* ct_in, const u64* bias, u64* out, u32 accumulate) {
    const u32 chunks = N / (2 * MAC_THREADS);
    u32 b = blockIdx.x;  // same order as the scalar kernel: slice, group of outputs, limb
    const u32 chunk = b % chunks; b /= chunks;
    const u32 tile_i = b % n_tiles;
    const u32 limb = b / n_tiles;
    const Tile tile = tiles[tile_i];
    const LimbConst& c = lt.c[limb];
    const u32 n = 2 * (chunk * MAC_THREADS + threadIdx.x);
    const size_t ct_stride = (size_t)2 * limbs * N;
    const size_t comp_stride = (size_t)limbs * N;
    const u64* x_base = ct_in + (size_t)limb * N + n;
    const u64* p_base = pt + (size_t)limb * N + n;
    const size_t pt_stride = (size_t)limbs * N;
    const u32* tc = term_ct + tile.term0;
    const u32 K = tile.n_terms;
    const u32* tp[G];
#pragma unroll
    for (int g = 0; g < G; g++) tp[g] = term_pt + off[tile.out0 + ((u32)g < tile.count ? g : 0)];

    MacAcc acc[4 * G];  // [output][component][slot]
#pragma unroll
    for (int g = 0; g < 4 * G; g++) acc_clear(acc[g]);
    u32 f = 0, r = 0;
    // The operands of term t + 1 are requested before term t is multiplied: twice the bytes in flight per wave
    // (the kernel is bound by HBM latency times the bytes outstanding).  Outputs beyond the group's count read the
    // first output's plaintexts again (tp[g] points there) and are not stored.
    ulonglong2 x0, x1, p[G];
    auto request = [&](u32 t, ulonglong2& a0, ulonglong2& a1, ulonglong2 (&w)[G]) {
        const u64* xp = x_base + (size_t)tc[t] * ct_stride;
        a0 = *reinterpret_cast<const ulonglong2*>(xp);
        a1 = *reinterpret_cast<const ulonglong2*>(xp + comp_stride);
#pragma unroll
        for (int g = 0; g < G; g++) {
            // read once: a non-temporal load keeps it from displacing the reused ciphertext rows in L2
            const u64* src = p_base + (size_t)tp[g][t] * pt_stride;
            w[g].x = __builtin_nontemporal_load(src);
            w[g].y = __builtin_nontemporal_load(src + 1);
        }
    };
    if (K > 0) request(0, x0, x1, p);
    for (u32 t = 0; t < K; t++) {
        ulonglong2 x0n = x0, x1n = x1, pn[G];
#pragma unroll
        for (int g = 0; g < G; g++) pn[g] = p[g];
        if (t + 1 < K) request(t + 1, x0n, x1n, pn);
        u32 xa[4], xb[4];  // [component][slot]
        split_operand(x0.x, c, xa[0], xb[0]);
        split_operand(x0.y, c, xa[1], xb[1]);
        split_operand(x1.x, c, xa[2], xb[2]);
        split_operand(x1.y, c, xa[3], xb[3]);
#pragma unroll
        for (int g = 0; g < G; g++) {
            u32 pa0, pb0, pa1, pb1;
            split_operand(p[g].x, c, pa0, pb0);
            split_operand(p[g].y, c, pa1, pb1);
            acc_mac(acc[4 * g + 0], xa[0], xb[0], pa0, pb0);
            acc_mac(acc[4 * g + 1], xa[1], xb[1], pa1, pb1);
            acc_mac(acc[4 * g + 2], xa[2], xb[2], pa0, pb0);
            acc_mac(acc[4 * g + 3], xa[3], xb[3], pa1, pb1);
        }
        ++f;
        ++r;
        if (t + 1 < K) housekeeping<4 * G>(acc, f, r, c.fold_every, c.reduce_every, c);
        x0 = x0n;
        x1 = x1n;
#pragma unroll
        for (int g = 0; g < G; g++) p[g] = pn[g];
    }
#pragma unroll
    for (int g = 0; g < G; g++) {
        if ((u32)g < tile.count) {
            const u32 o = tile.out0 + g;
            const u64 bv = bias != nullptr ? bias[(size_t)o * limbs + limb] : 0;
            ulonglong2 v0, v1;
            v0.x = add_mod(acc_reduce(acc[4 * g + 0], c), bv, c.q);
            v0.y = add_mod(acc_reduce(acc[4 * g + 1], c), bv, c.q);
            v1.x = acc_reduce(acc[4 * g + 2], c);
            v1.y = acc_reduce(acc[4 * g + 3], c);
            u64* dst = out + ((size_t)o * 2 * limbs + limb) * N + n;
            if (accumulate & MAC_ACCUMULATE) {
                const ulonglong2 o0 = *reinterpret_cast<const ulonglong2*>(dst), o1 = *reinterpret_cast<const ulonglong2*>(dst + comp_stride);
                v0.x = add_mod(v0.x, o0.x, c.q);
                v0.y = add_mod(v0.y, o0.y, c.q);
                v1.x = add_mod(v1.x, o1.x, c.q);
                v1.y = add_mod(v1.y, o1.y, c.q);
            }
            *reinterpret_cast<ulonglong2*>(dst) = v0;
            *reinterpret_cast<ulonglong2*>(dst + comp_stride) = v1;
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

}  // namespace

// tile classes: scalar plaintexts hold up to {1,4,16} outputs per thread, polynomial ones {1,2,4}
template <int G>
static int gather_scalar_class(he_ctx* ctx, const he_plan* plan, int cls, u32 limbs, const u64* pt, u64* wtab, hipStream_t s) {
    const u32 begin = plan->class_begin_s[cls], count = plan->class_begin_s[cls + 1] - begin;
    hipLaunchKernelGGL((gather_weights_kernel<G>), dim3(count * GATHER_BLOCKS), dim3(256), 0, s, ctx->limbs, plan->tiles_s_dev + begin,
                       plan->wbase_s_dev + begin, plan->wowner_s_dev + begin, count, limbs, plan->off_dev, plan->term_pt_dev, pt, wtab,
                       plan->wtab_elems);
    HE_HIP(hipGetLastError());
    return HE_OK;
}

// Grid of mac_scalar_kernel / mac_scalar_eight_kernel for a class: several groups per workgroup where the
// kernel can run from one into the next (see mac_scalar_kernel) and where enough workgroups remain to keep
// every compute unit's wave slots full several times over.
static int scalar_class_grid(he_ctx* ctx, const he_plan* plan, int cls, u32 limbs, ScalarClass& g) {
    const u32 begin = plan->class_begin_s[cls], count = plan->class_begin_s[cls + 1] - begin;
    const u64 per_group = (u64)limbs * 2 * (ctx->N / MAC_THREADS);
    u32 per_wg = plan->min_terms_s[cls] > BLOCK_TERMS ? GROUPS_PER_WG : 1;
    while (per_wg > 1 && (u64)((count + per_wg - 1) / per_wg) * per_group < MIN_WORKGROUPS) per_wg /= 2;
    const u64 blocks = (u64)((count + per_wg - 1) / per_wg) * per_group;
    if (blocks > 0x3FFFFFFFull) return HE_ERR_RANGE;
    g = ScalarClass{plan->tiles_s_dev + begin, plan->wbase_s_dev + begin, count, per_wg, plan->max_terms_s[cls], (u32)blocks};
    return HE_OK;
}

// groups of at most eight outputs: the kernel that multiplies only the first half of a table entry
static bool eight_outputs_suffice(he_ctx* ctx, const he_plan* plan, u32 limbs) {
    bool eight = plan->max_count_s[2] <= 8 && plan->min_terms_s[2] > 0;
    for (u32 i = 0; i < limbs; i++) eight = eight && ctx->limbs.c[i].fold_every >= BLOCK_TERMS;
    return eight;
}

template <int G>
static int launch_scalar_class(he_ctx* ctx, const he_plan* plan, int cls, u32 limbs, const u64* ct_in, const u64* pt,
                               const u64* bias, u64* out, u64* wtab, u32 accumulate, hipStream_t s) {
    const u32 begin = plan->class_begin_s[cls], count = plan->class_begin_s[cls + 1] - begin;
    if (count == 0) return HE_OK;
    const Tile* tiles = plan->tiles_s_dev + begin;
    const u64* wbase = plan->wbase_s_dev + begin;
    if (int rc = gather_scalar_class<G>(ctx, plan, cls, limbs, pt, wtab, s)) return rc;
    if constexpr (G == 1) {
        const u32 sl = ctx->N >= 2048 ? 4 : 2;
        const u64 blocks = (u64)count * limbs * 2 * (ctx->N / (MAC_THREADS * 2 * sl));
        if (blocks > 0x7FFFFFFFull) return HE_ERR_RANGE;
        if (sl == 4)
            hipLaunchKernelGGL((mac_scalar_single_kernel<4>), dim3((u32)blocks), dim3(MAC_THREADS), 0, s, ctx->limbs, limbs, ctx->N,
                               tiles, count, wbase, plan->term_ct_dev, wtab, plan->wtab_elems, ct_in, bias, out, accumulate);
        else
            hipLaunchKernelGGL((mac_scalar_single_kernel<2>), dim3((u32)blocks), dim3(MAC_THREADS), 0, s, ctx->limbs, limbs, ctx->N,
                               tiles, count, wbase, plan->term_ct_dev, wtab, plan->wtab_elems, ct_in, bias, out, accumulate);
        HE_HIP(hipGetLastError());
        return HE_OK;
    } else {
        ScalarClass g;
        if (int rc = scalar_class_grid(ctx, plan, cls, limbs, g)) return rc;
        if (G == 16 && eight_outputs_suffice(ctx, plan, limbs))
            hipLaunchKernelGGL(mac_scalar_eight_kernel, dim3(g.blocks), dim3(MAC_THREADS), 0, s, ctx->limbs, limbs, ctx->N, tiles, count,
                               g.per_wg, g.max_terms, wbase, plan->term_ct_dev, wtab, plan->wtab_elems, ct_in, bias, out, accumulate);
        else
            hipLaunchKernelGGL((mac_scalar_kernel<G>), dim3(g.blocks), dim3(MAC_THREADS), 0, s, ctx->limbs, limbs, ctx->N, tiles, count,
                               g.per_wg, g.max_terms, wbase, plan->term_ct_dev, wtab, plan->wtab_elems, ct_in, bias, out, accumulate);
        HE_HIP(hipGetLastError());
        return HE_OK;
    }
}

// Classes 1 (2..4 outputs) and 2 (5..16 outputs) together, in one launch, when the plan has both.
static int launch_scalar_classes_4_16(he_ctx* ctx, const he_plan* plan, u32 limbs, const u64* ct_in, const u64* pt, const u64* bias,
                                      u64* out, u64* wtab, u32 accumulate, hipStream_t s) {
    const bool has4 = plan->class_begin_s[2] > plan->class_begin_s[1], has16 = plan->class_begin_s[3] > plan->class_begin_s[2];
    if (!has4 || !has16 || eight_outputs_suffice(ctx, plan, limbs)) {
        if (int rc = launch_scalar_class<4>(ctx, plan, 1, limbs, ct_in, pt, bias, out, wtab, accumulate, s)) return rc;
        return launch_scalar_class<16>(ctx, plan, 2, limbs, ct_in, pt, bias, out, wtab, accumulate, s);
    }
    ScalarClass c4, c16;
    if (int rc = scalar_class_grid(ctx, plan, 1, limbs, c4)) return rc;
    if (int rc = scalar_class_grid(ctx, plan, 2, limbs, c16)) return rc;
    if (int rc = gather_scalar_class<4>(ctx, plan, 1, limbs, pt, wtab, s)) return rc;
    if (int rc = gather_scalar_class<16>(ctx, plan, 2, limbs, pt, wtab, s)) return rc;
    hipLaunchKernelGGL(mac_scalar_two_class_kernel, dim3(c16.blocks + c4.blocks), dim3(MAC_THREADS), 0, s, ctx->limbs, limbs, ctx->N, c16, c4,
                       plan->term_ct_dev, wtab, plan->wtab_elems, ct_in, bias, out, accumulate);
    HE_HIP(hipGetLastError());
    return HE_OK;
}

template <int G>
static int launch_poly_class(he_ctx* ctx, const he_plan* plan, int cls, u32 limbs, const u64* ct_in, const u64* pt,
                             const u64* bias, u64* out, u32 accumulate, hipStream_t s) {
    const u32 begin = plan->class_begin_p[cls], count = plan->class_begin_p[cls + 1] - begin;
    if (count == 0) return HE_OK;
    const u64 blocks = (u64)count * limbs * (ctx->N / (2 * MAC_THREADS));
    if (blocks > 0x7FFFFFFFull) return HE_ERR_RANGE;
    hipLaunchKernelGGL((mac_poly_kernel<G>), dim3((u32)blocks), dim3(MAC_THREADS), 0, s, ctx->limbs, limbs, ctx->N,
                       plan->tiles_p_dev + begin, count, plan->off_dev, plan->term_ct_dev, plan->term_pt_dev, pt, ct_in, bias, out, accumulate);
    HE_HIP(hipGetLastError());
    return HE_OK;
}

// The grid sizes launch_mac would use, checked without launching anything (the entry point calls this first,
// so that a plan too large for a grid is refused before any kernel of the call is on the stream).
int check_mac_launch(he_ctx* ctx, const he_plan* plan, u32 limbs, int pt_kind) {
    if (pt_kind == HE_PT_SCALAR) {
        const u64 singles = plan->class_begin_s[1] - plan->class_begin_s[0];
        const u32 sl = ctx->N >= 2048 ? 4 : 2;
        if (singles * limbs * 2 * (ctx->N / (MAC_THREADS * 2 * sl)) > 0x7FFFFFFFull) return HE_ERR_RANGE;
        u64 blocks = 0;
        for (int cls = 1; cls <= 2; cls++) {
            ScalarClass g;
            if (plan->class_begin_s[cls + 1] == plan->class_begin_s[cls]) continue;
            if (int rc = scalar_class_grid(ctx, plan, cls, limbs, g)) return rc;
            blocks += g.blocks;
        }
        if (blocks > 0x7FFFFFFFull) return HE_ERR_RANGE;  // the two classes may share one launch
    } else {
        for (int cls = 0; cls < 3; cls++) {
            const u64 count = plan->class_begin_p[cls + 1] - plan->class_begin_p[cls];
            if (count * limbs * (ctx->N / (2 * MAC_THREADS)) > 0x7FFFFFFFull) return HE_ERR_RANGE;
        }
    }
    return HE_OK;
}

int launch_mac(he_ctx* ctx, const he_plan* plan, u32 limbs, const u64* ct_in, const u64* pt, int pt_kind, const u64* bias,
               u64* out, u64* wtab, u32 accumulate, hipStream_t s) {
    int rc;
    if (pt_kind == HE_PT_SCALAR) {
        if ((rc = launch_scalar_class<1>(ctx, plan, 0, limbs, ct_in, pt, bias, out, wtab, accumulate, s)) != HE_OK) return rc;
        if ((rc = launch_scalar_classes_4_16(ctx, plan, limbs, ct_in, pt, bias, out, wtab, accumulate, s)) != HE_OK) return rc;
    } else {
        if ((rc = launch_poly_class<1>(ctx, plan, 0, limbs, ct_in, pt, bias, out, accumulate, s)) != HE_OK) return rc;
        if ((rc = launch_poly_class<2>(ctx, plan, 1, limbs, ct_in, pt, bias, out, accumulate, s)) != HE_OK) return rc;
        if ((rc = launch_poly_class<4>(ctx, plan, 2, limbs, ct_in, pt, bias, out, accumulate, s)) != HE_OK) return rc;
    }
    return HE_OK;
}
