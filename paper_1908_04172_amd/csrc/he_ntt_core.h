// The register-resident negacyclic transform's geometry and data movement, shared by the 64-bit and the packed
// 32-bit kernels: which index a register of a thread holds in each pass, the regrouping of the residues through
// the LDS between passes, and the loading of a pass's twiddles.  The butterflies themselves are the residue
// width's own (he_ntt.hip, he_packed32.hip).
//
// One workgroup transforms one polynomial limb (N residues).  Each of the T = N/16 threads keeps
// 16 residues in registers and runs up to four butterfly stages on them (a "pass") before the
// workgroup regroups the residues through LDS for the next pass.  Stage s (s = 0 .. log2N-1) pairs
// indices that differ in bit log2N-1-s, so pass p owns index bits [log2N-1-4p .. log2N-4-4p]; the
// last pass owns what is left at the bottom (1..4 stages) plus, to fill its 16 registers, the top
// bits again, so that consecutive threads hold consecutive short runs and global stores stay dense.
// A twiddle that is the same for the whole wavefront is read through the constant address space: a scalar
// load into scalar registers (the tables are never written by a kernel).  It takes no vector register, and it
// does not queue behind the vector stores of the previous row as a vector load would.
#pragma once
#include "he_arith.h"

namespace {

template <int LOGN>
struct Geo {
    static constexpr int N = 1 << LOGN;
    static constexpr int T = N / 16;
    static constexpr int NPASS = (LOGN + 3) / 4;
    static constexpr int REM = LOGN - 4 * (NPASS - 1);  // stages of the last pass, 1..4
};

// Index of register e of thread tid while pass P is being computed.  In the last pass the registers
// own the lowest REM index bits (the stages left) and, to fill 16 registers, the 4-REM bits just above
// the six bits that the lane number owns, so that a wavefront holds one aligned block of 1024.
template <int LOGN, int P>
__host__ __device__ constexpr u32 reg_index(u32 tid, u32 e) {
    using G = Geo<LOGN>;
    if constexpr (P < G::NPASS - 1) {
        constexpr int low = LOGN - 4 * (P + 1);
        u32 hi = tid >> low, lo = tid & ((1u << low) - 1);
        return (hi << (low + 4)) | (e << low) | lo;
    } else if constexpr (G::REM == 4) {
        return (tid << 4) | e;
    } else {
        u32 e_hi = e >> G::REM, e_lo = e & ((1u << G::REM) - 1);
        u32 wave = tid >> 6, lane = tid & 63u;
        return (wave << 10) | (e_hi << (G::REM + 6)) | (lane << G::REM) | e_lo;
    }
}

// True when, in pass P, every wavefront (64 consecutive threads) holds exactly the aligned block of
// 1024 indices with its own number: a regrouping between two such passes moves data only within
// wavefronts.  Checked over all threads and registers at compile time.
template <int LOGN, int P>
constexpr bool wave_holds_own_block() {
    for (u32 tid = 0; tid < (u32)Geo<LOGN>::T; tid++)
        for (u32 e = 0; e < 16; e++)
            if ((reg_index<LOGN, P>(tid, e) >> 10) != (tid >> 6)) return false;
    return true;
}

// LDS placement: XOR the low index bits with higher ones so that the strided access patterns of
// the regrouping steps spread over the banks.  A bijection on every aligned block of 1024 indices.
__host__ __device__ constexpr u32 lds_slot(u32 idx) {
    return idx ^ (((idx >> 6) & 0xFu) << 2) ^ ((idx >> 5) & 3u);
}

// Workgroup barrier that orders LDS traffic only: waits for this wave's LDS operations, then for the
// other waves.  (A full __syncthreads() would also wait for outstanding global loads, and the
// twiddles of the next pass are deliberately in flight across the regrouping.)
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// The same for data that stays within one wavefront: the LDS serves a wave's operations in the order
// they were issued, so the wave only has to keep that order (and nothing may be moved across by the
// compiler); other waves are not waited for and run ahead or behind freely.
__device__ __forceinline__ void lds_wave_order() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// (V: the residue type, u64 or u32; the row in the LDS is N of them)
template <int LOGN, int PFROM, int PTO, typename V>
__device__ __forceinline__ void regroup(V (&a)[16], V* lds, u32 tid) {
    constexpr bool WAVE_LOCAL = wave_holds_own_block<LOGN, PFROM>() && wave_holds_own_block<LOGN, PTO>();
    // reg_index(tid, e) = reg_index(tid, 0) ^ reg_index(0, e) (disjoint bits) and lds_slot is linear
    // over XOR, so each address is one XOR of a per-thread base with a compile-time constant
    // The two bases are derived from copies of the thread index that the optimizer cannot relate to
    // each other or to other passes: a regrouping writes where the previous one read, and addresses
    // kept alive from one to the next would cost more registers than the few operations they save.
    u32 tid_w = tid, tid_r = tid;
    asm("; regroup %1 write" : "+v"(tid_w) : "n"(PFROM * 16 + PTO));
    asm("; regroup %1 read" : "+v"(tid_r) : "n"(PFROM * 16 + PTO));
    // Addresses are formed as LDS byte addresses outright, one XOR per access: (row + from) ^ constant equals
    // row + (from ^ constant) because the row starts at LDS address 0 -- a workgroup's LDS addresses are relative
    // to its own allocation, and these kernels have no static LDS in front of the dynamic row (the launchers
    // check that: lds_row_starts_at_zero).
    typedef __attribute__((address_space(3))) V lds_v;
    constexpr u32 W = sizeof(V);
    const u32 row = (u32)(uintptr_t)(lds_v*)lds;
    const u32 from = row + lds_slot(reg_index<LOGN, PFROM>(tid_w, 0)) * W, to = row + lds_slot(reg_index<LOGN, PTO>(tid_r, 0)) * W;
    // earlier readers of the slots written here are done: all waves, or (wave-local) this wave only,
    // since its block of slots is then touched by no other wave until the next workgroup-wide regrouping
    if constexpr (WAVE_LOCAL) lds_wave_order(); else lds_barrier();
#pragma unroll
    for (u32 e = 0; e < 16; e++) *(lds_v*)(uintptr_t)(from ^ (lds_slot(reg_index<LOGN, PFROM>(0, e)) * W)) = a[e];
    if constexpr (WAVE_LOCAL) lds_wave_order(); else lds_barrier();
#pragma unroll
    for (u32 e = 0; e < 16; e++) a[e] = *(const lds_v*)(uintptr_t)(to ^ (lds_slot(reg_index<LOGN, PTO>(0, e)) * W));
}

// Tw: the twiddle type, Twiddle (two 64-bit words), Twiddle32 (two 32-bit words) or TwiddleF (one double): a table
// entry as it is stored.  For the two-word types Tw::raw is a vector type of the same layout, through which a
// wave-uniform entry is read with a scalar load.
template <typename Tw, bool UNIFORM>
__device__ __forceinline__ Tw load_twiddle(const Tw* tw, u32 k) {
    if constexpr (__is_same(Tw, TwiddleF)) {  // one double per entry
        if constexpr (UNIFORM) {
            k = __builtin_amdgcn_readfirstlane(k);
            return Tw{*(const __attribute__((address_space(4))) double*)(tw + k)};
        } else {
            return tw[k];
        }
    } else {
        typedef typename Tw::raw raw;
        static_assert(sizeof(raw) == sizeof(Tw), "a table entry is a pair of words");
        raw v;
        if constexpr (UNIFORM) {
            k = __builtin_amdgcn_readfirstlane(k);
            v = *(const __attribute__((address_space(4))) raw*)(tw + k);
        } else {
            v = *reinterpret_cast<const raw*>(tw + k);
        }
        return Tw{v.x, v.y};
    }
}

// Shape of pass P: its stages, and where the twiddle of (stage k, register e) sits among the
// pass's twiddles.  A thread's twiddles of stage k are 2^k consecutive table entries (per group of
// registers in the last pass), 15 entries per pass at most.
template <int LOGN, int P>
struct PassShape {
    using G = Geo<LOGN>;
    static constexpr bool LAST = (P == G::NPASS - 1);
    static constexpr int NST = LAST ? G::REM : 4;
    static constexpr int GROUPS = 16 >> NST;                 // independent register groups (last pass only > 1)
    static constexpr int PER_GROUP = (1 << NST) - 1;
    static constexpr int COUNT = GROUPS * PER_GROUP;
    // twiddles are the same for the whole wave when the thread-dependent part of the group index
    // is constant over 64 consecutive threads
    static constexpr bool UNIFORM = (P == 0) || (!LAST && (LOGN - 4 * (P + 1)) >= 6);
    __device__ static constexpr int slot(int k, u32 e) {
        return (int)(e >> NST) * PER_GROUP + ((1 << k) - 1) + (int)((e & ((1u << NST) - 1)) >> (NST - k));
    }
};

template <int LOGN, int P, typename Tw = Twiddle>
struct PassTwiddles {
    Tw t[PassShape<LOGN, P>::COUNT];
};

// All twiddles of pass P for this thread, requested in one go (the caller does this before the
// regrouping that precedes the pass, so the loads overlap the LDS traffic).
template <int LOGN, int P, typename Tw>
__device__ __forceinline__ void load_pass_twiddles(PassTwiddles<LOGN, P, Tw>& pt, const Tw* tw, u32 tid) {
    using S = PassShape<LOGN, P>;
    asm("; twiddles of pass %1" : "+v"(tid) : "n"(P));  // addresses are derived here, not ahead of earlier passes
#pragma unroll
    for (int k = 0; k < S::NST; k++) {
        const int s = 4 * P + k;
        const int bit = S::NST - 1 - k;
#pragma unroll
        for (u32 e = 0; e < 16; e++) {
            if (e & (1u << bit)) continue;
            if ((e & ((1u << S::NST) - 1)) & ((1u << bit) - 1)) continue;  // one load per distinct twiddle
            const u32 j = reg_index<LOGN, P>(tid, e);
            pt.t[S::slot(k, e)] = load_twiddle<Tw, S::UNIFORM>(tw, (1u << s) + (j >> (LOGN - s)));
        }
    }
}

// A copy of the thread index that the optimizer treats as a new value: addresses derived from it
// are computed where they are used instead of being carried (in registers the transform needs)
// from the top of the kernel.
__device__ __forceinline__ u32 fresh(u32 tid) {
    asm("; fresh thread index" : "+v"(tid));
    return tid;
}

}  // namespace
