// Building blocks shared by the ternary convolution kernels: activation/filter word groups,
// scalar-cache filter fetches, the four-instruction masked-Hamming step (Eq. 9) and the
// carry-flag bit assembly of the activation (Eq. 6).  Device code only.
#pragma once
#include "tern_internal.h"

namespace tern {
namespace {

template <int WC>
struct ActChunk {
    uint32_t m[WC];
    uint32_t s[WC];
};

// Filter words and cut points are read through the constant address space so that the
// wave-uniform loads go through the scalar cache (s_load) into SGPRs; neither is written by
// these kernels.
typedef const uint32_t __attribute__((address_space(4)))* scalar_ptr;

// word = (word << 1) | (thr < d): the comparison result goes through the carry flag into the
// low bit, two instructions per decision and no overflow cases.
__device__ __forceinline__ void shift_in_gt(uint32_t& word, int32_t d, int32_t thr)
{
    asm("v_cmp_lt_i32 vcc, %2, %1\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc"
        : "+v"(word) : "v"(d), "s"(thr) : "vcc");
}
// word = (word << 1) | (d < thr)
__device__ __forceinline__ void shift_in_lt(uint32_t& word, int32_t d, int32_t thr)
{
    asm("v_cmp_gt_i32 vcc, %2, %1\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc"
        : "+v"(word) : "v"(d), "s"(thr) : "vcc");
}

// Cut points of Eq. 6 for kCutBatch consecutive output channels.  The epilogue walks a pass's
// channels in such batches, two in flight (one being compared, one arriving), so that the cut
// points never occupy more than 32 SGPRs: fetching all 2 x CO_BLK of them at once left the
// register allocator short of SGPRs and it parked hundreds of them in VGPR lanes.
constexpr int kCutBatch = 8;
struct CutGroup {
    int32_t lo[kCutBatch];
    int32_t hi[kCutBatch];
};

// Channels c0 .. c0+7 of a pass; `valid` of them exist (channels past c_out get cut points that
// never fire, i.e. zero bits).  The full case is two contiguous 8-word scalar loads.
__device__ __forceinline__ void load_cuts(CutGroup& c, scalar_ptr thr_lo, scalar_ptr thr_hi, int c0,
                                          int valid, int c_out)
{
    if (valid >= kCutBatch) {
#pragma unroll
        for (int j = 0; j < kCutBatch; ++j) {
            c.lo[j] = (int32_t)thr_lo[c0 + j];
            c.hi[j] = (int32_t)thr_hi[c0 + j];
        }
    } else {
#pragma unroll
        for (int j = 0; j < kCutBatch; ++j) {
            const int cj = min(c0 + j, c_out - 1);
            const int32_t l = (int32_t)thr_lo[cj], h = (int32_t)thr_hi[cj];
            c.lo[j] = j < valid ? l : INT32_MIN;
            c.hi[j] = j < valid ? h : INT32_MAX;
        }
    }
}

// Same purpose as settle() for filter words: pins the wait for this batch's scalar loads here.
__device__ __forceinline__ void settle_cuts(const CutGroup& c)
{
    asm volatile("" ::"s"(c.lo[0]), "s"(c.lo[1]), "s"(c.lo[2]), "s"(c.lo[3]), "s"(c.lo[4]), "s"(c.lo[5]),
                 "s"(c.lo[6]), "s"(c.lo[7]), "s"(c.hi[0]), "s"(c.hi[1]), "s"(c.hi[2]), "s"(c.hi[3]),
                 "s"(c.hi[4]), "s"(c.hi[5]), "s"(c.hi[6]), "s"(c.hi[7]));
}

// Eq. 6 in integer form for one pass of CO_BLK channels: two decisions per (voxel, channel),
// highest channel first so that channel j ends up in bit j of pp (acc > hi) and pn (acc < lo).
template <int V, int CO_BLK>
__device__ __forceinline__ void ternarise_pass(const int32_t (&d)[V][CO_BLK], scalar_ptr thr_lo,
                                               scalar_ptr thr_hi, int cb, int co_left, int c_out,
                                               uint32_t (&pp)[V], uint32_t (&pn)[V])
{
    constexpr int NB = CO_BLK / kCutBatch;
    static_assert(CO_BLK % kCutBatch == 0, "whole batches");
    CutGroup cg[2];
    load_cuts(cg[(NB - 1) & 1], thr_lo, thr_hi, cb + (NB - 1) * kCutBatch, co_left - (NB - 1) * kCutBatch, c_out);
#pragma unroll
    for (int v = 0; v < V; ++v) pp[v] = pn[v] = 0u;
#pragma unroll
    for (int b = NB - 1; b >= 0; --b) {
        settle_cuts(cg[b & 1]);
        __builtin_amdgcn_sched_barrier(0);
        if (b > 0)
            load_cuts(cg[(b - 1) & 1], thr_lo, thr_hi, cb + (b - 1) * kCutBatch, co_left - (b - 1) * kCutBatch, c_out);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = kCutBatch - 1; j >= 0; --j) {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                shift_in_gt(pp[v], d[v][b * kCutBatch + j], cg[b & 1].hi[j]);   // +1 if acc > hi
                shift_in_lt(pn[v], d[v][b * kCutBatch + j], cg[b & 1].lo[j]);   // -1 if acc < lo
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// KG = output channels whose filter words are fetched together.  Two groups are in flight (one
// being used, one arriving).  With 32 channels per pass KG = 4 keeps the filter words within 32
// SGPRs, which leaves room for the loop's own scalars (8 per group made the compiler spill them);
// with 16 channels per pass KG = 8 fits and halves the number of waits, which matters when a
// SIMD holds a single wave and nothing else hides the scalar-cache latency; 8 channels per pass
// are two groups of 4.
template <int CO_BLK>
struct GroupOf {
    static constexpr int value = (CO_BLK >= 32 || CO_BLK <= 8) ? 4 : 8;
};

template <int WC, int KG>
struct WGroup {
    uint32_t m[KG][WC];
    uint32_t s[KG][WC];
};

// Fetch the filter words of KG consecutive channels of one step.  In the filter bank the
// channels of a step are contiguous (2*WC words each), so this is one contiguous block that
// the compiler turns into wide scalar loads with immediate offsets.
template <int WC, int KG>
__device__ __forceinline__ void load_wgroup(WGroup<WC, KG>& g, scalar_ptr wp)
{
#pragma unroll
    for (int j = 0; j < KG; ++j)
#pragma unroll
        for (int q = 0; q < WC; ++q) {
            g.m[j][q] = wp[j * 2 * WC + q];
            g.s[j][q] = wp[j * 2 * WC + WC + q];
        }
}

// Scalar loads return out of order, so the only safe wait is "all of them".  Naming the group's
// registers here makes the compiler place that wait at this point, i.e. before the loads of the
// following group are issued, so that those overlap the arithmetic on this group instead of
// being waited for together with it.
template <int WC, int KG>
__device__ __forceinline__ void settle(const WGroup<WC, KG>& g)
{
    static_assert(KG % 4 == 0, "groups of 4 channels per asm statement");
#pragma unroll
    for (int j = 0; j < KG; j += 4) {
        if constexpr (WC == 2) {
            asm volatile("" ::"s"(g.m[j][0]), "s"(g.m[j][1]), "s"(g.s[j][0]), "s"(g.s[j][1]),
                         "s"(g.m[j + 1][0]), "s"(g.m[j + 1][1]), "s"(g.s[j + 1][0]), "s"(g.s[j + 1][1]),
                         "s"(g.m[j + 2][0]), "s"(g.m[j + 2][1]), "s"(g.s[j + 2][0]), "s"(g.s[j + 2][1]),
                         "s"(g.m[j + 3][0]), "s"(g.m[j + 3][1]), "s"(g.s[j + 3][0]), "s"(g.s[j + 3][1]));
        } else {
            asm volatile("" ::"s"(g.m[j][0]), "s"(g.s[j][0]), "s"(g.m[j + 1][0]), "s"(g.s[j + 1][0]),
                         "s"(g.m[j + 2][0]), "s"(g.s[j + 2][0]), "s"(g.m[j + 3][0]), "s"(g.s[j + 3][0]));
        }
    }
}

// Eq. 9 for one (word pair, voxel) combination: acc_m += popcount(ma & mw), acc_n +=
// popcount(ma & mw & (sa ^ sw)) -- and, popcount-accumulate, three-input bit operation (truth
// table 0x48 = m & (sa ^ sw), index = sa<<2 | m<<1 | sw), popcount-accumulate; mw and sw are
// wave-uniform.
//
// Sixteen or thirty-two of these instructions make one asm statement (mac_quad below) because
// their order and spacing decide the issue rate on gfx950.  Measured with register-only loops of this mix (cycles per vector
// instruction at 2.4 GHz, four waves per SIMD): any order with no scalar instruction in between
// 3.95-4.0, also with another vector instruction between producer and popcount; one scalar
// instruction (s_nop 0 or any other) between the bit operation and its popcount 3.4; one between
// each producer and its popcount, as below, 3.1, a fifth less time per word pair; s_nop 1, v_nop or
// further nops between independent instructions lose the gain again.  The s_nop behind the bit
// operation is also the wait state the compiler itself puts between v_bitop3 and a reader of its
// result.  The compiler assumes that an asm statement's outputs may need such a wait state and
// puts an s_nop of its own in front of the next statement that touches one of them, which spoils
// the spacing: hence four or eight word pairs per statement, and two scratch registers taken in turn.
#define TERN_MAC_PAIR(P, C, ADD_M, ADD_N)                                           \
    "v_and_b32 %[t], %[mw" P "], %[ma" P "]\n\t"                                   \
    "s_nop 0\n\t"                                                                  \
    "v_bcnt_u32_b32 %[am" C "], %[t], " ADD_M "\n\t"                               \
    "v_bitop3_b32 %[t], %[sa" P "], %[t], %[sw" P "] bitop3:0x48\n\t"              \
    "s_nop 0\n\t"                                                                  \
    "v_bcnt_u32_b32 %[an" C "], %[t], " ADD_N "\n\t"
#define TERN_MAC_IN(P, MA, SA, MW, SW) [ma##P] "v"(MA), [sa##P] "v"(SA), [mw##P] "s"(MW), [sw##P] "s"(SW)

// All WC words of channels jg .. jg+4/V-1 of group g for all V voxels of a lane: combination c =
// (channel c / V, voxel c % V), 4 WC word pairs per statement.  SET: the accumulators hold
// nothing yet; the first word sets them instead of adding to them (a pass's first step does that,
// so they are never cleared).
template <int WC, int V, int CO_BLK, int KG, bool SET>
__device__ __forceinline__ void mac_quad(const ActChunk<WC> (&A)[V], const WGroup<WC, KG>& g, int jg, int j0,
                                         int32_t (&acc_m)[V][CO_BLK], int32_t (&acc_n)[V][CO_BLK],
                                         uint32_t& t)
{
    static_assert(V == 1 || V == 2 || V == 4, "four (channel, voxel) combinations per statement");
    static_assert(WC == 1 || WC == 2, "one or two words per chunk");
#define TERN_C(P) (jg + (P) / V)
#define TERN_X(P) ((P) % V)
#define TERN_ACC_SET(C) [am##C] "=&v"(acc_m[TERN_X(C)][j0 + TERN_C(C)]), [an##C] "=&v"(acc_n[TERN_X(C)][j0 + TERN_C(C)])
#define TERN_ACC_ADD(C) [am##C] "+v"(acc_m[TERN_X(C)][j0 + TERN_C(C)]), [an##C] "+v"(acc_n[TERN_X(C)][j0 + TERN_C(C)])
#define TERN_INS(P, C, Q) TERN_MAC_IN(P, A[TERN_X(C)].m[Q], A[TERN_X(C)].s[Q], g.m[TERN_C(C)][Q], g.s[TERN_C(C)][Q])
#define TERN_WORD0_SET TERN_MAC_PAIR("0", "0", "0", "0") TERN_MAC_PAIR("1", "1", "0", "0") \
                       TERN_MAC_PAIR("2", "2", "0", "0") TERN_MAC_PAIR("3", "3", "0", "0")
#define TERN_WORD0_ADD TERN_MAC_PAIR("0", "0", "%[am0]", "%[an0]") TERN_MAC_PAIR("1", "1", "%[am1]", "%[an1]") \
                       TERN_MAC_PAIR("2", "2", "%[am2]", "%[an2]") TERN_MAC_PAIR("3", "3", "%[am3]", "%[an3]")
#define TERN_WORD1_ADD TERN_MAC_PAIR("4", "0", "%[am0]", "%[an0]") TERN_MAC_PAIR("5", "1", "%[am1]", "%[an1]") \
                       TERN_MAC_PAIR("6", "2", "%[am2]", "%[an2]") TERN_MAC_PAIR("7", "3", "%[am3]", "%[an3]")
    if constexpr (WC == 2) {
        if constexpr (SET) {
            asm volatile(TERN_WORD0_SET TERN_WORD1_ADD
                         : TERN_ACC_SET(0), TERN_ACC_SET(1), TERN_ACC_SET(2), TERN_ACC_SET(3), [t] "+v"(t)
                         : TERN_INS(0, 0, 0), TERN_INS(1, 1, 0), TERN_INS(2, 2, 0), TERN_INS(3, 3, 0),
                           TERN_INS(4, 0, 1), TERN_INS(5, 1, 1), TERN_INS(6, 2, 1), TERN_INS(7, 3, 1));
        } else {
            asm volatile(TERN_WORD0_ADD TERN_WORD1_ADD
                         : TERN_ACC_ADD(0), TERN_ACC_ADD(1), TERN_ACC_ADD(2), TERN_ACC_ADD(3), [t] "+v"(t)
                         : TERN_INS(0, 0, 0), TERN_INS(1, 1, 0), TERN_INS(2, 2, 0), TERN_INS(3, 3, 0),
                           TERN_INS(4, 0, 1), TERN_INS(5, 1, 1), TERN_INS(6, 2, 1), TERN_INS(7, 3, 1));
        }
    } else {
        if constexpr (SET) {
            asm volatile(TERN_WORD0_SET
                         : TERN_ACC_SET(0), TERN_ACC_SET(1), TERN_ACC_SET(2), TERN_ACC_SET(3), [t] "+v"(t)
                         : TERN_INS(0, 0, 0), TERN_INS(1, 1, 0), TERN_INS(2, 2, 0), TERN_INS(3, 3, 0));
        } else {
            asm volatile(TERN_WORD0_ADD
                         : TERN_ACC_ADD(0), TERN_ACC_ADD(1), TERN_ACC_ADD(2), TERN_ACC_ADD(3), [t] "+v"(t)
                         : TERN_INS(0, 0, 0), TERN_INS(1, 1, 0), TERN_INS(2, 2, 0), TERN_INS(3, 3, 0));
        }
    }
#undef TERN_C
#undef TERN_X
#undef TERN_ACC_SET
#undef TERN_ACC_ADD
#undef TERN_INS
#undef TERN_WORD0_SET
#undef TERN_WORD0_ADD
#undef TERN_WORD1_ADD
}

// Two-digit inputs (sums of up to four ternary codes written in balanced ternary, low digit in
// the even word of a chunk and high digit, worth three, in the odd word): the same statement with
// the odd word's popcounts going to accumulators of their own, acc2_m / acc2_n.
template <int V, int CO_BLK, int KG, bool SET>
__device__ __forceinline__ void mac_quad_digits(const ActChunk<2> (&A)[V], const WGroup<2, KG>& g, int jg, int j0,
                                                int32_t (&acc_m)[V][CO_BLK], int32_t (&acc_n)[V][CO_BLK],
                                                int32_t (&acc2_m)[V][CO_BLK], int32_t (&acc2_n)[V][CO_BLK],
                                                uint32_t& t)
{
    static_assert(V == 1 || V == 2 || V == 4, "four (channel, voxel) combinations per statement");
#define TERN_C(P) (jg + (P) / V)
#define TERN_X(P) ((P) % V)
#define TERN_ACC(C, K, A1, A2) [am##C] K(A1##_m[TERN_X(C)][j0 + TERN_C(C)]), [an##C] K(A1##_n[TERN_X(C)][j0 + TERN_C(C)]), \
                               [bm##C] K(A2##_m[TERN_X(C)][j0 + TERN_C(C)]), [bn##C] K(A2##_n[TERN_X(C)][j0 + TERN_C(C)])
#define TERN_INS(P, C, Q) TERN_MAC_IN(P, A[TERN_X(C)].m[Q], A[TERN_X(C)].s[Q], g.m[TERN_C(C)][Q], g.s[TERN_C(C)][Q])
// the pair macro names its accumulators am<C> / an<C>; the odd word's pairs go through an alias
#define TERN_MAC_PAIR_B(P, C, ADD_M, ADD_N)                                          \
    "v_and_b32 %[t], %[mw" P "], %[ma" P "]\n\t"                                   \
    "s_nop 0\n\t"                                                                  \
    "v_bcnt_u32_b32 %[bm" C "], %[t], " ADD_M "\n\t"                               \
    "v_bitop3_b32 %[t], %[sa" P "], %[t], %[sw" P "] bitop3:0x48\n\t"              \
    "s_nop 0\n\t"                                                                  \
    "v_bcnt_u32_b32 %[bn" C "], %[t], " ADD_N "\n\t"
    if constexpr (SET) {
        asm volatile(TERN_MAC_PAIR("0", "0", "0", "0") TERN_MAC_PAIR("1", "1", "0", "0")
                     TERN_MAC_PAIR("2", "2", "0", "0") TERN_MAC_PAIR("3", "3", "0", "0")
                     TERN_MAC_PAIR_B("4", "0", "0", "0") TERN_MAC_PAIR_B("5", "1", "0", "0")
                     TERN_MAC_PAIR_B("6", "2", "0", "0") TERN_MAC_PAIR_B("7", "3", "0", "0")
                     : TERN_ACC(0, "=&v", acc, acc2), TERN_ACC(1, "=&v", acc, acc2), TERN_ACC(2, "=&v", acc, acc2),
                       TERN_ACC(3, "=&v", acc, acc2), [t] "+v"(t)
                     : TERN_INS(0, 0, 0), TERN_INS(1, 1, 0), TERN_INS(2, 2, 0), TERN_INS(3, 3, 0),
                       TERN_INS(4, 0, 1), TERN_INS(5, 1, 1), TERN_INS(6, 2, 1), TERN_INS(7, 3, 1));
    } else {
        asm volatile(TERN_MAC_PAIR("0", "0", "%[am0]", "%[an0]") TERN_MAC_PAIR("1", "1", "%[am1]", "%[an1]")
                     TERN_MAC_PAIR("2", "2", "%[am2]", "%[an2]") TERN_MAC_PAIR("3", "3", "%[am3]", "%[an3]")
                     TERN_MAC_PAIR_B("4", "0", "%[bm0]", "%[bn0]") TERN_MAC_PAIR_B("5", "1", "%[bm1]", "%[bn1]")
                     TERN_MAC_PAIR_B("6", "2", "%[bm2]", "%[bn2]") TERN_MAC_PAIR_B("7", "3", "%[bm3]", "%[bn3]")
                     : TERN_ACC(0, "+v", acc, acc2), TERN_ACC(1, "+v", acc, acc2), TERN_ACC(2, "+v", acc, acc2),
                       TERN_ACC(3, "+v", acc, acc2), [t] "+v"(t)
                     : TERN_INS(0, 0, 0), TERN_INS(1, 1, 0), TERN_INS(2, 2, 0), TERN_INS(3, 3, 0),
                       TERN_INS(4, 0, 1), TERN_INS(5, 1, 1), TERN_INS(6, 2, 1), TERN_INS(7, 3, 1));
    }
#undef TERN_C
#undef TERN_X
#undef TERN_ACC
#undef TERN_INS
#undef TERN_MAC_PAIR_B
}

template <int V, int CO_BLK, int KG, bool INIT = false>
__device__ __forceinline__ void mac_group_digits(const ActChunk<2> (&A)[V], const WGroup<2, KG>& g, int j0,
                                                 int32_t (&acc_m)[V][CO_BLK], int32_t (&acc_n)[V][CO_BLK],
                                                 int32_t (&acc2_m)[V][CO_BLK], int32_t (&acc2_n)[V][CO_BLK])
{
    constexpr int NCB = V == 4 ? 1 : 4 / V;
    static_assert(KG % NCB == 0, "whole statements");
    uint32_t t[2];
    asm volatile("" : "=v"(t[0]), "=v"(t[1]));
#pragma unroll
    for (int jg = 0, k = 0; jg < KG; jg += NCB, ++k)
        mac_quad_digits<V, CO_BLK, KG, INIT>(A, g, jg, j0, acc_m, acc_n, acc2_m, acc2_n, t[k & 1]);
}

// Four VALU instructions per (word pair, voxel) (Eq. 9 as popcount(M) - 2 popcount(M & X), the
// subtraction deferred).  INIT: the accumulators of these channels hold nothing yet.
template <int WC, int V, int CO_BLK, int KG, bool INIT = false>
__device__ __forceinline__ void mac_group(const ActChunk<WC> (&A)[V], const WGroup<WC, KG>& g, int j0,
                                          int32_t (&acc_m)[V][CO_BLK], int32_t (&acc_n)[V][CO_BLK])
{
    // (The statements are volatile so that they stay in this order; the empty statement hands out
    // two distinct scratch registers without an instruction.  The compiler's own s_nop in front of
    // a group's first statement, behind the scalar load of the next group's filter words, is
    // welcome: without it the loop measured 2 % slower.)
    constexpr int NCB = V == 4 ? 1 : 4 / V;   // channels per statement
    static_assert(KG % NCB == 0, "whole statements");
    uint32_t t[2];
    asm volatile("" : "=v"(t[0]), "=v"(t[1]));
#pragma unroll
    for (int jg = 0, k = 0; jg < KG; jg += NCB, ++k)
        mac_quad<WC, V, CO_BLK, KG, INIT>(A, g, jg, j0, acc_m, acc_n, t[k & 1]);
}


// ---- binary weights (Eq. 8) --------------------------------------------------------------------
// With weights in {-1, +1} the filter has no mask plane: a group is KG channels x WC sign words.
template <int WC, int KG>
struct WGroupB {
    uint32_t s[KG][WC];
};

// Binary filter bank: [step][co_pad][WC] sign words, the channels of a step contiguous.
template <int WC, int KG>
__device__ __forceinline__ void load_wgroup(WGroupB<WC, KG>& g, scalar_ptr wp)
{
#pragma unroll
    for (int j = 0; j < KG; ++j)
#pragma unroll
        for (int q = 0; q < WC; ++q) g.s[j][q] = wp[j * WC + q];
}

template <int WC, int KG>
__device__ __forceinline__ void settle(const WGroupB<WC, KG>& g)
{
    static_assert(KG % 8 == 0, "groups of 8 channels per asm statement");
#pragma unroll
    for (int j = 0; j < KG; j += 8) {
        if constexpr (WC == 2) {
            asm volatile("" ::"s"(g.s[j][0]), "s"(g.s[j][1]), "s"(g.s[j + 1][0]), "s"(g.s[j + 1][1]),
                         "s"(g.s[j + 2][0]), "s"(g.s[j + 2][1]), "s"(g.s[j + 3][0]), "s"(g.s[j + 3][1]),
                         "s"(g.s[j + 4][0]), "s"(g.s[j + 4][1]), "s"(g.s[j + 5][0]), "s"(g.s[j + 5][1]),
                         "s"(g.s[j + 6][0]), "s"(g.s[j + 6][1]), "s"(g.s[j + 7][0]), "s"(g.s[j + 7][1]));
        } else {
            asm volatile("" ::"s"(g.s[j][0]), "s"(g.s[j + 1][0]), "s"(g.s[j + 2][0]), "s"(g.s[j + 3][0]),
                         "s"(g.s[j + 4][0]), "s"(g.s[j + 5][0]), "s"(g.s[j + 6][0]), "s"(g.s[j + 7][0]));
        }
    }
}

// Eq. 8 with the activation's mask kept: for one (word pair, voxel) acc_n += popcount(ma & (sa ^
// sw)) -- one three-input bit operation (the same truth table as in the ternary step, with the
// activation mask in the place of M) and one popcount-accumulate, a scalar no-op between them.
// The other half of the sum, popcount(ma), does not depend on the filter and is counted once
// per voxel and step by the caller.  A zero activation (zero padding included) drops out
// through its mask exactly as in Eq. 9; with no zeros the result is c - 2 popcount(I xor W).
#define TERN_BIN_PAIR(P, C, ADD_N)                                                  \
    "v_bitop3_b32 %[t], %[sa" P "], %[ma" P "], %[sw" P "] bitop3:0x48\n\t"        \
    "s_nop 0\n\t"                                                                  \
    "v_bcnt_u32_b32 %[an" C "], %[t], " ADD_N "\n\t"
#define TERN_BIN_IN(P, MA, SA, SW) [ma##P] "v"(MA), [sa##P] "v"(SA), [sw##P] "s"(SW)

template <int WC, int V, int CO_BLK, int KG, bool SET>
__device__ __forceinline__ void mac_quad_bin(const ActChunk<WC> (&A)[V], const WGroupB<WC, KG>& g, int jg, int j0,
                                             int32_t (&acc_n)[V][CO_BLK], uint32_t& t)
{
    static_assert(V == 1 || V == 2 || V == 4, "four (channel, voxel) combinations per statement");
    static_assert(WC == 1 || WC == 2, "one or two words per chunk");
#define TERN_C(P) (jg + (P) / V)
#define TERN_X(P) ((P) % V)
#define TERN_ACC_SET(C) [an##C] "=&v"(acc_n[TERN_X(C)][j0 + TERN_C(C)])
#define TERN_ACC_ADD(C) [an##C] "+v"(acc_n[TERN_X(C)][j0 + TERN_C(C)])
#define TERN_INS(P, C, Q) TERN_BIN_IN(P, A[TERN_X(C)].m[Q], A[TERN_X(C)].s[Q], g.s[TERN_C(C)][Q])
#define TERN_WORD0_SET TERN_BIN_PAIR("0", "0", "0") TERN_BIN_PAIR("1", "1", "0") TERN_BIN_PAIR("2", "2", "0") \
                       TERN_BIN_PAIR("3", "3", "0")
#define TERN_WORD0_ADD TERN_BIN_PAIR("0", "0", "%[an0]") TERN_BIN_PAIR("1", "1", "%[an1]") \
                       TERN_BIN_PAIR("2", "2", "%[an2]") TERN_BIN_PAIR("3", "3", "%[an3]")
#define TERN_WORD1_ADD TERN_BIN_PAIR("4", "0", "%[an0]") TERN_BIN_PAIR("5", "1", "%[an1]") \
                       TERN_BIN_PAIR("6", "2", "%[an2]") TERN_BIN_PAIR("7", "3", "%[an3]")
    if constexpr (WC == 2) {
        if constexpr (SET) {
            asm volatile(TERN_WORD0_SET TERN_WORD1_ADD
                         : TERN_ACC_SET(0), TERN_ACC_SET(1), TERN_ACC_SET(2), TERN_ACC_SET(3), [t] "+v"(t)
                         : TERN_INS(0, 0, 0), TERN_INS(1, 1, 0), TERN_INS(2, 2, 0), TERN_INS(3, 3, 0),
                           TERN_INS(4, 0, 1), TERN_INS(5, 1, 1), TERN_INS(6, 2, 1), TERN_INS(7, 3, 1));
        } else {
            asm volatile(TERN_WORD0_ADD TERN_WORD1_ADD
                         : TERN_ACC_ADD(0), TERN_ACC_ADD(1), TERN_ACC_ADD(2), TERN_ACC_ADD(3), [t] "+v"(t)
                         : TERN_INS(0, 0, 0), TERN_INS(1, 1, 0), TERN_INS(2, 2, 0), TERN_INS(3, 3, 0),
                           TERN_INS(4, 0, 1), TERN_INS(5, 1, 1), TERN_INS(6, 2, 1), TERN_INS(7, 3, 1));
        }
    } else {
        if constexpr (SET) {
            asm volatile(TERN_WORD0_SET
                         : TERN_ACC_SET(0), TERN_ACC_SET(1), TERN_ACC_SET(2), TERN_ACC_SET(3), [t] "+v"(t)
                         : TERN_INS(0, 0, 0), TERN_INS(1, 1, 0), TERN_INS(2, 2, 0), TERN_INS(3, 3, 0));
        } else {
            asm volatile(TERN_WORD0_ADD
                         : TERN_ACC_ADD(0), TERN_ACC_ADD(1), TERN_ACC_ADD(2), TERN_ACC_ADD(3), [t] "+v"(t)
                         : TERN_INS(0, 0, 0), TERN_INS(1, 1, 0), TERN_INS(2, 2, 0), TERN_INS(3, 3, 0));
        }
    }
#undef TERN_C
#undef TERN_X
#undef TERN_ACC_SET
#undef TERN_ACC_ADD
#undef TERN_INS
#undef TERN_WORD0_SET
#undef TERN_WORD0_ADD
#undef TERN_WORD1_ADD
}

// Two VALU instructions per (word pair, voxel).  INIT: the accumulators hold nothing yet.
template <int WC, int V, int CO_BLK, int KG, bool INIT = false>
__device__ __forceinline__ void mac_group_bin(const ActChunk<WC> (&A)[V], const WGroupB<WC, KG>& g, int j0,
                                              int32_t (&acc_n)[V][CO_BLK])
{
    constexpr int NCB = V == 4 ? 1 : 4 / V;   // channels per statement
    static_assert(KG % NCB == 0, "whole statements");
    uint32_t t[2];
    asm volatile("" : "=v"(t[0]), "=v"(t[1]));
#pragma unroll
    for (int jg = 0, k = 0; jg < KG; jg += NCB, ++k)
        mac_quad_bin<WC, V, CO_BLK, KG, INIT>(A, g, jg, j0, acc_n, t[k & 1]);
}

}  // namespace
}  // namespace tern
