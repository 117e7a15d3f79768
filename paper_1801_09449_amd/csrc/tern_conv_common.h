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

// acc += popcount(x) as the single instruction the hardware has for it.
__device__ __forceinline__ void popc_acc(int32_t& acc, uint32_t x)
{
    asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(x));
}

// m & (sa ^ sw) as one three-input bit operation (truth-table index = sa<<2 | m<<1 | sw).
// Spelled out because the compiler otherwise sometimes forms (sa ^ sw) on its own and spends a
// fifth instruction per word pair.
__device__ __forceinline__ uint32_t and_xor(uint32_t m, uint32_t sa, uint32_t sw)
{
    uint32_t r;
    asm("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x48" : "=v"(r) : "v"(sa), "v"(m), "s"(sw));
    return r;
}

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

// KG = output channels whose filter words are fetched together.  Two groups are in flight (one
// being used, one arriving).  With 32 channels per pass KG = 4 keeps the filter words within 32
// SGPRs, which leaves room for the loop's own scalars (8 per group made the compiler spill them);
// with 16 channels per pass KG = 8 fits and halves the number of waits, which matters when a
// SIMD holds a single wave and nothing else hides the scalar-cache latency.
template <int CO_BLK>
struct GroupOf {
    static constexpr int value = CO_BLK >= 32 ? 4 : 8;
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

// Four VALU instructions per (word pair, voxel): and, popcount-accumulate, and-xor,
// popcount-accumulate (Eq. 9 as popcount(M) - 2 popcount(M & X), the subtraction deferred).
template <int WC, int V, int CO_BLK, int KG>
__device__ __forceinline__ void mac_group(const ActChunk<WC> (&A)[V], const WGroup<WC, KG>& g, int j0,
                                          int32_t (&acc_m)[V][CO_BLK], int32_t (&acc_n)[V][CO_BLK])
{
#pragma unroll
    for (int j = 0; j < KG; ++j)
#pragma unroll
        for (int q = 0; q < WC; ++q)
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const uint32_t M = A[v].m[q] & g.m[j][q];
                const uint32_t N = and_xor(M, A[v].s[q], g.s[j][q]);
                popc_acc(acc_m[v][j0 + j], M);
                popc_acc(acc_n[v][j0 + j], N);
            }
}

}  // namespace
}  // namespace tern
