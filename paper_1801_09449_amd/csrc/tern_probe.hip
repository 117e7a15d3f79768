// Diagnostic: sustained issue rate of the convolution's vector instructions with no memory
// traffic at all.  The benchmark uses variant 0 as the measured ceiling of the kernels' instruction
// mix next to the nominal 256 CU x 64 lanes x 2.4 GHz figure; the other variants take the mix
// apart (one opcode at a time, with and without a scalar instruction behind each vector
// instruction) to show which part of it issues faster than one wave instruction per four cycles.
//
//   0  the kernels' own statement: and, s_nop, popcount-accumulate, three-input bit operation,
//      s_nop, popcount-accumulate (a scalar no-op between each producer and its popcount)
//   1  the same four vector instructions per word pair in an order that needs no wait state and
//      with no scalar instruction in between (what a compiler's scheduler makes of them)
//   2 / 3    v_and_b32 with a wave-uniform operand, alone / each followed by s_nop 0
//   4 / 5    v_bcnt_u32_b32 accumulating into eight registers in turn, alone / with s_nop 0
//   6 / 7    v_bitop3_b32, alone / with s_nop 0
//   8 / 9    v_xor_b32 with a wave-uniform operand, alone / with s_nop 0
//   10 / 11  the two-instruction word pair of the binary convolution (Eq. 8), 32 pairs per round:
//            the kernels' own statement (three-input bit operation, s_nop, popcount-accumulate)
//            / the same two instructions with no scalar instruction between them
//   12 / 13  v_add_u32 with a wave-uniform operand (a plain integer add, for reference), alone /
//            with s_nop 0
//   14       v_xor_b32 on vector registers only
//   15       v_bitop3_b32 on vector registers only
//   16       v_and_b32 with a wave-uniform operand alternating with an independent v_add_u32 on
//            vector registers only
// Every variant issues 64 vector instructions plus one add per round and lane.
//
// What the variants show on MI355X (cycles per wave instruction and SIMD at 2.4 GHz, four waves
// per SIMD): an integer instruction whose operands are all vector registers retires in about two
// cycles (14, 15: 2.1-2.3; 32 lanes per clock and SIMD, the rate behind the published fp32
// vector peak), one that reads a wave-uniform (scalar register) operand in four (2, 6, 8, 12:
// 4.0), and so does v_bcnt_u32_b32 whatever its operands (4: 4.07); a vector-only instruction
// slips in beside a scalar-operand one (16: 2.15 on average).  A ternary word pair is therefore
// 2 + 4 + 2 + 4 = 12 cycles at best, 3.0 per instruction; the kernels' sequence reaches 3.16.
#include "tern_conv_common.h"
#include "tern_internal.h"

namespace tern {
namespace {

struct ProbeConsts { uint32_t k[32]; };

__global__ __launch_bounds__(512) void probe_kernel(ProbeConsts c, int iters, int32_t* sink)
{
    ActChunk<1> A[1];
    A[0].m[0] = threadIdx.x * 2654435761u + blockIdx.x;
    A[0].s[0] = A[0].m[0] ^ 0x9e3779b9u;
    WGroup<1, 8> g[2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            g[h].m[j][0] = c.k[8 * h + j];
            g[h].s[j][0] = c.k[16 + 8 * h + j];
        }
    int32_t acc_m[1][16], acc_n[1][16];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc_m[0][j] = acc_n[0][j] = 0;
    for (int it = 0; it < iters; ++it) {
        mac_group<1, 1, 16, 8>(A, g[0], 0, acc_m, acc_n);   // the kernels' own step, 16 word pairs
        mac_group<1, 1, 16, 8>(A, g[1], 8, acc_m, acc_n);
        A[0].m[0] += 0x01010101u;   // keeps the loop body from being hoisted; 1 extra op per 64
    }
    int32_t r = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) r += acc_m[0][j] - 2 * acc_n[0][j];
    if (r == 0x7fffffff) sink[0] = r;   // practically never true; keeps the work alive
}

// The same work per round as probe_kernel, unspaced: and, bit operation, popcount, popcount.
__global__ __launch_bounds__(512) void probe_unspaced_kernel(ProbeConsts c, int iters, int32_t* sink)
{
    uint32_t a = threadIdx.x * 2654435761u + blockIdx.x, b = a ^ 0x9e3779b9u;
    int32_t acc_m[16], acc_n[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc_m[j] = acc_n[j] = 0;
    for (int it = 0; it < iters; ++it) {
        // four word pairs per statement: the compiler puts an s_nop of its own between asm
        // statements, which would space single pairs after all
#define TERN_UNSPACED(P)                                                      \
    "v_and_b32 %[t], %[mw" P "], %[ma]\n\t"                                   \
    "v_bitop3_b32 %[u], %[sa], %[t], %[sw" P "] bitop3:0x48\n\t"              \
    "v_bcnt_u32_b32 %[am" P "], %[t], %[am" P "]\n\t"                         \
    "v_bcnt_u32_b32 %[an" P "], %[u], %[an" P "]\n\t"
#pragma unroll
        for (int j = 0; j < 16; j += 4) {
            uint32_t t, u;
            asm volatile(TERN_UNSPACED("0") TERN_UNSPACED("1") TERN_UNSPACED("2") TERN_UNSPACED("3")
                         : [am0] "+v"(acc_m[j]), [an0] "+v"(acc_n[j]), [am1] "+v"(acc_m[j + 1]),
                           [an1] "+v"(acc_n[j + 1]), [am2] "+v"(acc_m[j + 2]), [an2] "+v"(acc_n[j + 2]),
                           [am3] "+v"(acc_m[j + 3]), [an3] "+v"(acc_n[j + 3]), [t] "=&v"(t), [u] "=&v"(u)
                         : [ma] "v"(a), [sa] "v"(b), [mw0] "s"(c.k[j]), [sw0] "s"(c.k[16 + j]),
                           [mw1] "s"(c.k[j + 1]), [sw1] "s"(c.k[17 + j]), [mw2] "s"(c.k[j + 2]),
                           [sw2] "s"(c.k[18 + j]), [mw3] "s"(c.k[j + 3]), [sw3] "s"(c.k[19 + j]));
        }
#undef TERN_UNSPACED
        a += 0x01010101u;
    }
    int32_t r = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) r += acc_m[j] - 2 * acc_n[j];
    if (r == 0x7fffffff) sink[0] = r;
}

// The binary convolution's own step: 32 word pairs = 64 vector instructions per round.
__global__ __launch_bounds__(512) void probe_bin_kernel(ProbeConsts c, int iters, int32_t* sink)
{
    ActChunk<1> A[1];
    A[0].m[0] = threadIdx.x * 2654435761u + blockIdx.x;
    A[0].s[0] = A[0].m[0] ^ 0x9e3779b9u;
    WGroupB<1, 8> g[4];
#pragma unroll
    for (int h = 0; h < 4; ++h)
#pragma unroll
        for (int j = 0; j < 8; ++j) g[h].s[j][0] = c.k[8 * h + j];
    int32_t acc_n[1][32];
#pragma unroll
    for (int j = 0; j < 32; ++j) acc_n[0][j] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int h = 0; h < 4; ++h) mac_group_bin<1, 1, 32, 8>(A, g[h], 8 * h, acc_n);
        A[0].m[0] += 0x01010101u;
    }
    int32_t r = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) r += acc_n[0][j];
    if (r == 0x7fffffff) sink[0] = r;
}

// One opcode (or the binary word pair) at a time: eight instructions per statement on eight
// registers r0..r7 taken in turn, eight statements per round.  OP: 0 and, 1 popcount-accumulate,
// 2 three-input bit operation, 3 xor, 4 binary pair (bit operation into a scratch register, popcount
// of it accumulated; four pairs per statement), 5 add, each with one wave-uniform operand where the
// opcode takes one; 6 xor and 7 bit operation on vector registers only; 8 scalar-operand and beside
// an independent vector-only add.  NOP: s_nop 0 behind every vector instruction
// (binary pair: between the xor and its popcount).
#define TERN_P_AND(R, K)   "v_and_b32 %[r" R "], %[k" K "], %[a]\n\t"
#define TERN_P_BCNT(R, K)  "v_bcnt_u32_b32 %[r" R "], %[a], %[r" R "]\n\t"
#define TERN_P_BITOP(R, K) "v_bitop3_b32 %[r" R "], %[a], %[b], %[k" K "] bitop3:0x48\n\t"
#define TERN_P_XOR(R, K)   "v_xor_b32 %[r" R "], %[k" K "], %[a]\n\t"
#define TERN_P_ADD(R, K)   "v_add_u32 %[r" R "], %[k" K "], %[r" R "]\n\t"
#define TERN_P_XORV(R, K)  "v_xor_b32 %[r" R "], %[a], %[r" R "]\n\t"
#define TERN_P_BITOPV(R, K) "v_bitop3_b32 %[r" R "], %[a], %[b], %[r" R "] bitop3:0x48\n\t"
// scalar-operand and into r4..r7 beside an independent vector-only add on r0..r3
#define TERN_P_MIXED(R, T, K) "v_and_b32 %[r" T "], %[k" K "], %[a]\n\tv_add_u32 %[r" R "], %[b], %[r" R "]\n\t"
#define TERN_P_MIXED_FOUR TERN_P_MIXED("0", "4", "0") TERN_P_MIXED("1", "5", "1") TERN_P_MIXED("2", "6", "2") TERN_P_MIXED("3", "7", "3")
#define TERN_P_NOP "s_nop 0\n\t"
#define TERN_P_EIGHT(I, S)                                                                      \
    I("0", "0") S I("1", "1") S I("2", "2") S I("3", "3") S I("4", "0") S I("5", "1") S I("6", "2") S \
        I("7", "3") S
// binary pair: bit operation into t (registers r4..r7 serve as the scratch registers), popcount into r0..r3
#define TERN_P_BIN(R, T, K, S) \
    "v_bitop3_b32 %[r" T "], %[b], %[a], %[k" K "] bitop3:0x48\n\t" S "v_bcnt_u32_b32 %[r" R "], %[r" T "], %[r" R "]\n\t"
#define TERN_P_BIN_FOUR(S) \
    TERN_P_BIN("0", "4", "0", S) TERN_P_BIN("1", "5", "1", S) TERN_P_BIN("2", "6", "2", S) TERN_P_BIN("3", "7", "3", S)

template <int OP, bool NOP>
__global__ __launch_bounds__(512) void probe_opcode_kernel(ProbeConsts c, int iters, int32_t* sink)
{
    uint32_t a = threadIdx.x * 2654435761u + blockIdx.x, b = a ^ 0x9e3779b9u;
    uint32_t r[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = j;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int st = 0; st < 8; ++st) {
#define TERN_P_OPERANDS                                                                              \
    : [r0] "+v"(r[0]), [r1] "+v"(r[1]), [r2] "+v"(r[2]), [r3] "+v"(r[3]), [r4] "+v"(r[4]), [r5] "+v"(r[5]), \
      [r6] "+v"(r[6]), [r7] "+v"(r[7])                                                              \
    : [a] "v"(a), [b] "v"(b), [k0] "s"(c.k[4 * (st & 3)]), [k1] "s"(c.k[4 * (st & 3) + 1]),        \
      [k2] "s"(c.k[4 * (st & 3) + 2]), [k3] "s"(c.k[4 * (st & 3) + 3])
            if constexpr (OP == 0) {
                if constexpr (NOP) asm volatile(TERN_P_EIGHT(TERN_P_AND, TERN_P_NOP) TERN_P_OPERANDS);
                else asm volatile(TERN_P_EIGHT(TERN_P_AND, "") TERN_P_OPERANDS);
            } else if constexpr (OP == 1) {
                if constexpr (NOP) asm volatile(TERN_P_EIGHT(TERN_P_BCNT, TERN_P_NOP) TERN_P_OPERANDS);
                else asm volatile(TERN_P_EIGHT(TERN_P_BCNT, "") TERN_P_OPERANDS);
            } else if constexpr (OP == 2) {
                if constexpr (NOP) asm volatile(TERN_P_EIGHT(TERN_P_BITOP, TERN_P_NOP) TERN_P_OPERANDS);
                else asm volatile(TERN_P_EIGHT(TERN_P_BITOP, "") TERN_P_OPERANDS);
            } else if constexpr (OP == 3) {
                if constexpr (NOP) asm volatile(TERN_P_EIGHT(TERN_P_XOR, TERN_P_NOP) TERN_P_OPERANDS);
                else asm volatile(TERN_P_EIGHT(TERN_P_XOR, "") TERN_P_OPERANDS);
            } else if constexpr (OP == 4) {
                if constexpr (NOP) asm volatile(TERN_P_BIN_FOUR(TERN_P_NOP) TERN_P_OPERANDS);
                else asm volatile(TERN_P_BIN_FOUR("") TERN_P_OPERANDS);
            } else if constexpr (OP == 5) {
                if constexpr (NOP) asm volatile(TERN_P_EIGHT(TERN_P_ADD, TERN_P_NOP) TERN_P_OPERANDS);
                else asm volatile(TERN_P_EIGHT(TERN_P_ADD, "") TERN_P_OPERANDS);
            } else if constexpr (OP == 6) {
                asm volatile(TERN_P_EIGHT(TERN_P_XORV, "") TERN_P_OPERANDS);
            } else if constexpr (OP == 7) {
                asm volatile(TERN_P_EIGHT(TERN_P_BITOPV, "") TERN_P_OPERANDS);
            } else {
                asm volatile(TERN_P_MIXED_FOUR TERN_P_OPERANDS);
            }
#undef TERN_P_OPERANDS
        }
        a += 0x01010101u;
    }
    uint32_t x = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) x += r[j];
    if (x == 0x7fffffffu && b == 12345u) sink[0] = (int32_t)x;
}

}  // namespace
}  // namespace tern

extern "C" int tern_probe_valu(int32_t blocks, int32_t threads, int32_t iters, int32_t variant,
                               int32_t* sink, void* stream)
{
    using namespace tern;
    if (!sink) return TERN_ENULL;
    if (blocks < 1 || threads < 64 || threads > 512 || threads % 64 || iters < 1) return TERN_EARG;
    if (variant < 0 || variant >= TERN_PROBE_VARIANTS) return TERN_EARG;
    ProbeConsts c;
    for (int i = 0; i < 32; ++i) c.k[i] = 0x9e3779b9u * (uint32_t)(i + 1);
    typedef void (*kern_t)(ProbeConsts, int, int32_t*);
    static const kern_t table[TERN_PROBE_VARIANTS] = {
        probe_kernel, probe_unspaced_kernel,
        probe_opcode_kernel<0, false>, probe_opcode_kernel<0, true>,
        probe_opcode_kernel<1, false>, probe_opcode_kernel<1, true>,
        probe_opcode_kernel<2, false>, probe_opcode_kernel<2, true>,
        probe_opcode_kernel<3, false>, probe_opcode_kernel<3, true>,
        probe_bin_kernel, probe_opcode_kernel<4, false>,
        probe_opcode_kernel<5, false>, probe_opcode_kernel<5, true>,
        probe_opcode_kernel<6, false>, probe_opcode_kernel<7, false>, probe_opcode_kernel<8, false>,
    };
    hipLaunchKernelGGL(table[variant], dim3((unsigned)blocks), dim3((unsigned)threads), 0, (hipStream_t)stream, c,
                       iters, sink);
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}
