// Diagnostic: sustained issue rate of the convolution's instruction mix (and, popcount-accumulate,
// three-input bit operation, popcount-accumulate with wave-uniform second operands) with no
// memory traffic at all.  The benchmark uses it as the measured ceiling next to the nominal
// 256 CU x 64 lanes x 2.4 GHz figure.  Variant 0 runs the kernels' own statement (a scalar no-op
// between each producer and its popcount), variant 1 the same four instructions per word pair
// in an order that needs no wait state and with no scalar instruction in between, which is what
// a compiler's scheduler makes of them: the pair of figures shows what the spacing is worth.
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

}  // namespace
}  // namespace tern

extern "C" int tern_probe_valu(int32_t blocks, int32_t threads, int32_t iters, int32_t variant,
                               int32_t* sink, void* stream)
{
    using namespace tern;
    if (!sink) return TERN_ENULL;
    if (blocks < 1 || threads < 64 || threads > 512 || threads % 64 || iters < 1) return TERN_EARG;
    if (variant != 0 && variant != 1) return TERN_EARG;
    ProbeConsts c;
    for (int i = 0; i < 32; ++i) c.k[i] = 0x9e3779b9u * (uint32_t)(i + 1);
    hipLaunchKernelGGL(variant == 0 ? probe_kernel : probe_unspaced_kernel, dim3((unsigned)blocks),
                       dim3((unsigned)threads), 0, (hipStream_t)stream, c, iters, sink);
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}
