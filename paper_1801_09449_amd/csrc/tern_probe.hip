// Diagnostic: sustained issue rate of the convolution's instruction mix (and, popcount-accumulate,
// three-input bit operation, popcount-accumulate with wave-uniform second operands) with no
// memory traffic at all.  The benchmark uses it as the measured ceiling next to the nominal
// 256 CU x 64 lanes x 2.4 GHz figure.
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

}  // namespace
}  // namespace tern

extern "C" int tern_probe_valu(int32_t blocks, int32_t threads, int32_t iters, int32_t* sink,
                               void* stream)
{
    using namespace tern;
    if (!sink) return TERN_ENULL;
    if (blocks < 1 || threads < 64 || threads > 512 || threads % 64 || iters < 1) return TERN_EARG;
    ProbeConsts c;
    for (int i = 0; i < 32; ++i) c.k[i] = 0x9e3779b9u * (uint32_t)(i + 1);
    hipLaunchKernelGGL(probe_kernel, dim3((unsigned)blocks), dim3((unsigned)threads), 0,
                       (hipStream_t)stream, c, iters, sink);
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}
