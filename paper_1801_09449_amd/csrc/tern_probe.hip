// Diagnostic: sustained issue rate of the convolution's instruction mix (and, popcount-accumulate,
// three-input bit operation, popcount-accumulate with wave-uniform second operands) with no
// memory traffic at all.  The benchmark uses it as the measured ceiling next to the nominal
// 256 CU x 64 lanes x 2.4 GHz figure.
#include "tern_internal.h"

namespace tern {
namespace {

struct ProbeConsts { uint32_t k[32]; };

__device__ __forceinline__ void popc_acc(int32_t& acc, uint32_t x)
{
    asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(x));
}

__global__ __launch_bounds__(512) void probe_kernel(ProbeConsts c, int iters, int32_t* sink)
{
    uint32_t a = threadIdx.x * 2654435761u + blockIdx.x, b = a ^ 0x9e3779b9u;
    int32_t acc_m[16], acc_n[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc_m[j] = acc_n[j] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const uint32_t M = a & c.k[j];
            const uint32_t N = M & (b ^ c.k[16 + j]);
            popc_acc(acc_m[j], M);
            popc_acc(acc_n[j], N);
        }
        a += 0x01010101u;   // keeps the loop body from being hoisted; 1 extra op per 64
    }
    int32_t r = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) r += acc_m[j] - 2 * acc_n[j];
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
