// Fallback ternary convolution for geometries the tiled kernel does not take (halo tile larger
// than LDS).  One thread computes one accumulator (int32 output) or one 32-channel output word
// pair (packed output) straight from global memory.  Slow but general; same arithmetic as the
// tiled kernel: Eq. 9 as popcount(M) - 2*popcount(M & X), M = mask_w & mask_a,
// X = sign_w ^ sign_a, out-of-volume voxels contributing nothing; with binary filters (Eq. 8)
// M = mask_a.
#include "tern_internal.h"

namespace tern {
namespace {

__device__ __forceinline__ int32_t dot_at(const ConvParams& p, int n, int co, int z, int y, int x)
{
    const int Wd = p.wd_in;
    const int wc = p.wc, nchunk = Wd / wc;
    int32_t acc_m = 0, acc_n = 0;
    int32_t high_m = 0, high_n = 0;   // odd words of a two-digit input: they count three times
    for (int a = 0; a < p.kd; ++a) {
        const int iz = z * p.sd - p.pd + a * p.dd;
        if (iz < 0 || iz >= p.d) continue;
        for (int b = 0; b < p.kh; ++b) {
            const int iy = y * p.sh - p.ph + b * p.dh;
            if (iy < 0 || iy >= p.h) continue;
            for (int c = 0; c < p.kw; ++c) {
                const int ix = x * p.sw - p.pw + c * p.dw;
                if (ix < 0 || ix >= p.w) continue;
                const uint32_t* av =
                    p.in + ((((size_t)n * p.d + iz) * p.h + iy) * p.w + ix) * 2u * Wd;
                const int tap = (a * p.kh + b) * p.kw + c;
                if (p.tp_slots) {
                    // tap-packed bank: [tap / slots][co_pad][2][1], this tap's bits start at
                    // bit (tap % slots) * shift; the activation word has bits only below C_in
                    const int step = tap / p.tp_slots, sh = (tap - step * p.tp_slots) * p.tp_shift;
                    const uint32_t* wv = p.wgt + ((size_t)step * p.co_pad + co) * 2u;
                    const uint32_t live = (1u << p.c_in) - 1u;
                    const uint32_t M = av[0] & live & (wv[0] >> sh);
                    const uint32_t N = M & (av[1] ^ (wv[1] >> sh));
                    acc_m += __builtin_popcount(M);
                    acc_n += __builtin_popcount(N);
                    continue;
                }
                if (p.binary) {
                    // binary filter bank: [tap * nchunk + chunk][co_pad][wc] sign words; every
                    // nonzero activation counts, against the filter's sign (Eq. 8)
                    for (int q = 0; q < Wd; ++q) {
                        const uint32_t sw = p.wgt[((size_t)(tap * nchunk + q / wc) * p.co_pad + co) * wc + q % wc];
                        acc_m += __builtin_popcount(av[q]);
                        acc_n += __builtin_popcount(av[q] & (av[Wd + q] ^ sw));
                    }
                    continue;
                }
                for (int q = 0; q < Wd; ++q) {
                    // filter bank: [tap * nchunk + chunk][co_pad][2][wc]
                    const uint32_t* wv =
                        p.wgt + ((size_t)(tap * nchunk + q / wc) * p.co_pad + co) * 2u * wc + q % wc;
                    const uint32_t M = av[q] & wv[0];
                    const uint32_t N = M & (av[Wd + q] ^ wv[wc]);
                    if (p.digits && (q & 1)) {
                        high_m += __builtin_popcount(M);
                        high_n += __builtin_popcount(N);
                    } else {
                        acc_m += __builtin_popcount(M);
                        acc_n += __builtin_popcount(N);
                    }
                }
            }
        }
    }
    return (acc_m - 2 * acc_n) + 3 * (high_m - 2 * high_n);
}

__global__ __launch_bounds__(256) void conv_generic_acc(ConvParams p, int64_t total)
{
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= total) return;
    int64_t r = gid;
    const int x = (int)(r % p.ow); r /= p.ow;
    const int y = (int)(r % p.oh); r /= p.oh;
    const int z = (int)(r % p.od); r /= p.od;
    const int co = (int)(r % p.c_out);
    const int n = (int)(r / p.c_out);
    p.out_acc[gid] = dot_at(p, n, co, z, y, x);
}

__global__ __launch_bounds__(256) void conv_generic_packed(ConvParams p, int64_t total)
{
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= total) return;
    int64_t r = gid;
    const int q = (int)(r % p.wd_out); r /= p.wd_out;   // output word
    const int x = (int)(r % p.ow); r /= p.ow;
    const int y = (int)(r % p.oh); r /= p.oh;
    const int z = (int)(r % p.od);
    const int n = (int)(r / p.od);
    uint32_t m = 0, s = 0;
    const int cmax = min(32, p.c_out - 32 * q);
    for (int j = 0; j < cmax; ++j) {
        const int co = 32 * q + j;
        const int32_t acc = dot_at(p, n, co, z, y, x);
        const bool pos = acc > p.hi[co];
        const bool neg = (acc < p.lo[co]) && !pos;
        m |= ((pos || neg) ? 1u : 0u) << j;
        s |= (neg ? 1u : 0u) << j;
    }
    uint32_t* out = p.out_packed + ((((size_t)n * p.od + z) * p.oh + y) * p.ow + x) * 2u * p.wd_out;
    out[q] = m;
    out[p.wd_out + q] = s;
}

}  // namespace

int launch_conv3d_generic(const ConvParams& p, hipStream_t s)
{
    const int64_t vox = (int64_t)p.n * p.od * p.oh * p.ow;
    const int64_t total = p.out_acc ? vox * p.c_out : vox * p.wd_out;
    const int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffff) return TERN_ESHAPE;
    if (p.out_acc)
        hipLaunchKernelGGL(conv_generic_acc, dim3((unsigned)blocks), dim3(256), 0, s, p, total);
    else
        hipLaunchKernelGGL(conv_generic_packed, dim3((unsigned)blocks), dim3(256), 0, s, p, total);
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}

}  // namespace tern
