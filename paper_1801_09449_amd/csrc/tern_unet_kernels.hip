// The data movement a U-Net needs between ternary convolutions, done on packed bit-planes, and
// the real-weight prediction layer (paper, section 3, Table 1: Upsample2D rows, the "Skip"
// column, the Prediction row):
//   - concat_kernel: every output voxel gathers, per source, the voxel that nearest-neighbour
//     upsampling and cropping map onto it, and lays the sources' channel bits side by side;
//   - real_conv_kernel: cross-correlation of ternary codes with float weights (+ bias).
// Both are small HBM streams next to the convolutions; neither uses LDS.
#include "tern_internal.h"

namespace tern {
namespace {

constexpr int kBlock = 256;

// Read-only data addressed uniformly by a whole wave (the float filters): the constant address
// space lets the compiler fetch it with scalar loads.
typedef const __attribute__((address_space(4))) float* scalar_fptr;

// One thread per (output voxel, output word q).  Output bits [32q, 32q+32) are assembled from
// the one or two words of each source that overlap them; padding bits of a source are zero, so
// OR-ing the shifted pieces is enough.
__global__ __launch_bounds__(kBlock) void concat_kernel(ConcatParams p)
{
    const int64_t gid = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (gid >= p.total) return;
    const int q = (int)(gid % p.wd_out);
    int64_t vox = gid / p.wd_out;
    const int64_t vox_out = vox;
    const int x = (int)(vox % p.ow); vox /= p.ow;
    const int y = (int)(vox % p.oh); vox /= p.oh;
    const int z = (int)(vox % p.od);
    const int n = (int)(vox / p.od);

    uint32_t m = 0u, s = 0u;
    for (int i = 0; i < p.n_src; ++i) {
        const ConcatSrc& src = p.s[i];
        const int rel = 32 * q - src.bit0;          // bit of the source that lands on output bit 32q
        if (rel >= 32 * src.wd || rel <= -32) continue;
        const int sz = (z + src.first[0]) / src.up[0];
        const int sy = (y + src.first[1]) / src.up[1];
        const int sx = (x + src.first[2]) / src.up[2];
        const uint32_t* v = src.p + ((((size_t)n * src.d + sz) * src.h + sy) * src.w + sx) * 2u * src.wd;
        if (rel >= 0) {
            const int j = rel >> 5, sh = rel & 31;
            uint32_t mm = v[j] >> sh, ss = v[src.wd + j] >> sh;
            if (sh != 0 && j + 1 < src.wd) {
                mm |= v[j + 1] << (32 - sh);
                ss |= v[src.wd + j + 1] << (32 - sh);
            }
            m |= mm; s |= ss;
        } else {
            m |= v[0] << (-rel);
            s |= v[src.wd] << (-rel);
        }
    }
    uint32_t* o = p.out + (size_t)vox_out * 2u * p.wd_out;
    o[q] = m;
    o[p.wd_out + q] = s;
}

// One thread per output voxel; output channels in groups of CG accumulators.  For every tap
// and input channel the lane turns its two plane bits into the code (+1, 0, -1) once and feeds
// all CG accumulators; the weights of a (tap, channel) are the same for every lane, so they
// come through the scalar cache.  The sum runs over taps in (a, b, c) order and, within a tap,
// over the input channels in ascending order; every term is an exact +-w (or 0), added in fp32.
template <int CG>
__global__ __launch_bounds__(kBlock) void real_conv_kernel(RealConvParams p)
{
    int64_t vox = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (vox >= p.total) return;
    const int64_t vox_out = vox;
    const int x = (int)(vox % p.ow); vox /= p.ow;
    const int y = (int)(vox % p.oh); vox /= p.oh;
    const int z = (int)(vox % p.od);
    const int n = (int)(vox / p.od);
    const int T = p.kd * p.kh * p.kw;
    const size_t per_filter = (size_t)p.c_in * T;
    const size_t ospatial = (size_t)p.od * p.oh * p.ow;
    const size_t sp = vox_out - (size_t)n * ospatial;

    for (int co0 = 0; co0 < p.c_out; co0 += CG) {
        float acc[CG];
#pragma unroll
        for (int g = 0; g < CG; ++g) acc[g] = (p.bias && co0 + g < p.c_out) ? p.bias[co0 + g] : 0.0f;
        // filters past c_out: re-read the last one (its result is dropped)
        scalar_fptr wf[CG];
#pragma unroll
        for (int g = 0; g < CG; ++g)
            wf[g] = (scalar_fptr)(uintptr_t)(p.wgt + (size_t)min(co0 + g, p.c_out - 1) * per_filter);
        int tap = 0;
        for (int a = 0; a < p.kd; ++a)
            for (int b = 0; b < p.kh; ++b)
                for (int c = 0; c < p.kw; ++c, ++tap) {
                    const int iz = z * p.sd - p.pd + a * p.dd;
                    const int iy = y * p.sh - p.ph + b * p.dh;
                    const int ix = x * p.sw - p.pw + c * p.dw;
                    const bool inb = iz >= 0 && iz < p.d && iy >= 0 && iy < p.h && ix >= 0 && ix < p.w;
                    const uint32_t* v = p.in + ((((size_t)n * p.d + (inb ? iz : 0)) * p.h + (inb ? iy : 0)) * p.w +
                                                (inb ? ix : 0)) * 2u * p.wd_in;
                    for (int q = 0; q < p.wd_in; ++q) {
                        // out-of-volume taps read as zeros: the walk stays uniform over the wave
                        const uint32_t m = inb ? v[q] : 0u;
                        const uint32_t neg = inb ? (v[p.wd_in + q] & m) : 0u;   // sign counts only under the mask
                        const uint32_t pos = m & ~neg;
                        const int live = min(32, p.c_in - 32 * q);
                        // eight channels at a time: their weights are fetched together (scalar
                        // loads, independent of the data), then used.  Channels past c_in have
                        // zero bits; their weight index is clamped to stay inside the filter.
                        for (int j0 = 0; j0 < live; j0 += 8) {
                            float wv[CG][8];
#pragma unroll
                            for (int jj = 0; jj < 8; ++jj) {
                                const size_t wi = (size_t)min(32 * q + j0 + jj, p.c_in - 1) * T + tap;
#pragma unroll
                                for (int g = 0; g < CG; ++g) wv[g][jj] = wf[g][wi];
                            }
#pragma unroll
                            for (int jj = 0; jj < 8; ++jj) {
                                const int j = j0 + jj;
                                const float code = (float)((int)((pos >> j) & 1u) - (int)((neg >> j) & 1u));
#pragma unroll
                                for (int g = 0; g < CG; ++g) acc[g] = fmaf(code, wv[g][jj], acc[g]);
                            }
                        }
                    }
                }
#pragma unroll
        for (int g = 0; g < CG; ++g)
            if (co0 + g < p.c_out) p.out[((size_t)n * p.c_out + co0 + g) * ospatial + sp] = acc[g];
    }
}

}  // namespace

int launch_concat(const ConcatParams& p, hipStream_t s)
{
    const int64_t blocks = (p.total + kBlock - 1) / kBlock;
    if (blocks > 0x7fffffff) return TERN_ESHAPE;
    hipLaunchKernelGGL(concat_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, s, p);
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}

int launch_real_conv(const RealConvParams& p, hipStream_t s)
{
    const int64_t blocks = (p.total + kBlock - 1) / kBlock;
    if (blocks > 0x7fffffff) return TERN_ESHAPE;
    if (p.c_out <= 2)
        hipLaunchKernelGGL(real_conv_kernel<2>, dim3((unsigned)blocks), dim3(kBlock), 0, s, p);
    else
        hipLaunchKernelGGL(real_conv_kernel<4>, dim3((unsigned)blocks), dim3(kBlock), 0, s, p);
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}

}  // namespace tern
