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

// One thread per (output voxel, output channel), channel fastest.  The sum runs over taps in
// (a, b, c) order and, within a tap, over the nonzero input channels in ascending order; every
// term is an exact +-w, added in fp32.
__global__ __launch_bounds__(kBlock) void real_conv_kernel(RealConvParams p)
{
    const int64_t gid = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (gid >= p.total) return;
    const int co = (int)(gid % p.c_out);
    int64_t vox = gid / p.c_out;
    const int x = (int)(vox % p.ow); vox /= p.ow;
    const int y = (int)(vox % p.oh); vox /= p.oh;
    const int z = (int)(vox % p.od);
    const int n = (int)(vox / p.od);

    const int T = p.kd * p.kh * p.kw;
    const float* wco = p.wgt + (size_t)co * p.c_in * T;
    float acc = p.bias ? p.bias[co] : 0.0f;
    int tap = 0;
    for (int a = 0; a < p.kd; ++a)
        for (int b = 0; b < p.kh; ++b)
            for (int c = 0; c < p.kw; ++c, ++tap) {
                const int iz = z * p.sd - p.pd + a * p.dd;
                const int iy = y * p.sh - p.ph + b * p.dh;
                const int ix = x * p.sw - p.pw + c * p.dw;
                if (iz < 0 || iz >= p.d || iy < 0 || iy >= p.h || ix < 0 || ix >= p.w) continue;
                const uint32_t* v = p.in + ((((size_t)n * p.d + iz) * p.h + iy) * p.w + ix) * 2u * p.wd_in;
                for (int q = 0; q < p.wd_in; ++q) {
                    uint32_t m = v[q];
                    const uint32_t sg = v[p.wd_in + q];
                    while (m) {
                        const int j = __builtin_ctz(m);
                        m &= m - 1u;
                        const float wv = wco[(size_t)(32 * q + j) * T + tap];
                        acc += ((sg >> j) & 1u) ? -wv : wv;
                    }
                }
            }
    p.out[(((size_t)n * p.c_out + co) * p.od + z) * p.oh * p.ow + (size_t)y * p.ow + x] = acc;
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
    hipLaunchKernelGGL(real_conv_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, s, p);
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}

}  // namespace tern
