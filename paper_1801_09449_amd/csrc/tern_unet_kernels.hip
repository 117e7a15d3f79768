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

// The same sum with the filters of a channel group staged once per workgroup in LDS, transposed
// to [tap][channel][CG] (channels padded with zeros to a multiple of 4): a lane then gets the CG
// weights of four consecutive channels with 16-byte broadcast reads, a hundred cycles away
// instead of a scalar-cache round trip per eight channels.  Used whenever the group's filters
// fit in 48 KB; same order of operations, same bits as real_conv_kernel.
template <int CG>
__global__ __launch_bounds__(kBlock) void real_conv_lds_kernel(RealConvParams p, int c_pad)
{
    extern __shared__ __align__(16) float wl[];
    int64_t vox = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const bool active = vox < p.total;
    if (!active) vox = p.total - 1;
    const int64_t vox_out = vox;
    const int x = (int)(vox % p.ow); vox /= p.ow;
    const int y = (int)(vox % p.oh); vox /= p.oh;
    const int z = (int)(vox % p.od);
    const int n = (int)(vox / p.od);
    const int T = p.kd * p.kh * p.kw;
    const size_t per_filter = (size_t)p.c_in * T;
    const size_t ospatial = (size_t)p.od * p.oh * p.ow;
    const size_t sp = vox_out - (size_t)n * ospatial;
    const int rows = T * c_pad;

    for (int co0 = 0; co0 < p.c_out; co0 += CG) {
        if (co0 > 0) __syncthreads();          // everyone is done with the previous group's filters
        for (int i = threadIdx.x; i < rows * CG; i += kBlock) {
            const int g = i % CG;
            const int r = i / CG;
            const int c = r % c_pad, tap = r / c_pad;
            float wv = 0.0f;
            if (c < p.c_in) wv = p.wgt[(size_t)min(co0 + g, p.c_out - 1) * per_filter + (size_t)c * T + tap];
            wl[i] = wv;
        }
        __syncthreads();
        float acc[CG];
#pragma unroll
        for (int g = 0; g < CG; ++g) acc[g] = (p.bias && co0 + g < p.c_out) ? p.bias[co0 + g] : 0.0f;
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
                    const float* wt = wl + (size_t)tap * c_pad * CG;
                    for (int q = 0; q < p.wd_in; ++q) {
                        const uint32_t m = inb ? v[q] : 0u;
                        const uint32_t neg = inb ? (v[p.wd_in + q] & m) : 0u;
                        const uint32_t pos = m & ~neg;
                        const int live = min(32, c_pad - 32 * q);     // multiple of 4
                        for (int j0 = 0; j0 < live; j0 += 4) {
                            float wv[4 * CG];
#pragma unroll
                            for (int k = 0; k < 4 * CG; k += 4) {
                                const float4 r = *reinterpret_cast<const float4*>(wt + (size_t)(32 * q + j0) * CG + k);
                                wv[k] = r.x; wv[k + 1] = r.y; wv[k + 2] = r.z; wv[k + 3] = r.w;
                            }
#pragma unroll
                            for (int jj = 0; jj < 4; ++jj) {
                                const int j = j0 + jj;
                                const float code = (float)((int)((pos >> j) & 1u) - (int)((neg >> j) & 1u));
#pragma unroll
                                for (int g = 0; g < CG; ++g) acc[g] = fmaf(code, wv[jj * CG + g], acc[g]);
                            }
                        }
                    }
                }
        if (active) {
#pragma unroll
            for (int g = 0; g < CG; ++g)
                if (co0 + g < p.c_out) p.out[((size_t)n * p.c_out + co0 + g) * ospatial + sp] = acc[g];
        }
    }
}

// The same convolution through partial-sum tables: for every (tap, group of four input channels)
// LDS holds the 16 sums of the subsets of the group's four weights (per output channel of the
// group CG), built by the workgroup from the staged weights.  A voxel's +1 codes of such a group
// are a 4-bit index into the table and so are its -1 codes: two lookups, one addition and one
// subtraction per output channel replace four multiply-adds and the unpacking of four codes.
// A fixed order of operations again (table entries add their weights in channel order; the
// accumulator takes "+ entry of the +1 codes, - entry of the -1 codes" group by group), but not
// the order of real_conv_kernel: results agree within the rounding bound of a float sum of that
// many terms, not bit for bit.  Used when weights and tables (five times the weights) fit in 64 KB.
template <int CG>
__global__ __launch_bounds__(kBlock) void real_conv_lut_kernel(RealConvParams p, int c_pad)
{
    extern __shared__ __align__(16) float wl[];
    int64_t vox = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const bool active = vox < p.total;
    if (!active) vox = p.total - 1;
    const int64_t vox_out = vox;
    const int x = (int)(vox % p.ow); vox /= p.ow;
    const int y = (int)(vox % p.oh); vox /= p.oh;
    const int z = (int)(vox % p.od);
    const int n = (int)(vox / p.od);
    const int T = p.kd * p.kh * p.kw;
    const size_t per_filter = (size_t)p.c_in * T;
    const size_t ospatial = (size_t)p.od * p.oh * p.ow;
    const size_t sp = vox_out - (size_t)n * ospatial;
    const int rows = T * c_pad;                  // (tap, channel) pairs, channels padded to fours
    const int nq = c_pad / 4;                    // channel groups per tap
    float* lut = wl + (size_t)rows * CG;         // [tap][group][16][CG]

    for (int co0 = 0; co0 < p.c_out; co0 += CG) {
        if (co0 > 0) __syncthreads();            // everyone is done with the previous group's tables
        for (int i = threadIdx.x; i < rows * CG; i += kBlock) {
            const int g = i % CG;
            const int r = i / CG;
            const int c = r % c_pad, tap = r / c_pad;
            float wv = 0.0f;
            if (c < p.c_in) wv = p.wgt[(size_t)min(co0 + g, p.c_out - 1) * per_filter + (size_t)c * T + tap];
            wl[i] = wv;
        }
        __syncthreads();
        for (int i = threadIdx.x; i < T * nq * 16; i += kBlock) {
            const int v = i & 15;
            const float* w4 = wl + (size_t)(i >> 4) * 4 * CG;     // the group's four channels x CG
#pragma unroll
            for (int g = 0; g < CG; ++g) {
                float sum = 0.0f;
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    if ((v >> b) & 1) sum += w4[b * CG + g];
                lut[(size_t)i * CG + g] = sum;
            }
        }
        __syncthreads();
        float acc[CG];
#pragma unroll
        for (int g = 0; g < CG; ++g) acc[g] = (p.bias && co0 + g < p.c_out) ? p.bias[co0 + g] : 0.0f;
        // one tap's contribution from its voxel record (mask words, then sign words)
        auto add_tap = [&](int tap, const uint32_t* rec_m, const uint32_t* rec_s, int nwords) {
            const float* tt = lut + (size_t)tap * nq * 16 * CG;
            for (int q = 0; q < nwords; ++q) {
                const uint32_t m = rec_m[q];
                const uint32_t neg = rec_s[q] & m;
                const uint32_t pos = m & ~neg;
                const int live = min(32, c_pad - 32 * q);     // multiple of 4
                for (int j0 = 0; j0 < live; j0 += 4) {
                    const float* grp = tt + (size_t)(8 * q + (j0 >> 2)) * 16 * CG;
                    const float* ep = grp + ((pos >> j0) & 15u) * CG;
                    const float* en = grp + ((neg >> j0) & 15u) * CG;
#pragma unroll
                    for (int g = 0; g < CG; ++g) acc[g] = (acc[g] + ep[g]) - en[g];
                }
            }
        };
        auto tap_source = [&](int tap, bool& inb) -> const uint32_t* {
            const int c = tap % p.kw, r = tap / p.kw;
            const int b = r % p.kh, a = r / p.kh;
            const int iz = z * p.sd - p.pd + a * p.dd;
            const int iy = y * p.sh - p.ph + b * p.dh;
            const int ix = x * p.sw - p.pw + c * p.dw;
            inb = iz >= 0 && iz < p.d && iy >= 0 && iy < p.h && ix >= 0 && ix < p.w;
            return p.in + ((((size_t)n * p.d + (inb ? iz : 0)) * p.h + (inb ? iy : 0)) * p.w + (inb ? ix : 0)) *
                              2u * p.wd_in;
        };
        if (p.wd_in == 2) {
            // 16-byte records: the loads of up to nine taps are in flight together (one memory
            // round trip per batch instead of one per tap)
            constexpr int kBatch = 9;
            for (int t0 = 0; t0 < T; t0 += kBatch) {
                uint4 rec[kBatch];
#pragma unroll
                for (int k = 0; k < kBatch; ++k) {
                    rec[k] = make_uint4(0u, 0u, 0u, 0u);          // zero padding: every code is 0
                    if (t0 + k < T) {
                        bool inb;
                        const uint32_t* v = tap_source(t0 + k, inb);
                        if (inb) rec[k] = *reinterpret_cast<const uint4*>(v);
                    }
                }
#pragma unroll
                for (int k = 0; k < kBatch; ++k) {
                    if (t0 + k < T) {
                        const uint32_t mw[2] = {rec[k].x, rec[k].y}, sw[2] = {rec[k].z, rec[k].w};
                        add_tap(t0 + k, mw, sw, 2);
                    }
                }
            }
        } else {
            for (int tap = 0; tap < T; ++tap) {
                bool inb;
                const uint32_t* v = tap_source(tap, inb);
                if (inb) add_tap(tap, v, v + p.wd_in, p.wd_in);
            }
        }
        if (active) {
#pragma unroll
            for (int g = 0; g < CG; ++g)
                if (co0 + g < p.c_out) p.out[((size_t)n * p.c_out + co0 + g) * ospatial + sp] = acc[g];
        }
    }
}

// Per-channel code statistics of a packed tensor (the paper reports how sparse weights and
// activations become, section 4).  A wave takes 64 voxels at a time; for every channel bit the
// wave-wide vote of "this voxel's bit is set" is counted, lane j keeping the running nonzero
// count of channel 32q + j and lane 32 + j the count of its -1 codes.  One atomic add per
// (wave, channel) at the end.
__global__ __launch_bounds__(kBlock) void count_codes_kernel(const uint32_t* __restrict__ in, int64_t voxels,
                                                             int32_t wd, int32_t c,
                                                             unsigned long long* __restrict__ nonzero,
                                                             unsigned long long* __restrict__ negative)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * kBlock) >> 6;
    for (int q = 0; q < wd; ++q) {
        unsigned long long mine = 0ull;
        for (int64_t v0 = wave * 64; v0 < voxels; v0 += nwaves * 64) {
            const int64_t vox = v0 + lane;
            uint32_t m = 0u, sg = 0u;
            if (vox < voxels) {
                m = in[(size_t)vox * 2u * wd + q];
                sg = in[(size_t)vox * 2u * wd + wd + q] & m;
            }
            for (int j = 0; j < 32; ++j) {
                const unsigned long long vm = __ballot((m >> j) & 1u);
                const unsigned long long vs = __ballot((sg >> j) & 1u);
                if (lane == j) mine += (unsigned long long)__popcll(vm);
                if (lane == 32 + j) mine += (unsigned long long)__popcll(vs);
            }
        }
        const int ch = 32 * q + (lane & 31);
        if (ch < c && mine != 0ull) atomicAdd(lane < 32 ? &nonzero[ch] : &negative[ch], mine);
    }
}

// Sum pooling into two balanced-ternary digits.  The sum of up to four ternary codes lies in
// [-4, 4] and has exactly one representation low + 3 * high with both digits in {-1, 0, +1}, so a
// pooled tensor stays in the 2-bit format at twice the channel words (word 2k = low digits of
// channels 32k.., word 2k+1 = their high digits) and the convolution behind an average pooling
// (Table 1) costs two word pairs per pooled input word instead of one per unpooled voxel.
// All 32 channels of a word at once, on bit planes: count the +1 and the -1 codes of the window
// with one-bit adders (three-bit counts P and N), subtract, and read the digits off the 4-bit
// two's-complement difference.
struct PoolParams {
    const uint32_t* in;     // [N][d][h][w][2][wd]
    uint32_t* out;          // [N][od][oh][ow][2][2*wd]
    int32_t d, h, w, od, oh, ow, wd;
    int32_t pd, ph, pw;     // window, volume <= 4
    int64_t total;          // N * od * oh * ow * wd
};

__device__ __forceinline__ void count4(const uint32_t (&b)[4], uint32_t& c0, uint32_t& c1, uint32_t& c2)
{
    const uint32_t s1 = b[0] ^ b[1] ^ b[2];
    const uint32_t k1 = (b[0] & b[1]) | (b[2] & (b[0] ^ b[1]));   // carry of the first three
    c0 = s1 ^ b[3];
    const uint32_t k2 = s1 & b[3];
    c1 = k1 ^ k2;
    c2 = k1 & k2;
}

__global__ __launch_bounds__(kBlock) void pool_digits_kernel(PoolParams p)
{
    const int64_t gid = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (gid >= p.total) return;
    const int k = (int)(gid % p.wd);
    int64_t r = gid / p.wd;
    const int ox = (int)(r % p.ow); r /= p.ow;
    const int oy = (int)(r % p.oh); r /= p.oh;
    const int oz = (int)(r % p.od);
    const int64_t n = r / p.od;
    uint32_t pos[4] = {0u, 0u, 0u, 0u}, neg[4] = {0u, 0u, 0u, 0u};
    int idx = 0;
    for (int a = 0; a < p.pd; ++a)
        for (int b = 0; b < p.ph; ++b)
            for (int c = 0; c < p.pw; ++c, ++idx) {
                const size_t vox = (((size_t)n * p.d + (oz * p.pd + a)) * p.h + (oy * p.ph + b)) * p.w + (ox * p.pw + c);
                const uint32_t m = p.in[vox * 2u * p.wd + k];
                const uint32_t sg = p.in[vox * 2u * p.wd + p.wd + k];
                // (idx < 4 by the launcher's check on the window volume)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (q == idx) { pos[q] = m & ~sg; neg[q] = m & sg; }
            }
    uint32_t p0, p1, p2, n0, n1, n2;
    count4(pos, p0, p1, p2);
    count4(neg, n0, n1, n2);
    // s = P - N, four-bit two's complement, bit by bit with a borrow
    const uint32_t s0 = p0 ^ n0;
    const uint32_t b1 = ~p0 & n0;
    const uint32_t s1 = p1 ^ n1 ^ b1;
    const uint32_t b2 = (~p1 & n1) | (~(p1 ^ n1) & b1);
    const uint32_t s2 = p2 ^ n2 ^ b2;
    const uint32_t s3 = (~p2 & n2) | (~(p2 ^ n2) & b2);          // sign
    // high digit: nonzero for |s| >= 2 (positive: 2, 3, 4; negative: everything but -1 = 1111)
    const uint32_t hi_m = (~s3 & (s2 | s1)) | (s3 & ~(s2 & s1 & s0));
    const uint32_t hi_s = s3 & hi_m;
    // low digit s - 3 * high: zero for s in {-3, 0, 3} = {1101, 0000, 0011}, negative for
    // s in {-4, -1, 2} = {1100, 1111, 0010}
    const uint32_t z = (s3 & s2 & ~s1 & s0) | (~s3 & ~s2 & ~s1 & ~s0) | (~s3 & ~s2 & s1 & s0);
    const uint32_t lo_m = ~z;
    const uint32_t lo_s = (s3 & s2 & ~s1 & ~s0) | (s3 & s2 & s1 & s0) | (~s3 & ~s2 & s1 & ~s0);
    const size_t ovox = (size_t)(gid / p.wd);
    uint32_t* o = p.out + ovox * 4u * p.wd;     // 2 planes of 2*wd words
    *reinterpret_cast<uint2*>(o + 2 * k) = make_uint2(lo_m, hi_m);
    *reinterpret_cast<uint2*>(o + 2 * p.wd + 2 * k) = make_uint2(lo_s, hi_s);
}

__global__ void zero_counts_kernel(unsigned long long* a, unsigned long long* b, int32_t c)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < c) { a[i] = 0ull; b[i] = 0ull; }
}

}  // namespace

int launch_count_codes(const uint32_t* in, int64_t voxels, int32_t c, unsigned long long* nonzero,
                       unsigned long long* negative, hipStream_t s)
{
    // a small fill kernel rather than a memset, so that the call can be captured into a graph
    hipLaunchKernelGGL(zero_counts_kernel, dim3((unsigned)((c + 255) / 256)), dim3(256), 0, s, nonzero, negative, c);
    TERN_HIP_CHECK(hipGetLastError());
    const int wd = (c + 31) / 32;
    int64_t blocks = (voxels + kBlock - 1) / kBlock;
    if (blocks > 2048) blocks = 2048;      // grid-stride: a few waves per SIMD, few atomics
    hipLaunchKernelGGL(count_codes_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, s, in, voxels, wd, c, nonzero,
                       negative);
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}

int launch_pool_digits(const uint32_t* in, const tern_dims& in_dims, const int32_t window[3], uint32_t* out,
                       hipStream_t s)
{
    PoolParams p;
    p.in = in; p.out = out;
    p.d = in_dims.d; p.h = in_dims.h; p.w = in_dims.w;
    p.pd = window[0]; p.ph = window[1]; p.pw = window[2];
    p.od = in_dims.d / p.pd; p.oh = in_dims.h / p.ph; p.ow = in_dims.w / p.pw;
    p.wd = (in_dims.c + 31) / 32;
    p.total = (int64_t)in_dims.n * p.od * p.oh * p.ow * p.wd;
    if (p.total == 0) return TERN_OK;
    const int64_t blocks = (p.total + kBlock - 1) / kBlock;
    if (blocks > 0x7fffffff) return TERN_ESHAPE;
    hipLaunchKernelGGL(pool_digits_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, s, p);
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}

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
    const int cg = p.c_out <= 2 ? 2 : 4;
    const int c_pad = (p.c_in + 3) / 4 * 4;
    const int64_t lds = (int64_t)p.kd * p.kh * p.kw * c_pad * cg * 4;
    if (5 * lds <= 64 * 1024) {      // weights + partial-sum tables
        if (cg == 2)
            hipLaunchKernelGGL(real_conv_lut_kernel<2>, dim3((unsigned)blocks), dim3(kBlock), (size_t)(5 * lds), s, p, c_pad);
        else
            hipLaunchKernelGGL(real_conv_lut_kernel<4>, dim3((unsigned)blocks), dim3(kBlock), (size_t)(5 * lds), s, p, c_pad);
    } else if (lds <= 48 * 1024) {
        if (cg == 2)
            hipLaunchKernelGGL(real_conv_lds_kernel<2>, dim3((unsigned)blocks), dim3(kBlock), (size_t)lds, s, p, c_pad);
        else
            hipLaunchKernelGGL(real_conv_lds_kernel<4>, dim3((unsigned)blocks), dim3(kBlock), (size_t)lds, s, p, c_pad);
    } else if (cg == 2) {
        hipLaunchKernelGGL(real_conv_kernel<2>, dim3((unsigned)blocks), dim3(kBlock), 0, s, p);
    } else {
        hipLaunchKernelGGL(real_conv_kernel<4>, dim3((unsigned)blocks), dim3(kBlock), 0, s, p);
    }
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}

}  // namespace tern
