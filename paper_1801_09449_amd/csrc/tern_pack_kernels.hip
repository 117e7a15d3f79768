// Streaming kernels that turn an unpacked NCDHW tensor into channel-packed bit-planes
// (mask plane, sign plane; the 2-bit storage of the paper's Fig. 3):
//   - int8 ternary values                       (tern_pack)
//   - int32 accumulators against integer cut points, or float values against float cut points:
//     the hard activation of Eq. 6               (tern_threshold_pack)
// All three are HBM-bound streams.  A thread owns VPT consecutive voxels of one batch item and
// walks the channel words; for a fixed channel the lanes of a wave read consecutive addresses.
#include <type_traits>

#include "tern_conv_common.h"
#include "tern_internal.h"

namespace tern {
namespace {

constexpr int kBlock = 256;

// VPT voxels of type T starting at p (4 or 16 bytes, naturally aligned, when VPT > 1).
template <typename T, int VPT>
struct Vec {
    T v[VPT];
    __device__ void load(const T* p)
    {
        if constexpr (VPT == 1) {
            v[0] = *p;
        } else if constexpr (sizeof(T) * VPT == 4) {
            uint32_t raw = *reinterpret_cast<const uint32_t*>(p);
            __builtin_memcpy(v, &raw, 4);
        } else if constexpr (sizeof(T) * VPT == 8) {
            uint2 raw = *reinterpret_cast<const uint2*>(p);
            __builtin_memcpy(v, &raw, 8);
        } else {
            static_assert(sizeof(T) * VPT == 16, "unsupported vector width");
            uint4 raw = *reinterpret_cast<const uint4*>(p);
            __builtin_memcpy(v, &raw, 16);
        }
    }
};

// Decide VPT values of one channel and OR their bits into bit j of the voxels' words.
template <typename T, int VPT, int MODE>
__device__ __forceinline__ void classify(const Vec<T, VPT>& x, T tl, T th, int j, uint32_t (&m)[VPT],
                                         uint32_t (&s)[VPT])
{
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        bool nz, neg;
        if constexpr (MODE == 0) {
            nz = x.v[i] != 0;
            neg = x.v[i] < 0;
        } else {
            const bool pos = x.v[i] > th;
            neg = (x.v[i] < tl) && !pos;
            nz = pos || neg;
        }
        m[i] |= (nz ? 1u : 0u) << j;
        s[i] |= (neg ? 1u : 0u) << j;
    }
}

// int8 fast path.  A 32-bit word holds one channel's values of four consecutive voxels.  Per byte,
// "nonzero" and "negative" are single bits (any bit set / bit 7), so eight channels of four voxels
// are classified with a few word-wide operations each: flag bits land at bit 0 of every byte and
// are shifted to bit j of the byte for channel j of the octet.  The result has voxel i's eight
// channel bits in byte i; four octets are then transposed into the voxels' 32-channel words.
__device__ __forceinline__ void classify_octet(const uint32_t (&w)[8], int live, uint32_t& tm, uint32_t& ts)
{
    tm = ts = 0u;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t x = j < live ? w[j] : 0u;
        const uint32_t any = ((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x;   // bit 7 of a byte: byte != 0
        tm |= ((any >> 7) & 0x01010101u) << j;
        ts |= ((x >> 7) & 0x01010101u) << j;
    }
}

// byte i of t[0], t[1], t[2], t[3] -> one word (t[g] = channel octet g)
__device__ __forceinline__ uint32_t byte_column(const uint32_t (&t)[4], int i)
{
    const uint32_t sel = (uint32_t)i | ((uint32_t)(4 + i) << 8) | 0x0c0c0000u;   // 0x0c selects a zero byte
    const uint32_t lo = __builtin_amdgcn_perm(t[1], t[0], sel);
    const uint32_t hi = __builtin_amdgcn_perm(t[3], t[2], sel);
    return lo | (hi << 16);
}

// One 32-channel word group of VPT voxels from int8 data: channels c0 .. c0+31 (those >= C read
// a valid address and are masked out).  NW = VPT / 4 words of voxels per channel.
template <int VPT>
__device__ __forceinline__ void pack_group_i8(const int8_t* base, int64_t spatial, int c0, int C,
                                              uint32_t (&m)[VPT], uint32_t (&s)[VPT])
{
    constexpr int NW = VPT / 4;
    uint32_t tm[NW][4], ts[NW][4];
    if constexpr (NW == 1) {
        // all 32 channel loads in flight at once (128 bytes per lane)
        uint32_t w[4][8];
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int c = min(c0 + 8 * g + j, C - 1);
                w[g][j] = *reinterpret_cast<const uint32_t*>(base + (size_t)c * spatial);
            }
#pragma unroll
        for (int g = 0; g < 4; ++g) classify_octet(w[g], C - (c0 + 8 * g), tm[0][g], ts[0][g]);
    } else {
        // 16-byte loads: one octet of channels at a time (128 bytes per lane in flight)
        static_assert(NW == 4, "4 or 16 voxels per thread");
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint32_t r[8][NW];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int c = min(c0 + 8 * g + j, C - 1);
                const uint4 v = *reinterpret_cast<const uint4*>(base + (size_t)c * spatial);
                r[j][0] = v.x; r[j][1] = v.y; r[j][2] = v.z; r[j][3] = v.w;
            }
#pragma unroll
            for (int k = 0; k < NW; ++k) {
                uint32_t w[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) w[j] = r[j][k];
                classify_octet(w, C - (c0 + 8 * g), tm[k][g], ts[k][g]);
            }
        }
    }
#pragma unroll
    for (int k = 0; k < NW; ++k)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            m[4 * k + i] = byte_column(tm[k], i);
            s[4 * k + i] = byte_column(ts[k], i);
        }
}

// MODE 0: int8 ternary input.  MODE 1: thresholds (T = int32_t or float).
// WDT > 0: Wd is the compile-time constant WDT, all words of the VPT voxels stay in registers and
// every voxel is written with 16-byte stores (a thread writes VPT * 8 * Wd contiguous bytes).
// WDT == 0: any Wd, word-by-word stores.
template <typename T, int VPT, int MODE, int WDT>
__global__ __launch_bounds__(kBlock) void pack_kernel(const T* __restrict__ src,
                                                      uint32_t* __restrict__ dst,
                                                      const T* __restrict__ lo,
                                                      const T* __restrict__ hi, int32_t C,
                                                      int32_t Wd, int64_t spatial,
                                                      int64_t groups_per_n, int64_t total_groups)
{
    const int64_t gid = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (gid >= total_groups) return;
    const int64_t n = gid / groups_per_n;
    const int64_t v0 = (gid - n * groups_per_n) * VPT;  // first voxel (within batch item n)
    const T* base = src + (size_t)n * C * spatial + v0;

    if constexpr (WDT > 0) {
        uint32_t m[WDT][VPT], s[WDT][VPT];
#pragma unroll
        for (int q = 0; q < WDT; ++q) {
#pragma unroll
            for (int i = 0; i < VPT; ++i) m[q][i] = s[q][i] = 0u;
            const int cbase = 32 * q;
            if constexpr (MODE == 0 && sizeof(T) == 1 && VPT % 4 == 0) {
                if (cbase < C)
                    pack_group_i8<VPT>(reinterpret_cast<const int8_t*>(base), spatial, cbase, C, m[q], s[q]);
            } else if (cbase + 32 <= C) {
                // full word: batches of independent loads, at least 128 bytes in flight per lane
                constexpr int B = (sizeof(T) * VPT >= 16) ? 8 : 32;
#pragma unroll
                for (int j0 = 0; j0 < 32; j0 += B) {
                    Vec<T, VPT> x[B];
#pragma unroll
                    for (int j = 0; j < B; ++j) x[j].load(base + (size_t)(cbase + j0 + j) * spatial);
#pragma unroll
                    for (int j = 0; j < B; ++j) {
                        T tl = T(0), th = T(0);
                        if constexpr (MODE == 1) { tl = lo[cbase + j0 + j]; th = hi[cbase + j0 + j]; }
                        classify<T, VPT, MODE>(x[j], tl, th, j0 + j, m[q], s[q]);
                    }
                }
            } else {
                for (int j = 0; cbase + j < C; ++j) {
                    Vec<T, VPT> x;
                    x.load(base + (size_t)(cbase + j) * spatial);
                    T tl = T(0), th = T(0);
                    if constexpr (MODE == 1) { tl = lo[cbase + j]; th = hi[cbase + j]; }
                    classify<T, VPT, MODE>(x, tl, th, j, m[q], s[q]);
                }
            }
        }
        uint32_t* out = dst + ((size_t)n * spatial + v0) * 2u * WDT;
        if constexpr (WDT == 1) {
            static_assert(VPT % 2 == 0, "two 8-byte voxels per 16-byte store");
#pragma unroll
            for (int i = 0; i < VPT; i += 2)
                *reinterpret_cast<uint4*>(out + 2 * i) = make_uint4(m[0][i], s[0][i], m[0][i + 1], s[0][i + 1]);
        } else {
            static_assert(WDT % 2 == 0, "even word counts only");
#pragma unroll
            for (int i = 0; i < VPT; ++i) {
                uint32_t* o = out + (size_t)i * 2u * WDT;
                if constexpr (WDT == 2) {
                    *reinterpret_cast<uint4*>(o) = make_uint4(m[0][i], m[1][i], s[0][i], s[1][i]);
                } else {
#pragma unroll
                    for (int q = 0; q < WDT; q += 4) {
                        *reinterpret_cast<uint4*>(o + q) = make_uint4(m[q][i], m[q + 1][i], m[q + 2][i], m[q + 3][i]);
                        *reinterpret_cast<uint4*>(o + WDT + q) = make_uint4(s[q][i], s[q + 1][i], s[q + 2][i], s[q + 3][i]);
                    }
                }
            }
        }
    } else {
        uint32_t* out = dst + ((size_t)n * spatial + v0) * 2u * Wd;
        // blockIdx.y selects a slice of the channel words (one slice = all words, unless the
        // launch split them to get more threads out of a small volume with many channels)
        const int q_per_slice = (Wd + (int)gridDim.y - 1) / (int)gridDim.y;
        const int q_begin = blockIdx.y * q_per_slice;
        const int q_end = min(Wd, q_begin + q_per_slice);
        for (int q = q_begin; q < q_end; ++q) {
            uint32_t m[VPT], s[VPT];
#pragma unroll
            for (int i = 0; i < VPT; ++i) m[i] = s[i] = 0u;
            const int cmax = min(32, C - 32 * q);
            if constexpr (MODE == 0 && sizeof(T) == 1 && VPT % 4 == 0)
                pack_group_i8<VPT>(reinterpret_cast<const int8_t*>(base), spatial, 32 * q, C, m, s);
            else
#pragma unroll 8
            for (int j = 0; j < cmax; ++j) {
                const int c = 32 * q + j;
                Vec<T, VPT> x;
                x.load(base + (size_t)c * spatial);
                T tl = T(0), th = T(0);
                if constexpr (MODE == 1) { tl = lo[c]; th = hi[c]; }
                classify<T, VPT, MODE>(x, tl, th, j, m, s);
            }
#pragma unroll
            for (int i = 0; i < VPT; ++i) {
                out[(size_t)i * 2u * Wd + q] = m[i];
                out[(size_t)i * 2u * Wd + Wd + q] = s[i];
            }
        }
    }
}

template <typename T, int MODE>
int launch_pack_any(const T* src, tern_dims dims, const T* lo, const T* hi, uint32_t* dst,
                    hipStream_t s)
{
    const int64_t spatial = (int64_t)dims.d * dims.h * dims.w;
    const int32_t Wd = (dims.c + 31) / 32;
    // Voxels per thread: 4, or 16 for int8 when that still leaves a few thousand waves (a 16-byte
    // load per lane instead of a 4-byte one).
    constexpr bool kByte = sizeof(T) == 1;
    const bool ok4 = (spatial % 4 == 0) && (((uintptr_t)src % (4 * sizeof(T))) == 0);
    const bool ok16 = kByte && (spatial % 16 == 0) && (((uintptr_t)src % 16) == 0) &&
                      spatial * dims.n / 16 >= (int64_t)4096 * 64;
    const int vpt = ok16 ? 16 : (ok4 ? 4 : 1);
    const bool vec_ok = vpt > 1;
    const int64_t gpn = spatial / vpt;
    const int64_t total = gpn * dims.n;
    const int64_t blocks = (total + kBlock - 1) / kBlock;
    if (blocks > 0x7fffffff) return TERN_ESHAPE;
    // Few voxels but many channels (e.g. 256 channels on 32-cubed): one thread per channel word
    // instead of one per voxel group, through the word-by-word variant.
    const bool split_words = vpt == 4 && Wd >= 4 && total < (int64_t)1024 * 64;
    const dim3 grid((unsigned)blocks, split_words ? (unsigned)Wd : 1u), block(kBlock);
#define TERN_PACK_LAUNCH(VPT_, WDT_)                                                              \
    hipLaunchKernelGGL((pack_kernel<T, VPT_, MODE, WDT_>), grid, block, 0, s, src, dst, lo, hi, dims.c, \
                       Wd, spatial, gpn, total)
    if (vec_ok) {
        if (vpt == 16) {
            if constexpr (kByte) {
                switch (Wd) {   // 16 voxels x 2*Wd words stay in registers
                    case 1: TERN_PACK_LAUNCH(16, 1); break;
                    case 2: TERN_PACK_LAUNCH(16, 2); break;
                    case 4: TERN_PACK_LAUNCH(16, 4); break;
                    default: TERN_PACK_LAUNCH(16, 0); break;
                }
            }
        } else if (split_words) {
            TERN_PACK_LAUNCH(4, 0);
        } else {
            switch (Wd) {
                case 1: TERN_PACK_LAUNCH(4, 1); break;
                case 2: TERN_PACK_LAUNCH(4, 2); break;
                case 4: TERN_PACK_LAUNCH(4, 4); break;
                case 8: TERN_PACK_LAUNCH(4, 8); break;
                default: TERN_PACK_LAUNCH(4, 0); break;
            }
        }
    } else {
        TERN_PACK_LAUNCH(1, 0);
    }
#undef TERN_PACK_LAUNCH
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}

}  // namespace

int launch_pack_i8(const int8_t* src, tern_dims dims, uint32_t* dst, hipStream_t s)
{
    return launch_pack_any<int8_t, 0>(src, dims, nullptr, nullptr, dst, s);
}

int launch_threshold_pack_i32(const int32_t* src, tern_dims dims, const int32_t* lo,
                              const int32_t* hi, uint32_t* dst, hipStream_t s)
{
    return launch_pack_any<int32_t, 1>(src, dims, lo, hi, dst, s);
}

int launch_threshold_pack_f32(const float* src, tern_dims dims, const float* lo, const float* hi,
                              uint32_t* dst, hipStream_t s)
{
    return launch_pack_any<float, 1>(src, dims, lo, hi, dst, s);
}

// ---- first layer of a network on a scalar volume: gather the kernel taps into one word ----------
// With one input channel a packed voxel carries a single live bit per plane, and a convolution
// would have to collect its T <= 32 taps bit by bit for every output voxel and channel slice.
// This kernel does that collecting once, straight from the float intensities (applying the
// activation cut points on the way): output voxel o gets a mask string and a sign string whose
// bit t is the code of tap t = (a*kh + b)*kw + c of o's receptive field (0 outside the volume).
// The convolution then is a single-tap one over T "channels", and the tap-packed filter bank
// (bit t of its one word per channel = tap t) is exactly that convolution's plain bank.
// A thread owns one (ox, oy) column and kPatchZ consecutive output planes; with unit depth stride
// and dilation these share input planes, so kPatchZ + KD - 1 plane parts serve kPatchZ outputs.
// Instantiated for the usual first kernels, 3x3x3 and 1x3x3, and for the 15x3x3 stack kernel of
// Table 1, whose 135 taps make a five-word string (any in-plane stride, dilation, pad).
namespace {

// PZ = output planes per thread, WDP = words per plane of the gathered tap string.
// Tap strings of output voxels (ox, oy, oz0 .. oz0+PZ-1) of batch item n: wm[t][q], ws[t][q].
template <int KD, int KH, int KW, int PZ>
__device__ __forceinline__ void gather_taps(const PatchParams& p, int n, int ox, int oy, int oz0,
                                            uint32_t (&wm)[PZ][(KD * KH * KW + 31) / 32],
                                            uint32_t (&ws)[PZ][(KD * KH * KW + 31) / 32])
{
    constexpr int NB = KH * KW;   // taps per input plane
    constexpr int WDP = (KD * NB + 31) / 32;
    const float lo = p.lo[0], hi = p.hi[0];
    const float* src_n = p.src + (size_t)n * p.d * p.h * p.w;
    const size_t plane = (size_t)p.h * p.w;

    // In-plane offsets of this column's taps, fixed for the whole walk; taps outside the plane
    // read element 0 and are masked out afterwards, so every load is unconditional.
    int off[NB];
    uint32_t valid = 0u;
#pragma unroll
    for (int b = 0; b < KH; ++b)
#pragma unroll
        for (int c = 0; c < KW; ++c) {
            const int iy = oy * p.sh - p.ph + b * p.dh;
            const int ix = ox * p.sw - p.pw + c * p.dw;
            const bool ok = iy >= 0 && iy < p.h && ix >= 0 && ix < p.w;
            off[b * KW + c] = ok ? iy * p.w + ix : 0;
            valid |= (ok ? 1u : 0u) << (b * KW + c);
        }

    // All input planes this thread needs, fetched before any of them is used: one memory round
    // trip for the whole walk.  Planes outside the volume read plane 0 and are masked out.
    constexpr int NP = PZ + KD - 1;
    float v[NP][NB];
#pragma unroll
    for (int j = 0; j < NP; ++j) {
        const int iz = oz0 - p.pd + j;
        const float* pl = src_n + (size_t)((iz >= 0 && iz < p.d) ? iz : 0) * plane;
#pragma unroll
        for (int i = 0; i < NB; ++i) v[j][i] = pl[off[i]];
    }
    // codes of the in-plane taps of every fetched plane, tap (b, c) at bit b*KW + c
    uint32_t m[NP], s[NP];
#pragma unroll
    for (int j = 0; j < NP; ++j) {
        const int iz = oz0 - p.pd + j;
        uint32_t P = 0u, N = 0u;
#pragma unroll
        for (int i = NB - 1; i >= 0; --i) {
            // P = 2P + (hi < v), N = 2N + (v < lo): the comparison result travels through the
            // carry flag into the low bit (ordered comparisons: false for NaN, like the C ones)
            asm("v_cmp_lt_f32 vcc, %2, %1\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc"
                : "+v"(P) : "v"(v[j][i]), "s"(hi) : "vcc");
            asm("v_cmp_gt_f32 vcc, %2, %1\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc"
                : "+v"(N) : "v"(v[j][i]), "s"(lo) : "vcc");
        }
        const uint32_t vm = (iz >= 0 && iz < p.d) ? valid : 0u;
        P &= vm;
        N &= vm & ~P;          // +1 wins should the cut points be crossed (lo > hi)
        m[j] = P | N;
        s[j] = N;
    }
#pragma unroll
    for (int t = 0; t < PZ; ++t) {
        // plane a of the kernel occupies bits [a*NB, a*NB + NB) of the tap string
#pragma unroll
        for (int q = 0; q < WDP; ++q) wm[t][q] = ws[t][q] = 0u;
#pragma unroll
        for (int a = 0; a < KD; ++a) {
            constexpr int kNB = NB;
            const int word = (a * kNB) / 32, sh = (a * kNB) % 32;
            wm[t][word] |= m[t + a] << sh;
            ws[t][word] |= s[t + a] << sh;
            if (sh + kNB > 32) {
                wm[t][word + 1] |= m[t + a] >> (32 - sh);
                ws[t][word + 1] |= s[t + a] >> (32 - sh);
            }
        }
    }
}

template <int KD, int KH, int KW, int PZ>
__global__ __launch_bounds__(256) void patch_pack_f32_kernel(PatchParams p)
{
    constexpr int WDP = (KD * KH * KW + 31) / 32;
    const int ox = blockIdx.x * 64 + threadIdx.x;
    const int oy = blockIdx.y * 4 + threadIdx.y;
    const int nseg = (p.od + PZ - 1) / PZ;
    const int seg = blockIdx.z % nseg;
    const int n = blockIdx.z / nseg;
    if (ox >= p.ow || oy >= p.oh) return;
    const int oz0 = seg * PZ;
    uint32_t wm[PZ][WDP], ws[PZ][WDP];
    gather_taps<KD, KH, KW, PZ>(p, n, ox, oy, oz0, wm, ws);
    uint32_t* out = p.dst + ((((size_t)n * p.od + oz0) * p.oh + oy) * p.ow + ox) * 2u * WDP;
    const size_t ostep = (size_t)p.oh * p.ow * 2u * WDP;
#pragma unroll
    for (int t = 0; t < PZ; ++t) {
        if (oz0 + t >= p.od) break;
        uint32_t* o = out + (size_t)t * ostep;
        if constexpr (WDP == 1) {
            *reinterpret_cast<uint2*>(o) = make_uint2(wm[t][0], ws[t][0]);
        } else {
#pragma unroll
            for (int q = 0; q < WDP; ++q) { o[q] = wm[t][q]; o[WDP + q] = ws[t][q]; }
        }
    }
}

// The same gathering with layer 0's convolution behind it: the tap strings stay in registers and
// go straight through the word-pair sequence of the convolution kernels (Eq. 9 over the T
// gathered "channels"), the cut points of layer 0's activation (Eq. 6) and the re-packing, so
// that neither the ternarised input nor the tap strings ever reach memory.  Filter bank: the
// single-tap bank over T channels [WDP][co_pad][2][1], which is the tap-packed bank of the
// original kernel word for word.  VH voxels of a thread are convolved together (4 of the 8 planes
// of a column, or the single one).
template <int KD, int KH, int KW, int PZ>
__global__ __launch_bounds__(256) void patch_conv_f32_kernel(PatchParams p, FirstConvParams c)
{
    constexpr int WDP = (KD * KH * KW + 31) / 32;
    constexpr int VH = PZ >= 4 ? 4 : 1;
    constexpr int CO_BLK = 16;
    constexpr int KG = GroupOf<CO_BLK>::value;
    constexpr int NG = CO_BLK / KG;
    static_assert(PZ % VH == 0, "whole groups of voxels");
    const int ox = blockIdx.x * 64 + threadIdx.x;
    const int oy = blockIdx.y * 4 + threadIdx.y;
    const int nseg = (p.od + PZ - 1) / PZ;
    const int seg = blockIdx.z % nseg;
    const int n = blockIdx.z / nseg;
    if (ox >= p.ow || oy >= p.oh) return;   // (no cross-lane operation below)
    const int oz0 = seg * PZ;
    uint32_t wm[PZ][WDP], ws[PZ][WDP];
    gather_taps<KD, KH, KW, PZ>(p, n, ox, oy, oz0, wm, ws);

    const int step_words = c.co_pad * 2;   // filter-bank words per gathered word
    const size_t ostep = (size_t)p.oh * p.ow * 2u * c.wd_out;
    uint32_t* out = c.out_packed + ((((size_t)n * p.od + oz0) * p.oh + oy) * p.ow + ox) * 2u * c.wd_out;
#pragma unroll
    for (int h = 0; h < PZ / VH; ++h) {
        ActChunk<1> A[WDP][VH];
#pragma unroll
        for (int q = 0; q < WDP; ++q)
#pragma unroll
            for (int v = 0; v < VH; ++v) { A[q][v].m[0] = wm[h * VH + v][q]; A[q][v].s[0] = ws[h * VH + v][q]; }
        uint32_t pos_w[VH], neg_w[VH];
#pragma unroll
        for (int v = 0; v < VH; ++v) pos_w[v] = neg_w[v] = 0u;
        for (int cb = 0; cb < c.c_out; cb += CO_BLK) {
            int32_t acc_m[VH][CO_BLK], acc_n[VH][CO_BLK];   // set by the first word
            scalar_ptr wbase = (scalar_ptr)(uintptr_t)c.wgt + (size_t)cb * 2;
            WGroup<1, KG> g[2];
            load_wgroup<1, KG>(g[0], wbase);
            auto group_step = [&](int idx, auto init) {
                const int q = idx / NG, gi = idx % NG;
                settle<1, KG>(g[idx & 1]);
                __builtin_amdgcn_sched_barrier(0);
                if (idx + 1 < WDP * NG) {
                    const int nq = (idx + 1) / NG, ngi = (idx + 1) % NG;
                    load_wgroup<1, KG>(g[(idx + 1) & 1], wbase + (size_t)nq * step_words + ngi * KG * 2);
                }
                __builtin_amdgcn_sched_barrier(0);
                mac_group<1, VH, CO_BLK, KG, decltype(init)::value>(A[q], g[idx & 1], gi * KG, acc_m, acc_n);
                __builtin_amdgcn_sched_barrier(0);
            };
#pragma unroll
            for (int idx = 0; idx < NG; ++idx) group_step(idx, std::true_type{});
#pragma unroll
            for (int idx = NG; idx < WDP * NG; ++idx) group_step(idx, std::false_type{});

            int32_t d[VH][CO_BLK];
#pragma unroll
            for (int v = 0; v < VH; ++v)
#pragma unroll
                for (int j = 0; j < CO_BLK; ++j) d[v][j] = acc_m[v][j] - 2 * acc_n[v][j];
            uint32_t pp[VH], pn[VH];
            ternarise_pass<VH, CO_BLK>(d, (scalar_ptr)(uintptr_t)c.lo, (scalar_ptr)(uintptr_t)c.hi, cb,
                                       c.c_out - cb, c.c_out, pp, pn);
            const int sh = cb & 31;
#pragma unroll
            for (int v = 0; v < VH; ++v) { pos_w[v] |= pp[v] << sh; neg_w[v] |= pn[v] << sh; }
            if (((cb + CO_BLK) & 31) == 0 || cb + CO_BLK >= c.c_out) {
                const int q = cb >> 5;
#pragma unroll
                for (int v = 0; v < VH; ++v) {
                    const int t = h * VH + v;
                    if (oz0 + t < p.od) {
                        uint32_t* o = out + (size_t)t * ostep;
                        o[q] = pos_w[v] | neg_w[v];
                        o[c.wd_out + q] = neg_w[v] & ~pos_w[v];    // +1 wins if lo > hi
                    }
                    pos_w[v] = neg_w[v] = 0u;
                }
            }
        }
    }
}

// Kernel extents the gathering kernel is instantiated for -> output planes per thread (0: none).
// 15x3x3 is the stack-of-slices first layer of Table 1 (its output has a single plane).
inline int patch_planes_per_thread(int kd, int kh, int kw)
{
    if (kh != 3 || kw != 3) return 0;
    if (kd == 3 || kd == 1) return 8;
    if (kd == 15) return 1;
    return 0;
}

}  // namespace

bool patch_pack_applies(int32_t c_in, const tern_conv_geom& g, const tern_dims& out)
{
    const int pz = patch_planes_per_thread(g.k[0], g.k[1], g.k[2]);
    if (!(c_in == 1 && pz > 0 && g.stride[0] == 1 && g.dil[0] == 1)) return false;
    // launch grid limits of the gathering kernel
    const int64_t nseg = (out.d + pz - 1) / pz;
    return nseg * out.n <= 65535 && (out.h + 3) / 4 <= 65535;
}

int launch_patch_pack_f32(const PatchParams& p, int32_t n, hipStream_t s)
{
    const int pz = patch_planes_per_thread(p.kd, p.kh, p.kw);
    if (pz == 0) return TERN_EARG;
    const int nseg = (p.od + pz - 1) / pz;
    const dim3 grid((unsigned)((p.ow + 63) / 64), (unsigned)((p.oh + 3) / 4), (unsigned)(nseg * n)), block(64, 4);
    if (p.kd == 3)
        hipLaunchKernelGGL((patch_pack_f32_kernel<3, 3, 3, 8>), grid, block, 0, s, p);
    else if (p.kd == 1)
        hipLaunchKernelGGL((patch_pack_f32_kernel<1, 3, 3, 8>), grid, block, 0, s, p);
    else
        hipLaunchKernelGGL((patch_pack_f32_kernel<15, 3, 3, 1>), grid, block, 0, s, p);
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}

// Whether layer 0 should run behind the gathering in one kernel.  The 15x3x3 variant holds 135
// intensities per lane and fits only two waves per SIMD: good for one stack of slices (one launch
// instead of two latency-bound ones), slower than gathering and convolving separately for many.
bool patch_conv_pays(const PatchParams& p, int32_t n)
{
    if (p.kd != 15) return true;
    return (int64_t)n * p.od * p.oh * p.ow <= 131072;
}

int launch_patch_conv_f32(const PatchParams& p, const FirstConvParams& c, int32_t n, hipStream_t s)
{
    const int pz = patch_planes_per_thread(p.kd, p.kh, p.kw);
    if (pz == 0) return TERN_EARG;
    const int nseg = (p.od + pz - 1) / pz;
    const dim3 grid((unsigned)((p.ow + 63) / 64), (unsigned)((p.oh + 3) / 4), (unsigned)(nseg * n)), block(64, 4);
    if (p.kd == 3)
        hipLaunchKernelGGL((patch_conv_f32_kernel<3, 3, 3, 8>), grid, block, 0, s, p, c);
    else if (p.kd == 1)
        hipLaunchKernelGGL((patch_conv_f32_kernel<1, 3, 3, 8>), grid, block, 0, s, p, c);
    else
        hipLaunchKernelGGL((patch_conv_f32_kernel<15, 3, 3, 1>), grid, block, 0, s, p, c);
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}

// ---- filter bank ------------------------------------------------------------------------------
// Layout consumed by the convolution kernels (documented in include/tern.h).
// Plain: uint32 [T * nchunk][co_pad][2][wc]; step s = tap * nchunk + chunk holds, for every
// channel, wc mask words then wc sign words of input-channel words [chunk*wc, chunk*wc + wc).
// Tap-packed (C_in <= 16, T > 1): uint32 [ceil(T / slots)][co_pad][2][1]; the word of step s
// carries taps s*slots .. s*slots + slots - 1, tap i of the step in bits [i*shift, i*shift + C_in).
namespace {

__global__ __launch_bounds__(256) void pack_filters_kernel(const int8_t* __restrict__ w,
                                                           uint32_t* __restrict__ bank, int c_out,
                                                           int c_in, int T, BankShape b, int co_pad,
                                                           int64_t total)
{
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= total) return;
    // one thread per (step, channel, word-in-chunk)
    int64_t r = gid;
    const int q = (int)(r % b.wc); r /= b.wc;
    const int co = (int)(r % co_pad); r /= co_pad;
    const int step = (int)r;
    uint32_t m = 0u, s = 0u;
    if (co < c_out) {
        if (b.tp_slots) {
            for (int i = 0; i < b.tp_slots; ++i) {
                const int tap = step * b.tp_slots + i;
                if (tap >= T) break;
                for (int ci = 0; ci < c_in; ++ci) {
                    const int8_t v = w[((size_t)co * c_in + ci) * T + tap];
                    m |= (v != 0 ? 1u : 0u) << (i * b.tp_shift + ci);
                    s |= (v < 0 ? 1u : 0u) << (i * b.tp_shift + ci);
                }
            }
        } else {
            const int tap = step / b.nchunk, chunk = step - tap * b.nchunk;
            const int word = chunk * b.wc + q;
            for (int j = 0; j < 32; ++j) {
                const int ci = 32 * word + j;
                if (ci >= c_in) break;
                const int8_t v = w[((size_t)co * c_in + ci) * T + tap];
                m |= (v != 0 ? 1u : 0u) << j;
                s |= (v < 0 ? 1u : 0u) << j;
            }
        }
    }
    uint32_t* o = bank + ((size_t)step * co_pad + co) * 2u * b.wc;
    o[q] = m;
    o[b.wc + q] = s;
}

}  // namespace

// Binary filter bank (weights in {-1, +1}, Eq. 8): uint32 [T*nchunk][co_pad][wc] sign words, plain
// layout whatever C_in is; bit j of a word is set where the weight is negative.
namespace {
__global__ __launch_bounds__(256) void pack_filters_binary_kernel(const int8_t* __restrict__ w,
                                                                  uint32_t* __restrict__ bank, int c_out, int c_in,
                                                                  int T, int wc, int nchunk, int co_pad, int64_t total)
{
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= total) return;
    int64_t r = gid;
    const int q = (int)(r % wc); r /= wc;
    const int co = (int)(r % co_pad); r /= co_pad;
    const int step = (int)r;
    uint32_t s = 0u;
    if (co < c_out) {
        const int tap = step / nchunk, chunk = step - tap * nchunk;
        const int word = chunk * wc + q;
        for (int j = 0; j < 32; ++j) {
            const int ci = 32 * word + j;
            if (ci >= c_in) break;
            s |= (w[((size_t)co * c_in + ci) * T + tap] < 0 ? 1u : 0u) << j;
        }
    }
    bank[gid] = s;
}
}  // namespace

int launch_pack_filters_binary(const int8_t* w, int32_t c_out, int32_t c_in, int32_t kd, int32_t kh,
                               int32_t kw, uint32_t* bank, hipStream_t s)
{
    const int T = kd * kh * kw;
    const int wd = (c_in + 31) / 32, wc = (wd % 2 == 0) ? 2 : 1, nchunk = wd / wc;
    const int co_pad = (c_out + 31) / 32 * 32;
    const int64_t total = (int64_t)T * nchunk * co_pad * wc;
    const int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffff) return TERN_ESHAPE;
    hipLaunchKernelGGL(pack_filters_binary_kernel, dim3((unsigned)blocks), dim3(256), 0, s, w, bank, c_out, c_in,
                       T, wc, nchunk, co_pad, total);
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}

int launch_pack_filters(const int8_t* w, int32_t c_out, int32_t c_in, int32_t kd, int32_t kh,
                        int32_t kw, uint32_t* bank, hipStream_t s)
{
    const int T = kd * kh * kw;
    const BankShape b = bank_shape(c_in, T);
    const int co_pad = (c_out + 31) / 32 * 32;
    const int64_t total = (int64_t)b.nsteps * co_pad * b.wc;
    const int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffff) return TERN_ESHAPE;
    hipLaunchKernelGGL(pack_filters_kernel, dim3((unsigned)blocks), dim3(256), 0, s, w, bank, c_out,
                       c_in, T, b, co_pad, total);
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}

}  // namespace tern
