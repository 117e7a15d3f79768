// Pointwise ternary convolution for gfx950: a 1x1x1 kernel with unit stride and no padding
// (paper section 2, Eq. 9; the 1x1 rows of Table 1; also the second half of a one-channel first
// layer whose taps were gathered into one word per voxel).
//
// An output voxel depends on one input voxel only, so there is no halo and nothing to share:
// the volume is a flat list of voxels, a lane owns V of them (64 apart, so that a wave's loads
// and stores are contiguous runs), reads their packed words from global memory once into
// registers, and then walks the output channels CO_BLK at a time with the filter words coming
// through the scalar cache -- the same four vector instructions per word pair and the same
// epilogue as the tiled kernel, without its LDS tile, barrier and tap walk, whose fixed cost per
// wave would dominate here (a single-tap wave has only a few hundred instructions of real work).
#include <type_traits>

#include "tern_conv_common.h"
#include "tern_internal.h"

namespace tern {
namespace {

constexpr int kPointThreads = 256;

struct PointParams {
    const uint32_t* in;      // packed [voxels][2][WC*NCH] (batch items folded for packed output)
    const uint32_t* wgt;     // filter bank [NCH][co_pad][2][WC]
    const int32_t* lo;
    const int32_t* hi;
    int32_t* out_acc;        // [n][c_out][voxels] or null
    uint32_t* out_packed;    // [voxels][2][wd_out] or null
    int64_t voxels;          // per grid.z slice
    int32_t c_out, wd_out, co_pad;
    int32_t co_per_wave;     // multiple of 32 (or everything)
};

template <int WC, int NCH, int V, int CO_BLK, bool PACKED>
__global__ __launch_bounds__(kPointThreads) void conv_point_kernel(PointParams p)
{
    constexpr int WD = WC * NCH;
    constexpr int KG = GroupOf<CO_BLK>::value;
    constexpr int NG = CO_BLK / KG;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t wid = (int64_t)blockIdx.x * (kPointThreads / 64) + wave;
    const int64_t v0 = wid * (64 * V) + lane;           // this lane's first voxel
    if (wid * (64 * V) >= p.voxels) return;             // whole wave past the end
    const int n = blockIdx.z;
    const uint32_t* in_n = p.in + (size_t)n * p.voxels * 2u * WD;

    // ---- this lane's voxels, all chunks, straight into registers -----------------------------
    ActChunk<WC> A[NCH][V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int64_t vox = v0 + 64 * v;
        const bool live = vox < p.voxels;
        const uint32_t* src = in_n + (size_t)(live ? vox : 0) * 2u * WD;
        if constexpr (WD == 1) {
            uint2 r = *reinterpret_cast<const uint2*>(src);
            A[0][v].m[0] = live ? r.x : 0u;
            A[0][v].s[0] = live ? r.y : 0u;
        } else if constexpr (WC == 1) {   // odd word counts: records are only 8-byte aligned
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                const uint32_t m = src[ch], sg = src[WD + ch];
                A[ch][v].m[0] = live ? m : 0u;
                A[ch][v].s[0] = live ? sg : 0u;
            }
        } else {
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                const uint2 m = *reinterpret_cast<const uint2*>(src + 2 * ch);
                const uint2 sg = *reinterpret_cast<const uint2*>(src + WD + 2 * ch);
                A[ch][v].m[0] = live ? m.x : 0u; A[ch][v].m[1] = live ? m.y : 0u;
                A[ch][v].s[0] = live ? sg.x : 0u; A[ch][v].s[1] = live ? sg.y : 0u;
            }
        }
    }

    const int co_begin = blockIdx.y * p.co_per_wave;
    const int co_end = min(p.c_out, co_begin + p.co_per_wave);
    const int step_words = p.co_pad * 2 * WC;            // filter-bank words per chunk
    uint32_t pos_w[V], neg_w[V];
#pragma unroll
    for (int v = 0; v < V; ++v) pos_w[v] = neg_w[v] = 0u;

    for (int cb = co_begin; cb < co_end; cb += CO_BLK) {
        int32_t acc_m[V][CO_BLK], acc_n[V][CO_BLK];   // set by the first chunk, added to by the rest

        // (chunk, channel group) pairs in order, two filter-word groups in flight
        scalar_ptr wbase = (scalar_ptr)(uintptr_t)p.wgt + (size_t)cb * 2 * WC;
        WGroup<WC, KG> g[2];
        load_wgroup<WC, KG>(g[0], wbase);
        auto group_step = [&](int idx, auto init) {
            const int ch = idx / NG, gi = idx % NG;
            settle<WC, KG>(g[idx & 1]);
            __builtin_amdgcn_sched_barrier(0);
            if (idx + 1 < NCH * NG) {
                const int nch = (idx + 1) / NG, ngi = (idx + 1) % NG;
                load_wgroup<WC, KG>(g[(idx + 1) & 1], wbase + (size_t)nch * step_words + ngi * KG * 2 * WC);
            }
            __builtin_amdgcn_sched_barrier(0);
            mac_group<WC, V, CO_BLK, KG, decltype(init)::value>(A[ch], g[idx & 1], gi * KG, acc_m, acc_n);
            __builtin_amdgcn_sched_barrier(0);
        };
#pragma unroll
        for (int idx = 0; idx < NG; ++idx) group_step(idx, std::true_type{});
#pragma unroll
        for (int idx = NG; idx < NCH * NG; ++idx) group_step(idx, std::false_type{});

        int32_t d[V][CO_BLK];
#pragma unroll
        for (int v = 0; v < V; ++v)
#pragma unroll
            for (int j = 0; j < CO_BLK; ++j) d[v][j] = acc_m[v][j] - 2 * acc_n[v][j];

        const int co_left = co_end - cb;
        if constexpr (PACKED) {
            uint32_t pp[V], pn[V];
            ternarise_pass<V, CO_BLK>(d, (scalar_ptr)(uintptr_t)p.lo, (scalar_ptr)(uintptr_t)p.hi, cb,
                                      co_left, p.c_out, pp, pn);
            const int sh = cb & 31;
#pragma unroll
            for (int v = 0; v < V; ++v) { pos_w[v] |= pp[v] << sh; neg_w[v] |= pn[v] << sh; }
            // a wave's channel slice starts at a multiple of 32, so it always owns whole words
            if (((cb + CO_BLK) & 31) == 0 || cb + CO_BLK >= co_end) {
                const int q = cb >> 5;
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    const int64_t vox = v0 + 64 * v;
                    if (vox < p.voxels) {
                        uint32_t* o = p.out_packed + (size_t)vox * 2u * p.wd_out;
                        o[q] = pos_w[v] | neg_w[v];
                        o[p.wd_out + q] = neg_w[v] & ~pos_w[v];    // +1 wins if lo > hi
                    }
                    pos_w[v] = neg_w[v] = 0u;
                }
            }
        } else {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const int64_t vox = v0 + 64 * v;
                if (vox < p.voxels) {
                    int32_t* o = p.out_acc + (size_t)n * p.c_out * p.voxels + vox;
#pragma unroll
                    for (int j = 0; j < CO_BLK; ++j)
                        if (j < co_left) o[(size_t)(cb + j) * p.voxels] = d[v][j];
                }
            }
        }
    }
}

}  // namespace

bool conv_point_applies(const ConvParams& p)
{
    if (p.kd * p.kh * p.kw != 1) return false;
    if (p.sd != 1 || p.sh != 1 || p.sw != 1 || p.pd != 0 || p.ph != 0 || p.pw != 0) return false;
    if (p.tp_slots != 0) return false;
    return p.wd_in == 1 || p.wd_in == 2 || p.wd_in == 3 || p.wd_in == 4 || p.wd_in == 5 || p.wd_in == 8;
}

int launch_conv_point(const ConvParams& c, hipStream_t s)
{
    const bool packed = c.out_packed != nullptr;
    PointParams p;
    p.in = c.in; p.wgt = c.wgt; p.lo = c.lo; p.hi = c.hi;
    p.out_acc = c.out_acc; p.out_packed = c.out_packed;
    // packed output: batch items are just more voxels; int32 output keeps them apart (grid.z)
    const int64_t spatial = (int64_t)c.d * c.h * c.w;
    p.voxels = packed ? spatial * c.n : spatial;
    const int gz = packed ? 1 : c.n;
    if (gz > 65535) return TERN_ESHAPE;
    p.c_out = c.c_out; p.wd_out = c.wd_out; p.co_pad = c.co_pad;

    constexpr int V = 2;
    const int64_t waves0 = (p.voxels + 64 * V - 1) / (64 * V) * gz;
    // 32 channels per pass on large problems (half the passes), 16 on small ones or when the
    // last pass would be mostly padding
    const int tail = c.c_out % 32;
    const int co_blk = (waves0 * ((c.c_out + 31) / 32) >= 4096 && (tail == 0 || tail > 16)) ? 32 : 16;
    // One wave walks all output channels (its voxels are read once) unless that leaves the chip
    // short of waves; slices are whole 32-channel words.
    const int words = (c.c_out + 31) / 32;
    int slices = 1;
    if (waves0 < 2048) {
        slices = (int)((2048 + waves0 - 1) / waves0);
        if (slices > words) slices = words;
    }
    const int words_per_slice = (words + slices - 1) / slices;
    slices = (words + words_per_slice - 1) / words_per_slice;
    p.co_per_wave = words_per_slice * 32;

    const int64_t blocks = (waves0 / gz + kPointThreads / 64 - 1) / (kPointThreads / 64);
    if (blocks > 0x7fffffff || slices > 65535) return TERN_ESHAPE;
    const dim3 grid((unsigned)blocks, (unsigned)slices, (unsigned)gz), block(kPointThreads);
#define TERN_POINT(WC_, NCH_, CB_)                                                                        \
    do {                                                                                                  \
        if (packed) hipLaunchKernelGGL((conv_point_kernel<WC_, NCH_, V, CB_, true>), grid, block, 0, s, p); \
        else hipLaunchKernelGGL((conv_point_kernel<WC_, NCH_, V, CB_, false>), grid, block, 0, s, p);       \
    } while (0)
    switch (c.wd_in) {
        case 1: if (co_blk == 32) TERN_POINT(1, 1, 32); else TERN_POINT(1, 1, 16); break;
        case 2: if (co_blk == 32) TERN_POINT(2, 1, 32); else TERN_POINT(2, 1, 16); break;
        case 3: if (co_blk == 32) TERN_POINT(1, 3, 32); else TERN_POINT(1, 3, 16); break;
        case 4: if (co_blk == 32) TERN_POINT(2, 2, 32); else TERN_POINT(2, 2, 16); break;
        case 5: if (co_blk == 32) TERN_POINT(1, 5, 32); else TERN_POINT(1, 5, 16); break;
        case 8: if (co_blk == 32) TERN_POINT(2, 4, 32); else TERN_POINT(2, 4, 16); break;
        default: return TERN_EARG;
    }
#undef TERN_POINT
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}

}  // namespace tern
