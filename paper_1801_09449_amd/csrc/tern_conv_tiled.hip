// Tiled ternary 3D convolution for gfx950 (paper section 2, Eq. 9, evaluated as
// popcount(M) - 2*popcount(M & X) with M = mask_w & mask_a, X = sign_w ^ sign_a).
//
// Mapping
//   - A wave owns an 8 (x) by 8 (y) patch of output voxels, V voxels deep in z per lane; a
//     workgroup is an nwx * nwy * nwz arrangement of such waves and shares one LDS halo tile of
//     the packed input (out-of-volume voxels are stored as zero words = ternary 0).
//   - Output channels are processed CO_BLK at a time.  The two running bit counts of every
//     (voxel, channel) pair live in VGPRs: 2 * V * CO_BLK accumulators.
//   - Filter words are wave-uniform: they are fetched through the scalar cache into SGPRs and
//     used directly as VALU operands, so one word pair costs four VALU instructions per lane
//     (and, popcount-accumulate, and-xor as one three-input bit operation, popcount-accumulate).
//   - Input channels are walked in chunks of WC words per plane; LDS holds each voxel
//     chunk-interleaved ([chunk][WC mask words][WC sign words]) so that a lane fetches one chunk
//     with a single 8- or 16-byte LDS read.
//   - Epilogue: acc = M-count - 2 * N-count; either stored as int32 (NCDHW) or compared with the
//     per-channel cut points (Eq. 6 in integer form) and assembled into mask/sign words in-lane,
//     so that activations go back to memory at 2 bits per value.
#include "tern_internal.h"

namespace tern {

int launch_conv3d_generic(const ConvParams& p, hipStream_t s);

namespace {

constexpr int kMaxThreads = 512;         // 8 waves: at most 2 waves per SIMD, <= 256 VGPRs
constexpr int kLdsLimit = 160 * 1024;    // LDS per compute unit / per workgroup on gfx950

// Largest dynamic LDS allocation the current device grants one workgroup (queried once per
// device; 0 on error).
int lds_limit_for_current_device()
{
    static int cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (cached[dev] == 0) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess)
            return 0;
        cached[dev] = v < kLdsLimit ? v : kLdsLimit;
    }
    return cached[dev];
}

struct TileParams {
    int32_t nwx, nwy, nwz;        // waves per workgroup along x, y, z
    int32_t hx, hy, hz;           // halo tile extents in voxels
    int32_t tiles_x, tiles_y, tiles_z;
    int32_t vstride;              // LDS words per voxel (2*Wd plus padding)
    int32_t nchunk;               // Wd / WC
    int32_t co_per_wg;            // output channels handled by one workgroup (blockIdx.y)
};

template <int WC>
struct ActChunk {
    uint32_t m[WC];
    uint32_t s[WC];
};

template <int WC>
__device__ __forceinline__ ActChunk<WC> lds_read_chunk(const uint32_t* p)
{
    ActChunk<WC> a;
    if constexpr (WC == 1) {
        const uint2 r = *reinterpret_cast<const uint2*>(p);
        a.m[0] = r.x; a.s[0] = r.y;
    } else {
        static_assert(WC == 2, "WC must be 1 or 2");
        const uint4 r = *reinterpret_cast<const uint4*>(p);
        a.m[0] = r.x; a.m[1] = r.y; a.s[0] = r.z; a.s[1] = r.w;
    }
    return a;
}

// Filter words are read through the constant address space so that the wave-uniform loads go
// through the scalar cache (s_load) into SGPRs; the filter bank is never written by these
// kernels.
typedef const uint32_t __attribute__((address_space(4)))* scalar_ptr;

// acc += popcount(x) as the single instruction the hardware has for it.
__device__ __forceinline__ void popc_acc(int32_t& acc, uint32_t x)
{
    asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(x));
}

constexpr int kGroup = 8;  // output channels whose filter words are fetched together

template <int WC>
struct WGroup {
    uint32_t m[kGroup][WC];
    uint32_t s[kGroup][WC];
};

// Fetch the filter words of kGroup consecutive channels of one step.  In the filter bank the
// channels of a step are contiguous (2*WC words each), so this is one contiguous block that
// the compiler turns into wide scalar loads with immediate offsets.
template <int WC>
__device__ __forceinline__ void load_wgroup(WGroup<WC>& g, scalar_ptr wp)
{
#pragma unroll
    for (int j = 0; j < kGroup; ++j)
#pragma unroll
        for (int q = 0; q < WC; ++q) {
            g.m[j][q] = wp[j * 2 * WC + q];
            g.s[j][q] = wp[j * 2 * WC + WC + q];
        }
}

// Scalar loads return out of order, so the only safe wait is "all of them".  Naming the group's
// registers here makes the compiler place that wait at this point, i.e. before the loads of the
// following group are issued, so that those overlap the arithmetic on this group instead of
// being waited for together with it.
template <int WC>
__device__ __forceinline__ void settle(const WGroup<WC>& g)
{
#pragma unroll
    for (int j = 0; j < kGroup; j += 4) {
        if constexpr (WC == 2) {
            asm volatile("" ::"s"(g.m[j][0]), "s"(g.m[j][1]), "s"(g.s[j][0]), "s"(g.s[j][1]),
                         "s"(g.m[j + 1][0]), "s"(g.m[j + 1][1]), "s"(g.s[j + 1][0]), "s"(g.s[j + 1][1]),
                         "s"(g.m[j + 2][0]), "s"(g.m[j + 2][1]), "s"(g.s[j + 2][0]), "s"(g.s[j + 2][1]),
                         "s"(g.m[j + 3][0]), "s"(g.m[j + 3][1]), "s"(g.s[j + 3][0]), "s"(g.s[j + 3][1]));
        } else {
            asm volatile("" ::"s"(g.m[j][0]), "s"(g.s[j][0]), "s"(g.m[j + 1][0]), "s"(g.s[j + 1][0]),
                         "s"(g.m[j + 2][0]), "s"(g.s[j + 2][0]), "s"(g.m[j + 3][0]), "s"(g.s[j + 3][0]));
        }
    }
}

// Four VALU instructions per (word pair, voxel): and, popcount-accumulate, and-xor,
// popcount-accumulate (Eq. 9 as popcount(M) - 2 popcount(M & X), the subtraction deferred).
template <int WC, int V, int CO_BLK>
__device__ __forceinline__ void mac_group(const ActChunk<WC> (&A)[V], const WGroup<WC>& g, int j0,
                                          int32_t (&acc_m)[V][CO_BLK], int32_t (&acc_n)[V][CO_BLK])
{
#pragma unroll
    for (int j = 0; j < kGroup; ++j)
#pragma unroll
        for (int q = 0; q < WC; ++q)
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const uint32_t M = A[v].m[q] & g.m[j][q];
                const uint32_t N = M & (A[v].s[q] ^ g.s[j][q]);
                popc_acc(acc_m[v][j0 + j], M);
                popc_acc(acc_n[v][j0 + j], N);
            }
}

template <int WC, int V, int CO_BLK, bool PACKED>
__global__ __launch_bounds__(kMaxThreads) void conv_tiled_kernel(ConvParams p, TileParams t)
{
    extern __shared__ __align__(16) uint32_t lds[];

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- which tile ------------------------------------------------------------------------
    int bid = blockIdx.x;
    const int tix = bid % t.tiles_x; bid /= t.tiles_x;
    const int tiy = bid % t.tiles_y; bid /= t.tiles_y;
    const int tiz = bid % t.tiles_z;
    const int n = bid / t.tiles_z;
    const int TX = 8 * t.nwx, TY = 8 * t.nwy, TZ = V * t.nwz;
    const int ox0 = tix * TX, oy0 = tiy * TY, oz0 = tiz * TZ;

    // ---- stage the halo tile -------------------------------------------------------------
    {
        const int gx0 = ox0 * p.sw - p.pw, gy0 = oy0 * p.sh - p.ph, gz0 = oz0 * p.sd - p.pd;
        const int plane = t.hy * t.hx;
        const int wd = p.wd_in;
        const uint32_t* in_n = p.in + (size_t)n * p.d * p.h * p.w * 2u * wd;
        for (int hz = 0; hz < t.hz; ++hz) {
            const int gz = gz0 + hz;
            const bool zin = gz >= 0 && gz < p.d;
            for (int i = tid; i < plane; i += nthreads) {
                const int hy = i / t.hx;
                const int hxx = i - hy * t.hx;
                const int gy = gy0 + hy, gx = gx0 + hxx;
                const bool inb = zin && gy >= 0 && gy < p.h && gx >= 0 && gx < p.w;
                const uint32_t* src = in_n + (((size_t)gz * p.h + gy) * p.w + gx) * 2u * wd;
                uint32_t* dst = lds + (size_t)(hz * plane + i) * t.vstride;
                for (int ch = 0; ch < t.nchunk; ++ch) {
                    if constexpr (WC == 2) {
                        uint2 m = make_uint2(0u, 0u), s = make_uint2(0u, 0u);
                        if (inb) {
                            m = *reinterpret_cast<const uint2*>(src + 2 * ch);
                            s = *reinterpret_cast<const uint2*>(src + wd + 2 * ch);
                        }
                        *reinterpret_cast<uint4*>(dst + 4 * ch) = make_uint4(m.x, m.y, s.x, s.y);
                    } else {
                        uint32_t m = 0u, s = 0u;
                        if (inb) { m = src[ch]; s = src[wd + ch]; }
                        *reinterpret_cast<uint2*>(dst + 2 * ch) = make_uint2(m, s);
                    }
                }
            }
        }
    }
    __syncthreads();

    // ---- this wave's voxels --------------------------------------------------------------
    const int wx = wave % t.nwx;
    const int wy = (wave / t.nwx) % t.nwy;
    const int wz = wave / (t.nwx * t.nwy);
    const int lx = lane & 7, ly = lane >> 3;
    const int ox = ox0 + wx * 8 + lx;
    const int oy = oy0 + wy * 8 + ly;
    const int ozb = oz0 + wz * V;
    const int row_words = t.hx * t.vstride;
    const int plane_words = t.hy * row_words;
    // LDS word offset of the tap-(0,0,0) input voxel of this lane's output voxel v = 0
    const int lane_base = (wz * V * p.sd) * plane_words + (wy * 8 + ly) * p.sh * row_words +
                          (wx * 8 + lx) * p.sw * t.vstride;
    const int vstep = p.sd * plane_words;  // between consecutive v
    const uint32_t* lane_lds = lds + lane_base;

    const int T = p.kd * p.kh * p.kw;
    const int co_begin = blockIdx.y * t.co_per_wg;
    const int co_end = min(p.c_out, co_begin + t.co_per_wg);
    const int nsteps = T * t.nchunk;
    // scalar increments of the LDS offset when the tap advances along x / wraps to the next
    // row / wraps to the next plane
    const int inc_c = p.dw * t.vstride;
    const int inc_b = p.dh * row_words - (p.kw - 1) * inc_c;
    const int inc_a = p.dd * plane_words - (p.kh - 1) * p.dh * row_words - (p.kw - 1) * inc_c;
    const int step_words = p.co_pad * 2 * WC;  // filter-bank words per step
    constexpr int NG = CO_BLK / kGroup;
    static_assert(NG >= 2 && NG % 2 == 0, "CO_BLK must be a multiple of 2*kGroup");

    uint32_t out_m[V], out_s[V];  // packed mode: words being assembled
#pragma unroll
    for (int v = 0; v < V; ++v) out_m[v] = out_s[v] = 0u;

    // The filter bank is padded with all-zero channels up to a multiple of 32, so a channel
    // block may run past c_out: the surplus accumulators stay 0 and are dropped below.
    for (int cb = co_begin; cb < co_end; cb += CO_BLK) {
        int32_t acc_m[V][CO_BLK], acc_n[V][CO_BLK];
#pragma unroll
        for (int v = 0; v < V; ++v)
#pragma unroll
            for (int j = 0; j < CO_BLK; ++j) acc_m[v][j] = acc_n[v][j] = 0;

        const int co_left = co_end - cb;
        scalar_ptr wblk = (scalar_ptr)(uintptr_t)p.wgt + (size_t)cb * 2 * WC;

        // Software pipeline: while a channel group of step i is being accumulated, the scalar
        // loads of the following group and the LDS reads of step i+1 are in flight.
        ActChunk<WC> A[V];
        WGroup<WC> g0, g1;
#pragma unroll
        for (int v = 0; v < V; ++v) A[v] = lds_read_chunk<WC>(lane_lds + v * vstep);
        load_wgroup<WC>(g0, wblk);

        int tb = 0, tc = 0, ch = 0;  // row / column / chunk of the step being accumulated
        int toff = 0;                // its LDS word offset (tap part)
        scalar_ptr wcur = wblk;      // its filter words
        for (int step = 0; step < nsteps; ++step) {
            // LDS offset of the following step (after the last step: step 0 again, whose
            // prefetched data is not used; this keeps every address in bounds)
            int nch = ch + 1, ntoff = toff;
            if (nch == t.nchunk) {
                nch = 0;
                if (++tc == p.kw) {
                    tc = 0;
                    if (++tb == p.kh) { tb = 0; ntoff += inc_a; }
                    else ntoff += inc_b;
                } else ntoff += inc_c;
            }
            const bool last = step + 1 == nsteps;
            if (last) { nch = 0; ntoff = 0; }
            scalar_ptr wnext = last ? wblk : wcur + step_words;

            ActChunk<WC> An[V];
#pragma unroll
            for (int gi = 0; gi < NG; gi += 2) {
                settle<WC>(g0);
                __builtin_amdgcn_sched_barrier(0);
                if (gi == 0) {
                    // LDS reads of the following step, issued behind the wait so that they
                    // complete under the arithmetic of the first group
#pragma unroll
                    for (int v = 0; v < V; ++v)
                        An[v] = lds_read_chunk<WC>(lane_lds + v * vstep + ntoff + nch * 2 * WC);
                }
                load_wgroup<WC>(g1, wcur + (gi + 1) * kGroup * 2 * WC);
                __builtin_amdgcn_sched_barrier(0);
                mac_group<WC, V, CO_BLK>(A, g0, gi * kGroup, acc_m, acc_n);
                __builtin_amdgcn_sched_barrier(0);
                settle<WC>(g1);
                __builtin_amdgcn_sched_barrier(0);
                if (gi + 2 < NG) load_wgroup<WC>(g0, wcur + (gi + 2) * kGroup * 2 * WC);
                else load_wgroup<WC>(g0, wnext);
                __builtin_amdgcn_sched_barrier(0);
                mac_group<WC, V, CO_BLK>(A, g1, (gi + 1) * kGroup, acc_m, acc_n);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int v = 0; v < V; ++v) A[v] = An[v];
            ch = nch; toff = ntoff; wcur = wnext;
        }

        // ---- epilogue ----------------------------------------------------------------------
        if constexpr (PACKED) {
            scalar_ptr thr_lo = (scalar_ptr)(uintptr_t)p.lo;
            scalar_ptr thr_hi = (scalar_ptr)(uintptr_t)p.hi;
            // Shift one decision bit per channel into a partial word, highest channel first.
            uint32_t pm[V], ps[V];
#pragma unroll
            for (int v = 0; v < V; ++v) pm[v] = ps[v] = 0u;
#pragma unroll
            for (int j = CO_BLK - 1; j >= 0; --j) {
                const bool live = j < co_left;
                const int cj = min(cb + j, p.c_out - 1);
                // |acc| < 2^24, so cut points beyond +-2^30 decide like +-infinity and the
                // differences below cannot overflow.  Channels past c_out get cut points that
                // never fire, i.e. zero bits.
                int32_t hi = (int32_t)thr_hi[cj];
                int32_t lo = (int32_t)thr_lo[cj];
                hi = live ? max(min(hi, 1 << 30), -(1 << 30)) : (1 << 30);
                lo = live ? max(min(lo, 1 << 30), -(1 << 30)) : -(1 << 30);
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    const int32_t acc = acc_m[v][j] - 2 * acc_n[v][j];
                    const uint32_t pos = (uint32_t)(hi - acc) >> 31;            // acc > hi
                    const uint32_t neg = ((uint32_t)(acc - lo) >> 31) & ~pos;   // acc < lo
                    pm[v] = (pm[v] << 1) | (pos | neg);
                    ps[v] = (ps[v] << 1) | neg;
                }
            }
            const int sh = cb & 31;  // CO_BLK divides 32 or is a multiple of it
#pragma unroll
            for (int v = 0; v < V; ++v) {
                if constexpr (CO_BLK >= 32) { out_m[v] = pm[v]; out_s[v] = ps[v]; }
                else { out_m[v] |= pm[v] << sh; out_s[v] |= ps[v] << sh; }
            }
            const bool flush = ((cb + CO_BLK) & 31) == 0 || cb + CO_BLK >= co_end;
            if (flush) {
                const int q = cb >> 5;
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    const int oz = ozb + v;
                    if (ox < p.ow && oy < p.oh && oz < p.od) {
                        uint32_t* o = p.out_packed +
                                      ((((size_t)n * p.od + oz) * p.oh + oy) * p.ow + ox) * 2u * p.wd_out;
                        o[q] = out_m[v];
                        o[p.wd_out + q] = out_s[v];
                    }
                    out_m[v] = out_s[v] = 0u;
                }
            }
        } else {
            const size_t cstride = (size_t)p.od * p.oh * p.ow;
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const int oz = ozb + v;
                if (ox < p.ow && oy < p.oh && oz < p.od) {
                    int32_t* o = p.out_acc + (size_t)n * p.c_out * cstride +
                                 ((size_t)oz * p.oh + oy) * p.ow + ox;
#pragma unroll
                    for (int j = 0; j < CO_BLK; ++j)
                        if (j < co_left) o[(size_t)(cb + j) * cstride] = acc_m[v][j] - 2 * acc_n[v][j];
                }
            }
        }
    }
}

template <int WC, int V, int CO_BLK, bool PACKED>
int launch_variant(const ConvParams& p, const TileParams& t, size_t lds_bytes, dim3 grid,
                   int threads, hipStream_t s)
{
    auto kern = conv_tiled_kernel<WC, V, CO_BLK, PACKED>;
    if (lds_bytes > 64 * 1024) {
        static thread_local int raised_on_device = -1;
        int dev = 0;
        TERN_HIP_CHECK(hipGetDevice(&dev));
        if (raised_on_device != dev) {
            TERN_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize,
                                               lds_limit_for_current_device()));
            raised_on_device = dev;
        }
    }
    hipLaunchKernelGGL(kern, grid, dim3(threads), lds_bytes, s, p, t);
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}

inline int cdiv(int a, int b) { return (a + b - 1) / b; }

}  // namespace

int launch_conv3d(const ConvParams& p, hipStream_t s)
{
    const bool packed = p.out_packed != nullptr;
    const int wd = p.wd_in;
    const int WC = p.wc;
    const int V = 2, CO_BLK = 32;

    TileParams t;
    t.nchunk = wd / WC;
    t.vstride = 2 * wd + (wd >= 4 ? 4 : 0);

    // Workgroup shape: start from one wave per workgroup and stack waves along z while the
    // halo tile stays small and there are plenty of workgroups; dilated kernels amortise their
    // wide halo better over larger tiles.
    t.nwx = 1; t.nwy = 1; t.nwz = 1;
    auto halo = [&](int tiles_out, int stride, int k, int dil) { return (tiles_out - 1) * stride + (k - 1) * dil + 1; };
    auto lds_for = [&](const TileParams& q) {
        const int64_t hx = halo(8 * q.nwx, p.sw, p.kw, p.dw);
        const int64_t hy = halo(8 * q.nwy, p.sh, p.kh, p.dh);
        const int64_t hz = halo(V * q.nwz, p.sd, p.kd, p.dd);
        return hx * hy * hz * q.vstride * 4;
    };
    // Grow the tile while the per-wave LDS share is too large for two waves per SIMD
    // (8 waves per compute unit => 20 KB per wave of the 160 KB).
    for (int it = 0; it < 6; ++it) {
        const int waves = t.nwx * t.nwy * t.nwz;
        if (lds_for(t) <= (int64_t)waves * 20 * 1024 || waves >= 8) break;
        TileParams best = t;
        double best_share = 1e30;
        TileParams cand[3] = {t, t, t};
        cand[0].nwz *= 2; cand[1].nwy *= 2; cand[2].nwx *= 2;
        for (const TileParams& c : cand) {
            const double share = (double)lds_for(c) / (c.nwx * c.nwy * c.nwz);
            if (share < best_share) { best_share = share; best = c; }
        }
        t = best;
    }
    const int64_t lds_bytes = lds_for(t);
    if (lds_bytes > lds_limit_for_current_device()) return launch_conv3d_generic(p, s);

    t.hx = halo(8 * t.nwx, p.sw, p.kw, p.dw);
    t.hy = halo(8 * t.nwy, p.sh, p.kh, p.dh);
    t.hz = halo(V * t.nwz, p.sd, p.kd, p.dd);
    t.tiles_x = cdiv(p.ow, 8 * t.nwx);
    t.tiles_y = cdiv(p.oh, 8 * t.nwy);
    t.tiles_z = cdiv(p.od, V * t.nwz);
    const int64_t spatial_tiles = (int64_t)t.tiles_x * t.tiles_y * t.tiles_z * p.n;
    if (spatial_tiles > 0x7fffffff) return TERN_ESHAPE;

    // Split output channels over blockIdx.y when there are too few spatial tiles to fill the
    // chip (2048 wave slots at two waves per SIMD).  Packed output needs whole 32-channel words.
    const int waves_per_wg = t.nwx * t.nwy * t.nwz;
    const int co_gran = packed ? 32 : CO_BLK;
    int co_groups = cdiv(p.c_out, co_gran);
    int split = 1;
    while (split < co_groups && spatial_tiles * waves_per_wg * split < 2048) split *= 2;
    split = split < co_groups ? split : co_groups;
    t.co_per_wg = cdiv(co_groups, split) * co_gran;
    const int grid_y = cdiv(p.c_out, t.co_per_wg);

    const dim3 grid((unsigned)spatial_tiles, (unsigned)grid_y);
    const int threads = 64 * waves_per_wg;
    if (WC == 2) {
        return packed ? launch_variant<2, 2, 32, true>(p, t, (size_t)lds_bytes, grid, threads, s)
                      : launch_variant<2, 2, 32, false>(p, t, (size_t)lds_bytes, grid, threads, s);
    }
    return packed ? launch_variant<1, 2, 32, true>(p, t, (size_t)lds_bytes, grid, threads, s)
                  : launch_variant<1, 2, 32, false>(p, t, (size_t)lds_bytes, grid, threads, s);
}

}  // namespace tern
