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
#include <cmath>

#include "tern_conv_common.h"
#include "tern_internal.h"

namespace tern {

int launch_conv3d_generic(const ConvParams& p, hipStream_t s);

// Largest dynamic LDS allocation the current device grants one workgroup (queried once per
// device; 0 on error).
int lds_limit_for_current_device()
{
    constexpr int kLdsLimit = 160 * 1024;    // LDS per compute unit on gfx950
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

// Compute units of the current device (queried once per device; 0 on error).
static int compute_units_of_current_device()
{
    static int cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (cached[dev] == 0) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cached[dev] = v;
    }
    return cached[dev];
}

namespace {

constexpr int kMaxThreads = 512;         // 8 waves: at most 2 waves per SIMD, <= 256 VGPRs
constexpr int kStreamItems = 2;          // persistent kernel: halo items a thread prefetches per tile

struct TileParams {
    int32_t nwx, nwy, nwz;        // waves per workgroup along x, y, z
    int32_t hx, hy, hz;           // halo tile extents in voxels
    int32_t tiles_x, tiles_y, tiles_z;
    int32_t vstride;              // LDS words per voxel (2*Wd plus padding)
    int32_t nchunk;               // Wd / WC
    int32_t nwc;                  // waves per workgroup along the output-channel axis
    int32_t co_per_wave;          // output channels handled by one wave (multiple of 16)
    int32_t nks;                  // waves per workgroup that split the kernel taps of one slice
    int32_t red_off;              // LDS word offset of the partial-sum area (nks > 1)
    int32_t vy;                   // 1: a lane's V voxels are 8 rows apart along y (single-plane
                                  // outputs); 0: consecutive along z
    // flat halo fill: floor(e / d) = umulhi(e, m_d) with m_d = 0xffffffff / d + 1 for d = hx,
    // hy * hx and nchunk (valid for e * d < 2^32 and d > 1; m_ch is unused when nchunk = 1, m_hx
    // when hx = 1)
    uint32_t m_hx, m_pl, m_ch;
    // a wave's 64 lanes cover 2^lxb x 2^lyb x 64 / 2^(lxb + lyb) output voxels (x, y, z), x fastest
    int32_t lxb, lyb;
    int32_t flat;                 // 1: halo fill over one flat index space, 0: per plane position
    int32_t tiles_per_wg;         // persistent kernel: consecutive tiles one workgroup walks
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

// Scalar walk over the kernel taps.  Plain mode: one step = one (tap, channel chunk) and the
// cursor is the step whose activations were fetched last.  Tap-packed mode (C_in <= 16, one
// word per voxel): one step = up to `slots` consecutive taps whose channel bits are shifted into
// disjoint slots of a single word, and the cursor is the next tap to fetch.
struct StepCursor {
    int tb, tc, ch;   // kernel row, column and channel chunk
    int toff;         // LDS word offset of the tap
    int tap;          // linear tap index
};

// (The LDS offset increments for "next column / next row / next plane" travel as three separate
// by-value ints, not as members: as struct members the compiler turns the choice between them
// into an indexed load from a stack copy of the struct.)
// Loop-invariant scalars of the walk.
struct StepConsts {
    int kw, kh, nchunk;
    int step_words;            // filter-bank words per step
    int vstep;                 // LDS words between a lane's consecutive voxels
    int slots, shift;          // tap-packed mode: taps per word, bits per slot
    uint32_t slot_mask;        // tap-packed mode: (1 << C_in) - 1
    int tap_end;               // tap-packed mode: first tap this wave does not own
};

__device__ __forceinline__ void next_tap(StepCursor& c, const StepConsts& sc, int inc_c, int inc_b,
                                         int inc_a)
{
    ++c.tap;
    int inc = inc_c;
    if (++c.tc == sc.kw) {
        c.tc = 0;
        inc = inc_b;
        if (++c.tb == sc.kh) { c.tb = 0; inc = inc_a; }
    }
    c.toff += inc;
}

// Fetch the activations of one step into A.  Plain mode: advance to the following step unless
// `stay` (used for the prefetch after a wave's last step, which is discarded), then read.
template <int WC, int V, bool TP>
__device__ __forceinline__ void fetch_step(ActChunk<WC> (&A)[V], StepCursor& c, const StepConsts& sc,
                                           int inc_c, int inc_b, int inc_a,
                                           const uint32_t* lane_lds, bool advance)
{
    if constexpr (!TP) {
        if (advance) {
            if (++c.ch == sc.nchunk) { c.ch = 0; next_tap(c, sc, inc_c, inc_b, inc_a); }
        }
#pragma unroll
        for (int v = 0; v < V; ++v)
            A[v] = lds_read_chunk<WC>(lane_lds + v * sc.vstep + c.toff + c.ch * 2 * WC);
    } else {
        static_assert(WC == 1 || !TP, "tap packing uses one word per voxel");
#pragma unroll
        for (int v = 0; v < V; ++v) A[v].m[0] = A[v].s[0] = 0u;
        for (int i = 0; i < sc.slots && c.tap < sc.tap_end; ++i) {
            const int sh = i * sc.shift;
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const uint2 r = *reinterpret_cast<const uint2*>(lane_lds + v * sc.vstep + c.toff);
                A[v].m[0] |= (r.x & sc.slot_mask) << sh;
                A[v].s[0] |= (r.y & sc.slot_mask) << sh;
            }
            next_tap(c, sc, inc_c, inc_b, inc_a);
        }
    }
}

// Filter-word group of a kernel variant: ternary filters carry mask and sign words (2 WC words per
// channel in the bank), binary filters sign words only (WC words per channel, eight channels per
// group: sixteen SGPRs at most).
template <int WC, int CO_BLK, bool BIN>
struct GroupType {
    static constexpr int KG = GroupOf<CO_BLK>::value;
    static constexpr int CW = 2 * WC;   // bank words per channel and step
    using type = WGroup<WC, KG>;
};
template <int WC, int CO_BLK>
struct GroupType<WC, CO_BLK, true> {
    static constexpr int KG = 8;
    static constexpr int CW = WC;
    using type = WGroupB<WC, KG>;
};

// One step: accumulate CO_BLK channels from A0 (this step's activations) while fetching the next
// step's activations into A1.  Software pipeline: while a channel group is being accumulated,
// the scalar loads of the following group and the LDS reads of the next step are in flight.
// INIT marks the first step of a pass, which sets the accumulators instead of adding to them.
// DIG: two-digit input, the odd word of a chunk goes to the second accumulator set.
// BIN: binary filters (Eq. 8): only acc_n is used, and cnt collects popcount(mask_a) per voxel.
template <int WC, int V, int CO_BLK, bool TP, bool DIG, bool BIN, bool INIT = false, typename Acc2>
__device__ __forceinline__ void conv_step(const ActChunk<WC> (&A0)[V], ActChunk<WC> (&A1)[V], bool last,
                                          StepCursor& cur, const StepConsts& sc, int inc_c, int inc_b,
                                          int inc_a, typename GroupType<WC, CO_BLK, BIN>::type& g0,
                                          typename GroupType<WC, CO_BLK, BIN>::type& g1, scalar_ptr& wcur,
                                          const uint32_t* lane_lds,
                                          int32_t (&acc_m)[V][CO_BLK], int32_t (&acc_n)[V][CO_BLK],
                                          Acc2& acc2_m, Acc2& acc2_n, int32_t (&cnt)[V])
{
    using GT = GroupType<WC, CO_BLK, BIN>;
    constexpr int KG = GT::KG;
    constexpr int CW = GT::CW;
    constexpr int NG = CO_BLK / KG;
    // after a wave's last step the prefetches re-read the same (valid) addresses and are dropped
    scalar_ptr wnext = last ? wcur : wcur + sc.step_words;
    if constexpr (BIN) {
#pragma unroll
        for (int v = 0; v < V; ++v)
#pragma unroll
            for (int q = 0; q < WC; ++q) cnt[v] += __builtin_popcount(A0[v].m[q]);
    }
#pragma unroll
    for (int gi = 0; gi < NG; gi += 2) {
        settle<WC, KG>(g0);
        __builtin_amdgcn_sched_barrier(0);
        // issued behind the wait so that the LDS reads complete under the first group's arithmetic
        if (gi == 0) fetch_step<WC, V, TP>(A1, cur, sc, inc_c, inc_b, inc_a, lane_lds, !last);
        load_wgroup<WC, KG>(g1, wcur + (gi + 1) * KG * CW);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (BIN) mac_group_bin<WC, V, CO_BLK, KG, INIT>(A0, g0, gi * KG, acc_n);
        else if constexpr (DIG) mac_group_digits<V, CO_BLK, KG, INIT>(A0, g0, gi * KG, acc_m, acc_n, acc2_m, acc2_n);
        else mac_group<WC, V, CO_BLK, KG, INIT>(A0, g0, gi * KG, acc_m, acc_n);
        __builtin_amdgcn_sched_barrier(0);
        settle<WC, KG>(g1);
        __builtin_amdgcn_sched_barrier(0);
        if (gi + 2 < NG) load_wgroup<WC, KG>(g0, wcur + (gi + 2) * KG * CW);
        else load_wgroup<WC, KG>(g0, wnext);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (BIN) mac_group_bin<WC, V, CO_BLK, KG, INIT>(A0, g1, (gi + 1) * KG, acc_n);
        else if constexpr (DIG) mac_group_digits<V, CO_BLK, KG, INIT>(A0, g1, (gi + 1) * KG, acc_m, acc_n, acc2_m, acc2_n);
        else mac_group<WC, V, CO_BLK, KG, INIT>(A0, g1, (gi + 1) * KG, acc_m, acc_n);
        __builtin_amdgcn_sched_barrier(0);
    }
    wcur = wnext;
}

// End of one accumulation pass: channels [cb, cb + CO_BLK) of a wave whose slice is [co_begin,
// co_end).  PACKED: Eq. 6 in integer form, the decision bits collected in pos_w / neg_w until a
// 32-channel word (or the slice) is complete, then stored; else the raw accumulators (NCDHW).
// A lane's V voxels are (ox, oy, ozb + v), or (ox, oy + LY * v, ozb) for single-plane outputs.
template <int V, int CO_BLK, bool PACKED>
__device__ __forceinline__ void finish_pass(const int32_t (&d)[V][CO_BLK], const ConvParams& p, const TileParams& t,
                                            int cb, int co_begin, int co_end, int n, int ox, int oy, int ozb, int LY,
                                            uint32_t (&pos_w)[V], uint32_t (&neg_w)[V])
{
    const int co_left = co_end - cb;
    if constexpr (PACKED) {
        // Cut points of this block come through the scalar cache, a few channels at a time.
        uint32_t pp[V], pn[V];
        ternarise_pass<V, CO_BLK>(d, (scalar_ptr)(uintptr_t)p.lo, (scalar_ptr)(uintptr_t)p.hi, cb,
                                  co_left, p.c_out, pp, pn);
        const int sh = cb & 31;
#pragma unroll
        for (int v = 0; v < V; ++v) { pos_w[v] |= pp[v] << sh; neg_w[v] |= pn[v] << sh; }
        const bool flush = ((cb + CO_BLK) & 31) == 0 || cb + CO_BLK >= co_end;
        if (flush) {
            // This wave's bits of word q are [b0, b1), whole bytes.  A wave that owns only part
            // of the word stores that part (16- or 8-bit stores) so that the waves owning the
            // rest can store theirs without a read-modify-write; the wave that owns the last
            // existing channel of the word also stores the (zero) bytes behind it.
            const int q = cb >> 5;
            const int b0 = max(co_begin, q * 32) - q * 32;
            const int b1 = min(co_begin + t.co_per_wave, q * 32 + 32) - q * 32;
            const int B0 = b0 >> 3;
            const int B1 = (q * 32 + b1 >= p.c_out) ? 4 : (b1 >> 3);
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const int oz = t.vy ? ozb : ozb + v;
                const int oyv = t.vy ? oy + LY * v : oy;
                if (ox < p.ow && oyv < p.oh && oz < p.od) {
                    uint32_t* o = p.out_packed +
                                  ((((size_t)n * p.od + oz) * p.oh + oyv) * p.ow + ox) * 2u * p.wd_out;
                    const uint32_t mk = pos_w[v] | neg_w[v];      // nonzero mask
                    const uint32_t sg = neg_w[v] & ~pos_w[v];     // sign; +1 wins if lo > hi
                    if (B0 == 0 && B1 == 4) {
                        o[q] = mk;
                        o[p.wd_out + q] = sg;
                    } else if ((B0 & 1) == 0 && B1 - B0 == 2) {
                        reinterpret_cast<uint16_t*>(o + q)[B0 >> 1] = (uint16_t)(mk >> (8 * B0));
                        reinterpret_cast<uint16_t*>(o + p.wd_out + q)[B0 >> 1] = (uint16_t)(sg >> (8 * B0));
                    } else {
                        for (int B = B0; B < B1; ++B) {
                            reinterpret_cast<uint8_t*>(o + q)[B] = (uint8_t)(mk >> (8 * B));
                            reinterpret_cast<uint8_t*>(o + p.wd_out + q)[B] = (uint8_t)(sg >> (8 * B));
                        }
                    }
                }
                pos_w[v] = neg_w[v] = 0u;
            }
        }
    } else {
        const size_t cstride = (size_t)p.od * p.oh * p.ow;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const int oz = t.vy ? ozb : ozb + v;
            const int oyv = t.vy ? oy + LY * v : oy;
            if (ox < p.ow && oyv < p.oh && oz < p.od) {
                int32_t* o = p.out_acc + (size_t)n * p.c_out * cstride +
                             ((size_t)oz * p.oh + oyv) * p.ow + ox;
#pragma unroll
                for (int j = 0; j < CO_BLK; ++j)
                    if (j < co_left) o[(size_t)(cb + j) * cstride] = d[v][j];
            }
        }
    }
}

template <int WC, int V, int CO_BLK, bool PACKED, bool TP, bool DIG = false, bool BIN = false>
__global__ __launch_bounds__(kMaxThreads) void conv_tiled_kernel(ConvParams p, TileParams t)
{
    extern __shared__ __align__(16) uint32_t lds[];

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- which tile ------------------------------------------------------------------------
    // Workgroups are handed to the 8 XCDs round-robin by index; give each XCD a contiguous run
    // of tiles so that neighbouring tiles (which share halo voxels) meet in the same L2.
    int bid = blockIdx.x;
    {
        const int per_xcd = gridDim.x >> 3;
        if (bid < (per_xcd << 3)) bid = (bid & 7) * per_xcd + (bid >> 3);
    }
    const int tix = bid % t.tiles_x; bid /= t.tiles_x;
    const int tiy = bid % t.tiles_y; bid /= t.tiles_y;
    const int tiz = bid % t.tiles_z;
    const int n = bid / t.tiles_z;
    // A lane's V output voxels are stacked along z, or (vy: single-plane outputs) along y.
    const int LX = 1 << t.lxb, LY = 1 << t.lyb, LZ = 64 >> (t.lxb + t.lyb);   // lanes along x, y, z
    const int ywave = t.vy ? LY * V : LY, zwave = t.vy ? 1 : LZ * V;   // output extent of one wave
    const int TX = LX * t.nwx, TY = ywave * t.nwy, TZ = zwave * t.nwz;
    const int ox0 = tix * TX, oy0 = tiy * TY, oz0 = tiz * TZ;

    // ---- stage the halo tile -------------------------------------------------------------
    // All global loads of a batch of FB voxels are issued before the batch's first LDS write, so
    // a wave pays one memory round trip per batch instead of one per voxel.  Deep tiles: a thread
    // owns plane positions i = tid, tid + nthreads, ... of the (hy, hx) halo plane and a batch is
    // FB planes of one position.  Flat tiles (few planes, many positions per thread, as for
    // single-plane outputs): a batch is FB (position, chunk) items of the whole tile.
    {
        constexpr int FB = 8;
        const int gx0 = ox0 * p.sw - p.pw, gy0 = oy0 * p.sh - p.ph, gz0 = oz0 * p.sd - p.pd;
        const int plane = t.hy * t.hx;
        const int wd = p.wd_in;
        const uint32_t* in_n = p.in + (size_t)n * p.d * p.h * p.w * 2u * wd;
        const size_t zstride = (size_t)p.h * p.w * 2u * wd;   // words between input planes
        if (!t.flat) {
            for (int i = tid; i < plane; i += nthreads) {
                const int hy = i / t.hx;
                const int hxx = i - hy * t.hx;
                const int gy = gy0 + hy, gx = gx0 + hxx;
                const bool xy_in = gy >= 0 && gy < p.h && gx >= 0 && gx < p.w;
                const uint32_t* src_xy = in_n + ((size_t)(xy_in ? gy : 0) * p.w + (xy_in ? gx : 0)) * 2u * wd;
                uint32_t* dst_xy = lds + (size_t)i * t.vstride;
                for (int ch = 0; ch < t.nchunk; ++ch) {
                    for (int hz0 = 0; hz0 < t.hz; hz0 += FB) {
                        uint4 r[FB];
                        // the second half of a batch is skipped as a whole (a wave-uniform
                        // branch) when at most FB/2 planes are left, e.g. 4-plane tiles
                        const bool both = t.hz - hz0 > FB / 2;
    #pragma unroll
                        for (int half = 0; half < 2; ++half) {
                            if (half == 0 || both) {
    #pragma unroll
                                for (int j = half * (FB / 2); j < (half + 1) * (FB / 2); ++j) {
                                    const int gz = gz0 + hz0 + j;
                                    const bool inb = xy_in && hz0 + j < t.hz && gz >= 0 && gz < p.d;
                                    r[j] = make_uint4(0u, 0u, 0u, 0u);
                                    if (inb) {
                                        const uint32_t* src = src_xy + (size_t)gz * zstride;
                                        if constexpr (WC == 2) {
                                            const uint2 m = *reinterpret_cast<const uint2*>(src + 2 * ch);
                                            const uint2 sg = *reinterpret_cast<const uint2*>(src + wd + 2 * ch);
                                            r[j] = make_uint4(m.x, m.y, sg.x, sg.y);
                                        } else {
                                            r[j].x = src[ch];
                                            r[j].y = src[wd + ch];
                                        }
                                    }
                                }
                            }
                        }
    #pragma unroll
                        for (int half = 0; half < 2; ++half) {
                            if (half == 0 || both) {
    #pragma unroll
                                for (int j = half * (FB / 2); j < (half + 1) * (FB / 2); ++j) {
                                    if (hz0 + j < t.hz) {
                                        uint32_t* dst = dst_xy + (size_t)(hz0 + j) * plane * t.vstride;
                                        if constexpr (WC == 2) *reinterpret_cast<uint4*>(dst + 4 * ch) = r[j];
                                        else *reinterpret_cast<uint2*>(dst + 2 * ch) = make_uint2(r[j].x, r[j].y);
                                    }
                                }
                            }
                        }
                    }
                }
            }
        } else {
            // One index space over (plane, position, chunk), chunk fastest: neighbouring threads
            // read neighbouring words of one voxel record and write neighbouring LDS words, and
            // a thread's FB items are in flight together whatever plane and chunk they belong to
            // (with a loop per plane and chunk a 512-channel tile took 16 round trips).
            // The divisions are multiplications by host-made reciprocals; e is below the tile's
            // LDS words.
            const uint32_t nch = (uint32_t)t.nchunk;
            const uint32_t m_hx = t.m_hx, m_pl = t.m_pl, m_ch = t.m_ch;
            const uint32_t items = (uint32_t)t.hz * (uint32_t)plane * nch;
            for (uint32_t e0 = tid; e0 < items; e0 += FB * nthreads) {
                uint4 r[FB];
#pragma unroll
                for (int j = 0; j < FB; ++j) {
                    const uint32_t e = e0 + j * nthreads;
                    const uint32_t vox = nch > 1 ? __umulhi(e, m_ch) : e;   // plane * position index
                    const uint32_t ch = e - vox * nch;
                    const uint32_t hz = __umulhi(vox, m_pl);
                    const uint32_t i = vox - hz * plane;
                    const int hy = t.hx > 1 ? (int)__umulhi(i, m_hx) : (int)i;   // no 32-bit reciprocal of 1
                    const int hxx = (int)i - hy * t.hx;
                    const int gz = gz0 + (int)hz, gy = gy0 + hy, gx = gx0 + hxx;
                    const bool inb = e < items && gz >= 0 && gz < p.d && gy >= 0 && gy < p.h && gx >= 0 && gx < p.w;
                    r[j] = make_uint4(0u, 0u, 0u, 0u);
                    if (inb) {
                        const uint32_t* src = in_n + (((size_t)gz * p.h + gy) * p.w + gx) * 2u * wd;
                        if constexpr (WC == 2) {
                            const uint2 m = *reinterpret_cast<const uint2*>(src + 2 * ch);
                            const uint2 sg = *reinterpret_cast<const uint2*>(src + wd + 2 * ch);
                            r[j] = make_uint4(m.x, m.y, sg.x, sg.y);
                        } else {
                            r[j].x = src[ch];
                            r[j].y = src[wd + ch];
                        }
                    }
                }
#pragma unroll
                for (int j = 0; j < FB; ++j) {
                    const uint32_t e = e0 + j * nthreads;
                    if (e < items) {
                        const uint32_t vox = nch > 1 ? __umulhi(e, m_ch) : e;
                        uint32_t* dst = lds + vox * t.vstride + (e - vox * nch) * (2 * WC);
                        if constexpr (WC == 2) *reinterpret_cast<uint4*>(dst) = r[j];
                        else *reinterpret_cast<uint2*>(dst) = make_uint2(r[j].x, r[j].y);
                    }
                }
            }
        }
    }
    __syncthreads();

    // ---- this wave's voxels --------------------------------------------------------------
    const int nsp = t.nwx * t.nwy * t.nwz;
    const int wslot = wave % (nsp * t.nwc);           // (spatial, channel-slice) position
    const int ks = wave / (nsp * t.nwc);              // which share of the kernel taps
    const int wx = wslot % t.nwx;
    const int wy = (wslot / t.nwx) % t.nwy;
    const int wz = (wslot / (t.nwx * t.nwy)) % t.nwz;
    const int wch = wslot / nsp;                      // channel slice of this wave
    const int lx = lane & (LX - 1), ly = (lane >> t.lxb) & (LY - 1);
    const int lz = t.vy ? 0 : (lane >> (t.lxb + t.lyb)) * V;   // first of the lane's planes in the wave
    const int ox = ox0 + wx * LX + lx;
    const int oy = oy0 + wy * ywave + ly;
    const int ozb = oz0 + wz * zwave + lz;
    const int row_words = t.hx * t.vstride;
    const int plane_words = t.hy * row_words;
    // LDS word offset of the tap-(0,0,0) input voxel of this lane's output voxel v = 0
    const int lane_base = ((wz * zwave + lz) * p.sd) * plane_words + (wy * ywave + ly) * p.sh * row_words +
                          (wx * LX + lx) * p.sw * t.vstride;
    const int vstep = t.vy ? LY * p.sh * row_words : p.sd * plane_words;  // between consecutive v
    const uint32_t* lane_lds = lds + lane_base;

    const int T = p.kd * p.kh * p.kw;
    const int co_begin = (blockIdx.y * t.nwc + wch) * t.co_per_wave;
    const int co_end = min(p.c_out, co_begin + t.co_per_wave);
    const int nsteps = TP ? (T + p.tp_slots - 1) / p.tp_slots : T * t.nchunk;
    // this wave's share of the steps (all of them unless the taps are split over nks waves)
    const int steps_per_wave = (nsteps + t.nks - 1) / t.nks;
    const int s_begin = ks * steps_per_wave;
    const int s_end = min(nsteps, s_begin + steps_per_wave);
    StepConsts sc;
    sc.kw = p.kw; sc.kh = p.kh; sc.nchunk = t.nchunk;
    const int inc_c = p.dw * t.vstride;
    const int inc_b = p.dh * row_words - (p.kw - 1) * inc_c;
    const int inc_a = p.dd * plane_words - (p.kh - 1) * p.dh * row_words - (p.kw - 1) * inc_c;
    using GT = GroupType<WC, CO_BLK, BIN>;
    constexpr int CW = GT::CW;
    static_assert(!BIN || (!TP && !DIG), "binary filters use the plain bank layout and one-digit inputs");
    sc.step_words = p.co_pad * CW;
    sc.vstep = vstep;
    sc.slots = p.tp_slots; sc.shift = p.tp_shift;
    sc.slot_mask = TP ? ((1u << p.c_in) - 1u) : 0xffffffffu;
    sc.tap_end = TP ? min(T, s_end * p.tp_slots) : T;
    // cursor at this wave's first step
    StepCursor cur0 = {0, 0, 0, 0, 0};
    if (s_begin > 0) {
        const int tap0 = TP ? s_begin * p.tp_slots : s_begin / t.nchunk;
        cur0.ch = TP ? 0 : s_begin - tap0 * t.nchunk;
        cur0.tap = tap0;
        cur0.tc = tap0 % p.kw;
        const int r = tap0 / p.kw;
        cur0.tb = r % p.kh;
        const int ta = r / p.kh;
        cur0.toff = ta * p.dd * plane_words + cur0.tb * p.dh * row_words + cur0.tc * inc_c;
    }
    constexpr int KG = GT::KG;
    constexpr int NG = CO_BLK / KG;
    static_assert(NG >= 2 && NG % 2 == 0, "CO_BLK must be a multiple of twice the group size");
    static_assert(CO_BLK <= 32 && 32 % CO_BLK == 0 && CO_BLK % 8 == 0, "CO_BLK must divide 32 in whole bytes");

    uint32_t pos_w[V], neg_w[V];  // packed mode: decision bits of the 32-channel word in progress
#pragma unroll
    for (int v = 0; v < V; ++v) pos_w[v] = neg_w[v] = 0u;

    // The filter bank is padded with all-zero channels up to a multiple of 32, so a channel
    // block may run past c_out: the surplus accumulators stay 0 and are dropped below.
    // With split taps (nks > 1) a wave makes exactly one pass (co_per_wave == CO_BLK) and every
    // wave of the workgroup, with or without channels of its own, meets at the barrier below.
    for (int cb = co_begin;; cb += CO_BLK) {
        const bool active = cb < co_end;
        if (!active && t.nks == 1) break;
        int32_t d[V][CO_BLK];   // accumulators of this pass
        if (active && s_begin < s_end) {
            int32_t acc_m[V][CO_BLK], acc_n[V][CO_BLK];   // set by the pass's first step
            // second set for the high digits of a two-digit input (one dummy element otherwise)
            int32_t acc2_m[DIG ? V : 1][DIG ? CO_BLK : 1], acc2_n[DIG ? V : 1][DIG ? CO_BLK : 1];
            int32_t cnt[V];   // binary filters: nonzero activations met so far (the c of Eq. 8)
#pragma unroll
            for (int v = 0; v < V; ++v) cnt[v] = 0;
            scalar_ptr wcur = (scalar_ptr)(uintptr_t)p.wgt + (size_t)cb * CW +
                              (size_t)s_begin * sc.step_words;
            typename GT::type g0, g1;
            StepCursor cur = cur0;
            ActChunk<WC> Aa[V], Ab[V];
            fetch_step<WC, V, TP>(Aa, cur, sc, inc_c, inc_b, inc_a, lane_lds, false);
            load_wgroup<WC, KG>(g0, wcur);
            int step = s_begin + 1;
            conv_step<WC, V, CO_BLK, TP, DIG, BIN, true>(Aa, Ab, step == s_end, cur, sc, inc_c, inc_b, inc_a, g0, g1,
                                                         wcur, lane_lds, acc_m, acc_n, acc2_m, acc2_n, cnt);
            for (; step + 2 <= s_end; step += 2) {   // two steps per trip: no register copies
                conv_step<WC, V, CO_BLK, TP, DIG, BIN>(Ab, Aa, false, cur, sc, inc_c, inc_b, inc_a, g0, g1, wcur,
                                                       lane_lds, acc_m, acc_n, acc2_m, acc2_n, cnt);
                conv_step<WC, V, CO_BLK, TP, DIG, BIN>(Aa, Ab, step + 2 == s_end, cur, sc, inc_c, inc_b, inc_a, g0,
                                                       g1, wcur, lane_lds, acc_m, acc_n, acc2_m, acc2_n, cnt);
            }
            if (step < s_end)
                conv_step<WC, V, CO_BLK, TP, DIG, BIN>(Ab, Aa, true, cur, sc, inc_c, inc_b, inc_a, g0, g1, wcur,
                                                       lane_lds, acc_m, acc_n, acc2_m, acc2_n, cnt);
#pragma unroll
            for (int v = 0; v < V; ++v)
#pragma unroll
                for (int j = 0; j < CO_BLK; ++j) {
                    if constexpr (BIN) d[v][j] = cnt[v] - 2 * acc_n[v][j];   // c - 2 popcount, Eq. 8
                    else d[v][j] = acc_m[v][j] - 2 * acc_n[v][j];
                    if constexpr (DIG) d[v][j] += 3 * (acc2_m[v][j] - 2 * acc2_n[v][j]);   // high digit
                }
        } else if (active) {   // a tap share without steps (more shares than steps)
#pragma unroll
            for (int v = 0; v < V; ++v)
#pragma unroll
                for (int j = 0; j < CO_BLK; ++j) d[v][j] = 0;
        }

        if (t.nks > 1) {
            // Partial sums of the tap shares meet in LDS: shares 1.. store, share 0 adds them up
            // and carries on to the epilogue.
            int32_t* red = reinterpret_cast<int32_t*>(lds) + t.red_off;
            const int nslots = nsp * t.nwc;
            if (active && ks > 0) {
                int32_t* mine = red + (size_t)((ks - 1) * nslots + wslot) * (V * CO_BLK * 64) + lane;
#pragma unroll
                for (int v = 0; v < V; ++v)
#pragma unroll
                    for (int j = 0; j < CO_BLK; ++j) mine[(v * CO_BLK + j) * 64] = d[v][j];
            }
            __syncthreads();
            if (!active || ks > 0) break;
            for (int k = 1; k < t.nks; ++k) {
                const int32_t* theirs = red + (size_t)((k - 1) * nslots + wslot) * (V * CO_BLK * 64) + lane;
#pragma unroll
                for (int v = 0; v < V; ++v)
#pragma unroll
                    for (int j = 0; j < CO_BLK; ++j) d[v][j] += theirs[(v * CO_BLK + j) * 64];
            }
        }

        // ---- epilogue ----------------------------------------------------------------------
        finish_pass<V, CO_BLK, PACKED>(d, p, t, cb, co_begin, co_end, n, ox, oy, ozb, LY, pos_w, neg_w);
        if (t.nks > 1) break;
    }
}

// Persistent form of the kernel above for large launches of four-wave workgroups (one voxel per
// lane, whole kernel per wave): a workgroup walks a run of consecutive tiles and holds two halo
// tiles in LDS.  The global loads of the next tile are issued before the current tile's tap loop
// and land in registers under it; they are written to the other LDS buffer after the loop, so
// no wave waits for a halo fill except the very first.  Launched with as many workgroups as the
// chip holds at once (four per compute unit), so every SIMD keeps the same four waves from start
// to end and no second generation of workgroups has to ramp up.
template <int WC, int CO_BLK, bool PACKED, bool BIN>
__global__ __launch_bounds__(256) void conv_tiled_stream_kernel(ConvParams p, TileParams t)
{
    constexpr int V = 1;
    constexpr int NI = kStreamItems;
    extern __shared__ __align__(16) uint32_t lds[];

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- this workgroup's run of tiles (contiguous per XCD, as above) -------------------------
    int w = blockIdx.x;
    {
        const int per_xcd = gridDim.x >> 3;
        if (w < (per_xcd << 3)) w = (w & 7) * per_xcd + (w >> 3);
    }
    const int ntiles = t.tiles_x * t.tiles_y * t.tiles_z * p.n;
    const int first = w * t.tiles_per_wg;
    const int last = min(ntiles, first + t.tiles_per_wg);
    if (first >= last) return;   // whole workgroup

    const int LX = 1 << t.lxb, LY = 1 << t.lyb, LZ = 64 >> (t.lxb + t.lyb);
    const int TX = LX * t.nwx, TY = LY * t.nwy, TZ = LZ * t.nwz;
    const int plane = t.hy * t.hx;
    const int wd = p.wd_in;
    const uint32_t nch = (uint32_t)t.nchunk;
    const uint32_t items = (uint32_t)t.hz * (uint32_t)plane * nch;
    const int buf_words = t.hz * plane * t.vstride;

    struct Origin { int ox0, oy0, oz0, n; };
    auto origin_of = [&](int tile) {
        Origin o;
        const int tix = tile % t.tiles_x; tile /= t.tiles_x;
        const int tiy = tile % t.tiles_y; tile /= t.tiles_y;
        const int tiz = tile % t.tiles_z;
        o.n = tile / t.tiles_z;
        o.ox0 = tix * TX; o.oy0 = tiy * TY; o.oz0 = tiz * TZ;
        return o;
    };
    // Halo items e = tid + j * nthreads of one tile, (plane, position, chunk) with chunk fastest;
    // out-of-volume voxels read as zero words.  Slots that no lane of the wave uses are skipped.
    auto load_items = [&](const Origin& o, uint4 (&r)[NI]) {
        const int gx0 = o.ox0 * p.sw - p.pw, gy0 = o.oy0 * p.sh - p.ph, gz0 = o.oz0 * p.sd - p.pd;
        const uint32_t* in_n = p.in + (size_t)o.n * p.d * p.h * p.w * 2u * wd;
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            r[j] = make_uint4(0u, 0u, 0u, 0u);
            if ((uint32_t)(wave * 64 + j * nthreads) < items) {
                const uint32_t e = tid + j * nthreads;
                const uint32_t vox = nch > 1 ? __umulhi(e, t.m_ch) : e;
                const uint32_t ch = e - vox * nch;
                const uint32_t hz = __umulhi(vox, t.m_pl);
                const uint32_t i = vox - hz * plane;
                const int hy = t.hx > 1 ? (int)__umulhi(i, t.m_hx) : (int)i;
                const int hxx = (int)i - hy * t.hx;
                const int gz = gz0 + (int)hz, gy = gy0 + hy, gx = gx0 + hxx;
                if (e < items && gz >= 0 && gz < p.d && gy >= 0 && gy < p.h && gx >= 0 && gx < p.w) {
                    const uint32_t* src = in_n + (((size_t)gz * p.h + gy) * p.w + gx) * 2u * wd;
                    if constexpr (WC == 2) {
                        const uint2 m = *reinterpret_cast<const uint2*>(src + 2 * ch);
                        const uint2 sg = *reinterpret_cast<const uint2*>(src + wd + 2 * ch);
                        r[j] = make_uint4(m.x, m.y, sg.x, sg.y);
                    } else {
                        r[j].x = src[ch];
                        r[j].y = src[wd + ch];
                    }
                }
            }
        }
    };
    auto store_items = [&](uint32_t* buf, const uint4 (&r)[NI]) {
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const uint32_t e = tid + j * nthreads;
            if (e < items) {
                const uint32_t vox = nch > 1 ? __umulhi(e, t.m_ch) : e;
                uint32_t* dst = buf + vox * t.vstride + (e - vox * nch) * (2 * WC);
                if constexpr (WC == 2) *reinterpret_cast<uint4*>(dst) = r[j];
                else *reinterpret_cast<uint2*>(dst) = make_uint2(r[j].x, r[j].y);
            }
        }
    };

    // ---- this wave's voxels inside a tile, and its walk over the taps -------------------------
    const int nsp = t.nwx * t.nwy * t.nwz;
    const int wx = wave % t.nwx;
    const int wy = (wave / t.nwx) % t.nwy;
    const int wz = (wave / (t.nwx * t.nwy)) % t.nwz;
    const int wch = wave / nsp;
    const int lx = lane & (LX - 1), ly = (lane >> t.lxb) & (LY - 1);
    const int lz = lane >> (t.lxb + t.lyb);
    const int row_words = t.hx * t.vstride;
    const int plane_words = t.hy * row_words;
    const int lane_base = ((wz * LZ + lz) * p.sd) * plane_words + (wy * LY + ly) * p.sh * row_words +
                          (wx * LX + lx) * p.sw * t.vstride;
    const int T = p.kd * p.kh * p.kw;
    const int co_begin = wch * t.co_per_wave;
    const int co_end = min(p.c_out, co_begin + t.co_per_wave);
    const int nsteps = T * t.nchunk;
    StepConsts sc;
    sc.kw = p.kw; sc.kh = p.kh; sc.nchunk = t.nchunk;
    const int inc_c = p.dw * t.vstride;
    const int inc_b = p.dh * row_words - (p.kw - 1) * inc_c;
    const int inc_a = p.dd * plane_words - (p.kh - 1) * p.dh * row_words - (p.kw - 1) * inc_c;
    using GT = GroupType<WC, CO_BLK, BIN>;
    constexpr int CW = GT::CW;
    constexpr int KG = GT::KG;
    sc.step_words = p.co_pad * CW;
    sc.vstep = 0;
    sc.slots = 0; sc.shift = 0;
    sc.slot_mask = 0xffffffffu;
    sc.tap_end = T;

    uint4 r[NI];
    Origin here = origin_of(first);
    load_items(here, r);
    store_items(lds, r);
    __syncthreads();

    for (int tile = first, b = 0; tile < last; ++tile, b ^= 1) {
        const bool more = tile + 1 < last;
        Origin next = here;
        if (more) {
            next = origin_of(tile + 1);
            load_items(next, r);
        }
        __builtin_amdgcn_sched_barrier(0);
        const uint32_t* lane_lds = lds + b * buf_words + lane_base;
        const int ox = here.ox0 + wx * LX + lx;
        const int oy = here.oy0 + wy * LY + ly;
        const int oz = here.oz0 + wz * LZ + lz;

        uint32_t pos_w[V] = {0u}, neg_w[V] = {0u};
        for (int cb = co_begin; cb < co_end; cb += CO_BLK) {
            int32_t d[V][CO_BLK];
            {
                int32_t acc_m[V][CO_BLK], acc_n[V][CO_BLK];
                int32_t acc2_m[1][1], acc2_n[1][1];
                int32_t cnt[V] = {0};
                scalar_ptr wcur = (scalar_ptr)(uintptr_t)p.wgt + (size_t)cb * CW;
                typename GT::type g0, g1;
                StepCursor cur = {0, 0, 0, 0, 0};
                ActChunk<WC> Aa[V], Ab[V];
                fetch_step<WC, V, false>(Aa, cur, sc, inc_c, inc_b, inc_a, lane_lds, false);
                load_wgroup<WC, KG>(g0, wcur);
                int step = 1;
                conv_step<WC, V, CO_BLK, false, false, BIN, true>(Aa, Ab, step == nsteps, cur, sc, inc_c, inc_b,
                                                                  inc_a, g0, g1, wcur, lane_lds, acc_m, acc_n,
                                                                  acc2_m, acc2_n, cnt);
                for (; step + 2 <= nsteps; step += 2) {
                    conv_step<WC, V, CO_BLK, false, false, BIN>(Ab, Aa, false, cur, sc, inc_c, inc_b, inc_a, g0, g1,
                                                                wcur, lane_lds, acc_m, acc_n, acc2_m, acc2_n, cnt);
                    conv_step<WC, V, CO_BLK, false, false, BIN>(Aa, Ab, step + 2 == nsteps, cur, sc, inc_c, inc_b,
                                                                inc_a, g0, g1, wcur, lane_lds, acc_m, acc_n, acc2_m,
                                                                acc2_n, cnt);
                }
                if (step < nsteps)
                    conv_step<WC, V, CO_BLK, false, false, BIN>(Ab, Aa, true, cur, sc, inc_c, inc_b, inc_a, g0, g1,
                                                                wcur, lane_lds, acc_m, acc_n, acc2_m, acc2_n, cnt);
#pragma unroll
                for (int j = 0; j < CO_BLK; ++j) {
                    if constexpr (BIN) d[0][j] = cnt[0] - 2 * acc_n[0][j];
                    else d[0][j] = acc_m[0][j] - 2 * acc_n[0][j];
                }
            }
            finish_pass<V, CO_BLK, PACKED>(d, p, t, cb, co_begin, co_end, here.n, ox, oy, oz, LY, pos_w, neg_w);
        }
        if (more) {
            // the other buffer was last read before the barrier that ended the previous tile
            store_items(lds + (b ^ 1) * buf_words, r);
            __syncthreads();
        }
        here = next;
    }
}

template <int WC, int V, int CO_BLK, bool PACKED, bool TP, bool DIG = false, bool BIN = false>
int launch_variant(const ConvParams& p, const TileParams& t, size_t lds_bytes, dim3 grid,
                   int threads, hipStream_t s)
{
    auto kern = conv_tiled_kernel<WC, V, CO_BLK, PACKED, TP, DIG, BIN>;
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

// Tuning overrides (tern_set_option).  Per host thread: a launch decision reads only values its
// own thread has set, so no other thread can change the plan in the middle of it.
thread_local int g_lane_depth = 0;   // 0 = choose, 1, 2 or 4 = force that voxel depth per lane
thread_local int g_waves_z = 0;      // 0 = choose, else waves stacked along z per workgroup
thread_local int g_co_block = 0;     // 0 = choose, 16 or 32 = channels per accumulation pass
thread_local int g_co_per_wave = 0;  // 0 = choose, else channels per wave (multiple of 16)
thread_local int g_tap_split = 0;    // 0 = choose, else waves sharing the taps of one slice
thread_local int g_point = 1;        // 0 = never use the pointwise kernel
thread_local int g_lane_tile = 0;    // 0 = choose, else 100 * LX + LY lanes of a wave along x and y
thread_local int g_stream = 0;       // 1 = persistent workgroups with prefetched halo tiles where they apply
// plan of this thread's most recent convolution launch (tern_last_launch)
thread_local int32_t g_last[8] = {-1, 0, 0, 0, 0, 0, 0, 0};
void note_launch(int kind, int v, int cb, int nks, int threads, unsigned gx, unsigned gy, size_t lds)
{
    g_last[0] = kind; g_last[1] = v; g_last[2] = cb; g_last[3] = nks; g_last[4] = threads;
    g_last[5] = (int32_t)gx; g_last[6] = (int32_t)gy; g_last[7] = (int32_t)lds;
}

// Tile plan for a voxel depth V per lane and a wave of 2^lxb x 2^lyb x (64 / 2^(lxb + lyb)) lanes;
// returns false if no halo tile fits in LDS.  Single-plane outputs need lxb + lyb = 6.
bool plan_tiles(const ConvParams& p, int V, int lds_limit, TileParams& t, int64_t& lds_bytes,
                int lxb = 3, int lyb = 3)
{
    const int wd = p.wd_in;
    const int LX = 1 << lxb, LY = 1 << lyb, LZ = 64 >> (lxb + lyb);
    t.lxb = lxb; t.lyb = lyb; t.flat = 1;
    if (p.od == 1 && LZ != 1) return false;
    t.nchunk = wd / p.wc;
    t.vstride = 2 * wd + (wd >= 4 ? 4 : 0);
    t.nwx = 1; t.nwy = 1; t.nwz = g_waves_z > 0 ? g_waves_z : 1;
    // one voxel per lane: two waves share a halo tile from the start (along z, or along y for
    // single-plane outputs), which gives the same tile as one wave with two voxels per lane
    // (not for stacks of independent planes, kd = 1 with several output planes: stacking shares
    // nothing there and only makes workgroups coarser; measured 7-8 % slower on the 2-D layers
    // of a batch of 16)
    if (V == 1 && g_waves_z == 0) {
        if (p.od == 1) t.nwy = 2;
        else if (p.kd > 1) t.nwz = 2;
    }
    // Single-plane outputs (2-D convolutions): a lane's V voxels go along y instead of z.
    t.vy = p.od == 1 ? 1 : 0;
    const int vyx = t.vy ? V : 1, vzx = t.vy ? 1 : V * LZ;
    auto halo = [](int tiles_out, int stride, int k, int dil) { return (tiles_out - 1) * stride + (k - 1) * dil + 1; };
    auto lds_for = [&](const TileParams& q) {
        const int64_t hx = halo(LX * q.nwx, p.sw, p.kw, p.dw);
        const int64_t hy = halo(LY * vyx * q.nwy, p.sh, p.kh, p.dh);
        const int64_t hz = halo(vzx * q.nwz, p.sd, p.kd, p.dd);
        return hx * hy * hz * q.vstride * 4;
    };
    // Start from one wave per workgroup; grow the tile (stacking waves along the axis that
    // lowers LDS per wave the most) while the per-wave LDS share is too large for the waves a
    // compute unit is expected to hold: eight (20 KB each of the 160 KB) on a large problem,
    // fewer on a small one, where small tiles matter more because they give more workgroups.
    const int64_t waves1 = (int64_t)cdiv(p.ow, LX) * cdiv(p.oh, LY * vyx) * cdiv(p.od, vzx) * p.n * cdiv(p.c_out, 16);
    int per_cu = (int)((waves1 + 255) / 256);
    per_cu = per_cu < 1 ? 1 : (per_cu > 8 ? 8 : per_cu);
    const int64_t share_budget = (int64_t)(160 * 1024) / per_cu;
    for (int it = 0; it < 6; ++it) {
        const int waves = t.nwx * t.nwy * t.nwz;
        if (lds_for(t) <= (int64_t)waves * share_budget || waves >= 8) break;
        TileParams best = t;
        double best_share = 1e30;
        TileParams cand[3] = {t, t, t};
        cand[0].nwz *= 2; cand[1].nwy *= 2; cand[2].nwx *= 2;
        for (const TileParams& c : cand) {
            if (c.nwz != t.nwz && vzx * t.nwz >= p.od) continue;   // no planes left to stack
            if (lds_for(c) > lds_limit) continue;                  // would not fit at all
            const double share = (double)lds_for(c) / (c.nwx * c.nwy * c.nwz);
            if (share < best_share) { best_share = share; best = c; }
        }
        if (best_share == 1e30) break;   // nothing larger fits: keep what we have
        t = best;
    }
    lds_bytes = lds_for(t);
    if (lds_bytes > lds_limit) return false;
    t.hx = halo(LX * t.nwx, p.sw, p.kw, p.dw);
    t.hy = halo(LY * vyx * t.nwy, p.sh, p.kh, p.dh);
    t.hz = halo(vzx * t.nwz, p.sd, p.kd, p.dd);
    t.tiles_x = cdiv(p.ow, LX * t.nwx);
    t.tiles_y = cdiv(p.oh, LY * vyx * t.nwy);
    t.tiles_z = cdiv(p.od, vzx * t.nwz);
    t.m_hx = 0xffffffffu / (uint32_t)t.hx + 1u;
    t.m_pl = 0xffffffffu / (uint32_t)(t.hx * t.hy) + 1u;
    t.m_ch = t.nchunk > 1 ? 0xffffffffu / (uint32_t)t.nchunk + 1u : 0u;
    return true;
}

}  // namespace

void set_lane_depth(int v) { g_lane_depth = (v == 1 || v == 2 || v == 4) ? v : 0; }
void set_waves_z(int v) { g_waves_z = (v == 1 || v == 2 || v == 4 || v == 8) ? v : 0; }
void set_co_block(int v) { g_co_block = (v == 8 || v == 16 || v == 32) ? v : 0; }
void set_co_per_wave(int v) { g_co_per_wave = (v > 0 && v % 16 == 0) ? v : 0; }
void set_tap_split(int v) { g_tap_split = (v == 1 || v == 2 || v == 4 || v == 8) ? v : 0; }
void set_pointwise(int v) { g_point = v ? 1 : 0; }
void set_lane_tile(int v) { g_lane_tile = v; }
void set_stream(int v) { g_stream = v ? 1 : 0; }
void last_launch(int32_t* info) { for (int i = 0; i < 8; ++i) info[i] = g_last[i]; }

int launch_conv3d(const ConvParams& p_in, hipStream_t s)
{
    if (g_point && !p_in.digits && !p_in.binary && conv_point_applies(p_in)) {
        note_launch(TERN_KERNEL_POINTWISE, 0, 0, 0, 0, 0, 0, 0);
        return launch_conv_point(p_in, s);
    }
    ConvParams p = p_in;
    const bool packed = p.out_packed != nullptr;
    // A kernel of depth extent 1 with unit depth stride and no depth padding treats every input
    // plane by itself, so batch items are just more planes: [N][D] collapses to [1][N*D] and
    // planes of different batch items share tiles (stacks of 2-D slices have D = 1).  Packed
    // output only: the int32 layout has the channel axis between N and D.
    if (packed && p.n > 1 && p.kd == 1 && p.sd == 1 && p.pd == 0 && (int64_t)p.n * p.d <= INT32_MAX) {
        p.d *= p.n;
        p.od *= p.n;
        p.n = 1;
    }
    // A single tap with unit stride and no padding looks at no neighbour at all: the volume is
    // a flat list of voxels.  Laid out as rows of 8 it makes every wave's 8 x 16 tile one
    // contiguous run of 128 voxels, so the halo fill and the stores stream instead of touching
    // 64-byte pieces of many rows.
    if (p.kd * p.kh * p.kw == 1 && p.sd == 1 && p.sh == 1 && p.sw == 1 && p.pd == 0 && p.ph == 0 &&
        p.pw == 0) {
        const int64_t vox = (int64_t)p.d * p.h * p.w;
        if (vox % 8 == 0) {
            p.d = p.od = 1;
            p.h = p.oh = (int32_t)(vox / 8);
            p.w = p.ow = 8;
        }
    }
    const int lds_limit = lds_limit_for_current_device();

    // Kernel variants: voxels per lane V x channels per pass CO_BLK = accumulator pairs per lane.
    //   V=1, CO_BLK=32  (64 pairs, five waves per SIMD): large launches;
    //   V=1 or 2, CO_BLK=16  (32 or 64 pairs): smaller launches, the finest work split;
    //   V=2, CO_BLK=32  (128 pairs, three waves per SIMD): tap-packed layers and few-step kernels;
    //   V=4, CO_BLK=16: half the scalar-cache traffic per instruction (tuning option only).
    // One voxel per lane where a wave still has enough steps to amortise its fixed cost (not
    // the tap-packed layers, whose step set-up is per voxel): half the accumulators, so more
    // waves fit a SIMD (five instead of three with 32 channels per pass), and waves half as
    // long, which shortens the end of the launch where SIMDs run out of waves one by one.
    // Measured against two voxels per lane: +1-2 % on 64- and 32-cubed volumes of 64-256
    // channels, +5 % on 96-cubed ones, up to +10 % with int32 output, +30 % on 512-channel 2-D
    // modules; -3 % with only 9 steps per wave, hence the step limit.
    const int steps_all = p.kd * p.kh * p.kw * (p.wd_in / p.wc);
    auto lane_depth_for = [&](int cb) {
        const bool exists = p.tp_slots == 0 && (p.wc == 2 || cb == 32 || cb == 8);
        // (8 channels per pass: two voxels per lane unless told otherwise, measured faster on
        // every small launch tried but one)
        return (exists && (g_lane_depth == 1 || (g_lane_depth == 0 && steps_all >= 16 && cb != 8))) ? 1 : 2;
    };
    // Estimated launch time in vector instructions of the busiest SIMD, for cb channels per pass
    // and the kernel taps split over ks waves: workgroups are dealt to the 256 compute units
    // whole, a unit's waves spread over its four SIMDs, and a wave costs its share of the
    // contraction, its epilogue, about 560 fixed instructions and, with split taps, the exchange
    // of partial sums.
    auto estimate = [&](int cb, int ks) -> double {
        const int v = lane_depth_for(cb);
        TileParams q;
        int64_t bytes = 0;
        if (!plan_tiles(p, v, lds_limit, q, bytes)) return 1e300;
        const int nsp = q.nwx * q.nwy * q.nwz;
        if (nsp * ks > 8 || steps_all < 4 * ks) return 1e300;
        const int slices = cdiv(p.c_out, cb);
        int nwc = 8 / (nsp * ks);
        if (nwc > slices) nwc = slices;
        if (nwc < 1) nwc = 1;
        const double wgs = (double)q.tiles_x * q.tiles_y * q.tiles_z * p.n * cdiv(slices, nwc);
        const double per_wave = (double)steps_all / ks * cb * p.wc * v * (p.binary ? 2 : 4) + 5.0 * v * cb + 560.0 +
                                (ks > 1 ? 2.0 * (ks - 1) * v * cb + 300.0 : 0.0);
        // waves of the fullest compute unit, spread over its four SIMDs
        const double per_simd = std::ceil(std::ceil(wgs / 256.0) * (nsp * nwc * ks) / 4.0);
        // penalty for SIMDs with few waves.  The weights were the issue efficiency measured for
        // one, two, three and four or more waves before the word-pair sequence was spaced by hand
        // (it now loses less with few waves); they are kept because the choices they lead to
        // still measure best on the mid-size layers tried (the gentler weights 0.89 / 0.95 /
        // 0.98 / 1.0 picked a 50 % slower launch for 64 -> 64 channels on 32^3)
        const double eff = per_simd <= 1 ? 0.78 : per_simd <= 2 ? 0.90 : per_simd <= 3 ? 0.93 : 0.95;
        return per_simd * per_wave / eff;
    };
    int nks_pref = 0;   // tap split chosen together with the pass width (0: decided further down)
    int V = 2, co_blk = 16;
    if (g_lane_depth == 4 && p.tp_slots == 0) { V = 4; co_blk = 16; }
    else if (g_co_block == 32) { V = 2; co_blk = 32; }
    else if (g_co_block == 8 && p.tp_slots == 0 && !p.digits && !p.binary) { co_blk = 8; }
    else if (g_co_block == 0) {
        const int64_t tiles2 = p.od == 1 ? (int64_t)cdiv(p.ow, 8) * cdiv(p.oh, 16) * p.n
                                         : (int64_t)cdiv(p.ow, 8) * cdiv(p.oh, 8) * cdiv(p.od, 2) * p.n;
        const int tail = p.c_out % 32;   // a 32-channel pass over 1..16 live channels is half wasted
        const int64_t units = tiles2 * cdiv(p.c_out, 32);
        // large launches: 32 channels per pass (half the passes over the LDS tile, half the fixed
        // cost); tiny ones: 16 (they need every wave they can get and split the taps besides);
        // in between the two differ in how evenly the workgroups fill the chip: estimate both
        // the smallest launches (fewer 16-channel slices of two-voxel tiles than SIMDs): 8 channels
        // per pass.  They split the kernel taps over several waves anyway, and the partial sums
        // that those waves exchange through LDS shrink with the pass width: twice the slices at
        // half the split measured 8-23 % faster (24^3 x 32 channels 9.2 -> 7.1 us, 64 -> 128
        // channels on 16 x 16 x 8 outputs 9.2 -> 7.6 us, the layers between 3-6 %).
        if (tiles2 * cdiv(p.c_out, 16) < 1024 && p.tp_slots == 0 && !p.digits && !p.binary) {
            co_blk = 8;
        } else if (units >= 4096) {
            if (tail == 0 || tail > 16) co_blk = 32;
        } else if (units >= 512 && p.tp_slots == 0) {
            double best = 1e300;
            for (int cb = 16; cb <= 32; cb += 16) {
                if (cb == 32 && !(tail == 0 || tail > 16)) continue;
                for (int ks = 1; ks <= 2; ++ks) {
                    if (g_tap_split > 0 && ks != g_tap_split) continue;
                    const double e = estimate(cb, ks);
                    if (e < best) { best = e; co_blk = cb; nks_pref = ks; }
                }
            }
        }
    }
    if (V == 2) V = lane_depth_for(co_blk);
    if (p.digits) V = 1;   // the only variant built for two-digit inputs
    if (p.binary && V == 4) V = 2;   // binary filters: one or two voxels per lane
    // Shape of a wave's 64 output voxels.  8 x 8 in a plane by default.  Stacks of independent
    // planes (kd = 1) start from 4 x 8 in two planes instead (measured equal to 9 % faster than
    // 8 x 8 on the 2-D layers of a batch of 16, never slower).  Where the extents leave much of
    // the last tile of a row or column empty, a smaller footprint over more planes (8 x 4 x 2,
    // 4 x 4 x 4, and for plane stacks also 2 x 8 x 4, ...) wastes fewer lanes at the price of a
    // larger halo per output: 4-14 % faster on 3-D volumes of 100, 44 and 20 voxels per axis, no
    // difference where 8 x 8 tiles fit.  Estimate: word-pair instructions of all waves plus about
    // 32 instructions per halo item staged; another shape has to beat the starting one by 3 %.
    int lxb = 3, lyb = 3;
    if (p.od > 1 && g_lane_tile > 0) {
        const int lx = g_lane_tile / 100, ly = g_lane_tile % 100;
        for (int a = 0; a < 4; ++a)
            for (int b = 0; b < 4; ++b)
                if ((1 << a) == lx && (1 << b) == ly && a + b >= 2) { lxb = a; lyb = b; }
    } else if (p.od > 1 && g_lane_tile == 0 && p.tp_slots == 0) {
        const bool planes = p.kd == 1;   // independent planes
        auto score = [&](int a, int b) -> double {
            TileParams q;
            int64_t bytes = 0;
            if (!plan_tiles(p, V, lds_limit, q, bytes, a, b)) return 1e300;
            const int nsp = q.nwx * q.nwy * q.nwz;
            if (nsp > 8) return 1e300;
            const int slices = cdiv(p.c_out, co_blk);
            int nwc = 4 / nsp < 1 ? 1 : 4 / nsp;
            if (nwc > slices) nwc = slices;
            const double tiles = (double)q.tiles_x * q.tiles_y * q.tiles_z * p.n;
            const double mac = tiles * nsp * steps_all * p.wc * 4.0 * V * slices * co_blk;
            const double fill = tiles * cdiv(slices, nwc) * ((double)q.hx * q.hy * q.hz * q.nchunk / 64.0) * 32.0;
            return mac + fill;
        };
        double best = planes ? score(2, 3) : score(3, 3);
        if (best < 1e300) {
            if (planes) { lxb = 2; lyb = 3; }
            best *= 0.97;
        }
        for (int a = planes ? 0 : 2; a < 4; ++a)
            for (int b = planes ? 0 : 2; b < 4; ++b) {
                if (a + b < 2 || (a == lxb && b == lyb)) continue;
                const double e = score(a, b);
                if (e < best) { best = e; lxb = a; lyb = b; }
            }
    }
    TileParams t;
    int64_t lds_bytes = 0;
    if (!plan_tiles(p, V, lds_limit, t, lds_bytes, lxb, lyb)) {
        if (V == 4 && plan_tiles(p, 2, lds_limit, t, lds_bytes, lxb, lyb)) V = 2;
        else {
            note_launch(TERN_KERNEL_DIRECT, 0, 0, 0, 0, 0, 0, 0);
            return launch_conv3d_generic(p, s);
        }
    }
    const int64_t spatial_tiles = (int64_t)t.tiles_x * t.tiles_y * t.tiles_z * p.n;
    if (spatial_tiles > 0x7fffffff) return TERN_ESHAPE;
    // Output channels are cut into slices of co_per_wave (one accumulation pass by default:
    // many short waves keep every SIMD supplied with several resident waves, and a single wave
    // cannot issue a vector instruction every cycle by itself).  Up to 8 waves of one workgroup
    // take consecutive slices of the same spatial tile and share its LDS halo; further slices
    // go to blockIdx.y.
    const int nsp = t.nwx * t.nwy * t.nwz;
    int co_per_wave = g_co_per_wave > 0 ? g_co_per_wave : co_blk;
    co_per_wave = cdiv(co_per_wave, co_blk) * co_blk;
    int slices = cdiv(p.c_out, co_per_wave);

    // Small problems: when even 16-channel slices leave most SIMDs without a wave, the kernel
    // taps of one (tile, slice) are split over nks waves of the same workgroup, which add their
    // partial sums through LDS.
    const bool tp = p.tp_slots > 0;
    const int T = p.kd * p.kh * p.kw;
    const int nsteps = tp ? cdiv(T, p.tp_slots) : T * t.nchunk;
    int nks = 1;
    if (g_tap_split > 0) nks = g_tap_split;
    else if (nks_pref > 0) nks = nks_pref;
    else {
        const int64_t waves0 = spatial_tiles * nsp * slices;
        // double the split while that keeps the launch within two waves per SIMD
        while (nks * 2 * nsp <= 8 && waves0 * nks * 2 <= 2048 && nsteps >= 4 * nks) nks *= 2;
    }
    if (nks * nsp > 8) nks = 8 / nsp;
    if (nks < 1) nks = 1;
    if (nks > 1) { co_per_wave = co_blk; slices = cdiv(p.c_out, co_per_wave); }
    int nwc = 8 / (nsp * nks);
    if (nwc > slices) nwc = slices;
    // Large launches: workgroups of four waves rather than eight.  Sharing a halo tile between
    // more channel slices saves fills, but coarser workgroups fill the chip less evenly; measured
    // equal on 3-D layers and 8 % faster on the large 2-D layers of a batch of 16.
    if (nks == 1 && spatial_tiles * nsp * slices >= 4096 && nsp * nwc > 4) nwc = 4 / nsp;
    if (nwc < 1) nwc = 1;
    t.nwc = nwc;
    t.co_per_wave = co_per_wave;
    t.nks = nks;
    t.red_off = (int32_t)(lds_bytes / 4);
    if (nks > 1) {
        lds_bytes += (int64_t)(nks - 1) * nsp * nwc * V * co_blk * 64 * 4;
        if (lds_bytes > lds_limit) {   // no room for the partial sums: do without the split
            lds_bytes = (int64_t)t.red_off * 4;
            t.nks = nks = 1;
            t.nwc = nwc = (8 / nsp < slices) ? 8 / nsp : slices;
        }
    }
    const int grid_y = cdiv(slices, nwc);
    if (grid_y > 65535) return TERN_ESHAPE;

    const dim3 grid((unsigned)spatial_tiles, (unsigned)grid_y);
    const int threads = 64 * nsp * nwc * nks;
    // Halo fill: per plane position (a thread fetches up to 8 planes of one position and chunk
    // per round trip) for tiles of 4 planes or more, else over one flat index space.  Wave shapes
    // with a small footprint have few positions per plane: they take whichever needs fewer trips.
    t.flat = t.hz < 4 ? 1 : 0;
    if (!(lxb == 3 && lyb == 3) && !t.flat) {
        const int plane = t.hx * t.hy;
        const int64_t deep_trips = (int64_t)cdiv(plane, threads) * t.nchunk * cdiv(t.hz, 8);
        const int64_t flat_trips = ((int64_t)t.hz * plane * t.nchunk + 8 * threads - 1) / (8 * threads);
        if (flat_trips < deep_trips) t.flat = 1;
    }
    const size_t lb = (size_t)lds_bytes;
    // Persistent form: four-wave workgroups, one per (SIMD, wave slot) of the chip, each walking
    // a run of tiles with the next halo tile prefetched under the current tile's arithmetic.
    if (g_stream && V == 1 && co_blk == 32 && !tp && !p.digits && nks == 1 && grid_y == 1 && threads == 256 &&
        (int64_t)t.hx * t.hy * t.hz * t.nchunk <= (int64_t)kStreamItems * threads && 2 * lds_bytes <= 64 * 1024) {
        const int resident = 4 * compute_units_of_current_device();
        if (resident > 0 && spatial_tiles >= 2 * (int64_t)resident) {
            t.tiles_per_wg = (int32_t)((spatial_tiles + resident - 1) / resident);
            const unsigned wgs = (unsigned)((spatial_tiles + t.tiles_per_wg - 1) / t.tiles_per_wg);
            // at least a fifth of a compute unit's LDS per workgroup, so that no unit takes five
            size_t sb = 2 * lb;
            if (sb < 33 * 1024) sb = 33 * 1024;
#define TERN_LAUNCH_S(WC_, BIN_)                                                                          \
    do {                                                                                                  \
        if (packed) hipLaunchKernelGGL((conv_tiled_stream_kernel<WC_, 32, true, BIN_>), dim3(wgs), dim3(threads), sb, s, p, t);   \
        else hipLaunchKernelGGL((conv_tiled_stream_kernel<WC_, 32, false, BIN_>), dim3(wgs), dim3(threads), sb, s, p, t);        \
    } while (0)
            if (p.binary) { if (p.wc == 2) TERN_LAUNCH_S(2, true); else TERN_LAUNCH_S(1, true); }
            else { if (p.wc == 2) TERN_LAUNCH_S(2, false); else TERN_LAUNCH_S(1, false); }
#undef TERN_LAUNCH_S
            TERN_HIP_CHECK(hipGetLastError());
            note_launch(TERN_KERNEL_PERSISTENT, 1, 32, 1, threads, wgs, 1, sb);
            return TERN_OK;
        }
    }
    note_launch(TERN_KERNEL_TILED, V, co_blk, nks, threads, grid.x, grid.y, lb);
#define TERN_LAUNCH(WC_, V_, CB_, TP_)                                                       \
    (packed ? launch_variant<WC_, V_, CB_, true, TP_>(p, t, lb, grid, threads, s)            \
            : launch_variant<WC_, V_, CB_, false, TP_>(p, t, lb, grid, threads, s))
    if (p.digits) {   // two-digit input: one voxel per lane, two accumulator sets
        if (co_blk == 32)
            return packed ? launch_variant<2, 1, 32, true, false, true>(p, t, lb, grid, threads, s)
                          : launch_variant<2, 1, 32, false, false, true>(p, t, lb, grid, threads, s);
        return packed ? launch_variant<2, 1, 16, true, false, true>(p, t, lb, grid, threads, s)
                      : launch_variant<2, 1, 16, false, false, true>(p, t, lb, grid, threads, s);
    }
    if (p.binary) {   // Eq. 8: sign-only filter bank, two instructions per word pair
#define TERN_LAUNCH_B(WC_, V_, CB_)                                                                     \
    (packed ? launch_variant<WC_, V_, CB_, true, false, false, true>(p, t, lb, grid, threads, s)       \
            : launch_variant<WC_, V_, CB_, false, false, false, true>(p, t, lb, grid, threads, s))
        if (p.wc == 2) {
            if (V == 1) return co_blk == 32 ? TERN_LAUNCH_B(2, 1, 32) : TERN_LAUNCH_B(2, 1, 16);
            return co_blk == 32 ? TERN_LAUNCH_B(2, 2, 32) : TERN_LAUNCH_B(2, 2, 16);
        }
        if (V == 1) return TERN_LAUNCH_B(1, 1, 32);
        return co_blk == 32 ? TERN_LAUNCH_B(1, 2, 32) : TERN_LAUNCH_B(1, 2, 16);
#undef TERN_LAUNCH_B
    }
    if (tp) return co_blk == 32 ? TERN_LAUNCH(1, 2, 32, true) : TERN_LAUNCH(1, 2, 16, true);
    if (co_blk == 8) {   // the finest channel slices: small launches
        if (V == 4) V = 2;
        if (p.wc == 2) return V == 1 ? TERN_LAUNCH(2, 1, 8, false) : TERN_LAUNCH(2, 2, 8, false);
        return V == 1 ? TERN_LAUNCH(1, 1, 8, false) : TERN_LAUNCH(1, 2, 8, false);
    }
    if (p.wc == 2) {
        if (V == 1) return co_blk == 32 ? TERN_LAUNCH(2, 1, 32, false) : TERN_LAUNCH(2, 1, 16, false);
        if (V == 4) return TERN_LAUNCH(2, 4, 16, false);
        return co_blk == 32 ? TERN_LAUNCH(2, 2, 32, false) : TERN_LAUNCH(2, 2, 16, false);
    }
    if (V == 4) return TERN_LAUNCH(1, 4, 16, false);
    if (V == 1) return TERN_LAUNCH(1, 1, 32, false);
    return co_blk == 32 ? TERN_LAUNCH(1, 2, 32, false) : TERN_LAUNCH(1, 2, 16, false);
#undef TERN_LAUNCH
}

}  // namespace tern
