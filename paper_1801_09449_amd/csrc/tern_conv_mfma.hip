// Ternary convolution on the matrix cores: the inner product of section 2 (the quantity that
// Eq. 9 evaluates with two bit-counts) computed as a matrix product.  Activations stay in the
// packed two-plane layout in HBM; a workgroup expands its halo tile in LDS, one inner step at a
// time, and contracts it with an expanded filter bank.  Two kinds:
//   int8: one byte per code, a step is a word of 32 channels, v_mfma_i32_32x32x32_i8, int32 sums;
//   fp4:  four bits per code (E2M1: +1 = 0010, -1 = 1010), a step is a pair of words,
//         v_mfma_scale_f32_32x32x64_f8f6f4 with both scales 2^0, float sums, exact because every
//         partial sum is an integer below 2^24 (checked on the host); twice the rate.
// Same results as the bit-count kernels, bit for bit.  The fp4 kind also takes the two-digit tensors
// of tern_pool_digits (window sums -4 .. 4 as low + 3 * high): every such sum is an E2M1 value, so
// the staging turns a digit pair into the sum's code and the contraction is that of the pooled
// tensor with the layer's own weights.
//
// Implicit matrix product: rows = output voxels, columns = output channels, inner index =
// (kernel tap, input channel).  A wave owns 8 x 8 x 2 output voxels (four row blocks of 32:
// plane p in {0, 1} x y-half h in {0, 1}, voxel i of a block at x = i % 8, y = 4 h + i / 8; for a
// single output plane 8 x 16 x 1, the row blocks being its four y-quarters) and up
// to 64 output channels (two column blocks), i.e. eight 32 x 32 accumulator tiles; up to four
// waves stacked along z share a halo tile.  Per (tap, step) a wave reads four row fragments from
// LDS (one 16-byte read per lane each) and two column fragments from the filter bank (16 bytes
// per lane, 1 KB contiguous per fragment, served by the vector cache) and issues eight matrix
// instructions: LDS at half and the vector cache at half of what they can deliver.
//
// Operand layout of the instructions (two lane groups x 16 bytes of inner indices): lane l of
// the row operand holds row l % 32, lane l of the column operand holds column l % 32, and both
// hold the inner indices of lane group l / 32 in the same order, so any consistent assignment
// of channels to (lane group, position) gives the right sum; the one used is whatever makes the
// 2-bit -> operand expansion cheapest (see expand_word, expand_word_f4).  Result: lane l holds
// column l % 32, register v holds row 8 (v / 4) + 4 (l / 32) + v % 4.
#include <type_traits>

#include "tern_internal.h"

namespace tern {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kMaxWaves = 4;         // waves per workgroup (4, 2 or 1), stacked along z
constexpr int kMaxThreads = 64 * kMaxWaves;
constexpr int kTX = 8;               // output voxels per wave: 8 x 8 x 2 planes, or 8 x 16 of a single plane
// LDS tile: the two 16-byte halves of a halo voxel's 32 bytes (the row-fragment halves that lane
// groups 0 and 1 read) live in two regions, voxel records 16 bytes apart in each, the second
// region at an offset that is 64 modulo 128: eight lanes with neighbouring voxels read 128
// contiguous bytes, and four lanes of each group together read two runs of 64 bytes in
// different banks.  (Same speed as 48-byte records holding both halves, two thirds of the LDS.)
constexpr int kRec = 16;
inline int64_t half_offset(int64_t nvox) { return (nvox * kRec + 127) / 128 * 128 + 64; }
constexpr int kFill = 4;             // halo items a thread keeps in flight

struct MfmaPlan {
    int32_t hx, hy, hz;              // halo extents in voxels
    int32_t tiles_x, tiles_y, tiles_z;
    int32_t nblk;                    // 32-channel column blocks in the filter bank
    int32_t ksteps;                  // inner steps per tap: channel words (int8) or word pairs (fp4)
    uint32_t m_hx, m_pl;             // floor(e / hx) = umulhi(e, m_hx), likewise hx * hy
    int32_t half_off;                // LDS byte offset of the second region
    int32_t flat;                    // 1: single-plane output, a wave's four row blocks are y-quarters of 8 x 16
};

// The inner index of the matrix product may be laid out in any order that row and column operands
// share, so the expansions pick the order that costs the fewest instructions: bits are masked
// where they stand instead of being gathered.
//
// One byte per code from a word of 32 channels: +1 -> 0x01, -1 -> 0xff, 0 -> 0x00.  Dword d
// (0..7; lane group d / 4 reads dwords 4 (d / 4) .. + 3) holds channels d, d + 8, d + 16, d + 24 in
// its bytes 0..3: (m >> d) & 0x01010101 is their magnitude byte, and 0xfe times the same of the
// negative codes turns 0x01 into 0xff.
__device__ __forceinline__ void expand_word(uint32_t m, uint32_t s, uint4& lo16, uint4& hi16)
{
    const uint32_t neg = m & s;
    uint32_t o[8];
#pragma unroll
    for (int d = 0; d < 8; ++d)
        o[d] = ((m >> d) & 0x01010101u) | (((neg >> d) & 0x01010101u) * 0xfeu);
    lo16 = make_uint4(o[0], o[1], o[2], o[3]);
    hi16 = make_uint4(o[4], o[5], o[6], o[7]);
}

// Four bits per code (the E2M1 format of the scaled matrix instructions: +1 = 0010, -1 = 1010,
// 0 = 0000) from a word of 32 channels.  Dword q (0..3) holds channels q, q + 4, ..., q + 28 in its
// 4-bit fields 0..7: the magnitude bit of channel 4 i + q belongs at bit 4 i + 1 and its sign at
// bit 4 i + 3, a shift by q - 1 and by q - 3 away from where the words have them.
__device__ __forceinline__ uint4 expand_word_f4(uint32_t m, uint32_t s)
{
    const uint32_t neg = m & s;
    uint32_t o[4];
    o[0] = ((m << 1) & 0x22222222u) | ((neg << 3) & 0x88888888u);
    o[1] = (m & 0x22222222u) | ((neg << 2) & 0x88888888u);
    o[2] = ((m >> 1) & 0x22222222u) | ((neg << 1) & 0x88888888u);
    o[3] = ((m >> 2) & 0x22222222u) | (neg & 0x88888888u);
    return make_uint4(o[0], o[1], o[2], o[3]);
}

// Two balanced-ternary digits per value (tern_pool_digits: value = low + 3 * high, -4 .. 4), to the
// E2M1 code of the value (magnitudes 1, 2, 3, 4 = 0010, 0100, 0101, 0110), same field order as
// expand_word_f4.  Bit planes of the code from the digits' masks and signs: the sign is the high
// digit's where that is nonzero, else the low digit's; bit 2 says the high digit is nonzero; with
// it, bit 1 says the low digit has the same sign (3 + 1) and bit 0 that the low digit is zero.
__device__ __forceinline__ uint4 expand_digits_f4(uint32_t lm, uint32_t ls, uint32_t hm, uint32_t hs)
{
    const uint32_t b3 = (hm & hs) | (lm & ls & ~hm);
    const uint32_t b2 = hm;
    const uint32_t b1 = lm & ~(hm & (ls ^ hs));
    const uint32_t b0 = hm & ~lm;
    uint32_t o[4];
    o[0] = (b0 & 0x11111111u) | ((b1 << 1) & 0x22222222u) | ((b2 << 2) & 0x44444444u) | ((b3 << 3) & 0x88888888u);
    o[1] = ((b0 >> 1) & 0x11111111u) | (b1 & 0x22222222u) | ((b2 << 1) & 0x44444444u) | ((b3 << 2) & 0x88888888u);
    o[2] = ((b0 >> 2) & 0x11111111u) | ((b1 >> 1) & 0x22222222u) | (b2 & 0x44444444u) | ((b3 << 1) & 0x88888888u);
    o[3] = ((b0 >> 3) & 0x11111111u) | ((b1 >> 2) & 0x22222222u) | ((b2 >> 1) & 0x44444444u) | (b3 & 0x88888888u);
    return make_uint4(o[0], o[1], o[2], o[3]);
}

// Filter banks, [tap][step][column block][lane group g][column j][16 bytes], in the expansions'
// channel order.  int8 (step = word): byte b of dword q = code of filter 32 * block + j at input
// channel 32 * step + (4 g + q) + 8 b.  fp4 (step = pair of words): 4-bit field i of dword q = code
// at input channel 32 * (2 * step + g) + 4 i + q.  Zero past c_out and c_in.
template <bool F4>
__global__ __launch_bounds__(256) void expand_filters_kernel(const int8_t* __restrict__ w, int32_t c_out,
                                                             int32_t c_in, int32_t taps, int32_t ksteps,
                                                             int32_t nblk, uint32_t* __restrict__ bank,
                                                             int64_t dwords)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= dwords) return;
    const int q = (int)(e & 3);                  // dword within the 16 bytes
    const int j = (int)((e >> 2) & 31);
    const int g = (int)((e >> 7) & 1);
    int64_t r = e >> 8;                          // (tap * ksteps + step) * nblk + block
    const int blk = (int)(r % nblk); r /= nblk;
    const int ks = (int)(r % ksteps);
    const int tap = (int)(r / ksteps);
    const int co = blk * 32 + j;
    uint32_t out = 0u;
    if (co < c_out) {
        constexpr int PER = F4 ? 8 : 4;          // codes per dword
#pragma unroll
        for (int b = 0; b < PER; ++b) {
            const int c = F4 ? (2 * ks + g) * 32 + 4 * b + q : ks * 32 + (4 * g + q) + 8 * b;
            if (c < c_in) {
                const int v = w[((size_t)co * c_in + c) * taps + tap];
                if constexpr (F4) out |= (v > 0 ? 0x2u : v < 0 ? 0xau : 0u) << (4 * b);
                else out |= (v > 0 ? 0x01u : v < 0 ? 0xffu : 0u) << (8 * b);
            }
        }
    }
    bank[e] = out;
}

// Eq. 6 on one 32 x 32 accumulator tile: register V of lane l is (row 8 (V / 4) + 4 (l / 32) +
// V % 4, column l % 32).  A wave-wide comparison gives the 32 channel bits of two rows at once
// (lanes 0-31: row r, lanes 32-63: row r + 4); they go to lanes r and r + 4 of posw / negw.
// Four registers (one group of eight rows) per step: eight comparisons, then their sixteen lane
// writes behind one wait.  Thr is the accumulators' own type (the fp4 route compares floats: its
// sums are exact integers and the cut points are clamped to +-2^24, beyond every sum).
template <int V0, typename Acc, typename Thr>
__device__ __forceinline__ void decide_rows(const Acc& acc, Thr lo, Thr hi, uint32_t& posw, uint32_t& negw)
{
    if constexpr (V0 < 16) {
        constexpr int r = (V0 >> 2) * 8;         // rows r .. r + 3 from lane group 0, r + 4 .. r + 7 from group 1
        unsigned long long bp[4], bn[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            bp[j] = __ballot(acc[V0 + j] > hi);
            bn[j] = __ballot(acc[V0 + j] < lo);
        }
        // The compiler does not see inside the statement: the wait states that a lane write
        // needs after a comparison wrote its scalar result are spelled out.
        asm("s_nop 4\n\t"
            "v_writelane_b32 %[p], %[p0l], %[r0]\n\t"
            "v_writelane_b32 %[p], %[p0h], %[r4]\n\t"
            "v_writelane_b32 %[n], %[n0l], %[r0]\n\t"
            "v_writelane_b32 %[n], %[n0h], %[r4]\n\t"
            "v_writelane_b32 %[p], %[p1l], %[r1]\n\t"
            "v_writelane_b32 %[p], %[p1h], %[r5]\n\t"
            "v_writelane_b32 %[n], %[n1l], %[r1]\n\t"
            "v_writelane_b32 %[n], %[n1h], %[r5]\n\t"
            "v_writelane_b32 %[p], %[p2l], %[r2]\n\t"
            "v_writelane_b32 %[p], %[p2h], %[r6]\n\t"
            "v_writelane_b32 %[n], %[n2l], %[r2]\n\t"
            "v_writelane_b32 %[n], %[n2h], %[r6]\n\t"
            "v_writelane_b32 %[p], %[p3l], %[r3]\n\t"
            "v_writelane_b32 %[p], %[p3h], %[r7]\n\t"
            "v_writelane_b32 %[n], %[n3l], %[r3]\n\t"
            "v_writelane_b32 %[n], %[n3h], %[r7]"
            : [p] "+v"(posw), [n] "+v"(negw)
            : [p0l] "s"((uint32_t)bp[0]), [p0h] "s"((uint32_t)(bp[0] >> 32)), [n0l] "s"((uint32_t)bn[0]),
              [n0h] "s"((uint32_t)(bn[0] >> 32)), [p1l] "s"((uint32_t)bp[1]), [p1h] "s"((uint32_t)(bp[1] >> 32)),
              [n1l] "s"((uint32_t)bn[1]), [n1h] "s"((uint32_t)(bn[1] >> 32)), [p2l] "s"((uint32_t)bp[2]),
              [p2h] "s"((uint32_t)(bp[2] >> 32)), [n2l] "s"((uint32_t)bn[2]), [n2h] "s"((uint32_t)(bn[2] >> 32)),
              [p3l] "s"((uint32_t)bp[3]), [p3h] "s"((uint32_t)(bp[3] >> 32)), [n3l] "s"((uint32_t)bn[3]),
              [n3h] "s"((uint32_t)(bn[3] >> 32)), [r0] "n"(r), [r1] "n"(r + 1), [r2] "n"(r + 2), [r3] "n"(r + 3),
              [r4] "n"(r + 4), [r5] "n"(r + 5), [r6] "n"(r + 6), [r7] "n"(r + 7));
        decide_rows<V0 + 4, Acc, Thr>(acc, lo, hi, posw, negw);
    }
}

template <int NB, bool PACKED, bool F4, bool DIG = false>
__global__ __launch_bounds__(kMaxThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void conv_mfma_kernel(ConvParams p, MfmaPlan t)
{
    extern __shared__ __align__(16) uint8_t lds8[];
    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    int bid = blockIdx.x;
    {   // contiguous runs of tiles per XCD (workgroups go to the 8 XCDs round-robin)
        const int per_xcd = gridDim.x >> 3;
        if (bid < (per_xcd << 3)) bid = (bid & 7) * per_xcd + (bid >> 3);
    }
    const int tix = bid % t.tiles_x; bid /= t.tiles_x;
    const int tiy = bid % t.tiles_y; bid /= t.tiles_y;
    const int tiz = bid % t.tiles_z;
    const int n = bid / t.tiles_z;
    const int flat = t.flat;                     // wave = 8 x 16 x 1 instead of 8 x 8 x 2
    const int wplanes = flat ? 1 : 2;
    const int ox0 = tix * kTX, oy0 = tiy * (flat ? 16 : 8), oz0 = tiz * (nthreads >> 6) * wplanes;
    const int nb0 = blockIdx.y * NB;             // first column block of this workgroup

    const int gx0 = ox0 * p.sw - p.pw, gy0 = oy0 * p.sh - p.ph, gz0 = oz0 * p.sd - p.pd;
    const int plane = t.hx * t.hy;
    const int nvox = plane * t.hz;
    const int wd = p.wd_in;
    const uint32_t* in_n = p.in + (size_t)n * p.d * p.h * p.w * 2u * wd;

    const int i32 = lane & 31, g = lane >> 5;
    const int xl = i32 & 7, yl = i32 >> 3;
    const int row_b = t.hx * kRec, plane_b = t.hy * row_b;
    const int lane_off = (wave * wplanes * p.sd) * plane_b + (yl * p.sh) * row_b + (xl * p.sw) * kRec + g * t.half_off;
    int mboff[4];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
        mboff[mb] = flat ? (mb * 4 * p.sh) * row_b : ((mb >> 1) * p.sd) * plane_b + ((mb & 1) * 4 * p.sh) * row_b;

    const v4i* bank = reinterpret_cast<const v4i*>(p.wgt);
    const int T = p.kd * p.kh * p.kw;

    static_assert(F4 || !DIG, "two-digit inputs go through the 4-bit kind");
    // input words per inner step: a channel word (int8), a pair (fp4), or the low and high digit
    // words of a pair of channel words (two-digit input)
    constexpr int KW = DIG ? 4 : F4 ? 2 : 1;
    using Acc = typename std::conditional<F4, v16f, v16i>::type;
    Acc acc[4][NB];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0;

    // Halo staging of one inner step (a channel word, or a pair of them for fp4): global loads
    // (kFill voxels per thread in flight), then one byte (or four bits) per code into LDS.  A
    // thread's first kFill voxels of the next step are requested before this step's contraction
    // and stored after it.
    const int ksteps = t.ksteps;
    auto halo_load = [&](int ks, int e0, uint32_t (&m)[kFill][KW], uint32_t (&s)[kFill][KW]) {
#pragma unroll
        for (int k = 0; k < kFill; ++k) {
            const uint32_t e = (uint32_t)(e0 + k * nthreads);
            const uint32_t hz = __umulhi(e, t.m_pl);
            const uint32_t r = e - hz * plane;
            const int hy = (int)__umulhi(r, t.m_hx);
            const int hxx = (int)r - hy * t.hx;
            const int gz = gz0 + (int)hz, gy = gy0 + hy, gx = gx0 + hxx;
            const bool inb = e < (uint32_t)nvox && gz >= 0 && gz < p.d && gy >= 0 && gy < p.h && gx >= 0 && gx < p.w;
#pragma unroll
            for (int q = 0; q < KW; ++q) m[k][q] = s[k][q] = 0u;
            if (inb) {
                const uint32_t vox = (uint32_t)((gz * p.h + gy) * p.w + gx);   // below 2^31 voxels per item
                const uint32_t* src = in_n + (size_t)vox * (2u * wd);
                if (DIG && (wd & 3) == 0) {              // the four digit words with one load per plane
                    const uint4 mm = *reinterpret_cast<const uint4*>(src + ks * 4);
                    const uint4 ss = *reinterpret_cast<const uint4*>(src + wd + ks * 4);
                    m[k][0] = mm.x; m[k][1 % KW] = mm.y; m[k][2 % KW] = mm.z; m[k][3 % KW] = mm.w;
                    s[k][0] = ss.x; s[k][1 % KW] = ss.y; s[k][2 % KW] = ss.z; s[k][3 % KW] = ss.w;
                } else if (F4 && !DIG && (wd & 1) == 0) {   // both words of the pair with one load per plane
                    const uint2 mm = *reinterpret_cast<const uint2*>(src + ks * 2);
                    const uint2 ss = *reinterpret_cast<const uint2*>(src + wd + ks * 2);
                    m[k][0] = mm.x; m[k][1 % KW] = mm.y;
                    s[k][0] = ss.x; s[k][1 % KW] = ss.y;
                } else {
#pragma unroll
                    for (int q = 0; q < KW; ++q) {
                        const int word = ks * KW + q;
                        if (word < wd) {                 // an odd word count leaves the last pair half empty
                            m[k][q] = src[word];
                            s[k][q] = src[wd + word];
                        }
                    }
                }
            }
        }
    };
    auto halo_store = [&](int e0, const uint32_t (&m)[kFill][KW], const uint32_t (&s)[kFill][KW]) {
#pragma unroll
        for (int k = 0; k < kFill; ++k) {
            const int e = e0 + k * nthreads;
            if (e < nvox) {
                uint4* dst0 = reinterpret_cast<uint4*>(lds8 + (size_t)e * kRec);
                uint4* dst1 = reinterpret_cast<uint4*>(lds8 + t.half_off + (size_t)e * kRec);
                if constexpr (DIG) {          // words (low, high) of channel word 2 ks, then of 2 ks + 1
                    *dst0 = expand_digits_f4(m[k][0], s[k][0], m[k][1 % KW], s[k][1 % KW]);
                    *dst1 = expand_digits_f4(m[k][2 % KW], s[k][2 % KW], m[k][3 % KW], s[k][3 % KW]);
                } else if constexpr (F4) {
                    *dst0 = expand_word_f4(m[k][0], s[k][0]);
                    *dst1 = expand_word_f4(m[k][1 % KW], s[k][1 % KW]);
                } else {
                    uint4 a, b;
                    expand_word(m[k][0], s[k][0], a, b);
                    *dst0 = a;
                    *dst1 = b;
                }
            }
        }
    };
    uint32_t hm[kFill][KW], hs[kFill][KW];
    halo_load(0, tid, hm, hs);
    for (int ks = 0; ks < ksteps; ++ks) {
        if (ks > 0) __syncthreads();             // everyone is done reading the previous step's tile
        halo_store(tid, hm, hs);
        for (int e0 = tid + kFill * nthreads; e0 < nvox; e0 += kFill * nthreads) {
            uint32_t m2[kFill][KW], s2[kFill][KW];
            halo_load(ks, e0, m2, s2);
            halo_store(e0, m2, s2);
        }
        __syncthreads();
        if (ks + 1 < ksteps) halo_load(ks + 1, tid, hm, hs);

        // ---- contract: all taps of this step ----
        // Column fragments come from the vector cache, hundreds of cycles away: they are requested
        // two taps ahead (three register sets in rotation); row fragments come from LDS at the
        // start of their tap.
        const uint8_t* lane_lds = lds8 + lane_off;
        auto fetch_b = [&](v4i (&B)[NB], int tap) {
            const int tq = tap < T ? tap : T - 1;        // past the end: a harmless repeat
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                B[nb] = bank[((size_t)(tq * ksteps + ks) * t.nblk + nb0 + nb) * 64 + lane];
            __builtin_amdgcn_sched_barrier(0);           // keep the requests ahead of the matrix instructions
        };
        // LDS offset of the following tap (x fastest), as wave-uniform increments
        const int inc_c = p.dw * kRec;
        const int inc_b = p.dh * row_b - (p.kw - 1) * inc_c;
        const int inc_a = p.dd * plane_b - (p.kh - 1) * p.dh * row_b - (p.kw - 1) * inc_c;
        int tb = 0, tc = 0, toff = 0;
        auto contract = [&](const v4i (&B)[NB]) {
            v4i A[4];
#pragma unroll
            for (int mb = 0; mb < 4; ++mb)
                A[mb] = *reinterpret_cast<const v4i*>(lane_lds + toff + mboff[mb]);
#pragma unroll
            for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    if constexpr (F4) {
                        // 4-bit operands occupy the first four of the eight operand registers;
                        // both scales are 2^0 (E8M0 127 in every byte)
                        const v8i a8 = __builtin_shufflevector(A[mb], A[mb], 0, 1, 2, 3, -1, -1, -1, -1);
                        const v8i b8 = __builtin_shufflevector(B[nb], B[nb], 0, 1, 2, 3, -1, -1, -1, -1);
                        acc[mb][nb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                            a8, b8, acc[mb][nb], 4, 4, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
                    } else {
                        acc[mb][nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[mb], B[nb], acc[mb][nb], 0, 0, 0);
                    }
                }
            int inc = inc_c;                             // on to the next tap
            if (++tc == p.kw) {
                tc = 0;
                inc = inc_b;
                if (++tb == p.kh) { tb = 0; inc = inc_a; }
            }
            toff += inc;
        };
        v4i B0[NB], B1[NB], B2[NB];
        fetch_b(B0, 0);
        fetch_b(B1, 1);
        int tap = 0;
        for (; tap + 3 <= T; tap += 3) {
            fetch_b(B2, tap + 2);
            contract(B0);
            fetch_b(B0, tap + 3);
            contract(B1);
            fetch_b(B1, tap + 4);
            contract(B2);
        }
        if (tap < T) {
            contract(B0);
            if (tap + 1 < T) contract(B1);
        }
    }

    // ---- epilogue ----
    // lane l holds column l % 32 (output channel) and, in register v, row 8 (v / 4) + 4 g + v % 4
    // (voxel x = row % 8, y = row / 8 of the row block)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int co = (nb0 + nb) * 32 + i32;
        if constexpr (PACKED) {
            int32_t lo_i = INT32_MIN, hi_i = INT32_MAX;  // channels past c_out: code 0
            if (co < p.c_out) { lo_i = p.lo[co]; hi_i = p.hi[co]; }
            using Thr = typename std::conditional<F4, float, int32_t>::type;
            Thr lo, hi;
            if constexpr (F4) {                          // |sum| < 2^24: clamping changes no decision
                lo = (float)max(-(1 << 24), min(1 << 24, lo_i));
                hi = (float)max(-(1 << 24), min(1 << 24, hi_i));
            } else {
                lo = lo_i;
                hi = hi_i;
            }
            const int q = nb0 + nb;
            if (q < p.wd_out) {
#pragma unroll
                for (int mb = 0; mb < 4; ++mb) {
                    __builtin_amdgcn_sched_barrier(0);   // one tile at a time
                    uint32_t posw = 0u, negw = 0u;      // lane r (< 32): words of the block's voxel r
                    decide_rows<0, Acc, Thr>(acc[mb][nb], lo, hi, posw, negw);
                    const int ox = ox0 + xl, oy = oy0 + (flat ? mb : (mb & 1)) * 4 + yl;
                    const int oz = oz0 + wave * wplanes + (flat ? 0 : (mb >> 1));
                    if (g == 0 && ox < p.ow && oy < p.oh && oz < p.od) {
                        uint32_t* o = p.out_packed + ((((size_t)n * p.od + oz) * p.oh + oy) * p.ow + ox) * 2u * p.wd_out;
                        o[q] = posw | negw;
                        o[p.wd_out + q] = negw & ~posw;
                    }
                }
            }
        } else {
            const size_t cstride = (size_t)p.od * p.oh * p.ow;
#pragma unroll
            for (int mb = 0; mb < 4; ++mb) {
                __builtin_amdgcn_sched_barrier(0);       // one tile at a time
                const int oz = oz0 + wave * wplanes + (flat ? 0 : (mb >> 1));
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = (v >> 2) * 8 + g * 4 + (v & 3);
                    const int ox = ox0 + (r & 7), oy = oy0 + (flat ? mb : (mb & 1)) * 4 + (r >> 3);
                    if (co < p.c_out && ox < p.ow && oy < p.oh && oz < p.od)
                        p.out_acc[((size_t)n * p.c_out + co) * cstride + ((size_t)oz * p.oh + oy) * p.ow + ox] =
                            (int32_t)acc[mb][nb][v];
                }
            }
        }
    }
}

inline int cdiv(int a, int b) { return (a + b - 1) / b; }

template <int NB, bool PACKED, bool F4, bool DIG = false>
int launch_variant(const ConvParams& p, const MfmaPlan& t, size_t lds_bytes, dim3 grid, int threads,
                   hipStream_t s)
{
    auto kern = conv_mfma_kernel<NB, PACKED, F4, DIG>;
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

}  // namespace

// kind 0: one byte per code, an inner step is one channel word; kind 1: four bits per code, an
// inner step is a pair of channel words.  Either way a (tap, step, block of 32 filters) entry is
// 64 lanes x 16 bytes.
static int32_t steps_of(int32_t c_in, int kind) { return kind == 1 ? (c_in + 63) / 64 : (c_in + 31) / 32; }

size_t byte_bank_bytes(int32_t c_out, int32_t c_in, int32_t taps, int kind)
{
    const size_t nblk = (size_t)(c_out + 31) / 32;
    return (size_t)taps * (size_t)steps_of(c_in, kind) * nblk * 1024;
}

int launch_expand_filters(const int8_t* w, int32_t c_out, int32_t c_in, int32_t taps, int kind, uint32_t* bank,
                          hipStream_t s)
{
    const int32_t ksteps = steps_of(c_in, kind), nblk = (c_out + 31) / 32;
    const int64_t dwords = (int64_t)taps * ksteps * nblk * 256;
    const int64_t blocks = (dwords + 255) / 256;
    if (blocks > 0x7fffffff) return TERN_ESHAPE;
    if (kind == 1)
        hipLaunchKernelGGL(expand_filters_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, w, c_out, c_in,
                           taps, ksteps, nblk, bank, dwords);
    else
        hipLaunchKernelGGL(expand_filters_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, w, c_out, c_in,
                           taps, ksteps, nblk, bank, dwords);
    TERN_HIP_CHECK(hipGetLastError());
    return TERN_OK;
}

// p.wgt is the filter bank of that kind.  TERN_ESHAPE when the halo tile of even one wave's
// 8 x 8 x 2 output block does not fit in LDS (very large strides or dilations), and for the 4-bit
// kind when a sum could leave the integers a float holds exactly (k-volume * C_in >= 2^24).
// p.digits: the input is a two-digit tensor (tern_pool_digits) and the bank that of the undoubled
// weights, 4-bit kind.
int launch_conv3d_mfma(const ConvParams& p_in, int kind, hipStream_t s)
{
    ConvParams p = p_in;
    if (kind == 1 && (int64_t)p.kd * p.kh * p.kw * p.c_in >= (1 << 24)) return TERN_ESHAPE;
    // two-digit input (p.digits): 4-bit kind only; p.c_in counts digit channels (two per value, each
    // value up to 4 in magnitude), so a sum stays below 2 * k-volume * c_in
    if (p.digits && (kind != 1 || 2 * (int64_t)p.kd * p.kh * p.kw * p.c_in >= (1 << 24))) return TERN_ESHAPE;
    // A kernel of depth extent 1 with unit depth stride and no depth padding treats every input
    // plane by itself: batch items are just more planes, [N][D] collapses to [1][N*D], and a
    // workgroup's eight planes may come from different batch items (stacks of 2-D slices have
    // D = 1).  Packed output only: the int32 layout has the channel axis between N and D.
    if (p.out_packed && p.n > 1 && p.kd == 1 && p.sd == 1 && p.pd == 0 && (int64_t)p.n * p.d <= INT32_MAX) {
        p.d *= p.n;
        p.od *= p.n;
        p.n = 1;
    }
    MfmaPlan t;
    auto halo = [](int out, int stride, int k, int dil) { return (out - 1) * stride + (k - 1) * dil + 1; };
    t.hx = halo(kTX, p.sw, p.kw, p.dw);
    // single-plane outputs: a wave takes 8 x 16 of the plane instead of 8 x 8 of two planes
    t.flat = p.od == 1 ? 1 : 0;
    const int wplanes = t.flat ? 1 : 2;
    t.hy = halo(t.flat ? 16 : 8, p.sh, p.kh, p.dh);
    // Waves per workgroup (each adds two output planes to the shared halo tile): the count that
    // puts the most waves on a compute unit, LDS permitting (at most two per SIMD fit the
    // registers).  On a tie the larger tile where neighbouring waves read common input planes,
    // else the smaller: waves that share nothing gain nothing from one workgroup and only wait
    // for each other at its barriers.
    const int64_t kLds = lds_limit_for_current_device();   // what this device grants a workgroup
    if (kLds <= 0) return TERN_EHIP;
    int nw = 0, best_waves = 0;
    int w_max = kMaxWaves;
    while (w_max > 1 && w_max >= p.od) w_max /= 2;   // no more waves than there are pairs of output planes
    const bool shares_z = (p.kd - 1) * p.dd + 1 > p.sd;   // neighbouring waves' input planes overlap
    for (int w = w_max; w >= 1; w /= 2) {
        const int64_t nv = (int64_t)t.hx * t.hy * halo(wplanes * w, p.sd, p.kd, p.dd);
        const int64_t bytes = half_offset(nv) + nv * kRec;
        if (bytes > kLds) continue;
        int64_t waves = w * (kLds / bytes);
        if (waves > 8) waves = 8;
        if (waves > best_waves || (waves == best_waves && !shares_z)) { best_waves = (int)waves; nw = w; }
    }
    if (nw == 0) return TERN_ESHAPE;
    const int tz = wplanes * nw;
    t.hz = halo(tz, p.sd, p.kd, p.dd);
    const int64_t nvox = (int64_t)t.hx * t.hy * t.hz;
    t.half_off = (int32_t)half_offset(nvox);
    const int64_t lds = t.half_off + nvox * kRec;
    t.tiles_x = cdiv(p.ow, kTX);
    t.tiles_y = cdiv(p.oh, t.flat ? 16 : 8);
    t.tiles_z = cdiv(p.od, tz);
    t.nblk = (p.c_out + 31) / 32;
    t.m_hx = 0xffffffffu / (uint32_t)t.hx + 1u;           // hx >= 8
    t.m_pl = 0xffffffffu / (uint32_t)(t.hx * t.hy) + 1u;
    const int64_t tiles = (int64_t)t.tiles_x * t.tiles_y * t.tiles_z * p.n;
    if (tiles > 0x7fffffff) return TERN_ESHAPE;
    t.ksteps = p.digits ? (p.wd_in + 3) / 4 : steps_of(p.c_in, kind);
    const bool packed = p.out_packed != nullptr;
    // column blocks in pairs; an odd last block would be paired with a block the bank does not
    // hold, so odd counts run one block per workgroup
    const int nb = (t.nblk % 2 == 0) ? 2 : 1;
    const dim3 grid((unsigned)tiles, (unsigned)(t.nblk / nb));
    const int threads = 64 * nw;
    const size_t lb = (size_t)lds;
#define TERN_MFMA_LAUNCH(NB_, F4_)                                                    \
    (packed ? launch_variant<NB_, true, F4_>(p, t, lb, grid, threads, s)               \
            : launch_variant<NB_, false, F4_>(p, t, lb, grid, threads, s))
    if (p.digits) {
        if (nb == 2)
            return packed ? launch_variant<2, true, true, true>(p, t, lb, grid, threads, s)
                          : launch_variant<2, false, true, true>(p, t, lb, grid, threads, s);
        return packed ? launch_variant<1, true, true, true>(p, t, lb, grid, threads, s)
                      : launch_variant<1, false, true, true>(p, t, lb, grid, threads, s);
    }
    if (kind == 1) return nb == 2 ? TERN_MFMA_LAUNCH(2, true) : TERN_MFMA_LAUNCH(1, true);
    return nb == 2 ? TERN_MFMA_LAUNCH(2, false) : TERN_MFMA_LAUNCH(1, false);
#undef TERN_MFMA_LAUNCH
}

}  // namespace tern
