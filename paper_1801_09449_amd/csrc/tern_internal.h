// Internal declarations shared by the host entry points and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "tern.h"
#include "tern_matrix.h"
#include "tern_tuning.h"

namespace tern {

// Records a failing HIP call for tern_last_hip_error() and maps it to TERN_EHIP.
int record_hip_error(hipError_t e);

#define TERN_HIP_CHECK(expr)                                        \
    do {                                                            \
        hipError_t e__ = (expr);                                    \
        if (e__ != hipSuccess) return ::tern::record_hip_error(e__); \
    } while (0)

// Geometry of one convolution launch, passed to kernels by value.
struct ConvParams {
    const uint32_t* in;     // packed activations [N][D][H][W][2][Wd]
    const uint32_t* wgt;    // filter bank [T*nchunk][co_pad][2][wc] (see tern_pack_filters)
    const int32_t* lo;      // [Co] (packed output mode)
    const int32_t* hi;      // [Co]
    int32_t* out_acc;       // [N][Co][Do][Ho][Wo] or null
    uint32_t* out_packed;   // [N][Do][Ho][Wo][2][Wdo] or null
    int32_t n, c_in, d, h, w;
    int32_t c_out, od, oh, ow;
    int32_t kd, kh, kw;
    int32_t sd, sh, sw;
    int32_t pd, ph, pw;
    int32_t dd, dh, dw;
    int32_t wd_in;          // ceil(c_in/32)
    int32_t wd_out;         // ceil(c_out/32)
    int32_t wc;             // filter-bank chunk width in words: 2 if wd_in is even, else 1
    int32_t co_pad;         // c_out rounded up to a multiple of 32
    int32_t tp_slots;       // tap-packed filter bank: taps per word (0 = plain layout)
    int32_t tp_shift;       // tap-packed filter bank: bits per tap slot
    int32_t digits;         // 1: two-digit input (tern_pool_digits): odd words count three times
    int32_t binary;         // 1: binary filters, bank [T*nchunk][co_pad][wc] of sign words (Eq. 8)
};

// Filter-bank geometry for (c_in, taps): tap packing applies when a voxel is one word with at
// most 16 live channels and the kernel has more than one tap.
struct BankShape {
    int32_t wd, wc, nchunk;     // words per plane, words per chunk, chunks per tap
    int32_t tp_slots, tp_shift; // 0, 0 for the plain layout
    int32_t nsteps;             // rows of the bank
};
inline BankShape bank_shape(int32_t c_in, int32_t taps)
{
    BankShape b;
    b.wd = (c_in + 31) / 32;
    b.wc = (b.wd % 2 == 0) ? 2 : 1;
    b.nchunk = b.wd / b.wc;
    b.tp_slots = 0; b.tp_shift = 0;
    if (c_in <= 16 && taps > 1) {
        int sh = 1;
        while (sh < c_in) sh *= 2;
        b.tp_shift = sh;
        b.tp_slots = 32 / sh;
        if (b.tp_slots > taps) b.tp_slots = taps;
    }
    b.nsteps = b.tp_slots ? (taps + b.tp_slots - 1) / b.tp_slots : taps * b.nchunk;
    return b;
}

// tern_concat: one source after validation, and the whole launch (passed to the kernel by value).
struct ConcatSrc {
    const uint32_t* p;      // packed [N][d][h][w][2][wd]
    int32_t d, h, w, wd;
    int32_t bit0;           // first output channel this source fills
    int32_t up[3];          // nearest-neighbour factor per axis
    int32_t first[3];       // upsampled coordinate that lands on output voxel 0
};
struct ConcatParams {
    ConcatSrc s[TERN_MAX_SOURCES];
    int32_t n_src;
    int32_t od, oh, ow, wd_out;
    int64_t total;          // output voxels x wd_out
    uint32_t* out;
};

// tern_conv3d_real: ternary codes x float weights.
struct RealConvParams {
    const uint32_t* in;     // packed [N][D][H][W][2][wd_in]
    const float* wgt;       // [c_out][c_in][kd][kh][kw]
    const float* bias;      // [c_out] or null
    float* out;             // [N][c_out][od][oh][ow]
    int32_t c_in, d, h, w, wd_in;
    int32_t c_out, od, oh, ow;
    int32_t kd, kh, kw, sd, sh, sw, pd, ph, pw, dd, dh, dw;
    int64_t total;          // output voxels
};

// Gathering of the taps of a one-channel first layer (see patch_pack_f32_kernel).
struct PatchParams {
    const float* src;       // [N][1][d][h][w]
    const float* lo;        // [1] cut points of the input activation
    const float* hi;
    uint32_t* dst;          // [N][od][oh][ow][2][1]
    int32_t d, h, w, od, oh, ow;
    int32_t kd, kh, kw, sh, sw, pd, ph, pw, dh, dw;
};
// True when a first layer with c_in input channels, geometry g and output extents `out` can take
// that route.
bool patch_pack_applies(int32_t c_in, const tern_conv_geom& g, const tern_dims& out);
int launch_patch_pack_f32(const PatchParams& p, int32_t n, hipStream_t s);
// Layer 0 behind the gathering, in the same kernel (PatchParams::dst unused): single-tap filter
// bank over the gathered words, integer cut points, packed output [N][od][oh][ow][2][wd_out].
struct FirstConvParams {
    const uint32_t* wgt;    // [words of the tap string][co_pad][2][1]
    const int32_t* lo;      // [c_out]
    const int32_t* hi;
    uint32_t* out_packed;
    int32_t c_out, co_pad, wd_out;
};
int launch_patch_conv_f32(const PatchParams& p, const FirstConvParams& c, int32_t n, hipStream_t s);
bool patch_conv_pays(const PatchParams& p, int32_t n);

// Largest dynamic LDS allocation the current device grants one workgroup, at most the 160 KB of a
// gfx950 compute unit (queried once per device; 0 on error).
int lds_limit_for_current_device();

// Launchers implemented in the kernel translation units.  Each validates nothing (the entry
// points did) and returns a tern_status.
int launch_pack_i8(const int8_t* src, tern_dims dims, uint32_t* dst, hipStream_t s);
int launch_threshold_pack_i32(const int32_t* src, tern_dims dims, const int32_t* lo,
                              const int32_t* hi, uint32_t* dst, hipStream_t s);
int launch_threshold_pack_f32(const float* src, tern_dims dims, const float* lo, const float* hi,
                              uint32_t* dst, hipStream_t s);
int launch_conv3d(const ConvParams& p, hipStream_t s);
// 1x1x1 / stride 1 / no padding with 1, 2, 4 or 8 input words per plane: the pointwise kernel.
bool conv_point_applies(const ConvParams& p);
int launch_conv_point(const ConvParams& p, hipStream_t s);
// Matrix-core route: byte filter bank and the convolution that takes it as p.wgt.
size_t byte_bank_bytes(int32_t c_out, int32_t c_in, int32_t taps, int kind);
int launch_expand_filters(const int8_t* w, int32_t c_out, int32_t c_in, int32_t taps, int kind, uint32_t* bank,
                          hipStream_t s);
int launch_conv3d_mfma(const ConvParams& p, int kind, hipStream_t s);
int launch_concat(const ConcatParams& p, hipStream_t s);
int launch_pool_digits(const uint32_t* in, const tern_dims& in_dims, const int32_t window[3], uint32_t* out,
                       hipStream_t s);
int launch_real_conv(const RealConvParams& p, hipStream_t s);
int launch_count_codes(const uint32_t* in, int64_t voxels, int32_t c, unsigned long long* nonzero,
                       unsigned long long* negative, hipStream_t s);
void set_lane_depth(int v);
void set_waves_z(int v);
void set_co_block(int v);
void set_co_per_wave(int v);
void set_tap_split(int v);
void set_lane_tile(int v);
void set_pointwise(int v);
void set_stream(int v);
void last_launch(int32_t* info);
int launch_pack_filters(const int8_t* w, int32_t c_out, int32_t c_in, int32_t kd, int32_t kh,
                        int32_t kw, uint32_t* bank, hipStream_t s);
int launch_pack_filters_binary(const int8_t* w, int32_t c_out, int32_t c_in, int32_t kd, int32_t kh,
                               int32_t kw, uint32_t* bank, hipStream_t s);

}  // namespace tern
