// Host side of the C ABI declared in include/tern.h: argument validation and dispatch.
// Every entry point validates on the host, launches on the caller's stream and returns without
// synchronising.  Nothing here allocates device memory.
#include <limits.h>

#include <mutex>
#include <vector>

#include "tern_internal.h"

namespace tern {

static thread_local int g_last_hip_error = 0;

int record_hip_error(hipError_t e)
{
    g_last_hip_error = static_cast<int>(e);
    return TERN_EHIP;
}

static bool dims_ok(const tern_dims& d)
{
    return d.n > 0 && d.c > 0 && d.d > 0 && d.h > 0 && d.w > 0;
}

static int64_t voxels(const tern_dims& d)
{
    return (int64_t)d.n * d.d * d.h * d.w;
}

// Limits that keep every device-side index inside int32/uint32 where the kernels use them.
static bool sizes_ok(const tern_dims& d)
{
    if (!dims_ok(d)) return false;
    const int64_t vox = voxels(d);
    if (vox > (int64_t)INT32_MAX) return false;
    const int64_t wd = (d.c + 31) / 32;
    if (vox * 2 * wd > (int64_t)1 << 40) return false;
    if ((int64_t)d.c * (int64_t)d.d * d.h * d.w > (int64_t)1 << 40) return false;
    return true;
}

static int out_extent(int x, int k, int s, int p, int dil)
{
    const int64_t span = (int64_t)x + 2 * (int64_t)p - (int64_t)dil * (k - 1) - 1;
    if (span < 0) return 0;
    const int64_t o = span / s + 1;
    return o > INT32_MAX ? 0 : (int)o;
}

static bool filter_shape_ok(int32_t c_out, int32_t c_in, int32_t kd, int32_t kh, int32_t kw)
{
    if (c_out <= 0 || c_out > (1 << 19) || c_in <= 0 || kd < 1 || kh < 1 || kw < 1) return false;
    if (kd > 1024 || kh > 1024 || kw > 1024) return false;
    const int64_t taps = (int64_t)kd * kh * kw;
    if (taps * c_in >= (int64_t)1 << 24) return false;
    if (taps * ((c_in + 31) / 32) * ((int64_t)c_out + 31) >= (int64_t)1 << 31) return false;
    return true;
}

static int geom_check(const tern_dims& in, int32_t c_out, const tern_conv_geom& g, tern_dims* out)
{
    if (!sizes_ok(in) || c_out <= 0) return TERN_ESHAPE;
    for (int a = 0; a < 3; ++a) {
        if (g.k[a] < 1 || g.stride[a] < 1 || g.dil[a] < 1 || g.pad[a] < 0) return TERN_EARG;
        if (g.k[a] > 1024 || g.stride[a] > 1024 || g.dil[a] > 1024 || g.pad[a] > (1 << 20))
            return TERN_EARG;
    }
    if (!filter_shape_ok(c_out, in.c, g.k[0], g.k[1], g.k[2])) return TERN_ESHAPE;
    tern_dims o;
    o.n = in.n;
    o.c = c_out;
    o.d = out_extent(in.d, g.k[0], g.stride[0], g.pad[0], g.dil[0]);
    o.h = out_extent(in.h, g.k[1], g.stride[1], g.pad[1], g.dil[1]);
    o.w = out_extent(in.w, g.k[2], g.stride[2], g.pad[2], g.dil[2]);
    if (o.d < 1 || o.h < 1 || o.w < 1) return TERN_ESHAPE;
    if (!sizes_ok(o)) return TERN_ESHAPE;
    if (out) *out = o;
    return TERN_OK;
}

// Kernel parameters of one (already validated) convolution with output extents o.
static ConvParams conv_params(const uint32_t* in_packed, const tern_dims& in_dims,
                              const uint32_t* w_bank, int32_t c_out, const tern_conv_geom& g,
                              const tern_dims& o, const int32_t* thr_lo, const int32_t* thr_hi,
                              int32_t* out_acc, uint32_t* out_packed)
{
    ConvParams p;
    p.in = in_packed;
    p.wgt = w_bank;
    p.lo = thr_lo;
    p.hi = thr_hi;
    p.out_acc = out_acc;
    p.out_packed = out_packed;
    p.n = in_dims.n; p.c_in = in_dims.c; p.d = in_dims.d; p.h = in_dims.h; p.w = in_dims.w;
    p.c_out = c_out; p.od = o.d; p.oh = o.h; p.ow = o.w;
    p.kd = g.k[0]; p.kh = g.k[1]; p.kw = g.k[2];
    p.sd = g.stride[0]; p.sh = g.stride[1]; p.sw = g.stride[2];
    p.pd = g.pad[0]; p.ph = g.pad[1]; p.pw = g.pad[2];
    p.dd = g.dil[0]; p.dh = g.dil[1]; p.dw = g.dil[2];
    p.wd_in = tern_words(in_dims.c);
    p.wd_out = tern_words(c_out);
    const BankShape bs = bank_shape(in_dims.c, g.k[0] * g.k[1] * g.k[2]);
    p.wc = bs.wc;
    p.co_pad = (c_out + 31) / 32 * 32;
    p.tp_slots = bs.tp_slots;
    p.tp_shift = bs.tp_shift;
    p.digits = 0;
    p.binary = 0;
    return p;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace tern

using namespace tern;

extern "C" {

int32_t tern_words(int32_t c) { return c > 0 ? (c + 31) / 32 : 0; }

size_t tern_packed_bytes(tern_dims dims)
{
    if (!sizes_ok(dims)) return 0;
    return (size_t)voxels(dims) * 2u * (size_t)tern_words(dims.c) * sizeof(uint32_t);
}

int tern_conv_out_dims(tern_dims in_dims, int32_t c_out, tern_conv_geom g, tern_dims* out_dims)
{
    if (!out_dims) return TERN_ENULL;
    return geom_check(in_dims, c_out, g, out_dims);
}

int tern_last_hip_error(void) { return g_last_hip_error; }

const char* tern_status_string(int status)
{
    switch (status) {
        case TERN_OK: return "TERN_OK";
        case TERN_ENULL: return "TERN_ENULL: a required pointer is NULL";
        case TERN_ESHAPE: return "TERN_ESHAPE: invalid or unsupported tensor extents";
        case TERN_EARG: return "TERN_EARG: invalid argument combination";
        case TERN_EWORKSPACE: return "TERN_EWORKSPACE: workspace too small or misaligned";
        case TERN_EHIP: return "TERN_EHIP: a HIP call failed";
        default: return "unknown tern_status";
    }
}

int tern_set_option(int option, int value)
{
    if (option == TERN_OPT_LANE_DEPTH) {
        if (value != 0 && value != 1 && value != 2 && value != 4) return TERN_EARG;
        set_lane_depth(value);
        return TERN_OK;
    }
    if (option == TERN_OPT_CO_BLOCK) {
        if (value != 0 && value != 8 && value != 16 && value != 32) return TERN_EARG;
        set_co_block(value);
        return TERN_OK;
    }
    if (option == TERN_OPT_CO_PER_WAVE) {
        if (value < 0 || value % 16 != 0 || value > (1 << 20)) return TERN_EARG;
        set_co_per_wave(value);
        return TERN_OK;
    }
    if (option == TERN_OPT_TAP_SPLIT) {
        if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8) return TERN_EARG;
        set_tap_split(value);
        return TERN_OK;
    }
    if (option == TERN_OPT_POINTWISE) {
        if (value != 0 && value != 1) return TERN_EARG;
        set_pointwise(value);
        return TERN_OK;
    }
    if (option == TERN_OPT_LANE_TILE) {
        const int lx = value / 100, ly = value % 100;
        auto pow2 = [](int v) { return v == 1 || v == 2 || v == 4 || v == 8; };
        if (value != 0 && value != -1 && !(pow2(lx) && pow2(ly) && lx * ly >= 4)) return TERN_EARG;
        set_lane_tile(value);
        return TERN_OK;
    }
    if (option == TERN_OPT_STREAM) {
        if (value != 0 && value != 1) return TERN_EARG;
        set_stream(value);
        return TERN_OK;
    }
    if (option == TERN_OPT_WAVES_Z) {
        if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8) return TERN_EARG;
        set_waves_z(value);
        return TERN_OK;
    }
    return TERN_EARG;
}

int tern_last_launch(int32_t info[8])
{
    if (!info) return TERN_ENULL;
    last_launch(info);
    return TERN_OK;
}

int tern_pack(const int8_t* src, tern_dims dims, uint32_t* dst_packed, void* stream)
{
    if (!src || !dst_packed) return TERN_ENULL;
    if (!sizes_ok(dims)) return TERN_ESHAPE;
    if (!aligned16(dst_packed)) return TERN_EARG;
    return launch_pack_i8(src, dims, dst_packed, (hipStream_t)stream);
}

size_t tern_filter_bank_bytes(int32_t c_out, int32_t c_in, int32_t kd, int32_t kh, int32_t kw)
{
    if (!filter_shape_ok(c_out, c_in, kd, kh, kw)) return 0;
    const size_t co_pad = (size_t)(c_out + 31) / 32 * 32;
    const BankShape b = bank_shape(c_in, kd * kh * kw);
    return (size_t)b.nsteps * co_pad * 2u * (size_t)b.wc * sizeof(uint32_t);
}

int tern_pack_filters(const int8_t* w, int32_t c_out, int32_t c_in, int32_t kd, int32_t kh,
                      int32_t kw, uint32_t* bank, void* stream)
{
    if (!w || !bank) return TERN_ENULL;
    if (!filter_shape_ok(c_out, c_in, kd, kh, kw)) return TERN_ESHAPE;
    if (!aligned16(bank)) return TERN_EARG;
    return launch_pack_filters(w, c_out, c_in, kd, kh, kw, bank, (hipStream_t)stream);
}

int tern_threshold_pack(const void* src, tern_src_type t, tern_dims dims, const void* thr_lo,
                        const void* thr_hi, uint32_t* dst_packed, void* stream)
{
    if (!src || !thr_lo || !thr_hi || !dst_packed) return TERN_ENULL;
    if (t != TERN_SRC_I32 && t != TERN_SRC_F32) return TERN_EARG;
    if (!sizes_ok(dims)) return TERN_ESHAPE;
    if (!aligned16(dst_packed) || ((uintptr_t)src & 3u)) return TERN_EARG;
    if (t == TERN_SRC_I32)
        return launch_threshold_pack_i32((const int32_t*)src, dims, (const int32_t*)thr_lo,
                                         (const int32_t*)thr_hi, dst_packed, (hipStream_t)stream);
    return launch_threshold_pack_f32((const float*)src, dims, (const float*)thr_lo,
                                     (const float*)thr_hi, dst_packed, (hipStream_t)stream);
}

int tern_conv3d(const uint32_t* in_packed, tern_dims in_dims, const uint32_t* w_bank,
                int32_t c_out, tern_conv_geom g, const int32_t* thr_lo, const int32_t* thr_hi,
                int32_t* out_acc, uint32_t* out_packed, void* stream)
{
    if (!in_packed || !w_bank) return TERN_ENULL;
    if ((out_acc == nullptr) == (out_packed == nullptr)) return TERN_EARG;
    if (out_packed && (!thr_lo || !thr_hi)) return TERN_ENULL;
    tern_dims o;
    int rc = geom_check(in_dims, c_out, g, &o);
    if (rc != TERN_OK) return rc;
    if (!aligned16(in_packed) || !aligned16(w_bank)) return TERN_EARG;
    if (out_packed && !aligned16(out_packed)) return TERN_EARG;
    if (out_acc && ((uintptr_t)out_acc & 3u)) return TERN_EARG;

    const ConvParams p = conv_params(in_packed, in_dims, w_bank, c_out, g, o, thr_lo, thr_hi, out_acc,
                                     out_packed);
    return launch_conv3d(p, (hipStream_t)stream);
}

size_t tern_binary_bank_bytes(int32_t c_out, int32_t c_in, int32_t kd, int32_t kh, int32_t kw)
{
    if (!filter_shape_ok(c_out, c_in, kd, kh, kw)) return 0;
    const size_t co_pad = (size_t)(c_out + 31) / 32 * 32;
    return (size_t)kd * kh * kw * (size_t)tern_words(c_in) * co_pad * sizeof(uint32_t);
}

int tern_pack_filters_binary(const int8_t* w, int32_t c_out, int32_t c_in, int32_t kd, int32_t kh,
                             int32_t kw, uint32_t* bank, void* stream)
{
    if (!w || !bank) return TERN_ENULL;
    if (!filter_shape_ok(c_out, c_in, kd, kh, kw)) return TERN_ESHAPE;
    if (!aligned16(bank)) return TERN_EARG;
    return launch_pack_filters_binary(w, c_out, c_in, kd, kh, kw, bank, (hipStream_t)stream);
}

int tern_conv3d_binary(const uint32_t* in_packed, tern_dims in_dims, const uint32_t* w_bank,
                       int32_t c_out, tern_conv_geom g, const int32_t* thr_lo, const int32_t* thr_hi,
                       int32_t* out_acc, uint32_t* out_packed, void* stream)
{
    if (!in_packed || !w_bank) return TERN_ENULL;
    if ((out_acc == nullptr) == (out_packed == nullptr)) return TERN_EARG;
    if (out_packed && (!thr_lo || !thr_hi)) return TERN_ENULL;
    tern_dims o;
    int rc = geom_check(in_dims, c_out, g, &o);
    if (rc != TERN_OK) return rc;
    if (!aligned16(in_packed) || !aligned16(w_bank)) return TERN_EARG;
    if (out_packed && !aligned16(out_packed)) return TERN_EARG;
    if (out_acc && ((uintptr_t)out_acc & 3u)) return TERN_EARG;
    ConvParams p = conv_params(in_packed, in_dims, w_bank, c_out, g, o, thr_lo, thr_hi, out_acc, out_packed);
    p.binary = 1;
    p.tp_slots = 0;    // the binary bank has the plain layout whatever C_in is
    p.tp_shift = 0;
    return launch_conv3d(p, (hipStream_t)stream);
}

size_t tern_matrix_bank_bytes(int32_t c_out, int32_t c_in, int32_t kd, int32_t kh, int32_t kw, int32_t kind)
{
    if (!filter_shape_ok(c_out, c_in, kd, kh, kw) || (kind != TERN_MATRIX_I8 && kind != TERN_MATRIX_F4)) return 0;
    return byte_bank_bytes(c_out, c_in, kd * kh * kw, kind);
}

int tern_expand_filters(const int8_t* w, int32_t c_out, int32_t c_in, int32_t kd, int32_t kh,
                        int32_t kw, int32_t kind, uint32_t* matrix_bank, void* stream)
{
    if (!w || !matrix_bank) return TERN_ENULL;
    if (kind != TERN_MATRIX_I8 && kind != TERN_MATRIX_F4) return TERN_EARG;
    if (!filter_shape_ok(c_out, c_in, kd, kh, kw)) return TERN_ESHAPE;
    if (!aligned16(matrix_bank)) return TERN_EARG;
    return launch_expand_filters(w, c_out, c_in, kd * kh * kw, kind, matrix_bank, (hipStream_t)stream);
}

int tern_conv3d_mfma(const uint32_t* in_packed, tern_dims in_dims, const uint32_t* byte_bank, int32_t kind,
                     int32_t c_out, tern_conv_geom g, const int32_t* thr_lo, const int32_t* thr_hi,
                     int32_t* out_acc, uint32_t* out_packed, void* stream)
{
    if (!in_packed || !byte_bank) return TERN_ENULL;
    if (kind != TERN_MATRIX_I8 && kind != TERN_MATRIX_F4) return TERN_EARG;
    if ((out_acc == nullptr) == (out_packed == nullptr)) return TERN_EARG;
    if (out_packed && (!thr_lo || !thr_hi)) return TERN_ENULL;
    tern_dims o;
    int rc = geom_check(in_dims, c_out, g, &o);
    if (rc != TERN_OK) return rc;
    if (!aligned16(in_packed) || !aligned16(byte_bank)) return TERN_EARG;
    if (out_packed && !aligned16(out_packed)) return TERN_EARG;
    if (out_acc && ((uintptr_t)out_acc & 3u)) return TERN_EARG;
    const ConvParams p = conv_params(in_packed, in_dims, byte_bank, c_out, g, o, thr_lo, thr_hi, out_acc,
                                     out_packed);
    return launch_conv3d_mfma(p, kind, (hipStream_t)stream);
}

int tern_conv3d_mfma_digits(const uint32_t* in_packed, tern_dims in_dims, const uint32_t* matrix_bank,
                            int32_t c_out, tern_conv_geom g, const int32_t* thr_lo, const int32_t* thr_hi,
                            int32_t* out_acc, uint32_t* out_packed, void* stream)
{
    if (!in_packed || !matrix_bank) return TERN_ENULL;
    if ((out_acc == nullptr) == (out_packed == nullptr)) return TERN_EARG;
    if (out_packed && (!thr_lo || !thr_hi)) return TERN_ENULL;
    if (in_dims.c <= 0 || in_dims.c % 64 != 0) return TERN_EARG;   // whole (low, high) word pairs
    tern_dims o;
    int rc = geom_check(in_dims, c_out, g, &o);
    if (rc != TERN_OK) return rc;
    if (!aligned16(in_packed) || !aligned16(matrix_bank)) return TERN_EARG;
    if (out_packed && !aligned16(out_packed)) return TERN_EARG;
    if (out_acc && ((uintptr_t)out_acc & 3u)) return TERN_EARG;
    ConvParams p = conv_params(in_packed, in_dims, matrix_bank, c_out, g, o, thr_lo, thr_hi, out_acc, out_packed);
    p.digits = 1;
    return launch_conv3d_mfma(p, TERN_MATRIX_F4, (hipStream_t)stream);
}

int tern_conv3d_digits(const uint32_t* in_packed, tern_dims in_dims, const uint32_t* w_bank,
                       int32_t c_out, tern_conv_geom g, const int32_t* thr_lo, const int32_t* thr_hi,
                       int32_t* out_acc, uint32_t* out_packed, void* stream)
{
    if (!in_packed || !w_bank) return TERN_ENULL;
    if ((out_acc == nullptr) == (out_packed == nullptr)) return TERN_EARG;
    if (out_packed && (!thr_lo || !thr_hi)) return TERN_ENULL;
    if (in_dims.c <= 0 || in_dims.c % 64 != 0) return TERN_EARG;   // whole (low, high) word pairs
    tern_dims o;
    int rc = geom_check(in_dims, c_out, g, &o);
    if (rc != TERN_OK) return rc;
    // accumulators reach 2 * k-volume * c (every digit pair can contribute 1 + 3)
    if ((int64_t)g.k[0] * g.k[1] * g.k[2] * in_dims.c >= (1 << 23)) return TERN_ESHAPE;
    if (!aligned16(in_packed) || !aligned16(w_bank)) return TERN_EARG;
    if (out_packed && !aligned16(out_packed)) return TERN_EARG;
    if (out_acc && ((uintptr_t)out_acc & 3u)) return TERN_EARG;
    ConvParams p = conv_params(in_packed, in_dims, w_bank, c_out, g, o, thr_lo, thr_hi, out_acc, out_packed);
    p.digits = 1;
    return launch_conv3d(p, (hipStream_t)stream);
}

int tern_pool_digits(const uint32_t* in_packed, tern_dims in_dims, const int32_t window[3],
                     uint32_t* out_packed, void* stream)
{
    if (!in_packed || !window || !out_packed) return TERN_ENULL;
    if (!sizes_ok(in_dims)) return TERN_ESHAPE;
    for (int a = 0; a < 3; ++a)
        if (window[a] < 1 || window[a] > 4) return TERN_EARG;
    if (window[0] * window[1] * window[2] > 4) return TERN_EARG;   // sums beyond +-4 need a third digit
    if (!aligned16(in_packed) || !aligned16(out_packed)) return TERN_EARG;
    const int64_t c2 = 64 * (int64_t)tern_words(in_dims.c);
    if (c2 > INT32_MAX) return TERN_ESHAPE;
    return launch_pool_digits(in_packed, in_dims, window, out_packed, (hipStream_t)stream);
}

int tern_concat(const tern_source* srcs, int32_t n_src, tern_dims out_dims, uint32_t* out_packed,
                void* stream)
{
    if (!srcs || !out_packed) return TERN_ENULL;
    if (n_src < 1 || n_src > TERN_MAX_SOURCES) return TERN_EARG;
    if (!sizes_ok(out_dims)) return TERN_ESHAPE;
    if (!aligned16(out_packed)) return TERN_EARG;
    ConcatParams p;
    int64_t channels = 0;
    const int32_t oext[3] = {out_dims.d, out_dims.h, out_dims.w};
    for (int i = 0; i < n_src; ++i) {
        const tern_source& s = srcs[i];
        if (!s.packed) return TERN_ENULL;
        if (!sizes_ok(s.dims)) return TERN_ESHAPE;
        if (s.dims.n != out_dims.n) return TERN_EARG;
        if (!aligned16(s.packed)) return TERN_EARG;
        const int32_t sext[3] = {s.dims.d, s.dims.h, s.dims.w};
        for (int a = 0; a < 3; ++a) {
            if (s.up[a] < 1 || s.up[a] > 1024 || s.first[a] < 0) return TERN_EARG;
            if ((int64_t)s.first[a] + oext[a] > (int64_t)sext[a] * s.up[a]) return TERN_EARG;
        }
        ConcatSrc& c = p.s[i];
        c.p = s.packed;
        c.d = s.dims.d; c.h = s.dims.h; c.w = s.dims.w;
        c.wd = tern_words(s.dims.c);
        c.bit0 = (int32_t)channels;
        for (int a = 0; a < 3; ++a) { c.up[a] = s.up[a]; c.first[a] = s.first[a]; }
        channels += s.dims.c;
        if (channels > out_dims.c) return TERN_EARG;
    }
    if (channels != out_dims.c) return TERN_EARG;
    for (int i = n_src; i < TERN_MAX_SOURCES; ++i) p.s[i] = p.s[0];
    p.n_src = n_src;
    p.od = out_dims.d; p.oh = out_dims.h; p.ow = out_dims.w;
    p.wd_out = tern_words(out_dims.c);
    p.total = voxels(out_dims) * p.wd_out;
    p.out = out_packed;
    return launch_concat(p, (hipStream_t)stream);
}

int tern_conv3d_real(const uint32_t* in_packed, tern_dims in_dims, const float* w,
                     const float* bias, int32_t c_out, tern_conv_geom g, float* out, void* stream)
{
    if (!in_packed || !w || !out) return TERN_ENULL;
    tern_dims o;
    int rc = geom_check(in_dims, c_out, g, &o);
    if (rc != TERN_OK) return rc;
    if (!aligned16(in_packed) || ((uintptr_t)w & 3u) || ((uintptr_t)out & 3u) ||
        ((uintptr_t)bias & 3u))
        return TERN_EARG;
    RealConvParams p;
    p.in = in_packed; p.wgt = w; p.bias = bias; p.out = out;
    p.c_in = in_dims.c; p.d = in_dims.d; p.h = in_dims.h; p.w = in_dims.w;
    p.wd_in = tern_words(in_dims.c);
    p.c_out = c_out; p.od = o.d; p.oh = o.h; p.ow = o.w;
    p.kd = g.k[0]; p.kh = g.k[1]; p.kw = g.k[2];
    p.sd = g.stride[0]; p.sh = g.stride[1]; p.sw = g.stride[2];
    p.pd = g.pad[0]; p.ph = g.pad[1]; p.pw = g.pad[2];
    p.dd = g.dil[0]; p.dh = g.dil[1]; p.dw = g.dil[2];
    p.total = voxels(o);
    return launch_real_conv(p, (hipStream_t)stream);
}

int tern_count_codes(const uint32_t* in_packed, tern_dims dims, uint64_t* nonzero, uint64_t* negative,
                     void* stream)
{
    if (!in_packed || !nonzero || !negative) return TERN_ENULL;
    if (!sizes_ok(dims)) return TERN_ESHAPE;
    if (!aligned16(in_packed) || ((uintptr_t)nonzero & 7u) || ((uintptr_t)negative & 7u)) return TERN_EARG;
    return launch_count_codes(in_packed, voxels(dims), dims.c, (unsigned long long*)nonzero,
                              (unsigned long long*)negative, (hipStream_t)stream);
}

// Walks the chain once: validates channel continuity and geometry, and reports the packed size
// of the input and of every layer output.  Returns TERN_OK or the first error.
static int fcn_plan(tern_dims in_dims, const tern_layer* layers, int32_t n_layers,
                    size_t* ws_bytes, tern_dims* last)
{
    if (!layers) return TERN_ENULL;
    if (n_layers < 1 || n_layers > 1024) return TERN_EARG;
    if (!sizes_ok(in_dims)) return TERN_ESHAPE;
    size_t total = (tern_packed_bytes(in_dims) + 255u) & ~(size_t)255u;
    tern_dims cur = in_dims;
    for (int i = 0; i < n_layers; ++i) {
        if (layers[i].c_in != cur.c) return TERN_EARG;
        tern_dims o;
        int rc = geom_check(cur, layers[i].c_out, layers[i].g, &o);
        if (rc != TERN_OK) return rc;
        if (i == 0 && patch_pack_applies(in_dims.c, layers[0].g, o)) {
            // the first region then holds the gathered taps (one word pair per output voxel of
            // layer 0) instead of the packed input
            const tern_dims patches = {o.n, layers[0].g.k[0] * layers[0].g.k[1] * layers[0].g.k[2], o.d, o.h, o.w};
            total = (tern_packed_bytes(patches) + 255u) & ~(size_t)255u;
        }
        if (i + 1 < n_layers) total += (tern_packed_bytes(o) + 255u) & ~(size_t)255u;
        cur = o;
    }
    if (ws_bytes) *ws_bytes = total;
    if (last) *last = cur;
    return TERN_OK;
}

size_t tern_fcn_workspace_bytes(tern_dims in_dims, const tern_layer* layers, int32_t n_layers)
{
    size_t b = 0;
    if (fcn_plan(in_dims, layers, n_layers, &b, nullptr) != TERN_OK) return 0;
    return b;
}

// The chain behind tern_fcn_forward and tern_fcn_forward_static: everything validated, `workspace`
// holds at least the bytes fcn_plan asks for.
static int fcn_run(const float* in, tern_dims in_dims, const float* in_lo, const float* in_hi,
                   const tern_layer* layers, int32_t n_layers, void* workspace, uint32_t* out_packed,
                   uint32_t** layer_out, void* stream)
{
    char* ws = (char*)workspace;
    uint32_t* cur_buf = (uint32_t*)ws;
    tern_dims cur = in_dims;
    tern_dims o0;
    int rc = geom_check(in_dims, layers[0].c_out, layers[0].g, &o0);
    if (rc != TERN_OK) return rc;
    // A one-channel input with a 3x3x3, 1x3x3 or 15x3x3 first kernel: Eq. 6 and the gathering of
    // every output voxel's taps into a bit string happen in one pass over the intensities, and
    // layer 0 becomes a single-tap convolution over those strings (its tap-packed filter bank is already in the
    // matching layout).  Otherwise: Eq. 6 on the raw intensities, packed, then layer 0 as is.
    const bool gathered = patch_pack_applies(in_dims.c, layers[0].g, o0);
    PatchParams first = {};
    bool fused = false;
    if (gathered) {
        const tern_dims patches = {o0.n, layers[0].g.k[0] * layers[0].g.k[1] * layers[0].g.k[2], o0.d, o0.h, o0.w};
        ws += (tern_packed_bytes(patches) + 255u) & ~(size_t)255u;
        const tern_conv_geom& g = layers[0].g;
        PatchParams pp;
        pp.src = in; pp.lo = in_lo; pp.hi = in_hi; pp.dst = cur_buf;
        pp.d = in_dims.d; pp.h = in_dims.h; pp.w = in_dims.w;
        pp.od = o0.d; pp.oh = o0.h; pp.ow = o0.w;
        pp.kd = g.k[0]; pp.kh = g.k[1]; pp.kw = g.k[2];
        pp.sh = g.stride[1]; pp.sw = g.stride[2];
        pp.pd = g.pad[0]; pp.ph = g.pad[1]; pp.pw = g.pad[2];
        pp.dh = g.dil[1]; pp.dw = g.dil[2];
        // layer 0 runs behind the gathering in the same kernel (below) where that pays; the
        // region reserved for the tap strings then stays unused
        first = pp;
        fused = patch_conv_pays(pp, in_dims.n);
        rc = fused ? TERN_OK : launch_patch_pack_f32(pp, in_dims.n, (hipStream_t)stream);
    } else {
        ws += (tern_packed_bytes(in_dims) + 255u) & ~(size_t)255u;
        rc = tern_threshold_pack(in, TERN_SRC_F32, in_dims, in_lo, in_hi, cur_buf, stream);
    }
    if (rc != TERN_OK) return rc;
    for (int i = 0; i < n_layers; ++i) {
        tern_dims o;
        rc = geom_check(cur, layers[i].c_out, layers[i].g, &o);
        if (rc != TERN_OK) return rc;
        uint32_t* dst;
        if (i + 1 < n_layers) {
            dst = (uint32_t*)ws;
            ws += (tern_packed_bytes(o) + 255u) & ~(size_t)255u;
        } else {
            dst = out_packed;
        }
        if (i == 0 && gathered && !fused) {
            const int32_t taps = layers[0].g.k[0] * layers[0].g.k[1] * layers[0].g.k[2];
            const tern_dims pin = {o.n, taps, o.d, o.h, o.w};
            const tern_conv_geom unit = {{1, 1, 1}, {1, 1, 1}, {0, 0, 0}, {1, 1, 1}};
            if (!aligned16(layers[0].w_bank) || !aligned16(dst)) return TERN_EARG;
            rc = launch_conv3d(conv_params(cur_buf, pin, layers[0].w_bank, layers[0].c_out, unit, o,
                                           layers[0].thr_lo, layers[0].thr_hi, nullptr, dst),
                               (hipStream_t)stream);
        } else if (i == 0 && gathered) {
            if (!aligned16(layers[0].w_bank) || !aligned16(dst)) return TERN_EARG;
            FirstConvParams fc;
            fc.wgt = layers[0].w_bank; fc.lo = layers[0].thr_lo; fc.hi = layers[0].thr_hi;
            fc.out_packed = dst;
            fc.c_out = layers[0].c_out; fc.co_pad = (layers[0].c_out + 31) / 32 * 32;
            fc.wd_out = tern_words(layers[0].c_out);
            rc = launch_patch_conv_f32(first, fc, in_dims.n, (hipStream_t)stream);
        } else {
            rc = tern_conv3d(cur_buf, cur, layers[i].w_bank, layers[i].c_out, layers[i].g,
                             layers[i].thr_lo, layers[i].thr_hi, nullptr, dst, stream);
        }
        if (rc != TERN_OK) return rc;
        if (layer_out) layer_out[i] = dst;
        cur_buf = dst;
        cur = o;
    }
    return TERN_OK;
}

int tern_fcn_forward(const float* in, tern_dims in_dims, const float* in_lo, const float* in_hi,
                     const tern_layer* layers, int32_t n_layers, void* workspace,
                     size_t workspace_bytes, uint32_t* out_packed, tern_dims* out_dims,
                     uint32_t** layer_out, void* stream)
{
    if (!in || !in_lo || !in_hi || !layers || !workspace || !out_packed) return TERN_ENULL;
    size_t need = 0;
    tern_dims last;
    int rc = fcn_plan(in_dims, layers, n_layers, &need, &last);
    if (rc != TERN_OK) return rc;
    for (int i = 0; i < n_layers; ++i)
        if (!layers[i].w_bank || !layers[i].thr_lo || !layers[i].thr_hi) return TERN_ENULL;
    if (workspace_bytes < need || !aligned16(workspace)) return TERN_EWORKSPACE;
    if (!aligned16(out_packed)) return TERN_EARG;
    rc = fcn_run(in, in_dims, in_lo, in_hi, layers, n_layers, workspace, out_packed, layer_out, stream);
    if (rc != TERN_OK) return rc;
    if (out_dims) *out_dims = last;
    return TERN_OK;
}

// ---- the chain for callers that cannot allocate ---------------------------------------------
// The activations between layers live in a file-scope device array instead of a caller's
// workspace.  Every GPU the library runs on holds its own copy of the array at its own address;
// in host code the array's name is only a handle for hipGetSymbolAddress, never an address to
// pass to a kernel.  The address is looked up once per device, with that device current.
static constexpr size_t kStaticScratchBytes = (size_t)TERN_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on device i, or null

// Device address of the current device's copy of the scratch array (resolved on first use).
static int scratch_for_current_device(void** out)
{
    int dev = 0;
    TERN_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return TERN_EARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        TERN_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return TERN_EHIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return TERN_OK;
}

size_t tern_static_scratch_bytes(void) { return kStaticScratchBytes; }

int tern_fcn_forward_static(const float* in, tern_dims in_dims, const float* in_lo, const float* in_hi,
                            const tern_layer* layers, int32_t n_layers, uint32_t* out_packed,
                            tern_dims* out_dims, uint32_t** layer_out, void* stream)
{
    if (!in || !in_lo || !in_hi || !layers || !out_packed) return TERN_ENULL;
    size_t need = 0;
    tern_dims last;
    int rc = fcn_plan(in_dims, layers, n_layers, &need, &last);
    if (rc != TERN_OK) return rc;
    for (int i = 0; i < n_layers; ++i)
        if (!layers[i].w_bank || !layers[i].thr_lo || !layers[i].thr_hi) return TERN_ENULL;
    if (need > kStaticScratchBytes) return TERN_EWORKSPACE;   // chain too large for the fixed array
    if (!aligned16(out_packed)) return TERN_EARG;
    void* ws = nullptr;
    rc = scratch_for_current_device(&ws);
    if (rc != TERN_OK) return rc;
    // every region of the scratch that a kernel of the chain reads was written by an earlier
    // kernel of the same call, so nothing has to be cleared between calls
    rc = fcn_run(in, in_dims, in_lo, in_hi, layers, n_layers, ws, out_packed, layer_out, stream);
    if (rc != TERN_OK) return rc;
    if (out_dims) *out_dims = last;
    return TERN_OK;
}

// One walk over the modules: validates the wiring, reports extents, and lays the workspace out
// (regions of 256-byte granularity, in the order: packed input, then per module [concatenated
// input,] output).  With `run` the kernels are enqueued as well.
namespace {
struct NetWalk {
    const float* in; const float* in_lo; const float* in_hi;
    char* ws; hipStream_t stream; bool run;
    uint32_t** module_out; tern_dims* module_dims;
};

inline size_t region(const tern_dims& d) { return (tern_packed_bytes(d) + 255u) & ~(size_t)255u; }

int net_walk(tern_dims in_dims, const tern_module* mods, int32_t n_mods, NetWalk* w, size_t* total,
             tern_dims* last_dims, const uint32_t** last_ptr)
{
    if (!mods) return TERN_ENULL;
    if (n_mods < 1 || n_mods > 1024) return TERN_EARG;
    if (!sizes_ok(in_dims)) return TERN_ESHAPE;
    std::vector<tern_dims> odims((size_t)n_mods);
    std::vector<size_t> ooff((size_t)n_mods);
    size_t off = 0;
    const size_t in_off = off;
    // Module 0 on a one-channel input with a 3x3x3 / 1x3x3 kernel: the input region holds the
    // gathered taps of every output voxel instead of the packed input (see tern_fcn_forward).
    bool gathered = false;
    tern_dims o0 = in_dims;
    {
        const tern_module& m0 = mods[0];
        const bool plain = m0.skip_from == -1 && m0.up[0] == 1 && m0.up[1] == 1 && m0.up[2] == 1 &&
                           m0.pool[0] <= 1 && m0.pool[1] <= 1 && m0.pool[2] <= 1;
        if (plain && geom_check(in_dims, m0.c_out, m0.g, &o0) == TERN_OK)
            gathered = patch_pack_applies(in_dims.c, m0.g, o0);
    }
    if (gathered) {
        const tern_dims patches = {o0.n, mods[0].g.k[0] * mods[0].g.k[1] * mods[0].g.k[2], o0.d, o0.h, o0.w};
        off += region(patches);
    } else {
        off += region(in_dims);
    }
    PatchParams first = {};
    bool fused = false;
    if (w && w->run) {
        int rc;
        if (gathered) {
            const tern_conv_geom& g = mods[0].g;
            PatchParams pp;
            pp.src = w->in; pp.lo = w->in_lo; pp.hi = w->in_hi; pp.dst = (uint32_t*)(w->ws + in_off);
            pp.d = in_dims.d; pp.h = in_dims.h; pp.w = in_dims.w;
            pp.od = o0.d; pp.oh = o0.h; pp.ow = o0.w;
            pp.kd = g.k[0]; pp.kh = g.k[1]; pp.kw = g.k[2];
            pp.sh = g.stride[1]; pp.sw = g.stride[2];
            pp.pd = g.pad[0]; pp.ph = g.pad[1]; pp.pw = g.pad[2];
            pp.dh = g.dil[1]; pp.dw = g.dil[2];
            // module 0 runs behind the gathering in the same kernel (below) where that pays; the
            // region reserved for the tap strings then stays unused
            first = pp;
            fused = patch_conv_pays(pp, in_dims.n);
            rc = fused ? TERN_OK : launch_patch_pack_f32(pp, in_dims.n, w->stream);
        } else {
            rc = tern_threshold_pack(w->in, TERN_SRC_F32, in_dims, w->in_lo, w->in_hi,
                                     (uint32_t*)(w->ws + in_off), w->stream);
        }
        if (rc != TERN_OK) return rc;
    }
    tern_dims cur = in_dims;
    size_t cur_off = in_off;
    for (int i = 0; i < n_mods; ++i) {
        const tern_module& m = mods[i];
        if (m.skip_from >= i || m.skip_from < -1) return TERN_EARG;
        for (int a = 0; a < 3; ++a)
            if (m.up[a] < 1 || m.up[a] > 1024) return TERN_EARG;
        const bool resample = m.up[0] > 1 || m.up[1] > 1 || m.up[2] > 1 || m.skip_from >= 0;
        if (resample) {
            const int64_t ud = (int64_t)cur.d * m.up[0], uh = (int64_t)cur.h * m.up[1], uw = (int64_t)cur.w * m.up[2];
            if (ud > INT32_MAX || uh > INT32_MAX || uw > INT32_MAX) return TERN_ESHAPE;
            tern_dims cat = {cur.n, cur.c, (int32_t)ud, (int32_t)uh, (int32_t)uw};
            tern_source src[2];
            src[0].packed = w && w->run ? (const uint32_t*)(w->ws + cur_off) : nullptr;
            src[0].dims = cur;
            for (int a = 0; a < 3; ++a) { src[0].up[a] = m.up[a]; src[0].first[a] = 0; }
            int n_src = 1;
            if (m.skip_from >= 0) {
                const tern_dims& sd = odims[(size_t)m.skip_from];
                const int32_t first[3] = {(sd.d - cat.d) / 2, (sd.h - cat.h) / 2, (sd.w - cat.w) / 2};
                if (sd.d < cat.d || sd.h < cat.h || sd.w < cat.w) return TERN_EARG;
                if ((int64_t)cat.c + sd.c > INT32_MAX) return TERN_ESHAPE;
                src[1].packed = w && w->run ? (const uint32_t*)(w->ws + ooff[(size_t)m.skip_from]) : nullptr;
                src[1].dims = sd;
                for (int a = 0; a < 3; ++a) { src[1].up[a] = 1; src[1].first[a] = first[a]; }
                cat.c += sd.c;
                n_src = 2;
            }
            if (!sizes_ok(cat)) return TERN_ESHAPE;
            const size_t cat_off = off;
            off += region(cat);
            if (w && w->run) {
                int rc = tern_concat(src, n_src, cat, (uint32_t*)(w->ws + cat_off), w->stream);
                if (rc != TERN_OK) return rc;
            }
            cur = cat;
            cur_off = cat_off;
        }
        // sum pooling in front of the module: two balanced-ternary digits per channel
        const bool pooled = m.pool[0] > 1 || m.pool[1] > 1 || m.pool[2] > 1;
        if (pooled) {
            for (int a = 0; a < 3; ++a)
                if (m.pool[a] < 1 || m.pool[a] > 4) return TERN_EARG;
            if (m.pool[0] * m.pool[1] * m.pool[2] > 4) return TERN_EARG;
            const int64_t c2 = 64 * (int64_t)tern_words(cur.c);
            if (c2 > INT32_MAX) return TERN_ESHAPE;
            const tern_dims pd = {cur.n, (int32_t)c2, cur.d / m.pool[0], cur.h / m.pool[1], cur.w / m.pool[2]};
            if (!sizes_ok(pd)) return TERN_ESHAPE;
            const size_t pool_off = off;
            off += region(pd);
            if (w && w->run) {
                const int rcp = tern_pool_digits((const uint32_t*)(w->ws + cur_off), cur, m.pool,
                                                 (uint32_t*)(w->ws + pool_off), w->stream);
                if (rcp != TERN_OK) return rcp;
            }
            cur = pd;
            cur_off = pool_off;
        }
        tern_dims o;
        int rc = geom_check(cur, m.c_out, m.g, &o);
        if (rc != TERN_OK) return rc;
        odims[(size_t)i] = o;
        ooff[(size_t)i] = off;
        off += region(o);
        if (w && w->run) {
            if (!m.w_bank || !m.thr_lo || !m.thr_hi) return TERN_ENULL;
            if (i == 0 && gathered && !fused) {
                // single-tap convolution over the gathered words
                const int32_t taps = m.g.k[0] * m.g.k[1] * m.g.k[2];
                const tern_dims pin = {o.n, taps, o.d, o.h, o.w};
                const tern_conv_geom unit = {{1, 1, 1}, {1, 1, 1}, {0, 0, 0}, {1, 1, 1}};
                if (!aligned16(m.w_bank)) return TERN_EARG;
                rc = launch_conv3d(conv_params((const uint32_t*)(w->ws + cur_off), pin, m.w_bank, m.c_out, unit,
                                               o, m.thr_lo, m.thr_hi, nullptr,
                                               (uint32_t*)(w->ws + ooff[(size_t)i])),
                                   w->stream);
            } else if (i == 0 && gathered) {
                // gathering and single-tap convolution over the gathered words in one kernel
                if (!aligned16(m.w_bank)) return TERN_EARG;
                FirstConvParams fc;
                fc.wgt = m.w_bank; fc.lo = m.thr_lo; fc.hi = m.thr_hi;
                fc.out_packed = (uint32_t*)(w->ws + ooff[(size_t)i]);
                fc.c_out = m.c_out; fc.co_pad = (m.c_out + 31) / 32 * 32;
                fc.wd_out = tern_words(m.c_out);
                rc = launch_patch_conv_f32(first, fc, in_dims.n, w->stream);
            } else if (pooled) {
                rc = tern_conv3d_digits((const uint32_t*)(w->ws + cur_off), cur, m.w_bank, m.c_out, m.g,
                                        m.thr_lo, m.thr_hi, nullptr, (uint32_t*)(w->ws + ooff[(size_t)i]),
                                        w->stream);
            } else {
                rc = tern_conv3d((const uint32_t*)(w->ws + cur_off), cur, m.w_bank, m.c_out, m.g, m.thr_lo,
                                 m.thr_hi, nullptr, (uint32_t*)(w->ws + ooff[(size_t)i]), w->stream);
            }
            if (rc != TERN_OK) return rc;
            if (w->module_out) w->module_out[i] = (uint32_t*)(w->ws + ooff[(size_t)i]);
            if (w->module_dims) w->module_dims[i] = o;
        }
        cur = o;
        cur_off = ooff[(size_t)i];
    }
    if (total) *total = off;
    if (last_dims) *last_dims = cur;
    if (last_ptr) *last_ptr = w && w->run ? (const uint32_t*)(w->ws + cur_off) : nullptr;
    return TERN_OK;
}
}  // namespace

size_t tern_net_workspace_bytes(tern_dims in_dims, const tern_module* mods, int32_t n_mods)
{
    size_t total = 0;
    if (net_walk(in_dims, mods, n_mods, nullptr, &total, nullptr, nullptr) != TERN_OK) return 0;
    return total;
}

int tern_net_forward(const float* in, tern_dims in_dims, const float* in_lo, const float* in_hi,
                     const tern_module* mods, int32_t n_mods, const float* head_w, const float* head_b,
                     int32_t head_c_out, tern_conv_geom head_g, void* workspace, size_t workspace_bytes,
                     float* head_out, tern_dims* head_dims, uint32_t** module_out,
                     tern_dims* module_dims, void* stream)
{
    if (!in || !in_lo || !in_hi || !mods || !workspace) return TERN_ENULL;
    if (head_w && !head_out) return TERN_ENULL;
    if (n_mods >= 1 && n_mods <= 1024)
        for (int i = 0; i < n_mods; ++i)
            if (!mods[i].w_bank || !mods[i].thr_lo || !mods[i].thr_hi) return TERN_ENULL;
    size_t need = 0;
    tern_dims last;
    int rc = net_walk(in_dims, mods, n_mods, nullptr, &need, &last, nullptr);   // validate first
    if (rc != TERN_OK) return rc;
    tern_dims hd = last;
    if (head_w) {
        rc = geom_check(last, head_c_out, head_g, &hd);
        if (rc != TERN_OK) return rc;
    }
    if (workspace_bytes < need || !aligned16(workspace)) return TERN_EWORKSPACE;
    NetWalk w = {in, in_lo, in_hi, (char*)workspace, (hipStream_t)stream, true, module_out, module_dims};
    const uint32_t* last_ptr = nullptr;
    rc = net_walk(in_dims, mods, n_mods, &w, nullptr, nullptr, &last_ptr);
    if (rc != TERN_OK) return rc;
    if (head_w) {
        rc = tern_conv3d_real(last_ptr, last, head_w, head_b, head_c_out, head_g, head_out, stream);
        if (rc != TERN_OK) return rc;
        if (head_dims) *head_dims = hd;
    }
    return TERN_OK;
}

}  // extern "C"
