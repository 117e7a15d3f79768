/*
 * tern.h -- C ABI of the MI355X (gfx950) ternary 3D convolution library.
 *
 * The library implements the inference hot path of TernaryNet (Heinrich, Blendowski, Oktay,
 * "TernaryNet: Faster Deep Model Inference without GPUs for Medical 3D Segmentation using Sparse
 * and Binary Convolutions", arXiv 1801.09449): a convolution whose weights and activations are
 * both restricted to {-1, 0, +1}, evaluated as a masked Hamming distance on bit-planes (section 2,
 * Eq. 9), followed by the hard ternary activation (Eq. 6) and re-packing to 2 bits per value
 * (Fig. 3) so that modules can be chained (section 2, last paragraph).
 *
 * General rules
 *   - Every data pointer is a DEVICE pointer owned by the caller unless a comment says "host".
 *     The library never allocates, frees or retains caller memory and keeps no state between
 *     calls except the last HIP error code (tern_last_hip_error), the per-thread tuning
 *     overrides of tern_tuning.h and the fixed scratch array of tern_fcn_forward_static.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work
 *     on that stream and return without synchronising.
 *   - Return value: TERN_OK (0) or a negative tern_status.  No call throws or aborts.  Arguments
 *     are validated on the host before anything is launched; a failing call launches nothing.
 *   - Tensors with zero elements are rejected with TERN_ESHAPE.
 *
 * Unpacked tensors are contiguous NCDHW (W fastest).
 *
 * Packed ternary tensors (two bit-planes packed along the channel axis, Fig. 3 / section 2):
 *     uint32 [N][D][H][W][2][Wd],   Wd = tern_words(C) = ceil(C/32)
 *   plane 0 = nonzero mask, plane 1 = sign.  Bit j of word q describes channel 32q + j:
 *     value +1 -> mask 1, sign 0;   value -1 -> mask 1, sign 1;   value 0 -> mask 0, sign 0.
 *   Bits of channels >= C are 0 in both planes.  Producers in this library always emit this
 *   canonical form; consumers ignore sign bits under a clear mask bit.
 *   (The figure draws the complementary convention -- first bit set for +1, second bit a zero
 *   flag; the convolution result does not depend on the choice.)
 *   Packed buffers must be 16-byte aligned (any hipMalloc / torch allocation is).
 *
 * Filter banks (the ternary weights of one layer at two bits each, section 2) hold the same
 * two bit-planes but ordered for the convolution kernels, which fetch filter words through the
 * scalar cache one kernel tap at a time:
 *     uint32 [T * nchunk][co_pad][2][wc]
 *   T = kd*kh*kw taps in (a, b, c) order; Wd = ceil(C_in/32); wc = 2 if Wd is even, else 1;
 *   nchunk = Wd / wc; co_pad = C_out rounded up to a multiple of 32.  Entry [tap*nchunk + ch]
 *   [co][p][q] is plane p (0 mask, 1 sign) of input-channel word ch*wc + q of filter co at that
 *   tap; channels co >= C_out are all-zero.  Built by tern_pack_filters.
 *   Tap-packed variant, used when C_in <= 16 and T > 1 (a voxel's word would otherwise be mostly
 *   empty): shift = smallest power of two >= C_in, slots = min(32 / shift, T);
 *     uint32 [ceil(T / slots)][co_pad][2][1]
 *   and the word of row r holds taps r*slots .. r*slots + slots - 1, tap i of the row in bits
 *   [i*shift, i*shift + C_in).  The kernels build the matching activation word from the voxels of
 *   those taps, so one word pair covers up to 32 (tap, channel) products of Eq. 9.
 */
#ifndef TERN_H
#define TERN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TERN_OK = 0,
    TERN_ENULL = -1,        /* a required pointer is NULL                                   */
    TERN_ESHAPE = -2,       /* non-positive extent, empty output, or sizes beyond the limits */
    TERN_EARG = -3,         /* invalid combination of arguments                              */
    TERN_EWORKSPACE = -4,   /* workspace too small or misaligned                             */
    TERN_EHIP = -5          /* a HIP call failed; see tern_last_hip_error()                  */
} tern_status;

/* Logical NCDHW extents.  Limits: every extent >= 1; N*D*H*W <= 2^31 - 1 voxels per tensor (the
 * kernels count voxels in 32 bits; byte offsets are 64-bit, so tensors may exceed 4 GiB). */
typedef struct { int32_t n, c, d, h, w; } tern_dims;

/* Kernel extent, stride, zero padding (both sides) and dilation per axis, order (d, h, w).
 * Output extent per axis: floor((X + 2*pad - dil*(k-1) - 1)/stride) + 1; TERN_ESHAPE if < 1.
 * Limits: 1 <= k, stride, dil <= 1024 and 0 <= pad <= 2^20 per axis (else TERN_EARG);
 * k[0]*k[1]*k[2]*C_in < 2^24, which bounds |accumulator|, and C_out <= 2^19 (else TERN_ESHAPE). */
typedef struct { int32_t k[3], stride[3], pad[3], dil[3]; } tern_conv_geom;

typedef enum { TERN_SRC_I8 = 0, TERN_SRC_I32 = 1, TERN_SRC_F32 = 2 } tern_src_type;

/* ceil(c/32): 32-bit words per plane per voxel. */
int32_t tern_words(int32_t c);
/* Bytes of a packed tensor with these logical dims (0 if dims are invalid). */
size_t tern_packed_bytes(tern_dims dims);
/* Bytes of the filter bank of a layer (0 if the shape is invalid or beyond the limits). */
size_t tern_filter_bank_bytes(int32_t c_out, int32_t c_in, int32_t kd, int32_t kh, int32_t kw);
/* Output extents of a convolution; TERN_ESHAPE if the geometry does not fit. */
int tern_conv_out_dims(tern_dims in_dims, int32_t c_out, tern_conv_geom g, tern_dims* out_dims);
/* Raw hipError_t value recorded by the most recent call (on this host thread) that returned
 * TERN_EHIP. */
int tern_last_hip_error(void);
/* Human-readable name of a tern_status. */
const char* tern_status_string(int status);

/*
 * tern_pack -- 2-bit encoding of a ternary tensor (Fig. 3; section 2: two bits per entry, one
 * for the value, one for the sign).
 *   src        : int8 values in {-1, 0, +1}, contiguous [N][C][D][H][W].  Other values are not
 *                detected: a nonzero byte sets the mask bit and a negative one the sign bit.
 *   dst_packed : packed layout described above, tern_packed_bytes(dims) bytes.
 */
int tern_pack(const int8_t* src, tern_dims dims, uint32_t* dst_packed, void* stream);

/*
 * tern_pack_filters -- 2-bit encoding of a layer's ternary weights (section 2, last paragraph:
 * two bits are all a trained weight needs) in the filter-bank layout described above.
 *   w    : int8 values in {-1, 0, +1}, contiguous [C_out][C_in][kd][kh][kw] (other values are
 *          treated as in tern_pack).
 *   bank : tern_filter_bank_bytes(...) bytes, 16-byte aligned.
 * Done once per layer; the bank is then passed to tern_conv3d / tern_fcn_forward.
 */
int tern_pack_filters(const int8_t* w, int32_t c_out, int32_t c_in, int32_t kd, int32_t kh,
                      int32_t kw, uint32_t* bank, void* stream);

/*
 * tern_conv3d -- ternary convolution (cross-correlation) as a masked Hamming distance, Eq. 9:
 *   acc[n][co][z][y][x] = sum over taps (a,b,c) and channel words q of
 *        popcount(M) - 2*popcount(M & (sign_w ^ sign_a)),   M = mask_w & mask_a,
 *   with the activation voxel at (z*s - p + a*dil, ...) and all-zero words outside the volume
 *   (zero padding is the ternary value 0, which the mask excludes).  This equals the integer
 *   inner product of the ternary patch and filter.
 *
 *   in_packed : packed activations, logical dims in_dims (in_dims.c = C_in).
 *   w_bank    : filter bank of the layer (tern_pack_filters) for (c_out, C_in, g.k).
 *   Exactly one output mode per call:
 *     out_acc != NULL, out_packed == NULL : raw accumulators, int32 [N][c_out][Do][Ho][Wo];
 *                                           thr_lo / thr_hi are ignored.
 *     out_packed != NULL, out_acc == NULL : fused activation + re-pack (Eq. 6 with the
 *         per-channel scale and batch-norm folded into two integer cut points):
 *         code = +1 if acc > thr_hi[co]; -1 if acc < thr_lo[co]; else 0, written in the packed
 *         layout with logical dims {N, c_out, Do, Ho, Wo}.  thr_lo, thr_hi: int32[c_out] on the
 *         device, required, with thr_lo[co] <= thr_hi[co] + 1 (lo = hi + 1 is an empty zero
 *         band; not checked -- the values live on the device; if violated, +1 takes precedence
 *         where both comparisons hold).
 *   Both non-NULL or both NULL -> TERN_EARG.  Buffers must not overlap.
 */
int tern_conv3d(const uint32_t* in_packed, tern_dims in_dims,
                const uint32_t* w_bank, int32_t c_out, tern_conv_geom g,
                const int32_t* thr_lo, const int32_t* thr_hi,
                int32_t* out_acc, uint32_t* out_packed, void* stream);

/*
 * tern_pack_filters_binary / tern_conv3d_binary -- the binary special case, Eq. 8: with weights
 * and activations in {-1, +1} the inner product of c-element vectors is c - 2 * popcount(I xor W),
 * one xor and one bit count per word pair instead of the two of each that Eq. 9 needs.
 *
 * tern_conv3d_binary is tern_conv3d for filters without zeros.  The activations come in the same
 * packed layout and their mask plane is honoured, so that zero padding (the ternary value 0) and
 * any zero code drop out exactly as in Eq. 9:
 *   acc[n][co][z][y][x] = sum over taps and channel words of
 *        popcount(mask_a) - 2 * popcount(mask_a & (sign_a ^ sign_w)),
 * which for an input without zeros, away from the padded border, is Eq. 8 with c = k-volume *
 * C_in, and in general equals the integer inner product of the ternary patch with the +-1 filter.
 * Output modes, cut points, limits and errors as for tern_conv3d (cut points with lo = hi + 1 give
 * an output without zeros, i.e. the sign activation of a binary network).
 *   w      : int8 [C_out][C_in][kd][kh][kw] with values -1 / +1 (not checked: a negative byte is
 *            read as -1, anything else, 0 included, as +1).
 *   bank   : tern_binary_bank_bytes(...) bytes, 16-byte aligned: uint32 [T * nchunk][co_pad][wc]
 *            sign words (T, nchunk, wc, co_pad as for the ternary filter bank, always the plain
 *            layout); bit j of word q is set where the weight of input channel 32q + j is -1;
 *            filters co >= C_out and channels >= C_in are zero.
 */
size_t tern_binary_bank_bytes(int32_t c_out, int32_t c_in, int32_t kd, int32_t kh, int32_t kw);
int tern_pack_filters_binary(const int8_t* w, int32_t c_out, int32_t c_in, int32_t kd, int32_t kh,
                             int32_t kw, uint32_t* bank, void* stream);
int tern_conv3d_binary(const uint32_t* in_packed, tern_dims in_dims,
                       const uint32_t* w_bank, int32_t c_out, tern_conv_geom g,
                       const int32_t* thr_lo, const int32_t* thr_hi,
                       int32_t* out_acc, uint32_t* out_packed, void* stream);

/*
 * tern_threshold_pack -- the hard ternary activation of Eq. 6 followed by 2-bit packing, on a
 * tensor that is already in memory:  code = +1 if v > hi[c]; -1 if v < lo[c]; else 0.
 *   src    : contiguous [N][C][D][H][W] of type t (TERN_SRC_I32: int32 accumulators with int32
 *            cut points; TERN_SRC_F32: float values with float cut points, e.g. raw intensities
 *            at -0.5 / +0.5; a NaN becomes 0).  TERN_SRC_I8 is not accepted here (TERN_EARG).
 *   thr_lo, thr_hi : C entries of the source type, device memory, lo[c] <= hi[c] (int32:
 *            lo[c] <= hi[c] + 1); not checked.
 */
int tern_threshold_pack(const void* src, tern_src_type t, tern_dims dims,
                        const void* thr_lo, const void* thr_hi,
                        uint32_t* dst_packed, void* stream);

/* One TernaryNet module (section 2, last paragraph: ternary convolution, batch-norm, ternary
 * activation).  The struct lives in HOST memory; the pointers inside are DEVICE pointers. */
typedef struct {
    int32_t c_in, c_out;
    tern_conv_geom g;
    const uint32_t* w_bank;     /* filter bank from tern_pack_filters       */
    const int32_t* thr_lo;      /* [c_out] */
    const int32_t* thr_hi;      /* [c_out] */
} tern_layer;

/* Bytes of scratch that tern_fcn_forward needs for this chain (0 if the chain is invalid:
 * channel mismatch between consecutive layers or a geometry that does not fit). */
size_t tern_fcn_workspace_bytes(tern_dims in_dims, const tern_layer* layers /* host */,
                                int32_t n_layers);

/*
 * tern_fcn_forward -- a chain of modules with activations kept packed between layers.
 *   in        : float [N][C0][D][H][W] raw intensities, ternarised per channel at
 *               (in_lo[c], in_hi[c]) (device float[C0]; Eq. 6 uses -0.5 / +0.5) and packed;
 *   layers    : host array of n_layers >= 1 modules, layers[0].c_in == in_dims.c and
 *               layers[i].c_in == layers[i-1].c_out;
 *   workspace : device scratch of at least tern_fcn_workspace_bytes() bytes, 16-byte aligned;
 *               holds the packed activations of the input and of every layer but the last.
 *               (With a one-channel input and a 3x3x3, 1x3x3 or 15x3x3 first kernel of unit
 *               depth stride and dilation, the input region instead holds, per
 *               output voxel of layer 0, that voxel's kernel taps gathered into a bit string:
 *               Eq. 6 and the gathering run as one pass over the intensities and layer 0
 *               becomes a single-tap convolution, which usually runs in that same pass on the
 *               strings in registers; the region is then reserved but not written.  Results
 *               are identical either way.)
 *               When layer_out (host array of n_layers pointers, may be NULL) is given,
 *               layer_out[i] receives the device address of layer i's packed output (inside
 *               workspace, or out_packed for the last layer) so that callers can inspect every
 *               layer; nothing is overwritten within one call.
 *   out_packed: packed output of the last layer; out_dims (host, may be NULL) receives its
 *               logical dims.
 * All kernels are enqueued on `stream` in order; there is no host synchronisation.
 */
int tern_fcn_forward(const float* in, tern_dims in_dims, const float* in_lo, const float* in_hi,
                     const tern_layer* layers /* host */, int32_t n_layers,
                     void* workspace, size_t workspace_bytes,
                     uint32_t* out_packed, tern_dims* out_dims /* host */,
                     uint32_t** layer_out /* host, optional */, void* stream);

/*
 * tern_fcn_forward_static -- tern_fcn_forward for callers that cannot allocate device memory and
 * have no workspace to hand over: code recorded into a HIP graph, tight serving loops, harnesses
 * that forbid allocation.  Same arguments without the workspace, same results; the activations
 * between layers go to a fixed device array of TERN_STATIC_SCRATCH_BYTES that is part of the
 * library's code object (every GPU the library is used on holds its own copy until the process
 * ends).  The call allocates and frees nothing; a chain whose tern_fcn_workspace_bytes() exceeds
 * tern_static_scratch_bytes() is refused with TERN_EWORKSPACE before anything is launched.
 *   - All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU
 *     (different streams, or different host threads) race on it.  Calls on one stream are safe.
 *   - The array keeps the previous call's contents; nothing needs clearing, because every region a
 *     kernel of the chain reads was written earlier in the same call.
 *   - layer_out[i] (optional) receives addresses inside that array for every layer but the last;
 *     they are valid until the next call on the same GPU.
 *   - The first call on a device looks the array's address up (and thereby loads the library's
 *     code object if nothing has yet); make one ordinary call before recording a graph.
 */
#define TERN_STATIC_SCRATCH_BYTES (32u << 20)
size_t tern_static_scratch_bytes(void);
int tern_fcn_forward_static(const float* in, tern_dims in_dims, const float* in_lo, const float* in_hi,
                            const tern_layer* layers /* host */, int32_t n_layers,
                            uint32_t* out_packed, tern_dims* out_dims /* host */,
                            uint32_t** layer_out /* host, optional */, void* stream);

/*
 * U-Net plumbing on packed activations (section 3, Table 1: the Upsample2D rows, the "Skip"
 * column, the AvgPool2D rows and the Prediction row; section 2 notes that skip connections and
 * feature concatenation are usable with ternary convolutions).
 *
 * tern_concat -- output voxel (n, z, y, x) takes, from every source i in turn, the channels of
 * source voxel (n, (z + first[0]) / up[0], (y + first[1]) / up[1], (x + first[2]) / up[2])
 * (integer division: nearest-neighbour upsampling by `up`, then a crop that starts at `first`
 * in upsampled coordinates) and lays them side by side: source 0 fills channels
 * [0, c0), source 1 [c0, c0 + c1), ...  One source with up = 1 is a crop, with up = 2 an
 * upsampling; two sources are a decoder step (upsampled tensor + cropped skip tensor).
 *   srcs      : host array of n_src (1 .. TERN_MAX_SOURCES) descriptors; `packed` are device
 *               pointers in the packed layout of `dims`; dims.n == out_dims.n;
 *               1 <= up <= 1024, first >= 0, first + out extent <= dims extent * up per axis;
 *   out_dims  : out_dims.c must equal the sum of the sources' channel counts (any counts: bits
 *               are shifted across word boundaries when a count is not a multiple of 32);
 *   out_packed: packed output, must not overlap a source.
 * Errors: TERN_EARG for a violated constraint, TERN_ESHAPE for invalid extents.
 *
 * tern_conv3d_real -- the full-precision output layer: cross-correlation of packed ternary codes
 * with float weights w [c_out][C_in][kd][kh][kw] plus bias [c_out] (NULL = none), zero padding,
 * float output [N][c_out][Do][Ho][Wo].  Each term is +-w exactly; they are added in fp32 in the
 * order taps (d, h, w), then ascending input channel, starting from the bias, so the result
 * differs from exact arithmetic by at most (terms) * 2^-24 * (|bias| + sum |w| over the filter).
 * Meant for a handful of output channels (Table 1: 2); one thread per output voxel.
 *
 * tern_pool_digits / tern_digits_weights / tern_conv3d_digits -- average pooling in front of a
 * ternary convolution (Table 1: AvgPool 2x2 before modules 4, 6 and 8) at twice, not four times,
 * the cost of the pooled convolution.  The sum of up to four ternary codes lies in [-4, 4] and has
 * exactly one representation low + 3 * high with both digits in {-1, 0, +1} (balanced ternary).
 * tern_pool_digits writes, for non-overlapping windows of at most 4 voxels (window[a] >= 1,
 * product <= 4; trailing voxels that do not fill a window are dropped), the two digits of every
 * window sum as a packed tensor [N][d/wd][h/wh][w/ww] with 64 * words(C) channels: word 2k of a
 * plane holds the low digits of channels 32k .. 32k+31, word 2k+1 their high digits.
 * tern_conv3d_digits is tern_conv3d on such a tensor (in_dims.c = that channel count, a multiple
 * of 64) with the odd words counted three times, i.e. the exact convolution of the window sums;
 * the cut points then refer to sums, not averages (scale them by the window volume).  Its filter
 * bank is tern_pack_filters applied to the weights that tern_digits_weights (host arrays,
 * launches nothing) makes from w [c_out][c_in][taps]: w_out [c_out][64 * words(c_in)][taps] with
 * channel 64k + j and 64k + 32 + j both equal to channel 32k + j of w (zero past c_in).
 * Limits as for tern_conv3d with k-volume * in_dims.c < 2^23.
 *
 * tern_fold_avgpool (host arrays, launches nothing) -- average pooling between two ternary
 * modules, done exactly: pooling with window = stride = pool followed by a convolution with
 * kernel k, stride s, padding p, dilation 1 equals, up to the constant factor
 * P = pool[0]*pool[1]*pool[2], a convolution of the unpooled tensor with kernel k*pool (every
 * tap repeated pool times along each axis), stride s*pool and padding p*pool.  The helper
 * writes those repeated filters, w_out int8 [c_out][c_in][kd*pool[0]][kh*pool[1]][kw*pool[2]];
 * the accumulator of the folded convolution is P times that of the pooled one, so pass
 * scale/P to tern_fold_thresholds.  Without padding the output extents and values are identical
 * to pool-then-convolve for any input extent (trailing voxels that do not fill a pooling window
 * are never reached); with padding p > 0 the input extents must be multiples of the pooling
 * window, otherwise the folded convolution would read those trailing voxels where the pooled
 * one reads padding.
 */
#define TERN_MAX_SOURCES 8
typedef struct {
    const uint32_t* packed;     /* device: packed activations of this source           */
    tern_dims dims;             /* its logical extents                                  */
    int32_t up[3];              /* nearest-neighbour upsampling factor per axis (d,h,w) */
    int32_t first[3];           /* upsampled coordinate that lands on output voxel 0    */
} tern_source;
int tern_concat(const tern_source* srcs /* host */, int32_t n_src, tern_dims out_dims,
                uint32_t* out_packed, void* stream);
int tern_conv3d_real(const uint32_t* in_packed, tern_dims in_dims, const float* w,
                     const float* bias, int32_t c_out, tern_conv_geom g, float* out,
                     void* stream);
int tern_pool_digits(const uint32_t* in_packed, tern_dims in_dims, const int32_t window[3] /* host */,
                     uint32_t* out_packed, void* stream);
int tern_digits_weights(const int8_t* w /* host */, int32_t c_out, int32_t c_in, int64_t taps,
                        int8_t* w_out /* host */);
int tern_conv3d_digits(const uint32_t* in_packed, tern_dims in_dims, const uint32_t* w_bank,
                       int32_t c_out, tern_conv_geom g, const int32_t* thr_lo, const int32_t* thr_hi,
                       int32_t* out_acc, uint32_t* out_packed, void* stream);
/*
 * tern_net_forward -- a network of ternary modules with skip connections (the baseline U-Net of
 * section 3 / Table 1, or any encoder-decoder of that kind), run as one call: Eq. 6 on the float
 * input, then for every module, in order, [nearest upsampling of the incoming tensor and
 * appending of an earlier module's centre-cropped output, via the tern_concat kernel] and a
 * fused tern_conv3d; optionally a float-weight prediction layer (tern_conv3d_real) on the last
 * module's output.  Average pooling in front of a module is expressed either through the
 * module's filters and stride (tern_fold_avgpool; pool left at 1) or through pool[]: the
 * incoming tensor (after upsampling and concatenation, if any) is sum-pooled over windows of
 * pool[] voxels (product <= 4) into two digits (tern_pool_digits) and the convolution runs on
 * those (tern_conv3d_digits: w_bank then is the bank of tern_digits_weights' output, the cut
 * points refer to window sums).  A chain without skips and upsampling is what tern_fcn_forward
 * runs.
 *   mods       : host array; module i reads the output of module i-1 (the packed input for
 *                i = 0), upsampled by up[] when any factor is > 1, followed channel-wise by the
 *                output of module skip_from (-1 = none; must be < i), centre-cropped to the
 *                (upsampled) incoming extent: first voxel floor((X_skip - X)/2) per axis, which
 *                must not be negative.  w_bank holds filters for that total channel count.
 *   head_w     : float [head_c_out][C_last][k] on the device, NULL = no prediction layer (then
 *                head_b, head_out are ignored); head_b may be NULL; head_out receives
 *                [N][head_c_out][Do][Ho][Wo] floats, head_dims (host, optional) its extents.
 *   workspace  : device scratch of at least tern_net_workspace_bytes() bytes, 16-byte aligned;
 *                holds the packed input (or, as in tern_fcn_forward, the gathered taps of a
 *                one-channel input's first module), every module's output and every
 *                concatenated or pooled tensor, each in a region of its own (nothing is
 *                overwritten within a call).
 *   module_out / module_dims : optional host arrays of n_mods entries that receive the device
 *                address (inside workspace) and logical extents of every module's packed output.
 * Errors as for the calls it is made of; TERN_EARG for an invalid skip_from or crop,
 * TERN_EWORKSPACE for a workspace that is too small or misaligned.  Everything is enqueued on
 * `stream` in order; no host synchronisation.
 */
typedef struct {
    int32_t c_out;
    tern_conv_geom g;
    const uint32_t* w_bank;
    const int32_t* thr_lo;
    const int32_t* thr_hi;
    int32_t skip_from;
    int32_t up[3];
    int32_t pool[3];            /* {1,1,1} or all 0: none; else sum pooling through two digits */
} tern_module;
size_t tern_net_workspace_bytes(tern_dims in_dims, const tern_module* mods /* host */, int32_t n_mods);
int tern_net_forward(const float* in, tern_dims in_dims, const float* in_lo, const float* in_hi,
                     const tern_module* mods /* host */, int32_t n_mods,
                     const float* head_w, const float* head_b, int32_t head_c_out, tern_conv_geom head_g,
                     void* workspace, size_t workspace_bytes,
                     float* head_out, tern_dims* head_dims /* host, optional */,
                     uint32_t** module_out /* host, optional */, tern_dims* module_dims /* host, optional */,
                     void* stream);

/*
 * tern_count_codes -- per-channel statistics of a packed tensor (the paper discusses how sparse
 * the ternary weights and activations are, section 4): nonzero[c] = number of voxels (over the
 * whole batch) whose channel c is +1 or -1, negative[c] = number whose channel c is -1; the zero
 * fraction of channel c is 1 - nonzero[c] / (N*D*H*W).  Both arrays: device, dims.c entries of
 * uint64, 8-byte aligned, overwritten.  Sign bits under a clear mask bit are ignored.  Exact
 * (integer atomics); works on filter tensors too when they are packed with tern_pack as
 * {C_out, C_in, kd, kh, kw} (statistics then are per input channel).
 */
int tern_count_codes(const uint32_t* in_packed, tern_dims dims, uint64_t* nonzero, uint64_t* negative,
                     void* stream);
int tern_fold_avgpool(const int8_t* w /* host */, int32_t c_out, int32_t c_in, int32_t kd,
                      int32_t kh, int32_t kw, const int32_t pool[3], int8_t* w_out /* host */);

/*
 * Host-side model preparation.  These run on the CPU on HOST arrays and launch nothing.
 *
 * tern_ternarize_filters -- ternary weight approximation W ~ alpha * W~ (Eq. 4), per output
 * filter: Delta = 0.7/n * sum|W_i|;  W~_i = +1 if W_i > Delta, 0 if |W_i| <= Delta, -1 otherwise;
 * alpha = mean of |W_i| over the nonzero W~_i (0 if there are none).  Sums in double.
 *   w      : float [c_out][per_filter]  (per_filter = C_in*kd*kh*kw, the filter's own order)
 *   codes  : int8  [c_out][per_filter]  (ready for tern_pack_filters once copied to the device)
 *   alpha  : double[c_out]
 *
 * tern_ternarize_filters_sparse -- the same with a prescribed sparsity (section 2, the remark
 * after Eq. 9: Delta placed so that a given share of every kernel's entries, half in the paper's
 * example, is zero).  Per output filter the `zeros` entries of smallest magnitude become 0 (equal
 * magnitudes in index order), the others take their sign (an entry that is exactly 0 stays 0, so
 * there can be more zeros than asked for); alpha = mean magnitude of the nonzero codes' entries.
 * 0 <= zeros <= per_filter, else TERN_EARG.  Only the quantiser is provided: the convolution
 * treats such filters like any others (the paper does not say how the bit-counts would halve).
 *
 * tern_fold_thresholds -- integer cut points for the activation of Eq. 6 applied to
 * y = scale[c]*acc + shift[c] (scale and shift collect alpha and the batch-norm affine, which sit
 * between convolution and activation in a TernaryNet module, section 2).  For every integer acc
 * with |acc| <= acc_bound:  (+1 if acc > hi[c]; -1 if acc < lo[c]; else 0) equals the
 * double-precision evaluation (+1 if y > 0.5; 0 if |y| <= 0.5; else -1), ties included.
 * A channel with negative scale gets negate[c] = 1 and cut points for |scale|: the caller must
 * negate that filter's ternary codes (conv(-w) = -conv(w)).  scale = 0 gives a constant channel.
 * acc_bound: 1 .. 2^24-1, normally C_in*kd*kh*kw.  Non-finite scale/shift -> TERN_EARG.
 *
 * tern_fold_batchnorm -- the same with scale = alpha*gamma/sqrt(var+eps) and
 * shift = beta - gamma*mean/sqrt(var+eps) computed in double.
 */
int tern_ternarize_filters(const float* w /* host */, int32_t c_out, int64_t per_filter,
                           int8_t* codes /* host */, double* alpha /* host */);
int tern_ternarize_filters_sparse(const float* w /* host */, int32_t c_out, int64_t per_filter,
                                  int64_t zeros, int8_t* codes /* host */, double* alpha /* host */);
int tern_fold_thresholds(const double* scale /* host */, const double* shift /* host */, int32_t c,
                         int32_t acc_bound, int32_t* lo /* host */, int32_t* hi /* host */,
                         uint8_t* negate /* host */);
int tern_fold_batchnorm(const double* alpha, const double* gamma, const double* beta,
                        const double* mean, const double* var, double eps, int32_t c,
                        int32_t acc_bound, int32_t* lo, int32_t* hi, uint8_t* negate);

#ifdef __cplusplus
}
#endif
#endif /* TERN_H */
