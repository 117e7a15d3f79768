/*
 * tern_matrix.h -- an experiment beside the library's contract: the ternary convolution of tern.h
 * evaluated on the matrix instructions of gfx950 instead of by bit counts.  Nothing in tern.h
 * dispatches to these calls; they take the same packed activations and give the same bits as
 * tern_conv3d, and exist to compare the two ways of taking the inner products of section 2 on
 * this device.  Conventions (device pointers, streams, status codes) as in tern.h.
 */
#ifndef TERN_MATRIX_H
#define TERN_MATRIX_H

#include "tern.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * tern_conv3d_mfma -- the same convolution, same arguments, same results bit for bit, with the
 * inner products of section 2 (the sums that Eq. 9 evaluates by two bit-counts) taken by the
 * matrix instructions instead: activations stay packed in memory, a workgroup expands its halo
 * tile in LDS and multiplies it with an expanded filter bank.  Not the paper's scheme (which
 * exists because CPUs count bits faster than they multiply); provided because on this device the
 * matrix cores multiply faster than the vector units count.
 *   kind        : TERN_MATRIX_I8 -- one byte per code (0x01 / 0xff / 0x00), int8 products, int32
 *                 sums; TERN_MATRIX_F4 -- four bits per code (the E2M1 values +1, -1, 0), float
 *                 sums, exact because every partial sum is an integer below 2^24 (TERN_ESHAPE if
 *                 k-volume * C_in >= 2^24); twice the rate of the former.
 *   matrix_bank : tern_matrix_bank_bytes(...) bytes, 16-byte aligned, made once per layer by
 *                 tern_expand_filters from the same int8 weights [C_out][C_in][kd][kh][kw] that
 *                 tern_pack_filters takes.  Layout [tap][step][block of 32 filters][half g]
 *                 [filter j][4 dwords q]; I8: step = word of 32 input channels, byte b of dword q
 *                 = channel 32 step + (4 g + q) + 8 b; F4: step = pair of words, 4-bit field i of
 *                 dword q = channel 32 (2 step + g) + 4 i + q (the order in which the kernel's
 *                 expansion of an activation word leaves the channels).  Zero past C_out and C_in.
 * Returns TERN_ESHAPE when the halo of an 8 x 8 x 2 block of outputs does not fit in LDS (very
 * large strides or dilations); tern_conv3d has no such limit.
 */
typedef enum { TERN_MATRIX_I8 = 0, TERN_MATRIX_F4 = 1 } tern_matrix_kind;
size_t tern_matrix_bank_bytes(int32_t c_out, int32_t c_in, int32_t kd, int32_t kh, int32_t kw,
                              int32_t kind);
int tern_expand_filters(const int8_t* w, int32_t c_out, int32_t c_in, int32_t kd, int32_t kh,
                        int32_t kw, int32_t kind, uint32_t* matrix_bank, void* stream);
int tern_conv3d_mfma(const uint32_t* in_packed, tern_dims in_dims,
                     const uint32_t* matrix_bank, int32_t kind, int32_t c_out, tern_conv_geom g,
                     const int32_t* thr_lo, const int32_t* thr_hi,
                     int32_t* out_acc, uint32_t* out_packed, void* stream);
/*
 * tern_conv3d_mfma_digits -- tern_conv3d_digits (below) on the matrix cores: the convolution of
 * the window sums that a two-digit tensor of tern_pool_digits holds (values -4 .. 4, all of them
 * 4-bit float values), same results.  in_dims.c = 64 * words(C) as for tern_conv3d_digits;
 * matrix_bank is the TERN_MATRIX_F4 bank of the layer's own weights [C_out][C][taps] (not the
 * doubled ones of tern_digits_weights).  TERN_ESHAPE if 2 * k-volume * in_dims.c >= 2^24 or the
 * halo tile does not fit.
 */
int tern_conv3d_mfma_digits(const uint32_t* in_packed, tern_dims in_dims,
                            const uint32_t* matrix_bank, int32_t c_out, tern_conv_geom g,
                            const int32_t* thr_lo, const int32_t* thr_hi,
                            int32_t* out_acc, uint32_t* out_packed, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TERN_MATRIX_H */
