/*
 * tern_tuning.h -- tuning overrides and a diagnostic of the ternary convolution library.  Not part
 * of the library's contract (tern.h): results never depend on anything declared here.
 */
#ifndef TERN_TUNING_H
#define TERN_TUNING_H

#include "tern.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Tuning overrides.  They belong to the calling host thread: a launch reads the values set by
 * its own thread, so another thread's tern_set_option cannot change a plan half-way through; a
 * new thread starts with the defaults (everything chosen per call from the problem size).  TERN_OPT_LANE_DEPTH: output voxels per lane along z in
 * the tiled convolution kernel, 0 = choose automatically, 1, 2 or 4 = force (1 and 4 only
 * where that variant exists).  TERN_OPT_WAVES_Z: waves
 * stacked along z in one workgroup (sharing one LDS halo tile), 0 = choose, 1, 2, 4 or 8 = start
 * from that value.  TERN_OPT_CO_BLOCK: output channels per accumulation pass, 0 = choose, 16 or 32.
 * TERN_OPT_CO_PER_WAVE: output channels handled by one wave, 0 = choose, else a multiple of 16.
 * TERN_OPT_TAP_SPLIT: waves of one workgroup that share the kernel taps of one channel slice and
 * add their partial sums in LDS, 0 = choose, 1, 2, 4 or 8.  TERN_OPT_POINTWISE: 1 (default) = 1x1x1
 * convolutions with unit stride and no padding use the pointwise kernel when the input has 1, 2,
 * 3, 4, 5 or 8 words per plane, 0 = they go through the tiled kernel like any other.
 * TERN_OPT_LANE_TILE: the block of 64 output voxels that one wave of the tiled kernel computes,
 * 0 = choose (8 x 8 in a plane, or a smaller footprint over several planes where that wastes fewer
 * lanes on the edges of a stack of independent planes), -1 = always 8 x 8, 100 * X + Y with X, Y in
 * {1, 2, 4, 8} and X * Y >= 4 = X x Y voxels in 64 / (X * Y) planes wherever the output has more
 * than one plane.
 * TERN_OPT_STREAM: 1 = large launches of the tiled kernel (one voxel per lane, 32 channels per
 * pass, all output channels in one workgroup, at least eight tiles per compute unit) run as
 * persistent workgroups, four per compute unit, each walking a run of consecutive tiles with the
 * next halo tile loaded under the current tile's arithmetic; 0 (default) = one workgroup per tile.
 * Measured 5-18 % slower than the default on every shape tried, kept as an option for comparison.
 * Results never depend on options.  Returns TERN_EARG for an unknown option or
 * value. */
typedef enum { TERN_OPT_LANE_DEPTH = 1, TERN_OPT_WAVES_Z = 2, TERN_OPT_CO_BLOCK = 3,
               TERN_OPT_CO_PER_WAVE = 4, TERN_OPT_TAP_SPLIT = 5, TERN_OPT_POINTWISE = 6,
               TERN_OPT_LANE_TILE = 7, TERN_OPT_STREAM = 8 } tern_option;
int tern_set_option(int option, int value);

/*
 * tern_last_launch -- diagnostic: the plan of the calling thread's most recent convolution launch
 * (tern_conv3d, tern_conv3d_binary, tern_conv3d_digits, or the last layer of a network call), so
 * that a test can tell which kernel its input reached.  info (host, 8 values): [0] kernel, one of
 * the TERN_KERNEL_ values (-1 before the thread's first launch); for the tiled and persistent
 * kernels [1] output voxels per lane, [2] channels per pass, [3] waves sharing the taps of a slice,
 * [4] threads per workgroup, [5], [6] grid extents, [7] LDS bytes per workgroup; zeros otherwise.
 * TERN_ENULL for a NULL pointer.
 */
typedef enum { TERN_KERNEL_DIRECT = 0, TERN_KERNEL_TILED = 1, TERN_KERNEL_POINTWISE = 2,
               TERN_KERNEL_PERSISTENT = 3 } tern_kernel;
int tern_last_launch(int32_t info[8]);

/*
 * tern_probe_valu -- diagnostic, no counterpart in the paper: runs `iters` rounds of 64 integer
 * vector instructions plus one add per round and lane on blocks x threads lanes with no memory
 * traffic.  Timing it gives the sustained issue rate of those instructions on the device, the
 * measured ceiling for section 2's bit-count argument on this hardware.  variant:
 *    0  the word-pair sequence of the convolution kernels (and, popcount-accumulate, three-input
 *       bit operation, popcount-accumulate, a scalar no-op behind each producer), 16 word pairs;
 *    1  the same four instructions per word pair with no scalar instruction between them;
 *    2, 4, 6, 8, 12   one opcode alone: v_and_b32, v_bcnt_u32_b32, v_bitop3_b32, v_xor_b32,
 *       v_add_u32 (the last for reference);  3, 5, 7, 9, 13  the same with s_nop 0 behind every
 *       vector instruction;
 *   10  the word pair of the binary convolution (three-input bit operation, s_nop 0, popcount-
 *       accumulate), 32 pairs;
 *   11  the same without the no-op;
 *   14, 15  v_xor_b32 / v_bitop3_b32 with vector-register operands only;
 *   16  v_and_b32 with a wave-uniform operand alternating with an independent v_add_u32 on
 *       vector registers.
 * (2, 6, 8, 12 give their opcode one wave-uniform operand, as the convolution's filter words are.)
 * sink: device int32[1] (practically never written).  threads: multiple of 64, at most 512.
 * TERN_EARG for anything else.
 */
#define TERN_PROBE_VARIANTS 17
int tern_probe_valu(int32_t blocks, int32_t threads, int32_t iters, int32_t variant, int32_t* sink,
                    void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TERN_TUNING_H */
