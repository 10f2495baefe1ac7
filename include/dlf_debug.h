/*
 * libdlf testing hooks: process-wide switches that force the planner's choices, so that tests can
 * reach every kernel form and tile shape.  Not part of the serving interface: they are not
 * thread-safe, and a hook left set changes every plan made afterwards in the process -- reset each
 * one (its documented "automatic" value) before planning anything else.
 */
#ifndef DLF_DEBUG_H
#define DLF_DEBUG_H

#include "dlf.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Testing hook: th > 0 forces tile th x tw, register-tile variant, channel slicing, streaming and
 * channels per streaming round (kc: 32, 64 or 128; 0 = 32) for every group planned afterwards
 * (groups it does not fit become infeasible; for a fully connected layer nslices = 1, 2, 4 or 8
 * is the number of K slices); th = 0 restores the automatic choice.
 * Process-wide, not thread-safe. */
void dlf_debug_force_config(int32_t th, int32_t tw, int32_t variant, int32_t nslices,
                            int32_t slice_c, int32_t stream0, int32_t kc);
/* Testing hook, after dlf_debug_force_config (which resets it to 1): the forced tiling also splits K
 * over `ksplit` waves per work item (2, 4 or 8; single resident convolution, 32x64 register tile). */
void dlf_debug_force_ksplit(int32_t ksplit);

/* Testing hook: how single 1x1 convolutions choose between the fused-group kernel and the
 * pointwise kernel: 0 = by modelled cost (default), 1 = pointwise wherever it applies, 2 = never,
 * 3 / 4 / 5 = pointwise wherever it applies with 64x64 / 32x32 / split-K 64x64 work items,
 * 6 / 7 = with workgroup blocks of 128 channels x 128 pixels / 64 channels x 256 pixels whose
 * operands are shared through LDS, 8 = on the kernel for maps of many channels and few pixels (cin 256,
 * 512 or 1024, stride 1, no residual) wherever that applies.  Process-wide, not thread-safe. */
void dlf_debug_pointwise_mode(int32_t mode);

/* Testing hook: how a single depthwise 3x3 layer (pad 1, stride 1 or 2), or such a layer with the 1x1
 * convolution behind it, chooses between the fused-group kernel and the streaming depthwise kernel /
 * the depthwise + 1x1 kernels: 0 = by modelled cost (default), 1 = the depthwise kernels wherever
 * they apply (a pair: the tile kernel where its shape restrictions allow, else the register kernel),
 * 2 = never, 3 = as 1 but a pair always on the register kernel, 4 = a pair on the kernel for maps of many
 * channels and few pixels wherever that applies (channels a multiple of 256).  In mode 1 - 3 that kernel is
 * not considered.  Process-wide, not thread-safe. */
void dlf_debug_depthwise_mode(int32_t mode);
/* Testing hook: wx > 0 fixes the tile of the depthwise + 1x1 tile kernel for groups planned afterwards:
 * wx (1, 2 or 4) of its four waves side by side, each 512 / (2 * channels) pixels wide, rw output rows
 * per wave (a shape that does not fit falls back to the other kernels); wx = 0 restores the automatic
 * choice.  Under depthwise mode 4 the two values fix the other kernel's configuration instead: wx = channel
 * blocks per wave (1 or 2), rw = channels per pass (256 or 512).  Process-wide, not thread-safe. */
void dlf_debug_depthwise_tile(int32_t wx, int32_t rw);

/* Testing hook: how a single 3x3 stride-1 pad-1 convolution (with the 2x2 max pool folded behind
 * it, if any) chooses between the fused-group kernel and the block 3x3 kernel: mode 0 = by
 * modelled cost (default), 1 = the block kernel wherever it applies, 2 = never.  shape >= 0 also
 * fixes the block's shape and its th x tw pixel tile: shape 0 / 1 = 128 channels x up to 256
 * pixels with activations brought in 32 / 64 input channels at a time, 2 / 3 = 64 channels x up to
 * 512 pixels likewise, 4 = 128 channels x up to 512 pixels (32 input channels at a time), 5 = the kernel
 * for maps of many channels and few pixels (cin 256, 512, 1024 or 2048, no pool; th > 0 then
 * fixes the number of waves that share a channel block's K: 1, 2 or 4; tw is not used), 6 = the
 * kernel for a 3x3 layer (128 or 256 channels in and out) with a 1x1 layer behind it as one group
 * (th, tw > 0 then fix the tile the map is cut into equal parts for: at most 8 x 16 pixels), 7 = the
 * kernel for a whole bottleneck block (1x1 to 64 channels, 3x3, 1x1; th, tw as for 6, at most 64
 * pixels); a shape
 * that cannot be laid out falls back to the fused-group kernel.  Mode 2 keeps such a pair of layers
 * on the fused-group kernel as well.
 * Process-wide, not thread-safe. */
void dlf_debug_block3x3_mode(int32_t mode, int32_t shape, int32_t th, int32_t tw);

#ifdef __cplusplus
}
#endif
#endif /* DLF_DEBUG_H */
