// Shared between the host planner and the gfx950 kernels: the "group program" one workgroup
// interprets.  A fusion group (Sec. III-B of the paper: consecutive layers executed as one block
// with on-chip intermediates) is a short list of stages; each stage reads a region of its input
// feature map from LDS (stage 0 may stream its input from HBM instead) and writes its output
// region to LDS, or to HBM if it is the last stage.
#pragma once
#include <stdint.h>

#define DLF_MAX_STAGES 8
#define DLF_WG_THREADS 512
#define DLF_WAVES 8          // waves per workgroup
#define DLF_MMA_WAVES 4      // streaming CONV stage: waves 0..3 multiply, the others move data
#define DLF_LOAD_THREADS ((DLF_WAVES - DLF_MMA_WAVES) * 64)
#define DLF_CPAD 8          // halfs of padding per LDS pixel row: makes the row stride an odd
                            // multiple of 16 bytes, so 16-byte LDS accesses spread over all banks
#define DLF_STAGE_VECS 8    // 16-byte vectors a data-movement thread holds per streaming round

enum { DLF_ST_CONV = 0, DLF_ST_MAXPOOL = 1, DLF_ST_DW = 2 };

struct DlfStage {
    int32_t kind;
    int32_t cin;          // true input channels
    int32_t cin_pad;      // input channels padded to a multiple of 32 (zero weights beyond cin)
    int32_t kc;           // CONV streaming: channels brought in per round (32, 64 or 128)
    int32_t kc_shift;     // log2(kc / 8) = log2 of the 16-byte vectors per pixel per round
    int32_t cout;         // true output channels
    int32_t ncb;          // CONV: number of 32-wide output-channel blocks = ceil(cout/32)
    int32_t kh, kw, stride, pad, act;
    int32_t pool2;        // CONV: fused 2x2 stride-2 max pooling in the epilogue
    int32_t in_h, in_w;   // true size of the input feature map
    int32_t out_h, out_w; // true size of the output feature map (before the fused pool)
    int32_t rh, rw;       // output region this stage computes per tile (before the fused pool)
    int32_t ih, iw;       // input region = (rh-1)*stride+kh by (rw-1)*stride+kw
    int32_t oy_mul, oy_off, ox_mul, ox_off; // output region origin = tile origin * mul + off
    int32_t in_cs;        // halfs per pixel of the input LDS buffer
    int32_t out_cs;       // halfs per pixel of the output LDS buffer (if not last)
    int32_t in_off;       // LDS offset (halfs) of the input buffer (stream: first of two buffers)
    int32_t out_off;      // LDS offset (halfs) of the output buffer
    int32_t stream_buf;   // stream mode: halfs per chunk buffer
    int32_t nsteps;       // CONV: 16-wide K steps per output-channel block
    int32_t alias_out;    // last CONV stage: the output tile overwrites the stage's input in LDS; a
                          // barrier separates the last MFMA from the epilogue
    int32_t im2col;       // CONV stage 0 on a narrow input (cin % 8 != 0).  1: the staging gathers each
                          // output pixel's kh*kw*cin inputs into one LDS row and the stage then
                          // runs as a 1x1 convolution over cin_pad = roundup(kh*kw*cin, 32) channels.
                          // 2 (cin <= 4, even stride): the input patch is staged as 4-channel pixels
                          // and the stage runs with one tap per filter row over
                          // cin_pad = roundup(4*kw, 32) channels, in_cs = 4, kw = 1
    int32_t im_kh, im_kw, im_stride, im_pad, im_cin; // the real filter geometry of an im2col stage
    const void* w;        // CONV: packed fragments; DW: [kh][kw][c] fp16
    const float* bias;    // padded with zeros to ncb*32 (CONV) / c rounded up to 8 (DW)
    const void* res;      // residual operand in HBM, NHWC with this stage's output shape, or null
    int32_t ksplit;       // resident CONV stage: K (the 32-channel chunks) split over this many waves per
                          // work item (1, 2, 4 or 8; work items x ksplit <= 8); the partial sums meet in
    int32_t ks_off;       // an LDS area at this offset (halfs): [wave][FC * FP * 16][64] fp32
};

struct DlfGroupArgs {
    const void* in;       // group input tensor (HBM)
    void* out;            // group output tensor (HBM)
    int32_t nstages;
    int32_t stream0;      // stage 0 is a CONV that streams its input in K-chunks
    int32_t batch;
    int32_t in_h, in_w, in_c;         // group input tensor shape
    int32_t iy_mul, iy_off, ix_mul, ix_off; // group input region origin = tile origin*mul + off
    int32_t th, tw;       // tile of the last stage's output region (before its fused pool)
    int32_t tiles_y, tiles_x;
    int32_t nslices;      // channel slices (grid over output channels / channels)
    int32_t slice_c;      // channels per slice (multiple of 32 for CONV, of 8 otherwise)
    int32_t ntiles;       // batch * tiles_y * tiles_x * nslices
    int32_t out_h, out_w, out_c;      // group output tensor shape
    DlfStage st[DLF_MAX_STAGES];
};

struct DlfFcArgs {
    const void* x;        // [batch][k] fp16
    void* y;              // [batch][cout] fp16
    const void* w;        // packed fragments
    const float* bias;
    int32_t batch, k, cout, ncb, nsteps, act;
    int32_t ksplit;       // > 1: K is split over ksplit workgroups per pair of channel blocks ...
    float* part;          // ... which leave fp32 partial sums here: [batch block][ksplit][ncb][16][64]
};

// Pointwise (1x1, pad 0) convolution run without tiles or barriers: every wave owns work items
// of 64 x 64 (shape 0) or 32 x 32 (shape 1) output pixels x output channels (shape 2: a 64 x 64
// item shared by the four waves of a workgroup, each running a quarter of K), reads its activations
// straight from HBM in the MFMA operand layout and writes its result through a wave-private LDS
// transpose buffer.
#define DLF_PW_WAVES 4               // waves per workgroup
#define DLF_PWSK_PART_BYTES (4 * 3 * 16 * 64 * 4)   // split-K form (shape 2): partial sums in LDS
// block form of the pointwise kernel: K steps per LDS stage, stages in the ring; LDS = the ring
// (1 KiB per fragment) or the four waves' transpose buffers, whichever is larger
#ifndef DLF_PWB_KS
#define DLF_PWB_KS 2
#endif
#ifndef DLF_PWB_STAGES
#define DLF_PWB_STAGES 4
#endif
#define DLF_PWB_LDS_BYTES(WN, WM)                                                                   \
    ((DLF_PWB_STAGES * (2 * (WN) + 2 * (WM)) * DLF_PWB_KS * 1024) > (DLF_PW_WAVES * 64 * 72 * 2)      \
         ? (DLF_PWB_STAGES * (2 * (WN) + 2 * (WM)) * DLF_PWB_KS * 1024)                              \
         : (DLF_PW_WAVES * 64 * 72 * 2))
struct DlfPwArgs {
    const void* in;       // [batch][in_h][in_w][cin] fp16
    void* out;            // [batch][out_h][out_w][cout] fp16
    const void* w;        // packed fragments (same stream as a CONV stage)
    const float* bias;    // padded to ncb*32
    const void* res;      // residual operand, output shape, or null
    int32_t m;            // output pixels = batch * out_h * out_w
    int32_t cin, cout, ncb, nsteps, act;
    int32_t stride, in_h, in_w, out_h, out_w;
    int32_t n_pg, n_cg;   // groups of 64 (32) pixels, groups of 64 (32) output channels
    int32_t nitems;       // n_pg * n_cg
    // Second operand pair (block forms only; nsteps2 = 0: none): a second 1x1 convolution with the
    // same output shape whose result is added before the activation -- the projection shortcut of a
    // residual block run as further K steps of the same accumulators, out = act(w . in + bias +
    // w2 . in2 + bias2), instead of a tensor written to memory and read back as a residual.
    const void* in2;      // [batch][in_h2][in_w2][cin2] fp16
    const void* w2;       // packed fragments
    const float* bias2;   // padded to ncb*32
    int32_t cin2, nsteps2, stride2, in_h2, in_w2;
    // quantised form only (int8 tensors, `cin` = byte pairs per pixel, `act` != 0 = ReLU):
    const float* scale;   // requantisation scale per output channel, padded to ncb*32
};

// 3x3 stride-1 pad-1 convolution as a block kernel (one layer, optionally with the 2x2 max pool
// that follows it): a workgroup of eight waves computes 64 * WC output channels x 64 * (8 / WC)
// pixels of a th x tw tile, K streamed through LDS: the weights of all nine taps for the block's
// channels 16 input channels at a time (a ring of stages), the tile's halo region ACH input
// channels at a time (two buffers).  A wave's part is 64 channels x 32 * FP pixels.
// Shapes (WC, ACH, FP): 0 = (2, 32, 2), 1 = (2, 64, 2), 2 = (1, 32, 2), 3 = (1, 64, 2), 4 = (2, 32, 4).
#define DLF_C3_WAVES 8
#define DLF_C3_SHAPES 5
#define DLF_C3_LOAD_WAVES 4          // waves 0 .. 3 request the operands of all eight
#define DLF_C3_MAX_ACT_LOADS 16      // activation loads per requesting wave per block the kernel is built for
#define DLF_C3_EPI_BYTES (DLF_C3_WAVES * 64 * 72 * 2)   // transpose buffers of the epilogue
struct DlfC3Args {
    const void* in;       // [batch][h][w][cin] fp16
    void* out;            // [batch][h][w][cout] fp16 ([batch][h/2][w/2][cout] with pool2)
    const void* w;        // packed fragments (same stream as a CONV stage), zero steps behind them
    const float* bias;    // padded to ncb*32
    const void* res;      // residual operand, output shape, or null
    int32_t batch, h, w_, cin, cout, ncb, nsteps, act, pool2;
    int32_t th, tw, tiles_y, tiles_x;
    int32_t n_cg;         // groups of 64 * WC output channels
    int32_t ntiles;       // batch * tiles_y * tiles_x
    int32_t nitems;       // n_cg * ntiles (channel group slowest)
    int32_t npxh;         // (th + 2) * (tw + 2): pixels of the halo region
    int32_t na_i;         // ceil(npxh / (512 / ACH)): activation load instructions per block (1 KiB each)
    int32_t lpw_a;        // ceil(na_i / DLF_C3_LOAD_WAVES): ... per requesting wave
    int32_t nst;          // stages in the weight ring (2 .. 4)
    // quantised form only (int8 tensors, `cin` = byte pairs per pixel, `act` != 0 = ReLU):
    const float* scale;   // requantisation scale per output channel, padded to ncb*32
};

// Depthwise 3x3 convolution (pad 1, stride 1 or 2) as a streaming kernel without LDS or barriers:
// a wave owns 64 consecutive 16-byte vectors (8 channels each) of the output rows of a strip and
// walks down the strip with a sliding window of input rows in registers.
#define DLF_DW_WAVES 4               // waves per workgroup
#define DLF_DW_ROWS1 14              // output rows per strip, stride 1
#define DLF_DW_ROWS2 7               // output rows per strip, stride 2
struct DlfDwArgs {
    const void* in;       // [batch][h][w][c] fp16
    void* out;            // [batch][oh][ow][c] fp16
    const void* w;        // [9][cpad] fp16 (tap-major)
    const float* bias;    // [cpad]
    uint32_t in_bytes, res_bytes;    // size of the input tensor (below 2 GiB)
    int32_t batch, h, w_, c, cpad, oh, ow, stride, act;
    int32_t cg;           // c / 8: 16-byte vectors per pixel
    int32_t rowv;         // ow * cg: vectors per output row
    int32_t nxr;          // ceil(rowv / 64): runs of 64 vectors per output row
    int32_t nstrips;      // ceil(oh / rows per strip)
    int32_t nitems;       // batch * nstrips * nxr
};

// Depthwise 3x3 (pad 1, stride 1 or 2) followed by a 1x1 convolution, fused without a tile pipeline:
// a wave owns work items of 32 output pixels x 32 * NB output channels; per 16-channel K step every
// lane computes the depthwise result of its pixel and 8 channels in registers -- which is the MFMA
// "B" operand as it stands -- and the wave multiplies it with NB packed weight fragments.
#define DLF_DWPW_WAVES 4
#define DLF_DWPW_LDS_BYTES(C, NB) (22 * (C) + DLF_DWPW_WAVES * 32 * (32 * (NB) + 8) * 2)
struct DlfDwPwArgs {
    const void* in;       // [batch][h][w][c] fp16
    void* out;            // [batch][oh][ow][cout] fp16
    const void* wdw;      // depthwise weights [9][c] fp16 (tap-major)
    const float* bdw;     // depthwise bias [c]
    const void* wpw;      // pointwise weights, packed fragments
    const float* bpw;     // pointwise bias, padded to ncb * 32
    uint32_t in_bytes;    // size of the input tensor (below 2 GiB)
    int32_t batch, h, w_, c, oh, ow, stride, act_dw, act_pw;
    int32_t cout, ncb, nsteps;
    int32_t m;            // output pixels = batch * oh * ow
    int32_t n_pg, n_cg;   // groups of 32 pixels, groups of 32 * NB output channels
    int32_t nitems;       // n_pg * n_cg (channel group fastest)
};

// Depthwise 3x3 + 1x1 as a tile kernel: a workgroup of four waves owns a th x tw tile of output
// pixels.  Phase 1: the waves (wx x wy of them, each pxw = 512 / (2 c) pixels wide and rw rows high)
// compute the depthwise layer as k_dw does -- coalesced loads, window of input rows in registers --
// and leave its result in LDS as [pixel][c + 8].  Phase 2: the 1x1 layer on MFMA, its "B" fragments
// read from that LDS tile, work units of one 32-channel block x up to four 32-pixel blocks dealt
// to the waves; results leave through wave-private transpose buffers.
#define DLF_DWT_WAVES 4
#define DLF_DWT_EPI_HALFS (32 * (32 + 8))            // transpose buffer of a wave: 32 pixels x 32 channels
#define DLF_DWT_LDS_BYTES(TP, C) (((TP) * ((C) + 8) + DLF_DWT_WAVES * DLF_DWT_EPI_HALFS) * 2)
struct DlfDwtArgs {
    const void* in;       // [batch][h][w][c] fp16
    void* out;            // [batch][oh][ow][cout] fp16
    const void* wdw;      // depthwise weights [9][c] fp16 (tap-major)
    const float* bdw;     // depthwise bias [c]
    const void* wpw;      // pointwise weights, packed fragments
    const float* bpw;     // pointwise bias, padded to ncb * 32
    uint32_t in_bytes;    // size of the input tensor (below 2 GiB)
    int32_t batch, h, w_, c, oh, ow, stride, act_dw, act_pw;
    int32_t cout, ncb, nsteps;
    int32_t cg;           // c / 8 (a power of two, 4 .. 64)
    int32_t pxw;          // 64 / cg: pixels of a row a wave covers
    int32_t wx, wy, rw;   // waves along x and y (wx * wy = 4), rows per wave
    int32_t th, tw;       // tile: wy * rw rows x wx * pxw pixels
    int32_t tp;           // th * tw tile pixels (at most 256)
    int32_t npb;          // ceil(tp / 32) pixel blocks
    int32_t npg;          // ceil(npb / 4) groups of up to four pixel blocks
    int32_t tiles_y, tiles_x, ntiles;     // ntiles = batch * tiles_y * tiles_x
};

// Depthwise 3x3 + 1x1 convolution for maps of many channels and few pixels (channels a multiple of
// 256), where the tile kernel above has no tile to work with: one workgroup of eight waves per work
// item = (tile of at most 8 x 8 output pixels, slice of 8 * cbw 32-channel blocks of the 1x1 layer).
// Per pass over kh of the c channels: the tile's input region arrives in LDS by direct loads, the waves compute the depthwise layer from there
// into an LDS tile [pixel][kh + 8], then multiply it on MFMA, every wave cbw channel blocks x two
// 32-pixel blocks with its weight fragments streaming through a register ring.
#define DLF_DWS_WAVES 8
// a region: whole KiB of pixels, kh channels each
#define DLF_DWS_IN_BYTES(RP, KH) ((((RP) * (KH) * 2 + 1023) / 1024) * 1024)
#define DLF_DWS_EPI_BYTES(CBW) (DLF_DWS_WAVES * 32 * (32 * (CBW) + 8) * 2)
#define DLF_DWS_MID_BYTES(TP, KH) ((TP) * ((KH) + 8) * 2)
#define DLF_DWS_LDS_BYTES(RP, TP, KH, CBW, NBUF)                                                 \
    (((NBUF) * DLF_DWS_IN_BYTES(RP, KH) > DLF_DWS_EPI_BYTES(CBW) ? (NBUF) * DLF_DWS_IN_BYTES(RP, KH) \
                                                               : DLF_DWS_EPI_BYTES(CBW)) +         \
     DLF_DWS_MID_BYTES(TP, KH))
struct DlfDwsArgs {
    const void* in;       // [batch][h][w][c] fp16
    void* out;            // [batch][oh][ow][cout] fp16
    const void* wdw;      // depthwise weights [9][c] fp16 (tap-major)
    const float* bdw;     // depthwise bias [c]
    const void* wpw;      // pointwise weights, packed fragments
    const float* bpw;     // pointwise bias, padded to ncb * 32
    uint32_t in_bytes;    // size of the input tensor (below 2 GiB)
    int32_t batch, h, w_, c, oh, ow, stride, act_dw, act_pw;
    int32_t cout, ncb, nsteps;
    int32_t kh, nkh;      // channels per pass (256 or 512), passes = c / kh
    int32_t nbuf;         // region buffers in LDS: nkh (every pass's region is requested at the start) or 1
    int32_t th, tw, tp;   // tile of output pixels (each side <= 8), tp = th * tw
    int32_t rh, rw, rp;   // its input region: (th - 1) * stride + 3 rows, likewise columns; rp = rh * rw
    int32_t tiles_y, tiles_x, ntiles;     // ntiles = batch * tiles_y * tiles_x
    int32_t cbw;          // channel blocks per wave (1 or 2)
    int32_t nsl;          // slices of the output channels: ceil(ncb / (8 * cbw))
};

// 3x3 convolution, pad 1, stride 1 or 2 (or 1x1, stride 1) on maps of many channels and few pixels (cin 256 .. 2048),
// where the block kernel has too few blocks for the chip and the fused-group kernel's waves each
// stream their own weights: one workgroup of eight waves per work item = (tile of at most 8 x 8 output
// pixels, slice of 8 / ksplit 32-channel blocks); the tile's input region, all cin channels, goes to LDS
// by direct loads; ksplit waves share a channel block's K (whole 32-channel chunks each) and their
// partial sums meet in LDS.
#define DLF_C3S_WAVES 8
#define DLF_C3S_IN_BYTES(RP, CIN) ((((RP) * (CIN) * 2 + 1023) / 1024) * 1024)
#define DLF_C3S_RED_BYTES (6 * 2 * 16 * 64 * 4)      // up to six waves' accumulators (2 pixel blocks x 16 registers x 64 lanes)
#define DLF_C3S_EPI_BYTES (DLF_C3S_WAVES * 32 * (32 + 8) * 2)
#define DLF_C3S_LDS_BYTES(RP, CIN)                                                      \
    (DLF_C3S_IN_BYTES(RP, CIN) > DLF_C3S_RED_BYTES + DLF_C3S_EPI_BYTES ? DLF_C3S_IN_BYTES(RP, CIN) \
                                                                     : DLF_C3S_RED_BYTES + DLF_C3S_EPI_BYTES)
struct DlfC3sArgs {
    const void* in;       // [batch][h][w][cin] fp16
    void* out;            // [batch][oh][ow][cout] fp16
    const void* res;      // residual operand [batch][oh][ow][cout] fp16, or null
    const void* w;        // packed weight fragments, K step = (32-channel chunk, tap, half)
    const float* bias;    // padded to ncb * 32
    uint32_t in_bytes;    // size of the input tensor (below 2 GiB)
    int32_t batch, h, w_, oh, ow, cin, cout, ncb, nsteps, act;
    int32_t taps;         // 9: 3x3, pad 1; 1: 1x1
    int32_t stride;       // 1, or 2 (3x3 only)
    int32_t th, tw, tp;   // tile of output pixels (each side <= 8), tp = th * tw
    int32_t rw, rp;       // its input region: (tw - 1) * stride + 3 columns (1x1: tw), rows likewise, rp pixels
    int32_t tiles_y, tiles_x, ntiles;     // ntiles = batch * tiles_y * tiles_x
    int32_t ksplit;       // 1, 2 or 4 waves per channel block; divides cin / 32 (1x1: cin / 128)
    int32_t nsl;          // slices of the output channels: ceil(ncb / (8 / ksplit))
    int32_t slice_major;  // 1: an XCD keeps to one slice (nsl 2, 4 or 8); 0: the slices of a tile share an XCD
    // quantised form (int8 tensors, `cin` = byte pairs per pixel, `act` != 0 = ReLU) if not null:
    const float* scale;   // requantisation scale per output channel, padded to ncb * 32
    int32_t pool2;        // quantised 3x3 form: the 2x2 max pool behind the layer folded in (tw = 8, th even;
                          // oh, ow, th, tw count convolution pixels, the output map is [oh / 2][ow / 2])
};

// 3x3 convolution (stride 1, pad 1, cin = cout = c: 64, 128 or 256) and the 1x1 convolution behind it, with
// a residual operand added to the second layer's result: the second half of a bottleneck block, where
// the batch's tiles are no more than the chip's CUs (ResNet-50's 28 x 28 stage at batch 32).  One
// workgroup of eight waves per work item = (tile of up to 128 output pixels, slice of 16 channel
// blocks of the second layer); the input region goes to LDS by direct loads, the first layer's
// result stays in LDS as [pixel][c + 8].
#define DLF_C3PW_WAVES(C) ((C) == 64 ? 4 : 8)             /* 64 channels: four waves, two workgroups per CU */
#define DLF_C3PW_IN_BYTES(RP, C) ((((RP) * (C) * 2 + 1023) / 1024) * 1024)
#define DLF_C3PW_EPI_BYTES(C) (DLF_C3PW_WAVES(C) * 32 * (32 + 8) * 2)
#define DLF_C3PW_MID_BYTES(TP, C) ((TP) * ((C) + 8) * 2)
#define DLF_C3PW_RES_STRIDE(C) (DLF_C3PW_WAVES(C) * 128 + 64)   /* a pixel's residual row: the item's channels + 64 bytes */
// the first layer's result takes the region's place; behind it the waves' transpose buffers, then
// (past the region's end) the residual operand
#define DLF_C3PW_TB_OFF(TP, C) (((DLF_C3PW_MID_BYTES(TP, C) + 63) / 64) * 64)
#define DLF_C3PW_RES_OFF(RP, TP, C)                                                                        \
    (DLF_C3PW_IN_BYTES(RP, C) > DLF_C3PW_TB_OFF(TP, C) + DLF_C3PW_EPI_BYTES(C) ? DLF_C3PW_IN_BYTES(RP, C) \
                                                                                : DLF_C3PW_TB_OFF(TP, C) + DLF_C3PW_EPI_BYTES(C))
#define DLF_C3PW_BIAS_OFF(RP, TP, C, RES) (DLF_C3PW_RES_OFF(RP, TP, C) + ((RES) ? (TP) * DLF_C3PW_RES_STRIDE(C) : 0))
#define DLF_C3PW_LDS_BYTES(RP, TP, C, RES) (DLF_C3PW_BIAS_OFF(RP, TP, C, RES) + DLF_C3PW_WAVES(C) * 64 * 4)
struct DlfC3PwArgs {
    const void* in;       // [batch][h][w][c] fp16
    const void* res;      // residual operand [batch][h][w][cout] fp16, or null
    void* out;            // [batch][h][w][cout] fp16
    const void* w1;       // 3x3 weights, packed fragments (K step = 32-channel chunk, tap, half)
    const float* b1;      // padded to c
    const void* w2;       // 1x1 weights, packed fragments
    const float* b2;      // padded to ncb2 * 32
    uint32_t in_bytes;    // size of the input tensor (below 2 GiB)
    uint32_t res_bytes;   // size of the residual operand = of the output (below 2 GiB)
    int32_t batch, h, w_, c, cout, ncb2, act1, act2;
    int32_t th, tw, tp;   // tile of output pixels: th <= 8, tw <= 16, tp = th * tw <= 128
    int32_t rw, rp;       // its input region: tw + 2 columns, (th + 2) * (tw + 2) pixels
    int32_t tiles_y, tiles_x, ntiles;     // ntiles = batch * tiles_y * tiles_x
    int32_t nsl;          // slices of the second layer's channels: ceil(ncb2 / (2 * waves))
};

// A whole bottleneck block as one group: 1x1 (cin0 -> 64), 3x3 (64 -> 64, stride 1, pad 1), 1x1 (64 ->
// cout), the block's input added to the last layer's result where the block has an identity
// shortcut (then cout = cin0).  One workgroup of four waves per work item = (tile of up to 64 output
// pixels, slice of 8 channel blocks of the last layer), two workgroups to a CU.  LDS: the input
// region with all cin0 channels, the first layer's result on the region, the second layer's on the
// tile, the waves' transpose buffers, the last layer's bias.
#define DLF_BN_WAVES 4
#define DLF_BN_IN_BYTES(RP, CIN0) ((((RP) * (CIN0) * 2 + 1023) / 1024) * 1024)
#define DLF_BN_MA_BYTES(RP) ((((RP) * 128 + 1023) / 1024) * 1024)
#define DLF_BN_MB_BYTES(TP) ((((TP) * (64 + 8) * 2 + 63) / 64) * 64)
#define DLF_BN_EPI_BYTES (DLF_BN_WAVES * 32 * (32 + 8) * 2)
#define DLF_BN_MA_OFF(RP, CIN0) DLF_BN_IN_BYTES(RP, CIN0)
#define DLF_BN_MB_OFF(RP, CIN0) (DLF_BN_MA_OFF(RP, CIN0) + DLF_BN_MA_BYTES(RP))
#define DLF_BN_TB_OFF(RP, TP, CIN0) (DLF_BN_MB_OFF(RP, CIN0) + DLF_BN_MB_BYTES(TP))
#define DLF_BN_BIAS_OFF(RP, TP, CIN0) (DLF_BN_TB_OFF(RP, TP, CIN0) + DLF_BN_EPI_BYTES)
#define DLF_BN_LDS_BYTES(RP, TP, CIN0) (DLF_BN_BIAS_OFF(RP, TP, CIN0) + DLF_BN_WAVES * 64 * 4)
struct DlfBnArgs {
    const void* in;       // [batch][h][w][cin0] fp16: the block's input (and its residual operand)
    void* out;            // [batch][h][w][cout] fp16
    const void* w0;       // 1x1 weights cin0 -> 64, packed fragments
    const float* b0;
    const void* w1;       // 3x3 weights 64 -> 64, packed fragments (K step = 32-channel chunk, tap, half)
    const float* b1;
    const void* w2;       // 1x1 weights 64 -> cout, packed fragments
    const float* b2;      // padded to ncb2 * 32
    uint32_t in_bytes;    // size of the input tensor (below 2 GiB)
    int32_t batch, h, w_, cin0, cout, ncb2, act0, act1, act2;
    int32_t identity;     // 1: the input is added to the last layer's result (cout == cin0)
    int32_t th, tw, tp;   // tile of output pixels: th <= 8, tw <= 16, tp = th * tw <= 64
    int32_t rw, rp;       // its input region: tw + 2 columns, (th + 2) * (tw + 2) pixels
    int32_t tiles_y, tiles_x, ntiles;     // ntiles = batch * tiles_y * tiles_x
    int32_t nsl;          // slices of the last layer's channels: ceil(ncb2 / 8)
};

struct DlfGapArgs {
    const void* x;        // [batch][hw][c]
    void* y;              // [batch][c]
    int32_t batch, hw, c;
};

#ifdef __cplusplus
extern "C" {
#endif
// Launchers (defined with the kernels).  `variant` selects the per-wave register tile of CONV
// stages: 0 = 64 channels x 64 pixels, 1 = 32 x 128, 2 = 32 x 64, 3 = 32 x 64 compiled for 128
// registers so that two workgroups share a CU.
#define DLF_NUM_VARIANTS 4
int dlf_launch_group(const DlfGroupArgs* a, int variant, int grid, int lds_bytes, void* stream);
int dlf_launch_fc(const DlfFcArgs* a, void* stream);
int dlf_launch_gap(const DlfGapArgs* a, void* stream);
int dlf_launch_pw(const DlfPwArgs* a, int shape, int grid, void* stream);
int dlf_launch_c3(const DlfC3Args* a, int shape, int grid, int lds_bytes, void* stream);
int dlf_launch_pw_i8(const DlfPwArgs* a, int shape, int grid, void* stream);
int dlf_launch_c3_i8(const DlfC3Args* a, int shape, int grid, int lds_bytes, void* stream);
int dlf_launch_dw(const DlfDwArgs* a, int grid, void* stream);
int dlf_launch_dwpw(const DlfDwPwArgs* a, int nb, int grid, void* stream);
int dlf_launch_dwt(const DlfDwtArgs* a, int grid, int lds_bytes, void* stream);
int dlf_launch_dws(const DlfDwsArgs* a, int grid, int lds_bytes, void* stream);
int dlf_launch_c3s(const DlfC3sArgs* a, int grid, int lds_bytes, void* stream);
int dlf_launch_c3pw(const DlfC3PwArgs* a, int grid, int lds_bytes, void* stream);
int dlf_launch_bneck(const DlfBnArgs* a, int grid, int lds_bytes, void* stream);
int dlf_kernels_init(void);
// Attaches a start / stop event pair (hipEvent_t, either may be null) to this thread's next launch.
void dlf_next_launch_events(void* start, void* stop);
#ifdef __cplusplus
}
#endif
