/*
 * libdlf — fused-layer CNN inference on one MI355X (gfx950).
 *
 * A network is given as a linear layer list; dlf_plan() partitions it into contiguous fusion
 * groups and gives each group a budget of compute units (CUs); dlf_run() executes the plan with
 * one kernel launch per group, intermediate feature maps of a group staying on-chip (LDS).
 *
 * This is the execution model the paper tunes (Sec. II-A.2: the two knobs "number of cores" and
 * "layer fusion"; Sec. III-B: a fused block keeps intermediates on chip and pays for it with
 * halo recomputation; Algorithm 1: inputs = layer list, number of layers, OpCount_critical,
 * outputs = fusion_partition_index[], mp_of_fusionblock[]).  Here a "core" is a compute unit:
 * a group with budget b is launched as min(tiles, b * occupancy) persistent workgroups, where
 * occupancy (1 or 2 workgroups per CU) follows from the kernel variant's registers and LDS.
 *
 * Conventions
 *   - Every call returns a dlf_status; out-parameters are written only on DLF_OK.  Nothing
 *     throws or aborts across this boundary.  dlf_last_error() gives a thread-local message.
 *   - Activations are NHWC fp16, [batch][H][W][C], in DEVICE memory owned by the caller.
 *   - Weights/biases passed to dlf_net_create are HOST pointers, borrowed only for the duration
 *     of the call (the library repacks them into its own device buffers).
 *   - dlf_run is asynchronous on the given HIP stream and never synchronises or allocates.
 */
#ifndef DLF_H
#define DLF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DLF_OK = 0,
    DLF_ERR_INVALID_ARG = 1,  /* null pointer, negative size, bad enum value                  */
    DLF_ERR_SHAPE = 2,        /* layer list does not shape-check                               */
    DLF_ERR_UNSUPPORTED = 3,  /* valid network, but no kernel implements this layer            */
    DLF_ERR_INFEASIBLE = 4,   /* a requested fusion group does not fit on-chip memory          */
    DLF_ERR_OOM = 5,          /* host or device allocation failed, or workspace too small      */
    DLF_ERR_HIP = 6,          /* a HIP runtime call failed (see dlf_last_error)                */
    DLF_ERR_NO_WEIGHTS = 7    /* dlf_run on a shape-only network                               */
} dlf_status;

typedef enum { DLF_CONV = 0, DLF_DWCONV = 1, DLF_FC = 2, DLF_MAXPOOL = 3, DLF_GLOBAL_AVGPOOL = 4 } dlf_op;
typedef enum { DLF_ACT_NONE = 0, DLF_ACT_RELU = 1, DLF_ACT_RELU6 = 2 } dlf_act;

/* One layer.  Convolution is cross-correlation with zero padding; the operation count of a
 * layer is Eq. 1 (convolution: 2*Hout*Wout*Hk*Wk*Cin*Cout) or Eq. 2 (FC: 2*M*K*N, M = batch). */
typedef struct {
    int32_t op;            /* dlf_op                                                            */
    int32_t cin, cout;     /* channels (pooling: cin == cout; depthwise: cin == cout)           */
    int32_t kh, kw;        /* kernel size (FC, global avgpool: 1)                               */
    int32_t stride, pad;   /* spatial stride; symmetric padding (0 for conv, -inf for maxpool)  */
    int32_t has_bias;      /* 1: add bias[cout] (a folded batch-norm shift)                     */
    int32_t act;           /* dlf_act; applied after the residual add if there is one           */
    int32_t input_from;    /* -1: previous layer (net input for layer 0); else a layer index    */
    int32_t residual_from; /* -1: none; else index of the layer whose output is added: the layer's  */
                           /* own result (convolution + bias, fp32) is rounded to fp16, the fp16    */
                           /* operand is added and the sum rounded again, then the activation; the  */
                           /* result before the add must therefore lie in the fp16 range            */
    const void* weight;    /* HOST fp16 [cout][kh][kw][cin] (depthwise: [cout][kh][kw][1];      */
                           /* FC: [cout][cin], cin flattened in h,w,c order); NULL => shape-only */
    const float* bias;     /* HOST fp32 [cout], or NULL                                         */
} dlf_layer_desc;

typedef struct dlf_net_s dlf_net_t;
typedef struct dlf_plan_s dlf_plan_t;

/* Tuner modes. */
enum { DLF_TUNER_DP = 0,      /* exact minimum of the additive cost model over all plans        */
       DLF_TUNER_GREEDY = 1,  /* Algorithm 1 (greedy O(n) pass), then split of infeasible blocks */
       DLF_TUNER_MANUAL = 2,  /* caller gives group_last[] and budget[]                          */
       /* The comparison strategies of the paper's evaluation (Sec. V, table of strategies):      */
       DLF_TUNER_LAYERWISE = 3, /* no fusion; each layer's budget from Eq. 5 (strategy 3), or      */
                                /* fixed_budget for all (strategies 1 and 2)                       */
       DLF_TUNER_MAXFUSE = 4    /* longest groups the kernels can run, left to right, on the       */
                                /* largest allowed budget or fixed_budget (strategy 4)             */ };

typedef struct {
    int32_t mode;                     /* DLF_TUNER_*                                             */
    const int32_t* budgets;           /* allowed CU budgets (the MP set); NULL => {32,64,128,256} */
    int32_t n_budgets;
    double opcount_critical;          /* Algorithm 1: operations per core at which a block       */
                                      /* is closed; <= 0 => library default                      */
    double alpha, beta;               /* Eq. 5 weights of log2(C) and log2(OpCount); both 0 =>   */
                                      /* the paper's 0.316 / 0.659                               */
    double mp_scale, mp_offset;       /* Eq. 5 is a proportionality: MP = scale*score + offset;  */
                                      /* both 0 => library default                               */
    const int32_t* manual_group_last; /* DLF_TUNER_MANUAL: index of the last layer of each group */
    const int32_t* manual_budget;     /* DLF_TUNER_MANUAL: budget of each group                  */
    int32_t manual_n;                 /* number of manual groups                                 */
    int32_t max_lds_bytes;            /* on-chip memory one workgroup may use; <= 0 => 160 KiB   */
    int32_t fixed_budget;             /* > 0: every group of a GREEDY / LAYERWISE / MAXFUSE plan  */
                                      /* gets this budget (GREEDY: strategy 5 of the paper)      */
} dlf_tuner_opts;

/* Builds a network from `n` layers on an in_h x in_w x in_c input.  Validates and infers
 * shapes.  If every conv/depthwise/FC layer has a weight pointer, weights are repacked and
 * uploaded to the current HIP device (needs a GPU); if all weight pointers are NULL the result
 * is a shape-only network that can be planned but not run (works without a GPU).
 * Ranges: in_h, in_w, in_c, cin, cout <= 2^20 (FC: cin <= 2^24); kh, kw, stride, pad <= 1024;
 * anything above is DLF_ERR_INVALID_ARG. */
dlf_status dlf_net_create(const dlf_layer_desc* layers, int32_t n, int32_t in_h, int32_t in_w,
                          int32_t in_c, dlf_net_t** out);
void dlf_net_destroy(dlf_net_t* net);
int32_t dlf_net_num_layers(const dlf_net_t* net);
/* Output shape and operation count (Eq. 1 / Eq. 2 at batch 1; 0 for pooling) of layer i. */
dlf_status dlf_net_layer_info(const dlf_net_t* net, int32_t i, int32_t* out_h, int32_t* out_w,
                              int32_t* out_c, uint64_t* op_count);

/* Chooses fusion groups and budgets for `batch` images (Algorithm 1's outputs
 * fusion_partition_index[] and mp_of_fusionblock[]); opts == NULL => DLF_TUNER_DP defaults. */
dlf_status dlf_plan(const dlf_net_t* net, int32_t batch, const dlf_tuner_opts* opts,
                    dlf_plan_t** out);
void dlf_plan_destroy(dlf_plan_t* plan);
int32_t dlf_plan_num_groups(const dlf_plan_t* plan);
/* Group g covers layers [*first, *last] on *budget CUs; tile_h x tile_w output pixels per
 * workgroup step; model_cost in picoseconds of the cost model. Any out pointer may be NULL. */
dlf_status dlf_plan_group(const dlf_plan_t* plan, int32_t g, int32_t* first, int32_t* last,
                          int32_t* budget, int32_t* tile_h, int32_t* tile_w, uint64_t* model_cost);
/* Cost-model value (picoseconds) of running layers [first,last] as one group on `budget` CUs
 * for `batch` images, minimised over the tilings the library can use; DLF_ERR_INFEASIBLE if the
 * layers cannot be executed as one group (the paper times candidates on the device, Sec. V
 * "Oracle Case"; here an integer model stands in, so that dlf_plan can be checked against
 * exhaustive enumeration).  max_lds_bytes <= 0 => 160 KiB.  Works without a GPU. */
dlf_status dlf_group_cost(const dlf_net_t* net, int32_t batch, int32_t first, int32_t last,
                          int32_t budget, int32_t max_lds_bytes, uint64_t* cost);
/* Device bytes needed for the activations that cross group boundaries. */
size_t dlf_plan_workspace_bytes(const dlf_plan_t* plan);
/* Gives the plan its workspace (DEVICE pointer, caller-owned, 256-byte aligned, must outlive the
 * plan's runs).  A plan runs on one stream at a time per workspace. */
dlf_status dlf_plan_bind_workspace(dlf_plan_t* plan, void* dev_ptr, size_t bytes);
/* Runs the whole plan: in_dev [batch][in_h][in_w][in_c] fp16, out_dev = output of the last layer,
 * both DEVICE pointers that must not alias; hip_stream is a hipStream_t (NULL = default stream).
 * Asynchronous; reports launch errors only.  After its first call on a device (which sets kernel
 * attributes once) it allocates nothing and records only kernel launches, so a call may be captured
 * into a HIP graph (tested: replays equal the eager result; on MI355X a replay is no faster than
 * the eager launches, the step being bound on the GPU side). */
dlf_status dlf_run(const dlf_plan_t* plan, const void* in_dev, void* out_dev, void* hip_stream);
/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): dlf_run with the workspace -- the tensors that cross
 * group boundaries and the partial sums of a split-K FC layer -- in a static device array of
 * dlf_static_workspace_bytes() (32 MiB) that the library's code object holds on every GPU it runs
 * on until the process ends; no workspace has to be bound, and a bound one is not used.  in_dev /
 * out_dev as for dlf_run (DEVICE, caller-owned).  Calls no hipMalloc / hipFree and creates no
 * stream or event; every group runs in order on hip_stream (dlf_plan_set_overlap is ignored).
 * DLF_ERR_OOM if dlf_plan_workspace_bytes(plan) exceeds the static size.  All calls on one GPU share
 * that GPU's array, whatever the plan: two calls whose kernels overlap in time on one GPU (different
 * streams or threads) race; calls on one stream are ordered and safe.  Nothing in the array has to
 * start at zero: every byte a kernel reads was written earlier in the same call. */
dlf_status dlf_run_noalloc(const dlf_plan_t* plan, const void* in_dev, void* out_dev, void* hip_stream);
size_t dlf_static_workspace_bytes(void);
/* Branches of the network (the layer graph of a residual network is not a chain): with on != 0 a
 * group that does not read the output of the group in front of it -- the projection shortcut of a
 * residual block, placed behind the block's first layers -- is launched by dlf_run on a second
 * stream of the plan's own (default priority, created at the first such run), beside that group;
 * events order it behind its producers and its consumers behind it, and hip_stream waits for the
 * second stream before dlf_run returns, so the caller sees one stream.  Default off (every group
 * on hip_stream, in order): measured on MI355X the hand-over between the two hardware queues costs
 * more than the overlap gains (ResNet-18 batch 32: 313 -> 366 us per step).
 * dlf_plan_group_stream: the stream group g runs on under the current setting, 0 = the caller's,
 * 1 = the second one, -1 = bad argument.  dlf_run_profiled and dlf_plan_refine always run the
 * groups in order on one stream. */
dlf_status dlf_plan_set_overlap(dlf_plan_t* plan, int32_t on);
int32_t dlf_plan_group_stream(const dlf_plan_t* plan, int32_t g);
/* Profiling variant of dlf_run: runs the plan `reps` times with a HIP stop event attached to every
 * group launch on hip_stream (stamped with the end of that dispatch; a group's duration is taken
 * from the end of the previous dispatch to the end of its own), waits for the stream, and writes
 * the mean duration of each group
 * in milliseconds to group_ms[dlf_plan_num_groups] (HOST array).  Creates and destroys events,
 * synchronises: not for the serving path. */
dlf_status dlf_run_profiled(const dlf_plan_t* plan, const void* in_dev, void* out_dev,
                            void* hip_stream, int32_t reps, float* group_ms);
/* Runs only group g: in_dev = the group's input tensor, out_dev = its output tensor; a residual
 * operand produced outside the group (for a group of kind 8: its second input) is read from
 * res_dev (may be NULL if the group has none). */
dlf_status dlf_run_group(const dlf_plan_t* plan, int32_t g, const void* in_dev, const void* res_dev,
                         void* out_dev, void* hip_stream);
/* Device address inside the bound workspace of the output of layer i, or NULL if that tensor is
 * never materialised (it lives only on-chip) or is the network output. */
const void* dlf_plan_layer_output(const dlf_plan_t* plan, int32_t layer);

/* Kernel configuration chosen for group g: kind (0 fused-group kernel, 1 FC, 2 global avgpool,
 * 3 pointwise-convolution kernels: a single 1x1 layer, 4 block 3x3 kernel: a single 3x3 stride-1
 * pad-1 layer, with its folded 2x2 pool or residual); variant: for kind 0 the register tile
 * (per-wave accumulator tile, output channels x pixels: 0 = 64x64, 1 = 32x128, 2 = 32x64,
 * 3 = 32x64 built for two workgroups per CU), for kind 3 the work-item form (0 = 64x64 and
 * 1 = 32x32 per wave, 2 = 64x64 with K split over four waves, 3 = 128x128 and 4 = 64x256 blocks
 * shared through LDS), for kind 4 the block shape (0 / 1 = 128 channels x 256 pixels, 2 / 3 =
 * 64 x 512, odd: activations 64 input channels at a time, even: 32; 4 = 128 x 512), 5 streaming
 * depthwise kernel: a single depthwise 3x3 layer (variant = stride - 1), 6 fused depthwise 3x3 +
 * 1x1 kernel: a depthwise layer and the pointwise layer behind it, the depthwise result held in
 * registers (variant = 32-channel blocks of a wave's work item, 2 or 4), 7 depthwise + 1x1 tile
 * kernel: the same pair, the depthwise result of a pixel tile held in LDS (variant = stride - 1),
 * 8 two 1x1 convolutions into one output (the projection shortcut of a residual block and the
 * block's last layer, variant = block form as for kind 3; the group reads two tensors, reported by
 * dlf_plan_group_io as input = the last layer's input, residual = the projection's input),
 * 9 depthwise + 1x1 kernel for maps of 256 and more channels and few pixels (variant = 2 * (stride
 * - 1) + channel blocks per wave - 1), 10 small-map kernel: a single 3x3 layer (stride 1 or 2,
 * residual or not) or 1x1 layer on 256 .. 2048 input channels (variant = waves that share a channel
 * block's K: 1, 2 or 4; + 8 for a 1x1 layer), 11 a 3x3 layer of 64, 128 or 256 channels and the 1x1
 * layer behind it (variant = 32-pixel blocks of a tile: 2 or 4), 12 a whole bottleneck block, 1x1 to
 * 64 channels -> 3x3 -> 1x1 with the block's input as residual operand, or its first two layers
 * (variant = the block's input channels; dlf_plan_group_io reports no residual tensor: the kernel
 * takes it from its input);
 * channel slices, channels
 * per slice, whether stage 0 streams its input, LDS bytes per workgroup.  Any out pointer may be
 * NULL. */
dlf_status dlf_plan_group_config(const dlf_plan_t* plan, int32_t g, int32_t* kind, int32_t* variant,
                                 int32_t* nslices, int32_t* slice_c, int32_t* stream0,
                                 int32_t* lds_bytes);
/* Tensors group g reads from HBM: *in_layer = layer whose output is the group input (-1 = the
 * network input); *res_layer = layer whose output is added as a residual (-2 = none). */
dlf_status dlf_plan_group_io(const dlf_plan_t* plan, int32_t g, int32_t* in_layer, int32_t* res_layer);
/* Measured refinement of a plan, after the paper's search procedure that times candidates on the
 * hardware (Sec. V, the reduced brute-force search): for every fused group and every single 1x1 or
 * 3x3 layer, the top_k tilings by modelled cost (and each pointwise form, and the top_k block 3x3
 * shapes, that apply) are run
 * `reps` times on the group's real input (caches scrubbed, the input freshly written by the group
 * in front) and the fastest replaces the planned configuration if it is at least 10 % faster.  The partition into groups and the budgets stay as planned.
 * in_dev / out_dev: DEVICE, as for dlf_run; the workspace must be bound.  Runs the network once,
 * then the candidates, on hip_stream, and waits for them (this call synchronises the stream).
 * *changed (HOST, may be null): number of groups whose configuration changed.  The plan must
 * not be in use by another thread.  dlf_plan_group and dlf_plan_group_config report the new
 * configuration; model_cost is the modelled cost of that configuration.  With the environment
 * variable DLF_DEBUG set, one line per group with the measured times goes to stderr. */
dlf_status dlf_plan_refine(dlf_plan_t* plan, const void* in_dev, void* out_dev, void* hip_stream,
                           int32_t top_k, int32_t reps, int32_t* changed);

/* ---- Quantised (int8) convolution layer ------------------------------------------------------
 * The paper's chip offers an INT8 mode beside FP16 (table of the MLU100's specification); the paper
 * fixes no quantisation scheme.  This is one convolution layer, ksize = 3 (stride 1, zero padding 1)
 * or ksize = 1 (stride 1, no padding), on the int8 matrix instructions, with the usual integer scheme:
 *   acc = sum over taps and input channels of in * w, exact, in 32-bit integers;
 *   out = clamp(round_half_even(fma((float)acc, scale[co], bias[co])), relu ? 0 : -128, 127)
 * with one fp32 fused multiply-add per output ((float) rounds to nearest even above 2^24).  The
 * caller guarantees |acc| < 2^31 (always true for cin <= 14000).
 * pool = 1 (ksize = 3 only) folds the 2x2 stride-2 max pool behind the layer into it -- a fused block of
 * two layers in the sense of Sec. III-B: out[y][x] = max of the four requantised values of its window,
 * the output map is [h/2][w/2] (a last odd row or column is dropped, as by the pooling layer).
 * Tensors: in_dev int8 [batch][h][w][cin], out_dev int8 [batch][h][w][cout], DEVICE, caller-owned,
 * 16-byte aligned, below 2 GiB each.  weight: HOST int8 [cout][ksize][ksize][cin]; scale, bias: HOST fp32
 * [cout]; all three borrowed for the call only (repacked into device buffers the layer owns).  With
 * weight == NULL (then scale and bias are ignored) the layer is shape-only: it can be queried but not
 * run, and needs no GPU.  cin % 64 == 0 and cout % 16 == 0, else DLF_ERR_UNSUPPORTED.
 * budget: compute units the layer may use (<= 0: all 256). */
typedef struct dlf_i8conv_s dlf_i8conv_t;
dlf_status dlf_i8conv_create(int32_t batch, int32_t h, int32_t w, int32_t cin, int32_t cout, int32_t ksize,
                             int32_t relu, int32_t pool, const int8_t* weight, const float* scale, const float* bias, int32_t budget,
                             dlf_i8conv_t** out);
void dlf_i8conv_destroy(dlf_i8conv_t* layer);
/* Tile (th x tw convolution pixels per work item; 1 x pixels for a 1x1 layer on the block kernel), kernel
 * shape index (5: the kernel for maps of many channels and few pixels; else ksize = 3: 0 .. 4, the block
 * kernel's shapes -- output channels x pixels per workgroup 128 x 256, 128 x 256 with 128-byte activation
 * blocks, 64 x 512, 64 x 512 with 128-byte blocks, 128 x 512 --, ksize = 1: 3 = 128 x 128, 4 = 64 x 256),
 * workgroups launched, and the operation count of Eq. 1 for the whole batch.  Any out pointer may be NULL. */
dlf_status dlf_i8conv_info(const dlf_i8conv_t* layer, int32_t* th, int32_t* tw, int32_t* shape, int32_t* grid,
                           uint64_t* op_count);
/* One launch on hip_stream; asynchronous, allocates nothing.  DLF_ERR_NO_WEIGHTS on a shape-only layer. */
dlf_status dlf_i8conv_run(const dlf_i8conv_t* layer, const void* in_dev, void* out_dev, void* hip_stream);

const char* dlf_status_string(dlf_status s);
const char* dlf_last_error(void);
/* Version of the cost-model definition implemented by dlf_group_cost. */
int32_t dlf_cost_model_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DLF_H */
