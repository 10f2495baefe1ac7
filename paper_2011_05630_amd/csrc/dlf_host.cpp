// Host side of libdlf: network object, weight repacking, fusion-group construction, cost model,
// tuner (exact DP, Algorithm-1 greedy, manual) and the launch loop.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <limits>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/dlf.h"
#include "../../include/dlf_debug.h"
#include "dlf_internal.h"

// Workspace of dlf_run_noalloc: a file-scope device array, one copy per GPU the library runs on, held
// until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the device address it returns (per device) is what kernels are given.
#define DLF_STATIC_WS_BYTES ((size_t)32 << 20)
#define DLF_MAX_DEVICES 64
static __device__ __align__(256) unsigned char scratch[DLF_STATIC_WS_BYTES];

namespace {

thread_local std::string g_err;

dlf_status fail(dlf_status s, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return s;
}

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline int round_up(int a, int b) { return ceil_div(a, b) * b; }

struct Layer {
    dlf_layer_desc d;
    int in_h, in_w, in_c;     // input tensor shape
    int out_h, out_w, out_c;  // output tensor shape
    int src;                  // producer of the input (-1 = net input)
    uint64_t macs;            // multiply-accumulates at batch 1
    // packed parameters (device)
    void* d_w = nullptr;
    float* d_bias = nullptr;
    int kc = 0, cin_pad = 0, ncb = 0, nsteps = 0;
    bool im2col = false;     // narrow-input convolution run as a 1x1 over gathered rows
    bool rowfold = false;    // narrow-input convolution (cin <= 4, even stride) whose filter columns are
                             // folded into the channel dimension: input staged as 4-channel pixels,
                             // one tap per filter row over round_up(4 * kw, 32) "channels"
};

}  // namespace

struct dlf_net_s {
    std::vector<Layer> L;
    int in_h, in_w, in_c;
    bool has_weights;
};

namespace {

// ------------------------------------------------------------------------------------------
// Weight repacking
// ------------------------------------------------------------------------------------------

// MFMA "A" fragments for v_mfma_f32_32x32x16_f16: for output-channel block cb (32 channels) and
// K step t, lane l holds W[cb*32 + l%32][k(t) + (l/32)*8 + j], j = 0..7.  Steps run in the
// order the kernel consumes them: input-channel chunk (kc channels) -> filter tap -> 16-channel
// sub-step inside the chunk.
void pack_conv_weights(const uint16_t* w, int cout, int taps, int cin, int kc, int cin_pad,
                       std::vector<uint16_t>& out)
{
    const int ncb = ceil_div(cout, 32), nchunks = cin_pad / kc, nks = kc / 16;
    const size_t nsteps = (size_t)nchunks * taps * nks;
    out.assign((ncb * nsteps + 24) * 512, 0);  // 24 steps of zeros: the kernels prefetch up to 18 steps ahead
    for (int cb = 0; cb < ncb; ++cb)
        for (int chunk = 0; chunk < nchunks; ++chunk)
            for (int tap = 0; tap < taps; ++tap)
                for (int ks = 0; ks < nks; ++ks) {
                    const size_t step = ((size_t)chunk * taps + tap) * nks + ks;
                    uint16_t* dst = &out[(cb * nsteps + step) * 512];
                    for (int lane = 0; lane < 64; ++lane) {
                        const int co = cb * 32 + (lane & 31);
                        if (co >= cout) continue;
                        const int ci0 = chunk * kc + ks * 16 + (lane >> 5) * 8;
                        const uint16_t* src = w + ((size_t)co * taps + tap) * cin;
                        for (int j = 0; j < 8; ++j)
                            if (ci0 + j < cin) dst[lane * 8 + j] = src[ci0 + j];
                    }
                }
}

dlf_status upload(const void* host, size_t bytes, void** dev)
{
    hipError_t e = hipMalloc(dev, bytes);
    if (e != hipSuccess) return fail(DLF_ERR_OOM, "hipMalloc(%zu): %s", bytes, hipGetErrorString(e));
    e = hipMemcpy(*dev, host, bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) return fail(DLF_ERR_HIP, "hipMemcpy: %s", hipGetErrorString(e));
    return DLF_OK;
}

dlf_status pack_and_upload(Layer& L)
{
    const dlf_layer_desc& d = L.d;
    if (d.op == DLF_CONV || d.op == DLF_FC) {
        std::vector<uint16_t> packed;
        const int taps = d.kh * d.kw;
        if (L.rowfold) {
            // repack [cout][kh][kw][cin] as [cout][kh][cin_pad] with column kw*4 + c, zero elsewhere
            std::vector<uint16_t> w4((size_t)d.cout * d.kh * L.cin_pad, 0);
            const uint16_t* src = (const uint16_t*)d.weight;
            for (int co = 0; co < d.cout; ++co)
                for (int r = 0; r < d.kh; ++r)
                    for (int q = 0; q < d.kw; ++q)
                        for (int c = 0; c < d.cin; ++c)
                            w4[((size_t)co * d.kh + r) * L.cin_pad + q * 4 + c] =
                                src[(((size_t)co * d.kh + r) * d.kw + q) * d.cin + c];
            pack_conv_weights(w4.data(), d.cout, d.kh, L.cin_pad, L.kc, L.cin_pad, packed);
        } else if (L.im2col)   // [cout][kh][kw][cin] is already the gathered row order: a 1x1 over kh*kw*cin
            pack_conv_weights((const uint16_t*)d.weight, d.cout, 1, taps * d.cin, L.kc, L.cin_pad, packed);
        else
            pack_conv_weights((const uint16_t*)d.weight, d.cout, taps, d.cin, L.kc, L.cin_pad, packed);
        dlf_status s = upload(packed.data(), packed.size() * 2, &L.d_w);
        if (s != DLF_OK) return s;
        std::vector<float> b((size_t)L.ncb * 32, 0.0f);
        if (d.has_bias && d.bias) std::copy(d.bias, d.bias + d.cout, b.begin());
        return upload(b.data(), b.size() * 4, (void**)&L.d_bias);
    }
    if (d.op == DLF_DWCONV) {
        const int taps = d.kh * d.kw, cp = L.cin_pad;
        std::vector<uint16_t> w((size_t)taps * cp, 0);
        const uint16_t* src = (const uint16_t*)d.weight;
        for (int c = 0; c < d.cout; ++c)
            for (int t = 0; t < taps; ++t) w[(size_t)t * cp + c] = src[(size_t)c * taps + t];
        dlf_status s = upload(w.data(), w.size() * 2, &L.d_w);
        if (s != DLF_OK) return s;
        std::vector<float> b((size_t)cp, 0.0f);
        if (d.has_bias && d.bias) std::copy(d.bias, d.bias + d.cout, b.begin());
        return upload(b.data(), b.size() * 4, (void**)&L.d_bias);
    }
    return DLF_OK;
}

// ------------------------------------------------------------------------------------------
// Fusion groups
// ------------------------------------------------------------------------------------------

enum { GK_GROUP = 0, GK_FC = 1, GK_GAP = 2, GK_PW = 3, GK_C3 = 4, GK_DW = 5, GK_DWPW = 6, GK_DWT = 7, GK_PW2 = 8, GK_DWS = 9, GK_C3S = 10, GK_C3PW = 11, GK_BNECK = 12 };

struct TileCfg {
    int th, tw;      // tile of the group's final output tensor
    int variant;     // register tile of CONV stages
    int nslices, slice_c;
    int stream0;
    int kc;          // stream0: channels per streaming round (32, 64 or 128)
    int ksplit = 1;  // resident single CONV stage: waves that share a work item's K
};

struct GroupPlan {
    int first = 0, last = 0, budget = 0;
    int kind = GK_GROUP;
    int variant = 0, lds_bytes = 0, grid = 0, occ = 1;
    size_t scratch_bytes = 0, scratch_off = 0;   // device scratch in the workspace (split-K FC)
    int th = 0, tw = 0;
    uint64_t cost = 0;
    int in_layer = -1;   // producer of the group's input (-1 = net input)
    int res_layer = -2;  // producer of a residual operand read from HBM (-2 = none)
    int res_stage = -1;
    DlfGroupArgs ga;
    DlfFcArgs fa;
    DlfGapArgs pa;
    DlfPwArgs wa;
    DlfC3Args ca;
    DlfDwArgs da;
    DlfDwPwArgs dp;
    DlfDwtArgs dt;
    DlfDwsArgs ds;
    DlfC3sArgs cs; DlfC3PwArgs cp; DlfBnArgs bn;
};

const int VAR_FC[DLF_NUM_VARIANTS] = {2, 1, 1, 1};
const int VAR_FP[DLF_NUM_VARIANTS] = {2, 4, 2, 2};
const int VAR_OCC[DLF_NUM_VARIANTS] = {1, 1, 1, 2};   // workgroups per CU the registers allow

// Constants of the cost model, in GPU cycles unless noted (MI355X: 256 CUs at about 2.15 GHz
// under load, HBM about 3300 bytes per cycle for the whole chip).  All arithmetic is integer so
// that an independent implementation reproduces every cost bit for bit.
const int64_t PS_PER_CYCLE = 465;
const int64_t HBM_BYTES_PER_CYCLE = 3300;   // whole chip
const int64_t CU_BYTES_PER_CYCLE = 12;      // what the workgroups of one CU pull from HBM
const int64_t L2_BYTES_PER_CYCLE = 48;      // weight fragments, L2 -> one CU
const int64_t C_LAUNCH = 9000;              // kernel launch + drain
const int64_t C_TILE = 6000;                // per tile: decode, address setup, barriers
const int64_t C_LAT = 5000;                 // one exposed HBM/L2 round trip
const int64_t C_STAGE_VEC = 120;             // per 512 staged 16-byte vectors
const int64_t C_IM2COL = 150;                // per gathered element per 512 (pixel, row) pairs
const int64_t C_ROWFOLD = 400;               // per 512 staged narrow pixels (3 element loads, one 8-byte LDS write)
const int64_t C_ROUND = 1500;               // lower bound of a streaming round: loader latency ...
const int64_t C_ROUND_VEC = 300;            // ... plus this per 16-byte vector a data-movement thread brings in
const int64_t C_BARRIER = 500;
const int64_t C_KSPLIT = 2500;              // K split over waves: partial sums through LDS, a barrier
const int64_t C_EPI = 900;                  // epilogue per 32x32 accumulator block
const int64_t C_VALU = 100;                  // per tap per 512 (pixel, 8 channels) items
const int64_t C_STAGE = 1200;                // per VALU stage
const int64_t C_STORE_VEC = 80;             // per 512 stored 16-byte vectors
const int64_t C_STORE = 1600;
const int64_t MFMA_CYCLES = 32;             // one 32x32x16 MFMA on one SIMD
const int64_t FC_BYTES_PER_CYCLE = 1400;    // weight streaming rate of the FC kernel
const int64_t FC_SPLIT_HBM_BYTES_PER_CYCLE = 1900;   // the same with K split over all CUs
const int64_t GAP_BYTES_PER_CYCLE = 1000;
// pointwise kernel, per item shape: register tile (FC x FP blocks of 32), operand ring depth,
// independent waves per CU
// (shape 2: the split-K form, a 64 x 64 item per workgroup of four waves, two workgroups per CU)
// (shapes 3, 4: the block form, four waves share a block of 128 x 128 or 64 channels x 256 pixels
// through LDS, two workgroups per CU)
const int PW_SHAPES = 5;
const int PW_FC[PW_SHAPES] = {2, 1, 2, 4, 2};          // 32-channel blocks per item
const int PW_FP[PW_SHAPES] = {2, 1, 2, 4, 8};          // 32-pixel blocks per item
const int PW_WAVES_PER_CU[PW_SHAPES] = {8, 16, 1, 2, 2};     // items in flight per CU that cost no more than one
                                                             // (split-K: a second item on the CU doubles the time)
const int PW_KSPLIT[PW_SHAPES] = {1, 1, 4, 1, 1};
const bool PW_BLOCK[PW_SHAPES] = {false, false, false, true, true};
// fitted to per-launch HIP-event times of 1x1 layers of the ResNet-50 / MobileNet-v1 shapes
const int64_t C_PW_ITEM = 2500;             // per work item: address setup, epilogue
const int64_t C_PW_STEP[PW_SHAPES] = {470, 300, 470, 0, 0};   // per K step of a latency-bound wave ...
const int64_t C_PW_STEP_WAVE[PW_SHAPES] = {64, 100, 256, 0, 0};   // ... or of a CU whose waves share its vector-memory path
const int64_t C_PWB_BLOCK = 4000;           // block form, per round of two blocks on a CU: first operands, epilogue
const int64_t PWB_BYTES_PER_CYCLE = 28;     // rate at which a CU takes operand fragments in (block form of the pointwise kernel)
const int64_t PW_BYTES_PER_CYCLE = 25;      // ... the per-wave forms, the 1x1 phase of the depthwise tile kernel, the FC kernel
const int64_t C_PW_SK = 2000;               // split-K: exchange of partial sums through LDS
const int64_t C_PW_RES = 1000;              // residual loads
const int64_t PW_HBM_BYTES_PER_CYCLE = 2000;
// block 3x3 kernel: per work item (first stages of the ring, epilogue), per LDS stage of 16 input
// channels (nine taps x four MFMAs on each of two waves per SIMD, in tenths), intake of a stage
const int64_t C_C3_ITEM = 10000;
const int64_t C_C3_SHORT_K = 6000;          // per item when K has fewer than 8 stages: the ring never reaches its steady state
const int64_t C3_MMA_TENTHS = 15;
const int64_t C3_BYTES_PER_CYCLE = 27;
const int64_t C3_SHALLOW_RING = 300;        // per stage when the weight ring has two stages only

// streaming depthwise kernel: per work item (decode, weights, first rows of the window), per output
// row of a wave (about a hundred vector instructions; the waves of a SIMD share its issue slots),
// the rate at which the chip streams the tensors, waves in flight per CU
const int64_t C_DW_ITEM = 2500;
const int64_t C_DW_ROW = 420;
const int64_t DW_HBM_BYTES_PER_CYCLE = 2300;
const int64_t DW_CU_BYTES_PER_CYCLE = 24;
const int DW_WAVES_PER_CU = 16;

// fused depthwise + 1x1 kernel: per work item (decode, first loads, epilogue), per K step the vector
// instructions of a wave (nine taps x 8 channels of mixed-precision multiply-adds and their operands;
// the two waves of a SIMD share its issue slots), cycles a CU's vector-memory path needs per load
// instruction of a wave: a K step takes 16 of a pixel's channels, a quarter of a 128-byte line, and
// with eight waves' lines in flight the CU's cache does not keep a line until the next K step asks
// for it again, so 1 KiB of operands costs 4 KiB of intake (measured: 800 cycles per K step and item
// on a CU for 13 loads)
const int64_t C_DWPW_ITEM = 4000;
const int64_t C_DWPW_STEP = 470;
const int64_t C_DWPW_LOAD = 62;

// depthwise + 1x1 tile kernel: per tile (decode, barriers, first rows of the window in flight), per
// output row of the depthwise phase, per work unit of the 1x1 phase (first fragments, epilogue
// set-up), per K step and 32-pixel block of a unit (at least two blocks' worth: below that the
// operand reads, not the MFMAs, set the pace), per 32-pixel block of a unit's epilogue.  Fitted to
// the eight depthwise / 1x1 pairs of MobileNet-v1 at batch 64, every tile shape forced in turn; the
// workgroups that share a CU (two: registers) split its time.
const int64_t C_DWT_TILE = 6000;
const int64_t C_DWT_ROW = 630;
const int64_t C_DWT_UNIT = 2250;
const int64_t C_DWT_STEP = 48;
const int64_t C_DWT_EPI = 750;
// small-map depthwise + 1x1 kernel: per work item a fixed part (the first region's trip to memory,
// barriers, store drain), the trip of every further region that is not resident, per depthwise step
// of a wave pair, per K step and channel block of a wave, per channel block of a wave in the epilogue
const int64_t C_DWS_ITEM = 7000;
const int64_t C_DWS_REGION = 5000;
const int64_t C_DWS_STEP = 1070;
const int64_t C_DWS_MMA = 120;
const int64_t C_DWS_EPI = 2500;
const int64_t DWS_BYTES_PER_CYCLE = 64;
// small-map 3x3 kernel: per work item a fixed part (beyond the launch's own round trip), per K step of a
// wave two MFMAs beside those of the SIMD's other wave -- 128 cycles at the pipe's rate, measured on the
// 256-channel layers; the 512-channel layers (weights above 3 MiB, K loops of 30 thousand cycles) run at
// 215 whether an XCD's L2 holds all of its weights or not: the rate the matrix pipes sustain on such
// operands --, the exchange of partial sums, the epilogue; a CU's further items each pay the region's trip to memory
// and the store drain in full (one workgroup per CU: nothing overlaps them)
const int64_t C_C3S_ITEM = 3000;
const int64_t C_C3S_NEXT = 13000;
const int64_t C_C3S_STEP = 128;
const int64_t C_C3S_STEP_BIG = 215;
const int64_t C_C3S_BIG_BYTES = 3 << 20;
const int64_t C_C3S_RED = 1500;
const int64_t C_C3S_EPI = 2500;
// the fused 3x3 -> 1x1 kernel for small maps: per work item (decode, first loads), bytes per cycle of
// its LDS intake, cycles per MFMA of a SIMD, per K step of the first layer's weight ring (requests
// nine steps ahead against the L2's latency), per channel block of the first layer for the hand-over
// of its result, per item for the second layer's start, and the rate at which the chip takes the
// stores of all items of a round, which run their last phase together
const int64_t C_C3PW_ITEM = 3500;
const int64_t C3PW_BYTES_PER_CYCLE = 16;
const int64_t C_C3PW_MMA = 38;
const int64_t C_C3PW_STEP = 125;
const int64_t C_C3PW_MID = 600;
const int64_t C_C3PW_SECOND = 1000;
const int64_t C3PW_STORE_BYTES_PER_CYCLE = 2300;
const int64_t C_BN_ITEM = 14000;              // bottleneck kernel: per item, per tile pixel, per 16 input channels beyond 256
const int64_t C_BN_PIXEL = 245;
const int64_t C_BN_CHANNEL = 150;
const int64_t C_BN_LAST = 5000;              // ... less without the last layer
const int64_t C3PW_OVERLAP_PCT = 60;         // two workgroups per CU: what a further round of items adds, in per cent of an item

struct StageSpec {   // one stage, before tiling
    int layer;
    int kind;
    int pool2;
    int pool_layer;  // layer index of the folded pool, or -1
};

bool is_pool2(const dlf_layer_desc& d)
{
    return d.op == DLF_MAXPOOL && d.kh == 2 && d.kw == 2 && d.stride == 2 && d.pad == 0;
}

// Can layers [first,last] form one group?  Returns the stage list.
bool group_stages(const dlf_net_s& net, int first, int last, std::vector<StageSpec>& st, int& kind,
                  std::string& why)
{
    st.clear();
    const Layer& L0 = net.L[first];
    if (L0.d.op == DLF_FC || L0.d.op == DLF_GLOBAL_AVGPOOL) {
        if (first != last) { why = "FC / global pooling layers run as their own group"; return false; }
        kind = (L0.d.op == DLF_FC) ? GK_FC : GK_GAP;
        return true;
    }
    kind = GK_GROUP;
    // does any layer other than j+1 read tensor j, or does j+1 add it as a residual?
    auto escapes = [&](int j) {
        for (size_t k = 0; k < net.L.size(); ++k) {
            if (net.L[k].d.residual_from == j) return true;
            if ((int)k != j + 1 && net.L[k].src == j) return true;
        }
        return false;
    };
    for (int i = first; i <= last; ++i) {
        const Layer& L = net.L[i];
        const dlf_layer_desc& d = L.d;
        if (d.op == DLF_FC || d.op == DLF_GLOBAL_AVGPOOL) { why = "FC / global pooling inside a group"; return false; }
        if (i > first && L.src != i - 1) { why = "layer input is not the previous layer of the group"; return false; }
        if (d.residual_from >= first && d.residual_from <= last) { why = "residual operand produced inside the group"; return false; }
        if (d.residual_from >= 0 && d.op != DLF_CONV) { why = "residual add on a non-convolution layer"; return false; }
        if (d.residual_from >= 0 && i != last) { why = "a residual add must be the last layer of its group"; return false; }
        // a tensor produced inside the group (except the last) must not be used outside it
        if (i < last && escapes(i)) { why = "intermediate tensor is used outside the group"; return false; }
        StageSpec s;
        s.layer = i;
        s.pool2 = 0;
        s.pool_layer = -1;
        if (d.op == DLF_CONV) {
            s.kind = DLF_ST_CONV;
            if (d.cout % 4 != 0) { why = "convolution output channels must be a multiple of 4"; return false; }
            if (i + 1 <= last && is_pool2(net.L[i + 1].d) && net.L[i + 1].src == i && (L.out_h % 2 == 0)
                && (L.out_w % 2 == 0) && d.residual_from < 0) {
                // the pooled tensor replaces the convolution output (which nothing else reads:
                // checked above); the pooled tensor in turn must stay inside unless it is last
                if (i + 1 < last && escapes(i + 1)) { why = "intermediate tensor is used outside the group"; return false; }
                s.pool2 = 1;
                s.pool_layer = i + 1;
            }
        } else if (d.op == DLF_DWCONV) {
            s.kind = DLF_ST_DW;
            if (d.cin % 8 != 0) { why = "depthwise channels must be a multiple of 8"; return false; }
        } else {
            s.kind = DLF_ST_MAXPOOL;
            if (d.cin % 8 != 0) { why = "pooling channels must be a multiple of 8"; return false; }
            if (d.pad >= d.kh) { why = "pooling pad must be smaller than the window"; return false; }
        }
        st.push_back(s);
        if (s.pool2) ++i;
    }
    if ((int)st.size() > DLF_MAX_STAGES) { why = "too many stages"; return false; }
    // a CONV stage after stage 0 needs all its input channels in LDS: VALU producers must
    // write a multiple of the consumer's chunk size
    for (size_t k = 1; k < st.size(); ++k) {
        if (st[k].kind == DLF_ST_CONV && st[k - 1].kind != DLF_ST_CONV) {
            const Layer& C = net.L[st[k].layer];
            if (C.d.cin % 32 != 0) { why = "channel count not a multiple of the K chunk"; return false; }
        }
    }
    return true;
}

struct Built {
    bool ok = false;
    int lds_bytes = 0;
    int ntiles = 0;
    int64_t tile_cycles = 0;      // modelled cycles one workgroup spends per tile (compute side)
    int64_t tile_mma_cycles = 0;  // the part of them that occupies the matrix pipes
    int64_t tile_hbm_bytes = 0;   // activation bytes per tile (HBM side)
    int64_t tile_l2_bytes = 0;    // weight bytes per tile (L2 side)
    DlfGroupArgs ga;
};

// Builds the kernel arguments of a group for one tiling choice; ok=false if it does not fit.
Built build_group(const dlf_net_s& net, const std::vector<StageSpec>& specs, int batch,
                  const TileCfg& tc, int max_lds)
{
    Built b;
    DlfGroupArgs& ga = b.ga;
    memset(&ga, 0, sizeof ga);
    const int ns = (int)specs.size();
    const Layer& Lfirst = net.L[specs[0].layer];
    const StageSpec& slast = specs[ns - 1];
    const Layer& Llast = net.L[slast.pool2 ? slast.pool_layer : slast.layer];
    const int FCv = VAR_FC[tc.variant], FPv = VAR_FP[tc.variant];
    ga.nstages = ns;
    ga.stream0 = tc.stream0;
    ga.batch = batch;
    ga.in_h = Lfirst.in_h; ga.in_w = Lfirst.in_w; ga.in_c = Lfirst.in_c;
    ga.out_h = Llast.out_h; ga.out_w = Llast.out_w; ga.out_c = Llast.out_c;
    ga.th = tc.th; ga.tw = tc.tw;
    ga.tiles_y = ceil_div(ga.out_h, tc.th);
    ga.tiles_x = ceil_div(ga.out_w, tc.tw);
    ga.nslices = tc.nslices;
    ga.slice_c = tc.slice_c;
    ga.ntiles = batch * ga.tiles_y * ga.tiles_x * tc.nslices;
    b.ntiles = ga.ntiles;

    // backward region propagation
    int my = 1, oy = 0, mx = 1, ox = 0, h = tc.th, w = tc.tw;
    for (int s = ns - 1; s >= 0; --s) {
        const Layer& L = net.L[specs[s].layer];
        DlfStage& st = ga.st[s];
        st.kind = specs[s].kind;
        st.pool2 = specs[s].pool2;
        if (st.pool2) { my *= 2; oy *= 2; mx *= 2; ox *= 2; h *= 2; w *= 2; }
        st.cin = L.d.cin; st.cout = L.d.cout;
        st.kh = L.d.kh; st.kw = L.d.kw; st.stride = L.d.stride; st.pad = L.d.pad; st.act = L.d.act;
        st.in_h = L.in_h; st.in_w = L.in_w; st.out_h = L.out_h; st.out_w = L.out_w;
        st.rh = h; st.rw = w;
        st.oy_mul = my; st.oy_off = oy; st.ox_mul = mx; st.ox_off = ox;
        st.ih = (h - 1) * st.stride + st.kh;
        st.iw = (w - 1) * st.stride + st.kw;
        my *= st.stride; oy = oy * st.stride - st.pad;
        mx *= st.stride; ox = ox * st.stride - st.pad;
        h = st.ih; w = st.iw;
        st.im2col = 0;
        if (st.kind == DLF_ST_CONV && L.rowfold) {
            if (s != 0 || tc.stream0) return b;      // folded staging: resident stage 0 only
            st.im2col = 2;
            st.im_kh = st.kh; st.im_kw = st.kw; st.im_stride = st.stride; st.im_pad = st.pad;
            st.im_cin = L.d.cin;
            st.kw = 1;                                // what the MFMA loop sees: one tap per row
            st.iw = round_up(st.iw, 2);               // keeps every 16-byte LDS read aligned
        } else if (st.kind == DLF_ST_CONV && L.im2col) {
            if (s != 0 || tc.stream0) return b;      // gathered staging: resident stage 0 only
            st.im2col = 1;
            st.im_kh = st.kh; st.im_kw = st.kw; st.im_stride = st.stride; st.im_pad = st.pad;
            st.im_cin = L.d.cin;
            st.kh = st.kw = 1; st.stride = 1; st.pad = 0;   // what the MFMA loop sees
            st.ih = st.rh; st.iw = st.rw;
        }
        st.w = L.d_w; st.bias = L.d_bias; st.res = nullptr;
        if (st.kind == DLF_ST_CONV) {
            st.kc = (s == 0 && tc.stream0) ? tc.kc : 32;
            st.kc_shift = st.kc == 128 ? 4 : (st.kc == 64 ? 3 : 2);
            st.cin_pad = L.cin_pad; st.ncb = L.ncb; st.nsteps = L.nsteps;
            if (st.kc != 32 && st.kc != 64 && st.kc != 128) return b;
            if (L.cin_pad % st.kc != 0) return b;
            if (st.kc != 32 && (L.d.cin & 7) != 0) return b;
        } else {
            st.kc = 8; st.kc_shift = 0; st.cin_pad = round_up(L.d.cin, 8); st.ncb = 0; st.nsteps = 0;
        }
    }
    ga.iy_mul = my; ga.iy_off = oy; ga.ix_mul = mx; ga.ix_off = ox;

    // slicing rules
    if (tc.nslices > 1) {
        for (int s = 1; s < ns; ++s)
            if (ga.st[s].kind == DLF_ST_CONV) return b;  // later CONV stages need every channel
        if (ga.st[0].kind == DLF_ST_CONV && (tc.slice_c % 32) != 0) return b;
        if ((tc.slice_c % 8) != 0) return b;
        const int cslice = ga.st[0].kind == DLF_ST_CONV ? ga.st[0].cout : ga.st[0].cin;
        if ((int64_t)tc.nslices * tc.slice_c < cslice) return b;   // slices must cover every channel
    }
    // the kernels form element offsets into the input, output and residual tensors in 32 bits
    if ((int64_t)batch * ga.in_h * ga.in_w * ga.in_c >= (int64_t)1 << 31) return b;
    if ((int64_t)batch * (ga.out_h + 32) * (ga.out_w + 32) * ga.out_c >= (int64_t)1 << 31) return b;
    const int chan_local = (tc.nslices > 1) ? tc.slice_c : 0;   // 0 = all channels

    // LDS layout: stage s reads buffer s, writes buffer s+1; even buffers share one area,
    // odd buffers the other.
    int64_t area[2] = {0, 0};
    std::vector<int64_t> bufsz(ns + 1, 0);
    for (int s = 0; s < ns; ++s) {
        DlfStage& st = ga.st[s];
        int cs;
        if (st.kind == DLF_ST_CONV && st.im2col == 2) {
            cs = 4;
        } else if (st.kind == DLF_ST_CONV) {
            cs = (s == 0 && tc.stream0) ? st.kc + DLF_CPAD : st.cin_pad + DLF_CPAD;
        } else {
            const int c = chan_local ? chan_local : st.cin;
            cs = round_up(c, 8) + DLF_CPAD;
        }
        st.in_cs = cs;
        if (s > 0) ga.st[s - 1].out_cs = cs;
        int64_t sz = (int64_t)st.ih * st.iw * cs;
        if (st.kind == DLF_ST_CONV && st.im2col == 2) sz += 32;   // zeroed slack behind the last pixel
        if (s == 0 && tc.stream0) {
            st.stream_buf = (int)sz;
            sz *= 2;
            if ((int64_t)st.ih * st.iw * (st.kc / 8) > (int64_t)DLF_STAGE_VECS * DLF_LOAD_THREADS) return b;
        }
        bufsz[s] = sz;
        area[s & 1] = std::max(area[s & 1], sz);
    }
    // K split over waves: a single resident CONV stage on a register tile of at most 64 pixels x 32
    // channels (the partial sums of 8 waves must fit LDS), chunks divisible, one pass of work items
    for (int s = 0; s < ns; ++s) { ga.st[s].ksplit = 1; ga.st[s].ks_off = 0; }
    if (tc.ksplit != 1) {
        const DlfStage& st = ga.st[0];
        if (tc.ksplit != 2 && tc.ksplit != 4 && tc.ksplit != 8) return b;
        if (ns != 1 || st.kind != DLF_ST_CONV || tc.stream0 || st.im2col || FCv * FPv > 2) return b;
        if ((st.cin_pad / 32) % tc.ksplit != 0) return b;
        const int npb = ceil_div(st.rh * st.rw, 32), n_pg = ceil_div(npb, FPv);
        const int cbs = tc.nslices > 1 ? std::min(st.ncb, tc.slice_c / 32) : st.ncb;
        if (n_pg * ceil_div(cbs, FCv) * tc.ksplit > DLF_WAVES) return b;
    }
    // the last CONV stage leaves its tile in LDS (buffer ns); store_tile copies it to HBM.  Where
    // every wave has at most one work item of that stage (or the stage streams, which ends with a
    // barrier anyway), the tile may overwrite the stage's own input: one barrier between the
    // last MFMA and the epilogue, and the group needs that much less LDS.
    bool alias_out = false;
    if (ga.st[ns - 1].kind == DLF_ST_CONV) {
        DlfStage& st = ga.st[ns - 1];
        const int c = chan_local ? chan_local : st.cout;
        st.out_cs = round_up(c, 8) + DLF_CPAD;
        const int ph = st.pool2 ? st.rh / 2 : st.rh, pw = st.pool2 ? st.rw / 2 : st.rw;
        const int npb = ceil_div(st.rh * st.rw, 32), n_pg = ceil_div(npb, FPv);
        const int cbs = tc.nslices > 1 ? std::min(st.ncb, tc.slice_c / 32) : st.ncb;
        const int nitems = n_pg * ceil_div(cbs, FCv);
        const bool streaming = (ns == 1 && tc.stream0);
        alias_out = streaming || nitems <= DLF_WAVES;
        st.alias_out = alias_out ? 1 : 0;
        area[(alias_out ? ns - 1 : ns) & 1] =
            std::max(area[(alias_out ? ns - 1 : ns) & 1], (int64_t)ph * pw * st.out_cs);
    }
    // consistency: what stage s writes must be what stage s+1 reads
    for (int s = 0; s + 1 < ns; ++s) {
        const DlfStage& p = ga.st[s];
        const DlfStage& c = ga.st[s + 1];
        const int ph = p.pool2 ? p.rh / 2 : p.rh, pw = p.pool2 ? p.rw / 2 : p.rw;
        if (ph != c.ih || pw != c.iw) return b;
        if (p.pool2 && ((p.oy_off & 1) || (p.ox_off & 1) || (p.rh & 1) || (p.rw & 1))) return b;
    }
    if (ga.st[ns - 1].pool2 && ((tc.th * 2 != ga.st[ns - 1].rh))) return b;
    for (int s = 0; s < ns; ++s) {
        ga.st[s].in_off = (s & 1) ? (int)area[0] : 0;
        ga.st[s].out_off = ((s + 1) & 1) ? (int)area[0] : 0;
    }
    if (alias_out) ga.st[ns - 1].out_off = ga.st[ns - 1].in_off;
    int64_t lds_halfs = area[0] + area[1];
    if (tc.ksplit > 1) {
        ga.st[0].ksplit = tc.ksplit;
        lds_halfs = round_up((int)lds_halfs, 8);
        ga.st[0].ks_off = (int)lds_halfs;
        lds_halfs += (int64_t)DLF_WAVES * FCv * FPv * 16 * 64 * 2;      // fp32 = 2 halfs
    }
    if (lds_halfs * 2 > max_lds) return b;
    b.lds_bytes = (int)(lds_halfs * 2);

    // ---- cost model: cycles one workgroup spends on one tile ----
    int64_t cyc = C_TILE, l2 = 0, mma_total = 0;
    const DlfStage& s0 = ga.st[0];
    const int cin0 = (s0.kind != DLF_ST_CONV && chan_local) ? chan_local : s0.cin;
    if (tc.stream0) {
        cyc += C_LAT;
    } else if (s0.kind == DLF_ST_CONV && s0.im2col == 2) {
        cyc += C_LAT + (int64_t)ceil_div(s0.ih * s0.iw, DLF_WG_THREADS) * C_ROWFOLD;
    } else if (s0.kind == DLF_ST_CONV && s0.im2col) {
        cyc += C_LAT + (int64_t)ceil_div(s0.rh * s0.rw * s0.im_kh, DLF_WG_THREADS) * s0.im_kw * s0.im_cin * C_IM2COL;
    } else {
        const int cfill = s0.kind == DLF_ST_CONV ? s0.cin_pad : round_up(cin0, 8);
        cyc += C_LAT + (int64_t)ceil_div(s0.ih * s0.iw * (cfill / 8), DLF_WG_THREADS) * C_STAGE_VEC;
    }
    for (int s = 0; s < ns; ++s) {
        const DlfStage& st = ga.st[s];
        const int npix = st.rh * st.rw;
        if (st.kind == DLF_ST_CONV) {
            const int npb = ceil_div(npix, 32), n_pg = ceil_div(npb, FPv);
            int cbs = st.ncb;
            if (tc.nslices > 1) cbs = std::min(st.ncb, tc.slice_c / 32);
            const int n_cg = ceil_div(cbs, FCv);
            const int nitems = n_pg * n_cg * tc.ksplit;           // K slices run like work items
            const bool streaming = (s == 0 && tc.stream0);
            const int mma_waves = streaming ? DLF_MMA_WAVES : DLF_WAVES;
            if (streaming && nitems > mma_waves) return b;
            // items queue up on the 4 SIMDs; measured rounds run at 1.8 times the MFMA issue time
            // (a 32 x 128 register tile needs half the weight traffic per MFMA and runs closer to
            //  the issue rate: 1.3)
            int64_t mma = (int64_t)ceil_div(nitems, 4) * (st.nsteps / tc.ksplit) * FCv * FPv * MFMA_CYCLES * (FPv >= 4 ? 13 : 18) / 10;
            if (streaming) {
                const int64_t nrounds = st.cin_pad / st.kc;
                const int64_t vecs = ceil_div(st.ih * st.iw * (st.kc / 8), DLF_LOAD_THREADS);
                mma = std::max(mma, nrounds * (C_ROUND + vecs * C_ROUND_VEC)) + nrounds * C_BARRIER;
            }
            mma_total += mma;
            cyc += mma + (int64_t)ceil_div(nitems, mma_waves) * FCv * FPv * C_EPI + (tc.ksplit > 1 ? C_KSPLIT : 0);
            l2 += (int64_t)nitems * FCv * (st.nsteps / tc.ksplit) * 1024;
        } else {
            const int c = chan_local ? chan_local : st.cout;
            const int64_t items = (int64_t)npix * ceil_div(c, 8);
            cyc += (int64_t)ceil_div((int)items, DLF_WG_THREADS) * (st.kh * st.kw) * C_VALU + C_STAGE;
        }
    }
    const DlfStage& sl = ga.st[ns - 1];
    const int cout_l = chan_local ? std::min(chan_local, ga.out_c) : ga.out_c;
    const int has_res = net.L[specs[ns - 1].layer].d.residual_from >= 0 ? 1 : 0;
    if (sl.kind == DLF_ST_CONV)
        cyc += (int64_t)ceil_div(tc.th * tc.tw * ceil_div(cout_l, 8), DLF_WG_THREADS) * C_STORE_VEC + C_STORE
               + has_res * C_LAT;
    b.tile_hbm_bytes = (int64_t)s0.ih * s0.iw * cin0 * 2 + (int64_t)tc.th * tc.tw * cout_l * 2 * (1 + has_res);
    if (s0.kind == DLF_ST_CONV && s0.im2col == 2)
        b.tile_hbm_bytes = (int64_t)s0.ih * s0.iw * s0.im_cin * 2 + (int64_t)tc.th * tc.tw * cout_l * 2;
    else if (s0.kind == DLF_ST_CONV && s0.im2col)
        b.tile_hbm_bytes = (int64_t)s0.rh * s0.rw * s0.im_stride * s0.im_stride * s0.im_cin * 2
                           + (int64_t)tc.th * tc.tw * cout_l * 2;
    b.tile_l2_bytes = l2;
    b.tile_cycles = cyc;
    b.tile_mma_cycles = mma_total;
    b.ok = true;
    return b;
}

// Cost-model time of a built group on `budget` CUs, in picoseconds.
uint64_t group_cost_ps(const Built& b, int budget, int variant)
{
    const int occ = std::max(1, std::min(VAR_OCC[variant], (160 * 1024) / std::max(b.lds_bytes, 1)));
    const int64_t cu = std::min<int64_t>(budget, b.ntiles);
    const int64_t wg = std::min<int64_t>(b.ntiles, (int64_t)budget * occ);
    const int64_t conc = (wg + cu - 1) / cu;              // workgroups sharing a CU
    const int64_t tiles_cu = (b.ntiles + cu - 1) / cu;    // tiles one CU works through
    // Everything but the MFMA loops (staging, epilogues, VALU stages, stores, barriers) is a chain
    // of latencies: a workgroup alone on its CU pays them in full (5/4 of the fitted terms); two
    // workgroups fill each other's gaps (3/5 of the total), down to the time the matrix pipes
    // they share are busy.
    const int64_t tile = b.tile_mma_cycles + (b.tile_cycles - b.tile_mma_cycles) * 5 / 4;
    int64_t compute = tiles_cu * (conc >= 2 ? std::max(b.tile_mma_cycles, tile * 3 / 5) : tile);
    const int64_t bw = std::min<int64_t>(CU_BYTES_PER_CYCLE, std::max<int64_t>(1, HBM_BYTES_PER_CYCLE / cu));
    const int64_t mem = tiles_cu * (b.tile_hbm_bytes / bw + b.tile_l2_bytes / L2_BYTES_PER_CYCLE);
    return (uint64_t)((C_LAUNCH + std::max(compute, mem)) * PS_PER_CYCLE);
}

// Testing hook: when th > 0 every group is built with exactly this configuration.
TileCfg g_force = {0, 0, 0, 1, 0, 0, 32};

const int TILE_H[] = {2, 4, 7, 8, 14, 16};
const int TILE_W[] = {4, 7, 8, 14, 16, 28, 32};

// Chooses tile / register tile / slicing for a group at a given budget: minimum modelled cost;
// ties go to the earlier candidate in enumeration order.
bool choose_group(const dlf_net_s& net, const std::vector<StageSpec>& specs, int batch, int budget,
                  int max_lds, Built& best, TileCfg& best_tc, uint64_t& best_cost,
                  const TileCfg& force = g_force, std::vector<std::pair<uint64_t, TileCfg>>* all = nullptr)
{
    bool found = false;
    const int ns = (int)specs.size();
    if (force.th > 0) {
        Built b = build_group(net, specs, batch, force, max_lds);
        if (!b.ok) return false;
        best = b;
        best_tc = force;
        best_cost = group_cost_ps(b, budget, force.variant);
        return true;
    }
    const Layer& Llast = net.L[specs[ns - 1].pool2 ? specs[ns - 1].pool_layer : specs[ns - 1].layer];
    const Layer& L0 = net.L[specs[0].layer];
    const bool conv0 = specs[0].kind == DLF_ST_CONV;
    bool later_conv = false, any_conv = conv0;
    for (int s = 1; s < ns; ++s)
        if (specs[s].kind == DLF_ST_CONV) { later_conv = true; any_conv = true; }
    for (int th : TILE_H) {
        if (th > Llast.out_h && th != TILE_H[0] && (th - Llast.out_h) >= 4) continue;
        for (int tw : TILE_W) {
            if (tw > Llast.out_w && tw != TILE_W[0] && (tw - Llast.out_w) >= 4) continue;
            if (th * tw > 512) continue;
            for (int variant = 0; variant < DLF_NUM_VARIANTS; ++variant) {
                if (!any_conv && variant != 0 && variant != 3) continue;   // only occupancy differs
                std::vector<TileCfg> cands;
                if (conv0) {
                    // slicing over output channels: only if no later CONV stage
                    const int ncb = L0.ncb, FCv = VAR_FC[variant];
                    const bool pointwise = (L0.d.cin & 7) == 0;   // any filter may stream 32..128 channels per round
                    for (int stream0 = 1; stream0 >= 0; --stream0) {
                        for (int kc = 32; kc <= (stream0 && pointwise ? 128 : 32); kc *= 2) {
                            if (L0.cin_pad % kc != 0) continue;
                            TileCfg t{th, tw, variant, 1, 0, stream0, kc};
                            cands.push_back(t);
                            if (!stream0 && ns == 1 && FCv * VAR_FP[variant] <= 2) {
                                // a single resident CONV: K split over 2, 4 or 8 waves, whole or
                                // sliced over the output channels
                                for (int ks = 2; ks <= 8; ks *= 2) {
                                    TileCfg k{th, tw, variant, 1, 0, 0, 32, ks};
                                    cands.push_back(k);
                                    for (int cg = 1; cg <= 4; cg *= 2) {
                                        const int sc = FCv * cg * 32;
                                        if (sc >= ncb * 32) continue;
                                        TileCfg u{th, tw, variant, ceil_div(ncb * 32, sc), sc, 0, 32, ks};
                                        cands.push_back(u);
                                    }
                                }
                            }
                            if (!later_conv && stream0) {
                                for (int cg = 1; cg <= 4; cg *= 2) {
                                    const int sc = FCv * cg * 32;
                                    if (sc >= ncb * 32) continue;
                                    TileCfg u{th, tw, variant, ceil_div(ncb * 32, sc), sc, 1, kc};
                                    cands.push_back(u);
                                }
                            }
                        }
                    }
                } else {
                    TileCfg t{th, tw, variant, 1, 0, 0, 32};
                    cands.push_back(t);
                    if (!later_conv) {
                        for (int sc = 32; sc < L0.d.cin; sc *= 2) {
                            TileCfg u{th, tw, variant, ceil_div(L0.d.cin, sc), sc, 0, 32};
                            cands.push_back(u);
                        }
                    }
                }
                for (const TileCfg& tc : cands) {
                    Built b = build_group(net, specs, batch, tc, max_lds);
                    if (!b.ok) continue;
                    const uint64_t c = group_cost_ps(b, budget, tc.variant);
                    if (all) all->push_back(std::make_pair(c, tc));
                    if (!found || c < best_cost) {
                        found = true;
                        best = b;
                        best_tc = tc;
                        best_cost = c;
                    }
                }
            }
        }
    }
    return found;
}

// Testing hook: 0 = the pointwise kernel competes with the fused-group kernel on modelled cost,
// 1 = always where it applies, 2 = never, 3 .. 7 = always, with item shape 0 .. 4 (shape 2
// falls back to 0 where K does not split in four).
int g_pw_mode = 0;

// A convolution the pointwise kernel can run: 1x1, no padding, whole 32-channel K chunks.
bool pw_eligible(const Layer& L, int batch)
{
    const dlf_layer_desc& d = L.d;
    if (d.op != DLF_CONV || d.kh != 1 || d.kw != 1 || d.pad != 0) return false;
    if ((d.cin % 32) != 0 || (d.cout % 8) != 0) return false;
    if ((int64_t)batch * L.in_h * L.in_w * L.in_c >= (int64_t)1 << 31) return false;
    if ((int64_t)batch * L.out_h * L.out_w * L.out_c >= (int64_t)1 << 31) return false;
    return true;
}

uint64_t pw_shape_cost_ps(const Layer& L, int batch, int budget, int shape)
{
    const int64_t FCs = PW_FC[shape], FPs = PW_FP[shape], W = PW_WAVES_PER_CU[shape];
    const int64_t m = (int64_t)batch * L.out_h * L.out_w;
    const int64_t items = ((m + 32 * FPs - 1) / (32 * FPs)) * ((L.ncb + FCs - 1) / FCs);
    const int64_t items_cu = (items + budget - 1) / budget;
    const int64_t has_res = L.d.residual_from >= 0 ? 1 : 0;
    if (PW_BLOCK[shape]) {
        // a CU works through its blocks two at a time; what bounds a block is the stream of operand
        // fragments into the CU (1 KiB per 32 channels or pixels of the block and K step)
        const int64_t rounds = (items_cu + W - 1) / W;
        const int64_t frag_bytes = items_cu * L.nsteps * (FCs + FPs) * 1024;
        const int64_t compute = rounds * (C_PWB_BLOCK + has_res * C_PW_RES) + frag_bytes / PWB_BYTES_PER_CYCLE;
        const int64_t bytes = m * L.d.cin * 2 + m * L.d.cout * 2 * (1 + has_res) + (int64_t)L.ncb * L.nsteps * 1024;
        const int64_t mem = bytes / std::min<int64_t>(PW_HBM_BYTES_PER_CYCLE, (int64_t)budget * CU_BYTES_PER_CYCLE);
        return (uint64_t)((C_LAUNCH + std::max(compute, mem)) * PS_PER_CYCLE);
    }
    const int64_t step = std::max(C_PW_STEP[shape], std::min(items_cu, W) * C_PW_STEP_WAVE[shape]);
    const int64_t ks = PW_KSPLIT[shape];
    const int64_t item = C_PW_ITEM + (L.nsteps / ks) * step + (ks > 1 ? C_PW_SK : 0) + has_res * C_PW_RES;
    // ... and never faster than the CU takes in the operand fragments of its items
    const int64_t stream = items_cu * L.nsteps * (FCs + FPs) * 1024 / PW_BYTES_PER_CYCLE;
    const int64_t compute = std::max(((items_cu + W - 1) / W) * item, stream);
    const int64_t bytes = m * L.d.cin * 2 + m * L.d.cout * 2 * (1 + has_res) + (int64_t)L.ncb * L.nsteps * 1024;
    const int64_t mem = bytes / std::min<int64_t>(PW_HBM_BYTES_PER_CYCLE, (int64_t)budget * CU_BYTES_PER_CYCLE);
    return (uint64_t)((C_LAUNCH + std::max(compute, mem)) * PS_PER_CYCLE);
}

// May the planner choose this shape for the layer?  Split-K needs K steps that divide by four; of
// the block forms, 128 x 128 serves layers of more than 64 output channels, 64 x 256 the others.
bool pw_shape_ok(const Layer& L, int shape)
{
    if (PW_KSPLIT[shape] > 1 && (L.nsteps % PW_KSPLIT[shape] != 0 || L.nsteps < 16)) return false;
    if (shape == 3) return L.ncb >= 3;
    if (shape == 4) return L.ncb <= 2;
    return true;
}

// Cheapest of the shapes (ties: the block forms first, then the larger item).
uint64_t pw_cost_ps(const Layer& L, int batch, int budget, int& shape)
{
    static const int order[PW_SHAPES] = {3, 4, 0, 1, 2};
    uint64_t best = 0;
    shape = -1;
    for (int k = 0; k < PW_SHAPES; ++k) {
        const int sh = order[k];
        if (!pw_shape_ok(L, sh)) continue;
        const uint64_t c = pw_shape_cost_ps(L, batch, budget, sh);
        if (shape < 0 || c < best) { best = c; shape = sh; }
    }
    return best;
}

// ---- two 1x1 convolutions into one output: the projection shortcut of a residual block and the
// block's last 1x1 layer, out = act(conv(y) + conv_proj(x)), as one launch of the block pointwise kernel
// whose K loop runs over both operand pairs ----

// layers [first, last] = [projection, last 1x1]: the projection (no activation, read by nothing
// else) is the residual operand of the layer behind it, which reads a tensor from outside
bool pw2_eligible(const dlf_net_s& net, int first, int last, int batch)
{
    if (last != first + 1) return false;
    const Layer& P = net.L[first];
    const Layer& Q = net.L[last];
    if (!pw_eligible(P, batch) || !pw_eligible(Q, batch)) return false;
    if (Q.d.residual_from != first || Q.src >= first || P.d.residual_from >= 0 || P.d.act != DLF_ACT_NONE) return false;
    if (P.out_h != Q.out_h || P.out_w != Q.out_w || P.d.cout != Q.d.cout || Q.d.stride != 1) return false;
    for (size_t k = 0; k < net.L.size(); ++k) {
        if ((int)k != last && net.L[k].d.residual_from == first) return false;
        if (net.L[k].src == first) return false;
    }
    return true;
}

uint64_t pw2_cost_ps(const Layer& P, const Layer& Q, int batch, int budget, int shape)
{
    const int64_t FCs = PW_FC[shape], FPs = PW_FP[shape], W = PW_WAVES_PER_CU[shape];
    const int64_t m = (int64_t)batch * Q.out_h * Q.out_w;
    const int64_t nsteps = P.nsteps + Q.nsteps;
    const int64_t items = ((m + 32 * FPs - 1) / (32 * FPs)) * ((Q.ncb + FCs - 1) / FCs);
    const int64_t items_cu = (items + budget - 1) / budget;
    const int64_t rounds = (items_cu + W - 1) / W;
    const int64_t frag_bytes = items_cu * nsteps * (FCs + FPs) * 1024;
    const int64_t compute = rounds * C_PWB_BLOCK + frag_bytes / PWB_BYTES_PER_CYCLE;
    // a strided projection uses one pixel in stride^2 of its input, but fetches the lines of every
    // second pixel of every second row
    const int64_t in2 = (int64_t)batch * P.in_h * P.in_w * P.d.cin * 2 / P.d.stride;
    const int64_t bytes = m * Q.d.cin * 2 + in2 + m * Q.d.cout * 2 + (int64_t)Q.ncb * nsteps * 1024;
    const int64_t mem = bytes / std::min<int64_t>(PW_HBM_BYTES_PER_CYCLE, (int64_t)budget * CU_BYTES_PER_CYCLE);
    return (uint64_t)((C_LAUNCH + std::max(compute, mem)) * PS_PER_CYCLE);
}

// ---- block 3x3 kernel (one 3x3 stride-1 pad-1 convolution, optionally with its folded 2x2 pool) ----

// Testing hook: mode 0 = the block kernel competes with the fused-group kernel on modelled cost,
// 1 = always where it applies, 2 = never; wc > 0 forces the shape (wc x th x tw).
struct C3Force { int mode, shape, th, tw; };      // shape < 0: not forced
C3Force g_c3_force = {0, -1, 0, 0};
const int C3_WC[DLF_C3_SHAPES] = {2, 2, 1, 1, 2};
const int C3_ACH[DLF_C3_SHAPES] = {32, 64, 32, 64, 32};
const int C3_FP[DLF_C3_SHAPES] = {2, 2, 2, 2, 4};      // 32-pixel blocks of a wave's part

struct C3Cfg { int shape, th, tw, nst, lds_bytes, npxh, na_i, lpw_a; };

bool c3_eligible(const dlf_net_s& net, const std::vector<StageSpec>& specs, int batch)
{
    if (specs.size() != 1 || specs[0].kind != DLF_ST_CONV) return false;
    const Layer& L = net.L[specs[0].layer];
    const dlf_layer_desc& d = L.d;
    if (d.op != DLF_CONV || d.kh != 3 || d.kw != 3 || d.stride != 1 || d.pad != 1) return false;
    if (L.im2col || L.rowfold || (d.cin % 32) != 0 || (d.cout % 8) != 0) return false;
    // the input is read through a buffer resource whose range check supplies the padding: below 2 GiB
    if ((int64_t)batch * L.in_h * L.in_w * L.in_c * 2 >= (int64_t)1 << 31) return false;
    if ((int64_t)batch * L.out_h * L.out_w * L.out_c >= (int64_t)1 << 31) return false;
    return true;
}

// Lays one shape out: wc waves along the channels (64 each), 8 / wc along the pixels (64 each);
// two activation buffers of ACH channels, the rest of LDS (less a spare KiB) a ring of weight stages.
bool c3_build(int pool2, int cin, int shape, int th, int tw, int max_lds, C3Cfg& c)
{
    if (shape < 0 || shape >= DLF_C3_SHAPES) return false;
    const int wc = C3_WC[shape], ach = C3_ACH[shape];
    if (th < 1 || tw < 1 || th * tw > 32 * C3_FP[shape] * (DLF_C3_WAVES / wc) || (cin % ach) != 0) return false;
    if (pool2 && (((th | tw) & 1) != 0)) return false;
    c.shape = shape; c.th = th; c.tw = tw;
    c.npxh = (th + 2) * (tw + 2);
    c.na_i = ceil_div(c.npxh, 512 / ach);
    c.lpw_a = ceil_div(c.na_i, DLF_C3_LOAD_WAVES);
    if (c.lpw_a > DLF_C3_MAX_ACT_LOADS) return false;
    // ... and, behind the spare KiB, the requesting waves' table of halo-pixel offsets (4 bytes per pixel)
    const int act = 2 * c.na_i * 1024, wstage = 9 * 2 * wc * 1024;
    const int tab = (c.lpw_a * DLF_C3_LOAD_WAVES * (512 / ach) * 4 + 255) / 256 * 256;
    c.nst = std::min(4, (max_lds - 1024 - tab - act) / wstage);
    if (c.nst < 2) return false;
    c.lds_bytes = std::max(act + c.nst * wstage + 1024 + tab, (int)DLF_C3_EPI_BYTES);
    return c.lds_bytes <= max_lds;
}

uint64_t c3_cost_ps(const Layer& L, int pool2, int batch, int budget, const C3Cfg& c)
{
    const int wc = C3_WC[c.shape];
    const int64_t tiles = (int64_t)batch * ceil_div(L.out_h, c.th) * ceil_div(L.out_w, c.tw);
    const int64_t items = tiles * ceil_div(L.ncb, 2 * wc);
    const int64_t items_cu = (items + budget - 1) / budget;
    const int64_t stage_bytes = (int64_t)9 * 2 * wc * 1024 + (int64_t)c.npxh * 32;
    int64_t stage = std::max(9 * 2 * C3_FP[c.shape] * MFMA_CYCLES * 2 * C3_MMA_TENTHS / 10, stage_bytes / C3_BYTES_PER_CYCLE);
    if (c.nst == 2) stage += C3_SHALLOW_RING;
    const int64_t has_res = L.d.residual_from >= 0 ? 1 : 0;
    const int64_t kt = L.d.cin / 16;
    const int64_t compute = items_cu * (C_C3_ITEM + (kt < 8 ? C_C3_SHORT_K : 0) + has_res * C_PW_RES + kt * stage);
    const int64_t m = (int64_t)batch * L.out_h * L.out_w;
    const int64_t bytes = m * L.d.cin * 2 + (pool2 ? m / 4 : m) * L.d.cout * 2 * (1 + has_res) + (int64_t)L.ncb * L.nsteps * 1024;
    const int64_t mem = bytes / std::min<int64_t>(PW_HBM_BYTES_PER_CYCLE, (int64_t)budget * CU_BYTES_PER_CYCLE);
    return (uint64_t)((C_LAUNCH + std::max(compute, mem)) * PS_PER_CYCLE);
}

// Cheapest shape (ties: the first in the order of shapes; tile heights, tile widths ascending).
bool c3_choose(const Layer& L, int pool2, int batch, int budget, int max_lds, C3Cfg& best, uint64_t& cost,
               std::vector<std::pair<uint64_t, C3Cfg>>* all = nullptr)
{
    bool found = false;
    for (int shape = 0; shape < DLF_C3_SHAPES; ++shape)
        for (int th : TILE_H) {
            if (th > L.out_h && th != TILE_H[0] && (th - L.out_h) >= 4) continue;
            for (int tw : TILE_W) {
                if (tw > L.out_w && tw != TILE_W[0] && (tw - L.out_w) >= 4) continue;
                C3Cfg c;
                if (!c3_build(pool2, L.d.cin, shape, th, tw, max_lds, c)) continue;
                const uint64_t cc = c3_cost_ps(L, pool2, batch, budget, c);
                if (all) all->push_back(std::make_pair(cc, c));
                if (!found || cc < cost) { found = true; cost = cc; best = c; }
            }
        }
    return found;
}

// ---- streaming depthwise kernel (one depthwise 3x3 layer, pad 1, stride 1 or 2) ----

// Testing hook: 0 = the streaming kernel competes with the fused-group kernel on modelled cost,
// 1 = always where it applies, 2 = never.
int g_dw_mode = 0;

bool dw_eligible(const Layer& L, int batch)
{
    const dlf_layer_desc& d = L.d;
    if (d.op != DLF_DWCONV || d.kh != 3 || d.kw != 3 || d.pad != 1 || (d.stride != 1 && d.stride != 2)) return false;
    if ((d.cin % 8) != 0 || d.residual_from >= 0) return false;
    // byte offsets into the input are formed in 31 bits, element offsets into the output in 32
    if ((int64_t)batch * L.in_h * L.in_w * L.in_c * 2 >= (int64_t)1 << 31) return false;
    if ((int64_t)batch * L.out_h * L.out_w * L.out_c >= (int64_t)1 << 31) return false;
    return true;
}

void dw_fill(const Layer& L, int batch, DlfDwArgs& da)
{
    memset(&da, 0, sizeof da);
    da.w = L.d_w; da.bias = L.d_bias;
    da.in_bytes = (uint32_t)((int64_t)batch * L.in_h * L.in_w * L.in_c * 2);
    da.batch = batch; da.h = L.in_h; da.w_ = L.in_w; da.c = L.d.cin; da.cpad = L.cin_pad;
    da.oh = L.out_h; da.ow = L.out_w; da.stride = L.d.stride; da.act = L.d.act;
    da.cg = L.d.cin / 8;
    da.rowv = L.out_w * da.cg;
    da.nxr = ceil_div(da.rowv, 64);
    da.nstrips = ceil_div(L.out_h, L.d.stride == 1 ? DLF_DW_ROWS1 : DLF_DW_ROWS2);
    da.nitems = batch * da.nstrips * da.nxr;
}

uint64_t dw_cost_ps(const Layer& L, int batch, int budget, const DlfDwArgs& da)
{
    const int64_t rows = std::min<int64_t>(L.out_h, L.d.stride == 1 ? DLF_DW_ROWS1 : DLF_DW_ROWS2);
    // the items of a CU are dealt to its four SIMDs; a SIMD's waves share its instruction issue
    const int64_t items_simd = ((int64_t)da.nitems + (int64_t)budget * 4 - 1) / ((int64_t)budget * 4);
    const int64_t compute = C_LAT + items_simd * (C_DW_ITEM / (DW_WAVES_PER_CU / 4) + rows * C_DW_ROW);
    const int64_t bytes = (int64_t)da.in_bytes + (int64_t)batch * L.out_h * L.out_w * L.out_c * 2 + (int64_t)L.cin_pad * 22;
    const int64_t mem = bytes / std::min<int64_t>(DW_HBM_BYTES_PER_CYCLE, (int64_t)budget * DW_CU_BYTES_PER_CYCLE);
    return (uint64_t)((C_LAUNCH + std::max(compute, mem)) * PS_PER_CYCLE);
}

// ---- fused depthwise 3x3 + 1x1 kernel (a depthwise layer and the pointwise layer that reads it) ----

bool dwpw_eligible(const dlf_net_s& net, int first, int last, int batch)
{
    if (last != first + 1) return false;
    const Layer& D = net.L[first];
    const Layer& P = net.L[last];
    if (!dw_eligible(D, batch) || (D.d.cin % 32) != 0) return false;
    const dlf_layer_desc& p = P.d;
    if (p.op != DLF_CONV || p.kh != 1 || p.kw != 1 || p.pad != 0 || p.stride != 1 || P.src != first) return false;
    if (p.residual_from >= 0 || (p.cout % 8) != 0 || P.nsteps != D.d.cin / 16) return false;
    if ((int64_t)batch * P.out_h * P.out_w * P.out_c >= (int64_t)1 << 31) return false;
    if (DLF_DWPW_LDS_BYTES(D.d.cin, 4) > 64 * 1024) return false;
    // the depthwise output exists only in registers: nothing else may read it
    for (size_t k = 0; k < net.L.size(); ++k) {
        if (net.L[k].d.residual_from == first) return false;
        if ((int)k != last && net.L[k].src == first) return false;
    }
    return true;
}

void dwpw_fill(const Layer& D, const Layer& P, int batch, int nb, DlfDwPwArgs& dp)
{
    memset(&dp, 0, sizeof dp);
    dp.wdw = D.d_w; dp.bdw = D.d_bias; dp.wpw = P.d_w; dp.bpw = P.d_bias;
    dp.in_bytes = (uint32_t)((int64_t)batch * D.in_h * D.in_w * D.in_c * 2);
    dp.batch = batch; dp.h = D.in_h; dp.w_ = D.in_w; dp.c = D.d.cin;
    dp.oh = D.out_h; dp.ow = D.out_w; dp.stride = D.d.stride; dp.act_dw = D.d.act; dp.act_pw = P.d.act;
    dp.cout = P.d.cout; dp.ncb = P.ncb; dp.nsteps = P.nsteps;
    dp.m = batch * D.out_h * D.out_w;
    dp.n_pg = ceil_div(dp.m, 32);
    dp.n_cg = ceil_div(P.ncb, nb);
    dp.nitems = dp.n_pg * dp.n_cg;
}

uint64_t dwpw_cost_ps(const Layer& D, const Layer& P, int batch, int budget, int nb)
{
    const int64_t m = (int64_t)batch * D.out_h * D.out_w;
    const int64_t items = ((m + 31) / 32) * ceil_div(P.ncb, nb);
    const int64_t items_simd = (items + (int64_t)budget * 4 - 1) / ((int64_t)budget * 4);
    const int64_t items_cu = (items + budget - 1) / budget;
    const int64_t valu = items_simd * (C_DWPW_ITEM / 2 + P.nsteps * C_DWPW_STEP);
    const int64_t mfma = items_simd * P.nsteps * nb * MFMA_CYCLES;
    const int64_t loads = items_cu * P.nsteps * (9 + nb) * C_DWPW_LOAD;
    const int64_t compute = C_LAT + std::max(std::max(valu, mfma), loads);
    const int64_t bytes = (int64_t)batch * D.in_h * D.in_w * D.in_c * 2 + m * P.d.cout * 2 +
                          (int64_t)P.ncb * P.nsteps * 1024 + (int64_t)D.d.cin * 22;
    const int64_t mem = bytes / std::min<int64_t>(DW_HBM_BYTES_PER_CYCLE, (int64_t)budget * DW_CU_BYTES_PER_CYCLE);
    return (uint64_t)((C_LAUNCH + std::max(compute, mem)) * PS_PER_CYCLE);
}

// ---- depthwise + 1x1 tile kernel ----

bool dwt_eligible(const dlf_net_s& net, int first, int last, int batch)
{
    if (!dwpw_eligible(net, first, last, batch)) return false;
    const int cg = net.L[first].d.cin / 8;
    return cg >= 4 && cg <= 64 && (cg & (cg - 1)) == 0;
}

// One tile shape: wx x wy waves, rw rows per wave.
bool dwt_build(const Layer& D, const Layer& P, int batch, int wx, int rw, int max_lds, DlfDwtArgs& dt)
{
    memset(&dt, 0, sizeof dt);
    dt.cg = D.d.cin / 8;
    dt.pxw = 64 / dt.cg;
    dt.wx = wx; dt.wy = DLF_DWT_WAVES / wx; dt.rw = rw;
    dt.th = dt.wy * rw; dt.tw = wx * dt.pxw;
    dt.tp = dt.th * dt.tw;
    if (dt.tp > 256 || rw < 1) return false;
    if ((int)DLF_DWT_LDS_BYTES(dt.tp, D.d.cin) > max_lds) return false;
    dt.npb = ceil_div(dt.tp, 32);
    dt.npg = ceil_div(dt.npb, 4);
    dt.wdw = D.d_w; dt.bdw = D.d_bias; dt.wpw = P.d_w; dt.bpw = P.d_bias;
    dt.in_bytes = (uint32_t)((int64_t)batch * D.in_h * D.in_w * D.in_c * 2);
    dt.batch = batch; dt.h = D.in_h; dt.w_ = D.in_w; dt.c = D.d.cin;
    dt.oh = D.out_h; dt.ow = D.out_w; dt.stride = D.d.stride; dt.act_dw = D.d.act; dt.act_pw = P.d.act;
    dt.cout = P.d.cout; dt.ncb = P.ncb; dt.nsteps = P.nsteps;
    dt.tiles_y = ceil_div(D.out_h, dt.th); dt.tiles_x = ceil_div(D.out_w, dt.tw);
    dt.ntiles = batch * dt.tiles_y * dt.tiles_x;
    return true;
}

uint64_t dwt_cost_ps(const Layer& D, const Layer& P, int batch, int budget, const DlfDwtArgs& dt, int& occ)
{
    const int lds = (int)DLF_DWT_LDS_BYTES(dt.tp, dt.c);
    occ = std::max(1, std::min(2, (160 * 1024) / lds));
    const int64_t units_wave = ceil_div(dt.ncb * dt.npg, DLF_DWT_WAVES);
    const int64_t nb = std::min(4, dt.npb);
    const int64_t p1 = (int64_t)dt.rw * C_DWT_ROW;
    const int64_t p2 = units_wave * (C_DWT_UNIT + dt.nsteps * std::max<int64_t>(nb, 2) * C_DWT_STEP + nb * C_DWT_EPI);
    const int64_t tile = C_DWT_TILE + p1 + p2;
    const int64_t tiles_cu = ((int64_t)dt.ntiles + budget - 1) / budget;
    const int64_t conc = std::min<int64_t>(occ, tiles_cu);
    // ... but not the rate at which the CU takes in the weight fragments every tile streams anew
    const int64_t intake = tiles_cu * ((int64_t)dt.ncb * dt.npg * dt.nsteps * 1024) / PW_BYTES_PER_CYCLE;
    const int64_t compute = C_LAT + std::max(tiles_cu * tile / conc, intake);
    const int64_t m = (int64_t)batch * D.out_h * D.out_w;
    const int64_t bytes = (int64_t)batch * D.in_h * D.in_w * D.in_c * 2 + m * P.d.cout * 2 +
                          (int64_t)P.ncb * P.nsteps * 1024 + (int64_t)D.d.cin * 22;
    const int64_t mem = bytes / std::min<int64_t>(DW_HBM_BYTES_PER_CYCLE, (int64_t)budget * DW_CU_BYTES_PER_CYCLE);
    return (uint64_t)((C_LAUNCH + std::max(compute, mem)) * PS_PER_CYCLE);
}

const int DWT_RW[] = {1, 2, 4, 7, 8, 14, 16};

// Cheapest tile shape (ties: the first in the order waves along x 4, 2, 1; rows ascending).
bool dwt_choose(const Layer& D, const Layer& P, int batch, int budget, int max_lds, DlfDwtArgs& best,
                uint64_t& cost, int& occ)
{
    bool found = false;
    // tiles that overshoot the map by a whole wave's share are skipped, unless a map is so small that
    // every shape does
    for (int pass = 0; pass < 2 && !found; ++pass)
        for (int wx = 4; wx >= 1; wx /= 2)
            for (int rw : DWT_RW) {
                DlfDwtArgs dt;
                if (!dwt_build(D, P, batch, wx, rw, max_lds, dt)) continue;
                if (pass == 0 && dt.th - D.out_h >= rw && dt.wy > 1) continue;
                if (pass == 0 && dt.tw - D.out_w >= dt.pxw && wx > 1) continue;
                int o = 1;
                const uint64_t c = dwt_cost_ps(D, P, batch, budget, dt, o);
                if (!found || c < cost) { found = true; cost = c; best = dt; occ = o; }
            }
    return found;
}

// Testing hook of the tile kernel: wx > 0 forces its shape.
struct DwtForce { int wx, rw; };
DwtForce g_dwt_force = {0, 0};

// ---- 3x3 kernel for maps of many channels and few pixels ----

bool c3s_cin_ok(int cin) { return cin == 256 || cin == 512 || cin == 1024 || cin == 2048; }

bool c3s_eligible(const dlf_net_s& net, const std::vector<StageSpec>& specs, int batch)
{
    if (specs.size() != 1 || specs[0].kind != DLF_ST_CONV || specs[0].pool2) return false;
    const Layer& L = net.L[specs[0].layer];
    const dlf_layer_desc& d = L.d;
    if (d.op != DLF_CONV || d.kh != 3 || d.kw != 3 || (d.stride != 1 && d.stride != 2) || d.pad != 1) return false;
    if (L.im2col || L.rowfold || !c3s_cin_ok(d.cin) || (d.cout % 8) != 0) return false;
    // the input is read through a buffer resource whose range check supplies the padding: below 2 GiB
    if ((int64_t)batch * L.in_h * L.in_w * L.in_c * 2 >= (int64_t)1 << 31) return false;
    if ((int64_t)batch * L.out_h * L.out_w * L.out_c >= (int64_t)1 << 31) return false;
    return true;
}

// The same kernel takes 1x1 layers (stride 1, no residual) of those channel counts.
bool c3s_pw_eligible(const Layer& L, int batch)
{
    if (!pw_eligible(L, batch) || L.d.stride != 1 || L.d.residual_from >= 0) return false;
    if ((int64_t)batch * L.in_h * L.in_w * L.in_c * 2 >= (int64_t)1 << 31) return false;
    return c3s_cin_ok(L.d.cin);
}

// One configuration: ksplit waves per channel block, the map cut into `rows` x `cols` equal tiles
// (0: as few as tiles of at most 8 x 8 output pixels allow).
// pool2 (quantised 3x3 form only): the 2x2 max pool behind the layer folded in, which needs tiles 8 pixels
// wide and of even height.
bool c3s_build(const Layer& L, int batch, int ksplit, int rows, int cols, int max_lds, DlfC3sArgs& cs, int pool2 = 0)
{
    memset(&cs, 0, sizeof cs);
    cs.taps = L.d.kh * L.d.kw;
    cs.stride = L.d.stride;
    const int halo = cs.taps == 9 ? 1 : 0, chunks = L.d.cin / (cs.taps == 9 ? 32 : 128);
    if ((cs.taps != 9 && cs.taps != 1) || (ksplit != 1 && ksplit != 2 && ksplit != 4) || (chunks % ksplit) != 0) return false;
    if (rows <= 0) rows = ceil_div(L.out_h, 8);
    if (cols <= 0) cols = ceil_div(L.out_w, 8);
    cs.th = ceil_div(L.out_h, rows);
    cs.tw = ceil_div(L.out_w, cols);
    if (pool2) {
        if (L.d.kh != 3 || L.d.stride != 1 || L.out_h < 2 || L.out_w < 2) return false;
        cs.th = round_up(cs.th, 2);
        cs.tw = 8;
        cs.pool2 = 1;
    }
    if (cs.th > 8 || cs.tw > 8) return false;
    cs.tp = cs.th * cs.tw;
    cs.rw = (cs.tw - 1) * cs.stride + 1 + 2 * halo;
    cs.rp = ((cs.th - 1) * cs.stride + 1 + 2 * halo) * cs.rw;
    if ((int)DLF_C3S_LDS_BYTES(cs.rp, L.d.cin) > max_lds) return false;
    cs.w = L.d_w; cs.bias = L.d_bias;
    cs.in_bytes = (uint32_t)((int64_t)batch * L.in_h * L.in_w * L.in_c * 2);
    cs.batch = batch; cs.h = L.in_h; cs.w_ = L.in_w; cs.oh = L.out_h; cs.ow = L.out_w;
    cs.cin = L.d.cin; cs.cout = L.d.cout;
    cs.ncb = L.ncb; cs.nsteps = L.nsteps; cs.act = L.d.act;
    cs.tiles_y = ceil_div(L.out_h, cs.th); cs.tiles_x = ceil_div(L.out_w, cs.tw);
    cs.ntiles = batch * cs.tiles_y * cs.tiles_x;
    cs.ksplit = ksplit;
    cs.nsl = ceil_div(L.ncb, DLF_C3S_WAVES / ksplit);
    // weights that do not fit an XCD's L2: let every XCD keep to one slice of them
    cs.slice_major = ((int64_t)L.ncb * L.nsteps * 1024 > C_C3S_BIG_BYTES && (cs.nsl == 2 || cs.nsl == 4 || cs.nsl == 8)) ? 1 : 0;
    return true;
}

uint64_t c3s_cost_ps(const Layer& L, int batch, int budget, const DlfC3sArgs& cs)
{
    const int64_t wbytes = (int64_t)L.ncb * L.nsteps * 1024;
    const int64_t nitems = (int64_t)cs.ntiles * cs.nsl;
    const int64_t rounds = (nitems + budget - 1) / budget;
    const int64_t item = C_C3S_ITEM + (rounds > 1 ? C_C3S_NEXT : 0) + (int64_t)cs.rp * cs.cin * 2 / DWS_BYTES_PER_CYCLE +
                         (int64_t)(cs.nsteps / cs.ksplit) * (wbytes > C_C3S_BIG_BYTES ? C_C3S_STEP_BIG : C_C3S_STEP) *
                             (cs.tp > 32 ? 4 : 3) / 4 +        // one pixel block: half the MFMAs, the same weights

                         (cs.ksplit > 1 ? C_C3S_RED : 0) + C_C3S_EPI + (L.d.residual_from >= 0 ? C_PW_RES : 0);
    const int64_t compute = C_LAT + rounds * item;
    const int64_t m = (int64_t)batch * L.out_h * L.out_w;
    const int64_t bytes = (int64_t)batch * L.in_h * L.in_w * L.d.cin * 2 + m * L.d.cout * 2 * (L.d.residual_from >= 0 ? 2 : 1) +
                          (int64_t)L.ncb * L.nsteps * 1024;
    const int64_t mem = bytes / std::min<int64_t>(PW_HBM_BYTES_PER_CYCLE, (int64_t)budget * CU_BYTES_PER_CYCLE);
    return (uint64_t)((C_LAUNCH + std::max(compute, mem)) * PS_PER_CYCLE);
}

// Cheapest split of K over the waves and cut of the map (ties: the smaller split, the fewer tiles):
// the largest tiles first, then one more row or column of tiles while a region does not fit LDS.
bool c3s_choose(const Layer& L, int batch, int budget, int max_lds, DlfC3sArgs& best, uint64_t& cost, int pool2 = 0)
{
    bool found = false;
    const int r0 = ceil_div(L.out_h, 8), c0 = ceil_div(L.out_w, 8);
    for (int extra = 0; extra <= 6 && !found; ++extra)
        for (int er = 0; er <= extra; ++er)
            for (int ks = 1; ks <= 4; ks *= 2) {
                DlfC3sArgs cs;
                if (!c3s_build(L, batch, ks, r0 + er, c0 + extra - er, max_lds, cs, pool2)) continue;
                const uint64_t c = c3s_cost_ps(L, batch, budget, cs);
                if (!found || c < cost) { found = true; cost = c; best = cs; }
            }
    return found;
}

// ---- fused 3x3 -> 1x1 (+ residual) kernel for maps with no more tiles than CUs ----

bool c3pw_eligible(const dlf_net_s& net, const std::vector<StageSpec>& specs, int batch)
{
    if (specs.size() != 2 || specs[0].kind != DLF_ST_CONV || specs[1].kind != DLF_ST_CONV || specs[0].pool2 || specs[1].pool2)
        return false;
    const Layer& A = net.L[specs[0].layer];
    const Layer& P = net.L[specs[1].layer];
    const dlf_layer_desc& a = A.d;
    const dlf_layer_desc& p = P.d;
    if (a.kh != 3 || a.kw != 3 || a.stride != 1 || a.pad != 1 || A.im2col || A.rowfold || a.residual_from >= 0) return false;
    if ((a.cin != 64 && a.cin != 128 && a.cin != 256) || a.cout != a.cin) return false;
    if (p.kh != 1 || p.kw != 1 || p.stride != 1 || p.pad != 0 || P.im2col || P.rowfold || (p.cout % 8) != 0) return false;
    if ((int64_t)batch * A.in_h * A.in_w * a.cin * 2 >= (int64_t)1 << 31) return false;
    if ((int64_t)batch * P.out_h * P.out_w * p.cout * 2 >= (int64_t)1 << 31) return false;
    return true;
}

// One configuration: the map cut into rows x cols equal tiles.
bool c3pw_build(const Layer& A, const Layer& P, int batch, int rows, int cols, int max_lds, DlfC3PwArgs& cp)
{
    memset(&cp, 0, sizeof cp);
    if (rows <= 0 || cols <= 0) return false;
    cp.th = ceil_div(A.out_h, rows);
    cp.tw = ceil_div(A.out_w, cols);
    if (cp.th > 8 || cp.tw > 16 || cp.th * cp.tw > 128) return false;
    cp.tp = cp.th * cp.tw;
    cp.rw = cp.tw + 2;
    cp.rp = (cp.th + 2) * cp.rw;
    // 64 channels: items of four waves, two of them to a CU
    if ((int)DLF_C3PW_LDS_BYTES(cp.rp, cp.tp, A.d.cin, P.d.residual_from >= 0) > (A.d.cin == 64 ? std::min(max_lds, 80 * 1024) : max_lds))
        return false;
    cp.w1 = A.d_w; cp.b1 = A.d_bias; cp.w2 = P.d_w; cp.b2 = P.d_bias;
    cp.in_bytes = (uint32_t)((int64_t)batch * A.in_h * A.in_w * A.in_c * 2);
    cp.res_bytes = (uint32_t)((int64_t)batch * P.out_h * P.out_w * P.d.cout * 2);
    cp.batch = batch; cp.h = A.in_h; cp.w_ = A.in_w; cp.c = A.d.cin; cp.cout = P.d.cout;
    cp.ncb2 = P.ncb; cp.act1 = A.d.act; cp.act2 = P.d.act;
    cp.tiles_y = ceil_div(A.out_h, cp.th); cp.tiles_x = ceil_div(A.out_w, cp.tw);
    cp.ntiles = batch * cp.tiles_y * cp.tiles_x;
    cp.nsl = ceil_div(P.ncb, 2 * DLF_C3PW_WAVES(A.d.cin));
    return true;
}

// Workgroups of the kernel a CU holds: one of eight waves; of four waves as many as LDS and
// registers take (two with four 32-pixel blocks per wave, else three).
int c3pw_per_cu(const DlfC3PwArgs& cp, bool res)
{
    if (cp.c != 64) return 1;
    const int lds = (int)DLF_C3PW_LDS_BYTES(cp.rp, cp.tp, cp.c, res);
    return std::max(1, std::min(cp.tp > 64 ? 2 : 3, (160 * 1024) / lds));
}

uint64_t c3pw_cost_ps(const Layer& A, const Layer& P, int batch, int budget, const DlfC3PwArgs& cp)
{
    const int waves = DLF_C3PW_WAVES(cp.c), per_cu = c3pw_per_cu(cp, P.d.residual_from >= 0);
    const int64_t nitems = (int64_t)cp.ntiles * cp.nsl;
    const int64_t slots = (int64_t)budget * per_cu;
    const int64_t rounds = (nitems + slots - 1) / slots;
    const int64_t fp = cp.tp > 64 ? 4 : 2, ncb1 = cp.c / 32;
    const bool res = P.d.residual_from >= 0;
    const int64_t intake = (int64_t)cp.rp * cp.c * 2 + (res && ncb1 == waves ? (int64_t)cp.tp * 1024 : 0);
    const int64_t mma1 = (int64_t)A.nsteps * std::max(fp * C_C3PW_MMA * (ncb1 > 4 ? 2 : 1), C_C3PW_STEP);
    const int64_t pbs = ceil_div(cp.tp, 32);
    const int64_t cb_item = std::min<int64_t>(P.ncb, 2 * waves);
    const int64_t mma2 = pbs * P.nsteps * ceil_div(cb_item, 4) * C_C3PW_MMA;     // the waves of a SIMD, two blocks each
    const int64_t stores = std::min<int64_t>(nitems, slots) * cp.tp * cb_item * 64 / C3PW_STORE_BYTES_PER_CYCLE;
    const int64_t item = C_C3PW_ITEM + intake / C3PW_BYTES_PER_CYCLE + mma1 + ncb1 * C_C3PW_MID + C_C3PW_SECOND +
                         std::max(mma2, stores);
    // one workgroup per CU: a further item of a CU repeats every phase behind the first; two per
    // CU: their phases interleave, and the rounds cost what the chip's memory takes for them
    const int64_t compute = C_LAT + (per_cu == 1 ? rounds * item + (rounds > 1 ? (rounds - 1) * C_C3S_NEXT : 0)
                                                 : item + (rounds - 1) * item * C3PW_OVERLAP_PCT / 100);
    const int64_t m = (int64_t)batch * P.out_h * P.out_w;
    const int64_t bytes = (int64_t)batch * A.in_h * A.in_w * cp.c * 2 + m * cp.cout * 2 * (res ? 2 : 1) +
                          ((int64_t)A.ncb * A.nsteps + (int64_t)P.ncb * P.nsteps) * 1024;
    int64_t mem = bytes / std::min<int64_t>(PW_HBM_BYTES_PER_CYCLE, (int64_t)budget * CU_BYTES_PER_CYCLE);
    if (per_cu > 1) {
        // measured on the 56 x 56 pair of ResNet-50 (tiles 7x8, 4x14: 31.6 us; 7x14: 32.9; 8x8: 36.7;
        // 8x12: 36.9): three workgroups per CU hold the memory rate, two lose some of it, and
        // pixels of tiles that hang over the map's edge cost like real ones
        mem = mem * (per_cu >= 3 ? 100 : 104) / 100 * ((int64_t)cp.ntiles * cp.tp) / m;
    }
    return (uint64_t)((C_LAUNCH + std::max(compute, mem)) * PS_PER_CYCLE);
}

// Cheapest cut of the map (ties: the fewer tiles).
bool c3pw_choose(const Layer& A, const Layer& P, int batch, int budget, int max_lds, DlfC3PwArgs& best, uint64_t& cost)
{
    bool found = false;
    const int r0 = ceil_div(A.out_h, 8), c0 = ceil_div(A.out_w, 16);
    for (int rows = r0; rows <= r0 + 3; ++rows)
        for (int cols = c0; cols <= c0 + 3; ++cols) {
            DlfC3PwArgs cp;
            if (!c3pw_build(A, P, batch, rows, cols, max_lds, cp)) continue;
            const uint64_t c = c3pw_cost_ps(A, P, batch, budget, cp);
            if (!found || c < cost) { found = true; cost = c; best = cp; }
        }
    return found;
}

// ---- a whole bottleneck block (1x1 -> 3x3 -> 1x1, identity shortcut or none) as one group ----

// (two stages: the pair 1x1 -> 3x3, which the kernel runs without its last layer)
bool bneck_eligible(const dlf_net_s& net, const std::vector<StageSpec>& specs, int batch)
{
    if (specs.size() != 3 && specs.size() != 2) return false;
    for (const StageSpec& sp : specs)
        if (sp.kind != DLF_ST_CONV || sp.pool2) return false;
    const Layer& A = net.L[specs[0].layer];
    const Layer& B = net.L[specs[1].layer];
    const dlf_layer_desc& a = A.d;
    const dlf_layer_desc& b = B.d;
    if (A.im2col || A.rowfold || B.im2col || B.rowfold) return false;
    if (a.kh != 1 || a.kw != 1 || a.stride != 1 || a.pad != 0 || a.residual_from >= 0) return false;
    if ((a.cin != 64 && a.cin != 128 && a.cin != 256 && a.cin != 512) || a.cout != 64) return false;
    if (b.kh != 3 || b.kw != 3 || b.stride != 1 || b.pad != 1 || b.cin != 64 || b.cout != 64 || b.residual_from >= 0) return false;
    if ((int64_t)batch * A.in_h * A.in_w * a.cin * 2 >= (int64_t)1 << 31) return false;
    if (specs.size() == 2) return true;
    if (a.cin == 64) return false;
    const Layer& P = net.L[specs[2].layer];
    const dlf_layer_desc& p = P.d;
    if (P.im2col || P.rowfold) return false;
    if (p.kh != 1 || p.kw != 1 || p.stride != 1 || p.pad != 0 || p.cin != 64 || (p.cout % 8) != 0) return false;
    // the shortcut, if any, is the block's own input
    if (p.residual_from >= 0 && (p.residual_from != A.src || p.cout != a.cin)) return false;
    if ((int64_t)batch * P.out_h * P.out_w * p.cout * 2 >= (int64_t)1 << 31) return false;
    return true;
}

// One configuration: the map cut into rows x cols equal tiles of at most 64 pixels.  P is the last
// layer, or the second one again where there are only two.
bool bneck_build(const Layer& A, const Layer& B, const Layer& P, int batch, int rows, int cols, int max_lds, DlfBnArgs& bn)
{
    memset(&bn, 0, sizeof bn);
    if (rows <= 0 || cols <= 0) return false;
    bn.th = ceil_div(A.out_h, rows);
    bn.tw = ceil_div(A.out_w, cols);
    if (bn.th > 8 || bn.tw > 16 || bn.th * bn.tw > 64) return false;
    bn.tp = bn.th * bn.tw;
    bn.rw = bn.tw + 2;
    bn.rp = (bn.th + 2) * bn.rw;
    if ((int)DLF_BN_LDS_BYTES(bn.rp, bn.tp, A.d.cin) > std::min(max_lds, 80 * 1024)) return false;   // two to a CU
    const bool two = &P == &B;
    bn.w0 = A.d_w; bn.b0 = A.d_bias; bn.w1 = B.d_w; bn.b1 = B.d_bias; bn.w2 = two ? nullptr : P.d_w; bn.b2 = two ? nullptr : P.d_bias;
    bn.in_bytes = (uint32_t)((int64_t)batch * A.in_h * A.in_w * A.in_c * 2);
    bn.batch = batch; bn.h = A.in_h; bn.w_ = A.in_w; bn.cin0 = A.d.cin; bn.cout = P.d.cout;
    bn.ncb2 = two ? 0 : P.ncb; bn.act0 = A.d.act; bn.act1 = B.d.act; bn.act2 = P.d.act;
    bn.identity = !two && P.d.residual_from >= 0 ? 1 : 0;
    bn.tiles_y = ceil_div(A.out_h, bn.th); bn.tiles_x = ceil_div(A.out_w, bn.tw);
    bn.ntiles = batch * bn.tiles_y * bn.tiles_x;
    bn.nsl = two ? 1 : ceil_div(P.ncb, 2 * DLF_BN_WAVES);
    return true;
}

// Workgroups a CU holds: two or three, as LDS allows (182 - 256 registers for four waves: three fit).
int bneck_per_cu(const DlfBnArgs& bn)
{
    return std::max(1, std::min(bn.cin0 == 512 ? 2 : 3, (160 * 1024) / (int)DLF_BN_LDS_BYTES(bn.rp, bn.tp, bn.cin0)));
}

// An item is a chain of waits (region, first layer with one accumulator per wave, the 3x3 ring, the
// transposes of the last layer) that two workgroups per CU do not hide: C_BN_ITEM + C_BN_PIXEL per
// tile pixel, half of it where the chip is not full; the items of a CU's two places follow one
// another.  Fitted to seven forced tile shapes of ResNet-50's 56 x 56 block at batch 32 (49 - 72 us)
// and two at batch 1 (8.3, 10.1 us): modelled / measured 0.97 - 1.05.
uint64_t bneck_cost_ps(const Layer& A, const Layer& B, const Layer& P, int batch, int budget, const DlfBnArgs& bn)
{
    const int64_t nitems = (int64_t)bn.ntiles * bn.nsl;
    // (a third workgroup on a CU, where LDS has room for one, does not shorten the chains: priced as two)
    const int64_t slots = (int64_t)budget * 2;
    const bool two = bn.ncb2 == 0;
    int64_t item = C_BN_ITEM + C_BN_PIXEL * bn.tp + (bn.cin0 - 256) * C_BN_CHANNEL / 16 - (two ? C_BN_LAST : 0);
    if (nitems <= budget) item /= 2;
    const int64_t compute = nitems <= slots ? item : item * nitems / slots;
    const int64_t m = (int64_t)batch * P.out_h * P.out_w;
    const int64_t bytes = (int64_t)bn.ntiles * bn.rp * bn.cin0 * 2 + m * bn.cout * 2 +
                          ((int64_t)A.ncb * A.nsteps + (int64_t)B.ncb * B.nsteps + (two ? 0 : (int64_t)P.ncb * P.nsteps)) * 1024;
    const int64_t mem = bytes / std::min<int64_t>(PW_HBM_BYTES_PER_CYCLE, (int64_t)budget * CU_BYTES_PER_CYCLE);
    return (uint64_t)((C_LAUNCH + std::max(compute, mem)) * PS_PER_CYCLE);
}

bool bneck_choose(const Layer& A, const Layer& B, const Layer& P, int batch, int budget, int max_lds, DlfBnArgs& best, uint64_t& cost)
{
    bool found = false;
    const int r0 = ceil_div(A.out_h, 8), c0 = ceil_div(A.out_w, 16);
    for (int rows = r0; rows <= r0 + 8; ++rows)
        for (int cols = c0; cols <= c0 + 8; ++cols) {
            DlfBnArgs bn;
            if (!bneck_build(A, B, P, batch, rows, cols, max_lds, bn)) continue;
            const uint64_t c = bneck_cost_ps(A, B, P, batch, budget, bn);
            if (!found || c < cost) { found = true; cost = c; best = bn; }
        }
    return found;
}

// ---- depthwise + 1x1 kernel for maps of many channels and few pixels ----

bool dws_eligible(const dlf_net_s& net, int first, int last, int batch)
{
    if (!dwpw_eligible(net, first, last, batch)) return false;
    return (net.L[first].d.cin % 256) == 0;
}

// One configuration: kh channels per pass, cbw channel blocks per wave.
bool dws_build(const Layer& D, const Layer& P, int batch, int kh, int cbw, int max_lds, DlfDwsArgs& ds)
{
    memset(&ds, 0, sizeof ds);
    const int c = D.d.cin, s = D.d.stride;
    if ((kh != 256 && kh != 512) || (c % kh) != 0 || (cbw != 1 && cbw != 2)) return false;
    ds.kh = kh; ds.nkh = c / kh;
    // the map is cut into equal tiles of at most 8 x 8 output pixels
    ds.th = ceil_div(D.out_h, ceil_div(D.out_h, 8));
    ds.tw = ceil_div(D.out_w, ceil_div(D.out_w, 8));
    ds.tp = ds.th * ds.tw;
    ds.rh = (ds.th - 1) * s + 3; ds.rw = (ds.tw - 1) * s + 3; ds.rp = ds.rh * ds.rw;
    // all passes' regions in LDS where they fit (and the kernel's counted waits reach), else one
    ds.nbuf = ds.nkh;
    if ((int)DLF_DWS_LDS_BYTES(ds.rp, ds.tp, kh, cbw, ds.nbuf) > max_lds ||
        (ds.nbuf - 1) * ceil_div((int)(DLF_DWS_IN_BYTES(ds.rp, kh) / 1024), DLF_DWS_WAVES) + 16 + 11 > 48)
        ds.nbuf = 1;
    if ((int)DLF_DWS_LDS_BYTES(ds.rp, ds.tp, kh, cbw, ds.nbuf) > max_lds) return false;
    ds.wdw = D.d_w; ds.bdw = D.d_bias; ds.wpw = P.d_w; ds.bpw = P.d_bias;
    ds.in_bytes = (uint32_t)((int64_t)batch * D.in_h * D.in_w * D.in_c * 2);
    ds.batch = batch; ds.h = D.in_h; ds.w_ = D.in_w; ds.c = c;
    ds.oh = D.out_h; ds.ow = D.out_w; ds.stride = s; ds.act_dw = D.d.act; ds.act_pw = P.d.act;
    ds.cout = P.d.cout; ds.ncb = P.ncb; ds.nsteps = P.nsteps;
    ds.tiles_y = ceil_div(D.out_h, ds.th); ds.tiles_x = ceil_div(D.out_w, ds.tw);
    ds.ntiles = batch * ds.tiles_y * ds.tiles_x;
    ds.cbw = cbw;
    ds.nsl = ceil_div(P.ncb, DLF_DWS_WAVES * cbw);
    return true;
}

uint64_t dws_cost_ps(const Layer& D, const Layer& P, int batch, int budget, const DlfDwsArgs& ds)
{
    const int ppi = ds.kh == 512 ? 1 : 2;
    const int64_t steps = (int64_t)ds.nkh * ceil_div(ds.tp, DLF_DWS_WAVES * ppi);
    const int64_t dw = steps * C_DWS_STEP;
    const int64_t mma = (int64_t)ds.nsteps * ds.cbw * C_DWS_MMA;
    const int64_t blocks = std::min(ds.ncb, DLF_DWS_WAVES * ds.cbw);
    const int64_t intake = (blocks * ds.nsteps * 1024) / DWS_BYTES_PER_CYCLE;
    // a region that is not resident is waited for: a trip to memory per pass beyond the first
    const int64_t exposed = ds.nbuf == ds.nkh ? 0 : (int64_t)(ds.nkh - 1) * C_DWS_REGION;
    const int64_t item = C_DWS_ITEM + (int64_t)ds.rp * ds.c * 2 / DWS_BYTES_PER_CYCLE + exposed + dw + std::max(mma, intake) +
                         (int64_t)ds.cbw * C_DWS_EPI;
    const int64_t nitems = (int64_t)ds.ntiles * ds.nsl;
    const int64_t compute = C_LAT + ((nitems + budget - 1) / budget) * item;
    const int64_t m = (int64_t)batch * D.out_h * D.out_w;
    const int64_t bytes = (int64_t)batch * D.in_h * D.in_w * D.in_c * 2 + m * P.d.cout * 2 +
                          (int64_t)P.ncb * P.nsteps * 1024 + (int64_t)D.d.cin * 22;
    const int64_t mem = bytes / std::min<int64_t>(DW_HBM_BYTES_PER_CYCLE, (int64_t)budget * DW_CU_BYTES_PER_CYCLE);
    return (uint64_t)((C_LAUNCH + std::max(compute, mem)) * PS_PER_CYCLE);
}

// Cheapest configuration (ties: 512 channels per pass before 256, two channel blocks per wave before one).
bool dws_choose(const Layer& D, const Layer& P, int batch, int budget, int max_lds, DlfDwsArgs& best, uint64_t& cost)
{
    bool found = false;
    for (int kh = 512; kh >= 256; kh /= 2)
        for (int cbw = 2; cbw >= 1; --cbw) {
            DlfDwsArgs ds;
            if (cbw == 2 && P.ncb <= DLF_DWS_WAVES) continue;      // half the waves would have no channel block
            if (!dws_build(D, P, batch, kh, cbw, max_lds, ds)) continue;
            const uint64_t c = dws_cost_ps(D, P, batch, budget, ds);
            if (!found || c < cost) { found = true; cost = c; best = ds; }
        }
    return found;
}

// force_tc / pw_mode: explicit values for the two testing hooks (null / -1: the process-wide ones)
// Fully connected layer: one workgroup per 32 output channels streaming all of K, or, where that is
// cheaper, pairs of channel blocks with K split 2, 4 or 8 ways (at most 256 workgroups), a second
// launch adding the slices: what a workgroup then takes in per K step is 3 KiB for two MFMAs.
uint64_t fc_cost_ps(const Layer& L, int batch, int& ksplit)
{
    const int64_t nbb = ceil_div(batch, 32);
    const int64_t wbytes = (int64_t)L.ncb * L.nsteps * 1024 * nbb;
    uint64_t best = (uint64_t)((C_LAUNCH + C_LAT + wbytes / FC_BYTES_PER_CYCLE) * PS_PER_CYCLE);
    ksplit = 1;
    for (int ks = 2; ks <= 8; ks *= 2) {
        if (ceil_div(L.ncb, 2) * ks > 256 || L.nsteps < 64 * ks) continue;
        const int64_t intake = 3 * (int64_t)ceil_div(L.nsteps, ks) * 1024 * nbb / PW_BYTES_PER_CYCLE;
        const int64_t hbm = wbytes / FC_SPLIT_HBM_BYTES_PER_CYCLE;
        const uint64_t c = (uint64_t)((2 * C_LAUNCH + C_LAT + std::max(intake, hbm)) * PS_PER_CYCLE);
        if (c < best) { best = c; ksplit = ks; }
    }
    return best;
}

dlf_status make_group(const dlf_net_s& net, int batch, int first, int last, int budget, int max_lds,
                      GroupPlan& g, const TileCfg* force_tc = nullptr, int pw_mode = -1,
                      const C3Force* c3_force = nullptr)
{
    const TileCfg& force = force_tc ? *force_tc : g_force;
    const int pwm = pw_mode >= 0 ? pw_mode : g_pw_mode;
    const C3Force& c3f = c3_force ? *c3_force : g_c3_force;
    if (first < 0 || last >= (int)net.L.size() || first > last || budget <= 0)
        return fail(DLF_ERR_INVALID_ARG, "bad group [%d,%d] budget %d", first, last, budget);
    if (pwm != 2 && force.th <= 0 && pw2_eligible(net, first, last, batch)) {
        const Layer& P = net.L[first];
        const Layer& Q = net.L[last];
        const int shape = Q.ncb >= 3 ? 3 : 4;
        g = GroupPlan();
        g.first = first; g.last = last; g.budget = budget;
        g.in_layer = Q.src;                  // the 1x1 layer's input ...
        g.res_layer = P.src; g.res_stage = 0;   // ... and the projection's, handed over like a residual operand
        DlfPwArgs& wa = g.wa;
        memset(&wa, 0, sizeof wa);
        wa.w = Q.d_w; wa.bias = Q.d_bias;
        wa.m = batch * Q.out_h * Q.out_w;
        wa.cin = Q.d.cin; wa.cout = Q.d.cout; wa.ncb = Q.ncb; wa.nsteps = Q.nsteps;
        wa.act = Q.d.act; wa.stride = 1;
        wa.in_h = Q.in_h; wa.in_w = Q.in_w; wa.out_h = Q.out_h; wa.out_w = Q.out_w;
        wa.n_pg = ceil_div(wa.m, 32 * PW_FP[shape]); wa.n_cg = ceil_div(Q.ncb, PW_FC[shape]);
        wa.nitems = wa.n_pg * wa.n_cg;
        wa.w2 = P.d_w; wa.bias2 = P.d_bias; wa.cin2 = P.d.cin; wa.nsteps2 = P.nsteps; wa.stride2 = P.d.stride;
        wa.in_h2 = P.in_h; wa.in_w2 = P.in_w;
        g.kind = GK_PW2;
        g.cost = pw2_cost_ps(P, Q, batch, budget, shape);
        g.variant = shape;
        g.occ = 2;
        g.grid = std::max(8, std::min(budget * 2, ceil_div(wa.nitems, 8) * 8) / 8 * 8);
        g.th = 1; g.tw = 32 * PW_FP[shape];
        g.lds_bytes = shape == 3 ? DLF_PWB_LDS_BYTES(2, 2) : DLF_PWB_LDS_BYTES(1, 4);
        return DLF_OK;
    }
    std::vector<StageSpec> specs;
    std::string why;
    int kind;
    if (!group_stages(net, first, last, specs, kind, why))
        return fail(DLF_ERR_INFEASIBLE, "layers [%d,%d] cannot form a group: %s", first, last, why.c_str());
    g = GroupPlan();
    g.first = first; g.last = last; g.budget = budget; g.kind = kind;
    const Layer& L0 = net.L[first];
    g.in_layer = L0.src;
    if (kind == GK_FC) {
        DlfFcArgs& fa = g.fa;
        memset(&fa, 0, sizeof fa);
        fa.w = L0.d_w; fa.bias = L0.d_bias;
        fa.batch = batch; fa.k = L0.d.cin; fa.cout = L0.d.cout; fa.ncb = L0.ncb;
        fa.nsteps = L0.nsteps; fa.act = L0.d.act;
        int ksplit = 1;
        g.cost = fc_cost_ps(L0, batch, ksplit);
        if (force.th > 0 && (force.nslices == 1 || force.nslices == 2 || force.nslices == 4 || force.nslices == 8))
            ksplit = force.nslices;                     // testing hook
        fa.ksplit = ksplit;
        g.scratch_bytes = ksplit > 1 ? (size_t)ksplit * ceil_div(batch, 32) * L0.ncb * 4096 : 0;
        g.grid = L0.ncb;
        g.th = g.tw = 1;
        return DLF_OK;
    }
    if (kind == GK_GAP) {
        DlfGapArgs& pa = g.pa;
        memset(&pa, 0, sizeof pa);
        pa.batch = batch; pa.hw = L0.in_h * L0.in_w; pa.c = L0.d.cin;
        const int64_t bytes = (int64_t)batch * pa.hw * pa.c * 2;
        g.cost = (uint64_t)((C_LAUNCH + C_LAT + bytes / GAP_BYTES_PER_CYCLE) * PS_PER_CYCLE);
        g.grid = ceil_div(batch * pa.c, 256);
        g.th = L0.in_h; g.tw = L0.in_w;
        return DLF_OK;
    }
    Built b;
    TileCfg tc;
    uint64_t cost = 0;
    const bool tiled = choose_group(net, specs, batch, budget, max_lds, b, tc, cost, force);
    const bool pw_ok = first == last && pw_eligible(L0, batch) && pwm != 2 &&
                       (force.th <= 0 || pwm == 1 || pwm >= 3);
    // a 1x1 layer on the small-map kernel: pointwise mode 8 of the testing hook forces it
    DlfC3sArgs pcs;
    uint64_t pcsc = 0;
    const bool have_pcs = first == last && (pwm == 0 || pwm == 8) && (force.th <= 0 || pwm == 8) &&
                          c3s_pw_eligible(L0, batch) && c3s_choose(L0, batch, budget, max_lds, pcs, pcsc);
    auto take_pcs = [&]() {
        g.cs = pcs;
        g.kind = GK_C3S;
        g.cost = pcsc;
        g.variant = 8 + pcs.ksplit;
        g.occ = 1;
        g.grid = pcs.slice_major ? ceil_div(pcs.ntiles, 8 / pcs.nsl) * 8 : ceil_div(pcs.ntiles, 8) * 8 * pcs.nsl;
        g.th = pcs.th; g.tw = pcs.tw;
        g.lds_bytes = (int)DLF_C3S_LDS_BYTES(pcs.rp, pcs.cin);
        return DLF_OK;
    };
    if (have_pcs && pwm == 8) return take_pcs();
    if (pw_ok && pwm != 8) {
        int shape = 0;
        uint64_t pc = pw_cost_ps(L0, batch, budget, shape);
        if (have_pcs && pcsc < pc && (!tiled || pcsc < cost)) return take_pcs();
        if (pwm >= 3) {
            shape = pwm - 3;
            if (PW_KSPLIT[shape] > 1 && !pw_shape_ok(L0, shape)) shape = 0;
            pc = pw_shape_cost_ps(L0, batch, budget, shape);
        }
        if (!tiled || pwm == 1 || pwm >= 3 || pc < cost) {
            DlfPwArgs& wa = g.wa;
            memset(&wa, 0, sizeof wa);
            wa.w = L0.d_w; wa.bias = L0.d_bias;
            wa.m = batch * L0.out_h * L0.out_w;
            wa.cin = L0.d.cin; wa.cout = L0.d.cout; wa.ncb = L0.ncb; wa.nsteps = L0.nsteps;
            wa.act = L0.d.act; wa.stride = L0.d.stride;
            wa.in_h = L0.in_h; wa.in_w = L0.in_w; wa.out_h = L0.out_h; wa.out_w = L0.out_w;
            wa.n_pg = ceil_div(wa.m, 32 * PW_FP[shape]); wa.n_cg = ceil_div(L0.ncb, PW_FC[shape]);
            wa.nitems = wa.n_pg * wa.n_cg;
            g.kind = GK_PW;
            g.cost = pc;
            g.variant = shape;
            g.occ = (shape == 2 || PW_BLOCK[shape]) ? 2 : PW_WAVES_PER_CU[shape] / DLF_PW_WAVES;
            g.grid = PW_BLOCK[shape] ? std::max(8, std::min(budget * 2, ceil_div(wa.nitems, 8) * 8) / 8 * 8)
                     : shape == 2 ? std::min(budget * 2, wa.nitems)
                                : std::min(budget * g.occ, ceil_div(wa.nitems, DLF_PW_WAVES));
            g.th = 1; g.tw = 32 * PW_FP[shape];
            g.lds_bytes = shape == 3   ? DLF_PWB_LDS_BYTES(2, 2)
                          : shape == 4 ? DLF_PWB_LDS_BYTES(1, 4)
                                       : DLF_PW_WAVES * 32 * PW_FP[shape] * (32 * PW_FC[shape] + 8) * 2;
            if (L0.d.residual_from >= 0) { g.res_layer = L0.d.residual_from; g.res_stage = 0; }
            return DLF_OK;
        }
    }
    if ((g_dw_mode == 0 || g_dw_mode == 4) && (force.th <= 0 || g_dw_mode == 4) && dws_eligible(net, first, last, batch)) {
        const Layer& P = net.L[last];
        DlfDwsArgs ds;
        uint64_t sc = 0;
        bool have_s;
        if (g_dw_mode == 4 && g_dwt_force.wx > 0) {    // testing hook: channel blocks per wave, channels per pass
            have_s = dws_build(L0, P, batch, g_dwt_force.rw, g_dwt_force.wx, max_lds, ds);
            if (have_s) sc = dws_cost_ps(L0, P, batch, budget, ds);
        } else {
            have_s = dws_choose(L0, P, batch, budget, max_lds, ds, sc);
        }
        if (have_s) {
            // against the fused-group kernel and, where that one applies, the tile kernel
            uint64_t other = tiled ? cost : UINT64_MAX;
            if (g_dw_mode == 0 && g_dwt_force.wx <= 0 && dwt_eligible(net, first, last, batch)) {
                DlfDwtArgs dt;
                uint64_t dc = 0;
                int occ = 1;
                if (dwt_choose(L0, P, batch, budget, max_lds, dt, dc, occ)) other = std::min(other, dc);
            }
            if (g_dw_mode == 4 || sc < other) {
                g.ds = ds;
                g.kind = GK_DWS;
                g.cost = sc;
                g.variant = (L0.d.stride - 1) * 2 + (ds.cbw - 1);
                g.occ = 1;
                g.grid = ceil_div(ds.ntiles, 8) * 8 * ds.nsl;
                g.th = ds.th; g.tw = ds.tw;
                g.lds_bytes = (int)DLF_DWS_LDS_BYTES(ds.rp, ds.tp, ds.kh, ds.cbw, ds.nbuf);
                return DLF_OK;
            }
        }
    }
    if (g_dw_mode != 2 && g_dw_mode != 3 && (force.th <= 0 || g_dw_mode == 1) && dwt_eligible(net, first, last, batch)) {
        const Layer& P = net.L[last];
        DlfDwtArgs dt;
        uint64_t dc = 0;
        int occ = 1;
        bool have;
        if (g_dwt_force.wx > 0) {
            have = dwt_build(L0, P, batch, g_dwt_force.wx, g_dwt_force.rw, max_lds, dt);
            if (have) dc = dwt_cost_ps(L0, P, batch, budget, dt, occ);
        } else {
            have = dwt_choose(L0, P, batch, budget, max_lds, dt, dc, occ);
        }
        if (have && (!tiled || g_dw_mode == 1 || dc < cost)) {
            g.dt = dt;
            g.kind = GK_DWT;
            g.cost = dc;
            g.variant = L0.d.stride - 1;
            g.occ = occ;
            g.grid = std::min(budget * occ, dt.ntiles);
            g.th = dt.th; g.tw = dt.tw;
            g.lds_bytes = (int)DLF_DWT_LDS_BYTES(dt.tp, dt.c);
            return DLF_OK;
        }
    }
    if (g_dw_mode != 2 && (force.th <= 0 || g_dw_mode == 1 || g_dw_mode == 3) && dwpw_eligible(net, first, last, batch)) {
        const Layer& P = net.L[last];
        int nb = 4;
        uint64_t dc = dwpw_cost_ps(L0, P, batch, budget, 4);
        const uint64_t dc2 = dwpw_cost_ps(L0, P, batch, budget, 2);
        if (dc2 < dc || P.ncb <= 2) { nb = 2; dc = dc2; }
        if (!tiled || g_dw_mode == 1 || g_dw_mode == 3 || dc < cost) {
            dwpw_fill(L0, P, batch, nb, g.dp);
            g.kind = GK_DWPW;
            g.cost = dc;
            g.variant = nb;
            g.occ = 2;
            g.grid = std::min(budget * g.occ, ceil_div(g.dp.nitems, DLF_DWPW_WAVES));
            g.th = 1; g.tw = 32;
            g.lds_bytes = DLF_DWPW_LDS_BYTES(L0.d.cin, nb);
            return DLF_OK;
        }
    }
    if (first == last && g_dw_mode != 2 && (force.th <= 0 || g_dw_mode == 1) && dw_eligible(L0, batch)) {
        DlfDwArgs da;
        dw_fill(L0, batch, da);
        const uint64_t dc = dw_cost_ps(L0, batch, budget, da);
        if (!tiled || g_dw_mode == 1 || dc < cost) {
            g.da = da;
            g.kind = GK_DW;
            g.cost = dc;
            g.variant = L0.d.stride - 1;
            g.occ = DW_WAVES_PER_CU / DLF_DW_WAVES;
            g.grid = std::min(budget * g.occ, ceil_div(da.nitems, DLF_DW_WAVES));
            g.th = L0.d.stride == 1 ? DLF_DW_ROWS1 : DLF_DW_ROWS2;
            g.tw = 64;
            g.lds_bytes = 0;
            return DLF_OK;
        }
    }
    // a whole bottleneck block: shape DLF_C3_SHAPES + 2 of the testing hook (its th x tw then fix the tile)
    if ((first + 2 == last || first + 1 == last) && c3f.mode != 2 && (force.th <= 0 || c3f.mode == 1) &&
        (c3f.shape < 0 || c3f.shape == DLF_C3_SHAPES + 2) && bneck_eligible(net, specs, batch)) {
        const Layer& Bm = net.L[first + 1];
        const Layer& P = net.L[last];            // (two layers: the second one again)
        DlfBnArgs bn;
        uint64_t bc = 0;
        bool have;
        if (c3f.shape == DLF_C3_SHAPES + 2 && c3f.th > 0 && c3f.tw > 0) {
            have = bneck_build(L0, Bm, P, batch, ceil_div(L0.out_h, c3f.th), ceil_div(L0.out_w, c3f.tw), max_lds, bn);
            if (have) bc = bneck_cost_ps(L0, Bm, P, batch, budget, bn);
        } else {
            have = bneck_choose(L0, Bm, P, batch, budget, max_lds, bn, bc);
        }
        if (have && (!tiled || c3f.mode == 1 || bc < cost)) {
            g.bn = bn;
            g.kind = GK_BNECK;
            g.cost = bc;
            g.variant = bn.cin0;
            g.occ = bneck_per_cu(bn);
            g.grid = ceil_div(bn.ntiles, 8) * 8 * bn.nsl;
            g.th = bn.th; g.tw = bn.tw;
            g.lds_bytes = (int)DLF_BN_LDS_BYTES(bn.rp, bn.tp, bn.cin0);
            // (the shortcut is the group's own input: no second operand)
            return DLF_OK;
        }
    }
    // the fused 3x3 -> 1x1 kernel: shape DLF_C3_SHAPES + 1 of the testing hook (its th x tw then fix the tile)
    if (first + 1 == last && c3f.mode != 2 && (force.th <= 0 || c3f.mode == 1) &&
        (c3f.shape < 0 || c3f.shape == DLF_C3_SHAPES + 1) && c3pw_eligible(net, specs, batch)) {
        const Layer& P = net.L[last];
        DlfC3PwArgs cp;
        uint64_t pc = 0;
        bool have;
        if (c3f.shape == DLF_C3_SHAPES + 1 && c3f.th > 0 && c3f.tw > 0) {
            have = c3pw_build(L0, P, batch, ceil_div(L0.out_h, c3f.th), ceil_div(L0.out_w, c3f.tw), max_lds, cp);
            if (have) pc = c3pw_cost_ps(L0, P, batch, budget, cp);
        } else {
            have = c3pw_choose(L0, P, batch, budget, max_lds, cp, pc);
        }
        if (have && (!tiled || c3f.mode == 1 || pc < cost)) {
            g.cp = cp;
            g.kind = GK_C3PW;
            g.cost = pc;
            g.variant = cp.tp > 64 ? 4 : 2;
            g.occ = c3pw_per_cu(cp, P.d.residual_from >= 0);
            g.grid = ceil_div(cp.ntiles, 8) * 8 * cp.nsl;
            g.th = cp.th; g.tw = cp.tw;
            g.lds_bytes = (int)DLF_C3PW_LDS_BYTES(cp.rp, cp.tp, cp.c, P.d.residual_from >= 0);
            if (P.d.residual_from >= 0) { g.res_layer = P.d.residual_from; g.res_stage = 1; }
            return DLF_OK;
        }
    }
    // the small-map 3x3 kernel: shape DLF_C3_SHAPES of the testing hook (its th then fixes the split of K)
    DlfC3sArgs cs;
    uint64_t c3sc = 0;
    bool have_c3s = false;
    if (c3f.mode != 2 && (force.th <= 0 || c3f.mode == 1) && (c3f.shape < 0 || c3f.shape == DLF_C3_SHAPES) &&
        c3s_eligible(net, specs, batch)) {
        if (c3f.shape == DLF_C3_SHAPES && c3f.th > 0) {
            have_c3s = c3s_build(L0, batch, c3f.th, 0, 0, max_lds, cs);
            if (have_c3s) c3sc = c3s_cost_ps(L0, batch, budget, cs);
        } else {
            have_c3s = c3s_choose(L0, batch, budget, max_lds, cs, c3sc);
        }
    }
    if (c3f.mode != 2 && (force.th <= 0 || c3f.mode == 1) && c3f.shape != DLF_C3_SHAPES && c3_eligible(net, specs, batch)) {
        C3Cfg cc;
        uint64_t c3c = 0;
        const int pool2 = specs[0].pool2;
        bool have;
        if (c3f.shape >= 0) {
            have = c3_build(pool2, L0.d.cin, c3f.shape, c3f.th, c3f.tw, max_lds, cc);
            if (have) c3c = c3_cost_ps(L0, pool2, batch, budget, cc);
        } else {
            have = c3_choose(L0, pool2, batch, budget, max_lds, cc, c3c);
        }
        if (have && have_c3s && c3sc < c3c) have = false;       // the small-map kernel is cheaper: decided below
        if (have && (!tiled || c3f.mode == 1 || c3c < cost)) {
            DlfC3Args& ca = g.ca;
            memset(&ca, 0, sizeof ca);
            ca.w = L0.d_w; ca.bias = L0.d_bias;
            ca.batch = batch; ca.h = L0.out_h; ca.w_ = L0.out_w; ca.cin = L0.d.cin; ca.cout = L0.d.cout;
            ca.ncb = L0.ncb; ca.nsteps = L0.nsteps; ca.act = L0.d.act; ca.pool2 = pool2;
            ca.th = cc.th; ca.tw = cc.tw;
            ca.tiles_y = ceil_div(L0.out_h, cc.th); ca.tiles_x = ceil_div(L0.out_w, cc.tw);
            ca.n_cg = ceil_div(L0.ncb, 2 * C3_WC[cc.shape]);
            ca.ntiles = batch * ca.tiles_y * ca.tiles_x;
            ca.nitems = ca.n_cg * ca.ntiles;
            ca.npxh = cc.npxh; ca.na_i = cc.na_i; ca.lpw_a = cc.lpw_a; ca.nst = cc.nst;
            g.kind = GK_C3;
            g.cost = c3c;
            g.variant = cc.shape;
            g.occ = 1;
            g.grid = std::max(8, std::min(budget, ceil_div(ca.nitems, 8) * 8) / 8 * 8);
            g.th = cc.th; g.tw = cc.tw;
            g.lds_bytes = cc.lds_bytes;
            if (L0.d.residual_from >= 0) { g.res_layer = L0.d.residual_from; g.res_stage = 0; }
            return DLF_OK;
        }
    }
    if (have_c3s && (!tiled || c3f.mode == 1 || c3sc < cost)) {
        g.cs = cs;
        g.kind = GK_C3S;
        g.cost = c3sc;
        g.variant = cs.ksplit;
        g.occ = 1;
        g.grid = cs.slice_major ? ceil_div(cs.ntiles, 8 / cs.nsl) * 8 : ceil_div(cs.ntiles, 8) * 8 * cs.nsl;
        g.th = cs.th; g.tw = cs.tw;
        g.lds_bytes = (int)DLF_C3S_LDS_BYTES(cs.rp, cs.cin);
        if (L0.d.residual_from >= 0) { g.res_layer = L0.d.residual_from; g.res_stage = 0; }
        return DLF_OK;
    }
    if (!tiled)
        return fail(DLF_ERR_INFEASIBLE, "layers [%d,%d] do not fit on-chip memory as one group", first, last);
    g.ga = b.ga;
    g.variant = tc.variant;
    g.lds_bytes = b.lds_bytes;
    // the budget counts CUs; a CU holds as many workgroups as registers and LDS allow
    g.occ = std::max(1, std::min(VAR_OCC[tc.variant], (160 * 1024) / std::max(b.lds_bytes, 1)));
    g.grid = std::min(budget * g.occ, b.ntiles);
    g.th = tc.th; g.tw = tc.tw;
    g.cost = cost;
    for (size_t s = 0; s < specs.size(); ++s) {
        const int rf = net.L[specs[s].layer].d.residual_from;
        if (rf >= 0) { g.res_layer = rf; g.res_stage = (int)s; }
    }
    return DLF_OK;
}

}  // namespace

struct dlf_plan_s {
    const dlf_net_s* net;
    int batch;
    std::vector<GroupPlan> G;
    std::vector<size_t> layer_off;   // workspace offset of each layer's output, or SIZE_MAX
    size_t ws_bytes = 0;
    char* ws = nullptr;
    int max_lds = 160 * 1024;
    // Branches: a group that does not read the output of the group in front of it (the projection
    // shortcut of a residual block beside the block's first layers) runs on a second stream, beside
    // that group.  The streams meet through events: a group waits for each producer on the other
    // stream, and the caller's stream waits for the second one at the end of dlf_run.  Off unless
    // asked for: on this chip the hand-over between two hardware queues costs more than the
    // overlap of two such layers gains.
    bool overlap = false;
    std::vector<int> on_side;        // per group: 1 = second stream
    std::vector<int> dep_a, dep_b;   // per group: producer groups of its input / residual (-1: none)
    mutable hipStream_t side = nullptr;
    mutable std::vector<hipEvent_t> done;   // per group: recorded after it where another stream waits
    mutable hipEvent_t side_end = nullptr;
    ~dlf_plan_s()
    {
        for (hipEvent_t e : done) if (e) (void)hipEventDestroy(e);
        if (side_end) (void)hipEventDestroy(side_end);
        if (side) (void)hipStreamDestroy(side);
    }
};

namespace {

const int DEFAULT_BUDGETS[4] = {32, 64, 128, 256};

// Algorithm 1 of the paper (greedy joint fusion + MP pass).  Where the printed algorithm is silent
// or inconsistent: the running mean of the per-layer MP is kept as a sum and a count; the threshold
// test is skipped while the open block holds no convolution / FC layer; the walk covers every layer;
// layers left over at the end form a last block; pooling layers ride with the block before them;
// Eq. 5's proportionality is closed with a fitted scale and offset (MP = k * score + b, clamped),
// with C = min(Cin, Cout); a block's MP is its mean MP floored to a power of two, then the largest
// allowed budget not above it.
bool conv_like(const dlf_net_s& net, int i)
{
    const int op = net.L[i].d.op;
    return op == DLF_CONV || op == DLF_DWCONV || op == DLF_FC;
}

// Eq. 5 closed with a scale and an offset, clamped to [1, max_mp]
double layer_mp(const Layer& L, int batch, double alpha, double beta, double k, double b, int max_mp)
{
    const double ops = 2.0 * (double)L.macs * batch;
    const double score = alpha * std::log2((double)std::min(L.d.cin, L.d.cout)) + beta * std::log2(ops);
    return std::min((double)max_mp, std::max(1.0, k * score + b));
}

// mean MP of a block -> power of two below it -> largest allowed budget not above that
int round_mp(double avg, const std::vector<int>& allowed)
{
    const int p = 1 << (int)std::floor(std::log2(avg));
    int best = -1;
    for (int a : allowed) if (a <= p && a > best) best = a;
    if (best < 0) best = *std::min_element(allowed.begin(), allowed.end());
    return best;
}

void algorithm1(const dlf_net_s& net, int batch, double crit, double alpha, double beta, double k,
                double b, const std::vector<int>& allowed, std::vector<int>& part, std::vector<int>& mps)
{
    const int n = (int)net.L.size();
    const int max_mp = *std::max_element(allowed.begin(), allowed.end());
    auto conv_like = [&](int i) { return ::conv_like(net, i); };
    auto round_mp = [&](double avg) { return ::round_mp(avg, allowed); };
    double sum_op = 0, sum_mp = 0;
    int block = 0;
    for (int i = 0; i < n; ++i) {
        if (conv_like(i)) {
            const Layer& L = net.L[i];
            sum_mp += layer_mp(L, batch, alpha, beta, k, b, max_mp);
            sum_op += 2.0 * (double)L.macs * batch;
            ++block;
        }
        if (block > 0) {
            const double avg = sum_mp / block;
            if (sum_op / avg >= crit) {
                while (i + 1 < n && !conv_like(i + 1)) ++i;
                part.push_back(i);
                mps.push_back(round_mp(avg));
                sum_op = sum_mp = 0;
                block = 0;
            }
        }
    }
    const int covered = part.empty() ? 0 : part.back() + 1;
    if (covered < n) {
        if (block > 0) {
            part.push_back(n - 1);
            mps.push_back(round_mp(sum_mp / block));
        } else if (!part.empty()) {
            part.back() = n - 1;
        } else {
            part.push_back(n - 1);
            mps.push_back(*std::min_element(allowed.begin(), allowed.end()));
        }
    }
}

}  // namespace

extern "C" {

const char* dlf_status_string(dlf_status s)
{
    switch (s) {
    case DLF_OK: return "ok";
    case DLF_ERR_INVALID_ARG: return "invalid argument";
    case DLF_ERR_SHAPE: return "shape mismatch";
    case DLF_ERR_UNSUPPORTED: return "unsupported layer";
    case DLF_ERR_INFEASIBLE: return "fusion group infeasible";
    case DLF_ERR_OOM: return "out of memory";
    case DLF_ERR_HIP: return "HIP error";
    case DLF_ERR_NO_WEIGHTS: return "network has no weights";
    }
    return "unknown status";
}

const char* dlf_last_error(void) { return g_err.c_str(); }

int32_t dlf_cost_model_version(void) { return 3; }

dlf_status dlf_net_create(const dlf_layer_desc* layers, int32_t n, int32_t in_h, int32_t in_w,
                          int32_t in_c, dlf_net_t** out)
{
    if (!layers || !out || n <= 0 || in_h <= 0 || in_w <= 0 || in_c <= 0)
        return fail(DLF_ERR_INVALID_ARG, "dlf_net_create: null or non-positive argument");
    // Limits that keep every size computed from these fields inside 32-bit integers.
    const int32_t MAX_DIM = 1 << 20, MAX_WINDOW = 1 << 10;
    if (in_h > MAX_DIM || in_w > MAX_DIM || in_c > MAX_DIM)
        return fail(DLF_ERR_INVALID_ARG, "dlf_net_create: input dimension above %d", MAX_DIM);
    dlf_net_s* net = new (std::nothrow) dlf_net_s;
    if (!net) return fail(DLF_ERR_OOM, "host allocation failed");
    net->in_h = in_h; net->in_w = in_w; net->in_c = in_c;
    net->L.resize(n);
    int with_w = 0, need_w = 0;
    for (int i = 0; i < n; ++i) {
        Layer& L = net->L[i];
        L.d = layers[i];
        const dlf_layer_desc& d = L.d;
        auto bad = [&](dlf_status s, const char* msg) {
            delete net;
            return fail(s, "layer %d: %s", i, msg);
        };
        if (d.op < DLF_CONV || d.op > DLF_GLOBAL_AVGPOOL) return bad(DLF_ERR_INVALID_ARG, "bad op");
        if (d.act < DLF_ACT_NONE || d.act > DLF_ACT_RELU6) return bad(DLF_ERR_INVALID_ARG, "bad activation");
        if (d.cin <= 0 || d.cout <= 0 || d.kh <= 0 || d.kw <= 0 || d.stride <= 0 || d.pad < 0)
            return bad(DLF_ERR_INVALID_ARG, "non-positive size");
        if (d.cin > (d.op == DLF_FC ? (1 << 24) : MAX_DIM) || d.cout > MAX_DIM || d.kh > MAX_WINDOW || d.kw > MAX_WINDOW ||
            d.stride > MAX_WINDOW || d.pad > MAX_WINDOW)
            return bad(DLF_ERR_INVALID_ARG, "size above the supported range");
        if (d.input_from < -1 || d.input_from >= i) return bad(DLF_ERR_INVALID_ARG, "input_from must name an earlier layer");
        if (d.residual_from < -1 || d.residual_from >= i) return bad(DLF_ERR_INVALID_ARG, "residual_from must name an earlier layer");
        L.src = d.input_from >= 0 ? d.input_from : i - 1;
        if (L.src < 0) { L.in_h = in_h; L.in_w = in_w; L.in_c = in_c; }
        else { L.in_h = net->L[L.src].out_h; L.in_w = net->L[L.src].out_w; L.in_c = net->L[L.src].out_c; }
        L.macs = 0;
        switch (d.op) {
        case DLF_CONV: case DLF_DWCONV: case DLF_MAXPOOL:
            if (d.cin != L.in_c) return bad(DLF_ERR_SHAPE, "cin does not match the input tensor");
            if (d.op != DLF_CONV && d.cin != d.cout) return bad(DLF_ERR_SHAPE, "cin must equal cout");
            if (L.in_h + 2 * d.pad < d.kh || L.in_w + 2 * d.pad < d.kw) return bad(DLF_ERR_SHAPE, "kernel larger than padded input");
            L.out_h = (L.in_h + 2 * d.pad - d.kh) / d.stride + 1;
            L.out_w = (L.in_w + 2 * d.pad - d.kw) / d.stride + 1;
            L.out_c = d.cout;
            if (d.op == DLF_CONV) L.macs = (uint64_t)L.out_h * L.out_w * d.kh * d.kw * d.cin * d.cout;
            if (d.op == DLF_DWCONV) L.macs = (uint64_t)L.out_h * L.out_w * d.kh * d.kw * d.cout;
            if (d.op == DLF_MAXPOOL && d.has_bias) return bad(DLF_ERR_INVALID_ARG, "pooling has no bias");
            break;
        case DLF_FC:
            if ((int64_t)d.cin != (int64_t)L.in_h * L.in_w * L.in_c) return bad(DLF_ERR_SHAPE, "FC cin must equal H*W*C of its input");
            if (d.kh != 1 || d.kw != 1) return bad(DLF_ERR_INVALID_ARG, "FC kernel must be 1x1");
            L.out_h = L.out_w = 1; L.out_c = d.cout;
            L.macs = (uint64_t)d.cin * d.cout;
            break;
        case DLF_GLOBAL_AVGPOOL:
            if (d.cin != L.in_c || d.cout != d.cin) return bad(DLF_ERR_SHAPE, "channel mismatch");
            L.out_h = L.out_w = 1; L.out_c = d.cout;
            break;
        }
        if (d.residual_from >= 0) {
            const Layer& R = net->L[d.residual_from];
            if (R.out_h != L.out_h || R.out_w != L.out_w || R.out_c != L.out_c)
                return bad(DLF_ERR_SHAPE, "residual operand shape differs from the layer output");
        }
        if (d.op == DLF_CONV && (d.cout % 4) != 0)
            return bad(DLF_ERR_UNSUPPORTED, "convolution needs cout % 4 == 0");
        if (d.op == DLF_FC && (d.cin % 8) != 0)
            return bad(DLF_ERR_UNSUPPORTED, "FC needs cin % 8 == 0");
        if ((d.op == DLF_DWCONV || d.op == DLF_MAXPOOL) && (d.cin % 8) != 0)
            return bad(DLF_ERR_UNSUPPORTED, "depthwise / pooling layers need channels % 8 == 0");
        if (d.op == DLF_MAXPOOL && d.pad >= d.kh)
            return bad(DLF_ERR_UNSUPPORTED, "pooling pad must be smaller than the window");
        if (d.op == DLF_CONV || d.op == DLF_FC) {
            L.kc = 32;
            const bool narrow = d.op == DLF_CONV && (d.cin % 8) != 0;
            L.rowfold = narrow && d.cin <= 4 && (d.stride % 2) == 0 && d.kw * 4 <= 128;
            L.im2col = narrow && !L.rowfold;
            if (narrow && L.src >= 0)
                return bad(DLF_ERR_UNSUPPORTED, "a convolution with cin % 8 != 0 must read the network input");
            if (L.im2col && L.src >= 0)
                return bad(DLF_ERR_UNSUPPORTED, "a convolution with cin % 8 != 0 must read the network input");
            if (L.im2col && d.kh * d.kw * d.cin > 1024)
                return bad(DLF_ERR_UNSUPPORTED, "narrow-input convolution too large");
            L.cin_pad = round_up(L.rowfold ? d.kw * 4 : (L.im2col ? d.kh * d.kw * d.cin : d.cin), L.kc);
            L.ncb = ceil_div(d.cout, 32);
            L.nsteps = L.rowfold ? (L.cin_pad / 16) * d.kh
                                 : (L.im2col ? L.cin_pad / 16 : (L.cin_pad / L.kc) * d.kh * d.kw * (L.kc / 16));
        } else if (d.op == DLF_DWCONV) {
            L.kc = 8; L.cin_pad = round_up(d.cin, 8);
        }
        if (d.op == DLF_CONV || d.op == DLF_FC || d.op == DLF_DWCONV) {
            ++need_w;
            if (d.weight) ++with_w;
        }
    }
    if (with_w != 0 && with_w != need_w) {
        delete net;
        return fail(DLF_ERR_INVALID_ARG, "either all or none of the weighted layers must have weights");
    }
    net->has_weights = (with_w == need_w) && (with_w > 0 || need_w == 0);
    if (net->has_weights && need_w > 0) {
        for (int i = 0; i < n; ++i) {
            dlf_status s = pack_and_upload(net->L[i]);
            if (s != DLF_OK) { dlf_net_destroy(net); return s; }
        }
    }
    for (int i = 0; i < n; ++i) { net->L[i].d.weight = nullptr; net->L[i].d.bias = nullptr; }
    *out = net;
    return DLF_OK;
}

void dlf_net_destroy(dlf_net_t* net)
{
    if (!net) return;
    for (Layer& L : net->L) {
        if (L.d_w) (void)hipFree(L.d_w);
        if (L.d_bias) (void)hipFree(L.d_bias);
    }
    delete net;
}

int32_t dlf_net_num_layers(const dlf_net_t* net) { return net ? (int32_t)net->L.size() : 0; }

dlf_status dlf_net_layer_info(const dlf_net_t* net, int32_t i, int32_t* out_h, int32_t* out_w,
                              int32_t* out_c, uint64_t* op_count)
{
    if (!net || i < 0 || i >= (int)net->L.size()) return fail(DLF_ERR_INVALID_ARG, "bad layer index");
    const Layer& L = net->L[i];
    if (out_h) *out_h = L.out_h;
    if (out_w) *out_w = L.out_w;
    if (out_c) *out_c = L.out_c;
    if (op_count) *op_count = 2 * L.macs;
    return DLF_OK;
}

dlf_status dlf_group_cost(const dlf_net_t* net, int32_t batch, int32_t first, int32_t last,
                          int32_t budget, int32_t max_lds_bytes, uint64_t* cost)
{
    if (!net || !cost || batch <= 0) return fail(DLF_ERR_INVALID_ARG, "dlf_group_cost: bad argument");
    GroupPlan g;
    dlf_status s = make_group(*net, batch, first, last, budget, max_lds_bytes > 0 ? max_lds_bytes : 160 * 1024, g);
    if (s != DLF_OK) return s;
    *cost = g.cost;
    return DLF_OK;
}

dlf_status dlf_plan(const dlf_net_t* net, int32_t batch, const dlf_tuner_opts* opts, dlf_plan_t** out)
{
    if (!net || !out || batch <= 0) return fail(DLF_ERR_INVALID_ARG, "dlf_plan: bad argument");
    dlf_tuner_opts o;
    memset(&o, 0, sizeof o);
    if (opts) o = *opts;
    const int n = (int)net->L.size();
    const int max_lds = o.max_lds_bytes > 0 ? o.max_lds_bytes : 160 * 1024;
    std::vector<int> budgets;
    if (o.budgets && o.n_budgets > 0) budgets.assign(o.budgets, o.budgets + o.n_budgets);
    else budgets.assign(DEFAULT_BUDGETS, DEFAULT_BUDGETS + 4);
    for (int b : budgets) if (b <= 0) return fail(DLF_ERR_INVALID_ARG, "budgets must be positive");

    std::vector<GroupPlan> groups;
    if (o.mode == DLF_TUNER_MANUAL) {
        if (!o.manual_group_last || !o.manual_budget || o.manual_n <= 0)
            return fail(DLF_ERR_INVALID_ARG, "manual plan needs group_last[], budget[] and a count");
        int first = 0;
        for (int g = 0; g < o.manual_n; ++g) {
            const int last = o.manual_group_last[g];
            if (last < first || last >= n) return fail(DLF_ERR_INVALID_ARG, "manual group_last[] must be increasing and < n");
            GroupPlan gp;
            dlf_status s = make_group(*net, batch, first, last, o.manual_budget[g], max_lds, gp);
            if (s != DLF_OK) return s;
            groups.push_back(gp);
            first = last + 1;
        }
        if (first != n) return fail(DLF_ERR_INVALID_ARG, "manual groups must cover every layer");
    } else if (o.mode == DLF_TUNER_DP) {
        // cost[f][l][b] for every contiguous range and budget; infeasible = no entry
        const uint64_t INF = std::numeric_limits<uint64_t>::max();
        const int nb = (int)budgets.size();
        std::vector<GroupPlan> table((size_t)n * n * nb);
        std::vector<char> ok((size_t)n * n * nb, 0);
        auto idx = [&](int f, int l, int b) { return ((size_t)f * n + l) * nb + b; };
        for (int f = 0; f < n; ++f)
            for (int l = f; l < n; ++l) {
                bool any = false;
                for (int b = 0; b < nb; ++b) {
                    GroupPlan gp;
                    if (make_group(*net, batch, f, l, budgets[b], max_lds, gp) == DLF_OK) {
                        table[idx(f, l, b)] = gp;
                        ok[idx(f, l, b)] = 1;
                        any = true;
                    }
                }
                if (!any && l > f) {
                    // a range that cannot be a group: longer ranges starting at f may still be
                    // (e.g. conv + pool + conv), so keep scanning
                }
            }
        // best[i] = best plan for the suffix starting at layer i under the total order
        // (cost, number of groups, group_last lexicographic, budgets lexicographic)
        struct Sfx { uint64_t cost; int ngroups; std::vector<int> lasts, buds; bool valid; };
        std::vector<Sfx> best(n + 1);
        best[n] = Sfx{0, 0, {}, {}, true};
        for (int i = n - 1; i >= 0; --i) {
            Sfx bs{INF, 0, {}, {}, false};
            for (int l = i; l < n; ++l) {
                if (!best[l + 1].valid) continue;
                for (int b = 0; b < nb; ++b) {
                    if (!ok[idx(i, l, b)]) continue;
                    Sfx c;
                    c.valid = true;
                    c.cost = table[idx(i, l, b)].cost + best[l + 1].cost;
                    c.ngroups = 1 + best[l + 1].ngroups;
                    c.lasts.push_back(l);
                    c.lasts.insert(c.lasts.end(), best[l + 1].lasts.begin(), best[l + 1].lasts.end());
                    c.buds.push_back(budgets[b]);
                    c.buds.insert(c.buds.end(), best[l + 1].buds.begin(), best[l + 1].buds.end());
                    bool better = !bs.valid;
                    if (!better) {
                        if (c.cost != bs.cost) better = c.cost < bs.cost;
                        else if (c.ngroups != bs.ngroups) better = c.ngroups < bs.ngroups;
                        else if (c.lasts != bs.lasts) better = c.lasts < bs.lasts;
                        else better = c.buds < bs.buds;
                    }
                    if (better) bs = c;
                }
            }
            best[i] = bs;
        }
        if (!best[0].valid) return fail(DLF_ERR_INFEASIBLE, "no feasible plan");
        int first = 0;
        for (size_t g = 0; g < best[0].lasts.size(); ++g) {
            const int last = best[0].lasts[g];
            int bi = 0;
            for (int b = 0; b < nb; ++b) if (budgets[b] == best[0].buds[g]) { bi = b; break; }
            groups.push_back(table[idx(first, last, bi)]);
            first = last + 1;
        }
    } else if (o.mode == DLF_TUNER_GREEDY) {
        const double alpha = (o.alpha == 0 && o.beta == 0) ? 0.316 : o.alpha;
        const double beta = (o.alpha == 0 && o.beta == 0) ? 0.659 : o.beta;
        const double k = (o.mp_scale == 0 && o.mp_offset == 0) ? 64.0 : o.mp_scale;
        const double b0 = (o.mp_scale == 0 && o.mp_offset == 0) ? -1056.0 : o.mp_offset;
        const double crit = o.opcount_critical > 0 ? o.opcount_critical : 2.0e7;
        std::vector<int> part, mps;
        algorithm1(*net, batch, crit, alpha, beta, k, b0, budgets, part, mps);
        // legalisation: a block the kernels cannot run as one group is split left to right into
        // maximal feasible groups, all with the block's budget
        int first = 0;
        for (size_t g = 0; g < part.size(); ++g) {
            const int blk_last = part[g];
            while (first <= blk_last) {
                int l = blk_last;
                GroupPlan gp;
                dlf_status s = DLF_ERR_INFEASIBLE;
                for (; l >= first; --l) {
                    s = make_group(*net, batch, first, l, o.fixed_budget > 0 ? o.fixed_budget : mps[g], max_lds, gp);
                    if (s == DLF_OK) break;
                }
                if (s != DLF_OK) return s;
                groups.push_back(gp);
                first = l + 1;
            }
        }
    } else if (o.mode == DLF_TUNER_LAYERWISE) {
        // every layer a group of its own; a layer without Eq. 5 features (pooling) takes the
        // budget of the convolution before it
        const double alpha = (o.alpha == 0 && o.beta == 0) ? 0.316 : o.alpha;
        const double beta = (o.alpha == 0 && o.beta == 0) ? 0.659 : o.beta;
        const double k = (o.mp_scale == 0 && o.mp_offset == 0) ? 64.0 : o.mp_scale;
        const double b0 = (o.mp_scale == 0 && o.mp_offset == 0) ? -1056.0 : o.mp_offset;
        const int max_mp = *std::max_element(budgets.begin(), budgets.end());
        int bud = *std::min_element(budgets.begin(), budgets.end());
        for (int i = 0; i < n; ++i) {
            if (conv_like(*net, i)) bud = round_mp(layer_mp(net->L[i], batch, alpha, beta, k, b0, max_mp), budgets);
            GroupPlan gp;
            dlf_status s = make_group(*net, batch, i, i, o.fixed_budget > 0 ? o.fixed_budget : bud, max_lds, gp);
            if (s != DLF_OK) return s;
            groups.push_back(gp);
        }
    } else if (o.mode == DLF_TUNER_MAXFUSE) {
        const int bud = o.fixed_budget > 0 ? o.fixed_budget : *std::max_element(budgets.begin(), budgets.end());
        int first = 0;
        while (first < n) {
            int l = n - 1;
            GroupPlan gp;
            dlf_status s = DLF_ERR_INFEASIBLE;
            for (; l >= first; --l) {
                s = make_group(*net, batch, first, l, bud, max_lds, gp);
                if (s == DLF_OK) break;
            }
            if (s != DLF_OK) return s;
            groups.push_back(gp);
            first = l + 1;
        }
    } else {
        return fail(DLF_ERR_INVALID_ARG, "unknown tuner mode %d", o.mode);
    }

    dlf_plan_s* plan = new (std::nothrow) dlf_plan_s;
    if (!plan) return fail(DLF_ERR_OOM, "host allocation failed");
    plan->net = net;
    plan->batch = batch;
    plan->G = groups;
    plan->max_lds = max_lds;
    // workspace: the output of each group except the last, 256-byte aligned slots
    plan->layer_off.assign(n, (size_t)-1);
    size_t off = 0;
    for (size_t g = 0; g + 1 < groups.size(); ++g) {
        const Layer& L = net->L[groups[g].last];
        const size_t bytes = (size_t)batch * L.out_h * L.out_w * L.out_c * 2;
        plan->layer_off[groups[g].last] = off;
        off += (bytes + 255) & ~(size_t)255;
    }
    for (GroupPlan& G : plan->G)
        if (G.scratch_bytes > 0) {
            G.scratch_off = off;
            off += (G.scratch_bytes + 255) & ~(size_t)255;
        }
    plan->ws_bytes = off;
    {
        const size_t ng = groups.size();
        std::vector<int> owner(n, -1);               // group that produces a layer's output
        for (size_t g = 0; g < ng; ++g)
            for (int l = groups[g].first; l <= groups[g].last; ++l) owner[l] = (int)g;
        plan->on_side.assign(ng, 0);
        plan->dep_a.assign(ng, -1);
        plan->dep_b.assign(ng, -1);
        for (size_t g = 0; g < ng; ++g) {
            const GroupPlan& G = groups[g];
            if (G.in_layer >= 0) plan->dep_a[g] = owner[G.in_layer];
            if (G.res_stage >= 0 && G.res_layer >= 0) plan->dep_b[g] = owner[G.res_layer];
            if (g >= 1 && g + 1 < ng && plan->on_side[g - 1] == 0 && plan->dep_a[g] != (int)g - 1 &&
                plan->dep_b[g] != (int)g - 1)
                plan->on_side[g] = 1;
        }
    }
    for (const GroupPlan& G : groups) {
        const bool in_ok = G.in_layer < 0 || plan->layer_off[G.in_layer] != (size_t)-1;
        const bool res_ok = G.res_stage < 0 || G.res_layer < 0 || plan->layer_off[G.res_layer] != (size_t)-1;
        if (!in_ok || !res_ok) {
            delete plan;
            return fail(DLF_ERR_INFEASIBLE, "group [%d,%d] reads a tensor that is not the output of an earlier group",
                        G.first, G.last);
        }
    }
    *out = plan;
    return DLF_OK;
}

void dlf_plan_destroy(dlf_plan_t* plan) { delete plan; }

int32_t dlf_plan_num_groups(const dlf_plan_t* plan) { return plan ? (int32_t)plan->G.size() : 0; }

dlf_status dlf_plan_group(const dlf_plan_t* plan, int32_t g, int32_t* first, int32_t* last,
                          int32_t* budget, int32_t* tile_h, int32_t* tile_w, uint64_t* model_cost)
{
    if (!plan || g < 0 || g >= (int)plan->G.size()) return fail(DLF_ERR_INVALID_ARG, "bad group index");
    const GroupPlan& G = plan->G[g];
    if (first) *first = G.first;
    if (last) *last = G.last;
    if (budget) *budget = G.budget;
    if (tile_h) *tile_h = G.th;
    if (tile_w) *tile_w = G.tw;
    if (model_cost) *model_cost = G.cost;
    return DLF_OK;
}

dlf_status dlf_plan_group_config(const dlf_plan_t* plan, int32_t g, int32_t* kind, int32_t* variant,
                                 int32_t* nslices, int32_t* slice_c, int32_t* stream0, int32_t* lds_bytes)
{
    if (!plan || g < 0 || g >= (int)plan->G.size()) return fail(DLF_ERR_INVALID_ARG, "bad group index");
    const GroupPlan& G = plan->G[g];
    if (kind) *kind = G.kind;
    if (variant) *variant = G.variant;
    if (nslices) *nslices = G.kind == GK_GROUP ? G.ga.nslices : 1;
    if (slice_c) *slice_c = G.kind == GK_GROUP ? G.ga.slice_c : 0;
    if (stream0) *stream0 = G.kind == GK_GROUP ? G.ga.stream0 : 0;
    if (lds_bytes) *lds_bytes = G.lds_bytes;
    return DLF_OK;
}

dlf_status dlf_plan_group_io(const dlf_plan_t* plan, int32_t g, int32_t* in_layer, int32_t* res_layer)
{
    if (!plan || g < 0 || g >= (int)plan->G.size()) return fail(DLF_ERR_INVALID_ARG, "bad group index");
    const GroupPlan& G = plan->G[g];
    if (in_layer) *in_layer = G.in_layer;
    if (res_layer) *res_layer = G.res_stage >= 0 ? G.res_layer : -2;
    return DLF_OK;
}

void dlf_debug_pointwise_mode(int32_t mode) { g_pw_mode = (mode >= 0 && mode <= 8) ? mode : 0; }

void dlf_debug_depthwise_mode(int32_t mode) { g_dw_mode = (mode >= 0 && mode <= 4) ? mode : 0; }

void dlf_debug_depthwise_tile(int32_t wx, int32_t rw) { g_dwt_force = DwtForce{wx, rw}; }

void dlf_debug_block3x3_mode(int32_t mode, int32_t shape, int32_t th, int32_t tw)
{
    g_c3_force = C3Force{(mode >= 0 && mode <= 2) ? mode : 0, shape, th, tw};
}

void dlf_debug_force_ksplit(int32_t ksplit) { g_force.ksplit = ksplit > 0 ? ksplit : 1; }

void dlf_debug_force_config(int32_t th, int32_t tw, int32_t variant, int32_t nslices, int32_t slice_c,
                            int32_t stream0, int32_t kc)
{
    g_force = TileCfg{th, tw, variant, nslices < 1 ? 1 : nslices, slice_c, stream0, kc > 0 ? kc : 32};
}

size_t dlf_plan_workspace_bytes(const dlf_plan_t* plan) { return plan ? plan->ws_bytes : 0; }

dlf_status dlf_plan_bind_workspace(dlf_plan_t* plan, void* dev_ptr, size_t bytes)
{
    if (!plan) return fail(DLF_ERR_INVALID_ARG, "null plan");
    if (bytes < plan->ws_bytes) return fail(DLF_ERR_OOM, "workspace too small: %zu < %zu", bytes, plan->ws_bytes);
    if (plan->ws_bytes > 0 && (!dev_ptr || ((uintptr_t)dev_ptr & 255) != 0))
        return fail(DLF_ERR_INVALID_ARG, "workspace must be a 256-byte aligned device pointer");
    plan->ws = (char*)dev_ptr;
    return DLF_OK;
}

const void* dlf_plan_layer_output(const dlf_plan_t* plan, int32_t layer)
{
    if (!plan || layer < 0 || layer >= (int)plan->layer_off.size()) return nullptr;
    if (plan->layer_off[layer] == (size_t)-1 || !plan->ws) return nullptr;
    return plan->ws + plan->layer_off[layer];
}

static std::once_flag g_kernels_once;
static int g_kernels_rc = 0;

// ws: base of the workspace this run uses (the plan's bound one, or the static array)
static dlf_status launch_one(const dlf_plan_s* plan, const GroupPlan& G, const void* in, const void* res,
                             void* out, void* stream, char* ws)
{
    int e = 0;
    std::call_once(g_kernels_once, [] { g_kernels_rc = dlf_kernels_init(); });
    if (g_kernels_rc != 0)
        return fail(DLF_ERR_HIP, "kernel setup failed: %s", hipGetErrorString((hipError_t)g_kernels_rc));
    if (G.kind == GK_FC) {
        DlfFcArgs fa = G.fa;
        fa.x = in; fa.y = out;
        if (fa.ksplit > 1) {
            if (!ws) return fail(DLF_ERR_INVALID_ARG, "no workspace bound");
            fa.part = (float*)(ws + G.scratch_off);
        }
        e = dlf_launch_fc(&fa, stream);
    } else if (G.kind == GK_GAP) {
        DlfGapArgs pa = G.pa;
        pa.x = in; pa.y = out;
        e = dlf_launch_gap(&pa, stream);
    } else if (G.kind == GK_PW2) {
        DlfPwArgs wa = G.wa;
        wa.in = in; wa.out = out;
        if (!res) return fail(DLF_ERR_INVALID_ARG, "group [%d,%d] needs its second input", G.first, G.last);
        wa.in2 = res;
        e = dlf_launch_pw(&wa, G.variant, G.grid, stream);
    } else if (G.kind == GK_PW) {
        DlfPwArgs wa = G.wa;
        wa.in = in; wa.out = out;
        if (G.res_stage >= 0) {
            if (!res) return fail(DLF_ERR_INVALID_ARG, "group [%d,%d] needs its residual operand", G.first, G.last);
            wa.res = res;
        }
        e = dlf_launch_pw(&wa, G.variant, G.grid, stream);
    } else if (G.kind == GK_DW) {
        DlfDwArgs da = G.da;
        da.in = in; da.out = out;
        e = dlf_launch_dw(&da, G.grid, stream);
    } else if (G.kind == GK_DWT) {
        DlfDwtArgs dt = G.dt;
        dt.in = in; dt.out = out;
        e = dlf_launch_dwt(&dt, G.grid, G.lds_bytes, stream);
    } else if (G.kind == GK_C3S) {
        DlfC3sArgs cs = G.cs;
        cs.in = in; cs.out = out;
        if (G.res_stage >= 0) {
            if (!res) return fail(DLF_ERR_INVALID_ARG, "group [%d,%d] needs its residual operand", G.first, G.last);
            cs.res = res;
        }
        e = dlf_launch_c3s(&cs, G.grid, G.lds_bytes, stream);
    } else if (G.kind == GK_C3PW) {
        DlfC3PwArgs cp = G.cp;
        cp.in = in; cp.out = out;
        if (G.res_stage >= 0) {
            if (!res) return fail(DLF_ERR_INVALID_ARG, "group [%d,%d] needs its residual operand", G.first, G.last);
            cp.res = res;
        }
        e = dlf_launch_c3pw(&cp, G.grid, G.lds_bytes, stream);
    } else if (G.kind == GK_BNECK) {
        DlfBnArgs bn = G.bn;
        bn.in = in; bn.out = out;
        e = dlf_launch_bneck(&bn, G.grid, G.lds_bytes, stream);
    } else if (G.kind == GK_DWS) {
        DlfDwsArgs ds = G.ds;
        ds.in = in; ds.out = out;
        e = dlf_launch_dws(&ds, G.grid, G.lds_bytes, stream);
    } else if (G.kind == GK_DWPW) {
        DlfDwPwArgs dp = G.dp;
        dp.in = in; dp.out = out;
        e = dlf_launch_dwpw(&dp, G.variant, G.grid, stream);
    } else if (G.kind == GK_C3) {
        DlfC3Args ca = G.ca;
        ca.in = in; ca.out = out;
        if (G.res_stage >= 0) {
            if (!res) return fail(DLF_ERR_INVALID_ARG, "group [%d,%d] needs its residual operand", G.first, G.last);
            ca.res = res;
        }
        e = dlf_launch_c3(&ca, G.variant, G.grid, G.lds_bytes, stream);
    } else {
        DlfGroupArgs ga = G.ga;
        ga.in = in; ga.out = out;
        if (G.res_stage >= 0) {
            if (!res) return fail(DLF_ERR_INVALID_ARG, "group [%d,%d] needs its residual operand", G.first, G.last);
            ga.st[G.res_stage].res = res;
        }
        e = dlf_launch_group(&ga, G.variant, G.grid, G.lds_bytes, stream);
    }
    if (e != 0) return fail(DLF_ERR_HIP, "launch of group [%d,%d] failed: %s", G.first, G.last,
                            hipGetErrorString((hipError_t)e));
    (void)plan;
    return DLF_OK;
}

dlf_status dlf_run_group(const dlf_plan_t* plan, int32_t g, const void* in_dev, const void* res_dev,
                         void* out_dev, void* hip_stream)
{
    if (!plan || g < 0 || g >= (int)plan->G.size() || !in_dev || !out_dev)
        return fail(DLF_ERR_INVALID_ARG, "dlf_run_group: bad argument");
    if (!plan->net->has_weights) return fail(DLF_ERR_NO_WEIGHTS, "network was created without weights");
    return launch_one(plan, plan->G[g], in_dev, res_dev, out_dev, hip_stream, plan->ws);
}

static void group_pointers(const dlf_plan_s* plan, size_t g, const void* in_dev, void* out_dev,
                           const void** in, const void** res, void** out)
{
    const GroupPlan& G = plan->G[g];
    *in = G.in_layer < 0 ? in_dev : plan->ws + plan->layer_off[G.in_layer];
    *res = G.res_stage < 0 ? nullptr : G.res_layer < 0 ? in_dev : plan->ws + plan->layer_off[G.res_layer];
    *out = (g + 1 == plan->G.size()) ? out_dev : (void*)(plan->ws + plan->layer_off[G.last]);
}

dlf_status dlf_plan_refine(dlf_plan_t* plan, const void* in_dev, void* out_dev, void* hip_stream,
                           int32_t top_k, int32_t reps, int32_t* changed)
{
    if (!plan || !in_dev || !out_dev || top_k <= 0 || reps <= 0)
        return fail(DLF_ERR_INVALID_ARG, "dlf_plan_refine: bad argument");
    if (!plan->net->has_weights) return fail(DLF_ERR_NO_WEIGHTS, "network was created without weights");
    if (plan->ws_bytes > 0 && !plan->ws) return fail(DLF_ERR_INVALID_ARG, "no workspace bound");
    const dlf_net_s& net = *plan->net;
    hipStream_t st = (hipStream_t)hip_stream;
    // every group's input must hold real data before groups are timed one by one
    dlf_status rs = dlf_run(plan, in_dev, out_dev, hip_stream);
    if (rs != DLF_OK) return rs;
    if (hipStreamSynchronize(st) != hipSuccess) return fail(DLF_ERR_HIP, "stream synchronise failed");
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return fail(DLF_ERR_HIP, "hipEventCreate failed");
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return fail(DLF_ERR_HIP, "hipEventCreate failed"); }
    // A group is timed the way it runs inside the network: weights and everything else it reads
    // are no longer in the caches (a scratch buffer larger than the last-level cache is rewritten
    // first), except its input, which the group in front of it has just produced.
    const size_t scrub_bytes = (size_t)320 << 20;
    void* scrub = nullptr;
    if (hipMalloc(&scrub, scrub_bytes) != hipSuccess) {
        (void)hipGetLastError();
        scrub = nullptr;                 // no room: time with warm caches
    }
    // candidates take turns, repetition by repetition, so that none of them profits from what the
    // others left behind (page translations, clocks)
    auto time_groups = [&](size_t g, const std::vector<GroupPlan>& list, const void* in, const void* res,
                           void* out, std::vector<float>& ms) {
        dlf_status r = DLF_OK;
        std::vector<double> sum(list.size(), 0.0);
        // a candidate's residual operand is its own: the kernel for a whole bottleneck block takes it
        // from its input, the fused-group kernel on the same layers as a second tensor
        (void)res;
        auto res_of = [&](const GroupPlan& c) -> const void* {
            if (c.res_stage < 0) return nullptr;
            return c.res_layer < 0 ? in_dev : (const void*)(plan->ws + plan->layer_off[c.res_layer]);
        };
        for (size_t i = 0; i < list.size() && r == DLF_OK; ++i)
            r = launch_one(plan, list[i], in, res_of(list[i]), out, hip_stream, plan->ws);          // warm-up
        for (int rep = 0; rep < reps && r == DLF_OK; ++rep)
            for (size_t i = 0; i < list.size() && r == DLF_OK; ++i) {
                if (scrub) (void)hipMemsetAsync(scrub, rep, scrub_bytes, st);
                if (g > 0) {
                    const void *pin, *pres;
                    void* pout;
                    group_pointers(plan, g - 1, in_dev, out_dev, &pin, &pres, &pout);
                    r = launch_one(plan, plan->G[g - 1], pin, pres, pout, hip_stream, plan->ws);
                    if (r != DLF_OK) break;
                }
                (void)hipEventRecord(e0, st);
                r = launch_one(plan, list[i], in, res_of(list[i]), out, hip_stream, plan->ws);
                (void)hipEventRecord(e1, st);
                if (hipEventSynchronize(e1) != hipSuccess && r == DLF_OK)
                    r = fail(DLF_ERR_HIP, "event synchronise failed");
                float t = 0;
                if (r == DLF_OK) { (void)hipEventElapsedTime(&t, e0, e1); sum[i] += t; }
            }
        ms.resize(list.size());
        for (size_t i = 0; i < list.size(); ++i) ms[i] = (float)(sum[i] / reps);
        return r;
    };
    TileCfg none{};
    none.th = 0;
    int nchanged = 0;
    for (size_t g = 0; g < plan->G.size() && rs == DLF_OK; ++g) {
        const GroupPlan cur = plan->G[g];
        if (cur.kind == GK_FC || cur.kind == GK_GAP || cur.kind == GK_PW2) continue;
        const void *in, *res;
        void* out;
        group_pointers(plan, g, in_dev, out_dev, &in, &res, &out);
        std::vector<GroupPlan> cands;
        std::vector<StageSpec> specs;
        std::string why;
        int kind;
        if (!group_stages(net, cur.first, cur.last, specs, kind, why)) continue;
        {   // the top_k tilings by modelled cost
            std::vector<std::pair<uint64_t, TileCfg>> all;
            Built b;
            TileCfg tc;
            uint64_t c = 0;
            choose_group(net, specs, plan->batch, cur.budget, plan->max_lds, b, tc, c, none, &all);
            std::stable_sort(all.begin(), all.end(),
                             [](const std::pair<uint64_t, TileCfg>& x, const std::pair<uint64_t, TileCfg>& y) {
                                 return x.first < y.first;
                             });
            for (size_t i = 0; i < all.size() && (int)i < top_k; ++i) {
                GroupPlan gp;
                const C3Force never = {2, -1, 0, 0};
                if (make_group(net, plan->batch, cur.first, cur.last, cur.budget, plan->max_lds, gp,
                               &all[i].second, 2, &never) == DLF_OK)
                    cands.push_back(gp);
            }
        }
        if (c3_eligible(net, specs, plan->batch)) {
            std::vector<std::pair<uint64_t, C3Cfg>> all;
            C3Cfg cc;
            uint64_t c = 0;
            c3_choose(net.L[cur.first], specs[0].pool2, plan->batch, cur.budget, plan->max_lds, cc, c, &all);
            std::stable_sort(all.begin(), all.end(),
                             [](const std::pair<uint64_t, C3Cfg>& x, const std::pair<uint64_t, C3Cfg>& y) {
                                 return x.first < y.first;
                             });
            for (size_t i = 0; i < all.size() && (int)i < top_k; ++i) {
                GroupPlan gp;
                const C3Force f = {1, all[i].second.shape, all[i].second.th, all[i].second.tw};
                if (make_group(net, plan->batch, cur.first, cur.last, cur.budget, plan->max_lds, gp, &none, 2,
                               &f) == DLF_OK)
                    cands.push_back(gp);
            }
        }
        if (cur.first == cur.last && pw_eligible(net.L[cur.first], plan->batch)) {
            for (int sh = 0; sh < PW_SHAPES; ++sh) {
                if (!pw_shape_ok(net.L[cur.first], sh)) continue;
                GroupPlan gp;
                if (make_group(net, plan->batch, cur.first, cur.last, cur.budget, plan->max_lds, gp, &none,
                               3 + sh) == DLF_OK)
                    cands.push_back(gp);
            }
        }
        cands.insert(cands.begin(), cur);
        std::vector<float> ms;
        rs = time_groups(g, cands, in, res, out, ms);
        if (rs != DLF_OK) break;
        const float cur_ms = ms[0];
        float best_ms = cur_ms;
        int best = -1;
        for (size_t i = 1; i < cands.size(); ++i)
            if (ms[i] < best_ms) { best_ms = ms[i]; best = (int)i; }
        if (getenv("DLF_DEBUG"))
            fprintf(stderr, "dlf_plan_refine [%d,%d]: planned %.2f us (variant %d tile %dx%d), best of %zu: %.2f us (kind %d variant %d tile %dx%d lds %d)\n",
                    cur.first, cur.last, cur_ms * 1e3, cur.variant, cur.th, cur.tw, cands.size() - 1, best_ms * 1e3,
                    best >= 0 ? cands[best].kind : cur.kind, best >= 0 ? cands[best].variant : cur.variant,
                    best >= 0 ? cands[best].th : cur.th, best >= 0 ? cands[best].tw : cur.tw,
                    best >= 0 ? cands[best].lds_bytes : cur.lds_bytes);
        // A candidate replaces the planned configuration only if it is clearly faster: timed one
        // by one, kernels of 15-20 us differ by a microsecond or two from how they run between
        // their neighbours in the network, in either direction.
        if (rs == DLF_OK && best >= 0 && best_ms < cur_ms * 0.90f) {
            plan->G[g] = cands[best];
            ++nchanged;
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (scrub) (void)hipFree(scrub);
    if (rs == DLF_OK && changed) *changed = nchanged;
    return rs;
}

dlf_status dlf_run_profiled(const dlf_plan_t* plan, const void* in_dev, void* out_dev, void* hip_stream,
                            int32_t reps, float* group_ms)
{
    if (!plan || !in_dev || !out_dev || !group_ms || reps <= 0)
        return fail(DLF_ERR_INVALID_ARG, "dlf_run_profiled: bad argument");
    if (!plan->net->has_weights) return fail(DLF_ERR_NO_WEIGHTS, "network was created without weights");
    if (plan->ws_bytes > 0 && !plan->ws) return fail(DLF_ERR_INVALID_ARG, "no workspace bound");
    const size_t ng = plan->G.size();
    hipStream_t st = (hipStream_t)hip_stream;
    // One stop event per launch, stamped by the runtime with the end of that dispatch; a group's
    // duration is the time from the end of the previous dispatch to the end of its own, i.e. the
    // kernel plus the hand-over gap in front of it, which is also what it costs in dlf_run.
    std::vector<hipEvent_t> ev((size_t)ng * reps + 1);
    for (hipEvent_t& e : ev)
        if (hipEventCreate(&e) != hipSuccess) return fail(DLF_ERR_HIP, "hipEventCreate failed");
    dlf_status rs = DLF_OK;
    (void)hipEventRecord(ev[0], st);
    for (int r = 0; r < reps && rs == DLF_OK; ++r)
        for (size_t g = 0; g < ng; ++g) {
            const void *in, *res;
            void* out;
            group_pointers(plan, g, in_dev, out_dev, &in, &res, &out);
            dlf_next_launch_events(nullptr, ev[1 + r * ng + g]);
            rs = launch_one(plan, plan->G[g], in, res, out, hip_stream, plan->ws);
            dlf_next_launch_events(nullptr, nullptr);
            if (rs != DLF_OK) break;
        }
    if (hipStreamSynchronize(st) != hipSuccess && rs == DLF_OK) rs = fail(DLF_ERR_HIP, "stream synchronise failed");
    if (rs == DLF_OK) {
        for (size_t g = 0; g < ng; ++g) {
            double sum = 0;
            for (int r = 0; r < reps; ++r) {
                float ms = 0;
                (void)hipEventElapsedTime(&ms, ev[r * ng + g], ev[1 + r * ng + g]);
                sum += ms;
            }
            group_ms[g] = (float)(sum / reps);
        }
    }
    for (hipEvent_t& e : ev) (void)hipEventDestroy(e);
    return rs;
}

dlf_status dlf_run(const dlf_plan_t* plan, const void* in_dev, void* out_dev, void* hip_stream)
{
    if (!plan || !in_dev || !out_dev) return fail(DLF_ERR_INVALID_ARG, "dlf_run: null argument");
    if (!plan->net->has_weights) return fail(DLF_ERR_NO_WEIGHTS, "network was created without weights");
    if (plan->ws_bytes > 0 && !plan->ws) return fail(DLF_ERR_INVALID_ARG, "no workspace bound");
    const size_t ng = plan->G.size();
    bool any_side = false;
    if (plan->overlap)
        for (size_t g = 0; g < ng; ++g) any_side = any_side || plan->on_side[g] != 0;
    if (any_side && plan->side == nullptr) {
        // created on first use, with the default priority
        if (hipStreamCreateWithFlags(&plan->side, hipStreamNonBlocking) != hipSuccess)
            return fail(DLF_ERR_HIP, "hipStreamCreateWithFlags failed");
        plan->done.assign(ng, nullptr);
        for (size_t g = 0; g < ng; ++g) {
            bool watched = false;      // does a group on the other stream read this group's output?
            for (size_t c = g + 1; c < ng; ++c)
                if ((plan->dep_a[c] == (int)g || plan->dep_b[c] == (int)g) && plan->on_side[c] != plan->on_side[g])
                    watched = true;
            if (watched && hipEventCreateWithFlags(&plan->done[g], hipEventDisableTiming) != hipSuccess)
                return fail(DLF_ERR_HIP, "hipEventCreate failed");
        }
        if (hipEventCreateWithFlags(&plan->side_end, hipEventDisableTiming) != hipSuccess)
            return fail(DLF_ERR_HIP, "hipEventCreate failed");
    }
    hipStream_t main_s = (hipStream_t)hip_stream;
    if (any_side) {
        // the second stream starts behind everything the caller's stream holds at this point (the
        // producer of the network input, the previous run's readers of the buffers about to be
        // rewritten), not behind the groups of this run
        if (hipEventRecord(plan->side_end, main_s) != hipSuccess ||
            hipStreamWaitEvent(plan->side, plan->side_end, 0) != hipSuccess)
            return fail(DLF_ERR_HIP, "stream fork failed");
    }
    for (size_t g = 0; g < ng; ++g) {
        const GroupPlan& G = plan->G[g];
        const void* in = G.in_layer < 0 ? in_dev : plan->ws + plan->layer_off[G.in_layer];
        const void* res = nullptr;
        if (G.res_stage >= 0) res = G.res_layer < 0 ? in_dev : plan->ws + plan->layer_off[G.res_layer];
        void* out = (g + 1 == ng) ? out_dev : (void*)(plan->ws + plan->layer_off[G.last]);
        hipStream_t st = main_s;
        if (any_side) {
            const int side = plan->on_side[g];
            st = side ? plan->side : main_s;
            const int deps[2] = {plan->dep_a[g], plan->dep_b[g]};
            for (int d : deps)
                if (d >= 0 && plan->on_side[d] != side && plan->done[d] != nullptr &&
                    hipStreamWaitEvent(st, plan->done[d], 0) != hipSuccess)
                    return fail(DLF_ERR_HIP, "hipStreamWaitEvent failed");
        }
        dlf_status s = launch_one(plan, G, in, res, out, (void*)st, plan->ws);
        if (s != DLF_OK) return s;
        if (any_side && plan->done[g] != nullptr && hipEventRecord(plan->done[g], st) != hipSuccess)
            return fail(DLF_ERR_HIP, "hipEventRecord failed");
    }
    if (any_side) {
        // join: whatever follows on the caller's stream comes after the second stream's work
        if (hipEventRecord(plan->side_end, plan->side) != hipSuccess ||
            hipStreamWaitEvent(main_s, plan->side_end, 0) != hipSuccess)
            return fail(DLF_ERR_HIP, "stream join failed");
    }
    return DLF_OK;
}

// Device address of this GPU's copy of the static workspace, looked up once per device.
static dlf_status static_workspace(char** base)
{
    static std::mutex mu;
    static void* ptr[DLF_MAX_DEVICES] = {nullptr};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(DLF_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= DLF_MAX_DEVICES) return fail(DLF_ERR_UNSUPPORTED, "device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(mu);
    if (ptr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || p == nullptr)
            return fail(DLF_ERR_HIP, "hipGetSymbolAddress(static workspace): %s", hipGetErrorString(e));
        ptr[dev] = p;
    }
    *base = (char*)ptr[dev];
    return DLF_OK;
}

// ------------------------------------------------------------------------------------------
// Quantised (int8) convolution layer on the block kernels (3x3: k_c3b, 1x1: k_pwb)
// ------------------------------------------------------------------------------------------

struct dlf_i8conv_s {
    int ksize = 3;
    bool small_map = false;      // runs on the small-map kernel (cs), else on a block kernel (ca / wa)
    DlfC3Args ca;
    DlfPwArgs wa;
    DlfC3sArgs cs;
    int th = 0, tw = 0;
    int shape = 0, grid = 0, lds_bytes = 0;
    uint64_t ops = 0;
    void* d_w = nullptr;
    float* d_scale = nullptr;
    float* d_bias = nullptr;
};

void dlf_i8conv_destroy(dlf_i8conv_t* l)
{
    if (!l) return;
    if (l->d_w) (void)hipFree(l->d_w);
    if (l->d_scale) (void)hipFree(l->d_scale);
    if (l->d_bias) (void)hipFree(l->d_bias);
    delete l;
}

dlf_status dlf_i8conv_create(int32_t batch, int32_t h, int32_t w, int32_t cin, int32_t cout, int32_t ksize,
                             int32_t relu, int32_t pool, const int8_t* weight, const float* scale, const float* bias, int32_t budget,
                             dlf_i8conv_t** out)
{
    if (!out) return fail(DLF_ERR_INVALID_ARG, "dlf_i8conv_create: null out pointer");
    if (batch < 1 || h < 1 || w < 1 || cin < 1 || cout < 1 || h > (1 << 20) || w > (1 << 20) || cin > (1 << 20) ||
        cout > (1 << 20))
        return fail(DLF_ERR_INVALID_ARG, "dlf_i8conv_create: sizes out of range");
    if (weight && (!scale || !bias)) return fail(DLF_ERR_INVALID_ARG, "dlf_i8conv_create: weights without scale / bias");
    if (ksize != 1 && ksize != 3) return fail(DLF_ERR_UNSUPPORTED, "the int8 layer is a 1x1 or a 3x3 convolution");
    if (pool != 0 && pool != 1) return fail(DLF_ERR_INVALID_ARG, "dlf_i8conv_create: pool is 0 or 1");
    if (pool && (ksize != 3 || h < 2 || w < 2))
        return fail(DLF_ERR_UNSUPPORTED, "the 2x2 max pool folds into the 3x3 layer only, on maps of at least 2 x 2");
    if ((cin % 64) != 0 || (cout % 16) != 0)
        return fail(DLF_ERR_UNSUPPORTED, "the int8 layer needs cin %% 64 == 0 and cout %% 16 == 0");
    if ((int64_t)batch * h * w * cin >= (int64_t)1 << 31 || (int64_t)batch * h * w * cout >= (int64_t)1 << 31)
        return fail(DLF_ERR_UNSUPPORTED, "the int8 layer needs tensors below 2 GiB");
    if (budget <= 0 || budget > 256) budget = 256;
    // to the operand path an int8 tensor of cin channels is an fp16 tensor of cin / 2
    Layer L;
    memset(&L.d, 0, sizeof L.d);
    const int taps = ksize * ksize;
    L.d.op = DLF_CONV; L.d.cin = cin / 2; L.d.cout = cout; L.d.kh = L.d.kw = ksize; L.d.stride = 1; L.d.pad = ksize / 2;
    L.d.residual_from = -1; L.d.input_from = -1;
    L.in_h = L.out_h = h; L.in_w = L.out_w = w; L.in_c = cin / 2; L.out_c = cout;
    L.kc = 32; L.cin_pad = cin / 2; L.ncb = ceil_div(cout, 32); L.nsteps = (L.cin_pad / 32) * taps * 2;
    std::unique_ptr<dlf_i8conv_s> l(new dlf_i8conv_s);
    l->ksize = ksize;
    l->ops = (uint64_t)2 * batch * h * w * taps * (uint64_t)cin * cout;
    memset(&l->ca, 0, sizeof l->ca);
    memset(&l->wa, 0, sizeof l->wa);
    memset(&l->cs, 0, sizeof l->cs);
    C3Cfg cc;
    uint64_t cost = 0;
    // Maps of many channels and few pixels: the small-map kernel, where it applies (512 .. 4096 int8
    // channels) and its modelled cost is below the block kernel's.  Testing hook: shape DLF_C3_SHAPES
    // forces it (th > 0: the split of K), a block shape excludes it.
    DlfC3sArgs cs;
    uint64_t cost_s = 0;
    bool have_s = false;
    if (c3s_cin_ok(L.d.cin) && !(g_c3_force.shape >= 0 && g_c3_force.shape < DLF_C3_SHAPES)) {
        if (g_c3_force.shape == DLF_C3_SHAPES && g_c3_force.th > 0) {
            have_s = c3s_build(L, batch, g_c3_force.th, 0, 0, 160 * 1024, cs, pool);
            if (!have_s) return fail(DLF_ERR_INFEASIBLE, "the forced split of K does not fit this layer");
        } else {
            have_s = c3s_choose(L, batch, budget, 160 * 1024, cs, cost_s, pool);
        }
        if (have_s && g_c3_force.shape != DLF_C3_SHAPES) {
            uint64_t other = UINT64_MAX;
            C3Cfg c2;
            if (ksize == 1) other = pw_shape_cost_ps(L, batch, budget, pw_shape_ok(L, 3) ? 3 : 4);
            else if (!c3_choose(L, pool, batch, budget, 160 * 1024, c2, other)) other = UINT64_MAX;
            if (other <= cost_s) have_s = false;
        }
    } else if (g_c3_force.shape == DLF_C3_SHAPES) {
        return fail(DLF_ERR_INFEASIBLE, "the small-map kernel does not take this channel count");
    }
    if (have_s) {
        l->small_map = true;
        l->cs = cs;
        l->cs.act = relu ? 1 : 0;
        l->shape = DLF_C3_SHAPES;
        l->grid = cs.slice_major ? ceil_div(cs.ntiles, 8 / cs.nsl) * 8 : ceil_div(cs.ntiles, 8) * 8 * cs.nsl;
        l->lds_bytes = (int)DLF_C3S_LDS_BYTES(cs.rp, cs.cin);
        l->th = cs.th; l->tw = cs.tw;
    } else if (ksize == 1) {
        // the block pointwise kernel: 128 channels x 128 pixels per workgroup, or 64 x 256 for few channels
        const int shape = pw_shape_ok(L, 3) ? 3 : 4;
        DlfPwArgs& wa = l->wa;
        wa.m = batch * h * w;
        wa.cin = cin / 2; wa.cout = cout; wa.ncb = L.ncb; wa.nsteps = L.nsteps;
        wa.act = relu ? 1 : 0; wa.stride = 1;
        wa.in_h = wa.out_h = h; wa.in_w = wa.out_w = w;
        wa.n_pg = ceil_div(wa.m, 32 * PW_FP[shape]); wa.n_cg = ceil_div(L.ncb, PW_FC[shape]);
        wa.nitems = wa.n_pg * wa.n_cg;
        l->shape = shape;
        l->grid = std::max(8, std::min(budget * 2, ceil_div(wa.nitems, 8) * 8) / 8 * 8);
        l->th = 1; l->tw = 32 * PW_FP[shape];
    } else {
    if (g_c3_force.shape >= 0 && g_c3_force.shape < DLF_C3_SHAPES) {      // testing hook: shape and tile as given
        if (!c3_build(pool, L.d.cin, g_c3_force.shape, g_c3_force.th, g_c3_force.tw, 160 * 1024, cc))
            return fail(DLF_ERR_INFEASIBLE, "the forced shape and tile do not fit this layer");
    } else if (!c3_choose(L, pool, batch, budget, 160 * 1024, cc, cost))
        return fail(DLF_ERR_INFEASIBLE, "no tile of the block kernel fits this layer");
    DlfC3Args& ca = l->ca;
    ca.batch = batch; ca.h = h; ca.w_ = w; ca.cin = cin / 2; ca.cout = cout;
    ca.ncb = L.ncb; ca.nsteps = L.nsteps; ca.act = relu ? 1 : 0; ca.pool2 = pool;
    ca.th = cc.th; ca.tw = cc.tw;
    ca.tiles_y = ceil_div(h, cc.th); ca.tiles_x = ceil_div(w, cc.tw);
    ca.n_cg = ceil_div(L.ncb, 2 * C3_WC[cc.shape]);
    ca.ntiles = batch * ca.tiles_y * ca.tiles_x;
    ca.nitems = ca.n_cg * ca.ntiles;
    ca.npxh = cc.npxh; ca.na_i = cc.na_i; ca.lpw_a = cc.lpw_a; ca.nst = cc.nst;
    l->shape = cc.shape;
    l->grid = std::max(8, std::min(budget, ceil_div(ca.nitems, 8) * 8) / 8 * 8);
    l->lds_bytes = cc.lds_bytes;
    l->th = cc.th; l->tw = cc.tw;
    }
    if (weight) {
        std::vector<uint16_t> packed;
        pack_conv_weights((const uint16_t*)weight, cout, taps, cin / 2, 32, cin / 2, packed);
        dlf_status s = upload(packed.data(), packed.size() * 2, &l->d_w);
        if (s != DLF_OK) { dlf_i8conv_destroy(l.release()); return s; }
        std::vector<float> sc((size_t)L.ncb * 32, 0.0f), bi((size_t)L.ncb * 32, 0.0f);
        std::copy(scale, scale + cout, sc.begin());
        std::copy(bias, bias + cout, bi.begin());
        s = upload(sc.data(), sc.size() * 4, (void**)&l->d_scale);
        if (s == DLF_OK) s = upload(bi.data(), bi.size() * 4, (void**)&l->d_bias);
        if (s != DLF_OK) { dlf_i8conv_destroy(l.release()); return s; }
        l->ca.w = l->wa.w = l->cs.w = l->d_w;
        l->ca.scale = l->wa.scale = l->cs.scale = l->d_scale;
        l->ca.bias = l->wa.bias = l->cs.bias = l->d_bias;
    }
    *out = l.release();
    return DLF_OK;
}

dlf_status dlf_i8conv_info(const dlf_i8conv_t* l, int32_t* th, int32_t* tw, int32_t* shape, int32_t* grid,
                           uint64_t* op_count)
{
    if (!l) return fail(DLF_ERR_INVALID_ARG, "dlf_i8conv_info: null layer");
    if (th) *th = l->th;
    if (tw) *tw = l->tw;
    if (shape) *shape = l->shape;
    if (grid) *grid = l->grid;
    if (op_count) *op_count = l->ops;
    return DLF_OK;
}

dlf_status dlf_i8conv_run(const dlf_i8conv_t* l, const void* in_dev, void* out_dev, void* hip_stream)
{
    if (!l || !in_dev || !out_dev) return fail(DLF_ERR_INVALID_ARG, "dlf_i8conv_run: null argument");
    if (!l->d_w) return fail(DLF_ERR_NO_WEIGHTS, "the layer was created without weights");
    if ((((uintptr_t)in_dev | (uintptr_t)out_dev) & 15) != 0)
        return fail(DLF_ERR_INVALID_ARG, "dlf_i8conv_run: tensors must be 16-byte aligned");
    std::call_once(g_kernels_once, [] { g_kernels_rc = dlf_kernels_init(); });
    if (g_kernels_rc != 0)
        return fail(DLF_ERR_HIP, "kernel setup failed: %s", hipGetErrorString((hipError_t)g_kernels_rc));
    int e;
    if (l->small_map) {
        DlfC3sArgs cs = l->cs;
        cs.in = in_dev; cs.out = out_dev;
        e = dlf_launch_c3s(&cs, l->grid, l->lds_bytes, hip_stream);
    } else if (l->ksize == 1) {
        DlfPwArgs wa = l->wa;
        wa.in = in_dev; wa.out = out_dev;
        e = dlf_launch_pw_i8(&wa, l->shape, l->grid, hip_stream);
    } else {
        DlfC3Args ca = l->ca;
        ca.in = in_dev; ca.out = out_dev;
        e = dlf_launch_c3_i8(&ca, l->shape, l->grid, l->lds_bytes, hip_stream);
    }
    if (e != 0) return fail(DLF_ERR_HIP, "launch of the int8 layer failed: %s", hipGetErrorString((hipError_t)e));
    return DLF_OK;
}

size_t dlf_static_workspace_bytes(void) { return DLF_STATIC_WS_BYTES; }

dlf_status dlf_run_noalloc(const dlf_plan_t* plan, const void* in_dev, void* out_dev, void* hip_stream)
{
    if (!plan || !in_dev || !out_dev) return fail(DLF_ERR_INVALID_ARG, "dlf_run_noalloc: null argument");
    if (!plan->net->has_weights) return fail(DLF_ERR_NO_WEIGHTS, "network was created without weights");
    if (plan->ws_bytes > DLF_STATIC_WS_BYTES)
        return fail(DLF_ERR_OOM, "dlf_run_noalloc: the plan needs %zu bytes of workspace, the static one holds %zu",
                    plan->ws_bytes, (size_t)DLF_STATIC_WS_BYTES);
    char* ws = nullptr;
    dlf_status s = static_workspace(&ws);
    if (s != DLF_OK) return s;
    // every group in order on the caller's stream: nothing here creates a stream or an event
    const size_t ng = plan->G.size();
    for (size_t g = 0; g < ng; ++g) {
        const GroupPlan& G = plan->G[g];
        const void* in = G.in_layer < 0 ? in_dev : ws + plan->layer_off[G.in_layer];
        const void* res = G.res_stage < 0 ? nullptr : G.res_layer < 0 ? in_dev : ws + plan->layer_off[G.res_layer];
        void* out = (g + 1 == ng) ? out_dev : (void*)(ws + plan->layer_off[G.last]);
        s = launch_one(plan, G, in, res, out, hip_stream, ws);
        if (s != DLF_OK) return s;
    }
    return DLF_OK;
}

dlf_status dlf_plan_set_overlap(dlf_plan_t* plan, int32_t on)
{
    if (!plan) return fail(DLF_ERR_INVALID_ARG, "null plan");
    plan->overlap = on != 0;
    return DLF_OK;
}

int32_t dlf_plan_group_stream(const dlf_plan_t* plan, int32_t g)
{
    if (!plan || g < 0 || g >= (int)plan->G.size()) return -1;
    return plan->overlap ? plan->on_side[g] : 0;
}

}  // extern "C"
