// gfx950 (CDNA4) kernels of libdlf.
//
// k_group: one workgroup executes a fusion group (paper Sec. III-B: consecutive layers run as one
// block, intermediates on chip, halo recomputed per tile) on one tile at a time, looping over
// tiles persistently (grid size = the group's workgroup budget, the analogue of the paper's MP).
//
// Convolution stages are implicit GEMMs on v_mfma_f32_32x32x16_f16:
//     D[co][pixel] += W[co][k] * X[k][pixel],   k = (kh, kw, ci)
// The weights are the MFMA "A" operand (32 output channels x 16 k), pre-packed on the host in
// exactly the register layout, so a wave fetches one 1 KiB fragment with one coalesced 16-byte
// load per lane, straight from L2 into registers.  The activations are the "B" operand
// (16 k x 32 pixels), read from LDS where a pixel's channels are contiguous (NHWC), so the
// im2col gather is just an address offset per filter tap.  With this orientation each lane ends
// up holding 4 consecutive output channels of one pixel, which is what an NHWC store wants.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <type_traits>
#include "dlf_internal.h"

typedef _Float16 half_t;
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef float f4v __attribute__((ext_vector_type(4)));
typedef unsigned u4v __attribute__((ext_vector_type(4)));
typedef unsigned u2v __attribute__((ext_vector_type(2)));

extern __shared__ __attribute__((aligned(16))) half_t lds[];

// A byte offset no tensor reaches (the host keeps tensors that are read through buffer resources
// below 2 GiB): a buffer load at this offset fails the hardware's range check and returns zeros.
#define DLF_OOB ((int)0x80000000)
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i16v __attribute__((ext_vector_type(16)));
template <bool I8> struct AccOf { typedef f16v type; };
template <> struct AccOf<true> { typedef i16v type; };
// Requantisation of one accumulator: (float)acc, one fused multiply-add with the channel's scale and bias,
// clamp, round half to even.  The clamp comes first (the bounds are integers and rounding is monotone, so
// the result is that of rounding first), and the rounding is the addition of 1.5 * 2^23, whose fp32 sum has
// a unit in the last place of 1: the sum is the rounded value, and the low byte of its bit pattern is the
// result as a two's-complement int8.  Four vector instructions per output, and the maximum of a pooling
// window can be taken on the sums as they are.
__device__ __forceinline__ float requant_biased(int acc, float sc, float bi, float lo)
{
    const float t = __builtin_fmaf((float)acc, sc, bi);
    return __builtin_amdgcn_fmed3f(t, lo, 127.0f) + 12582912.0f;
}
// ... and the low bytes of four such sums as one dword (three byte permutes)
__device__ __forceinline__ unsigned pack_low_bytes(float a, float b, float c, float d)
{
    const unsigned ab = __builtin_amdgcn_perm(__builtin_bit_cast(unsigned, b), __builtin_bit_cast(unsigned, a), 0x0c0c0400u);
    const unsigned cd = __builtin_amdgcn_perm(__builtin_bit_cast(unsigned, d), __builtin_bit_cast(unsigned, c), 0x0c0c0400u);
    return __builtin_amdgcn_perm(cd, ab, 0x05040100u);
}
// Transpose buffer of the quantised epilogues: rows of 64 bytes (a wave's 64 int8 channels of one
// pixel), written one dword per lane by 32 lanes that hold 32 consecutive rows, read 16 bytes per
// lane.  Row r keeps its 16-byte part c at position c ^ (r / 2) % 4 and, inside a part, dword d at
// d ^ (r / 8) % 4: with bit 4 of the bank number being r % 2, the 32 rows of a write fall into 32
// different banks.  A reader takes the part as it lies and undoes the dword permutation in registers.
__device__ __forceinline__ int i8t_write_off(int row, int c16, int d)
{
    return row * 64 + (((c16 ^ (row >> 1)) & 3) << 4) + (((d ^ (row >> 3)) & 3) << 2);
}
__device__ __forceinline__ u4v i8t_read(const unsigned char* tb, int row, int part)
{
    const u4v v = *(const u4v*)(tb + row * 64 + (((part ^ (row >> 1)) & 3) << 4));
    const int k = row >> 3;
    const u4v a = (k & 1) ? u4v{v.y, v.x, v.w, v.z} : v;
    return (k & 2) ? u4v{a.z, a.w, a.x, a.y} : a;
}
__device__ i32x4 raw_buffer_load_x4(i32x4 rsrc, int voffset, int soffset, int aux) __asm("llvm.amdgcn.raw.buffer.load.v4i32");
__device__ __forceinline__ i32x4 make_rsrc(const void* p, unsigned bytes)
{
    const unsigned long long a = (unsigned long long)p;
    i32x4 r;
    r.x = __builtin_amdgcn_readfirstlane((int)(unsigned)a);
    r.y = __builtin_amdgcn_readfirstlane((int)((unsigned)(a >> 32) & 0xffffu));   // stride 0: raw buffer
    r.z = __builtin_amdgcn_readfirstlane((int)bytes);                              // bytes that may be read
    r.w = 0x00020000;                                                              // 32-bit raw data
    return r;
}


// 16 bytes per lane of the packed weights, read through a buffer resource: address = base +
// 16 * lane + a uniform byte offset (a scalar register).  The per-lane part never changes, so a
// wave's walk through its fragments is scalar arithmetic only.  (A per-lane 64-bit pointer would be
// stepped with 64-bit vector instructions, and those get a slot on a SIMD only when its matrix
// pipe pauses: under MFMA load the weight stream of such a loop runs at a fraction of its rate.)
__device__ __forceinline__ h8 wfrag(const i32x4 rw, int lane16, unsigned soff)
{
    return __builtin_bit_cast(h8, raw_buffer_load_x4(rw, lane16, (int)soff, 0));
}

__device__ __forceinline__ float apply_act(float v, int act)
{
    if (act >= 1) v = fmaxf(v, 0.0f);
    if (act == 2) v = fminf(v, 6.0f);
    return v;
}

// Division of a small non-negative integer by a wave-uniform divisor d as one multiply:
// q = (n * m) >> 32 with m = floor((2^32 - 1) / d) + 1, exact while n * d < 2^32 (d = 1 wraps m to
// 0, which stands for "divide by one").  The general integer division costs some 40 vector
// instructions; the address arithmetic of staging, epilogue and store phases is full of them.
__device__ __forceinline__ unsigned div_magic(int d) { return 0xFFFFFFFFu / (unsigned)d + 1u; }
__device__ __forceinline__ int div_by(int n, unsigned m)
{
    return m == 0 ? n : (int)__umulhi((unsigned)n, m);
}

// Region pixel index -> (row, col); rw_m = div_magic(rw), or div_magic(rw / 2) with `quad`.  With
// `quad` the 4 pixels of a 2x2 pooling window are consecutive indices, so they sit in 4 adjacent
// lanes of the MFMA result.
__device__ __forceinline__ void pix_to_rc(int p, int rw, unsigned rw_m, int quad, int& ry, int& rx)
{
    if (quad) {
        const int q = p >> 2, d = p & 3, hw = rw >> 1;
        const int qy = div_by(q, rw_m), qx = q - qy * hw;
        ry = 2 * qy + (d >> 1);
        rx = 2 * qx + (d & 1);
    } else {
        ry = div_by(p, rw_m);
        rx = p - ry * rw;
    }
}

// Two packed fp16 values per 32-bit register: max / min / add on both halves at once.
__device__ __forceinline__ unsigned pk_max(unsigned a, unsigned b)
{
    unsigned r;
    asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ unsigned pk_min(unsigned a, unsigned b)
{
    unsigned r;
    asm("v_pk_min_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ unsigned pk_add(unsigned a, unsigned b)
{
    unsigned r;
    asm("v_pk_add_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
// Rounds two fp32 values to fp16 (nearest even) into one register.
__device__ __forceinline__ unsigned cvt_pk(float a, float b)
{
    typedef float f2v __attribute__((ext_vector_type(2)));
    typedef _Float16 h2v __attribute__((ext_vector_type(2)));
    const f2v f = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f, h2v));
}
// The activation as a clamp on packed fp16: none = [-inf, +inf], ReLU = [0, +inf], ReLU6 = [0, 6].
// Clamping after the rounding to fp16 gives the same result as before it: rounding is monotone
// and 0 and 6 are exact in fp16.
__device__ __forceinline__ unsigned act_lo(int act) { return act == 0 ? 0xFC00FC00u : 0u; }
__device__ __forceinline__ unsigned act_hi(int act) { return act == 2 ? 0x46004600u : 0x7C007C00u; }

// Output of the block pointwise kernel: to memory with the streaming hint (nothing in the same
// launch reads it again).  Measured per kernel: it shortens k_pwb's launches by 1 - 3 us; on the
// outputs of the other kernels the next layer loses what the storing one gains.
__device__ __forceinline__ void store_out(half_t* p, u4v v) { __builtin_nontemporal_store(v, (u4v*)p); }

__device__ __forceinline__ unsigned quad_max_pk(unsigned v)
{
    // max over the 4 lanes of a quad with two DPP quad permutes: [1,0,3,2] then [2,3,0,1]
    unsigned o = (unsigned)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);
    v = pk_max(v, o);
    o = (unsigned)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);
    return pk_max(v, o);
}

// Loads 8 channels [c, c+8) of input pixel (n, gy, gx); zero outside the image or beyond c_end.
__device__ __forceinline__ h8 load_px8(const half_t* in, int n, int gy, int gx, int H, int W,
                                       int C, int c, int c_end)
{
    h8 v = {0, 0, 0, 0, 0, 0, 0, 0};
    if (gy >= 0 && gy < H && gx >= 0 && gx < W && c < c_end) {
        // the host rejects tensors of 2^31 elements or more, so offsets fit 32 bits
        const half_t* p = in + (unsigned)(((n * H + gy) * W + gx) * C + c);
        if ((C & 7) == 0 && c + 8 <= c_end) {
            v = *(const h8*)p;
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = (c + j < c_end) ? p[j] : (half_t)0;
        }
    }
    return v;
}

// Copies the input region [iy0, iy0+ih) x [ix0, ix0+iw), channels [c0, c0+cfill), into LDS as
// [pixel][cs]; zero padding outside the image and beyond channel c_end.
__device__ __forceinline__ void stage_region(const half_t* in, int n, int H, int W, int C,
                                             int iy0, int ix0, int ih, int iw, int c0, int cfill,
                                             int c_end, int cs, half_t* dst)
{
    const int nvec = cfill >> 3;
    const int total = ih * iw * nvec;
    const unsigned nvec_m = div_magic(nvec), iw_m = div_magic(iw);
    // Batches of 8 parts per thread, loaded and then stored.  Each load sits under its own bounds
    // check, and the compiler waits for it at the end of that branch, so the eight round trips of
    // a batch follow one another.  A form without branches (every lane loads from a clamped
    // address, the value is chosen afterwards) does issue all eight at once, and measured 1-2 %
    // slower on whole networks: with two workgroups per CU the other workgroup's multiply phase
    // already covers this one's latency, and the burst only adds contention.
    constexpr int U = 8;
    for (int v0 = threadIdx.x; v0 < total; v0 += DLF_WG_THREADS * U) {
        h8 val[U];
        int doff[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int v = v0 + u * DLF_WG_THREADS;
            if (v < total) {
                const int pix = div_by(v, nvec_m), part = v - pix * nvec;
                const int ry = div_by(pix, iw_m), rx = pix - ry * iw;
                doff[u] = pix * cs + part * 8;
                val[u] = load_px8(in, n, iy0 + ry, ix0 + rx, H, W, C, c0 + part * 8, c_end);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int v = v0 + u * DLF_WG_THREADS;
            if (v < total) *(h8*)(dst + doff[u]) = val[u];
        }
    }
}

// Pointers with their address space spelled out, for the helpers below that are not inlined: a
// plain pointer is generic there and every access becomes a flat one, which waits on both memory
// counters at once and serialises what should be a batch of independent loads.
typedef const __attribute__((address_space(1))) half_t* gconst_h;
typedef __attribute__((address_space(3))) half_t* lds_h;
typedef __attribute__((address_space(3))) u4v* lds_u4v;
typedef __attribute__((address_space(3))) h4* lds_h4;

// im2col staging for a convolution on a narrow input (3 channels): LDS row p holds the
// kh*kw*cin inputs of output pixel p in (kh, kw, ci) order, zero padded to kfill halfs, so that the
// convolution becomes a 1x1 convolution over kfill channels: K = 27 -> 32 for a 3x3 filter on RGB
// instead of 9 taps x 32 padded channels.
__device__ __forceinline__ void stage_im2col_direct(const half_t* in_, int n, int H, int W, int C, int oy0,
                                             int ox0, int rh, int rw, int kh, int kw, int stride,
                                             int pad, int kfill, int cs, half_t* dst_)
{
    const gconst_h in = (gconst_h)in_;
    const lds_h dst = (lds_h)dst_;
    const int rowlen = kw * C;                     // contiguous in NHWC
    const int total = rh * rw * kh;
    for (int v = threadIdx.x; v < total; v += DLF_WG_THREADS) {
        const int pix = v / kh, r = v - pix * kh;
        const int oy = pix / rw, ox = pix - oy * rw;
        const int iy = (oy0 + oy) * stride - pad + r;
        const int ix0 = (ox0 + ox) * stride - pad;
        const lds_h d = dst + pix * cs + r * rowlen;
        const bool rowok = iy >= 0 && iy < H;
        const gconst_h src = in + (((size_t)n * H + (rowok ? iy : 0)) * W) * C;
        for (int j = 0; j < rowlen; ++j) {
            const int ix = ix0 + j / C;
            half_t val = (half_t)0;
            if (rowok && ix >= 0 && ix < W) val = src[ix0 * C + j];
            d[j] = val;
        }
        if (r == kh - 1)
            for (int j = kh * rowlen; j < kfill; ++j) dst[pix * cs + j] = (half_t)0;
    }
}

// The same in two steps through LDS, where a spare area `tmp` is at hand (the stage's output buffer,
// not yet in use; it must hold the patch and one half more): the input patch [ih][iw][C] is
// brought in first, rows of the image being contiguous in memory, zero outside the image; the
// im2col rows are then copied out of it -- a filter row of an output pixel is kw * C consecutive
// halfs of a patch row.  No bounds checks, no global access and no division by a run-time value
// per element in the second step.
__device__ __forceinline__ void stage_im2col_lds(const half_t* in_, int n, int H, int W, int C, int oy0,
                                                 int ox0, int rh, int rw, int kh, int kw, int stride,
                                                 int pad, int kfill, int cs, half_t* tmp_, half_t* dst_)
{
    const gconst_h in = (gconst_h)in_;
    const lds_h tmp = (lds_h)tmp_, dst = (lds_h)dst_;
    const int ih = (rh - 1) * stride + kh, iw = (rw - 1) * stride + kw;
    const int iy0 = oy0 * stride - pad, ix0 = ox0 * stride - pad;
    const int rowh = iw * C;                       // halfs per patch row
    const unsigned rowh_m = div_magic(rowh), c_m = div_magic(C);
    // batches of 4 loads per thread are issued before any is stored: the round trip to HBM is paid
    // once per batch, not once per element
    constexpr int U = 4;
    const int ptotal = ih * rowh;
    for (int v0 = threadIdx.x; v0 < ptotal; v0 += DLF_WG_THREADS * U) {
        half_t val[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int v = v0 + u * DLF_WG_THREADS;
            // every lane loads, from the nearest element inside the image where it has nothing to
            // fetch, and the value is chosen afterwards: a load under a divergent branch is waited
            // for at the end of its branch
            const int vv = min(v, ptotal - 1);
            const int r = div_by(vv, rowh_m), j = vv - r * rowh;
            const int px = div_by(j, c_m), ch = j - px * C;
            const int gy = iy0 + r, gx = ix0 + px;
            const bool ok = v < ptotal && gy >= 0 && gy < H && gx >= 0 && gx < W;
            const int gyc = min(max(gy, 0), H - 1), gxc = min(max(gx, 0), W - 1);
            const half_t x = in[(unsigned)(((n * H + gyc) * W + gxc) * C + ch)];
            val[u] = ok ? x : (half_t)0;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int v = v0 + u * DLF_WG_THREADS;
            if (v < ptotal) tmp[v] = val[u];
        }
    }
    if (threadIdx.x == 0) tmp[ptotal] = (half_t)0;                 // the zero that row padding reads
    __syncthreads();
    // One task = 8 consecutive k of one output pixel, written with a single 16-byte store.  Along k a
    // pixel's row is kh runs of kw*C halfs, each contiguous in the patch.  This phase is bound by
    // vector ALU issue (four waves share a SIMD), so what counts is instructions per element.
    const int rowlen = kw * C, per_pix = kh * rowlen, nq = kfill >> 3;
    const unsigned nq_m = div_magic(nq), rowlen_m = div_magic(rowlen), rw_m = div_magic(rw);
    if (DLF_WG_THREADS % nq == 0) {
        // The workgroup's stride is a multiple of the parts per row, so a thread serves the same part
        // of every row it visits: the eight offsets of its elements inside a pixel's window are
        // found once (padding beyond kh*kw*C points at the zero behind the patch), and an element
        // costs one addition and one read.
        const int j0 = (int)(threadIdx.x % (unsigned)nq) << 3;
        int off[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int j = j0 + e, r = div_by(j, rowlen_m);
            off[e] = j < per_pix ? r * rowh + (j - r * rowlen) : -1;
        }
        for (int u = threadIdx.x; u < rh * rw * nq; u += DLF_WG_THREADS) {
            const int pix = div_by(u, nq_m);
            const int oy = div_by(pix, rw_m), ox = pix - oy * rw;
            const int base = oy * stride * rowh + ox * stride * C;
            half_t v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = tmp[off[e] < 0 ? ptotal : base + off[e]];
            *(lds_u4v)(dst + pix * cs + j0) = *(const u4v*)v;
        }
        return;
    }
    // otherwise the source index is stepped along the row, with a jump at the end of each run
    for (int u = threadIdx.x; u < rh * rw * nq; u += DLF_WG_THREADS) {
        const int pix = div_by(u, nq_m), j0 = (u - pix * nq) << 3;
        const int oy = div_by(pix, rw_m), ox = pix - oy * rw;
        const int r = div_by(j0, rowlen_m);
        int jj = j0 - r * rowlen;
        int src = (oy * stride + r) * rowh + ox * stride * C + jj;
        half_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            // read without a branch (slot 0 where there is nothing to read) and choose afterwards,
            // so that the eight reads are in flight together
            const bool ok = j0 + e < per_pix;
            const half_t x = tmp[ok ? src : 0];
            v[e] = ok ? x : (half_t)0;
            ++src;
            if (++jj == rowlen) {
                jj = 0;
                src += rowh - rowlen;
            }
        }
        *(lds_u4v)(dst + pix * cs + j0) = *(const u4v*)v;
    }
}

// One entry for both forms, so that the kernel holds a single call: `tmp` is the spare LDS area of the
// two-step form, or null for the direct one.
__device__ __attribute__((noinline)) void stage_im2col(const half_t* in, int n, int H, int W, int C, int oy0,
                                             int ox0, int rh, int rw, int kh, int kw, int stride,
                                             int pad, int kfill, int cs, half_t* tmp, half_t* dst)
{
    if (tmp != nullptr)
        stage_im2col_lds(in, n, H, W, C, oy0, ox0, rh, rw, kh, kw, stride, pad, kfill, cs, tmp, dst);
    else
        stage_im2col_direct(in, n, H, W, C, oy0, ox0, rh, rw, kh, kw, stride, pad, kfill, cs, dst);
}

// Staging for a convolution on a narrow input (cin <= 4) with an even stride: the input patch goes
// to LDS as 4-channel pixels [ih][iw][4] (missing channels and pixels outside the image zero).
// The convolution stage then treats a filter row as one tap over round_up(4 * kw, 32) "channels":
// the 16-byte reads of a tap start at a pixel and run on over its right-hand neighbours, which are
// exactly the filter columns; the columns beyond kw meet zero weights (so the 32 halfs behind the
// last pixel only have to be finite: they are zeroed here).  No gather, K = kh * 32 per 7x7 row
// set instead of kh * kw * cin copies per output pixel.
__device__ __attribute__((noinline)) void stage_rowfold(const half_t* in_, int n, int H, int W, int C, int iy0,
                                              int ix0, int ih, int iw, half_t* dst_)
{
    const gconst_h in = (gconst_h)in_;
    const lds_h dst = (lds_h)dst_;
    const int total = ih * iw;
    const unsigned iw_m = div_magic(iw);
    constexpr int U = 4;
    for (int v0 = threadIdx.x; v0 < total; v0 += DLF_WG_THREADS * U) {
        h4 val[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int v = v0 + u * DLF_WG_THREADS;
            // every lane loads, from the nearest pixel inside the image where it has nothing to
            // fetch, and the value is chosen afterwards: a load under a divergent branch is waited
            // for at the end of its branch
            const int vv = min(v, total - 1);
            const int py = div_by(vv, iw_m), pxx = vv - py * iw;
            const int gy = iy0 + py, gx = ix0 + pxx;
            const bool ok = v < total && gy >= 0 && gy < H && gx >= 0 && gx < W;
            const int gyc = min(max(gy, 0), H - 1), gxc = min(max(gx, 0), W - 1);
            const gconst_h p = in + (unsigned)(((n * H + gyc) * W + gxc) * C);
            const half_t z = (half_t)0;
            const half_t c0 = p[0];
            const half_t c1 = C > 1 ? p[1] : z;
            const half_t c2 = C > 2 ? p[2] : z;
            const half_t c3 = C > 3 ? p[3] : z;
            const h4 px = {ok ? c0 : z, ok ? c1 : z, ok ? c2 : z, ok ? c3 : z};
            val[u] = px;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int v = v0 + u * DLF_WG_THREADS;
            if (v < total) *(lds_h4)(dst + v * 4) = val[u];
        }
    }
    if (threadIdx.x < 4) {
        const u4v z = {0, 0, 0, 0};
        *(lds_u4v)(dst + total * 4 + threadIdx.x * 8) = z;
    }
}

// One 32-channel K chunk of a convolution stage: every filter tap, two 16-channel MFMA steps per
// tap.  A "step" is one K step of 16 channels; the packed weight stream holds one 1 KiB fragment
// per output-channel block per step, in exactly the order the steps run.
//
// Weights: ring `ar` of RA steps.  Right after the MFMAs of step s were issued, ar[s % RA] is
// re-fetched with step s + RA, so every weight fragment is requested RA steps (several hundred
// cycles, an L2 round trip) before it is used, and one wave alone keeps the MFMA pipe busy.
// Activations (3x3 path): both K steps of the next tap are read from LDS while the current tap
// is multiplied.
// TAPS = 9 (3x3, RA = 6 or 18) is fully unrolled so that every ring index is static and the
// compiler places each wait exactly; TAPS = 1 (1x1) and TAPS = 0 (any other filter, a loop) use
// RA = 2.  A wave's weight stream is bound by (ring bytes) / (round trip): with 6 KiB in flight and
// 0.5-1.3 us to L2 or HBM a wave gets 5-13 GB/s, which is what a layer with a long K and few
// pixels (3x3 on 14 x 14 or 7 x 7 maps) then runs at; the 32 x 64 register tile has the registers
// for a ring of a whole 18-step chunk (not in the build for 128 registers).
template <int TAPS, int FC, int FP, bool LEAN> struct RingSize {
    static constexpr int value = TAPS != 9 ? 2 : (FC * FP <= 2 && !LEAN) ? 18 : (FC * FP < 8 ? 6 : 2);
};

template <int FC, int FP, int TAPS, int RA>
__device__ __forceinline__ void mma_chunk(const half_t* src, const int (&pbase)[FP], const i32x4 rw, int lane16,
                                          unsigned (&wo)[FC], h8 (&ar)[RA][FC],
                                          f16v (&acc)[FC][FP], int cs, int iw, int kw, int ntaps)
{
    static_assert(RA == 2 || (TAPS == 9 && 18 % RA == 0), "ring depths this loop is written for");
    // Per-tap LDS addresses are formed right before each load; the empty asm keeps the compiler
    // from precomputing all of them outside the chunk loop, which would cost TAPS x FP registers.
    int pb[FP];
#pragma unroll
    for (int p = 0; p < FP; ++p) {
        pb[p] = pbase[p];
        asm volatile("" : "+v"(pb[p]));
    }
    if constexpr (RA > 2) {
        h8 b[2][2][FP];
#pragma unroll
        for (int p = 0; p < FP; ++p) {
            b[0][0][p] = *(const h8*)(src + pb[p]);
            b[0][1][p] = *(const h8*)(src + pb[p] + 16);
        }
        // A wave issues in order, so a load placed between two MFMAs is issued while the first
        // one still occupies the matrix pipe: one LDS read (and, at the end of a step, the weight
        // refills) follows each MFMA, and scheduling barriers keep exactly this order.
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const int nextoff = (((t + 1) / 3) * iw + ((t + 1) % 3)) * cs;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const int sidx = (2 * t + ks) % RA;
#pragma unroll
                for (int f = 0; f < FC; ++f)
#pragma unroll
                    for (int p = 0; p < FP; ++p) {
                        acc[f][p] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ar[sidx][f], b[t & 1][ks][p],
                                                                           acc[f][p], 0, 0, 0);
                        const int li = (ks * FC + f) * FP + p;     // loads so far in this tap
                        if (t + 1 < 9 && li < 2 * FP)
                            b[(t + 1) & 1][li / FP][li % FP] =
                                *(const h8*)(src + pb[li % FP] + nextoff + (li / FP) * 16);
                        if (f == FC - 1 && p == FP - 1) {
#pragma unroll
                            for (int f2 = 0; f2 < FC; ++f2)
                                ar[sidx][f2] = wfrag(rw, lane16, wo[f2] + (2 * t + ks + RA) * 1024);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
            }
        }
#pragma unroll
        for (int f = 0; f < FC; ++f) wo[f] += 18 * 1024;
    } else {
        h8 b0[FP], b1[FP];
#pragma unroll
        for (int p = 0; p < FP; ++p) b0[p] = *(const h8*)(src + pb[p]);
        const int nt = (TAPS == 1) ? 1 : ntaps;
        const int rowskip = (iw - kw) * cs;
        int tapoff = 0, kwc = 0;
        for (int t = 0; t < nt; ++t) {
#pragma unroll
            for (int p = 0; p < FP; ++p) b1[p] = *(const h8*)(src + pb[p] + tapoff + 16);
#pragma unroll
            for (int f = 0; f < FC; ++f)
#pragma unroll
                for (int p = 0; p < FP; ++p)
                    acc[f][p] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ar[0][f], b0[p], acc[f][p], 0, 0, 0);
#pragma unroll
            for (int f = 0; f < FC; ++f) ar[0][f] = wfrag(rw, lane16, wo[f] + 2 * 1024);
            tapoff += cs;
            if (++kwc == kw) { kwc = 0; tapoff += rowskip; }
            if (t + 1 < nt) {
#pragma unroll
                for (int p = 0; p < FP; ++p) b0[p] = *(const h8*)(src + pb[p] + tapoff);
            }
#pragma unroll
            for (int f = 0; f < FC; ++f)
#pragma unroll
                for (int p = 0; p < FP; ++p)
                    acc[f][p] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ar[1][f], b1[p], acc[f][p], 0, 0, 0);
#pragma unroll
            for (int f = 0; f < FC; ++f) { ar[1][f] = wfrag(rw, lane16, wo[f] + 3 * 1024); wo[f] += 2 * 1024; }
        }
    }
}

// Keeps a wave-uniform value in a scalar register: without this the compiler prefers to re-load
// kernel-argument fields from memory wherever they are used, and every such load is a stall.
__device__ __forceinline__ int pin_s(int x)
{
    x = __builtin_amdgcn_readfirstlane(x);
    asm volatile("" : "+s"(x));
    return x;
}

// Epilogue of a convolution work item: fp16 rounding, optional 2x2 max pooling across the 4 lanes
// of a quad, activation, store of 4 consecutive channels per lane into the LDS tile
// [pixel][out_cs].  Pixels outside the true feature map are stored as zero (the padding value the
// next convolution of the group must see).
template <int FC, int FP, bool POOL>
__device__ __forceinline__ void conv_epilogue(f16v (&acc)[FC][FP], int cbl, int ncbv, int pg,
                                              int npix, int rw, unsigned rw_m, int ry0, int rx0,
                                              int out_h, int out_w, int act, int out_off, int out_cs)
{
    const int lane = threadIdx.x & 63, l32 = lane & 31, lhi = lane >> 5;
    const int cmax = out_cs - DLF_CPAD;
    const unsigned lo_act = act_lo(act), hi_act = act_hi(act);
#pragma unroll
    for (int p = 0; p < FP; ++p) {
        const int pix = (pg * FP + p) * 32 + l32;
        const bool valid = pix < npix;
        int ry, rx;
        pix_to_rc(valid ? pix : 0, rw, rw_m, POOL ? 1 : 0, ry, rx);
        const int gy = ry0 + ry, gx = rx0 + rx;
        bool keep, store;
        int row;
        if (POOL) {
            const int py = gy >> 1, px = gx >> 1;
            keep = gy >= 0 && gx >= 0 && py < (out_h >> 1) && px < (out_w >> 1);
            store = valid && (l32 & 3) == 0;
            row = pix >> 2;
        } else {
            keep = gy >= 0 && gy < out_h && gx >= 0 && gx < out_w;
            store = valid;
            row = pix;
        }
        // a pixel outside the feature map is clamped to [0, 0]: the zero padding the next
        // convolution must see, at no extra instruction
        const unsigned lo = keep ? lo_act : 0u, hi = keep ? hi_act : 0u;
        half_t* dst = lds + out_off + row * out_cs + lhi * 4;
#pragma unroll
        for (int f = 0; f < FC; ++f) {
            if (f < ncbv) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int lc = (cbl + f) * 32 + q * 8;
                    unsigned u0 = cvt_pk(acc[f][p][q * 4 + 0], acc[f][p][q * 4 + 1]);
                    unsigned u1 = cvt_pk(acc[f][p][q * 4 + 2], acc[f][p][q * 4 + 3]);
                    if (POOL) {
                        u0 = quad_max_pk(u0);
                        u1 = quad_max_pk(u1);
                    }
                    u0 = pk_min(pk_max(u0, lo), hi);
                    u1 = pk_min(pk_max(u1, lo), hi);
                    if (store && lc + lhi * 4 < cmax) {
                        const u2v uu = {u0, u1};
                        *(u2v*)(dst + lc) = uu;
                    }
                }
            }
        }
    }
}

// A convolution stage.
//
// STREAM: the input is not resident; it is brought from HBM in rounds of st.kc channels (a
// multiple of 32) into two alternating LDS buffers.  The workgroup is split by role: waves
// 0..3 multiply (one work item each), waves 4..7 only move data (HBM -> registers -> LDS for the
// next round).  The roles must be different waves because the hardware's load counter retires in
// order: a wave that had both the long-latency activation loads and the just-in-time weight
// fragment loads in flight would stall its MFMAs on the activation loads.
// Resident (not STREAM): the input region is already in LDS and all 8 waves multiply.
template <int FC, int FP, bool STREAM, int TAPS, bool LEAN, bool KSP>
__device__ __forceinline__ void conv_stage(const DlfGroupArgs& a, const DlfStage& st, int n,
                                           int ty0, int tx0, int slice, bool defer_act)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    const int npix = st.rh * st.rw;
    const int npb = (npix + 31) >> 5;
    const int n_pg = (npb + FP - 1) / FP;
    int cb_begin = 0, cb_end = st.ncb;
    if (a.nslices > 1) {
        cb_begin = slice * (a.slice_c >> 5);
        cb_end = min(st.ncb, cb_begin + (a.slice_c >> 5));
    }
    const int n_cg = (cb_end - cb_begin + FC - 1) / FC;
    const int nitems = n_pg * n_cg;
    const int ry0 = ty0 * st.oy_mul + st.oy_off, rx0 = tx0 * st.ox_mul + st.ox_off;
    const unsigned rw_m = div_magic(st.pool2 ? st.rw >> 1 : st.rw);
    const int kc = STREAM ? st.kc : 32;         // channels per round
    const int cpr = kc >> 5;                    // 32-channel chunks per round
    const int nrounds = st.cin_pad / kc;
    const int cs = st.in_cs;
    const int ntaps = st.kh * st.kw;
    const half_t* in = (const half_t*)a.in;
    const i32x4 rin = make_rsrc(a.in, 0xffffffffu);
    constexpr int MMA_WAVES = STREAM ? DLF_MMA_WAVES : DLF_WAVES;

    if (STREAM && wave >= DLF_MMA_WAVES) {
        // ---------------- data-movement waves ----------------
        const int lt = tid - DLF_MMA_WAVES * 64;                 // 0 .. DLF_LOAD_THREADS-1
        const int vshift = st.kc_shift;              // log2(16-byte vectors per pixel per round)
        const int vmask = (1 << vshift) - 1;
        const int s_total = (st.ih * st.iw) << vshift;
        const unsigned iw_m = div_magic(st.iw);
        const int iy0 = ty0 * a.iy_mul + a.iy_off, ix0 = tx0 * a.ix_mul + a.ix_off;
        // Element offset of the pixel each vector comes from -- clamped into the image and into the
        // region, so that it can always be loaded from -- and whether the vector is real or zero fill.
        // Every vector of a round is loaded without a branch and the zero chosen afterwards: a load
        // under a divergent check is waited for at the end of its branch, which would make a round as
        // many trips to memory, one after the other, as a thread has vectors; the multiplying waves
        // wait for nothing else.
        int s_goff[DLF_STAGE_VECS];
        unsigned s_ok = 0;
        if ((st.cin & 7) != 0) {
            // narrow inputs (e.g. 3 channels): one round, element-wise copy
            for (int v = lt; v < s_total; v += DLF_LOAD_THREADS) {
                const int pix = v >> vshift, part = v & vmask;
                const int ry = div_by(pix, iw_m), rx = pix - ry * st.iw;
                *(h8*)(lds + st.in_off + pix * cs + part * 8) =
                    load_px8(in, n, iy0 + ry, ix0 + rx, a.in_h, a.in_w, a.in_c, part * 8, st.cin);
            }
            __syncthreads();
            for (int round = 0; round < nrounds; ++round) __syncthreads();
            return;
        }
#pragma unroll
        for (int i = 0; i < DLF_STAGE_VECS; ++i) {
            const int v = lt + i * DLF_LOAD_THREADS;
            const int pix = min(v, s_total - 1) >> vshift;
            const int ry = div_by(pix, iw_m), rx = pix - ry * st.iw;
            const int gy = iy0 + ry, gx = ix0 + rx;
            if (v < s_total && gy >= 0 && gy < a.in_h && gx >= 0 && gx < a.in_w) s_ok |= 1u << i;
            const int gyc = min(max(gy, 0), a.in_h - 1), gxc = min(max(gx, 0), a.in_w - 1);
            s_goff[i] = ((n * a.in_h + gyc) * a.in_w + gxc) * a.in_c;
        }
        for (int round = 0; round <= nrounds; ++round) {
            // round r of this loop fills the buffer that the multiplying waves read in round r
            if (round < nrounds) {
                const int coff = round * kc;
                half_t* dst = lds + st.in_off + (round & 1) * st.stream_buf;
                h8 s_reg[DLF_STAGE_VECS];
#pragma unroll
                for (int i = 0; i < DLF_STAGE_VECS; ++i) {
                    const int c = coff + ((lt + i * DLF_LOAD_THREADS) & vmask) * 8;
                    const h8 x = wfrag(rin, (s_goff[i] + min(c, st.cin - 8)) * 2, 0);     // 32-bit offsets: the tensor is below 4 GiB
                    const h8 z = {0, 0, 0, 0, 0, 0, 0, 0};
                    s_reg[i] = ((s_ok >> i) & 1u) != 0 && c < st.cin ? x : z;
                }
#pragma unroll
                for (int i = 0; i < DLF_STAGE_VECS; ++i) {
                    const int vi = lt + i * DLF_LOAD_THREADS;
                    if (vi < s_total) *(h8*)(dst + (vi >> vshift) * cs + (vi & vmask) * 8) = s_reg[i];
                }
            }
            __syncthreads();
        }
        return;
    }

    // K split over waves (resident stages with few work items and a long K, where a wave's weight
    // stream, not the matrix pipe, sets the pace): ksplit waves share a work item, each runs a
    // contiguous share of the 32-channel chunks, the partial sums meet in LDS and the first wave of
    // the item finishes it.  The host guarantees work items x ksplit <= waves: one pass.  Only the
    // KSP builds of the kernel carry this form; in the others ksplit is the constant 1.
    const int ksplit = (KSP && !STREAM) ? max(st.ksplit, 1) : 1;    // a power of two
    const int ks_shift = __builtin_ctz(ksplit);
    const i32x4 rw = make_rsrc(st.w, 0xffffffffu);       // every offset the streams form lies inside the packed weights
    const int lane16 = lane * 16;
    const int kpart = wave & (ksplit - 1);
    const int iwave = wave >> ks_shift;
    const int items_per_pass = MMA_WAVES >> ks_shift;
    bool first_pass = true;
    for (int item0 = 0; item0 < nitems; item0 += items_per_pass) {
        const int item = item0 + iwave;
        const bool active = item < nitems;
        if (!STREAM && !active) {
            // the barrier in front of the other waves' epilogues
            if (st.alias_out || ksplit > 1) __syncthreads();
            continue;
        }
        const int itc = active ? item : 0;
        const int cg = itc / n_pg, pg = itc - cg * n_pg;

        int pbase[FP];
#pragma unroll
        for (int p = 0; p < FP; ++p) {
            const int pix = (pg * FP + p) * 32 + l32;
            int ry, rx;
            pix_to_rc(pix < npix ? pix : 0, st.rw, rw_m, st.pool2, ry, rx);
            pbase[p] = ((ry * st.stride) * st.iw + rx * st.stride) * cs + lhi * 8;
        }
        const int rounds_mine = nrounds / ksplit;           // the host guarantees divisibility
        const int round_first = kpart * rounds_mine;
        // the wave's weight streams: uniform byte offsets into the packed weights (below 4 GiB)
        unsigned wo[FC];
#pragma unroll
        for (int f = 0; f < FC; ++f) {
            const int cb = min(cb_begin + cg * FC + f, cb_end - 1);
            wo[f] = (unsigned)__builtin_amdgcn_readfirstlane((cb * st.nsteps + round_first * cpr * ntaps * 2) * 1024);
        }
        // accumulators start at the bias of their output channel (in the item's first wave)
        f16v acc[FC][FP];
#pragma unroll
        for (int f = 0; f < FC; ++f) {
            const int cb = min(cb_begin + cg * FC + f, cb_end - 1);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                f4v bv = *(const f4v*)(st.bias + cb * 32 + q * 8 + lhi * 4);
                if (kpart != 0) bv = f4v{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int p = 0; p < FP; ++p)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[f][p][q * 4 + r] = bv[r];
            }
        }

        constexpr int RA = RingSize<TAPS, FC, FP, LEAN>::value;
        h8 ar[RA][FC];
#pragma unroll
        for (int i = 0; i < RA; ++i)
#pragma unroll
            for (int f = 0; f < FC; ++f) ar[i][f] = wfrag(rw, lane16, wo[f] + i * 1024);

        if (STREAM && first_pass) {
            __syncthreads();          // round 0 is in LDS
            first_pass = false;
        }
        for (int round = round_first; round < round_first + rounds_mine; ++round) {
            const half_t* src = STREAM ? lds + st.in_off + (round & 1) * st.stream_buf
                                       : lds + st.in_off + round * 32;
            if (active) {
                if constexpr (TAPS == 1) {
                    int j = 0;
                    for (; j + 1 < cpr; j += 2) {
                        mma_chunk<FC, FP, 1, RA>(src + j * 32, pbase, rw, lane16, wo, ar, acc, cs, st.iw, 1, 1);
                        mma_chunk<FC, FP, 1, RA>(src + j * 32 + 32, pbase, rw, lane16, wo, ar, acc, cs, st.iw, 1, 1);
                    }
                    if (j < cpr)
                        mma_chunk<FC, FP, 1, RA>(src + j * 32, pbase, rw, lane16, wo, ar, acc, cs, st.iw, 1, 1);
                } else {
                    for (int j = 0; j < cpr; ++j)
                        mma_chunk<FC, FP, TAPS, RA>(src + j * 32, pbase, rw, lane16, wo, ar, acc, cs, st.iw, st.kw,
                                                ntaps);
                }
            }
            if (STREAM) __syncthreads();
        }

        // partial sums of a split K: every wave but the item's first leaves its accumulators in LDS
        if (!STREAM && ksplit > 1 && kpart != 0) {
            float* sc = (float*)(lds + st.ks_off) + wave * (FC * FP * 16 * 64) + lane;
#pragma unroll
            for (int f = 0; f < FC; ++f)
#pragma unroll
                for (int p = 0; p < FP; ++p)
#pragma unroll
                    for (int r = 0; r < 16; ++r) sc[((f * FP + p) * 16 + r) * 64] = acc[f][p][r];
        }
        // the output tile may overwrite this stage's input: every wave must be done reading it
        // (a streaming stage has just passed its last round's barrier)
        if (!STREAM && (st.alias_out || ksplit > 1)) __syncthreads();
        if (!STREAM && ksplit > 1) {
            if (kpart != 0) continue;
            for (int k = 1; k < ksplit; ++k) {
                const float* sc = (const float*)(lds + st.ks_off) + (wave + k) * (FC * FP * 16 * 64) + lane;
#pragma unroll
                for (int f = 0; f < FC; ++f)
#pragma unroll
                    for (int p = 0; p < FP; ++p)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[f][p][r] += sc[((f * FP + p) * 16 + r) * 64];
            }
        }
        // ---- epilogue: activation, (pool), fp16 -> LDS tile [pixel][channel] ----
        // (the last stage's tile is then written to HBM by store_tile with full-line stores,
        //  which also adds the residual operand and applies the activation after it)
        if (!active) continue;
        const int act = (defer_act && st.res != nullptr) ? 0 : st.act;
        const int cbl = cg * FC;                       // first local channel block of the item
        const int ncbv = min(FC, cb_end - cb_begin - cbl);
        if (st.pool2)
            conv_epilogue<FC, FP, true>(acc, cbl, ncbv, pg, npix, pin_s(st.rw), rw_m, ry0, rx0,
                                        pin_s(st.out_h), pin_s(st.out_w), act, pin_s(st.out_off),
                                        pin_s(st.out_cs));
        else
            conv_epilogue<FC, FP, false>(acc, cbl, ncbv, pg, npix, pin_s(st.rw), rw_m, ry0, rx0,
                                         pin_s(st.out_h), pin_s(st.out_w), act, pin_s(st.out_off),
                                         pin_s(st.out_cs));
    }
}

// Writes the finished output tile of a CONV stage from LDS to HBM: consecutive threads write
// consecutive 16-byte pieces of a pixel's channels, so every store instruction covers whole
// cache lines (the MFMA result layout itself would give 8-byte pieces 2*Cout bytes apart).
__device__ __forceinline__ void store_tile(const DlfGroupArgs& a, const DlfStage& st, int n, int ty0,
                                           int tx0, int slice)
{
    const int ph = st.pool2 ? st.rh >> 1 : st.rh, pw = st.pool2 ? st.rw >> 1 : st.rw;
    int oy = ty0 * st.oy_mul + st.oy_off, ox = tx0 * st.ox_mul + st.ox_off;
    if (st.pool2) { oy >>= 1; ox >>= 1; }
    int c0 = 0, ccnt = st.cout;
    if (a.nslices > 1) {
        c0 = slice * a.slice_c;
        ccnt = min(a.slice_c, st.cout - c0);
    }
    half_t* outp = (half_t*)a.out;
    const half_t* resp = (const half_t*)st.res;   // same shape as the output; added, then activation
    if ((st.cout & 7) == 0) {
        const int nvec = ccnt >> 3;
        const int total = ph * pw * nvec;
        const unsigned nvec_m = div_magic(nvec), pw_m = div_magic(pw);
        const unsigned lo = act_lo(st.act), hi = act_hi(st.act);
        constexpr int U = 4;     // residual loads of a batch are all in flight together
        for (int v0 = threadIdx.x; v0 < total; v0 += DLF_WG_THREADS * U) {
            unsigned go[U];      // element offsets fit 32 bits (checked on the host)
            u4v val[U], rv[U];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int v = v0 + u * DLF_WG_THREADS;
                const int vc = v < total ? v : 0;
                const int pix = div_by(vc, nvec_m), part = vc - pix * nvec;
                const int y = div_by(pix, pw_m), x = pix - y * pw;
                const int gy = oy + y, gx = ox + x;
                ok[u] = v < total && gy < a.out_h && gx < a.out_w;
                go[u] = (unsigned)(((n * a.out_h + gy) * a.out_w + gx) * a.out_c + c0 + part * 8);
                if (resp != nullptr && ok[u]) rv[u] = *(const u4v*)(resp + go[u]);
                val[u] = *(const u4v*)(lds + st.out_off + pix * st.out_cs + part * 8);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (ok[u]) {
                    if (resp != nullptr) {
                        // fp16 + fp16 correctly rounded, then the activation as a clamp
                        val[u].x = pk_min(pk_max(pk_add(val[u].x, rv[u].x), lo), hi);
                        val[u].y = pk_min(pk_max(pk_add(val[u].y, rv[u].y), lo), hi);
                        val[u].z = pk_min(pk_max(pk_add(val[u].z, rv[u].z), lo), hi);
                        val[u].w = pk_min(pk_max(pk_add(val[u].w, rv[u].w), lo), hi);
                    }
                    *(u4v*)(outp + go[u]) = val[u];
                }
            }
        }
    } else {
        const int nvec = ccnt >> 2;
        for (int v = threadIdx.x; v < ph * pw * nvec; v += DLF_WG_THREADS) {
            const int pix = v / nvec, part = v - pix * nvec;
            const int y = pix / pw, x = pix - y * pw;
            const int gy = oy + y, gx = ox + x;
            if (gy < a.out_h && gx < a.out_w) {
                const size_t go = (((size_t)n * a.out_h + gy) * a.out_w + gx) * a.out_c + c0 + part * 4;
                h4 val = *(const h4*)(lds + st.out_off + pix * st.out_cs + part * 4);
                if (resp != nullptr) {
                    const h4 rv = *(const h4*)(resp + go);
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        val[j] = (half_t)apply_act((float)val[j] + (float)rv[j], st.act);
                }
                *(h4*)(outp + go) = val;
            }
        }
    }
}

// Max pooling and depthwise convolution on the vector ALUs: one work item = one output pixel x
// 8 channels, input read from LDS (16 bytes per tap), fp32 arithmetic.
// HOIST: keep the 3x3 depthwise weights of the lane's channel group in registers across work
// items (44 registers; not in the 128-register build, where they are re-read per item).
template <bool HOIST>
__device__ __forceinline__ void valu_stage(const DlfGroupArgs& a, const DlfStage& st, bool last,
                                           int n, int ty0, int tx0, int slice)
{
    const int npix = st.rh * st.rw;
    int c0 = 0, ccnt = st.cout;
    if (a.nslices > 1) {
        c0 = slice * a.slice_c;
        ccnt = min(a.slice_c, st.cout - c0);
    }
    const int ncg = (ccnt + 7) >> 3;
    const unsigned ncg_m = div_magic(ncg), rw_m = div_magic(st.rw);
    const int ry0 = ty0 * st.oy_mul + st.oy_off, rx0 = tx0 * st.ox_mul + st.ox_off;
    const half_t* wdw = (const half_t*)st.w;
    half_t* outp = (half_t*)a.out;
    const bool k3 = st.kind == DLF_ST_DW && st.kh == 3 && st.kw == 3;
    // a thread's channel group is it % ncg with it advancing by the workgroup size
    const bool fixed_g = HOIST && (DLF_WG_THREADS % ncg) == 0;
    h8 w3[9];
    f4v b0, b1;
    if (k3 && fixed_g) {
        const int lc = (threadIdx.x % ncg) * 8;
#pragma unroll
        for (int t = 0; t < 9; ++t) w3[t] = *(const h8*)(wdw + t * st.cin_pad + c0 + lc);
        b0 = *(const f4v*)(st.bias + c0 + lc);
        b1 = *(const f4v*)(st.bias + c0 + lc + 4);
    }
    for (int it = threadIdx.x; it < npix * ncg; it += DLF_WG_THREADS) {
        const int pix = div_by(it, ncg_m), g = it - pix * ncg;
        const int ry = div_by(pix, rw_m), rx = pix - ry * st.rw;
        const int gy = ry0 + ry, gx = rx0 + rx;
        const bool inimg = gy >= 0 && gy < st.out_h && gx >= 0 && gx < st.out_w;
        const int lc = g * 8;
        u4v hv;
        if (st.kind == DLF_ST_MAXPOOL) {
            // max of fp16 values is exact: stay in packed fp16
            hv = u4v{0xFC00FC00u, 0xFC00FC00u, 0xFC00FC00u, 0xFC00FC00u};   // -inf
            if (st.kh == 3 && st.kw == 3) {
                // 3x3: all nine reads are issued before the first maximum (one LDS round trip per
                // work item instead of nine); taps outside the feature map count as -inf
                const int iy = gy * st.stride - st.pad, ix = gx * st.stride - st.pad;
                const half_t* xp = lds + st.in_off + ((ry * st.stride) * st.iw + rx * st.stride) * st.in_cs + lc;
                const int rowstep = st.iw * st.in_cs;
                u4v x[9];
#pragma unroll
                for (int t = 0; t < 9; ++t) x[t] = *(const u4v*)(xp + (t / 3) * rowstep + (t % 3) * st.in_cs);
#pragma unroll
                for (int t = 0; t < 9; ++t) {
                    const int ty = iy + t / 3, tx = ix + t % 3;
                    const bool ok = ty >= 0 && ty < st.in_h && tx >= 0 && tx < st.in_w;
                    const unsigned m = ok ? 0u : 0xFC00FC00u;      // max(x, -inf) = x
                    hv.x = pk_max(hv.x, ok ? x[t].x : m);
                    hv.y = pk_max(hv.y, ok ? x[t].y : m);
                    hv.z = pk_max(hv.z, ok ? x[t].z : m);
                    hv.w = pk_max(hv.w, ok ? x[t].w : m);
                }
            } else
            for (int kh = 0; kh < st.kh; ++kh) {
                const int iy = gy * st.stride - st.pad + kh;
                if (iy < 0 || iy >= st.in_h) continue;
                for (int kw = 0; kw < st.kw; ++kw) {
                    const int ix = gx * st.stride - st.pad + kw;
                    if (ix < 0 || ix >= st.in_w) continue;
                    const u4v x = *(const u4v*)(lds + st.in_off
                                                    + ((ry * st.stride + kh) * st.iw + rx * st.stride + kw)
                                                          * st.in_cs + lc);
                    hv.x = pk_max(hv.x, x.x);
                    hv.y = pk_max(hv.y, x.y);
                    hv.z = pk_max(hv.z, x.z);
                    hv.w = pk_max(hv.w, x.w);
                }
            }
        } else {
            float v[8];
            if (k3) {
                // 3x3: taps unrolled, the 9 weight vectors and the bias of the lane's channel
                // group held in registers (loaded once when the group never changes)
                if (!fixed_g) {
#pragma unroll
                    for (int t = 0; t < 9; ++t) w3[t] = *(const h8*)(wdw + t * st.cin_pad + c0 + lc);
                    b0 = *(const f4v*)(st.bias + c0 + lc);
                    b1 = *(const f4v*)(st.bias + c0 + lc + 4);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) { v[j] = b0[j]; v[j + 4] = b1[j]; }
                const half_t* xp = lds + st.in_off + ((ry * st.stride) * st.iw + rx * st.stride) * st.in_cs + lc;
                const int rowstep = st.iw * st.in_cs;
#pragma unroll
                for (int kh = 0; kh < 3; ++kh) {
                    h8 x[3];
#pragma unroll
                    for (int kw = 0; kw < 3; ++kw) x[kw] = *(const h8*)(xp + kh * rowstep + kw * st.in_cs);
#pragma unroll
                    for (int kw = 0; kw < 3; ++kw)
#pragma unroll
                        for (int j = 0; j < 8; ++j)
                            v[j] = fmaf((float)x[kw][j], (float)w3[kh * 3 + kw][j], v[j]);
                }
            } else {
                const f4v c0v = *(const f4v*)(st.bias + c0 + lc);
                const f4v c1v = *(const f4v*)(st.bias + c0 + lc + 4);
#pragma unroll
                for (int j = 0; j < 4; ++j) { v[j] = c0v[j]; v[j + 4] = c1v[j]; }
                for (int kh = 0; kh < st.kh; ++kh) {
                    for (int kw = 0; kw < st.kw; ++kw) {
                        const h8 x = *(const h8*)(lds + st.in_off
                                                  + ((ry * st.stride + kh) * st.iw + rx * st.stride + kw)
                                                        * st.in_cs + lc);
                        const h8 w = *(const h8*)(wdw + (kh * st.kw + kw) * st.cin_pad + c0 + lc);
#pragma unroll
                        for (int j = 0; j < 8; ++j) v[j] = fmaf((float)x[j], (float)w[j], v[j]);
                    }
                }
            }
            const unsigned lo = act_lo(st.act), hi = act_hi(st.act);
            hv.x = pk_min(pk_max(cvt_pk(v[0], v[1]), lo), hi);
            hv.y = pk_min(pk_max(cvt_pk(v[2], v[3]), lo), hi);
            hv.z = pk_min(pk_max(cvt_pk(v[4], v[5]), lo), hi);
            hv.w = pk_min(pk_max(cvt_pk(v[6], v[7]), lo), hi);
        }
        if (last) {
            if (inimg) {
                half_t* o = outp + (unsigned)(((n * a.out_h + gy) * a.out_w + gx) * a.out_c + c0 + lc);
                if (lc + 8 <= ccnt) {
                    *(u4v*)o = hv;
                } else {
                    const h8 hh = __builtin_bit_cast(h8, hv);
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (lc + j < ccnt) o[j] = hh[j];
                }
            }
        } else {
            const u4v z = {0, 0, 0, 0};
            *(u4v*)(lds + st.out_off + pix * st.out_cs + lc) = inimg ? hv : z;
        }
    }
}

// MINW = minimum waves per SIMD the register allocation must allow: 2 (up to 256 registers, one
// workgroup per CU) or 4 (128 registers, two workgroups per CU, for bandwidth-bound groups whose
// load, multiply and store phases then overlap across workgroups).
template <int FC, int FP, int MINW, bool KSP = false>
__global__ __launch_bounds__(DLF_WG_THREADS, MINW) void k_group(const DlfGroupArgs a)
{
    for (int t = blockIdx.x; t < a.ntiles; t += gridDim.x) {
        int r = t;
        const int slice = r % a.nslices;
        r /= a.nslices;
        const int tx = r % a.tiles_x;
        r /= a.tiles_x;
        const int ty = r % a.tiles_y;
        const int n = r / a.tiles_y;
        const int ty0 = ty * a.th, tx0 = tx * a.tw;
        if (!a.stream0) {
            const DlfStage& s0 = a.st[0];
            int c0 = 0, cfill = s0.cin_pad, cend = s0.cin;
            if (a.nslices > 1 && s0.kind != DLF_ST_CONV) {
                c0 = slice * a.slice_c;
                cend = min(s0.cin, c0 + a.slice_c);
                cfill = (cend - c0 + 7) & ~7;
            }
            if (s0.kind == DLF_ST_CONV && s0.im2col == 2)
                stage_rowfold((const half_t*)a.in, n, a.in_h, a.in_w, a.in_c, ty0 * a.iy_mul + a.iy_off,
                              tx0 * a.ix_mul + a.ix_off, s0.ih, s0.iw, lds + s0.in_off);
            else if (s0.kind == DLF_ST_CONV && s0.im2col) {
                // through the stage's output buffer where there is one of its own and the patch fits it
                const int pih = (s0.rh - 1) * s0.im_stride + s0.im_kh, piw = (s0.rw - 1) * s0.im_stride + s0.im_kw;
                const bool two_step = a.nstages > 1 && !s0.alias_out && s0.out_off != s0.in_off &&
                                      ((s0.cin_pad | s0.in_cs) & 7) == 0 &&
                                      pih * piw * a.in_c < (s0.pool2 ? (s0.rh >> 1) * (s0.rw >> 1) : s0.rh * s0.rw) * s0.out_cs;
                stage_im2col((const half_t*)a.in, n, a.in_h, a.in_w, a.in_c,
                             ty0 * s0.oy_mul + s0.oy_off, tx0 * s0.ox_mul + s0.ox_off, s0.rh, s0.rw,
                             s0.im_kh, s0.im_kw, s0.im_stride, s0.im_pad, s0.cin_pad, s0.in_cs,
                             two_step ? lds + s0.out_off : nullptr, lds + s0.in_off);
            }
            else
                stage_region((const half_t*)a.in, n, a.in_h, a.in_w, a.in_c,
                             ty0 * a.iy_mul + a.iy_off, tx0 * a.ix_mul + a.ix_off, s0.ih, s0.iw, c0,
                             cfill, cend, s0.in_cs, lds + s0.in_off);
            __syncthreads();
        }
        for (int s = 0; s < a.nstages; ++s) {
            const DlfStage& st = a.st[s];
            const bool last = (s == a.nstages - 1);
            if (st.kind == DLF_ST_CONV) {
                const int taps = st.kh * st.kw;
                const int kind = (taps == 9 && st.kw == 3) ? 9 : (taps == 1 ? 1 : 0);
                if (s == 0 && a.stream0) {
                    if (kind == 9) conv_stage<FC, FP, true, 9, (MINW >= 4), false>(a, st, n, ty0, tx0, slice, last);
                    else if (kind == 1) conv_stage<FC, FP, true, 1, (MINW >= 4), false>(a, st, n, ty0, tx0, slice, last);
                    else conv_stage<FC, FP, true, 0, (MINW >= 4), false>(a, st, n, ty0, tx0, slice, last);
                } else {
                    if (kind == 9) conv_stage<FC, FP, false, 9, (MINW >= 4), KSP>(a, st, n, ty0, tx0, slice, last);
                    else if (kind == 1) conv_stage<FC, FP, false, 1, (MINW >= 4), KSP>(a, st, n, ty0, tx0, slice, last);
                    else conv_stage<FC, FP, false, 0, (MINW >= 4), KSP>(a, st, n, ty0, tx0, slice, last);
                }
                if (last) {
                    __syncthreads();
                    store_tile(a, st, n, ty0, tx0, slice);
                }
            } else {
                valu_stage<(MINW < 4)>(a, st, last, n, ty0, tx0, slice);
            }
            __syncthreads();
        }
    }
}

// Pointwise convolution, one wave per work item (32*FP output pixels x 32*FC output channels), no
// workgroup barrier anywhere: the layers this serves are bound by HBM traffic or by the latency of
// a long K loop, and eight to sixteen independent waves per CU, each with its own loads in
// flight, hide the memory latency that a tile pipeline with barriers exposes phase by phase.
//   B operand (activations): lane (pixel l%32, k half l/32) loads 16 bytes of its pixel's
//     channels per K step directly from HBM/L2 -- the MFMA layout, no LDS staging;
//   A operand (weights): packed fragments from L2, as in the fused-group kernel;
//   both through D-deep register rings refilled right behind the MFMAs that used the slot; the
//     first operands of the wave's next item are requested before the epilogue of the current one;
//   result: fp16 into the wave's transpose buffer, read back 16 bytes per lane so that the
//     stores (and the residual loads) cover whole runs of 64 * FC bytes.
// Shapes: (2,2) with D = 4 for large layers (each operand byte feeds two MFMAs); (1,1) with D = 8
// where the layer has too few 64 x 64 items to occupy the chip (small feature maps, long K).
template <int FP>
__device__ __forceinline__ void pw_item_setup(const DlfPwArgs& a, int item, int lane, int (&bo)[FP],
                                              int& pg, int& cg)
{
    const int l32 = lane & 31, lhi = lane >> 5;
    pg = item / a.n_cg;
    cg = item - pg * a.n_cg;
#pragma unroll
    for (int p = 0; p < FP; ++p) {
        int pix = (pg * FP + p) * 32 + l32;
        pix = pix < a.m ? pix : a.m - 1;          // clamped lanes compute a result nobody stores
        unsigned off;
        if (a.stride == 1) {
            off = (unsigned)pix * (unsigned)a.cin;
        } else {
            const int hw = a.out_h * a.out_w;
            const int n = pix / hw, r = pix - n * hw;
            const int oy = r / a.out_w, ox = r - oy * a.out_w;
            off = (unsigned)(((n * a.in_h + oy * a.stride) * a.in_w + ox * a.stride) * a.cin);
        }
        bo[p] = (int)((off + lhi * 8) * 2u);       // byte offset of the lane's 16 bytes of K step 0
    }
}

template <int FC, int FP, int D, int MINB>
__global__ __launch_bounds__(DLF_PW_WAVES * 64, MINB) void k_pw(const DlfPwArgs a)
{
    constexpr int ROW = 32 * FC + 8;                 // halfs per pixel row of the transpose buffer
    constexpr int LPP = 4 * FC;                      // lanes (16-byte vectors) per pixel
    constexpr int NPASS = 2 * FC * FP;               // read-back passes of 64 vectors
    // (the wave index as a scalar: what is derived from it -- work items, loop exits, weight offsets --
    // is then uniform for the compiler too)
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    half_t* tb = lds + wave * (32 * FP * ROW);
    const half_t* resp = (const half_t*)a.res;
    half_t* outp = (half_t*)a.out;
    const int nwaves = gridDim.x * DLF_PW_WAVES;
    const int nsteps = a.nsteps;
    const int act_epi = resp != nullptr ? 0 : a.act;     // with a residual the activation comes after the add
    const unsigned lo_e = act_lo(act_epi), hi_e = act_hi(act_epi);
    const unsigned lo_r = act_lo(a.act), hi_r = act_hi(a.act);

    int item = blockIdx.x * DLF_PW_WAVES + wave;
    if (item >= a.nitems) return;
    // operands through buffer resources: 32-bit lane offsets + uniform K-step offsets, so that the
    // wave's walk along K is scalar arithmetic (see wfrag)
    const i32x4 rw = make_rsrc(a.w, 0xffffffffu), rin = make_rsrc(a.in, 0xffffffffu);
    const int lane16 = lane * 16;
    int bo[FP];
    unsigned wo[FC];
    int pg, cg;
    h8 ar[D][FC], br[D][FP];
    auto request_first = [&]() {
        pw_item_setup<FP>(a, item, lane, bo, pg, cg);
#pragma unroll
        for (int f = 0; f < FC; ++f) {
            const int cb = min(cg * FC + f, a.ncb - 1);
            wo[f] = (unsigned)__builtin_amdgcn_readfirstlane(cb * nsteps * 1024);
        }
#pragma unroll
        for (int j = 0; j < D; ++j) {
            if (j < nsteps) {
#pragma unroll
                for (int f = 0; f < FC; ++f) ar[j][f] = wfrag(rw, lane16, wo[f] + j * 1024);
#pragma unroll
                for (int p = 0; p < FP; ++p) br[j][p] = wfrag(rin, bo[p], j * 32);
            }
        }
    };
    request_first();
    for (;;) {
        f16v acc[FC][FP];
#pragma unroll
        for (int f = 0; f < FC; ++f)
#pragma unroll
            for (int p = 0; p < FP; ++p)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[f][p][r] = 0.0f;
        for (int s = 0; s < nsteps; s += D) {
#pragma unroll
            for (int j = 0; j < D; ++j) {
                if (s + j < nsteps) {
#pragma unroll
                    for (int f = 0; f < FC; ++f)
#pragma unroll
                        for (int p = 0; p < FP; ++p)
                            acc[f][p] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ar[j][f], br[j][p], acc[f][p], 0, 0, 0);
                    if (s + j + D < nsteps) {       // never read activations beyond the pixel's channels
#pragma unroll
                        for (int f = 0; f < FC; ++f) ar[j][f] = wfrag(rw, lane16, wo[f] + (s + j + D) * 1024);
#pragma unroll
                        for (int p = 0; p < FP; ++p) br[j][p] = wfrag(rin, bo[p], (s + j + D) * 32);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        // bias first, then the next item's operands: the epilogue waits for the bias only
        f4v bias[FC][4];
#pragma unroll
        for (int f = 0; f < FC; ++f) {
            const int cb = min(cg * FC + f, a.ncb - 1);
#pragma unroll
            for (int q = 0; q < 4; ++q) bias[f][q] = *(const f4v*)(a.bias + cb * 32 + q * 8 + lhi * 4);
        }
        const int cur_pg = pg, cur_cg = cg;
        item += nwaves;
        const bool more = item < a.nitems;
        if (more) request_first();
        __builtin_amdgcn_sched_barrier(0);
        // ---- result (+ bias) -> wave-private transpose buffer [pixel][channel] ----
#pragma unroll
        for (int p = 0; p < FP; ++p)
#pragma unroll
            for (int f = 0; f < FC; ++f)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    unsigned u0 = cvt_pk(acc[f][p][q * 4 + 0] + bias[f][q][0], acc[f][p][q * 4 + 1] + bias[f][q][1]);
                    unsigned u1 = cvt_pk(acc[f][p][q * 4 + 2] + bias[f][q][2], acc[f][p][q * 4 + 3] + bias[f][q][3]);
                    u0 = pk_min(pk_max(u0, lo_e), hi_e);
                    u1 = pk_min(pk_max(u1, lo_e), hi_e);
                    const u2v uu = {u0, u1};
                    *(u2v*)(tb + (p * 32 + l32) * ROW + f * 32 + q * 8 + lhi * 4) = uu;
                }
        __builtin_amdgcn_wave_barrier();
        // ---- 16 bytes per lane: LPP lanes cover the 32*FC channels of one pixel ----
        const int part = lane % LPP;
        const int c = cur_cg * (32 * FC) + part * 8;
        constexpr int HP = NPASS > 1 ? NPASS / 2 : 1;          // two rounds keep the register need down
#pragma unroll
        for (int h = 0; h < NPASS / HP; ++h) {
            u4v val[HP], rv[HP];
            bool ok[HP];
            unsigned go[HP];
#pragma unroll
            for (int i = 0; i < HP; ++i) {
                const int px = (h * HP + i) * (64 / LPP) + lane / LPP;
                const int gpix = cur_pg * (32 * FP) + px;
                ok[i] = gpix < a.m && c < a.cout;
                go[i] = (unsigned)gpix * (unsigned)a.cout + (unsigned)c;
                if (resp != nullptr && ok[i]) rv[i] = *(const u4v*)(resp + go[i]);
                val[i] = *(const u4v*)(tb + px * ROW + part * 8);
            }
#pragma unroll
            for (int i = 0; i < HP; ++i) {
                if (ok[i]) {
                    if (resp != nullptr) {
                        val[i].x = pk_min(pk_max(pk_add(val[i].x, rv[i].x), lo_r), hi_r);
                        val[i].y = pk_min(pk_max(pk_add(val[i].y, rv[i].y), lo_r), hi_r);
                        val[i].z = pk_min(pk_max(pk_add(val[i].z, rv[i].z), lo_r), hi_r);
                        val[i].w = pk_min(pk_max(pk_add(val[i].w, rv[i].w), lo_r), hi_r);
                    }
                    *(u4v*)(outp + go[i]) = val[i];
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
        if (!more) break;
    }
}

// Split-K form of the pointwise kernel, for layers with few work items and a long K loop (small
// feature maps, many input channels), where one wave per item leaves most of the chip idle behind a
// serial chain of operand round trips: the four waves of a workgroup share one 64 x 64 item, each
// runs a quarter of the K steps, the partial sums meet in LDS and each wave finishes one of the
// four 32 x 32 blocks (bias, activation, residual, store).
__global__ __launch_bounds__(DLF_PW_WAVES * 64, 2) void k_pw_sk(const DlfPwArgs a)
{
    constexpr int D = 6;
    constexpr int ROW = 32 + 8;
    // (the wave index as a scalar: what is derived from it -- work items, loop exits, weight offsets --
    // is then uniform for the compiler too)
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    float* part = (float*)lds;                                  // [block][3 senders][16][64] fp32
    half_t* tb = lds + DLF_PWSK_PART_BYTES / 2 + wave * (32 * ROW);
    const half_t* resp = (const half_t*)a.res;
    half_t* outp = (half_t*)a.out;
    const int per = a.nsteps / DLF_PW_WAVES;                    // the host guarantees divisibility
    const int s0 = wave * per;
    const i32x4 rw = make_rsrc(a.w, 0xffffffffu), rin = make_rsrc(a.in, 0xffffffffu);
    const int lane16 = lane * 16;
    const int act_epi = resp != nullptr ? 0 : a.act;
    const unsigned lo_e = act_lo(act_epi), hi_e = act_hi(act_epi);
    const unsigned lo_r = act_lo(a.act), hi_r = act_hi(a.act);
    for (int item = blockIdx.x; item < a.nitems; item += gridDim.x) {
        int bo[2];
        unsigned wo[2];
        int pg, cg;
        pw_item_setup<2>(a, item, lane, bo, pg, cg);
#pragma unroll
        for (int p = 0; p < 2; ++p) bo[p] += s0 * 32;
#pragma unroll
        for (int f = 0; f < 2; ++f) {
            const int cb = min(cg * 2 + f, a.ncb - 1);
            wo[f] = (unsigned)__builtin_amdgcn_readfirstlane((cb * a.nsteps + s0) * 1024);
        }
        h8 ar[D][2], br[D][2];
#pragma unroll
        for (int j = 0; j < D; ++j) {
            if (j < per) {
#pragma unroll
                for (int f = 0; f < 2; ++f) ar[j][f] = wfrag(rw, lane16, wo[f] + j * 1024);
#pragma unroll
                for (int p = 0; p < 2; ++p) br[j][p] = wfrag(rin, bo[p], j * 32);
            }
        }
        f16v acc[2][2];
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[f][p][r] = 0.0f;
        for (int s = 0; s < per; s += D) {
#pragma unroll
            for (int j = 0; j < D; ++j) {
                if (s + j < per) {
#pragma unroll
                    for (int f = 0; f < 2; ++f)
#pragma unroll
                        for (int p = 0; p < 2; ++p)
                            acc[f][p] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ar[j][f], br[j][p], acc[f][p], 0, 0, 0);
                    if (s + j + D < per) {          // stays inside this wave's share of the channels
#pragma unroll
                        for (int f = 0; f < 2; ++f) ar[j][f] = wfrag(rw, lane16, wo[f] + (s + j + D) * 1024);
#pragma unroll
                        for (int p = 0; p < 2; ++p) br[j][p] = wfrag(rin, bo[p], (s + j + D) * 32);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        // ---- exchange: block b = 2 * f + p is finished by wave b; the others send their partials ----
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            if (b != wave) {
                const int k = wave < b ? wave : wave - 1;
#pragma unroll
                for (int r = 0; r < 16; ++r) part[((b * 3 + k) * 16 + r) * 64 + lane] = acc[b >> 1][b & 1][r];
            }
        }
        __syncthreads();
        f16v own = wave == 0 ? acc[0][0] : (wave == 1 ? acc[0][1] : (wave == 2 ? acc[1][0] : acc[1][1]));
#pragma unroll
        for (int k = 0; k < 3; ++k)
#pragma unroll
            for (int r = 0; r < 16; ++r) own[r] += part[((wave * 3 + k) * 16 + r) * 64 + lane];
        const int fo = wave >> 1, po = wave & 1;
        const int cb = cg * 2 + fo;
        if (cb < a.ncb) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f4v bv = *(const f4v*)(a.bias + cb * 32 + q * 8 + lhi * 4);
                unsigned u0 = cvt_pk(own[q * 4 + 0] + bv[0], own[q * 4 + 1] + bv[1]);
                unsigned u1 = cvt_pk(own[q * 4 + 2] + bv[2], own[q * 4 + 3] + bv[3]);
                u0 = pk_min(pk_max(u0, lo_e), hi_e);
                u1 = pk_min(pk_max(u1, lo_e), hi_e);
                const u2v uu = {u0, u1};
                *(u2v*)(tb + l32 * ROW + q * 8 + lhi * 4) = uu;
            }
            __builtin_amdgcn_wave_barrier();
            // 32 pixels x 4 vectors of 8 channels: two per lane
            const int partv = lane & 3;
            const int c = cb * 32 + partv * 8;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int px = i * 16 + (lane >> 2);
                const int gpix = (pg * 2 + po) * 32 + px;
                if (gpix < a.m && c < a.cout) {
                    const unsigned go = (unsigned)gpix * (unsigned)a.cout + (unsigned)c;
                    u4v val = *(const u4v*)(tb + px * ROW + partv * 8);
                    if (resp != nullptr) {
                        const u4v rv = *(const u4v*)(resp + go);
                        val.x = pk_min(pk_max(pk_add(val.x, rv.x), lo_r), hi_r);
                        val.y = pk_min(pk_max(pk_add(val.y, rv.y), lo_r), hi_r);
                        val.z = pk_min(pk_max(pk_add(val.z, rv.z), lo_r), hi_r);
                        val.w = pk_min(pk_max(pk_add(val.w, rv.w), lo_r), hi_r);
                    }
                    *(u4v*)(outp + go) = val;
                }
            }
        }
        __syncthreads();        // the partial-sum area is rewritten by the next item
    }
}

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Direct-to-LDS load of 16 bytes per lane, lane l from base + off into LDS at dst + 16 l, in the
// instruction's scalar-base form: `base` (uniform) in a scalar register pair, `off` a 32-bit lane
// offset, `dst` (uniform) through M0.  A request then costs the wave no vector ALU instruction.
// Written as an instruction because the compiler, given the same address as base + off, folds it
// into a 64-bit vector-register pointer per request.  Counted by vmcnt like any load; the compiler
// does not see it.  (The kernels that use it keep their uniform values within the scalar register
// file: a spilled `base` cannot be named by the instruction.  tests/test_build.py checks the
// generated code for that.)
__device__ __forceinline__ void dma16s(const void* base, unsigned off, unsigned dst)
{
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(dst) : "memory", "m0");
}
// The same load through the compiler's own instruction selection (any register class for base).
__device__ __forceinline__ void dma16(const void* base, unsigned off, half_t* dst)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)((const char*)base + off),
                                     (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
}

// An LDS read issued as an instruction (16 bytes per lane at byte address addr + OFF), invisible to
// the compiler's own wait insertion: the value may be used only behind an lds_arrive that covers it.
template <int OFF> __device__ __forceinline__ h8 lds_read16(unsigned addr)
{
    h8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
// Waits until at most N LDS reads of the wave are outstanding (they return in order) and passes the
// four fragments through, so that their users depend on the wait.
template <int N> __device__ __forceinline__ void lds_arrive(h8& a, h8& b, h8& c, h8& d)
{
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N));
}
template <int N> __device__ __forceinline__ void lds_arrive1(h8& a)
{
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a) : "n"(N));
}
template <int N> __device__ __forceinline__ void lds_arrive2(h8& a, h8& b)
{
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N));
}
template <int I, int N, typename F> __device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>());
        static_for<I + 1, N>(f);
    }
}

// Block form of the pointwise kernel, for layers whose operand traffic from L2 bounds the
// one-wave-per-item form: a workgroup of four waves computes 64 * WN output channels x 64 * WM
// pixels (2 x 2 or 1 x 4 waves, each a 64 x 64 part), and the block's operands pass through LDS, so
// every byte fetched from L2 feeds WM (weights) or WN (activations) waves.
//   Global -> LDS: 16-byte direct loads (no registers in between); a wave's 64 lanes deposit
//     1 KiB, lane l at byte 16 l -- for weights one packed MFMA fragment as it lies in memory, for
//     activations 2 KS adjacent lanes fetch the stage's 32 KS bytes of one pixel, so that a request
//     covers whole runs of memory (16-byte pieces of many different cache lines cost a CU several
//     times their size in intake).
//   LDS is a ring of NST stages of KS K steps; stage t + NST - 1 is requested when stage t is
//     about to be multiplied.  Loads retire in issue order: "at most n x loads-per-stage
//     outstanding" means that all but the wave's last n requested stages have landed, and the
//     barrier that follows extends that to all waves (and tells every wave that stage t - 1 has
//     been read by all, so its slot may be refilled).
//   The barrier is the bare instruction: the fence of __syncthreads() would wait for every load
//     in flight and serialise the ring.
//   Epilogue as in k_pw, through a wave-private transpose buffer that reuses the ring.
// One block per workgroup; consecutive blocks (same pixels, next channels) are dealt to the same
// XCD so that they meet in its L2.
// I8: the quantised form (int8 tensors seen as fp16 tensors of half the channels, int32
// accumulators on v_mfma_i32_32x32x32_i8, requantising epilogue; see k_c3b).  No residual operand
// and no second operand pair in this form.
template <int WN, int WM, bool P2, bool I8 = false>
__global__ __launch_bounds__(DLF_PW_WAVES * 64, 2) void k_pwb(const DlfPwArgs a)
{
    static_assert(!(I8 && P2), "the quantised form takes one operand pair");
    constexpr int KS = DLF_PWB_KS, NST = DLF_PWB_STAGES;
    constexpr int NA = 2 * WN * KS, NB = 2 * WM * KS, NF = NA + NB;   // fragments per stage
    constexpr int LPW = NF / DLF_PW_WAVES;                            // loads per wave per stage
    constexpr int STAGE = NF * 512;                                   // halfs per stage
    constexpr int LPX = 2 * KS, PPI = 64 / LPX;      // activation loads: lanes per pixel, pixels per instruction
    static_assert(KS == 2 || KS == 4, "a pixel's part of a stage is 64 or 128 bytes: 4 or 8 lanes");
    static_assert(WN * WM == DLF_PW_WAVES && NA % DLF_PW_WAVES == 0 && NB % DLF_PW_WAVES == 0, "fragment roles are per wave");
    static_assert(KS % 2 == 0 && NST >= 4, "two register sets alternate per K step; one stage is read ahead");
    constexpr int ROW = 64 + 8;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) half_t*)lds;
    // blockIdx.x % 8 is the XCD: give each XCD a contiguous range of blocks (the grid is a
    // multiple of 8; a workgroup takes every (gridDim.x / 8)-th block of its XCD's range)
    const int per_xcd = (a.nitems + 7) >> 3;
    bool again = false;
    for (int li = blockIdx.x >> 3; li < per_xcd; li += gridDim.x >> 3) {
    const int item = (blockIdx.x & 7) * per_xcd + li;
    if (item >= a.nitems) break;
    if (again) {
        // the stores of the previous block must not be counted among the loads of the ring, and
        // the transpose buffers of all waves must have been read before the ring is refilled
        wait_vmcnt<0>();
        asm volatile("s_barrier" ::: "memory");
    }
    again = true;
    const int pg = item / a.n_cg, cg = item - pg * a.n_cg;
    const int wn = WN == 1 ? 0 : (wave & (WN - 1)), wm = WN == 1 ? wave : wave / WN;
    const int wcg = cg * WN + wn, wpg = pg * WM + wm;       // the wave's 64-channel / 64-pixel part
    const half_t* resp = (const half_t*)a.res;
    half_t* outp = (half_t*)a.out;
    const int act_epi = resp != nullptr ? 0 : a.act;
    const unsigned lo_e = act_lo(act_epi), hi_e = act_hi(act_epi);
    const unsigned lo_r = act_lo(a.act), hi_r = act_hi(a.act);

    // the oldest loads in flight: complete by the first wait of the ring
    f4v bias[2][4];
#pragma unroll
    for (int f = 0; f < 2; ++f) {
        const int cb = min(wcg * 2 + f, a.ncb - 1);
#pragma unroll
        for (int q = 0; q < 4; ++q) bias[f][q] = *(const f4v*)(a.bias + cb * 32 + q * 8 + lhi * 4);
        if (P2) {
#pragma unroll
            for (int q = 0; q < 4; ++q) bias[f][q] += *(const f4v*)(a.bias2 + cb * 32 + q * 8 + lhi * 4);
        }
    }

    // ... and so does the residual operand of the wave's part (8 lanes cover the 64 channels of a
    // pixel, as in the epilogue): requested here, it has arrived long before the epilogue, where
    // the round trip to HBM would otherwise be paid in full, twice
    u4v rvp[2][4];
    if (resp != nullptr) {
        const int c = wcg * 64 + (lane & 7) * 8;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int gpix = wpg * 64 + (h * 4 + i) * 8 + (lane >> 3);
                if (gpix < a.m && c < a.cout)
                    rvp[h][i] = *(const u4v*)(resp + (unsigned)gpix * (unsigned)a.cout + (unsigned)c);
            }
    }

    // This wave's loads of a stage: fragments wave, wave + 4, ...  Every load is "uniform base +
    // 32-bit lane offset" (dma16): the bases live in scalar registers and move by scalar adds, the
    // lane offsets are fixed for the block, so that a request costs the wave no vector ALU
    // instruction -- on a SIMD whose matrix pipe another wave keeps busy a wave gets a vector ALU
    // slot only every few dozen cycles, and requests that need one each arrive at a quarter of
    // the rate.  Weight fragments: base = the fragment, offset 16 * lane.  Activations: base = the
    // tensor + the stage's channel offset, offset = the lane's pixel and 16-byte part.  base2 /
    // off2: the same for the second operand pair, which the stream of stages switches to after the
    // first pair's K steps.
    unsigned off[LPW], off2[LPW];
    auto operand_offsets = [&](int nsteps, int cin, int stride, int in_h, int in_w, unsigned (&op)[LPW])
                               __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int f = wave + DLF_PW_WAVES * i;
            if (DLF_PW_WAVES * i < NA) {
                const int cbl = f / KS, ks = f - cbl * KS;
                const int cb = min(cg * (2 * WN) + cbl, a.ncb - 1);
                op[i] = (unsigned)((cb * nsteps + ks) * 1024 + lane * 16);   // packed weights: < 4 GiB
            } else {
                // instruction `sub` of 32-pixel block pbl: PPI pixels, LPX adjacent lanes fetching
                // the stage's 32 * KS bytes of one pixel (a whole run of memory per pixel, not a
                // 32-byte piece of it); the 16-byte parts are stored permuted, see actb_off
                const int j = f - NA;
                const int pbl = j / KS, sub = j - pbl * KS;
                const int pl = sub * PPI + lane / LPX;
                const int q = (lane & (LPX - 1)) ^ ((pl / (16 / LPX)) & (LPX - 1));
                int pix = (pg * (2 * WM) + pbl) * 32 + pl;
                pix = pix < a.m ? pix : a.m - 1;          // clamped lanes compute a result nobody stores
                unsigned o;
                if (stride == 1) {
                    o = (unsigned)pix * (unsigned)cin;
                } else {
                    const int hw = a.out_h * a.out_w;
                    const int n = pix / hw, r = pix - n * hw;
                    const int oy = r / a.out_w, ox = r - oy * a.out_w;
                    o = (unsigned)(((n * in_h + oy * stride) * in_w + ox * stride) * cin);
                }
                op[i] = (o + (unsigned)q * 8u) * 2u;      // bytes; a tensor is smaller than 4 GiB
            }
        }
    };
    operand_offsets(a.nsteps, a.cin, a.stride, a.in_h, a.in_w, off);
    const int KT1 = a.nsteps / KS;
    if (P2) operand_offsets(a.nsteps2, a.cin2, a.stride2, a.in_h2, a.in_w2, off2);
    // the two bases of the stage being requested (weights, activations), for either operand pair
    const half_t* wb = (const half_t*)a.w;
    const half_t* ib = (const half_t*)a.in;
    const half_t* wb2 = P2 ? (const half_t*)a.w2 : nullptr;
    const half_t* ib2 = P2 ? (const half_t*)a.in2 : nullptr;
    int nissued = 0;
    auto issue = [&](int slot) {
        const bool first = !P2 || nissued < KT1;                   // uniform
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const half_t* b = (DLF_PW_WAVES * i < NA) ? (first ? wb : wb2) : (first ? ib : ib2);
            // (with two operand pairs the kernel's uniform values no longer fit the scalar register
            // file, and the compiler chooses the registers of the address)
            if constexpr (P2) dma16(b, first ? off[i] : off2[i], lds + slot * STAGE + (wave + DLF_PW_WAVES * i) * 512);
            else dma16s(b, off[i], lds0 + (unsigned)((slot * STAGE + (wave + DLF_PW_WAVES * i) * 512) * 2));
        }
        if (first) {
            wb += KS * 512;
            ib += KS * 16;
        } else {
            wb2 += KS * 512;
            ib2 += KS * 16;
        }
        ++nissued;
    };
    const int KT = (a.nsteps + (P2 ? a.nsteps2 : 0)) / KS;
#pragma unroll
    for (int t = 0; t < NST - 1; ++t)
        if (t < KT) issue(t);

    typename AccOf<I8>::type acc[2][2];
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[f][p][r] = 0;

    // Stage t is multiplied while the fragments of the next K step -- the last one of a stage
    // reads ahead into stage t + 1 -- are on their way from LDS, so stage t + 1 must be visible
    // when iteration t starts: NST - 3 requested stages stay in flight behind it.
    // A 32-pixel block of a stage lies in LDS as [pixel][32 * KS bytes]; part q (16 bytes: K step
    // q / 2, K half q % 2) of pixel p sits at position q ^ f(p), f(p) = (p / (16 / LPX)) % LPX, so
    // that the 16 lanes LDS serves per cycle -- 16 consecutive pixels, one part each -- fall into
    // 16 different 16-byte bank groups.
    int actb_off[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        actb_off[ks] = l32 * (KS * 16) + (((2 * ks + lhi) ^ ((l32 / (16 / LPX)) & (LPX - 1))) << 3);
    // The fragment reads are written as instructions, with their waits: while a direct-to-LDS load
    // is pending the compiler turns every wait for an LDS read into a wait for all of them, the
    // ones just issued for the next K step included (one full LDS round trip per step).  LDS reads
    // return in order, so "at most 4 outstanding" behind the 4 requests of the next step means the
    // current step's fragments have arrived; lds_arrive hands them to the MFMAs (a data dependence:
    // nothing that uses them can move above the wait).
    const unsigned a_addr = lds0 + (unsigned)(((wn * 2) * KS * 512 + lane * 8) * 2);
    unsigned b_addr[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) b_addr[ks] = lds0 + (unsigned)(((NA + (wm * 2) * KS) * 512 + actb_off[ks]) * 2);
    auto request = [&](unsigned slot_bytes, auto kc, h8 (&af)[2], h8 (&bf)[2]) __attribute__((always_inline)) {
        constexpr int K = decltype(kc)::value;
        af[0] = lds_read16<(0 * KS + K) * 1024>(a_addr + slot_bytes);
        af[1] = lds_read16<(1 * KS + K) * 1024>(a_addr + slot_bytes);
        bf[0] = lds_read16<(0 * KS) * 1024>(b_addr[K] + slot_bytes);
        bf[1] = lds_read16<(1 * KS) * 1024>(b_addr[K] + slot_bytes);
    };
    h8 af[2][2], bf[2][2];
    if (KT > NST - 2) wait_vmcnt<(NST - 2) * LPW>(); else wait_vmcnt<0>();
    asm volatile("s_barrier" ::: "memory");
    request(0u, std::integral_constant<int, 0>(), af[0], bf[0]);
    int slot = 0;
    for (int kt = 0; kt < KT; ++kt) {
        const int nslot = slot + 1 == NST ? 0 : slot + 1;
        if (kt + 1 < KT) {
            if (kt + NST - 2 < KT) wait_vmcnt<(NST - 3) * LPW>();
            else wait_vmcnt<0>();
        }
        asm volatile("s_barrier" ::: "memory");
        if (kt + NST - 1 < KT) issue(slot == 0 ? NST - 1 : slot - 1);
        const unsigned sb = (unsigned)(slot * STAGE * 2), nb = (unsigned)(nslot * STAGE * 2);
        static_for<0, KS>([&](auto kc) __attribute__((always_inline)) {
            constexpr int K = decltype(kc)::value, cur = K & 1, nxt = cur ^ 1;
            // (behind the last stage the read-ahead takes stale fragments nobody multiplies)
            if constexpr (K + 1 < KS) request(sb, std::integral_constant<int, K + 1>(), af[nxt], bf[nxt]);
            else request(nb, std::integral_constant<int, 0>(), af[nxt], bf[nxt]);
            lds_arrive<4>(af[cur][0], af[cur][1], bf[cur][0], bf[cur][1]);
#pragma unroll
            for (int f = 0; f < 2; ++f)
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    if constexpr (I8)
                        acc[f][p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4, af[cur][f]),
                                                                          __builtin_bit_cast(i32x4, bf[cur][p]), acc[f][p], 0, 0, 0);
                    else
                        acc[f][p] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[cur][f], bf[cur][p], acc[f][p], 0, 0, 0);
                }
            __builtin_amdgcn_sched_barrier(0);
        });
        slot = nslot;
    }
    // the read-ahead of the last step lands in registers nobody reads: it must have landed before
    // they are used for anything else
    lds_arrive<0>(af[0][0], af[0][1], bf[0][0], bf[0][1]);
    // every wave is done with the ring (all loads were waited for above): reuse it
    asm volatile("s_barrier" ::: "memory");
    if constexpr (I8) {
        // requantise, transpose through 64-byte rows (i8t_write_off), and
        // store 16 bytes per lane: 4 lanes cover the wave's 64 channels of a pixel, 16 pixels per pass
        unsigned char* tb8 = (unsigned char*)lds + wave * (64 * 64);
        signed char* out8 = (signed char*)a.out;
        const float lo = a.act != 0 ? 0.0f : -128.0f;
#pragma unroll
        for (int f = 0; f < 2; ++f) {
            const int cb = min(wcg * 2 + f, a.ncb - 1);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f4v sv = *(const f4v*)(a.scale + cb * 32 + q * 8 + lhi * 4);
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    const unsigned u = pack_low_bytes(requant_biased(acc[f][p][q * 4 + 0], sv[0], bias[f][q][0], lo),
                                                      requant_biased(acc[f][p][q * 4 + 1], sv[1], bias[f][q][1], lo),
                                                      requant_biased(acc[f][p][q * 4 + 2], sv[2], bias[f][q][2], lo),
                                                      requant_biased(acc[f][p][q * 4 + 3], sv[3], bias[f][q][3], lo));
                    *(unsigned*)(tb8 + i8t_write_off(p * 32 + l32, f * 2 + (q >> 1), (q & 1) * 2 + lhi)) = u;
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
        const int part = lane & 3;
        const int c = wcg * 64 + part * 16;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int px = it * 16 + (lane >> 2);
            const int gpix = wpg * 64 + px;
            const u4v v = i8t_read(tb8, px, part);
            if (gpix < a.m && c < a.cout)
                __builtin_nontemporal_store(v, (u4v*)(out8 + (size_t)gpix * (size_t)a.cout + (size_t)c));
        }
    } else {
    half_t* tb = lds + wave * (64 * ROW);
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                unsigned u0 = cvt_pk(acc[f][p][q * 4 + 0] + bias[f][q][0], acc[f][p][q * 4 + 1] + bias[f][q][1]);
                unsigned u1 = cvt_pk(acc[f][p][q * 4 + 2] + bias[f][q][2], acc[f][p][q * 4 + 3] + bias[f][q][3]);
                u0 = pk_min(pk_max(u0, lo_e), hi_e);
                u1 = pk_min(pk_max(u1, lo_e), hi_e);
                const u2v uu = {u0, u1};
                *(u2v*)(tb + (p * 32 + l32) * ROW + f * 32 + q * 8 + lhi * 4) = uu;
            }
    __builtin_amdgcn_wave_barrier();
    // 16 bytes per lane: 8 lanes cover the 64 channels of one pixel, 8 pixels per pass
    const int part = lane & 7;
    const int c = wcg * 64 + part * 8;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        u4v val[4], rv[4];
        bool ok[4];
        unsigned go[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int px = (h * 4 + i) * 8 + (lane >> 3);
            const int gpix = wpg * 64 + px;
            ok[i] = gpix < a.m && c < a.cout;
            go[i] = (unsigned)gpix * (unsigned)a.cout + (unsigned)c;
            rv[i] = rvp[h][i];
            val[i] = *(const u4v*)(tb + px * ROW + part * 8);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (ok[i]) {
                if (resp != nullptr) {
                    val[i].x = pk_min(pk_max(pk_add(val[i].x, rv[i].x), lo_r), hi_r);
                    val[i].y = pk_min(pk_max(pk_add(val[i].y, rv[i].y), lo_r), hi_r);
                    val[i].z = pk_min(pk_max(pk_add(val[i].z, rv[i].z), lo_r), hi_r);
                    val[i].w = pk_min(pk_max(pk_add(val[i].w, rv[i].w), lo_r), hi_r);
                }
                store_out(outp + go[i], val[i]);
            }
        }
    }
    }
    }
}

// Waits until at most n of this wave's loads are outstanding, for a wave-uniform n known only at
// run time (the count is an immediate of the instruction); counts above 48 wait for everything.
__device__ __forceinline__ void wait_vmcnt_dyn(int n)
{
    switch (__builtin_amdgcn_readfirstlane(n)) {
#define DLF_WAIT_CASE(N) case N: wait_vmcnt<N>(); break;
    DLF_WAIT_CASE(1) DLF_WAIT_CASE(2) DLF_WAIT_CASE(3) DLF_WAIT_CASE(4) DLF_WAIT_CASE(5) DLF_WAIT_CASE(6)
    DLF_WAIT_CASE(7) DLF_WAIT_CASE(8) DLF_WAIT_CASE(9) DLF_WAIT_CASE(10) DLF_WAIT_CASE(11) DLF_WAIT_CASE(12)
    DLF_WAIT_CASE(13) DLF_WAIT_CASE(14) DLF_WAIT_CASE(15) DLF_WAIT_CASE(16) DLF_WAIT_CASE(17) DLF_WAIT_CASE(18)
    DLF_WAIT_CASE(19) DLF_WAIT_CASE(20) DLF_WAIT_CASE(21) DLF_WAIT_CASE(22) DLF_WAIT_CASE(23) DLF_WAIT_CASE(24)
    DLF_WAIT_CASE(25) DLF_WAIT_CASE(26) DLF_WAIT_CASE(27) DLF_WAIT_CASE(28) DLF_WAIT_CASE(29) DLF_WAIT_CASE(30)
    DLF_WAIT_CASE(31) DLF_WAIT_CASE(32) DLF_WAIT_CASE(33) DLF_WAIT_CASE(34) DLF_WAIT_CASE(35) DLF_WAIT_CASE(36)
    DLF_WAIT_CASE(37) DLF_WAIT_CASE(38) DLF_WAIT_CASE(39) DLF_WAIT_CASE(40) DLF_WAIT_CASE(41) DLF_WAIT_CASE(42)
    DLF_WAIT_CASE(43) DLF_WAIT_CASE(44) DLF_WAIT_CASE(45) DLF_WAIT_CASE(46) DLF_WAIT_CASE(47) DLF_WAIT_CASE(48)
#undef DLF_WAIT_CASE
    default: wait_vmcnt<0>(); break;
    }
}

// 3x3 convolution, stride 1, pad 1, as a block kernel: one layer (with the 2x2 max pool behind it
// folded into the epilogue, or a residual operand added there), for layers where the fused-group
// kernel is bound by the weight stream of its waves.  A workgroup of eight waves computes
// 64 * WC output channels x a th x tw tile of up to 64 * (8 / WC) pixels, every wave a 64 x 64
// part, and streams K through LDS:
//   weights: a ring of 2 .. 4 stages, each the nine taps' fragments of the block's channels for 16
//     input channels (9 * 2 * WC KiB, the packed fragments as they lie in memory);
//   activations: two buffers, each the tile's halo region, (th + 2) x (tw + 2) pixels, for ACH
//     input channels (ACH / 16 weight stages); block b + 1 is requested when block b is first used;
//   global -> LDS by 16-byte direct loads, a wave's 64 lanes filling 1 KiB per instruction.  For
//     activations ACH / 8 adjacent lanes fetch the ACH channels of one pixel, so that a request
//     covers whole 64- or 128-byte runs of memory (16-byte pieces of different cache lines cost a
//     CU several times their size in intake); lanes of pixels outside the image fetch from the
//     zero steps behind the packed weights (the padding arrives as data); every wave issues the
//     same number of loads (surplus ones go to a spare KiB), so one count of outstanding loads
//     means the same for all of them;
//   within a pixel's ACH channels the 16-byte parts are stored permuted, part q of halo pixel h at
//     position q ^ f(h): an MFMA "B" fragment reads one part of 32 consecutive pixels, LDS serves
//     16 lanes (256 bytes) per cycle, and with f(h) = (h / 2) % 8 (128 bytes per pixel) or
//     (h / 4) % 4 (64 bytes) any 16 consecutive pixels land in 16 different 16-byte bank groups,
//     whatever the filter tap's shift;
//   one bare barrier per weight stage, as in k_pwb; fragments of tap t + 1 are read while tap t is
//     multiplied.
// Every byte from L2 feeds eight waves' worth of MFMAs: 128 channels x 256 pixels take in
// 1 byte per ~200 FLOP, against ~50-100 for the per-wave weight streams of the fused-group kernel.
// Work items: channel group slowest, so that the workgroups running at one time share weights; each
// XCD gets a contiguous range of items.
//
// I8: the quantised form of the same layer.  An int8 tensor of C channels has the bytes of an fp16
// tensor of C / 2 channels, and v_mfma_i32_32x32x32_i8 takes its operands as the fp16 instruction
// does (16 bytes per lane, the two halves of the wave the two halves of a K step), so the operand
// path above serves as it stands with `cin` counting byte pairs: one K step is 32 int8 channels.
// What differs: exact int32 accumulators that start at zero, and an epilogue that requantises --
// (float)acc, one fused multiply-add with the channel's scale and bias, round half to even, clamp
// to [-128 or 0, 127] -- and stores int8, four lanes of 16 bytes covering a wave's 64 channels of
// a pixel.  The 2x2 max pool behind the layer can be folded in (on the requantised values); no residual
// operand in this form.
template <int WC, int ACH, int FP, bool I8 = false>
__global__ __launch_bounds__(DLF_C3_WAVES * 64, 1) void k_c3b(const DlfC3Args a)
{
    using acc_t = typename AccOf<I8>::type;
    constexpr int NCBW = 2 * WC;                     // 32-channel blocks of the workgroup
    constexpr int NWF = 9 * NCBW;                    // weight fragments per stage
    constexpr int LW = DLF_C3_LOAD_WAVES;              // waves that request operands (one per SIMD)
    constexpr int LPW_W = (NWF + LW - 1) / LW;
    constexpr int W_HALFS = NWF * 512;
    constexpr int LPP = ACH / 8;                     // lanes (16-byte parts) per pixel
    constexpr int PPI = 64 / LPP;                    // pixels per load instruction
    constexpr int SH = LPP == 8 ? 1 : 2;             // f(h) = (h >> SH) % LPP
    constexpr int CPB = ACH / 16;                    // weight stages per activation block
    constexpr int MAXA = DLF_C3_MAX_ACT_LOADS;
    constexpr int ROW = 64 + 8;
    static_assert(FP == 2 || FP == 4, "a wave's part: 64 channels x 32 * FP pixels");
    static_assert(ACH == 32 || ACH == 64, "activation block: 64 or 128 bytes per pixel");
    // the wave index as a scalar: everything derived from it (fragment numbers, LDS targets, weight
    // addresses) then lives in scalar registers
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    const int wc = WC == 1 ? 0 : (wave & (WC - 1)), wp = WC == 1 ? wave : wave / WC;
    const int pw = a.tw + 2;
    const int npxh = a.npxh, na_i = a.na_i, lpa = a.lpw_a, nst = a.nst;
    const int act_halfs = na_i * 512;
    half_t* const wring = lds + 2 * act_halfs;
    half_t* const trash = wring + nst * W_HALFS;
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) half_t*)lds;
    const int KT = a.cin >> 4, NB = a.cin / ACH;
    const unsigned pw_m = div_magic(pw);
    const unsigned tw_m = div_magic(a.pool2 ? a.tw >> 1 : a.tw);
    const half_t* resp = (const half_t*)a.res;
    half_t* outp = (half_t*)a.out;
    const int act_epi = resp != nullptr ? 0 : a.act;
    const unsigned lo_e = act_lo(act_epi), hi_e = act_hi(act_epi);
    const unsigned lo_r = act_lo(a.act), hi_r = act_hi(a.act);
    const int npix = a.th * a.tw;
    const int per_xcd = (a.nitems + 7) >> 3;
    int li = blockIdx.x >> 3;
    {
        const int first = (blockIdx.x & 7) * per_xcd + li;
        if (li >= per_xcd || first >= a.nitems) return;
    }

    // the wave's FP 32-pixel blocks: halo index of each lane's pixel under tap (0, 0)
    int hp0[FP];
#pragma unroll
    for (int p = 0; p < FP; ++p) {
        int pix = wp * (32 * FP) + p * 32 + l32;
        pix = pix < npix ? pix : 0;               // surplus lanes compute a result nobody stores
        int ry, rx;
        pix_to_rc(pix, a.tw, tw_m, a.pool2, ry, rx);
        hp0[p] = ry * pw + rx;
    }

    // Load side: the item whose operands are being requested.  The first stages of item i + 1 are
    // requested before the epilogue of item i, so that they arrive while it runs.
    // A request must cost the requesting wave as little vector arithmetic as possible: its SIMD's
    // matrix pipe is kept busy by the other wave, a vector ALU instruction gets a slot only every
    // few dozen cycles, and loads that need address arithmetic in vector registers arrive at a
    // quarter of the rate the memory pipe could take them.
    //   weights: uniform base (scalar arithmetic) + 16 * lane, the scalar-base form of the load;
    //   activations: the byte offset of a halo pixel is the same for all of an item's channel
    //     blocks: it is computed once per item into a table in LDS (wave-private: no barrier), and
    //     a request is one 4-byte LDS read, one 32-bit add of the lane's 16-byte part, and a buffer
    //     load (32-bit offsets) whose scalar offset selects the block; pixels outside the image
    //     hold an offset beyond the tensor, for which the hardware's range check delivers zeros
    //     (the padding arrives as data, without a source of zeros in memory).  The part a lane
    //     fetches, (lane % LPP) ^ f(halo pixel), is the same in all of a wave's instructions:
    //     instruction wave + LW i starts at halo pixel (wave + LW i) PPI, and LW (PPI >> SH) is a
    //     multiple of LPP.
    int cg = 0, n = 0, ty0 = 0, tx0 = 0;
    static_assert(((LW * (PPI >> SH)) % LPP) == 0 && (PPI % (1 << SH)) == 0, "the permuted part of a lane is the same in all of a wave's load instructions");
    unsigned* const atab = (unsigned*)(trash + 512) + wave * PPI + lane / LPP;   // pixel entry of load i at atab[i * LW * PPI]
    const unsigned part16 =
        (unsigned)(((lane & (LPP - 1)) ^ ((wave * (PPI >> SH) + ((lane / LPP) >> SH)) & (LPP - 1))) << 4);
    const __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(
        (void*)a.in, 0, (int)((unsigned)(a.batch * a.h * a.w_) * (unsigned)a.cin * 2u), 0x00020000);
    auto setup = [&](int item) __attribute__((always_inline)) {
        cg = item / a.ntiles;
        int t = item - cg * a.ntiles;
        const int tx = t % a.tiles_x;
        t /= a.tiles_x;
        const int ty = t % a.tiles_y;
        n = t / a.tiles_y;
        ty0 = ty * a.th;
        tx0 = tx * a.tw;
        if (wave < LW) {
            // instruction j = wave + LW * i covers PPI halo pixels x LPP parts
#pragma unroll 1
            for (int i = 0; i < lpa; ++i) {
                const int j = wave + LW * i;
                const int hpx = j * PPI + lane / LPP;
                unsigned off = DLF_OOB;
                if (hpx < npxh) {
                    const int hy = div_by(hpx, pw_m), hx = hpx - hy * pw;
                    const int gy = ty0 - 1 + hy, gx = tx0 - 1 + hx;
                    if (gy >= 0 && gy < a.h && gx >= 0 && gx < a.w_)
                        off = (unsigned)(((n * a.h + gy) * a.w_ + gx) * a.cin) * 2u;
                }
                atab[i * (LW * PPI)] = off;       // (the LPP lanes of a pixel write the same value)
            }
        }
    };
    // one weight load (the wave's i-th of stage c, into ring slot `slot`): fragment fi = wave +
    // LW * i (tap-major) of the block's channels, K chunk c
    const unsigned lane16 = (unsigned)lane * 16u;
    auto issue_w1 = [&](int i, int c, int slot) __attribute__((always_inline)) {
        const int fi = wave + LW * i;
        const int tap = fi / NCBW, cbi = fi - tap * NCBW;
        const int cb = min(cg * NCBW + cbi, a.ncb - 1);
        const int ks = (c >> 1) * 18 + tap * 2 + (c & 1);       // stage c = 16-channel chunk c of tap `tap`
        const bool real = fi < NWF;                             // uniform; surplus loads re-read the first fragment
        const half_t* base = (const half_t*)a.w + (real ? (size_t)(cb * a.nsteps + ks) * 512 : (size_t)0);
        const unsigned dst = lds0 + (unsigned)((real ? 2 * act_halfs + slot * W_HALFS + fi * 512
                                                     : 2 * act_halfs + nst * W_HALFS) * 2);
        dma16s(base, lane16, dst);
    };
    // one activation load (the wave's i-th of block b)
    auto issue_a1 = [&](int i, int b) __attribute__((always_inline)) {
        const int j = wave + LW * i;
        half_t* dst = j < na_i ? lds + (b & 1) * act_halfs + j * 512 : trash;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rin, (__attribute__((address_space(3))) void*)dst, 16,
                                                 atab[i * (LW * PPI)] + part16, b * (ACH * 2), 0, 0);
    };
    auto issue_w = [&](int c, int slot) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < LPW_W; ++i) issue_w1(i, c, slot);
    };
    auto issue_a = [&](int b) __attribute__((always_inline)) {
        // a loop, not unrolled: the addresses are formed one load at a time (unrolled, the compiler
        // forms all of them first, in registers the accumulators need)
#pragma unroll 1
        for (int i = 0; i < lpa; ++i) issue_a1(i, b);
    };
    const bool loader = wave < LW;
    auto first_stages = [&]() __attribute__((always_inline)) {
        if (!loader) return;
        issue_a(0);
        for (int c = 0; c < nst - 1; ++c)
            if (c < KT) issue_w(c, c);
    };
    setup((blockIdx.x & 7) * per_xcd + li);
    first_stages();

    for (;;) {
        // accumulators start at the bias
        acc_t acc[2][FP];
#pragma unroll
        for (int f = 0; f < 2; ++f) {
            const int cb = min(cg * NCBW + wc * 2 + f, a.ncb - 1);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if constexpr (I8) {
#pragma unroll
                    for (int p = 0; p < FP; ++p)
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[f][p][q * 4 + r] = 0;
                } else {
                    const f4v bv = *(const f4v*)(a.bias + cb * 32 + q * 8 + lhi * 4);
#pragma unroll
                    for (int p = 0; p < FP; ++p)
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[f][p][q * 4 + r] = bv[r];
                }
            }
        }

        // Loads retire in issue order: first A0 W0 .. W(nst-2); then iteration i requests W(i + nst - 1)
        // and, when it starts block i / CPB, the next block, all at the top of the stage.  A CU
        // takes one such instruction per 16 cycles, so the requests of a stage keep the issuing
        // waves, which issue in order, from their MFMAs for about a thousand cycles.  Only waves
        // 0-3, one per SIMD, request operands: while such a wave waits, the other wave of its SIMD
        // (4-7, which never touches memory in the K loop) has the matrix pipe to itself, and is
        // waiting at the next barrier by the time the first catches up.  (Requesting one load per
        // filter tap from every wave, or in mid-stage from half of them, was slower.)
        // Iteration c needs W(c), requested in iteration c - nst + 1, and block c / CPB, requested in
        // iteration (c / CPB - 1) * CPB: it may leave outstanding what was requested in the
        // iterations after both of these.
        auto w_thr = [&](int i) __attribute__((always_inline)) { return i >= 0 ? min(KT, i + nst) : min(KT, nst - 1); };     // stages requested through iteration i
        auto a_thr = [&](int i) __attribute__((always_inline)) { return i >= 0 ? 1 + min(NB - 1, i / CPB + 1) : 1; };        // blocks
        int slot = 0;
        for (int c = 0; c < KT; ++c) {
            const int blk = c / CPB, kq = c - blk * CPB;
            if (loader) {
                const int need = max(max(c - nst + 1, (blk - 1) * CPB), -1);
                wait_vmcnt_dyn(LPW_W * (w_thr(c - 1) - w_thr(need)) + lpa * (a_thr(c - 1) - a_thr(need)));
            }
            asm volatile("s_barrier" ::: "memory");
            // every wave is done with stage c - 1 (and, at the start of a block, with the block
            // before it; at c = 0, with the previous item's epilogue): their places may be refilled
            const bool do_w = c + nst - 1 < KT, do_a = kq == 0 && blk + 1 < NB;
            const int nslot = slot == 0 ? nst - 1 : slot - 1;
            if (loader) {
                if (do_w) issue_w(c + nst - 1, nslot);
                if (do_a) issue_a(blk + 1);
            }
            const unsigned wf = lds0 + (unsigned)((2 * act_halfs + slot * W_HALFS + (wc * 2) * 512 + lane * 8) * 2);
            const unsigned ab = lds0 + (unsigned)(((blk & 1) * act_halfs) * 2);
            const int q = 2 * kq + lhi;
            // halo pixel h, part q: byte address of h * ACH halfs + 8 * (q ^ f(h))
            auto b_at = [&](int h) __attribute__((always_inline)) {
                return ab + (unsigned)((h * ACH + ((((h >> SH) & (LPP - 1)) ^ q) << 3)) * 2);
            };
            // (with four pixel blocks the empty asm keeps the compiler from precomputing the tap
            // addresses of a stage outside the K loop, which costs two registers per tap and pixel
            // block; with two blocks there is room, and three instructions per address less)
            int h[FP];
#pragma unroll
            for (int p = 0; p < FP; ++p) {
                h[p] = hp0[p];
                if (FP > 2) asm volatile("" : "+v"(h[p]));
            }
            // Fragment reads are issued as instructions and waited for by count (LDS reads return
            // in order; while a direct-to-LDS load is pending the compiler would turn every wait
            // into a wait for all reads, the newest included).  Request order of a tap: A0, B0,
            // B1 .. B(FP-1), A1 -- the order its MFMAs need them -- each request of tap t + 1
            // placed behind an MFMA of tap t.  Before MFMA (f, p) of tap t the reads that may still
            // be outstanding are the tap's own later ones plus what has been requested of tap
            // t + 1 so far: FP before (0, 0); FP + 1 before (0, p > 0) and (1, 0); at the last tap,
            // with nothing requested behind it, FP - p and 0.
            h8 af[2][2], bf[2][FP];
            af[0][0] = lds_read16<0>(wf);
#pragma unroll
            for (int p = 0; p < FP; ++p) bf[0][p] = lds_read16<0>(b_at(h[p]));
            af[0][1] = lds_read16<1024>(wf);
            static_for<0, 9>([&](auto tc) __attribute__((always_inline)) {
                constexpr int tap = decltype(tc)::value, cur = tap & 1, nxt = cur ^ 1;
                constexpr bool more = tap + 1 < 9;
                const int toff = ((tap + 1) / 3) * pw + ((tap + 1) % 3);
                unsigned nb[FP];
#pragma unroll
                for (int p = 0; p < FP; ++p) nb[p] = more ? b_at(h[p] + toff) : 0u;
                __builtin_amdgcn_sched_barrier(0);
                lds_arrive2<FP>(af[cur][0], bf[cur][0]);
                static_for<0, 2 * FP>([&](auto kc) __attribute__((always_inline)) {
                    constexpr int kk = decltype(kc)::value, f = kk / FP, p = kk % FP;
                    if constexpr (f == 0 && p > 0) lds_arrive1<more ? FP + 1 : FP - p>(bf[cur][p]);
                    if constexpr (f == 1 && p == 0) lds_arrive1<more ? FP + 1 : 0>(af[cur][1]);
                    if constexpr (I8)
                        acc[f][p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4, af[cur][f]),
                                                                          __builtin_bit_cast(i32x4, bf[cur][p]), acc[f][p], 0, 0, 0);
                    else
                        acc[f][p] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[cur][f], bf[cur][p], acc[f][p], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if constexpr (more) {
                        if constexpr (kk == 0) {
                            af[nxt][0] = lds_read16<((tap + 1) * NCBW) * 1024>(wf);
                            bf[nxt][0] = lds_read16<0>(nb[0]);
                        } else if constexpr (kk < FP) {
                            bf[nxt][kk] = lds_read16<0>(nb[kk]);
                        } else if constexpr (kk == FP) {
                            af[nxt][1] = lds_read16<((tap + 1) * NCBW + 1) * 1024>(wf);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                });
            });
            slot = slot + 1 == nst ? 0 : slot + 1;
        }
        // every wave is done with the ring and the buffers (all loads were waited for above)
        asm volatile("s_barrier" ::: "memory");
        const int e_cg = cg, e_n = n, e_ty0 = ty0, e_tx0 = tx0;
        li += gridDim.x >> 3;
        const int next = (blockIdx.x & 7) * per_xcd + li;
        const bool more = li < per_xcd && next < a.nitems;
        if (more) {
            setup(next);
            first_stages();
        }

        // Epilogue, in passes of R pixels per wave through a transpose buffer in the last slot of
        // the weight ring, which the first stages of the next item do not touch: fp16, (pool),
        // activation; then 16 bytes per lane, 8 lanes covering the wave's 64 channels of a pixel.
        if constexpr (I8) {
            // Quantised form: a pass per 32-pixel block.  A lane holds, per channel block f and q, four
            // consecutive channels of its pixel: one dword of the pixel's 64-byte row in the wave's
            // transpose buffer (i8t_write_off); then lane 4 r + c stores part c of row r.
            static_assert(DLF_C3_WAVES * 32 * 64 <= W_HALFS * 2, "the transpose buffers fit one slot of the ring");
            unsigned char* tb8 = (unsigned char*)(wring + (nst - 1) * W_HALFS) + wave * (32 * 64);
            signed char* out8 = (signed char*)a.out;
            const float lo = a.act != 0 ? 0.0f : -128.0f;
            const int part = lane & 3;
            const int cch = (e_cg * NCBW + wc * 2) * 32 + part * 16;
            // with the 2x2 max pool folded in, the window is the 4 lanes of a quad (pix_to_rc): the maximum
            // is taken on the requantised values (the pooled layer's definition), lane 0 of a quad writes
            // row l32 / 4, and a pass stores 8 pooled pixels
            const bool pool = a.pool2 != 0;
            const int oh = pool ? a.h >> 1 : a.h, ow = pool ? a.w_ >> 1 : a.w_, otw = pool ? a.tw >> 1 : a.tw;
            const int oy0 = pool ? e_ty0 >> 1 : e_ty0, ox0 = pool ? e_tx0 >> 1 : e_tx0;
            const int onpix = pool ? npix >> 2 : npix;
#pragma unroll
            for (int p = 0; p < FP; ++p) {
#pragma unroll
                for (int f = 0; f < 2; ++f) {
                    const int cb = min(e_cg * NCBW + wc * 2 + f, a.ncb - 1);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const f4v sv = *(const f4v*)(a.scale + cb * 32 + q * 8 + lhi * 4);
                        const f4v bv = *(const f4v*)(a.bias + cb * 32 + q * 8 + lhi * 4);
                        float tv[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            float t = requant_biased(acc[f][p][q * 4 + r], sv[r], bv[r], lo);
                            if (pool) {
                                t = __builtin_fmaxf(t, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, t), 0xB1, 0xF, 0xF, true)));
                                t = __builtin_fmaxf(t, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, t), 0x4E, 0xF, 0xF, true)));
                            }
                            tv[r] = t;
                        }
                        const unsigned u = pack_low_bytes(tv[0], tv[1], tv[2], tv[3]);
                        if (!pool || (l32 & 3) == 0)
                            *(unsigned*)(tb8 + i8t_write_off(pool ? l32 >> 2 : l32, f * 2 + (q >> 1), (q & 1) * 2 + lhi)) = u;
                    }
                }
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int it = 0; it < 2; ++it) {
                    const int row = it * 16 + (lane >> 2);
                    const int opix = pool ? wp * (8 * FP) + p * 8 + row : wp * (32 * FP) + p * 32 + row;
                    const int ry = div_by(opix, tw_m), rx = opix - ry * otw;
                    const int gy = oy0 + ry, gx = ox0 + rx;
                    const bool ok = (!pool || row < 8) && opix < onpix && gy < oh && gx < ow && cch < a.cout;
                    const u4v v = i8t_read(tb8, row, part);
                    if (ok) *(u4v*)(out8 + (size_t)((e_n * oh + gy) * ow + gx) * (size_t)a.cout + cch) = v;
                }
                __builtin_amdgcn_wave_barrier();
            }
        } else {
        constexpr int R = (W_HALFS / (DLF_C3_WAVES * ROW)) >= 32 ? 32 : 16;
        static_assert(DLF_C3_WAVES * R * ROW <= W_HALFS, "the transpose buffers fit one slot of the ring");
        half_t* tb = wring + (nst - 1) * W_HALFS + wave * (R * ROW);
        const int part = lane & 7;
        const int cch = (e_cg * NCBW + wc * 2) * 32 + part * 8;
        const int rows_pass = a.pool2 ? R / 4 : R;
        const int oh = a.pool2 ? a.h >> 1 : a.h, ow = a.pool2 ? a.w_ >> 1 : a.w_;
        const int otw = a.pool2 ? a.tw >> 1 : a.tw;
        const int oy0 = a.pool2 ? e_ty0 >> 1 : e_ty0, ox0 = a.pool2 ? e_tx0 >> 1 : e_tx0;
        const int onpix = a.pool2 ? npix >> 2 : npix;
#pragma unroll
        for (int s = 0; s < 32 * FP / R; ++s) {
            const int p = s / (32 / R), sub = s % (32 / R);
            if (l32 / R == sub) {
#pragma unroll
                for (int f = 0; f < 2; ++f)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        unsigned u0 = cvt_pk(acc[f][p][q * 4 + 0], acc[f][p][q * 4 + 1]);
                        unsigned u1 = cvt_pk(acc[f][p][q * 4 + 2], acc[f][p][q * 4 + 3]);
                        int row = l32 % R;
                        bool wr = true;
                        if (a.pool2) {
                            // the 2x2 window is the 4 lanes of a quad (monotone rounding and clamps
                            // commute with the maximum)
                            u0 = quad_max_pk(u0);
                            u1 = quad_max_pk(u1);
                            wr = (l32 & 3) == 0;
                            row >>= 2;
                        }
                        u0 = pk_min(pk_max(u0, lo_e), hi_e);
                        u1 = pk_min(pk_max(u1, lo_e), hi_e);
                        const u2v uu = {u0, u1};
                        if (wr) *(u2v*)(tb + row * ROW + f * 32 + q * 8 + lhi * 4) = uu;
                    }
            }
            __builtin_amdgcn_wave_barrier();
            const int obase = wp * (a.pool2 ? 8 * FP : 32 * FP) + ((p * 32 + sub * R) >> (a.pool2 ? 2 : 0));
            for (int r0 = 0; r0 < rows_pass; r0 += 16) {
                u4v val[2], rv[2];
                bool ok[2];
                unsigned go[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int row = r0 + i * 8 + (lane >> 3);
                    const int opix = obase + row;
                    const int ry = div_by(opix, tw_m), rx = opix - ry * otw;
                    const int gy = oy0 + ry, gx = ox0 + rx;
                    ok[i] = row < rows_pass && opix < onpix && gy < oh && gx < ow && cch < a.cout;
                    go[i] = (unsigned)(((e_n * oh + gy) * ow + gx) * a.cout + cch);
                    if (resp != nullptr && ok[i]) rv[i] = *(const u4v*)(resp + go[i]);
                    val[i] = *(const u4v*)(tb + (row & (R - 1)) * ROW + part * 8);
                }
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    if (ok[i]) {
                        if (resp != nullptr) {
                            val[i].x = pk_min(pk_max(pk_add(val[i].x, rv[i].x), lo_r), hi_r);
                            val[i].y = pk_min(pk_max(pk_add(val[i].y, rv[i].y), lo_r), hi_r);
                            val[i].z = pk_min(pk_max(pk_add(val[i].z, rv[i].z), lo_r), hi_r);
                            val[i].w = pk_min(pk_max(pk_add(val[i].w, rv[i].w), lo_r), hi_r);
                        }
                        *(u4v*)(outp + go[i]) = val[i];
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        }
        if (!more) break;
        // this item's stores must not be counted among the loads of the next item's ring
        wait_vmcnt<0>();
    }
}

// ---- buffer loads: a tensor behind a buffer resource, so that the hardware's range check turns the
// loads of padding positions into zeros (an offset beyond the tensor returns 0: no branch, no
// select).  Offsets are bytes; DLF_OOB is an offset no tensor reaches (the host keeps tensors
// below 2 GiB on these paths).
// Mixed-precision multiply-add on one half of two packed fp16 pairs: c + a.lo * b.lo / c + a.hi * b.hi
// in fp32.  Written out because the compiler, given (float)a * (float)b + c in a loop that reuses b,
// converts b to fp32 once and keeps it there: twice the registers and a conversion per operand.
__device__ __forceinline__ float fma_mix_lo(unsigned a, unsigned b, float c)
{
    float d;
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[1,1,0]" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}
__device__ __forceinline__ float fma_mix_hi(unsigned a, unsigned b, float c)
{
    float d;
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,1,0] op_sel_hi:[1,1,0]" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}
// v[0..7] += x[0..7] * w[0..7] (8 channels of one filter tap)
__device__ __forceinline__ void dw_tap(float (&v)[8], const u4v& x, const u4v& w)
{
    v[0] = fma_mix_lo(x.x, w.x, v[0]);
    v[1] = fma_mix_hi(x.x, w.x, v[1]);
    v[2] = fma_mix_lo(x.y, w.y, v[2]);
    v[3] = fma_mix_hi(x.y, w.y, v[3]);
    v[4] = fma_mix_lo(x.z, w.z, v[4]);
    v[5] = fma_mix_hi(x.z, w.z, v[5]);
    v[6] = fma_mix_lo(x.w, w.w, v[6]);
    v[7] = fma_mix_hi(x.w, w.w, v[7]);
}

// Depthwise 3x3 convolution, pad 1, stride S, + bias + activation: the layer the paper's evaluation
// shows to be bound by memory, not arithmetic (Sec. V: layers of low operation count).  No LDS, no
// barrier: a wave owns 64 consecutive 16-byte vectors of the output rows of a strip (a run of
// (pixel, 8 channels) pairs, contiguous in NHWC) and walks down the strip.  Each lane keeps a window
// of input rows in registers -- the three columns x-1, x, x+1 of its 8 channels -- so every input
// vector is requested once per lane that needs it (three per row instead of nine per output), the
// rows one iteration ahead of their use; the 9 weight vectors and the bias of the lane's channels
// stay in registers for the whole strip.  Multiply-adds are mixed precision (fp16 operands, fp32
// sum).  Loads and stores are whole 1 KiB runs per wave.
template <int S>
__global__ __launch_bounds__(DLF_DW_WAVES * 64, 4) void k_dw(const DlfDwArgs a)
{
    constexpr int ROWS = S == 1 ? DLF_DW_ROWS1 : DLF_DW_ROWS2;
    constexpr int RING = S == 1 ? 4 : 5;                  // input rows in registers
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const i32x4 rin = make_rsrc(a.in, a.in_bytes);
    const unsigned cg_m = div_magic(a.cg);
    const half_t* wdw = (const half_t*)a.w;
    half_t* outp = (half_t*)a.out;
    const unsigned lo = act_lo(a.act), hi = act_hi(a.act);
    const int rowbytes = a.w_ * a.c * 2;
    const int nwaves = gridDim.x * DLF_DW_WAVES;
    for (int item = blockIdx.x * DLF_DW_WAVES + wave; item < a.nitems; item += nwaves) {
        int t = item;
        const int xr = t % a.nxr;
        t /= a.nxr;
        const int strip = t % a.nstrips, n = t / a.nstrips;
        const int e = xr * 64 + lane;
        const bool lv = e < a.rowv;
        const int ec = lv ? e : 0;
        const int ox = div_by(ec, cg_m), g = ec - ox * a.cg;
        u4v w[9];
#pragma unroll
        for (int k = 0; k < 9; ++k) w[k] = *(const u4v*)(wdw + k * a.cpad + g * 8);
        const f4v b0 = *(const f4v*)(a.bias + g * 8), b1 = *(const f4v*)(a.bias + g * 8 + 4);
        int voff[3];
#pragma unroll
        for (int d = 0; d < 3; ++d) {
            const int ix = ox * S - 1 + d;
            voff[d] = (lv && ix >= 0 && ix < a.w_) ? (ix * a.cg + g) * 16 : DLF_OOB;
        }
        const int oy0 = strip * ROWS;
        const int iy0 = oy0 * S - 1;                       // input row of window slot 0
        u4v win[RING][3];
        auto load_row = [&](int k) __attribute__((always_inline)) {
            const int iy = iy0 + k;
            const bool rok = iy >= 0 && iy < a.h;          // uniform; a row of padding reads zeros
            const int so = rok ? (n * a.h + iy) * rowbytes : 0;
#pragma unroll
            for (int d = 0; d < 3; ++d)
                win[k % RING][d] = __builtin_bit_cast(u4v, raw_buffer_load_x4(rin, rok ? voff[d] : DLF_OOB, so, 0));
        };
#pragma unroll
        for (int k = 0; k < RING - 1; ++k) load_row(k);
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            const int oy = oy0 + r;
            if (oy >= a.oh) break;
            // the rows of the next output row are requested before this one is computed
#pragma unroll
            for (int k = r * S + RING - S; k < r * S + RING; ++k) load_row(k);
            float v[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) { v[j] = b0[j]; v[j + 4] = b1[j]; }
#pragma unroll
            for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) dw_tap(v, win[(r * S + kh) % RING][kw], w[kh * 3 + kw]);
            u4v hv;
            hv.x = pk_min(pk_max(cvt_pk(v[0], v[1]), lo), hi);
            hv.y = pk_min(pk_max(cvt_pk(v[2], v[3]), lo), hi);
            hv.z = pk_min(pk_max(cvt_pk(v[4], v[5]), lo), hi);
            hv.w = pk_min(pk_max(cvt_pk(v[6], v[7]), lo), hi);
            if (lv) *(u4v*)(outp + ((size_t)((n * a.oh + oy) * a.rowv + e) << 3)) = hv;
        }
    }
}

// Depthwise 3x3 + 1x1 convolution fused (the pair MobileNet-style networks are made of: the
// depthwise layer has nine multiply-adds per value it reads and writes, so run alone it is pure
// memory traffic, and its output is read again at once by the 1x1 layer; Sec. V: layers of low
// operation count gain most from fusion).  The depthwise output never exists in memory: lane
// (pixel l % 32, K half l / 32) of a wave computes, for each 16-channel K step, the depthwise
// result of its pixel and its 8 channels from nine 16-byte loads (range-checked buffer loads:
// padding positions read zero), applies bias and activation, rounds to fp16 -- and holds exactly
// the MFMA "B" fragment of that K step, which is multiplied at once with the NB weight fragments
// (32 output channels each) of the wave's channel group.  No LDS between the two layers, no
// workgroup barrier in the loop; the loads of K step k + 1 are in flight while step k is computed.
// The depthwise weights and bias sit in LDS (read once per workgroup), the 1x1 fragments stream
// from L2 as in k_pw.  Waves of a workgroup take consecutive items, channel group fastest, so the
// channel groups of one pixel group find their inputs in the CU's cache.
template <int NB>
__global__ __launch_bounds__(DLF_DWPW_WAVES * 64, 2) void k_dwpw(const DlfDwPwArgs a)
{
    constexpr int ROW = 32 * NB + 8;                 // halfs per pixel row of the transpose buffer
    constexpr int LPP = 4 * NB;                      // lanes (16-byte vectors) per pixel
    constexpr int NPASS = 2 * NB;                    // read-back passes of 64 vectors
    // (the wave index as a scalar: what is derived from it -- work items, loop exits, weight offsets --
    // is then uniform for the compiler too)
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    const int c = a.c;
    half_t* wl = lds;                                // [9][c] fp16
    float* bl = (float*)(lds + 9 * c);               // [c] fp32
    half_t* tb = lds + 11 * c + wave * (32 * ROW);
    for (int i = threadIdx.x; i < (9 * c) >> 3; i += DLF_DWPW_WAVES * 64) ((u4v*)wl)[i] = ((const u4v*)a.wdw)[i];
    for (int i = threadIdx.x; i < c >> 2; i += DLF_DWPW_WAVES * 64) ((f4v*)bl)[i] = ((const f4v*)a.bdw)[i];
    __syncthreads();
    const i32x4 rin = make_rsrc(a.in, a.in_bytes);
    half_t* outp = (half_t*)a.out;
    const unsigned lo_d = act_lo(a.act_dw), hi_d = act_hi(a.act_dw);
    const unsigned lo_p = act_lo(a.act_pw), hi_p = act_hi(a.act_pw);
    const int nsteps = a.nsteps;                     // even: c is a multiple of 32
    const int ohw = a.oh * a.ow;
    const unsigned ohw_m = div_magic(ohw), ow_m = div_magic(a.ow), ncg_m = div_magic(a.n_cg);
    const int nwaves = gridDim.x * DLF_DWPW_WAVES;
    for (int item = blockIdx.x * DLF_DWPW_WAVES + wave; item < a.nitems; item += nwaves) {
        const int pg = div_by(item, ncg_m), cg = item - pg * a.n_cg;
        int pix = pg * 32 + l32;
        pix = pix < a.m ? pix : a.m - 1;             // clamped lanes compute a result nobody stores
        const int n = div_by(pix, ohw_m), r = pix - n * ohw;
        const int oy = div_by(r, ow_m), ox = r - oy * a.ow;
        // byte offsets of the nine taps' 16 bytes (K step 0), or out of range for padding
        int voff[9];
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                const int iy = oy * a.stride - 1 + kh, ix = ox * a.stride - 1 + kw;
                const bool ok = iy >= 0 && iy < a.h && ix >= 0 && ix < a.w_;
                voff[kh * 3 + kw] = ok ? (((n * a.h + iy) * a.w_ + ix) * c + lhi * 8) * 2 : DLF_OOB;
            }
        const h8* wp[NB];
#pragma unroll
        for (int f = 0; f < NB; ++f) {
            const int cb = min(cg * NB + f, a.ncb - 1);
            wp[f] = (const h8*)a.wpw + (size_t)cb * nsteps * 64 + lane;
        }
        f16v acc[NB];
#pragma unroll
        for (int f = 0; f < NB; ++f)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[f][q] = 0.0f;
        u4v x[2][9];
        h8 ar[2][NB];
        // K step ks: inputs and weight fragments of step ks + 1 are requested first (the last step
        // requests a step that does not exist: the loads land in the next pixel's channels or
        // beyond the tensor, where the range check returns zero, and in the zero steps behind the
        // packed weights; nothing uses them)
        auto request = [&](int ks, u4v (&xn)[9], h8 (&an)[NB]) __attribute__((always_inline)) {
#pragma unroll
            for (int k = 0; k < 9; ++k)
                xn[k] = __builtin_bit_cast(u4v, raw_buffer_load_x4(rin, voff[k], ks * 32, 0));
#pragma unroll
            for (int f = 0; f < NB; ++f) an[f] = wp[f][ks * 64];
        };
        auto step = [&](int ks, const u4v (&xc)[9], u4v (&xn)[9], const h8 (&ac)[NB], h8 (&an)[NB])
                        __attribute__((always_inline)) {
            request(ks + 1, xn, an);
            __builtin_amdgcn_sched_barrier(0);       // all of them before the arithmetic, not sunk into it
            const int ch = ks * 16 + lhi * 8;
            const f4v b0 = *(const f4v*)(bl + ch), b1 = *(const f4v*)(bl + ch + 4);
            float v[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) { v[j] = b0[j]; v[j + 4] = b1[j]; }
#pragma unroll
            for (int k = 0; k < 9; ++k) dw_tap(v, xc[k], *(const u4v*)(wl + k * c + ch));
            u4v hv;
            hv.x = pk_min(pk_max(cvt_pk(v[0], v[1]), lo_d), hi_d);
            hv.y = pk_min(pk_max(cvt_pk(v[2], v[3]), lo_d), hi_d);
            hv.z = pk_min(pk_max(cvt_pk(v[4], v[5]), lo_d), hi_d);
            hv.w = pk_min(pk_max(cvt_pk(v[6], v[7]), lo_d), hi_d);
            const h8 b = __builtin_bit_cast(h8, hv);
#pragma unroll
            for (int f = 0; f < NB; ++f) acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ac[f], b, acc[f], 0, 0, 0);
        };
        request(0, x[0], ar[0]);
        for (int ks = 0; ks < nsteps; ks += 2) {
            step(ks, x[0], x[1], ar[0], ar[1]);
            step(ks + 1, x[1], x[0], ar[1], ar[0]);
        }
        // ---- result + bias -> activation -> wave-private transpose buffer [pixel][channel] ----
#pragma unroll
        for (int f = 0; f < NB; ++f) {
            const int cb = min(cg * NB + f, a.ncb - 1);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f4v bv = *(const f4v*)(a.bpw + cb * 32 + q * 8 + lhi * 4);
                unsigned u0 = cvt_pk(acc[f][q * 4 + 0] + bv[0], acc[f][q * 4 + 1] + bv[1]);
                unsigned u1 = cvt_pk(acc[f][q * 4 + 2] + bv[2], acc[f][q * 4 + 3] + bv[3]);
                u0 = pk_min(pk_max(u0, lo_p), hi_p);
                u1 = pk_min(pk_max(u1, lo_p), hi_p);
                const u2v uu = {u0, u1};
                *(u2v*)(tb + l32 * ROW + f * 32 + q * 8 + lhi * 4) = uu;
            }
        }
        __builtin_amdgcn_wave_barrier();
        // ---- 16 bytes per lane: LPP lanes cover the 32 * NB channels of one pixel ----
        const int part = lane % LPP;
        const int cc = cg * (32 * NB) + part * 8;
#pragma unroll
        for (int i = 0; i < NPASS; ++i) {
            const int px = i * (64 / LPP) + lane / LPP;
            const int gpix = pg * 32 + px;
            if (gpix < a.m && cc < a.cout)
                *(u4v*)(outp + (size_t)gpix * a.cout + cc) = *(const u4v*)(tb + px * ROW + part * 8);
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// Depthwise 3x3 + 1x1 convolution as a tile kernel.  What k_dwpw gets wrong is its memory access (a
// K step of 16 channels per pixel uses a quarter of each line); here the depthwise phase reads
// exactly as k_dw does -- a wave's 64 lanes cover whole pixels' channels, contiguous in memory, a
// window of input rows slides down in registers -- and hands its result to the 1x1 phase through an
// LDS tile [pixel][c + 8] (the 8 halfs of padding spread the pixels over the banks).  One barrier
// between the phases, one before the tile buffer is reused; several workgroups share a CU, so one's
// vector arithmetic overlaps another's MFMAs and stores.
//   Phase 2 work units: (32-channel block, group of up to four 32-pixel blocks), dealt round-robin
// to the four waves; weight fragments stream from L2 through a register ring, "B" fragments come
// from the tile with one 16-byte LDS read per lane.
// Phase 1 of k_dwt for a wave: RW output rows of the depthwise layer, stride S, written to the LDS
// tile.  Everything about the row window is static (RW is a template parameter: the kernel
// switches once per tile), so the compiler knows at every use how many newer loads may still be
// outstanding; with a run-time row count the loads sit under conditions and every join waits for
// all of them.  Input rows of output row r + PF are requested before row r is computed.
template <int S, int RW>
__device__ __forceinline__ void dwt_phase1(const i32x4 rin, const int (&voff)[3], int img_row0, int h, int rowbytes,
                                           int iy0, const u4v (&w)[9], const f4v b0, const f4v b1, unsigned lo_d,
                                           unsigned hi_d, half_t* dst, int row_halfs)
{
    constexpr int NR = (RW - 1) * S + 3;             // input rows the wave needs
    constexpr int PF = S == 1 ? 3 : 2;
    constexpr int RING = NR < PF * S + 3 ? NR : PF * S + 3;
    u4v win[RING][3];
    auto load_row = [&](int k) __attribute__((always_inline)) {
        const int iy = iy0 + k;
        const bool rok = iy >= 0 && iy < h;          // uniform; a row of padding reads zeros
        const int so = rok ? (img_row0 + iy) * rowbytes : 0;
#pragma unroll
        for (int d = 0; d < 3; ++d)
            win[k % RING][d] = __builtin_bit_cast(u4v, raw_buffer_load_x4(rin, rok ? voff[d] : DLF_OOB, so, 0));
    };
    constexpr int FIRST = NR < RING - S + (RING == NR ? S : 0) ? NR : RING - S + (RING == NR ? S : 0);
#pragma unroll
    for (int k = 0; k < FIRST; ++k) load_row(k);
#pragma unroll
    for (int r = 0; r < RW; ++r) {
#pragma unroll
        for (int q = 0; q < S; ++q) {
            const int k = (r + PF) * S + 3 - S + q;  // a row of output row r + PF not yet requested
            if (k >= FIRST && k < NR) load_row(k);
        }
        float v[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) { v[i] = b0[i]; v[i + 4] = b1[i]; }
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) dw_tap(v, win[(r * S + kh) % RING][kw], w[kh * 3 + kw]);
        u4v hv;
        hv.x = pk_min(pk_max(cvt_pk(v[0], v[1]), lo_d), hi_d);
        hv.y = pk_min(pk_max(cvt_pk(v[2], v[3]), lo_d), hi_d);
        hv.z = pk_min(pk_max(cvt_pk(v[4], v[5]), lo_d), hi_d);
        hv.w = pk_min(pk_max(cvt_pk(v[6], v[7]), lo_d), hi_d);
        *(u4v*)(dst + r * row_halfs) = hv;
    }
}

// Phase 2 of k_dwt for a wave: its work units of the 1x1 layer.  The weight fragments of all the
// wave's units form one stream through a ring of D K steps (D divides the K steps of a unit, so
// ring slots are static): a fragment is requested D steps before its use, across unit boundaries,
// and the round trip to L2 is paid once per tile, not once per ring turn.
template <int D>
__device__ __forceinline__ void dwt_phase2(const DlfDwtArgs& a, const half_t* tile, half_t* tb, int cs, int wave,
                                           int lane, int n, int ty0, int tx0, unsigned tw_m, unsigned lo_p,
                                           unsigned hi_p)
{
    constexpr int ROW = 32 + 8;
    const int l32 = lane & 31, lhi = lane >> 5;
    half_t* outp = (half_t*)a.out;
    const int nunits = a.ncb * a.npg;
    int pf_u = wave, pf_ks = 0;                      // the stream's next fragment: unit, K step
    const i32x4 rw = make_rsrc(a.wpw, 0xffffffffu);
    const int lane16 = lane * 16;
    auto next_frag = [&]() __attribute__((always_inline)) {
        // past the last unit the stream re-reads the last block's first fragment (never used)
        const int cbp = min(pf_u, nunits - 1) / a.npg;
        const h8 f = wfrag(rw, lane16, (unsigned)__builtin_amdgcn_readfirstlane((cbp * a.nsteps + pf_ks) * 1024));
        const bool live = pf_u < nunits;
        const int nks = live ? pf_ks + 1 : pf_ks;
        const bool wrap = nks == a.nsteps;
        pf_ks = wrap ? 0 : nks;
        pf_u = wrap ? pf_u + DLF_DWT_WAVES : pf_u;
        return f;
    };
    h8 ar[D];
#pragma unroll
    for (int j = 0; j < D; ++j) ar[j] = next_frag();
    for (int u = wave; u < nunits; u += DLF_DWT_WAVES) {
        const int cb = u / a.npg, pgi = u - cb * a.npg;
        const int pb0 = pgi * 4;
        const int nb = min(4, a.npb - pb0);          // pixel blocks of this unit (uniform)
        const half_t* bsrc[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            // blocks beyond the tile repeat its last pixel: multiplied, never stored
            const int px = min((pb0 + p) * 32 + l32, a.tp - 1);
            bsrc[p] = tile + px * cs + lhi * 8;
        }
        f16v acc[4];
#pragma unroll
        for (int p = 0; p < 4; ++p)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[p][q] = 0.0f;
        // the K loop, one copy per number of pixel blocks (a switch per unit, nothing conditional inside)
        auto kloop = [&](auto nbc) __attribute__((always_inline)) {
            constexpr int NBK = decltype(nbc)::value;
            for (int s0 = 0; s0 < a.nsteps; s0 += D) {
#pragma unroll
                for (int j = 0; j < D; ++j) {
                    h8 bf[NBK];
#pragma unroll
                    for (int p = 0; p < NBK; ++p) bf[p] = *(const h8*)(bsrc[p] + (s0 + j) * 16);
#pragma unroll
                    for (int p = 0; p < NBK; ++p)
                        acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ar[j], bf[p], acc[p], 0, 0, 0);
                    ar[j] = next_frag();
                }
            }
        };
        if (nb == 4) kloop(std::integral_constant<int, 4>());
        else if (nb == 3) kloop(std::integral_constant<int, 3>());
        else if (nb == 2) kloop(std::integral_constant<int, 2>());
        else kloop(std::integral_constant<int, 1>());
        // epilogue: bias, activation, fp16; 32 pixels at a time through the wave's transpose buffer
        f4v bias[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) bias[q] = *(const f4v*)(a.bpw + cb * 32 + q * 8 + lhi * 4);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            if (p < nb) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    unsigned u0 = cvt_pk(acc[p][q * 4 + 0] + bias[q][0], acc[p][q * 4 + 1] + bias[q][1]);
                    unsigned u1 = cvt_pk(acc[p][q * 4 + 2] + bias[q][2], acc[p][q * 4 + 3] + bias[q][3]);
                    u0 = pk_min(pk_max(u0, lo_p), hi_p);
                    u1 = pk_min(pk_max(u1, lo_p), hi_p);
                    const u2v uu = {u0, u1};
                    *(u2v*)(tb + l32 * ROW + q * 8 + lhi * 4) = uu;
                }
                __builtin_amdgcn_wave_barrier();
                // 4 lanes cover the 32 channels of a pixel: 16 pixels per pass
                const int part = lane & 3;
                const int cc = cb * 32 + part * 8;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int pl = i * 16 + (lane >> 2);
                    const int px = (pb0 + p) * 32 + pl;
                    const int row = div_by(px, tw_m), colp = px - row * a.tw;
                    const int oy = ty0 + row, ox = tx0 + colp;
                    if (px < a.tp && oy < a.oh && ox < a.ow && cc < a.cout)
                        *(u4v*)(outp + ((size_t)((n * a.oh + oy) * a.ow + ox) * a.cout + cc)) =
                            *(const u4v*)(tb + pl * ROW + part * 8);
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
    }
}

template <int S>
__global__ __launch_bounds__(DLF_DWT_WAVES * 64, 2) void k_dwt(const DlfDwtArgs a)
{
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int c = a.c, cs = c + 8;
    half_t* tile = lds;                              // [tp][c + 8]
    half_t* tb = lds + a.tp * cs + wave * DLF_DWT_EPI_HALFS;
    const i32x4 rin = make_rsrc(a.in, a.in_bytes);
    const half_t* wdw = (const half_t*)a.wdw;
    const unsigned lo_d = act_lo(a.act_dw), hi_d = act_hi(a.act_dw);
    const unsigned lo_p = act_lo(a.act_pw), hi_p = act_hi(a.act_pw);
    const int rowbytes = a.w_ * c * 2;
    const unsigned tw_m = div_magic(a.tw);
    // phase 1 role of the lane: column pxl of the wave's pxw pixels, channel group g
    const int cg_shift = __builtin_ctz(a.cg);
    const int pxl = lane >> cg_shift, g = lane & (a.cg - 1);
    const int wxi = wave % a.wx, wyi = wave / a.wx;
    // the lane's nine weight vectors and bias stay in registers over all tiles
    u4v w[9];
#pragma unroll
    for (int k = 0; k < 9; ++k) w[k] = *(const u4v*)(wdw + k * c + g * 8);
    const f4v b0 = *(const f4v*)(a.bdw + g * 8), b1 = *(const f4v*)(a.bdw + g * 8 + 4);

    // (work item i goes to XCD i % 8 when the grid is a multiple of 8: an XCD's items are a
    // contiguous eighth of the tiles, so the rows neighbouring tiles share are in its L2)
    const int per_xcd = (a.ntiles + 7) >> 3;
    for (int i = blockIdx.x; i < 8 * per_xcd; i += gridDim.x) {
        const int t = (i & 7) * per_xcd + (i >> 3);
        if (t >= a.ntiles) continue;
        int r_ = t;
        const int tx = r_ % a.tiles_x;
        r_ /= a.tiles_x;
        const int ty = r_ % a.tiles_y, n = r_ / a.tiles_y;
        const int ty0 = ty * a.th, tx0 = tx * a.tw;
        // ---------------- phase 1: depthwise rows of this wave -> LDS tile ----------------
        {
            const int col = wxi * a.pxw + pxl;                 // column inside the tile
            const int ox = tx0 + col;
            const bool lv = ox < a.ow;
            int voff[3];
#pragma unroll
            for (int d = 0; d < 3; ++d) {
                const int ix = ox * S - 1 + d;
                voff[d] = (lv && ix >= 0 && ix < a.w_) ? (ix * a.cg + g) * 16 : DLF_OOB;
            }
            const int oyw = ty0 + wyi * a.rw;                  // first output row of the wave
            const int iy0 = oyw * S - 1;
            half_t* dst = tile + ((wyi * a.rw) * a.tw + col) * cs + g * 8;
            const int rh = a.tw * cs;
            switch (a.rw) {                                    // the shapes the host offers
            case 1: dwt_phase1<S, 1>(rin, voff, n * a.h, a.h, rowbytes, iy0, w, b0, b1, lo_d, hi_d, dst, rh); break;
            case 2: dwt_phase1<S, 2>(rin, voff, n * a.h, a.h, rowbytes, iy0, w, b0, b1, lo_d, hi_d, dst, rh); break;
            case 4: dwt_phase1<S, 4>(rin, voff, n * a.h, a.h, rowbytes, iy0, w, b0, b1, lo_d, hi_d, dst, rh); break;
            case 7: dwt_phase1<S, 7>(rin, voff, n * a.h, a.h, rowbytes, iy0, w, b0, b1, lo_d, hi_d, dst, rh); break;
            case 8: dwt_phase1<S, 8>(rin, voff, n * a.h, a.h, rowbytes, iy0, w, b0, b1, lo_d, hi_d, dst, rh); break;
            case 14: dwt_phase1<S, 14>(rin, voff, n * a.h, a.h, rowbytes, iy0, w, b0, b1, lo_d, hi_d, dst, rh); break;
            default: dwt_phase1<S, 16>(rin, voff, n * a.h, a.h, rowbytes, iy0, w, b0, b1, lo_d, hi_d, dst, rh); break;
            }
        }
        __syncthreads();
        // ---------------- phase 2: 1x1 convolution of the tile ----------------
        if (a.nsteps >= 8) dwt_phase2<8>(a, tile, tb, cs, wave, lane, n, ty0, tx0, tw_m, lo_p, hi_p);
        else if (a.nsteps == 4) dwt_phase2<4>(a, tile, tb, cs, wave, lane, n, ty0, tx0, tw_m, lo_p, hi_p);
        else dwt_phase2<2>(a, tile, tb, cs, wave, lane, n, ty0, tx0, tw_m, lo_p, hi_p);
        __syncthreads();                 // every wave is done reading the tile
    }
}


// Depthwise 3x3 + 1x1 convolution where a map has many channels and few pixels (MobileNet's 14 x 14
// and 7 x 7 maps of 256 - 1024 channels).  There the layers are small, a launch costs about as much
// as the arithmetic, and the depthwise result is best never written: Sec. V finds exactly these
// low-operation-count layers to gain most from fusion.  The tile kernel above cannot take them (a
// wave's 64 lanes cover one pixel's 512 channels: its tiles degenerate to columns).
//   Work item = (tile of up to 8 x 8 output pixels, slice of 8 * CBW channel blocks of the 1x1 layer):
// one workgroup of eight waves, one item, one workgroup per CU.  The slices of a tile run on the same
// XCD (workgroups i, i + 8, ...), so their common input reaches that L2 once.
//   The c channels are taken kh = 256 or 512 at a time; per pass
//     1. region: the tile's input region, kh channels per pixel, global -> LDS by direct loads, one
//        instruction = 1 KiB = one pixel's 512 channels or two pixels' 256; pixels outside the
//        image are requested beyond the buffer's range and arrive as zeros (the padding is data,
//        no branch).  Behind the pixels the same way: the pass's depthwise weights (nine taps,
//        "pixels" of their own) and bias, so that no lane has loads of its own for them.  Where
//        LDS holds the regions of all passes they are all requested at the start (a region takes
//        a trip to memory, 4 - 5 thousand cycles), else one after the other;
//     2. depthwise: a wave takes every eighth pixel (pair), lane = 8 channels; nine 16-byte LDS reads,
//        fp32 sums in the order of k_dw (same bits), result to the LDS tile [pixel][kh + 8];
//     3. 1x1: every wave CBW channel blocks x the tile's two 32-pixel blocks, accumulators kept over
//        the passes; "B" fragments from the tile, weight fragments through a register ring of 8 K
//        steps, first requested behind the regions (the ring's trip to L2 hides behind step 2, and
//        the regions do not share the CU's intake with it).
//   Steps 2 and 3 were also built as a pipeline over 128-channel passes with half of the waves
// filtering while the other half multiplies: the two halves slowed each other down by what the
// overlap should have gained, and the phases' barriers came on top (20 us against 19).
//   Results leave through wave-private transpose buffers (in the regions' space), 64 * CBW bytes
// per pixel and instruction group.
template <int S, int CBW>
__global__ __launch_bounds__(DLF_DWS_WAVES * 64, 1) void k_dws(const DlfDwsArgs a)
{
    constexpr int D = 8;
    constexpr int ROW = 32 * CBW + 8;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    const int KH = a.kh, cs = KH + 8;
    const int ng_shift = KH == 512 ? 6 : 5;                  // lanes per pixel = kh / 8
    const int ppi = 64 >> ng_shift;                          // pixels per load instruction and per wave step
    const int g = lane & ((1 << ng_shift) - 1), psub = lane >> ng_shift;
    const int per8 = blockIdx.x >> 3;
    // (an XCD takes a contiguous eighth of the tiles: the halo a tile shares with its neighbours is in that XCD's L2)
    const int sl = per8 % a.nsl, tile = (blockIdx.x & 7) * ((a.ntiles + 7) >> 3) + per8 / a.nsl;
    if (tile >= a.ntiles) return;
    int r_ = tile;
    const int tx = r_ % a.tiles_x;
    r_ /= a.tiles_x;
    const int ty = r_ % a.tiles_y, n = r_ / a.tiles_y;
    const int oy0 = ty * a.th, ox0 = tx * a.tw;
    const int iy0 = oy0 * S - 1, ix0 = ox0 * S - 1;
    const int in_halfs = DLF_DWS_IN_BYTES(a.rp, KH) / 2, epi_halfs = DLF_DWS_EPI_BYTES(CBW) / 2;
    const bool resident = a.nbuf == a.nkh;                   // every pass has a region buffer of its own
    half_t* const inb = lds;
    half_t* const mid = lds + (a.nbuf * in_halfs > epi_halfs ? a.nbuf * in_halfs : epi_halfs);
    half_t* const tb = lds + wave * (32 * ROW);
    half_t* outp = (half_t*)a.out;
    const unsigned lo_d = act_lo(a.act_dw), hi_d = act_hi(a.act_dw);
    const unsigned lo_p = act_lo(a.act_pw), hi_p = act_hi(a.act_pw);
    const unsigned tw_m = div_magic(a.tw), rw_m = div_magic(a.rw);

    // ---- the wave's weight stream: CBW fragments per K step, D steps ahead ----
    const i32x4 rwt = make_rsrc(a.wpw, 0xffffffffu);
    const int lane16 = lane * 16;
    const int cb0 = (sl * DLF_DWS_WAVES + wave) * CBW;
    const bool live = cb0 < a.ncb;                           // uniform: a wave beyond the last block only loads and filters
    unsigned wo[CBW];
#pragma unroll
    for (int j = 0; j < CBW; ++j)
        wo[j] = (unsigned)__builtin_amdgcn_readfirstlane(min(cb0 + j, a.ncb - 1) * a.nsteps * 1024);
    int pf_ks = 0;
    h8 ar[D][CBW];
    auto request = [&](int slot) __attribute__((always_inline)) {
        const unsigned so = (unsigned)min(pf_ks, a.nsteps - 1) * 1024u;      // past the end: re-read, never used
#pragma unroll
        for (int j = 0; j < CBW; ++j) ar[slot][j] = wfrag(rwt, lane16, wo[j] + so);
        ++pf_ks;
    };

    // ---- step 1: this wave's share of a region's load instructions ----
    // (written as instructions: of a direct-to-LDS load the compiler only knows that it writes LDS
    // at some time, and it would put a wait for all loads in front of every LDS read that follows;
    // here the waits are counted by hand)
    const i32x4 rin = make_rsrc(a.in, a.in_bytes);
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) half_t*)lds;
    const int ni = (a.rp + ppi - 1) >> (6 - ng_shift);
    auto issue_in = [&](int pass) __attribute__((always_inline)) {
        const unsigned dst0 = lds0 + (unsigned)((resident ? pass : 0) * in_halfs) * 2u;
#pragma unroll 1
        for (int i = wave; i < ni; i += DLF_DWS_WAVES) {
            const int rp = i * ppi + psub;
            unsigned off = (unsigned)DLF_OOB;
            if (rp < a.rp) {
                const int ry = div_by(rp, rw_m), rx = rp - ry * a.rw;
                const int gy = iy0 + ry, gx = ix0 + rx;
                if (gy >= 0 && gy < a.h && gx >= 0 && gx < a.w_)
                    off = (unsigned)(((n * a.h + gy) * a.w_ + gx) * a.c + pass * KH + g * 8) * 2u;
            }
            asm volatile("s_mov_b32 m0, %2\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds" ::"v"(off), "s"(rin),
                         "s"(dst0 + (unsigned)i * 1024u)
                         : "memory", "m0");
        }
    };

    // the depthwise weights and bias of the lane's 8 channels, for one pass (uniform parts of the
    // addresses in scalar registers: one lane offset serves all eleven loads)
    const i32x4 rdw = make_rsrc(a.wdw, (unsigned)(9 * a.c * 2)), rdb = make_rsrc(a.bdw, (unsigned)(a.c * 4));
    u4v w[9];
    f4v b0, b1;
    auto load_dw_weights = [&](int pass) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < 9; ++k)
            w[k] = __builtin_bit_cast(u4v, raw_buffer_load_x4(rdw, g * 16, (k * a.c + pass * KH) * 2, 0));
        b0 = __builtin_bit_cast(f4v, raw_buffer_load_x4(rdb, g * 32, pass * KH * 4, 0));
        b1 = __builtin_bit_cast(f4v, raw_buffer_load_x4(rdb, g * 32 + 16, pass * KH * 4, 0));
    };

    f16v acc[CBW][2];
#pragma unroll
    for (int j = 0; j < CBW; ++j)
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[j][p][q] = 0.0f;

    // Loads retire in the order of their requests, so "region q has landed" is "at most the requests
    // behind it are outstanding".
    const int n_in = (ni - wave + DLF_DWS_WAVES - 1) / DLF_DWS_WAVES;     // this wave's loads per region
    const int n_ring = live ? D * CBW : 0;
    const int ahead = resident ? a.nkh : 1;
    load_dw_weights(0);                                      // (requested first: the oldest loads)
    asm volatile("" ::: "memory");
    for (int q = 0; q < ahead; ++q) issue_in(q);
    // (the ring's first turn behind the regions: requested only when the first region has landed it
    // slows the depthwise step by what the region gains)
    if (live) {
#pragma unroll
        for (int d = 0; d < D; ++d) request(d);
    }
    for (int pass = 0; pass < a.nkh; ++pass) {
        // behind region `pass`: the later regions (if all were requested at the start) and the ring
        wait_vmcnt_dyn((resident ? (a.nkh - 1 - pass) * n_in : 0) + n_ring);
        asm volatile("s_barrier" ::: "memory");      // the region has landed; everyone is done multiplying the previous tile
        // ---- step 2: depthwise ----
        {
            const half_t* const region = inb + (resident ? pass : 0) * in_halfs;
            if (pass > 0) load_dw_weights(pass);
#pragma unroll 1
            for (int p0 = wave * ppi; p0 < a.tp; p0 += DLF_DWS_WAVES * ppi) {
                const int p = p0 + psub;
                const int pc = min(p, a.tp - 1);
                const int py = div_by(pc, tw_m), px = pc - py * a.tw;
                const half_t* src = region + ((py * S) * a.rw + px * S) * KH + g * 8;
                float v[8];
#pragma unroll
                for (int i = 0; i < 4; ++i) { v[i] = b0[i]; v[i + 4] = b1[i]; }
#pragma unroll
                for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                    for (int kw = 0; kw < 3; ++kw) {
                        const u4v x = *(const u4v*)(src + (kh * a.rw + kw) * KH);
                        dw_tap(v, x, w[kh * 3 + kw]);
                    }
                u4v hv;
                hv.x = pk_min(pk_max(cvt_pk(v[0], v[1]), lo_d), hi_d);
                hv.y = pk_min(pk_max(cvt_pk(v[2], v[3]), lo_d), hi_d);
                hv.z = pk_min(pk_max(cvt_pk(v[4], v[5]), lo_d), hi_d);
                hv.w = pk_min(pk_max(cvt_pk(v[6], v[7]), lo_d), hi_d);
                if (p < a.tp) *(u4v*)(mid + p * cs + g * 8) = hv;
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");      // the tile is complete; the region may be overwritten
        if (!resident && pass + 1 < a.nkh) issue_in(pass + 1);
        // ---- step 3: 1x1 on MFMA ----
        if (live) {
            const half_t* bsrc[2];
#pragma unroll
            for (int p = 0; p < 2; ++p) bsrc[p] = mid + min(p * 32 + l32, a.tp - 1) * cs + lhi * 8;
            // the fragments of step s + 1 are read before step s is multiplied, and the ring slot of
            // step s is requested again right behind its multiplies (the scheduler would otherwise
            // gather a turn's requests at its end: one exposed trip to L2 per turn)
            const int last_s = (KH >> 4) - 1;
            h8 bf[2][2];
#pragma unroll
            for (int p = 0; p < 2; ++p) bf[0][p] = *(const h8*)(bsrc[p]);
            for (int s0 = 0; s0 <= last_s; s0 += D) {
#pragma unroll
                for (int j = 0; j < D; ++j) {
                    const int sn = min(s0 + j + 1, last_s);
#pragma unroll
                    for (int p = 0; p < 2; ++p) bf[(j + 1) & 1][p] = *(const h8*)(bsrc[p] + sn * 16);
#pragma unroll
                    for (int c = 0; c < CBW; ++c)
#pragma unroll
                        for (int p = 0; p < 2; ++p)
                            acc[c][p] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ar[j][c], bf[j & 1][p], acc[c][p], 0, 0, 0);
                    request(j);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    }
    if (!live) return;
    // ---- epilogue: bias, activation, fp16; 32 pixels x 32 * CBW channels at a time ----
    // (the transpose buffers lie in the regions' space: nobody reads a region after the last
    // barrier, and no load into one is outstanding)
    constexpr int LPX = 4 * CBW;                             // lanes per pixel in the store phase
    constexpr int PPP = 64 / LPX;                            // pixels per store instruction
    // (the bias before the first store: a load behind a store waits for the store as well)
    f4v biasv[CBW][4];
#pragma unroll
    for (int c = 0; c < CBW; ++c)
#pragma unroll
        for (int q = 0; q < 4; ++q) biasv[c][q] = *(const f4v*)(a.bpw + min(cb0 + c, a.ncb - 1) * 32 + q * 8 + lhi * 4);
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        if (p * 32 < a.tp) {
#pragma unroll
            for (int c = 0; c < CBW; ++c) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f4v bias = biasv[c][q];
                    unsigned u0 = cvt_pk(acc[c][p][q * 4 + 0] + bias[0], acc[c][p][q * 4 + 1] + bias[1]);
                    unsigned u1 = cvt_pk(acc[c][p][q * 4 + 2] + bias[2], acc[c][p][q * 4 + 3] + bias[3]);
                    u0 = pk_min(pk_max(u0, lo_p), hi_p);
                    u1 = pk_min(pk_max(u1, lo_p), hi_p);
                    const u2v uu = {u0, u1};
                    *(u2v*)(tb + l32 * ROW + c * 32 + q * 8 + lhi * 4) = uu;
                }
            }
            __builtin_amdgcn_wave_barrier();
            const int part = lane & (LPX - 1);
            const int cc = cb0 * 32 + part * 8;
#pragma unroll
            for (int i = 0; i < 32 / PPP; ++i) {
                const int pl = i * PPP + lane / LPX;
                const int px_ = p * 32 + pl;
                const int row = div_by(px_, tw_m), colp = px_ - row * a.tw;
                const int oy = oy0 + row, ox = ox0 + colp;
                if (px_ < a.tp && oy < a.oh && ox < a.ow && cc < a.cout)
                    *(u4v*)(outp + ((size_t)((n * a.oh + oy) * a.ow + ox) * a.cout + cc)) =
                        *(const u4v*)(tb + pl * ROW + part * 8);
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// 3x3 convolution (pad 1, stride 1 or 2; + residual operand) or 1x1 convolution (stride 1), + bias + activation, where a map has
// many channels and few pixels: the 14 x 14 and 7 x 7 maps of ResNet-50's and VGG-16's last stages.  The block kernel k_c3b has too
// few 128-channel x 256-pixel blocks there to fill the chip, and in the fused-group kernel every wave
// streams weights for one or two pixel blocks of its own.  Built like k_dws:
//   Work item = (tile of up to 8 x 8 output pixels, slice of 8 / ksplit channel blocks): one workgroup
// of eight waves, one item, one workgroup per CU; the slices of a tile run on one XCD.
//   1. The tile's input region, all cin channels, global -> LDS by direct loads with the hardware's
//      range check supplying the padding (written as instructions, waits counted by hand, as in
//      k_dws).  Within a pixel the 16-byte parts are stored permuted, part q of the region pixel in
//      row r, column c at position q ^ ((r * tw + c) % 16): a pixel's cin * 2 bytes are a multiple
//      of all 64 banks, so the position alone picks the bank group; an MFMA "B" fragment reads one
//      part of 32 consecutive tile pixels shifted by a tap, for which r * tw + c runs through
//      consecutive integers (tile pixel + a constant): any 16 of them read conflict-free.  (With
//      the region's own pixel index in its place the row breaks of a 7-wide tile in a 9-wide
//      region repeat two of 16 values: SQ_LDS_BANK_CONFLICT at 48 % of the LDS cycles.)
//   2. Every wave one channel block x the tile's two 32-pixel blocks; ksplit waves share a channel
//      block, each taking whole 32-channel chunks of K (18 K steps a chunk: nine taps x two halves,
//      the order the weights are packed in, so a wave's fragments are one contiguous stream through
//      a register ring of 9 K steps).  The tap of a K step is static in the unrolled chunk, so the
//      lane's nine (tap-shifted pixel, permutation) pairs stay in registers.
//   3. Partial sums of the waves of a channel block meet in LDS (in the region's space, behind a
//      barrier); bias, fp16, residual operand if there is one (its vectors requested right behind
//      the K loop), activation, transpose, 64-byte runs per pixel to memory.
// I8: the quantised form (int8 tensors seen as fp16 tensors of half the channels, int32 accumulators on
// v_mfma_i32_32x32x32_i8 -- the partial sums that meet in LDS are integers, so the split of K changes no
// bit -- and a requantising epilogue, see k_c3b); stride 1, no residual operand.
template <int TAPS, int S, int FP, bool I8 = false>
__global__ __launch_bounds__(DLF_C3S_WAVES * 64, 1) void k_c3s(const DlfC3sArgs a)
{
    static_assert(!I8 || S == 1, "the quantised form has stride 1");
    typedef typename AccOf<I8>::type acc_t;
    typedef decltype(acc_t{}[0] + 0) red_t;            // float, or int in the quantised form
    static_assert(TAPS == 9 || (TAPS == 1 && S == 1), "3x3 (pad 1, stride 1 or 2) or 1x1 (pad 0, stride 1)");
    static_assert(S == 1 || S == 2, "stride");
    static_assert(FP == 1 || FP == 2, "32-pixel blocks of a tile");
    constexpr int HALO = TAPS == 9 ? 1 : 0;
    constexpr int CH = TAPS == 9 ? 32 : 128;                 // channels of a chunk of K
    constexpr int STEPS = TAPS * CH / 16;                    // its K steps: 18 or 8, in the order the weights are packed
    constexpr int D = TAPS == 9 ? 9 : 8;                     // ring depth: divides STEPS
    constexpr int ROW = 32 + 8;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    const int pp_shift = __builtin_ctz(a.cin) - 3;           // 16-byte parts per pixel = cin / 8 (32 .. 256)
    // Work item of the workgroup.  Workgroup i runs on XCD i % 8.  Either the slices of a tile share an
    // XCD (its L2 fetches the tile's region once, and every XCD fetches all the weights), or an XCD
    // keeps to one slice (8 / nsl XCDs share the tiles of a slice: each L2 holds 1 / nsl of the weights
    // and fetches every region its tiles need) -- the host chooses by which of the two is larger.
    const int per8 = blockIdx.x >> 3, xcd = blockIdx.x & 7;
    int sl, tile;
    if (a.slice_major) {
        sl = xcd % a.nsl;
        tile = per8 * (8 / a.nsl) + xcd / a.nsl;
    } else {
        sl = per8 % a.nsl;
        tile = xcd * ((a.ntiles + 7) >> 3) + per8 / a.nsl;     // a contiguous eighth of the tiles: halos meet in the XCD's L2
    }
    if (tile >= a.ntiles) return;
    int r_ = tile;
    const int tx = r_ % a.tiles_x;
    r_ /= a.tiles_x;
    const int ty = r_ % a.tiles_y, n = r_ / a.tiles_y;
    const int oy0 = ty * a.th, ox0 = tx * a.tw;
    const int ncbw = DLF_C3S_WAVES / a.ksplit;               // channel blocks of the item
    const int cbw = wave % ncbw, kpart = wave / ncbw;
    const int cb = sl * ncbw + cbw;
    const bool live = cb < a.ncb;                            // uniform
    half_t* outp = (half_t*)a.out;
    const unsigned lo_e = act_lo(a.act), hi_e = act_hi(a.act);
    const unsigned tw_m = div_magic(a.tw), rw_m = div_magic(a.rw);

    // ---- step 1: the region ----
    const i32x4 rin = make_rsrc(a.in, a.in_bytes);
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) half_t*)lds;
    const int nparts = a.rp << pp_shift;
    const int ni = (nparts + 63) >> 6;
#pragma unroll 1
    for (int i = wave; i < ni; i += DLF_C3S_WAVES) {
        const int idx = i * 64 + lane;
        const int hp = idx >> pp_shift, pos = idx & ((1 << pp_shift) - 1);
        unsigned off = (unsigned)DLF_OOB;
        if (hp < a.rp) {
            const int ry = div_by(hp, rw_m), rx = hp - ry * a.rw;
            const int gy = oy0 * S - HALO + ry, gx = ox0 * S - HALO + rx;
            if (gy >= 0 && gy < a.h && gx >= 0 && gx < a.w_)
                off = (unsigned)(((n * a.h + gy) * a.w_ + gx) * a.cin + ((pos ^ (((ry / S) * a.tw + rx / S) & 15)) << 3)) * 2u;
        }
        asm volatile("s_mov_b32 m0, %2\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds" ::"v"(off), "s"(rin),
                     "s"(lds0 + (unsigned)i * 1024u)
                     : "memory", "m0");
    }

    // ---- the wave's weight stream ----
    const i32x4 rwt = make_rsrc(a.w, 0xffffffffu);
    const int lane16 = lane * 16;
    const int nchunk = (a.cin / CH) / a.ksplit;              // chunks of this wave
    const int c32_0 = kpart * nchunk;
    const unsigned wo = (unsigned)__builtin_amdgcn_readfirstlane((min(cb, a.ncb - 1) * a.nsteps + c32_0 * STEPS) * 1024);
    const int n_mine = nchunk * STEPS;
    int pf_ks = 0;
    h8 ar[D];
    auto request = [&](int slot) __attribute__((always_inline)) {
        ar[slot] = wfrag(rwt, lane16, wo + (unsigned)min(pf_ks, n_mine - 1) * 1024u);   // past the end: re-read, never used
        ++pf_ks;
    };
    if (live) {
#pragma unroll
        for (int d = 0; d < D; ++d) request(d);
    }

    // the lane's two pixels under each of the nine taps: byte offset of the region pixel, and the
    // permutation of that pixel combined with the lane's K half, as a byte offset (16 * (h % 16 ^ lhi))
    int bt[TAPS][FP], ft[TAPS][FP];
#pragma unroll
    for (int p = 0; p < FP; ++p) {
        const int px_ = min(p * 32 + l32, a.tp - 1);
        const int py = div_by(px_, tw_m), pxx = px_ - py * a.tw;
#pragma unroll
        for (int t = 0; t < TAPS; ++t) {
            const int ry = py * S + t / 3, rx = pxx * S + t % 3;
            bt[t][p] = (ry * a.rw + rx) * a.cin * 2;
            ft[t][p] = ((((ry / S) * a.tw + rx / S) & 15) ^ lhi) << 4;
        }
    }
    acc_t acc[FP];
#pragma unroll
    for (int p = 0; p < FP; ++p)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[p][q] = 0;

    if (live) wait_vmcnt<D>(); else wait_vmcnt<0>();         // the region has landed: only the ring's requests are behind it
    asm volatile("s_barrier" ::: "memory");

    // ---- step 2: K loop ----
    if (live) {
        const char* const region = (const char*)lds;
        // (the fragments of step s + 1 are read before step s is multiplied; a ring slot is requested
        // again right behind its multiplies)
        h8 bf[2][FP];
#pragma unroll
        for (int p = 0; p < FP; ++p) bf[0][p] = *(const h8*)(region + bt[0][p] + ((c32_0 * (CH * 2)) ^ ft[0][p]));
#pragma unroll 1
        for (int c = 0; c < nchunk; ++c) {
            const int q16 = (c32_0 + c) * (CH * 2);          // byte offset of the chunk's first part, before the permutation
            const int q16n = (c32_0 + min(c + 1, nchunk - 1)) * (CH * 2);
#pragma unroll
            for (int j = 0; j < STEPS; ++j) {
                // step j of a chunk: 3x3: tap j / 2, channels (j % 2) * 16 ..; 1x1: channels j * 16 ..
                const int jn = (j + 1) % STEPS, tn = TAPS == 9 ? jn >> 1 : 0;
                const int qn = (j == STEPS - 1 ? q16n : q16) + (TAPS == 9 ? (jn & 1) : jn) * 32;
#pragma unroll
                for (int p = 0; p < FP; ++p) bf[(j + 1) & 1][p] = *(const h8*)(region + bt[tn][p] + (qn ^ ft[tn][p]));
#pragma unroll
                for (int p = 0; p < FP; ++p) {
                    if constexpr (I8)
                        acc[p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4, ar[j % D]),
                                                                       __builtin_bit_cast(i32x4, bf[j & 1][p]), acc[p], 0, 0, 0);
                    else
                        acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ar[j % D], bf[j & 1][p], acc[p], 0, 0, 0);
                }
                request(j % D);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    // ---- step 3: partial sums, epilogue ----
    red_t* const red = (red_t*)lds;
    half_t* const tb = lds + DLF_C3S_RED_BYTES / 2 + wave * (32 * ROW);
    // the residual vectors of the pixels and channels this lane will store, and the bias: requested
    // here, ahead of the exchange of partial sums and of the first store (a load behind a store
    // waits for the store as well)
    const half_t* const resp = (const half_t*)a.res;
    u4v rv[FP][2];
    f4v biasv[4];
    if (live && kpart == 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) biasv[q] = *(const f4v*)(a.bias + cb * 32 + q * 8 + lhi * 4);
        if (resp != nullptr) {
            const int cc = cb * 32 + (lane & 3) * 8;
#pragma unroll
            for (int p = 0; p < FP; ++p)
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int px_ = min(p * 32 + i * 16 + (lane >> 2), a.tp - 1);
                    const int row = div_by(px_, tw_m), colp = px_ - row * a.tw;
                    const int oy = min(oy0 + row, a.oh - 1), ox = min(ox0 + colp, a.ow - 1);
                    rv[p][i] = *(const u4v*)(resp + ((size_t)((n * a.oh + oy) * a.ow + ox) * a.cout + min(cc, a.cout - 8)));
                }
        }
    }
    if (a.ksplit > 1) {
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");      // everyone is done reading the region
        if (kpart > 0 && live) {
            red_t* dst = red + (wave - ncbw) * (2 * 16 * 64) + lane;
#pragma unroll
            for (int p = 0; p < FP; ++p)
#pragma unroll
                for (int q = 0; q < 16; ++q) dst[(p * 16 + q) * 64] = acc[p][q];
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (kpart > 0 || !live) return;
        for (int k = 1; k < a.ksplit; ++k) {
            const red_t* src = red + (k * ncbw + cbw - ncbw) * (2 * 16 * 64) + lane;
#pragma unroll
            for (int p = 0; p < FP; ++p)
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[p][q] += src[(p * 16 + q) * 64];
        }
    } else {
        if (!live) return;
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");      // the transpose buffers lie in the region's space
    }
    if constexpr (I8) {
        // requantise; the wave's 32 channels of a pixel are a row of 32 bytes in its transpose buffer
        // (16-byte part c of row r at c ^ (r / 4) % 2, dword d of a part at d ^ (r / 8) % 4: the 32 rows
        // of a write fall into 32 banks); then lane 2 r + c stores part c of row r
        unsigned char* const tb8 = (unsigned char*)tb;
        signed char* const out8 = (signed char*)a.out;
        const float lo = a.act != 0 ? 0.0f : -128.0f;
        f4v scv[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) scv[q] = *(const f4v*)(a.scale + cb * 32 + q * 8 + lhi * 4);
        // With the 2x2 max pool folded in (tiles 8 pixels wide and of even height): a 32-pixel block is four
        // tile rows, lane l32 holds tile pixel (l32 / 8, l32 % 8) of them, so a window is the lanes
        // {l, l ^ 1, l ^ 8, l ^ 9}: one quad permute and one rotation by 8 inside the row of 16 lanes; the
        // lane of the window's first pixel writes pooled pixel (l32 / 16) * 4 + (l32 % 8) / 2 of the block's 8.
        const bool pool = a.pool2 != 0;
        const int poh = a.oh >> 1, pow_ = a.ow >> 1;
#pragma unroll
        for (int p = 0; p < FP; ++p) {
            if (p * 32 < a.tp) {
                const int wrow = pool ? ((l32 >> 4) << 2) + ((l32 & 7) >> 1) : l32;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float tv[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float t = requant_biased(acc[p][q * 4 + r], scv[q][r], biasv[q][r], lo);
                        if (pool) {
                            t = __builtin_fmaxf(t, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, t), 0xB1, 0xF, 0xF, true)));
                            t = __builtin_fmaxf(t, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, t), 0x128, 0xF, 0xF, true)));
                        }
                        tv[r] = t;
                    }
                    const unsigned u = pack_low_bytes(tv[0], tv[1], tv[2], tv[3]);
                    if (!pool || (l32 & 9) == 0)
                        *(unsigned*)(tb8 + wrow * 32 + ((((q >> 1) ^ (wrow >> 2)) & 1) << 4) + (((((q & 1) * 2 + lhi) ^ (wrow >> 3)) & 3) << 2)) = u;
                }
                __builtin_amdgcn_wave_barrier();
                const int part = lane & 1, pl = lane >> 1;
                const int cc = cb * 32 + part * 16;
                const u4v v = *(const u4v*)(tb8 + pl * 32 + (((part ^ (pl >> 2)) & 1) << 4));
                const int k = pl >> 3;
                const u4v v1 = (k & 1) ? u4v{v.y, v.x, v.w, v.z} : v;
                const u4v v2 = (k & 2) ? u4v{v1.z, v1.w, v1.x, v1.y} : v1;
                if (pool) {
                    // pooled pixel pl (< 8) of the block: pooled tile row 2 p + pl / 4, column pl % 4
                    const int qy = 2 * p + (pl >> 2), qx = pl & 3;
                    const int oy = (oy0 >> 1) + qy, ox = (ox0 >> 1) + qx;
                    if (pl < 8 && 2 * qy < a.th && oy < poh && ox < pow_ && cc < a.cout)
                        *(u4v*)(out8 + ((size_t)((n * poh + oy) * pow_ + ox) * a.cout + cc)) = v2;
                } else {
                    const int px_ = p * 32 + pl;
                    const int row = div_by(px_, tw_m), colp = px_ - row * a.tw;
                    const int oy = oy0 + row, ox = ox0 + colp;
                    if (px_ < a.tp && oy < a.oh && ox < a.ow && cc < a.cout)
                        *(u4v*)(out8 + ((size_t)((n * a.oh + oy) * a.ow + ox) * a.cout + cc)) = v2;
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
        return;
    }
    // with a residual operand the activation follows the add (fp16 + fp16, as in the other kernels)
    const unsigned lo_t = resp != nullptr ? act_lo(0) : lo_e, hi_t = resp != nullptr ? act_hi(0) : hi_e;
#pragma unroll
    for (int p = 0; p < FP; ++p) {
        if (p * 32 < a.tp) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f4v bias = biasv[q];
                unsigned u0 = cvt_pk(acc[p][q * 4 + 0] + bias[0], acc[p][q * 4 + 1] + bias[1]);
                unsigned u1 = cvt_pk(acc[p][q * 4 + 2] + bias[2], acc[p][q * 4 + 3] + bias[3]);
                u0 = pk_min(pk_max(u0, lo_t), hi_t);
                u1 = pk_min(pk_max(u1, lo_t), hi_t);
                const u2v uu = {u0, u1};
                *(u2v*)(tb + l32 * ROW + q * 8 + lhi * 4) = uu;
            }
            __builtin_amdgcn_wave_barrier();
            const int part = lane & 3;
            const int cc = cb * 32 + part * 8;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int pl = i * 16 + (lane >> 2);
                const int px_ = p * 32 + pl;
                const int row = div_by(px_, tw_m), colp = px_ - row * a.tw;
                const int oy = oy0 + row, ox = ox0 + colp;
                if (px_ < a.tp && oy < a.oh && ox < a.ow && cc < a.cout) {
                    u4v v = *(const u4v*)(tb + pl * ROW + part * 8);
                    if (resp != nullptr) {
                        v.x = pk_min(pk_max(pk_add(v.x, rv[p][i].x), lo_e), hi_e);
                        v.y = pk_min(pk_max(pk_add(v.y, rv[p][i].y), lo_e), hi_e);
                        v.z = pk_min(pk_max(pk_add(v.z, rv[p][i].z), lo_e), hi_e);
                        v.w = pk_min(pk_max(pk_add(v.w, rv[p][i].w), lo_e), hi_e);
                    }
                    *(u4v*)(outp + ((size_t)((n * a.oh + oy) * a.ow + ox) * a.cout + cc)) = v;
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// 3x3 convolution (stride 1, pad 1, c -> c channels, c = 64, 128 or 256) + bias + activation, and the 1x1
// convolution behind it + bias + residual operand + activation: the second half of a bottleneck block
// (Sec. III-B: the intermediate tensor never leaves the chip), where the fused-group kernel's tile
// pipeline is bound by the latency of its steps.  Work item = (tile of up to 8 x 16 output pixels,
// slice of the second layer's channel blocks, two per wave); one item per workgroup.
//   c = 128, 256: workgroups of eight waves, one to a CU, for batches with no more tiles than CUs.
// Every workgroup of the chip is then in the same phase at the same time, so the phases are
// arranged for memory and matrix pipes to work side by side: the residual operand comes in while
// the first layer multiplies.
//   c = 64: workgroups of four waves, two or three to a CU and more items than places: the phases
// of neighbouring items overlap by themselves (ResNet-50's 56 x 56 groups: 116 MB in 31 us).
//   1. The tile's input region, all c channels, global -> LDS by direct loads, as in k_c3s (range
//      check as padding, parts permuted by (r * tw + c) % 16).  Behind it the residual operand of the
//      item's pixels x 512 (four waves: 256) channels, likewise to LDS (one load per pixel, rows of
//      1024 + 64 (512 + 64) bytes; of an item of four waves the upper lanes take no part), by
//      the waves that have no part in the first layer, once the region has landed (requested beside
//      it, it doubles the time until the first layer can start); with eight channel blocks in the
//      first layer every wave has one, and they all request it before they start.
//   2. First layer: waves 0 .. c / 32 - 1 take one channel block x all FP 32-pixel blocks each, K in the
//      packed order through a register ring of 9 steps.  (With four channel blocks the other four
//      waves have nothing to multiply here: two waves of a SIMD would take turns on its matrix pipe
//      anyway.)  Once every wave is done with the region: result (bias included), activation, fp16 to an LDS
//      tile [pixel][c + 8] in the region's place.
//   3. Second layer: every wave two channel blocks, one after the other, all of K (c / 16 steps)
//      with both blocks' weight fragments in registers (requested as early as the wave has room for
//      them), 32 pixels at a time: the MFMAs run, the results go through the wave's transpose
//      buffer, the residual is added to the rounded sum (fp16 + fp16, as in the other kernels),
//      activation, and a pixel's 2 x 64 bytes go to memory in adjacent instructions.
template <int FP, int C>
__global__ __launch_bounds__(DLF_C3PW_WAVES(C) * 64, C == 64 ? 2 : 1) void k_c3pw(const DlfC3PwArgs a)
{
    constexpr int D = 9;
    constexpr int ROW = 32 + 8;
    static_assert(FP == 2 || FP == 4, "32-pixel blocks of a tile");
    static_assert(C == 64 || C == 128 || C == 256, "channels of the first layer");
    constexpr int W = DLF_C3PW_WAVES(C);
    constexpr int PP = C / 8;                                // 16-byte parts per pixel: 8, 16 or 32
    constexpr int RES_STRIDE = DLF_C3PW_RES_STRIDE(C);
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    constexpr int pp_shift = C == 64 ? 3 : (C == 128 ? 4 : 5);
    constexpr int PERM = PP < 16 ? PP - 1 : 15;              // the permutation stays inside a pixel
    constexpr int cs = C + 8;
    const int per8 = blockIdx.x >> 3;
    // (an XCD takes a contiguous eighth of the tiles: the halo a tile shares with its neighbours is in that XCD's L2)
    const int sl = per8 % a.nsl, tile = (blockIdx.x & 7) * ((a.ntiles + 7) >> 3) + per8 / a.nsl;
    if (tile >= a.ntiles) return;
    int r_ = tile;
    const int tx = r_ % a.tiles_x;
    r_ /= a.tiles_x;
    const int ty = r_ % a.tiles_y, n = r_ / a.tiles_y;
    const int oy0 = ty * a.th, ox0 = tx * a.tw;
    half_t* const mid = lds;                                 // takes the region's place
    half_t* const tb = lds + DLF_C3PW_TB_OFF(a.tp, C) / 2 + wave * (32 * ROW);
    const int res_off = DLF_C3PW_RES_OFF(a.rp, a.tp, C);
    half_t* outp = (half_t*)a.out;
    const bool has_res = a.res != nullptr;
    const unsigned lo1 = act_lo(a.act1), hi1 = act_hi(a.act1);
    const unsigned lo2 = act_lo(a.act2), hi2 = act_hi(a.act2);
    const unsigned tw_m = div_magic(a.tw), rw_m = div_magic(a.rw);

    // ---- step 1: the region, the residual operand ----
    const i32x4 rin = make_rsrc(a.in, a.in_bytes);
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) half_t*)lds;
    const int ni = ((a.rp << pp_shift) + 63) >> 6;
#pragma unroll 1
    for (int i = wave; i < ni; i += W) {
        const int idx = i * 64 + lane;
        const int hp = idx >> pp_shift, pos = idx & ((1 << pp_shift) - 1);
        unsigned off = (unsigned)DLF_OOB;
        if (hp < a.rp) {
            const int ry = div_by(hp, rw_m), rx = hp - ry * a.rw;
            const int gy = oy0 - 1 + ry, gx = ox0 - 1 + rx;
            if (gy >= 0 && gy < a.h && gx >= 0 && gx < a.w_)
                off = (unsigned)(((n * a.h + gy) * a.w_ + gx) * C + ((pos ^ ((ry * a.tw + rx) & PERM)) << 3)) * 2u;
        }
        asm volatile("s_mov_b32 m0, %2\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds" ::"v"(off), "s"(rin),
                     "s"(lds0 + (unsigned)i * 1024u)
                     : "memory", "m0");
    }
    const int lane16 = lane * 16;
    constexpr int ncb1 = C / 32, nsteps1 = ncb1 * 18, nsteps2 = C / 16;
    const bool conv1 = wave < ncb1;                          // uniform
    // the residual operand of pixels first, first + every, ..: one load per pixel
    auto request_res = [&](int first, int every) __attribute__((always_inline)) {
        const i32x4 rres = make_rsrc(a.res, a.res_bytes);
        const int ch = sl * (2 * W * 32) + lane * 8;
#pragma unroll 1
        for (int p = first; p < a.tp; p += every) {
            const int row = div_by(p, tw_m), colp = p - row * a.tw;
            const int oy = oy0 + row, ox = ox0 + colp;
            unsigned off = (unsigned)DLF_OOB;
            if (oy < a.h && ox < a.w_ && ch < a.cout) off = (unsigned)(((n * a.h + oy) * a.w_ + ox) * a.cout + ch) * 2u;
            // (an item of four waves has 256 channels: the upper lanes take no part and write nothing)
            if (W == 8 || lane < W * 8)
                asm volatile("s_mov_b32 m0, %2\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds" ::"v"(off), "s"(rres),
                             "s"(lds0 + (unsigned)(res_off + p * RES_STRIDE))
                             : "memory", "m0");
        }
    };
    if (ncb1 == W && has_res) request_res(wave, W);

    // the second layer's weights of this wave: both channel blocks, all of K
    const int cb0 = (sl * W + wave) * 2;
    const bool live = cb0 < a.ncb2;                          // uniform
    const i32x4 rw2 = make_rsrc(a.w2, 0xffffffffu);
    h8 a2[2][nsteps2];
    auto load_a2 = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const unsigned wo2 = (unsigned)__builtin_amdgcn_readfirstlane(min(cb0 + j, a.ncb2 - 1) * nsteps2 * 1024);
#pragma unroll
            for (int k = 0; k < nsteps2; ++k) a2[j][k] = wfrag(rw2, lane16, wo2 + (unsigned)k * 1024u);
        }
    };

    // its bias values, to a wave-private place in LDS (they start the accumulators below)
    float* const bl = (float*)((char*)lds + DLF_C3PW_BIAS_OFF(a.rp, a.tp, C, has_res)) + wave * 64;
    bl[lane] = a.b2[min(cb0 * 32 + lane, a.ncb2 * 32 - 1)];

    // ---- step 2: the first layer ----
    f16v acc[FP];
    if (conv1) {
        const i32x4 rw1 = make_rsrc(a.w1, 0xffffffffu);
        const unsigned wo = (unsigned)__builtin_amdgcn_readfirstlane(wave * nsteps1 * 1024);
        // the accumulators start from the bias
        f4v bias1[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) bias1[q] = *(const f4v*)(a.b1 + wave * 32 + q * 8 + lhi * 4);
        int pf_ks = 0;
        h8 ar[D];
        auto request = [&](int slot) __attribute__((always_inline)) {
            ar[slot] = wfrag(rw1, lane16, wo + (unsigned)min(pf_ks, nsteps1 - 1) * 1024u);   // past the end: re-read, never used
            ++pf_ks;
        };
#pragma unroll
        for (int d = 0; d < D; ++d) request(d);
        int bt[9][FP], ft[9][FP];
#pragma unroll
        for (int p = 0; p < FP; ++p) {
            const int px_ = min(p * 32 + l32, a.tp - 1);
            const int py = div_by(px_, tw_m), pxx = px_ - py * a.tw;
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                const int ry = py + t / 3, rx = pxx + t % 3;
                bt[t][p] = (ry * a.rw + rx) * C * 2;
                ft[t][p] = (((ry * a.tw + rx) & PERM) ^ lhi) << 4;
            }
        }
#pragma unroll
        for (int p = 0; p < FP; ++p)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[p][q] = bias1[q >> 2][q & 3];
        wait_vmcnt<D>();                                     // the region has landed: only the ring's requests are behind it
        asm volatile("s_barrier" ::: "memory");
        const char* const region = (const char*)lds;
        h8 bf[2][FP];
#pragma unroll
        for (int p = 0; p < FP; ++p) bf[0][p] = *(const h8*)(region + bt[0][p] + ft[0][p]);
#pragma unroll 1
        for (int c = 0; c < ncb1; ++c) {
            const int q16 = c * 64, q16n = min(c + 1, ncb1 - 1) * 64;
#pragma unroll
            for (int j = 0; j < 18; ++j) {
                const int jn = (j + 1) % 18, tn = jn >> 1;
                const int qn = (j == 17 ? q16n : q16) + (jn & 1) * 32;
#pragma unroll
                for (int p = 0; p < FP; ++p) bf[(j + 1) & 1][p] = *(const h8*)(region + bt[tn][p] + (qn ^ ft[tn][p]));
#pragma unroll
                for (int p = 0; p < FP; ++p)
                    acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ar[j % D], bf[j & 1][p], acc[p], 0, 0, 0);
                request(j % D);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    } else {
        wait_vmcnt<0>();
        asm volatile("s_barrier" ::: "memory");              // the region has landed
        if (has_res) request_res(wave - ncb1, W - ncb1);
        if (live) load_a2();
    }
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");      // nobody reads the region any more
    if (conv1) {
        // activation, fp16, to the tile: the accumulator holds channels q * 8 + lhi * 4 .. + 3 of pixel l32
#pragma unroll
        for (int p = 0; p < FP; ++p) {
            const int px_ = p * 32 + l32;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                unsigned u0 = cvt_pk(acc[p][q * 4 + 0], acc[p][q * 4 + 1]);
                unsigned u1 = cvt_pk(acc[p][q * 4 + 2], acc[p][q * 4 + 3]);
                u0 = pk_min(pk_max(u0, lo1), hi1);
                u1 = pk_min(pk_max(u1, lo1), hi1);
                const u2v uu = {u0, u1};
                if (px_ < a.tp) *(u2v*)(mid + px_ * cs + wave * 32 + q * 8 + lhi * 4) = uu;
            }
        }
        if (live) load_a2();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    } else {
        wait_vmcnt<0>();                                     // this wave's part of the residual operand has landed
    }
    asm volatile("s_barrier" ::: "memory");                  // the tile and the residual operand are complete
    if (!live) return;

    // everything this wave has asked memory for is in its registers from here on: the loop below
    // issues stores only and never waits for them
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int k = 0; k < nsteps2; ++k) asm volatile("" : "+v"(a2[j][k]));

    // ---- step 3: the second layer ----
    constexpr int LPX = 4, PPP = 64 / LPX;                   // store phase: 4 lanes per pixel and channel block, 16 pixels per instruction
    const int part = lane & (LPX - 1);
    const char* const resl = (const char*)lds + res_off + (wave * 2 * LPX + part) * 16;
    const int cc = cb0 * 32 + part * 8;                      // of the first block; the second one's are 32 further
#pragma unroll 1
    for (int pb = 0; pb * 32 < a.tp; ++pb) {
        f16v acc2[2];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f4v bias = *(const f4v*)(bl + j * 32 + q * 8 + lhi * 4);
#pragma unroll
                for (int i = 0; i < 4; ++i) acc2[j][q * 4 + i] = bias[i];
            }
        const half_t* const bsrc = mid + min(pb * 32 + l32, a.tp - 1) * cs + lhi * 8;
#pragma unroll
        for (int k = 0; k < nsteps2; ++k) {
            const h8 b = *(const h8*)(bsrc + k * 16);
#pragma unroll
            for (int j = 0; j < 2; ++j) acc2[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2[j][k], b, acc2[j], 0, 0, 0);
        }
        // both blocks through the transpose buffer, then each pixel's 2 x 64 bytes to memory back to back
        u4v val[2][32 / PPP];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const unsigned u0 = cvt_pk(acc2[j][q * 4 + 0], acc2[j][q * 4 + 1]);
                const unsigned u1 = cvt_pk(acc2[j][q * 4 + 2], acc2[j][q * 4 + 3]);
                const u2v uu = {u0, u1};
                *(u2v*)(tb + l32 * ROW + q * 8 + lhi * 4) = uu;
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int i = 0; i < 32 / PPP; ++i) val[j][i] = *(const u4v*)(tb + (i * PPP + lane / LPX) * ROW + part * 8);
            __builtin_amdgcn_wave_barrier();
        }
#pragma unroll
        for (int i = 0; i < 32 / PPP; ++i) {
            const int px_ = pb * 32 + i * PPP + lane / LPX;
            const int pc = min(px_, a.tp - 1);
            const int row = div_by(pc, tw_m), colp = pc - row * a.tw;
            const int oy = oy0 + row, ox = ox0 + colp;
            const bool inside = px_ < a.tp && oy < a.h && ox < a.w_;
            half_t* const dst = outp + ((size_t)((n * a.h + oy) * a.w_ + ox) * a.cout + cc);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if (inside && cc + j * 32 < a.cout) {
                    u4v v = val[j][i];
                    if (has_res) {
                        const u4v rv = *(const u4v*)(resl + pc * RES_STRIDE + j * (LPX * 16));
                        v.x = pk_add(v.x, rv.x);
                        v.y = pk_add(v.y, rv.y);
                        v.z = pk_add(v.z, rv.z);
                        v.w = pk_add(v.w, rv.w);
                    }
                    v.x = pk_min(pk_max(v.x, lo2), hi2);
                    v.y = pk_min(pk_max(v.y, lo2), hi2);
                    v.z = pk_min(pk_max(v.z, lo2), hi2);
                    v.w = pk_min(pk_max(v.w, lo2), hi2);
                    *(u4v*)(dst + j * 32) = v;
                }
            }
        }
    }
}

// (With ncb2 = 0 the kernel stops after the second layer and stores its tile: the pair 1x1 -> 3x3.)
// A bottleneck block as one group: 1x1 (cin0 -> 64) + 3x3 (64 -> 64, stride 1, pad 1) + 1x1 (64 -> cout),
// each with bias and activation, and the block's input added before the last activation where the
// block has an identity shortcut (Sec. III-B: neither intermediate tensor leaves the chip, and the
// residual operand is the input region that is in LDS already).  Built from the parts of k_c3pw's
// 64-channel form: one workgroup of four waves per work item = (tile of up to 64 output pixels,
// slice of 8 channel blocks of the last layer), two workgroups to a CU, more items than places, so
// that the load, multiply and store phases of neighbouring items overlap.
//   1. The tile's input region, all cin0 channels, global -> LDS by direct loads (range check as
//      padding, parts permuted by (r * tw + c) % 16).
//   2. First layer on every pixel of the region (the halo is computed again by the neighbouring
//      tiles): wave w takes channel block w % 2 and every second 32-pixel block, all of K with the
//      weight fragments in registers; bias, activation, zero for pixels outside the map (they are
//      the second layer's padding), fp16 into a second region [pixel][64] with the permutation the
//      3x3 loop reads by.
//   3. Second layer: waves 0 and 1 one channel block x the tile's two pixel blocks each, K through a
//      register ring of 9 steps, as in k_c3pw; result to an LDS tile [pixel][64 + 8].
//   4. Last layer: every wave two channel blocks, all of K in registers, 32 pixels at a time through
//      the wave's transpose buffer; + the input's centre pixels from the first region (fp16 + fp16),
//      activation, a pixel's 2 x 64 bytes stored by adjacent instructions.
template <int CIN0>
__global__ __launch_bounds__(DLF_BN_WAVES * 64, 2) void k_bneck(const DlfBnArgs a)
{
    constexpr int D = 9, ROW = 32 + 8, C = 64, W = DLF_BN_WAVES, FP = 2, cs = C + 8;
    static_assert(CIN0 == 64 || CIN0 == 128 || CIN0 == 256 || CIN0 == 512, "channels of the block's input");
    constexpr int pp0 = CIN0 == 64 ? 3 : (CIN0 == 128 ? 4 : (CIN0 == 256 ? 5 : 6));   // log2 of the input's 16-byte parts per pixel
    constexpr int PERM0 = CIN0 == 64 ? 7 : 15;               // the permutation stays inside a pixel
    constexpr int NS0 = CIN0 / 16;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    // Workgroup i runs on XCD i % 8: an XCD takes a contiguous eighth of the tiles (whole rows of
    // tiles, whole images), in order, so that the halo a tile shares with its neighbours is in that
    // XCD's L2 when the neighbour asks for it
    const int per8 = blockIdx.x >> 3;
    const int sl = per8 % a.nsl, tile = (blockIdx.x & 7) * ((a.ntiles + 7) >> 3) + per8 / a.nsl;
    if (tile >= a.ntiles) return;
    int r_ = tile;
    const int tx = r_ % a.tiles_x;
    r_ /= a.tiles_x;
    const int ty = r_ % a.tiles_y, n = r_ / a.tiles_y;
    const int oy0 = ty * a.th, ox0 = tx * a.tw;
    char* const r0 = (char*)lds;
    char* const ma = r0 + DLF_BN_MA_OFF(a.rp, CIN0);
    half_t* const mid = (half_t*)(r0 + DLF_BN_MB_OFF(a.rp, CIN0));
    half_t* const tb = (half_t*)(r0 + DLF_BN_TB_OFF(a.rp, a.tp, CIN0)) + wave * (32 * ROW);
    float* const bl = (float*)(r0 + DLF_BN_BIAS_OFF(a.rp, a.tp, CIN0)) + wave * 64;
    half_t* outp = (half_t*)a.out;
    const unsigned lo0 = act_lo(a.act0), hi0 = act_hi(a.act0);
    const unsigned lo1 = act_lo(a.act1), hi1 = act_hi(a.act1);
    const unsigned lo2 = act_lo(a.act2), hi2 = act_hi(a.act2);
    const unsigned tw_m = div_magic(a.tw), rw_m = div_magic(a.rw);
    const int lane16 = lane * 16;

    // ---- step 1: the region ----
    const i32x4 rin = make_rsrc(a.in, a.in_bytes);
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) half_t*)lds;
    const int ni = ((a.rp << pp0) + 63) >> 6;
#pragma unroll 1
    for (int i = wave; i < ni; i += W) {
        const int idx = i * 64 + lane;
        const int hp = idx >> pp0, pos = idx & ((1 << pp0) - 1);
        unsigned off = (unsigned)DLF_OOB;
        if (hp < a.rp) {
            const int ry = div_by(hp, rw_m), rx = hp - ry * a.rw;
            const int gy = oy0 - 1 + ry, gx = ox0 - 1 + rx;
            if (gy >= 0 && gy < a.h && gx >= 0 && gx < a.w_)
                off = (unsigned)(((n * a.h + gy) * a.w_ + gx) * CIN0 + ((pos ^ ((ry * a.tw + rx) & PERM0)) << 3)) * 2u;
        }
        asm volatile("s_mov_b32 m0, %2\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds" ::"v"(off), "s"(rin),
                     "s"(lds0 + (unsigned)i * 1024u)
                     : "memory", "m0");
    }
    // the first layer's weights of this wave's channel block, all of K; the last layer's bias to LDS
    const int cb_a = wave & 1;
    h8 a0[NS0];
    {
        const i32x4 rw0 = make_rsrc(a.w0, 0xffffffffu);
        const unsigned wo0 = (unsigned)(cb_a * NS0 * 1024);
#pragma unroll
        for (int k = 0; k < NS0; ++k) a0[k] = wfrag(rw0, lane16, wo0 + (unsigned)k * 1024u);
    }
    f4v bias0[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) bias0[q] = *(const f4v*)(a.b0 + cb_a * 32 + q * 8 + lhi * 4);
    const bool last = a.ncb2 > 0;                            // uniform: is there a third layer
    const int cb0 = (sl * W + wave) * 2;
    const bool live = cb0 < a.ncb2;                          // uniform
    if (last) bl[lane] = a.b2[min(cb0 * 32 + lane, a.ncb2 * 32 - 1)];
    // the last layer's weights of this wave (both channel blocks, all of K) and, on the two waves of
    // the second layer, the first turn of its ring: everything is requested before the first wait
    constexpr int nsteps1 = 2 * 18, nsteps2 = C / 16;
    h8 a2[2][nsteps2];
    if (last) {
        const i32x4 rw2 = make_rsrc(a.w2, 0xffffffffu);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const unsigned wo2 = (unsigned)__builtin_amdgcn_readfirstlane(min(cb0 + j, a.ncb2 - 1) * nsteps2 * 1024);
#pragma unroll
            for (int k = 0; k < nsteps2; ++k) a2[j][k] = wfrag(rw2, lane16, wo2 + (unsigned)k * 1024u);
        }
    }
    const i32x4 rw1 = make_rsrc(a.w1, 0xffffffffu);
    const unsigned wo = (unsigned)__builtin_amdgcn_readfirstlane((wave & 1) * nsteps1 * 1024);
    int pf_ks = 0;
    h8 ar[D];
    auto request = [&](int slot) __attribute__((always_inline)) {
        ar[slot] = wfrag(rw1, lane16, wo + (unsigned)min(pf_ks, nsteps1 - 1) * 1024u);   // past the end: re-read, never used
        ++pf_ks;
    };
    if (wave < 2) {
#pragma unroll
        for (int d = 0; d < D; ++d) request(d);
    }
    wait_vmcnt<0>();
    asm volatile("s_barrier" ::: "memory");                  // the region has landed

    // ---- step 2: the first layer, on the region ----
    {
        const int npb = (a.rp + 31) >> 5;
#pragma unroll 1
        for (int pb = wave >> 1; pb < npb; pb += W / 2) {
            const int px_ = pb * 32 + l32, pc = min(px_, a.rp - 1);
            const int ry = div_by(pc, rw_m), rx = pc - ry * a.rw;
            const int perm = (ry * a.tw + rx) & 15;          // (the first region uses PERM0 of its bits, the second 7)
            const char* const src = r0 + pc * (CIN0 * 2);
            f16v acc;
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[q] = bias0[q >> 2][q & 3];
#pragma unroll
            for (int k = 0; k < NS0; ++k)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0[k], *(const h8*)(src + (((2 * k + lhi) ^ (perm & PERM0)) << 4)), acc, 0, 0, 0);
            const int gy = oy0 - 1 + ry, gx = ox0 - 1 + rx;
            const bool inside = gy >= 0 && gy < a.h && gx >= 0 && gx < a.w_;
            char* const dst = ma + pc * (C * 2) + lhi * 8;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                unsigned u0 = cvt_pk(acc[q * 4 + 0], acc[q * 4 + 1]);
                unsigned u1 = cvt_pk(acc[q * 4 + 2], acc[q * 4 + 3]);
                u0 = inside ? pk_min(pk_max(u0, lo0), hi0) : 0u;
                u1 = inside ? pk_min(pk_max(u1, lo0), hi0) : 0u;
                const u2v uu = {u0, u1};
                if (px_ < a.rp) *(u2v*)(dst + (((cb_a * 4 + q) ^ (perm & 7)) << 4)) = uu;
            }
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");      // the second region is complete

    // ---- step 3: the second layer ----
    if (wave < 2) {
        f4v bias1[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) bias1[q] = *(const f4v*)(a.b1 + wave * 32 + q * 8 + lhi * 4);
        int bt[9][FP], ft[9][FP];
#pragma unroll
        for (int p = 0; p < FP; ++p) {
            const int px_ = min(p * 32 + l32, a.tp - 1);
            const int py = div_by(px_, tw_m), pxx = px_ - py * a.tw;
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                const int ry = py + t / 3, rx = pxx + t % 3;
                bt[t][p] = (ry * a.rw + rx) * C * 2;
                ft[t][p] = (((ry * a.tw + rx) & 7) ^ lhi) << 4;
            }
        }
        f16v acc[FP];
#pragma unroll
        for (int p = 0; p < FP; ++p)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[p][q] = bias1[q >> 2][q & 3];
        const char* const region = ma;
        h8 bf[2][FP];
#pragma unroll
        for (int p = 0; p < FP; ++p) bf[0][p] = *(const h8*)(region + bt[0][p] + ft[0][p]);
#pragma unroll 1
        for (int c = 0; c < 2; ++c) {
            const int q16 = c * 64, q16n = min(c + 1, 1) * 64;
#pragma unroll
            for (int j = 0; j < 18; ++j) {
                const int jn = (j + 1) % 18, tn = jn >> 1;
                const int qn = (j == 17 ? q16n : q16) + (jn & 1) * 32;
#pragma unroll
                for (int p = 0; p < FP; ++p) bf[(j + 1) & 1][p] = *(const h8*)(region + bt[tn][p] + (qn ^ ft[tn][p]));
#pragma unroll
                for (int p = 0; p < FP; ++p)
                    acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ar[j % D], bf[j & 1][p], acc[p], 0, 0, 0);
                request(j % D);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int p = 0; p < FP; ++p) {
            const int px_ = p * 32 + l32;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                unsigned u0 = cvt_pk(acc[p][q * 4 + 0], acc[p][q * 4 + 1]);
                unsigned u1 = cvt_pk(acc[p][q * 4 + 2], acc[p][q * 4 + 3]);
                u0 = pk_min(pk_max(u0, lo1), hi1);
                u1 = pk_min(pk_max(u1, lo1), hi1);
                const u2v uu = {u0, u1};
                if (px_ < a.tp) *(u2v*)(mid + px_ * cs + wave * 32 + q * 8 + lhi * 4) = uu;
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    asm volatile("s_barrier" ::: "memory");                  // the tile is complete
    if (!last) {
        // two layers only: the tile goes to memory as it is, 16 bytes per lane
        for (int idx = threadIdx.x; idx < a.tp * (C / 8); idx += W * 64) {
            const int px_ = idx >> 3, q = idx & 7;
            const int row = div_by(px_, tw_m), colp = px_ - row * a.tw;
            const int oy = oy0 + row, ox = ox0 + colp;
            if (oy < a.h && ox < a.w_)
                *(u4v*)(outp + ((size_t)((n * a.h + oy) * a.w_ + ox) * C + q * 8)) = *(const u4v*)(mid + px_ * cs + q * 8);
        }
        return;
    }
    if (!live) return;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int k = 0; k < nsteps2; ++k) asm volatile("" : "+v"(a2[j][k]));

    // ---- step 4: the last layer ----
    constexpr int LPX = 4, PPP = 64 / LPX;
    const int part = lane & (LPX - 1);
    const int cc = cb0 * 32 + part * 8;
#pragma unroll 1
    for (int pb = 0; pb * 32 < a.tp; ++pb) {
        f16v acc2[2];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f4v bias = *(const f4v*)(bl + j * 32 + q * 8 + lhi * 4);
#pragma unroll
                for (int i = 0; i < 4; ++i) acc2[j][q * 4 + i] = bias[i];
            }
        const half_t* const bsrc = mid + min(pb * 32 + l32, a.tp - 1) * cs + lhi * 8;
#pragma unroll
        for (int k = 0; k < nsteps2; ++k) {
            const h8 b = *(const h8*)(bsrc + k * 16);
#pragma unroll
            for (int j = 0; j < 2; ++j) acc2[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2[j][k], b, acc2[j], 0, 0, 0);
        }
        u4v val[2][32 / PPP];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const unsigned u0 = cvt_pk(acc2[j][q * 4 + 0], acc2[j][q * 4 + 1]);
                const unsigned u1 = cvt_pk(acc2[j][q * 4 + 2], acc2[j][q * 4 + 3]);
                const u2v uu = {u0, u1};
                *(u2v*)(tb + l32 * ROW + q * 8 + lhi * 4) = uu;
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int i = 0; i < 32 / PPP; ++i) val[j][i] = *(const u4v*)(tb + (i * PPP + lane / LPX) * ROW + part * 8);
            __builtin_amdgcn_wave_barrier();
        }
#pragma unroll
        for (int i = 0; i < 32 / PPP; ++i) {
            const int px_ = pb * 32 + i * PPP + lane / LPX;
            const int pc = min(px_, a.tp - 1);
            const int row = div_by(pc, tw_m), colp = pc - row * a.tw;
            const int oy = oy0 + row, ox = ox0 + colp;
            const bool inside = px_ < a.tp && oy < a.h && ox < a.w_;
            half_t* const dst = outp + ((size_t)((n * a.h + oy) * a.w_ + ox) * a.cout + cc);
            // the same pixel of the input region: one row and one column in
            const int rpx = (row + 1) * a.rw + colp + 1;
            const int rperm = ((row + 1) * a.tw + colp + 1) & PERM0;
            const char* const rsrc = r0 + rpx * (CIN0 * 2);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if (inside && cc + j * 32 < a.cout) {
                    u4v v = val[j][i];
                    if (a.identity) {
                        const u4v rv = *(const u4v*)(rsrc + ((((cb0 + j) * 4 + part) ^ rperm) << 4));
                        v.x = pk_add(v.x, rv.x);
                        v.y = pk_add(v.y, rv.y);
                        v.z = pk_add(v.z, rv.z);
                        v.w = pk_add(v.w, rv.w);
                    }
                    v.x = pk_min(pk_max(v.x, lo2), hi2);
                    v.y = pk_min(pk_max(v.y, lo2), hi2);
                    v.z = pk_min(pk_max(v.z, lo2), hi2);
                    v.w = pk_min(pk_max(v.w, lo2), hi2);
                    *(u4v*)(dst + j * 32) = v;
                }
            }
        }
    }
}

extern "C" int dlf_launch_dw(const DlfDwArgs* a, int grid, void* stream);

// Fully connected layer (Eq. 2 with M = batch): y[n][co] = act(bias[co] + sum_k x[n][k] w[co][k]).
// One workgroup per 32 output channels; its 8 waves split K, each streaming a contiguous share
// of the packed weight fragments from HBM exactly once; partial sums meet in LDS.
#define DLF_FC_WAVES 8
#define DLF_FC_BROW 144                                      // bytes of an activation row in LDS: 4 K steps + 16
#define DLF_FC_BBYTES (32 * DLF_FC_BROW)                     // per wave

// K steps [t0, t1) of one block of 32 images for NA streams of weight fragments, on one wave.
//   Weights: an 8-deep ring of fragments per stream (8 KiB in flight per wave and stream), a slot
// refilled right behind the MFMA that used it.  A load under a condition is waited for where its
// branch ends, and the compiler cannot count the loads behind it, so a ring refilled under "if
// there is a step t + 8" drains at every turn.  Hence: the first fill clamps its step index instead
// of testing it; while at least 16 steps remain, every refill exists and is issued without a test;
// the last one or two turns of the ring use the tested form.
//   Activations: the "B" fragment of a step is 16 bytes of each of 32 rows of x, a row per image:
// read as it is used, one load touches 32 lines for a quarter of a line each, and with 8 waves at
// their own places of K the CU's vector cache does not keep those lines for the next three steps
// (VGG-16's 25088 -> 4096 layer: 45 us at batch 1, 67 us at batch 16 for the same weights).  So a
// wave fetches the rows' 128 bytes of four steps at once, 8 lanes to a row, four loads for 32 rows,
// two such groups ahead; the lanes exchange them through the wave's own LDS rows (144 bytes apart:
// the fragment reads of 32 rows are conflict-free) into the fragments of the four steps.  Beyond K
// a piece is read from the start of the weights and written as zero.
template <int NA>
__device__ __forceinline__ void fc_steps(const DlfFcArgs& a, const h8* const (&wp)[NA], int nb, int t0, int t1,
                                         char* bb, int lane, f16v (&acc)[NA])
{
    const int l32 = lane & 31, lhi = lane >> 5, rrow = lane >> 3, piece = lane & 7;
    const half_t* xrow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        xrow[i] = (const half_t*)a.x + (size_t)min(nb + i * 8 + rrow, a.batch - 1) * a.k + piece * 8;
    char* const wr = bb + rrow * DLF_FC_BROW + piece * 16;
    const char* const rd = bb + l32 * DLF_FC_BROW + lhi * 16;
    h8 av[NA][8], raw[2][4], bv[4];
    const h8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    auto fetch = [&](int slot, int tg) __attribute__((always_inline)) {      // the group of steps tg .. tg + 3
        const bool ok = tg * 16 + piece * 8 + 8 <= a.k;
#pragma unroll
        for (int i = 0; i < 4; ++i) raw[slot][i] = *(const h8*)(ok ? xrow[i] + tg * 16 : (const half_t*)a.w);
    };
    auto exchange = [&](int slot, int tg) __attribute__((always_inline)) {
        const bool ok = tg * 16 + piece * 8 + 8 <= a.k;
#pragma unroll
        for (int i = 0; i < 4; ++i) *(h8*)(wr + i * 8 * DLF_FC_BROW) = ok ? raw[slot][i] : zero8;
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int s_ = 0; s_ < 4; ++s_) bv[s_] = *(const h8*)(rd + s_ * 32);
        __builtin_amdgcn_wave_barrier();
    };
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int t = max(min(t0 + j, t1 - 1), 0);
#pragma unroll
        for (int n = 0; n < NA; ++n) av[n][j] = __builtin_nontemporal_load(wp[n] + (size_t)t * 64);
    }
    fetch(0, t0);
    fetch(1, t0 + 4);
    int tb = t0;
    for (; tb + 16 <= t1; tb += 8) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (j == 0) { exchange(0, tb); fetch(0, tb + 8); }
            if (j == 4) { exchange(1, tb + 4); fetch(1, tb + 12); }
#pragma unroll
            for (int n = 0; n < NA; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[n][j], bv[j & 3], acc[n], 0, 0, 0);
            const int tn = tb + j + 8;
#pragma unroll
            for (int n = 0; n < NA; ++n) av[n][j] = __builtin_nontemporal_load(wp[n] + (size_t)tn * 64);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    for (; tb < t1; tb += 8) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (j == 0) {
                exchange(0, tb);
                if (tb + 8 < t1) fetch(0, tb + 8);
            }
            if (j == 4) {
                exchange(1, tb + 4);
                if (tb + 12 < t1) fetch(1, tb + 12);
            }
            const int t = tb + j;
            if (t < t1) {
#pragma unroll
                for (int n = 0; n < NA; ++n)
                    acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[n][j], bv[j & 3], acc[n], 0, 0, 0);
                const int tn = t + 8;
                if (tn < t1) {
#pragma unroll
                    for (int n = 0; n < NA; ++n) av[n][j] = __builtin_nontemporal_load(wp[n] + (size_t)tn * 64);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
}

__global__ __launch_bounds__(DLF_FC_WAVES * 64) void k_fc(const DlfFcArgs a)
{
    // the waves' activation rows during the K loop, their partial sums behind it
    __shared__ __align__(16) char smem[DLF_FC_WAVES * DLF_FC_BBYTES];
    static_assert(sizeof(smem) >= DLF_FC_WAVES * 16 * 64 * 4, "partial sums");
    float (*const red)[16][64] = (float (*)[16][64])smem;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cb = blockIdx.x;
    half_t* y = (half_t*)a.y;
    const h8* const wp[1] = {(const h8*)a.w + (size_t)cb * a.nsteps * 64 + lane};
    // each wave a contiguous eighth of the K steps, whole groups of four
    const int per = ((a.nsteps + DLF_FC_WAVES - 1) / DLF_FC_WAVES + 3) & ~3;
    const int t0 = min(wave * per, a.nsteps), t1 = min(a.nsteps, t0 + per);
    for (int nb = 0; nb < a.batch; nb += 32) {
        f16v acc[1];
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[0][i] = 0.0f;
        fc_steps<1>(a, wp, nb, t0, t1, smem + wave * DLF_FC_BBYTES, lane, acc);
        __syncthreads();                                     // the sums take the rows' place
#pragma unroll
        for (int i = 0; i < 16; ++i) red[wave][i][lane] = acc[0][i];
        __syncthreads();
        for (int e = tid; e < 16 * 64; e += DLF_FC_WAVES * 64) {
            const int i = e >> 6, ln = e & 63;
            float s = 0.0f;
#pragma unroll
            for (int w = 0; w < DLF_FC_WAVES; ++w) s += red[w][i][ln];
            const int co = cb * 32 + (i >> 2) * 8 + (ln >> 5) * 4 + (i & 3);
            const int im = nb + (ln & 31);
            if (co < a.cout && im < a.batch)
                y[(size_t)im * a.cout + co] = (half_t)apply_act(s + a.bias[co], a.act);
        }
        __syncthreads();
    }
}

// Split-K form of the fully connected layer, for long K and few output channels per CU (VGG's
// 25088 -> 4096): a workgroup takes two 32-channel blocks (the activation fragment of a K step
// feeds two MFMAs) and one of `ksplit` slices of K, so that the operand bytes a CU has to take in
// drop from 2 KiB to 0.75 KiB per MFMA and ksplit times as many CUs share them.  The partial sums
// (fp32, in the MFMA accumulator layout) go to scratch memory; k_fc_fin adds the slices in a fixed
// order, the bias and the activation.
__global__ __launch_bounds__(DLF_FC_WAVES * 64) void k_fc_sk(const DlfFcArgs a)
{
    __shared__ __align__(16) char smem[DLF_FC_WAVES * DLF_FC_BBYTES];
    float (*const red)[16][64] = (float (*)[16][64])smem;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ks = blockIdx.x % a.ksplit, cbp = blockIdx.x / a.ksplit;
    const int cb0 = cbp * 2, cb1 = min(cb0 + 1, a.ncb - 1);
    const h8* const wp[2] = {(const h8*)a.w + (size_t)cb0 * a.nsteps * 64 + lane,
                             (const h8*)a.w + (size_t)cb1 * a.nsteps * 64 + lane};
    // slices and the waves' shares of a slice: whole groups of four K steps
    const int per_ks = ((a.nsteps + a.ksplit - 1) / a.ksplit + 3) & ~3;
    const int s0 = min(ks * per_ks, a.nsteps), s1 = min(a.nsteps, s0 + per_ks);
    const int per = ((s1 - s0 + DLF_FC_WAVES - 1) / DLF_FC_WAVES + 3) & ~3;
    const int t0 = min(s0 + wave * per, s1), t1 = min(s1, t0 + per);
    for (int nb = 0; nb < a.batch; nb += 32) {
        f16v acc[2];
#pragma unroll
        for (int i = 0; i < 16; ++i) { acc[0][i] = 0.0f; acc[1][i] = 0.0f; }
        fc_steps<2>(a, wp, nb, t0, t1, smem + wave * DLF_FC_BBYTES, lane, acc);
        __syncthreads();                                     // the sums take the rows' place
        float* pbase = a.part + (size_t)((nb >> 5) * a.ksplit + ks) * a.ncb * 1024;
#pragma unroll
        for (int f = 0; f < 2; ++f) {
            if (f == 1 && cb0 + 1 >= a.ncb) break;          // uniform: an odd number of blocks
#pragma unroll
            for (int i = 0; i < 16; ++i) red[wave][i][lane] = acc[f][i];
            __syncthreads();
            for (int e = tid; e < 16 * 64; e += DLF_FC_WAVES * 64) {
                const int i = e >> 6, ln = e & 63;
                float sum = 0.0f;
#pragma unroll
                for (int w = 0; w < DLF_FC_WAVES; ++w) sum += red[w][i][ln];
                pbase[(size_t)(cb0 + f) * 1024 + e] = sum;
            }
            __syncthreads();
        }
    }
}

__global__ __launch_bounds__(256) void k_fc_fin(const DlfFcArgs a)
{
    const int cb = blockIdx.x % a.ncb, nbi = blockIdx.x / a.ncb;
    half_t* y = (half_t*)a.y;
    for (int e = threadIdx.x; e < 16 * 64; e += 256) {
        const int i = e >> 6, ln = e & 63;
        float s = 0.0f;
        for (int ks = 0; ks < a.ksplit; ++ks)
            s += a.part[((size_t)(nbi * a.ksplit + ks) * a.ncb + cb) * 1024 + e];
        const int co = cb * 32 + (i >> 2) * 8 + (ln >> 5) * 4 + (i & 3);
        const int im = nbi * 32 + (ln & 31);
        if (co < a.cout && im < a.batch)
            y[(size_t)im * a.cout + co] = (half_t)apply_act(s + a.bias[co], a.act);
    }
}

// Global average pooling: fp32 sum over H*W, mean, fp16.
__global__ __launch_bounds__(256) void k_gap(const DlfGapArgs a)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= a.batch * a.c) return;
    const int n = idx / a.c, c = idx - n * a.c;
    const half_t* p = (const half_t*)a.x + (size_t)n * a.hw * a.c + c;
    float s = 0.0f;
#pragma unroll 7
    for (int i = 0; i < a.hw; ++i) s += (float)p[(size_t)i * a.c];
    ((half_t*)a.y)[idx] = (half_t)(s / (float)a.hw);
}

// Profiling: a start / stop event pair attached to the next launch of this thread.  The runtime
// stamps such events with the dispatch's own begin and end, so their difference is the kernel's
// duration (what a kernel trace reports), free of the gaps around events recorded on the stream.
static thread_local hipEvent_t g_ev_start = nullptr, g_ev_stop = nullptr;
extern "C" void dlf_next_launch_events(void* start, void* stop)
{
    g_ev_start = (hipEvent_t)start;
    g_ev_stop = (hipEvent_t)stop;
}

template <typename K, typename A>
static void launch(K k, dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream, const A& a)
{
    if (g_ev_start != nullptr || g_ev_stop != nullptr) {
        hipExtLaunchKernelGGL(k, grid, block, lds_bytes, stream, g_ev_start, g_ev_stop, 0, a);
        g_ev_start = g_ev_stop = nullptr;
    } else {
        hipLaunchKernelGGL(k, grid, block, lds_bytes, stream, a);
    }
}

typedef void (*group_kernel_t)(const DlfGroupArgs);
static group_kernel_t group_kernel(int variant, bool ksplit)
{
    switch (variant) {
    case 0: return ksplit ? nullptr : k_group<2, 2, 2>;
    case 1: return ksplit ? nullptr : k_group<1, 4, 2>;
    case 2: return ksplit ? k_group<1, 2, 2, true> : k_group<1, 2, 2>;
    case 3: return ksplit ? k_group<1, 2, 4, true> : k_group<1, 2, 4>;
    default: return nullptr;
    }
}

typedef void (*c3s_kernel_t)(const DlfC3sArgs);
static c3s_kernel_t c3s_kernel(int taps, int stride, int fp)
{
    if (taps == 9 && stride == 1) return fp == 2 ? k_c3s<9, 1, 2> : k_c3s<9, 1, 1>;
    if (taps == 9 && stride == 2) return fp == 2 ? k_c3s<9, 2, 2> : k_c3s<9, 2, 1>;
    if (taps == 1 && stride == 1) return fp == 2 ? k_c3s<1, 1, 2> : k_c3s<1, 1, 1>;
    return nullptr;
}
static c3s_kernel_t c3s_kernel_i8(int taps, int fp)
{
    if (taps == 9) return fp == 2 ? k_c3s<9, 1, 2, true> : k_c3s<9, 1, 1, true>;
    if (taps == 1) return fp == 2 ? k_c3s<1, 1, 2, true> : k_c3s<1, 1, 1, true>;
    return nullptr;
}

typedef void (*c3_kernel_t)(const DlfC3Args);
static c3_kernel_t c3_kernel(int shape)
{
    switch (shape) {
    case 0: return k_c3b<2, 32, 2>;
    case 1: return k_c3b<2, 64, 2>;
    case 2: return k_c3b<1, 32, 2>;
    case 3: return k_c3b<1, 64, 2>;
    case 4: return k_c3b<2, 32, 4>;
    default: return nullptr;
    }
}
static c3_kernel_t c3_kernel_i8(int shape)
{
    switch (shape) {
    case 0: return k_c3b<2, 32, 2, true>;
    case 1: return k_c3b<2, 64, 2, true>;
    case 2: return k_c3b<1, 32, 2, true>;
    case 3: return k_c3b<1, 64, 2, true>;
    case 4: return k_c3b<2, 32, 4, true>;
    default: return nullptr;
    }
}

extern "C" int dlf_kernels_init(void)
{
    for (int v = 0; v < 2 * DLF_NUM_VARIANTS; ++v) {
        group_kernel_t k = group_kernel(v >> 1, (v & 1) != 0);
        if (k == nullptr) continue;
        hipError_t e = hipFuncSetAttribute((const void*)k, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           160 * 1024);
        if (e != hipSuccess) return (int)e;
    }
    {
        hipError_t e = hipFuncSetAttribute((const void*)k_dwt<1>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void*)k_dwt<2>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return (int)e;
    }
    {
        hipError_t e2 = hipFuncSetAttribute((const void*)k_c3pw<2, 128>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e2 == hipSuccess) e2 = hipFuncSetAttribute((const void*)k_c3pw<4, 128>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e2 == hipSuccess) e2 = hipFuncSetAttribute((const void*)k_c3pw<2, 256>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e2 == hipSuccess) e2 = hipFuncSetAttribute((const void*)k_c3pw<4, 256>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e2 == hipSuccess) e2 = hipFuncSetAttribute((const void*)k_c3pw<2, 64>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e2 == hipSuccess) e2 = hipFuncSetAttribute((const void*)k_c3pw<4, 64>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e2 == hipSuccess) e2 = hipFuncSetAttribute((const void*)k_bneck<64>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e2 == hipSuccess) e2 = hipFuncSetAttribute((const void*)k_bneck<128>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e2 == hipSuccess) e2 = hipFuncSetAttribute((const void*)k_bneck<256>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e2 == hipSuccess) e2 = hipFuncSetAttribute((const void*)k_bneck<512>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e2 != hipSuccess) return (int)e2;
        for (int v = 0; v < 6; ++v) {
            hipError_t e = hipFuncSetAttribute((const void*)c3s_kernel(v < 4 ? 9 : 1, (v >> 1) == 1 ? 2 : 1, (v & 1) + 1),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return (int)e;
        }
        for (int v = 0; v < 4; ++v) {
            hipError_t e = hipFuncSetAttribute((const void*)c3s_kernel_i8(v < 2 ? 9 : 1, (v & 1) + 1),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return (int)e;
        }
    }
    {
        const void* ks[4] = {(const void*)k_dws<1, 1>, (const void*)k_dws<1, 2>, (const void*)k_dws<2, 1>, (const void*)k_dws<2, 2>};
        for (const void* k : ks) {
            hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return (int)e;
        }
    }
    for (int sh = 0; sh < 2 * DLF_C3_SHAPES; ++sh) {
        const c3_kernel_t k = sh < DLF_C3_SHAPES ? c3_kernel(sh) : c3_kernel_i8(sh - DLF_C3_SHAPES);
        hipError_t e = hipFuncSetAttribute((const void*)k, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return (int)e;
    }
    return 0;
}

extern "C" int dlf_launch_c3(const DlfC3Args* a, int shape, int grid, int lds_bytes, void* stream)
{
    c3_kernel_t k = c3_kernel(shape);
    if (k == nullptr || grid < 8 || (grid & 7) != 0 || lds_bytes <= 0) return (int)hipErrorInvalidValue;
    launch(k, dim3(grid), dim3(DLF_C3_WAVES * 64), (size_t)lds_bytes, (hipStream_t)stream, *a);
    return (int)hipGetLastError();
}

extern "C" int dlf_launch_c3_i8(const DlfC3Args* a, int shape, int grid, int lds_bytes, void* stream)
{
    c3_kernel_t k = c3_kernel_i8(shape);
    if (k == nullptr || grid < 8 || (grid & 7) != 0 || lds_bytes <= 0 || a->scale == nullptr || a->res != nullptr ||
        (a->cout & 15) != 0 || (a->pool2 != 0 && (((a->th | a->tw) & 1) != 0 || a->h < 2 || a->w_ < 2)))
        return (int)hipErrorInvalidValue;
    launch(k, dim3(grid), dim3(DLF_C3_WAVES * 64), (size_t)lds_bytes, (hipStream_t)stream, *a);
    return (int)hipGetLastError();
}

extern "C" int dlf_launch_group(const DlfGroupArgs* a, int variant, int grid, int lds_bytes,
                                void* stream)
{
    const bool ksplit = a->nstages == 1 && a->st[0].kind == DLF_ST_CONV && a->st[0].ksplit > 1;
    group_kernel_t k = group_kernel(variant, ksplit);
    if (k == nullptr || grid <= 0) return (int)hipErrorInvalidValue;
    launch(k, dim3(grid), dim3(DLF_WG_THREADS), (size_t)lds_bytes, (hipStream_t)stream, *a);
    return (int)hipGetLastError();
}

extern "C" int dlf_launch_fc(const DlfFcArgs* a, void* stream)
{
    if (a->ksplit > 1) {
        if (a->part == nullptr) return (int)hipErrorInvalidValue;
        // a stop event requested for "the next launch" belongs to the second of the two
        hipEvent_t stop = g_ev_stop;
        g_ev_stop = nullptr;
        launch(k_fc_sk, dim3(((a->ncb + 1) / 2) * a->ksplit), dim3(DLF_FC_WAVES * 64), 0,
               (hipStream_t)stream, *a);
        g_ev_stop = stop;
        launch(k_fc_fin, dim3(a->ncb * ((a->batch + 31) / 32)), dim3(256), 0, (hipStream_t)stream, *a);
        return (int)hipGetLastError();
    }
    launch(k_fc, dim3(a->ncb), dim3(DLF_FC_WAVES * 64), 0, (hipStream_t)stream, *a);
    return (int)hipGetLastError();
}

extern "C" int dlf_launch_pw(const DlfPwArgs* a, int shape, int grid, void* stream)
{
    if (grid <= 0) return (int)hipErrorInvalidValue;
    // a second operand pair: block forms only, whole stages of K steps, both operands present
    if (a->nsteps2 != 0 && ((shape != 3 && shape != 4) || a->nsteps2 < 0 || (a->nsteps2 % DLF_PWB_KS) != 0 ||
                            a->in2 == nullptr || a->w2 == nullptr || a->bias2 == nullptr || a->res != nullptr))
        return (int)hipErrorInvalidValue;
    if (shape == 0)
        launch(k_pw<2, 2, 6, 2>, dim3(grid), dim3(DLF_PW_WAVES * 64),
                           (size_t)(DLF_PW_WAVES * 64 * (64 + 8) * 2), (hipStream_t)stream, *a);
    else if (shape == 1)
        launch(k_pw<1, 1, 8, 4>, dim3(grid), dim3(DLF_PW_WAVES * 64),
                           (size_t)(DLF_PW_WAVES * 32 * (32 + 8) * 2), (hipStream_t)stream, *a);
    else if (shape == 2)
        launch(k_pw_sk, dim3(grid), dim3(DLF_PW_WAVES * 64),
                           (size_t)(DLF_PWSK_PART_BYTES + DLF_PW_WAVES * 32 * (32 + 8) * 2),
                           (hipStream_t)stream, *a);
    else if (shape == 3)
        launch(a->nsteps2 != 0 ? k_pwb<2, 2, true> : k_pwb<2, 2, false>, dim3(grid), dim3(DLF_PW_WAVES * 64),
               (size_t)DLF_PWB_LDS_BYTES(2, 2), (hipStream_t)stream, *a);
    else if (shape == 4)
        launch(a->nsteps2 != 0 ? k_pwb<1, 4, true> : k_pwb<1, 4, false>, dim3(grid), dim3(DLF_PW_WAVES * 64),
               (size_t)DLF_PWB_LDS_BYTES(1, 4), (hipStream_t)stream, *a);
    else
        return (int)hipErrorInvalidValue;
    return (int)hipGetLastError();
}

extern "C" int dlf_launch_pw_i8(const DlfPwArgs* a, int shape, int grid, void* stream)
{
    if (grid < 8 || (grid & 7) != 0 || a->scale == nullptr || a->res != nullptr || a->nsteps2 != 0 || a->stride != 1 ||
        (a->nsteps % DLF_PWB_KS) != 0 || (a->cout & 15) != 0)
        return (int)hipErrorInvalidValue;
    if (shape == 3)
        launch(k_pwb<2, 2, false, true>, dim3(grid), dim3(DLF_PW_WAVES * 64), (size_t)DLF_PWB_LDS_BYTES(2, 2), (hipStream_t)stream, *a);
    else if (shape == 4)
        launch(k_pwb<1, 4, false, true>, dim3(grid), dim3(DLF_PW_WAVES * 64), (size_t)DLF_PWB_LDS_BYTES(1, 4), (hipStream_t)stream, *a);
    else
        return (int)hipErrorInvalidValue;
    return (int)hipGetLastError();
}

extern "C" int dlf_launch_dw(const DlfDwArgs* a, int grid, void* stream)
{
    if (grid <= 0 || (a->stride != 1 && a->stride != 2) || a->in_bytes >= 0x80000000u || (a->c & 7) != 0)
        return (int)hipErrorInvalidValue;
    if (a->stride == 1)
        launch(k_dw<1>, dim3(grid), dim3(DLF_DW_WAVES * 64), 0, (hipStream_t)stream, *a);
    else
        launch(k_dw<2>, dim3(grid), dim3(DLF_DW_WAVES * 64), 0, (hipStream_t)stream, *a);
    return (int)hipGetLastError();
}

extern "C" int dlf_launch_dwpw(const DlfDwPwArgs* a, int nb, int grid, void* stream)
{
    if (grid <= 0 || (a->stride != 1 && a->stride != 2) || a->in_bytes >= 0x80000000u || (a->c & 31) != 0 ||
        a->nsteps != a->c / 16 || (a->cout & 7) != 0)
        return (int)hipErrorInvalidValue;
    if (nb == 2)
        launch(k_dwpw<2>, dim3(grid), dim3(DLF_DWPW_WAVES * 64), (size_t)DLF_DWPW_LDS_BYTES(a->c, 2), (hipStream_t)stream, *a);
    else if (nb == 4)
        launch(k_dwpw<4>, dim3(grid), dim3(DLF_DWPW_WAVES * 64), (size_t)DLF_DWPW_LDS_BYTES(a->c, 4), (hipStream_t)stream, *a);
    else
        return (int)hipErrorInvalidValue;
    return (int)hipGetLastError();
}

extern "C" int dlf_launch_dwt(const DlfDwtArgs* a, int grid, int lds_bytes, void* stream)
{
    // what the kernel's indexing assumes
    if (grid <= 0 || (a->stride != 1 && a->stride != 2) || a->in_bytes >= 0x80000000u) return (int)hipErrorInvalidValue;
    if (a->cg * 8 != a->c || a->cg < 4 || a->cg > 64 || (a->cg & (a->cg - 1)) != 0 || a->pxw * a->cg != 64)
        return (int)hipErrorInvalidValue;
    if (a->rw != 1 && a->rw != 2 && a->rw != 4 && a->rw != 7 && a->rw != 8 && a->rw != 14 && a->rw != 16)
        return (int)hipErrorInvalidValue;
    if ((a->nsteps & (a->nsteps - 1)) != 0 || a->nsteps < 2) return (int)hipErrorInvalidValue;
    if (a->wx * a->wy != DLF_DWT_WAVES || a->th != a->wy * a->rw || a->tw != a->wx * a->pxw || a->tp != a->th * a->tw ||
        a->tp > 256 || a->npb != (a->tp + 31) / 32 || a->npg != (a->npb + 3) / 4 || a->nsteps != a->c / 16 ||
        (a->cout & 7) != 0 || lds_bytes != (int)DLF_DWT_LDS_BYTES(a->tp, a->c) || lds_bytes > 160 * 1024)
        return (int)hipErrorInvalidValue;
    if (a->stride == 1)
        launch(k_dwt<1>, dim3(grid), dim3(DLF_DWT_WAVES * 64), (size_t)lds_bytes, (hipStream_t)stream, *a);
    else
        launch(k_dwt<2>, dim3(grid), dim3(DLF_DWT_WAVES * 64), (size_t)lds_bytes, (hipStream_t)stream, *a);
    return (int)hipGetLastError();
}

extern "C" int dlf_launch_dws(const DlfDwsArgs* a, int grid, int lds_bytes, void* stream)
{
    // what the kernel's indexing assumes
    if (grid <= 0 || (grid & 7) != 0 || (a->stride != 1 && a->stride != 2) || a->in_bytes >= 0x80000000u)
        return (int)hipErrorInvalidValue;
    if ((a->kh != 256 && a->kh != 512) || a->nkh < 1 || a->kh * a->nkh != a->c || a->nsteps != a->c / 16 || (a->cout & 7) != 0)
        return (int)hipErrorInvalidValue;
    if (a->th < 1 || a->th > 8 || a->tw < 1 || a->tw > 8 || a->tp != a->th * a->tw || a->rh != (a->th - 1) * a->stride + 3 ||
        a->rw != (a->tw - 1) * a->stride + 3 || a->rp != a->rh * a->rw)
        return (int)hipErrorInvalidValue;
    if ((a->cbw != 1 && a->cbw != 2) || a->nsl != (a->ncb + 8 * a->cbw - 1) / (8 * a->cbw) ||
        a->tiles_y != (a->oh + a->th - 1) / a->th || a->tiles_x != (a->ow + a->tw - 1) / a->tw ||
        a->ntiles != a->batch * a->tiles_y * a->tiles_x || grid != (a->ntiles + 7) / 8 * 8 * a->nsl)
        return (int)hipErrorInvalidValue;
    if ((a->nbuf != a->nkh && a->nbuf != 1) || lds_bytes != (int)DLF_DWS_LDS_BYTES(a->rp, a->tp, a->kh, a->cbw, a->nbuf) ||
        lds_bytes > 160 * 1024)
        return (int)hipErrorInvalidValue;
    // (the counted waits of the kernel go up to 48 outstanding loads)
    if ((a->nbuf - 1) * ((int)(DLF_DWS_IN_BYTES(a->rp, a->kh) / 1024 + DLF_DWS_WAVES - 1) / DLF_DWS_WAVES) + 16 + 11 > 48)
        return (int)hipErrorInvalidValue;
    const dim3 block(DLF_DWS_WAVES * 64);
    if (a->stride == 1 && a->cbw == 1) launch(k_dws<1, 1>, dim3(grid), block, (size_t)lds_bytes, (hipStream_t)stream, *a);
    else if (a->stride == 1) launch(k_dws<1, 2>, dim3(grid), block, (size_t)lds_bytes, (hipStream_t)stream, *a);
    else if (a->cbw == 1) launch(k_dws<2, 1>, dim3(grid), block, (size_t)lds_bytes, (hipStream_t)stream, *a);
    else launch(k_dws<2, 2>, dim3(grid), block, (size_t)lds_bytes, (hipStream_t)stream, *a);
    return (int)hipGetLastError();
}

extern "C" int dlf_launch_c3s(const DlfC3sArgs* a, int grid, int lds_bytes, void* stream)
{
    // what the kernel's indexing assumes
    if (grid <= 0 || (grid & 7) != 0 || a->in_bytes >= 0x80000000u) return (int)hipErrorInvalidValue;
    if ((a->taps != 9 && a->taps != 1) || (a->stride != 1 && a->stride != 2) || (a->taps == 1 && a->stride != 1) ||
        (a->cin != 256 && a->cin != 512 && a->cin != 1024 && a->cin != 2048) || a->nsteps != a->taps * a->cin / 16 ||
        (a->cout & 7) != 0)
        return (int)hipErrorInvalidValue;
    const int halo = a->taps == 9 ? 1 : 0, chunks = a->cin / (a->taps == 9 ? 32 : 128), s = a->stride;
    if ((a->ksplit != 1 && a->ksplit != 2 && a->ksplit != 4) || (chunks % a->ksplit) != 0 ||
        a->nsl != (a->ncb + DLF_C3S_WAVES / a->ksplit - 1) / (DLF_C3S_WAVES / a->ksplit))
        return (int)hipErrorInvalidValue;
    if (a->th < 1 || a->th > 8 || a->tw < 1 || a->tw > 8 || a->tp != a->th * a->tw ||
        a->rw != (a->tw - 1) * s + 1 + 2 * halo || a->rp != ((a->th - 1) * s + 1 + 2 * halo) * a->rw ||
        a->oh != (a->h + 2 * halo - (a->taps == 9 ? 3 : 1)) / s + 1 || a->ow != (a->w_ + 2 * halo - (a->taps == 9 ? 3 : 1)) / s + 1 ||
        a->tiles_y != (a->oh + a->th - 1) / a->th || a->tiles_x != (a->ow + a->tw - 1) / a->tw ||
        a->ntiles != a->batch * a->tiles_y * a->tiles_x ||
        (a->slice_major != 0 && a->slice_major != 1) ||
        (a->slice_major && (a->nsl != 2 && a->nsl != 4 && a->nsl != 8)) ||
        grid != (a->slice_major ? (a->ntiles + 8 / a->nsl - 1) / (8 / a->nsl) * 8 : (a->ntiles + 7) / 8 * 8 * a->nsl))
        return (int)hipErrorInvalidValue;
    if (lds_bytes != (int)DLF_C3S_LDS_BYTES(a->rp, a->cin) || lds_bytes > 160 * 1024) return (int)hipErrorInvalidValue;
    if (a->scale != nullptr) {       // the quantised form
        if (s != 1 || a->res != nullptr || (a->cout & 15) != 0) return (int)hipErrorInvalidValue;
        if (a->pool2 != 0 && (a->pool2 != 1 || a->taps != 9 || a->tw != 8 || (a->th & 1) != 0 || a->oh < 2 || a->ow < 2))
            return (int)hipErrorInvalidValue;
        launch(c3s_kernel_i8(a->taps, a->tp > 32 ? 2 : 1), dim3(grid), dim3(DLF_C3S_WAVES * 64), (size_t)lds_bytes,
               (hipStream_t)stream, *a);
        return (int)hipGetLastError();
    }
    if (a->pool2 != 0) return (int)hipErrorInvalidValue;
    launch(c3s_kernel(a->taps, s, a->tp > 32 ? 2 : 1), dim3(grid), dim3(DLF_C3S_WAVES * 64), (size_t)lds_bytes,
           (hipStream_t)stream, *a);
    return (int)hipGetLastError();
}

extern "C" int dlf_launch_c3pw(const DlfC3PwArgs* a, int grid, int lds_bytes, void* stream)
{
    // what the kernel's indexing assumes
    if (grid <= 0 || (grid & 7) != 0 || a->in_bytes >= 0x80000000u || a->res_bytes >= 0x80000000u) return (int)hipErrorInvalidValue;
    if (a->c != 64 && a->c != 128 && a->c != 256) return (int)hipErrorInvalidValue;
    const int waves = DLF_C3PW_WAVES(a->c);
    if ((a->cout & 7) != 0 || a->ncb2 != (a->cout + 31) / 32 || a->nsl != (a->ncb2 + 2 * waves - 1) / (2 * waves))
        return (int)hipErrorInvalidValue;
    if (a->th < 1 || a->th > 8 || a->tw < 1 || a->tw > 16 || a->tp != a->th * a->tw || a->tp > 128 || a->rw != a->tw + 2 ||
        a->rp != (a->th + 2) * (a->tw + 2) || a->tiles_y != (a->h + a->th - 1) / a->th ||
        a->tiles_x != (a->w_ + a->tw - 1) / a->tw || a->ntiles != a->batch * a->tiles_y * a->tiles_x ||
        grid != (a->ntiles + 7) / 8 * 8 * a->nsl)
        return (int)hipErrorInvalidValue;
    if (lds_bytes != (int)DLF_C3PW_LDS_BYTES(a->rp, a->tp, a->c, a->res != nullptr) || lds_bytes > 160 * 1024)
        return (int)hipErrorInvalidValue;
    void (*const kern)(DlfC3PwArgs) = a->c == 64    ? (a->tp > 64 ? k_c3pw<4, 64> : k_c3pw<2, 64>)
                                      : a->c == 128 ? (a->tp > 64 ? k_c3pw<4, 128> : k_c3pw<2, 128>)
                                                    : (a->tp > 64 ? k_c3pw<4, 256> : k_c3pw<2, 256>);
    launch(kern, dim3(grid), dim3(waves * 64), (size_t)lds_bytes, (hipStream_t)stream, *a);
    return (int)hipGetLastError();
}

extern "C" int dlf_launch_bneck(const DlfBnArgs* a, int grid, int lds_bytes, void* stream)
{
    // what the kernel's indexing assumes
    if (grid <= 0 || (grid & 7) != 0 || a->in_bytes >= 0x80000000u) return (int)hipErrorInvalidValue;
    if (a->cin0 != 64 && a->cin0 != 128 && a->cin0 != 256 && a->cin0 != 512) return (int)hipErrorInvalidValue;
    if (a->ncb2 == 0) {                                      // two layers: the output is the second layer's
        if (a->cout != 64 || a->nsl != 1 || a->identity) return (int)hipErrorInvalidValue;
    } else if (a->cin0 == 64 || (a->cout & 7) != 0 || a->ncb2 != (a->cout + 31) / 32 ||
               a->nsl != (a->ncb2 + 2 * DLF_BN_WAVES - 1) / (2 * DLF_BN_WAVES) || (a->identity && a->cout != a->cin0)) {
        return (int)hipErrorInvalidValue;
    }
    if (a->th < 1 || a->th > 8 || a->tw < 1 || a->tw > 16 || a->tp != a->th * a->tw || a->tp > 64 || a->rw != a->tw + 2 ||
        a->rp != (a->th + 2) * (a->tw + 2) || a->tiles_y != (a->h + a->th - 1) / a->th ||
        a->tiles_x != (a->w_ + a->tw - 1) / a->tw || a->ntiles != a->batch * a->tiles_y * a->tiles_x ||
        grid != (a->ntiles + 7) / 8 * 8 * a->nsl)
        return (int)hipErrorInvalidValue;
    if (lds_bytes != (int)DLF_BN_LDS_BYTES(a->rp, a->tp, a->cin0) || lds_bytes > 160 * 1024) return (int)hipErrorInvalidValue;
    void (*const kern)(DlfBnArgs) = a->cin0 == 64 ? k_bneck<64> : (a->cin0 == 128 ? k_bneck<128> : (a->cin0 == 256 ? k_bneck<256> : k_bneck<512>));
    launch(kern, dim3(grid), dim3(DLF_BN_WAVES * 64), (size_t)lds_bytes, (hipStream_t)stream, *a);
    return (int)hipGetLastError();
}

extern "C" int dlf_launch_gap(const DlfGapArgs* a, void* stream)
{
    const int total = a->batch * a->c;
    launch(k_gap, dim3((total + 255) / 256), dim3(256), 0, (hipStream_t)stream, *a);
    return (int)hipGetLastError();
}
