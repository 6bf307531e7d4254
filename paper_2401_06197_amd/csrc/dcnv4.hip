// DCNv4 spatial aggregation for MI355X (gfx950): kernels and the C ABI of include/dcnv4.h.
//
// Operator: paper Sec. 3.1, Eq. 1-2 without the softmax.  Work organisation follows the
// idea of Sec. 3.2 (one thread serves a run of channels of one group at one output pixel,
// so one offset/mask read and one set of bilinear coefficients is shared, and the channel
// run is moved with 128-bit memory instructions); everything below that idea is laid out
// for CDNA4: wave64, raw buffer loads whose hardware range check supplies the zero for
// rows outside the image, offset/mask tiles staged through LDS with 128-bit coalesced
// loads, tiles handed to XCDs in contiguous bands so that neighbouring outputs share an L2.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "dcnv4.h"

namespace {

constexpr int kThreads = 256;
constexpr int kTaps = 9;
constexpr int kXcds = 8;
// Word 3 of a gfx9-family raw buffer descriptor: 32-bit data format, no swizzle, no stride.
constexpr int kRsrcWord3 = 0x00020000;
// A byte offset no descriptor of ours reaches (images are validated below 2^31 bytes):
// loads through it return zero, atomics through it are dropped.
constexpr int kOutside = (int)0x80000000u;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __amdgpu_buffer_rsrc_t rsrc_t;

// n / d for 0 <= n < 2^31 as mulhi + add + shift (d >= 1), constants made on the host.
struct FastDiv {
    unsigned mul, shift;
};

__device__ __forceinline__ int fdiv(int n, FastDiv f)
{
    return (int)((__umulhi((unsigned)n, f.mul) + (unsigned)n) >> f.shift);
}

struct Geo {
    int H, W, Ho, Wo, G;
    int sh, sw, ph, pw, dh, dw;
    float scale;        // offset_scale
    float dmax;         // scaled offsets are clamped to [-dmax, dmax]; beyond that every corner is outside
    int pgi;            // (pixel, group) pairs per image = Ho*Wo*G
    int tiles_per_image, ntiles, tiles_per_xcd, remap;
    FastDiv div_g, div_wo, div_tpi;
    int x_img_bytes;    // H*W*C*sizeof(T)
    int y_img_bytes;    // Ho*Wo*C*sizeof(T)
    int row_bytes;      // W*C*sizeof(T)
    int pix_bytes;      // C*sizeof(T)
};

__device__ __forceinline__ rsrc_t make_rsrc(const void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, kRsrcWord3);
}

// blockIdx -> tile.  Hardware deals consecutive workgroups to the 8 XCDs in turn; with the
// remap XCD i works through tiles [i*tiles_per_xcd, (i+1)*tiles_per_xcd) in order, so the
// tiles in flight on one XCD are spatial neighbours and their input pixels hit that XCD's L2.
__device__ __forceinline__ int tile_of_block(const Geo &p)
{
    const int b = blockIdx.x;
    return p.remap ? (b & (kXcds - 1)) * p.tiles_per_xcd + (b >> 3) : b;
}

// Copy `bytes` of a tensor region starting at byte `start` (of `base`, 16-byte aligned) into
// LDS, beginning at the 16-byte boundary below `start`; returns how many bytes of lead-in
// precede the region in LDS.  All global reads are aligned 128-bit loads whose dwords are
// range-checked one by one against a descriptor that ends exactly at the region's end, so
// nothing past the tensor is touched.  A region of 2-byte elements can end in the middle of a
// dword; the hardware zeroes that whole dword, so the thread that holds it fetches the last
// element again with a 16-bit load.
template <int CAP_BYTES, int ELEM_BYTES>
__device__ __forceinline__ int stage_region(char *lds, const char *base, long long start, int bytes)
{
    const long long aligned = start & ~15LL;
    const int delta = (int)(start - aligned);
    const int total = delta + bytes;                       // < CAP_BYTES by construction
    const rsrc_t r = make_rsrc(base + aligned, (unsigned)total);
#pragma unroll
    for (int o = 0; o < CAP_BYTES; o += kThreads * 16) {
        const int off = o + (int)threadIdx.x * 16;
        if (off < total) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
            *reinterpret_cast<u32x4 *>(lds + off) = v;
            if (ELEM_BYTES == 2 && (total & 2) && off + 16 >= total) {
                const unsigned short tail = __builtin_amdgcn_raw_buffer_load_b16(r, total - 2, 0, 0);
                *reinterpret_cast<unsigned short *>(lds + total - 2) = tail;
            }
        }
    }
    return delta;
}

template <typename T, int CPT> struct Vec;          // CPT channels of one pixel in registers
template <int CPT> struct Vec<_Float16, CPT> {
    static constexpr int kRegs = CPT / 8;
    f16x8 v[kRegs];
    __device__ __forceinline__ void load(rsrc_t r, int off)
    {
#pragma unroll
        for (int i = 0; i < kRegs; ++i)
            v[i] = __builtin_bit_cast(f16x8, __builtin_amdgcn_raw_buffer_load_b128(r, off + 16 * i, 0, 0));
    }
    __device__ __forceinline__ float get(int c) const { return (float)v[c / 8][c % 8]; }
};
template <int CPT> struct Vec<float, CPT> {
    static constexpr int kRegs = CPT / 4;
    f32x4 v[kRegs];
    __device__ __forceinline__ void load(rsrc_t r, int off)
    {
#pragma unroll
        for (int i = 0; i < kRegs; ++i)
            v[i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, off + 16 * i, 0, 0));
    }
    __device__ __forceinline__ float get(int c) const { return v[c / 4][c % 4]; }
};
template <> struct Vec<float, 2> {              // narrow runs: the backward's lane-per-channel layouts
    float v[2];
    __device__ __forceinline__ void load(rsrc_t r, int off)
    {
        // two dword loads (the 64-bit raw buffer load builtin of this compiler fetches one dword only)
        v[0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0));
        v[1] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, off + 4, 0, 0));
    }
    __device__ __forceinline__ float get(int c) const { return v[c]; }
};
template <> struct Vec<float, 1> {
    float v;
    __device__ __forceinline__ void load(rsrc_t r, int off)
    {
        v = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0));
    }
    __device__ __forceinline__ float get(int) const { return v; }
};

template <int CPT>
__device__ __forceinline__ void store_run(rsrc_t r, int off, const float (&a)[CPT], _Float16 *)
{
#pragma unroll
    for (int i = 0; i < CPT / 8; ++i) {
        f16x8 h;
#pragma unroll
        for (int c = 0; c < 8; ++c)
            h[c] = (_Float16)a[8 * i + c];                 // round to nearest even, once
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, h), r, off + 16 * i, 0, 0);
    }
}
template <int CPT>
__device__ __forceinline__ void store_run(rsrc_t r, int off, const float (&a)[CPT], float *)
{
#pragma unroll
    for (int i = 0; i < CPT / 4; ++i) {
        f32x4 f = {a[4 * i], a[4 * i + 1], a[4 * i + 2], a[4 * i + 3]};
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, f), r, off + 16 * i, 0, 0);
    }
}

// One tap's sampling geometry: fractional parts, the byte offsets of the 4 neighbours inside
// the image's descriptor (kOutside where the column is outside; rows outside fall out of the
// descriptor's range by themselves) -- Eq. 1's x_g(p0 + p_k + dp_gk).
struct Tap {
    float lh, lw;
    int o00, o01, o10, o11;
};

// Byte offsets of the 4 neighbours of a sampling position given as whole-pixel window origin
// (base_h, base_w) plus the already scaled displacement (dy, dx).
__device__ __forceinline__ Tap tap_offsets(float dy, float dx, int base_h, int base_w, int chan_bytes, float dmax,
                                           int W, int row_bytes, int pix_bytes)
{
    // The whole-pixel part of the sampling position is kept in integers and only the scaled
    // offset goes through fp32, so the fractional parts carry no error from the magnitude of
    // the pixel coordinate.  Beyond +-dmax every neighbour is outside, so clamping changes nothing.
    dy = __builtin_fminf(__builtin_fmaxf(dy, -dmax), dmax);
    dx = __builtin_fminf(__builtin_fmaxf(dx, -dmax), dmax);
    const float fy = __builtin_floorf(dy), fx = __builtin_floorf(dx);
    Tap t;
    t.lh = dy - fy;
    t.lw = dx - fx;
    const int h0 = base_h + (int)fy, w0 = base_w + (int)fx;
    const int o = h0 * row_bytes + w0 * pix_bytes + chan_bytes;
    const bool in0 = (unsigned)w0 < (unsigned)W, in1 = (unsigned)(w0 + 1) < (unsigned)W;
    t.o00 = in0 ? o : kOutside;
    t.o10 = in0 ? o + row_bytes : kOutside;
    t.o01 = in1 ? o + pix_bytes : kOutside;
    t.o11 = in1 ? o + row_bytes + pix_bytes : kOutside;
    return t;
}

__device__ __forceinline__ Tap tap_geometry(float dY, float dX, int base_h, int base_w, int chan_bytes,
                                            const Geo &p)
{
    return tap_offsets(p.scale * dY, p.scale * dX, base_h, base_w, chan_bytes, p.dmax, p.W, p.row_bytes,
                       p.pix_bytes);
}

__device__ __forceinline__ int cvt_floor_i32(float v)
{
    int r;
    asm("v_cvt_flr_i32_f32 %0, %1" : "=v"(r) : "v"(v));       // floor, saturating, NaN -> 0
    return r;
}

__device__ __forceinline__ int cvt_round_i32(float v)      // floor(v + 0.5), saturating
{
    int r;
    asm("v_cvt_rpi_i32_f32 %0, %1" : "=v"(r) : "v"(v));
    return r;
}

__device__ __forceinline__ int med3i(int v, int lo, int hi)     // clamp to [lo, hi] in one instruction
{
    int r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
    return r;
}

// channel c of a 16-byte unit, widened to fp32
template <typename T> __device__ __forceinline__ float unit_get(const u32x4 &v, int c);
template <> __device__ __forceinline__ float unit_get<_Float16>(const u32x4 &v, int c)
{
    return (float)__builtin_bit_cast(f16x8, v)[c];
}
template <> __device__ __forceinline__ float unit_get<float>(const u32x4 &v, int c)
{
    return __builtin_bit_cast(f32x4, v)[c];
}

// store one 16-byte unit of results (8 fp16 or 4 fp32 values, one rounding to nearest even)
template <typename T> __device__ __forceinline__ void store_unit(rsrc_t r, int off, const float *a);
template <> __device__ __forceinline__ void store_unit<_Float16>(rsrc_t r, int off, const float *a)
{
    f16x8 h;
#pragma unroll
    for (int c = 0; c < 8; ++c)
        h[c] = (_Float16)a[c];
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, h), r, off, 0, 0);
}
template <> __device__ __forceinline__ void store_unit<float>(rsrc_t r, int off, const float *a)
{
    f32x4 f = {a[0], a[1], a[2], a[3]};
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, f), r, off, 0, 0);
}

// Shared per-thread decode: which (pixel, group, channel run) this thread serves.
struct Item {
    int n, pg0, npg;          // image, first (pixel,group) of the tile, pairs in the tile
    int pgl, sub;             // pair inside the tile, channel run inside the group
    int pix, g, oh, ow;
    bool active;
};

template <int TPG>
__device__ __forceinline__ Item decode_item(const Geo &p, int tile)
{
    constexpr int PGB = kThreads / TPG;
    Item it;
    it.n = fdiv(tile, p.div_tpi);
    it.pg0 = (tile - it.n * p.tiles_per_image) * PGB;
    it.npg = min(PGB, p.pgi - it.pg0);
    it.pgl = (int)threadIdx.x / TPG;
    it.sub = (int)threadIdx.x % TPG;
    it.active = it.pgl < it.npg;
    const int pg = it.pg0 + min(it.pgl, it.npg - 1);
    it.pix = fdiv(pg, p.div_g);
    it.g = pg - it.pix * p.G;
    it.oh = fdiv(it.pix, p.div_wo);
    it.ow = it.pix - it.oh * p.Wo;
    return it;
}

}  // namespace

// ------------------------------------------------------------------------------------------
// Forward (Eq. 1-2): thread = (output pixel, group, run of CPT channels).
// ------------------------------------------------------------------------------------------
template <typename T, int CG, int CPT, int KH = 3, int KW = 3>
__global__ __launch_bounds__(kThreads) void dcnv4_fwd_kernel(const T *__restrict__ x, const T *__restrict__ offset,
                                                             const T *__restrict__ mask, T *__restrict__ y, Geo p)
{
    constexpr int TPG = CG / CPT;
    constexpr int KT = KH * KW;                 // sampling points of the window
    constexpr int PGB = kThreads / TPG;
    constexpr int OFF_CAP = PGB * 2 * KT * (int)sizeof(T) + 16;
    constexpr int MSK_CAP = PGB * KT * (int)sizeof(T) + 16;
    __shared__ __attribute__((aligned(16))) char s_off[OFF_CAP];
    __shared__ __attribute__((aligned(16))) char s_msk[MSK_CAP];

    const int tile = tile_of_block(p);
    if (tile >= p.ntiles)
        return;
    const Item it = decode_item<TPG>(p, tile);

    const long long pg_first = (long long)it.n * p.pgi + it.pg0;
    const int d_off = stage_region<OFF_CAP, (int)sizeof(T)>(s_off, (const char *)offset, pg_first * (2 * KT * (int)sizeof(T)),
                                            it.npg * 2 * KT * (int)sizeof(T));
    const int d_msk = stage_region<MSK_CAP, (int)sizeof(T)>(s_msk, (const char *)mask, pg_first * (KT * (int)sizeof(T)),
                                            it.npg * KT * (int)sizeof(T));
    __syncthreads();
    if (!it.active)
        return;

    const T *my_off = reinterpret_cast<const T *>(s_off + d_off) + it.pgl * 2 * KT;
    const T *my_msk = reinterpret_cast<const T *>(s_msk + d_msk) + it.pgl * KT;
    const rsrc_t rx = make_rsrc((const char *)x + (long long)it.n * p.x_img_bytes, (unsigned)p.x_img_bytes);
    const int chan_bytes = (it.g * CG + it.sub * CPT) * (int)sizeof(T);
    const int bh = it.oh * p.sh - p.ph, bw = it.ow * p.sw - p.pw;

    float acc[CPT];
#pragma unroll
    for (int c = 0; c < CPT; ++c)
        acc[c] = 0.f;

#pragma unroll
    for (int j = 0; j < KW; ++j) {
#pragma unroll
        for (int i = 0; i < KH; ++i) {
            const int k = j * KH + i;
            const Tap t = tap_geometry((float)my_off[2 * k + 1], (float)my_off[2 * k], bh + i * p.dh, bw + j * p.dw,
                                       chan_bytes, p);
            Vec<T, CPT> v00, v01, v10, v11;
            v00.load(rx, t.o00);
            v01.load(rx, t.o01);
            v10.load(rx, t.o10);
            v11.load(rx, t.o11);
            const float m = (float)my_msk[k];
            const float mh0 = m * (1.f - t.lh), mh1 = m * t.lh;
            const float w00 = mh0 * (1.f - t.lw), w01 = mh0 * t.lw, w10 = mh1 * (1.f - t.lw), w11 = mh1 * t.lw;
#pragma unroll
            for (int c = 0; c < CPT; ++c) {
                float a = acc[c];
                a = __builtin_fmaf(v00.get(c), w00, a);
                a = __builtin_fmaf(v01.get(c), w01, a);
                a = __builtin_fmaf(v10.get(c), w10, a);
                a = __builtin_fmaf(v11.get(c), w11, a);
                acc[c] = a;
            }
        }
    }

    const rsrc_t ry = make_rsrc((char *)y + (long long)it.n * p.y_img_bytes, (unsigned)p.y_img_bytes);
    store_run<CPT>(ry, it.pix * p.pix_bytes + chan_bytes, acc, (T *)nullptr);
}

#include "dcnv4_tiled.inc"
#include "dcnv4_ring.inc"
#include "dcnv4_linear.inc"

// ------------------------------------------------------------------------------------------
// Backward (chain rule on Eq. 1), fp32, in one pass with grad_x added straight to memory; used
// where the LDS-staged kernels do not apply (groups wider than 16 channels, tiny images).  A group
// is spread over TPG lanes of CPT channels each -- by default one channel per lane, so that a
// wave's atomic instruction covers a few whole cache lines; the L2 atomic units then sustain about
// eight times the rate they reach when every lane adds to a line of its own.  The lanes' partial
// sums for grad_offset/grad_mask are combined with DPP exchanges inside a 16-lane row (plus one
// swizzle for 32 lanes).
// grad_offset / grad_mask leave through the same LDS tile the inputs came in by.
// ------------------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v)
{
    const int o = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false);
    return v + __builtin_bit_cast(float, o);
}

template <int TPG>
__device__ __forceinline__ float group_sum(float v)
{
    if (TPG >= 2) v = dpp_add<0xB1>(v);      // quad_perm [1,0,3,2]
    if (TPG >= 4) v = dpp_add<0x4E>(v);      // quad_perm [2,3,0,1]
    if (TPG >= 8) v = dpp_add<0x141>(v);     // row_half_mirror
    if (TPG >= 16) v = dpp_add<0x140>(v);    // row_mirror
    if (TPG >= 32)                           // the other 16-lane row of the 32-lane half: swizzle, lane ^ 16
        v += __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F));
    return v;
}

template <int CG, int CPT, int KH = 3, int KW = 3>
__global__ __launch_bounds__(kThreads) void dcnv4_bwd_kernel(const float *__restrict__ x,
                                                             const float *__restrict__ offset,
                                                             const float *__restrict__ mask,
                                                             const float *__restrict__ grad_y,
                                                             float *__restrict__ grad_x,
                                                             float *__restrict__ grad_offset,
                                                             float *__restrict__ grad_mask, Geo p)
{
    typedef float T;
    constexpr int TPG = CG / CPT;
    constexpr int KT = KH * KW;
    constexpr int PGB = kThreads / TPG;
    constexpr int OFF_CAP = PGB * 2 * KT * (int)sizeof(T) + 16;
    constexpr int MSK_CAP = PGB * KT * (int)sizeof(T) + 16;
    __shared__ __attribute__((aligned(16))) char s_off[OFF_CAP];
    __shared__ __attribute__((aligned(16))) char s_msk[MSK_CAP];

    const int tile = tile_of_block(p);
    if (tile >= p.ntiles)
        return;
    const Item it = decode_item<TPG>(p, tile);

    const long long pg_first = (long long)it.n * p.pgi + it.pg0;
    const int d_off = stage_region<OFF_CAP, (int)sizeof(T)>(s_off, (const char *)offset, pg_first * (2 * KT * (int)sizeof(T)),
                                            it.npg * 2 * KT * (int)sizeof(T));
    const int d_msk = stage_region<MSK_CAP, (int)sizeof(T)>(s_msk, (const char *)mask, pg_first * (KT * (int)sizeof(T)),
                                            it.npg * KT * (int)sizeof(T));
    __syncthreads();

    T *tile_off = reinterpret_cast<T *>(s_off + d_off);
    T *tile_msk = reinterpret_cast<T *>(s_msk + d_msk);
    if (it.active) {
        T *my_off = tile_off + it.pgl * 2 * KT;
        T *my_msk = tile_msk + it.pgl * KT;
        const rsrc_t rx = make_rsrc((const char *)x + (long long)it.n * p.x_img_bytes, (unsigned)p.x_img_bytes);
        const rsrc_t rgx = make_rsrc((char *)grad_x + (long long)it.n * p.x_img_bytes, (unsigned)p.x_img_bytes);
        const rsrc_t rgy =
            make_rsrc((const char *)grad_y + (long long)it.n * p.y_img_bytes, (unsigned)p.y_img_bytes);
        const int chan_bytes = (it.g * CG + it.sub * CPT) * (int)sizeof(T);
        const int bh = it.oh * p.sh - p.ph, bw = it.ow * p.sw - p.pw;

        Vec<T, CPT> gy;
        gy.load(rgy, it.pix * p.pix_bytes + chan_bytes);

#pragma unroll
        for (int j = 0; j < KW; ++j) {
#pragma unroll
            for (int i = 0; i < KH; ++i) {
                const int k = j * KH + i;
                const Tap t = tap_geometry(my_off[2 * k + 1], my_off[2 * k], bh + i * p.dh, bw + j * p.dw,
                                           chan_bytes, p);
                Vec<T, CPT> v00, v01, v10, v11;
                v00.load(rx, t.o00);
                v01.load(rx, t.o01);
                v10.load(rx, t.o10);
                v11.load(rx, t.o11);
                const float m = my_msk[k];
                const float hh = 1.f - t.lh, hw = 1.f - t.lw;
                // grad_x: m * corner weight * gy, dropped by the descriptor where the corner is outside
                const float w00 = m * hh * hw, w01 = m * hh * t.lw, w10 = m * t.lh * hw, w11 = m * t.lh * t.lw;
                float d00 = 0.f, d01 = 0.f, d10 = 0.f, d11 = 0.f;
#pragma unroll
                for (int c = 0; c < CPT; ++c) {
                    const float g = gy.get(c);
                    d00 = __builtin_fmaf(g, v00.get(c), d00);
                    d01 = __builtin_fmaf(g, v01.get(c), d01);
                    d10 = __builtin_fmaf(g, v10.get(c), d10);
                    d11 = __builtin_fmaf(g, v11.get(c), d11);
                    __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_f32(w00 * g, rgx, t.o00 + 4 * c, 0, 0);
                    __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_f32(w01 * g, rgx, t.o01 + 4 * c, 0, 0);
                    __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_f32(w10 * g, rgx, t.o10 + 4 * c, 0, 0);
                    __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_f32(w11 * g, rgx, t.o11 + 4 * c, 0, 0);
                }
                d00 = group_sum<TPG>(d00);
                d01 = group_sum<TPG>(d01);
                d10 = group_sum<TPG>(d10);
                d11 = group_sum<TPG>(d11);
                // grad_mask = sum_c gy*S;  grad_offset = scale * m * sum_c gy * dS/d(wx, hy)
                const float gm = hh * (hw * d00 + t.lw * d01) + t.lh * (hw * d10 + t.lw * d11);
                const float gdy = p.scale * m * (hw * (d10 - d00) + t.lw * (d11 - d01));
                const float gdx = p.scale * m * (hh * (d01 - d00) + t.lh * (d11 - d10));
                if (it.sub == 0) {                       // after every lane of the pair has read tap k
                    my_off[2 * k] = gdx;
                    my_off[2 * k + 1] = gdy;
                    my_msk[k] = gm;
                }
            }
        }
    }
    __syncthreads();
    float *go = grad_offset + pg_first * (2 * KT);
    float *gm = grad_mask + pg_first * KT;
    for (int e = threadIdx.x; e < it.npg * 2 * KT; e += kThreads)
        go[e] = tile_off[e];
    for (int e = threadIdx.x; e < it.npg * KT; e += kThreads)
        gm[e] = tile_msk[e];
}

// Zero-fill of `bytes` bytes (a multiple of 4) at a 16-byte aligned address: 128-bit stores, then the
// last few dwords one by one.  A kernel rather than a memset node, so that a call can be captured
// into a graph.
__global__ __launch_bounds__(kThreads) void dcnv4_zero_kernel(u32x4 *__restrict__ dst, long long bytes)
{
    const long long n16 = bytes / 16;
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < n16; i += (long long)gridDim.x * kThreads)
        dst[i] = z;
    const int tail = (int)((bytes - n16 * 16) / 4);
    if (blockIdx.x == 0 && (int)threadIdx.x < tail)
        reinterpret_cast<unsigned *>(dst + n16)[threadIdx.x] = 0u;
}

// ------------------------------------------------------------------------------------------
// Host side: validation, launch geometry, dispatch.
// ------------------------------------------------------------------------------------------
namespace {

// Test and benchmark switches (dcnv4_set_option): they force a path or a tile shape so that every
// kernel can be checked on every shape; 0 = the library's own choice.  Not meant for applications.
struct Options {
    int fwd_path = 0;      // 1 direct global gather, 2 rectangle staged in LDS, 3 ring of record rows in LDS
    int bwd_path = 0;      // 1 direct (global atomics), 2 LDS-staged (two passes)
    int fwd_cpt = 0;       // channels per lane of the direct forward (8 or 16)
    int bwd_cpt = 0;       // channels per lane of the direct backward (1, 2, 4, 8, 16)
    int xcd_remap = 1;     // consecutive tiles go to one XCD (0: plain block order)
    int halo = 0;          // displacement in pixels (rows, for the ring) the staged window allows for
    int lds_kb = 0;        // LDS budget per workgroup of the staged kernels (8..160)
    int fwd_threads = 0;   // workgroup size of the staged forward kernels (64, 128, 256, 512, 640, 768)
    int wg_per_cu = 0;     // persistent workgroups per compute unit of the rectangle kernels (1..32)
    int fwd_single = 0;    // rectangle buffers of the staged gather kernels: 1 always two, 2 always one
    int gx_threads = 0;    // workgroup size of the grad_x kernel (256, 512, 768)
    int gom_coop = 0;      // 1: the fp32 grad_offset/grad_mask pass goes through LDS slices even for whole groups
    int module_rows = 0;   // 1: the module keeps its tensors channel-last between the layers (default: plane-major)
} g_opt;

char g_last_kernel[2][96];

FastDiv make_div(unsigned d)
{
    unsigned s = 0;
    while ((1ull << s) < d)
        ++s;
    FastDiv f;
    f.shift = s;
    f.mul = (unsigned)(((1ull << 32) * ((1ull << s) - d)) / d + 1);
    return f;
}

int esize(int dtype) { return dtype == DCNV4_F16 ? 2 : 4; }

struct Problem {
    int N, H, W, G, Cg, Ho, Wo;
    int kh, kw;     // window: 3x3 everywhere; 1x1 and 5x5 through the direct kernels only
    int sh, sw, ph, pw, dh, dw;
    float scale;
    int dtype;
    int merged;     // offsets and mask values share one buffer of 32 values per (pixel, group)
    int softmax;    // the mask tensor holds logits, normalised over the 9 taps inside the kernels
};

int validate(const Problem &q, int kh, int kw, const void *const *ptrs, int nptrs)
{
    for (int i = 0; i < nptrs; ++i)
        if (!ptrs[i])
            return DCNV4_ERR_NULL;
    if (q.N < 1 || q.H < 1 || q.W < 1 || q.G < 1 || q.Cg < 1 || kh < 1 || kw < 1 || q.sh < 1 || q.sw < 1 ||
        q.ph < 0 || q.pw < 0 || q.dh < 1 || q.dw < 1)
        return DCNV4_ERR_SHAPE;
    if (q.Ho < 1 || q.Wo < 1)
        return DCNV4_ERR_SHAPE;
    if (kh != kw || (kh != 1 && kh != 3 && kh != 5))
        return DCNV4_ERR_UNSUPPORTED;
    if (q.dtype != DCNV4_F32 && q.dtype != DCNV4_F16)
        return DCNV4_ERR_UNSUPPORTED;
    if (q.Cg != 8 && q.Cg != 16 && q.Cg != 32 && q.Cg != 64)
        return DCNV4_ERR_UNSUPPORTED;
    if (!(q.scale == q.scale) || q.scale > 3.0e38f || q.scale < -3.0e38f)
        return DCNV4_ERR_UNSUPPORTED;
    for (int i = 0; i < nptrs; ++i)
        if (reinterpret_cast<uintptr_t>(ptrs[i]) & 15u)
            return DCNV4_ERR_ALIGN;
    return DCNV4_OK;
}

// Fills the kernel's geometry block; returns DCNV4_ERR_UNSUPPORTED when 32-bit byte offsets
// inside one image could overflow.
int make_geo(const Problem &q, int tpg, Geo *out)
{
    Geo p;
    memset(&p, 0, sizeof(p));
    const long long es = esize(q.dtype), C = (long long)q.G * q.Cg;
    p.H = q.H; p.W = q.W; p.Ho = q.Ho; p.Wo = q.Wo; p.G = q.G;
    p.sh = q.sh; p.sw = q.sw; p.ph = q.ph; p.pw = q.pw; p.dh = q.dh; p.dw = q.dw;
    p.scale = q.scale;
    // window origin of any tap lies in [-pad, (out-1)*stride - pad + (k-1)*dil]
    const long long bh = (long long)(q.Ho - 1) * q.sh + (long long)(q.kh - 1) * q.dh + q.ph;
    const long long bw = (long long)(q.Wo - 1) * q.sw + (long long)(q.kw - 1) * q.dw + q.pw;
    const long long reach = (q.H > q.W ? q.H : q.W) + (bh > bw ? bh : bw) + 4;
    if (reach >= (1 << 22))
        return DCNV4_ERR_UNSUPPORTED;
    p.dmax = (float)reach;
    // |row| <= 2*reach+1, |col| <= 2*reach+1 after clamping: the byte offset must fit in int32
    const long long worst = (2 * reach + 2) * ((long long)q.W + 1) * C * es + (2 * reach + 2) * C * es;
    const long long ximg = (long long)q.H * q.W * C * es, yimg = (long long)q.Ho * q.Wo * C * es;
    if (worst >= (1LL << 31) || ximg >= (1LL << 31) || yimg >= (1LL << 31))
        return DCNV4_ERR_UNSUPPORTED;
    const long long pgi = (long long)q.Ho * q.Wo * q.G;
    const int pgb = kThreads / tpg;
    const long long tpi = (pgi + pgb - 1) / pgb;
    const long long ntiles = tpi * q.N;
    if (pgi >= (1LL << 31) || ntiles >= (1LL << 30))
        return DCNV4_ERR_UNSUPPORTED;
    p.pgi = (int)pgi;
    p.tiles_per_image = (int)tpi;
    p.ntiles = (int)ntiles;
    p.tiles_per_xcd = (int)((ntiles + kXcds - 1) / kXcds);
    p.remap = g_opt.xcd_remap;
    p.div_g = make_div((unsigned)q.G);
    p.div_wo = make_div((unsigned)q.Wo);
    p.div_tpi = make_div((unsigned)tpi);
    p.x_img_bytes = (int)ximg;
    p.y_img_bytes = (int)yimg;
    p.row_bytes = (int)(q.W * C * es);
    p.pix_bytes = (int)(C * es);
    *out = p;
    return DCNV4_OK;
}

unsigned grid_of(const Geo &p) { return (unsigned)(p.remap ? p.tiles_per_xcd * kXcds : p.ntiles); }

// Eight channels per lane in the direct forward: 16-byte (fp16) or 32-byte (fp32) runs, so that
// neighbouring lanes share cache lines.
constexpr int kDefaultFwdCpt = 8;
// One or two channels per lane: a wave's atomic instruction then covers a few whole cache lines
// (16 lanes x 4 or 8 bytes per pixel) instead of 64 different ones, and the L2 atomic rate follows.
int default_bwd_cpt(int Cg) { return Cg <= 32 ? 1 : Cg / 32; }

int pick_fwd_cpt(int Cg)
{
    int c = g_opt.fwd_cpt ? g_opt.fwd_cpt : kDefaultFwdCpt;
    if (c > Cg) c = Cg;
    if (Cg / c > 8) c = Cg / 8;        // at most 8 lanes per group
    return c;
}
int pick_bwd_cpt(int Cg)
{
    int c = g_opt.bwd_cpt ? g_opt.bwd_cpt : default_bwd_cpt(Cg);
    if (c > Cg) c = Cg;
    if (Cg / c > 32) c = Cg / 32;      // the lane reduction spans at most two 16-lane rows
    return c;
}

template <typename T, int CG, int CPT, int KS = 3>
int launch_fwd(const void *x, const void *off, const void *msk, void *y, const Problem &q, hipStream_t s)
{
    Geo p;
    int rc = make_geo(q, CG / CPT, &p);
    if (rc)
        return rc;
    hipLaunchKernelGGL((dcnv4_fwd_kernel<T, CG, CPT, KS, KS>), dim3(grid_of(p)), dim3(kThreads), 0, s, (const T *)x,
                       (const T *)off, (const T *)msk, (T *)y, p);
    if (KS == 3)
        snprintf(g_last_kernel[0], sizeof(g_last_kernel[0]), "dcnv4_fwd_kernel<%s, %d, %d>",
                 sizeof(T) == 2 ? "_Float16" : "float", CG, CPT);
    else
        snprintf(g_last_kernel[0], sizeof(g_last_kernel[0]), "dcnv4_fwd_kernel<%s, %d, %d, %d, %d>",
                 sizeof(T) == 2 ? "_Float16" : "float", CG, CPT, KS, KS);
    return hipGetLastError() == hipSuccess ? DCNV4_OK : DCNV4_ERR_LAUNCH;
}

// Windows other than 3x3 (1x1, 5x5): the direct kernel, eight channels per lane.  A 5x5 window keeps
// 75 values per (pixel, group) in the kernel's static LDS tiles, which fit for groups of 16 channels
// or more (128 pairs per workgroup).
template <typename T, int KS>
int dispatch_fwd_window(const void *x, const void *off, const void *msk, void *y, const Problem &q, hipStream_t s)
{
    switch (q.Cg) {
    case 8:
        if constexpr (KS <= 3)
            return launch_fwd<T, 8, 8, KS>(x, off, msk, y, q, s);
        return DCNV4_ERR_UNSUPPORTED;
    case 16: return launch_fwd<T, 16, 8, KS>(x, off, msk, y, q, s);
    case 32: return launch_fwd<T, 32, 8, KS>(x, off, msk, y, q, s);
    case 64: return launch_fwd<T, 64, 8, KS>(x, off, msk, y, q, s);
    }
    return DCNV4_ERR_UNSUPPORTED;
}

template <typename T, int CG>
int dispatch_fwd_cpt(int cpt, const void *x, const void *off, const void *msk, void *y, const Problem &q,
                     hipStream_t s)
{
    if constexpr (CG >= 16) {
        if (cpt == 16) return launch_fwd<T, CG, 16>(x, off, msk, y, q, s);
    }
    if constexpr (CG <= 64) {
        if (cpt == 8) return launch_fwd<T, CG, 8>(x, off, msk, y, q, s);
    }
    return DCNV4_ERR_UNSUPPORTED;
}


// (pitch + 2) staged pixels of zeros follow the slices; the chooser reserves room for the widest pitch
constexpr int kTiledZeroPixelsExtra = 2;
constexpr int kDefaultHalo = 6;
constexpr int kDefaultHaloGradX = 4;
constexpr int kDefaultLdsKb = 158;
constexpr int kMaxLdsBytes = 160 * 1024;

// Tile choice for the LDS-staged forward: full-width row bands when a band with a useful
// number of rows fits the LDS budget, otherwise split the columns too.  Returns false when
// no tile with at least as many output rows/cols as the halo fits (the rectangle would be
// mostly halo); the caller then uses the direct kernel.
// Per-device caches (compute-unit count, dynamic-LDS grants) are indexed by the HIP device number.
constexpr int kMaxDevices = 64;
int current_device()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return -1;
    return dev;
}

// Number of compute units of the current device (persistent kernels launch one workgroup each).
int device_cus()
{
    static int cus[kMaxDevices];
    const int dev = current_device();
    if (dev < 0)
        return 0;
    if (cus[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < kXcds)
            return 0;
        cus[dev] = n;
    }
    return cus[dev];
}

// Lets `kern` use `lds` bytes of dynamic LDS on the current device (asked for once per device and size).
bool grant_lds(const void *kern, int lds, int (&granted)[kMaxDevices])
{
    if (lds <= 64 * 1024)
        return true;
    const int dev = current_device();
    if (dev < 0)
        return false;
    if (lds > granted[dev]) {
        if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
            return false;
        granted[dev] = lds;
    }
    return true;
}

bool choose_tile(const Problem &q, int threads, int halo, int lds_bytes, int nbuf, int pb, bool accum, bool with_slices,
                 int chan_slices, TGeo *out, double *cost_out = nullptr)
{
    const int es = esize(q.dtype);
    // per-wave LDS slices for the 27 offset/mask values of 64 pixels (grad_offset/grad_mask pass only)
    const int slices = with_slices ? (threads / 64) * 64 * 27 * es : 0;
    const int need = halo > 4 ? halo : 4;
    const int waves = threads / 64;
    int cus = device_cus();
    if (cus <= 0) cus = 256;                 // no device in this process (host-only checks): assume a full MI355X
    // Cost of a candidate (column splits kq, band height R), in units of one round (= every wave
    // of a workgroup doing one batch of 64 output pixels): a tile of B batches takes ceil(B / waves)
    // rounds plus about four for the switch (barrier, drained pipeline; measured; six with a single
    // buffer, whose refill is not hidden), and a workgroup
    // works through ceil(tiles / CUs) tiles -- so few, huge tiles that leave CUs idle lose against
    // more, smaller ones.
    double best_cost = 1e30;
    bool found = false;
    int splits_tried = 0;
    for (int kq = 1; kq <= q.Wo && splits_tried < 12; ++kq) {
        const int Q = (q.Wo + kq - 1) / kq;
        if (kq > 1 && Q == (q.Wo + kq - 2) / (kq - 1))
            continue;                        // same tile width as the previous split count
        long long cols = (long long)(Q - 1) * q.sw + 2LL * q.dw + 2LL * halo + 2;
        if (cols > q.W + 4) cols = q.W + 4;
        // the rectangle buffers (each a multiple of 1 KiB) share what the slices leave, after
        // a block of zeros (pitch + 2 pixels) or one more dword per rectangle pixel (the bound words of the grad_x accumulator)
        const long long zero_bytes = accum ? 16 : ((cols + kTiledZeroPixelsExtra) * pb + 15) & ~15LL;
        const long long budget_px =
            ((((long long)lds_bytes - slices - zero_bytes) * pb / (pb + (accum ? 4 : 0)) / nbuf) & ~1023LL) / pb;
        if (budget_px < 64)
            continue;
        const long long rows_max = budget_px / cols;
        long long Rmax = (rows_max - 2LL * q.dh - 2LL * halo - 2) / q.sh + 1;
        if (rows_max >= q.H + 4) Rmax = q.Ho;               // the whole (clipped) height fits
        if (Rmax > q.Ho) Rmax = q.Ho;
        if (Rmax < 1 || (Rmax < need && Rmax < q.Ho) || (Q < need && Q < q.Wo))
            continue;
        ++splits_tried;
        const int tiles_q = (q.Wo + Q - 1) / Q;
        const long long Rlow = Rmax < need ? Rmax : need;
        for (long long R = Rmax; R >= Rlow; --R) {
            const long long bands = (q.Ho + R - 1) / R, Rlast = q.Ho - (bands - 1) * R;
            const long long b_full = (R * Q + 63) / 64, b_last = (Rlast * Q + 63) / 64;
            const double rounds_img = tiles_q * ((bands - 1) * (double)((b_full + waves - 1) / waves) +
                                                 (double)((b_last + waves - 1) / waves) + (nbuf == 1 && !accum ? 6.0 : 4.0) * bands);
            const long long tiles = (long long)q.N * q.G * chan_slices * bands * tiles_q;
            const double per_tile = rounds_img / (double)(bands * tiles_q);
            const double cost = (double)((tiles + cus - 1) / cus) * per_tile;
            if (cost < best_cost - 1e-9) {
                best_cost = cost;
                found = true;
                long long rows = (R - 1) * q.sh + 2LL * q.dh + 2LL * halo + 2;
                if (rows > q.H + 4) rows = q.H + 4;
                out->R = (int)R;
                out->Q = Q;
                out->halo = halo;
                out->pitch = (int)cols;
                out->tiles_q = tiles_q;
                out->tiles_per_img = (int)(bands * tiles_q);
                out->xtile_bytes = (int)((rows * cols * pb + 1023) & ~1023LL);
            }
        }
    }
    if (cost_out)
        *cost_out = best_cost;
    return found;
}

// `mode`: kTiledGradX has a single LDS rectangle of Cg + 1 dwords per pixel (fixed-point sums and a bound word);
// kTiledGradOM additionally keeps per-wave slices for the offset/mask values.
int make_tgeo(const Problem &q, int threads, int mode, TGeo *out, int cg_kernel = 0, int want_nbuf = 0)
{
    const bool gradx = mode == kTiledGradX, with_slices = mode == kTiledGradOM;
    // a group wider than the kernel's channel run is cut into slices that are tiles of their own
    const int cgk = cg_kernel ? cg_kernel : q.Cg;
    // (the grad_offset/grad_mask pass can combine slices only in fp32, where it adds them up atomically)
    if (q.Cg % cgk != 0 || (with_slices && cgk != q.Cg && q.dtype != DCNV4_F32))
        return DCNV4_ERR_UNSUPPORTED;
    const int chan_slices = q.Cg / cgk;
    Geo base;
    int rc = make_geo(q, 1, &base);          // shares the 32-bit offset validation
    if (rc)
        return rc;
    TGeo p;
    memset(&p, 0, sizeof(p));
    // the grad_x kernel sends far samples straight to memory without waiting for them, so it can
    // afford a tighter rectangle (taller tiles, fewer flushes)
    const int halo = g_opt.halo ? g_opt.halo : (gradx ? kDefaultHaloGradX : kDefaultHalo);
    int lds = (g_opt.lds_kb ? g_opt.lds_kb : kDefaultLdsKb) * 1024;
    if (lds > kMaxLdsBytes) lds = kMaxLdsBytes;
    const int pb = cgk * esize(q.dtype);
    if (gradx) {
        if (!choose_tile(q, threads, halo, lds, 1, cgk * 4, true, false, chan_slices, &p))
            return DCNV4_ERR_UNSUPPORTED;
        p.nbuf = 1;
    } else {
        // Two buffers overlap the copy of the next tile with the work on this one; one buffer holds a
        // rectangle twice as big (taller bands, fewer tile switches, less halo).  Take the cheaper one
        // by the chooser's own estimate.
        TGeo one;
        memset(&one, 0, sizeof(one));
        double cost2 = 0, cost1 = 0;
        const int pick = g_opt.fwd_single ? g_opt.fwd_single : want_nbuf == 1 ? 2 : want_nbuf == 2 ? 1 : 0;
        const bool ok2 = pick != 2 && choose_tile(q, threads, halo, lds, 2, pb, false, with_slices, chan_slices, &p, &cost2);
        const bool ok1 = pick != 1 && choose_tile(q, threads, halo, lds, 1, pb, false, with_slices, chan_slices, &one, &cost1);
        if (!ok2 && !ok1)
            return DCNV4_ERR_UNSUPPORTED;
        if (!ok2 || (ok1 && cost1 < cost2)) {
            p = one;
            p.nbuf = 1;
        } else {
            p.nbuf = 2;
        }
    }
    const long long es = esize(q.dtype);
    const long long pgi = (long long)q.Ho * q.Wo * q.G;
    if (pgi >= 0x1000000)                    // offset/mask byte offsets inside one image stay in int32
        return DCNV4_ERR_UNSUPPORTED;
    p.H = q.H; p.W = q.W; p.Ho = q.Ho; p.Wo = q.Wo; p.G = q.G;
    p.sh = q.sh; p.sw = q.sw; p.ph = q.ph; p.pw = q.pw; p.dh = q.dh; p.dw = q.dw;
    p.scale = q.scale;
    p.dmax = base.dmax;
    const long long nblocks = (long long)q.N * p.tiles_per_img * q.G * chan_slices;
    if (nblocks >= (1LL << 30))
        return DCNV4_ERR_UNSUPPORTED;
    p.nblocks = (int)nblocks;
    p.blocks_per_xcd = (int)((nblocks + kXcds - 1) / kXcds);
    p.remap = g_opt.xcd_remap;
    p.blocked = 0;                          // (contiguous runs per wave leave waves without work when a tile has few batches)
    p.div_g = make_div((unsigned)q.G);
    p.div_s = make_div((unsigned)chan_slices);
    p.slices = chan_slices;
    p.group_bytes = q.Cg * esize(q.dtype);
    p.div_tpi = make_div((unsigned)p.tiles_per_img);
    p.div_tq = make_div((unsigned)p.tiles_q);
    p.div_q = make_div((unsigned)p.Q);
    p.div_pitch = make_div((unsigned)p.pitch);
    p.x_img_bytes = base.x_img_bytes;
    p.y_img_bytes = base.y_img_bytes;
    p.row_bytes = base.row_bytes;
    p.pix_bytes = base.pix_bytes;
    p.softmax = q.softmax;
    p.og_bytes = (int)((q.merged ? 32 : 18) * es);
    p.mg_bytes = (int)((q.merged ? 32 : 9) * es);
    // (idle lanes point at (pixel, group) number 2^24 of the image, which has to lie past its end)
    if (pgi * p.og_bytes >= (1LL << 31) || pgi >= (1LL << 24))
        return DCNV4_ERR_UNSUPPORTED;
    p.off_img_bytes = (int)(pgi * p.og_bytes);
    p.msk_img_bytes = (int)(pgi * p.mg_bytes);
    p.off_ext_bytes = (int)((pgi - 1) * p.og_bytes + 18 * es);
    p.msk_ext_bytes = (int)((pgi - 1) * p.mg_bytes + 9 * es);
    *out = p;
    return DCNV4_OK;
}

// A launch of the LDS-staged kernel in one of its modes, in two steps: prepare_tiled does everything
// that can refuse (tile choice, LDS size, LDS grant, device query) and launches nothing; run_tiled
// launches what was prepared.  `which` = 0 forward, 1 backward (for the kernel-name record).
struct TiledLaunch {
    TGeo p;
    int lds;
    unsigned grid;
};

template <typename T, int CG, int THREADS, int MODE>
int prepare_tiled(const Problem &q, bool any_tile_size, int want_nbuf, int want_per_cu, TiledLaunch *out)
{
    TGeo p;
    constexpr bool kGradX = MODE == kTiledGradX;
    int rc = make_tgeo(q, THREADS, MODE, &p, CG, want_nbuf);
    if (rc)
        return rc;
    // a tile of one or two 64-pixel batches leaves most of the workgroup's waves idle and pays the
    // tile switch for almost no work: such images are left to the direct kernel unless forced
    if (!any_tile_size && p.R * p.Q < 128)
        return DCNV4_ERR_UNSUPPORTED;
    const int px_bytes = kGradX ? CG * 4 : CG * (int)sizeof(T);
    const int tail = kGradX ? (p.xtile_bytes / px_bytes) * 4 + 16 : ((p.pitch + kTiledZeroPixelsExtra) * px_bytes + 15) & ~15;
    const int slices = MODE == kTiledGradOM ? (THREADS / 64) * 64 * 27 * (int)sizeof(T) : 0;     // (not kTiledGradOMDirect)
    const int lds = p.nbuf * p.xtile_bytes + slices + tail;
    if (lds > kMaxLdsBytes)
        return DCNV4_ERR_UNSUPPORTED;
    static int granted[kMaxDevices];         // largest dynamic-LDS size already requested for this kernel, per device
    if (!grant_lds(reinterpret_cast<const void *>(dcnv4_tiled_kernel<T, CG, THREADS, MODE>), lds, granted))
        return DCNV4_ERR_LAUNCH;
    // persistent workgroups: one per compute unit (or fewer when there are fewer tiles)
    const int cus = device_cus();
    if (cus <= 0)
        return DCNV4_ERR_LAUNCH;
    // several persistent workgroups per compute unit when their LDS and registers fit: their tile
    // switches (barrier, drained pipeline) then overlap with each other's work
    int per_cu = g_opt.wg_per_cu ? g_opt.wg_per_cu : want_per_cu ? want_per_cu : (MODE != kTiledFwd || CG * sizeof(T) >= 64 ? 1 : THREADS == 256 ? 2 : THREADS == 64 ? 16 : 1);
    while (per_cu > 1 && (per_cu * lds > kMaxLdsBytes || per_cu * THREADS > 2048))
        --per_cu;
    const int slots = cus * per_cu;
    unsigned grid;
    if (p.remap) {
        const int per = slots / kXcds < p.blocks_per_xcd ? slots / kXcds : p.blocks_per_xcd;
        grid = (unsigned)(per * kXcds);
    } else {
        grid = (unsigned)(slots < p.nblocks ? slots : p.nblocks);
    }
    out->p = p;
    out->lds = lds;
    out->grid = grid;
    return DCNV4_OK;
}

template <typename T, int CG, int THREADS, int MODE>
int run_tiled(const TiledLaunch &l, const void *x, const void *off, const void *msk, const void *gy, void *o1, void *o2,
              hipStream_t s, int which)
{
    hipLaunchKernelGGL((dcnv4_tiled_kernel<T, CG, THREADS, MODE>), dim3(l.grid), dim3(THREADS), l.lds, s, (const T *)x,
                       (const T *)off, (const T *)msk, (const T *)gy, (T *)o1, (T *)o2, l.p);
    snprintf(g_last_kernel[which], sizeof(g_last_kernel[which]), "dcnv4_tiled_kernel<%s, %d, %d, %d>",
             sizeof(T) == 2 ? "_Float16" : "float", CG, THREADS, MODE);
    return hipGetLastError() == hipSuccess ? DCNV4_OK : DCNV4_ERR_LAUNCH;
}

template <typename T, int CG, int THREADS, int MODE>
int launch_tiled(const void *x, const void *off, const void *msk, const void *gy, void *o1, void *o2,
                 const Problem &q, hipStream_t s, int which, bool any_tile_size, int want_nbuf = 0, int want_per_cu = 0)
{
    TiledLaunch l;
    const int rc = prepare_tiled<T, CG, THREADS, MODE>(q, any_tile_size, want_nbuf, want_per_cu, &l);
    if (rc)
        return rc;
    return run_tiled<T, CG, THREADS, MODE>(l, x, off, msk, gy, o1, o2, s, which);
}

template <typename T, int CG, int THREADS>
int launch_fwd_tiled(const void *x, const void *off, const void *msk, void *y, const Problem &q, hipStream_t s)
{
    return launch_tiled<T, CG, THREADS, kTiledFwd>(x, off, msk, nullptr, y, nullptr, q, s, 0, g_opt.fwd_path == 2 || q.merged || q.softmax);
}

// The tiled kernel keeps Cg fp32 accumulators and 4*Cg input values per lane, so it is built
// for staged pixels of up to 64 bytes.
template <typename T, int CG>
int dispatch_fwd_tiled(const void *x, const void *off, const void *msk, void *y, const Problem &q, hipStream_t s)
{
    if constexpr (CG * sizeof(T) <= 64 && CG * sizeof(T) >= 16) {
        if constexpr (CG * sizeof(T) == 64) {
            // 64-byte pixels: eight waves still fit the register file (no LDS slices, no exchange registers)
            if (g_opt.fwd_threads == 256)
                return launch_fwd_tiled<T, CG, 256>(x, off, msk, y, q, s);
            return launch_fwd_tiled<T, CG, 512>(x, off, msk, y, q, s);
        }
        if (g_opt.fwd_threads == 256)
            return launch_fwd_tiled<T, CG, 256>(x, off, msk, y, q, s);
        if constexpr (CG * sizeof(T) < 64) {
            // Small whole-image tiles: several four-wave workgroups per compute unit, whose tile
            // switches overlap with each other's work, beat one big workgroup.
            if (g_opt.fwd_threads == 64)
                return launch_fwd_tiled<T, CG, 64>(x, off, msk, y, q, s);
            if (g_opt.fwd_threads == 128)
                return launch_fwd_tiled<T, CG, 128>(x, off, msk, y, q, s);
            if (g_opt.fwd_threads == 768)
                return launch_fwd_tiled<T, CG, 768>(x, off, msk, y, q, s);
            if (g_opt.fwd_threads == 0 && g_opt.fwd_path != 1) {
                // An image of one or two batches: one-wave workgroups, eight to a compute unit, so that
                // no wave idles while another works (beats the direct kernel on 7x7 maps).
                TGeo tiny;
                if (make_tgeo(q, 64, kTiledFwd, &tiny, CG) == DCNV4_OK && tiny.tiles_per_img == 1 && tiny.R * tiny.Q <= 128)
                    return launch_tiled<T, CG, 64, kTiledFwd>(x, off, msk, nullptr, y, nullptr, q, s, 0, true);
            }
            if (g_opt.fwd_threads == 0) {
                TGeo probe;
                // (one rectangle buffer each: with several workgroups on the unit, one computes while
                // another refills, and the halved LDS lets three of them in)
                if (make_tgeo(q, 256, kTiledFwd, &probe, CG, 1) == DCNV4_OK && probe.tiles_per_img == 1 &&
                    probe.R * probe.Q <= 16 * 64)
                    return launch_tiled<T, CG, 256, kTiledFwd>(x, off, msk, nullptr, y, nullptr, q, s, 0,
                                                               g_opt.fwd_path == 2 || q.merged || q.softmax, 1, 3);
            }
            if (g_opt.fwd_threads == 512)
                return launch_fwd_tiled<T, CG, 512>(x, off, msk, y, q, s);
            // pixels of up to 32 bytes leave room for twelve waves in the register file (measured: 2-5 %
            // over eight)
            return launch_fwd_tiled<T, CG, 768>(x, off, msk, y, q, s);
        } else {
            return DCNV4_ERR_UNSUPPORTED;
        }
    }
    return DCNV4_ERR_UNSUPPORTED;
}

template <typename T>
int dispatch_fwd_tiled_cg(const void *x, const void *off, const void *msk, void *y, const Problem &q, hipStream_t s)
{
    constexpr int kWidest = 64 / (int)sizeof(T);     // channels of a 64-byte pixel: the widest run a lane keeps
    switch (q.Cg) {
    case 8: return dispatch_fwd_tiled<T, 8>(x, off, msk, y, q, s);
    case 16: return dispatch_fwd_tiled<T, 16>(x, off, msk, y, q, s);
    case 32:
    case 64:
        // wider groups go through in slices of 64 bytes (same offsets and mask, own channels)
        if (q.Cg <= kWidest)
            return dispatch_fwd_tiled<T, 32>(x, off, msk, y, q, s);
        return dispatch_fwd_tiled<T, kWidest>(x, off, msk, y, q, s);
    }
    return DCNV4_ERR_UNSUPPORTED;
}

// ---- forward out of a ring of record rows (fp16, 16 channels per group, full-width tiles) ----
// Chooses how many record rows the LDS ring holds and the row halo: a host-side walk over the
// rounds of one workgroup (same arithmetic as the kernel's) finds the largest halo, up to 8 rows,
// for which the rows of two consecutive rounds always fit the ring, and checks that one round can
// stage the rows the next one adds.  Returns DCNV4_ERR_UNSUPPORTED where the kernel does not apply.
int make_rgeo(const Problem &q, int waves, int grid_wgs, RGeo *out)
{
    if (q.dtype != DCNV4_F16 || q.Cg != 16)
        return DCNV4_ERR_UNSUPPORTED;
    Geo base;
    int rc = make_geo(q, 1, &base);
    if (rc)
        return rc;
    RGeo p;
    memset(&p, 0, sizeof(p));
    const long long C = (long long)q.G * q.Cg;
    const long long xbytes = (long long)q.N * q.H * q.W * C * 2;
    const long long pgi = (long long)q.Ho * q.Wo * q.G;
    if (xbytes >= (1LL << 31) || pgi >= 0x1000000 || (long long)q.N * q.G >= (1LL << 24))
        return DCNV4_ERR_UNSUPPORTED;
    p.H = q.H; p.W = q.W; p.Ho = q.Ho; p.Wo = q.Wo; p.G = q.G;
    p.sh = q.sh; p.sw = q.sw; p.ph = q.ph; p.pw = q.pw; p.dh = q.dh; p.dw = q.dw;
    p.scale = q.scale;
    p.dmax = base.dmax;
    p.pitch = q.W + 4;
    p.VR = q.H + 3;
    p.npx = q.Ho * q.Wo;
    p.B = (p.npx + 63) / 64;
    const int lds_budget = (g_opt.lds_kb ? g_opt.lds_kb : 160) * 1024 - 128;
    p.ring = lds_budget / (p.pitch * kRingRecBytes);
    p.ntiles = q.N * q.G;
    p.tiles_per_xcd = (p.ntiles + kXcds - 1) / kXcds;
    p.remap = g_opt.xcd_remap;
    p.cbn = (p.pitch + 31) / 32;
    p.max_groups_round = kRingMaxTasks * ring_staging_waves(waves) / p.cbn;
    if (p.ring < 2 * kRingTaskRows || p.max_groups_round < 1)
        return DCNV4_ERR_UNSUPPORTED;
    // tiles the busiest workgroup walks
    int S;
    if (p.remap) {
        const int per = grid_wgs / kXcds;
        S = (p.tiles_per_xcd + per - 1) / per;
    } else {
        S = (p.ntiles + grid_wgs - 1) / grid_wgs;
    }
    const int RK = kRingTaskRows;
    if (p.ring > (S * p.VR + RK - 1) / RK * RK)
        p.ring = (S * p.VR + RK - 1) / RK * RK;      // no use for more rows than the workgroup ever stages
    const int NB = S * p.B;
    auto need = [&](int gb, int hr, int *lo, int *hi) {
        const int s = gb / p.B, b = gb - s * p.B;
        const int q0 = b * 64, q1 = q0 + 63 < p.npx - 1 ? q0 + 63 : p.npx - 1;
        const int oa = q0 / p.Wo, ob = q1 / p.Wo;
        int l = oa * p.sh - p.ph - hr, h = ob * p.sh - p.ph + 2 * p.dh + hr;
        l = l < -2 ? -2 : l > p.H ? p.H : l;
        h = h > p.H ? p.H : h < -2 ? -2 : h;
        *lo = s * p.VR + 2 + l;
        *hi = s * p.VR + 2 + h;
    };
    const int rounds = (NB + waves - 1) / waves;
    const int sim_rounds = rounds < 4096 ? rounds : 4096;
    int best = -1;
    const int hr_cap = g_opt.halo ? g_opt.halo : 8;
    for (int hr = hr_cap; hr >= 2 && best < 0; --hr) {
        bool ok = true;
        for (int t = 0; t < sim_rounds && ok; ++t) {
            int lo_first, hi_dummy, lo_dummy, hi_next, hi_this;
            need(t * waves, hr, &lo_first, &hi_dummy);
            const int last_this = (t + 1) * waves < NB ? (t + 1) * waves - 1 : NB - 1;
            const int last_next = (t + 2) * waves < NB ? (t + 2) * waves - 1 : NB - 1;
            need(last_this, hr, &lo_dummy, &hi_this);
            need(last_next, hr, &lo_dummy, &hi_next);
            const int g_this = (hi_this + RK) / RK, g_next = (hi_next + RK) / RK;    // row groups staged by then
            if (g_next * RK > lo_first + p.ring)
                ok = false;                                   // two rounds' rows do not fit
            if (t == 0 && g_this * RK > p.ring)
                ok = false;
            if (g_next - g_this > p.max_groups_round)
                ok = false;                                   // one round cannot stage the next one's rows
        }
        if (ok)
            best = hr;
    }
    if (best < 0)
        return DCNV4_ERR_UNSUPPORTED;
    p.hr = best;
    p.div_g = make_div((unsigned)q.G);
    p.div_wo = make_div((unsigned)q.Wo);
    p.div_cbn = make_div((unsigned)p.cbn);
    p.div_vr = make_div((unsigned)p.VR);
    p.div_ring = make_div((unsigned)p.ring);
    p.div_b = make_div((unsigned)p.B);
    p.x_bytes = (int)xbytes;
    p.x_img_bytes = base.x_img_bytes;
    p.y_img_bytes = base.y_img_bytes;
    p.row_bytes = base.row_bytes;
    p.pix_bytes = base.pix_bytes;
    p.og_bytes = q.merged ? 64 : 36;
    p.mg_bytes = q.merged ? 64 : 18;
    p.off_img_bytes = (int)(pgi * p.og_bytes);
    p.msk_img_bytes = (int)(pgi * p.mg_bytes);
    p.off_ext_bytes = (int)((pgi - 1) * p.og_bytes + 36);
    p.msk_ext_bytes = (int)((pgi - 1) * p.mg_bytes + 18);
    *out = p;
    return DCNV4_OK;
}

template <int WAVES, bool SOFTMAX = false>
int launch_ring_fwd(const void *x, const void *off, const void *msk, void *y, const Problem &q, hipStream_t s)
{
    const int cus = device_cus();
    if (cus <= 0)
        return DCNV4_ERR_LAUNCH;
    const long long ntiles = (long long)q.N * q.G;
    const long long tiles_per_xcd = (ntiles + kXcds - 1) / kXcds;
    unsigned grid;
    if (g_opt.xcd_remap) {
        const long long per = cus / kXcds < tiles_per_xcd ? cus / kXcds : tiles_per_xcd;
        grid = (unsigned)(per * kXcds);
    } else {
        grid = (unsigned)(cus < ntiles ? cus : ntiles);
    }
    RGeo p;
    int rc = make_rgeo(q, WAVES, (int)grid, &p);
    if (rc)
        return rc;
    const int lds = p.ring * p.pitch * kRingRecBytes + 128;
    if (lds > kMaxLdsBytes)
        return DCNV4_ERR_UNSUPPORTED;
    auto kern = dcnv4_ring_fwd_kernel<WAVES, SOFTMAX>;
    static int granted[kMaxDevices];
    if (!grant_lds(reinterpret_cast<const void *>(kern), lds, granted))
        return DCNV4_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WAVES * 64), lds, s, (const _Float16 *)x, (const _Float16 *)off,
                       (const _Float16 *)msk, (_Float16 *)y, p);
    snprintf(g_last_kernel[0], sizeof(g_last_kernel[0]), SOFTMAX ? "dcnv4_ring_fwd_kernel<%d, softmax>" : "dcnv4_ring_fwd_kernel<%d>", WAVES);
    return hipGetLastError() == hipSuccess ? DCNV4_OK : DCNV4_ERR_LAUNCH;
}

int dispatch_ring_fwd(const void *x, const void *off, const void *msk, void *y, const Problem &q, hipStream_t s)
{
    // eight waves: two per SIMD, 256 registers each (four waves on request, for tests)
    if (q.softmax)
        return g_opt.fwd_threads == 256 ? launch_ring_fwd<4, true>(x, off, msk, y, q, s) : launch_ring_fwd<8, true>(x, off, msk, y, q, s);
    if (g_opt.fwd_threads == 256)
        return launch_ring_fwd<4>(x, off, msk, y, q, s);
    return launch_ring_fwd<8>(x, off, msk, y, q, s);
}

template <typename T>
int dispatch_fwd(const void *x, const void *off, const void *msk, void *y, const Problem &q, hipStream_t s)
{
    if (q.kh != 3) {
        if (q.merged || q.softmax || g_opt.fwd_path >= 2)
            return DCNV4_ERR_UNSUPPORTED;
        return q.kh == 1 ? dispatch_fwd_window<T, 1>(x, off, msk, y, q, s) : dispatch_fwd_window<T, 5>(x, off, msk, y, q, s);
    }
    // (maps of a few batches per image leave most of a ring workgroup idle: the rectangle kernels,
    // with several small workgroups per compute unit, are faster there -- measured at 14x14 and 7x7)
    if (sizeof(T) == 2 && (g_opt.fwd_path == 3 || (g_opt.fwd_path == 0 && q.Ho * q.Wo >= 512))) {
        const int rc = dispatch_ring_fwd(x, off, msk, y, q, s);
        if (rc != DCNV4_ERR_UNSUPPORTED || g_opt.fwd_path == 3)
            return rc;
    }
    if (g_opt.fwd_path == 3)
        return DCNV4_ERR_UNSUPPORTED;
    if (g_opt.fwd_path != 1) {
        const int rc = dispatch_fwd_tiled_cg<T>(x, off, msk, y, q, s);
        if (rc != DCNV4_ERR_UNSUPPORTED || g_opt.fwd_path == 2)
            return rc;
    }
    if (q.merged || q.softmax)               // (the direct kernels read two separate tensors and take m as given)
        return DCNV4_ERR_UNSUPPORTED;
    const int cpt = pick_fwd_cpt(q.Cg);
    switch (q.Cg) {
    case 8: return dispatch_fwd_cpt<T, 8>(cpt, x, off, msk, y, q, s);
    case 16: return dispatch_fwd_cpt<T, 16>(cpt, x, off, msk, y, q, s);
    case 32: return dispatch_fwd_cpt<T, 32>(cpt, x, off, msk, y, q, s);
    case 64: return dispatch_fwd_cpt<T, 64>(cpt, x, off, msk, y, q, s);
    }
    return DCNV4_ERR_UNSUPPORTED;
}

template <int CG, int CPT, int KS = 3>
int launch_bwd(const void *x, const void *off, const void *msk, const void *gy, void *gx, void *go, void *gm,
               const Problem &q, hipStream_t s)
{
    Geo p;
    int rc = make_geo(q, CG / CPT, &p);
    if (rc)
        return rc;
    const long long zbytes = (long long)q.N * p.x_img_bytes;
    long long zb = (zbytes / 16 + kThreads - 1) / kThreads;
    if (zb > 8192) zb = 8192;
    hipLaunchKernelGGL(dcnv4_zero_kernel, dim3((unsigned)zb), dim3(kThreads), 0, s, (u32x4 *)gx, zbytes);
    hipLaunchKernelGGL((dcnv4_bwd_kernel<CG, CPT, KS, KS>), dim3(grid_of(p)), dim3(kThreads), 0, s, (const float *)x,
                       (const float *)off, (const float *)msk, (const float *)gy, (float *)gx, (float *)go,
                       (float *)gm, p);
    if (KS == 3)
        snprintf(g_last_kernel[1], sizeof(g_last_kernel[1]), "dcnv4_bwd_kernel<%d, %d>", CG, CPT);
    else
        snprintf(g_last_kernel[1], sizeof(g_last_kernel[1]), "dcnv4_bwd_kernel<%d, %d, %d, %d>", CG, CPT, KS, KS);
    return hipGetLastError() == hipSuccess ? DCNV4_OK : DCNV4_ERR_LAUNCH;
}

template <int CG>
int dispatch_bwd_cpt(int cpt, const void *x, const void *off, const void *msk, const void *gy, void *gx, void *go,
                     void *gm, const Problem &q, hipStream_t s)
{
    if constexpr (CG >= 16) {
        if (cpt == 16) return launch_bwd<CG, 16>(x, off, msk, gy, gx, go, gm, q, s);
    }
    if (cpt == 8) return launch_bwd<CG, 8>(x, off, msk, gy, gx, go, gm, q, s);
    if constexpr (CG <= 64) {
        if (cpt == 4) return launch_bwd<CG, 4>(x, off, msk, gy, gx, go, gm, q, s);
    }
    if constexpr (CG <= 64) {
        if (cpt == 2) return launch_bwd<CG, 2>(x, off, msk, gy, gx, go, gm, q, s);
    }
    if constexpr (CG <= 32) {
        if (cpt == 1) return launch_bwd<CG, 1>(x, off, msk, gy, gx, go, gm, q, s);
    }
    return DCNV4_ERR_UNSUPPORTED;
}

// Backward through the LDS-staged kernels: zero-fill of grad_x, then the grad_offset/grad_mask
// pass (gathers, like the forward) and the grad_x pass (LDS-private accumulation, one flush per
// tile).  Both passes are prepared -- everything that can refuse -- before anything is launched,
// so a call that returns an error has written nothing.
template <typename T, int CG>
int launch_bwd_tiled(const void *x, const void *off, const void *msk, const void *gy, void *gx, void *go, void *gm,
                     const Problem &q, hipStream_t s)
{
    // the gather pass keeps 4*Cg inputs and gy per lane: eight waves fit the register file with pixels of up to
    // 32 bytes, four with 64-byte pixels
    constexpr int THREADS = CG * sizeof(T) >= 64 ? 256 : 512;
    // CG is the kernels' channel run; a wider group (q.Cg) goes through as q.Cg / CG slices whose
    // grad_offset/grad_mask parts are added up in zero-filled outputs
    const bool sliced = q.Cg != CG;
    // whole fp32 groups: the lanes read and write their own pixels' values, no LDS slices, eight waves
    bool gom_direct = false;
    if constexpr (sizeof(T) == 4)
        gom_direct = !sliced && g_opt.gom_coop == 0;
    // (for fp16 there is no other backward, so the tile-size heuristic does not apply)
    const bool any_size = g_opt.bwd_path == 2 || sizeof(T) == 2 || q.merged || q.softmax;
    // the grad_x pass: twelve waves keep the LDS busiest (measured)
    const int gxt = g_opt.gx_threads ? g_opt.gx_threads : 768;
    TiledLaunch l_gom, l_gx;
    int rc;
    if constexpr (sizeof(T) == 4) {
        rc = gom_direct ? prepare_tiled<T, CG, 512, kTiledGradOMDirect>(q, any_size, 0, 0, &l_gom)
                        : prepare_tiled<T, CG, THREADS, kTiledGradOM>(q, any_size, 0, 0, &l_gom);
    } else {
        rc = prepare_tiled<T, CG, THREADS, kTiledGradOM>(q, any_size, 0, 0, &l_gom);
    }
    if (rc)
        return rc;
    rc = gxt == 768   ? prepare_tiled<T, CG, 768, kTiledGradX>(q, any_size, 0, 0, &l_gx)
         : gxt == 512 ? prepare_tiled<T, CG, 512, kTiledGradX>(q, any_size, 0, 0, &l_gx)
                      : prepare_tiled<T, CG, 256, kTiledGradX>(q, any_size, 0, 0, &l_gx);
    if (rc)
        return rc;
    auto zero = [&](void *ptr, long long bytes) {
        long long zb = (bytes / 16 + kThreads - 1) / kThreads;
        if (zb > 8192) zb = 8192;
        if (zb < 1) zb = 1;
        hipLaunchKernelGGL(dcnv4_zero_kernel, dim3((unsigned)zb), dim3(kThreads), 0, s, (u32x4 *)ptr, bytes);
    };
    zero(gx, (long long)q.N * l_gx.p.x_img_bytes);
    if (q.merged) {
        zero(go, (long long)q.N * l_gom.p.off_img_bytes);       // one buffer: gradients and padding
    } else if (sliced) {
        zero(go, (long long)q.N * l_gom.p.off_img_bytes);
        zero(gm, (long long)q.N * l_gom.p.msk_img_bytes);
    }
    if constexpr (sizeof(T) == 4) {
        rc = gom_direct ? run_tiled<T, CG, 512, kTiledGradOMDirect>(l_gom, x, off, msk, gy, go, gm, s, 1)
                        : run_tiled<T, CG, THREADS, kTiledGradOM>(l_gom, x, off, msk, gy, go, gm, s, 1);
    } else {
        rc = run_tiled<T, CG, THREADS, kTiledGradOM>(l_gom, x, off, msk, gy, go, gm, s, 1);
    }
    if (rc == DCNV4_OK)
        rc = gxt == 768   ? run_tiled<T, CG, 768, kTiledGradX>(l_gx, x, off, msk, gy, gx, nullptr, s, 1)
             : gxt == 512 ? run_tiled<T, CG, 512, kTiledGradX>(l_gx, x, off, msk, gy, gx, nullptr, s, 1)
                          : run_tiled<T, CG, 256, kTiledGradX>(l_gx, x, off, msk, gy, gx, nullptr, s, 1);
    return rc;
}

int fill_problem(Problem *q, int N, int H, int W, int G, int Cg, int kh, int kw, int sh, int sw, int ph, int pw,
                 int dh, int dw, float scale, int dtype)
{
    q->N = N; q->H = H; q->W = W; q->G = G; q->Cg = Cg;
    q->kh = kh; q->kw = kw;
    q->sh = sh; q->sw = sw; q->ph = ph; q->pw = pw; q->dh = dh; q->dw = dw;
    q->scale = scale; q->dtype = dtype;
    q->merged = 0;
    q->softmax = 0;
    q->Ho = q->Wo = 0;
    if (H < 1 || W < 1 || kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0 || dh < 1 || dw < 1)
        return DCNV4_ERR_SHAPE;
    return dcnv4_output_hw(H, W, kh, kw, sh, sw, ph, pw, dh, dw, &q->Ho, &q->Wo);
}

}  // namespace

extern "C" {

int dcnv4_output_hw(int H, int W, int kernel_h, int kernel_w, int stride_h, int stride_w, int pad_h, int pad_w,
                    int dil_h, int dil_w, int *H_out, int *W_out)
{
    if (!H_out || !W_out)
        return DCNV4_ERR_NULL;
    if (H < 1 || W < 1 || kernel_h < 1 || kernel_w < 1 || stride_h < 1 || stride_w < 1 || pad_h < 0 || pad_w < 0 ||
        dil_h < 1 || dil_w < 1)
        return DCNV4_ERR_SHAPE;
    const long long eh = (long long)H + 2LL * pad_h - (long long)dil_h * (kernel_h - 1) - 1;
    const long long ew = (long long)W + 2LL * pad_w - (long long)dil_w * (kernel_w - 1) - 1;
    if (eh < 0 || ew < 0)
        return DCNV4_ERR_SHAPE;
    *H_out = (int)(eh / stride_h + 1);
    *W_out = (int)(ew / stride_w + 1);
    return DCNV4_OK;
}

namespace {

int forward_impl(const void *x, const void *offset, const void *mask, void *y, int N, int H, int W, int G, int Cg,
                 int kernel_h, int kernel_w, int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
                 float offset_scale, int dtype, void *stream, bool merged, bool softmax = false)
{
    const void *ptrs[4] = {x, offset, y, mask};
    for (int i = 0; i < (merged ? 3 : 4); ++i)
        if (!ptrs[i])
            return DCNV4_ERR_NULL;
    Problem q;
    int rc = fill_problem(&q, N, H, W, G, Cg, kernel_h, kernel_w, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w,
                          offset_scale, dtype);
    if (rc)
        return rc;
    rc = validate(q, kernel_h, kernel_w, ptrs, merged ? 3 : 4);
    if (rc)
        return rc;
    q.softmax = softmax;
    if (merged) {
        // the mask values follow the 18 offsets of their (pixel, group) in the same buffer
        q.merged = 1;
        mask = (const char *)offset + 18 * esize(dtype);
    }
    hipStream_t s = (hipStream_t)stream;
    return dtype == DCNV4_F16 ? dispatch_fwd<_Float16>(x, offset, mask, y, q, s)
                              : dispatch_fwd<float>(x, offset, mask, y, q, s);
}

int backward_impl(const void *x, const void *offset, const void *mask, const void *grad_y, void *grad_x,
                  void *grad_offset, void *grad_mask, int N, int H, int W, int G, int Cg, int kernel_h,
                  int kernel_w, int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
                  float offset_scale, int dtype, void *stream, bool merged, bool softmax = false)
{
    const void *ptrs[7] = {x, offset, grad_y, grad_x, grad_offset, mask, grad_mask};
    for (int i = 0; i < (merged ? 5 : 7); ++i)
        if (!ptrs[i])
            return DCNV4_ERR_NULL;
    Problem q;
    int rc = fill_problem(&q, N, H, W, G, Cg, kernel_h, kernel_w, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w,
                          offset_scale, dtype);
    if (rc)
        return rc;
    rc = validate(q, kernel_h, kernel_w, ptrs, merged ? 5 : 7);
    if (rc)
        return rc;
    q.softmax = softmax;
    if (merged) {
        q.merged = 1;
        mask = (const char *)offset + 18 * esize(dtype);
        grad_mask = (char *)grad_offset + 18 * esize(dtype);
    }
    hipStream_t s = (hipStream_t)stream;
    if (kernel_h != 3) {
        // 1x1 and 5x5 windows: the direct fp32 kernel, one channel per lane (two for groups of 64)
        if (merged || softmax || dtype != DCNV4_F32 || g_opt.bwd_path == 2)
            return DCNV4_ERR_UNSUPPORTED;
        if (kernel_h == 1) {
            switch (Cg) {
            case 8: return launch_bwd<8, 1, 1>(x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, q, s);
            case 16: return launch_bwd<16, 1, 1>(x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, q, s);
            case 32: return launch_bwd<32, 1, 1>(x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, q, s);
            case 64: return launch_bwd<64, 2, 1>(x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, q, s);
            }
        } else {
            switch (Cg) {
            case 8: return launch_bwd<8, 1, 5>(x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, q, s);
            case 16: return launch_bwd<16, 1, 5>(x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, q, s);
            case 32: return launch_bwd<32, 1, 5>(x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, q, s);
            case 64: return launch_bwd<64, 2, 5>(x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, q, s);
            }
        }
        return DCNV4_ERR_UNSUPPORTED;
    }
    if (dtype == DCNV4_F16) {
        // fp16 storage, fp32 arithmetic; only the LDS-staged kernels exist for it (Cg 8, 16 or 32)
        if (g_opt.bwd_path == 1)
            return DCNV4_ERR_UNSUPPORTED;
        if (Cg == 8)
            return launch_bwd_tiled<_Float16, 8>(x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, q, s);
        if (Cg == 16)
            return launch_bwd_tiled<_Float16, 16>(x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, q, s);
        if (Cg == 32)                                  // 64-byte pixels, like fp32 groups of 16
            return launch_bwd_tiled<_Float16, 32>(x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, q, s);
        return DCNV4_ERR_UNSUPPORTED;
    }
    if (g_opt.bwd_path != 1 || merged || softmax) {
        rc = DCNV4_ERR_UNSUPPORTED;
        if (Cg == 8)
            rc = launch_bwd_tiled<float, 8>(x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, q, s);
        else if (Cg == 16 || Cg == 32 || Cg == 64)     // wider groups: 64-byte channel slices
            rc = launch_bwd_tiled<float, 16>(x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, q, s);
        if (rc != DCNV4_ERR_UNSUPPORTED || g_opt.bwd_path == 2 || merged || softmax)
            return rc;
    }
    const int cpt = pick_bwd_cpt(Cg);
    switch (Cg) {
    case 8: return dispatch_bwd_cpt<8>(cpt, x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, q, s);
    case 16: return dispatch_bwd_cpt<16>(cpt, x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, q, s);
    case 32: return dispatch_bwd_cpt<32>(cpt, x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, q, s);
    case 64: return dispatch_bwd_cpt<64>(cpt, x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, q, s);
    }
    return DCNV4_ERR_UNSUPPORTED;
}

// ---- the module's linear layers ----------------------------------------------------------------
// One layer of the linear kernel's work list, checked: K * element size a multiple of 32 bytes (one
// MFMA group), nout a multiple of 32 (one MFMA block), 32-bit byte offsets inside every tensor.
int add_linear_segment(LinGeo *g, long long P, int K, int dtype, const void *w, const void *b, void *y, int nout,
                       int plane_shift = 0)
{
    if (!w || !y)
        return DCNV4_ERR_NULL;
    if (nout < 1)
        return DCNV4_ERR_SHAPE;
    const long long es = esize(dtype);
    if (nout % 32 || (long long)nout * K * es >= (1LL << 31) || P * nout * es >= (1LL << 31) || g->nseg >= kLinMaxSeg)
        return DCNV4_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(w) & 15u) || (reinterpret_cast<uintptr_t>(y) & 15u) ||
        (reinterpret_cast<uintptr_t>(b) & (uintptr_t)(es - 1)))
        return DCNV4_ERR_ALIGN;
    LinSeg &sg = g->seg[g->nseg++];
    sg.w = w; sg.b = b; sg.y = y; sg.nout = nout;
    sg.plane_shift = plane_shift;
    sg.nblocks = (nout + kLinBlock - 1) / kLinBlock;
    return DCNV4_OK;
}

int begin_linear(LinGeo *g, const void *x, long long P, int K, int dtype)
{
    memset(g, 0, sizeof(*g));
    if (!x)
        return DCNV4_ERR_NULL;
    if (P < 1 || K < 1)
        return DCNV4_ERR_SHAPE;
    if (dtype != DCNV4_F32 && dtype != DCNV4_F16)
        return DCNV4_ERR_UNSUPPORTED;
    const long long kbytes = (long long)K * esize(dtype);
    if (kbytes % 32 || P * kbytes >= (1LL << 31))
        return DCNV4_ERR_UNSUPPORTED;
    if (reinterpret_cast<uintptr_t>(x) & 15u)
        return DCNV4_ERR_ALIGN;
    g->P = (int)P;
    g->kbytes = (int)kbytes;
    g->nchunks = (int)((kbytes + kLinChunk - 1) / kLinChunk);
    return DCNV4_OK;
}

int launch_linear(const void *x, const LinGeo &g, int dtype, hipStream_t s)
{
    const int tiles = (g.P + kLinPixels - 1) / kLinPixels;
    // maps of few pixels and many channels: the passes over blocks of output channels are spread over
    // workgroups as well, until there are about two workgroups per compute unit
    int npass = 0;
    for (int i = 0; i < g.nseg; ++i)
        npass += g.seg[i].nblocks;
    const int want = 2 * device_cus();
    int split = (want + tiles - 1) / tiles;
    if (split > npass) split = npass;
    if (split < 1) split = 1;
    const dim3 grid((unsigned)tiles, (unsigned)split);
    const bool single = g.nchunks == 1;
    if (dtype == DCNV4_F16) {
        if (single)
            hipLaunchKernelGGL((dcnv4_linear_kernel<_Float16, true>), grid, dim3(256), 0, s, (const _Float16 *)x, g);
        else
            hipLaunchKernelGGL((dcnv4_linear_kernel<_Float16, false>), grid, dim3(256), 0, s, (const _Float16 *)x, g);
    } else {
        if (single)
            hipLaunchKernelGGL((dcnv4_linear_kernel<float, true>), grid, dim3(256), 0, s, (const float *)x, g);
        else
            hipLaunchKernelGGL((dcnv4_linear_kernel<float, false>), grid, dim3(256), 0, s, (const float *)x, g);
    }
    return hipGetLastError() == hipSuccess ? DCNV4_OK : DCNV4_ERR_LAUNCH;
}

int launch_depthwise(const void *x, const void *w, const void *b, void *y, int N, int H, int W, int C, int dtype,
                     hipStream_t s)
{
    if (!x || !w || !y)
        return DCNV4_ERR_NULL;
    if (N < 1 || H < 1 || W < 1 || C < 1)
        return DCNV4_ERR_SHAPE;
    if (dtype != DCNV4_F32 && dtype != DCNV4_F16)
        return DCNV4_ERR_UNSUPPORTED;
    const long long es = esize(dtype), pix_bytes = (long long)C * es;
    const long long bytes = (long long)N * H * W * pix_bytes;
    if (pix_bytes % 16 || bytes >= (1LL << 31))
        return DCNV4_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(x) & 15u) || (reinterpret_cast<uintptr_t>(w) & 15u) ||
        (reinterpret_cast<uintptr_t>(y) & 15u) || (reinterpret_cast<uintptr_t>(b) & 15u))
        return DCNV4_ERR_ALIGN;
    DwGeo g;
    g.H = H; g.W = W;
    g.units = (int)(pix_bytes / 16);
    g.total = (int)(bytes / 16);
    g.row_bytes = (int)(W * pix_bytes);
    g.pix_bytes = (int)pix_bytes;
    g.div_units = make_div((unsigned)g.units);
    g.div_w = make_div((unsigned)W);
    g.div_h = make_div((unsigned)H);
    const unsigned grid = (unsigned)((g.total + 255) / 256);
    if (dtype == DCNV4_F16)
        hipLaunchKernelGGL(dcnv4_depthwise3x3_kernel<_Float16>, dim3(grid), dim3(256), 0, s, (const _Float16 *)x,
                           (const _Float16 *)w, (const _Float16 *)b, (_Float16 *)y, g);
    else
        hipLaunchKernelGGL(dcnv4_depthwise3x3_kernel<float>, dim3(grid), dim3(256), 0, s, (const float *)x,
                           (const float *)w, (const float *)b, (float *)y, g);
    return hipGetLastError() == hipSuccess ? DCNV4_OK : DCNV4_ERR_LAUNCH;
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace

int dcnv4_forward(const void *x, const void *offset, const void *mask, void *y, int N, int H, int W, int G, int Cg,
                  int kernel_h, int kernel_w, int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
                  float offset_scale, int dtype, void *stream)
{
    return forward_impl(x, offset, mask, y, N, H, W, G, Cg, kernel_h, kernel_w, stride_h, stride_w, pad_h, pad_w, dil_h,
                        dil_w, offset_scale, dtype, stream, false);
}

int dcnv4_forward_merged(const void *x, const void *offset_mask, void *y, int N, int H, int W, int G, int Cg,
                         int kernel_h, int kernel_w, int stride_h, int stride_w, int pad_h, int pad_w, int dil_h,
                         int dil_w, float offset_scale, int dtype, void *stream)
{
    return forward_impl(x, offset_mask, nullptr, y, N, H, W, G, Cg, kernel_h, kernel_w, stride_h, stride_w, pad_h, pad_w,
                        dil_h, dil_w, offset_scale, dtype, stream, true);
}

int dcnv4_backward(const void *x, const void *offset, const void *mask, const void *grad_y, void *grad_x,
                   void *grad_offset, void *grad_mask, int N, int H, int W, int G, int Cg, int kernel_h,
                   int kernel_w, int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
                   float offset_scale, int dtype, void *stream)
{
    return backward_impl(x, offset, mask, grad_y, grad_x, grad_offset, grad_mask, N, H, W, G, Cg, kernel_h, kernel_w,
                         stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, offset_scale, dtype, stream, false);
}

int dcnv4_forward_softmax(const void *x, const void *offset, const void *mask_logits, void *y, int N, int H, int W,
                          int G, int Cg, int kernel_h, int kernel_w, int stride_h, int stride_w, int pad_h, int pad_w,
                          int dil_h, int dil_w, float offset_scale, int dtype, void *stream)
{
    return forward_impl(x, offset, mask_logits, y, N, H, W, G, Cg, kernel_h, kernel_w, stride_h, stride_w, pad_h, pad_w,
                        dil_h, dil_w, offset_scale, dtype, stream, false, true);
}

int dcnv4_backward_softmax(const void *x, const void *offset, const void *mask_logits, const void *grad_y,
                           void *grad_x, void *grad_offset, void *grad_mask_logits, int N, int H, int W, int G,
                           int Cg, int kernel_h, int kernel_w, int stride_h, int stride_w, int pad_h, int pad_w,
                           int dil_h, int dil_w, float offset_scale, int dtype, void *stream)
{
    return backward_impl(x, offset, mask_logits, grad_y, grad_x, grad_offset, grad_mask_logits, N, H, W, G, Cg, kernel_h,
                         kernel_w, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, offset_scale, dtype, stream, false,
                         true);
}

int dcnv4_backward_merged(const void *x, const void *offset_mask, const void *grad_y, void *grad_x,
                          void *grad_offset_mask, int N, int H, int W, int G, int Cg, int kernel_h, int kernel_w,
                          int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w, float offset_scale,
                          int dtype, void *stream)
{
    return backward_impl(x, offset_mask, nullptr, grad_y, grad_x, grad_offset_mask, nullptr, N, H, W, G, Cg, kernel_h,
                         kernel_w, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, offset_scale, dtype, stream, true);
}

long long dcnv4_forward_algorithmic_bytes(int N, int H, int W, int G, int Cg, int H_out, int W_out, int dtype)
{
    const long long es = esize(dtype), C = (long long)G * Cg;
    const long long P = (long long)N * H_out * W_out;
    return es * ((long long)N * H * W * C + P * C + P * G * 27);
}

long long dcnv4_backward_algorithmic_bytes(int N, int H, int W, int G, int Cg, int H_out, int W_out, int dtype)
{
    const long long es = esize(dtype), C = (long long)G * Cg;
    const long long P = (long long)N * H_out * W_out;
    return es * (2 * (long long)N * H * W * C + P * C + 2 * P * G * 27);
}

long long dcnv4_forward_merged_algorithmic_bytes(int N, int H, int W, int G, int Cg, int H_out, int W_out, int dtype)
{
    const long long es = esize(dtype), C = (long long)G * Cg;
    const long long P = (long long)N * H_out * W_out;
    return es * ((long long)N * H * W * C + P * C + P * G * 32);
}

long long dcnv4_backward_merged_algorithmic_bytes(int N, int H, int W, int G, int Cg, int H_out, int W_out, int dtype)
{
    const long long es = esize(dtype), C = (long long)G * Cg;
    const long long P = (long long)N * H_out * W_out;
    return es * (2 * (long long)N * H * W * C + P * C + 2 * P * G * 32);
}

int dcnv4_linear(const void *x, const void *w, const void *b, void *y, long long P, int K, int Nout, int dtype,
                 void *stream)
{
    LinGeo g;
    int rc = begin_linear(&g, x, P, K, dtype);
    if (rc)
        return rc;
    rc = add_linear_segment(&g, P, K, dtype, w, b, y, Nout);
    if (rc)
        return rc;
    return launch_linear(x, g, dtype, (hipStream_t)stream);
}

int dcnv4_depthwise3x3(const void *x, const void *w, const void *b, void *y, int N, int H, int W, int C, int dtype,
                       void *stream)
{
    return launch_depthwise(x, w, b, y, N, H, W, C, dtype, (hipStream_t)stream);
}

long long dcnv4_module_workspace_bytes(int N, int H, int W, int G, int Cg, int dtype, int lightweight, int depthwise)
{
    if (N < 1 || H < 1 || W < 1 || G < 1 || Cg < 1 || (dtype != DCNV4_F32 && dtype != DCNV4_F16))
        return -1;
    const long long P = (long long)N * H * W, es = esize(dtype), C = (long long)G * Cg;
    const long long om = (long long)align256((size_t)(P * G * 32 * es)), act = (long long)align256((size_t)(P * C * es));
    return om + (lightweight ? 0 : 2 * act) + (depthwise ? act : 0);
}

namespace {

// Built-in workspace of dcnv4_module_forward_static: one copy per GPU, held until the process ends.
constexpr long long kScratchBytes = 32ll << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// Device address of `scratch` on the current device (the array's name is only a host-side stand-in:
// every GPU has its own copy at its own address), looked up once per device; null on failure.
void *scratch_address()
{
    static void *ptr[kMaxDevices];
    const int dev = current_device();
    if (dev < 0)
        return nullptr;
    if (!ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess)
            return nullptr;
        ptr[dev] = p;
    }
    return ptr[dev];
}

int module_forward_impl(const void *x, const void *w_in, const void *b_in, const void *w_dw, const void *b_dw,
                        const void *w_om, const void *b_om, const void *w_out, const void *b_out, void *workspace,
                        long long workspace_bytes, void *y, int N, int H, int W, int G, int Cg, int kernel_h,
                        int kernel_w, int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
                        float offset_scale, int dtype, void *stream)
{
    if (!x || !w_om || !workspace || !y)
        return DCNV4_ERR_NULL;
    if ((w_in == nullptr) != (w_out == nullptr))        // the two projections come together (or not at all)
        return DCNV4_ERR_NULL;
    const bool light = w_in == nullptr, dw = w_dw != nullptr;
    Problem q;
    int rc = fill_problem(&q, N, H, W, G, Cg, kernel_h, kernel_w, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w,
                          offset_scale, dtype);
    if (rc)
        return rc;
    const void *ptrs[3] = {x, workspace, y};
    rc = validate(q, kernel_h, kernel_w, ptrs, 3);
    if (rc)
        return rc;
    // the merged layer predicts one set of offsets per INPUT pixel: the window must keep the map's size
    if (q.Ho != H || q.Wo != W || kernel_h != 3)
        return DCNV4_ERR_UNSUPPORTED;
    const long long need = dcnv4_module_workspace_bytes(N, H, W, G, Cg, dtype, light ? 1 : 0, dw ? 1 : 0);
    if (workspace_bytes < need)
        return DCNV4_ERR_SHAPE;
    const long long P = (long long)N * H * W, es = esize(dtype);
    const int C = G * Cg;
    const size_t act = align256((size_t)(P * C * es));
    char *om = (char *)workspace;
    char *next = om + align256((size_t)(P * G * 32 * es));
    char *value = nullptr, *y_op = nullptr, *x_dw = nullptr;
    if (!light) {
        value = next;
        y_op = next + act;
        next += 2 * act;
    }
    if (dw)
        x_dw = next;
    // Between its layers the full module keeps value, offsets/scalars and the operator's output plane-major,
    // [image][group][pixel][channels of the group]: the operator then sees N*G images of ONE group whose
    // pixels are whole, contiguous pieces (a workgroup of its kernels reads full cache lines instead of a
    // quarter of each), and the linear layers write and read 1 KB runs.  (Not the lightweight variant, whose
    // value tensor is the caller's channel-last x; not groups whose bytes are no power of two in 32..128.)
    int vshift = 0;
    for (int sft = 5; sft <= 7; ++sft)
        if ((long long)Cg * es == (1LL << sft))
            vshift = sft;
    const bool planar = !light && vshift != 0 && g_opt.module_rows == 0;
    const int oshift = planar ? (es == 2 ? 6 : 7) : 0;            // 32 entries per (pixel, group)
    if (!planar)
        vshift = 0;
    // Everything that can refuse is checked before the first launch.  Without the depthwise convolution
    // both layers that read x are one launch; with it the offset/scalar layer reads the convolved map.
    LinGeo first, second, last;
    const bool fused = !dw && !light;
    rc = begin_linear(&first, x, P, C, dtype);
    if (!rc && !light)
        rc = add_linear_segment(&first, P, C, dtype, w_in, b_in, value, C, vshift);
    if (!rc && (fused || light) && !dw)
        rc = add_linear_segment(&first, P, C, dtype, w_om, b_om, om, G * 32, oshift);
    first.hw = H * W;
    first.div_hw = make_div((unsigned)(H * W));
    if (!rc && dw) {
        rc = begin_linear(&second, x_dw, P, C, dtype);
        if (!rc)
            rc = add_linear_segment(&second, P, C, dtype, w_om, b_om, om, G * 32, oshift);
        second.hw = H * W;
        second.div_hw = make_div((unsigned)(H * W));
        if (!rc && ((reinterpret_cast<uintptr_t>(w_dw) & 15u) || (reinterpret_cast<uintptr_t>(b_dw) & 15u)))
            rc = DCNV4_ERR_ALIGN;
        if (!rc && (P * C * es >= (1LL << 31) || (C * es) % 16))
            rc = DCNV4_ERR_UNSUPPORTED;
    }
    if (!rc && !light) {
        rc = begin_linear(&last, y_op, P, C, dtype);
        if (!rc)
            rc = add_linear_segment(&last, P, C, dtype, w_out, b_out, y, C);
        last.hw = H * W;
        last.div_hw = make_div((unsigned)(H * W));
        last.in_plane_shift = vshift;
    }
    if (rc)
        return rc;
    hipStream_t s = (hipStream_t)stream;
    if (first.nseg > 0) {
        rc = launch_linear(x, first, dtype, s);
        if (rc)
            return rc;
    }
    if (dw) {
        rc = launch_depthwise(x, w_dw, b_dw, x_dw, N, H, W, C, dtype, s);
        if (rc)
            return rc;
        rc = launch_linear(x_dw, second, dtype, s);
        if (rc)
            return rc;
    }
    if (planar)
        rc = forward_impl(value, om, nullptr, y_op, N * G, H, W, 1, Cg, kernel_h, kernel_w, stride_h, stride_w, pad_h, pad_w,
                          dil_h, dil_w, offset_scale, dtype, stream, true);
    else
        rc = forward_impl(light ? x : (const void *)value, om, nullptr, light ? y : (void *)y_op, N, H, W, G, Cg, kernel_h,
                          kernel_w, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, offset_scale, dtype, stream, true);
    if (rc || light)
        return rc;
    return launch_linear(y_op, last, dtype, s);
}

}  // namespace

int dcnv4_module_forward(const void *x, const void *w_in, const void *b_in, const void *w_dw, const void *b_dw,
                         const void *w_om, const void *b_om, const void *w_out, const void *b_out, void *workspace,
                         long long workspace_bytes, void *y, int N, int H, int W, int G, int Cg, int kernel_h,
                         int kernel_w, int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
                         float offset_scale, int dtype, void *stream)
{
    return module_forward_impl(x, w_in, b_in, w_dw, b_dw, w_om, b_om, w_out, b_out, workspace, workspace_bytes, y, N, H, W,
                               G, Cg, kernel_h, kernel_w, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, offset_scale,
                               dtype, stream);
}

long long dcnv4_module_static_workspace_limit(void) { return kScratchBytes; }

int dcnv4_module_forward_static(const void *x, const void *w_in, const void *b_in, const void *w_dw, const void *b_dw,
                                const void *w_om, const void *b_om, const void *w_out, const void *b_out, void *y,
                                int N, int H, int W, int G, int Cg, int kernel_h, int kernel_w, int stride_h,
                                int stride_w, int pad_h, int pad_w, int dil_h, int dil_w, float offset_scale, int dtype,
                                void *stream)
{
    if (!x || !w_om || !y)
        return DCNV4_ERR_NULL;
    if ((w_in == nullptr) != (w_out == nullptr))
        return DCNV4_ERR_NULL;
    const long long need = dcnv4_module_workspace_bytes(N, H, W, G, Cg, dtype, w_in == nullptr, w_dw != nullptr);
    if (need < 0)
        return (dtype != DCNV4_F32 && dtype != DCNV4_F16) ? DCNV4_ERR_UNSUPPORTED : DCNV4_ERR_SHAPE;
    if (need > kScratchBytes)
        return DCNV4_ERR_TOO_LARGE;
    void *ws = scratch_address();
    if (!ws)
        return DCNV4_ERR_LAUNCH;
    return module_forward_impl(x, w_in, b_in, w_dw, b_dw, w_om, b_om, w_out, b_out, ws, kScratchBytes, y, N, H, W, G, Cg,
                               kernel_h, kernel_w, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, offset_scale, dtype,
                               stream);
}

int dcnv4_set_option(const char *key, int value)
{
    if (!key)
        return DCNV4_ERR_NULL;
    if (!strcmp(key, "reset")) {             // every switch back to the library's own choice
        g_opt = Options();
        return DCNV4_OK;
    }
    if (!strcmp(key, "fwd_cpt") && (value == 0 || value == 8 || value == 16)) {
        g_opt.fwd_cpt = value;
        return DCNV4_OK;
    }
    if (!strcmp(key, "bwd_cpt") && (value == 0 || value == 1 || value == 2 || value == 4 || value == 8 || value == 16)) {
        g_opt.bwd_cpt = value;
        return DCNV4_OK;
    }
    if (!strcmp(key, "xcd_remap") && (value == 0 || value == 1)) {
        g_opt.xcd_remap = value;
        return DCNV4_OK;
    }
    if (!strcmp(key, "fwd_path") && value >= 0 && value <= 3) {
        g_opt.fwd_path = value;
        return DCNV4_OK;
    }
    if (!strcmp(key, "gx_threads") && (value == 0 || value == 256 || value == 512 || value == 768)) {
        g_opt.gx_threads = value;
        return DCNV4_OK;
    }
    if (!strcmp(key, "fwd_single") && value >= 0 && value <= 2) {
        g_opt.fwd_single = value;
        return DCNV4_OK;
    }
    if (!strcmp(key, "module_rows") && (value == 0 || value == 1)) {
        g_opt.module_rows = value;
        return DCNV4_OK;
    }
    if (!strcmp(key, "gom_coop") && (value == 0 || value == 1)) {
        g_opt.gom_coop = value;
        return DCNV4_OK;
    }
    if (!strcmp(key, "wg_per_cu") && value >= 0 && value <= 32) {
        g_opt.wg_per_cu = value;
        return DCNV4_OK;
    }
    if (!strcmp(key, "bwd_path") && value >= 0 && value <= 2) {
        g_opt.bwd_path = value;
        return DCNV4_OK;
    }
    if (!strcmp(key, "halo") && value >= 0 && value <= 64) {
        g_opt.halo = value;
        return DCNV4_OK;
    }
    if (!strcmp(key, "lds_kb") && (value == 0 || (value >= 8 && value <= 160))) {
        g_opt.lds_kb = value;
        return DCNV4_OK;
    }
    if (!strcmp(key, "fwd_threads") && (value == 0 || value == 64 || value == 128 || value == 256 || value == 512 || value == 640 || value == 768)) {
        g_opt.fwd_threads = value;
        return DCNV4_OK;
    }
    return DCNV4_ERR_UNSUPPORTED;
}

const char *dcnv4_last_kernel_name(int backward)
{
    const char *n = g_last_kernel[backward ? 1 : 0];
    return n[0] ? n : nullptr;
}

const char *dcnv4_status_string(int status)
{
    switch (status) {
    case DCNV4_OK: return "ok";
    case DCNV4_ERR_NULL: return "null pointer";
    case DCNV4_ERR_SHAPE: return "bad shape: a size is non-positive or the window does not fit";
    case DCNV4_ERR_UNSUPPORTED: return "unsupported kernel size, group width, dtype, option or tensor size";
    case DCNV4_ERR_ALIGN: return "tensor pointer not 16-byte aligned";
    case DCNV4_ERR_LAUNCH: return "HIP launch failed";
    case DCNV4_ERR_TOO_LARGE: return "the call needs more workspace than the built-in scratch buffer holds";
    }
    return "unknown status";
}

}  // extern "C"
