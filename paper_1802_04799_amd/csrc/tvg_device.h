// Device-side helpers shared by the libtvg kernels: element types, bf16
// conversion and the fused element-wise tail.
#ifndef TVG_DEVICE_H
#define TVG_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tvg.h"

namespace tvg {

typedef uint16_t bf16_t;   // raw bfloat16 bits

typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(uint32_t(b) << 16); }

// fp32 -> bf16, round to nearest, ties to even: the hardware conversion of gfx950
// (v_cvt_pk_bf16_f32), one instruction per pair of values.
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    return __builtin_bit_cast(bf16_t, static_cast<__bf16>(f));
}

__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi)
{
    typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
    typedef float f2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{lo, hi}, bf2));
}

// Output store with or without the non-temporal hint (the TVG_STREAM_OUT flag of the call), a
// compile-time choice: the wide stores of the staged tail and of the depthwise kernels take
// it.  With the hint y neither displaces the operands in L2 nor waits there, dirty, for the
// write-back at the end of the kernel (measured on twelve unrelated layers in a row: 333 us
// plain, 299 us hinted); without it the next kernel finds y in the memory-side cache (measured
// on the 21-launch ResNet-18 chain at batch 32: 0.437 ms plain, 0.450 ms hinted).  Narrow
// stores are always plain: hinted, the element-wise tail of 7x7 maps was 30-60 % slower.
template <bool NT, typename V>
__device__ __forceinline__ void stream_store(V *p, V v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// Exact floor division of small non-negative integers through the float reciprocal:
// a and b below 2^22, inv_b = 1.0f / b.  The float quotient is within one of the true
// quotient, and one correction step settles it.  About 8 vector instructions instead of
// the 35 or so of the emulated 32-bit integer division.
__device__ __forceinline__ int fast_div(int a, int b, float inv_b, int *rem)
{
    int q = (int)(__int2float_rn(a) * inv_b);
    int r = a - q * b;
    if (r < 0) { --q; r += b; }
    else if (r >= b) { ++q; r -= b; }
    *rem = r;
    return q;
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float *p, int i) { return p[i]; }
    static __device__ __forceinline__ void store(float *p, int i, float v) { p[i] = v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t *p, int i) { return bf16_to_f32(p[i]); }
    static __device__ __forceinline__ void store(bf16_t *p, int i, float v) { p[i] = f32_to_bf16(v); }
};

// The element-wise operators fused onto the convolution's output (TVM paper,
// Section 3, operator fusion): bias, folded batch-norm scale/shift, residual
// add, ReLU, applied to the fp32 accumulator before the single store.
template <typename T>
__device__ __forceinline__ void fused_tail_store(float acc, float scale, float shift, float bias,
                                                 const T *residual, T *y, int out_index, bool relu)
{
    float t = (acc + bias) * scale + shift;
    if (residual) t += Elem<T>::load(residual, out_index);
    if (relu) t = fmaxf(t, 0.0f);
    Elem<T>::store(y, out_index, t);
}

// ---------------------------------------------------------------------------------------
// Tile epilogue shared by the MFMA kernels.
//
// The kernels feed the MFMA with the pixel operand first and the weight operand second, so
// a 32x32 accumulator tile comes out as D[pixel][channel]: value v of lane l belongs to
// channel l%32 and pixel 8*(v/4) + 4*(l/32) + v%4, i.e. a lane holds four groups of four
// CONSECUTIVE pixels of ONE output channel.  The fused tail (one FMA with the channel's
// scale and offset, residual add, ReLU clamp, rounding) is therefore applied in place, with
// one (scale, offset) pair per lane, and a group packs into one 8-byte (bf16) or 16-byte
// (fp32) piece of an NCHW row without any data exchange.  Three store modes, chosen on the
// host from OH*OW and the pointers' alignment:
//   8  (bf16, OH*OW % 8 == 0)  the packed groups go through a wave-private LDS area
//      (32 channel rows x 64 B, row stride 80 B) and leave as 16-byte stores, four lanes per
//      channel row = 64 contiguous bytes;
//   4  (OH*OW % 4 == 0)        each group is stored directly (8 or 16 bytes per lane);
//   1  (anything else)         element-wise stores with a per-pixel index.
// Four consecutive pixels starting at a multiple of four lie in one image and are contiguous
// and aligned in NCHW exactly when OH*OW is a multiple of four.
// ---------------------------------------------------------------------------------------
struct TailArgs {
    const float *scale, *shift, *bias;
    const void *residual;
    void *y;
    int OC, OHW, npix, relu;      // relu: bit 0 = ReLU, bit 1 = hinted stores on the staged fast path
};

constexpr int kStageRow = 80;                          // bytes per staged channel row
constexpr int kStageBytes = 32 * kStageRow;            // per wave
constexpr int kStageFloats = kStageBytes / 4;

// Puts the per-channel multiplier and offset of a tile's `rows` output channels into LDS as
// (scale, bias*scale + shift) pairs, so the epilogue reads them with LDS latency instead of
// issuing dependent global loads.  (acc + bias)*scale + shift == acc*scale + that offset.
// Call before a barrier that precedes the first store_tile.
__device__ __forceinline__ void stage_scale_shift(float *ss, int m0, int rows, const float *scale,
                                                  const float *shift, const float *bias, int OC,
                                                  int tid, int nthreads)
{
    for (int r = tid; r < rows; r += nthreads) {
        const int oc = m0 + r;
        float sc = 0.0f, sf = 0.0f;
        if (oc < OC) {
            sc = scale[oc];
            sf = bias ? fmaf(bias[oc], sc, shift[oc]) : shift[oc];
        }
        ss[2 * r] = sc;
        ss[2 * r + 1] = sf;
    }
}

typedef uint32_t uint2v __attribute__((ext_vector_type(2)));

// Four fp32 values -> the dtype's packed group, and a packed group -> four fp32 values.
template <typename T> struct Group4;
template <> struct Group4<bf16_t> {
    typedef uint2v vec;
    static __device__ __forceinline__ vec pack(const float *f)
    {
        return vec{f32x2_to_bf16x2(f[0], f[1]), f32x2_to_bf16x2(f[2], f[3])};
    }
    static __device__ __forceinline__ void unpack(const vec &r, float *f)
    {
        f[0] = __uint_as_float(r[0] << 16); f[1] = __uint_as_float(r[0] & 0xFFFF0000u);
        f[2] = __uint_as_float(r[1] << 16); f[3] = __uint_as_float(r[1] & 0xFFFF0000u);
    }
};
template <> struct Group4<float> {
    typedef float4v vec;
    static __device__ __forceinline__ vec pack(const float *f) { return vec{f[0], f[1], f[2], f[3]}; }
    static __device__ __forceinline__ void unpack(const vec &r, float *f)
    {
        f[0] = r[0]; f[1] = r[1]; f[2] = r[2]; f[3] = r[3];
    }
};

// acc: one 32x32 accumulator tile in the D[pixel][channel] orientation described above.
// oc0 / p0: output channel of column 0 / flattened pixel of row 0 (a multiple of 32).
// ss: staged (scale, offset) pairs of the workgroup tile, row0: index of oc0 in that tile.
// stage: kStageBytes of wave-private LDS (used by bf16 modes 8 and 1).
template <typename T>
__device__ __forceinline__ void store_tile(const float16v &acc, unsigned char *stage, int lane,
                                           int oc0, int p0, const TailArgs &t, int vmode,
                                           const float *ss, int row0)
{
    typedef typename Group4<T>::vec gvec;
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int oc = oc0 + lrow;
    const float sc = ss[2 * (row0 + lrow)], sf = ss[2 * (row0 + lrow) + 1];
    const float floor_v = (t.relu & 1) ? 0.0f : -INFINITY;     // no ReLU = clamp at minus infinity
    const T *res = static_cast<const T *>(t.residual);
    T *y = static_cast<T *>(t.y);
    // image index of the tile's first pixel: uniform, one scalar division; later pixels
    // reach later images by repeated subtraction (at most once when OH*OW >= 32)
    const int p0u = __builtin_amdgcn_readfirstlane(p0);
    const int n0 = p0u / t.OHW, rem0 = p0u - n0 * t.OHW;

    // Fast path (uniform test): the tile's 32 pixels lie in one image and neither the pixel
    // nor the channel range is ragged, so every index is base + constant and nothing is
    // masked.  This is the case for all but the boundary tiles.
    if (vmode != 1 && rem0 + 32 <= t.OHW && p0u + 32 <= t.npix &&
        __builtin_amdgcn_readfirstlane(oc0) + 32 <= t.OC) {
        const int base = (n0 * t.OC + oc) * t.OHW + rem0 + 4 * lhalf;     // lane's group 0
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            float f[4], r[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (res) Group4<T>::unpack(*reinterpret_cast<const gvec *>(res + base + 8 * gq), r);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                f[q] = fmaxf(fmaf(acc[4 * gq + q], sc, sf) + r[q], floor_v);
            const gvec packed = Group4<T>::pack(f);
            if (sizeof(T) == 2 && vmode == 8)
                *reinterpret_cast<gvec *>(stage + lrow * kStageRow + (8 * gq + 4 * lhalf) * 2) = packed;
            else
                *reinterpret_cast<gvec *>(y + base + 8 * gq) = packed;
        }
        if (sizeof(T) == 2 && vmode == 8) {
            __builtin_amdgcn_wave_barrier();
            const int row = lane >> 2, g = lane & 3;
            const int b2 = (n0 * t.OC + oc0 + row) * t.OHW + rem0 + 8 * g;
#pragma unroll
            for (int it = 0; it < 2; ++it)
                *reinterpret_cast<uint4v *>(y + b2 + it * 16 * t.OHW) =
                    *reinterpret_cast<const uint4v *>(stage + (row + 16 * it) * kStageRow + g * 16);
            __builtin_amdgcn_wave_barrier();
        }
        return;
    }

    if constexpr (sizeof(T) == 2) {
        if (vmode == 1) {
            // Odd-sized maps (7x7 = 49 pixels): nothing is aligned, every element is stored on
            // its own.  In the accumulator layout a store instruction would scatter its 64
            // two-byte elements over 64 cache lines (measured: 2-4 us of tail on the 7x7
            // layers, the address unit taking a line per cycle); transposed through the
            // stage, its lanes write two channel rows of 32 adjacent pixels.  The residual
            // comes in the same way.
            const int px = lane & 31, rsel = lane >> 5;
            int n = n0, rem = rem0 + px;
            while (rem >= t.OHW) { rem -= t.OHW; ++n; }
            const bool pok = p0 + px < t.npix;
            const int rbase = (n * t.OC + oc0) * t.OHW + rem;        // (row 0, this lane's pixel)
            if (res) {
#pragma unroll
                for (int it = 0; it < 16; ++it) {
                    const int row = 2 * it + rsel;
                    T v = 0;
                    if (pok && oc0 + row < t.OC) v = res[rbase + row * t.OHW];
                    *reinterpret_cast<T *>(stage + row * kStageRow + px * 2) = v;
                }
                __builtin_amdgcn_wave_barrier();
            }
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                gvec *slot = reinterpret_cast<gvec *>(stage + lrow * kStageRow + (8 * gq + 4 * lhalf) * 2);
                float f[4], r[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                if (res) Group4<T>::unpack(*slot, r);
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    f[q] = fmaxf(fmaf(acc[4 * gq + q], sc, sf) + r[q], floor_v);
                *slot = Group4<T>::pack(f);
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int it = 0; it < 16; ++it) {
                const int row = 2 * it + rsel;
                if (pok && oc0 + row < t.OC)
                    y[rbase + row * t.OHW] = *reinterpret_cast<const T *>(stage + row * kStageRow + px * 2);
            }
            __builtin_amdgcn_wave_barrier();
            return;
        }
    }

    if (vmode == 1) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int pl = 8 * (v >> 2) + 4 * lhalf + (v & 3);
            if (oc < t.OC && p0 + pl < t.npix) {
                int n = n0, rem = rem0 + pl;
                while (rem >= t.OHW) { rem -= t.OHW; ++n; }
                const int idx = (n * t.OC + oc) * t.OHW + rem;
                float o = fmaf(acc[v], sc, sf);
                if (res) o += Elem<T>::load(res, idx);
                Elem<T>::store(y, idx, fmaxf(o, floor_v));
            }
        }
        return;
    }

#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
        const int pl = 8 * gq + 4 * lhalf;
        const bool ok = oc < t.OC && p0 + pl < t.npix;      // npix % 4 == 0: whole group or none
        int n = n0, rem = rem0 + pl;
        while (rem >= t.OHW) { rem -= t.OHW; ++n; }
        const int idx = ok ? (n * t.OC + oc) * t.OHW + rem : 0;
        float f[4], r[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (res && ok) Group4<T>::unpack(*reinterpret_cast<const gvec *>(res + idx), r);
#pragma unroll
        for (int q = 0; q < 4; ++q) f[q] = fmaxf(fmaf(acc[4 * gq + q], sc, sf) + r[q], floor_v);
        const gvec packed = Group4<T>::pack(f);
        if constexpr (sizeof(T) == 2) {
            if (vmode == 8) {
                *reinterpret_cast<gvec *>(stage + lrow * kStageRow + pl * 2) = packed;
                continue;
            }
        }
        if (ok) *reinterpret_cast<gvec *>(y + idx) = packed;
    }

    if constexpr (sizeof(T) == 2) {
        if (vmode == 8) {
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int task = it * 64 + lane;
                const int row = task >> 2, g = task & 3;
                const int c = oc0 + row, p = p0 + 8 * g;
                if (c < t.OC && p < t.npix) {
                    int n = n0, rem = rem0 + 8 * g;
                    while (rem >= t.OHW) { rem -= t.OHW; ++n; }
                    const int idx = (n * t.OC + c) * t.OHW + rem;
                    *reinterpret_cast<uint4v *>(y + idx) =
                        *reinterpret_cast<const uint4v *>(stage + row * kStageRow + g * 16);
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// All MI x NJ accumulator tiles of a wave (acc[i][j]: channel block i, pixel block j).
template <typename T, int MI, int NJ>
__device__ __forceinline__ void store_acc_tiles(const float16v (&acc)[MI][NJ], unsigned char *stage,
                                                int lane, int oc_base, int p_base,
                                                const TailArgs &t, int vmode, const float *ss,
                                                int row_base)
{
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            store_tile<T>(acc[i][j], stage, lane, oc_base + i * 32, p_base + j * 32, t, vmode, ss,
                          row_base + i * 32);
}

// The fast-path body of store_acc_tiles_batched: tile (i, j) starts at channel ocu + 32 i and
// at pixel rem0[j] of image n0[j]; everything is in range.  BT tiles share one LDS round trip.
template <int MI, int NJ, int BT, bool HAS_RES, bool NT>
__device__ __forceinline__ void store_fast_tiles(const float16v (&acc)[MI][NJ], unsigned char *stage,
                                                 int lane, int ocu, const int (&n0)[NJ],
                                                 const int (&rem0)[NJ], const TailArgs &t,
                                                 const float *ss, int row_base)
{
    constexpr int T = MI * NJ;
    // a short last batch would let the pair store below pick up a stale staged tile
    static_assert(T % BT == 0, "the batch size must divide the number of tiles of a wave");
    const int lrow = lane & 31, lhalf = lane >> 5;
    const float floor_v = (t.relu & 1) ? 0.0f : -INFINITY;
    const bf16_t *res = static_cast<const bf16_t *>(t.residual);
    bf16_t *y = static_cast<bf16_t *>(t.y);
    const int row = lane >> 2, g = lane & 3;
#pragma unroll
    for (int b0 = 0; b0 < T; b0 += BT) {
#pragma unroll
        for (int k = 0; k < BT; ++k) {
            // (the last batch may be short; clamped indices keep every subscript a constant)
            const int tix = b0 + k < T ? b0 + k : T - 1;
            const int i = tix / NJ, j = tix % NJ;
            if (b0 + k < T) {
                const float sc = ss[2 * (row_base + i * 32 + lrow)];
                const float sf = ss[2 * (row_base + i * 32 + lrow) + 1];
                unsigned char *st = stage + k * kStageBytes;
                const int base = (n0[j] * t.OC + ocu + i * 32 + lrow) * t.OHW + rem0[j] + 4 * lhalf;
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    float f[4], r[4];
                    if (HAS_RES)
                        Group4<bf16_t>::unpack(*reinterpret_cast<const uint2v *>(res + base + 8 * gq), r);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float v = fmaf(acc[i][j][4 * gq + q], sc, sf);
                        if (HAS_RES) v += r[q];
                        f[q] = fmaxf(v, floor_v);
                    }
                    *reinterpret_cast<uint2v *>(st + lrow * kStageRow + (8 * gq + 4 * lhalf) * 2) =
                        Group4<bf16_t>::pack(f);
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
        // Two staged tiles that are neighbours along the pixels (same channels, the next 32
        // pixels of the same image) leave together: eight lanes write the 128 contiguous bytes
        // of a channel row - a whole cache line when the map size is a multiple of 64 -
        // instead of two instructions writing half of it each.
        constexpr bool kPairs = BT % 2 == 0 && NJ % 2 == 0;
#pragma unroll
        for (int k = 0; k < BT; ++k) {
            const int tix = b0 + k < T ? b0 + k : T - 1;
            const int i = tix / NJ, j = tix % NJ;
            if constexpr (kPairs) {
                // (b0 and NJ even: tiles k, k + 1 of an even k share their channel block)
                const int jn = j + 1 < NJ ? j + 1 : j;
                if (k % 2 == 0 && n0[jn] == n0[j]) {
                    const int row8 = lane >> 3, g8 = lane & 7;
                    const unsigned char *st = stage + (k + (g8 >> 2)) * kStageBytes;
                    const int b2 = (n0[j] * t.OC + ocu + i * 32 + row8) * t.OHW + rem0[j] + 8 * g8;
#pragma unroll
                    for (int it = 0; it < 4; ++it)
                        stream_store<NT>(reinterpret_cast<uint4v *>(y + b2 + it * 8 * t.OHW),
                                         *reinterpret_cast<const uint4v *>(st + (row8 + 8 * it) * kStageRow + (g8 & 3) * 16));
                    continue;
                }
                if (k % 2 == 1 && n0[j] == n0[j - (j > 0 ? 1 : 0)]) continue;   // left with its neighbour
            }
            if (b0 + k < T) {
                const unsigned char *st = stage + k * kStageBytes;
                const int b2 = (n0[j] * t.OC + ocu + i * 32 + row) * t.OHW + rem0[j] + 8 * g;
#pragma unroll
                for (int it = 0; it < 2; ++it)
                    stream_store<NT>(reinterpret_cast<uint4v *>(y + b2 + it * 16 * t.OHW),
                                     *reinterpret_cast<const uint4v *>(st + (row + 16 * it) * kStageRow + g * 16));
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// store_acc_tiles for bf16 with BT*kStageBytes of wave-private LDS at `stage`: when every tile
// of the wave is on store_tile's fast path (mode 8, nothing ragged, each tile within one
// image) BT tiles at a time are converted and staged first and stored afterwards, so the LDS
// round trip and the store issue are paid once per batch instead of once per tile.
template <int MI, int NJ, int BT = MI * NJ>
__device__ __forceinline__ void store_acc_tiles_batched(const float16v (&acc)[MI][NJ],
                                                        unsigned char *stage, int lane, int oc_base,
                                                        int p_base, const TailArgs &t, int vmode,
                                                        const float *ss, int row_base)
{
    const int pbu = __builtin_amdgcn_readfirstlane(p_base);
    const int ocu = __builtin_amdgcn_readfirstlane(oc_base);
    bool fast = vmode == 8 && ocu + MI * 32 <= t.OC && pbu + NJ * 32 <= t.npix;
    int n0[NJ], rem0[NJ];
    n0[0] = pbu / t.OHW;
    rem0[0] = pbu - n0[0] * t.OHW;
    fast = fast && rem0[0] + 32 <= t.OHW;
#pragma unroll
    for (int j = 1; j < NJ; ++j) {
        // the previous tile ended inside its image, so this one starts at most at its end
        const bool wrap = rem0[j - 1] + 32 >= t.OHW;
        n0[j] = n0[j - 1] + (wrap ? 1 : 0);
        rem0[j] = wrap ? 0 : rem0[j - 1] + 32;
        fast = fast && rem0[j] + 32 <= t.OHW;
    }
    if (!fast) {
        store_acc_tiles<bf16_t, MI, NJ>(acc, stage, lane, oc_base, p_base, t, vmode, ss, row_base);
        return;
    }
    // the residual test is hoisted out: a branch per group would fence the tiles from each other
    // (so is the store hint, a compile-time property of the store instruction)
    const bool nt = (t.relu & 2) != 0;
    if (t.residual) {
        if (nt) store_fast_tiles<MI, NJ, BT, true, true>(acc, stage, lane, ocu, n0, rem0, t, ss, row_base);
        else store_fast_tiles<MI, NJ, BT, true, false>(acc, stage, lane, ocu, n0, rem0, t, ss, row_base);
    } else {
        if (nt) store_fast_tiles<MI, NJ, BT, false, true>(acc, stage, lane, ocu, n0, rem0, t, ss, row_base);
        else store_fast_tiles<MI, NJ, BT, false, false>(acc, stage, lane, ocu, n0, rem0, t, ss, row_base);
    }
}

// Host side: the store mode the problem allows (see store_tile).
inline int pick_store_vmode(int dtype, int OHW, const void *y, const void *residual)
{
    const bool aligned = reinterpret_cast<uintptr_t>(y) % 16 == 0 &&
                         reinterpret_cast<uintptr_t>(residual) % 16 == 0;
    if (!aligned) return 1;
    if (dtype == TVG_BF16 && OHW % 8 == 0) return 8;
    if (OHW % 4 == 0) return 4;
    return 1;
}

}  // namespace tvg
#endif
