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
// A 32x32 fp32 accumulator tile (rows = output channels, columns = consecutive
// output pixels) leaves the MFMA with one pixel per lane, which would mean one
// 2- or 4-byte store per value.  Instead the wave transposes the tile through a
// private 32 x 36 float staging area in LDS so that each lane owns V consecutive
// pixels of one channel, applies the fused tail to them and moves residual and y
// as 8- or 16-byte vectors (64 contiguous bytes or more per channel row).
// V consecutive pixels starting at a multiple of V lie in one image and are
// contiguous and aligned in NCHW exactly when OH*OW is a multiple of V; the
// caller selects V accordingly (V = 1: no staging, direct stores).
// ---------------------------------------------------------------------------------------
struct TailArgs {
    const float *scale, *shift, *bias;
    const void *residual;
    void *y;
    int OC, OHW, npix, relu;
};

constexpr int kStageStride = 36;                       // floats per staged row (32 + 4 padding)
constexpr int kStageFloats = 32 * kStageStride;        // per wave

// Puts the per-channel multiplier and offset of a tile's `rows` output channels into LDS as
// (scale, bias*scale + shift) pairs, so the epilogue reads them with LDS latency instead of
// issuing dependent global loads per store.  (acc + bias)*scale + shift == acc*scale + that
// offset.  Call before a barrier that precedes the first staged store.
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

template <typename T, int V> struct VecIO;
template <> struct VecIO<bf16_t, 8> {
    typedef uint4v vec;
    static __device__ __forceinline__ void unpack(const vec &r, float *f)
    {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            f[2 * q] = __uint_as_float(r[q] << 16);
            f[2 * q + 1] = __uint_as_float(r[q] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ vec pack(const float *f)
    {
        vec r;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            r[q] = f32x2_to_bf16x2(f[2 * q], f[2 * q + 1]);
        return r;
    }
};
template <> struct VecIO<bf16_t, 4> {
    typedef uint32_t vec __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ void unpack(const vec &r, float *f)
    {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            f[2 * q] = __uint_as_float(r[q] << 16);
            f[2 * q + 1] = __uint_as_float(r[q] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ vec pack(const float *f)
    {
        vec r;
#pragma unroll
        for (int q = 0; q < 2; ++q)
            r[q] = f32x2_to_bf16x2(f[2 * q], f[2 * q + 1]);
        return r;
    }
};
template <> struct VecIO<float, 4> {
    typedef float4v vec;
    static __device__ __forceinline__ void unpack(const vec &r, float *f)
    {
#pragma unroll
        for (int q = 0; q < 4; ++q) f[q] = r[q];
    }
    static __device__ __forceinline__ vec pack(const float *f) { return vec{f[0], f[1], f[2], f[3]}; }
};

// acc: one 32x32 MFMA accumulator tile (value v of lane l = row 8*(v/4) + 4*(l/32) + v%4,
// column l%32).  oc0 / p0: output channel of row 0 / flattened pixel of column 0.
// ss: staged (scale, offset) pairs of the workgroup tile, row0: row of oc0 inside that tile.
template <typename T, int V>
__device__ __forceinline__ void store_tile_staged(const float16v &acc, float *stage, int lane,
                                                  int oc0, int p0, const TailArgs &t,
                                                  const float *ss, int row0)
{
    typedef typename VecIO<T, V>::vec vec;
    const int lrow = lane & 31, lhalf = lane >> 5;
#pragma unroll
    for (int v = 0; v < 16; ++v)
        stage[(8 * (v >> 2) + 4 * lhalf + (v & 3)) * kStageStride + lrow] = acc[v];
    __builtin_amdgcn_wave_barrier();
    constexpr int G = 32 / V;                      // lane groups per row
    // image index of the tile's first pixel: uniform, so one scalar division; a tile of 32
    // pixels crosses into later images by repeated subtraction (at most once for OH*OW >= 32)
    const int p0u = __builtin_amdgcn_readfirstlane(p0);
    const int n0 = p0u / t.OHW, rem0 = p0u - n0 * t.OHW;
#pragma unroll
    for (int it = 0; it < 32 * G / 64; ++it) {
        const int task = it * 64 + lane;
        const int row = task / G, g = task - row * G;
        const int oc = oc0 + row, p = p0 + g * V;
        if (oc < t.OC && p < t.npix) {
            int n = n0, rem = rem0 + g * V;
            while (rem >= t.OHW) { rem -= t.OHW; ++n; }
            const size_t idx = (size_t)(n * t.OC + oc) * t.OHW + rem;
            const float sc = ss[2 * (row0 + row)], sf = ss[2 * (row0 + row) + 1];
            float f[V], r[V];
#pragma unroll
            for (int q = 0; q < V; ++q) {
                f[q] = stage[row * kStageStride + g * V + q];
                r[q] = 0.0f;
            }
            if (t.residual)
                VecIO<T, V>::unpack(*reinterpret_cast<const vec *>(static_cast<const T *>(t.residual) + idx), r);
            // no per-element selects: a missing residual adds zeros, a missing ReLU clamps
            // at minus infinity
            const float floor_v = t.relu ? 0.0f : -INFINITY;
#pragma unroll
            for (int q = 0; q < V; ++q) f[q] = fmaxf(fmaf(f[q], sc, sf) + r[q], floor_v);
            *reinterpret_cast<vec *>(static_cast<T *>(t.y) + idx) = VecIO<T, V>::pack(f);
        }
    }
    __builtin_amdgcn_wave_barrier();
}

// Direct (unstaged) stores of one accumulator tile: any OH*OW, any alignment.
template <typename T>
__device__ __forceinline__ void store_tile_direct(const float16v &acc, int lane, int oc0, int p0,
                                                  const TailArgs &t)
{
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int p = p0 + lrow;
    if (p >= t.npix) return;
    const int n = p / t.OHW, rem = p - n * t.OHW;
    const int obase = n * t.OC * t.OHW + rem;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int oc = oc0 + 8 * (v >> 2) + 4 * lhalf + (v & 3);
        if (oc >= t.OC) continue;
        fused_tail_store<T>(acc[v], t.scale[oc], t.shift[oc], t.bias ? t.bias[oc] : 0.0f,
                            static_cast<const T *>(t.residual), static_cast<T *>(t.y),
                            obase + oc * t.OHW, t.relu != 0);
    }
}

// vmode: pixels per vector store (8, 4) or 1 for direct stores; chosen on the host.
template <typename T>
__device__ __forceinline__ void store_tile(const float16v &acc, float *stage, int lane, int oc0,
                                           int p0, const TailArgs &t, int vmode, const float *ss,
                                           int row0)
{
    if constexpr (sizeof(T) == 2) {
        if (vmode == 8) return store_tile_staged<bf16_t, 8>(acc, stage, lane, oc0, p0, t, ss, row0);
        if (vmode == 4) return store_tile_staged<bf16_t, 4>(acc, stage, lane, oc0, p0, t, ss, row0);
    } else {
        if (vmode == 4) return store_tile_staged<float, 4>(acc, stage, lane, oc0, p0, t, ss, row0);
    }
    store_tile_direct<T>(acc, lane, oc0, p0, t);
}

// All MI x NJ accumulator tiles of a wave, one after the other through ONE copy of the
// store code: the loop is kept rolled and the tile is picked by uniform selects, because
// inlining the epilogue per tile multiplies the code size and the kernels' hot loops then
// no longer fit the instruction cache.
template <typename T, int MI, int NJ>
__device__ __forceinline__ void store_acc_tiles(const float16v (&acc)[MI][NJ], float *stage,
                                                int lane, int oc_base, int p_base,
                                                const TailArgs &t, int vmode, const float *ss,
                                                int row_base)
{
#pragma unroll 1
    for (int k = 0; k < MI * NJ; ++k) {
        float16v cur = acc[0][0];
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                if (i * NJ + j == k) cur = acc[i][j];
        const int i = k / NJ, j = k - i * NJ;
        store_tile<T>(cur, stage, lane, oc_base + i * 32, p_base + j * 32, t, vmode, ss,
                      row_base + i * 32);
    }
}

// Host side: widest staged store the problem allows.
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
