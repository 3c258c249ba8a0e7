// Device-side helpers shared by the libtvg kernels: element types, bf16
// conversion and the fused element-wise tail.
#ifndef TVG_DEVICE_H
#define TVG_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tvg {

typedef uint16_t bf16_t;   // raw bfloat16 bits

typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(uint32_t(b) << 16); }

// fp32 -> bf16, round to nearest, ties to even (finite inputs).
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return bf16_t(u >> 16);
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

}  // namespace tvg
#endif
