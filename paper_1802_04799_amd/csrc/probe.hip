// Measurement probes: what this GPU sustains, measured beside the operators in the same run.
//   tvg_probe_copy  a plain device copy with 16-byte accesses (the achievable HBM rate when the
//                   buffers exceed the caches)
//   tvg_probe_mfma  a register-resident loop of matrix instructions, nothing else: the achievable
//                   matrix rate at the clock the chip sustains under that load
// Neither is part of the operators; they give the denominators "achievable" next to the
// data-sheet peaks.
#include "tvg_device.h"
#include "tvg_internal.h"

namespace tvg {

namespace {

__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4v *__restrict__ src,
                                                        uint4v *__restrict__ dst, size_t words)
{
    // grid-stride, four independent 16-byte accesses in flight per lane
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < words; i += 4 * stride) {
        const uint4v a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        __builtin_nontemporal_store(a, dst + i);
        __builtin_nontemporal_store(b, dst + i + stride);
        __builtin_nontemporal_store(c, dst + i + 2 * stride);
        __builtin_nontemporal_store(d, dst + i + 3 * stride);
    }
    for (; i < words; i += stride) __builtin_nontemporal_store(src[i], dst + i);
}

// Four independent accumulator tiles per wave, so that consecutive matrix instructions never
// wait for each other; operands stay in registers.
template <int DTYPE>
__global__ __launch_bounds__(256) void probe_mfma_kernel(float *out, int iters)
{
    float16v acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
    const uint4v a = {threadIdx.x, 1u, 2u, 3u}, b = {4u, 5u, 6u, threadIdx.x};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if constexpr (DTYPE == TVG_BF16) {
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8v, a),
                                                                 __builtin_bit_cast(bf16x8v, b), acc[i], 0, 0, 0);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)      // 4 x (32x32x2): the flops of 32x32x8
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[e]) * 1e-30f,
                                                                  __uint_as_float(b[e]) * 1e-30f, acc[i], 0, 0, 0);
            }
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

}  // namespace tvg

extern "C" {

tvg_status tvg_probe_copy(const void *src, void *dst, size_t bytes, void *hip_stream)
{
    if (!src || !dst) return TVG_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0) return TVG_ERR_BAD_SHAPE;
    if (reinterpret_cast<uintptr_t>(src) % 16 != 0 || reinterpret_cast<uintptr_t>(dst) % 16 != 0)
        return TVG_ERR_UNSUPPORTED;
    const size_t words = bytes / 16;
    size_t blocks = (words + 4 * 256 - 1) / (4 * 256);
    const size_t cap = (size_t)tvg::kComputeUnits * 32;          // plenty of waves per CU, then stride
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(tvg::probe_copy_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const tvg::uint4v *>(src),
                       static_cast<tvg::uint4v *>(dst), words);
    return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
}

tvg_status tvg_probe_mfma(int32_t dtype, int32_t iters, int32_t workgroups, float *out,
                          double *flops, void *hip_stream)
{
    if (!out || !flops) return TVG_ERR_NULL;
    if (iters < 1 || workgroups < 1 || workgroups > 65536) return TVG_ERR_BAD_SHAPE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    double per_mfma_group;
    if (dtype == TVG_BF16) {
        per_mfma_group = 2.0 * 32 * 32 * 16;
        hipLaunchKernelGGL((tvg::probe_mfma_kernel<TVG_BF16>), dim3((unsigned)workgroups), dim3(256), 0,
                           stream, out, iters);
    } else if (dtype == TVG_F32) {
        per_mfma_group = 2.0 * 32 * 32 * 2 * 4;
        hipLaunchKernelGGL((tvg::probe_mfma_kernel<TVG_F32>), dim3((unsigned)workgroups), dim3(256), 0,
                           stream, out, iters);
    } else {
        return TVG_ERR_UNSUPPORTED;
    }
    *flops = per_mfma_group * 4.0 /*tiles*/ * 4.0 /*waves*/ * (double)iters * (double)workgroups;
    return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
}

}  // extern "C"
