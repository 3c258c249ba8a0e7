// 3x3 stride-2 pad-1 max-pool, NCHW.  Support operator for the ResNet-18 body
// (between the stem convolution and the first residual stage); padded taps are
// ignored.  bf16 maps with rows of a multiple of 8 pixels: a lane computes four adjacent outputs
// from three 16-byte row loads (the ResNet-18 pool at batch 32, 51 MB in and 13 MB out: 45 us
// with one lane per output, nine 2-byte loads each).  Everything else: one lane per output
// element, lanes contiguous along the output row.
#include "tvg_device.h"
#include "tvg_internal.h"

namespace tvg {

namespace {

template <typename T>
__global__ __launch_bounds__(256) void maxpool3x3s2_kernel(const T *__restrict__ x, T *__restrict__ y,
                                                          int planes, int H, int W, int OH, int OW)
{
    const int ow = blockIdx.x * 64 + (threadIdx.x & 63);
    const int oh = blockIdx.y * 4 + (threadIdx.x >> 6);
    const int plane = blockIdx.z;
    if (ow >= OW || oh >= OH) return;
    const T *src = x + (size_t)plane * H * W;
    float best = -INFINITY;
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int ih = oh * 2 - 1 + r;
        if (ih < 0 || ih >= H) continue;
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            const int iw = ow * 2 - 1 + s;
            if (iw < 0 || iw >= W) continue;
            best = fmaxf(best, Elem<T>::load(src, ih * W + iw));
        }
    }
    Elem<T>::store(y + (size_t)plane * OH * OW, oh * OW + ow, best);
}

// Four outputs per lane; grid.y = plane, lanes run over (output row, group of four outputs).
__global__ __launch_bounds__(256) void maxpool3x3s2_bf16x4_kernel(const bf16_t *__restrict__ x,
                                                                 bf16_t *__restrict__ y, int H, int W,
                                                                 int OH, int OW, float inv_qw)
{
    const int QW = OW >> 2;
    const int g = blockIdx.x * 256 + threadIdx.x;
    if (g >= OH * QW) return;
    int q;
    const int oh = fast_div(g, QW, inv_qw, &q);
    const bf16_t *src = x + (size_t)blockIdx.y * H * W + 8 * q;     // input column 2 * (4 q)
    float m[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int ih = oh * 2 - 1 + r;
        if (ih < 0 || ih >= H) continue;
        const bf16_t *row = src + ih * W;
        const uint4v v = *reinterpret_cast<const uint4v *>(row);    // columns 8q .. 8q + 7
        float px[9];
        px[0] = q > 0 ? bf16_to_f32(row[-1]) : -INFINITY;           // column 8q - 1
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            px[1 + 2 * k] = __uint_as_float(v[k] << 16);
            px[2 + 2 * k] = __uint_as_float(v[k] & 0xFFFF0000u);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) m[j] = fmaxf(m[j], fmaxf(px[2 * j], fmaxf(px[2 * j + 1], px[2 * j + 2])));
    }
    // the maximum is one of the inputs: its upper half is the bf16 value, exactly
    uint2v out;
    out[0] = (__float_as_uint(m[0]) >> 16) | (__float_as_uint(m[1]) & 0xFFFF0000u);
    out[1] = (__float_as_uint(m[2]) >> 16) | (__float_as_uint(m[3]) & 0xFFFF0000u);
    *reinterpret_cast<uint2v *>(y + ((size_t)blockIdx.y * OH + oh) * OW + 4 * q) = out;
}

}  // namespace

tvg_status launch_maxpool3x3s2(int N, int C, int H, int W, int dtype, const void *x, void *y,
                               hipStream_t stream)
{
    const int OH = (H - 1) / 2 + 1, OW = (W - 1) / 2 + 1;
    const int planes = N * C;
    // grid.z is limited to 65535 planes per launch; larger problems go in slices
    const bool vec4 = dtype == TVG_BF16 && W % 8 == 0 && OH * (OW / 4) < (1 << 22) &&
                      reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(y) % 8 == 0;
    for (int p0 = 0; p0 < planes; p0 += 65535) {
        const int np = planes - p0 < 65535 ? planes - p0 : 65535;
        dim3 grid((OW + 63) / 64, (OH + 3) / 4, np);
        if (vec4)
            hipLaunchKernelGGL(maxpool3x3s2_bf16x4_kernel, dim3((OH * (OW / 4) + 255) / 256, np), dim3(256),
                               0, stream, static_cast<const bf16_t *>(x) + (size_t)p0 * H * W,
                               static_cast<bf16_t *>(y) + (size_t)p0 * OH * OW, H, W, OH, OW,
                               1.0f / (float)(OW / 4));
        else if (dtype == TVG_BF16)
            hipLaunchKernelGGL((maxpool3x3s2_kernel<bf16_t>), grid, dim3(256), 0, stream,
                               static_cast<const bf16_t *>(x) + (size_t)p0 * H * W,
                               static_cast<bf16_t *>(y) + (size_t)p0 * OH * OW, np, H, W, OH, OW);
        else
            hipLaunchKernelGGL((maxpool3x3s2_kernel<float>), grid, dim3(256), 0, stream,
                               static_cast<const float *>(x) + (size_t)p0 * H * W,
                               static_cast<float *>(y) + (size_t)p0 * OH * OW, np, H, W, OH, OW);
        if (hipGetLastError() != hipSuccess) return TVG_ERR_LAUNCH;
    }
    return TVG_OK;
}

}  // namespace tvg
