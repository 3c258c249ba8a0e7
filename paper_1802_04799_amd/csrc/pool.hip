// 3x3 stride-2 pad-1 max-pool, NCHW.  Support operator for the ResNet-18 body
// (between the stem convolution and the first residual stage); padded taps are
// ignored.  One lane per output element, lanes contiguous along the output row.
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

}  // namespace

tvg_status launch_maxpool3x3s2(int N, int C, int H, int W, int dtype, const void *x, void *y,
                               hipStream_t stream)
{
    const int OH = (H - 1) / 2 + 1, OW = (W - 1) / 2 + 1;
    const int planes = N * C;
    // grid.z is limited to 65535 planes per launch; larger problems go in slices
    for (int p0 = 0; p0 < planes; p0 += 65535) {
        const int np = planes - p0 < 65535 ? planes - p0 : 65535;
        dim3 grid((OW + 63) / 64, (OH + 3) / 4, np);
        if (dtype == TVG_BF16)
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
