// Depthwise fused 3x3 conv2d (TVM paper, Table 2 operators D1..D9, channel
// multiplier 1) as a bandwidth kernel: 18 FLOP per output against 8 bytes of
// compulsory traffic, so the vector ALUs suffice and the matrix cores are not
// used.  There is no reduction across lanes: each output sums its own 9 taps.
//
// One workgroup owns PT channel planes x RT output rows (full width).  It
// stages the haloed input rows of its planes in LDS with zero borders
// (coalesced along the row; Section 4.2's cooperative fetch), so the compute
// phase has no bounds checks; each lane then walks a column strip of 4 output
// rows, re-using the 3 input rows shared by vertically adjacent outputs, and
// stores row segments that are contiguous across lanes.  The fused tail
// (Section 3, operator fusion) is applied in registers.
#include "tvg_device.h"
#include "tvg_internal.h"

namespace tvg {

namespace {

struct DwArgs {
    const void *x, *w;
    const float *scale, *shift, *bias;
    const void *residual;
    void *y;
    int planes, C, H, W, OH, OW;
    int PT, RT, row_tiles;     // planes per workgroup, output rows per workgroup (4 << k)
    int strips_log2;           // log2(RT / 4)
    int wp_log2, ow_log2;      // log2 of (W + 2) and OW rounded up to a power of two
    int relu;
};

constexpr int kStrip = 4;      // output rows per lane
constexpr int kPrm = 12;       // per-plane parameters in LDS: 9 taps, scale, shift, bias

template <typename T, int STRIDE>
__global__ __launch_bounds__(256) void dwconv3x3_kernel(const DwArgs a)
{
    extern __shared__ float smem[];
    const int IR = (a.RT - 1) * STRIDE + 3;     // staged input rows per plane
    const int WP = a.W + 2;                     // staged row length, one zero column each side
    const int per_plane = IR * WP;
    float *tile = smem;
    float *prm = smem + a.PT * per_plane;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ptile = blockIdx.x / a.row_tiles, rtile = blockIdx.x - ptile * a.row_tiles;
    const int p0 = ptile * a.PT;
    const int np = min(a.PT, a.planes - p0);
    const int oh0 = rtile * a.RT;
    const int ih_base = oh0 * STRIDE - 1;
    const T *__restrict__ xg = static_cast<const T *>(a.x);
    const T *__restrict__ wg = static_cast<const T *>(a.w);

    // ---- stage the haloed rows: lanes run along a row, several short rows per pass ------
    {
        const int wpr = 1 << a.wp_log2;
        const int rows_per_pass = wpr >= 64 ? 1 : 64 >> a.wp_log2;
        const int col_passes = wpr >= 64 ? (wpr >> 6) : 1;
        const int rsub = wpr >= 64 ? 0 : lane >> a.wp_log2;
        const int col0 = wpr >= 64 ? lane : lane & (wpr - 1);
        for (int p = 0; p < np; ++p) {
            const T *plane = xg + (size_t)(p0 + p) * a.H * a.W;
            float *dst = tile + p * per_plane;
            for (int row = wave * rows_per_pass + rsub; row < IR; row += 4 * rows_per_pass) {
                const int ih = ih_base + row;
                const bool rok = ih >= 0 && ih < a.H;
                for (int cp = 0; cp < col_passes; ++cp) {
                    const int col = col0 + (cp << 6);
                    if (col < WP) {
                        const int iw = col - 1;
                        const bool ok = rok && iw >= 0 && iw < a.W;
                        const float v = Elem<T>::load(plane, ok ? ih * a.W + iw : 0);
                        dst[row * WP + col] = ok ? v : 0.0f;
                    }
                }
            }
        }
        for (int l = tid; l < np * kPrm; l += 256) {
            const int p = l / kPrm, e = l - p * kPrm;
            const int c = (p0 + p) % a.C;
            float v;
            if (e < 9) v = Elem<T>::load(wg, c * 9 + e);
            else if (e == 9) v = a.scale[c];
            else if (e == 10) v = a.shift[c];
            else v = a.bias ? a.bias[c] : 0.0f;
            prm[l] = v;
        }
    }
    __syncthreads();

    // ---- compute: lane = output column, 4 output rows per lane -------------------------
    const T *res = static_cast<const T *>(a.residual);
    T *yg = static_cast<T *>(a.y);
    const int owr = 1 << a.ow_log2;
    const int pairs_per_pass = owr >= 64 ? 1 : 64 >> a.ow_log2;
    const int col_passes = owr >= 64 ? (owr >> 6) : 1;
    const int sub = owr >= 64 ? 0 : lane >> a.ow_log2;
    const int ow0 = owr >= 64 ? lane : lane & (owr - 1);
    const int npairs = np << a.strips_log2;                 // (plane, strip) pairs
    constexpr int ROWS = (kStrip - 1) * STRIDE + 3;
    for (int q = wave * pairs_per_pass + sub; q < npairs; q += 4 * pairs_per_pass) {
        const int p = q >> a.strips_log2;
        const int orow0 = (q - (p << a.strips_log2)) * kStrip;
        const float *pp = prm + p * kPrm;
        float wt[9];
#pragma unroll
        for (int e = 0; e < 9; ++e) wt[e] = pp[e];
        const float scale = pp[9], shift = pp[10], bias = pp[11];
        for (int cp = 0; cp < col_passes; ++cp) {
            const int ow = ow0 + (cp << 6);
            if (ow >= a.OW) continue;
            const float *src = tile + p * per_plane + orow0 * STRIDE * WP + ow * STRIDE;
            float acc[kStrip] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int rr = 0; rr < ROWS; ++rr) {
                const float v0 = src[rr * WP], v1 = src[rr * WP + 1], v2 = src[rr * WP + 2];
#pragma unroll
                for (int o = 0; o < kStrip; ++o) {
                    const int r = rr - o * STRIDE;
                    if (r >= 0 && r < 3)
                        acc[o] += v0 * wt[r * 3] + v1 * wt[r * 3 + 1] + v2 * wt[r * 3 + 2];
                }
            }
#pragma unroll
            for (int o = 0; o < kStrip; ++o) {
                const int oh = oh0 + orow0 + o;
                if (oh < a.OH) {
                    const int idx = ((p0 + p) * a.OH + oh) * a.OW + ow;
                    fused_tail_store<T>(acc[o], scale, shift, bias, res, yg, idx, a.relu != 0);
                }
            }
        }
    }
}

int ceil_log2(int v)
{
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

}  // namespace

tvg_status launch_dwconv3x3(const ConvProblem &p, const ConvPointers &ptr, hipStream_t stream)
{
    DwArgs a;
    a.x = ptr.x; a.w = ptr.w; a.scale = ptr.scale; a.shift = ptr.shift; a.bias = ptr.bias;
    a.residual = ptr.residual; a.y = ptr.y;
    a.planes = p.N * p.IC; a.C = p.IC; a.H = p.H; a.W = p.W; a.OH = p.OH; a.OW = p.OW;
    a.relu = p.relu;
    const int stride = p.sh;

    // Output rows per workgroup: 4 << k, the smallest that covers OH, capped at 16.
    int rt = kStrip;
    while (rt < p.OH && rt < 16) rt <<= 1;
    const long total = (long)a.planes * p.OH * p.OW;
    long target = total / 1024;                 // outputs per workgroup: aim at >= 1024 workgroups
    if (target < 256) target = 256;
    if (target > 2048) target = 2048;
    // shrink the row band of large planes towards the target
    while (rt > kStrip && (long)rt * p.OW > target) rt >>= 1;
    const int ir = (rt - 1) * stride + 3, wp = p.W + 2;
    int pt = (int)(target / ((long)rt * p.OW));
    if (pt < 1) pt = 1;
    if (pt > a.planes) pt = a.planes;
    const size_t lds_cap = 48 * 1024;
    while (pt > 1 && (size_t)pt * (ir * wp + kPrm) * sizeof(float) > lds_cap) --pt;
    const size_t lds_bytes = (size_t)pt * (ir * wp + kPrm) * sizeof(float);
    if (lds_bytes > 64 * 1024) return TVG_ERR_UNSUPPORTED;   // a single row band does not fit

    a.PT = pt; a.RT = rt;
    a.row_tiles = (p.OH + rt - 1) / rt;
    a.strips_log2 = ceil_log2(rt / kStrip);
    a.wp_log2 = ceil_log2(wp);
    a.ow_log2 = ceil_log2(p.OW);
    const unsigned grid = (unsigned)(((a.planes + pt - 1) / pt) * a.row_tiles);

    if (p.dtype == TVG_BF16) {
        if (stride == 1)
            hipLaunchKernelGGL((dwconv3x3_kernel<bf16_t, 1>), dim3(grid), dim3(256), lds_bytes, stream, a);
        else
            hipLaunchKernelGGL((dwconv3x3_kernel<bf16_t, 2>), dim3(grid), dim3(256), lds_bytes, stream, a);
    } else {
        if (stride == 1)
            hipLaunchKernelGGL((dwconv3x3_kernel<float, 1>), dim3(grid), dim3(256), lds_bytes, stream, a);
        else
            hipLaunchKernelGGL((dwconv3x3_kernel<float, 2>), dim3(grid), dim3(256), lds_bytes, stream, a);
    }
    return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
}

}  // namespace tvg
