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

// Register-blocked variant for fp32 planes whose rows are multiples of four: no LDS.
// A lane computes a block of RB (4, 2 or 1) output rows x 4 output columns of one plane; every input
// row of the block is read as 16-byte vectors plus the halo scalars, re-used in registers
// by the (up to three) output rows that need it, and each output row leaves as one 16-byte
// store.  Neighbouring lanes read neighbouring vectors of the same row; the overlap
// between blocks (halo rows and columns) is served by the caches.
struct DwDirectArgs {
    const float *x, *w;
    const float *scale, *shift, *bias;
    const float *residual;
    float *y;
    int C, H, W, OH, OW;
    int CB;            // 4-column blocks per output row
    int tpp;           // lane tasks per plane: row blocks x CB
    int total;         // tasks in total
    float inv_cb;
    int relu;
};



template <int STRIDE, bool NT, int RB = 4>
__global__ __launch_bounds__(256) void dwconv3x3_direct_kernel(const DwDirectArgs a)
{
    const int g = blockIdx.x * 256 + threadIdx.x;
    if (g >= a.total) return;
    const int plane = g / a.tpp;
    int cb;
    const int rb = fast_div(g - plane * a.tpp, a.CB, a.inv_cb, &cb);
    const int c = plane % a.C;
    const int oh0 = rb * RB, ow0 = cb * 4;
    const int H = a.H, W = a.W;
    const float *__restrict__ xp = a.x + (size_t)plane * H * W;

    float wt[9];
#pragma unroll
    for (int e = 0; e < 9; ++e) wt[e] = a.w[c * 9 + e];
    const float sc = a.scale[c];
    const float sf = a.bias ? fmaf(a.bias[c], sc, a.shift[c]) : a.shift[c];

    constexpr int IR = (RB - 1) * STRIDE + 3;        // input rows of the block
    constexpr int NV = 3 * STRIDE + 3;                // input columns of the block
    float acc[RB][4];
#pragma unroll
    for (int o = 0; o < RB; ++o)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[o][q] = 0.0f;

    const int iw0 = ow0 * STRIDE;                     // first in-image column of the vectors
#pragma unroll
    for (int rr = 0; rr < IR; ++rr) {
        // A padding row is read from the nearest image row and replaced by zeros: with no
        // branch around the loads all rows of the block are in flight at once (one memory round
        // trip per lane instead of one per row, which is what a launch of few waves waits for).
        const int ih = oh0 * STRIDE - 1 + rr;
        const bool rowok = ih >= 0 && ih < H;
        const float *row = xp + min(max(ih, 0), H - 1) * W + iw0;
        float v[NV];                                  // columns iw0 - 1 .. iw0 + NV - 2
        v[0] = iw0 > 0 ? row[-1] : 0.0f;
        const float4v m0 = *reinterpret_cast<const float4v *>(row);
        v[1] = m0[0]; v[2] = m0[1]; v[3] = m0[2]; v[4] = m0[3];
        if (STRIDE == 1) {
            v[5] = iw0 + 4 < W ? row[4] : 0.0f;
        } else {
            const float4v m1 = *reinterpret_cast<const float4v *>(row + 4);
            v[5] = m1[0]; v[6] = m1[1]; v[7] = m1[2]; v[8] = m1[3];
        }
#pragma unroll
        for (int e = 0; e < NV; ++e) v[e] = rowok ? v[e] : 0.0f;
#pragma unroll
        for (int o = 0; o < RB; ++o) {
            const int r = rr - o * STRIDE;
            if (r < 0 || r > 2) continue;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                acc[o][q] += v[q * STRIDE] * wt[r * 3] + v[q * STRIDE + 1] * wt[r * 3 + 1] +
                             v[q * STRIDE + 2] * wt[r * 3 + 2];
        }
    }

    const float floor_v = a.relu ? 0.0f : -INFINITY;
#pragma unroll
    for (int o = 0; o < RB; ++o) {
        const int oh = oh0 + o;
        if (oh >= a.OH) continue;
        const size_t idx = ((size_t)plane * a.OH + oh) * a.OW + ow0;
        float4v r = {0.0f, 0.0f, 0.0f, 0.0f};
        if (a.residual) r = *reinterpret_cast<const float4v *>(a.residual + idx);
        float4v out;
#pragma unroll
        for (int q = 0; q < 4; ++q) out[q] = fmaxf(fmaf(acc[o][q], sc, sf) + r[q], floor_v);
        stream_store<NT>(reinterpret_cast<float4v *>(a.y + idx), out);
    }
}

// The same register blocking for bf16 planes: a lane computes 4 output rows x CW output
// columns (CW = 8 or 4, the output row must be a multiple of it).  An input row of the block
// is CW * STRIDE pixels in one or two vector loads of 8 or 16 bytes plus the halo pixel(s);
// an output row leaves as one 16- or 8-byte store.  Sums are fp32, as everywhere.
struct DwDirectBf16Args {
    const bf16_t *x, *w;
    const float *scale, *shift, *bias;
    const bf16_t *residual;
    bf16_t *y;
    int C, H, W, OH, OW;
    int CB;            // column blocks per output row
    int tpp;           // lane tasks per plane: row blocks x CB
    int total;         // tasks in total
    float inv_cb;
    int relu;
};

template <int STRIDE, int CW, bool NT, int RB = 4>
__global__ __launch_bounds__(256) void dwconv3x3_direct_bf16_kernel(const DwDirectBf16Args a)
{
    const int g = blockIdx.x * 256 + threadIdx.x;
    if (g >= a.total) return;
    const int plane = g / a.tpp;
    int cb;
    const int rb = fast_div(g - plane * a.tpp, a.CB, a.inv_cb, &cb);
    const int c = plane % a.C;
    const int oh0 = rb * RB, ow0 = cb * CW;
    const int H = a.H, W = a.W;
    const bf16_t *__restrict__ xp = a.x + (size_t)plane * H * W;

    float wt[9];
#pragma unroll
    for (int e = 0; e < 9; ++e) wt[e] = bf16_to_f32(a.w[c * 9 + e]);
    const float sc = a.scale[c];
    const float sf = a.bias ? fmaf(a.bias[c], sc, a.shift[c]) : a.shift[c];

    constexpr int IR = (RB - 1) * STRIDE + 3;        // input rows of the block
    constexpr int NIN = CW * STRIDE;                  // input pixels fetched as vectors
    constexpr int NW = NIN / 2;                       // ... in 4-byte words
    constexpr int NV = NIN + 2;                       // columns iw0 - 1 .. iw0 + NIN
    float acc[RB][CW];
#pragma unroll
    for (int o = 0; o < RB; ++o)
#pragma unroll
        for (int q = 0; q < CW; ++q) acc[o][q] = 0.0f;

    const int iw0 = ow0 * STRIDE;
#pragma unroll
    for (int rr = 0; rr < IR; ++rr) {
        // (the branch stays here: hoisting all rows of a block, up to 9 x 18 pixels, costs this
        // kernel more in occupancy than the serial round trips do - 14 -> 18 us on the 112x112
        // MobileNet layers at batch 32 - where the fp32 kernel above gains 12-20 %)
        const int ih = oh0 * STRIDE - 1 + rr;
        if (ih < 0 || ih >= H) continue;              // a padding row contributes nothing
        const bf16_t *row = xp + ih * W + iw0;
        uint32_t wd[NW];
        if (NW == 2) {
            const uint2v m = *reinterpret_cast<const uint2v *>(row);
            wd[0] = m[0]; wd[1] = m[1];
        } else {
#pragma unroll
            for (int k = 0; k < NW / 4; ++k) {
                const uint4v m = reinterpret_cast<const uint4v *>(row)[k];
#pragma unroll
                for (int e = 0; e < 4; ++e) wd[4 * k + e] = m[e];
            }
        }
        float v[NV];
        v[0] = iw0 > 0 ? bf16_to_f32(row[-1]) : 0.0f;
#pragma unroll
        for (int k = 0; k < NW; ++k) {
            v[1 + 2 * k] = __uint_as_float(wd[k] << 16);
            v[2 + 2 * k] = __uint_as_float(wd[k] & 0xFFFF0000u);
        }
        if (STRIDE == 1) v[NV - 1] = iw0 + NIN < W ? bf16_to_f32(row[NIN]) : 0.0f;
#pragma unroll
        for (int o = 0; o < RB; ++o) {
            const int r = rr - o * STRIDE;
            if (r < 0 || r > 2) continue;
#pragma unroll
            for (int q = 0; q < CW; ++q)
                acc[o][q] += v[q * STRIDE] * wt[r * 3] + v[q * STRIDE + 1] * wt[r * 3 + 1] +
                             v[q * STRIDE + 2] * wt[r * 3 + 2];
        }
    }

    typedef uint32_t outv __attribute__((ext_vector_type(CW / 2)));
    const float floor_v = a.relu ? 0.0f : -INFINITY;
#pragma unroll
    for (int o = 0; o < RB; ++o) {
        const int oh = oh0 + o;
        if (oh >= a.OH) continue;
        const size_t idx = ((size_t)plane * a.OH + oh) * a.OW + ow0;
        outv r;
#pragma unroll
        for (int k = 0; k < CW / 2; ++k) r[k] = 0u;
        if (a.residual) r = *reinterpret_cast<const outv *>(a.residual + idx);
        outv out;
#pragma unroll
        for (int k = 0; k < CW / 2; ++k) {
            const float lo = fmaxf(fmaf(acc[o][2 * k], sc, sf) + __uint_as_float(r[k] << 16), floor_v);
            const float hi = fmaxf(fmaf(acc[o][2 * k + 1], sc, sf) + __uint_as_float(r[k] & 0xFFFF0000u),
                                   floor_v);
            out[k] = f32x2_to_bf16x2(lo, hi);
        }
        stream_store<NT>(reinterpret_cast<outv *>(a.y + idx), out);
    }
}

template <int STRIDE, int CW, int RB>
void launch_direct_bf16_rb(const DwDirectBf16Args &d, bool nt, unsigned blocks, hipStream_t stream)
{
    if (nt)
        hipLaunchKernelGGL((dwconv3x3_direct_bf16_kernel<STRIDE, CW, true, RB>), dim3(blocks), dim3(256), 0,
                           stream, d);
    else
        hipLaunchKernelGGL((dwconv3x3_direct_bf16_kernel<STRIDE, CW, false, RB>), dim3(blocks), dim3(256), 0,
                           stream, d);
}

template <int STRIDE, int CW>
void launch_direct_bf16(const DwDirectBf16Args &d, int rb, bool nt, unsigned blocks, hipStream_t stream)
{
    if (rb == 2) launch_direct_bf16_rb<STRIDE, CW, 2>(d, nt, blocks, stream);
    else launch_direct_bf16_rb<STRIDE, CW, 4>(d, nt, blocks, stream);
}

// Variant for small planes (at most 256 outputs per plane: 14x14 and 7x7 maps).  A
// workgroup copies PG whole planes, which are one contiguous run of memory, into LDS (as
// fp32) with 16-byte loads and no per-element index arithmetic; every lane then keeps ONE
// output position (oh, ow) for the whole kernel, with its nine tap offsets and in-image
// mask computed once, and walks over the planes of the group.
struct DwSmallArgs {
    const void *x, *w;
    const float *scale, *shift, *bias;
    const void *residual;
    void *y;
    int planes, C, H, W, OH, OW, PG, relu;
};

template <typename T, int STRIDE, bool NT>
__global__ __launch_bounds__(256) void dwconv3x3_smallplane_kernel(const DwSmallArgs a)
{
    extern __shared__ float smem[];
    const int HW = a.H * a.W, OHW = a.OH * a.OW;
    float *tile = smem;                   // [PG][H*W]
    float *prm = smem + a.PG * HW;        // [PG][12]: 9 taps, scale, offset, unused
    const int tid = threadIdx.x;
    const int p0 = blockIdx.x * a.PG;
    const int np = min(a.PG, a.planes - p0);
    const T *__restrict__ wg = static_cast<const T *>(a.w);

    // ---- copy the planes: contiguous, 16-byte aligned start (PG * sizeof(T) is a multiple of 16)
    const T *src = static_cast<const T *>(a.x) + (size_t)p0 * HW;
    const int nelem = np * HW;
    constexpr int VE = 16 / sizeof(T);    // elements per 16-byte vector
    const int nvec = nelem / VE;
    for (int i = tid; i < nvec; i += 256) {
        if (sizeof(T) == 4) {
            reinterpret_cast<float4v *>(tile)[i] = reinterpret_cast<const float4v *>(src)[i];
        } else {
            const uint4v m = reinterpret_cast<const uint4v *>(src)[i];
            float4v lo, hi;
            lo[0] = __uint_as_float(m[0] << 16); lo[1] = __uint_as_float(m[0] & 0xFFFF0000u);
            lo[2] = __uint_as_float(m[1] << 16); lo[3] = __uint_as_float(m[1] & 0xFFFF0000u);
            hi[0] = __uint_as_float(m[2] << 16); hi[1] = __uint_as_float(m[2] & 0xFFFF0000u);
            hi[2] = __uint_as_float(m[3] << 16); hi[3] = __uint_as_float(m[3] & 0xFFFF0000u);
            reinterpret_cast<float4v *>(tile)[2 * i] = lo;
            reinterpret_cast<float4v *>(tile)[2 * i + 1] = hi;
        }
    }
    for (int i = nvec * VE + tid; i < nelem; i += 256) tile[i] = Elem<T>::load(src, i);
    for (int l = tid; l < np * 12; l += 256) {
        const int p = l / 12, e = l - p * 12;
        const int c = (p0 + p) % a.C;
        float v = 0.0f;
        if (e < 9) v = Elem<T>::load(wg, c * 9 + e);
        else if (e == 9) v = a.scale[c];
        else if (e == 10) v = a.bias ? fmaf(a.bias[c], a.scale[c], a.shift[c]) : a.shift[c];
        prm[l] = v;
    }

    // ---- this lane's output position and taps, fixed for the kernel -------------------------
    const int G = 256 / OHW;              // planes handled per pass of the workgroup
    const int sub = tid / OHW, r0 = tid - sub * OHW;
    const int oh = r0 / a.OW, ow = r0 - oh * a.OW;
    int toff[9];
    uint32_t mask = 0;
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            const int ih = oh * STRIDE - 1 + r, iw = ow * STRIDE - 1 + s;
            const bool ok = ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
            toff[r * 3 + s] = ok ? ih * a.W + iw : 0;
            mask |= (uint32_t)ok << (r * 3 + s);
        }
    __syncthreads();
    if (sub >= G) return;

    const T *res = static_cast<const T *>(a.residual);
    T *yg = static_cast<T *>(a.y);
    const float floor_v = a.relu ? 0.0f : -INFINITY;
    for (int p = sub; p < np; p += G) {
        const float *pl = tile + p * HW;
        const float *pp = prm + p * 12;
        float acc = 0.0f;
#pragma unroll
        for (int e = 0; e < 9; ++e) {
            const float v = pl[toff[e]];
            acc += ((mask >> e) & 1u) ? v * pp[e] : 0.0f;
        }
        const size_t idx = (size_t)(p0 + p) * OHW + r0;
        float o = fmaf(acc, pp[9], pp[10]);
        if (res) o += Elem<T>::load(res + idx, 0);
        o = fmaxf(o, floor_v);
        // a wave's lanes write one contiguous run; the hint pays on 4-byte elements only
        if (sizeof(T) == 4) stream_store<NT>(reinterpret_cast<float *>(yg) + idx, o);
        else Elem<T>::store(yg + idx, 0, o);
    }
}

template <typename T, int STRIDE>
void launch_smallplane(const DwSmallArgs &d, bool nt, unsigned blocks, size_t lds, hipStream_t stream)
{
    if (nt && sizeof(T) == 4)
        hipLaunchKernelGGL((dwconv3x3_smallplane_kernel<T, STRIDE, true>), dim3(blocks), dim3(256), lds,
                           stream, d);
    else
        hipLaunchKernelGGL((dwconv3x3_smallplane_kernel<T, STRIDE, false>), dim3(blocks), dim3(256), lds,
                           stream, d);
}

// Variant for the narrow maps of the late layers (output rows of 14 or 7 pixels: D6..D9 of Table 2
// and the MobileNet body behind them) when there are enough planes to fill the chip.  A lane owns
// ONE output row of one plane: it reads its three input rows whole (rows of 14 or 28 pixels are 28
// to 112 contiguous bytes, fetched as dword-aligned 16-byte vectors plus a remainder), keeps them
// in registers with a zero column on either side, and writes the output row as one contiguous run.
// There is no LDS, no barrier and no per-element index arithmetic: the small-plane kernel above
// spends some 60 vector instructions per output (offsets, masks, LDS reads of taps that change with
// every plane) and was bound by instruction issue, not by memory - 11.1 us against 4.9 us here on
// the 14x14x512 bf16 layer at batch 32; a lane per output-row PAIR or per plane is slower again
// (5.9, 11.2 us: fewer, fatter waves).  Neighbouring lanes re-read two of the three rows; the
// caches serve that.  With few planes (batch 1) the small-plane kernel's finer split wins.
typedef uint32_t uint4a __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t uint3a __attribute__((ext_vector_type(3), aligned(4)));
typedef uint32_t uint2a __attribute__((ext_vector_type(2), aligned(4)));

template <int NW>
__device__ __forceinline__ void load_words(const uint32_t *p, uint32_t (&w)[NW])
{
#pragma unroll
    for (int k = 0; k + 4 <= NW; k += 4) {
        const uint4a m = *reinterpret_cast<const uint4a *>(p + k);
        w[k] = m[0]; w[k + 1] = m[1]; w[k + 2] = m[2]; w[k + 3] = m[3];
    }
    constexpr int B = NW / 4 * 4;
    if constexpr (NW % 4 == 3) {
        const uint3a m = *reinterpret_cast<const uint3a *>(p + B);
        w[B] = m[0]; w[B + 1] = m[1]; w[B + 2] = m[2];
    }
    if constexpr (NW % 4 == 2) {
        const uint2a m = *reinterpret_cast<const uint2a *>(p + B);
        w[B] = m[0]; w[B + 1] = m[1];
    }
    if constexpr (NW % 4 == 1) w[B] = p[B];
}

template <bool NT, int NW>
__device__ __forceinline__ void store_words(uint32_t *p, const uint32_t (&w)[NW])
{
#pragma unroll
    for (int k = 0; k + 4 <= NW; k += 4) {
        uint4a m;
        m[0] = w[k]; m[1] = w[k + 1]; m[2] = w[k + 2]; m[3] = w[k + 3];
        if constexpr (NT) __builtin_nontemporal_store(m, reinterpret_cast<uint4a *>(p + k));
        else *reinterpret_cast<uint4a *>(p + k) = m;
    }
    constexpr int B = NW / 4 * 4;
    if constexpr (NW % 4 == 3) {
        uint3a m;
        m[0] = w[B]; m[1] = w[B + 1]; m[2] = w[B + 2];
        if constexpr (NT) __builtin_nontemporal_store(m, reinterpret_cast<uint3a *>(p + B));
        else *reinterpret_cast<uint3a *>(p + B) = m;
    }
    if constexpr (NW % 4 == 2) {
        uint2a m;
        m[0] = w[B]; m[1] = w[B + 1];
        if constexpr (NT) __builtin_nontemporal_store(m, reinterpret_cast<uint2a *>(p + B));
        else *reinterpret_cast<uint2a *>(p + B) = m;
    }
    if constexpr (NW % 4 == 1) stream_store<NT>(p + B, w[B]);
}

struct DwRowsArgs {
    const void *x, *w;
    const float *scale, *shift, *bias;
    const void *residual;
    void *y;
    int C, H, OH;
    int total;         // lanes with work: planes x OH
    float inv_oh;
    int relu;
    uint32_t x_bytes;  // size of x rounded up to a whole word (odd rows only)
};

template <typename T, int STRIDE, int OW, bool NT>
__global__ __launch_bounds__(256) void dwconv3x3_rows_kernel(const DwRowsArgs a)
{
    constexpr int W = OW * STRIDE;                  // input row, pixels
    constexpr int EW = 4 / sizeof(T);               // pixels per 32-bit word
    // Rows of an odd number of bf16 pixels (7: 14 bytes) start on any 2-byte boundary.  Such a row
    // is fetched as the four aligned words from the one that holds its first pixel - through a
    // buffer descriptor whose size is the tensor's rounded up to a whole word, so that the last
    // word of the tensor is readable - and moved down by 16 bits where it started in a word's
    // upper half (one funnel shift per word).
    constexpr bool kOdd = W % EW != 0;
    static_assert(!kOdd || (sizeof(T) == 2 && W == 7), "odd rows: seven bf16 pixels");
    constexpr int NW = (W + EW - 1) / EW;
    const int g = blockIdx.x * 256 + threadIdx.x;
    if (g >= a.total) return;
    int oh;
    const int plane = fast_div(g, a.OH, a.inv_oh, &oh);
    const int c = plane % a.C;
    const T *__restrict__ wg = static_cast<const T *>(a.w);
    float wt[9];
#pragma unroll
    for (int e = 0; e < 9; ++e) wt[e] = Elem<T>::load(wg, c * 9 + e);
    const float sc = a.scale[c];
    const float sf = a.bias ? fmaf(a.bias[c], sc, a.shift[c]) : a.shift[c];

    // the three input rows; a padding row is read from the nearest image row and zeroed, so that
    // all loads are in flight together
    const T *xp = static_cast<const T *>(a.x) + (size_t)plane * a.H * W;
    float v[3][W + 2];
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int ih = oh * STRIDE - 1 + r;
        const bool ok = ih >= 0 && ih < a.H;
        uint32_t wd[NW];
        const int ihc = min(max(ih, 0), a.H - 1);
        if constexpr (kOdd) {
            const uint32_t start = ((uint32_t)plane * a.H + ihc) * (uint32_t)(W * 2);   // byte offset in x
            const uint4v m = __builtin_bit_cast(
                uint4v, __builtin_amdgcn_raw_buffer_load_b128(
                            __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.x), 0, a.x_bytes, 0x00020000),
                            start & ~3u, 0, 0));
            const uint32_t sh = (start & 2u) * 8u;
            wd[0] = __builtin_amdgcn_alignbit(m[1], m[0], sh);
            wd[1] = __builtin_amdgcn_alignbit(m[2], m[1], sh);
            wd[2] = __builtin_amdgcn_alignbit(m[3], m[2], sh);
            wd[3] = m[3] >> sh;
        } else {
            load_words<NW>(reinterpret_cast<const uint32_t *>(xp + ihc * W), wd);
        }
        v[r][0] = 0.0f;
#pragma unroll
        for (int k = 0; k < NW; ++k) {
            if constexpr (sizeof(T) == 4) {
                v[r][1 + k] = ok ? __uint_as_float(wd[k]) : 0.0f;
            } else {
                v[r][1 + 2 * k] = ok ? __uint_as_float(wd[k] << 16) : 0.0f;
                if (2 + 2 * k <= W) v[r][2 + 2 * k] = ok ? __uint_as_float(wd[k] & 0xFFFF0000u) : 0.0f;
            }
        }
        v[r][W + 1] = 0.0f;
    }

    float out[OW];
#pragma unroll
    for (int q = 0; q < OW; ++q) {
        float acc = 0.0f;
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int t = 0; t < 3; ++t) acc += v[r][q * STRIDE + t] * wt[r * 3 + t];
        out[q] = fmaf(acc, sc, sf);
    }

    const size_t idx = ((size_t)plane * a.OH + oh) * OW;
    const float floor_v = a.relu ? 0.0f : -INFINITY;
    T *yp = static_cast<T *>(a.y) + idx;
    const T *rp = a.residual ? static_cast<const T *>(a.residual) + idx : nullptr;
    constexpr bool kWords = (OW * sizeof(T)) % 4 == 0;      // the output row is whole words
    if constexpr (kWords) {
        constexpr int NO = OW * sizeof(T) / 4;
        uint32_t ow_[NO];
        if (a.residual) {
            load_words<NO>(reinterpret_cast<const uint32_t *>(rp), ow_);
#pragma unroll
            for (int k = 0; k < NO; ++k) {
                if constexpr (sizeof(T) == 4) {
                    out[k] += __uint_as_float(ow_[k]);
                } else {
                    out[2 * k] += __uint_as_float(ow_[k] << 16);
                    out[2 * k + 1] += __uint_as_float(ow_[k] & 0xFFFF0000u);
                }
            }
        }
#pragma unroll
        for (int k = 0; k < NO; ++k) {
            if constexpr (sizeof(T) == 4) ow_[k] = __float_as_uint(fmaxf(out[k], floor_v));
            else ow_[k] = f32x2_to_bf16x2(fmaxf(out[2 * k], floor_v), fmaxf(out[2 * k + 1], floor_v));
        }
        store_words<NT, NO>(reinterpret_cast<uint32_t *>(yp), ow_);
    } else {
        // rows of an odd number of bf16 pixels start on any 2-byte boundary: element by element
#pragma unroll
        for (int q = 0; q < OW; ++q) {
            float o = out[q];
            if (a.residual) o += Elem<T>::load(rp, q);
            Elem<T>::store(yp, q, fmaxf(o, floor_v));
        }
    }
}

template <typename T, int STRIDE, int OW>
void launch_rows(const DwRowsArgs &d, bool nt, hipStream_t stream)
{
    const unsigned blocks = (unsigned)((d.total + 255) / 256);
    // (the non-temporal hint pays on the 4-byte type's wide stores only, as in the kernels above)
    if (nt && sizeof(T) == 4)
        hipLaunchKernelGGL((dwconv3x3_rows_kernel<T, STRIDE, OW, true>), dim3(blocks), dim3(256), 0, stream, d);
    else
        hipLaunchKernelGGL((dwconv3x3_rows_kernel<T, STRIDE, OW, false>), dim3(blocks), dim3(256), 0, stream, d);
}

// Lanes below which the rows kernel leaves a launch to the small-plane kernel (a batch-1 layer has
// 3.5 to 7 thousand output rows: too few waves to hide a lane's three-row fetch).
constexpr long kRowsMinLanes = 16384;

int ceil_log2(int v)
{
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

}  // namespace

tvg_status launch_dwconv3x3(const ConvProblem &p, const ConvPointers &ptr, hipStream_t stream)
{
    const int stride0 = p.sh;
    const bool ptr16 = reinterpret_cast<uintptr_t>(ptr.x) % 16 == 0 &&
                       reinterpret_cast<uintptr_t>(ptr.y) % 16 == 0 &&
                       reinterpret_cast<uintptr_t>(ptr.residual) % 16 == 0;
    // narrow output rows, many planes: one lane per output row
    const long rows_total = (long)p.N * p.IC * p.OH;
    const int esz = p.dtype == TVG_BF16 ? 2 : 4;
    // (rows of 28 pixels: bf16 only, 11.1 -> 9.3 us on the 256-channel layer at batch 32; in fp32 a
    // lane's three rows are 90 registers and 112-byte strides, and D5 at batch 64 took 73 us against
    // the register-blocked kernel's 33)
    if ((p.OW == 14 || p.OW == 7 || (p.OW == 28 && stride0 == 1 && p.dtype == TVG_BF16)) &&
        p.W == p.OW * stride0 && ((p.W * esz) % 4 == 0 || (p.dtype == TVG_BF16 && p.W == 7)) &&
        rows_total >= kRowsMinLanes && rows_total < (1L << 22) &&
        reinterpret_cast<uintptr_t>(ptr.x) % 4 == 0 && reinterpret_cast<uintptr_t>(ptr.y) % 4 == 0 &&
        reinterpret_cast<uintptr_t>(ptr.residual) % 4 == 0 && reinterpret_cast<uintptr_t>(ptr.w) % esz == 0) {
        DwRowsArgs d;
        d.x = ptr.x; d.w = ptr.w;
        d.scale = ptr.scale; d.shift = ptr.shift; d.bias = ptr.bias;
        d.residual = ptr.residual; d.y = ptr.y;
        d.C = p.IC; d.H = p.H; d.OH = p.OH;
        d.total = (int)rows_total;
        d.inv_oh = 1.0f / (float)p.OH;
        // (a depthwise problem has fewer than 2^31 elements, so the byte count fits)
        d.x_bytes = (uint32_t)(((size_t)p.N * p.IC * p.H * p.W * esz + 3) & ~(size_t)3);
        d.relu = p.relu;
        const bool nt = p.stream_out != 0;
        const bool f32 = p.dtype == TVG_F32;
        if (p.OW == 28) launch_rows<bf16_t, 1, 28>(d, nt, stream);
        else if (p.OW == 14 && stride0 == 1) f32 ? launch_rows<float, 1, 14>(d, nt, stream) : launch_rows<bf16_t, 1, 14>(d, nt, stream);
        else if (p.OW == 14) f32 ? launch_rows<float, 2, 14>(d, nt, stream) : launch_rows<bf16_t, 2, 14>(d, nt, stream);
        else if (stride0 == 2) f32 ? launch_rows<float, 2, 7>(d, nt, stream) : launch_rows<bf16_t, 2, 7>(d, nt, stream);
        else f32 ? launch_rows<float, 1, 7>(d, nt, stream) : launch_rows<bf16_t, 1, 7>(d, nt, stream);
        return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
    }

    // output rows per lane (measured at batch 64 and batch 1, us with 4 / 2 / 1 rows): stride 2 wants
    // one (D2 49.6 / 48.7 / 45.1, D4 31.4 / 29.9 / 25.0: a block of 4 rows is 9 input rows of
    // registers), stride 1 four on the wide maps (D1 42.9 / 50.3 / 65.8) and two on 28-pixel rows
    // (D5 33.4 / 31.5 / 33.5); a launch of few lanes wants the finest split (batch 1: 4.4-5.4 /
    // 3.8-4.4 / 3.3-3.8)
    const long tasks4 = (long)p.N * p.IC * ((p.OH + 3) / 4) * (p.OW / 4);
    const int frb = (stride0 == 2 || tasks4 < 131072) ? 1 : p.W <= 28 ? 2 : 4;
    const long tasks = (long)p.N * p.IC * ((p.OH + frb - 1) / frb) * (p.OW / 4);
    if (p.dtype == TVG_F32 && ptr16 && p.W % 4 == 0 && p.OW % 4 == 0 && p.W >= 8 &&
        tasks < (1L << 31) && (p.OH + frb - 1) / frb * (p.OW / 4) < (1 << 22)) {
        DwDirectArgs d;
        d.x = static_cast<const float *>(ptr.x); d.w = static_cast<const float *>(ptr.w);
        d.scale = ptr.scale; d.shift = ptr.shift; d.bias = ptr.bias;
        d.residual = static_cast<const float *>(ptr.residual); d.y = static_cast<float *>(ptr.y);
        d.C = p.IC; d.H = p.H; d.W = p.W; d.OH = p.OH; d.OW = p.OW;
        d.CB = p.OW / 4;
        d.tpp = (p.OH + frb - 1) / frb * d.CB;
        d.total = (int)tasks;
        d.inv_cb = 1.0f / (float)d.CB;
        d.relu = p.relu;
        const unsigned blocks = (unsigned)((tasks + 255) / 256);
#define TVG_DW_LAUNCH(RB_)                                                                           \
        do {                                                                                         \
            if (stride0 == 1 && p.stream_out)                                                         \
                hipLaunchKernelGGL((dwconv3x3_direct_kernel<1, true, RB_>), dim3(blocks), dim3(256), 0, stream, d);  \
            else if (stride0 == 1)                                                                    \
                hipLaunchKernelGGL((dwconv3x3_direct_kernel<1, false, RB_>), dim3(blocks), dim3(256), 0, stream, d); \
            else if (p.stream_out)                                                                    \
                hipLaunchKernelGGL((dwconv3x3_direct_kernel<2, true, RB_>), dim3(blocks), dim3(256), 0, stream, d);  \
            else                                                                                      \
                hipLaunchKernelGGL((dwconv3x3_direct_kernel<2, false, RB_>), dim3(blocks), dim3(256), 0, stream, d); \
        } while (0)
        if (frb == 1) TVG_DW_LAUNCH(1);
        else if (frb == 2) TVG_DW_LAUNCH(2);
        else TVG_DW_LAUNCH(4);
#undef TVG_DW_LAUNCH
        return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
    }

    // bf16: 8 output columns per lane where the row allows, else 4; planes of at most 256
    // outputs whose rows allow neither go to the small-plane kernel below
    const int cw = p.OW % 8 == 0 ? 8 : p.OW % 4 == 0 ? 4 : 0;
    // output rows per lane: 4, under stride 2 two (a block of 4 is 9 input rows; the 112 -> 56 and
    // 56 -> 28 MobileNet layers at batch 32: 14.2 -> 13.7 and 9.2 -> 8.5 us; one row: 14.0, 9.0, and
    // 40 % slower under stride 1)
    const int brb = stride0 == 2 ? 2 : 4;
    const long btasks = cw ? (long)p.N * p.IC * ((p.OH + brb - 1) / brb) * (p.OW / cw) : 0;
    if (p.dtype == TVG_BF16 && ptr16 && cw && (stride0 == 1 || p.W == 2 * p.OW) &&
        reinterpret_cast<uintptr_t>(ptr.w) % 2 == 0 && btasks < (1L << 31) &&
        (p.OH + brb - 1) / brb * (p.OW / cw) < (1 << 22)) {
        DwDirectBf16Args d;
        d.x = static_cast<const bf16_t *>(ptr.x); d.w = static_cast<const bf16_t *>(ptr.w);
        d.scale = ptr.scale; d.shift = ptr.shift; d.bias = ptr.bias;
        d.residual = static_cast<const bf16_t *>(ptr.residual); d.y = static_cast<bf16_t *>(ptr.y);
        d.C = p.IC; d.H = p.H; d.W = p.W; d.OH = p.OH; d.OW = p.OW;
        d.CB = p.OW / cw;
        d.tpp = (p.OH + brb - 1) / brb * d.CB;
        d.total = (int)btasks;
        d.inv_cb = 1.0f / (float)d.CB;
        d.relu = p.relu;
        const unsigned blocks = (unsigned)((btasks + 255) / 256);
        const bool nt = p.stream_out != 0;
        if (stride0 == 1 && cw == 8) launch_direct_bf16<1, 8>(d, brb, nt, blocks, stream);
        else if (stride0 == 1) launch_direct_bf16<1, 4>(d, brb, nt, blocks, stream);
        else if (cw == 8) launch_direct_bf16<2, 8>(d, brb, nt, blocks, stream);
        else launch_direct_bf16<2, 4>(d, brb, nt, blocks, stream);
        return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
    }

    if (p.OH * p.OW <= 256 && reinterpret_cast<uintptr_t>(ptr.x) % 16 == 0) {
        DwSmallArgs d;
        d.x = ptr.x; d.w = ptr.w;
        d.scale = ptr.scale; d.shift = ptr.shift; d.bias = ptr.bias;
        d.residual = ptr.residual; d.y = ptr.y;
        d.planes = p.N * p.IC; d.C = p.IC; d.H = p.H; d.W = p.W; d.OH = p.OH; d.OW = p.OW;
        d.relu = p.relu;
        // planes per workgroup: a multiple of the unit that makes every group start on a 16-byte
        // boundary (1 when a plane is itself a multiple of 16 bytes, else 4 for fp32 and 8 for
        // bf16), about 2048 outputs, at most 40 KB of LDS, and no larger than leaves about four
        // workgroups per CU - or, with so few planes that this is below the unit (batch 1), one
        // workgroup per CU: D6 at batch 1 used to run 32 workgroups of 8 planes on 256 CUs
        const int hw = p.H * p.W, ohw = p.OH * p.OW;
        const int esize = p.dtype == TVG_BF16 ? 2 : 4;
        const int unit = (hw * esize) % 16 == 0 ? 1 : 16 / esize;
        int pg = 2048 / ohw;
        const int cap_lds = (40 * 1024 / 4) / (hw + 12);
        if (pg > cap_lds) pg = cap_lds;
        int cap_fill = d.planes / (4 * kComputeUnits);
        if (cap_fill < unit) cap_fill = d.planes / kComputeUnits;
        if (cap_fill < unit) cap_fill = unit;
        if (pg > cap_fill) pg = cap_fill;
        pg = pg / unit * unit;
        if (pg >= unit) {
            d.PG = pg;
            const size_t lds = (size_t)pg * (hw + 12) * sizeof(float);
            const unsigned blocks = (unsigned)((d.planes + pg - 1) / pg);
            const bool nt = p.stream_out != 0;
            if (p.dtype == TVG_BF16) {
                if (stride0 == 1) launch_smallplane<bf16_t, 1>(d, nt, blocks, lds, stream);
                else launch_smallplane<bf16_t, 2>(d, nt, blocks, lds, stream);
            } else {
                if (stride0 == 1) launch_smallplane<float, 1>(d, nt, blocks, lds, stream);
                else launch_smallplane<float, 2>(d, nt, blocks, lds, stream);
            }
            return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
        }
    }

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
    // (the host interface has already rejected rows whose narrowest band does not fit)
    if (lds_bytes > 64 * 1024) return TVG_ERR_UNSUPPORTED;

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
