// bf16 3x3 (pad 1, stride 1 or 2) fused conv2d: implicit GEMM on MFMA with the
// input staged ONCE per input-channel chunk as a zero-padded spatial patch in LDS
// and re-read from there by all nine filter taps.
//
// Why a second dense kernel: the generic implicit-GEMM kernel gathers every
// (pixel, k) operand from global memory, i.e. each input value is fetched nine
// times for a 3x3 filter, one 2-byte load each, and the address arithmetic of
// those loads outweighs the MFMA work.  Here a workgroup's NT consecutive output
// pixels (n, oh, ow flattened) need a contiguous range of input rows; those
// rows are fetched once per chunk of 16 input channels (cooperative fetch into
// the shared scope, TVM paper Section 4.2), transposed on the way so that the 8
// channels an MFMA lane consumes are one 16-byte LDS word, and every tap reads
// the same patch at a shifted address.  Weights for the chunk (all nine taps)
// are fetched as contiguous 144-byte runs of the OIHW tensor and transposed in
// registers to tap-major.  The reduction order is (ic chunk, tap, ic in chunk).
//
// Patch geometry.  "Virtual rows": image n owns rows n*(H+2) .. n*(H+2)+H+1,
// the first and last being zero padding, so a pixel (n, oh, ow) and tap (r, s)
// read virtual row n*(H+2) + oh*stride + r, column ow*stride + s of a
// (W+2)-wide padded row.  A pixel tile therefore needs one contiguous range of
// virtual rows even when it straddles images.  For stride 2 a row is stored even
// columns first, odd columns after them, so that the pixels of consecutive lanes
// (two columns apart) are adjacent positions again.
//
// Pipeline per chunk: global loads of chunk c+1 are issued into registers, the
// 9 taps x MFMA phase of chunk c runs from LDS, then (barrier) the registers are
// written to LDS (barrier).  Two workgroups per CU overlap each other's phases
// (Section 4.4: hide memory latency behind compute).
#include <stdio.h>
#include <stdlib.h>

#include <numeric>
#include <algorithm>

#include "tvg_device.h"
#include "tvg_internal.h"

namespace tvg {

namespace {

struct PatchArgs {
    const bf16_t *x, *w;
    const float *scale, *shift, *bias;
    const bf16_t *residual;
    bf16_t *y;
    int N, IC, H, W, OC, OH, OW, npix, relu, mtiles;
    int vmode;        // pixels per vector store in the epilogue (8, 4 or 1)
    uint32_t x_bytes, w_bytes;
    int ss_offset;    // byte offset in LDS of the staged (scale, offset) pairs
    int ntiles, m_major;
    // Two heads (tvg_conv2d_fused_dual): output channels [0, oc1) go to y with `relu` and the
    // residual, channels [oc1, OC) to y2 with relu2; oc1 = 0: one head.  centre2: the filters of
    // head 2 are zero outside their centre tap (a 1x1 convolution of the same input), its tiles
    // skip the other eight taps.  A tile lies within one head (oc1 is a multiple of MT).
    int oc1, relu2, centre2;
    bf16_t *y2;
};

// LDS layout: the two channel octets of a chunk live in separate PLANES of dense 16-byte words
// (position-major), so the 16-byte reads of 16 consecutive lanes are 256 consecutive bytes:
// conflict-free without padding (a 48-byte position stride did the same with half as much again
// of LDS, which cost the 64-channel layers their third workgroup per CU).
constexpr int kWordBytes = 16;
constexpr int kChunk = 16;       // input channels per chunk = K of one 32x32x16 MFMA
constexpr int kRsrcFlags = 0x00020000;   // raw buffer descriptor word 3 on gfx9-family targets

__device__ __forceinline__ int xcd_remap(int bid, int nb)
{
    const int q = nb >> 3, rem = nb & 7;
    const int xcd = bid & 7, local = bid >> 3;
    return xcd < rem ? xcd * (q + 1) + local : rem * (q + 1) + (xcd - rem) * q + local;
}

// (half `ha` of a) | (half `hb` of b) << 16 in one byte permute (v_perm_b32 takes its selector
// bytes 0-3 from the second source, 4-7 from the first); written as shifts and masks the same
// pair costs two to three instructions, and the staging of a chunk was a third of the loop's
// instruction stream, which is what bounds the layers of this kernel
__device__ __forceinline__ uint32_t pack_halves(uint32_t a, int ha, uint32_t b, int hb)
{
    const uint32_t sel = (ha ? 0x0302u : 0x0100u) | ((hb ? 0x0706u : 0x0504u) << 16);
    return __builtin_amdgcn_perm(b, a, sel);
}

// MT x NT output tile per workgroup of 256 threads; PT = patch load tasks per thread; PX =
// horizontally adjacent pixels fetched per load (2, 4 or 8 need W to be a multiple: 32-, 64- or
// 128-bit loads, a half to an eighth of the vector memory instructions).
// DUAL = the two-head variant (instances exist for the 64-channel tiles of 128 and 256 pixels).
template <int MT, int NT, int STRIDE, int PT, int PX, bool DUAL = false>
// (Three workgroups per CU were measured on C2 once the plane layout had made room in LDS: the
// compiler then keeps the 64 x 256 tile in 168 registers with 16 spilled, 33.2 us against 23.6.)
__global__ __launch_bounds__(256, 2) void conv3x3_patch_kernel(const PatchArgs a)
{
    // four waves as 2 x 2, or 1 x 4 for the wide 64 x 256 tile (the weights of a chunk weigh
    // about six times the input patch per tile side, so a wide pixel tile moves the fewest
    // operand bytes per MFMA through the vector memory path)
    // wave layout: under a 64-channel tile the four waves sit side by side, each all 64 channels x
    // NT / 4 pixels (for 128 pixels that is two weight reads and one pixel read per pair of
    // MFMAs instead of one and two: C7 19.0 -> 18.4 us); a 128-channel tile is 2 x 2 waves
    constexpr int WM = (NT >= 256 || (MT == 64 && NT == 128)) ? 1 : 2, WN = 4 / WM;
    constexpr int WTM = MT / WM, WTN = NT / WN;
    constexpr int MI = WTM / 32, NJ = WTN / 32;
    constexpr int APLANE = 9 * MT * kWordBytes + 128;     // (+128: the two planes' stores fall on different banks)
    constexpr int ABYTES = 2 * APLANE;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *As = smem;              // [octet][tap][oc] 16-byte words
    unsigned char *Ps = smem + ABYTES;     // [octet][virtual row][W + 2] 16-byte words

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int lrow = lane & 31, lhalf = lane >> 5;

    const int tile = xcd_remap(blockIdx.x, gridDim.x);
    // Consecutive tiles (which share an XCD's L2) share the larger operand: the same pixel
    // tile under all channel tiles, or - when the weights outweigh the input - the same
    // channel tile over consecutive pixel tiles.
    const int m0 = (a.m_major ? tile / a.ntiles : tile % a.mtiles) * MT;
    const int n0 = (a.m_major ? tile % a.ntiles : tile / a.mtiles) * NT;

    const int H = a.H, W = a.W, HW = H * W, OHW = a.OH * a.OW;
    const int VH = H + 2, PW = W + 2;
    // Stride 2: a patch row holds its even columns first and its odd columns from position
    // HALF on, so that the 32 pixels of an MFMA operand (input columns two apart) are 32
    // adjacent positions, which 16-byte reads cover without bank conflicts; interleaved, they
    // would be 96 bytes apart and collide in pairs.
    const int HALF = (PW + 1) / 2;

    // Index arithmetic below divides by OH*OW, OW, W and H+2 only; the host admits this
    // kernel when every dividend stays below 2^22, where fast_div is exact.
    const float inv_ohw = 1.0f / (float)OHW, inv_ow = 1.0f / (float)a.OW;
    const float inv_vh = 1.0f / (float)VH;

    // ---- tile geometry (uniform) ---------------------------------------------------------
    const int p_last = min(n0 + NT, a.npix) - 1;
    const int na = n0 / OHW, oha = (n0 - na * OHW) / a.OW;
    const int nb = p_last / OHW, ohb = (p_last - nb * OHW) / a.OW;
    const int vr_lo = na * VH + oha * STRIDE;
    const int nrows = nb * VH + ohb * STRIDE + 2 - vr_lo + 1;
    const int npos = nrows * PW;
    const int pplane = npos * kWordBytes;          // one octet plane of this tile's patch

    float *ss_lds = reinterpret_cast<float *>(smem + a.ss_offset);

    // ---- per-thread patch load tasks: (virtual row, iw, channel octet), fixed for all chunks
    uint32_t goff[PT];      // byte offset of the task's first channel within a chunk of x
    int loff[PT];           // byte offset of its 16-byte slot in the patch
    int nvalid[PT];         // pixels of the task to store: 0 = nothing to do, < PX = the row's ragged end
    {
        // a row that is not a multiple of PX ends in a task with fewer pixels; its load reads on
        // into the next row (or, at the very end of x, past the buffer: zeros), 4-byte aligned
        const int WPX = (W + PX - 1) / PX;
        const float inv_wpx = 1.0f / (float)WPX;
        const int per_octet = nrows * WPX;
#pragma unroll
        for (int j = 0; j < PT; ++j) {
            const int t = tid + j * 256;
            goff[j] = 0;
            loff[j] = 0;
            nvalid[j] = 0;
            if (t < 2 * per_octet) {
                const int octet = t >= per_octet;
                const int rem = t - octet * per_octet;
                int iw, vi;
                const int vrow = fast_div(rem, WPX, inv_wpx, &iw);
                iw *= PX;
                const int n = fast_div(vr_lo + vrow, VH, inv_vh, &vi);
                const int ih = vi - 1;
                if (ih >= 0 && ih < H && n < a.N) {
                    goff[j] = 2u * (uint32_t)((n * a.IC + octet * 8) * HW + ih * W + iw);
                    const int col = iw + 1;       // patch column (0 = left padding)
                    const int pos = STRIDE == 2 ? ((col & 1) ? HALF + (col >> 1) : (col >> 1)) : col;
                    loff[j] = octet * pplane + (vrow * PW + pos) * kWordBytes;
                    nvalid[j] = min(PX, W - iw);
                }
            }
        }
    }

    // ---- per-lane LDS offsets of this lane's pixels (MFMA B operand) -----------------------
    int pb[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int p = n0 + wn * WTN + j * 32 + lrow;
        pb[j] = lhalf * pplane;
        if (p < a.npix) {
            int rem, ow;
            const int n = fast_div(p, OHW, inv_ohw, &rem);
            const int oh = fast_div(rem, a.OW, inv_ow, &ow);
            // (stride 2: column 2*ow is even, at position ow of its row)
            pb[j] += ((n * VH + oh * STRIDE - vr_lo) * PW + ow) * kWordBytes;
        }
    }

    // ---- weight task: one output channel, one octet of input channels, all nine taps -------
    const bool wtask = tid < MT * 2;
    const int w_ocl = tid >> 1, w_oct = tid & 1;
    // rows past OC read row 0: their products land in accumulators that are never stored
    const bool wvalid = wtask && (m0 + w_ocl) < a.OC;
    const uint32_t woff = 2u * (uint32_t)(((wvalid ? m0 + w_ocl : 0) * a.IC + w_oct * 8) * 9);

    // Loaded values stay unpacked until store_chunk so that nothing waits on the loads
    // before the MFMA phase of the current chunk.
    constexpr int W32 = PX >= 2 ? PX / 2 : 1;  // registers per load
    uint32_t praw[PT][8][W32];
    uint4v wreg[9];

    // Buffer loads: a uniform descriptor + per-lane 32-bit byte offset + scalar offset, so
    // the loads of a chunk cost no vector address arithmetic at all.
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(a.x), 0, a.x_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(a.w), 0, a.w_bytes, kRsrcFlags);

    auto load_chunk = [&](int c) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int soff = (c * kChunk + q) * HW * 2;
#pragma unroll
            for (int j = 0; j < PT; ++j)
                if constexpr (PX == 8) {
                    const uint4v t4 = __builtin_bit_cast(
                        uint4v, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, goff[j], soff, 0));
#pragma unroll
                    for (int d = 0; d < 4; ++d) praw[j][q][d] = t4[d];
                } else if constexpr (PX == 4) {
                    const uint2v t2 = __builtin_bit_cast(
                        uint2v, __builtin_amdgcn_raw_buffer_load_b64(xrsrc, goff[j], soff, 0));
                    praw[j][q][0] = t2[0];
                    praw[j][q][1] = t2[1];
                } else if constexpr (PX == 2) {
                    praw[j][q][0] = __builtin_amdgcn_raw_buffer_load_b32(xrsrc, goff[j], soff, 0);
                } else {
                    praw[j][q][0] = __builtin_amdgcn_raw_buffer_load_b16(xrsrc, goff[j], soff, 0);
                }
        }
        if (wtask) {
            const int soff = c * kChunk * 9 * 2;
#pragma unroll
            for (int i = 0; i < 9; ++i)
                wreg[i] = __builtin_bit_cast(
                    uint4v, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, woff + i * 16, soff, 0));
        }
    };

    auto store_chunk = [&]() {
#pragma unroll
        for (int j = 0; j < PT; ++j) {
            // pixel k of the task sits in half (k & 1) of register k >> 1 of each channel;
            // rows are even when PX > 1, so a ragged task ends on a pixel pair
            constexpr int STEP = PX > 1 ? 2 : 1;
#pragma unroll
            for (int k0 = 0; k0 < PX; k0 += STEP) {
                if (k0 < nvalid[j]) {
#pragma unroll
                    for (int k = k0; k < k0 + STEP; ++k) {
                        uint32_t o[4];
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            o[q] = pack_halves(praw[j][2 * q][k >> 1], k & 1, praw[j][2 * q + 1][k >> 1], k & 1);
                        // stride 2 (PX > 1: the task starts on an odd patch column): pixels
                        // alternate between the odd and the even half of the row
                        const int koff = STRIDE == 2 ? ((k & 1) ? (1 - HALF) * kWordBytes : 0) + (k >> 1) * kWordBytes
                                                     : k * kWordBytes;
                        *reinterpret_cast<uint4v *>(Ps + loff[j] + koff) = uint4v{o[0], o[1], o[2], o[3]};
                    }
                }
            }
        }
        if (wtask) {
            // wreg holds 8 channels x 9 taps, tap fastest; emit one 8-channel vector per tap
            uint32_t d[36];
#pragma unroll
            for (int i = 0; i < 9; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) d[i * 4 + q] = wreg[i][q];
#pragma unroll
            for (int tap = 0; tap < 9; ++tap) {
                uint32_t o[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int e0 = (2 * q) * 9 + tap, e1 = (2 * q + 1) * 9 + tap;
                    o[q] = pack_halves(d[e0 >> 1], e0 & 1, d[e1 >> 1], e1 & 1);
                }
                *reinterpret_cast<uint4v *>(As + w_oct * APLANE + (tap * MT + w_ocl) * kWordBytes) =
                    uint4v{o[0], o[1], o[2], o[3]};
            }
        }
    };

    float16v acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int nchunks = a.IC / kChunk;
    // The first chunk's loads go out before the rest of the set-up, which then runs under
    // their latency: zero the patch once (padding rows and columns are never written
    // again) and stage the tile's (scale, offset) pairs.
    load_chunk(0);
    for (int i = tid; i < 2 * npos; i += 256)
        reinterpret_cast<uint4v *>(Ps)[i] = uint4v{0u, 0u, 0u, 0u};
    stage_scale_shift(ss_lds, m0, MT, a.scale, a.shift, a.bias, a.OC, tid, 256);
    __syncthreads();          // patch zeroing complete before the first real data lands
    store_chunk();
    __syncthreads();

    const bool head2 = DUAL && m0 >= a.oc1;                 // (uniform)
    const bool centre_only = head2 && a.centre2 != 0;
    const unsigned char *Abase = As + lhalf * APLANE + (wm * WTM + lrow) * kWordBytes;
    for (int c = 0; c < nchunks; ++c) {
        // All of the next chunk's loads are issued before this chunk's MFMAs: measured, issuing
        // them in slices between the taps leaves them too little time to arrive.
        if (c + 1 < nchunks) load_chunk(c + 1);

        // operands of tap t+1 are requested from LDS before the MFMAs of tap t issue
        uint4v af[2][MI], bf[2][NJ];
        auto fetch = [&](int tap, int slot) {
            const int r = tap / 3, s = tap - r * 3;
            const int toff = (r * PW + (STRIDE == 2 ? (s == 1 ? HALF : (s >> 1)) : s)) * kWordBytes;
#pragma unroll
            for (int i = 0; i < MI; ++i)
                af[slot][i] =
                    *reinterpret_cast<const uint4v *>(Abase + (tap * MT + i * 32) * kWordBytes);
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                bf[slot][j] = *reinterpret_cast<const uint4v *>(Ps + pb[j] + toff);
        };
        if (centre_only) {
            // a 1x1 convolution riding in a 3x3 launch: the centre tap alone
            fetch(4, 0);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8v, bf[0][j]),
                        __builtin_bit_cast(bf16x8v, af[0][i]), acc[i][j], 0, 0, 0);
        } else {
        fetch(0, 0);
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) {
            const int cur = tap & 1;
            if (tap + 1 < 9) fetch(tap + 1, cur ^ 1);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    // pixel operand first: the accumulator tile is D[pixel][channel]
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8v, bf[cur][j]),
                        __builtin_bit_cast(bf16x8v, af[cur][i]), acc[i][j], 0, 0, 0);
            // keep the order written here: next tap's LDS reads first, then this tap's MFMAs
            if (tap + 1 < 9) __builtin_amdgcn_sched_group_barrier(0x100, MI + NJ, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, MI * NJ, 0);
        }
        }

        if (c + 1 < nchunks) {
            __syncthreads();
            store_chunk();
            __syncthreads();
        }
    }

    // ---- fused tail: transpose each 32x32 tile through LDS, vector stores -----------------
    __syncthreads();                       // every wave is done reading the operand tiles
    // up to two tiles per wave are staged at a time: 20 KB (the host sizes the LDS for it)
    constexpr int BT = MI * NJ >= 2 ? 2 : 1;
    unsigned char *stage = smem + wave * (BT * kStageBytes);
    if (head2) {
        // head 2: its own tensor of OC - oc1 channels, no residual, its own ReLU and store hint
        const TailArgs tail2{a.scale, a.shift, a.bias, nullptr, a.y2, a.OC - a.oc1, OHW, a.npix, a.relu2};
        store_acc_tiles_batched<MI, NJ, BT>(acc, stage, lane, m0 - a.oc1 + wm * WTM, n0 + wn * WTN,
                                            tail2, a.vmode, ss_lds, wm * WTM);
        return;
    }
    const TailArgs tail{a.scale, a.shift, a.bias, a.residual, a.y, DUAL ? a.oc1 : a.OC, OHW,
                        a.npix, a.relu};
    store_acc_tiles_batched<MI, NJ, BT>(acc, stage, lane, m0 + wm * WTM, n0 + wn * WTN, tail,
                                        a.vmode, ss_lds, wm * WTM);
}

// Largest number of virtual rows any pixel tile of NT pixels needs.
int max_patch_rows(const ConvProblem &p, int nt)
{
    const int OHW = p.OH * p.OW, VH = p.H + 2;
    int best = 0;
    // the row count of a tile depends only on where in an image it starts, which repeats after
    // OHW / gcd(OHW, nt) tiles: one period covers every case (this runs on every call)
    const long period = (long)nt * (OHW / std::gcd(OHW, nt));
    for (long n0 = 0; n0 < p.npix && n0 < period; n0 += nt) {
        const long last = (n0 + nt < p.npix ? n0 + nt : p.npix) - 1;
        const int na = (int)(n0 / OHW), oha = (int)((n0 - (long)na * OHW) / p.OW);
        const int nb = (int)(last / OHW), ohb = (int)((last - (long)nb * OHW) / p.OW);
        const int rows = nb * VH + ohb * p.sh + 2 - (na * VH + oha * p.sh) + 1;
        if (rows > best) best = rows;
    }
    return best;
}

template <int MT, int NT, int STRIDE, int PT, int PX, bool DUAL = false>
tvg_status launch_instance_d(const PatchArgs &a, int ntiles, size_t lds, hipStream_t stream)
{
    auto kernel = conv3x3_patch_kernel<MT, NT, STRIDE, PT, PX, DUAL>;
    static bool configured = false;      // opt in to > 64 KB of dynamic LDS once per instance
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return TVG_ERR_LAUNCH;
        configured = true;
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)(a.mtiles * ntiles)), dim3(256), lds, stream, a);
    return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
}

template <int MT, int NT, int STRIDE, int PT, int PX>
tvg_status launch_instance(const PatchArgs &a, int ntiles, size_t lds, hipStream_t stream)
{
    if (a.oc1 > 0) {
        if constexpr (MT == 64 && NT >= 128) return launch_instance_d<MT, NT, STRIDE, PT, PX, true>(a, ntiles, lds, stream);
        else return TVG_ERR_UNSUPPORTED;
    }
    return launch_instance_d<MT, NT, STRIDE, PT, PX, false>(a, ntiles, lds, stream);
}

template <int MT, int NT, int STRIDE>
tvg_status launch_pt(const PatchArgs &a, int ntiles, size_t lds, int pt, int px, hipStream_t stream)
{
    {
        // wide loads keep the number of vector memory instructions down
        if (px == 8) {
            if (pt <= 1) return launch_instance<MT, NT, STRIDE, 1, 8>(a, ntiles, lds, stream);
            return launch_instance<MT, NT, STRIDE, 2, 8>(a, ntiles, lds, stream);
        }
        if (px == 4) {
            if (pt <= 1) return launch_instance<MT, NT, STRIDE, 1, 4>(a, ntiles, lds, stream);
            if (pt <= 2) return launch_instance<MT, NT, STRIDE, 2, 4>(a, ntiles, lds, stream);
            return launch_instance<MT, NT, STRIDE, 4, 4>(a, ntiles, lds, stream);
        }
    }
    if (px == 2) {
        if (pt <= 2) return launch_instance<MT, NT, STRIDE, 2, 2>(a, ntiles, lds, stream);
        return launch_instance<MT, NT, STRIDE, 4, 2>(a, ntiles, lds, stream);
    }
    if (pt <= 2) return launch_instance<MT, NT, STRIDE, 2, 1>(a, ntiles, lds, stream);
    if (pt <= 4) return launch_instance<MT, NT, STRIDE, 4, 1>(a, ntiles, lds, stream);
    return launch_instance<MT, NT, STRIDE, 8, 1>(a, ntiles, lds, stream);
}

template <int MT, int NT>
tvg_status launch_stride(const PatchArgs &a, int stride, int ntiles, size_t lds, int pt, int px,
                         hipStream_t stream)
{
    return stride == 1 ? launch_pt<MT, NT, 1>(a, ntiles, lds, pt, px, stream)
                       : launch_pt<MT, NT, 2>(a, ntiles, lds, pt, px, stream);
}

}  // namespace

bool conv3x3_patch_pointers_ok(const ConvPointers &ptr)
{
    // weights and input pixels are read as vectors of up to 16 bytes
    return reinterpret_cast<uintptr_t>(ptr.w) % 16 == 0 && reinterpret_cast<uintptr_t>(ptr.x) % 16 == 0;
}

bool plan_conv3x3_patch(const ConvProblem &p, Patch3x3Plan *plan, int single_stage_mt_divides)
{
    if (p.dtype != TVG_BF16 || p.R != 3 || p.S != 3 || p.ph != 1 || p.pw != 1) return false;
    if (p.sh != p.sw || (p.sh != 1 && p.sh != 2)) return false;
    if (p.IC % kChunk != 0) return false;
    if (p.npix >= (1 << 22) || (long)p.N * (p.H + 2) >= (1 << 22)) return false;   // fast_div range
    // (two-head launches: the single-stage kernel only, channel tiles that divide head 1)
    const bool dual = single_stage_mt_divides > 0;
    const Knobs knobs = dual ? Knobs{0, 0, 1, 0, 0, 0} : forced_knobs(p);
    const int force_mt = knobs.mt, force_nt = knobs.nt;
    const bool use_dbuf = knobs.stages != 1;
    // Tile choice (measured on MI355X at batch 64): take the largest tile that still gives at
    // least 1.5 workgroups per CU, wider in pixels on a tie; if none does, the tile shape with
    // the most workgroups.  A 128-channel tile with more than 4 patch tasks per thread (wide
    // stride-2 patches) runs out of registers and is skipped.
    // (128 x 256 exists in the pipelined kernel only, as its channel-split variant, and is taken
    // when a caller names it)
    // (64 x 512: single-stage kernel, stride 1, rows of 8n pixels; first in line for the layers the
    // pipelined kernel does not take - fewer than eight chunks - where it still gives 1.5 workgroups
    // per CU: C2 at batch 64, 392 tiles in one round instead of 784 in two, 24.6 -> 22.6 us)
    const int cands[7][2] = {{64, 512}, {64, 256}, {128, 128}, {64, 128}, {128, 64}, {64, 64}, {128, 256}};
    Patch3x3Plan best{};
    bool found = false, best_fills = false;
    for (const auto &c : cands) {
        const int mt = c[0], nt = c[1];
        if (mt == 128 && p.OC <= 64) continue;
        if (dual && (mt != 64 || nt < 128 || single_stage_mt_divides % mt != 0)) continue;
        if (force_mt && mt != force_mt) continue;
        if (force_nt && nt != force_nt) continue;
        if (mt == 128 && nt == 256 && !(force_mt == 128 && force_nt == 256)) continue;
        if (nt == 512 && (p.sh != 1 || dual || p.W % 8 != 0 || (force_nt != 512 && p.IC >= 8 * kChunk))) continue;
        const int rows = max_patch_rows(p, nt);
        // two pixels per load when the rows are even (32-bit aligned pairs) and that keeps the
        // task count within the instances built for it
        int px = p.W % 2 == 0 ? 2 : 1;
        // 16- or 8-byte loads where the rows allow them (x is 16-byte aligned, and so is every
        // row when W % 8 == 0): a stride-2 patch is four times the output tile (measured at
        // batch 64 with the split rows: C4 26.0 -> 24.2 us, C7 unchanged); at stride 1 they pay
        // under the 256-pixel tile only (C2 30.5 -> 28.9 us; under 64x128 31.4 -> 32.9: the wider
        // a task, the more of its lanes' 16-byte LDS stores fall on the same banks)
        if ((p.sh == 2 || nt >= 256) && p.W % 2 == 0) {
            // (a row that is no multiple of the load ends in a shorter task, loads 4-byte aligned)
            const auto tasks = [&](int q) { return (2 * rows * ((p.W + q - 1) / q) + 255) / 256; };
            if (p.W >= 8 && tasks(8) <= 2 && (p.W % 8 == 0 || tasks(8) < tasks(4))) px = 8;
            else if (p.W >= 4 && tasks(4) <= 4) px = 4;
        }
        int pt = (2 * rows * ((p.W + px - 1) / px) + 255) / 256;
        if (px == 2 && pt > 4) { px = 1; pt = (2 * rows * p.W + 255) / 256; }
        // operand planes (the tail's staging areas, 20 KB, reuse them) + (scale, offset) pairs
        const size_t lds = std::max(2 * ((size_t)9 * mt * kWordBytes + 128) + 2 * (size_t)rows * (p.W + 2) * kWordBytes,
                                    (size_t)4 * 2 * kStageBytes) + (size_t)mt * 8;
        const long tiles = (long)((p.OC + mt - 1) / mt) * ((p.npix + nt - 1) / nt);
        Patch3x3Plan cand{mt, nt, pt, px, rows, lds, tiles, 0, 0, 0, 0, 0, 1,
                          knobs.split_k, knobs.lds_pitch, knobs.row_loads, knobs.stages};
        if (dual && nt == 256 && pt > 1) continue;    // (those two-head instances run out of registers)
        if (nt == 512 && !(px == 8 && pt <= 1)) continue;      // (the one instance built)
        if (!(use_dbuf && plan_conv3x3_dbuf(p, &cand))) {
            if (knobs.stages == 2) continue;      // the caller asked for the pipelined kernel
            if (mt == 128 && nt == 256) continue; // (no single-stage instance of that tile)
            if (pt > 8 || lds > 80 * 1024) continue;
            if (mt == 128 && pt > 4 && !force_mt) continue;
        }
        // the pipelined kernel keeps a CU busy with one workgroup: three quarters of the CUs
        // covered is enough for it; the single-stage kernel wants 1.5 workgroups per CU
        const bool fills = cand.dbuf ? 4 * tiles >= 3 * kComputeUnits : 2 * tiles >= 3 * kComputeUnits;
        if (!found || (!best_fills && (fills || tiles > best.tiles))) {
            best = cand;
            best_fills = fills;
            found = true;
        }
    }
    if (!found) return false;
    *plan = best;
    return true;
}

tvg_status launch_conv3x3_patch(const ConvProblem &p, const Patch3x3Plan &plan,
                                const ConvPointers &ptr, hipStream_t stream, const DualHead *dual)
{
    if (plan.dbuf) return dual ? TVG_ERR_UNSUPPORTED : launch_conv3x3_dbuf(p, plan, ptr, stream);
    PatchArgs a;
    a.oc1 = dual ? dual->oc1 : 0;
    a.relu2 = dual ? dual->relu2 : 0;
    a.centre2 = dual ? dual->centre2 : 0;
    a.y2 = dual ? static_cast<bf16_t *>(dual->y2) : nullptr;
    a.x = static_cast<const bf16_t *>(ptr.x); a.w = static_cast<const bf16_t *>(ptr.w);
    a.scale = ptr.scale; a.shift = ptr.shift; a.bias = ptr.bias;
    a.residual = static_cast<const bf16_t *>(ptr.residual); a.y = static_cast<bf16_t *>(ptr.y);
    a.N = p.N; a.IC = p.IC; a.H = p.H; a.W = p.W; a.OC = p.OC; a.OH = p.OH; a.OW = p.OW;
    a.npix = p.npix; a.relu = p.relu | (p.stream_out << 1);
    a.mtiles = (p.OC + plan.mt - 1) / plan.mt;
    a.vmode = pick_store_vmode(p.dtype, p.OH * p.OW, ptr.y, ptr.residual);
    if (dual && pick_store_vmode(p.dtype, p.OH * p.OW, dual->y2, nullptr) < a.vmode)
        a.vmode = pick_store_vmode(p.dtype, p.OH * p.OW, dual->y2, nullptr);
    a.ss_offset = (int)(plan.lds_bytes - (size_t)plan.mt * 8);
    a.x_bytes = (uint32_t)((size_t)p.N * p.IC * p.H * p.W * 2);
    a.w_bytes = (uint32_t)((size_t)p.OC * p.IC * 9 * 2);
    const int ntiles = (p.npix + plan.nt - 1) / plan.nt;
    a.ntiles = ntiles;
    a.m_major = (size_t)p.OC * p.IC * 9 > (size_t)p.N * p.IC * p.H * p.W;
    if (plan.nt == 512) {
        if (p.sh == 1 && plan.px == 8 && plan.pt <= 1 && !dual)
            return launch_instance_d<64, 512, 1, 1, 8, false>(a, ntiles, plan.lds_bytes, stream);
        return TVG_ERR_UNSUPPORTED;
    }
    if (plan.nt == 256)
        return launch_stride<64, 256>(a, p.sh, ntiles, plan.lds_bytes, plan.pt, plan.px, stream);
    if (plan.mt == 128 && plan.nt == 128)
        return launch_stride<128, 128>(a, p.sh, ntiles, plan.lds_bytes, plan.pt, plan.px, stream);
    if (plan.mt == 128)
        return launch_stride<128, 64>(a, p.sh, ntiles, plan.lds_bytes, plan.pt, plan.px, stream);
    if (plan.nt == 128)
        return launch_stride<64, 128>(a, p.sh, ntiles, plan.lds_bytes, plan.pt, plan.px, stream);
    return launch_stride<64, 64>(a, p.sh, ntiles, plan.lds_bytes, plan.pt, plan.px, stream);
}

}  // namespace tvg
