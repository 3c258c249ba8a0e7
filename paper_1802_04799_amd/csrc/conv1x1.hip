// bf16 1x1 (pointwise) fused conv2d, stride 1 or 2, on MFMA: y[oc, p] = sum_ic w[oc, ic] *
// x[ic, pixel p], a GEMM whose K axis (ic) is the slowest axis of the NCHW input.
//
// These layers (Table 2's C3, C5, C8, C11) have 20-80 FLOP per byte at batch 64, far
// below the bf16 ridge of the chip, so the kernel is organised around the memory side:
// no filter taps, no halo and no bounds masks; every thread owns fixed (pixel, channel
// octet) slots whose byte offsets are computed once, and per K chunk of 32 channels it
// issues its loads through a buffer descriptor (uniform base + per-lane offset + scalar
// channel offset, i.e. no vector address arithmetic), packs 8 channels of one pixel into
// a 16-byte LDS word (the transposition NCHW -> K-innermost happens in registers) and the
// wave tiles run 32x32x16 MFMAs from LDS.  Weight rows are contiguous in ic and are copied
// as 16-byte vectors.  Loads of chunk c+1 are in flight during the MFMAs of chunk c
// (cooperative fetch + latency hiding, TVM paper Sections 4.2 and 4.4); the fused tail
// (Section 3) runs on the accumulators with vector stores.
#include <stdio.h>
#include <stdlib.h>
#include "tvg_device.h"
#include "tvg_internal.h"

namespace tvg {

namespace {

struct PwArgs {
    const bf16_t *x, *w;
    const float *scale, *shift, *bias;
    const bf16_t *residual;
    bf16_t *y;
    int N, IC, H, W, OC, OH, OW, stride, npix, relu, mtiles, vmode;
    uint32_t x_bytes, w_bytes;
    int ntiles, m_major;
};

constexpr int kRow = 80;                 // bytes per LDS row: 32 channels (64 B) + 16 B padding
constexpr int kKC = 32;                  // channels per K chunk
constexpr int kRsrcFlags = 0x00020000;   // raw buffer descriptor word 3 on gfx9-family targets
constexpr uint32_t kOutOfRange = 0xFFFFFFF0u;

__device__ __forceinline__ int xcd_remap(int bid, int nb)
{
    const int q = nb >> 3, rem = nb & 7;
    const int xcd = bid & 7, local = bid >> 3;
    return xcd < rem ? xcd * (q + 1) + local : rem * (q + 1) + (xcd - rem) * q + local;
}

// NCH > 0: the reduction is exactly NCH chunks and all of them are fetched before the first is
// used, each into registers of its own.  These layers do 4 to 16 MFMAs per wave and chunk, so
// with one chunk in flight at a time every chunk costs a full memory latency (measured: 8
// chunks, 12 us); with all in flight the latency is paid once.  NCH = 0: any number of whole
// chunks, a rolling window of them ahead (see PF below).  NCH < 0: any channel count, the last
// chunk ragged, one chunk ahead.
template <int MT, int NT, int NCH>
__global__ __launch_bounds__(256) void conv1x1_kernel(const PwArgs a)
{
    constexpr int WTM = MT / 2, WTN = NT / 2;
    constexpr int MI = WTM / 32, NJ = WTN / 32;
    constexpr int BT = NT * 4 / 256;          // (pixel, octet) slots per thread
    constexpr int AT = MT * 4 / 256;          // weight vectors per thread
    static_assert(MT % 64 == 0 && NT % 64 == 0, "whole load slots per thread");
    constexpr int OPER = (MT + NT) * kRow;
    constexpr int STAGE = 4 * MI * NJ * kStageBytes;    // the epilogue stages all of a wave's tiles
    __shared__ __attribute__((aligned(16))) unsigned char lds[OPER > STAGE ? OPER : STAGE];
    __shared__ float ss_lds[2 * MT];
    unsigned char *As = lds, *Bs = lds + MT * kRow;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int tile = xcd_remap(blockIdx.x, gridDim.x);
    // Consecutive tiles (which share an XCD's L2) share the larger operand: the same pixel
    // tile under all channel tiles, or - when the weights outweigh the input - the same
    // channel tile over consecutive pixel tiles.
    const int m0 = (a.m_major ? tile / a.ntiles : tile % a.mtiles) * MT;
    const int n0 = (a.m_major ? tile % a.ntiles : tile / a.mtiles) * NT;
    const int HW = a.H * a.W, OHW = a.OH * a.OW;

    stage_scale_shift(ss_lds, m0, MT, a.scale, a.shift, a.bias, a.OC, tid, 256);

    // ---- fixed load slots ------------------------------------------------------------------
    uint32_t boff[BT];          // byte offset of (pixel, channel 8*octet) in x, or out of range
    int bdst[BT], boct[BT];
#pragma unroll
    for (int j = 0; j < BT; ++j) {
        const int t = tid + j * 256;
        const int pl = t % NT, octet = t / NT;      // lanes run over pixels: coalesced loads
        const int p = n0 + pl;
        boct[j] = octet;
        bdst[j] = pl * kRow + octet * 16;
        boff[j] = 0;       // pixels past the end read pixel 0; their columns are never stored
        if (p < a.npix) {
            const int n = p / OHW, rem = p - n * OHW;
            const int oh = rem / a.OW, ow = rem - oh * a.OW;
            boff[j] = 2u * (uint32_t)((n * a.IC + octet * 8) * HW + oh * a.stride * a.W +
                                      ow * a.stride);
        }
    }
    uint32_t aoff[AT];
    int adst[AT], akv[AT];
#pragma unroll
    for (int i = 0; i < AT; ++i) {
        const int v = tid + i * 256;
        const int row = v >> 2, kv = v & 3;
        akv[i] = kv;
        adst[i] = row * kRow + kv * 16;
        // rows past OC read row 0; their accumulators are never stored
        aoff[i] = 2u * (uint32_t)((m0 + row < a.OC ? m0 + row : 0) * a.IC + kv * 8);
    }

    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(a.x), 0, a.x_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(a.w), 0, a.w_bytes, kRsrcFlags);

    // NCH = 0: PF chunks ahead, each in a register set of its own that is refilled as soon as its
    // chunk has gone to LDS.  With one chunk ahead every chunk cost a memory latency, because the
    // 4 to 8 MFMAs of a chunk are over long before its successor arrives, and a layer that leaves
    // a CU one or two workgroups has nothing else to run meanwhile (512 -> 512 channels on 6272
    // pixels: 16 chunks, 17.4 us, 190 TFLOP/s).
    constexpr int PF = (MT == 128 && NT == 128) ? 2 : 4;
    constexpr int NS = NCH > 0 ? NCH : NCH == 0 ? PF : 1;     // register sets
    uint32_t braw[NS][BT][8];
    uint4v areg[NS][AT];
    // Full chunks (all 32 channels below IC) use the scalar offset operand for the channel
    // term; a ragged last chunk builds complete per-lane offsets so that channels past IC
    // are unambiguously out of range of the descriptor and read as zeros.
    auto load_chunk = [&](int c, int set) __attribute__((always_inline)) {
        const int c0 = c * kKC;
        if (NCH >= 0 || c0 + kKC <= a.IC) {
#pragma unroll
            for (int j = 0; j < BT; ++j)
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    braw[set][j][q] =
                        __builtin_amdgcn_raw_buffer_load_b16(xrsrc, boff[j], (c0 + q) * HW * 2, 0);
#pragma unroll
            for (int i = 0; i < AT; ++i)
                areg[set][i] = __builtin_bit_cast(
                    uint4v, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, aoff[i], c0 * 2, 0));
        } else {
#pragma unroll
            for (int j = 0; j < BT; ++j) {
                const bool ok = c0 + boct[j] * 8 < a.IC;
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const uint32_t off = ok ? boff[j] + (uint32_t)((c0 + q) * HW * 2) : kOutOfRange;
                    braw[set][j][q] = __builtin_amdgcn_raw_buffer_load_b16(xrsrc, off, 0, 0);
                }
            }
#pragma unroll
            for (int i = 0; i < AT; ++i) {
                const uint32_t off = (c0 + akv[i] * 8 < a.IC) ? aoff[i] + (uint32_t)(c0 * 2) : kOutOfRange;
                areg[set][i] = __builtin_bit_cast(
                    uint4v, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, off, 0, 0));
            }
        }
    };
    auto store_chunk = [&](int set) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < BT; ++j)
            *reinterpret_cast<uint4v *>(Bs + bdst[j]) = uint4v{
                braw[set][j][0] | (braw[set][j][1] << 16), braw[set][j][2] | (braw[set][j][3] << 16),
                braw[set][j][4] | (braw[set][j][5] << 16), braw[set][j][6] | (braw[set][j][7] << 16)};
#pragma unroll
        for (int i = 0; i < AT; ++i)
            *reinterpret_cast<uint4v *>(As + adst[i]) = areg[set][i];
    };

    float16v acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    auto mfma_chunk = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            uint4v af[MI], bf[NJ];
#pragma unroll
            for (int i = 0; i < MI; ++i)
                af[i] = *reinterpret_cast<const uint4v *>(
                    As + (wm * WTM + i * 32 + lrow) * kRow + ks * 32 + lhalf * 16);
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                bf[j] = *reinterpret_cast<const uint4v *>(
                    Bs + (wn * WTN + j * 32 + lrow) * kRow + ks * 32 + lhalf * 16);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    // pixel operand first: the accumulator tile is D[pixel][channel]
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8v, bf[j]), __builtin_bit_cast(bf16x8v, af[i]),
                        acc[i][j], 0, 0, 0);
        }
    };

    if constexpr (NCH > 0) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) load_chunk(c, c);
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            store_chunk(c);
            __syncthreads();
            mfma_chunk();
            __syncthreads();          // (the last one frees the operand tiles for the tail)
        }
    } else if constexpr (NCH < 0) {
        const int nchunks = (a.IC + kKC - 1) / kKC;
        load_chunk(0, 0);
        store_chunk(0);
        __syncthreads();
        for (int c = 0; c < nchunks; ++c) {
            if (c + 1 < nchunks) load_chunk(c + 1, 0);
            mfma_chunk();
            __syncthreads();
            if (c + 1 < nchunks) {
                store_chunk(0);
                __syncthreads();
            }
        }
    } else {
        // (a multiple of PF chunks, the launcher sees to that.  Every load below is issued
        // unconditionally - the last group of PF chunks is peeled off for that - because a wait on
        // the memory counter can leave the younger loads in flight only if they are certain to
        // have been issued: behind a branch they force a wait for everything.)
        const int nchunks = a.IC / kKC;
#pragma unroll
        for (int s = 0; s < PF; ++s) {
            load_chunk(s, s);
            __builtin_amdgcn_sched_barrier(0);    // (issue order = consumption order)
        }
        for (int c0 = 0; c0 + PF < nchunks; c0 += PF) {
#pragma unroll
            for (int s = 0; s < PF; ++s) {
                store_chunk(s);
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
                load_chunk(c0 + s + PF, s);
                __builtin_amdgcn_sched_barrier(0);
                mfma_chunk();
                __syncthreads();
            }
        }
#pragma unroll
        for (int s = 0; s < PF; ++s) {    // the last group: nothing left to fetch
            store_chunk(s);
            __syncthreads();
            mfma_chunk();
            __syncthreads();              // (the last one frees the operand tiles for the tail)
        }
    }

    unsigned char *stage = lds + wave * (MI * NJ * kStageBytes);
    const TailArgs tail{a.scale, a.shift, a.bias, a.residual, a.y, a.OC, OHW, a.npix, a.relu};
    store_acc_tiles_batched<MI, NJ>(acc, stage, lane, m0 + wm * WTM, n0 + wn * WTN, tail, a.vmode,
                                    ss_lds, wm * WTM);
}

}  // namespace

bool plan_conv1x1(const ConvProblem &p, Pw1x1Plan *plan)
{
    if (p.dtype != TVG_BF16 || p.R != 1 || p.S != 1 || p.ph != 0 || p.pw != 0) return false;
    if (p.sh != p.sw || (p.sh != 1 && p.sh != 2)) return false;
    if (p.IC % 8 != 0) return false;
    if ((size_t)p.N * p.IC * p.H * p.W * 2 > (size_t)kOutOfRange) return false;
    // Tile choice (measured on MI355X at batch 64 over the ResNet-18, MobileNet and ResNet-50
    // pointwise shapes): a narrow pixel tile under as many output channels as possible - the
    // input is what costs loads, one per element, so it should be fetched by few workgroups -
    // as long as that gives 1.5 workgroups per CU; (128, 64) was best or within 10 % of the best
    // on 17 of 20 shapes, the wider tiles on none by more.  A single-chunk reduction under a
    // 64-channel tile is bound by its output stream and prefers the wide tile.
    const int deep[4][2] = {{128, 64}, {64, 64}, {128, 128}, {64, 128}};
    const int shallow[4][2] = {{64, 128}, {64, 64}, {128, 64}, {128, 128}};
    const auto &cands = (p.OC <= 64 && p.IC < 64) ? shallow : deep;
    bool found = false, fills_best = false;
    int force_mt = 0, force_nt = 0;       // tuning override, as for the 3x3 kernels
    {
        const Knobs knobs = forced_knobs(p);
        force_mt = knobs.mt;
        force_nt = knobs.nt;
    }
    for (const auto &c : cands) {
        const int mt = c[0], nt = c[1];
        if (mt == 128 && p.OC <= 64) continue;
        if ((force_mt && mt != force_mt) || (force_nt && nt != force_nt)) continue;
        const long tiles = (long)((p.OC + mt - 1) / mt) * ((p.npix + nt - 1) / nt);
        const bool fills = 2 * tiles >= 3 * kComputeUnits;
        if (!found || (!fills_best && (fills || tiles > plan->tiles))) {
            plan->mt = mt; plan->nt = nt; plan->tiles = tiles;
            fills_best = fills;
            found = true;
        }
    }
    return found;
}

bool conv1x1_pointers_ok(const ConvPointers &ptr)
{
    return reinterpret_cast<uintptr_t>(ptr.w) % 16 == 0 && reinterpret_cast<uintptr_t>(ptr.x) % 2 == 0;
}

tvg_status launch_conv1x1(const ConvProblem &p, const Pw1x1Plan &plan, const ConvPointers &ptr,
                          hipStream_t stream)
{
    PwArgs a;
    a.x = static_cast<const bf16_t *>(ptr.x); a.w = static_cast<const bf16_t *>(ptr.w);
    a.scale = ptr.scale; a.shift = ptr.shift; a.bias = ptr.bias;
    a.residual = static_cast<const bf16_t *>(ptr.residual); a.y = static_cast<bf16_t *>(ptr.y);
    a.N = p.N; a.IC = p.IC; a.H = p.H; a.W = p.W; a.OC = p.OC; a.OH = p.OH; a.OW = p.OW;
    a.stride = p.sh; a.npix = p.npix; a.relu = p.relu | (p.stream_out << 1);
    a.mtiles = (p.OC + plan.mt - 1) / plan.mt;
    a.ntiles = (p.npix + plan.nt - 1) / plan.nt;
    a.m_major = (size_t)p.OC * p.IC > (size_t)p.N * p.IC * p.H * p.W;
    a.vmode = pick_store_vmode(p.dtype, p.OH * p.OW, ptr.y, ptr.residual);
    a.x_bytes = (uint32_t)((size_t)p.N * p.IC * p.H * p.W * 2);
    a.w_bytes = (uint32_t)((size_t)p.OC * p.IC * 2);
    const unsigned grid = (unsigned)plan.tiles;
    // whole reduction in flight at once when it is 2, 4 or 8 full chunks and the registers fit
    // (measured at batch 64: C11, 8 chunks, 13.0 -> 11.5 us)
    int nch = p.IC % kKC == 0 ? p.IC / kKC : -1;
    if (nch > 0 && ((nch != 2 && nch != 4 && nch != 8) || (nch == 8 && plan.mt == 128 && plan.nt == 128))) {
        // the rolling window takes whole groups of PF chunks (4, or 2 under the 128 x 128 tile;
        // eight sets under the 64-pixel tiles, refilled one by one or four at a time, were slower:
        // 512 -> 512 at 14x14 14.6 and 15.4 us against 13.1; two LDS stages with one barrier per
        // chunk made single layers 3-10 % faster in a warm loop and changed the chains and the
        // step by less than 1 % either way on one box: not kept)
        const int pf = (plan.mt == 128 && plan.nt == 128) ? 2 : 4;
        nch = nch % pf == 0 ? 0 : -1;
    }
#define TVG_PW_LAUNCH(MT_, NT_)                                                                     \
    do {                                                                                           \
        if (nch == 2)                                                                              \
            hipLaunchKernelGGL((conv1x1_kernel<MT_, NT_, 2>), dim3(grid), dim3(256), 0, stream, a);   \
        else if (nch == 4)                                                                         \
            hipLaunchKernelGGL((conv1x1_kernel<MT_, NT_, 4>), dim3(grid), dim3(256), 0, stream, a);   \
        else if (nch == 8)                                                                         \
            hipLaunchKernelGGL((conv1x1_kernel<MT_, NT_, (MT_ == 128 && NT_ == 128) ? 2 : 8>),       \
                               dim3(grid), dim3(256), 0, stream, a);                               \
        else if (nch == 0)                                                                         \
            hipLaunchKernelGGL((conv1x1_kernel<MT_, NT_, 0>), dim3(grid), dim3(256), 0, stream, a);   \
        else                                                                                       \
            hipLaunchKernelGGL((conv1x1_kernel<MT_, NT_, -1>), dim3(grid), dim3(256), 0, stream, a);  \
    } while (0)
    if (plan.mt == 128 && plan.nt == 128) TVG_PW_LAUNCH(128, 128);
    else if (plan.mt == 128) TVG_PW_LAUNCH(128, 64);
    else if (plan.nt == 128) TVG_PW_LAUNCH(64, 128);
    else TVG_PW_LAUNCH(64, 64);
#undef TVG_PW_LAUNCH
    return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
}

}  // namespace tvg
