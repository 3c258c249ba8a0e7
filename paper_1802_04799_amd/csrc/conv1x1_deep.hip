// bf16 1x1 (pointwise) fused conv2d, stride 1, for DEEP reductions (IC a multiple of 128): the
// 512 -> 512 and 1024 -> 1024 layers of MobileNet and the bottleneck layers of ResNet-50.
//
// The general pointwise kernel fetches its pixel operand one element per load (the channel axis
// is the slowest of NCHW) and keeps one 32-channel chunk in flight; on a reduction of 512
// channels over a 14x14 map that is 16 round trips to memory and 10 load instructions per 4
// matrix instructions (measured 16.5 us for 3.3 GFLOP at batch 32).  Here (TVM paper Section 4.2,
// cooperative fetch; Section 4.4, latency hiding):
//   - a load task is a run of 4 or 8 CONSECUTIVE pixels of one channel (8 or 16 bytes; pixels of
//     an image are contiguous whatever the row length, a 1x1 filter has no halo), eight channels
//     per task, transposed in registers (v_perm_b32) into the 16-byte words [pixel][8 channels]
//     that the matrix instruction consumes;
//   - a step covers 64 channels, and the loads of two steps are in flight while a third is
//     multiplied: two register sets, two LDS stages, one barrier per step;
//   - operands live in LDS as planes of dense 16-byte words, [channel octet][row]: the 16-byte
//     reads of 16 consecutive lanes are consecutive words (conflict-free, no padding).
// Tile: 64 output channels x 128 pixels, four waves of 32 x 64.
#include <type_traits>

#include "tvg_device.h"
#include "tvg_internal.h"

namespace tvg {

namespace {

struct PwDeepArgs {
    const bf16_t *x, *w;
    const float *scale, *shift, *bias;
    const bf16_t *residual;
    bf16_t *y;
    int IC, HW, OC, npix, relu, mtiles, vmode;
    uint32_t x_bytes, w_bytes;
    float inv_hw;
};

constexpr int kMT = 64, kNT = 128;
constexpr int kKS = 64;                  // channels per step: 8 octets, 4 matrix-instruction k-steps
constexpr int kAWords = 8 * kMT, kBWords = 8 * kNT;
constexpr int kStage = (kAWords + kBWords) * 16;
constexpr int kRsrcFlags = 0x00020000;   // raw buffer descriptor word 3 on gfx9-family targets
constexpr uint32_t kOutOfRange = 0x80000000u;

__device__ __forceinline__ int xcd_remap(int bid, int nb)
{
    const int q = nb >> 3, rem = nb & 7;
    const int xcd = bid & 7, local = bid >> 3;
    return xcd < rem ? xcd * (q + 1) + local : rem * (q + 1) + (xcd - rem) * q + local;
}

// 16-bit half `ha` of a in the low half of the result, half `hb` of b in the high half.
__device__ __forceinline__ uint32_t pack_halves(uint32_t a, int ha, uint32_t b, int hb)
{
    const uint32_t sel = (ha ? 0x0302u : 0x0100u) | (hb ? 0x07060000u : 0x05040000u);
    return __builtin_amdgcn_perm(b, a, sel);
}

// PX = pixels per load: 8 (HW % 8 == 0, 16-byte loads; the tile's 128 tasks sit in waves 0 and 1)
// or 4 (HW % 4 == 0, 8-byte loads; one task per thread).
template <int PX>
__global__ __launch_bounds__(256) void conv1x1_deep_kernel(const PwDeepArgs a)
{
    constexpr int MI = 1, NJ = 2;                 // wave tile: 32 channels x 64 pixels
    constexpr int PW32 = PX / 2;                  // registers per load
    constexpr int NTASK = (kNT / PX) * 8;         // 256 or 128
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * kStage];
    __shared__ float ss_lds[2 * kMT];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int tile = xcd_remap(blockIdx.x, gridDim.x);
    // consecutive tiles (one XCD's L2) are the channel tiles over one pixel range
    const int m0 = (tile % a.mtiles) * kMT;
    const int n0 = (tile / a.mtiles) * kNT;
    const int HW = a.HW;

    stage_scale_shift(ss_lds, m0, kMT, a.scale, a.shift, a.bias, a.OC, tid, 256);

    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(a.x), 0, a.x_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(a.w), 0, a.w_bytes, kRsrcFlags);

    // ---- fixed load slots ------------------------------------------------------------------
    // weights: word wi = row wi % 64 of octet wi / 64; rows past OC read row 0 (never stored)
    uint32_t aoff[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int wi = tid + 256 * i, o = wi >> 6, r = wi & 63;
        aoff[i] = 2u * (uint32_t)((m0 + r < a.OC ? m0 + r : 0) * a.IC + o * 8);
    }
    // pixels: task = (group of PX consecutive pixels, channel octet), groups fastest over the lanes
    const bool loader = NTASK == 256 || tid < NTASK;          // uniform per wave
    const int grp = tid % (kNT / PX), oct = tid / (kNT / PX);
    uint32_t boff = kOutOfRange;                                // groups past the end read zeros
    {
        const int p = n0 + grp * PX;
        if (loader && p < a.npix) {
            int rem;
            const int n = fast_div(p, HW, a.inv_hw, &rem);
            boff = 2u * (uint32_t)((n * a.IC + oct * 8) * HW + rem);
        }
    }
    const int bdst = kAWords * 16 + (oct * kNT + grp * PX) * 16;
    const int hw2 = HW * 2;

    uint4v areg[2][2];
    uint32_t braw[2][8][PW32];
    auto issue = [&](int s, auto setc) __attribute__((always_inline)) {
        constexpr int R = decltype(setc)::value;
#pragma unroll
        for (int i = 0; i < 2; ++i)
            areg[R][i] = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, aoff[i], s * kKS * 2, 0));
        // (threads without a task load too, from an out-of-range offset: a conditional load would make
        // the compiler's wait before a commit cover every outstanding load, and the look-ahead is lost)
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int soff = (s * kKS + q) * hw2;
            if constexpr (PX == 8) {
                const uint4v t4 = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, boff, soff, 0));
#pragma unroll
                for (int d = 0; d < 4; ++d) braw[R][q][d] = t4[d];
            } else {
                const uint2v t2 = __builtin_bit_cast(uint2v, __builtin_amdgcn_raw_buffer_load_b64(xrsrc, boff, soff, 0));
                braw[R][q][0] = t2[0];
                braw[R][q][1] = t2[1];
            }
        }
    };
    // register set R -> LDS stage st: the weights as they are, the pixels transposed
    auto commit = [&](auto setc, int st) __attribute__((always_inline)) {
        constexpr int R = decltype(setc)::value;
        unsigned char *base = lds + st * kStage;
#pragma unroll
        for (int i = 0; i < 2; ++i) *reinterpret_cast<uint4v *>(base + (tid + 256 * i) * 16) = areg[R][i];
        if (loader) {
#pragma unroll
            for (int k = 0; k < PX; ++k) {
                uint4v o;
#pragma unroll
                for (int d = 0; d < 4; ++d)
                    o[d] = pack_halves(braw[R][2 * d][k >> 1], k & 1, braw[R][2 * d + 1][k >> 1], k & 1);
                *reinterpret_cast<uint4v *>(base + bdst + k * 16) = o;
            }
        }
    };

    float16v acc[MI][NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[0][j][v] = 0.0f;

    auto multiply = [&](int st) __attribute__((always_inline)) {
        const unsigned char *As = lds + st * kStage, *Bs = As + kAWords * 16;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int o = 2 * ks + lhalf;
            const uint4v af = *reinterpret_cast<const uint4v *>(As + (o * kMT + wm * 32 + lrow) * 16);
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const uint4v bf = *reinterpret_cast<const uint4v *>(Bs + (o * kNT + wn * 64 + j * 32 + lrow) * 16);
                // pixel operand first: the accumulator tile is D[pixel][channel]
                acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8v, bf), __builtin_bit_cast(bf16x8v, af), acc[0][j], 0, 0, 0);
            }
        }
    };

    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    // The number of steps is even (IC % 128 == 0).  Loads are issued unconditionally - past the end
    // they fetch the last step again - so that the waits before a commit count instructions.
    const int nsteps = a.IC / kKS, last = nsteps - 1;
    issue(0, S0{});
    issue(1, S1{});
    commit(S0{}, 0);
    issue(min(2, last), S0{});
    __syncthreads();
    for (int s = 0; s < nsteps; s += 2) {
        // stage 0 holds step s; set 1 holds step s + 1, set 0 step s + 2
        commit(S1{}, 1);
        multiply(0);
        issue(min(s + 3, last), S1{});
        __syncthreads();
        // stage 1 holds step s + 1; set 0 holds step s + 2, set 1 step s + 3
        if (s + 2 < nsteps) commit(S0{}, 0);
        multiply(1);
        issue(min(s + 4, last), S0{});
        __syncthreads();
    }

    unsigned char *stage = lds + wave * (MI * NJ * kStageBytes);
    const TailArgs tail{a.scale, a.shift, a.bias, a.residual, a.y, a.OC, HW, a.npix, a.relu};
    store_acc_tiles_batched<MI, NJ>(acc, stage, lane, m0 + wm * 32, n0 + wn * 64, tail, a.vmode, ss_lds,
                                    wm * 32);
}

}  // namespace

bool plan_conv1x1_deep(const ConvProblem &p, PwDeepPlan *plan)
{
    if (p.dtype != TVG_BF16 || p.R != 1 || p.S != 1 || p.ph != 0 || p.pw != 0) return false;
    if (p.sh != 1 || p.sw != 1) return false;
    if (p.IC % 128 != 0) return false;
    const int HW = p.H * p.W;
    if (HW % 4 != 0) return false;
    if ((size_t)p.N * p.IC * HW * 2 >= (size_t)kOutOfRange || p.npix >= (1 << 22)) return false;
    plan->px = HW % 8 == 0 ? 8 : 4;
    plan->tiles = (long)((p.OC + kMT - 1) / kMT) * ((p.npix + kNT - 1) / kNT);
    return true;
}

bool conv1x1_deep_pointers_ok(const ConvPointers &ptr)
{
    return reinterpret_cast<uintptr_t>(ptr.w) % 16 == 0 && reinterpret_cast<uintptr_t>(ptr.x) % 16 == 0;
}

tvg_status launch_conv1x1_deep(const ConvProblem &p, const PwDeepPlan &plan, const ConvPointers &ptr,
                               hipStream_t stream)
{
    PwDeepArgs a;
    a.x = static_cast<const bf16_t *>(ptr.x); a.w = static_cast<const bf16_t *>(ptr.w);
    a.scale = ptr.scale; a.shift = ptr.shift; a.bias = ptr.bias;
    a.residual = static_cast<const bf16_t *>(ptr.residual); a.y = static_cast<bf16_t *>(ptr.y);
    a.IC = p.IC; a.HW = p.H * p.W; a.OC = p.OC; a.npix = p.npix;
    a.relu = p.relu | (p.stream_out << 1);
    a.mtiles = (p.OC + kMT - 1) / kMT;
    a.vmode = pick_store_vmode(p.dtype, a.HW, ptr.y, ptr.residual);
    a.x_bytes = (uint32_t)((size_t)p.N * p.IC * a.HW * 2);
    a.w_bytes = (uint32_t)((size_t)p.OC * p.IC * 2);
    a.inv_hw = 1.0f / (float)a.HW;
    const unsigned grid = (unsigned)plan.tiles;
    if (plan.px == 8) hipLaunchKernelGGL(conv1x1_deep_kernel<8>, dim3(grid), dim3(256), 0, stream, a);
    else hipLaunchKernelGGL(conv1x1_deep_kernel<4>, dim3(grid), dim3(256), 0, stream, a);
    return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
}

}  // namespace tvg
