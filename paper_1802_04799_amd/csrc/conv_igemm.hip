// Dense fused conv2d as an implicit GEMM on the gfx950 matrix cores.
//
// GEMM view (TVM paper, Table 2 operators C1..C12; Section 4.3 "tensorization":
// the reduction loop is a sequence of calls to a hardware tensor intrinsic):
//     rows    M = output channels
//     columns N = output pixels (n, oh, ow) flattened
//     depth   K = (ic, r, s) flattened in OIHW order
// so that NCHW output stores and the gathered input loads are contiguous along
// `ow` across the lanes of a wavefront, and weight rows are contiguous in K.
//
// One workgroup = 256 threads = 4 wavefronts computes an MT x 128 tile.  Per K
// chunk of 64 bytes (16 fp32 / 32 bf16 values) the workgroup cooperatively
// stages the weight tile and the gathered input tile in LDS (Section 4.2,
// cooperative fetch into a shared memory scope), out-of-image taps as zeros,
// both K-innermost so that every lane reads its MFMA operand as one 16-byte
// LDS load.  The next chunk's global loads are issued before the MFMAs of the
// current chunk and land in the other LDS buffer (Section 4.4's latency hiding,
// done here with register prefetch + double buffering).  The fused tail runs on
// the accumulators; nothing but y (or split-K partials) is written to memory.
#include "tvg_device.h"
#include "tvg_internal.h"

namespace tvg {

namespace {

struct IgemmArgs {
    const void *x, *w;
    const float *scale, *shift, *bias;
    const void *residual;
    void *y;
    float *ws;
    int N, IC, H, W, OC, R, S, sh, sw, ph, pw, OH, OW;
    int K, npix, relu;
    int mtiles, splits, k_per_split;
    int w_vec_ok;      // weight rows may be read as aligned 16-byte vectors
    int vmode;         // pixels per vector store in the epilogue (8, 4 or 1)
};

constexpr int kThreads = 256;
constexpr int kNT = 128;        // pixels per workgroup tile
constexpr int kLdsRow = 80;     // bytes per LDS row: 64 of data + 16 of padding (conflict-free b128)

// Workgroups are dealt round-robin to the 8 XCDs; hand each XCD a contiguous
// range of tiles so that neighbouring tiles (shared halos, shared weights) meet
// in the same L2.
__device__ __forceinline__ int xcd_remap(int bid, int nb)
{
    const int q = nb >> 3, rem = nb & 7;
    const int xcd = bid & 7, local = bid >> 3;
    return xcd < rem ? xcd * (q + 1) + local : rem * (q + 1) + (xcd - rem) * q + local;
}

template <typename T> struct Mma;

template <> struct Mma<float> {
    // Lane l holds 4 consecutive K values of row/column l%32; half-wave h = l/32
    // owns K offsets 4h..4h+3 of each 8-wide step, fed through four 32x32x2 MFMAs.
    static __device__ __forceinline__ void run(float16v &acc, const uint4v &a, const uint4v &b)
    {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[e]), __uint_as_float(b[e]),
                                                       acc, 0, 0, 0);
    }
};

template <> struct Mma<bf16_t> {
    static __device__ __forceinline__ void run(float16v &acc, const uint4v &a, const uint4v &b)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8v, a),
                                                      __builtin_bit_cast(bf16x8v, b), acc, 0, 0, 0);
    }
};

// FK selects a compile-time filter size (1, 3, 7) or 0 for run-time R and S.
template <typename T, int MT, int FK>
__global__ __launch_bounds__(kThreads) void conv_igemm_kernel(const IgemmArgs a)
{
    constexpr int VE = 16 / (int)sizeof(T);       // elements per 16-byte vector
    constexpr int KT = 4 * VE;                    // K elements per chunk
    constexpr int HALF = KT / 2;                  // K elements gathered per thread per chunk
    constexpr int WTM = MT / 2;                   // wave tile rows
    constexpr int MI = WTM / 32, NJ = 2;          // 32x32 MFMA tiles per wave
    constexpr int AV = MT * 4 / kThreads;         // weight vectors per thread per chunk
    constexpr int BUF = (MT + kNT) * kLdsRow;

    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * BUF];
    __shared__ float ss_lds[2 * MT];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;

    const int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int m0 = (tile % a.mtiles) * MT;
    const int n0 = (tile / a.mtiles) * kNT;
    const int split = blockIdx.y;
    const int kbeg = split * a.k_per_split;
    const int kend = min(a.K, kbeg + a.k_per_split);
    const int nchunks = (kend - kbeg + KT - 1) / KT;

    const int R = FK ? FK : a.R, S = FK ? FK : a.S, RS = R * S;
    const int HW = a.H * a.W, OHW = a.OH * a.OW;
    const T *__restrict__ xg = static_cast<const T *>(a.x);
    const T *__restrict__ wg = static_cast<const T *>(a.w);

    // ---- per-thread gather coordinates: one pixel, half of each K chunk ----------------
    const int pl = tid & (kNT - 1);
    const int kslot = __builtin_amdgcn_readfirstlane(tid >> 7);   // uniform within a wavefront
    const int pg = n0 + pl;
    const bool pvalid = pg < a.npix;
    int base = 0;
    uint32_t rowmask = 0, colmask = 0;
    if (pvalid) {
        const int n = pg / OHW, rem = pg - n * OHW;
        const int oh = rem / a.OW, ow = rem - oh * a.OW;
        const int ih0 = oh * a.sh - a.ph, iw0 = ow * a.sw - a.pw;
        base = n * a.IC * HW + ih0 * a.W + iw0;
        for (int r = 0; r < R; ++r) rowmask |= (uint32_t)(ih0 + r >= 0 && ih0 + r < a.H) << r;
        for (int s = 0; s < S; ++s) colmask |= (uint32_t)(iw0 + s >= 0 && iw0 + s < a.W) << s;
    }

    alignas(16) T breg[HALF];
    uint4v areg[AV];

    auto load_chunk = [&](int c) {
        const int kc = kbeg + c * KT;
        // weights: rows of the OIHW tensor are contiguous in K
#pragma unroll
        for (int i = 0; i < AV; ++i) {
            const int v = tid + i * kThreads;
            const int row = v >> 2, kv = v & 3;
            const int oc = m0 + row, k = kc + kv * VE;
            uint4v val = {0u, 0u, 0u, 0u};
            if (a.w_vec_ok) {
                if (oc < a.OC && k < kend)
                    val = *reinterpret_cast<const uint4v *>(wg + (size_t)oc * a.K + k);
            } else if (oc < a.OC) {
                T tmp[VE];
#pragma unroll
                for (int e = 0; e < VE; ++e) {
                    const bool ok = k + e < kend;
                    const T t = wg[(size_t)oc * a.K + (ok ? k + e : 0)];
                    tmp[e] = ok ? t : T(0);
                }
                val = __builtin_bit_cast(uint4v, tmp);
            }
            areg[i] = val;
        }
        // input: one pixel per lane, HALF consecutive K indices, out-of-image taps read as 0
        const int k0 = kc + kslot * HALF;
#pragma unroll
        for (int j = 0; j < HALF; ++j) {
            const int k = k0 + j;
            int ic, r, s;
            if (FK == 1) {
                ic = k; r = 0; s = 0;
            } else {
                ic = k / RS;
                const int rs = k - ic * RS;
                r = rs / S;
                s = rs - r * S;
            }
            const bool ok = pvalid && k < kend && ((rowmask >> r) & (colmask >> s) & 1u);
            const int idx = ok ? base + ic * HW + r * a.W + s : 0;
            const T t = xg[idx];
            breg[j] = ok ? t : T(0);
        }
    };

    auto store_chunk = [&](int buf) {
        unsigned char *A = lds + buf * BUF;
        unsigned char *B = A + MT * kLdsRow;
#pragma unroll
        for (int i = 0; i < AV; ++i) {
            const int v = tid + i * kThreads;
            *reinterpret_cast<uint4v *>(A + (v >> 2) * kLdsRow + (v & 3) * 16) = areg[i];
        }
        const uint4v *bv = reinterpret_cast<const uint4v *>(breg);
        unsigned char *dst = B + pl * kLdsRow + kslot * 32;
        *reinterpret_cast<uint4v *>(dst) = bv[0];
        *reinterpret_cast<uint4v *>(dst + 16) = bv[1];
    };

    float16v acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    if (a.splits == 1)
        stage_scale_shift(ss_lds, m0, MT, a.scale, a.shift, a.bias, a.OC, tid, kThreads);
    if (nchunks > 0) {
        load_chunk(0);
        store_chunk(0);
    }
    __syncthreads();

    const int lrow = lane & 31, lhalf = lane >> 5;
    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        if (c + 1 < nchunks) load_chunk(c + 1);

        const unsigned char *A = lds + buf * BUF;
        const unsigned char *B = A + MT * kLdsRow;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            uint4v af[MI], bf[NJ];
#pragma unroll
            for (int i = 0; i < MI; ++i)
                af[i] = *reinterpret_cast<const uint4v *>(
                    A + (wm * WTM + i * 32 + lrow) * kLdsRow + ks * 32 + lhalf * 16);
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                bf[j] = *reinterpret_cast<const uint4v *>(
                    B + (wn * 64 + j * 32 + lrow) * kLdsRow + ks * 32 + lhalf * 16);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                // pixel operand first: the accumulator tile is D[pixel][channel]
                for (int j = 0; j < NJ; ++j) Mma<T>::run(acc[i][j], bf[j], af[i]);
        }

        if (c + 1 < nchunks) store_chunk(buf ^ 1);
        __syncthreads();
    }

    // ---- fused tail on the accumulators (or raw partials when the reduction is split) -----
    if (a.splits == 1) {
        // the loop ended on a barrier: the operand buffers are free to stage the transposes
        unsigned char *stage = lds + wave * kStageBytes;
        const TailArgs tail{a.scale, a.shift, a.bias, a.residual, a.y, a.OC, OHW, a.npix, a.relu};
        store_acc_tiles<T, MI, NJ>(acc, stage, lane, m0 + wm * WTM, n0 + wn * 64, tail, a.vmode,
                                   ss_lds, wm * WTM);
        return;
    }
    // Accumulator v of lane l in a 32x32 tile: pixel 8*(v/4) + 4*(l/32) + v%4, channel l%32.
    // A group of four values is four consecutive pixels of one channel: one 16-byte store when
    // the map size is a multiple of four (a group then lies within one image); the image index
    // comes from one uniform division per tile and a step at an image end (the first version
    // divided per value and stored 4 bytes at a time: 4-8 us of a 10-17 us kernel at batch 1).
    const size_t total = (size_t)a.npix * a.OC;
    float *wsp = a.ws + (size_t)split * total;
    const bool vec = OHW % 4 == 0;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        const int oc = m0 + wm * WTM + i * 32 + lrow;
        if (oc >= a.OC) continue;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int p0t = __builtin_amdgcn_readfirstlane(n0 + wn * 64 + j * 32);
            const int nt0 = p0t / OHW, remt = p0t - nt0 * OHW;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int pl = 8 * g + 4 * lhalf;
                int n = nt0, rem = remt + pl;
                while (rem >= OHW) { rem -= OHW; ++n; }
                if (vec) {
                    if (p0t + pl < a.npix)        // npix % 4 == 0: a whole group or none
                        *reinterpret_cast<float4v *>(wsp + (size_t)(n * a.OC + oc) * OHW + rem) =
                            float4v{acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2],
                                    acc[i][j][4 * g + 3]};
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if (p0t + pl + q < a.npix) wsp[(size_t)(n * a.OC + oc) * OHW + rem] = acc[i][j][4 * g + q];
                        if (++rem >= OHW) { rem -= OHW; ++n; }
                    }
                }
            }
        }
    }
}

// Sums the split-K partials in a fixed order and applies the fused tail.
template <typename T>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const IgemmArgs a)
{
    const int OHW = a.OH * a.OW;
    const int total = a.npix * a.OC;
    const int o = blockIdx.x * 256 + threadIdx.x;
    if (o >= total) return;
    float acc = 0.0f;
    for (int s = 0; s < a.splits; ++s) acc += a.ws[(size_t)s * total + o];
    const int oc = (o / OHW) % a.OC;
    fused_tail_store<T>(acc, a.scale[oc], a.shift[oc], a.bias ? a.bias[oc] : 0.0f,
                        static_cast<const T *>(a.residual), static_cast<T *>(a.y), o, a.relu != 0);
}

template <typename T, int MT>
void launch_fk(const IgemmArgs &a, dim3 grid, hipStream_t stream)
{
    if (a.R == 1 && a.S == 1)
        hipLaunchKernelGGL((conv_igemm_kernel<T, MT, 1>), grid, dim3(kThreads), 0, stream, a);
    else if (a.R == 3 && a.S == 3)
        hipLaunchKernelGGL((conv_igemm_kernel<T, MT, 3>), grid, dim3(kThreads), 0, stream, a);
    else if (a.R == 7 && a.S == 7)
        hipLaunchKernelGGL((conv_igemm_kernel<T, MT, 7>), grid, dim3(kThreads), 0, stream, a);
    else
        hipLaunchKernelGGL((conv_igemm_kernel<T, MT, 0>), grid, dim3(kThreads), 0, stream, a);
}

template <typename T>
tvg_status launch_typed(const IgemmArgs &a, int mt, hipStream_t stream)
{
    const int ntiles = (a.npix + kNT - 1) / kNT;
    dim3 grid((unsigned)(a.mtiles * ntiles), (unsigned)a.splits);
    if (mt == 64)
        launch_fk<T, 64>(a, grid, stream);
    else
        launch_fk<T, 128>(a, grid, stream);
    if (hipGetLastError() != hipSuccess) return TVG_ERR_LAUNCH;
    if (a.splits > 1) {
        const int total = a.npix * a.OC;
        hipLaunchKernelGGL((splitk_reduce_kernel<T>), dim3((total + 255) / 256), dim3(256), 0,
                           stream, a);
        if (hipGetLastError() != hipSuccess) return TVG_ERR_LAUNCH;
    }
    return TVG_OK;
}

}  // namespace

ConvPlan plan_conv(const ConvProblem &p, bool allow_split)
{
    ConvPlan plan;
    const int kt = p.dtype == TVG_BF16 ? 32 : 16;
    const Knobs knobs = forced_knobs(p);
    plan.mt = knobs.mt == 64 || knobs.mt == 128 ? knobs.mt : p.OC <= 64 ? 64 : 128;
    plan.nt = kNT;
    const long tiles = (long)((p.OC + plan.mt - 1) / plan.mt) * ((p.npix + kNT - 1) / kNT);
    const int chunks = (p.K + kt - 1) / kt;
    int splits = 1;
    if (allow_split && tiles < kComputeUnits) {
        const int want = (int)((2 * kComputeUnits + tiles - 1) / tiles);
        splits = want < chunks / 4 ? want : chunks / 4;   // keep at least 4 chunks per partition
        if (splits > 32) splits = 32;
        if (splits < 1) splits = 1;
    }
    if (allow_split && knobs.split_k > 0)              // fixed by the caller, at most one per chunk
        splits = knobs.split_k < chunks ? (knobs.split_k > 32 ? 32 : knobs.split_k) : chunks;
    int per = (chunks + splits - 1) / splits;
    plan.k_per_split = per * kt;
    plan.splits = (p.K + plan.k_per_split - 1) / plan.k_per_split;
    plan.workspace_bytes =
        plan.splits > 1 ? (size_t)plan.splits * (size_t)p.npix * (size_t)p.OC * sizeof(float) : 0;
    return plan;
}

tvg_status launch_splitk_reduce(const ConvProblem &p, int splits, const ConvPointers &ptr,
                                hipStream_t stream)
{
    IgemmArgs a{};
    a.scale = ptr.scale; a.shift = ptr.shift; a.bias = ptr.bias;
    a.residual = ptr.residual; a.y = ptr.y; a.ws = ptr.workspace;
    a.OC = p.OC; a.OH = p.OH; a.OW = p.OW; a.npix = p.npix; a.relu = p.relu;
    a.splits = splits;
    const int total = p.npix * p.OC;
    if (p.dtype == TVG_BF16)
        hipLaunchKernelGGL((splitk_reduce_kernel<bf16_t>), dim3((total + 255) / 256), dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((splitk_reduce_kernel<float>), dim3((total + 255) / 256), dim3(256), 0, stream, a);
    return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
}

tvg_status launch_conv_igemm(const ConvProblem &p, const ConvPlan &plan, const ConvPointers &ptr,
                             hipStream_t stream)
{
    IgemmArgs a;
    a.x = ptr.x; a.w = ptr.w; a.scale = ptr.scale; a.shift = ptr.shift; a.bias = ptr.bias;
    a.residual = ptr.residual; a.y = ptr.y; a.ws = ptr.workspace;
    a.N = p.N; a.IC = p.IC; a.H = p.H; a.W = p.W; a.OC = p.OC; a.R = p.R; a.S = p.S;
    a.sh = p.sh; a.sw = p.sw; a.ph = p.ph; a.pw = p.pw; a.OH = p.OH; a.OW = p.OW;
    a.K = p.K; a.npix = p.npix; a.relu = p.relu;
    a.mtiles = (p.OC + plan.mt - 1) / plan.mt;
    a.splits = plan.splits;
    a.k_per_split = plan.k_per_split;
    const int ve = p.dtype == TVG_BF16 ? 8 : 4;
    a.w_vec_ok = (p.K % ve == 0) && (reinterpret_cast<uintptr_t>(ptr.w) % 16 == 0);
    a.vmode = pick_store_vmode(p.dtype, p.OH * p.OW, ptr.y, ptr.residual);
    return p.dtype == TVG_BF16 ? launch_typed<bf16_t>(a, plan.mt, stream)
                               : launch_typed<float>(a, plan.mt, stream);
}

}  // namespace tvg
