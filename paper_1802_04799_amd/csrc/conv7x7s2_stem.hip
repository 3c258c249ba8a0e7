// bf16 stride-2 fused conv2d for very few input channels - 7x7 pad 3 (the ResNet stem, Table 2's
// C1: 3 -> 64 channels on 224x224) and 3x3 pad 1 (the MobileNet stem, 3 -> 32) - on MFMA.  The
// text below describes the 7x7 case; R is a template parameter, and a 3x3 filter row sits in
// slots 3..5 of the same 8-slot window (the window of pixel (oh, ow) covers input columns
// 2*ow - 4 .. 2*ow + 3 whatever R is).
//
// With IC = 3 the reduction (147) is too short and too ragged for the channel-
// chunked kernels, and at batch 64 the layer is bound by writing its output
// (103 MB against 19 MB of input), so this kernel is built around three ideas:
//
//  * Reduction order (ic, r, s') with the filter row padded to 8 taps on the LEFT
//    (s' = 0 is a zero weight, s' = 1..7 are the real taps).  One MFMA lane then
//    consumes 8 horizontally adjacent input values of one (ic, r) pair, which are
//    contiguous in the NCHW input: the input patch is staged in LDS in its
//    natural layout with plain 16-byte copies, no transposition, and the operand
//    of pixel (oh, ow) for pair (ic, r) starts at column 2*ow of the staged row
//    (the staged row begins 4 columns left of the image).  K per MFMA = 2 pairs,
//    ceil(7*IC/2) MFMAs cover the whole reduction: there is no K loop.
//  * The weights (OC tile x 7*IC pairs x 8) are staged once per workgroup and
//    re-used for every pixel tile the workgroup walks over (persistent
//    workgroups), so the per-tile work is: copy a few input rows, 11 x 4 MFMAs
//    per wave, store 64 x 256 outputs.
//  * Rows that fall outside the image are fetched through a buffer descriptor at
//    an out-of-range offset, which returns zeros: no branches in the copy.
//
// The next tile's rows are requested before the current tile's MFMAs and are
// written to the other LDS buffer afterwards (one barrier per tile).
#include <numeric>
#include "tvg_device.h"
#include "tvg_internal.h"

namespace tvg {

namespace {

struct StemArgs {
    const bf16_t *x, *w;
    const float *scale, *shift, *bias;
    const bf16_t *residual;
    bf16_t *y;
    int N, IC, H, W, OC, OH, OW, npix, relu, vmode;
    int nrows;          // staged virtual rows per tile (maximum over tiles)
    int ntiles, mtiles, wg_per_mtile;
    uint32_t x_bytes, w_bytes;
};

constexpr int kNT = 256;                 // pixels per tile
// (output channels per tile: MT = 64, or 32 for layers of at most 32 channels - the MobileNet
// stem - which would otherwise run half of their MFMAs and half of the tail on rows nobody stores)
constexpr int kRsrcFlags = 0x00020000;   // raw buffer descriptor word 3 on gfx9-family targets
constexpr uint32_t kOutOfRange = 0xFFFFFFF0u;

// IC = input channels (compile time, so the reduction loop unrolls completely and the LDS
// reads of one MFMA step overlap the previous step's MFMAs); LT = 16-byte copy tasks per
// thread per tile.
template <int R, int IC, int LT, int MT>
__global__ __launch_bounds__(256, 2) void conv_stem_s2_kernel(const StemArgs a)
{
    constexpr int kMT = MT, MI = MT / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int PAD = R / 2;
    constexpr int npairs = IC * R;
    constexpr int NM = (npairs + 1) / 2;                 // MFMAs over the reduction
    const int H = a.H, W = a.W, OHW = a.OH * a.OW;
    const int VH = H + 2 * PAD;                          // virtual rows per image (pad + H + pad)
    const int pitch = (W + 8) * 2;                       // bytes per staged row
    const int nrows = a.nrows;
    const int a_bytes = 2 * NM * kMT * 16;
    const int patch_bytes = IC * nrows * pitch;
    unsigned char *As = smem;                            // [pair][oc][8 taps]
    unsigned char *Ps = smem + a_bytes;                  // 2 x [ic][row][W + 8]
    // per wave: staging for two accumulator tiles at a time
    unsigned char *stage = smem + a_bytes + 2 * patch_bytes + (threadIdx.x >> 6) * 2 * kStageBytes;
    float *ss_lds = reinterpret_cast<float *>(smem + a_bytes + 2 * patch_bytes) + 8 * kStageFloats;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int mtile = blockIdx.x % a.mtiles, wg = blockIdx.x / a.mtiles;
    const int m0 = mtile * kMT;

    stage_scale_shift(ss_lds, m0, kMT, a.scale, a.shift, a.bias, a.OC, tid, 256);

    // ---- zero both patch buffers (their padding columns stay zero) and the weight area ----
    for (int i = tid; i < 2 * patch_bytes / 16; i += 256)
        reinterpret_cast<uint4v *>(Ps)[i] = uint4v{0u, 0u, 0u, 0u};
    for (int i = tid; i < a_bytes / 16; i += 256)
        reinterpret_cast<uint4v *>(As)[i] = uint4v{0u, 0u, 0u, 0u};
    // ---- stage the weights: the tile's channels are one contiguous run of [oc][ic][r][s], read
    // as 16-byte vectors that are all in flight together, then scattered element by element
    // into [pair = (ic, r)][oc][slot = s + 1] (slot 0, the odd pair and absent channels stay 0)
    {
        constexpr int KW = IC * R * R;                   // weights per output channel
        constexpr int WV = (kMT * KW + 7) / 8;           // vectors per full tile
        constexpr int WT = (WV + 255) / 256;             // vectors per thread
        const int count = min(kMT, a.OC - m0) * KW;
        const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<bf16_t *>(a.w), 0, a.w_bytes, kRsrcFlags);
        const uint32_t wbase = (uint32_t)m0 * KW * 2u;
        uint4v wv[WT];
#pragma unroll
        for (int j = 0; j < WT; ++j) {
            const int v = tid + j * 256;
            const uint32_t voff = v * 8 < count ? wbase + (uint32_t)v * 16u : kOutOfRange;
            wv[j] = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, voff, 0, 0));
        }
        __syncthreads();                                 // the zeros are in place
#pragma unroll
        for (int j = 0; j < WT; ++j) {
            const int f0 = (tid + j * 256) * 8;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int f = f0 + k;
                const int ocl = f / KW, rem = f - ocl * KW;
                const int pair = rem / R, sp = rem - pair * R + (4 - PAD);
                const bf16_t v = (bf16_t)(k & 1 ? wv[j][k >> 1] >> 16 : wv[j][k >> 1] & 0xffffu);
                if (f < count) reinterpret_cast<bf16_t *>(As)[(pair * kMT + ocl) * 8 + sp] = v;
            }
        }
    }

    // ---- per-thread copy tasks: (ic, row slot, 16-byte column group), fixed for all tiles --
    const int VPR = W / 8;
    const int ntasks = IC * nrows * VPR;
    uint32_t cgoff[LT];
    int rslot[LT], ldst[LT];
#pragma unroll
    for (int j = 0; j < LT; ++j) {
        const int t = tid + j * 256;
        const int pr = t / VPR, v = t - pr * VPR;
        const int ic = pr / nrows, rs = pr - ic * nrows;
        cgoff[j] = (uint32_t)(ic * H * W * 2 + v * 16);
        rslot[j] = t < ntasks ? rs : -1;
        ldst[j] = (ic * nrows + rs) * pitch + 8 + v * 16;
    }

    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(a.x), 0, a.x_bytes, kRsrcFlags);
    const TailArgs tail{a.scale, a.shift, a.bias, a.residual, a.y, a.OC, OHW, a.npix, a.relu};

    uint4v lreg[LT];
    // index arithmetic through the float reciprocal (exact below 2^22, checked on the host)
    const float inv_ohw = 1.0f / (float)OHW, inv_ow = 1.0f / (float)a.OW, inv_vh = 1.0f / (float)VH;
    auto first_vrow = [&](int tile) {
        int rem, ow;
        const int n = fast_div(tile * kNT, OHW, inv_ohw, &rem);
        const int oh = fast_div(rem, a.OW, inv_ow, &ow);
        return n * VH + oh * 2;
    };
    auto load_tile = [&](int tile) {
        const int vr_lo = first_vrow(tile);
        int vi_lo;
        const int n_lo = fast_div(vr_lo, VH, inv_vh, &vi_lo);
#pragma unroll
        for (int j = 0; j < LT; ++j) {
            int vi = vi_lo + rslot[j], n = n_lo;
            if (vi >= VH) { vi -= VH; n += 1; }
            const int ih = vi - PAD;
            const bool ok = rslot[j] >= 0 && ih >= 0 && ih < H && n < a.N;
            const uint32_t voff = ok ? cgoff[j] + (uint32_t)((n * IC * H + ih) * W) * 2u : kOutOfRange;
            lreg[j] = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, voff, 0, 0));
        }
    };
    auto store_tile_rows = [&](int buf) {
        unsigned char *P = Ps + buf * patch_bytes;
#pragma unroll
        for (int j = 0; j < LT; ++j)
            if (rslot[j] >= 0) {
                typedef uint32_t u2 __attribute__((ext_vector_type(2)));
                *reinterpret_cast<u2 *>(P + ldst[j]) = u2{lreg[j][0], lreg[j][1]};
                *reinterpret_cast<u2 *>(P + ldst[j] + 8) = u2{lreg[j][2], lreg[j][3]};
            }
    };

    int tile = wg;
    if (tile < a.ntiles) load_tile(tile);
    __syncthreads();
    if (tile < a.ntiles) store_tile_rows(0);
    __syncthreads();

    for (int it = 0; tile < a.ntiles; tile += a.wg_per_mtile, ++it) {
        const int next = tile + a.wg_per_mtile;
        if (next < a.ntiles) load_tile(next);

        const unsigned char *P = Ps + (it & 1) * patch_bytes;
        const int p0 = tile * kNT;
        const int vr_lo = first_vrow(tile);
        int pb[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int p = p0 + wave * 64 + j * 32 + lrow;
            pb[j] = 0;
            if (p < a.npix) {
                int rem, ow;
                const int n = fast_div(p, OHW, inv_ohw, &rem);
                const int oh = fast_div(rem, a.OW, inv_ow, &ow);
                pb[j] = (n * VH + oh * 2 - vr_lo) * pitch + ow * 4;
            }
        }
        float16v acc[MI][2];
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

#pragma unroll
        for (int m = 0; m < NM; ++m) {
            // the two half-waves hold pairs 2m and 2m+1; both offsets are uniform values
            const int pa = 2 * m, pq = 2 * m + 1 < npairs ? 2 * m + 1 : 0;
            const int offa = ((pa / R) * nrows + pa % R) * pitch;
            const int offq = ((pq / R) * nrows + pq % R) * pitch;
            const int poff = lhalf ? offq : offa;
            uint4v af[MI], bf[2];
#pragma unroll
            for (int i = 0; i < MI; ++i)
                af[i] = *reinterpret_cast<const uint4v *>(As + ((2 * m + lhalf) * kMT + i * 32 + lrow) * 16);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const uint32_t *src = reinterpret_cast<const uint32_t *>(P + pb[j] + poff);
                bf[j] = uint4v{src[0], src[1], src[2], src[3]};
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    // pixel operand first: the accumulator tile is D[pixel][channel]
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8v, bf[j]), __builtin_bit_cast(bf16x8v, af[i]),
                        acc[i][j], 0, 0, 0);
        }

        // The next tile's rows have arrived during the MFMAs: put them into the other buffer
        // now, so that waiting for those loads does not also wait for this tile's stores.
        if (next < a.ntiles) store_tile_rows((it + 1) & 1);

        store_acc_tiles_batched<MI, 2, 2>(acc, stage, lane, m0, p0 + wave * 64, tail, a.vmode, ss_lds, 0);
        __syncthreads();
    }
}

int max_stem_rows(const ConvProblem &p)
{
    const int OHW = p.OH * p.OW, VH = p.H + 2 * p.ph;
    int best = 0;
    // the row count of a tile depends only on where in an image it starts, which repeats after
    // OHW / gcd(OHW, kNT) tiles: one period covers every case (this runs on every call)
    const long period = (long)kNT * (OHW / std::gcd(OHW, kNT));
    for (long p0 = 0; p0 < p.npix && p0 < period; p0 += kNT) {
        const long last = (p0 + kNT < p.npix ? p0 + kNT : p.npix) - 1;
        const int na = (int)(p0 / OHW), oha = (int)((p0 - (long)na * OHW) / p.OW);
        const int nb = (int)(last / OHW), ohb = (int)((last - (long)nb * OHW) / p.OW);
        const int rows = nb * VH + ohb * 2 + (p.R - 1) - (na * VH + oha * 2) + 1;
        if (rows > best) best = rows;
    }
    return best;
}

template <int R, int IC, int LT, int MT = 64>
tvg_status launch_lt(const StemArgs &a, unsigned grid, size_t lds, hipStream_t stream)
{
    auto kernel = conv_stem_s2_kernel<R, IC, LT, MT>;
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return TVG_ERR_LAUNCH;
        configured = true;
    }
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), lds, stream, a);
    return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
}

}  // namespace

bool plan_conv7x7s2_stem(const ConvProblem &p, StemPlan *plan)
{
    if (p.dtype != TVG_BF16 || (p.R != 7 && p.R != 3) || p.S != p.R || p.sh != 2 || p.sw != 2 ||
        p.ph != p.R / 2 || p.pw != p.R / 2)
        return false;
    if (p.IC > 4 || p.W % 8 != 0) return false;
    if (p.npix >= (1 << 22) || (long)p.N * (p.H + 2 * p.ph) >= (1 << 22)) return false;   // fast_div range
    if ((size_t)p.N * p.IC * p.H * p.W * 2 > (size_t)kOutOfRange) return false;
    const int rows = max_stem_rows(p);
    if (rows > p.H + 2 * p.ph) return false;            // a tile may wrap into the next image once
    const int nm = (p.IC * p.R + 1) / 2;
    // (the narrow channel tile exists for the case that needs it, the 3x3 three-channel stem)
    const int mt = (p.OC <= 32 && p.R == 3 && p.IC == 3) ? 32 : 64;
    const size_t lds = (size_t)2 * nm * mt * 16 + (size_t)2 * p.IC * rows * (p.W + 8) * 2 +
                       (size_t)8 * kStageBytes + (size_t)mt * 8;
    const int lt = (p.IC * rows * (p.W / 8) + 255) / 256;
    if (lds > 80 * 1024 || lt > 8) return false;
    plan->rows = rows;
    plan->mt = mt;
    plan->lt = lt;
    plan->lds_bytes = lds;
    return true;
}

bool conv7x7s2_stem_pointers_ok(const ConvPointers &ptr)
{
    // input rows and the weights are read as 16-byte vectors
    return reinterpret_cast<uintptr_t>(ptr.x) % 16 == 0 && reinterpret_cast<uintptr_t>(ptr.w) % 16 == 0;
}

tvg_status launch_conv7x7s2_stem(const ConvProblem &p, const StemPlan &plan, const ConvPointers &ptr,
                                 hipStream_t stream)
{
    StemArgs a;
    a.x = static_cast<const bf16_t *>(ptr.x); a.w = static_cast<const bf16_t *>(ptr.w);
    a.scale = ptr.scale; a.shift = ptr.shift; a.bias = ptr.bias;
    a.residual = static_cast<const bf16_t *>(ptr.residual); a.y = static_cast<bf16_t *>(ptr.y);
    a.N = p.N; a.IC = p.IC; a.H = p.H; a.W = p.W; a.OC = p.OC; a.OH = p.OH; a.OW = p.OW;
    a.npix = p.npix; a.relu = p.relu | (p.stream_out << 1);
    a.vmode = pick_store_vmode(p.dtype, p.OH * p.OW, ptr.y, ptr.residual);
    a.nrows = plan.rows;
    a.ntiles = (p.npix + kNT - 1) / kNT;
    a.mtiles = (p.OC + plan.mt - 1) / plan.mt;
    // persistent workgroups: two per CU, shared between the output-channel tiles
    int per = 2 * kComputeUnits / a.mtiles;
    if (per < 1) per = 1;
    if (per > a.ntiles) per = a.ntiles;
    a.wg_per_mtile = per;
    a.x_bytes = (uint32_t)((size_t)p.N * p.IC * p.H * p.W * 2);
    // Buffer loads are range-checked per 4-byte word: an odd number of weights (odd OC x IC)
    // would leave the last one unreadable, so the size is rounded up to whole words (the two
    // bytes past the tensor lie in the same aligned word as its last element).
    a.w_bytes = ((uint32_t)((size_t)p.OC * p.IC * p.R * p.R * 2) + 3u) & ~3u;
    const unsigned grid = (unsigned)(per * a.mtiles);
    if (p.R == 3) {
        if (plan.mt == 32)
            return plan.lt <= 5 ? launch_lt<3, 3, 5, 32>(a, grid, plan.lds_bytes, stream)
                                : launch_lt<3, 3, 8, 32>(a, grid, plan.lds_bytes, stream);
        if (p.IC == 3 && plan.lt <= 5) return launch_lt<3, 3, 5>(a, grid, plan.lds_bytes, stream);
        switch (p.IC) {
        case 1: return launch_lt<3, 1, 8>(a, grid, plan.lds_bytes, stream);
        case 2: return launch_lt<3, 2, 8>(a, grid, plan.lds_bytes, stream);
        case 3: return launch_lt<3, 3, 8>(a, grid, plan.lds_bytes, stream);
        default: return launch_lt<3, 4, 8>(a, grid, plan.lds_bytes, stream);
        }
    }
    if (p.IC == 3 && plan.lt <= 5) return launch_lt<7, 3, 5>(a, grid, plan.lds_bytes, stream);
    switch (p.IC) {
    case 1: return launch_lt<7, 1, 8>(a, grid, plan.lds_bytes, stream);
    case 2: return launch_lt<7, 2, 8>(a, grid, plan.lds_bytes, stream);
    case 3: return launch_lt<7, 3, 8>(a, grid, plan.lds_bytes, stream);
    default: return launch_lt<7, 4, 8>(a, grid, plan.lds_bytes, stream);
    }
}

}  // namespace tvg
