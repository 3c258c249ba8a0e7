// bf16 MobileNet block in one kernel: y = tail_pw(w_pw * bf16(tail_dw(depthwise3x3(x)))).
//
// Operator fusion (TVM paper, Section 3) carried across the two operators of the block: the
// depthwise result (Table 2, rows D) is never written to memory.  The kernel is the 1x1 GEMM
// kernel (rows = output channels, columns = 64 consecutive output pixels, K chunks of 32
// channels, 32x32x16 MFMAs from LDS) with a different producer for its pixel operand:
//   * per K chunk the workgroup copies, for each of the 32 channels, the input rows that its
//     pixel tile touches (its rows plus one above and below; a tile may span up to three
//     images, each giving one contiguous run per channel) into LDS with 4-byte loads,
//     widened to fp32 on the way in, together with the chunk's depthwise parameters;
//   * thread (pixel, channel octet) then sums the nine taps of its 8 channels from LDS with
//     tap cells it computed once (padding taps point at a zero cell), applies the depthwise
//     tail, rounds to bf16 and writes the 16-byte operand word the MFMAs read.
// The next chunk's rows and weights are in flight while the current chunk is summed and
// multiplied (Section 4.4, latency hiding).  Stride 1, channels a multiple of 32.
#include <stdlib.h>
#include <numeric>
#include "tvg_device.h"
#include "tvg_internal.h"

namespace tvg {

namespace {

struct DwPwArgs {
    const bf16_t *x, *w_dw;
    const float *scale_dw, *shift_dw;
    const bf16_t *w_pw;
    const float *scale, *shift, *bias;
    const bf16_t *residual;
    bf16_t *y;
    int N, C, H, W, OC, npix, relu, relu_dw, mtiles, vmode;
    uint32_t x_bytes, w_bytes;
};

constexpr int kRow = 80;                 // bytes per operand row in LDS: 32 channels + padding
constexpr int kKC = 32;                  // channels per K chunk
constexpr int kNT = 64;                  // pixels per workgroup
constexpr int kRsrcFlags = 0x00020000;   // raw buffer descriptor word 3 on gfx9-family targets
constexpr uint32_t kOutOfRange = 0xFFFFFFF0u;
constexpr int kSets = 4;                 // register sets of loads: kSets - 1 chunks in flight
constexpr int kGroup = 2;                // channels whose taps are fetched from LDS together
constexpr int kSegs = 3;                 // images a 64-pixel tile can span (maps of >= 32 pixels)

__device__ __forceinline__ int xcd_remap(int bid, int nb)
{
    const int q = nb >> 3, rem = nb & 7;
    const int xcd = bid & 7, local = bid >> 3;
    return xcd < rem ? xcd * (q + 1) + local : rem * (q + 1) + (xcd - rem) * q + local;
}

// The input rows of one image that a run of output pixels [lo, hi) of that image touches.
struct Seg {
    int estart;      // first element (ih_lo * W)
    int len;         // elements
    int ndw;         // 4-byte words reserved for the run in an LDS channel row (0 = empty)
};

__host__ __device__ inline Seg make_seg(int lo, int hi, int H, int W)
{
    Seg s{0, 0, 0};
    if (hi <= lo) return s;
    const int oh_lo = lo / W, oh_hi = (hi - 1) / W;
    const int ih_lo = oh_lo > 0 ? oh_lo - 1 : 0;
    const int ih_hi = oh_hi + 1 < H ? oh_hi + 1 : H - 1;
    s.estart = ih_lo * W;
    // the run starts on an even or odd element: one spare word covers either phase
    s.len = (ih_hi - ih_lo + 1) * W;
    s.ndw = s.len / 2 + 1;
    return s;
}

template <int MT, int LT>
__global__ __launch_bounds__(256, MT <= 128 ? 2 : 1) void dwpw_kernel(const DwPwArgs a)
{
    constexpr int MI = MT / 64;                    // 32x32 tiles per wave along channels
    constexpr int AT = MT * 4 / 256;               // weight vectors per thread
    // A channel row of the patch, in fp32 cells: per run one leading cell, its elements and up
    // to two cells of slack (a run is fetched as whole 4-byte words from an even element), then
    // two dump cells for idle loader slots and the zero cell that padding taps read.
    constexpr int CELLS = 16 * LT + 10;
    constexpr int kDump = 16 * LT + 6, kZero = 16 * LT + 9;
    constexpr int kPrm = 208;                      // parameter words per chunk as loaded: 144 of
                                                   // taps (32 x 9 bf16), 32 scales, 32 shifts
    constexpr int OPER = (MT + kNT) * kRow + kKC * CELLS * 4 + kKC * 12 * 4;
    constexpr int STAGE = 4 * MI * kStageBytes;
    __shared__ __attribute__((aligned(16))) unsigned char lds[OPER > STAGE ? OPER : STAGE];
    __shared__ float ss_lds[2 * MT];
    unsigned char *As = lds, *Bs = lds + MT * kRow;
    float *Pr = reinterpret_cast<float *>(lds + (MT + kNT) * kRow);      // [32][12]: taps, scale, shift
    float *Ps = Pr + kKC * 12;                                            // [32][CELLS]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int m0 = (tile % a.mtiles) * MT;        // consecutive tiles share the pixel tile
    const int n0 = (tile / a.mtiles) * kNT;
    const int H = a.H, W = a.W, HW = H * W;

    stage_scale_shift(ss_lds, m0, MT, a.scale, a.shift, a.bias, a.OC, tid, 256);

    // ---- the runs of input rows this tile needs (uniform over the workgroup) ----------------
    const int nA = n0 / HW;
    const int pend = min(n0 + kNT, a.npix);
    Seg seg[kSegs];
    int dstart[kSegs + 1], cbase[kSegs];
    dstart[0] = 0;
#pragma unroll
    for (int s = 0; s < kSegs; ++s) {
        const int base = (nA + s) * HW;
        seg[s] = make_seg(max(n0, base) - base, min(pend, base + HW) - base, H, W);
        dstart[s + 1] = dstart[s] + seg[s].ndw;
        cbase[s] = 2 * dstart[s] + 2 * s;          // every run owns 2 * ndw + 2 cells
    }

    // ---- loader: wave w fetches the rows of channels 8w .. 8w + 7 of the chunk, one channel
    // per instruction, lanes along the row (256 contiguous bytes per load).  Word d of a row
    // maps to the same run and offset for every channel, up to the parity of the run's first
    // element when the map has an odd number of pixels: one offset pair per pass. -----------
    constexpr int WPASS = (LT * 8 + 63) / 64;      // passes of 64 words over a row
    uint32_t goff[WPASS][2];       // [pass][channel parity]: byte offset within the image stack
    int cl[WPASS][2];              // cell of the word's low half; the high half goes to the next
#pragma unroll
    for (int ps = 0; ps < WPASS; ++ps) {
        const int d = lane + 64 * ps;
        const int s = (d >= dstart[1] ? 1 : 0) + (d >= dstart[2] ? 1 : 0);
        const int es = s == 0 ? seg[0].estart : s == 1 ? seg[1].estart : seg[2].estart;
        const int ds = s == 0 ? dstart[0] : s == 1 ? dstart[1] : dstart[2];
        const int cb = s == 0 ? cbase[0] : s == 1 ? cbase[1] : cbase[2];
        const int len = s == 0 ? seg[0].len : s == 1 ? seg[1].len : seg[2].len;
#pragma unroll
        for (int par = 0; par < 2; ++par) {
            // first element of the run, less the channel's own term (which is scalar); the
            // chunk's first channel and 8 wave are even, so the parity is that of the slot
            const int g = (nA + s) * a.C * HW + es;
            const int ph = (g + par * HW) & 1;
            // only words that hold an element of the run: none of them passes the tensor's end
            const bool live = d < dstart[kSegs] && d - ds < (len + 1 + ph) / 2;
            // (the scalar channel term is rounded down to a whole word below: an odd channel of
            // an odd-sized map gives its two bytes back here, so both parts stay word-aligned)
            goff[ps][par] = live ? (uint32_t)(2 * (g - ph) + 4 * (d - ds) + 2 * (par & HW & 1))
                                 : kOutOfRange;
            cl[ps][par] = wave * 8 * CELLS + (live ? cb + 1 + 2 * (d - ds) - ph : kDump);
        }
    }
    // One word of the chunk's depthwise parameters per thread (threads 208.. have none).  They
    // travel with the patch, so the depthwise stage never waits on memory, and are widened to
    // fp32 on the way into LDS.
    const bool ptap = tid < 144;
    const uint32_t *pptr = ptap ? reinterpret_cast<const uint32_t *>(a.w_dw) + tid
                         : tid < 176 ? reinterpret_cast<const uint32_t *>(a.scale_dw) + (tid - 144)
                                     : reinterpret_cast<const uint32_t *>(a.shift_dw) + (tid - 176);
    const int pstep = ptap ? 144 : 32;             // words per chunk
    const int pd0 = ptap ? (2 * tid) / 9 * 12 + (2 * tid) % 9
                         : tid < 176 ? (tid - 144) * 12 + 9 : (tid - 176) * 12 + 10;
    const int pd1 = (2 * tid + 1) / 9 * 12 + (2 * tid + 1) % 9;

    // ---- this thread's pixel: the cells of its nine taps, fixed for the kernel --------------
    int tb[9];
    {
        const int p = n0 + lane;
        const int n = p / HW, rem = p - n * HW;
        const int oh = rem / W, ow = rem - oh * W;
        const int s = n - nA;
        const int es = s == 0 ? seg[0].estart : s == 1 ? seg[1].estart : seg[2].estart;
        const int cb = s == 0 ? cbase[0] : s == 1 ? cbase[1] : cbase[2];
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int q = 0; q < 3; ++q) {
                const int ih = oh - 1 + r, iw = ow - 1 + q;
                const bool ok = p < pend && s < kSegs && ih >= 0 && ih < H && iw >= 0 && iw < W;
                tb[r * 3 + q] = wave * 8 * CELLS + (ok ? cb + 1 + ih * W + iw - es : kZero);
            }
    }

    uint32_t aoff[AT];
    int adst[AT];
#pragma unroll
    for (int i = 0; i < AT; ++i) {
        const int v = tid + i * 256;
        const int row = v >> 2, kv = v & 3;
        adst[i] = row * kRow + kv * 16;
        // rows past OC read row 0; their accumulators are never stored
        aoff[i] = 2u * (uint32_t)((m0 + row < a.OC ? m0 + row : 0) * a.C + kv * 8);
    }

    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(a.x), 0, a.x_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(a.w_pw), 0, a.w_bytes, kRsrcFlags);

    // The loads run kSets - 1 chunks ahead of their use, each chunk into registers of its own.
    uint32_t raw[kSets][WPASS][8], praw[kSets];
    uint4v areg[kSets][AT];
    auto load_chunk = [&](int c, int set) __attribute__((always_inline)) {
        // (made scalar by hand: seen as per-lane values, the chunk offsets turn every load into
        // a loop over lanes)
        const int c0 = __builtin_amdgcn_readfirstlane(c * kKC);
        const int xoff = __builtin_amdgcn_readfirstlane(c0 * HW * 2);
        praw[set] = tid < kPrm ? pptr[c * pstep] : 0u;
#pragma unroll
        for (int ps = 0; ps < WPASS; ++ps)
#pragma unroll
            for (int k = 0; k < 8; ++k)        // channel c0 + 8 wave + k: its term is scalar
                raw[set][ps][k] = __builtin_amdgcn_raw_buffer_load_b32(
                    xrsrc, goff[ps][k & 1], xoff + (((wave * 8 + k) * HW * 2) & ~3), 0);
#pragma unroll
        for (int i = 0; i < AT; ++i)
            areg[set][i] = __builtin_bit_cast(
                uint4v, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, aoff[i], c0 * 2, 0));
    };
    auto store_patch = [&](int set) __attribute__((always_inline)) {
#pragma unroll
        for (int ps = 0; ps < WPASS; ++ps)
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                Ps[cl[ps][k & 1] + k * CELLS] = __uint_as_float(raw[set][ps][k] << 16);
                Ps[cl[ps][k & 1] + k * CELLS + 1] = __uint_as_float(raw[set][ps][k] & 0xFFFF0000u);
            }
        if (tid < kPrm) {
            Pr[pd0] = __uint_as_float(ptap ? praw[set] << 16 : praw[set]);
            if (ptap) Pr[pd1] = __uint_as_float(praw[set] & 0xFFFF0000u);
        }
    };
    auto store_weights = [&](int set) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < AT; ++i) *reinterpret_cast<uint4v *>(As + adst[i]) = areg[set][i];
    };

    float16v acc[MI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;

    if (tid < kKC) Ps[tid * CELLS + kZero] = 0.0f;

    const int nchunks = a.C / kKC;
#pragma unroll
    for (int u = 0; u < kSets - 1; ++u)
        if (u < nchunks) load_chunk(u, u);
    store_patch(0);
    store_weights(0);
    __syncthreads();

    const float floor_dw = a.relu_dw ? 0.0f : -INFINITY;
    // One chunk: `steady` = inside the main loop, where every load and store below happens
    // (no conditions: the compiler then knows how many loads are in flight at each wait; with
    // conditional loads it waits for all of them, i.e. for the newest, and the look-ahead is
    // lost).  Chunk c lives in register set u = c % kSets.
    auto chunk_step = [&](int c, int u, bool steady) __attribute__((always_inline)) {
        if (steady || c + kSets - 1 < nchunks) load_chunk(c + kSets - 1, (u + kSets - 1) % kSets);

        // ---- depthwise stage for (pixel = lane, channels 32 c + 8 wave .. + 7) ----------------
        // kGroup channels at a time: their parameters (the same words for every lane) and all
        // their taps are requested before the first is used, so the LDS latency is paid once per
        // group and not once per tap (the scheduler is fenced: it would otherwise pair each
        // read with its multiply-add).
        uint32_t packed[4];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int grp = 0; grp < 8 / kGroup; ++grp) {
            float4v prm[kGroup][3];
            float px[kGroup][9];
#pragma unroll
            for (int qq = 0; qq < kGroup; ++qq) {
                const int q = grp * kGroup + qq;
#pragma unroll
                for (int v = 0; v < 3; ++v)
                    prm[qq][v] = *reinterpret_cast<const float4v *>(Pr + (wave * 8 + q) * 12 + v * 4);
#pragma unroll
                for (int e = 0; e < 9; ++e) px[qq][e] = Ps[tb[e] + q * CELLS];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int qq = 0; qq < kGroup; ++qq) {
                const int q = grp * kGroup + qq;
                float sum = 0.0f;
#pragma unroll
                for (int e = 0; e < 9; ++e) sum = fmaf(px[qq][e], prm[qq][e >> 2][e & 3], sum);
                const float t = fmaxf(fmaf(sum, prm[qq][2][1], prm[qq][2][2]), floor_dw);
                if (q & 1) packed[q >> 1] = f32x2_to_bf16x2(__uint_as_float(packed[q >> 1]), t);
                else packed[q >> 1] = __float_as_uint(t);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        *reinterpret_cast<uint4v *>(Bs + lane * kRow + wave * 16) =
            uint4v{packed[0], packed[1], packed[2], packed[3]};
        __syncthreads();          // the operand is complete; the patch rows are free

        // ---- 1x1 stage ------------------------------------------------------------------------
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            uint4v af[MI];
#pragma unroll
            for (int i = 0; i < MI; ++i)
                af[i] = *reinterpret_cast<const uint4v *>(
                    As + (wm * (MT / 2) + i * 32 + lrow) * kRow + ks * 32 + lhalf * 16);
            const uint4v bf = *reinterpret_cast<const uint4v *>(
                Bs + (wn * 32 + lrow) * kRow + ks * 32 + lhalf * 16);
#pragma unroll
            for (int i = 0; i < MI; ++i)
                // pixel operand first: the accumulator tile is D[pixel][channel]
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8v, bf), __builtin_bit_cast(bf16x8v, af[i]), acc[i], 0, 0, 0);
        }
        if (steady || c + 1 < nchunks) store_patch((u + 1) % kSets);
        __syncthreads();          // every wave has read the weights (and the operand) of chunk c
        if (steady || c + 1 < nchunks) store_weights((u + 1) % kSets);
    };
    int cb0 = 0;
    for (; cb0 + 2 * kSets - 1 <= nchunks; cb0 += kSets) {
#pragma unroll
        for (int u = 0; u < kSets; ++u) chunk_step(cb0 + u, u, true);
    }
    for (; cb0 < nchunks; cb0 += kSets) {
#pragma unroll
        for (int u = 0; u < kSets; ++u)
            if (cb0 + u < nchunks) chunk_step(cb0 + u, u, false);
    }

    float16v acc2[MI][1];
#pragma unroll
    for (int i = 0; i < MI; ++i) acc2[i][0] = acc[i];
    unsigned char *stage = lds + wave * (MI * kStageBytes);
    const TailArgs tail{a.scale, a.shift, a.bias, a.residual, a.y, a.OC, HW, a.npix, a.relu};
    store_acc_tiles_batched<MI, 1>(acc2, stage, lane, m0 + wm * (MT / 2), n0 + wn * 32, tail, a.vmode,
                                   ss_lds, wm * (MT / 2));
}

// Largest number of patch words a channel row needs over all tiles of the problem (tile
// starts repeat with period HW / gcd(HW, 64) tiles).
int max_patch_words(const ConvProblem &dw)
{
    const int HW = dw.H * dw.W;
    const long npix = (long)dw.N * HW;
    const long period = HW / std::gcd(HW, kNT);
    const long ntiles = (npix + kNT - 1) / kNT;
    int worst = 0;
    for (long t = 0; t < period + 1 && t < ntiles; ++t) {
        const long n0 = t * kNT, pend = n0 + kNT < npix ? n0 + kNT : npix;
        const long nA = n0 / HW;
        int total = 0;
        for (int s = 0; s < kSegs; ++s) {
            const long base = (nA + s) * HW;
            const long lo = (n0 > base ? n0 : base) - base;
            const long hi = (pend < base + HW ? pend : base + HW) - base;
            total += make_seg((int)lo, (int)hi, dw.H, dw.W).ndw;
        }
        if (total > worst) worst = total;
    }
    return worst;
}

}  // namespace

bool plan_dwpw(const ConvProblem &dw, int OC, DwPwPlan *plan)
{
    if (dw.dtype != TVG_BF16 || dw.sh != 1 || dw.sw != 1 || dw.ph != 1 || dw.pw != 1) return false;
    if (dw.IC % kKC != 0 || dw.H * dw.W < 32 || OC < 1) return false;
    if ((size_t)dw.N * dw.IC * dw.H * dw.W * 2 > (size_t)kOutOfRange) return false;
    if ((size_t)OC * dw.IC * 2 > (size_t)kOutOfRange) return false;
    const int words = max_patch_words(dw);
    if (words > 16 * 8) return false;
    plan->lt = words <= 8 * 8 ? 8 : 16;            // one or two passes of 64 words over a row
    // every channel tile repeats the depthwise stage of its pixels, so tall tiles where the
    // accumulators allow (measured: 512 -> 512 at 14x14, batch 32: 37 us with 128, 29 with 256)
    plan->mt = OC <= 64 ? 64 : (OC >= 256 && dw.IC <= 512) ? 256 : 128;
    plan->tiles = (long)((OC + plan->mt - 1) / plan->mt) * ((dw.npix + kNT - 1) / kNT);
    return plan->tiles < (1L << 31);
}

tvg_status launch_dwpw(const ConvProblem &dw, int OC, int pw_relu, int pw_stream_out,
                       const DwPwPlan &plan, const DwPwPointers &ptr, hipStream_t stream)
{
    if (reinterpret_cast<uintptr_t>(ptr.w_dw) % 4 != 0) return TVG_ERR_UNSUPPORTED;
    DwPwArgs a;
    a.x = static_cast<const bf16_t *>(ptr.x); a.w_dw = static_cast<const bf16_t *>(ptr.w_dw);
    a.scale_dw = ptr.scale_dw; a.shift_dw = ptr.shift_dw;
    a.w_pw = static_cast<const bf16_t *>(ptr.w_pw);
    a.scale = ptr.scale_pw; a.shift = ptr.shift_pw; a.bias = ptr.bias_pw;
    a.residual = static_cast<const bf16_t *>(ptr.residual); a.y = static_cast<bf16_t *>(ptr.y);
    a.N = dw.N; a.C = dw.IC; a.H = dw.H; a.W = dw.W; a.OC = OC; a.npix = dw.npix;
    a.relu = pw_relu | (pw_stream_out << 1);
    a.relu_dw = dw.relu;
    a.mtiles = (OC + plan.mt - 1) / plan.mt;
    a.vmode = pick_store_vmode(TVG_BF16, dw.H * dw.W, ptr.y, ptr.residual);
    a.x_bytes = (uint32_t)((size_t)dw.N * dw.IC * dw.H * dw.W * 2);
    a.w_bytes = (uint32_t)((size_t)OC * dw.IC * 2);
    const dim3 grid((unsigned)plan.tiles), block(256);
#define TVG_DWPW(MT_, LT_) hipLaunchKernelGGL((dwpw_kernel<MT_, LT_>), grid, block, 0, stream, a)
    if (plan.mt == 256) {
        if (plan.lt == 8) TVG_DWPW(256, 8);
        else TVG_DWPW(256, 16);
    } else if (plan.mt == 128) {
        if (plan.lt == 8) TVG_DWPW(128, 8);
        else TVG_DWPW(128, 16);
    } else {
        if (plan.lt == 8) TVG_DWPW(64, 8);
        else TVG_DWPW(64, 16);
    }
#undef TVG_DWPW
    return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
}

}  // namespace tvg
