// fp32 fused conv2d for launch-bound problems (batch 1: the ResNet-18 shapes of Table 2 have
// roofline times of 0.1 - 1.5 us, far below the cost of a launch): 1x1 and 3x3 filters, stride 1
// or 2, "same" padding.  One launch, nothing but y written (TVM paper Section 4.2 cooperative
// fetch, Section 4.3 tensorization; Section 3 fusion for the tail).
//
// What makes fp32 different from the bf16 kernels: v_mfma_f32_32x32x2_f32 takes ONE k value per
// lane (lanes 0-31: k, lanes 32-63: k + 1), so nothing has to be transposed.
//   - The pixel operand of tap (r, s) is the fp32 input itself at a shifted address: the input
//     rows a tile needs are copied into LDS in their natural [channel][row][column] layout with
//     zero borders, and 32 consecutive pixels are 32 consecutive words.
//   - The weight operand of lane (oc, half) over a run of k values is a CONTIGUOUS run of floats
//     of the OIHW tensor (k = (ic, r, s) is its innermost order).  A wave copies the 32 runs of
//     a pass (32 output channels x 8 input channels x taps) into LDS with 16-byte loads whose
//     lanes walk along the runs, and every lane then reads its own run's floats one by one.
//     (The first version loaded each lane's run straight into registers: every lane then touches
//     cache lines of its own, a wave's load instruction 64 of them, and with 8 to 16 waves per CU
//     the lines are evicted and fetched again for each of a run's nine loads - C12 at batch 1
//     took 28 us, C9 18 us, bound by the CU's address unit.)
// A workgroup owns 32 output channels x 32 consecutive pixels of one image; its NW waves (1 to
// 16) split the reduction: in every pass wave w takes 8 input channels (4 per half-wave), copies
// their rows into LDS of its own, and needs no barrier to use them.  At the end the waves add
// their accumulators through LDS (one barrier pair) and 256 threads apply the fused tail and
// store rows of 4 consecutive pixels.  The reduction order is fixed, results are deterministic.
#include "tvg_device.h"
#include "tvg_internal.h"

namespace tvg {

namespace {

constexpr int kCPH = 4;              // input channels per half-wave and pass
// patch loads per lane and pass (16-, 8- or 4-byte loads for rows of 4n, 2n, other pixel counts);
// workgroups of 16 waves (4 per SIMD, 128 registers each) hold fewer
constexpr int kMaxSlots = 16, kMaxBig = 8;
constexpr int kPartPitch = 65;       // floats per (wave, register) row of the partial sums
constexpr int kWRow = 73;            // floats of one weight run in LDS (3x3: 72 + 1); a tile's runs: T x 73, a 16-byte multiple
constexpr int kRsrc = 0x00020000;

struct F32Args {
    const float *x, *w, *scale, *shift, *bias, *residual;
    float *y;
    int N, IC, H, W, OC, OH, OW, relu;
    int mtiles, tpi;        // channel tiles, pixel tiles per image
    int nw, passes;         // waves per workgroup, passes over the channels (per slice)
    int ksplit;             // slices of the reduction across workgroups (blockIdx.y); > 1: raw sums to ws
    float *ws;              // [ksplit][N][OC][OH][OW] partial sums
    int pitch, region;      // LDS row pitch and floats per wave region
    int vec_out;            // y (and residual) rows of 4 pixels are aligned 16-byte pieces
    uint32_t x_bytes, w_bytes;
};

// T = tile edge: 32 (v_mfma_f32_32x32x2_f32: the two half-waves hold k and k + 1) or 16
// (v_mfma_f32_16x16x4_f32: four quarter-waves, four k values).  The small tile is for layers that
// leave most CUs without a 32 x 32 tile: every wave of a workgroup issues its MFMAs to the matrix
// pipe of its SIMD, 36 of 64 cycles each per pass of a 3x3 layer, and with 16 waves on a CU that
// is 9200 cycles (4.4 us) while three quarters of the chip idle; a quarter of the tile is a quarter
// of that on four times the CUs.
template <int R, int STRIDE, int VEC, bool BIG, int T>
__global__ __launch_bounds__(BIG ? 1024 : 512) void conv_f32_small_kernel(const F32Args a)
{
    constexpr int KG = 64 / T;                     // k values per MFMA = groups of T lanes
    constexpr int CPG = 2 * kCPH / KG;             // input channels per group and pass
    constexpr int NV = T * T / 64;                 // accumulator registers
    constexpr int kWRegion = T * kWRow;
    constexpr int RS = R * R, PAD = R / 2;
    constexpr int WROW = 2 * kCPH * RS;            // floats of one output channel's run per pass
    constexpr int WPITCH = WROW + 1;               // its pitch in LDS (odd: conflict-free reads)
    constexpr int WPIECES = T * WROW / 4;          // 16-byte pieces of the T runs
    constexpr int WSLOTS = (WPIECES + 63) / 64;    // per lane
    extern __shared__ __attribute__((aligned(16))) float smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lp = lane & (T - 1), half = lane / T;        // (half: the lane's k group)
    int b = blockIdx.x;
    const int mt = b % a.mtiles;
    b /= a.mtiles;
    const int pt = b % a.tpi, n = b / a.tpi;
    const int m0 = mt * T, p0 = pt * T;
    const int OHW = a.OH * a.OW, W = a.W, H = a.H;
    const int npx = min(T, OHW - p0);
    const int oh_lo = p0 / a.OW, oh_hi = (p0 + npx - 1) / a.OW;
    const int ih_lo = oh_lo * STRIDE - PAD;
    const int nr = (oh_hi - oh_lo) * STRIDE + R;          // input rows of the tile (with padding rows)
    const int pitch = a.pitch, plane = nr * pitch;
    // rows that exist in the image: one contiguous run per channel
    const int ih_first = max(ih_lo, 0), ih_last = min(ih_lo + nr - 1, H - 1);
    const int E = (ih_last - ih_first + 1) * W;           // floats per channel to copy
    const int row_shift = ih_first - ih_lo;

    float *reg = smem + wave * (a.region + kWRegion);
    float *wl = reg + a.region;                            // the wave's 32 weight runs
    // zero the wave's region once: border columns and rows outside the image stay zero, the
    // interior is overwritten by every pass
    for (int i = lane * 4; i < a.region; i += 256)
        *reinterpret_cast<float4v *>(reg + i) = float4v{0.0f, 0.0f, 0.0f, 0.0f};

    const __amdgpu_buffer_rsrc_t xrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.x), 0, a.x_bytes, kRsrc);
    const __amdgpu_buffer_rsrc_t wrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.w), 0, a.w_bytes, kRsrc);

    // this lane's pixel (lanes past the tile's end shadow pixel 0; their results are dropped)
    const int pp = lp < npx ? lp : 0;
    const int oh = (p0 + pp) / a.OW, ow = (p0 + pp) - oh * a.OW;
    const int bbase = half * CPG * plane + (oh - oh_lo) * STRIDE * pitch + ow * STRIDE;
    // weight copy slots: piece q of the 32 runs -> (run, part); runs past OC shadow the last one
    uint32_t wsrc[WSLOTS];
    int wdst[WSLOTS];
#pragma unroll
    for (int k = 0; k < WSLOTS; ++k) {
        const int q = lane + 64 * k;
        const int run = q / (WROW / 4), part = q - run * (WROW / 4);
        wdst[k] = q < WPIECES ? run * WPITCH + part * 4 : -1;
        wsrc[k] = 4u * (uint32_t)(min(m0 + run, a.OC - 1) * a.IC * RS) + 16u * (uint32_t)part;
    }
    const int abase = lp * WPITCH + half * CPG * RS;

    // copy slots of this lane: element i of the wave's 8 x E floats -> (channel, row, column)
    const float inv_e = 1.0f / (float)E, inv_w = 1.0f / (float)W;
    constexpr int NSLOT = BIG ? kMaxBig : kMaxSlots;
    constexpr int STEP = VEC;                      // floats per copy: 4, 2 or 1
    uint32_t src_off[NSLOT];      // byte offset within channel block 0 of the image (per pass: + channels)
    int dst_off[NSLOT];           // float offset in the wave's region, -1 = no element
#pragma unroll
    for (int k = 0; k < NSLOT; ++k) {
        const int i = (lane + 64 * k) * STEP;
        dst_off[k] = -1;
        src_off[k] = 0;
        if (i < 2 * kCPH * E) {
            int e, col;
            const int ch = fast_div(i, E, inv_e, &e);
            const int row = fast_div(e, W, inv_w, &col);
            src_off[k] = 4u * (uint32_t)((ch * H + ih_first) * W + e);
            dst_off[k] = ch * plane + (row + row_shift) * pitch + col + PAD;
        }
    }

    typedef float accv __attribute__((ext_vector_type(NV)));
    accv acc;
#pragma unroll
    for (int v = 0; v < NV; ++v) acc[v] = 0.0f;

    for (int pass = 0; pass < a.passes; ++pass) {
        // this wave's 8 channels (slice blockIdx.y of the reduction takes a.passes passes)
        const int ic0 = (((int)blockIdx.y * a.passes + pass) * a.nw + wave) * 2 * kCPH;
        // weights: the runs of channels ic0 .. ic0 + 7 (WROW contiguous floats per output channel)
        uint4v wv[WSLOTS];
#pragma unroll
        for (int k = 0; k < WSLOTS; ++k)
            if (wdst[k] >= 0)
                wv[k] = __builtin_bit_cast(
                    uint4v, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, wsrc[k], ic0 * RS * 4, 0));
        // the patch rows of the 8 channels
        const int cbase = 4 * ((n * a.IC + ic0) * H * W);
        float pv[NSLOT][STEP];
#pragma unroll
        for (int k = 0; k < NSLOT; ++k) {
            if (dst_off[k] >= 0) {                       // (the same lanes in every pass)
                if constexpr (VEC == 4) {
                    const uint4v t4 = __builtin_bit_cast(
                        uint4v, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, src_off[k], cbase, 0));
#pragma unroll
                    for (int d = 0; d < 4; ++d) pv[k][d] = __uint_as_float(t4[d]);
                } else if constexpr (VEC == 2) {
                    const uint2v t2 = __builtin_bit_cast(
                        uint2v, __builtin_amdgcn_raw_buffer_load_b64(xrsrc, src_off[k], cbase, 0));
                    pv[k][0] = __uint_as_float(t2[0]);
                    pv[k][1] = __uint_as_float(t2[1]);
                } else {
                    pv[k][0] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(xrsrc, src_off[k], cbase, 0));
                }
            }
        }
#pragma unroll
        for (int k = 0; k < WSLOTS; ++k)
            if (wdst[k] >= 0) {
#pragma unroll
                for (int d = 0; d < 4; ++d) wl[wdst[k] + d] = __uint_as_float(wv[k][d]);
            }
#pragma unroll
        for (int k = 0; k < NSLOT; ++k)
            if (dst_off[k] >= 0) {
#pragma unroll
                for (int d = 0; d < STEP; ++d) reg[dst_off[k] + d] = pv[k][d];
            }
        // a wave reads only what it wrote itself: LDS operations of a wave complete in order
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int c = 0; c < CPG; ++c)
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int s = 0; s < R; ++s) {
                    const float bv = reg[bbase + c * plane + r * pitch + s];
                    const float av = wl[abase + c * RS + r * R + s];
                    // pixel operand first: the accumulator tile is D[pixel][channel]
                    if constexpr (T == 32) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av, acc, 0, 0, 0);
                    else acc = __builtin_amdgcn_mfma_f32_16x16x4f32(bv, av, acc, 0, 0, 0);
                }
        __builtin_amdgcn_wave_barrier();      // the next pass overwrites the rows just read
    }

    // ---- the waves' partial sums meet in LDS (over the patch regions, which are done with) ----
    __syncthreads();
    float *part = smem;
#pragma unroll
    for (int v = 0; v < NV; ++v) part[(wave * NV + v) * kPartPitch + lane] = acc[v];
    __syncthreads();
    // T = 32: value v of lane l is channel l % 32, pixel 8*(v/4) + 4*(l/32) + v%4; T = 16: channel
    // l % 16, pixel 4*(l/16) + v.  Thread t of the first T*T/4 takes channel t / (T/4) and the 4
    // consecutive pixels from 4 * (t % (T/4)) on.
    for (int t = tid; t < T * T / 4; t += (int)blockDim.x) {
        const int cc = t / (T / 4), pb = (t % (T / 4)) * 4;
        const int src_lane = T == 32 ? cc + 32 * ((pb >> 2) & 1) : cc + 16 * (pb >> 2);
        const int v0 = T == 32 ? 4 * (pb >> 3) : 0;
        float sum[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int s = 0; s < a.nw; ++s)
#pragma unroll
            for (int q = 0; q < 4; ++q) sum[q] += part[(s * NV + v0 + q) * kPartPitch + src_lane];
        const int oc = m0 + cc;
        if (oc >= a.OC || pb >= npx) continue;
        if (a.ksplit > 1) {       // a slice of the reduction: raw sums, the reduce launch finishes
            float *dst = a.ws + (size_t)blockIdx.y * ((size_t)a.N * a.OC * OHW) +
                         (size_t)(n * a.OC + oc) * OHW + p0 + pb;
            if (OHW % 4 == 0) *reinterpret_cast<float4v *>(dst) = float4v{sum[0], sum[1], sum[2], sum[3]};
            else
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (pb + q < npx) dst[q] = sum[q];
            continue;
        }
        const float sc = a.scale[oc];
        const float sf = a.bias ? fmaf(a.bias[oc], sc, a.shift[oc]) : a.shift[oc];
        const float floor_v = a.relu ? 0.0f : -INFINITY;
        const int idx = (n * a.OC + oc) * OHW + p0 + pb;
        if (a.vec_out) {                               // OHW % 4 == 0: the whole group is inside
            float4v r4 = {0.0f, 0.0f, 0.0f, 0.0f};
            if (a.residual) r4 = *reinterpret_cast<const float4v *>(a.residual + idx);
            float4v o;
#pragma unroll
            for (int q = 0; q < 4; ++q) o[q] = fmaxf(fmaf(sum[q], sc, sf) + r4[q], floor_v);
            *reinterpret_cast<float4v *>(a.y + idx) = o;
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (pb + q < npx) {
                    float o = fmaf(sum[q], sc, sf);
                    if (a.residual) o += a.residual[idx + q];
                    a.y[idx + q] = fmaxf(o, floor_v);
                }
        }
    }
}

template <int R, int STRIDE, int T>
tvg_status launch_rs(const F32Args &a, int vec, dim3 grid, size_t lds, hipStream_t stream)
{
    // opt in to > 64 KB of dynamic LDS (a cheap host call, made before every launch: the four
    // instances below would each need a flag of their own)
    auto set = [&](auto kernel) {
        return hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) == hipSuccess;
    };
#define TVG_F32_LAUNCH(VEC_, BIG_)                                                             \
    do {                                                                                       \
        auto kernel = conv_f32_small_kernel<R, STRIDE, VEC_, BIG_, T>;                         \
        if (!set(kernel)) return TVG_ERR_LAUNCH;                                               \
        hipLaunchKernelGGL(kernel, grid, dim3(64 * a.nw), lds, stream, a);                     \
    } while (0)
    if (a.nw == 16) {
        if (vec == 4) TVG_F32_LAUNCH(4, true);
        else if (vec == 2) TVG_F32_LAUNCH(2, true);
        else TVG_F32_LAUNCH(1, true);
    } else {
        if (vec == 4) TVG_F32_LAUNCH(4, false);
        else if (vec == 2) TVG_F32_LAUNCH(2, false);
        else TVG_F32_LAUNCH(1, false);
    }
#undef TVG_F32_LAUNCH
    return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
}

// ---------------------------------------------------------------------------------------------
// The same idea for the 7x7 stride-2 pad-3 stem with up to four input channels (C1 of Table 2 at
// batch 1: K = 147, too short and too ragged to split by channels).  A workgroup owns 32 output
// channels x 64 consecutive pixels of one image and has SEVEN waves, one per filter row: wave r
// multiplies filter row r of every input channel - 8 tap slots per (channel, row), slot 0 a zero
// weight, so that the window of pixel (oh, ow) starts at the even padded column 2 ow - into its
// own accumulators; the seven partial tiles are added through LDS and the fused tail stores rows
// of four pixels.  The input rows of the tile are staged once, shared by all waves, in their
// natural layout with four zero columns on either side; the 32 x IC x 49 weights of the tile
// are one contiguous run of the OIHW tensor, copied with coalesced loads into [row][channel]
// [slot][oc] order, so that the 32 lanes of an operand read are 32 consecutive words.
struct F32StemArgs {
    const float *x, *w, *scale, *shift, *bias, *residual;
    float *y;
    int N, H, W, OC, OH, OW, relu;
    int mtiles, tpi, nr, pw4;          // channel tiles, pixel tiles per image, staged rows, 16-byte words per staged row
    float inv_rowwords, inv_pw4;       // reciprocals of nr * pw4 and pw4
    int vec_out;
    uint32_t x_bytes, w_bytes;
};

constexpr int kStemWaves = 7, kStemThreads = 64 * kStemWaves, kStemPix = 64;

template <int IC>
__global__ __launch_bounds__(kStemThreads) void conv_f32_stem_kernel(const F32StemArgs a)
{
    constexpr int R = 7, KW = IC * 49;
    constexpr int WFLOATS = R * IC * 8 * 32;                 // staged weights
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lp = lane & 31, half = lane >> 5;
    int b = blockIdx.x;
    const int mt = b % a.mtiles;
    b /= a.mtiles;
    const int pt = b % a.tpi, n = b / a.tpi;
    const int m0 = mt * 32, p0 = pt * kStemPix;
    const int OHW = a.OH * a.OW, W = a.W, H = a.H;
    const int npx = min(kStemPix, OHW - p0);
    const int oh_lo = p0 / a.OW;
    const int ih_lo = oh_lo * 2 - 3;
    const int PW = a.pw4 * 4, nr = a.nr, plane = nr * PW;
    float *wl = smem;                                        // [r][ic][slot][oc]
    float *patch = smem + WFLOATS;                           // [ic][row][PW]

    const __amdgpu_buffer_rsrc_t xrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.x), 0, a.x_bytes, kRsrc);
    const __amdgpu_buffer_rsrc_t wrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.w), 0, a.w_bytes, kRsrc);

    // ---- weights: element e of the tile's contiguous run -> (oc, ic, r, s); rows past OC read zeros
    constexpr int WN = (32 * KW + kStemThreads - 1) / kStemThreads;
    float wv[WN];
#pragma unroll
    for (int j = 0; j < WN; ++j) {
        const int e = tid + j * kStemThreads;
        const uint32_t off = e < 32 * KW ? 4u * (uint32_t)(m0 * KW + e) : 0xFFFFFFFCu;
        wv[j] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(wrsrc, off, 0, 0));
    }
    // ---- patch: task = one 16-byte word of a staged row; the first and last word of a row are
    // padding, rows outside the image come back as zeros (out-of-range offset)
    const int ntask = IC * nr * a.pw4;
    for (int t = tid; t < ntask; t += kStemThreads) {
        int rem, j;
        const int ic = fast_div(t, nr * a.pw4, a.inv_rowwords, &rem);
        const int row = fast_div(rem, a.pw4, a.inv_pw4, &j);
        const int ih = ih_lo + row;
        const bool ok = j > 0 && j < a.pw4 - 1 && ih >= 0 && ih < H;
        const uint32_t off = ok ? 4u * (uint32_t)(((n * IC + ic) * H + ih) * W + 4 * (j - 1)) : 0xFFFFFFF0u;
        const uint4v v = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, off, 0, 0));
        *reinterpret_cast<uint4v *>(patch + (ic * nr + row) * PW + 4 * j) = v;
    }
#pragma unroll
    for (int j = 0; j < WN; ++j) {
        const int e = tid + j * kStemThreads;
        if (e < 32 * KW) {
            const int oc = e / KW, rem = e - oc * KW;
            const int ic = rem / 49, t = rem - ic * 49;
            const int r = t / 7, s = t - r * 7;
            wl[((r * IC + ic) * 8 + s + 1) * 32 + oc] = wv[j];
        }
    }
    for (int i = tid; i < R * IC * 32; i += kStemThreads)   // slot 0 of every (row, channel)
        wl[(i >> 5) * 8 * 32 + (i & 31)] = 0.0f;
    __syncthreads();

    // ---- wave r: filter row r of every channel, two blocks of 32 pixels ---------------------
    int bbase[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int q = j * 32 + lp;
        const int pp = q < npx ? q : 0;                      // lanes past the end shadow pixel 0
        const int oh = (p0 + pp) / a.OW, ow = (p0 + pp) - oh * a.OW;
        bbase[j] = ((oh - oh_lo) * 2 + wave) * PW + 2 * ow + half;
    }
    const int abase = (wave * IC * 8 + half) * 32 + lp;
    float16v acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;
#pragma unroll
    for (int ic = 0; ic < IC; ++ic)
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            const float av = wl[abase + (ic * 8 + 2 * st) * 32];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const float bv = patch[bbase[j] + ic * plane + 2 * st];
                // pixel operand first: the accumulator tile is D[pixel][channel]
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av, acc[j], 0, 0, 0);
            }
        }

    // ---- the seven partial tiles meet in LDS (over the operands, which are done with) --------
    __syncthreads();
    float *part = smem;                                      // [block][wave][16][kPartPitch]
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) part[((j * kStemWaves + wave) * 16 + v) * kPartPitch + lane] = acc[j][v];
    __syncthreads();
    for (int g = tid; g < 512; g += kStemThreads) {
        const int j = g >> 8, t = g & 255;
        const int cc = t >> 3, pb = (t & 7) * 4;
        const int src_lane = cc + 32 * ((pb >> 2) & 1), v0 = 4 * (pb >> 3);
        float sum[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int s = 0; s < kStemWaves; ++s)
#pragma unroll
            for (int q = 0; q < 4; ++q) sum[q] += part[((j * kStemWaves + s) * 16 + v0 + q) * kPartPitch + src_lane];
        const int oc = m0 + cc, px = j * 32 + pb;
        if (oc >= a.OC || px >= npx) continue;
        const float sc = a.scale[oc];
        const float sf = a.bias ? fmaf(a.bias[oc], sc, a.shift[oc]) : a.shift[oc];
        const float floor_v = a.relu ? 0.0f : -INFINITY;
        const int idx = (n * a.OC + oc) * OHW + p0 + px;
        if (a.vec_out) {                                     // OHW % 4 == 0: the whole group is inside
            float4v r4 = {0.0f, 0.0f, 0.0f, 0.0f};
            if (a.residual) r4 = *reinterpret_cast<const float4v *>(a.residual + idx);
            float4v o;
#pragma unroll
            for (int q = 0; q < 4; ++q) o[q] = fmaxf(fmaf(sum[q], sc, sf) + r4[q], floor_v);
            *reinterpret_cast<float4v *>(a.y + idx) = o;
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (px + q < npx) {
                    float o = fmaf(sum[q], sc, sf);
                    if (a.residual) o += a.residual[idx + q];
                    a.y[idx + q] = fmaxf(o, floor_v);
                }
        }
    }
}

// Rows of input a tile of 64 consecutive pixels can touch, and the LDS it needs.
static bool f32_stem_geometry(const ConvProblem &p, int *nr, int *pw4, size_t *lds)
{
    const int OHW = p.OH * p.OW;
    const int orows = std::min(p.OH, (std::min(kStemPix, OHW) + p.OW - 2) / p.OW + 1);
    *nr = (orows - 1) * 2 + 7;
    *pw4 = p.W / 4 + 2;
    const size_t operands = ((size_t)7 * p.IC * 8 * 32 + (size_t)p.IC * *nr * *pw4 * 4) * 4;
    const size_t partials = (size_t)2 * kStemWaves * 16 * kPartPitch * 4;
    *lds = std::max(operands, partials);
    return *lds <= 80 * 1024;
}

}  // namespace

bool plan_conv_f32_small(const ConvProblem &p, F32SmallPlan *plan)
{
    plan->stem = 0;
    if (p.dtype == TVG_F32 && p.R == 7 && p.S == 7 && p.sh == 2 && p.sw == 2 && p.ph == 3 && p.pw == 3 &&
        p.IC <= 4 && p.W % 4 == 0) {
        // the 7x7 stem of launch-bound problems: one launch, seven waves split the filter rows
        const Knobs knobs = forced_knobs(p);
        if (knobs.split_k > 0 || knobs.mt > 0) return false;
        const long gtiles = (long)((p.OC + 127) / 128) * ((p.npix + 127) / 128);
        if (gtiles >= kComputeUnits) return false;
        int nr, pw4;
        size_t lds;
        if (!f32_stem_geometry(p, &nr, &pw4, &lds)) return false;
        if ((long)p.IC * nr * pw4 >= (1 << 22)) return false;                  // fast_div range
        if ((size_t)p.N * p.IC * p.H * p.W >= ((size_t)1 << 30) || (size_t)p.OC * p.K >= ((size_t)1 << 30))
            return false;                                                      // 32-bit byte offsets
        if ((long)p.N * ((p.OH * p.OW + kStemPix - 1) / kStemPix) * ((p.OC + 31) / 32) >= (1L << 31)) return false;
        plan->stem = 1;
        plan->tile = 32;
        plan->nw = kStemWaves;
        plan->passes = 1;
        plan->ksplit = 1;
        plan->workspace_bytes = 0;
        plan->pitch = pw4 * 4;
        plan->region = nr;
        plan->vec = 4;
        plan->lds_bytes = lds;
        return true;
    }
    if (p.dtype != TVG_F32 || p.R != p.S || (p.R != 1 && p.R != 3)) return false;
    if (p.ph != p.R / 2 || p.pw != p.R / 2 || p.sh != p.sw || (p.sh != 1 && p.sh != 2)) return false;
    if (p.IC % (2 * kCPH) != 0) return false;
    const Knobs knobs = forced_knobs(p);
    if (knobs.split_k > 0 || knobs.mt > 0) return false;     // the caller shapes the generic kernel
    // launch-bound problems only: those the generic kernel cannot fill the chip with in one pass
    const long gtiles = (long)((p.OC + 127) / 128) * ((p.npix + 127) / 128);
    if (gtiles >= kComputeUnits) return false;
    const int OHW = p.OH * p.OW;
    const int pitch = p.W + 2 * (p.R / 2);
    const int vec = p.W % 4 == 0 ? 4 : p.W % 2 == 0 ? 2 : 1;
    if ((size_t)p.N * p.IC * p.H * p.W >= ((size_t)1 << 30) || (size_t)p.OC * p.K >= ((size_t)1 << 30))
        return false;                                        // 32-bit byte offsets
    // the geometry of a plan with tiles of T x T outputs
    auto geometry = [&](int T, F32SmallPlan *g) {
        const int orows = std::min(p.OH, (std::min(T, OHW) + p.OW - 2) / p.OW + 1);   // rows T pixels can touch
        const int nr = (orows - 1) * p.sh + p.R;
        const int region = (2 * kCPH * nr * pitch + 3) / 4 * 4;
        const long elems = (long)2 * kCPH * std::min(nr, p.H) * p.W;
        const long slots = (elems / vec + 63) / 64;
        if (slots > kMaxSlots) return false;
        if (elems >= (1 << 22)) return false;                    // fast_div range
        int nw = slots <= kMaxBig ? 16 : 8;
        auto lds_for = [&](int w) {
            return std::max((size_t)w * (region + T * kWRow) * 4, (size_t)w * (T * T / 64) * kPartPitch * 4);
        };
        while (nw > 1 && (p.IC % (2 * kCPH * nw) != 0 || lds_for(nw) > 160 * 1024)) nw >>= 1;
        const size_t lds = lds_for(nw);
        if (lds > 160 * 1024) return false;
        const long wgs = (long)p.N * ((OHW + T - 1) / T) * ((p.OC + T - 1) / T);
        if (wgs >= (1L << 31)) return false;
        // Deep reductions on few tiles (C9, C10, C12 at batch 1: 4 to 8 passes of about 3.6 us each
        // under the large tile, the matrix pipes of a few CUs doing all the work): slices of the
        // reduction go to different workgroups, their sums to the workspace, and the reduce launch
        // of the generic kernel adds them in a fixed order.  A second launch costs about 4 us, so
        // only from three passes on.
        const int passes = p.IC / (2 * kCPH * nw);
        int ksplit = 1;
        if (passes >= 3 && wgs < kComputeUnits) {
            ksplit = passes;
            while (ksplit > 1 && (passes % ksplit != 0 || wgs * (ksplit / 2) >= 2 * kComputeUnits)) --ksplit;
        }
        g->tile = T;
        g->nw = nw;
        g->ksplit = ksplit;
        g->passes = passes / ksplit;
        g->workspace_bytes = ksplit > 1 ? (size_t)ksplit * p.npix * p.OC * sizeof(float) : 0;
        g->pitch = pitch;
        g->region = region;
        g->vec = vec;
        g->lds_bytes = lds;
        g->stem = 0;
        return true;
    };
    // 16 x 16 tiles where 32 x 32 ones would leave three quarters of the CUs without a workgroup,
    // provided the small tiles then need no second launch (measured at batch 1, us with 32 / 16:
    // C7 12.0 / 7.9, C9 11.3 / 9.1, C11 10.9 / 7.9, C10 12.1 / 11.6, C8 7.9 / 7.9; with more tiles
    // the small ones lose - C2 8.3 / 20.2, C4 9.8 / 11.8, C6 11.0 / 12.3 - as does C12, 12.5 / 16.2,
    // whose reduction stays split either way and whose 49 pixels make four tiles of 16, one of them
    // a single pixel)
    const long wgs32 = (long)p.N * ((OHW + 31) / 32) * ((p.OC + 31) / 32);
    if (wgs32 <= kComputeUnits / 4) {
        F32SmallPlan small;
        if (geometry(16, &small) && small.ksplit == 1) {
            *plan = small;
            return true;
        }
    }
    return geometry(32, plan);
}

bool conv_f32_small_pointers_ok(const ConvPointers &ptr)
{
    return reinterpret_cast<uintptr_t>(ptr.x) % 16 == 0 && reinterpret_cast<uintptr_t>(ptr.w) % 4 == 0;
}

static tvg_status launch_conv_f32_stem(const ConvProblem &p, const F32SmallPlan &plan, const ConvPointers &ptr,
                                       hipStream_t stream)
{
    F32StemArgs a;
    a.x = static_cast<const float *>(ptr.x); a.w = static_cast<const float *>(ptr.w);
    a.scale = ptr.scale; a.shift = ptr.shift; a.bias = ptr.bias;
    a.residual = static_cast<const float *>(ptr.residual); a.y = static_cast<float *>(ptr.y);
    a.N = p.N; a.H = p.H; a.W = p.W; a.OC = p.OC; a.OH = p.OH; a.OW = p.OW;
    a.relu = p.relu;
    a.mtiles = (p.OC + 31) / 32;
    a.tpi = (p.OH * p.OW + kStemPix - 1) / kStemPix;
    a.nr = plan.region;
    a.pw4 = plan.pitch / 4;
    a.inv_rowwords = 1.0f / (float)(a.nr * a.pw4);
    a.inv_pw4 = 1.0f / (float)a.pw4;
    a.vec_out = (p.OH * p.OW) % 4 == 0 && reinterpret_cast<uintptr_t>(ptr.y) % 16 == 0 &&
                reinterpret_cast<uintptr_t>(ptr.residual) % 16 == 0;
    a.x_bytes = (uint32_t)((size_t)p.N * p.IC * p.H * p.W * 4);
    a.w_bytes = (uint32_t)((size_t)p.OC * p.IC * 49 * 4);
    const dim3 grid((unsigned)((long)a.mtiles * a.tpi * p.N));
    auto go = [&](auto kernel) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return TVG_ERR_LAUNCH;
        hipLaunchKernelGGL(kernel, grid, dim3(kStemThreads), plan.lds_bytes, stream, a);
        return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
    };
    switch (p.IC) {
    case 1: return go(conv_f32_stem_kernel<1>);
    case 2: return go(conv_f32_stem_kernel<2>);
    case 3: return go(conv_f32_stem_kernel<3>);
    default: return go(conv_f32_stem_kernel<4>);
    }
}

tvg_status launch_conv_f32_small(const ConvProblem &p, const F32SmallPlan &plan, const ConvPointers &ptr,
                                 hipStream_t stream)
{
    if (plan.stem) return launch_conv_f32_stem(p, plan, ptr, stream);
    F32Args a;
    a.x = static_cast<const float *>(ptr.x); a.w = static_cast<const float *>(ptr.w);
    a.scale = ptr.scale; a.shift = ptr.shift; a.bias = ptr.bias;
    a.residual = static_cast<const float *>(ptr.residual); a.y = static_cast<float *>(ptr.y);
    a.N = p.N; a.IC = p.IC; a.H = p.H; a.W = p.W; a.OC = p.OC; a.OH = p.OH; a.OW = p.OW;
    a.relu = p.relu;
    a.mtiles = (p.OC + plan.tile - 1) / plan.tile;
    a.tpi = (p.OH * p.OW + plan.tile - 1) / plan.tile;
    a.nw = plan.nw; a.passes = plan.passes; a.pitch = plan.pitch; a.region = plan.region;
    a.ksplit = plan.ksplit; a.ws = ptr.workspace;
    a.vec_out = (p.OH * p.OW) % 4 == 0 && reinterpret_cast<uintptr_t>(ptr.y) % 16 == 0 &&
                reinterpret_cast<uintptr_t>(ptr.residual) % 16 == 0;
    a.x_bytes = (uint32_t)((size_t)p.N * p.IC * p.H * p.W * 4);
    a.w_bytes = (uint32_t)((size_t)p.OC * p.IC * p.R * p.S * 4);
    const dim3 grid((unsigned)((long)a.mtiles * a.tpi * p.N), (unsigned)plan.ksplit);
    const int vec = plan.vec;
    tvg_status st;
    if (plan.tile == 16) {
        if (p.R == 3) st = p.sh == 1 ? launch_rs<3, 1, 16>(a, vec, grid, plan.lds_bytes, stream)
                                     : launch_rs<3, 2, 16>(a, vec, grid, plan.lds_bytes, stream);
        else st = p.sh == 1 ? launch_rs<1, 1, 16>(a, vec, grid, plan.lds_bytes, stream)
                            : launch_rs<1, 2, 16>(a, vec, grid, plan.lds_bytes, stream);
    } else {
        if (p.R == 3) st = p.sh == 1 ? launch_rs<3, 1, 32>(a, vec, grid, plan.lds_bytes, stream)
                                     : launch_rs<3, 2, 32>(a, vec, grid, plan.lds_bytes, stream);
        else st = p.sh == 1 ? launch_rs<1, 1, 32>(a, vec, grid, plan.lds_bytes, stream)
                            : launch_rs<1, 2, 32>(a, vec, grid, plan.lds_bytes, stream);
    }
    if (st != TVG_OK || plan.ksplit == 1) return st;
    return launch_splitk_reduce(p, plan.ksplit, ptr, stream);
}

}  // namespace tvg
