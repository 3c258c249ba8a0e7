// bf16 3x3 (pad 1, stride 1 or 2) fused conv2d, software-pipelined variant of the patch
// kernel: the operand tiles of an input-channel chunk live in one of TWO LDS stages, so the
// registers holding chunk c+1 are transposed and written to the idle stage BETWEEN the MFMAs
// of chunk c, and one barrier per chunk is all the synchronisation left.  The global loads of
// chunk c+3 are issued as soon as those registers are free (two register sets).  (TVM paper
// Section 4.2:
// cooperative fetch into the shared scope; Section 4.4: memory latency hidden behind compute -
// here inside one workgroup instead of by switching between workgroups.)
//
// Tile: 64 output channels x NT pixels (NT = 256, 128 or 64), 256 threads.
//
// LDS layout of a stage.  An MFMA lane consumes 8 channels (16 bytes) of one pixel or one
// filter row; the two channel octets of a chunk are kept in two separate PLANES, each a dense
// array of 16-byte words indexed by position, so that 16 consecutive lanes (which read the same
// octet of 16 consecutive positions) touch 256 consecutive bytes: conflict-free without
// padding, and the byte offset of a tap is one constant for all lanes.
//   A planes: [octet][tap][oc]      16 B each (+128 B between the planes: spreads the writes)
//   P planes: [octet][virtual row][column]   16 B each
// Virtual rows are those of the patch kernel: image n owns rows n*(H+2) .. n*(H+2)+H+1, first
// and last being zero padding.  For stride 2 a row is stored even columns first, then odd
// columns, so that the pixels of consecutive lanes (two columns apart) are again consecutive
// 16-byte words.
#include <stdio.h>
#include <stdlib.h>

#include <algorithm>
#include <type_traits>

#include "tvg_device.h"
#include "tvg_internal.h"

namespace tvg {

namespace {

struct DbufArgs {
    const bf16_t *x, *w;
    const float *scale, *shift, *bias;
    const bf16_t *residual;
    bf16_t *y;
    int N, IC, H, W, OC, OH, OW, npix, relu, mtiles;
    int vmode;        // pixels per vector store in the epilogue (8, 4 or 1)
    uint32_t x_bytes, w_bytes;
    int pplane;       // bytes of one channel-octet plane of the patch
    int pws;          // 16-byte words per patch row in a plane
    int xp16;         // extra bytes between the rows of consecutive images in a plane
    int stage_bytes;  // weight planes + patch planes + dump area
    int ss_offset;    // byte offset in LDS of the staged (scale, offset) pairs
    int ntiles, m_major;
    // reciprocals for fast_div (host-computed 1.0f / x): of the tile-order divisor, OH*OW, OW,
    // H + 2 and W / PX
    float inv_tdiv, inv_ohw, inv_ow, inv_vh, inv_wpx;
};

constexpr int kMT = 64;
constexpr int kChunk = 16;                       // input channels per chunk = K of one MFMA
constexpr int kAPlane = 9 * kMT * 16 + 128;      // bytes of one weight plane
constexpr int kRsrcFlags = 0x00020000;           // raw buffer descriptor word 3 on gfx9-family targets

__device__ __forceinline__ int xcd_remap(int bid, int nb)
{
    const int q = nb >> 3, rem = nb & 7;
    const int xcd = bid & 7, local = bid >> 3;
    return xcd < rem ? xcd * (q + 1) + local : rem * (q + 1) + (xcd - rem) * q + local;
}

// 16-bit half `ha` of a in the low half of the result, half `hb` of b in the high half.
__device__ __forceinline__ uint32_t pack_halves(uint32_t a, int ha, uint32_t b, int hb)
{
    // v_perm_b32 selects bytes 0..3 from its second source and 4..7 from its first
    const uint32_t sel = (ha ? 0x0302u : 0x0100u) | (hb ? 0x07060000u : 0x05040000u);
    return __builtin_amdgcn_perm(b, a, sel);
}

// s_waitcnt immediate for "at most vm vector-memory and lgkm LDS/scalar operations pending"
// (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8; 63 / 15 = no wait).
constexpr int waitcnt_imm(int vm, int lgkm)
{
    return (vm & 0xF) | ((vm >> 4) << 14) | (7 << 4) | (lgkm << 8);
}

// PT = patch load tasks per thread; PX = horizontally adjacent pixels per load (W must be a
// multiple: 16- to 128-bit loads).
//
// What limits this kernel is the number of instructions a SIMD has to issue per MFMA, so the
// loop body is kept to the bone: every LDS address is a register computed once per stage plus
// an immediate, one explicit wait covers all loads of a register set, and
// the widest load the row length admits is used.
//
// WM = waves along the 64 output channels (1 or 2), NJ = 32-pixel blocks per wave: the tile is
// 64 x NT with NT = (4 / WM) * NJ * 32.  (Tiles of 448 and 832 pixels - one workgroup per CU with
// 112 or 208 accumulator registers per lane - were measured: slower, a single wave per SIMD
// issues an MFMA plus its LDS operand read in 27 ns against 16 ns for two waves.)
//
// KG = 2: two groups of four waves share one tile and split the reduction - group g takes the
// chunks 2j + g, with LDS stages of its own - and add their accumulators through LDS at the
// end, each group finishing half of the tile.  For grids of at most one workgroup per CU: a lone
// group of four waves is bound by the latency of its own chain (barrier, operand reads, 36
// matrix instructions: about 1 us per chunk on C9, the matrix pipe busy for 0.58 of it), and
// no second workgroup is there to fill the gaps; the second group is.
//
// UNAL (with PX = 8, stride 1, rows of at most 7 pixels): rows that start at any 2-byte address.
// A row of an odd-sized map (7x7: 98-byte planes) begins 4-byte aligned or 2 bytes past that,
// alternating with the row and, when the plane is odd, with the channel.  Element-wise 2-byte
// loads (16 per thread and chunk on C12 against 18 matrix instructions per wave) kept the CU's
// address unit busier than its matrix pipes.  Instead a task is one row of one PAIR of channels:
// it fetches, per channel, the 16 bytes from the aligned address at or just below the row's
// start - the whole row in one load - and, when it comes to transposing, first moves each
// channel's four registers down by 16 bits where the row started in the upper half (one funnel
// shift per register, the amount a per-lane value), then writes pixel k's two channels as one
// 4-byte piece of the pixel's 16-byte word.  (A task of all eight channels, 16-byte stores, was
// measured first: the few threads that own a row - 60 of 256 on C12 - became the critical path,
// 31.4 us against 25.6; pairs spread the same rows over 240 threads.)  Pixels past the end of
// the row (the eighth element and beyond) go to the dump area.
//
// MG: two groups of four waves split the OUTPUT CHANNELS of a 128-channel tile - group g owns
// channels 64 g .. 64 g + 63 with weight planes of its own - and share one patch: the 512 threads
// stage it together (half the patch tasks per thread), every patch word feeds twice the matrix
// instructions, and a CU holds two waves per SIMD that run the same chunk.  For grids that fit
// the chip at one such workgroup per CU: stride-2 layers, whose patch is four times the output
// tile (their two stages then fit one workgroup per CU only), and stride-1 grids that would
// otherwise put two workgroups on some CUs and one on the rest.
template <int WM, int NJ, int STRIDE, int PT, int PX, int KG = 1, bool UNAL = false, bool MG = false>
__global__ __launch_bounds__(256 * (MG ? 2 : KG), 2) void conv3x3_dbuf_kernel(const DbufArgs a)
{
    static_assert(!UNAL || (PX == 8 && STRIDE == 1), "unaligned rows: whole rows of at most 7 pixels");
    static_assert(!(MG && (KG != 1 || UNAL)), "the channel-split variant has one reduction group and aligned rows");
    constexpr int MT = kMT;
    constexpr int WN = 4 / WM;
    constexpr int WTM = MT / WM, WTN = NJ * 32, NT = WN * WTN;
    constexpr int MI = WTM / 32;
    constexpr int PW32 = PX >= 2 ? PX / 2 : 1;        // registers per patch load
    constexpr int kWLoads = 5;                        // a weight task's 72 bytes: 4 x 16 + 8
    constexpr int NCH = UNAL ? 2 : 8;                 // channels per patch task
    constexpr int kLoads = kWLoads + NCH * PT;        // vector memory loads per thread and chunk
    constexpr int kP0 = 9 + kWLoads;                  // first patch item

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    // tid, wave: position within the thread's group of four waves (task lists, tile position)
    const int tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;
    const int group = (KG == 2 || MG) ? __builtin_amdgcn_readfirstlane(threadIdx.x >> 8) : 0;
    const int gbase = KG == 2 ? group * 2 * a.stage_bytes : 0;      // the group's two stages
    const int kgroup = KG == 2 ? group : 0;                          // which chunks the group takes
    // MG: the group's pair of weight planes within a stage; the patch planes follow all of them
    constexpr int kWAll = (MG ? 4 : 2) * kAPlane;
    const int agrp = MG ? group * 2 * kAPlane : 0;
    // the patch is staged by all threads of the workgroup
    constexpr int PTH = MG ? 512 : 256;
    const int ptid = MG ? (int)threadIdx.x : tid;
    const int wm = wave % WM, wn = wave / WM;
    const int lrow = lane & 31, lhalf = lane >> 5;

    const int H = a.H, W = a.W, HW = H * W, OHW = a.OH * a.OW;
    const int VH = H + 2;
    // 16-byte words per patch row, and where the odd columns start (stride 2 only)
    const int PWS = a.pws, PWH = PWS >> 1;
    const int stage_bytes = a.stage_bytes;

    // All index arithmetic divides through host-computed float reciprocals; the host admits
    // this kernel when every dividend stays below 2^22, where fast_div is exact.
    int m0, n0;
    {
        const int tile = xcd_remap(blockIdx.x, gridDim.x);
        int r;
        const int q = fast_div(tile, a.m_major ? a.ntiles : a.mtiles, a.inv_tdiv, &r);
        m0 = (a.m_major ? q : r) * (MG ? 2 * MT : MT) + (MG ? group * MT : 0);
        n0 = (a.m_major ? r : q) * NT;
    }

    // ---- weight task: one output channel, four input channels, all nine taps ----------------
    const int w_ocl = tid >> 2, w_quad = tid & 3;
    // rows past OC read row 0: their products land in accumulators that are never stored
    const uint32_t woff =
        2u * (uint32_t)((((m0 + w_ocl) < a.OC ? m0 + w_ocl : 0) * a.IC + w_quad * 4) * 9);
    // LDS byte addresses are kept per stage (index 0 / 1), so that the loop adds nothing to them
    int wbase[2];           // where tap 0 of the weight task goes
    wbase[0] = gbase + agrp + (w_quad >> 1) * kAPlane + w_ocl * 16 + (w_quad & 1) * 8;
    wbase[1] = wbase[0] + stage_bytes;

    uint32_t goff[PT];      // byte offset of a patch task's first channel within a chunk of x
    // UNAL: the same for the odd channels of the octet (one channel further, re-aligned), the
    // funnel shifts (0 or 16 bits) of the even and of the odd channels, and the task's dump words
    uint32_t goffo[UNAL ? PT : 1];
    int shift_e[UNAL ? PT : 1], shift_o[UNAL ? PT : 1], pwdump[2][UNAL ? PT : 1];
    int pwbase[2][PT];      // where the first pixel of a patch task goes
    int pwbase2[2][PT];     // stride 2: its second pixel (the even-column half of the row)
    // PX = 4: where pixels 2 and 3 go - behind the first pair, or, for the short last task of a
    // row of 4m + 2 pixels, to the dump area (its load then reads on into the next row)
    int pwtail[2][PX == 4 ? PT : 1], pwtail2[2][PX == 4 && STRIDE == 2 ? PT : 1];
    // two register sets: while one is transposed into LDS (chunk c+1) the other is still in
    // flight (chunk c+2), so a load has two chunks of MFMA time to arrive
    uint32_t praw[2][PT][NCH][PW32];
    uint32_t wraw[2][18];

    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(a.x), 0, a.x_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(a.w), 0, a.w_bytes, kRsrcFlags);
    const int hw2 = HW * 2;

    // The staging work of a chunk as a list of small items, so that it can be dealt out between
    // the MFMAs of an earlier chunk.  A register is reloaded right after the item that consumed
    // it (chunk c+1) - with chunk c+3, the other set holding chunk c+2:
    //   0..8    transpose filter tap i of the weights into the stage
    //   9..13   load the weight task's 72-byte run (4 x 16 bytes + 8 bytes)
    //   then per patch task: PX transposes (one pixel each), 8 loads (one channel each)
    // `set` = which register set the item works on = which stage a transpose writes to;
    // cbase = byte offset of the chunk to load within an image of x.
    constexpr int kItems = kP0 + PT * (PX + NCH);
    auto work_item = [&](int it, int set, bool do_pack, bool do_load, int c, int cbase) __attribute__((always_inline)) {
        if (it < 9) {
            if (!do_pack) return;
            const int tap = it;
            uint32_t o[2];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int e0 = (2 * q) * 9 + tap, e1 = (2 * q + 1) * 9 + tap;
                o[q] = pack_halves(wraw[set][e0 >> 1], e0 & 1, wraw[set][e1 >> 1], e1 & 1);
            }
            *reinterpret_cast<uint2v *>(smem + wbase[set] + tap * MT * 16) = uint2v{o[0], o[1]};
        } else if (it < kP0) {
            if (!do_load) return;
            // the task's run of 72 bytes starts 8-byte aligned: 16-byte loads need 4
            const int i = it - 9;
            if (i < 4) {
                const uint4v t4 = __builtin_bit_cast(
                    uint4v, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, woff + i * 16, (c * KG + kgroup) * kChunk * 9 * 2, 0));
#pragma unroll
                for (int d = 0; d < 4; ++d) wraw[set][4 * i + d] = t4[d];
            } else {
                const uint2v t2 = __builtin_bit_cast(
                    uint2v, __builtin_amdgcn_raw_buffer_load_b64(wrsrc, woff + 64, (c * KG + kgroup) * kChunk * 9 * 2, 0));
                wraw[set][16] = t2[0];
                wraw[set][17] = t2[1];
            }
        } else {
            const int j = (it - kP0) / (PX + NCH), r = (it - kP0) % (PX + NCH);
            if (r < PX) {
                if (!do_pack) return;
                const int k = r;
                if constexpr (UNAL) {
                    if (k == 0) {       // bring both channels' rows down to bit 0 of their registers
#pragma unroll
                        for (int q = 0; q < 2; ++q) {
                            const int sh = q ? shift_o[j] : shift_e[j];
#pragma unroll
                            for (int d = 0; d < 3; ++d)
                                praw[set][j][q][d] = __builtin_amdgcn_alignbit(praw[set][j][q][d + 1],
                                                                               praw[set][j][q][d], sh);
                            praw[set][j][q][3] >>= sh;
                        }
                    }
                    const uint32_t o2 = pack_halves(praw[set][j][0][k >> 1], k & 1,
                                                    praw[set][j][1][k >> 1], k & 1);
                    // (uniform test: the pixels past the row's end)
                    *reinterpret_cast<uint32_t *>(smem + (k < W ? pwbase[set][j] + k * 16
                                                                : pwdump[set][j] + k * 256)) = o2;
                    return;
                }
                uint32_t o[4];
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    o[q] = pack_halves(praw[set][j][2 * q][k >> 1], k & 1,
                                       praw[set][j][2 * q + 1][k >> 1], k & 1);
                // consecutive words; for stride 2 alternately the odd- and the even-column half
                unsigned char *dst = STRIDE == 2 ? smem + ((k & 1) ? pwbase2[set][j] : pwbase[set][j]) + (k >> 1) * 16
                                                 : smem + pwbase[set][j] + k * 16;
                if constexpr (PX == 4) {
                    if (k >= 2)
                        dst = STRIDE == 2 ? smem + (k == 3 ? pwtail2[set][j] : pwtail[set][j])
                                          : smem + pwtail[set][j] + (k - 2) * 16;
                }
                *reinterpret_cast<uint4v *>(dst) = uint4v{o[0], o[1], o[2], o[3]};
            } else {
                if (!do_load) return;
                const int q = r - PX;
                const int soff = cbase + q * hw2;
                if constexpr (UNAL) {
                    // the odd channel: its channel stride is part of its (re-aligned) lane offset
                    const uint4v t4 = __builtin_bit_cast(
                        uint4v, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, q ? goffo[j] : goff[j], cbase, 0));
#pragma unroll
                    for (int d = 0; d < 4; ++d) praw[set][j][q][d] = t4[d];
                } else if constexpr (PX == 8) {
                    const uint4v t4 = __builtin_bit_cast(
                        uint4v, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, goff[j], soff, 0));
#pragma unroll
                    for (int d = 0; d < 4; ++d) praw[set][j][q][d] = t4[d];
                } else if constexpr (PX == 4) {
                    const uint2v t2 = __builtin_bit_cast(
                        uint2v, __builtin_amdgcn_raw_buffer_load_b64(xrsrc, goff[j], soff, 0));
                    praw[set][j][q][0] = t2[0];
                    praw[set][j][q][1] = t2[1];
                } else if constexpr (PX == 2) {
                    praw[set][j][q][0] = __builtin_amdgcn_raw_buffer_load_b32(xrsrc, goff[j], soff, 0);
                } else {
                    praw[set][j][q][0] = __builtin_amdgcn_raw_buffer_load_b16(xrsrc, goff[j], soff, 0);
                }
            }
        }
    };
    auto all_items = [&](int first, int last, int set, bool do_pack, bool do_load, int c) __attribute__((always_inline)) {
        const int cbase = (c * KG + kgroup) * kChunk * hw2;
#pragma unroll
        for (int it = first; it < last; ++it) work_item(it, set, do_pack, do_load, c, cbase);
    };

    // The first chunk's loads go out as early as their addresses are known - the weights
    // first, they need no geometry - and the rest of the set-up runs under their latency.
    all_items(9, kP0, 0, false, true, 0);
    // likewise the tile's per-channel multiplier and offset, needed only by the fused tail
    float ss_scale = 0.0f, ss_shift = 0.0f, ss_bias = 0.0f;
    if ((MG || group == 0) && tid < MT && m0 + tid < a.OC) {
        ss_scale = a.scale[m0 + tid];
        ss_shift = a.shift[m0 + tid];
        if (a.bias) ss_bias = a.bias[m0 + tid];
    }

    // ---- tile geometry (uniform values) ----------------------------------------------------
    int vr_lo, nrows, na;
    {
        const int p_last = min(n0 + NT, a.npix) - 1;
        int ra, rb, t;
        na = fast_div(n0, OHW, a.inv_ohw, &ra);
        const int oha = fast_div(ra, a.OW, a.inv_ow, &t);
        const int nb = fast_div(p_last, OHW, a.inv_ohw, &rb), ohb = fast_div(rb, a.OW, a.inv_ow, &t);
        vr_lo = na * VH + oha * STRIDE;
        nrows = nb * VH + ohb * STRIDE + 2 - vr_lo + 1;
    }

    // ---- per-thread patch load tasks: (virtual row, iw, channel octet), fixed for all chunks
    {
        const int WPX = (W + PX - 1) / PX;       // (PX = 4 also serves rows of 4m + 2 pixels)
        const int per_octet = nrows * WPX;
        // second pixel of a stride-2 task: first pixel in an odd padded column, the second in
        // the following even column
        const int pair_step = 16 - PWH * 16;
#pragma unroll
        for (int j = 0; j < PT; ++j) {
            // (UNAL: four tasks per row and octet, one per pair of channels)
            const int pair = UNAL ? (tid & 3) : 0;
            const int t = UNAL ? (tid + j * 256) >> 2 : ptid + j * PTH;
            const int octet = t >= per_octet;
            const int rem = t - (octet ? per_octet : 0);
            int iw, vi;
            const int vrow = fast_div(rem, WPX, a.inv_wpx, &iw);
            iw *= PX;
            const int n = fast_div(vr_lo + vrow, VH, a.inv_vh, &vi);
            const int ih = vi - 1;
            const bool live = t < 2 * per_octet && ih >= 0 && ih < H && n < a.N;
            const int col = iw + 1;
            const int word = STRIDE == 2 ? (col & 1) * PWH + (col >> 1) : col;
            // tasks with nothing to fetch (padding rows, past the tile) load element 0 and
            // write it to a dump area behind the planes, so that no store needs a predicate
            goff[j] = live ? 2u * (uint32_t)((n * a.IC + octet * 8) * HW + ih * W + iw) : 0u;
            if constexpr (UNAL) {
                // element offsets of the row in the pair's even and odd channel; each load
                // starts at the 4-byte boundary at or below its row
                const uint32_t ee = live ? (uint32_t)((n * a.IC + octet * 8 + pair * 2) * HW + ih * W) : 0u;
                const uint32_t eo = ee + (uint32_t)HW;
                shift_e[j] = (int)(ee & 1u) * 16;
                shift_o[j] = (int)(eo & 1u) * 16;
                goff[j] = 2u * (ee & ~1u);
                goffo[j] = 2u * (eo & ~1u);
            }
            pwbase[0][j] = gbase +
                           (live ? kWAll + octet * a.pplane + (vrow * PWS + word) * 16 + (n - na) * a.xp16
                                 : kWAll + 2 * a.pplane + (tid & 15) * (PX > 1 ? PX * 16 : 32) +
                                       (STRIDE == 2 && PX > 1 ? 16 - pair_step : 0));
            if constexpr (UNAL) pwbase[0][j] += pair * 4;     // the pair's 4 bytes of a pixel's word
            pwbase[1][j] = pwbase[0][j] + stage_bytes;
            if constexpr (UNAL) {
                // (64 lanes write 256 consecutive bytes: conflict-free)
                pwdump[0][j] = gbase + kWAll + 2 * a.pplane + (tid & 63) * 4;
                pwdump[1][j] = pwdump[0][j] + stage_bytes;
            }
            pwbase2[0][j] = pwbase[0][j] + pair_step;
            pwbase2[1][j] = pwbase[1][j] + pair_step;
            if constexpr (PX == 4) {
                const bool whole = !live || iw + 4 <= W;
                const int dump = gbase + kWAll + 2 * a.pplane + (tid & 15) * 64;
                pwtail[0][j] = whole ? pwbase[0][j] + (STRIDE == 2 ? 16 : 32) : dump + 32;
                pwtail[1][j] = pwtail[0][j] + stage_bytes;
                if constexpr (STRIDE == 2) {
                    pwtail2[0][j] = whole ? pwbase2[0][j] + 16 : dump + 48;
                    pwtail2[1][j] = pwtail2[0][j] + stage_bytes;
                }
            }
        }
    }
    all_items(kP0, kItems, 0, false, true, 0);
    // The second chunk goes into the other register set (the channel count is a multiple of
    // 32).  A vector memory instruction takes the address unit some 60 cycles, and a wave issues
    // in order: its loads are dealt out between the pieces of set-up arithmetic that follow,
    // which would otherwise wait behind them.
    constexpr int kSecond = kItems - 9;            // items 9 .. kItems-1 (transposes are skipped)
    auto second_chunk_loads = [&](int part, int parts) __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
        all_items(9 + part * kSecond / parts, 9 + (part + 1) * kSecond / parts, 1, false, true, 1);
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- per-lane addresses of the MFMA operands --------------------------------------------
    // pixel operand: the word of filter row 0, column 0 of pixel block j in this lane's octet
    // plane of stage 0; stage, filter row (uniform values) and column (an immediate) are added
    // at the read - one vector add per read is free, a register per combination is not
    int bpix[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        if (j < 4) second_chunk_loads(j, NJ < 4 ? NJ + 2 : 6);
        const int p = n0 + wn * WTN + j * 32 + lrow;
        int rem, ow;
        const int n = fast_div(p, OHW, a.inv_ohw, &rem);
        const int oh = fast_div(rem, a.OW, a.inv_ow, &ow);
        bpix[j] = gbase + kWAll + lhalf * a.pplane +
                  (p < a.npix ? ((n * VH + oh * STRIDE - vr_lo) * PWS + ow) * 16 + (n - na) * a.xp16 : 0);
    }
    int abase[2];
    abase[0] = gbase + agrp + lhalf * kAPlane + (wm * WTM + lrow) * 16;
    abase[1] = abase[0] + stage_bytes;
    second_chunk_loads(NJ < 4 ? NJ : 4, NJ < 4 ? NJ + 2 : 6);

    float *ss_lds = reinterpret_cast<float *>(smem + a.ss_offset);

    float16v acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    second_chunk_loads(NJ < 4 ? NJ + 1 : 5, NJ < 4 ? NJ + 2 : 6);

    const int nchunks = a.IC / (kChunk * KG);     // chunks of this group
    // zero the patch planes of both stages once (padding rows and columns are never written
    // again) and stage the tile's (scale, offset) pairs
    {
        const int words = 2 * a.pplane / 16;
        for (int s = 0; s < 2; ++s) {
            uint4v *pz = reinterpret_cast<uint4v *>(smem + gbase + s * stage_bytes + kWAll);
            for (int i = ptid; i < words; i += PTH) pz[i] = uint4v{0u, 0u, 0u, 0u};
        }
    }
    if constexpr (MG) ss_lds += group * 2 * MT;          // each group's 64 channels
    if ((MG || group == 0) && tid < MT) {
        // (acc + bias)*scale + shift == acc*scale + (bias*scale + shift)
        ss_lds[2 * tid] = ss_scale;
        ss_lds[2 * tid + 1] = fmaf(ss_bias, ss_scale, ss_shift);
    }
    __syncthreads();          // zeroing complete before the first real data lands
    all_items(0, kItems, 0, true, nchunks > 2, 2);
    __syncthreads();

    // MFMA operands are requested from LDS ahead of their use: the weight operands of tap t+1
    // before the MFMAs of tap t, the pixel operands (one per 32-pixel block and tap, in the
    // order of use) kAhead operands ahead through a ring of registers.
    constexpr int kAhead = 4, kRing = kAhead + 1, kSeq = 9 * NJ;
    uint4v af[2][MI], bfr[kRing];
    auto fetch_a = [&](int st, int tap, int slot) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
            af[slot][i] = *reinterpret_cast<const uint4v *>(smem + abase[st] + (tap * MT + i * 32) * 16);
    };
    // q = tap * NJ + block; rowoff[r] = stage offset + filter row r (uniform)
    auto fetch_b = [&](const int (&rowoff)[3], int q) __attribute__((always_inline)) {
        const int tap = q / NJ, j = q % NJ, r = tap / 3, s = tap - r * 3;
        bfr[q % kRing] = *reinterpret_cast<const uint4v *>(
            smem + bpix[j] + rowoff[r] + (STRIDE == 2 ? (s & 1) * PWH * 16 + (s >> 1) * 16 : s * 16));
    };
    // One filter tap of chunk c (stage PAR): request later operands, then this tap's MFMAs, each
    // followed by its share of the staging items of chunks c+1 (transposes into the other
    // stage) and c+3 (loads into the registers just transposed): a few byte permutes and an LDS
    // store, or a few loads, which issue while the MFMA runs.  The order written here is kept:
    // the fences stop the compiler from regrouping it.
    // MODE 2 = transposes and loads, 1 = transposes only, 0 = neither.
    auto tap_step = [&](auto tapc, auto modec, auto parc, const int (&rowoff)[3], int cl, int cbase) __attribute__((always_inline)) {
        constexpr int tap = decltype(tapc)::value;
        constexpr int mode = decltype(modec)::value;
        constexpr int par = decltype(parc)::value;
        constexpr int nm = MI * NJ;
        if constexpr (tap + 1 < 9) fetch_a(par, tap + 1, (tap + 1) & 1);
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int q = tap * NJ + j;
            if (q + kAhead < kSeq) fetch_b(rowoff, q + kAhead);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                // pixel operand first: the accumulator tile is D[pixel][channel]
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8v, bfr[q % kRing]),
                    __builtin_bit_cast(bf16x8v, af[tap & 1][i]), acc[i][j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (mode > 0) {
                    const int g = tap * nm + j * MI + i;
#pragma unroll
                    for (int it = g * kItems / (9 * nm); it < (g + 1) * kItems / (9 * nm); ++it)
                        work_item(it, par ^ 1, true, mode == 2, cl, cbase);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    };
    // Chunk c of parity PAR reads stage PAR, transposes register set PAR^1 (chunk c+1) into
    // stage PAR^1 and reloads that set with chunk c+3.
    auto chunk = [&](auto parc, auto modec, int c) __attribute__((always_inline)) {
        constexpr int par = decltype(parc)::value;
        constexpr int mode = decltype(modec)::value;
        const int cbase = ((c + 3) * KG + kgroup) * kChunk * hw2;
        // (hidden from loop-invariant code motion, which would spend a register per
        // combination of stage, filter row and pixel block on precomputed addresses)
        int so = par * stage_bytes;
        asm volatile("" : "+s"(so));
        const int rowoff[3] = {so, so + PWS * 16, so + 2 * PWS * 16};
        fetch_a(par, 0, 0);
#pragma unroll
        for (int q = 0; q < kAhead && q < kSeq; ++q) fetch_b(rowoff, q);
        // The set to transpose was loaded two chunks ago; only the other set's loads (issued
        // during the previous chunk) may still be in flight.  One wait instead of one per
        // register.  (Where fewer loads are pending, the compiler's own waits take over.)
        if constexpr (mode > 0) __builtin_amdgcn_s_waitcnt(waitcnt_imm(kLoads, 15));
        tap_step(std::integral_constant<int, 0>{}, modec, parc, rowoff, c + 3, cbase);
        tap_step(std::integral_constant<int, 1>{}, modec, parc, rowoff, c + 3, cbase);
        tap_step(std::integral_constant<int, 2>{}, modec, parc, rowoff, c + 3, cbase);
        tap_step(std::integral_constant<int, 3>{}, modec, parc, rowoff, c + 3, cbase);
        tap_step(std::integral_constant<int, 4>{}, modec, parc, rowoff, c + 3, cbase);
        tap_step(std::integral_constant<int, 5>{}, modec, parc, rowoff, c + 3, cbase);
        tap_step(std::integral_constant<int, 6>{}, modec, parc, rowoff, c + 3, cbase);
        tap_step(std::integral_constant<int, 7>{}, modec, parc, rowoff, c + 3, cbase);
        tap_step(std::integral_constant<int, 8>{}, modec, parc, rowoff, c + 3, cbase);
        if constexpr (mode > 0) __syncthreads();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using M0 = std::integral_constant<int, 0>;
    using M1 = std::integral_constant<int, 1>;
    using M2 = std::integral_constant<int, 2>;
    // steady state in pairs (the chunk count is even), then the last four or two chunks, which
    // have less and finally nothing left to stage
    int c = 0;
    for (; c + 4 < nchunks; c += 2) {
        chunk(P0{}, M2{}, c);
        chunk(P1{}, M2{}, c + 1);
    }
    if (c + 4 == nchunks) {
        chunk(P0{}, M2{}, c);
        chunk(P1{}, M1{}, c + 1);
        c += 2;
    }
    chunk(P0{}, M1{}, c);
    chunk(P1{}, M0{}, c + 1);

    // ---- fused tail: per-wave staging in LDS, vector stores --------------------------------
    __syncthreads();                       // every wave is done reading the operand tiles
    const TailArgs tail{a.scale, a.shift, a.bias, a.residual, a.y, a.OC, OHW, a.npix, a.relu};
    if constexpr (KG == 1) {
        constexpr int BT = MI * NJ < 4 ? MI * NJ : 4;                 // tiles staged at a time
        // (four waves: <= 40 KB < two stages; MG: eight waves, the host sizes the LDS for them)
        unsigned char *stage = smem + ((MG ? group * 4 : 0) + wave) * (BT * kStageBytes);
        store_acc_tiles_batched<MI, NJ, BT>(acc, stage, lane, m0 + wm * WTM, n0 + wn * WTN, tail,
                                            a.vmode, ss_lds, wm * WTM);
    } else {
        // The two groups hold partial sums of the same tile.  Group g finishes pixel block g of
        // every wave tile: it hands its partial sums of the other block to its partner wave
        // through LDS (16-byte words, lane-contiguous: conflict-free) and adds what it receives.
        static_assert(NJ == 2, "the split-reduction variant halves a wave tile of two pixel blocks");
        constexpr int kXWave = MI * 16 * 64 * 4;                  // bytes a wave hands over
        float4v *xout = reinterpret_cast<float4v *>(smem + (wave * 2 + group) * kXWave);
        const float4v *xin = reinterpret_cast<const float4v *>(smem + (wave * 2 + (group ^ 1)) * kXWave);
        auto hand_over = [&](auto jc) __attribute__((always_inline)) {
            constexpr int js = decltype(jc)::value;               // the block this group gives away
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    xout[(i * 4 + q) * 64 + lane] = float4v{acc[i][js][4 * q], acc[i][js][4 * q + 1],
                                                            acc[i][js][4 * q + 2], acc[i][js][4 * q + 3]};
        };
        if (group == 0) hand_over(std::integral_constant<int, 1>{});
        else hand_over(std::integral_constant<int, 0>{});
        __syncthreads();
        float16v mine[MI][1];
        auto take_in = [&](auto jc) __attribute__((always_inline)) {
            constexpr int jk = decltype(jc)::value;               // the block this group keeps
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4v o = xin[(i * 4 + q) * 64 + lane];
#pragma unroll
                    for (int e = 0; e < 4; ++e) mine[i][0][4 * q + e] = acc[i][jk][4 * q + e] + o[e];
                }
        };
        if (group == 0) take_in(std::integral_constant<int, 0>{});
        else take_in(std::integral_constant<int, 1>{});
        // the staging areas of the tail lie behind the exchange area (a wave may still be
        // reading its partner's sums while another has started to store)
        constexpr int BT = MI;
        unsigned char *stage = smem + 8 * kXWave + (wave * 2 + group) * (BT * kStageBytes);
        store_acc_tiles_batched<MI, 1, BT>(mine, stage, lane, m0 + wm * WTM,
                                           n0 + wn * WTN + group * 32, tail, a.vmode, ss_lds, wm * WTM);
    }
}

template <int WM, int NJ, int STRIDE, int PT, int PX, int KG = 1, bool UNAL = false, bool MG = false>
tvg_status launch_instance(const DbufArgs &a, size_t lds, hipStream_t stream)
{
    auto kernel = conv3x3_dbuf_kernel<WM, NJ, STRIDE, PT, PX, KG, UNAL, MG>;
    static bool configured = false;      // opt in to > 64 KB of dynamic LDS once per instance
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return TVG_ERR_LAUNCH;
        configured = true;
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)(a.mtiles * a.ntiles)), dim3(256 * (MG ? 2 : KG)), lds, stream, a);
    return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
}

// The split-reduction variant (two groups of four waves): stride 1, wave tiles of two pixel blocks.
template <int WM, int NJ>
tvg_status launch_pt_kg2(const DbufArgs &a, size_t lds, int pt, int px, hipStream_t stream)
{
    if constexpr (NJ == 2) {
        if (px == 8 && a.W < 8) {
            if (pt <= 1) return launch_instance<WM, NJ, 1, 1, 8, 2, true>(a, lds, stream);
            return launch_instance<WM, NJ, 1, 2, 8, 2, true>(a, lds, stream);
        }
        switch (px) {
        case 8: return launch_instance<WM, NJ, 1, 1, 8, 2>(a, lds, stream);
        case 4:
            if (pt <= 1) return launch_instance<WM, NJ, 1, 1, 4, 2>(a, lds, stream);
            return launch_instance<WM, NJ, 1, 2, 4, 2>(a, lds, stream);
        case 2:
            if (pt <= 2) return launch_instance<WM, NJ, 1, 2, 2, 2>(a, lds, stream);
            return launch_instance<WM, NJ, 1, 4, 2, 2>(a, lds, stream);
        default:
            if (pt <= 2) return launch_instance<WM, NJ, 1, 2, 1, 2>(a, lds, stream);
            return launch_instance<WM, NJ, 1, 4, 1, 2>(a, lds, stream);
        }
    }
    return TVG_ERR_UNSUPPORTED;
}

// The channel-split variant (two groups of four waves, 128 output channels): wave tiles of two
// pixel blocks, aligned rows, one or two patch tasks per thread.
template <int WM, int NJ>
tvg_status launch_pt_mg(const DbufArgs &a, size_t lds, int stride, int pt, int px, hipStream_t stream)
{
    if constexpr (NJ == 2) {
        if (pt > 2) return TVG_ERR_UNSUPPORTED;
#define TVG_MG(S_, PX_)                                                                              \
    (pt <= 1 ? launch_instance<WM, NJ, S_, 1, PX_, 1, false, true>(a, lds, stream)                    \
             : launch_instance<WM, NJ, S_, 2, PX_, 1, false, true>(a, lds, stream))
        // (the host admits 16-byte loads with one task per thread only: registers)
        if (px == 8 && pt > 1) return TVG_ERR_UNSUPPORTED;
        if (stride == 2) {
            if (px == 8) return launch_instance<WM, NJ, 2, 1, 8, 1, false, true>(a, lds, stream);
            if (px == 4) return TVG_MG(2, 4);
            if (px == 2) return TVG_MG(2, 2);
            return TVG_ERR_UNSUPPORTED;
        }
        switch (px) {
        case 8: return launch_instance<WM, NJ, 1, 1, 8, 1, false, true>(a, lds, stream);
        case 4: return TVG_MG(1, 4);
        case 2: return TVG_MG(1, 2);
        default: return TVG_MG(1, 1);
        }
#undef TVG_MG
    }
    return TVG_ERR_UNSUPPORTED;
}

template <int WM, int NJ>
tvg_status launch_pt(const DbufArgs &a, size_t lds, int stride, int pt, int px, int kg,
                     hipStream_t stream)
{
    if (kg == 3) return launch_pt_mg<WM, NJ>(a, lds, stride, pt, px, stream);
    if (kg == 2) return stride == 1 ? launch_pt_kg2<WM, NJ>(a, lds, pt, px, stream) : TVG_ERR_UNSUPPORTED;
    if (stride == 2) {
        // instances exist for the 128- and 256-pixel tiles and even rows (see the plan)
        if constexpr (NJ == 2 || (WM == 1 && NJ == 1)) {
            if (px == 8) return launch_instance<WM, NJ, 2, 1, 8>(a, lds, stream);
            if (px == 4) {
                if (pt <= 1) return launch_instance<WM, NJ, 2, 1, 4>(a, lds, stream);
                return launch_instance<WM, NJ, 2, 2, 4>(a, lds, stream);
            }
            if (px == 2) {
                if (pt <= 2) return launch_instance<WM, NJ, 2, 2, 2>(a, lds, stream);
                return launch_instance<WM, NJ, 2, 4, 2>(a, lds, stream);
            }
        }
        return TVG_ERR_UNSUPPORTED;
    }
    if (px == 8 && a.W < 8) {
        if (pt <= 1) return launch_instance<WM, NJ, 1, 1, 8, 1, true>(a, lds, stream);
        return launch_instance<WM, NJ, 1, 2, 8, 1, true>(a, lds, stream);
    }
    switch (px) {
    case 8: return launch_instance<WM, NJ, 1, 1, 8>(a, lds, stream);
    case 4:
        if (pt <= 1) return launch_instance<WM, NJ, 1, 1, 4>(a, lds, stream);
        return launch_instance<WM, NJ, 1, 2, 4>(a, lds, stream);
    case 2:
        if (pt <= 2) return launch_instance<WM, NJ, 1, 2, 2>(a, lds, stream);
        return launch_instance<WM, NJ, 1, 4, 2>(a, lds, stream);
    default:
        if (pt <= 2) return launch_instance<WM, NJ, 1, 2, 1>(a, lds, stream);
        return launch_instance<WM, NJ, 1, 4, 1>(a, lds, stream);
    }
}

}  // namespace

// Fills the double-buffered fields of a plan whose mt/nt/rows are set; false if the two
// stages do not fit or the tile shape has no instance.
bool plan_conv3x3_dbuf(const ConvProblem &p, Patch3x3Plan *plan)
{
    // 128-channel tiles: the channel-split variant (two wave groups, one workgroup per CU)
    const bool mg = plan->mt == 2 * kMT;
    if (plan->mt != kMT && !mg) return false;
    // Measured at batch 64: C6 21.4 us against 21.7 with 64 x 256 tiles, C7 18.7 against 18.9 in the
    // single-stage kernel, C10 30.0 against 21.7 (100 workgroups instead of 200) - the operand reads
    // of a 32 x 64 or 64 x 64 wave tile keep the LDS as busy as before, whoever stages the patch.
    // Not a rule, then: the variant runs where a caller names it (tile 128 x nt, two stages).
    if (mg && (plan->want_stages != 2 || plan->tiles > kComputeUnits || plan->nt < 128 || p.OC <= kMT))
        return false;
    if (p.IC % (2 * kChunk) != 0) return false;      // the chunk loop runs in pairs
    // Measured at batch 64: with fewer than eight chunks the deeper pipeline's longer start-up
    // (three chunks in flight before the first MFMA) costs more than the loop gains.  (A caller
    // that asks for this kernel by name gets it from four chunks on.)
    if (p.IC < (plan->want_stages == 2 ? 4 : 8) * kChunk || plan->nt > 256) return false;
    // Stride 2: a patch is four times the output tile, so its two stages fill the LDS of a CU
    // and the kernel pays only where one workgroup per CU covers the problem (instances: the
    // 128- and 256-pixel tiles, even rows).
    if (p.sh == 2 && (plan->nt < 128 || p.W % 2 != 0 || plan->tiles > kComputeUnits)) return false;
    // Row pitch of the patch planes.  The 16 lanes of one LDS access read the words of 16
    // consecutive pixels; they are conflict-free when those words are consecutive modulo 16,
    // also across the end of an image row and of an image.  Stride 1: a pitch of W + 16 words
    // makes the step at a row end 1 (mod 16), and xp extra words between images do the same
    // for the step from an image's last pixel to the next image's first.  Stride 1 keeps the
    // plain pitch when the padded planes would cost the second workgroup per CU.
    // Stride 2: the 16 lanes of an access read word (output row * 4 * pwh + output column) of one
    // column half, so the step at the end of an output row is 4 * pwh - OW words; up to three
    // spare words per half row are added where they make more of those 16 words fall into
    // different banks (counted over the first four groups of 16 pixels of an image).
    int pwh = (p.W + 3) / 2;
    if (p.sh == 2 && plan->want_pitch != 1) {
        int best_d = 0, best_n = -1;
        for (int d = 0; d < 4; ++d) {
            int distinct = 0;
            for (int g = 0; g < 4; ++g) {
                unsigned seen = 0;
                for (int l = 0; l < 16; ++l) {
                    const int pix = g * 16 + l, row = pix / p.OW, col = pix % p.OW;
                    seen |= 1u << ((row * 4 * (pwh + d) + col) & 15);
                }
                distinct += __builtin_popcount(seen);
            }
            if (distinct > best_n) { best_n = distinct; best_d = d; }
        }
        pwh += best_d;
    }
    const int images = (plan->nt - 1) / (p.OH * p.OW) + 1;     // image ends a tile can span
    int pws = p.sh == 2 ? 2 * pwh : p.W + 16;
    int xp = p.sh == 2 ? 0 : ((p.H * p.W - (p.H + 2) * pws) % 16 + 16) % 16;
    int pplane = (plan->rows * pws + images * xp) * 16;
    // the widest load that divides a row (and an image plane: every row then starts aligned)
    // (rows of 4m + 2 pixels take 8-byte loads too, 4-byte aligned, the last one of a row short)
    // (odd rows of at most 7 pixels, stride 1, one task per thread: whole rows by one 16-byte load
    // from the aligned address below the row's start, see the kernel's UNAL)
    int px = p.W % 8 == 0 ? 8 : p.W % 4 == 0 ? 4 : p.W % 2 != 0 ? 1 : p.W >= 6 ? 4 : 2;
    // (C12 at batch 64, found by the knob search: whole rows + one wave group + padded pitch 23.1 us;
    // element loads + two wave groups 25.9; element loads + one group 28.1; whole rows with the
    // plain pitch 28.1 - the 4-byte stores of a row's pieces then collide)
    const bool odd_rows = px == 1;
    const bool unal = px == 1 && p.W <= 7 && p.sh == 1 && 8 * plan->rows <= 512 && plan->want_rows != 1 && !mg;
    if (unal) px = 8;
    // (unaligned rows: four tasks per row and octet, each two channels)
    const int pth = mg ? 512 : 256;                   // threads that share the patch tasks
    const int pt = unal ? (8 * plan->rows + 255) / 256
                        : (2 * plan->rows * ((p.W + px - 1) / px) + pth - 1) / pth;
    if (!unal && pt * (px >= 2 ? px / 2 : 1) > 4) return false;       // registers of a task's loads
    if (mg && pt > 2) return false;                                    // instances built
    // behind the planes of a stage: 32 bytes for each of 16 lanes, where idle patch tasks store
    // (a stride-2 pair stores its two pixels pwh - 1 words apart)
    const int dump = 16 * (px > 1 ? px * 16 : 32) + (p.sh == 2 ? pwh * 16 : 0);
    const int wplanes = (mg ? 4 : 2) * kAPlane;
    const size_t ss_bytes = (size_t)plan->mt * 8;
    // (the tail's staging areas, one per wave, reuse the stages; eight waves need 80 KB)
    const size_t tail_bytes = mg ? (size_t)8 * 4 * kStageBytes : 0;
    int stage = wplanes + 2 * pplane + dump;
    size_t lds = std::max(2 * (size_t)stage, tail_bytes) + ss_bytes;
    // (a grid of at most one workgroup per CU may take the whole LDS for the conflict-free pitch:
    // C9 20.9 -> 19.7 us)
    const bool lone = plan->tiles <= kComputeUnits;
    if (p.sh == 1 && (plan->want_pitch == 1 ||
                      (plan->want_pitch == 0 && lds > (size_t)(lone ? 160 : 80) * 1024))) {
        pws = p.W + 2;
        xp = 0;
        pplane = plan->rows * pws * 16;
        stage = wplanes + 2 * pplane + dump;
        lds = std::max(2 * (size_t)stage, tail_bytes) + ss_bytes;
    }
    // Grids of at most one workgroup per CU (stride 1, wave tiles of two pixel blocks, whole
    // pairs of chunks for each half of the reduction): two groups of four waves split the
    // reduction, each with two stages of its own.  Four stages must fit; the conflict-free
    // pitch is given up for the plain one if that is what it takes.  After the loop the same
    // memory holds the accumulators the groups exchange and the staging areas of the tail.
    int kg = 1;
    // Rule (measured at batch 64, warm): it pays where the rows are odd and fetched element by
    // element (C12: 28.1 -> 25.6 us), it loses on C9 (20.9 -> 21.4 us, and the four stages cost C9
    // the conflict-free pitch: 19.7 us with it); tvg_conv2d_set_knobs overrides the rule.
    const bool kg_rule = plan->want_kg == 2 || (plan->want_kg == 0 && odd_rows && !unal);
    if (!mg && p.sh == 1 && plan->tiles <= kComputeUnits && plan->nt >= 128 && p.IC % (4 * kChunk) == 0 &&
        p.IC >= 8 * kChunk && kg_rule) {
        const int mi = plan->nt == 256 ? 2 : 1;
        const size_t after = (size_t)8 * mi * 4096 + (size_t)8 * mi * kStageBytes;
        auto fits = [&](int st) { return 4 * (size_t)st + (size_t)kMT * 8 <= 160 * 1024; };
        if (!fits(stage) && plan->want_pitch != 2) {
            const int pws2 = p.W + 2, pplane2 = plan->rows * pws2 * 16;
            const int stage2 = 2 * kAPlane + 2 * pplane2 + dump;
            if (fits(stage2)) { pws = pws2; xp = 0; pplane = pplane2; stage = stage2; }
        }
        if (fits(stage)) {
            kg = 2;
            lds = 4 * (size_t)stage;
            if (lds < after) lds = after;
            lds += (size_t)kMT * 8;
        }
    }
    // two workgroups per CU, or one per CU when the whole grid is resident at once anyway
    if (kg == 1 && lds > 80 * 1024 && !(lds <= 160 * 1024 && plan->tiles <= kComputeUnits)) return false;
    if (plan->tiles >= (1 << 22)) return false;      // fast_div range of the tile index
    if (mg) kg = 3;                                   // (the launch's name for the channel split)
    plan->kg = kg;
    plan->dbuf = 1;
    plan->pt = pt;
    plan->px = px;
    plan->pplane = pplane;
    plan->pws = pws;
    plan->xp16 = xp * 16;
    plan->stage_bytes = stage;
    plan->lds_bytes = lds;
    return true;
}

tvg_status launch_conv3x3_dbuf(const ConvProblem &p, const Patch3x3Plan &plan,
                               const ConvPointers &ptr, hipStream_t stream)
{
    DbufArgs a;
    a.x = static_cast<const bf16_t *>(ptr.x); a.w = static_cast<const bf16_t *>(ptr.w);
    a.scale = ptr.scale; a.shift = ptr.shift; a.bias = ptr.bias;
    a.residual = static_cast<const bf16_t *>(ptr.residual); a.y = static_cast<bf16_t *>(ptr.y);
    a.N = p.N; a.IC = p.IC; a.H = p.H; a.W = p.W; a.OC = p.OC; a.OH = p.OH; a.OW = p.OW;
    a.npix = p.npix; a.relu = p.relu | (p.stream_out << 1);
    a.mtiles = (p.OC + plan.mt - 1) / plan.mt;
    a.vmode = pick_store_vmode(p.dtype, p.OH * p.OW, ptr.y, ptr.residual);
    a.pplane = plan.pplane;
    a.pws = plan.pws;
    a.xp16 = plan.xp16;
    a.stage_bytes = plan.stage_bytes;
    a.ss_offset = (int)(plan.lds_bytes - (size_t)plan.mt * 8);
    a.x_bytes = (uint32_t)((size_t)p.N * p.IC * p.H * p.W * 2);
    a.w_bytes = (uint32_t)((size_t)p.OC * p.IC * 9 * 2);
    a.ntiles = (p.npix + plan.nt - 1) / plan.nt;
    a.m_major = (size_t)p.OC * p.IC * 9 > (size_t)p.N * p.IC * p.H * p.W;
    a.inv_tdiv = 1.0f / (float)(a.m_major ? a.ntiles : a.mtiles);
    a.inv_ohw = 1.0f / (float)(p.OH * p.OW);
    a.inv_ow = 1.0f / (float)p.OW;
    a.inv_vh = 1.0f / (float)(p.H + 2);
    a.inv_wpx = 1.0f / (float)((p.W + plan.px - 1) / plan.px);
    switch (plan.nt) {
    case 256: return launch_pt<1, 2>(a, plan.lds_bytes, p.sh, plan.pt, plan.px, plan.kg, stream);
    case 128:
        // one group of four waves: side by side, each all 64 channels x 32 pixels - two weight
        // reads and one pixel read per pair of MFMAs instead of one and two (the weight reads never
        // collide, the pixel reads of short or strided rows do): C12 23.1 -> 22.4 us, C10 21.7 ->
        // 20.6 us at batch 64, the 256-channel 14x14 layer at batch 32 16.0 -> 15.5 us
        if (p.sh == 1 && plan.kg == 1 && plan.px == 8 && p.W < 8 && plan.pt <= 1)
            return launch_instance<1, 1, 1, 1, 8, 1, true>(a, plan.lds_bytes, stream);
        if (plan.kg == 1)
            return launch_pt<1, 1>(a, plan.lds_bytes, p.sh, plan.pt, plan.px, plan.kg, stream);
        return launch_pt<2, 2>(a, plan.lds_bytes, p.sh, plan.pt, plan.px, plan.kg, stream);
    default: return launch_pt<2, 1>(a, plan.lds_bytes, p.sh, plan.pt, plan.px, plan.kg, stream);
    }
}

}  // namespace tvg
