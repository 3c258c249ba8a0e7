// Winograd F(2x2, 3x3) path with pre-transformed weights for bf16 3x3 stride-1 pad-1 convolutions
// (TVM paper, Section 6.1: the "TVM PT" variant of the GPU per-operator benchmark, "pre-transformed
// Winograd" convolution).  A 2x2 block of outputs is computed from a 4x4 block of inputs with 16
// multiplications per input channel instead of 36:
//     Y = A^T [ sum_ic (G g G^T) .* (B^T d B) ] A
//     B^T = | 1  0 -1  0 |   G = | 1    0    0  |   A^T = | 1  1  1  0 |
//           | 0  1  1  0 |       | 1/2  1/2  1/2|         | 0  1 -1 -1 |
//           | 0 -1  1  0 |       | 1/2 -1/2  1/2|
//           | 0  1  0 -1 |       | 0    0    1  |
// (the minimal filtering algorithm F(2,3) nested in both directions; correlation, no filter flip).
//
// Three kernels:
//   wino_weight_kernel   once per weight tensor (tvg_conv2d_prepack): U = G g G^T in fp32, stored as
//                        fp16 in the layout the contraction reads, [16 positions][IC/8][OC][8].
//   wino_input_kernel    per call: V = B^T d B for every 4x4 input block (tile) and channel, fp16,
//                        [16 positions][IC/8][tiles][8] in the caller's workspace.
//   wino_gemm_kernel     per call: for a tile of 64 output channels x 64 tiles, the 16
//                        contractions M_k = U_k V_k over the input channels on the matrix cores
//                        (v_mfma_f32_32x32x16_f16), one position after the other; after each
//                        position M_k is added, with its +-1 coefficients of A^T, into the four fp32
//                        accumulators of the 2x2 outputs, so M never leaves the registers; then the
//                        fused tail and the store.
// Both transformed operands are 16-byte words of 8 consecutive input channels, words of
// consecutive rows (output channels, tiles) adjacent: global loads, LDS stores and the MFMA
// operand reads are all contiguous 16-byte accesses without any transposition.
// Precision: the transformed operands are fp16 (11-bit significand; the inputs are bf16, 8 bits):
// B^T d B adds four bf16 values, so |V| <= 4 max|x| must stay below 65504.  Accumulation, the
// inverse transform and the tail are fp32.
#include "tvg_device.h"
#include "tvg_internal.h"

namespace tvg {
namespace {

typedef _Float16 half_t;
typedef _Float16 f16x8v __attribute__((ext_vector_type(8)));
constexpr int kRsrcFlags = 0x00020000;   // raw buffer descriptor word 3 on gfx9-family targets
constexpr int kMT = 64;                  // output channels per workgroup
constexpr int kKC = 64;                  // input channels are taken in multiples of this
constexpr int kKS = 32;                  // channel octets per step of the contraction kernel

// ---------------------------------------------------------------------------------------------
struct WinoWArgs {
    const bf16_t *w;
    half_t *u;
    int OC, IC;
};

__global__ __launch_bounds__(256) void wino_weight_kernel(const WinoWArgs a)
{
    const int IC8 = a.IC >> 3;
    const int idx = blockIdx.x * 256 + threadIdx.x;       // (channel octet, oc), oc fastest
    if (idx >= IC8 * a.OC) return;
    const int oc = idx % a.OC, oct = idx / a.OC;
    // the 8 x 9 weights of this (oc, octet): 144 contiguous bytes, 16-byte aligned
    const uint4v *src = reinterpret_cast<const uint4v *>(a.w + ((size_t)oc * a.IC + oct * 8) * 9);
    uint32_t raw[36];
#pragma unroll
    for (int i = 0; i < 9; ++i) {
        const uint4v v = src[i];
        raw[4 * i] = v[0]; raw[4 * i + 1] = v[1]; raw[4 * i + 2] = v[2]; raw[4 * i + 3] = v[3];
    }
    f16x8v out[16];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        float g[9];
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const int e = c * 9 + t;
            g[t] = __uint_as_float((e & 1) ? (raw[e >> 1] & 0xFFFF0000u) : (raw[e >> 1] << 16));
        }
        float tg[4][3];                                    // G g
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            tg[0][s] = g[s];
            tg[1][s] = 0.5f * (g[s] + g[3 + s] + g[6 + s]);
            tg[2][s] = 0.5f * (g[s] - g[3 + s] + g[6 + s]);
            tg[3][s] = g[6 + s];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {                      // (G g) G^T
            out[4 * i + 0][c] = (half_t)tg[i][0];
            out[4 * i + 1][c] = (half_t)(0.5f * (tg[i][0] + tg[i][1] + tg[i][2]));
            out[4 * i + 2][c] = (half_t)(0.5f * (tg[i][0] - tg[i][1] + tg[i][2]));
            out[4 * i + 3][c] = (half_t)tg[i][2];
        }
    }
#pragma unroll
    for (int k = 0; k < 16; ++k)
        *reinterpret_cast<f16x8v *>(a.u + ((size_t)(k * IC8 + oct) * a.OC + oc) * 8) = out[k];
}

// ---------------------------------------------------------------------------------------------
struct WinoIArgs {
    const bf16_t *x;
    half_t *v;
    int IC, H, W, TW, THW, T;       // THW = tile rows x tile columns of one image
    float inv_thw, inv_tw;
    uint32_t x_bytes;
};

// One thread per (tile, channel octet); lanes run over tiles, so the 16-byte stores of a position
// are contiguous.  EVENW: rows of an even number of pixels start 4-byte aligned, and the four
// columns 2 tw - 1 .. 2 tw + 2 of a tile come from three aligned pixel pairs.
template <bool EVENW>
__global__ __launch_bounds__(256) void wino_input_kernel(const WinoIArgs a)
{
    const int IC8 = a.IC >> 3;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)IC8 * a.T) return;
    const int t = (int)(idx % a.T), oct = (int)(idx / a.T);
    int rem, tw;
    const int n = fast_div(t, a.THW, a.inv_thw, &rem);
    const int th = fast_div(rem, a.TW, a.inv_tw, &tw);
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(a.x), 0, a.x_bytes, kRsrcFlags);
    const uint32_t kOut = 0xFFFFFFFFu;                    // beyond any tensor: the load returns zero
    const int ih0 = 2 * th - 1, iw0 = 2 * tw - 1;
    f16x8v out[16];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const uint32_t plane = (uint32_t)((n * a.IC + oct * 8 + c) * a.H) * (uint32_t)a.W;   // elements
        float d[4][4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int ih = ih0 + r;
            const bool rv = ih >= 0 && ih < a.H;
            const uint32_t row = plane + (uint32_t)(ih * a.W);
            if constexpr (EVENW) {
                const uint32_t o0 = (rv && tw > 0) ? 2u * (row + iw0 - 1) : kOut;
                const uint32_t o1 = rv ? 2u * (row + iw0 + 1) : kOut;
                const uint32_t o2 = (rv && iw0 + 3 < a.W) ? 2u * (row + iw0 + 3) : kOut;
                const uint32_t p0 = __builtin_amdgcn_raw_buffer_load_b32(xrsrc, o0, 0, 0);
                const uint32_t p1 = __builtin_amdgcn_raw_buffer_load_b32(xrsrc, o1, 0, 0);
                const uint32_t p2 = __builtin_amdgcn_raw_buffer_load_b32(xrsrc, o2, 0, 0);
                d[r][0] = __uint_as_float(p0 & 0xFFFF0000u);
                d[r][1] = __uint_as_float(p1 << 16);
                d[r][2] = __uint_as_float(p1 & 0xFFFF0000u);
                d[r][3] = __uint_as_float(p2 << 16);
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int iw = iw0 + q;
                    const uint32_t o = (rv && iw >= 0 && iw < a.W) ? 2u * (row + iw) : kOut;
                    const uint32_t e = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(xrsrc, o, 0, 0);
                    d[r][q] = __uint_as_float(e << 16);
                }
            }
        }
        float bt[4][4];                                    // B^T d
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            bt[0][q] = d[0][q] - d[2][q];
            bt[1][q] = d[1][q] + d[2][q];
            bt[2][q] = d[2][q] - d[1][q];
            bt[3][q] = d[1][q] - d[3][q];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {                      // (B^T d) B
            out[4 * i + 0][c] = (half_t)(bt[i][0] - bt[i][2]);
            out[4 * i + 1][c] = (half_t)(bt[i][1] + bt[i][2]);
            out[4 * i + 2][c] = (half_t)(bt[i][2] - bt[i][1]);
            out[4 * i + 3][c] = (half_t)(bt[i][1] - bt[i][3]);
        }
    }
#pragma unroll
    for (int k = 0; k < 16; ++k)
        *reinterpret_cast<f16x8v *>(a.v + ((size_t)(k * IC8 + oct) * a.T + t) * 8) = out[k];
}

// ---------------------------------------------------------------------------------------------
struct WinoArgs {
    const half_t *u, *v;
    const float *scale, *shift, *bias;
    const bf16_t *residual;
    bf16_t *y;
    int IC, OC, OH, OW, TW, THW, T;
    float inv_thw, inv_tw;
    int relu;
    int mtiles;
    uint32_t u_bytes, v_bytes;
};

// Coefficient of position k = (ki, kj) in output (a, b): A^T[a][ki] * A^T[b][kj].
__host__ __device__ constexpr int at_coef(int a, int k)
{
    return a == 0 ? (k < 3 ? 1 : 0) : (k == 0 ? 0 : k == 1 ? 1 : -1);
}

// A workgroup owns 64 output channels x 64 tiles (four waves, 32 x 32 each).  A step brings kKS
// channel octets of the flattened [position][octet] axis into LDS - four positions at once for 64
// input channels, one position in several steps for 512 - so that few, large steps stand between
// a workgroup and its result: the chain of steps is what a small problem's time consists of.
// OMODE: how a lane stores its outputs - 2: eight consecutive pixels of an output row as one
// 16-byte store (OW % 8 == 0), 1: the pixel pair of a tile row as one 4-byte store (OW even),
// 0: element by element.
template <int OMODE>
__global__ __launch_bounds__(256, 2) void wino_gemm_kernel(const WinoArgs a)
{
    constexpr int NB = 1;
    constexpr int NT = 64;
    constexpr int AL = kKS * kMT / 256, BL = kKS * NT / 256;      // words per thread and step
    __shared__ __attribute__((aligned(16))) unsigned char lds[(kKS * kMT + kKS * NT) * 16];
    __shared__ float ss_lds[2 * kMT];
    unsigned char *As = lds, *Bs = lds + kKS * kMT * 16;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int lrow = lane & 31, lhalf = lane >> 5;
    // Workgroups are dealt to the eight XCDs in turn; renumbered so that one XCD gets a contiguous
    // run of tiles, the channel tiles of one tile range (which read the same transformed input)
    // share that XCD's L2 instead of each fetching it from HBM (C6: 105 -> 57 MB fetched).
    const int nbk = gridDim.x, bid = blockIdx.x;
    const int xq = nbk >> 3, xr = nbk & 7, xcd = bid & 7, local = bid >> 3;
    const int tile = xcd < xr ? xcd * (xq + 1) + local : xr * (xq + 1) + (xcd - xr) * xq + local;
    const int m0 = (tile % a.mtiles) * kMT;
    const int t0 = (tile / a.mtiles) * NT;

    stage_scale_shift(ss_lds, m0, kMT, a.scale, a.shift, a.bias, a.OC, tid, 256);

    const __amdgpu_buffer_rsrc_t ursrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<half_t *>(a.u), 0, a.u_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t vrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<half_t *>(a.v), 0, a.v_bytes, kRsrcFlags);
    // Fixed load slots: word wi of a step is row wi % 64 of octet wi / 64; step s starts kKS rows
    // of OC (of T) words further along the flattened axis.
    uint32_t aoff[AL], boff[BL];
#pragma unroll
    for (int i = 0; i < AL; ++i) {
        const int wi = tid + 256 * i, o = wi >> 6, r = wi & 63;
        aoff[i] = (uint32_t)(o * a.OC + m0 + r) * 16u;
    }
#pragma unroll
    for (int i = 0; i < BL; ++i) {
        const int wi = tid + 256 * i, o = wi / NT, r = wi % NT;
        // tiles past the end read zeros (an offset beyond the buffer); they are never stored
        boff[i] = t0 + r < a.T ? (uint32_t)(o * a.T + t0 + r) * 16u : 0x80000000u;
    }
    const uint32_t astep = (uint32_t)kKS * (uint32_t)a.OC * 16u, bstep = (uint32_t)kKS * (uint32_t)a.T * 16u;
    const int IC8 = a.IC >> 3;
    const int steps = 16 * IC8 / kKS;

    uint4v areg[AL], breg[BL];
    auto issue = [&](int s) {
#pragma unroll
        for (int i = 0; i < AL; ++i)
            areg[i] = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(ursrc, aoff[i], s * astep, 0));
#pragma unroll
        for (int i = 0; i < BL; ++i)
            breg[i] = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(vrsrc, boff[i], s * bstep, 0));
    };
    auto commit = [&]() {
#pragma unroll
        for (int i = 0; i < AL; ++i) *reinterpret_cast<uint4v *>(As + (tid + 256 * i) * 16) = areg[i];
#pragma unroll
        for (int i = 0; i < BL; ++i) *reinterpret_cast<uint4v *>(Bs + (tid + 256 * i) * 16) = breg[i];
    };

    float16v yacc[2][2][NB], macc[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            macc[j][e] = 0.0f;
            yacc[0][0][j][e] = 0.0f; yacc[0][1][j][e] = 0.0f; yacc[1][0][j][e] = 0.0f; yacc[1][1][j][e] = 0.0f;
        }
    }

    issue(0);
    commit();
    __syncthreads();
    for (int s = 0; s < steps; ++s) {
        const bool more = s + 1 < steps;
        if (more) issue(s + 1);
#pragma unroll
        for (int sub = 0; sub < kKS / 8; ++sub) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int oct = sub * 8 + 2 * ks + lhalf;
                const f16x8v af = *reinterpret_cast<const f16x8v *>(As + (oct * kMT + wm * 32 + lrow) * 16);
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const f16x8v bf = *reinterpret_cast<const f16x8v *>(
                        Bs + (oct * NT + wn * (NT / 2) + j * 32 + lrow) * 16);
                    macc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf, af, macc[j], 0, 0, 0);
                }
            }
            // the last octets of a position: Y[p][q] += A^T[p][ki] A^T[q][kj] M_k.  The
            // coefficients are 0 or +-1 and uniform, so a zero one is a skipped branch.
            const int fend = s * kKS + sub * 8 + 8;
            if (fend % IC8 == 0) {
                const int k = fend / IC8 - 1;
#pragma unroll
                for (int p = 0; p < 2; ++p)
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        const int cf = at_coef(p, k >> 2) * at_coef(q, k & 3);
                        if (cf != 0) {
                            const float f = (float)cf;
#pragma unroll
                            for (int j = 0; j < NB; ++j)
#pragma unroll
                                for (int e = 0; e < 16; ++e)
                                    yacc[p][q][j][e] = fmaf(f, macc[j][e], yacc[p][q][j][e]);
                        }
                    }
#pragma unroll
                for (int j = 0; j < NB; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) macc[j][e] = 0.0f;
            }
        }
        __syncthreads();
        if (more) commit();
        __syncthreads();
    }

    // ---- fused tail and store -------------------------------------------------------------
    // Value e of a lane's 32x32 block belongs to output channel lrow and tile
    // 8 (e / 4) + 4 lhalf + e % 4: four groups of four consecutive tiles.
    const int oc = m0 + wm * 32 + lrow;
    if (oc >= a.OC) return;
    const float sc = ss_lds[2 * (wm * 32 + lrow)], sf = ss_lds[2 * (wm * 32 + lrow) + 1];
    const bool relu = a.relu & 1;
    auto finish = [&](float acc, float res) {
        float v = fmaf(acc, sc, sf) + res;
        return relu ? fmaxf(v, 0.0f) : v;
    };
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int tb = t0 + wn * (NT / 2) + j * 32 + g * 8 + lhalf * 4;
            if constexpr (OMODE == 2) {
                // OW % 8 == 0: four consecutive tiles from a multiple of four share a tile row
                if (tb >= a.T) continue;
                int rem, tw;
                const int n = fast_div(tb, a.THW, a.inv_thw, &rem);
                const int th = fast_div(rem, a.TW, a.inv_tw, &tw);
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    const int oh = 2 * th + p;
                    if (oh >= a.OH) continue;
                    const size_t o = ((size_t)(n * a.OC + oc) * a.OH + oh) * a.OW + 2 * tw;
                    uint4v r4 = {0, 0, 0, 0};
                    if (a.residual) r4 = *reinterpret_cast<const uint4v *>(a.residual + o);
                    uint4v o4;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float lo = finish(yacc[p][0][j][g * 4 + i], __uint_as_float(r4[i] << 16));
                        const float hi = finish(yacc[p][1][j][g * 4 + i], __uint_as_float(r4[i] & 0xFFFF0000u));
                        o4[i] = f32x2_to_bf16x2(lo, hi);
                    }
                    *reinterpret_cast<uint4v *>(a.y + o) = o4;
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int t = tb + i;
                    if (t >= a.T) continue;
                    int rem, tw;
                    const int n = fast_div(t, a.THW, a.inv_thw, &rem);
                    const int th = fast_div(rem, a.TW, a.inv_tw, &tw);
#pragma unroll
                    for (int p = 0; p < 2; ++p) {
                        const int oh = 2 * th + p;
                        if (oh >= a.OH) continue;
                        const size_t o = ((size_t)(n * a.OC + oc) * a.OH + oh) * a.OW + 2 * tw;
                        if constexpr (OMODE == 1) {
                            uint32_t r2 = 0;
                            if (a.residual) r2 = *reinterpret_cast<const uint32_t *>(a.residual + o);
                            const float lo = finish(yacc[p][0][j][g * 4 + i], __uint_as_float(r2 << 16));
                            const float hi = finish(yacc[p][1][j][g * 4 + i], __uint_as_float(r2 & 0xFFFF0000u));
                            *reinterpret_cast<uint32_t *>(a.y + o) = f32x2_to_bf16x2(lo, hi);
                        } else {
#pragma unroll
                            for (int q = 0; q < 2; ++q) {
                                if (2 * tw + q >= a.OW) continue;
                                const float res = a.residual ? bf16_to_f32(a.residual[o + q]) : 0.0f;
                                a.y[o + q] = f32_to_bf16(finish(yacc[p][q][j][g * 4 + i], res));
                            }
                        }
                    }
                }
            }
        }
}

}  // namespace

bool plan_conv3x3_winograd(const ConvProblem &p, WinoPlan *plan)
{
    if (p.dtype != TVG_BF16 || p.R != 3 || p.S != 3 || p.sh != 1 || p.sw != 1 || p.ph != 1 || p.pw != 1)
        return false;
    if (p.IC % kKC != 0 || p.OC % kMT != 0) return false;
    const long th = (p.OH + 1) / 2, tw = (p.OW + 1) / 2;
    const long T = (long)p.N * th * tw;
    const size_t v_bytes = (size_t)16 * p.IC * T * 2, u_bytes = (size_t)16 * p.IC * p.OC * 2;
    // tile indices go through the float-reciprocal division; buffer offsets are 32 bits, and an
    // offset of 2^31 must lie beyond V
    if (T >= (1 << 22) || v_bytes >= ((size_t)1 << 31) || u_bytes >= ((size_t)1 << 31)) return false;
    if ((size_t)p.N * p.IC * p.H * p.W * 2 >= ((size_t)1 << 32)) return false;
    plan->TH = (int)th; plan->TW = (int)tw; plan->T = (int)T;
    plan->u_bytes = u_bytes; plan->v_bytes = v_bytes;
    const long mtiles = p.OC / kMT;
    plan->nb = 1;
    plan->tiles = mtiles * ((T + 63) / 64);
    return true;
}

tvg_status launch_winograd_prepack(const ConvProblem &p, const void *w, void *packed, hipStream_t stream)
{
    WinoWArgs a{static_cast<const bf16_t *>(w), static_cast<half_t *>(packed), p.OC, p.IC};
    const unsigned grid = (unsigned)(((long)(p.IC / 8) * p.OC + 255) / 256);
    hipLaunchKernelGGL(wino_weight_kernel, dim3(grid), dim3(256), 0, stream, a);
    return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
}

tvg_status launch_conv3x3_winograd(const ConvProblem &p, const WinoPlan &plan, const void *packed,
                                   const ConvPointers &ptr, hipStream_t stream)
{
    WinoIArgs ia;
    ia.x = static_cast<const bf16_t *>(ptr.x); ia.v = reinterpret_cast<half_t *>(ptr.workspace);
    ia.IC = p.IC; ia.H = p.H; ia.W = p.W; ia.TW = plan.TW; ia.THW = plan.TH * plan.TW; ia.T = plan.T;
    ia.inv_thw = 1.0f / (float)ia.THW; ia.inv_tw = 1.0f / (float)plan.TW;
    ia.x_bytes = (uint32_t)((size_t)p.N * p.IC * p.H * p.W * 2);
    const unsigned igrid = (unsigned)(((long)(p.IC / 8) * plan.T + 255) / 256);
    const bool evenw = p.W % 2 == 0 && reinterpret_cast<uintptr_t>(ptr.x) % 4 == 0;
    if (evenw) hipLaunchKernelGGL(wino_input_kernel<true>, dim3(igrid), dim3(256), 0, stream, ia);
    else hipLaunchKernelGGL(wino_input_kernel<false>, dim3(igrid), dim3(256), 0, stream, ia);

    WinoArgs a;
    a.u = static_cast<const half_t *>(packed); a.v = ia.v;
    a.scale = ptr.scale; a.shift = ptr.shift; a.bias = ptr.bias;
    a.residual = static_cast<const bf16_t *>(ptr.residual); a.y = static_cast<bf16_t *>(ptr.y);
    a.IC = p.IC; a.OC = p.OC; a.OH = p.OH; a.OW = p.OW; a.TW = plan.TW; a.THW = ia.THW; a.T = plan.T;
    a.inv_thw = ia.inv_thw; a.inv_tw = ia.inv_tw;
    a.relu = p.relu;
    a.mtiles = p.OC / kMT;
    a.u_bytes = (uint32_t)plan.u_bytes; a.v_bytes = (uint32_t)plan.v_bytes;
    const uintptr_t al = reinterpret_cast<uintptr_t>(ptr.y) | reinterpret_cast<uintptr_t>(ptr.residual);
    const int omode = (p.OW % 8 == 0 && al % 16 == 0) ? 2 : (p.OW % 2 == 0 && al % 4 == 0) ? 1 : 0;
    const unsigned grid = (unsigned)plan.tiles;
    if (omode == 2) hipLaunchKernelGGL((wino_gemm_kernel<2>), dim3(grid), dim3(256), 0, stream, a);
    else if (omode == 1) hipLaunchKernelGGL((wino_gemm_kernel<1>), dim3(grid), dim3(256), 0, stream, a);
    else hipLaunchKernelGGL((wino_gemm_kernel<0>), dim3(grid), dim3(256), 0, stream, a);
    return hipGetLastError() == hipSuccess ? TVG_OK : TVG_ERR_LAUNCH;
}

}  // namespace tvg
