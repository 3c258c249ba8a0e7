// Internal declarations shared by the translation units of libtvg (not installed).
#ifndef TVG_INTERNAL_H
#define TVG_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tvg.h"

namespace tvg {

// Number of compute units the launch heuristics are tuned for (MI355X).  A
// constant, not a device query, so that workspace sizes are a pure function of
// the descriptor.
constexpr int kComputeUnits = 256;

// Depthwise: floats of LDS that the narrowest row band of the general kernel may take (four
// output rows = 3*stride + 3 input rows of W + 2 columns, plus 12 per-plane parameters, in
// 64 KB).  The host rejects wider rows for every depthwise call, whichever kernel would run.
constexpr int kDwBandFloats = 64 * 1024 / 4 - 12;

struct ConvProblem {
    int N, IC, H, W, OC, R, S, sh, sw, ph, pw, OH, OW;
    int K;          // IC * R * S, the reduction length of the implicit GEMM
    int npix;       // N * OH * OW, the number of GEMM columns
    int dtype;      // tvg_dtype
    int relu;
    int stream_out; // TVG_STREAM_OUT: y is stored with the non-temporal hint
};

struct Knobs {
    int mt, nt;       // workgroup tile
    int stages;       // bf16 3x3: 1 = single-stage kernel, 2 = software-pipelined kernel
    int split_k;      // generic kernel: partitions of the reduction; pipelined 3x3: wave groups (1, 2)
    int lds_pitch;    // pipelined 3x3: 1 = plain patch pitch, 2 = conflict-free padded pitch
    int row_loads;    // pipelined 3x3, odd rows of at most 7 pixels: 1 = element loads, 2 = whole rows
};

struct ConvPointers {
    const void *x, *w;
    const float *scale, *shift, *bias;
    const void *residual;
    void *y;
    float *workspace;
};

// How the dense kernel is launched for a problem; a pure function of the problem.
struct ConvPlan {
    int mt;             // rows (output channels) per workgroup tile: 64 or 128
    int nt;             // columns (pixels) per workgroup tile: 128
    int splits;         // partitions of the reduction axis (1 = none)
    int k_per_split;    // reduction elements per partition, a multiple of the K chunk
    size_t workspace_bytes;
};

// Schedule knobs fixed for this exact problem by tvg_conv2d_set_knobs / tvg_conv2d_set_tile
// (all zero when there are none; a zero field leaves that choice to the planner's rule).
Knobs forced_knobs(const ConvProblem &p);

// `allow_split` = false plans a single pass over the reduction (no workspace).
ConvPlan plan_conv(const ConvProblem &p, bool allow_split = true);

// Launch shape of the bf16 3x3 patch kernel; a pure function of the problem.
struct Patch3x3Plan {
    int mt, nt;         // output channels x pixels per workgroup
    int pt;             // patch load tasks per thread
    int px;             // pixels per load (1, 2 or 4)
    int rows;           // virtual input rows staged per tile (maximum over tiles)
    size_t lds_bytes;
    long tiles;
    int dbuf;           // 1 = the software-pipelined kernel with two LDS stages runs the tile
    int pplane;         // its bytes per channel-octet plane of the patch
    int stage_bytes;    // its bytes per LDS stage
    int pws, xp16;      // its patch row pitch (16-byte words) and extra bytes between images
    int kg;             // its groups of four waves that split the reduction (1 or 2)
    // inputs to plan_conv3x3_dbuf, from the knobs (0 = the planner's rule): wave groups,
    // pitch (1 plain, 2 padded), row loads (1 element-wise, 2 whole rows)
    int want_kg, want_pitch, want_rows, want_stages;
};

// True when the problem is one the patch kernel is built for (bf16, 3x3, pad 1,
// stride 1 or 2, IC a multiple of 16).  Pointer alignment is checked at launch.
// single_stage_mt_divides > 0 (two-head launches): plan the single-stage kernel only, with a
// channel tile that divides this number (the channels of head 1).
bool plan_conv3x3_patch(const ConvProblem &p, Patch3x3Plan *plan, int single_stage_mt_divides = 0);
bool conv3x3_patch_pointers_ok(const ConvPointers &ptr);
// The second head of a two-head launch: output channels [oc1, OC) go to y2 with their own flags.
struct DualHead {
    int oc1, relu2, centre2;     // relu2: bit 0 ReLU, bit 1 store hint
    void *y2;
};
tvg_status launch_conv3x3_patch(const ConvProblem &p, const Patch3x3Plan &plan,
                                const ConvPointers &ptr, hipStream_t stream,
                                const DualHead *dual = nullptr);
// Two-stage variant (64-channel tiles): completes a plan whose mt, nt and rows are set.
bool plan_conv3x3_dbuf(const ConvProblem &p, Patch3x3Plan *plan);
tvg_status launch_conv3x3_dbuf(const ConvProblem &p, const Patch3x3Plan &plan,
                               const ConvPointers &ptr, hipStream_t stream);

// bf16 7x7 stride-2 pad-3 kernel for IC <= 4 (the ResNet stem).
struct StemPlan {
    int rows;           // virtual input rows staged per tile
    int mt;             // output channels per tile (64, or 32 for narrow layers)
    int lt;             // 16-byte copy tasks per thread per tile
    size_t lds_bytes;
};
bool plan_conv7x7s2_stem(const ConvProblem &p, StemPlan *plan);
bool conv7x7s2_stem_pointers_ok(const ConvPointers &ptr);
tvg_status launch_conv7x7s2_stem(const ConvProblem &p, const StemPlan &plan,
                                 const ConvPointers &ptr, hipStream_t stream);

// bf16 1x1 (pointwise) kernel, stride 1 or 2, IC a multiple of 8.
struct Pw1x1Plan {
    int mt, nt;
    long tiles;
};
bool plan_conv1x1(const ConvProblem &p, Pw1x1Plan *plan);
bool conv1x1_pointers_ok(const ConvPointers &ptr);
tvg_status launch_conv1x1(const ConvProblem &p, const Pw1x1Plan &plan, const ConvPointers &ptr,
                          hipStream_t stream);

// bf16 1x1 stride-1 kernel for deep reductions (IC a multiple of 128, maps of 4n pixels): wide
// pixel loads transposed in registers, two steps of 64 channels in flight.
struct PwDeepPlan {
    int px;             // pixels per load: 8 or 4
    long tiles;
};
bool plan_conv1x1_deep(const ConvProblem &p, PwDeepPlan *plan);
bool conv1x1_deep_pointers_ok(const ConvPointers &ptr);
tvg_status launch_conv1x1_deep(const ConvProblem &p, const PwDeepPlan &plan, const ConvPointers &ptr,
                               hipStream_t stream);

// bf16 MobileNet block in one kernel: depthwise 3x3 (pad 1, stride 1) computed in LDS as the
// pixel operand of the 1x1 stage.  `dw` is the depthwise problem, OC the 1x1 stage's channels.
struct DwPwPlan {
    int mt, lt;        // output channels per workgroup, patch dwords per loader thread
    long tiles;
};
struct DwPwPointers {
    const void *x, *w_dw;
    const float *scale_dw, *shift_dw;
    const void *w_pw;
    const float *scale_pw, *shift_pw, *bias_pw;
    const void *residual;
    void *y;
};
bool plan_dwpw(const ConvProblem &dw, int OC, DwPwPlan *plan);
tvg_status launch_dwpw(const ConvProblem &dw, int OC, int pw_relu, int pw_stream_out,
                       const DwPwPlan &plan, const DwPwPointers &ptr, hipStream_t stream);

// fp32 1x1 / 3x3 kernel for launch-bound problems: one launch, the waves of a workgroup split the
// reduction and add their accumulators through LDS.
struct F32SmallPlan {
    int tile;           // output tile edge: 32 or 16
    int nw, passes;     // waves per workgroup, passes over the input channels
    int pitch, region;  // LDS row pitch and floats per wave
    int vec;            // floats per patch load: 4, 2 or 1 (rows of 4n, 2n, other pixel counts)
    int ksplit;         // slices of the reduction across workgroups (1 = none, else a reduce launch follows)
    int stem;           // 1 = the 7x7 stride-2 variant (seven waves, one per filter row; region = staged rows)
    size_t lds_bytes, workspace_bytes;
};
// Adds `splits` partial results [splits][N][OC][OH][OW] in ptr.workspace in a fixed order and
// applies the fused tail (the second launch of every reduction that is split across workgroups).
tvg_status launch_splitk_reduce(const ConvProblem &p, int splits, const ConvPointers &ptr,
                                hipStream_t stream);
bool plan_conv_f32_small(const ConvProblem &p, F32SmallPlan *plan);
bool conv_f32_small_pointers_ok(const ConvPointers &ptr);
tvg_status launch_conv_f32_small(const ConvProblem &p, const F32SmallPlan &plan, const ConvPointers &ptr,
                                 hipStream_t stream);

// bf16 3x3 stride-1 pad-1 convolution by Winograd F(2x2, 3x3) with pre-transformed weights
// (IC and OC multiples of 64).  The packed weights are u_bytes of fp16, the per-call workspace
// (the transformed input) v_bytes.
struct WinoPlan {
    int TH, TW, T;      // 2x2 output tiles per image column, row, and in all
    int nb;             // 32-tile blocks per wave (1: the workgroup covers 64 channels x 64 tiles)
    long tiles;
    size_t u_bytes, v_bytes;
};
bool plan_conv3x3_winograd(const ConvProblem &p, WinoPlan *plan);
tvg_status launch_winograd_prepack(const ConvProblem &p, const void *w, void *packed, hipStream_t stream);
// ptr.w is unused (the weights come packed), ptr.workspace is the transformed-input area.
tvg_status launch_conv3x3_winograd(const ConvProblem &p, const WinoPlan &plan, const void *packed,
                                   const ConvPointers &ptr, hipStream_t stream);

tvg_status launch_conv_igemm(const ConvProblem &p, const ConvPlan &plan, const ConvPointers &ptr,
                             hipStream_t stream);
tvg_status launch_dwconv3x3(const ConvProblem &p, const ConvPointers &ptr, hipStream_t stream);
tvg_status launch_maxpool3x3s2(int N, int C, int H, int W, int dtype, const void *x, void *y,
                               hipStream_t stream);

}  // namespace tvg

#endif
