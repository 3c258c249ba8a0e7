/*
 * libtvg - fused conv2d and depthwise conv2d operators for one AMD MI355X (gfx950).
 *
 * These are hand-written versions of the fused tensor operators that the TVM
 * paper (arXiv 1802.04799) generates: a convolution with the element-wise
 * operators that follow it applied to its output inside the same kernel
 * (Section 3, "Operator Fusion": conv2d is "complex-out-fusable"), for the
 * operator shapes of Table 2 (conv2d C1..C12 of ResNet-18, depthwise conv2d
 * D1..D9 of MobileNet) and any other shape within the stated limits.
 *
 * Conventions common to every entry point
 *   - Plain C ABI.  Every data pointer is a DEVICE pointer owned by the caller;
 *     the descriptor and the size_t outputs are HOST pointers.
 *   - The library never allocates, frees or synchronises.  Work is enqueued on
 *     `hip_stream` (a hipStream_t passed as void*; NULL = the default stream) and
 *     the call returns at once.
 *   - Tensors are dense and contiguous: activations NCHW, dense weights OIHW
 *     [k][c][r][s], depthwise weights [c][1][r][s].  x, w, residual and y share
 *     `dtype`; scale, shift and bias are fp32 [k] whatever the dtype.
 *   - Cross-correlation (no kernel flip), symmetric zero padding, dilation 1.
 *     Output extent OH = floor((H + 2*pad_h - R) / stride_h) + 1 (must be >= 1).
 *   - Fused tail applied to the fp32 accumulator, in this order:
 *       t = acc + bias[k] (if bias); t = t*scale[k] + shift[k];
 *       t += residual[n,k,oh,ow] (if residual); t = max(t, 0) (if TVG_RELU);
 *       y = t rounded to dtype (bf16: round to nearest, ties to even).
 *   - y must not overlap x or w.  y may be the same buffer as residual (each
 *     element is read and then written by the same lane).
 *   - All arguments are validated on the host before any device call, so error
 *     paths can be exercised on a machine without a GPU.  Errors are return
 *     codes; nothing is thrown, logged or aborted.  On error nothing is launched.
 *   - Results are deterministic run to run (no floating-point atomics).
 *   - Limits: every tensor must hold fewer than 2^31 elements; R, S <= 16;
 *     strides 1..8; pad < kernel extent.  Depthwise calls also need
 *     (3*stride + 3) * (w + 2) <= 16372, i.e. w <= 2726 at stride 1 and w <= 1817 at stride 2
 *     (one band of input rows is staged in 64 KB of LDS); the size query and the operator
 *     both answer TVG_ERR_UNSUPPORTED beyond that.
 *   - Which kernel runs a problem, its launch shape and its workspace size depend on the
 *     descriptor (flags aside) and on what tvg_conv2d_set_tile has fixed, on nothing else: no
 *     environment variable is read.  Plans are remembered per problem; a size query and the
 *     call that follows it therefore agree unless tvg_conv2d_set_tile runs in between.
 */
#ifndef TVG_H
#define TVG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TVG_OK = 0,
    TVG_ERR_NULL = 1,          /* a required pointer is NULL */
    TVG_ERR_BAD_SHAPE = 2,     /* non-positive extent, empty output, stride/pad out of range */
    TVG_ERR_UNSUPPORTED = 3,   /* unknown dtype or flag, tensor too large, kernel size not built */
    TVG_ERR_WORKSPACE = 4,     /* workspace NULL, smaller than the query says or misaligned */
    TVG_ERR_LAUNCH = 5         /* the HIP runtime refused the launch */
} tvg_status;

typedef enum { TVG_F32 = 0, TVG_BF16 = 1 } tvg_dtype;

/* Bits of tvg_conv_desc.flags.
 * TVG_RELU        clamp the output at zero (last step of the fused tail).
 * TVG_STREAM_OUT  a hint, results are identical with and without it: y is stored with the
 *                 non-temporal cache hint.  Right when nothing reads y soon (an operator run
 *                 on its own, an output larger than the caches): the kernel and its successor
 *                 then run faster, since y neither displaces the operands in L2 nor waits
 *                 there to be written back.  Wrong between the layers of a network whose
 *                 activations fit the memory-side cache: the next layer would fetch from
 *                 HBM what it could have found there.  Off by default.  Kernels without wide
 *                 stores (the generic kernel that takes fp32 and odd shapes, the element-wise
 *                 tail of unaligned maps) ignore it. */
enum { TVG_RELU = 1u, TVG_STREAM_OUT = 2u };
/* Only in the flags2 argument of tvg_conv2d_fused_dual: see there. */
enum { TVG_CENTRE_TAP_ONLY = 4u };

typedef struct {
    int32_t n, c, h, w;        /* input N, C (= IC), H, W                                   */
    int32_t k, r, s;           /* output channels, kernel height, kernel width              */
    int32_t stride_h, stride_w, pad_h, pad_w;
    int32_t dtype;             /* tvg_dtype of x, w, residual, y                            */
    uint32_t flags;            /* TVG_RELU | TVG_STREAM_OUT, or 0                           */
} tvg_conv_desc;               /* depthwise: k == c, r == s == 3                            */

/*
 * Bytes of scratch that tvg_conv2d_fused needs for this problem (0 when the
 * problem is not split along the reduction axis).  Pure host computation.
 * `bytes` is a host pointer.  Returns TVG_OK or the same validation error the
 * operator itself would return.
 */
tvg_status tvg_conv2d_workspace_size(const tvg_conv_desc *desc, size_t *bytes);

/* Always 0 bytes; present so both operators are driven the same way. */
tvg_status tvg_dwconv2d_workspace_size(const tvg_conv_desc *desc, size_t *bytes);

/*
 * Dense fused conv2d (Table 2, rows C; fused tail per Section 3).  Implicit
 * GEMM on the matrix cores: rows = output channels, columns = output pixels
 * (n, oh, ow), reduction = (c, r, s); fp32 accumulate for both dtypes.
 *   x        device, [n][c][h][w], dtype
 *   w        device, [k][c][r][s], dtype
 *   scale    device, fp32 [k]  (required; pass ones for a bare convolution)
 *   shift    device, fp32 [k]  (required; pass zeros for a bare convolution)
 *   bias     device, fp32 [k], or NULL
 *   residual device, [n][k][oh][ow], dtype, or NULL
 *   y        device, [n][k][oh][ow], dtype, written completely
 *   workspace device, at least tvg_conv2d_workspace_size() bytes, 256-byte
 *            aligned; may be NULL when that size is 0.  Contents are scratch.
 */
tvg_status tvg_conv2d_fused(const tvg_conv_desc *desc, const void *x, const void *w,
                            const float *scale, const float *shift, const float *bias,
                            const void *residual, void *y,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Two fused convolutions of the SAME input in one launch (Section 3, operator fusion, applied to
 * sibling operators that share their input): bf16, 3x3, pad 1, stride 1 or 2, c a multiple of 16.
 * desc describes both together, desc->k = k1 + k2 output channels with weights [k1 + k2][c][3][3]
 * and scale, shift, bias of k1 + k2 entries:
 *   head 1   channels [0, k1): y1 [n][k1][oh][ow], tail with desc->flags and residual1
 *            ([n][k1][oh][ow] or NULL)
 *   head 2   channels [k1, k1 + k2): y2 [n][k2][oh][ow], tail with flags2 (TVG_RELU,
 *            TVG_STREAM_OUT), no residual
 * What it is for: the down-sampling block of a residual network, whose first 3x3 stride-2
 * convolution and whose 1x1 stride-2 projection shortcut read the same tensor.  A 1x1 convolution
 * with stride s and no padding is the centre tap of a 3x3 convolution with stride s and pad 1, so
 * the projection rides along as head 2 with filters that are zero outside their centre tap
 * (w[k1 + j][i][1][1] = the 1x1 weight, the caller builds the tensor once); TVG_CENTRE_TAP_ONLY in
 * flags2 is the caller's promise of exactly that, and head 2's tiles then skip the other eight
 * taps.  Without the flag head 2 is a full 3x3 convolution.  One launch and one pass over x
 * instead of two.
 * Errors: TVG_ERR_BAD_SHAPE unless 0 < k1 < desc->k; TVG_ERR_UNSUPPORTED for problems outside the
 * single-stage 3x3 kernel (other dtype, filter, padding; k1 no multiple of 64; x or w not
 * 16-byte aligned) - run the two convolutions separately then.  y1, y2 must not overlap x, w or
 * each other.  No workspace.
 */
tvg_status tvg_conv2d_fused_dual(const tvg_conv_desc *desc, int32_t k1, uint32_t flags2,
                                 const void *x, const void *w, const float *scale,
                                 const float *shift, const float *bias, const void *residual1,
                                 void *y1, void *y2, void *hip_stream);

/*
 * Convolution with pre-transformed weights (Section 6.1: the "TVM PT" rows of the GPU operator
 * benchmark - Winograd convolution whose weight transform is done once, ahead of time).
 * bf16, 3x3, stride 1, pad 1, c and k multiples of 64: a 2x2 block of outputs is computed from a
 * 4x4 block of inputs by Winograd's minimal filtering F(2x2, 3x3), 16 multiplications per input
 * channel instead of 36.  Three calls:
 *   tvg_conv2d_prepack_size     bytes of the packed weights and of the per-call workspace
 *   tvg_conv2d_prepack          w [k][c][3][3] (device, bf16, 16-byte aligned) -> packed (device,
 *                               16-byte aligned, at least packed_bytes): G g G^T of every filter in
 *                               fp16, laid out as the contraction reads it.  Once per weight tensor.
 *   tvg_conv2d_fused_prepacked  tvg_conv2d_fused with `packed` in place of w.  workspace: device,
 *                               256-byte aligned, at least the queried size; it receives the
 *                               transformed input (16 values per 2x2 output block and channel).
 * Same definition of the operator as tvg_conv2d_fused (the fused tail included), different
 * arithmetic: the transformed operands are fp16 (the sums of four bf16 inputs do not fit bf16's 8
 * bits; fp16 keeps 11), accumulation, inverse transform and tail are fp32.  Results agree with
 * the direct kernels within 1e-2 of the output's RMS instead of one bf16 rounding; inputs must
 * satisfy 4 max|x| < 65504 (fp16's range), which the caller guarantees.
 * Errors: TVG_ERR_UNSUPPORTED for every other problem (and for tensors beyond 2 GiB of
 * transformed input); TVG_ERR_WORKSPACE for a short or misaligned packed / workspace buffer;
 * otherwise as tvg_conv2d_fused.  The calls allocate nothing and never synchronise.
 */
tvg_status tvg_conv2d_prepack_size(const tvg_conv_desc *desc, size_t *packed_bytes,
                                   size_t *workspace_bytes);
tvg_status tvg_conv2d_prepack(const tvg_conv_desc *desc, const void *w, void *packed,
                              size_t packed_bytes, void *hip_stream);
tvg_status tvg_conv2d_fused_prepacked(const tvg_conv_desc *desc, const void *x, const void *packed,
                                      const float *scale, const float *shift, const float *bias,
                                      const void *residual, void *y, void *workspace,
                                      size_t workspace_bytes, void *hip_stream);

/*
 * tvg_conv2d_fused for callers that cannot allocate device memory and so have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same operator, same kernels, same results bit for bit; the scratch that a split reduction
 * needs comes from an array inside the library (tvg_static_scratch_bytes() = 16 MiB per GPU,
 * held from the library's load to the end of the process) instead of a workspace argument.
 *   - A problem whose tvg_conv2d_workspace_size() exceeds that is TVG_ERR_WORKSPACE (use
 *     tvg_conv2d_fused with a workspace); all other arguments and errors as tvg_conv2d_fused.
 *   - The call allocates and frees nothing and never synchronises.  The device that owns
 *     hip_stream and the pointers must be the current device: the array's address is looked up
 *     for the current device on the first call that needs it (TVG_ERR_LAUNCH if the runtime
 *     cannot resolve it).
 *   - Every call on a GPU shares that GPU's array.  Calls on one stream are ordered and safe;
 *     calls that may overlap on one GPU (different streams, concurrent graphs) race on it and
 *     give wrong results.  Nothing in the array needs clearing between calls: every partial sum
 *     is written before it is read.
 */
tvg_status tvg_conv2d_fused_static(const tvg_conv_desc *desc, const void *x, const void *w,
                                   const float *scale, const float *shift, const float *bias,
                                   const void *residual, void *y, void *hip_stream);
size_t tvg_static_scratch_bytes(void);

/*
 * Depthwise fused 3x3 conv2d, channel multiplier 1 (Table 2, rows D; same fused
 * tail).  Bandwidth kernel on the vector ALUs, no matrix cores.  Arguments as
 * above with w = [c][1][3][3]; desc->k must equal desc->c and r == s == 3;
 * stride_h == stride_w in {1, 2}; pad_h == pad_w == 1 (Table 2's "SAME" padding; anything
 * else is TVG_ERR_UNSUPPORTED).  The workspace arguments are ignored.
 */
tvg_status tvg_dwconv2d_fused(const tvg_conv_desc *desc, const void *x, const void *w,
                              const float *scale, const float *shift, const float *bias,
                              const void *residual, void *y,
                              void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * MobileNet block: depthwise 3x3 conv2d and the 1x1 conv2d that follows it, as one operator
 * (Section 3, operator fusion, carried across the two operators of the block; Table 2 rows D
 * are its first stage):
 *   t = tail_dw(depthwise3x3(x, w_dw)), rounded to dtype     tail_dw: t*scale_dw[c] + shift_dw[c],
 *                                                            max(t, 0) if dw_desc->flags has TVG_RELU
 *   y = tail_pw(conv1x1(t, w_pw))                            the fused tail of tvg_conv2d_fused with
 *                                                            scale_pw, shift_pw, bias_pw, residual,
 *                                                            pw_flags (TVG_RELU, TVG_STREAM_OUT)
 * dw_desc describes the depthwise stage as for tvg_dwconv2d_fused (k == c, 3x3, pad 1, stride 1
 * or 2); pw_k is the number of output channels of the 1x1 stage.
 *   x [n][c][h][w]; w_dw [c][1][3][3]; w_pw [pw_k][c][1][1]; scale_dw, shift_dw fp32 [c];
 *   scale_pw, shift_pw fp32 [pw_k]; bias_pw fp32 [pw_k] or NULL; residual [n][pw_k][oh][ow] or
 *   NULL; y [n][pw_k][oh][ow], written completely.  All device pointers; x, w_pw, residual and y
 *   must be 16-byte aligned (TVG_ERR_UNSUPPORTED otherwise).
 * Two forms compute this, and the workspace argument selects between them:
 *   - with a workspace of at least tvg_dwpw_workspace_size() bytes (256-byte aligned): the two
 *     kernels back to back, t held in the workspace.  This is the faster form on every shape
 *     measured so far and what a caller with memory to spare should use.
 *   - with workspace == NULL: ONE kernel, for callers that cannot spare the intermediate; t is
 *     produced in LDS as the pixel operand of the 1x1 stage and never reaches memory.  Exists
 *     for bf16, stride 1, c a multiple of 32 and maps whose rows are short enough
 *     (tvg_dwpw_one_kernel() says whether a problem qualifies); TVG_ERR_WORKSPACE otherwise.
 *     This form also needs w_dw 4-byte aligned (TVG_ERR_UNSUPPORTED otherwise).
 * A workspace that is too small or misaligned is TVG_ERR_WORKSPACE.  Both forms follow the
 * definition above (t rounded to dtype between the stages).
 */
tvg_status tvg_dwpw_workspace_size(const tvg_conv_desc *dw_desc, int32_t pw_k, size_t *bytes);
/* *available = 1 if the one-kernel form exists for this problem, else 0.  Host only. */
tvg_status tvg_dwpw_one_kernel(const tvg_conv_desc *dw_desc, int32_t pw_k, int32_t *available);
tvg_status tvg_dwpw_fused(const tvg_conv_desc *dw_desc, int32_t pw_k, uint32_t pw_flags,
                          const void *x, const void *w_dw, const float *scale_dw,
                          const float *shift_dw, const void *w_pw, const float *scale_pw,
                          const float *shift_pw, const float *bias_pw, const void *residual,
                          void *y, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * 3x3 stride-2 pad-1 max-pool, NCHW, padded taps ignored.  Support operator
 * for running the ResNet-18 body (the stem's 112x112 output must become the
 * 56x56 input of Table 2's C2).  x [n][c][h][w] -> y [n][c][oh][ow] with
 * oh = floor((h - 1) / 2) + 1.  dtype as in tvg_dtype.
 */
tvg_status tvg_maxpool2d_3x3s2(int32_t n, int32_t c, int32_t h, int32_t w, int32_t dtype,
                               const void *x, void *y, void *hip_stream);

/*
 * Static memory plan (TVM paper Section 3: after fusion a static memory planning pass
 * pre-allocates the memory of every intermediate tensor).  Host-only.  Given each tensor's size
 * and the launches during which it must stay intact - from the launch that writes it
 * (first_step) to the last launch that reads it (last_step), both inclusive - the call assigns
 * byte offsets in one arena so that tensors whose intervals intersect never overlap (so an
 * operator's output never overlaps its own inputs) while tensors that are never alive together
 * share memory.  Offsets are multiples of 256.  Greedy: largest tensor first, lowest offset that
 * is free over its whole interval; deterministic.
 *   tensors  host, `count` entries (1 <= count <= 4096; bytes >= 1; 0 <= first_step <= last_step)
 *   offsets  host, `count` entries, written
 *   arena_bytes  host, written: the arena's size (a multiple of 256)
 * Returns TVG_ERR_NULL, TVG_ERR_BAD_SHAPE (count or an entry out of range) or TVG_OK.
 */
typedef struct tvg_tensor_life {
    uint64_t bytes;
    int32_t first_step;
    int32_t last_step;
} tvg_tensor_life;
tvg_status tvg_plan_arena(const tvg_tensor_life *tensors, int32_t count, uint64_t *offsets,
                          uint64_t *arena_bytes);

/*
 * Tuning (TVM paper Section 5: the schedule of an operator is chosen per shape by measurement).
 * The tile shape of a kernel - output channels x pixels per workgroup - is its main knob; the
 * library picks one by a measured rule, and a caller that has timed the alternatives on its own
 * problem can fix the choice.  Host-only calls, safe to use from several threads.
 *
 * tvg_conv2d_set_tile: from now on plan this exact problem (every descriptor field but flags)
 * with tiles of mt x nt (the problem's other knobs, see tvg_conv2d_set_knobs, stay as they are),
 * one of 64x512, 64x256, 128x256, 128x128, 64x128, 128x64, 64x64 (anything else:
 * TVG_ERR_UNSUPPORTED; 64x512 exists in the single-stage 3x3 kernel for stride 1 and rows of 8n
 * pixels, 128x256 in the pipelined 3x3 kernel); mt = nt = 0 forgets the problem.  A tile shape that the problem's kernel
 * cannot use makes the call fall back to the generic kernel, which is correct but slow: time
 * before you fix.  At most 1024 problems are remembered.
 * tvg_conv2d_get_plan: which kernel and tile shape a call with this descriptor would use now
 * (alignment of the pointers aside).  kernel, mt, nt are host pointers.
 */
typedef enum {
    TVG_KERNEL_GENERIC = 0,        /* implicit GEMM with gathered operands, any shape      */
    TVG_KERNEL_3X3 = 1,            /* bf16 3x3, input patch in LDS, one stage              */
    TVG_KERNEL_3X3_PIPELINED = 2,  /* bf16 3x3, two LDS stages, software-pipelined         */
    TVG_KERNEL_STEM = 3,           /* bf16 7x7 or 3x3 stride 2, few input channels (mt 64|32) */
    TVG_KERNEL_1X1 = 4,            /* bf16 1x1                                             */
    TVG_KERNEL_F32_SMALL = 5,      /* fp32 1x1 / 3x3 / 7x7 stem of launch-bound problems (mt = nt = 32 or 16; stem 32 x 64) */
    TVG_KERNEL_1X1_DEEP = 6        /* bf16 1x1 stride 1, reductions of 128 n channels       */
} tvg_kernel;
tvg_status tvg_conv2d_set_tile(const tvg_conv_desc *desc, int32_t mt, int32_t nt);
tvg_status tvg_conv2d_get_plan(const tvg_conv_desc *desc, int32_t *kernel, int32_t *mt, int32_t *nt);

/*
 * The whole schedule space of a problem (TVM paper Section 5.1: a schedule template with knobs
 * per operator; Section 5.3: the space is explored by measurement).  Every knob is a set of
 * compiled kernel instances or a launch parameter; 0 leaves a knob to the library's rule.
 *   mt, nt      workgroup tile, as for tvg_conv2d_set_tile (with it the wave tile: 64x64, 32x64,
 *               64x32 or 32x32 outputs per wave)
 *               128 x 256 (and 128 x 128 with stages = 2) name the pipelined 3x3 kernel's
 *               channel-split variant: two groups of four waves own 64 output channels each and
 *               share one patch (at most one workgroup per CU, more than 64 output channels)
 *   stages      bf16 3x3: 1 = the single-stage kernel, 2 = the software-pipelined kernel with two
 *               LDS stages (from 64 input channels on, a multiple of 32; 64-channel tiles)
 *               bf16 1x1, stride 1: 2 = the kernel for deep reductions (c a multiple of 128, maps
 *               of 4n pixels: wide pixel loads, two steps of 64 channels in flight)
 *   split_k     partitions of the reduction.  Generic kernel (fp32, odd shapes): 1..32 partitions
 *               across workgroups, summed by a second launch - tvg_conv2d_workspace_size follows
 *               the knob.  Pipelined 3x3: 1 or 2 groups of four waves inside one workgroup that
 *               take alternate input-channel chunks and add their accumulators through LDS
 *               (grids of at most one workgroup per CU, stride 1, 128- or 256-pixel tiles, input
 *               channels a multiple of 64)
 *   lds_pitch   pipelined 3x3, stride 1: 1 = patch rows of W + 2 words, 2 = rows of W + 16 words
 *               (operand reads free of bank conflicts across row ends, more LDS)
 *   row_loads   pipelined 3x3, odd rows of at most 7 pixels: 1 = element loads, 2 = one 16-byte
 *               load per row and channel from the aligned address below the row, shifted into place
 * tvg_conv2d_set_knobs: fix the knobs of this exact problem (every descriptor field but flags);
 * knobs == NULL or all zero forgets the problem.  Values outside the ranges above are
 * TVG_ERR_UNSUPPORTED.  A combination the problem's kernel cannot use (say, two stages that do
 * not fit the LDS) makes the call fall back - to the other 3x3 kernel or to the generic kernel,
 * correct but possibly slow - so time before you fix; tvg_conv2d_get_knobs tells what a call
 * would really use now (0 where a knob does not apply to the kernel that runs).
 */
typedef struct {
    int32_t mt, nt, stages, split_k, lds_pitch, row_loads;
} tvg_conv_knobs;
tvg_status tvg_conv2d_set_knobs(const tvg_conv_desc *desc, const tvg_conv_knobs *knobs);
tvg_status tvg_conv2d_get_knobs(const tvg_conv_desc *desc, tvg_conv_knobs *knobs);

/*
 * Measurement probes (not operators): what the GPU sustains, to be timed by the caller beside
 * the operators in the same run, so that a fraction of the data-sheet peak can be read next to a
 * fraction of what is achievable (the paper's Section 6 evaluates against measured baselines on
 * the same device; these are the device's own ceilings).
 * tvg_probe_copy: dst[0..bytes) = src[0..bytes) with 16-byte accesses; src, dst device pointers,
 *   16-byte aligned, bytes a positive multiple of 16, the ranges disjoint.  Algorithmic traffic:
 *   2 * bytes.
 * tvg_probe_mfma: `workgroups` workgroups of four waves each issue iters * 4 matrix instruction
 *   groups on register operands (TVG_BF16: v_mfma_f32_32x32x16_bf16; TVG_F32: four
 *   v_mfma_f32_32x32x2_f32); out is a device buffer of workgroups * 256 floats (written so that the
 *   loop is live), *flops (host) receives the floating-point operations the launch performs.
 */
tvg_status tvg_probe_copy(const void *src, void *dst, size_t bytes, void *hip_stream);
tvg_status tvg_probe_mfma(int32_t dtype, int32_t iters, int32_t workgroups, float *out,
                          double *flops, void *hip_stream);

/* Static, NUL-terminated description of a status code (never NULL). */
const char *tvg_status_string(tvg_status status);

/* Library version as major*10000 + minor*100 + patch. */
int tvg_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TVG_H */
