// C ABI of libtvg: argument validation (host only, before any device call),
// planning and dispatch to the kernel launchers.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <initializer_list>
#include <utility>
#include <mutex>
#include <vector>
#include "tvg_internal.h"

namespace {

using tvg::ConvProblem;

const int64_t kMaxElems = (int64_t)1 << 31;

// Product of positive extents, saturating at kMaxElems (every factor is below 2^31, so a
// partial product below 2^31 times the next factor stays inside 64 bits).
int64_t count_elems(std::initializer_list<int64_t> extents)
{
    int64_t n = 1;
    for (int64_t e : extents) {
        n *= e;
        if (n >= kMaxElems) return kMaxElems;
    }
    return n;
}

tvg_status make_problem(const tvg_conv_desc *d, bool depthwise, ConvProblem *out)
{
    if (!d) return TVG_ERR_NULL;
    if (d->n < 1 || d->c < 1 || d->h < 1 || d->w < 1 || d->k < 1 || d->r < 1 || d->s < 1)
        return TVG_ERR_BAD_SHAPE;
    if (d->stride_h < 1 || d->stride_w < 1 || d->stride_h > 8 || d->stride_w > 8)
        return TVG_ERR_BAD_SHAPE;
    // The filter extent is bounded before anything is computed from the padding: with r, s <= 16
    // and pad < r every sum below stays far inside the int range (h, w < 2^31 - 32 is implied by
    // the element-count limit, checked in 64 bits).
    if (d->r > 16 || d->s > 16) return TVG_ERR_UNSUPPORTED;
    if (d->pad_h < 0 || d->pad_w < 0 || d->pad_h >= d->r || d->pad_w >= d->s)
        return TVG_ERR_BAD_SHAPE;
    if ((int64_t)d->h + 2 * d->pad_h < d->r || (int64_t)d->w + 2 * d->pad_w < d->s)
        return TVG_ERR_BAD_SHAPE;
    if (d->dtype != TVG_F32 && d->dtype != TVG_BF16) return TVG_ERR_UNSUPPORTED;
    if (d->flags & ~(uint32_t)(TVG_RELU | TVG_STREAM_OUT)) return TVG_ERR_UNSUPPORTED;
    if (count_elems({d->n, d->c, d->h, d->w}) >= kMaxElems) return TVG_ERR_UNSUPPORTED;
    if (depthwise) {
        if (d->k != d->c) return TVG_ERR_BAD_SHAPE;
        if (d->r != 3 || d->s != 3) return TVG_ERR_UNSUPPORTED;
        if (d->stride_h != d->stride_w || d->stride_h > 2) return TVG_ERR_UNSUPPORTED;
        if (d->pad_h != 1 || d->pad_w != 1) return TVG_ERR_UNSUPPORTED;
        // one band of input rows (4 output rows) of one plane must fit 64 KB of LDS as fp32
        if ((int64_t)(3 * d->stride_h + 3) * ((int64_t)d->w + 2) > tvg::kDwBandFloats)
            return TVG_ERR_UNSUPPORTED;
    }
    ConvProblem p;
    p.N = d->n; p.IC = d->c; p.H = d->h; p.W = d->w; p.OC = d->k; p.R = d->r; p.S = d->s;
    p.sh = d->stride_h; p.sw = d->stride_w; p.ph = d->pad_h; p.pw = d->pad_w;
    const int64_t oh = ((int64_t)d->h + 2 * d->pad_h - d->r) / d->stride_h + 1;
    const int64_t ow = ((int64_t)d->w + 2 * d->pad_w - d->s) / d->stride_w + 1;
    if (oh >= kMaxElems || ow >= kMaxElems) return TVG_ERR_UNSUPPORTED;
    p.OH = (int)oh;
    p.OW = (int)ow;
    const int64_t ny = count_elems({d->n, d->k, p.OH, p.OW});
    const int64_t nw = count_elems({d->k, depthwise ? 1 : d->c, d->r, d->s});
    if (ny >= kMaxElems || nw >= kMaxElems) return TVG_ERR_UNSUPPORTED;
    p.K = (depthwise ? 1 : d->c) * d->r * d->s;
    p.npix = d->n * p.OH * p.OW;
    p.dtype = d->dtype;
    p.relu = (d->flags & TVG_RELU) ? 1 : 0;
    p.stream_out = (d->flags & TVG_STREAM_OUT) ? 1 : 0;
    *out = p;
    return TVG_OK;
}

// Problems whose tile shape a caller has fixed (tvg_conv2d_set_tile): a short list under a
// mutex - planning reads it on every call, a tuner writes it a few times per shape.
struct TileEntry {
    int key[12];
    tvg::Knobs knobs;
};
std::mutex g_tile_mutex;
std::vector<TileEntry> g_tiles;
constexpr size_t kMaxTileEntries = 1024;

void tile_key(const ConvProblem &p, int (&key)[12])
{
    const int k[12] = {p.N, p.IC, p.H, p.W, p.OC, p.R, p.S, p.sh, p.sw, p.ph, p.pw, p.dtype};
    memcpy(key, k, sizeof(k));
}

// Everything planning derives from a problem, computed once per distinct problem: which
// kernel takes it and with what launch shape.  The descriptor's flags do not enter (no plan
// depends on them).  A short list under a mutex, scanned linearly; tvg_conv2d_set_tile empties
// it.  The launch-bound batch-1 layers spend 1-5 us per call in planning otherwise.
struct Dispatch {
    int key[12];
    bool patch_shape, stem_shape, pw_shape, pwd_shape, f32_shape;
    tvg::Patch3x3Plan patch;
    tvg::StemPlan stem;
    tvg::Pw1x1Plan pw;
    tvg::PwDeepPlan pwd;            // the deep-reduction 1x1 kernel, where its rule (or a knob) picks it
    tvg::F32SmallPlan f32;
    tvg::ConvPlan generic;          // the generic kernel's plan, reduction split allowed
    tvg::ConvPlan generic_single;   // the same in a single pass (no workspace)
};
std::mutex g_dispatch_mutex;
std::vector<Dispatch> g_dispatch;
size_t g_dispatch_next = 0;
constexpr size_t kMaxDispatchEntries = 256;

Dispatch dispatch_for(const ConvProblem &p)
{
    int key[12];
    tile_key(p, key);
    {
        std::lock_guard<std::mutex> lock(g_dispatch_mutex);
        for (const Dispatch &d : g_dispatch)
            if (memcmp(d.key, key, sizeof(key)) == 0) return d;
    }
    Dispatch d{};
    memcpy(d.key, key, sizeof(key));
    d.patch_shape = tvg::plan_conv3x3_patch(p, &d.patch);
    d.stem_shape = !d.patch_shape && tvg::plan_conv7x7s2_stem(p, &d.stem);
    d.pw_shape = !d.patch_shape && !d.stem_shape && tvg::plan_conv1x1(p, &d.pw);
    {
        // stages knob of a 1x1 problem: 2 = the deep-reduction kernel.  No rule picks it: measured at
        // batch 32 / 64 over thirteen MobileNet and ResNet-50 pointwise shapes it takes 1.15-1.5 times
        // as long as the general kernel (512 -> 512 at 14x14: 15.7 against 12.5 us).
        const int want = tvg::forced_knobs(p).stages;
        d.pwd_shape = d.pw_shape && want == 2 && tvg::plan_conv1x1_deep(p, &d.pwd);
    }
    d.f32_shape = tvg::plan_conv_f32_small(p, &d.f32);
    d.generic = tvg::plan_conv(p, true);
    d.generic_single = tvg::plan_conv(p, false);
    std::lock_guard<std::mutex> lock(g_dispatch_mutex);
    if (g_dispatch.size() < kMaxDispatchEntries) g_dispatch.push_back(d);
    else g_dispatch[g_dispatch_next++ % kMaxDispatchEntries] = d;     // replace the oldest slot
    return d;
}

void forget_dispatch()
{
    std::lock_guard<std::mutex> lock(g_dispatch_mutex);
    g_dispatch.clear();
}

// Scratch memory of tvg_conv2d_fused_static: the split-reduction partials of the generic kernel
// live in this array instead of a caller's workspace.  Every GPU that loads the library holds
// its own copy at its own address until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress; kernels are given the resolved device address.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];      // device address of `scratch` per device, once resolved

// The current device's copy of `scratch`; resolved on the first call per device.
tvg_status static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TVG_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return TVG_ERR_LAUNCH;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return TVG_OK;
}

}  // namespace

namespace tvg {

Knobs forced_knobs(const ConvProblem &p)
{
    int key[12];
    tile_key(p, key);
    std::lock_guard<std::mutex> lock(g_tile_mutex);
    for (const TileEntry &e : g_tiles)
        if (memcmp(e.key, key, sizeof(key)) == 0) return e.knobs;
    return Knobs{0, 0, 0, 0, 0, 0};
}

}  // namespace tvg

extern "C" {

// Stores, replaces or (knobs all zero) forgets the problem's entry in the knob table.
static tvg_status store_knobs(const ConvProblem &p, const tvg::Knobs &k)
{
    const bool clear = !k.mt && !k.nt && !k.stages && !k.split_k && !k.lds_pitch && !k.row_loads;
    int key[12];
    tile_key(p, key);
    forget_dispatch();                     // plans made under the old table are stale
    std::lock_guard<std::mutex> lock(g_tile_mutex);
    for (size_t i = 0; i < g_tiles.size(); ++i)
        if (memcmp(g_tiles[i].key, key, sizeof(key)) == 0) {
            if (clear) g_tiles.erase(g_tiles.begin() + (long)i);
            else g_tiles[i].knobs = k;
            return TVG_OK;
        }
    if (clear) return TVG_OK;
    if (g_tiles.size() >= kMaxTileEntries) return TVG_ERR_UNSUPPORTED;
    TileEntry e;
    memcpy(e.key, key, sizeof(key));
    e.knobs = k;
    g_tiles.push_back(e);
    return TVG_OK;
}

static bool known_tile(int mt, int nt)
{
    return (mt == 64 && (nt == 512 || nt == 256 || nt == 128 || nt == 64)) || (mt == 128 && (nt == 256 || nt == 128 || nt == 64));
}

tvg_status tvg_conv2d_set_tile(const tvg_conv_desc *desc, int32_t mt, int32_t nt)
{
    ConvProblem p;
    tvg_status st = make_problem(desc, false, &p);
    if (st != TVG_OK) return st;
    if (!(mt == 0 && nt == 0) && !known_tile(mt, nt)) return TVG_ERR_UNSUPPORTED;
    tvg::Knobs k = tvg::forced_knobs(p);      // the other knobs stay as they are
    k.mt = mt;
    k.nt = nt;
    return store_knobs(p, k);
}

tvg_status tvg_conv2d_set_knobs(const tvg_conv_desc *desc, const tvg_conv_knobs *knobs)
{
    ConvProblem p;
    tvg_status st = make_problem(desc, false, &p);
    if (st != TVG_OK) return st;
    if (!knobs) return store_knobs(p, tvg::Knobs{0, 0, 0, 0, 0, 0});
    if (!((knobs->mt == 0 && knobs->nt == 0) || known_tile(knobs->mt, knobs->nt))) return TVG_ERR_UNSUPPORTED;
    if (knobs->stages < 0 || knobs->stages > 2 || knobs->split_k < 0 || knobs->split_k > 32 ||
        knobs->lds_pitch < 0 || knobs->lds_pitch > 2 || knobs->row_loads < 0 || knobs->row_loads > 2)
        return TVG_ERR_UNSUPPORTED;
    return store_knobs(p, tvg::Knobs{knobs->mt, knobs->nt, knobs->stages, knobs->split_k,
                                     knobs->lds_pitch, knobs->row_loads});
}

tvg_status tvg_conv2d_get_knobs(const tvg_conv_desc *desc, tvg_conv_knobs *knobs)
{
    if (!knobs) return TVG_ERR_NULL;
    ConvProblem p;
    tvg_status st = make_problem(desc, false, &p);
    if (st != TVG_OK) return st;
    const Dispatch d = dispatch_for(p);
    tvg_conv_knobs k = {0, 0, 0, 0, 0, 0};
    if (d.patch_shape) {
        k.mt = d.patch.mt;
        k.nt = d.patch.nt;
        k.stages = d.patch.dbuf ? 2 : 1;
        if (d.patch.dbuf) {
            k.split_k = d.patch.kg == 2 ? 2 : 1;       // (kg 3 names the channel split: mt = 128)
            if (p.sh == 1) k.lds_pitch = d.patch.pws == p.W + 2 ? 1 : 2;
            if (p.W % 2 != 0 && p.W <= 7 && p.sh == 1) k.row_loads = d.patch.px == 8 ? 2 : 1;
        }
    } else if (d.stem_shape) {
        k.mt = d.stem.mt;
        k.nt = 256;
        k.stages = 1;
    } else if (d.pwd_shape) {
        k.mt = 64;
        k.nt = 128;
        k.stages = 2;
    } else if (d.pw_shape) {
        k.mt = d.pw.mt;
        k.nt = d.pw.nt;
        k.stages = 1;
    } else if (d.f32_shape) {
        k.stages = 1;
        k.split_k = d.f32.nw * d.f32.ksplit;     // waves of a workgroup x slices across workgroups
    } else {
        k.mt = d.generic.mt;
        k.nt = d.generic.nt;
        k.stages = 2;
        k.split_k = d.generic.splits;
    }
    *knobs = k;
    return TVG_OK;
}

tvg_status tvg_conv2d_get_plan(const tvg_conv_desc *desc, int32_t *kernel, int32_t *mt, int32_t *nt)
{
    if (!kernel || !mt || !nt) return TVG_ERR_NULL;
    ConvProblem p;
    tvg_status st = make_problem(desc, false, &p);
    if (st != TVG_OK) return st;
    const Dispatch d = dispatch_for(p);
    if (d.patch_shape) {
        *kernel = d.patch.dbuf ? TVG_KERNEL_3X3_PIPELINED : TVG_KERNEL_3X3;
        *mt = d.patch.mt;
        *nt = d.patch.nt;
    } else if (d.stem_shape) {
        *kernel = TVG_KERNEL_STEM;
        *mt = d.stem.mt;
        *nt = 256;
    } else if (d.pwd_shape) {
        *kernel = TVG_KERNEL_1X1_DEEP;
        *mt = 64;
        *nt = 128;
    } else if (d.pw_shape) {
        *kernel = TVG_KERNEL_1X1;
        *mt = d.pw.mt;
        *nt = d.pw.nt;
    } else if (d.f32_shape) {
        *kernel = TVG_KERNEL_F32_SMALL;
        *mt = d.f32.stem ? 32 : d.f32.tile;
        *nt = d.f32.stem ? 64 : d.f32.tile;
    } else {
        *kernel = TVG_KERNEL_GENERIC;
        *mt = d.generic.mt;
        *nt = d.generic.nt;
    }
    return TVG_OK;
}


tvg_status tvg_conv2d_workspace_size(const tvg_conv_desc *desc, size_t *bytes)
{
    if (!bytes) return TVG_ERR_NULL;
    ConvProblem p;
    tvg_status st = make_problem(desc, false, &p);
    if (st != TVG_OK) return st;
    const Dispatch d = dispatch_for(p);
    const bool single_pass = d.patch_shape || d.stem_shape || d.pw_shape;
    *bytes = single_pass ? 0 : d.f32_shape ? d.f32.workspace_bytes : d.generic.workspace_bytes;
    return TVG_OK;
}

tvg_status tvg_dwconv2d_workspace_size(const tvg_conv_desc *desc, size_t *bytes)
{
    if (!bytes) return TVG_ERR_NULL;
    ConvProblem p;
    tvg_status st = make_problem(desc, true, &p);
    if (st != TVG_OK) return st;
    *bytes = 0;
    return TVG_OK;
}

tvg_status tvg_conv2d_fused(const tvg_conv_desc *desc, const void *x, const void *w,
                            const float *scale, const float *shift, const float *bias,
                            const void *residual, void *y, void *workspace,
                            size_t workspace_bytes, void *hip_stream)
{
    ConvProblem p;
    tvg_status st = make_problem(desc, false, &p);
    if (st != TVG_OK) return st;
    if (!x || !w || !scale || !shift || !y) return TVG_ERR_NULL;
    tvg::ConvPointers ptr{x, w, scale, shift, bias, residual, y, static_cast<float *>(workspace)};
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const Dispatch d = dispatch_for(p);
    if (d.patch_shape && tvg::conv3x3_patch_pointers_ok(ptr))
        return tvg::launch_conv3x3_patch(p, d.patch, ptr, stream);
    if (d.stem_shape && tvg::conv7x7s2_stem_pointers_ok(ptr))
        return tvg::launch_conv7x7s2_stem(p, d.stem, ptr, stream);
    if (d.pwd_shape && tvg::conv1x1_deep_pointers_ok(ptr)) return tvg::launch_conv1x1_deep(p, d.pwd, ptr, stream);
    if (d.pw_shape && tvg::conv1x1_pointers_ok(ptr)) return tvg::launch_conv1x1(p, d.pw, ptr, stream);
    const auto workspace_short = [&](size_t need) {
        return need > 0 && (!workspace || workspace_bytes < need ||
                            reinterpret_cast<uintptr_t>(workspace) % 256 != 0);
    };
    if (d.f32_shape && tvg::conv_f32_small_pointers_ok(ptr)) {
        if (workspace_short(d.f32.workspace_bytes)) return TVG_ERR_WORKSPACE;
        return tvg::launch_conv_f32_small(p, d.f32, ptr, stream);
    }
    // A problem shaped for a specialised kernel reported a zero workspace; if its pointers
    // rule that kernel out, the generic kernel runs it in a single pass over the reduction.
    // (an fp32 problem whose x is not 16-byte aligned: the generic kernel, within the workspace
    // that the query reported for the fp32 kernel if that is all the caller has)
    const tvg::ConvPlan &plan =
        (d.patch_shape || d.stem_shape || d.pw_shape ||
         (d.f32_shape && workspace_short(d.generic.workspace_bytes))) ? d.generic_single : d.generic;
    if (workspace_short(plan.workspace_bytes)) return TVG_ERR_WORKSPACE;
    return tvg::launch_conv_igemm(p, plan, ptr, stream);
}

tvg_status tvg_conv2d_fused_dual(const tvg_conv_desc *desc, int32_t k1, uint32_t flags2,
                                 const void *x, const void *w, const float *scale,
                                 const float *shift, const float *bias, const void *residual1,
                                 void *y1, void *y2, void *hip_stream)
{
    ConvProblem p;
    tvg_status st = make_problem(desc, false, &p);
    if (st != TVG_OK) return st;
    if (k1 < 1 || k1 >= p.OC) return TVG_ERR_BAD_SHAPE;
    if (flags2 & ~(uint32_t)(TVG_RELU | TVG_STREAM_OUT | TVG_CENTRE_TAP_ONLY)) return TVG_ERR_UNSUPPORTED;
    if (!x || !w || !scale || !shift || !y1 || !y2) return TVG_ERR_NULL;
    tvg::Patch3x3Plan plan;
    if (!tvg::plan_conv3x3_patch(p, &plan, k1)) return TVG_ERR_UNSUPPORTED;
    const tvg::ConvPointers ptr{x, w, scale, shift, bias, residual1, y1, nullptr};
    if (!tvg::conv3x3_patch_pointers_ok(ptr)) return TVG_ERR_UNSUPPORTED;
    const tvg::DualHead dual{k1, (int)((flags2 & TVG_RELU ? 1 : 0) | (flags2 & TVG_STREAM_OUT ? 2 : 0)),
                             (flags2 & TVG_CENTRE_TAP_ONLY) ? 1 : 0, y2};
    return tvg::launch_conv3x3_patch(p, plan, ptr, static_cast<hipStream_t>(hip_stream), &dual);
}

tvg_status tvg_conv2d_fused_static(const tvg_conv_desc *desc, const void *x, const void *w,
                                   const float *scale, const float *shift, const float *bias,
                                   const void *residual, void *y, void *hip_stream)
{
    size_t need = 0;
    tvg_status st = tvg_conv2d_workspace_size(desc, &need);       // validates the descriptor
    if (st != TVG_OK) return st;
    if (!x || !w || !scale || !shift || !y) return TVG_ERR_NULL;
    if (need > kStaticScratchBytes) return TVG_ERR_WORKSPACE;     // before any device call
    void *ws = nullptr;
    if (need > 0) {
        st = static_scratch(&ws);
        if (st != TVG_OK) return st;
    }
    return tvg_conv2d_fused(desc, x, w, scale, shift, bias, residual, y, ws, need, hip_stream);
}

size_t tvg_static_scratch_bytes(void) { return kStaticScratchBytes; }

tvg_status tvg_conv2d_prepack_size(const tvg_conv_desc *desc, size_t *packed_bytes, size_t *workspace_bytes)
{
    if (!packed_bytes || !workspace_bytes) return TVG_ERR_NULL;
    ConvProblem p;
    tvg_status st = make_problem(desc, false, &p);
    if (st != TVG_OK) return st;
    tvg::WinoPlan plan;
    if (!tvg::plan_conv3x3_winograd(p, &plan)) return TVG_ERR_UNSUPPORTED;
    *packed_bytes = plan.u_bytes;
    *workspace_bytes = plan.v_bytes;
    return TVG_OK;
}

tvg_status tvg_conv2d_prepack(const tvg_conv_desc *desc, const void *w, void *packed,
                              size_t packed_bytes, void *hip_stream)
{
    ConvProblem p;
    tvg_status st = make_problem(desc, false, &p);
    if (st != TVG_OK) return st;
    tvg::WinoPlan plan;
    if (!tvg::plan_conv3x3_winograd(p, &plan)) return TVG_ERR_UNSUPPORTED;
    if (!w || !packed) return TVG_ERR_NULL;
    if (packed_bytes < plan.u_bytes || reinterpret_cast<uintptr_t>(packed) % 16 != 0) return TVG_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(w) % 16 != 0) return TVG_ERR_UNSUPPORTED;
    return tvg::launch_winograd_prepack(p, w, packed, static_cast<hipStream_t>(hip_stream));
}

tvg_status tvg_conv2d_fused_prepacked(const tvg_conv_desc *desc, const void *x, const void *packed,
                                      const float *scale, const float *shift, const float *bias,
                                      const void *residual, void *y, void *workspace,
                                      size_t workspace_bytes, void *hip_stream)
{
    ConvProblem p;
    tvg_status st = make_problem(desc, false, &p);
    if (st != TVG_OK) return st;
    tvg::WinoPlan plan;
    if (!tvg::plan_conv3x3_winograd(p, &plan)) return TVG_ERR_UNSUPPORTED;
    if (!x || !packed || !scale || !shift || !y) return TVG_ERR_NULL;
    if (!workspace || workspace_bytes < plan.v_bytes || reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
        return TVG_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(packed) % 16 != 0 || reinterpret_cast<uintptr_t>(x) % 2 != 0 ||
        reinterpret_cast<uintptr_t>(y) % 2 != 0 || reinterpret_cast<uintptr_t>(residual) % 2 != 0)
        return TVG_ERR_UNSUPPORTED;
    const tvg::ConvPointers ptr{x, nullptr, scale, shift, bias, residual, y, static_cast<float *>(workspace)};
    return tvg::launch_conv3x3_winograd(p, plan, packed, ptr, static_cast<hipStream_t>(hip_stream));
}

tvg_status tvg_dwconv2d_fused(const tvg_conv_desc *desc, const void *x, const void *w,
                              const float *scale, const float *shift, const float *bias,
                              const void *residual, void *y, void *workspace,
                              size_t workspace_bytes, void *hip_stream)
{
    (void)workspace;
    (void)workspace_bytes;
    ConvProblem p;
    tvg_status st = make_problem(desc, true, &p);
    if (st != TVG_OK) return st;
    if (!x || !w || !scale || !shift || !y) return TVG_ERR_NULL;
    tvg::ConvPointers ptr{x, w, scale, shift, bias, residual, y, nullptr};
    return tvg::launch_dwconv3x3(p, ptr, static_cast<hipStream_t>(hip_stream));
}

// The 1x1 stage of the block as a problem of its own: reads the depthwise stage's output.
static tvg_status make_pw_problem(const tvg_conv_desc *dw_desc, const ConvProblem &dw, int32_t pw_k,
                                  uint32_t pw_flags, ConvProblem *pw)
{
    if (pw_k < 1) return TVG_ERR_BAD_SHAPE;
    tvg_conv_desc d = *dw_desc;
    d.h = dw.OH; d.w = dw.OW; d.k = pw_k; d.r = d.s = 1;
    d.stride_h = d.stride_w = 1; d.pad_h = d.pad_w = 0;
    d.flags = pw_flags;
    return make_problem(&d, false, pw);
}

static size_t dwpw_workspace(const ConvProblem &dw, const ConvProblem &pw)
{
    const size_t elem = dw.dtype == TVG_BF16 ? 2 : 4;
    size_t bytes = ((size_t)dw.N * dw.IC * dw.OH * dw.OW * elem + 255) & ~(size_t)255;
    tvg::Pw1x1Plan p1;
    if (!tvg::plan_conv1x1(pw, &p1)) bytes += tvg::plan_conv(pw).workspace_bytes;   // split-K scratch
    return bytes;
}

tvg_status tvg_dwpw_workspace_size(const tvg_conv_desc *dw_desc, int32_t pw_k, size_t *bytes)
{
    if (!bytes) return TVG_ERR_NULL;
    ConvProblem dw, pw;
    tvg_status st = make_problem(dw_desc, true, &dw);
    if (st != TVG_OK) return st;
    st = make_pw_problem(dw_desc, dw, pw_k, 0, &pw);
    if (st != TVG_OK) return st;
    *bytes = dwpw_workspace(dw, pw);
    return TVG_OK;
}

tvg_status tvg_dwpw_one_kernel(const tvg_conv_desc *dw_desc, int32_t pw_k, int32_t *available)
{
    if (!available) return TVG_ERR_NULL;
    ConvProblem dw, pw;
    tvg_status st = make_problem(dw_desc, true, &dw);
    if (st != TVG_OK) return st;
    st = make_pw_problem(dw_desc, dw, pw_k, 0, &pw);
    if (st != TVG_OK) return st;
    tvg::DwPwPlan plan;
    *available = tvg::plan_dwpw(dw, pw.OC, &plan) ? 1 : 0;
    return TVG_OK;
}

tvg_status tvg_dwpw_fused(const tvg_conv_desc *dw_desc, int32_t pw_k, uint32_t pw_flags,
                          const void *x, const void *w_dw, const float *scale_dw,
                          const float *shift_dw, const void *w_pw, const float *scale_pw,
                          const float *shift_pw, const float *bias_pw, const void *residual,
                          void *y, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    ConvProblem dw, pw;
    tvg_status st = make_problem(dw_desc, true, &dw);
    if (st != TVG_OK) return st;
    st = make_pw_problem(dw_desc, dw, pw_k, pw_flags, &pw);
    if (st != TVG_OK) return st;
    if (!x || !w_dw || !scale_dw || !shift_dw || !w_pw || !scale_pw || !shift_pw || !y)
        return TVG_ERR_NULL;
    for (const void *q : {x, w_pw, residual, (const void *)y})
        if (reinterpret_cast<uintptr_t>(q) % 16 != 0) return TVG_ERR_UNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    tvg::DwPwPlan plan;
    if (!workspace && workspace_bytes == 0) {          // the caller asks for the one-kernel form
        if (!tvg::plan_dwpw(dw, pw.OC, &plan)) return TVG_ERR_WORKSPACE;
        const tvg::DwPwPointers ptr{x, w_dw, scale_dw, shift_dw, w_pw, scale_pw, shift_pw, bias_pw,
                                    residual, y};
        return tvg::launch_dwpw(dw, pw.OC, pw.relu, pw.stream_out, plan, ptr, stream);
    }
    const size_t need = dwpw_workspace(dw, pw);
    if (!workspace || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
        return TVG_ERR_WORKSPACE;
    const size_t elem = dw.dtype == TVG_BF16 ? 2 : 4;
    const size_t t_bytes = ((size_t)dw.N * dw.IC * dw.OH * dw.OW * elem + 255) & ~(size_t)255;
    dw.stream_out = 0;                       // t is read by the next launch
    const tvg::ConvPointers dptr{x, w_dw, scale_dw, shift_dw, nullptr, nullptr, workspace, nullptr};
    st = tvg::launch_dwconv3x3(dw, dptr, stream);
    if (st != TVG_OK) return st;
    const tvg::ConvPointers pptr{workspace, w_pw, scale_pw, shift_pw, bias_pw, residual, y,
                                 reinterpret_cast<float *>(static_cast<char *>(workspace) + t_bytes)};
    tvg::Pw1x1Plan p1;
    if (tvg::plan_conv1x1(pw, &p1) && tvg::conv1x1_pointers_ok(pptr))
        return tvg::launch_conv1x1(pw, p1, pptr, stream);
    return tvg::launch_conv_igemm(pw, tvg::plan_conv(pw), pptr, stream);
}

tvg_status tvg_plan_arena(const tvg_tensor_life *tensors, int32_t count, uint64_t *offsets,
                          uint64_t *arena_bytes)
{
    if (!tensors || !offsets || !arena_bytes) return TVG_ERR_NULL;
    if (count < 1 || count > 4096) return TVG_ERR_BAD_SHAPE;
    for (int32_t i = 0; i < count; ++i)
        if (tensors[i].bytes < 1 || tensors[i].bytes > ((uint64_t)1 << 48) ||
            tensors[i].first_step < 0 || tensors[i].last_step < tensors[i].first_step)
            return TVG_ERR_BAD_SHAPE;
    const uint64_t kAlign = 256;
    std::vector<int32_t> order(count);
    for (int32_t i = 0; i < count; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        return tensors[a].bytes > tensors[b].bytes;          // ties keep their index order
    });
    std::vector<char> placed(count, 0);
    std::vector<std::pair<uint64_t, uint64_t>> busy;          // [begin, end) of conflicting tensors
    uint64_t arena = 0;
    for (int32_t oi = 0; oi < count; ++oi) {
        const int32_t t = order[oi];
        const uint64_t size = (tensors[t].bytes + kAlign - 1) / kAlign * kAlign;
        busy.clear();
        for (int32_t j = 0; j < count; ++j)
            if (placed[j] && tensors[j].first_step <= tensors[t].last_step &&
                tensors[t].first_step <= tensors[j].last_step) {
                const uint64_t sz = (tensors[j].bytes + kAlign - 1) / kAlign * kAlign;
                busy.emplace_back(offsets[j], offsets[j] + sz);
            }
        std::sort(busy.begin(), busy.end());
        uint64_t at = 0;                                      // lowest gap that holds `size`
        for (const auto &b : busy) {
            if (b.first >= at + size) break;
            if (b.second > at) at = b.second;
        }
        offsets[t] = at;
        placed[t] = 1;
        if (at + size > arena) arena = at + size;
    }
    *arena_bytes = arena;
    return TVG_OK;
}

tvg_status tvg_maxpool2d_3x3s2(int32_t n, int32_t c, int32_t h, int32_t w, int32_t dtype,
                               const void *x, void *y, void *hip_stream)
{
    if (n < 1 || c < 1 || h < 1 || w < 1) return TVG_ERR_BAD_SHAPE;
    if (dtype != TVG_F32 && dtype != TVG_BF16) return TVG_ERR_UNSUPPORTED;
    if (count_elems({n, c, h, w}) >= kMaxElems) return TVG_ERR_UNSUPPORTED;
    if (!x || !y) return TVG_ERR_NULL;
    return tvg::launch_maxpool3x3s2(n, c, h, w, dtype, x, y, static_cast<hipStream_t>(hip_stream));
}

const char *tvg_status_string(tvg_status status)
{
    switch (status) {
    case TVG_OK: return "ok";
    case TVG_ERR_NULL: return "a required pointer is NULL";
    case TVG_ERR_BAD_SHAPE: return "bad shape, stride or padding";
    case TVG_ERR_UNSUPPORTED: return "unsupported dtype, flag, size or kernel extent";
    case TVG_ERR_WORKSPACE: return "workspace missing or too small";
    case TVG_ERR_LAUNCH: return "HIP launch failed";
    }
    return "unknown status";
}

int tvg_version(void) { return 100; }

}  // extern "C"
