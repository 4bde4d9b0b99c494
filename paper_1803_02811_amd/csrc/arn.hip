// C ABI of the library (declared in include/arn.h): argument checks on the host,
// then a fixed sequence of kernel launches on the caller's stream.
#include <hip/hip_runtime.h>

#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "arn_gemm.h"
#include "arn_layout.h"
#include "arn_problems.h"
#include "arn_pv_head.h"
#include "arn_resident.h"
#include "arn_resident_conv.h"
#include "arn_conv_bwd.h"
#include "arn_conv23_fwd.h"
#include "arn_infer_fwd.h"
#include "arn_small_kernels.h"
#include "arn_update.h"

using namespace arn;

// Scratch memory of arn_policy_forward_static, the entry point for callers that cannot allocate: one copy per
// GPU the library runs on, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress (static_scratch_ptr below); kernels receive the device address that call returns.
static __device__ __align__(256) unsigned char scratch[ARN_STATIC_SCRATCH_BYTES];

namespace {

std::mutex g_lazy_mutex;   // guards the lazily filled per-device tables below (first calls from several host threads)

inline bool aligned(const void *p, size_t a) { return p && (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline bool known_head(int k) { return k == ARN_HEAD_PV || k == ARN_HEAD_C51 || k == ARN_HEAD_Q || k == ARN_HEAD_DUEL; }

// gfx950 check, cached per device
int check_arch() {
    static int cached[64];   // 0 unknown, 1 ok, -1 wrong arch, -2 hip error
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return ARN_EHIP;
    if (dev < 0 || dev >= 64) return ARN_EHIP;
    std::lock_guard<std::mutex> lock(g_lazy_mutex);
    if (cached[dev] == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) cached[dev] = -2;
        else cached[dev] = strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : -1;
    }
    return cached[dev] == 1 ? ARN_OK : (cached[dev] == -1 ? ARN_EARCH : ARN_EHIP);
}

inline int launched() { return hipGetLastError() == hipSuccess ? ARN_OK : ARN_EHIP; }

// Optional instrumentation (arn_profile_enable): a pair of HIP events around every launch.
struct ProfRecord {
    const char *name;
    hipEvent_t start, stop;
};
bool g_prof_on = false;
std::vector<ProfRecord> g_prof;
struct ProfScope {
    hipStream_t s;
    bool on;
    ProfScope(const char *name, hipStream_t stream) : s(stream), on(g_prof_on) {
        if (!on) return;
        ProfRecord r{name, nullptr, nullptr};
        if (hipEventCreate(&r.start) != hipSuccess || hipEventCreate(&r.stop) != hipSuccess) { on = false; return; }
        (void)hipEventRecord(r.start, s);
        g_prof.push_back(r);
    }
    ~ProfScope() {
        if (on) (void)hipEventRecord(g_prof.back().stop, s);
    }
};

inline unsigned cdiv(long a, long b) { return (unsigned)((a + b - 1) / b); }

// A second, library-owned stream (default priority) on which the weight-gradient kernels and their
// reductions run next to the input-gradient chain of the caller's stream; joined back with events
// before the call returns.  Created once per device on first use.  ARN_SINGLE_STREAM=1 disables it.
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t fork[5] = {}, join = nullptr;
    int state = 0;   // 0 unknown, 1 ready, -1 unavailable
};
SideStream *side_stream() {
    static SideStream per_dev[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    SideStream &ss = per_dev[dev];
    std::lock_guard<std::mutex> lock(g_lazy_mutex);
    if (ss.state == 0) {
        const char *off = getenv("ARN_SINGLE_STREAM");
        bool ok = !(off && off[0] == '1');
        ok = ok && hipStreamCreateWithFlags(&ss.stream, hipStreamNonBlocking) == hipSuccess;
        for (int i = 0; ok && i < 5; ++i) ok = hipEventCreateWithFlags(&ss.fork[i], hipEventDisableTiming) == hipSuccess;
        ok = ok && hipEventCreateWithFlags(&ss.join, hipEventDisableTiming) == hipSuccess;
        ss.state = ok ? 1 : -1;
    }
    return ss.state == 1 ? &ss : nullptr;
}

// Device address of this GPU's copy of `scratch`, looked up once per device with that device current.
void *static_scratch_ptr() {
    static void *per_dev[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(g_lazy_mutex);
    if (!per_dev[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        per_dev[dev] = ptr;
    }
    return per_dev[dev];
}

template <class P>
void launch_nt(const char *name, const P &p, long M, int n_tiles, int z, hipStream_t s) {
    ProfScope ps(name, s);
    hipLaunchKernelGGL((gemm_nt_kernel<P, false>), dim3(cdiv(M, P::BM), n_tiles, z), dim3(ThreadsOf<P>::value), 0, s, p);
}
template <class P>
void launch_nt_split(const char *name, const P &p, long M, int n_tiles, int z, hipStream_t s) {
    ProfScope ps(name, s);
    hipLaunchKernelGGL((gemm_nt_kernel<P, true>), dim3(cdiv(M, P::BM), n_tiles, z), dim3(ThreadsOf<P>::value), 0, s, p);
}

template <class P>
void launch_tn(const char *name, const P &p, float *part, long M, int N1, int KP, int splits, hipStream_t s) {
    ProfScope ps(name, s);
    long rows = (M + splits - 1) / splits;
    rows = (rows + 63) / 64 * 64;
    hipLaunchKernelGGL(gemm_tn_kernel<P>, dim3(KP / P::BK2, N1 / P::BN1, splits), dim3(256), 0, s, p, part,
                       (int)rows);
}

// sample-resident convolution: a fixed, contiguous range of samples per workgroup
template <class C>
void launch_resident(const char *name, const typename C::Args &a, int B, hipStream_t s) {
    ProfScope ps(name, s);
    const int groups = (B + C::G - 1) / C::G;
    constexpr int waves = ResWaves<C>::value;
    const int target = C::NBUF == 1 && waves == 4 ? 512 : 256;               // single-buffered four-wavefront kernels share a CU
    const int spw = resident_spw(groups, target) * C::G;
    // with few sample groups, the position tiles of a group are dealt to several workgroups
    constexpr int tiles = (C::G * C::P + 15) / 16;
    const int wgs = (int)cdiv(B, spw);
    int parts = 128 / wgs;   // every extra workgroup repeats the weight fetch and the staging: measured to pay only up to about 128 workgroups
    parts = parts < 1 ? 1 : parts > tiles ? tiles : parts;
    hipLaunchKernelGGL(resident_conv_kernel<C>, dim3(wgs, parts), dim3(64 * waves), 0, s, a, B, spw);
}

template <class F>
void launch_reduce(const char *name, const F &f, const float *part, float *dW, long wcount, long bcount, int splits,
                   float wscale, hipStream_t s) {
    ProfScope ps(name, s);
    const long block = wcount + bcount;
    const int ng = splits >= 64 ? 8 : splits >= 16 ? 4 : splits >= 4 ? 2 : 1;
    hipLaunchKernelGGL(reduce_partials_kernel<F>, dim3(cdiv(block, 256 / ng)), dim3(256), 0, s, f, part, dW, block,
                       wcount, splits, wscale, ng);
}

struct Packed {   // typed views of the packed blob
    const __bf16 *w1, *w2, *w3, *wfc, *wh, *whd, *wfcd, *w3d, *w2d;
    const __bf16 *w1l, *w2l, *w3l, *wfcl, *whl;
    const _Float16 *w1h, *w2h, *w3h, *wfch;   // fp16 forward layouts
    const float *b1, *b2, *b3, *bfc, *bh;
};
Packed view_packed(const void *blob, const Dims &d) {
    const PackedOffsets o = packed_offsets(d);
    const char *b = (const char *)blob;
    Packed p;
    p.w1 = (const __bf16 *)(b + o.w1);
    p.w2 = (const __bf16 *)(b + o.w2);
    p.w3 = (const __bf16 *)(b + o.w3);
    p.wfc = (const __bf16 *)(b + o.wfc);
    p.wh = (const __bf16 *)(b + o.wh);
    p.b1 = (const float *)(b + o.b1);
    p.b2 = (const float *)(b + o.b2);
    p.b3 = (const float *)(b + o.b3);
    p.bfc = (const float *)(b + o.bfc);
    p.bh = (const float *)(b + o.bh);
    p.whd = (const __bf16 *)(b + o.whd);
    p.wfcd = (const __bf16 *)(b + o.wfcd);
    p.w3d = (const __bf16 *)(b + o.w3d);
    p.w2d = (const __bf16 *)(b + o.w2d);
    p.w1l = (const __bf16 *)(b + o.w1l);
    p.w2l = (const __bf16 *)(b + o.w2l);
    p.w3l = (const __bf16 *)(b + o.w3l);
    p.wfcl = (const __bf16 *)(b + o.wfcl);
    p.whl = (const __bf16 *)(b + o.whl);
    p.w1h = (const _Float16 *)(b + o.w1h);
    p.w2h = (const _Float16 *)(b + o.w2h);
    p.w3h = (const _Float16 *)(b + o.w3h);
    p.wfch = (const _Float16 *)(b + o.wfch);
    return p;
}

// fc layer and, for the categorical head, the head GEMM; shared by both geometries.  F16: act3 and the fc
// weights are fp16 and the layer is one product (no-gradient forward); otherwise three bf16 products.
template <int FEAT_, bool F16 = false>
void fc_and_head_launches(const Dims &d, const Packed &w, int B, char *ws, const Workspace &o, float *z_out,
                          int zstride, hipStream_t s) {
    __bf16 *a3 = (__bf16 *)(ws + o.a3), *a3l = (__bf16 *)(ws + o.a3l);
    __bf16 *h = (__bf16 *)(ws + o.h), *hl = (__bf16 *)(ws + o.hl);
    {
        typedef typename std::conditional<F16, FcFwdF16T<FEAT_>, FcFwdT<FEAT_>>::type Fc;
        Fc p;
        p.in = a3; p.lo_off = a3l - a3; p.M = B; p.w = F16 ? (const __bf16 *)w.wfch : w.wfc; p.w_lo = w.wfcl; p.bias = w.bfc;
        p.out = h; p.out_lo = hl; p.ksplit = fc_ksplit(B, F16); p.partial = (float *)(ws + o.fcp);
        p.to_partial = p.ksplit > 1 || d.small;
        if constexpr (F16) launch_nt("fc_fwd", p, B, HID / Fc::BN, p.ksplit, s);
        else launch_nt_split("fc_fwd", p, B, HID / Fc::BN, p.ksplit, s);
        if (p.ksplit > 1 && !d.small) {
            ProfScope ps("fc_finish", s);
            const long total = (long)B * HID;
            hipLaunchKernelGGL(fc_finish_kernel, dim3(cdiv(total / 4, 256)), dim3(256), 0, s, p.partial, p.ksplit,
                               w.bfc, h, hl, total);
        }
    }
    if (d.head == ARN_HEAD_C51) {
        HeadFwdC51 p;
        p.in = h; p.lo_off = hl - h; p.M = B; p.w = w.wh; p.w_lo = w.whl; p.bias = w.bh; p.z = z_out; p.ZW = d.NH; p.ZS = zstride;
        launch_nt_split("head_fwd", p, B, d.NHP / 64, 1, s);
    }
    // policy/value and action-value heads: the caller launches pv_head_kernel on the fc partial sums
}

// Which configurations of the sample-resident kernels a geometry uses: the 84x84 network has hand-laid LDS
// images, any other geometry the ones whose padding is computed from its map sizes.
template <class G>
struct ConvConfigs {
    typedef ResConv2FwdGeo<G> Fwd2;
    typedef ResConv3FwdGeo<G> Fwd3;
    typedef ResConv3DgradGeo<G> Dgrad3;
    typedef ResConv2DgradGeo<G> Dgrad2;
    static int conv1_parts(int) { return 1; }
    // conv2 -> conv3 through LDS needs both layers' images in one CU's LDS: not with the bordered images of this geometry
    static bool fused_conv23(int) { return false; }
    static void launch_conv23(const Conv23Args &, int, int, hipStream_t) {}
    static void launch_conv123(const uint8_t *, const __bf16 *, const __bf16 *, const float *, uint8_t *, const Conv23Args &, int,
                               int, hipStream_t) {}
};
template <>
struct ConvConfigs<Geo84> {
    typedef ResConv2Fwd Fwd2;
    typedef ResConv3Fwd Fwd3;
    typedef ResConv3Dgrad Dgrad3;
    typedef ResConv2Dgrad Dgrad2;
    // few samples: three workgroups share one (one workgroup fits per CU)
    static int conv1_parts(int B) { return 3 * B <= 256 ? 3 : 1; }
    // one workgroup per sample range and no tile splitting: measured equal to the two kernels at B = 64, faster above
    static bool fused_conv23(int B) { return B >= 64; }
    static void launch_conv23(const Conv23Args &p, int B, int spw, hipStream_t s) {
        hipLaunchKernelGGL((conv23_fwd_fused_kernel<ResConv2Fwd, ResConv3Fwd>), dim3((B + spw - 1) / spw), dim3(C23_THREADS), 0,
                           s, p, B, spw);
    }
    static void launch_conv123(const uint8_t *obs, const __bf16 *w1, const __bf16 *w1l, const float *b1, uint8_t *m1,
                               const Conv23Args &p, int B, int spw, hipStream_t s) {
        hipLaunchKernelGGL((conv123_fwd_kernel<Geo84, ResConv2Fwd, ResConv3Fwd>), dim3((B + spw - 1) / spw), dim3(C23_THREADS),
                           0, s, obs, w1, w1l, b1, m1, p, B, spw);
    }
};

// Forward pass for geometry G in three-product bf16 precision (conv1's pixel operand is exact: two products).
template <class G>
void forward_trunk(const Dims &d, const Packed &w, const uint8_t *obs, int B, char *ws, const Workspace &o,
                   float *z_out, int zstride, bool masks, hipStream_t s) {
    typedef ConvConfigs<G> Cfg;
    __bf16 *a1 = (__bf16 *)(ws + o.a1), *a2 = (__bf16 *)(ws + o.a2), *a3 = (__bf16 *)(ws + o.a3);
    __bf16 *a1l = (__bf16 *)(ws + o.a1l), *a2l = (__bf16 *)(ws + o.a2l), *a3l = (__bf16 *)(ws + o.a3l);
    const bool chained = Cfg::fused_conv23(B) && Cfg::conv1_parts(B) == 1;
    if (!chained) {
        ProfScope ps("conv1_fwd", s);
        const int spw = resident_spw(B, 256);
        hipLaunchKernelGGL(conv1_fwd_resident_kernel<G>, dim3(cdiv(B, spw), Cfg::conv1_parts(B)), dim3(RES_THREADS), 0, s,
                           obs, w.w1, w.w1l, w.b1, a1, a1l, masks ? (uint8_t *)(ws + o.m1) : nullptr, B, spw);
    }
    if (Cfg::fused_conv23(B)) {
        // conv2 and conv3 in one kernel: act2 passes through LDS; with one workgroup per sample range in conv1 too,
        // conv1 runs in the same launch, ahead of them in every workgroup
        ProfScope ps(chained ? "conv123_fwd" : "conv23_fwd", s);
        Conv23Args p;
        p.a1 = a1; p.a1_lo = a1l; p.w2 = w.w2; p.w2_lo = w.w2l; p.w3 = w.w3; p.w3_lo = w.w3l; p.b2 = w.b2; p.b3 = w.b3;
        p.a2 = masks ? a2 : nullptr; p.a3 = a3; p.a3_lo = a3l;
        p.m2 = masks ? (uint8_t *)(ws + o.m2) : nullptr; p.m3 = masks ? (uint8_t *)(ws + o.m3) : nullptr;
        const int spw = resident_spw(B, 256);
        if (chained) Cfg::launch_conv123(obs, w.w1, w.w1l, w.b1, masks ? (uint8_t *)(ws + o.m1) : nullptr, p, B, spw, s);
        else Cfg::launch_conv23(p, B, spw, s);
    } else {
        {
            typename Cfg::Fwd2::Args p;
            p.in = a1; p.in_lo = a1l; p.w = w.w2; p.w_lo = w.w2l; p.mask = nullptr; p.bias = w.b2; p.out = a2; p.out_lo = a2l;
            p.mask_out = masks ? (uint8_t *)(ws + o.m2) : nullptr;
            launch_resident<typename Cfg::Fwd2>("conv2_fwd", p, B, s);
        }
        {
            typename Cfg::Fwd3::Args p;
            p.in = a2; p.in_lo = a2l; p.w = w.w3; p.w_lo = w.w3l; p.mask = nullptr; p.bias = w.b3; p.out = a3; p.out_lo = a3l;
            p.mask_out = masks ? (uint8_t *)(ws + o.m3) : nullptr;
            launch_resident<typename Cfg::Fwd3>("conv3_fwd", p, B, s);
        }
    }
    fc_and_head_launches<G::FEAT>(d, w, B, ws, o, z_out, zstride, s);
}

// Forward pass that carries no gradient (action selection): the three convolutions in one kernel and one fp16
// product per layer, act3 in fp16, then the fc layer in fp16.  The heads run as in the training forward.
template <class G>
void infer_trunk(const Dims &d, const Packed &w, const uint8_t *obs, int B, char *ws, const Workspace &o,
                 float *z_out, int zstride, hipStream_t s) {
    typedef ConvConfigs<G> Cfg;
    {
        ProfScope ps("conv_infer", s);
        InferConvArgs p;
        p.obs = obs; p.w1 = w.w1h; p.w2 = w.w2h; p.w3 = w.w3h; p.b1 = w.b1; p.b2 = w.b2; p.b3 = w.b3;
        p.a3 = (_Float16 *)(ws + o.a3);
        const int spw = resident_spw(B, 256);
        // the software-pipelined variant where its 17 KB of weights and biases fit beside the LDS images (84x84)
        if constexpr (infer_pipelined_fits<G, typename Cfg::Fwd2, typename Cfg::Fwd3>())
            hipLaunchKernelGGL((infer_conv_pipelined_kernel<G, typename Cfg::Fwd2, typename Cfg::Fwd3>), dim3(cdiv(B, spw)),
                               dim3(INF_THREADS), 0, s, p, B, spw);
        else
            hipLaunchKernelGGL((infer_conv_kernel<G, typename Cfg::Fwd2, typename Cfg::Fwd3>), dim3(cdiv(B, spw)),
                               dim3(INF_THREADS), 0, s, p, B, spw);
    }
    fc_and_head_launches<G::FEAT, true>(d, w, B, ws, o, z_out, zstride, s);
}
void infer_launches(const Dims &d, const Packed &w, const uint8_t *obs, int B, char *ws, const Workspace &o,
                    float *z_out, int zstride, hipStream_t s) {
    if (d.geom == ARN_GEOM_PAPER) infer_trunk<GeoPaper>(d, w, obs, B, ws, o, z_out, zstride, s);
    else infer_trunk<Geo84>(d, w, obs, B, ws, o, z_out, zstride, s);
}

// trunk + heads forward.  C51: z_out = atom logits, rows of zstride floats (NH = dense, or NHP for the
// library's own buffers).  PV, Q, DUEL: stops after the fc GEMM, whose fp32 partial sums (o.fcp) the fused head
// kernel consumes.  masks: also write the ReLU sign bits of act1..3 for the backward pass (training forward on
// the online weights).
void forward_launches(const Dims &d, const Packed &w, const uint8_t *obs, int B, char *ws, const Workspace &o,
                      float *z_out, int zstride, bool masks, hipStream_t s) {
    if (d.geom == ARN_GEOM_PAPER) forward_trunk<GeoPaper>(d, w, obs, B, ws, o, z_out, zstride, masks, s);
    else forward_trunk<Geo84>(d, w, obs, B, ws, o, z_out, zstride, masks, s);
}

// Events that let work queued on the side stream see everything queued on the caller's stream so far.
struct Fork {
    SideStream *ss = nullptr;
    hipStream_t s = nullptr, s2 = nullptr;
    int n = 0;
    void operator()() {
        if (!ss) return;
        (void)hipEventRecord(ss->fork[n], s);
        (void)hipStreamWaitEvent(s2, ss->fork[n], 0);
        ++n;
    }
};

// Backward pass below d(pre_fc) for geometry G.  Everything that needs only d(pre_fc) -- the fc weight gradient
// and its reduction, next to the head's -- runs on the side stream; the chain fc dgrad -> conv3 dgrad ->
// conv2 dgrad (fused with conv1's weight gradient), the other convolutions' weight gradients and one reduction
// kernel for all three of them stay on the caller's stream.  (Every cross-stream event costs the waiting and the recording stream about 6 us, and two
// heavy kernels side by side mostly share the memory system, so more overlap than this measured slower.)
template <class G>
void backward_trunk(const Packed &w, const uint8_t *obs, int B, char *ws, const Workspace &o, const ParamOffsets &po,
                    const Splits &sp, float *dW, Fork &fk) {
    typedef ConvConfigs<G> Cfg;
    hipStream_t s = fk.s, s2 = fk.s2;
    __bf16 *a1 = (__bf16 *)(ws + o.a1), *a2 = (__bf16 *)(ws + o.a2), *a3 = (__bf16 *)(ws + o.a3);
    __bf16 *dph = (__bf16 *)(ws + o.dph), *dp3 = (__bf16 *)(ws + o.dp3);
    __bf16 *dp2 = (__bf16 *)(ws + o.dp2);
    float *part1 = (float *)(ws + o.pw1), *part2 = (float *)(ws + o.pw2), *part3 = (float *)(ws + o.pw3);
    {
        typedef Wgrad<DenseGather<G::FEAT>, 128, 64, 2, HID, G::FEAT> FcW;
        FcW p;
        p.in = a3; p.M = B; p.dy = dph;
        float *part = (float *)(ws + o.pwfc);
        launch_tn("fc_wgrad", p, part, B, HID, G::FEAT, sp.fc, s2);
        ProfScope ps("fc_reduce", s2);
        hipLaunchKernelGGL((fc_reduce_kernel<G::FEAT, G::P3>), dim3(HID + 1), dim3(256), 0, s2, part, dW, (long)po.wfc,
                           (long)po.bfc, sp.fc);
    }
    {
        // 128 x 128 tiles from 1024 samples up (fewer operand bytes from the L2 per flop), 128 x 64 below (more workgroups)
        auto launch = [&](auto p) {
            p.in = dph; p.M = B; p.w = w.wfcd; p.maskbits = (const uint8_t *)(ws + o.m3); p.out = dp3;
            launch_nt("fc_dgrad", p, B, (G::FEAT + p.BN - 1) / p.BN, 1, s);
        };
        if (B >= 1024) launch(FcDgradT<G::FEAT, 128>());
        else launch(FcDgradT<G::FEAT, 64>());
    }
    {
        typename Cfg::Dgrad3::Args p;
        p.in = dp3; p.in_lo = nullptr; p.w = w.w3d; p.w_lo = nullptr; p.mask = (const uint8_t *)(ws + o.m2); p.out = dp2;
        launch_resident<typename Cfg::Dgrad3>("conv3_dgrad", p, B, s);
    }
    {
        // One launch for everything that is left once d(pre2) exists: conv2's input gradient fused with conv1's
        // weight gradient (conv1's input is data, so d(pre1) has this one consumer and stays in LDS), and the
        // weight gradients of conv2 and conv3 -- three ranges of workgroups, longest first.
        ProfScope ps("conv_bwd", s);
        ConvBackwardArgs p;
        p.obs = obs; p.dp2 = dp2; p.w2d = w.w2d; p.mask1 = (const uint8_t *)(ws + o.m1); p.part1 = part1;
        p.a1 = a1; p.a2 = a2; p.dp3 = dp3; p.part2 = part2; p.part3 = part3;
        p.B = B; p.n1 = sp.c1; p.n2 = sp.c2;
        constexpr int geom = std::is_same<G, Geo84>::value ? ARN_GEOM_84 : ARN_GEOM_PAPER;
        p.spw1 = resident_spw(B, 256);
        p.spw2 = resident_spw((B + CONV2_WG_G - 1) / CONV2_WG_G, wgrad_wgs2(geom)) * CONV2_WG_G;
        p.spw3 = resident_spw((B + CONV3_WG_G - 1) / CONV3_WG_G, wgrad_wgs3(geom)) * CONV3_WG_G;
        hipLaunchKernelGGL((conv_backward_kernel<G, typename Cfg::Dgrad2>), dim3(sp.c1 + sp.c2 + sp.c3),
                           dim3(ConvBackward<G, typename Cfg::Dgrad2>::THREADS), 0, s, p);
    }
    {
        // one launch adds the partials of all three convolutions (x = u8/255: conv1's pixel scale comes out of
        // the contraction and is applied here; bias gradients have no such factor)
        ProfScope ps("conv_reduce", s);
        ConvReducePlan pl;
        pl.seg[0] = make_reduce_seg(part1, (long)C1 * KW1, C1, sp.c1, 1.f / 255.f);
        pl.seg[1] = make_reduce_seg(part2, (long)C2 * KW2, C2, sp.c2, 1.f);
        pl.seg[2] = make_reduce_seg(part3, (long)C3 * KW3, C3, sp.c3, 1.f);
        pl.w1 = (long)po.w1; pl.b1 = (long)po.b1; pl.w2 = (long)po.w2; pl.b2 = (long)po.b2;
        pl.w3 = (long)po.w3; pl.b3 = (long)po.b3;
        int blk = 0;
        for (int k = 0; k < 3; ++k) {
            pl.seg[k].first_block = blk;
            blk += (int)cdiv(pl.seg[k].block, 256 / pl.seg[k].ng);
        }
        hipLaunchKernelGGL(conv_reduce_kernel, dim3(blk), dim3(256), 0, s, pl, dW);
    }
}

// Samples per workgroup of the head kernel in the inference calls: small batches are spread over more CUs
inline int infer_rows_per_block(int B) { return B <= 512 ? 4 : B <= 4096 ? 8 : PVH_ROWS; }

// Arguments of the fused policy/value head kernel that both entry points share.
// f16: the fc partial sums come from the no-gradient forward (its own number of k ranges)
PvHeadArgs pv_head_args(const Dims &d, const Packed &w, int B, char *ws, const Workspace &o, bool f16) {
    PvHeadArgs p = {};
    p.partial = (const float *)(ws + o.fcp); p.ks = fc_ksplit(B, f16); p.bfc = w.bfc;
    p.wh = w.wh; p.whl = w.whl; p.bh = w.bh; p.B = B; p.A = d.A;
    p.qmode = d.head == ARN_HEAD_Q ? 1 : d.head == ARN_HEAD_DUEL ? 2 : 0;
    return p;
}

// Lays the flat fp32 parameters out in every packed form, one launch.
void launch_pack_all(const Dims &d, const float *w_fp32, void *w_packed, hipStream_t s) {
    if (d.a3c) {
        // the 2-convolution network: its parameters are first laid into the embedding network's flat vector, kept
        // in the tail of the packed blob, and that vector is packed
        ProfScope ps("a3c_embed", s);
        float *big = (float *)((char *)w_packed + packed_offsets(d).a3c_flat);
        const A3cMap m = make_a3c_map(d);
        const long total = (long)m.e.total;
        hipLaunchKernelGGL(a3c_fill_kernel, dim3(cdiv(total, 256)), dim3(256), 0, s, big, total, (long)m.e.w3);
        hipLaunchKernelGGL(a3c_scatter_kernel, dim3(cdiv(m.total, 256)), dim3(256), 0, s, m, w_fp32, big);
        w_fp32 = big;
    }
    ProfScope ps("pack_all", s);
    const PackPlan pl = make_pack_plan(d, w_packed);
    hipLaunchKernelGGL(pack_all_kernel, dim3(pl.blocks), dim3(256), 0, s, pl, w_fp32);
}

// Shared argument checks of the update entry points.  Returns ARN_OK and fills *d_out when a repack is asked for.
int check_update(size_t n, const arn_config *cfg, const void *w_packed, bool *repack, Dims *d_out) {
    if (n == 0 || n > ((size_t)1 << 40)) return ARN_EINVAL;
    *repack = w_packed != nullptr;
    if (*repack) {
        if (!cfg) return ARN_EINVAL;
        if (!known_head(cfg->head_kind)) return ARN_EKIND;
        *d_out = make_dims(cfg);
        if (!d_out->ok) return ARN_ESHAPE;
        if (n != public_param_count(*d_out)) return ARN_ESHAPE;
        if (!aligned(w_packed, 256)) return ARN_EINVAL;
    }
    return ARN_OK;
}
inline bool unit_interval(float b) { return b >= 0.f && b < 1.f; }
inline unsigned update_blocks(size_t n) { return (unsigned)((n + 1023) / 1024); }

}  // namespace

extern "C" {

const char *arn_status_string(int status) {
    switch (status) {
        case ARN_OK: return "ok";
        case ARN_EINVAL: return "invalid argument (null or misaligned pointer, B <= 0 or B > 2^20)";
        case ARN_ESHAPE: return "unsupported shape (num_actions, num_atoms or head for this call)";
        case ARN_EKIND: return "unknown head_kind, loss_kind or mode";
        case ARN_EWORKSPACE: return "workspace too small";
        case ARN_EARCH: return "device is not gfx950";
        case ARN_EHIP: return "HIP runtime error";
        case ARN_ESTATIC: return "batch too large for the library's static scratch buffer (arn_policy_forward_static)";
        default: return "unknown status";
    }
}

size_t arn_param_count(const arn_config *cfg) {
    const Dims d = make_dims(cfg);
    return d.ok ? public_param_count(d) : 0;
}

size_t arn_packed_bytes(const arn_config *cfg) {
    const Dims d = make_dims(cfg);
    return d.ok ? packed_offsets(d).total : 0;
}

size_t arn_workspace_bytes(const arn_config *cfg, int B, int mode) {
    const Dims d = make_dims(cfg);
    if (!d.ok || B <= 0 || B > (1 << 20) || (mode != ARN_MODE_FORWARD && mode != ARN_MODE_TRAIN)) return 0;
    return make_workspace(d, B, mode).total;
}

int arn_weights_prepare(const arn_config *cfg, const float *w_fp32, void *w_packed, void *stream) {
    if (!cfg) return ARN_EINVAL;
    if (!known_head(cfg->head_kind)) return ARN_EKIND;
    const Dims d = make_dims(cfg);
    if (!d.ok) return ARN_ESHAPE;
    if (!aligned(w_fp32, 16) || !aligned(w_packed, 256)) return ARN_EINVAL;
    if (int e = check_arch()) return e;
    hipStream_t s = (hipStream_t)stream;
    launch_pack_all(d, w_fp32, w_packed, s);
    return launched();
}

namespace {
// Argument checks shared by arn_policy_forward and arn_policy_forward_static; fills *d_out.
int check_policy_forward(const arn_config *cfg, const void *w_packed, const uint8_t *obs, int B, float *logits,
                         float *value, float *probs, int32_t *greedy, Dims *d_out) {
    if (!cfg || B <= 0 || B > (1 << 20)) return ARN_EINVAL;
    if (!known_head(cfg->head_kind)) return ARN_EKIND;
    const Dims d = make_dims(cfg);
    if (!d.ok) return ARN_ESHAPE;
    if (!aligned(w_packed, 256) || !aligned(obs, 16) || !aligned(logits, 16)) return ARN_EINVAL;
    if (d.small && !aligned(value, 16)) return ARN_EINVAL;
    if ((value && !aligned(value, 16)) || (probs && !aligned(probs, 16)) || (greedy && !aligned(greedy, 16)))
        return ARN_EINVAL;
    if (d.qhead && probs) return ARN_ESHAPE;
    *d_out = d;
    return ARN_OK;
}

// The launches of one inference call; `ws` holds make_workspace(d, B, ARN_MODE_FORWARD).total bytes.
int policy_forward_launches(const arn_config *cfg, const Dims &d, const Workspace &o, const void *w_packed,
                            const uint8_t *obs, int B, float *logits, float *value, float *probs, int32_t *greedy,
                            char *ws, hipStream_t s) {
    const Packed w = view_packed(w_packed, d);
    infer_launches(d, w, obs, B, ws, o, logits, d.NH, s);
    if (d.small) {
        ProfScope ps("pv_head", s);
        PvHeadArgs p = pv_head_args(d, w, B, ws, o, true);
        p.logits = logits; p.value = value; p.probs = probs; p.greedy = greedy;
        p.rpb = infer_rows_per_block(B);
        hipLaunchKernelGGL(pv_head_kernel<false>, dim3(cdiv(B, p.rpb)), dim3(PVH_THREADS), 0, s, p);
    } else if (value || probs || greedy) {
        ProfScope ps("c51_dist", s);
        hipLaunchKernelGGL(c51_dist_kernel, dim3(cdiv(B, C51_WAVES)), dim3(64 * C51_WAVES), 0, s, logits, d.NH, B, d.A,
                           d.atoms, cfg->v_min, cfg->v_max, cfg->gamma, (const float *)nullptr,
                           (const uint8_t *)nullptr, probs, value, greedy, (float *)nullptr);
    }
    return launched();
}
}  // namespace

int arn_policy_forward(const arn_config *cfg, const void *w_packed, const uint8_t *obs, int B, float *logits,
                       float *value, float *probs, int32_t *greedy, void *workspace, size_t workspace_bytes,
                       void *stream) {
    Dims d;
    if (int e = check_policy_forward(cfg, w_packed, obs, B, logits, value, probs, greedy, &d)) return e;
    if (!aligned(workspace, 256)) return ARN_EINVAL;
    const Workspace o = make_workspace(d, B, ARN_MODE_FORWARD);
    if (workspace_bytes < o.total) return ARN_EWORKSPACE;
    if (int e = check_arch()) return e;
    return policy_forward_launches(cfg, d, o, w_packed, obs, B, logits, value, probs, greedy, (char *)workspace,
                                   (hipStream_t)stream);
}

int arn_policy_forward_static(const arn_config *cfg, const void *w_packed, const uint8_t *obs, int B, float *logits,
                              float *value, float *probs, int32_t *greedy, void *stream) {
    Dims d;
    if (int e = check_policy_forward(cfg, w_packed, obs, B, logits, value, probs, greedy, &d)) return e;
    const Workspace o = make_workspace(d, B, ARN_MODE_FORWARD);
    if (o.total > (size_t)ARN_STATIC_SCRATCH_BYTES) return ARN_ESTATIC;
    if (int e = check_arch()) return e;
    void *ptr = static_scratch_ptr();
    if (!ptr) return ARN_EHIP;
    return policy_forward_launches(cfg, d, o, w_packed, obs, B, logits, value, probs, greedy, (char *)ptr,
                                   (hipStream_t)stream);
}

int arn_policy_act(const arn_config *cfg, const void *w_packed, const uint8_t *obs, int B, const float *u,
                   const float *u2, float epsilon, int32_t *action, float *logp, void *workspace,
                   size_t workspace_bytes, void *stream) {
    if (!cfg || B <= 0 || B > (1 << 20)) return ARN_EINVAL;
    if (!known_head(cfg->head_kind)) return ARN_EKIND;
    const Dims d = make_dims(cfg);
    if (!d.ok) return ARN_ESHAPE;
    if (!aligned(w_packed, 256) || !aligned(obs, 16) || !aligned(u, 16) || !aligned(action, 16) ||
        !aligned(workspace, 256))
        return ARN_EINVAL;
    const bool policy = d.head == ARN_HEAD_PV;
    if (!policy && (!aligned(u2, 16) || !(epsilon >= 0.f && epsilon <= 1.f))) return ARN_EINVAL;
    if (logp && (!policy || !aligned(logp, 16))) return policy ? ARN_EINVAL : ARN_ESHAPE;
    const Workspace o = make_workspace(d, B, ARN_MODE_FORWARD);
    if (workspace_bytes < o.total) return ARN_EWORKSPACE;
    if (int e = check_arch()) return e;
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    const Packed w = view_packed(w_packed, d);
    float *z = (float *)(ws + o.z);   // categorical head only
    infer_launches(d, w, obs, B, ws, o, z, d.NHP, s);
    if (d.small) {
        ProfScope ps("pv_head", s);
        PvHeadArgs p = pv_head_args(d, w, B, ws, o, true);
        p.u = u; p.u2 = u2; p.epsilon = epsilon; p.act_out = action; p.logp_out = logp;
        p.rpb = infer_rows_per_block(B);
        hipLaunchKernelGGL(pv_head_kernel<false>, dim3(cdiv(B, p.rpb)), dim3(PVH_THREADS), 0, s, p);
    } else {
        ProfScope ps("c51_dist", s);
        hipLaunchKernelGGL(c51_dist_kernel, dim3(cdiv(B, C51_WAVES)), dim3(64 * C51_WAVES), 0, s, z, d.NHP, B, d.A, d.atoms,
                           cfg->v_min, cfg->v_max, cfg->gamma, (const float *)nullptr, (const uint8_t *)nullptr,
                           (float *)nullptr, (float *)nullptr, action, (float *)nullptr);
        hipLaunchKernelGGL(epsilon_greedy_kernel, dim3(cdiv(B, 256)), dim3(256), 0, s, action, u, u2, epsilon, d.A, B);
    }
    return launched();
}

int arn_train_step_grads(const arn_config *cfg, const void *w_packed, const arn_batch *batch, int B, int loss_kind,
                         float *dW, float *loss, void *workspace, size_t workspace_bytes, void *stream) {
    if (!cfg || !batch || B <= 0 || B > (1 << 20)) return ARN_EINVAL;
    if (!known_head(cfg->head_kind)) return ARN_EKIND;
    if (loss_kind != ARN_LOSS_A2C && loss_kind != ARN_LOSS_PPO && loss_kind != ARN_LOSS_C51 &&
        loss_kind != ARN_LOSS_DQN)
        return ARN_EKIND;
    const Dims d = make_dims(cfg);
    if (!d.ok) return ARN_ESHAPE;
    if ((loss_kind == ARN_LOSS_C51) != (d.head == ARN_HEAD_C51)) return ARN_ESHAPE;
    if ((loss_kind == ARN_LOSS_DQN) != d.qhead) return ARN_ESHAPE;
    if (!aligned(w_packed, 256) || !aligned(batch->obs, 16) || !aligned(batch->action, 16) || !aligned(dW, 16) ||
        !aligned(loss, 16) || !aligned(workspace, 256))
        return ARN_EINVAL;
    if (loss_kind == ARN_LOSS_A2C || loss_kind == ARN_LOSS_PPO) {
        if (!aligned(batch->adv, 16) || !aligned(batch->ret, 16)) return ARN_EINVAL;
        if (loss_kind == ARN_LOSS_PPO && !aligned(batch->old_logp, 16)) return ARN_EINVAL;
    } else {
        if (!aligned(batch->next_obs, 16) || !aligned(batch->reward, 16) || !aligned(batch->done, 16) ||
            !aligned(batch->w_target_packed, 256))
            return ARN_EINVAL;
        if (batch->next_action && !aligned(batch->next_action, 16)) return ARN_EINVAL;
    }
    const Workspace o = make_workspace(d, B, ARN_MODE_TRAIN);
    if (workspace_bytes < o.total) return ARN_EWORKSPACE;
    if (int e = check_arch()) return e;

    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    const Packed w = view_packed(w_packed, d);
    const ParamOffsets po = param_offsets(d);
    const Splits sp = make_splits(d, B);
    float *const dW_out = dW;
    if (d.a3c) dW = (float *)(ws + o.a3c_dw);   // the embedding network's gradient; the caller's entries are gathered from it at the end
    float *z = (float *)(ws + o.z);
    __bf16 *h = (__bf16 *)(ws + o.h);
    __bf16 *dz = (__bf16 *)(ws + o.dz), *dph = (__bf16 *)(ws + o.dph);
    float *lossp = (float *)(ws + o.lossp), *hbp = (float *)(ws + o.hbp);
    const int lblocks = loss_blocks(d, B);
    // Double-DQN: the online network's greedy action on the next states, kept where the caller asked for it
    int32_t *const astar = batch->next_action ? batch->next_action : (int32_t *)(ws + o.astar);

    // ---- forward and objective ----
    // The passes that carry no gradient (target network, Double-DQN selection) are one fp16 product per layer.
    if (loss_kind == ARN_LOSS_C51) {
        // target network on next states -> projected target m; its activations are then overwritten
        const Packed wt = view_packed(batch->w_target_packed, d);
        float *ztgt = (float *)(ws + o.ztgt), *m = (float *)(ws + o.m);
        infer_launches(d, wt, batch->next_obs, B, ws, o, ztgt, d.NHP, s);
        {
            ProfScope ps("c51_target", s);
            hipLaunchKernelGGL(c51_dist_kernel, dim3(cdiv(B, C51_WAVES)), dim3(64 * C51_WAVES), 0, s, ztgt, d.NHP, B, d.A,
                               d.atoms, cfg->v_min, cfg->v_max, cfg->gamma, batch->reward, batch->done,
                               (float *)nullptr, (float *)nullptr, batch->next_action, m);
        }
        forward_launches(d, w, batch->obs, B, ws, o, z, d.NHP, true, s);
        ProfScope ps("loss", s);
        hipLaunchKernelGGL(c51_loss_kernel, dim3(lblocks), dim3(64 * C51_WAVES), 0, s, z, d.NHP, m, batch->action, B, d.A,
                           d.atoms, d.NHP, c51_loss_spw(B), dz, lossp, hbp);
    } else {
        const Packed *wt = nullptr;
        Packed wt_view;
        if (loss_kind == ARN_LOSS_DQN) {
            // target network on the next states -> Q(s', .); with Double-DQN the online network on the next
            // states -> its greedy action.  The activations of these passes are then overwritten.
            wt_view = view_packed(batch->w_target_packed, d);
            wt = &wt_view;
            infer_launches(d, *wt, batch->next_obs, B, ws, o, nullptr, 0, s);
            {
                ProfScope ps("q_target", s);
                PvHeadArgs p = pv_head_args(d, *wt, B, ws, o, true);
                p.logits = (float *)(ws + o.qt);
                if (!cfg->double_q) p.greedy = batch->next_action;
                p.rpb = loss_block(B);
                hipLaunchKernelGGL(pv_head_kernel<false>, dim3(lblocks), dim3(PVH_THREADS), 0, s, p);
            }
            if (cfg->double_q) {
                infer_launches(d, w, batch->next_obs, B, ws, o, nullptr, 0, s);
                ProfScope ps("q_select", s);
                PvHeadArgs p = pv_head_args(d, w, B, ws, o, true);
                p.greedy = astar;
                p.rpb = loss_block(B);
                hipLaunchKernelGGL(pv_head_kernel<false>, dim3(lblocks), dim3(PVH_THREADS), 0, s, p);
            }
        }
        forward_launches(d, w, batch->obs, B, ws, o, nullptr, 0, true, s);
        // fc finish, head, objective, dz and the head's input gradient d(pre_fc) in one kernel
        ProfScope ps("pv_head", s);
        PvHeadArgs p = pv_head_args(d, w, B, ws, o, false);
        p.action = batch->action; p.adv = batch->adv; p.ret = batch->ret; p.old_logp = batch->old_logp;
        p.objective = loss_kind == ARN_LOSS_PPO ? 1 : loss_kind == ARN_LOSS_DQN ? 2 : 0;
        p.clip_eps = cfg->clip_eps; p.value_coef = cfg->value_coef; p.entropy_coef = cfg->entropy_coef;
        if (loss_kind == ARN_LOSS_DQN) {
            p.q_next = (const float *)(ws + o.qt);
            p.a_star = cfg->double_q ? astar : nullptr;
            p.reward = batch->reward; p.done = batch->done; p.gamma = cfg->gamma;
        }
        p.whd = w.whd; p.h = h; p.dz = dz; p.dph = dph; p.lossp = lossp; p.hbp = hbp;
        p.rpb = loss_block(B);
        hipLaunchKernelGGL(pv_head_kernel<true>, dim3(lblocks), dim3(PVH_THREADS), 0, s, p);
    }

    // ---- backward ----
    // The input-gradient chain (head -> fc -> conv3 -> conv2, then conv1's weight gradient) runs on the
    // caller's stream; every other weight gradient and its reduction runs on the side stream as soon as
    // the gradient it consumes exists.
    Fork fk;
    fk.ss = side_stream();
    fk.s = s;
    fk.s2 = fk.ss ? fk.ss->stream : s;
    SideStream *ss = fk.ss;
    hipStream_t s2 = fk.s2;
    fk();   // dz (and, for the policy/value head, d(pre_fc))
    {
        // the reported loss values are off the critical path: block partial sums are added on the side stream
        ProfScope ps("loss_finalize", s2);
        const bool pv = loss_kind == ARN_LOSS_A2C || loss_kind == ARN_LOSS_PPO;
        hipLaunchKernelGGL(loss_finalize_kernel, dim3(1), dim3(64), 0, s2, lossp, lblocks, B,
                           pv ? cfg->value_coef : 0.f, pv ? cfg->entropy_coef : 0.f, loss);
    }
    {
        HeadWgrad p;
        p.in = h; p.M = B; p.N1 = d.NHP; p.dy = dz;
        float *part = (float *)(ws + o.pwh);
        launch_tn("head_wgrad", p, part, B, d.NHP, HID, sp.hd, s2);
        launch_reduce("head_reduce", UnmapHead{head_rows(d, po), d.NHP}, part, dW, (long)d.NHP * HID, d.NHP, sp.hd, 1.f, s2);
        // the head's bias gradient: the loss kernel's fp32 block partials, added in block order
        launch_reduce("head_bias", UnmapHeadBias{head_rows(d, po)}, hbp, dW, 0, d.small ? 32 : d.NHP, lblocks, 1.f, s2);
    }
    if (d.head == ARN_HEAD_C51) {
        HeadDgrad p;
        p.in = dz; p.M = B; p.K = d.NHP; p.w = w.whd; p.h = h; p.out = dph;
        launch_nt("head_dgrad", p, B, HID / HeadDgrad::BN, 1, s);
    }
    if (d.head == ARN_HEAD_C51) fk();   // d(pre_fc) comes from the head's input-gradient GEMM above
    if (d.geom == ARN_GEOM_PAPER) backward_trunk<GeoPaper>(w, batch->obs, B, ws, o, po, sp, dW, fk);
    else backward_trunk<Geo84>(w, batch->obs, B, ws, o, po, sp, dW, fk);
    if (ss) {   // join: the caller's stream continues only after the side stream's work
        (void)hipEventRecord(ss->join, s2);
        (void)hipStreamWaitEvent(s, ss->join, 0);
    }
    if (d.a3c) {
        ProfScope ps("a3c_gather", s);
        const A3cMap m = make_a3c_map(d);
        hipLaunchKernelGGL(a3c_gather_kernel, dim3(cdiv(m.total, 256)), dim3(256), 0, s, m, dW, dW_out);
    }
    return launched();
}

int arn_rmsprop_update(size_t n, float *theta, const float *g, float *accu, float lr, float rho, float eps,
                       const arn_config *cfg, void *w_packed, void *stream) {
    bool repack;
    Dims d;
    if (int e = check_update(n, cfg, w_packed, &repack, &d)) return e;
    if (!aligned(theta, 16) || !aligned(g, 16) || !aligned(accu, 16)) return ARN_EINVAL;
    if (!unit_interval(rho) || !(eps >= 0.f) || !(lr == lr)) return ARN_EINVAL;
    if (int e = check_arch()) return e;
    hipStream_t s = (hipStream_t)stream;
    UpdateArgs p = {};
    p.theta = theta; p.g = g; p.v = accu; p.n = (long)n; p.a = lr; p.beta2 = rho; p.eps = eps;
    {
        ProfScope ps("rmsprop", s);
        hipLaunchKernelGGL(update_kernel<RULE_RMSPROP>, dim3(update_blocks(n)), dim3(256), 0, s, p);
    }
    if (repack) launch_pack_all(d, theta, w_packed, s);
    return launched();
}

namespace {
// a = r sqrt(1 - beta2^t) / (1 - beta1^t), formed in fp64
float adam_scale(int64_t t, float r, float beta1, float beta2) {
    const double c1 = 1.0 - pow((double)beta1, (double)t), c2 = 1.0 - pow((double)beta2, (double)t);
    return (float)((double)r * sqrt(c2) / c1);
}
}  // namespace

int arn_adam_update(size_t n, float *theta, const float *g, float *m, float *v, int64_t t, float r, float beta1,
                    float beta2, float eps, const arn_config *cfg, void *w_packed, void *stream) {
    bool repack;
    Dims d;
    if (int e = check_update(n, cfg, w_packed, &repack, &d)) return e;
    if (!aligned(theta, 16) || !aligned(g, 16) || !aligned(m, 16) || !aligned(v, 16)) return ARN_EINVAL;
    if (t < 1 || !unit_interval(beta1) || !unit_interval(beta2) || !(eps >= 0.f) || !(r == r)) return ARN_EINVAL;
    if (int e = check_arch()) return e;
    hipStream_t s = (hipStream_t)stream;
    UpdateArgs p = {};
    p.theta = theta; p.g = g; p.m = m; p.v = v; p.n = (long)n;
    p.a = adam_scale(t, r, beta1, beta2); p.beta1 = beta1; p.beta2 = beta2; p.eps = eps;
    {
        ProfScope ps("adam", s);
        hipLaunchKernelGGL(update_kernel<RULE_ADAM>, dim3(update_blocks(n)), dim3(256), 0, s, p);
    }
    if (repack) launch_pack_all(d, theta, w_packed, s);
    return launched();
}

int arn_async_adam_local_step(size_t n, float *theta, const float *g, float *m, float *v, float *a_g, float *a_g2,
                              float *a_s, int64_t t, float r, float beta1, float beta2, float eps,
                              const arn_config *cfg, void *w_packed, void *stream) {
    bool repack;
    Dims d;
    if (int e = check_update(n, cfg, w_packed, &repack, &d)) return e;
    if (!aligned(theta, 16) || !aligned(g, 16) || !aligned(m, 16) || !aligned(v, 16) || !aligned(a_g, 16) ||
        !aligned(a_g2, 16) || !aligned(a_s, 16))
        return ARN_EINVAL;
    if (t < 1 || !unit_interval(beta1) || !unit_interval(beta2) || !(eps >= 0.f) || !(r == r)) return ARN_EINVAL;
    if (int e = check_arch()) return e;
    hipStream_t s = (hipStream_t)stream;
    UpdateArgs p = {};
    p.theta = theta; p.g = g; p.m = m; p.v = v; p.a_g = a_g; p.a_g2 = a_g2; p.a_s = a_s; p.n = (long)n;
    p.a = adam_scale(t, r, beta1, beta2); p.beta1 = beta1; p.beta2 = beta2; p.eps = eps;
    {
        ProfScope ps("adam_local", s);
        hipLaunchKernelGGL(update_kernel<RULE_ADAM_LOCAL>, dim3(update_blocks(n)), dim3(256), 0, s, p);
    }
    if (repack) launch_pack_all(d, theta, w_packed, s);
    return launched();
}

int arn_async_adam_merge(size_t n, float *theta_c, float *m_c, float *v_c, float *theta, float *m, float *v,
                         float *a_g, float *a_g2, float *a_s, int n_local, float beta1, float beta2,
                         const arn_config *cfg, void *w_packed, void *stream) {
    bool repack;
    Dims d;
    if (int e = check_update(n, cfg, w_packed, &repack, &d)) return e;
    if (!aligned(theta_c, 16) || !aligned(m_c, 16) || !aligned(v_c, 16) || !aligned(theta, 16) || !aligned(m, 16) ||
        !aligned(v, 16) || !aligned(a_g, 16) || !aligned(a_g2, 16) || !aligned(a_s, 16))
        return ARN_EINVAL;
    if (theta_c == theta || m_c == m || v_c == v) return ARN_EINVAL;
    if (n_local < 0 || !unit_interval(beta1) || !unit_interval(beta2)) return ARN_EINVAL;
    if (int e = check_arch()) return e;
    hipStream_t s = (hipStream_t)stream;
    UpdateArgs p = {};
    p.theta_c = theta_c; p.m_c = m_c; p.v_c = v_c; p.theta = theta; p.m = m; p.v = v;
    p.a_g = a_g; p.a_g2 = a_g2; p.a_s = a_s; p.n = (long)n; p.beta1 = beta1; p.beta2 = beta2;
    p.beta1_n = (float)pow((double)beta1, (double)n_local);
    p.beta2_n = (float)pow((double)beta2, (double)n_local);
    {
        ProfScope ps("adam_merge", s);
        hipLaunchKernelGGL(merge_kernel, dim3(update_blocks(n)), dim3(256), 0, s, p);
    }
    if (repack) launch_pack_all(d, theta, w_packed, s);
    return launched();
}

int arn_profile_null(void *stream) {
    // an event pair around nothing: what the instrumentation itself adds to every recorded duration
    ProfScope ps("null", (hipStream_t)stream);
    return ARN_OK;
}

int arn_profile_enable(int on) {
    g_prof_on = on != 0;
    return ARN_OK;
}

int arn_profile_collect(char *names, float *ms, int cap) {
    int n = 0;
    for (const ProfRecord &r : g_prof) {
        float t = 0.f;
        if (r.stop && hipEventSynchronize(r.stop) == hipSuccess) (void)hipEventElapsedTime(&t, r.start, r.stop);
        if (n < cap && names && ms) {
            strncpy(names + (size_t)n * 32, r.name, 31);
            names[(size_t)n * 32 + 31] = 0;
            ms[n] = t;
            ++n;
        }
        if (r.start) (void)hipEventDestroy(r.start);
        if (r.stop) (void)hipEventDestroy(r.stop);
    }
    g_prof.clear();
    return n;
}

}  // extern "C"
