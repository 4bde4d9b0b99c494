// Shapes of the Nature CNN, the packed-weight blob and the workspace carve-up.
// Host-side arithmetic only; shared by the API layer and the kernel launchers.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "../../include/arn.h"

namespace arn {

// network geometry (appendix "Atari Frame Processing": the standard
// 3-convolutional-layer network; 84x84 frames, no padding)
constexpr int IN_C = 4, IN_H = 84, IN_W = 84;
constexpr int OBS_BYTES = IN_C * IN_H * IN_W;            // 28224
constexpr int C1 = 32, K1 = 8, S1 = 4, H1 = 20;          // conv1 out 20x20
constexpr int C2 = 64, K2 = 4, S2 = 2, H2 = 9;           // conv2 out 9x9
constexpr int C3 = 64, K3 = 3, S3 = 1, H3 = 7;           // conv3 out 7x7
constexpr int P1 = H1 * H1, P2 = H2 * H2, P3 = H3 * H3;  // 400, 81, 49
constexpr int KW1 = IN_C * K1 * K1;                      // 256
constexpr int KW2 = C1 * K2 * K2;                        // 512
constexpr int KW3 = C2 * K3 * K3;                        // 576
constexpr int FEAT = C3 * P3;                            // 3136
constexpr int HID = 512;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Frame size and padding of the convolution stack as compile-time constants (the filter shapes above are
// common to both).  Geo84 restates the constants above; GeoPaper is the appendix's own setting: 104x80
// frames, no padding on conv1, padding 1 on conv2 and conv3.
template <int IN_H_, int IN_W_, int PAD2_, int PAD3_>
struct Geometry {
    static constexpr int IN_H = IN_H_, IN_W = IN_W_, PAD2 = PAD2_, PAD3 = PAD3_;
    static constexpr int H1 = (IN_H - K1) / S1 + 1, W1 = (IN_W - K1) / S1 + 1;
    static constexpr int H2 = (H1 + 2 * PAD2 - K2) / S2 + 1, W2 = (W1 + 2 * PAD2 - K2) / S2 + 1;
    static constexpr int H3 = (H2 + 2 * PAD3 - K3) / S3 + 1, W3 = (W2 + 2 * PAD3 - K3) / S3 + 1;
    static constexpr int P1 = H1 * W1, P2 = H2 * W2, P3 = H3 * W3;
    static constexpr int OBS_BYTES = IN_C * IN_H * IN_W, FEAT = C3 * P3;
};
typedef Geometry<84, 84, 0, 0> Geo84;
typedef Geometry<104, 80, 1, 1> GeoPaper;
static_assert(Geo84::P1 == P1 && Geo84::P2 == P2 && Geo84::P3 == P3 && Geo84::FEAT == FEAT, "84x84 constants");
static_assert(GeoPaper::H1 == 25 && GeoPaper::W1 == 19 && GeoPaper::H2 == 12 && GeoPaper::W2 == 9 &&
              GeoPaper::H3 == 12 && GeoPaper::W3 == 9 && GeoPaper::FEAT == 6912, "appendix: 25x19 -> 12x9 -> 12x9");

struct Dims {
    int A = 0, head = 0, atoms = 0;
    int NH = 0;    // real head rows: A+1 (PV, DUEL), A (Q) or A*atoms (C51)
    int NHP = 0;   // head rows padded to a multiple of 64 (MFMA k-tile of the head dgrad)
    bool small = false;   // at most 32 head rows: the fused head kernel follows the fc GEMM (PV, Q, DUEL)
    bool vrow = false;    // the row after the A action rows is a state value (PV, DUEL)
    bool qhead = false;   // the head outputs are action values (Q, DUEL)
    int geom = ARN_GEOM_84;   // geometry of the kernels that run: ARN_GEOM_84 or ARN_GEOM_PAPER
    bool a3c = false;         // the 2-convolution network, embedded in the ARN_GEOM_PAPER network
    int p1 = P1, p2 = P2, p3 = P3, feat = FEAT, obs_bytes = OBS_BYTES;   // positions per sample after conv1..3, fc inputs, bytes per observation
    bool ok = false;
};

inline Dims make_dims(const arn_config *c) {
    Dims d;
    if (!c) return d;
    d.A = c->num_actions;
    d.head = c->head_kind;
    d.geom = c->geometry;
    if (d.geom == ARN_GEOM_A3C) {
        d.a3c = true;
        d.geom = ARN_GEOM_PAPER;
    }
    if (d.geom == ARN_GEOM_PAPER) {
        d.p1 = GeoPaper::P1; d.p2 = GeoPaper::P2; d.p3 = GeoPaper::P3;
        d.feat = GeoPaper::FEAT; d.obs_bytes = GeoPaper::OBS_BYTES;
    } else if (d.geom != ARN_GEOM_84) {
        return d;
    }
    if (d.head == ARN_HEAD_PV || d.head == ARN_HEAD_Q || d.head == ARN_HEAD_DUEL) {
        if (d.A < 1 || d.A > 31) return d;
        d.atoms = 1;
        d.small = true;
        d.vrow = d.head != ARN_HEAD_Q;
        d.qhead = d.head != ARN_HEAD_PV;
        d.NH = d.A + (d.vrow ? 1 : 0);
    } else if (d.head == ARN_HEAD_C51) {
        d.atoms = c->num_atoms;
        if (d.A < 1 || d.A > 18 || d.atoms < 2 || d.atoms > 64) return d;
        if (!(c->v_max > c->v_min)) return d;
        d.NH = d.A * d.atoms;
    } else {
        return d;
    }
    d.NHP = (int)align_up((size_t)d.NH, 64);
    d.ok = true;
    return d;
}

// offsets (in fp32 entries) into the canonical flat parameter vector
struct ParamOffsets {
    size_t w1, b1, w2, b2, w3, b3, wfc, bfc, wh, bh, wv, bv, total;
};
inline ParamOffsets param_offsets(const Dims &d) {
    ParamOffsets o{};
    size_t p = 0;
    o.w1 = p; p += (size_t)C1 * KW1;
    o.b1 = p; p += C1;
    o.w2 = p; p += (size_t)C2 * KW2;
    o.b2 = p; p += C2;
    o.w3 = p; p += (size_t)C3 * KW3;
    o.b3 = p; p += C3;
    o.wfc = p; p += (size_t)HID * d.feat;
    o.bfc = p; p += HID;
    if (d.vrow) {
        o.wh = p; p += (size_t)d.A * HID;
        o.bh = p; p += d.A;
        o.wv = p; p += HID;
        o.bv = p; p += 1;
    } else {
        o.wh = p; p += (size_t)d.NH * HID;
        o.bh = p; p += d.NH;
        o.wv = o.bv = p;
    }
    o.total = p;
    return o;
}

// The 2-convolution network (16 and 32 filters, 256 hidden units, 104x80 frames) as a sub-network of the
// three-convolution one: its filters, hidden units and head columns are the leading ones, everything else is
// zero and conv3 is the identity (centre tap 1 on the diagonal, zero bias).  ReLU of a non-negative map is that
// map, and the sign bits of act3 equal those of act2, so function and gradients are those of the small network.
constexpr int A3C_C1 = 16, A3C_C2 = 32, A3C_HID = 256, A3C_FEAT = A3C_C2 * 12 * 9;
struct A3cMap {   // index of the small network's flat vector -> index of the embedding network's
    long w1, b1, w2, b2, wfc, bfc, wh, bh, wv, bv, total;   // offsets in the small vector
    ParamOffsets e;                                         // offsets in the embedding vector
    int feat;                                               // fc inputs of the embedding network
#if defined(__HIPCC__)
    __host__ __device__
#endif
    long operator()(long i) const {
        if (i < b1) return (long)e.w1 + i;                                   // filters 0..15: the leading rows
        if (i < w2) return (long)e.b1 + (i - b1);
        if (i < b2) {
            const long j = i - w2, co = j / (A3C_C1 * 16), r = j % (A3C_C1 * 16);
            return (long)e.w2 + co * (C1 * 16) + r;                          // [co][ci][4][4]: ci < 16 of 32
        }
        if (i < wfc) return (long)e.b2 + (i - b2);
        if (i < bfc) {
            const long j = i - wfc, n = j / A3C_FEAT, k = j % A3C_FEAT;
            return (long)e.wfc + n * feat + k;                               // input index c*108 + pos, c < 32
        }
        if (i < wh) return (long)e.bfc + (i - bfc);
        if (i < bh) {
            const long j = i - wh;
            return (long)e.wh + (j / A3C_HID) * HID + j % A3C_HID;
        }
        if (i < wv) return (long)e.bh + (i - bh);
        if (i < bv) return (long)e.wv + (i - wv);
        return (long)e.bv + (i - bv);
    }
};
inline A3cMap make_a3c_map(const Dims &d) {
    A3cMap m{};
    long p = 0;
    m.w1 = p; p += (long)A3C_C1 * KW1;
    m.b1 = p; p += A3C_C1;
    m.w2 = p; p += (long)A3C_C2 * A3C_C1 * 16;
    m.b2 = p; p += A3C_C2;
    m.wfc = p; p += (long)A3C_HID * A3C_FEAT;
    m.bfc = p; p += A3C_HID;
    const int rows = d.vrow ? d.A : d.NH;
    m.wh = p; p += (long)rows * A3C_HID;
    m.bh = p; p += rows;
    m.wv = p; p += d.vrow ? A3C_HID : 0;
    m.bv = p; p += d.vrow ? 1 : 0;
    m.total = p;
    m.e = param_offsets(d);
    m.feat = d.feat;
    return m;
}
// entries of the flat parameter / gradient vector at the interface
inline size_t public_param_count(const Dims &d) { return d.a3c ? (size_t)make_a3c_map(d).total : param_offsets(d).total; }

// byte offsets into the packed blob
struct PackedOffsets {
    size_t w1, w2, w3, wfc, wh;          // forward layouts  [N][K'] bf16 (high parts)
    size_t b1, b2, b3, bfc, bh;          // fp32 biases
    size_t w1l, w2l, w3l, wfcl, whl;     // low parts (w - hi) for the three-product inference path
    size_t whd, wfcd, w3d, w2d;          // input-gradient layouts
    size_t w1h, w2h, w3h, wfch;          // fp16 copies of the forward layouts (single-product, no-gradient forward)
    size_t a3c_flat;                     // the embedding network's flat fp32 vector (2-convolution network only)
    size_t fwd_bytes, total;
};
inline PackedOffsets packed_offsets(const Dims &d) {
    PackedOffsets o{};
    size_t p = 0;
    auto take = [&](size_t bytes) { size_t at = p; p = align_up(p + bytes, 256); return at; };
    o.w1 = take((size_t)C1 * KW1 * 2);
    o.w2 = take((size_t)C2 * KW2 * 2);
    o.w3 = take((size_t)C3 * KW3 * 2);
    o.wfc = take((size_t)HID * d.feat * 2);
    o.wh = take((size_t)d.NHP * HID * 2);
    o.b1 = take(C1 * 4);
    o.b2 = take(C2 * 4);
    o.b3 = take(C3 * 4);
    o.bfc = take(HID * 4);
    o.bh = take((size_t)d.NHP * 4);
    o.fwd_bytes = p;
    o.w1l = take((size_t)C1 * KW1 * 2);
    o.w2l = take((size_t)C2 * KW2 * 2);
    o.w3l = take((size_t)C3 * KW3 * 2);
    o.wfcl = take((size_t)HID * d.feat * 2);
    o.whl = take((size_t)d.NHP * HID * 2);
    o.whd = take((size_t)HID * d.NHP * 2);
    o.wfcd = take((size_t)d.feat * HID * 2);
    o.w3d = take((size_t)C2 * KW3 * 2);
    o.w2d = take((size_t)4 * C1 * 4 * C2 * 2);
    o.w1h = take((size_t)C1 * KW1 * 2);
    o.w2h = take((size_t)C2 * KW2 * 2);
    o.w3h = take((size_t)C3 * KW3 * 2);
    o.wfch = take((size_t)HID * d.feat * 2);
    o.a3c_flat = take(d.a3c ? param_offsets(d).total * 4 : 0);
    o.total = p;
    return o;
}

// how many batch slices each weight-gradient GEMM is cut into (fixed function
// of B only, so the summation order -- and the bits of dW -- never change)
struct Splits {
    int c1, c2, c3, fc, hd;
};
inline int pick_split(long rows, int tiles, int target_wgs) {
    long iters = (rows + 63) / 64;
    long s = target_wgs / tiles;
    if (s < 1) s = 1;
    if (s > iters) s = iters;
    return (int)s;
}
// workgroups of the conv2 / conv3 weight gradients: each writes a full fp32 partial of dW, so fewer workgroups
// mean less partial traffic (and a cheaper reduction).  The two are ranges of one grid (conv_backward_kernel) and
// run side by side, one per CU, so together they fill the 256 CUs; the split follows the measured time per sample
// of the two (84x84 network: conv2's 81 positions x 512 columns against conv3's 49 x 576), so that both ranges
// finish together.
inline int wgrad_wgs2(int geom) { return geom == ARN_GEOM_84 ? 148 : 128; }
inline int wgrad_wgs3(int geom) { return 256 - wgrad_wgs2(geom); }
constexpr int CONV2_WG_G = 2, CONV3_WG_G = 4;   // samples staged per iteration by the conv2 / conv3 weight-gradient kernels
// sample-resident weight-gradient kernels: samples per workgroup and number of workgroups
inline int resident_spw(int B, int target_wgs) { return (B + target_wgs - 1) / target_wgs; }
inline int resident_groups(int B, int target_wgs) {
    const int spw = resident_spw(B, target_wgs);
    return (B + spw - 1) / spw;
}
inline Splits make_splits(const Dims &d, int B) {
    Splits s;
    if (d.geom != ARN_GEOM_84) {
        // the dense layers' weight-gradient GEMMs are cut along the batch so that about 512 workgroups exist;
        // the convolutions use the sample-resident kernels, as below
        s.c1 = resident_groups(B, 256);
        s.c2 = resident_groups((B + CONV2_WG_G - 1) / CONV2_WG_G, wgrad_wgs2(d.geom));   // sample-resident kernels, as below
        s.c3 = resident_groups((B + CONV3_WG_G - 1) / CONV3_WG_G, wgrad_wgs3(d.geom));
        s.fc = pick_split(B, (d.feat / 64) * 4, 512);
        s.hd = pick_split(B, 4 * (d.NHP / 64), 256);
        return s;
    }
    s.c1 = resident_groups(B, 256);
    s.c2 = resident_groups((B + CONV2_WG_G - 1) / CONV2_WG_G, wgrad_wgs2(d.geom));
    s.c3 = resident_groups((B + CONV3_WG_G - 1) / CONV3_WG_G, wgrad_wgs3(d.geom));
    s.fc = pick_split(B, 49 * 4, 392);
    s.hd = pick_split(B, 4 * (d.NHP / 64), 256);
    return s;
}

// number of k ranges the fc forward GEMM is cut into (fills the chip when B/128 * 4 tiles are too few)
// f16: the one-product fc layer of the no-gradient forward, whose GEMM is a third of the work: from 128 samples up
// eight ranges are the better trade (inference at 256 samples 25.4 -> 23.8 us per call, at 512 33.7 -> 31.6; at 64 and
// below sixteen stay ahead by half a microsecond, and the three-product layer of the gradient step at every size).
inline int fc_ksplit(int B, bool f16 = false) {
    const int tiles = ((B + 127) / 128) * 4;
    int ks = 256 / tiles;
    if (ks < 1) ks = 1;
    const int cap = f16 && B >= 128 ? 8 : 16;   // the consumer adds the ranges one after the other: more of them costs it more than the GEMM gains
    if (ks > cap) ks = cap;
    return ks;
}

// Samples per workgroup of the fused policy/value head kernel in the gradient step (at most 16): eight keep all
// CUs busy at a few thousand samples; above that sixteen fill the MFMA's 16 sample columns and halve the workgroups;
// small batches are spread over more CUs, four samples each (one CU's L1 rate bounds the addition of the fc partials).
inline int loss_block(int B) { return B >= 4096 ? 16 : B <= 512 ? 4 : 8; }
constexpr int C51_WAVES = 4;      // wavefronts per block in the C51 kernels (one sample per wavefront at a time)
// Samples each wavefront of c51_loss_kernel takes one after the other: a block also writes one fp32 partial of the
// head's bias gradient, so large batches use fewer, longer blocks.
inline int c51_loss_spw(int B) { return B <= 2048 ? 1 : 4; }

// byte offsets into the workspace
struct Workspace {
    size_t a1, a2, a3, h;               // bf16 NHWC activations
    size_t a1l, a2l, a3l, hl;           // their low parts (written and read by the forward pass only)
    size_t fcp;                         // fp32 [ksplit][B][512] partial sums of the fc forward GEMM
    size_t z, zv;                       // categorical head: fp32 atom logits, rows padded to NHP floats
    size_t ztgt, m;                     // C51: target-net atom logits, projected target
    size_t qt, astar;                   // DQN: target-net Q(s',.) fp32 [B][A]; Double-DQN: online greedy action on s' int32 [B]
    size_t m1, m2, m3;                  // ReLU sign bits of act1..3 (bit e&7 of byte e>>3, NHWC element e), written by the forward
    size_t dz, dph, dp3, dp2;           // bf16 gradients at pre-activations (d(pre1) never leaves the chip)
    size_t lossp;                       // fp32 [blocks][4] partial loss sums
    size_t hbp;                         // fp32 [blocks][32 or NHP] partial sums of the head's bias gradient
    size_t pw1, pw2, pw3, pwfc, pwh;    // fp32 weight-gradient partials [split][N*K' + N]
    size_t a3c_dw;                      // gradient of the embedding network (2-convolution network only)
    size_t total;
};
inline int loss_blocks(const Dims &d, int B) {
    const int per = d.small ? loss_block(B) : C51_WAVES * c51_loss_spw(B);
    return (B + per - 1) / per;
}
inline Workspace make_workspace(const Dims &d, int B, int mode) {
    Workspace w{};
    size_t p = 0;
    auto take = [&](size_t bytes) { size_t at = p; p = align_up(p + bytes, 256); return at; };
    const size_t b = (size_t)B;
    const size_t p1 = (size_t)d.p1, p2 = (size_t)d.p2, feat = (size_t)d.feat;
    w.a1 = take(b * p1 * C1 * 2);
    w.a2 = take(b * p2 * C2 * 2);
    w.a3 = take(b * feat * 2);
    w.h = take(b * HID * 2);
    w.a1l = take(b * p1 * C1 * 2);
    w.a2l = take(b * p2 * C2 * 2);
    w.a3l = take(b * feat * 2);
    w.hl = take(b * HID * 2);
    // the fused policy/value head kernel always reads fp32 partials; the categorical path only when k is split
    w.fcp = take((size_t)(fc_ksplit(B) > 1 || d.small ? fc_ksplit(B) : 0) * b * HID * 4);
    // categorical head: atom logits of arn_policy_act (arn_policy_forward writes them to its `logits` argument)
    if (mode == ARN_MODE_FORWARD) w.z = take(d.small ? 0 : b * (size_t)d.NHP * 4);
    if (mode == ARN_MODE_TRAIN) {
        w.z = take(d.small ? 0 : b * (size_t)d.NHP * 4);
        w.zv = 0;
        if (d.qhead) {
            w.qt = take(b * (size_t)d.A * 4);
            w.astar = take(b * 4);
        }
        if (d.head == ARN_HEAD_C51) {
            w.ztgt = take(b * (size_t)d.NHP * 4);
            w.m = take(b * (size_t)d.atoms * 4);
        }
        w.m1 = take(b * p1 * C1 / 8);
        w.m2 = take(b * p2 * C2 / 8);
        w.m3 = take(b * feat / 8);
        w.dz = take(b * (size_t)d.NHP * 2);
        w.dph = take(b * HID * 2);
        w.dp3 = take(b * feat * 2);
        w.dp2 = take(b * p2 * C2 * 2);
        w.lossp = take((size_t)loss_blocks(d, B) * 4 * 4);
        w.hbp = take((size_t)loss_blocks(d, B) * (d.small ? 32 : d.NHP) * 4);
        const Splits s = make_splits(d, B);
        w.pw1 = take((size_t)s.c1 * ((size_t)C1 * KW1 + C1) * 4);
        w.pw2 = take((size_t)s.c2 * ((size_t)C2 * KW2 + C2) * 4);
        w.pw3 = take((size_t)s.c3 * ((size_t)C3 * KW3 + C3) * 4);
        w.pwfc = take((size_t)s.fc * ((size_t)HID * feat + HID) * 4);
        w.pwh = take((size_t)s.hd * ((size_t)d.NHP * HID + d.NHP) * 4);
        w.a3c_dw = take(d.a3c ? param_offsets(d).total * 4 : 0);
    }
    w.total = p;
    return w;
}

}  // namespace arn
