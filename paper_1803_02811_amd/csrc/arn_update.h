// Parameter update rules on the flat fp32 vector (appendix "Update Rule for Multi-Step Asynchronous Adam";
// RMSProp as named in appendix "Experiment Details"), and the single-launch conversion of the flat
// parameters into every packed layout the network kernels read.
//
// The update kernels are elementwise and HBM-bound: every thread owns four consecutive parameters and moves
// each state array with one 16-byte load and one 16-byte store.  All arithmetic is fp32; scalars that
// depend on the step count (the bias-correction factor a, beta^n of a merge) are formed on the host in
// fp64 and passed in.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "arn_gemm.h"
#include "arn_layout.h"
#include "arn_small_kernels.h"

namespace arn {

typedef float f32x4u __attribute__((ext_vector_type(4)));

enum { RULE_RMSPROP = 0, RULE_ADAM = 1, RULE_ADAM_LOCAL = 2, RULE_MERGE = 3 };

struct UpdateArgs {
    float *theta, *m, *v;          // RMSProp: v = accumulator of squared gradients, m unused
    const float *g;
    float *a_g, *a_g2, *a_s;       // local accumulators (RULE_ADAM_LOCAL, RULE_MERGE)
    float *theta_c, *m_c, *v_c;    // central values (RULE_MERGE)
    long n;
    float a;                       // RMSProp: learning rate; Adam: r*sqrt(1-beta2^t)/(1-beta1^t)
    float beta1, beta2;            // RMSProp: beta2 = rho.  RULE_MERGE: coefficients (1-beta1), (1-beta2) use these
    float eps;
    float beta1_n, beta2_n;        // RULE_MERGE: beta^n
};

// One element of a rule.  State goes in and out through references so that the vector and the tail path
// share the arithmetic.
template <int RULE>
struct Elem {
    static __device__ __forceinline__ void apply(const UpdateArgs &p, float &th, float &m, float &v, float g,
                                                  float &ag, float &ag2, float &as) {
        if constexpr (RULE == RULE_RMSPROP) {
            v = p.beta2 * v + (1.f - p.beta2) * g * g;
            th = th - p.a * g / sqrtf(v + p.eps);
        } else {
            m = p.beta1 * m + (1.f - p.beta1) * g;
            v = p.beta2 * v + (1.f - p.beta2) * g * g;
            const float s = p.a * m / (sqrtf(v) + p.eps);
            th = th - s;
            if constexpr (RULE == RULE_ADAM_LOCAL) {
                ag = p.beta1 * ag + g;
                ag2 = p.beta2 * ag2 + g * g;
                as = as + s;
            }
        }
    }
};

template <int RULE>
__global__ __launch_bounds__(256) void update_kernel(UpdateArgs p) {
    const long q = (long)blockIdx.x * 256 + threadIdx.x;   // group of four
    const long i0 = q * 4;
    if (i0 >= p.n) return;
    if (i0 + 4 <= p.n) {
        f32x4u th = *(const f32x4u *)(p.theta + i0), g = *(const f32x4u *)(p.g + i0);
        f32x4u v = *(const f32x4u *)(p.v + i0), m = 0.f, ag = 0.f, ag2 = 0.f, as = 0.f;
        if constexpr (RULE != RULE_RMSPROP) m = *(const f32x4u *)(p.m + i0);
        if constexpr (RULE == RULE_ADAM_LOCAL) {
            ag = *(const f32x4u *)(p.a_g + i0);
            ag2 = *(const f32x4u *)(p.a_g2 + i0);
            as = *(const f32x4u *)(p.a_s + i0);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float t = th[e], mm = m[e], vv = v[e], x = ag[e], y = ag2[e], z = as[e];
            Elem<RULE>::apply(p, t, mm, vv, g[e], x, y, z);
            th[e] = t; m[e] = mm; v[e] = vv; ag[e] = x; ag2[e] = y; as[e] = z;
        }
        *(f32x4u *)(p.theta + i0) = th;
        *(f32x4u *)(p.v + i0) = v;
        if constexpr (RULE != RULE_RMSPROP) *(f32x4u *)(p.m + i0) = m;
        if constexpr (RULE == RULE_ADAM_LOCAL) {
            *(f32x4u *)(p.a_g + i0) = ag;
            *(f32x4u *)(p.a_g2 + i0) = ag2;
            *(f32x4u *)(p.a_s + i0) = as;
        }
    } else {
        for (long i = i0; i < p.n; ++i) {
            float t = p.theta[i], vv = p.v[i], mm = 0.f, x = 0.f, y = 0.f, z = 0.f;
            if constexpr (RULE != RULE_RMSPROP) mm = p.m[i];
            if constexpr (RULE == RULE_ADAM_LOCAL) { x = p.a_g[i]; y = p.a_g2[i]; z = p.a_s[i]; }
            Elem<RULE>::apply(p, t, mm, vv, p.g[i], x, y, z);
            p.theta[i] = t; p.v[i] = vv;
            if constexpr (RULE != RULE_RMSPROP) p.m[i] = mm;
            if constexpr (RULE == RULE_ADAM_LOCAL) { p.a_g[i] = x; p.a_g2[i] = y; p.a_s[i] = z; }
        }
    }
}

// Merge of one learner's accumulated steps into the central values; the local copies take the new
// central values and the accumulators are cleared (third block of equations of the appendix).
__global__ __launch_bounds__(256) void merge_kernel(UpdateArgs p) {
    const long i0 = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i0 >= p.n) return;
    const float c1 = 1.f - p.beta1, c2 = 1.f - p.beta2;
    if (i0 + 4 <= p.n) {
        const f32x4u th = *(const f32x4u *)(p.theta_c + i0) - *(const f32x4u *)(p.a_s + i0);
        const f32x4u m = p.beta1_n * *(const f32x4u *)(p.m_c + i0) + c1 * *(const f32x4u *)(p.a_g + i0);
        const f32x4u v = p.beta2_n * *(const f32x4u *)(p.v_c + i0) + c2 * *(const f32x4u *)(p.a_g2 + i0);
        const f32x4u zero = 0.f;
        *(f32x4u *)(p.theta_c + i0) = th; *(f32x4u *)(p.theta + i0) = th;
        *(f32x4u *)(p.m_c + i0) = m; *(f32x4u *)(p.m + i0) = m;
        *(f32x4u *)(p.v_c + i0) = v; *(f32x4u *)(p.v + i0) = v;
        *(f32x4u *)(p.a_g + i0) = zero; *(f32x4u *)(p.a_g2 + i0) = zero; *(f32x4u *)(p.a_s + i0) = zero;
    } else {
        for (long i = i0; i < p.n; ++i) {
            const float th = p.theta_c[i] - p.a_s[i];
            const float m = p.beta1_n * p.m_c[i] + c1 * p.a_g[i];
            const float v = p.beta2_n * p.v_c[i] + c2 * p.a_g2[i];
            p.theta_c[i] = th; p.theta[i] = th;
            p.m_c[i] = m; p.m[i] = m;
            p.v_c[i] = v; p.v[i] = v;
            p.a_g[i] = 0.f; p.a_g2[i] = 0.f; p.a_s[i] = 0.f;
        }
    }
}

// ------------------------- all packed layouts in one launch -------------------------
// The packed blob has 14 regions (five forward weight matrices with their lo parts, five bias vectors,
// four input-gradient layouts).  One launch covers them all: a block finds the region its index falls in
// (uniform per block) and applies that region's index map.
enum {
    PK_W1 = 0, PK_W2, PK_W3, PK_WFC, PK_WH, PK_B1, PK_B2, PK_B3, PK_BFC, PK_BH, PK_WHD, PK_WFCD, PK_W3D, PK_W2D,
    PK_COUNT
};
struct PackSeg {
    int first_block;
    long n;
    void *out, *out_lo;
    void *out_f16;     // fp16 copy of a forward layout, or null
};
// The fc matrix (95 % of the parameters) is laid out by tile blocks instead: elementwise maps would read it with
// a stride of one row (input-gradient layout) or of P3 floats (forward layout).  A tile is PACK_FC_ROWS hidden
// units x PACK_FC_CH conv3 channels x all P3 positions -- contiguous runs of PACK_FC_CH * P3 floats in the flat
// vector -- staged in LDS and written out as 16-byte words of eight channels (forward layout, hi and lo) and of
// eight hidden units (input-gradient layout).  Eight rows per tile measured best (12.2 us for the whole launch
// against 13.1 with sixteen and 16 with thirty-two; the elementwise maps took 18.3).
constexpr int PACK_FC_ROWS = 8, PACK_FC_CH = 8;
// fp16 copy of a weight: values beyond the largest half are clamped to it instead of becoming infinite
__device__ __forceinline__ _Float16 to_f16_finite(float v) { return (_Float16)fminf(fmaxf(v, -65504.f), 65504.f); }
constexpr int PACK_FC_MAX_P3 = 108;   // 12 x 9 positions after conv3 on 104 x 80 frames
static_assert(P3 <= PACK_FC_MAX_P3 && GeoPaper::P3 <= PACK_FC_MAX_P3, "fc tile buffer");
static_assert(HID % PACK_FC_ROWS == 0 && C3 % PACK_FC_CH == 0 && PACK_FC_CH == 8 && PACK_FC_ROWS % 8 == 0, "fc tile shape");
struct PackPlan {
    PackSeg seg[PK_COUNT];
    int fc_first_block;                      // blocks from here on are fc tiles
    __bf16 *fc_hi, *fc_lo, *fc_dgrad;
    _Float16 *fc_f16;
    long w1, w2, w3, wfc, b1, b2, b3, bfc;   // offsets in the flat vector
    MapHeadRow hr;
    int NHP;
    int small_head; // the head's matrices are read by pv_head_kernel as register fragments: fragment order
    int feat, p3;   // fc inputs and positions after conv3
    int blocks;
};

inline PackPlan make_pack_plan(const Dims &d, void *w_packed) {
    const ParamOffsets po = param_offsets(d);
    const PackedOffsets o = packed_offsets(d);
    char *b = (char *)w_packed;
    PackPlan pl;
    pl.w1 = (long)po.w1; pl.w2 = (long)po.w2; pl.w3 = (long)po.w3; pl.wfc = (long)po.wfc;
    pl.b1 = (long)po.b1; pl.b2 = (long)po.b2; pl.b3 = (long)po.b3; pl.bfc = (long)po.bfc;
    pl.hr = head_rows(d, po);
    pl.NHP = d.NHP;
    pl.small_head = d.small ? 1 : 0;
    pl.feat = d.feat;
    pl.p3 = d.p3;
    auto set = [&](int k, long n, size_t out, size_t lo, bool has_lo) {
        pl.seg[k].n = n;
        pl.seg[k].out = b + out;
        pl.seg[k].out_lo = has_lo ? b + lo : nullptr;
        pl.seg[k].out_f16 = nullptr;
    };
    set(PK_W1, (long)C1 * KW1, o.w1, o.w1l, true);
    set(PK_W2, (long)C2 * KW2, o.w2, o.w2l, true);
    set(PK_W3, (long)C3 * KW3, o.w3, o.w3l, true);
    set(PK_WFC, 0, o.wfc, o.wfcl, true);          // by tile blocks, below
    set(PK_WH, (long)d.NHP * HID, o.wh, o.whl, true);
    set(PK_B1, C1, o.b1, 0, false);
    set(PK_B2, C2, o.b2, 0, false);
    set(PK_B3, C3, o.b3, 0, false);
    set(PK_BFC, HID, o.bfc, 0, false);
    set(PK_BH, d.NHP, o.bh, 0, false);
    set(PK_WHD, (long)HID * d.NHP, o.whd, 0, false);
    set(PK_WFCD, 0, o.wfcd, 0, false);            // by tile blocks, below
    pl.seg[PK_W1].out_f16 = b + o.w1h; pl.seg[PK_W2].out_f16 = b + o.w2h; pl.seg[PK_W3].out_f16 = b + o.w3h;
    pl.fc_hi = (__bf16 *)(b + o.wfc); pl.fc_lo = (__bf16 *)(b + o.wfcl); pl.fc_dgrad = (__bf16 *)(b + o.wfcd);
    pl.fc_f16 = (_Float16 *)(b + o.wfch);
    set(PK_W3D, (long)C2 * KW3, o.w3d, 0, false);
    set(PK_W2D, (long)4 * C1 * 256, o.w2d, 0, false);
    int blk = 0;
    for (int k = 0; k < PK_COUNT; ++k) {
        pl.seg[k].first_block = blk;
        blk += (int)((pl.seg[k].n + 255) / 256);
    }
    pl.fc_first_block = blk;
    pl.blocks = blk + (HID / PACK_FC_ROWS) * (C3 / PACK_FC_CH);
    return pl;
}

// One fc tile: hidden units n0 .. n0 + PACK_FC_ROWS - 1, conv3 channels c0 .. c0 + PACK_FC_CH - 1.
// Flat order Wfc[n][c * P3 + pos]; forward layout [n][pos * 64 + c]; input-gradient layout [pos * 64 + c][n].
template <int P3_>
__device__ __forceinline__ void pack_fc_tile(const PackPlan &pl, const float *__restrict__ w, int tile,
                                             float (&s_t)[PACK_FC_ROWS][PACK_FC_CH * PACK_FC_MAX_P3]) {
    constexpr int p3 = P3_, feat = C3 * P3_, run = PACK_FC_CH * p3;
    constexpr int NL = (PACK_FC_ROWS * run + 255) / 256;
    const int n0 = (tile / (C3 / PACK_FC_CH)) * PACK_FC_ROWS, c0 = (tile % (C3 / PACK_FC_CH)) * PACK_FC_CH;
    const int tid = threadIdx.x;
    float v_in[NL];   // all loads of the tile in flight before the first is used
#pragma unroll
    for (int j = 0; j < NL; ++j) {
        int i = tid + 256 * j;
        i = i < PACK_FC_ROWS * run ? i : PACK_FC_ROWS * run - 1;
        const int r = i / run, e = i - r * run;
        v_in[j] = w[pl.wfc + (long)(n0 + r) * feat + (long)c0 * p3 + e];
    }
#pragma unroll
    for (int j = 0; j < NL; ++j) {
        const int i = tid + 256 * j;
        if (i < PACK_FC_ROWS * run) s_t[i / run][i % run] = v_in[j];
    }
    __syncthreads();
    // forward layout: one 16-byte word = channels c0 .. c0+7 of (row r, position pos)
    for (int i = tid; i < PACK_FC_ROWS * p3; i += 256) {
        const int r = i / p3, pos = i - r * p3;
        float v[PACK_FC_CH];
#pragma unroll
        for (int c = 0; c < PACK_FC_CH; ++c) v[c] = s_t[r][c * p3 + pos];
        bf16x8 hi, lo;
        f16x8 hf;
#pragma unroll
        for (int c = 0; c < PACK_FC_CH; ++c) {
            hi[c] = (__bf16)v[c];
            lo[c] = (__bf16)(v[c] - (float)hi[c]);
            hf[c] = to_f16_finite(v[c]);
        }
        const size_t at = (size_t)(n0 + r) * feat + (size_t)pos * C3 + c0;
        *reinterpret_cast<bf16x8 *>(pl.fc_hi + at) = hi;
        *reinterpret_cast<bf16x8 *>(pl.fc_lo + at) = lo;
        *reinterpret_cast<f16x8 *>(pl.fc_f16 + at) = hf;
    }
    // input-gradient layout: one 16-byte word = hidden units n0 + 8h .. + 7 of (position pos, channel c)  (h = 0 with eight rows)
    for (int i = tid; i < (PACK_FC_ROWS / 8) * run; i += 256) {
        const int h = i / run, e = i - h * run, c = e / p3, pos = e - c * p3;
        bf16x8 hi;
#pragma unroll
        for (int r = 0; r < 8; ++r) hi[r] = (__bf16)s_t[8 * h + r][e];
        *reinterpret_cast<bf16x8 *>(pl.fc_dgrad + ((size_t)pos * C3 + c0 + c) * HID + n0 + 8 * h) = hi;
    }
}

// ---- the 2-convolution network inside the three-convolution one (A3cMap, arn_layout.h) ----
// fill: zeros everywhere, ones on conv3's identity taps W3[c][c][1][1]
__global__ __launch_bounds__(256) void a3c_fill_kernel(float *__restrict__ big, long total, long w3) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    float v = 0.f;
    const long j = i - w3;
    if (j >= 0 && j < (long)C3 * KW3) {
        const long co = j / KW3, r = j % KW3, ci = r / (K3 * K3), t = r % (K3 * K3);
        v = (co == ci && t == (K3 * K3) / 2) ? 1.f : 0.f;
    }
    big[i] = v;
}
// scatter the small network's parameters into the embedding vector / gather its gradient out of it
__global__ __launch_bounds__(256) void a3c_scatter_kernel(A3cMap m, const float *__restrict__ small, float *__restrict__ big) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i < m.total) big[m(i)] = small[i];
}
__global__ __launch_bounds__(256) void a3c_gather_kernel(A3cMap m, const float *__restrict__ big, float *__restrict__ small) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i < m.total) small[i] = big[m(i)];
}

__global__ __launch_bounds__(256) void pack_all_kernel(PackPlan pl, const float *__restrict__ w) {
    if ((int)blockIdx.x >= pl.fc_first_block) {
        __shared__ float s_t[PACK_FC_ROWS][PACK_FC_CH * PACK_FC_MAX_P3];
        const int tile = (int)blockIdx.x - pl.fc_first_block;
        if (pl.p3 == P3) pack_fc_tile<P3>(pl, w, tile, s_t);
        else pack_fc_tile<GeoPaper::P3>(pl, w, tile, s_t);
        return;
    }
    int k = 0;
#pragma unroll
    for (int j = 1; j < PK_COUNT; ++j) k = (int)blockIdx.x >= pl.seg[j].first_block ? j : k;
    // region fields selected without dynamic indexing of the argument block
    int first = 0;
    long n = 0;
    void *out = nullptr, *out_lo = nullptr, *out_f16 = nullptr;
#pragma unroll
    for (int j = 0; j < PK_COUNT; ++j)
        if (j == k) { first = pl.seg[j].first_block; n = pl.seg[j].n; out = pl.seg[j].out; out_lo = pl.seg[j].out_lo; out_f16 = pl.seg[j].out_f16; }
    const long i = (long)((int)blockIdx.x - first) * 256 + threadIdx.x;
    if (i >= n) return;
    long s;
    switch (k) {
    case PK_W1: s = pl.w1 + i; break;
    case PK_W2: s = MapConvFwd<C1, K2>{pl.w2}(i); break;
    case PK_W3: s = MapConvFwd<C2, K3>{pl.w3}(i); break;
    case PK_WFC: s = MapFcFwd{pl.wfc, pl.feat, pl.p3}(i); break;
    case PK_WH: s = MapHeadFwd{pl.hr}(i); break;
    case PK_B1: s = pl.b1 + i; break;
    case PK_B2: s = pl.b2 + i; break;
    case PK_B3: s = pl.b3 + i; break;
    case PK_BFC: s = pl.bfc + i; break;
    case PK_BH: s = MapHeadBias{pl.hr}(i); break;
    case PK_WHD: s = MapHeadDgrad{pl.hr, pl.NHP}(i); break;
    case PK_WFCD: s = MapFcDgrad{pl.wfc, pl.feat, pl.p3}(i); break;
    case PK_W3D: s = MapConv3Dgrad{pl.w3}(i); break;
    default: s = MapConv2Dgrad{pl.w2}(i); break;
    }
    const float v = s >= 0 ? w[s] : 0.f;
    if (k >= PK_B1 && k <= PK_BH) {
        ((float *)out)[i] = v;
    } else {
        // the convolution weights live in registers as MFMA fragments: packed in fragment order (frag_index)
        long o = i;
        if (k == PK_W1) o = frag_index(i / KW1, i % KW1, KW1);
        else if (k == PK_W2) o = frag_index(i / KW2, i % KW2, KW2);
        else if (k == PK_W3 || k == PK_W3D) o = frag_index(i / KW3, i % KW3, KW3);
        else if (k == PK_W2D) o = frag_index(i / 256, i % 256, 256);
        else if (k == PK_WH && pl.small_head) o = frag_index(i / HID, i % HID, HID);
        else if (k == PK_WHD && pl.small_head) o = frag_index(i / 64, i % 64, 64);
        const __bf16 hi = (__bf16)v;
        ((__bf16 *)out)[o] = hi;
        if (out_lo) ((__bf16 *)out_lo)[o] = (__bf16)(v - (float)hi);
        if (out_f16) ((_Float16 *)out_f16)[o] = to_f16_finite(v);
    }
}

}  // namespace arn
