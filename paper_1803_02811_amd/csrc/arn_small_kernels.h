// Everything that is not a contraction: weight packing, the softmax / loss /
// categorical-projection kernels (plain fp32 ALU work with wavefront and block
// reductions in a fixed order), and the ordered reduction of weight-gradient
// partials into the canonical flat gradient vector.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "arn_lanes.h"
#include "arn_layout.h"

namespace arn {

// ----------------------------- weight packing ------------------------------
// F maps a packed element index to the index of its source in the flat fp32
// vector (or -1 for padding); pack_all_kernel applies the maps, writing
// hi = bf16(w) and, for forward layouts, the residual lo = bf16(w - hi) used by
// the three-product forward path.
struct MapIdentity {   // conv1: canonical order is already [co][ci*64+ky*8+kx]
    long off;
    __device__ long operator()(long i) const { return off + i; }
};
template <int CIN, int KS>
struct MapConvFwd {    // packed [co][(ky*KS+kx)*CIN+ci]  <-  W[co][ci][ky][kx]
    long off;
    __device__ long operator()(long i) const {
        constexpr int KW = CIN * KS * KS;
        const int co = (int)(i / KW), k = (int)(i % KW);
        const int tap = k / CIN, ci = k % CIN, ky = tap / KS, kx = tap % KS;
        return off + (((long)co * CIN + ci) * KS + ky) * KS + kx;
    }
};
struct MapFcFwd {      // packed [n][pos*64+c]  <-  Wfc[n][c*P3+pos]   (P3 positions after conv3, feat = 64 P3)
    long off;
    int feat, p3;
    __device__ long operator()(long i) const {
        const int n = (int)(i / feat), k = (int)(i % feat), pos = k >> 6, c = k & 63;
        return off + (long)n * feat + c * p3 + pos;
    }
};
struct MapHeadRow {    // head row r of the packed head -> offset of its weight row / bias, or -1 (pv: A action rows then a value row)
    long wh, wv, bh, bv;
    int A, NH, pv;
    __device__ long wrow(int r) const {
        if (pv) return r < A ? wh + (long)r * HID : (r == A ? wv : -1);
        return r < NH ? wh + (long)r * HID : -1;
    }
    __device__ long brow(int r) const {
        if (pv) return r < A ? bh + r : (r == A ? bv : -1);
        return r < NH ? bh + r : -1;
    }
};
inline MapHeadRow head_rows(const Dims &d, const ParamOffsets &po) {
    MapHeadRow h;
    h.wh = (long)po.wh; h.wv = (long)po.wv; h.bh = (long)po.bh; h.bv = (long)po.bv;
    h.A = d.A; h.NH = d.NH; h.pv = d.vrow;
    return h;
}
struct MapHeadFwd {    // packed [r][j]
    MapHeadRow h;
    __device__ long operator()(long i) const {
        const long b = h.wrow((int)(i / HID));
        return b < 0 ? -1 : b + i % HID;
    }
};
struct MapHeadBias {
    MapHeadRow h;
    __device__ long operator()(long i) const { return h.brow((int)i); }
};
struct MapHeadDgrad {  // packed [j][r]  (NHP columns)
    MapHeadRow h;
    int NHP;
    __device__ long operator()(long i) const {
        const long b = h.wrow((int)(i % NHP));
        return b < 0 ? -1 : b + i / NHP;
    }
};
struct MapFcDgrad {    // packed [pos*64+c][n]  <-  Wfc[n][c*P3+pos]
    long off;
    int feat, p3;
    __device__ long operator()(long i) const {
        const int k = (int)(i / HID), n = (int)(i % HID), pos = k >> 6, c = k & 63;
        return off + (long)n * feat + c * p3 + pos;
    }
};
struct MapConv3Dgrad { // packed [ci][(ty*3+tx)*64+co]  <-  W3[co][ci][2-ty][2-tx]
    long off;
    __device__ long operator()(long i) const {
        const int ci = (int)(i / KW3), k = (int)(i % KW3), tap = k >> 6, co = k & 63, ty = tap / 3, tx = tap % 3;
        return off + (((long)co * C2 + ci) * K3 + (2 - ty)) * K3 + (2 - tx);
    }
};
struct MapConv2Dgrad { // packed [z][ci][(ty*2+tx)*64+co]  <-  W2[co][ci][py+2(1-ty)][px+2(1-tx)]
    long off;
    __device__ long operator()(long i) const {
        const int z = (int)(i / (C1 * 256)), rem = (int)(i % (C1 * 256));
        const int ci = rem / 256, k = rem % 256, tap = k >> 6, co = k & 63, ty = tap >> 1, tx = tap & 1;
        const int ky = (z >> 1) + 2 * (1 - ty), kx = (z & 1) + 2 * (1 - tx);
        return off + (((long)co * C1 + ci) * K2 + ky) * K2 + kx;
    }
};

// --------------------- ordered reduction of wgrad partials ------------------
// dW[map(n,k)] = wscale * sum_s part[s][n*KP + k];  db[bmap(n)] = sum_s part[s][N1*KP + n]
// F maps an index of the [N1*KP + N1] partial block to the flat gradient index (or -1);
// the first `wcount` entries of the block are weights, the rest biases.
// A block of 256 threads reduces 256/ng outputs: ng thread groups (1, 2, 4 or 8)
// each add a contiguous share of the splits in split order, then the group sums
// are added in group order -- a fixed association, so the result is bit-reproducible.
template <class F>
__global__ __launch_bounds__(256) void reduce_partials_kernel(F f, const float *__restrict__ part,
                                                              float *__restrict__ dW, long block, long wcount,
                                                              int splits, float wscale, int ng) {
    __shared__ float red[256];
    const int opb = 256 / ng;
    const int o = threadIdx.x % opb, q = threadIdx.x / opb;
    const long i = (long)blockIdx.x * opb + o;
    const int per = (splits + ng - 1) / ng;
    const int k0 = q * per, k1 = k0 + per < splits ? k0 + per : splits;
    float s = 0.f;
    if (i < block) {
        int k = k0;
        for (; k + 8 <= k1; k += 8) {     // eight independent loads in flight, added in split order
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = part[(size_t)(k + j) * block + i];
#pragma unroll
            for (int j = 0; j < 8; ++j) s += v[j];
        }
        for (; k < k1; ++k) s += part[(size_t)k * block + i];
    }
    red[threadIdx.x] = s;
    __syncthreads();
    if (q == 0 && i < block) {
        const long dst = f(i);
        if (dst < 0) return;
        float t = red[o];
        for (int g = 1; g < ng; ++g) t += red[g * opb + o];
        dW[dst] = i < wcount ? t * wscale : t;
    }
}
// The same reduction for the three convolutions in one launch: a block finds the layer its index falls in
// (uniform per block) and applies that layer's index map.
struct ReduceSeg {
    const float *part;
    long block, wcount;     // entries per partial ([N*K' + N]); how many of them are weights
    int splits, ng, first_block;
    float wscale;
};
inline ReduceSeg make_reduce_seg(const float *part, long wcount, long bcount, int splits, float wscale) {
    ReduceSeg g;
    g.part = part; g.block = wcount + bcount; g.wcount = wcount; g.splits = splits; g.wscale = wscale;
    g.ng = splits >= 64 ? 8 : splits >= 16 ? 4 : splits >= 4 ? 2 : 1;
    g.first_block = 0;
    return g;
}
struct ConvReducePlan {
    ReduceSeg seg[3];       // conv1, conv2, conv3
    long w1, b1, w2, b2, w3, b3;
};

// The fc layer's partials are [n][pos*64 + c] while the canonical weight is [n][c*P3 + pos]: one workgroup
// per output row n adds the splits with contiguous reads, permutes the row in LDS (stride 49 words at
// 84x84: no bank conflicts) and writes it out contiguously.  Workgroup HID handles the bias gradient.
template <int FEAT, int P3>
__global__ __launch_bounds__(256) void fc_reduce_kernel(const float *__restrict__ part, float *__restrict__ dW,
                                                        long woff, long boff, int splits) {
    __shared__ float row[FEAT];
    constexpr long block = (long)HID * FEAT + HID;
    const int n = blockIdx.x, tid = threadIdx.x;
    if (n == HID) {
        for (int j = tid; j < HID; j += 256) {
            float s = 0.f;
            for (int k = 0; k < splits; ++k) s += part[(size_t)k * block + (long)HID * FEAT + j];
            dW[boff + j] = s;
        }
        return;
    }
    // four consecutive k per thread and pass (same position, channels c .. c+3); all loads of a split are issued
    // before the first is added, and the splits are added in order
    static_assert(FEAT % 4 == 0 && ((long)HID * FEAT + HID) % 4 == 0, "16-byte loads of the partials");
    constexpr int NV = (FEAT / 4 + 255) / 256;
    float4 acc[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int q = 0; q < splits; ++q) {
        const float4 *src = reinterpret_cast<const float4 *>(part + (size_t)q * block + (long)n * FEAT);
        float4 v[NV];
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int k4 = tid + 256 * j;
            v[j] = src[k4 < FEAT / 4 ? k4 : FEAT / 4 - 1];
        }
#pragma unroll
        for (int j = 0; j < NV; ++j) { acc[j].x += v[j].x; acc[j].y += v[j].y; acc[j].z += v[j].z; acc[j].w += v[j].w; }
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int k = 4 * (tid + 256 * j);
        if (k < FEAT) {
            const int at = (k & 63) * P3 + (k >> 6);
            row[at] = acc[j].x; row[at + P3] = acc[j].y; row[at + 2 * P3] = acc[j].z; row[at + 3 * P3] = acc[j].w;
        }
    }
    __syncthreads();
    for (int i = tid; i < FEAT; i += 256) dW[woff + (long)n * FEAT + i] = row[i];
}

template <int CIN, int KS, int COUT>
struct UnmapConv {     // partial [co][(ky*KS+kx)*CIN+ci] then [co] bias
    long woff, boff;
    __device__ long operator()(long i) const {
        constexpr int KW = CIN * KS * KS;
        if (i >= (long)COUT * KW) return boff + (i - (long)COUT * KW);
        const int co = (int)(i / KW), k = (int)(i % KW);
        const int tap = k / CIN, ci = k % CIN, ky = tap / KS, kx = tap % KS;
        return woff + (((long)co * CIN + ci) * KS + ky) * KS + kx;
    }
};
struct UnmapConv1 {
    long woff, boff;
    __device__ long operator()(long i) const { return i >= C1 * KW1 ? boff + (i - C1 * KW1) : woff + i; }
};
__global__ __launch_bounds__(256) void conv_reduce_kernel(ConvReducePlan pl, float *__restrict__ dW) {
    __shared__ float red[256];
    const int k = (int)blockIdx.x >= pl.seg[2].first_block ? 2 : ((int)blockIdx.x >= pl.seg[1].first_block ? 1 : 0);
    // segment fields selected without dynamic indexing of the argument block
    const ReduceSeg g = k == 2 ? pl.seg[2] : (k == 1 ? pl.seg[1] : pl.seg[0]);
    const int opb = 256 / g.ng;
    const int o = threadIdx.x % opb, q = threadIdx.x / opb;
    const long i = (long)((int)blockIdx.x - g.first_block) * opb + o;
    const int per = (g.splits + g.ng - 1) / g.ng;
    const int k0 = q * per, k1 = k0 + per < g.splits ? k0 + per : g.splits;
    float s = 0.f;
    if (i < g.block) {
        int z = k0;
        for (; z + 8 <= k1; z += 8) {     // eight independent loads in flight, added in split order
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = g.part[(size_t)(z + j) * g.block + i];
#pragma unroll
            for (int j = 0; j < 8; ++j) s += v[j];
        }
        for (; z < k1; ++z) s += g.part[(size_t)z * g.block + i];
    }
    red[threadIdx.x] = s;
    __syncthreads();
    if (q == 0 && i < g.block) {
        const long dst = k == 2 ? UnmapConv<C2, K3, C3>{pl.w3, pl.b3}(i)
                                : (k == 1 ? UnmapConv<C1, K2, C2>{pl.w2, pl.b2}(i) : UnmapConv1{pl.w1, pl.b1}(i));
        float t = red[o];
        for (int j = 1; j < g.ng; ++j) t += red[j * opb + o];
        dW[dst] = i < g.wcount ? t * g.wscale : t;
    }
}

struct UnmapHeadBias {   // index = head row -> its bias entry in the flat gradient (or -1)
    MapHeadRow h;
    __device__ long operator()(long i) const { return h.brow((int)i); }
};
struct UnmapHead {       // the weight-gradient GEMM's partial block; its bias sums (of bf16 values) are not used
    MapHeadRow h;
    int NHP;
    __device__ long operator()(long i) const {
        if (i >= (long)NHP * HID) return -1;
        const long b = h.wrow((int)(i / HID));
        return b < 0 ? -1 : b + i % HID;
    }
};

// h = relu(sum_z partial[z] + bias), written as bf16 hi (and lo = residual) -- the
// second half of the split-k fc layer.  One thread per four outputs.
__global__ void fc_finish_kernel(const float *__restrict__ partial, int ksplit, const float *__restrict__ bias,
                                 __bf16 *__restrict__ out, __bf16 *__restrict__ out_lo, long total) {
    const long i = ((long)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= total) return;
    float4 s = *reinterpret_cast<const float4 *>(partial + i);
    for (int z = 1; z < ksplit; ++z) {
        const float4 v = *reinterpret_cast<const float4 *>(partial + (size_t)z * total + i);
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    const float4 b = *reinterpret_cast<const float4 *>(bias + (i & (HID - 1)));
    const float r0 = fmaxf(s.x + b.x, 0.f), r1 = fmaxf(s.y + b.y, 0.f), r2 = fmaxf(s.z + b.z, 0.f),
                r3 = fmaxf(s.w + b.w, 0.f);
    typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
    const bf16x4_t h = {(__bf16)r0, (__bf16)r1, (__bf16)r2, (__bf16)r3};
    *reinterpret_cast<u32x2 *>(out + i) = __builtin_bit_cast(u32x2, h);
    if (out_lo) {
        const bf16x4_t l = {(__bf16)(r0 - (float)h[0]), (__bf16)(r1 - (float)h[1]), (__bf16)(r2 - (float)h[2]),
                            (__bf16)(r3 - (float)h[3])};
        *reinterpret_cast<u32x2 *>(out_lo + i) = __builtin_bit_cast(u32x2, l);
    }
}

// loss[0..3] = {total, policy|cross-entropy, value mse, entropy}: one wavefront;
// lane l adds the partials of blocks l, l+64, ... in that order, then the lanes
// are added in a fixed tree -- the same association on every run.
__global__ __launch_bounds__(64) void loss_finalize_kernel(const float *__restrict__ lossp, int blocks, int B,
                                                           float value_coef, float entropy_coef,
                                                           float *__restrict__ loss) {
    if (blockIdx.x != 0) return;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f;
    for (int b = threadIdx.x; b < blocks; b += 64) {
        s0 += lossp[b * 4 + 0];
        s1 += lossp[b * 4 + 1];
        s2 += lossp[b * 4 + 2];
    }
    s0 = wave_sum(s0); s1 = wave_sum(s1); s2 = wave_sum(s2);
    if (threadIdx.x != 0) return;
    const float inv = 1.f / (float)B;
    s0 *= inv; s1 *= inv; s2 *= inv;
    loss[0] = s0 + value_coef * s1 - entropy_coef * s2;
    loss[1] = s0;
    loss[2] = s1;
    loss[3] = s2;
}

// epsilon-greedy on top of a greedy action: u < epsilon takes the uniformly random action floor(u2 * A)
__global__ void epsilon_greedy_kernel(int32_t *__restrict__ action, const float *__restrict__ u,
                                      const float *__restrict__ u2, float epsilon, int A, int B) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= B) return;
    if (u[n] < epsilon) {
        const int r = (int)((double)u2[n] * (double)A);   // exact product of an fp32 and a small integer
        action[n] = r < A - 1 ? r : A - 1;
    }
}

// ------------------------- Categorical DQN target ---------------------------
constexpr int C51_MAX_A = 18;     // most actions the categorical head supports
constexpr int C51_MAX_ATOMS = 64;
constexpr int C51_LANES = 3;      // lanes that share one action's row (3 * 18 <= 64)
constexpr int C51_PER = (C51_MAX_ATOMS + C51_LANES - 1) / C51_LANES;   // most atoms one lane holds
// One wavefront per sample.  From atom logits [A][atoms] of one network (rows of `zstride` floats): per-action
// softmax, expected values Q, lowest-index argmax.  With `m_out`, also the projection of the greedy action's
// distribution onto the support after the shift T_j = clip(r + gamma (1-done) z_j):
//     m_i = sum_j p_j max(0, 1 - |T_j - z_i| / delta).
// The sample's logits go through LDS (coalesced reads); then three neighbouring lanes share one action, each
// holding a third of its atoms in registers, so that the softmax of all actions is one serial pass over at most
// C51_PER values per lane and three cross-lane exchanges, instead of three wavefront reductions per action.
// The partial sums of the three lanes are added in lane order: the same association on every run.  The
// projection runs with lane i = atom i over (p_j, b_j = (T_j - v_min) / delta) pairs broadcast from LDS.
__global__ __launch_bounds__(64 * C51_WAVES) void c51_dist_kernel(
    const float *__restrict__ zin, int zstride, int B, int A, int atoms, float v_min, float v_max, float gamma,
    const float *__restrict__ reward, const uint8_t *__restrict__ done, float *__restrict__ probs,
    float *__restrict__ q_out, int32_t *__restrict__ greedy, float *__restrict__ m_out) {
    __shared__ float s_x[C51_WAVES][C51_MAX_A * C51_MAX_ATOMS];
    __shared__ float2 s_pb[C51_WAVES][C51_MAX_ATOMS];
    const int lane = threadIdx.x & 63, wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = blockIdx.x * C51_WAVES + wv;
    if (n >= B) return;                       // whole wavefronts leave; the kernel has no block-wide barrier
    float *sx = s_x[wv];
    const int ZW = A * atoms;
    const float delta = (v_max - v_min) / (float)(atoms - 1), inv_delta = 1.f / delta;
    // every row of the sample is fetched before the first is used: one memory latency per sample
    {
        float v[C51_MAX_A];
        const float *src = zin + (size_t)n * zstride;
#pragma unroll
        for (int t = 0; t < C51_MAX_A; ++t) {
            const int c = t * 64 + lane;
            v[t] = c < ZW ? src[c] : 0.f;
        }
#pragma unroll
        for (int t = 0; t < C51_MAX_A; ++t) sx[t * 64 + lane] = v[t];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();

    const int a = lane / C51_LANES, part = lane - a * C51_LANES;
    const int per = (atoms + C51_LANES - 1) / C51_LANES;          // wavefront-uniform
    const int j0 = part * per;
    const bool live = a < A;
    const int cnt = live ? max(0, min(per, atoms - j0)) : 0;
    const int at = (live ? a : 0) * atoms + j0;
    float x[C51_PER];
    float mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < C51_PER; ++k) {
        if (k < per) {
            x[k] = k < cnt ? sx[at + k] : -INFINITY;
            mx = fmaxf(mx, x[k]);
        }
    }
    const int base = lane - part;
    mx = fmaxf(fmaxf(__shfl(mx, base, 64), __shfl(mx, base + 1, 64)), __shfl(mx, base + 2, 64));
    float s = 0.f, w = 0.f;
#pragma unroll
    for (int k = 0; k < C51_PER; ++k) {
        if (k < per) {
            const float e = k < cnt ? expf(x[k] - mx) : 0.f;
            x[k] = e;
            s += e;
            w += e * (v_min + delta * (float)(j0 + k));
        }
    }
    s = (__shfl(s, base, 64) + __shfl(s, base + 1, 64)) + __shfl(s, base + 2, 64);
    w = (__shfl(w, base, 64) + __shfl(w, base + 1, 64)) + __shfl(w, base + 2, 64);
    const float inv_s = 1.f / s;
    const float q = live ? w * inv_s : -INFINITY;
    // lowest-index argmax over the actions (a NaN anywhere gives action 0)
    const float qmax = wave_max(q);
    int best_a = (int)-wave_max((live && q == qmax) ? -(float)a : -64.f);
    if (best_a >= A) best_a = 0;
    if (q_out && live && part == 0) q_out[(size_t)n * A + a] = q;
    if (greedy && lane == 0) greedy[n] = best_a;
    if (probs) {
#pragma unroll
        for (int k = 0; k < C51_PER; ++k)
            if (k < per && k < cnt) sx[at + k] = x[k] * inv_s;      // in place of this lane's own logits
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        float *dst = probs + (size_t)n * ZW;
#pragma unroll
        for (int t = 0; t < C51_MAX_A; ++t) {
            const int c = t * 64 + lane;
            if (c < ZW) dst[c] = sx[c];
        }
    }
    if (m_out) {
        float2 *pb = s_pb[wv];
        if (live && a == best_a) {
#pragma unroll
            for (int k = 0; k < C51_PER; ++k)
                if (k < per && k < cnt) pb[j0 + k].x = x[k] * inv_s;
        }
        if (lane < atoms) {
            const float shrink = done[n] ? 0.f : gamma;
            const float T = fminf(fmaxf(reward[n] + shrink * (v_min + delta * (float)lane), v_min), v_max);
            pb[lane].y = (T - v_min) * inv_delta;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const float fi = (float)lane;
        float m = 0.f;
#pragma unroll 4
        for (int j = 0; j < atoms; ++j) {
            const float2 v = pb[j];
            m += v.x * fmaxf(0.f, 1.f - fabsf(v.y - fi));
        }
        if (lane < atoms) m_out[(size_t)n * atoms + lane] = m;
    }
}

// Categorical cross-entropy against the projected target and its gradient:
// L_n = -sum_i m_i log p_i(s_n, a_n);  d/dlogit[a_n][i] = (p_i sum(m) - m_i)/B, other rows 0.
// A wavefront takes `spw` consecutive samples one after the other and writes each one's whole bf16 gradient
// row [NHP].  The head's bias gradient (the sum of those rows over the batch) is accumulated from the fp32
// values -- per wavefront in LDS, in sample order, then over the block's wavefronts in order -- and written as
// one partial per block; a sum of the bf16-rounded rows would be off by about 2^-9 of its largest terms, which
// is most of the result when they cancel.
constexpr int C51_MAX_NHP = 18 * 64;
__global__ __launch_bounds__(64 * C51_WAVES) void c51_loss_kernel(
    const float *__restrict__ z, int zstride, const float *__restrict__ m_in, const int32_t *__restrict__ action,
    int B, int A, int atoms, int NHP, int spw, __bf16 *__restrict__ dz, float *__restrict__ lossp,
    float *__restrict__ hbp) {
    __shared__ float red[C51_WAVES];
    __shared__ float sb[C51_WAVES][C51_MAX_NHP];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    for (int c = lane; c < NHP; c += 64) sb[wv][c] = 0.f;
    float ce = 0.f;
    const bool on = lane < atoms;
    const int n0 = (blockIdx.x * C51_WAVES + wv) * spw;           // wavefront-uniform
    // the operands of sample i + 1 are fetched while sample i is worked on
    int a_next = 0;
    float x_next = -INFINITY, m_next = 0.f;
    auto fetch = [&](int n) __attribute__((always_inline)) {
        if (n < B) {
            a_next = min(max(action[n], 0), A - 1);   // an out-of-range action must not become an out-of-range read
            x_next = on ? z[(size_t)n * zstride + a_next * atoms + lane] : -INFINITY;
            m_next = on ? m_in[(size_t)n * atoms + lane] : 0.f;
        }
    };
    fetch(n0);
    for (int i = 0; i < spw; ++i) {
        const int n = n0 + i;
        if (n >= B) break;
        const int a = a_next;
        const float x = x_next, m = m_next;
        if (i + 1 < spw) fetch(n + 1);
        const float mx = wave_max(x);
        const float e = on ? expf(x - mx) : 0.f;
        const float s = wave_sum(e);
        const float lp = x - mx - logf(s);
        ce += -wave_sum(on ? m * lp : 0.f);
        const float msum = wave_sum(m);
        const float g = on ? (e / s * msum - m) / (float)B : 0.f;
        const int lo = a * atoms;
        if (on) sb[wv][lo + lane] += g;                 // this wavefront's own row of LDS: no other writer
        __bf16 *row = dz + (size_t)n * NHP;
        for (int c0 = 0; c0 < NHP; c0 += 64) {
            const int c = c0 + lane, src = c - lo;
            const float gv = __shfl(g, src & 63, 64);
            row[c] = (__bf16)((src >= 0 && src < atoms) ? gv : 0.f);
        }
    }
    if (lane == 0) red[wv] = ce;
    __syncthreads();
    for (int c = threadIdx.x; c < NHP; c += 64 * C51_WAVES) {
        float t = sb[0][c];
#pragma unroll
        for (int w = 1; w < C51_WAVES; ++w) t += sb[w][c];
        hbp[(size_t)blockIdx.x * NHP + c] = t;
    }
    if (threadIdx.x == 0) {
        float s = 0.f;
        for (int i = 0; i < C51_WAVES; ++i) s += red[i];
        lossp[blockIdx.x * 4 + 0] = s;
        lossp[blockIdx.x * 4 + 1] = 0.f;
        lossp[blockIdx.x * 4 + 2] = 0.f;
    }
}

}  // namespace arn
