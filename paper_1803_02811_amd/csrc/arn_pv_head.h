// Everything after the fc layer's GEMM for the policy/value network, in one kernel per 16 samples:
//   1. h = relu(sum_z partial[z] + b_fc)               (finishes the split-k fc layer; hi/lo bf16 pair kept in LDS)
//   2. z = W_head h + b_head                            (three-product bf16 MFMA, 32 head rows x 16 samples x 512)
//   3. inference: logits, value, softmax, lowest-index greedy action                    (section "Synchronized Sampling")
//      training:  A2C / PPO objective terms and their gradient dz at the head outputs   (section "RL Algorithm Background")
//   4. training: d(pre_fc) = (W_head^T dz) * [h > 0]    (single bf16 MFMA, contraction over the 32 head rows)
// The same kernel serves the action-value heads (scalar Q rows, or advantage rows + a value row combined as
// Q = V + A - mean(A)): inference then returns Q, max Q and the greedy action; training evaluates the DQN
// objective mean((y - Q(s,a))^2) with y from the target network's values on the next state (section "RL
// Algorithm Background").  With random numbers as inputs the inference variant also draws the action
// (categorical by inverse CDF, or epsilon-greedy), as the paper's sampler returns actions, not logits.
// The head is tiny (at most 32 rows); as separate launches these steps cost several times their arithmetic in
// launch latency and in trips of h through HBM, and they all sit on the critical path between the forward
// and the backward pass.
//
// MFMA used: v_mfma_f32_16x16x32_bf16.  Operand layout (checked on hardware): A (16 x 32): lane l holds
// row l%16, k = 8*(l/16)..+7;  B (32 x 16): lane l holds column l%16, same k;  D (16 x 16): lane l holds column
// l%16, rows 4*(l/16)+r, r = 0..3.  Weights go in as A and samples as B, so a lane ends up with four consecutive
// output rows of one sample.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "arn_gemm.h"
#include "arn_lanes.h"
#include "arn_layout.h"

namespace arn {

constexpr int PVH_ROWS = 16;          // samples per workgroup
constexpr int PVH_THREADS = 256;
constexpr int PVH_HS = HID + 8;       // LDS row stride of h in bf16 (16-byte aligned rows, staggered banks)
constexpr int PVH_DZS = 40;           // LDS row stride of dz in bf16

struct PvHeadArgs {
    const float *partial;   // fp32 [ks][B][512] partial sums of the fc GEMM
    int ks;
    const float *bfc;       // [512]
    const __bf16 *wh, *whl; // head weights [64][512] hi / lo in fragment order (frag_index); rows A+1.. are zero
    const float *bh;        // [64] head bias (policy rows then the value row)
    int B, A;
    int rpb;                // samples per workgroup (1..16; 0 = 16).  Small batches spread over more
                            // workgroups, because one CU's L1 rate bounds the addition of the fc partial sums
    int qmode;              // 0: policy logits + value row; 1: scalar Q rows; 2: advantage rows + value row -> Q
    // inference outputs (each may be null)
    float *logits, *value, *probs;
    int32_t *greedy;
    // action draw (inference): u, u2 uniform [0,1) per sample; qmode 0: categorical by inverse CDF with u;
    // otherwise epsilon-greedy (u < epsilon: floor(u2 * A)); act_out null = no draw
    const float *u, *u2;
    float epsilon;
    int32_t *act_out;
    float *logp_out;        // qmode 0: log pi(drawn action), or null
    // training inputs
    const int32_t *action;
    const float *adv, *ret, *old_logp;
    int objective;          // 0 a2c, 1 ppo, 2 dqn
    // dqn: target-network values on the next state [B][A]; the action that is bootstrapped from (null: the
    // argmax of q_next itself); reward, done, discount
    const float *q_next;
    const int32_t *a_star;
    const float *reward;
    const uint8_t *done;
    float gamma;
    float clip_eps, value_coef, entropy_coef;
    const __bf16 *whd;      // head weights for the input gradient [512][64] (k = head row), in fragment order
    // training outputs
    __bf16 *h;              // [B][512] fc activations (bf16), read by the head's weight gradient
    __bf16 *dz;             // [B][64]
    __bf16 *dph;            // [B][512] d(pre_fc)
    float *lossp;           // [blocks][4] partial sums {policy, value, entropy}
    float *hbp;             // [blocks][32] this block's sum of dz per head row, from the fp32 values (the bias gradient)
};

__device__ __forceinline__ float group16_sum(float v) { return row16_sum(v); }   // same bits in all 16 lanes of the group
__device__ __forceinline__ float group16_scan(float v, int c) {   // inclusive prefix sum over the 16 lanes of the group
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {
        const float t = __shfl_up(v, o, 16);
        if (c >= o) v += t;
    }
    return v;
}
__device__ __forceinline__ int group16_min(int v) { return row16_min(v); }
__device__ __forceinline__ float group16_max(float v) { return row16_max(v); }

template <bool TRAIN>
__global__ __launch_bounds__(PVH_THREADS) void pv_head_kernel(const PvHeadArgs p) {
    __shared__ __attribute__((aligned(16))) __bf16 sH[PVH_ROWS * PVH_HS];
    __shared__ __attribute__((aligned(16))) __bf16 sL[PVH_ROWS * PVH_HS];
    __shared__ float sZ[4][32][PVH_ROWS];                 // per-wave partial head outputs [wave][row][sample]
    __shared__ __attribute__((aligned(16))) __bf16 sDz[PVH_ROWS * PVH_DZS];
    __shared__ float sRed[3][PVH_ROWS];
    __shared__ float sG[TRAIN ? PVH_ROWS : 1][32];        // fp32 dz, for the bias gradient

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rpb = p.rpb <= 0 ? PVH_ROWS : p.rpb;
    const int n0 = blockIdx.x * rpb;
    const int srow = tid >> 4, c = tid & 15;              // sample within the block, lane within its group of 16
    const int n = n0 + srow;
    const bool live = srow < rpb && n < p.B;

    // weight fragments and per-sample scalars do not depend on step 1: their loads go first
    const int fi = lane & 15, fg = lane >> 4;
    bf16x8 wa[4][2], wl[4][2];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const size_t at = frag_base(t, HID, lane) + FRAG_STEP * (wave * 4 + s);   // fragment order (frag_index)
            wa[s][t] = as_bf16x8(*reinterpret_cast<const u32x4 *>(p.wh + at));
            wl[s][t] = as_bf16x8(*reinterpret_cast<const u32x4 *>(p.whl + at));
        }
    u32x4 wd[TRAIN ? 8 : 1];
    int a = 0;
    float ad = 0.f, rt = 0.f, olp = 0.f;
    if constexpr (TRAIN) {
        if (live) {
            a = min(max(p.action[n], 0), p.A - 1);
            if (p.objective == 2) {
                ad = p.reward[n];                       // dqn: reward
                rt = p.done[n] ? 0.f : p.gamma;          //      discount of the bootstrap term
            } else {
                ad = p.adv[n];
                rt = p.ret[n];
                if (p.objective == 1) olp = p.old_logp[n];
            }
        }
    }
    const float bz0 = p.bh[c], bz1 = p.bh[c + 16];

    // ---- 1. finish the fc layer for 16 samples ----
    {
        const size_t plane = (size_t)p.B * HID;
        const float *src = p.partial + (size_t)(live ? n : 0) * HID + c * 4;
        float4 acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (live) {   // rows past the batch (or past this block's share) load nothing
            // the k ranges are added in order; four ranges (32 loads), then two, then one are in flight at a time
            auto add_planes = [&](int z, auto count) __attribute__((always_inline)) {
                constexpr int Q = decltype(count)::value;
                float4 v[Q][8];
#pragma unroll
                for (int q = 0; q < Q; ++q)
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        v[q][j] = *reinterpret_cast<const float4 *>(src + (size_t)(z + q) * plane + 64 * j);
#pragma unroll
                for (int q = 0; q < Q; ++q)
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        acc[j].x += v[q][j].x; acc[j].y += v[q][j].y; acc[j].z += v[q][j].z; acc[j].w += v[q][j].w;
                    }
            };
            int z = 0;
            for (; z + 4 <= p.ks; z += 4) add_planes(z, std::integral_constant<int, 4>());
            if (z + 2 <= p.ks) { add_planes(z, std::integral_constant<int, 2>()); z += 2; }
            if (z < p.ks) add_planes(z, std::integral_constant<int, 1>());
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int col = c * 4 + 64 * j;
            const float4 b = *reinterpret_cast<const float4 *>(p.bfc + col);
            float r[4] = {fmaxf(acc[j].x + b.x, 0.f), fmaxf(acc[j].y + b.y, 0.f), fmaxf(acc[j].z + b.z, 0.f),
                          fmaxf(acc[j].w + b.w, 0.f)};
            if (!live) r[0] = r[1] = r[2] = r[3] = 0.f;
            const bf16x4 hi = {(__bf16)r[0], (__bf16)r[1], (__bf16)r[2], (__bf16)r[3]};
            const bf16x4 lo = {(__bf16)(r[0] - (float)hi[0]), (__bf16)(r[1] - (float)hi[1]),
                               (__bf16)(r[2] - (float)hi[2]), (__bf16)(r[3] - (float)hi[3])};
            *reinterpret_cast<u32x2 *>(sH + srow * PVH_HS + col) = __builtin_bit_cast(u32x2, hi);
            *reinterpret_cast<u32x2 *>(sL + srow * PVH_HS + col) = __builtin_bit_cast(u32x2, lo);
            if (TRAIN && live) *reinterpret_cast<u32x2 *>(p.h + (size_t)n * HID + col) = __builtin_bit_cast(u32x2, hi);
        }
    }
    __syncthreads();
    // the weights of step 4 are asked for only now: fetched with the others they would compete with the fc partial
    // sums of step 1 for the L2, and steps 2 and 3 are long enough to cover them
    if constexpr (TRAIN) {
#pragma unroll
        for (int t = 0; t < 8; ++t)
            wd[t] = *reinterpret_cast<const u32x4 *>(p.whd + frag_base(wave * 8 + t, 64, lane));   // fragment order
    }

    // ---- 2. head GEMM: wave w takes k = 128 w .. 128 w + 127 for both 16-row tiles ----
    {
        f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int at = fi * PVH_HS + (wave * 4 + s) * 32 + fg * 8;
            const bf16x8 hh = as_bf16x8(*reinterpret_cast<const u32x4 *>(sH + at));
            const bf16x8 hl = as_bf16x8(*reinterpret_cast<const u32x4 *>(sL + at));
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wl[s][t], hh, acc[t], 0, 0, 0);
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[s][t], hl, acc[t], 0, 0, 0);
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[s][t], hh, acc[t], 0, 0, 0);
            }
        }
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) sZ[wave][16 * t + 4 * fg + r][fi] = acc[t][r];
    }
    __syncthreads();

    // lane c of sample srow owns head rows c and c + 16; partial sums are added in wave order
    float z0 = bz0, z1 = bz1;
    {
        float a0 = sZ[0][c][srow], a1 = sZ[0][c + 16][srow];
#pragma unroll
        for (int w = 1; w < 4; ++w) { a0 += sZ[w][c][srow]; a1 += sZ[w][c + 16][srow]; }
        z0 += a0; z1 += a1;
    }
    const int A = p.A;
    const bool on0 = c < A, on1 = c + 16 < A;
    // value = head row A (policy/value and dueling heads)
    const float vsel = A < 16 ? z0 : z1;
    const float v = __shfl(vsel, A & 15, 16);
    if (p.qmode == 2) {   // Q = V + A - mean(A)
        const float mean = group16_sum((on0 ? z0 : 0.f) + (on1 ? z1 : 0.f)) / (float)A;
        z0 = v + z0 - mean;
        z1 = v + z1 - mean;
    }
    const float x0 = on0 ? z0 : -INFINITY, x1 = on1 ? z1 : -INFINITY;
    const float mx = group16_max(fmaxf(x0, x1));
    // lowest index among the maxima: the maximum is known, take the smallest index that attains it
    const int arg = group16_min(x0 == mx ? c : (x1 == mx ? c + 16 : 64));

    if constexpr (!TRAIN) {
        const bool policy = p.qmode == 0;
        float e0 = 0.f, e1 = 0.f, s = 1.f;
        if (policy) {
            e0 = on0 ? expf(x0 - mx) : 0.f;
            e1 = on1 ? expf(x1 - mx) : 0.f;
            s = group16_sum(e0 + e1);
        }
        if (live) {
            if (p.logits) {
                if (on0) p.logits[(size_t)n * A + c] = z0;
                if (on1) p.logits[(size_t)n * A + c + 16] = z1;
            }
            if (p.value && c == 0) p.value[n] = policy ? v : mx;
            if (p.probs && policy) {
                const float inv = 1.f / s;
                if (on0) p.probs[(size_t)n * A + c] = e0 * inv;
                if (on1) p.probs[(size_t)n * A + c + 16] = e1 * inv;
            }
            if (p.greedy && c == 0) p.greedy[n] = arg;
        }
        if (p.act_out) {
            const float uu = live ? p.u[n] : 0.f;
            int act;
            if (policy) {
                // inverse CDF on the unnormalised weights: first k with sum_{j<=k} e_j > u * s
                const float c0 = group16_scan(e0, c);
                const float tot0 = __shfl(c0, 15, 16);
                const float c1 = tot0 + group16_scan(e1, c);
                const float thr = uu * s;
                act = group16_min(on0 && c0 > thr ? c : (on1 && c1 > thr ? c + 16 : 64));
                act = act < A ? act : A - 1;
                if (p.logp_out) {
                    const float lse = mx + logf(s);
                    const float lp = group16_sum((c == act ? x0 - lse : 0.f) + (c + 16 == act ? x1 - lse : 0.f));
                    if (live && c == 0) p.logp_out[n] = lp;
                }
            } else {
                const int rnd = min((int)((double)(live ? p.u2[n] : 0.f) * (double)A), A - 1);   // exact product
                act = uu < p.epsilon ? rnd : arg;
            }
            if (live && c == 0) p.act_out[n] = act;
        }
        return;
    } else {
        // ---- 3. objective terms and the gradient at the head outputs ----
        const float invB = 1.f / (float)p.B;
        float g0, g1, t0 = 0.f, t1 = 0.f, t2 = 0.f;   // dz of the lane's two rows; the sample's three loss terms
        if (p.objective == 2) {
            // DQN: y = r + gamma (1 - done) Q(s', a*; target network); ad = reward, rt = discount
            float qn0 = on0 && live ? p.q_next[(size_t)n * A + c] : -INFINITY;
            float qn1 = on1 && live ? p.q_next[(size_t)n * A + c + 16] : -INFINITY;
            int as;
            if (p.a_star) {
                as = live ? p.a_star[n] : 0;
            } else {
                const float qm = group16_max(fmaxf(qn0, qn1));
                as = group16_min(qn0 == qm ? c : (qn1 == qm ? c + 16 : 64));
            }
            const float boot = group16_sum((c == as && on0 ? qn0 : 0.f) + (c + 16 == as && on1 ? qn1 : 0.f));
            const float y = ad + rt * (live ? boot : 0.f);
            const float qa = group16_sum((c == a && on0 ? z0 : 0.f) + (c + 16 == a && on1 ? z1 : 0.f));
            const float td = qa - y;
            t0 = td * td;
            const float g = 2.f * td * invB;
            if (p.qmode == 2) {   // through Q = V + A - mean(A): dA_k = g (delta_ka - 1/A), dV = g
                const float share = g / (float)A;
                g0 = on0 ? (c == a ? g : 0.f) - share : 0.f;
                g1 = on1 ? (c + 16 == a ? g : 0.f) - share : 0.f;
                if (c == A) g0 = g;
                if (c + 16 == A) g1 = g;
            } else {
                g0 = on0 && c == a ? g : 0.f;
                g1 = on1 && c + 16 == a ? g : 0.f;
            }
        } else {
            const float e0 = on0 ? expf(x0 - mx) : 0.f, e1 = on1 ? expf(x1 - mx) : 0.f;
            const float s = group16_sum(e0 + e1);
            const float lse = mx + logf(s);
            const float lp0 = x0 - lse, lp1 = x1 - lse;                 // log-probabilities (-inf where off)
            const float q0 = on0 ? expf(lp0) : 0.f, q1 = on1 ? expf(lp1) : 0.f;
            const float H = -group16_sum((on0 ? q0 * lp0 : 0.f) + (on1 ? q1 * lp1 : 0.f));
            const float lpa = group16_sum((c == a ? lp0 : 0.f) + (c + 16 == a ? lp1 : 0.f));
            float pol, w;   // w = d(surrogate)/d(log pi(a))
            if (p.objective == 1) {
                const float rho = expf(lpa - olp);
                const float clipped = fminf(fmaxf(rho, 1.f - p.clip_eps), 1.f + p.clip_eps);
                pol = -fminf(rho * ad, clipped * ad);
                const bool active = (ad >= 0.f && rho <= 1.f + p.clip_eps) || (ad < 0.f && rho >= 1.f - p.clip_eps);
                w = active ? ad * rho : 0.f;
            } else {
                pol = -lpa * ad;
                w = ad;
            }
            const float dv = v - rt;
            g0 = on0 ? (-w * ((c == a ? 1.f : 0.f) - q0) + p.entropy_coef * q0 * (lp0 + H)) * invB : 0.f;
            g1 = on1 ? (-w * ((c + 16 == a ? 1.f : 0.f) - q1) + p.entropy_coef * q1 * (lp1 + H)) * invB : 0.f;
            const float gv = p.value_coef * 2.f * dv * invB;
            if (c == A) g0 = gv;
            if (c + 16 == A) g1 = gv;
            t0 = pol; t1 = dv * dv; t2 = H;
        }
        if (!live) g0 = g1 = 0.f;
        sDz[srow * PVH_DZS + c] = (__bf16)g0;
        sDz[srow * PVH_DZS + c + 16] = (__bf16)g1;
        sG[srow][c] = g0;
        sG[srow][c + 16] = g1;
        if (c == 0) {
            sRed[0][srow] = live ? t0 : 0.f;
            sRed[1][srow] = live ? t1 : 0.f;
            sRed[2][srow] = live ? t2 : 0.f;
        }
        __syncthreads();
        if (tid < 3) {   // block partial sums in sample order
            float t = 0.f;
#pragma unroll
            for (int i = 0; i < PVH_ROWS; ++i) t += sRed[tid][i];
            p.lossp[blockIdx.x * 4 + tid] = t;
        }
        // The head's bias gradient is the sum of dz over the batch.  It is taken from the fp32 values, in sample
        // order: a sum of bf16-rounded terms is off by about 2^-9 of its largest terms, which is most of the
        // result when the terms happen to cancel -- and these are tensors of one to a few dozen entries.
        if (tid >= 64 && tid < 96) {
            const int r = tid - 64;
            float t = 0.f;
#pragma unroll
            for (int i = 0; i < PVH_ROWS; ++i) t += sG[i][r];
            p.hbp[blockIdx.x * 32 + r] = t;
        }
        if (tid < PVH_ROWS * 8) {   // dz rows [64] as eight 16-byte words; columns 32.. are zero
            const int r = tid >> 3, q = tid & 7;
            if (r < rpb && n0 + r < p.B) {
                const u32x4 val = q < 4 ? *reinterpret_cast<const u32x4 *>(sDz + r * PVH_DZS + 8 * q) : zero_u4();
                *reinterpret_cast<u32x4 *>(p.dz + (size_t)(n0 + r) * 64 + 8 * q) = val;
            }
        }

        // ---- 4. input gradient of the head: 32 tiles of 16 hidden units, 8 per wave ----
        const bf16x8 dzf = as_bf16x8(*reinterpret_cast<const u32x4 *>(sDz + fi * PVH_DZS + fg * 8));
        const bool row_live = fi < rpb && n0 + fi < p.B;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int j0 = (wave * 8 + t) * 16;
            const bf16x8 wf = as_bf16x8(wd[t]);
            f32x4 d = {0.f, 0.f, 0.f, 0.f};
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, dzf, d, 0, 0, 0);
            const int j = j0 + 4 * fg;
            const f32x4 hv = unpack_bf16x4(*reinterpret_cast<const u32x2 *>(sH + fi * PVH_HS + j));
            if (row_live)
                *reinterpret_cast<u32x2 *>(p.dph + (size_t)(n0 + fi) * HID + j) =
                    pack_bf16x4(hv[0] > 0.f ? d[0] : 0.f, hv[1] > 0.f ? d[1] : 0.f, hv[2] > 0.f ? d[2] : 0.f,
                                hv[3] > 0.f ? d[3] : 0.f);
        }
    }
}

}  // namespace arn
