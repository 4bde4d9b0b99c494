// The three convolution layers of a forward pass that carries no gradient (action selection, section
// "Synchronized Sampling"), in one kernel and in one fp16 product per layer.
//
// Without a backward pass nothing but the last layer's output has to leave the chip, and the ReLU masks need
// not be exact, so fp16 operands (11 significant bits, fp32 accumulation) meet the output tolerance in a single
// MFMA product per k-step.  One workgroup of eight wavefronts takes a range of samples, one sample at a time:
//   frame (uint8, converted once to an fp16 image in LDS)
//     -> conv1: fragments read straight from that image; epilogue writes act1 into conv2's LDS image
//     -> conv2: fragments from that image; epilogue writes act2 into conv3's LDS image
//     -> conv3: epilogue writes act3 (fp16, NHWC = the fc layer's input order) to global memory.
// All eight wavefronts work on each layer (a wavefront owns one 16-channel tile and every second, or fourth,
// position tile), with two workgroup barriers per sample.  A wavefront keeps its share of conv2's and conv3's
// weights in registers for the whole kernel; conv1's (8 fragments) are fetched again for every sample, while
// conv3 of the sample before runs, because all three layers' weights do not fit the register file at once.
// The LDS images are the ones of the sample-resident training kernels (same padding rule, hence conflict-free
// 16-byte fragment reads), in a single fp16 part.  infer_conv_kernel is this scheme as it stands, for any geometry;
// infer_conv_pipelined_kernel (below) is its software-pipelined form for geometries that leave it 17 KB of LDS.
#pragma once
#include "arn_resident_conv.h"

namespace arn {

constexpr int INF_THREADS = 512;
constexpr float F16_MAX = 65504.f;

// eight uint8 (two little-endian words) -> eight fp16, exact
__device__ __forceinline__ u32x4 u8x8_to_f16x8(uint32_t lo, uint32_t hi) {
    auto two = [](uint32_t b0, uint32_t b1) -> uint32_t {
        const f16x2 h = {(_Float16)(float)b0, (_Float16)(float)b1};
        return __builtin_bit_cast(uint32_t, h);
    };
    u32x4 r;
    r.x = two(lo & 0xff, (lo >> 8) & 0xff);
    r.y = two((lo >> 16) & 0xff, lo >> 24);
    r.z = two(hi & 0xff, (hi >> 8) & 0xff);
    r.w = two((hi >> 16) & 0xff, hi >> 24);
    return r;
}

// relu(v) as four fp16 (finite: clamped to the largest half)
__device__ __forceinline__ u32x2 relu_f16x4(float a, float b, float c, float d) {
    const f16x4 h = {(_Float16)fminf(fmaxf(a, 0.f), F16_MAX), (_Float16)fminf(fmaxf(b, 0.f), F16_MAX),
                     (_Float16)fminf(fmaxf(c, 0.f), F16_MAX), (_Float16)fminf(fmaxf(d, 0.f), F16_MAX)};
    return __builtin_bit_cast(u32x2, h);
}

struct InferConvArgs {
    const uint8_t *obs;                 // [B][4][IN_H][IN_W]
    const _Float16 *w1, *w2, *w3;       // forward weights [co][k'] in fragment order (frag_index)
    const float *b1, *b2, *b3;
    _Float16 *a3;                       // [B][P3][64]
};

// P2 / P3: LDS image descriptions of conv2's and conv3's input (ResConv2Fwd / ResConv3Fwd or their bordered
// variants); only the addressing members are used, for one sample and a single part.
template <class Geo, class P2, class P3>
constexpr int infer_conv_lds_bytes() { return 2 * Geo::OBS_BYTES + P2::IMG + P3::IMG; }

template <class Geo, class P2, class P3>
__global__ __launch_bounds__(INF_THREADS) void infer_conv_kernel(const InferConvArgs a, int B, int spw) {
    constexpr int IN_H = Geo::IN_H, IN_W = Geo::IN_W, W1 = Geo::W1, NP1 = Geo::P1, NP2 = Geo::P2, NP3 = Geo::P3;
    constexpr int OBS_BYTES = Geo::OBS_BYTES, IMG_U4 = OBS_BYTES / 16, NL = (IMG_U4 + INF_THREADS - 1) / INF_THREADS;
    constexpr int KS1 = KW1 / 32, KS2 = KW2 / 32, KS3 = KW3 / 32;     // 8, 16, 18 k-steps
    constexpr int NT1 = (NP1 + 15) / 16, NT2 = (NP2 + 15) / 16, NT3 = (NP3 + 15) / 16;
    constexpr int Q2 = 4, Q3 = 6;                                      // k-steps per fragment batch (two batches in flight)
    static_assert(KS2 % Q2 == 0 && (KS2 / Q2) % 2 == 0 && KS3 % Q3 == 0, "fragment batches");
    static_assert(P2::CI == C1 && P3::CI == C2 && P2::PSB == C1 * 2 + 32 && P3::PSB == C2 * 2 + 32, "image descriptions");
    static_assert(layout_is_uniform<P2>() && layout_is_uniform<P3>(), "fragment rows must advance by one pixel stride modulo 256 bytes");
    static_assert(OBS_BYTES % 16 == 0 && P2::IMG % 16 == 0 && P3::IMG % 16 == 0 && infer_conv_lds_bytes<Geo, P2, P3>() <= 160 * 1024, "LDS budget");

    __shared__ u32x4 lds[infer_conv_lds_bytes<Geo, P2, P3>() / 16];
    u32x4 *const s_img = lds;                                          // fp16 [4][IN_H][IN_W]
    char *const img = reinterpret_cast<char *>(lds);
    char *const a1l = img + 2 * OBS_BYTES;                             // conv2's input image
    char *const a2l = a1l + P2::IMG;                                   // conv3's input image

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, lg = lane >> 4;
    const int s_begin = blockIdx.x * spw;
    const int s_end = s_begin + spw < B ? s_begin + spw : B;
    if (s_begin >= s_end) return;

    // frame of the next sample, in registers until the image buffer is free
    u32x4 rimg[NL];
    auto gload = [&](int s) __attribute__((always_inline)) {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(a.obs + (size_t)s * OBS_BYTES);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int idx = tid + INF_THREADS * i;
            rimg[i] = src[idx < IMG_U4 ? idx : IMG_U4 - 1];
        }
    };
    auto stage = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int idx = tid + INF_THREADS * i;
            if (idx < IMG_U4) {
                s_img[2 * idx] = u8x8_to_f16x8(rimg[i].x, rimg[i].y);
                s_img[2 * idx + 1] = u8x8_to_f16x8(rimg[i].z, rimg[i].w);
            }
        }
    };
    gload(s_begin);

    // conv1: wavefront w owns channel tile w & 1 and position tiles (w >> 1) + 4 j
    const int ct1 = wave & 1, t1_first = wave >> 1;
    // conv2 / conv3: wavefront w owns channel tile w & 3 and position tiles (w >> 2) + 2 j
    const int ct = wave & 3, t_first = wave >> 2;
    f16x8 w1[KS1];
    auto load_w1 = [&]() __attribute__((always_inline)) {
        const size_t r1 = frag_base(ct1, KW1, lane);
#pragma unroll
        for (int ks = 0; ks < KS1; ++ks) w1[ks] = as_f16x8(*reinterpret_cast<const u32x4 *>(a.w1 + r1 + FRAG_STEP * ks));
    };
    load_w1();
    f16x8 w2[KS2], w3[KS3];
    {
        const size_t r2 = frag_base(ct, KW2, lane), r3 = frag_base(ct, KW3, lane);
#pragma unroll
        for (int ks = 0; ks < KS2; ++ks) w2[ks] = as_f16x8(*reinterpret_cast<const u32x4 *>(a.w2 + r2 + FRAG_STEP * ks));
#pragma unroll
        for (int ks = 0; ks < KS3; ++ks) w3[ks] = as_f16x8(*reinterpret_cast<const u32x4 *>(a.w3 + r3 + FRAG_STEP * ks));
    }
    const float4 bias1 = *reinterpret_cast<const float4 *>(a.b1 + ct1 * 16 + 4 * lg);
    const float4 bias2 = *reinterpret_cast<const float4 *>(a.b2 + ct * 16 + 4 * lg);
    const float4 bias3 = *reinterpret_cast<const float4 *>(a.b3 + ct * 16 + 4 * lg);
    if constexpr (P2::ZERO_FILL || P3::ZERO_FILL) {   // zero borders of the padded layers, written once
        for (int i = tid; i < (P2::IMG + P3::IMG) / 16; i += INF_THREADS) lds[2 * IMG_U4 + i] = zero_u4();
    }
    stage();                      // needs the frame only: the weight loads were issued after it
    __syncthreads();
    if (s_begin + 1 < s_end) gload(s_begin + 1);

    // One sample.  FIRST: conv1 starts as soon as its own weights have arrived (the loads return in issue order);
    // the other layers' weights are waited for once, after it, so that no wait for them is left inside the loop
    // (there it could not be told from a wait for the prefetched frame).
    auto sample = [&](int s, auto first) __attribute__((always_inline)) {
        // ---- conv1: frame image -> act1 image ----
#pragma unroll 1
        for (int t = t1_first; t < NT1; t += 4) {
            int pos = t * 16 + li;
            const bool valid = pos < NP1;
            pos = valid ? pos : NP1 - 1;
            const int oy = pos / W1, ox = pos - oy * W1;
            const int base = ((S1 * oy + lg) * IN_W + S1 * ox) * 2;
            u32x2 f[2 * KS1];
#pragma unroll
            for (int ks = 0; ks < KS1; ++ks) {
                const int off = base + ((ks >> 1) * (IN_H * IN_W) + (ks & 1) * 4 * IN_W) * 2;
                f[2 * ks] = *reinterpret_cast<const u32x2 *>(img + off);
                f[2 * ks + 1] = *reinterpret_cast<const u32x2 *>(img + off + 8);
            }
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS1; ++ks) {
                const f16x8 b = as_f16x8(u32x4{f[2 * ks].x, f[2 * ks].y, f[2 * ks + 1].x, f[2 * ks + 1].y});
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(w1[ks], b, acc, 0, 0, 0);
            }
            constexpr float sc = 1.0f / 255.0f;
            if (valid)
                *reinterpret_cast<u32x2 *>(a1l + P2::dst_off(pos) + (ct1 * 16 + 4 * lg) * 2) =
                    relu_f16x4(acc[0] * sc + bias1.x, acc[1] * sc + bias1.y, acc[2] * sc + bias1.z, acc[3] * sc + bias1.w);
        }
        if constexpr (decltype(first)::value) wait_global_loads();
        __syncthreads();          // act1 complete; every read of the frame image done
        if (s + 1 < s_end) stage();   // the next frame, prefetched earlier

        // ---- conv2: act1 image -> act2 image ----
#pragma unroll 1
        for (int t = t_first; t < NT2; t += 2) {
            int row = t * 16 + li;
            const bool valid = row < NP2;
            row = valid ? row : NP2 - 1;
            const int base = P2::base_off(row) + 16 * lg;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            f16x8 fa[Q2], fb[Q2];
            auto load_q = [&](int q, f16x8 (&f)[Q2]) __attribute__((always_inline)) {
#pragma unroll
                for (int j = 0; j < Q2; ++j) {
                    const int ks = q * Q2 + j;
                    const int tap = (32 * ks) / C1, ci0 = (32 * ks) % C1;
                    f[j] = as_f16x8(*reinterpret_cast<const u32x4 *>(a1l + base + P2::tap_off(tap) + ci0 * 2));
                }
            };
            load_q(0, fa);
#pragma unroll
            for (int q = 0; q < KS2 / Q2; q += 2) {
                load_q(q + 1, fb);
#pragma unroll
                for (int j = 0; j < Q2; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(w2[q * Q2 + j], fa[j], acc, 0, 0, 0);
                if (q + 2 < KS2 / Q2) load_q(q + 2, fa);
#pragma unroll
                for (int j = 0; j < Q2; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(w2[(q + 1) * Q2 + j], fb[j], acc, 0, 0, 0);
            }
            if (valid)
                *reinterpret_cast<u32x2 *>(a2l + P3::dst_off(row) + (ct * 16 + 4 * lg) * 2) =
                    relu_f16x4(acc[0] + bias2.x, acc[1] + bias2.y, acc[2] + bias2.z, acc[3] + bias2.w);
        }
        __syncthreads();          // act2 complete; every read of the act1 image done; the next frame image staged
        if (s + 1 < s_end) load_w1();   // conv1's weights for the next sample arrive while conv3 runs
        if (s + 2 < s_end) gload(s + 2);   // the frame after the next: not in registers while conv2 runs

        // ---- conv3: act2 image -> act3 in global memory ----
#pragma unroll 1
        for (int t = t_first; t < NT3; t += 2) {
            int row = t * 16 + li;
            const bool valid = row < NP3;
            row = valid ? row : NP3 - 1;
            const int base = P3::base_off(row) + 16 * lg;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            f16x8 fa[Q3], fb[Q3];
            auto load_q = [&](int q, f16x8 (&f)[Q3]) __attribute__((always_inline)) {
#pragma unroll
                for (int j = 0; j < Q3; ++j) {
                    const int ks = q * Q3 + j;
                    const int tap = (32 * ks) / C2, ci0 = (32 * ks) % C2;
                    f[j] = as_f16x8(*reinterpret_cast<const u32x4 *>(a2l + base + P3::tap_off(tap) + ci0 * 2));
                }
            };
            load_q(0, fa);
            load_q(1, fb);
#pragma unroll
            for (int j = 0; j < Q3; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(w3[j], fa[j], acc, 0, 0, 0);
            load_q(2, fa);
#pragma unroll
            for (int j = 0; j < Q3; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(w3[Q3 + j], fb[j], acc, 0, 0, 0);
#pragma unroll
            for (int j = 0; j < Q3; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(w3[2 * Q3 + j], fa[j], acc, 0, 0, 0);
            if (valid)
                *reinterpret_cast<u32x2 *>(a.a3 + ((size_t)s * NP3 + row) * C3 + ct * 16 + 4 * lg) =
                    relu_f16x4(acc[0] + bias3.x, acc[1] + bias3.y, acc[2] + bias3.z, acc[3] + bias3.w);
        }
        // no barrier here: conv1 of the next sample writes the act1 image (its readers passed the barrier above)
        // and reads the frame image staged before that barrier; conv2 of the next sample, which overwrites the
        // act2 image, starts only after the barrier that follows conv1
    };
    sample(s_begin, std::true_type());
    for (int s = s_begin + 1; s < s_end; ++s) sample(s, std::false_type());
}

// ---------------------------------------------------------------------------
// The same forward where 17 KB of LDS are left beside the three images (the 84x84 network), with the tile loops as
// software pipelines.  In infer_conv_kernel above the register file is full (conv2's and conv3's weights 136, conv1's 32,
// the prefetched frame 16, biases 12), and what the compiler makes of its two-batch loops is a chain of
// read -> wait -> MFMA on a single set of fragment registers.  Here
//   * conv1's weights live in LDS (copied once) and are read back into registers at the start of every sample's
//     conv1, the biases are read from LDS in the epilogues, and the frame after the next is fetched only when conv3
//     starts: conv2 has 64 registers for fragments, conv3 48, conv1 32;
//   * every tile loop is a rolling pipeline over two sets of fragment registers: the reads of the next batch of
//     k-steps -- of the next position tile, at the end of a tile -- are issued before the MFMAs on the batch just
//     read (scheduling barriers keep that order), so an MFMA never waits for a read issued right before it.
// Wavefronts wait at s_waitcnt for 34 % of their cycles instead of 53 %, the kernel takes 166 instead of 177 us at
// 8192 samples and is then bound by the LDS itself (71 % busy: every 16-byte fragment read feeds one MFMA).
// Same results bit for bit (same products in the same order).
constexpr int INF_W1_BYTES = C1 * KW1 * 2;           // conv1's fp16 weights in fragment order
constexpr int INF_BIAS_BYTES = (C1 + C2 + C3) * 4;   // the three layers' biases
template <class Geo, class P2, class P3>
constexpr int infer_pipelined_lds_bytes() { return 2 * Geo::OBS_BYTES + P2::IMG + P3::IMG + INF_BIAS_BYTES + INF_W1_BYTES; }
template <class Geo, class P2, class P3>
constexpr bool infer_pipelined_fits() { return infer_pipelined_lds_bytes<Geo, P2, P3>() <= 160 * 1024; }

template <class Geo, class P2, class P3>
__global__ __launch_bounds__(INF_THREADS) void infer_conv_pipelined_kernel(const InferConvArgs a, int B, int spw) {
    constexpr int IN_H = Geo::IN_H, IN_W = Geo::IN_W, W1 = Geo::W1, NP1 = Geo::P1, NP2 = Geo::P2, NP3 = Geo::P3;
    constexpr int OBS_BYTES = Geo::OBS_BYTES, IMG_U4 = OBS_BYTES / 16, NL = (IMG_U4 + INF_THREADS - 1) / INF_THREADS;
    constexpr int IMG1 = 2 * OBS_BYTES;
    constexpr int KS1 = KW1 / 32, KS2 = KW2 / 32, KS3 = KW3 / 32;     // 8, 16, 18 k-steps
    constexpr int NT1 = (NP1 + 15) / 16, NT2 = (NP2 + 15) / 16, NT3 = (NP3 + 15) / 16;
    constexpr int Q1 = KS1 / 2, Q2 = KS2 / 2, Q3 = KS3 / 3;           // k-steps per fragment batch: 4, 8, 6
    constexpr int NB2 = KS2 / Q2;                                      // batches per tile in conv2 (even)
    static_assert(KS1 % 2 == 0 && KS2 % Q2 == 0 && NB2 % 2 == 0 && KS3 % 3 == 0, "fragment batches");
    static_assert(P2::CI == C1 && P3::CI == C2 && P2::PSB == C1 * 2 + 32 && P3::PSB == C2 * 2 + 32, "image descriptions");
    static_assert(layout_is_uniform<P2>() && layout_is_uniform<P3>(), "fragment rows must advance by one pixel stride modulo 256 bytes");
    static_assert(IMG1 % 16 == 0 && P2::IMG % 16 == 0 && P3::IMG % 16 == 0 && infer_pipelined_lds_bytes<Geo, P2, P3>() <= 160 * 1024, "LDS budget");
    static_assert(INF_W1_BYTES / 16 == 2 * INF_THREADS, "conv1's weights are copied in two 16-byte words per thread");

    __shared__ u32x4 lds[infer_pipelined_lds_bytes<Geo, P2, P3>() / 16];
    u32x4 *const s_img = lds;                                          // fp16 [4][IN_H][IN_W]
    char *const img = reinterpret_cast<char *>(lds);
    char *const a1l = img + IMG1;                                      // conv2's input image
    char *const a2l = a1l + P2::IMG;                                   // conv3's input image
    float *const s_bias = reinterpret_cast<float *>(a2l + P3::IMG);    // b1, b2, b3
    u32x4 *const s_w1 = reinterpret_cast<u32x4 *>(a2l + P3::IMG + INF_BIAS_BYTES);   // conv1's weights [ct][ks][lane]

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, lg = lane >> 4;
    const int s_begin = blockIdx.x * spw;
    const int s_end = s_begin + spw < B ? s_begin + spw : B;
    if (s_begin >= s_end) return;

    // frame of a later sample, in registers until the image buffer is free
    // frame of a later sample, in registers until the image buffer is free
    u32x4 rimg[NL];
    auto gload = [&](int s) __attribute__((always_inline)) {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(a.obs + (size_t)s * OBS_BYTES);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int idx = tid + INF_THREADS * i;
            rimg[i] = src[idx < IMG_U4 ? idx : IMG_U4 - 1];
        }
    };
    auto stage = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int idx = tid + INF_THREADS * i;
            if (idx < IMG_U4) {
                s_img[2 * idx] = u8x8_to_f16x8(rimg[i].x, rimg[i].y);
                s_img[2 * idx + 1] = u8x8_to_f16x8(rimg[i].z, rimg[i].w);
            }
        }
    };
    gload(s_begin);
    // conv1: wavefront w owns channel tile w & 1 and position tiles (w >> 1) + 4 j
    const int ct1 = wave & 1, t1_first = wave >> 1;
    // conv1's weights go to LDS once
    const u32x4 w1a = reinterpret_cast<const u32x4 *>(a.w1)[tid], w1b = reinterpret_cast<const u32x4 *>(a.w1)[tid + INF_THREADS];
    // conv2 / conv3: wavefront w owns channel tile w & 3 and position tiles (w >> 2) + 2 j
    const int ct = wave & 3, t_first = wave >> 2;
    f16x8 w2[KS2], w3[KS3];
    {
        const size_t r2 = frag_base(ct, KW2, lane), r3 = frag_base(ct, KW3, lane);
#pragma unroll
        for (int ks = 0; ks < KS2; ++ks) w2[ks] = as_f16x8(*reinterpret_cast<const u32x4 *>(a.w2 + r2 + FRAG_STEP * ks));
#pragma unroll
        for (int ks = 0; ks < KS3; ++ks) w3[ks] = as_f16x8(*reinterpret_cast<const u32x4 *>(a.w3 + r3 + FRAG_STEP * ks));
    }
    if (tid < C1 + C2 + C3) s_bias[tid] = tid < C1 ? a.b1[tid] : tid < C1 + C2 ? a.b2[tid - C1] : a.b3[tid - C1 - C2];
    const float4 *const bias1p = reinterpret_cast<const float4 *>(s_bias + ct1 * 16 + 4 * lg);
    const float4 *const bias2p = reinterpret_cast<const float4 *>(s_bias + C1 + ct * 16 + 4 * lg);
    const float4 *const bias3p = reinterpret_cast<const float4 *>(s_bias + C1 + C2 + ct * 16 + 4 * lg);
    if constexpr (P2::ZERO_FILL || P3::ZERO_FILL) {   // zero borders of the padded layers, written once
        for (int i = tid; i < (P2::IMG + P3::IMG) / 16; i += INF_THREADS) lds[IMG1 / 16 + i] = zero_u4();
    }
    s_w1[tid] = w1a;              // needs conv1's weights and (below) the frame only: the other weight loads were issued after them
    s_w1[tid + INF_THREADS] = w1b;
    stage();
    __syncthreads();
    if (s_begin + 1 < s_end) gload(s_begin + 1);

    // One sample.  FIRST: conv1 starts as soon as the frame and its own weights have arrived (loads return in issue order); the
    // other layers' weights are waited for once, after it, so that no wait for them is left inside the loop (there
    // it could not be told from a wait for the prefetched frame).
    auto sample = [&](int s, auto first) __attribute__((always_inline)) {
        // ---- conv1: frame image -> act1 image ----
        {
            f16x8 w1[KS1];
#pragma unroll
            for (int ks = 0; ks < KS1; ++ks) w1[ks] = as_f16x8(s_w1[(ct1 * KS1 + ks) * 64 + lane]);
            auto tile_at = [&](int t, int &pos, bool &valid) __attribute__((always_inline)) -> int {
                pos = t * 16 + li;
                valid = pos < NP1;
                pos = valid ? pos : NP1 - 1;
                const int oy = pos / W1, ox = pos - oy * W1;
                return ((S1 * oy + lg) * IN_W + S1 * ox) * 2;
            };
            auto load_h = [&](int base, int h, u32x2 (&f)[2 * Q1]) __attribute__((always_inline)) {
#pragma unroll
                for (int j = 0; j < Q1; ++j) {
                    const int ks = h * Q1 + j;
                    const int off = base + ((ks >> 1) * (IN_H * IN_W) + (ks & 1) * 4 * IN_W) * 2;
                    f[2 * j] = *reinterpret_cast<const u32x2 *>(img + off);
                    f[2 * j + 1] = *reinterpret_cast<const u32x2 *>(img + off + 8);
                }
            };
            u32x2 fa[2 * Q1], fb[2 * Q1];
            int pos, pos_n;
            bool valid, valid_n;
            int t = t1_first;
            int base = tile_at(t, pos, valid);
            load_h(base, 0, fa);
            load_h(base, 1, fb);
#pragma unroll 1
            for (;;) {
                const int tn = t + 4;
                const bool more = tn < NT1;                 // wavefront-uniform
                const int base_n = tile_at(more ? tn : t, pos_n, valid_n);
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < Q1; ++j)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(w1[j], as_f16x8(u32x4{fa[2 * j].x, fa[2 * j].y, fa[2 * j + 1].x, fa[2 * j + 1].y}), acc, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (more) load_h(base_n, 0, fa);
                const float4 bias1 = *bias1p;
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < Q1; ++j)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(w1[Q1 + j], as_f16x8(u32x4{fb[2 * j].x, fb[2 * j].y, fb[2 * j + 1].x, fb[2 * j + 1].y}), acc, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (more) load_h(base_n, 1, fb);
                __builtin_amdgcn_sched_barrier(0);
                constexpr float sc = 1.0f / 255.0f;
                if (valid)
                    *reinterpret_cast<u32x2 *>(a1l + P2::dst_off(pos) + (ct1 * 16 + 4 * lg) * 2) =
                        relu_f16x4(acc[0] * sc + bias1.x, acc[1] * sc + bias1.y, acc[2] * sc + bias1.z, acc[3] * sc + bias1.w);
                if (!more) break;
                t = tn; pos = pos_n; valid = valid_n;
            }
        }
        if constexpr (decltype(first)::value) wait_global_loads();
        __syncthreads();          // act1 complete; every read of the frame image done
        if (s + 1 < s_end) stage();   // the next frame, prefetched earlier

        // ---- conv2: act1 image -> act2 image ----
        {
            auto tile_at = [&](int t, int &row, bool &valid) __attribute__((always_inline)) -> int {
                row = t * 16 + li;
                valid = row < NP2;
                row = valid ? row : NP2 - 1;
                return P2::base_off(row) + 16 * lg;
            };
            auto load_q = [&](int base, int q, f16x8 (&f)[Q2]) __attribute__((always_inline)) {
#pragma unroll
                for (int j = 0; j < Q2; ++j) {
                    const int ks = q * Q2 + j;
                    const int tap = (32 * ks) / C1, ci0 = (32 * ks) % C1;
                    f[j] = as_f16x8(*reinterpret_cast<const u32x4 *>(a1l + base + P2::tap_off(tap) + ci0 * 2));
                }
            };
            f16x8 fa[Q2], fb[Q2];
            int row, row_n;
            bool valid, valid_n;
            int t = t_first;
            int base = tile_at(t, row, valid);
            load_q(base, 0, fa);
#pragma unroll 1
            for (;;) {
                const int tn = t + 2;
                const bool more = tn < NT2;
                const int base_n = tile_at(more ? tn : t, row_n, valid_n);
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                float4 bias2;
#pragma unroll
                for (int q = 0; q < NB2; q += 2) {
                    __builtin_amdgcn_sched_barrier(0);
                    load_q(base, q + 1, fb);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int j = 0; j < Q2; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(w2[q * Q2 + j], fa[j], acc, 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (q + 2 < NB2) {
                        load_q(base, q + 2, fa);
                    } else {
                        if (more) load_q(base_n, 0, fa);
                        bias2 = *bias2p;
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int j = 0; j < Q2; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(w2[(q + 1) * Q2 + j], fb[j], acc, 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (valid)
                    *reinterpret_cast<u32x2 *>(a2l + P3::dst_off(row) + (ct * 16 + 4 * lg) * 2) =
                        relu_f16x4(acc[0] + bias2.x, acc[1] + bias2.y, acc[2] + bias2.z, acc[3] + bias2.w);
                if (!more) break;
                t = tn; base = base_n; row = row_n; valid = valid_n;
            }
        }
        __syncthreads();          // act2 complete; every read of the act1 image done; the next frame image staged
        if (s + 2 < s_end) gload(s + 2);   // in registers while conv3 and the next sample's conv1 run

        // ---- conv3: act2 image -> act3 in global memory ----
        {
            auto tile_at = [&](int t, int &row, bool &valid) __attribute__((always_inline)) -> int {
                row = t * 16 + li;
                valid = row < NP3;
                row = valid ? row : NP3 - 1;
                return P3::base_off(row) + 16 * lg;
            };
            auto load_q = [&](int base, int q, f16x8 (&f)[Q3]) __attribute__((always_inline)) {
#pragma unroll
                for (int j = 0; j < Q3; ++j) {
                    const int ks = q * Q3 + j;
                    const int tap = (32 * ks) / C2, ci0 = (32 * ks) % C2;
                    f[j] = as_f16x8(*reinterpret_cast<const u32x4 *>(a2l + base + P3::tap_off(tap) + ci0 * 2));
                }
            };
            f16x8 fa[Q3], fb[Q3];
            int t = t_first;
            int row, row_n;
            bool valid, valid_n;
            int base = tile_at(t, row, valid), base_n;
            bool more;
            // one position tile: batch 0 of its fragments is in x, batch 1 in y; afterwards the next tile's batch 0 is in y
            // and its batch 1 in x
            auto tile = [&](f16x8 (&x)[Q3], f16x8 (&y)[Q3]) __attribute__((always_inline)) {
                const int tn = t + 2;
                more = tn < NT3;
                base_n = tile_at(more ? tn : t, row_n, valid_n);
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < Q3; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(w3[j], x[j], acc, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                load_q(base, 2, x);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < Q3; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(w3[Q3 + j], y[j], acc, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (more) load_q(base_n, 0, y);
                const float4 bias3 = *bias3p;
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < Q3; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(w3[2 * Q3 + j], x[j], acc, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (more) load_q(base_n, 1, x);
                __builtin_amdgcn_sched_barrier(0);
                if (valid)
                    *reinterpret_cast<u32x2 *>(a.a3 + ((size_t)s * NP3 + row) * C3 + ct * 16 + 4 * lg) =
                        relu_f16x4(acc[0] + bias3.x, acc[1] + bias3.y, acc[2] + bias3.z, acc[3] + bias3.w);
                t = tn; base = base_n; row = row_n; valid = valid_n;
            };
            load_q(base, 0, fa);
            load_q(base, 1, fb);
#pragma unroll 1
            for (;;) {
                tile(fa, fb);
                if (!more) break;
                tile(fb, fa);
                if (!more) break;
            }
        }
        // no barrier here: conv1 of the next sample writes the act1 image (its readers passed the barrier above)
        // and reads the frame image staged before that barrier; conv2 of the next sample, which overwrites the
        // act2 image, starts only after the barrier that follows conv1
    };
    sample(s_begin, std::true_type());
    for (int s = s_begin + 1; s < s_end; ++s) sample(s, std::false_type());
}

}  // namespace arn
