// conv2 and conv3 forward in one kernel: act2 goes from one layer to the next through LDS.
//
// Both layers keep their weights in registers and read their input from an LDS image (resident_conv_kernel).
// Here the eight wavefronts of a workgroup have two roles, as in conv1_bwd_fused_body: four "producers" hold
// conv2's weights (16 output channels each, hi and lo parts) and compute act2 of sample s+1 from the staged act1
// image; their epilogue (bias, ReLU, hi/lo split) writes the 16 x 16 tile straight into conv3's LDS image, one of
// two buffers.  Four "consumers" hold conv3's weights and compute act3 of sample s from the other buffer.  act2's
// low part never exists in HBM, its high part and sign bits are written only when the backward pass will need
// them, and conv3 has no staging phase.  The two roles sit in two branches that execute the same barriers, so
// registers are allocated for one role only (conv2's 128 + conv3's 144 weight registers would not fit one
// wavefront).  All three products of the split-bf16 forward are kept.
#pragma once
#include "arn_resident_conv.h"

namespace arn {

constexpr int C23_THREADS = 512;   // four consumer wavefronts (0-3), four producers (4-7); one workgroup per CU

struct Conv23Args {
    const __bf16 *a1, *a1_lo;        // act1 [B][P1][32], hi and lo
    const __bf16 *w2, *w2_lo, *w3, *w3_lo;
    const float *b2, *b3;
    __bf16 *a2;                      // act2 hi [B][P2][64] for the backward pass, or null
    __bf16 *a3, *a3_lo;              // act3 [B][P3][64], hi and lo
    uint8_t *m2, *m3;                // sign bits of act2 / act3 for the backward pass, or null
};

// LDS bytes of conv23_fwd_fused_body<P2, P3>: conv2's input image and two of conv3's, hi and lo parts each
template <class P2, class P3>
constexpr int conv23_fwd_lds_bytes() { return 2 * P2::IMG + 4 * P3::IMG; }

// The work of workgroup `block` (of C23_THREADS threads) in the caller's LDS buffer.
// P2, P3: the LDS image descriptions of conv2 forward (one sample per iteration) and conv3 forward.
// FULL: act2, act3's lo part and all sign bits are written unconditionally (see conv1_fwd_resident_body).
template <class P2, class P3, bool FULL = false>
__device__ __forceinline__ void conv23_fwd_fused_body(u32x4 *lds, int block, const Conv23Args &a, int B, int spw) {
    // conv2 (producers)
    constexpr int CI2 = P2::CI, NCH2 = CI2 / 8, IMG2 = P2::IMG, KS2 = P2::K / 32;
    constexpr int PARTS2 = 8, KH2 = KS2 / PARTS2;                // a tile's k-steps in eight parts: two sets of 16 fragment registers
    constexpr int R2 = P2::P, NT2 = (R2 + 15) / 16;
    constexpr int NQ2 = P2::SRC_PIX * NCH2, NL2 = (NQ2 + C23_THREADS - 1) / C23_THREADS;   // 16-byte chunks of a sample's act1, per part and per thread
    // conv3 (consumers), one sample per iteration
    constexpr int CI3 = P3::CI, IMG3 = P3::IMG, KS3 = P3::K / 32;
    constexpr int PARTS3 = 2, KH3 = KS3 / PARTS3;                // two halves of nine k-steps
    constexpr int R3 = P3::P, NT3 = (R3 + 15) / 16;
    static_assert(P2::G == 1 && P2::SPLIT && P3::SPLIT && !P2::ZERO_FILL && !P3::ZERO_FILL, "three-product layers without borders");
    static_assert(P2::CO == 64 && P3::CO == 64 && P2::CO == CI3 && P2::P == P3::SRC_PIX, "conv2's output is conv3's input");
    static_assert(KS2 % PARTS2 == 0 && PARTS2 % 2 == 0 && KS3 % PARTS3 == 0 && PARTS3 % 2 == 0 && P2::PSB == CI2 * 2 + 32 && P3::PSB == CI3 * 2 + 32, "k-steps in an even number of parts");
    static_assert(layout_is_uniform<P2>() && layout_is_uniform<P3>(), "fragment rows must advance by one pixel stride modulo 256 bytes");
    static_assert(conv23_fwd_lds_bytes<P2, P3>() <= 160 * 1024 && IMG2 % 16 == 0 && IMG3 % 16 == 0, "LDS budget");

    char *const a1l = reinterpret_cast<char *>(lds);                 // act1 image of one sample, hi then lo
    char *const a2l = a1l + 2 * IMG2;                                // two act2 images (hi then lo each): double buffered

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, lg = lane >> 4;
    const bool producer = wave >= 4;
    const int s_begin = block * spw;
    const int s_end = s_begin + spw < B ? s_begin + spw : B;
    if (s_begin >= s_end) return;

    // act1 of consecutive samples is prefetched and staged by all eight wavefronts: one persistent pointer per load,
    // advanced by a sample after each use; the lo tensor is at a fixed distance from the hi tensor
    u32x4 rh[NL2], rl[NL2];
    const u32x4 *ph[NL2];
    const ptrdiff_t lo_at = reinterpret_cast<const u32x4 *>(a.a1_lo) - reinterpret_cast<const u32x4 *>(a.a1);
#pragma unroll
    for (int i = 0; i < NL2; ++i) {
        const int q = tid + C23_THREADS * i;
        ph[i] = reinterpret_cast<const u32x4 *>(a.a1 + (size_t)s_begin * (NQ2 * 8) + (size_t)(q < NQ2 ? q : NQ2 - 1) * 8);
    }
    auto gload = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NL2; ++i) {
            rh[i] = *ph[i];
            rl[i] = *(ph[i] + lo_at);
            ph[i] += NQ2;
        }
    };
    auto stage = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NL2; ++i) {
            const int q = tid + C23_THREADS * i;
            if (q < NQ2) {
                const int p = q / NCH2, c = q - p * NCH2;
                const int off = P2::dst_off(p) + c * 16;
                *reinterpret_cast<u32x4 *>(a1l + off) = rh[i];
                *reinterpret_cast<u32x4 *>(a1l + IMG2 + off) = rl[i];
            }
        }
    };
    gload();

    // Both roles run the same sequence of barriers: one in the prologue and two per sample.
    if (producer) {
        const int pw = wave - 4;
        const int n0 = pw * 16 + 4 * lg;                         // this lane's four output channels
        bf16x8 wh[KS2], wl[KS2];
        {
            const size_t row = frag_base(pw, P2::K, lane);
#pragma unroll
            for (int ks = 0; ks < KS2; ++ks) {
                wh[ks] = as_bf16x8(*reinterpret_cast<const u32x4 *>(a.w2 + row + FRAG_STEP * ks));
                wl[ks] = as_bf16x8(*reinterpret_cast<const u32x4 *>(a.w2_lo + row + FRAG_STEP * ks));
            }
        }
        const float4 bias = *reinterpret_cast<const float4 *>(a.b2 + n0);
        wait_global_loads();
        // per-lane addresses of the position tiles: fragment base in the act1 image, and where the lane's four
        // channels of its position go in an act2 image (-1: padded row)
        int t_base[NT2], t_dst[NT2];
#pragma unroll
        for (int t = 0; t < NT2; ++t) {
            const int row = t * 16 + li;
            const int rowc = row < R2 ? row : R2 - 1;            // padded rows recompute the last one; never stored
            t_base[t] = P2::base_off(rowc) + 16 * lg;
            t_dst[t] = row < R2 ? P3::dst_off(rowc) + n0 * 2 : -1;
        }
        auto load_half = [&](int base, int half, bf16x8 (&fh)[KH2], bf16x8 (&fl)[KH2]) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < KH2; ++j) {
                const int ks = half * KH2 + j;
                const int tap = (32 * ks) / CI2, ci0 = (32 * ks) % CI2;
                const int off = base + P2::tap_off(tap) + ci0 * 2;
                fh[j] = as_bf16x8(*reinterpret_cast<const u32x4 *>(a1l + off));
                fl[j] = as_bf16x8(*reinterpret_cast<const u32x4 *>(a1l + IMG2 + off));
            }
        };
        auto mfma_half = [&](int half, const bf16x8 (&fh)[KH2], const bf16x8 (&fl)[KH2], f32x4 &acc) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < KH2; ++j) {
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wl[half * KH2 + j], fh[j], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[half * KH2 + j], fl[j], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[half * KH2 + j], fh[j], acc, 0, 0, 0);
            }
        };
        // act2 of sample s (its act1 image is staged) into the LDS image dst, and what the backward pass needs of it
        auto produce = [&](char *dst, int s) __attribute__((always_inline)) {
            // the fragments of the next part (an eighth of a tile's k-steps) are read while the MFMAs of the current
            // one run: two register sets, statically alternated (an even number of parts per tile)
            bf16x8 fh[2][KH2], fl[2][KH2];
            load_half(t_base[0], 0, fh[0], fl[0]);
#pragma unroll
            for (int t = 0; t < NT2; ++t) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int part = 0; part < PARTS2; ++part) {
                    const bool last = part + 1 == PARTS2;
                    const int tn = last ? (t + 1 < NT2 ? t + 1 : t) : t;     // the last tile repeats its own first reads
                    load_half(t_base[tn], last ? 0 : part + 1, fh[(part + 1) & 1], fl[(part + 1) & 1]);
                    __builtin_amdgcn_sched_barrier(0);
                    mfma_half(part, fh[part & 1], fl[part & 1], acc);
                    __builtin_amdgcn_sched_barrier(0);
                }
                const float r0 = fmaxf(acc[0] + bias.x, 0.f), r1 = fmaxf(acc[1] + bias.y, 0.f);
                const float r2 = fmaxf(acc[2] + bias.z, 0.f), r3 = fmaxf(acc[3] + bias.w, 0.f);
                const bf16x4 h = {(__bf16)r0, (__bf16)r1, (__bf16)r2, (__bf16)r3};
                const u32x2 hi = __builtin_bit_cast(u32x2, h);
                const u32x2 lo = pack_bf16x4(r0 - (float)h[0], r1 - (float)h[1], r2 - (float)h[2], r3 - (float)h[3]);
                const bool valid = t_dst[t] >= 0;
                const int pos = t * 16 + li;
                const size_t at = ((size_t)s * R2 + pos) * P2::CO + n0;
                if (valid) {
                    *reinterpret_cast<u32x2 *>(dst + t_dst[t]) = hi;
                    *reinterpret_cast<u32x2 *>(dst + IMG3 + t_dst[t]) = lo;
                    if (FULL || a.a2) *reinterpret_cast<u32x2 *>(a.a2 + at) = hi;
                }
                if (FULL || a.m2) {
                    const uint32_t bits = sign_bits16(r0, r1, r2, r3, lg);     // all lanes take part
                    if (lg == 0 && valid) *reinterpret_cast<uint16_t *>(a.m2 + (at >> 3)) = (uint16_t)bits;
                }
            }
        };

        stage();
        __syncthreads();
        if (s_begin + 1 < s_end) gload();
        produce(a2l, s_begin);     // first sample: its act2 before the loop
        int cur = 0;
        for (int s = s_begin; s < s_end; ++s) {
            // act2 of s is complete in buffer cur; conv3 of s-1 has read the other buffer; all producers are done
            // with the act1 image of s
            __syncthreads();
            if (s + 1 < s_end) stage();
            __syncthreads();
            if (s + 2 < s_end) gload();
            if (s + 1 < s_end) produce(a2l + (cur ^ 1) * (2 * IMG3), s + 1);
            cur ^= 1;
        }
    } else {
        const int n0 = wave * 16 + 4 * lg;
        // The first act1 image goes to LDS before this role's weights are asked for: the producers cannot start
        // before it is there (prologue barrier) and before their own weights are, while conv3's weights are not
        // needed until the producers have finished the first sample -- fetched now they would only compete with
        // the producers' for the L2.
        stage();
        __syncthreads();
        if (s_begin + 1 < s_end) gload();
        bf16x8 wh[KS3], wl[KS3];
        {
            const size_t row = frag_base(wave, P3::K, lane);
#pragma unroll
            for (int ks = 0; ks < KS3; ++ks) {
                wh[ks] = as_bf16x8(*reinterpret_cast<const u32x4 *>(a.w3 + row + FRAG_STEP * ks));
                wl[ks] = as_bf16x8(*reinterpret_cast<const u32x4 *>(a.w3_lo + row + FRAG_STEP * ks));
            }
        }
        const float4 bias = *reinterpret_cast<const float4 *>(a.b3 + n0);
        wait_global_loads();
        int t_base[NT3];
#pragma unroll
        for (int t = 0; t < NT3; ++t) {
            const int row = t * 16 + li;
            t_base[t] = P3::base_off(row < R3 ? row : R3 - 1) + 16 * lg;
        }
        auto load_half = [&](const char *src, int base, int half, bf16x8 (&fh)[KH3], bf16x8 (&fl)[KH3]) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < KH3; ++j) {
                const int ks = half * KH3 + j;
                const int tap = (32 * ks) / CI3, ci0 = (32 * ks) % CI3;
                const int off = base + P3::tap_off(tap) + ci0 * 2;
                fh[j] = as_bf16x8(*reinterpret_cast<const u32x4 *>(src + off));
                fl[j] = as_bf16x8(*reinterpret_cast<const u32x4 *>(src + IMG3 + off));
            }
        };
        auto mfma_half = [&](int half, const bf16x8 (&fh)[KH3], const bf16x8 (&fl)[KH3], f32x4 &acc) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < KH3; ++j) {
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wl[half * KH3 + j], fh[j], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[half * KH3 + j], fl[j], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[half * KH3 + j], fh[j], acc, 0, 0, 0);
            }
        };
        int cur = 0;
        for (int s = s_begin; s < s_end; ++s) {
            __syncthreads();                          // act2 of s is complete; the producers are done with act1 of s
            if (s + 1 < s_end) stage();
            __syncthreads();
            if (s + 2 < s_end) gload();
            const char *src = a2l + cur * (2 * IMG3);
#pragma unroll
            for (int t = 0; t < NT3; ++t) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                bf16x8 fh[KH3], fl[KH3];
#pragma unroll
                for (int part = 0; part < PARTS3; ++part) {
                    load_half(src, t_base[t], part, fh, fl);
                    mfma_half(part, fh, fl, acc);
                }
                const float r0 = fmaxf(acc[0] + bias.x, 0.f), r1 = fmaxf(acc[1] + bias.y, 0.f);
                const float r2 = fmaxf(acc[2] + bias.z, 0.f), r3 = fmaxf(acc[3] + bias.w, 0.f);
                const int pos = t * 16 + li;
                const bool valid = pos < R3;
                const size_t at = ((size_t)s * R3 + pos) * P3::CO + n0;
                if (valid) store_bf16x4_split(a.a3, a.a3_lo, at, r0, r1, r2, r3, std::integral_constant<bool, FULL>());
                if (FULL || a.m3) {
                    const uint32_t bits = sign_bits16(r0, r1, r2, r3, lg);     // all lanes take part
                    if (lg == 0 && valid) *reinterpret_cast<uint16_t *>(a.m3 + (at >> 3)) = (uint16_t)bits;
                }
            }
            cur ^= 1;
        }
    }
}

template <class P2, class P3>
__global__ __launch_bounds__(C23_THREADS) void conv23_fwd_fused_kernel(const Conv23Args a, int B, int spw) {
    __shared__ u32x4 lds[conv23_fwd_lds_bytes<P2, P3>() / 16];
    conv23_fwd_fused_body<P2, P3>(lds, blockIdx.x, a, B, spw);
}

// conv1, conv2 and conv3 forward of a workgroup's sample range, one layer pair after the other, in one launch: the
// three layers are independent across samples, so a workgroup only waits for its own act1 (a barrier)
// instead of for the whole grid, and the launch boundary between conv1 and the fused conv2/conv3 kernel is gone.
// act1 still goes through global memory (the backward pass needs it, and the layers' LDS images do not fit side by
// side).  Both bodies use the same sample ranges (spw per workgroup) and 512 threads.
template <class Geo, class P2, class P3>
__global__ __launch_bounds__(C23_THREADS) void conv123_fwd_kernel(const uint8_t *__restrict__ obs, const __bf16 *__restrict__ w1,
                                                                  const __bf16 *__restrict__ w1_lo, const float *__restrict__ b1,
                                                                  uint8_t *__restrict__ m1, const Conv23Args a, int B, int spw) {
    static_assert(RES_THREADS == C23_THREADS, "one block size for both bodies");
    constexpr int L1 = conv1_fwd_lds_bytes<Geo>(), L23 = conv23_fwd_lds_bytes<P2, P3>();
    __shared__ u32x4 lds[(L1 > L23 ? L1 : L23) / 16];
    conv1_fwd_resident_body<Geo, true>(lds, blockIdx.x, 0, 1, obs, w1, w1_lo, b1, const_cast<__bf16 *>(a.a1), const_cast<__bf16 *>(a.a1_lo),
                                 m1, B, spw);
    // The barrier orders this workgroup's act1 stores before its own reads (a workgroup's wavefronts share the CU's
    // vector cache).  A device-wide fence here is ruinous: it writes back and invalidates the whole L2 of the XCD,
    // once per workgroup (measured: 186 instead of 97 us).
    __syncthreads();
    conv23_fwd_fused_body<P2, P3, true>(lds, blockIdx.x, a, B, spw);
}

}  // namespace arn
