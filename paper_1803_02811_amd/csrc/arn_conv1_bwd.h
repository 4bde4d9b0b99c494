// conv2's input gradient and conv1's weight gradient in one workgroup body (a range of conv_backward_kernel).
//
// d(pre1) -- the largest tensor of the backward pass -- has a single consumer, conv1's weight gradient
// (conv1's input is data, so there is no input gradient below it).  Here a workgroup produces a sample's
// d(pre1) into LDS and contracts it there against the sample's frame: d(pre1) never goes to HBM.
//
// The eight wavefronts of a workgroup have two roles.  Four "producers" compute d(pre1) of sample s+1: the
// stride-2 input gradient as one 2x2 stride-1 correlation with 4 x 32 phase channels (one phase per wavefront,
// all k of its weights in registers, fragments read from the zero-bordered d(pre2) image as in
// resident_conv_kernel), masked by the sign bits of act1, written as bf16 rows into one of two LDS buffers.
// Meanwhile four "consumers" contract d(pre1) of sample s (the other buffer) against the bf16 image of the
// frame with transposing LDS reads that address the 8x8 windows directly, as in the weight-gradient kernels.
// Consumer w owns the two 32-column tiles of dW1 that belong to input channel w, so it is the only reader of
// that channel's plane of the image: it loads, converts and stores the plane itself, after its own contraction,
// with no barrier.  The producers stage d(pre2) and the mask words, which all four of them read.  The producers
// mostly use the MFMA pipe and VALU, the consumers the LDS, so the two roles fill each other's gaps on a SIMD;
// their code sits in two branches that execute the same barriers, so registers are allocated for one role only.
//
// Each workgroup owns a fixed, contiguous range of samples and accumulates dW1 in registers; partial results
// go to part[workgroup][32*256 + 32] and are summed in workgroup order by the reduction kernel.
#pragma once
#include "arn_resident.h"
#include "arn_resident_conv.h"

namespace arn {

constexpr int C1B_THREADS = 512;   // four consumer wavefronts (0-3), four producers (4-7); one workgroup per CU

// LDS layout of a d(pre1) buffer: rows of 32 bf16 (64 bytes); inside every 256-byte block of four rows the
// eight 32-byte granules are rotated by the block index.  A producer writes 16 positions two pixels apart
// (32 bytes each) per instruction: unrotated they would share two of the eight granule slots (an eight-way bank
// conflict, measured as a bottleneck); rotated they cover all eight.  The consumers' transposing reads take
// four consecutive rows of one block and stay conflict free.
__device__ __forceinline__ constexpr int dy1_offset(int row, int byte) {
    return (row >> 2) * 256 + ((((row & 3) * 2 + (byte >> 5) + (row >> 2)) & 7) << 5) + (byte & 31);
}

// LDS bytes of conv1_bwd_fused_body<Geo, D>
template <class Geo, class D>
constexpr int conv1_bwd_lds_bytes() {
    constexpr int RPAD = (Geo::P1 + 15) / 16 * 16;
    return 8 * Geo::IN_H * Geo::IN_W + 2 * RPAD * C1 * 2 + D::IMG + Geo::P1 * C1 / 8 + (80 % Geo::W1 != 0 ? RPAD : 4) * 4;
}

// The work of workgroup `block` (of C1B_THREADS threads) in the caller's LDS buffer `lds`.
// Geo: frame geometry; D: the description of conv2's input gradient (ResConv2Dgrad / ResConv2DgradGeo: the
// d(pre2) image of one sample).  obs u8 [B][4][IN_H][IN_W]; dy2 = d(pre2) bf16 [B][P2][64]; w2d: the packed
// input-gradient weights [phase*32 + ci][(ty*2 + tx)*64 + co]; mask1: sign bits of act1 (P1*32/8 bytes per sample).
template <class Geo, class D>
__device__ __forceinline__ void conv1_bwd_fused_body(u32x4 *lds, int block, const uint8_t *__restrict__ obs,
                                                     const __bf16 *__restrict__ dy2, const __bf16 *__restrict__ w2d,
                                                     const uint8_t *__restrict__ mask1, float *__restrict__ part, int B,
                                                     int spw) {
    constexpr int IN_H = Geo::IN_H, IN_W = Geo::IN_W, W1 = Geo::W1, P1 = Geo::P1, OBS_BYTES = Geo::OBS_BYTES;
    constexpr int NT = C1B_THREADS, NR = NT / 2;                 // threads in all, and per role
    // consumer side (a weight-gradient contraction over the P1 positions, as in conv_wgrad_resident_body)
    constexpr int PLANE_U4 = IN_H * IN_W / 16;                   // one input channel of the frame, 16 pixels per word
    constexpr int NI = (PLANE_U4 + 63) / 64;                     // words per lane of the wavefront that owns the plane
    constexpr int KSTEPS = (P1 + 15) / 16, RPAD = KSTEPS * 16;   // contraction steps; d(pre1) rows P1..RPAD stay zero
    constexpr int DYB = RPAD * C1 * 2;                           // bytes of one d(pre1) buffer
    constexpr int TX = 2;                                        // column tiles of dW1 per consumer: one input channel
    constexpr bool TABLE = 80 % W1 != 0;
    // producer side (as resident_conv_kernel<D> with one sample)
    constexpr int CI = D::CI, NCH = CI / 8, KS = D::K / 32, KH = KS / 2, CT = D::CO / 64;
    constexpr int NQ = D::SRC_PIX * NCH, NG = (NQ + NR - 1) / NR;
    constexpr int DT = (D::P + 15) / 16;                         // position tiles of the 2x2 correlation
    constexpr int MWORDS = P1 * C1 / 32, NM = (MWORDS + NR - 1) / NR;   // 4-byte words of act1 sign bits per sample
    static_assert((IN_H * IN_W) % 16 == 0 && OBS_BYTES == 4 * IN_H * IN_W, "a channel plane is copied in 16-byte words");
    static_assert(D::CO == 4 * C1 && CT == 2 && D::PSB == CI * 2 + 32, "four phases of 32 channels, one phase per producer");
    static_assert((P1 * C1) % 32 == 0, "whole mask words per sample");
    static_assert(!D::SPLIT && D::ZERO_FILL && D::G == 1, "single-product input gradient over a zero-bordered image, one sample");
    static_assert(layout_is_uniform<D>(), "fragment rows must advance by one pixel stride modulo 256 bytes");
    static_assert(D::IMG % 16 == 0 && DYB % 16 == 0, "16-byte aligned LDS regions");
    static_assert(conv1_bwd_lds_bytes<Geo, D>() == 8 * PLANE_U4 * 16 + 2 * DYB + D::IMG + 4 * MWORDS + 4 * (TABLE ? RPAD : 4) &&
                      conv1_bwd_lds_bytes<Geo, D>() <= 160 * 1024, "LDS budget");
    static_assert(4 * 16 * C1 * 4 <= DYB, "bias-gradient scratch");

    u32x4 *const s_img = lds;                                    // bf16 [4][IN_H][IN_W]
    u32x4 *const s_dy = s_img + 8 * PLANE_U4;                    // d(pre1), bf16 [2][RPAD][32], rows laid out by dy1_offset
    u32x4 *const s_g = s_dy + 2 * DYB / 16;                      // bordered d(pre2) image
    uint32_t *const s_mask = reinterpret_cast<uint32_t *>(s_g + D::IMG / 16);   // word p: the 32 sign bits of act1 at position p
    int *const s_win = reinterpret_cast<int *>(s_mask + MWORDS); // byte offset of the window origin of output position m in s_img

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, lg = lane >> 4;
    const bool producer = wave >= 4;
    const int s_begin = block * spw;
    const int s_end = s_begin + spw < B ? s_begin + spw : B;
    if (s_begin >= s_end) return;

    for (int i = tid; i < D::IMG / 16; i += NT) s_g[i] = zero_u4();
    if constexpr (RPAD > P1) {
        // rows P1..RPAD of both buffers stay zero: the blocks that hold them are cleared whole (their valid rows
        // are rewritten for every sample)
        constexpr int Z0 = (P1 & ~3) * C1 * 2 / 16, ZN = DYB / 16 - Z0;
        for (int i = tid; i < 2 * ZN; i += NT) s_dy[(i / ZN) * (DYB / 16) + Z0 + i % ZN] = zero_u4();
    }
    auto window = [&](int m) __attribute__((always_inline)) {
        const int mm = RPAD > P1 && m >= P1 ? P1 - 1 : m;   // rows past the last position (their dY is zero) take its window
        const int oy = mm / W1, ox = mm - oy * W1;
        return (S1 * oy * IN_W + S1 * ox) * 2;
    };
    if constexpr (TABLE)
        for (int m = tid; m < RPAD; m += NT) s_win[m] = window(m);

    char *const img = reinterpret_cast<char *>(s_img);
    char *const dyl = reinterpret_cast<char *>(s_dy);
    char *const gl = reinterpret_cast<char *>(s_g);
    float *out = part + (size_t)block * (C1 * KW1 + C1);
    float *red = reinterpret_cast<float *>(s_dy);      // epilogue scratch

    // Both roles run the same sequence of barriers: two in the prologue, two per sample, two in the epilogue.
    // Every global load of the sample loop has a persistent pointer, advanced by a sample after each use, so that
    // the prefetch needs no address arithmetic in registers that an earlier load may still be filling.
    if (producer) {
        const int ptid = tid - NR;
        // phase = (wavefront - 4): 32 channels, all k of their weights as A-operand fragments
        const int phase = wave - 4;
        bf16x8 wd[CT][KS];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            const size_t row = frag_base(phase * 2 + ct, D::K, lane);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) wd[ct][ks] = as_bf16x8(*reinterpret_cast<const u32x4 *>(w2d + row + FRAG_STEP * ks));
        }
        // d(pre2) and mask words of consecutive samples
        u32x4 rg[NG];
        uint32_t rm[NM];
        const u32x4 *pg[NG];
        const uint32_t *pm[NM];
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            const int idx = ptid + NR * i;
            pg[i] = reinterpret_cast<const u32x4 *>(dy2 + (size_t)s_begin * D::SRC_PIX * CI) + (idx < NQ ? idx : NQ - 1);
        }
#pragma unroll
        for (int i = 0; i < NM; ++i) {
            const int idx = ptid + NR * i;
            pm[i] = reinterpret_cast<const uint32_t *>(mask1 + (size_t)s_begin * (MWORDS * 4)) + (idx < MWORDS ? idx : MWORDS - 1);
        }
        auto gload_g = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < NG; ++i) {
                rg[i] = *pg[i];
                pg[i] += D::SRC_PIX * CI * 2 / 16;
            }
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                rm[i] = *pm[i];
                pm[i] += MWORDS;
            }
        };
        auto stage_g = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < NG; ++i) {
                const int q = ptid + NR * i;
                if (q < NQ) {
                    const int p = q / NCH, c = q - p * NCH;
                    *reinterpret_cast<u32x4 *>(gl + D::dst_off(p) + c * 16) = rg[i];
                }
            }
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                const int q = ptid + NR * i;
                if (q < MWORDS) s_mask[q] = rm[i];
            }
        };
        gload_g();
        wait_global_loads();
        // bias gradient: what this lane writes into d(pre1), channels ct*16 + 4*lg + r, added in fp32
        float bs[CT][4];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int r = 0; r < 4; ++r) bs[ct][r] = 0.f;

        // Per-lane addresses of the position tiles, which do not depend on the sample: fragment base in the d(pre2)
        // image, where channels ct*16 + 4*lg .. + 3 of the lane's position land in a d(pre1) buffer (-1: padded row
        // or outside the map), and the position's mask word.
        int t_base[DT], t_dst[DT][CT], t_mask[DT];
#pragma unroll
        for (int t = 0; t < DT; ++t) {
            int row = t * 16 + li;
            const bool valid = row < D::P;
            row = valid ? row : D::P - 1;                 // padded rows recompute the last one; never stored
            const int pix = valid ? D::out_pixel(row, phase) : -1;
            t_base[t] = D::base_off(row) + 16 * lg;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) t_dst[t][ct] = pix < 0 ? -1 : dy1_offset(pix, (ct * 16 + 4 * lg) * 2);
            t_mask[t] = pix < 0 ? 0 : pix;
        }
        // The fragment reads are pipelined by half-tiles: the second half of a tile's k-steps is in flight during
        // the MFMAs of the first, the first half of the next tile (and its mask word) during those of the second.
        auto load_half = [&](int base, int half, bf16x8 (&f)[KH]) __attribute__((always_inline)) {
#pragma unroll
            for (int jk = 0; jk < KH; ++jk) {
                const int ks = half * KH + jk;
                const int tap = (32 * ks) / CI, ci0 = (32 * ks) % CI;
                f[jk] = as_bf16x8(*reinterpret_cast<const u32x4 *>(gl + base + D::tap_off(tap) + ci0 * 2));
            }
        };
        auto mfma_half = [&](int half, const bf16x8 (&f)[KH], f32x4 (&da)[CT]) __attribute__((always_inline)) {
#pragma unroll
            for (int jk = 0; jk < KH; ++jk)
#pragma unroll
                for (int ct = 0; ct < CT; ++ct)
                    da[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wd[ct][half * KH + jk], f[jk], da[ct], 0, 0, 0);
        };
        // d(pre1) of the sample whose d(pre2) image and mask are staged, into dst
        auto produce = [&](char *dst) __attribute__((always_inline)) {
            bf16x8 fa[KH], fb[KH];
            uint32_t mk, mk_next;
            load_half(t_base[0], 0, fa);
            mk = s_mask[t_mask[0]];
#pragma unroll
            for (int t = 0; t < DT; ++t) {
                const int tn = t + 1 < DT ? t + 1 : t;        // the last tile repeats its own reads
                f32x4 da[CT];
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) da[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
                load_half(t_base[t], 1, fb);
                __builtin_amdgcn_sched_barrier(0);
                mfma_half(0, fa, da);
                __builtin_amdgcn_sched_barrier(0);
                load_half(t_base[tn], 0, fa);
                mk_next = s_mask[t_mask[tn]];
                __builtin_amdgcn_sched_barrier(0);
                mfma_half(1, fb, da);
                __builtin_amdgcn_sched_barrier(0);
                if (t_dst[t][0] >= 0) {
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) {
                        const int m = (int)(mk >> (ct * 16 + 4 * lg));   // bit r: channel ct*16 + 4*lg + r
                        float v[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) {         // bit r set: keep the value (AND with all ones), else zero
                            const float x = da[ct][r];
                            v[r] = __int_as_float(__float_as_int(x) & -((m >> r) & 1));
                            bs[ct][r] += v[r];
                        }
                        *reinterpret_cast<u32x2 *>(dst + t_dst[t][ct]) = pack_bf16x4(v[0], v[1], v[2], v[3]);
                    }
                }
                mk = mk_next;
            }
        };

        __syncthreads();                              // zero fill done
        stage_g();
        __syncthreads();
        if (s_begin + 1 < s_end) gload_g();
        produce(dyl);                                 // first sample: its d(pre1) before the loop
        int cur = 0;
        for (int s = s_begin; s < s_end; ++s) {
            // d(pre1) of s is complete in buffer cur; the contraction of s-1 has read the other buffer; all producers
            // are done with the d(pre2) image of s
            __syncthreads();
            if (s + 1 < s_end) stage_g();
            __syncthreads();
            if (s + 2 < s_end) gload_g();
            if (s + 1 < s_end) produce(dyl + (cur ^ 1) * DYB);
            cur ^= 1;
        }
        __syncthreads();
        // bias gradient: channel c = ct*16 + 4*lg + r is held by lanes (li = 0..15, lg) of all producers
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[(phase * 16 + li) * C1 + ct * 16 + 4 * lg + r] = bs[ct][r];
        __syncthreads();
    } else {
        // wavefront w: input channel w, i.e. column tiles 2w (kernel rows 0-3) and 2w+1 (rows 4-7) of dW1, and the
        // channel's plane of the image
        f32x16 acc[TX];
#pragma unroll
        for (int b = 0; b < TX; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[b][r] = 0.f;
        u32x4 rimg[NI];
        const u32x4 *pimg[NI];
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int idx = lane + 64 * i;
            pimg[i] = reinterpret_cast<const u32x4 *>(obs + (size_t)s_begin * OBS_BYTES) + wave * PLANE_U4 +
                      (idx < PLANE_U4 ? idx : PLANE_U4 - 1);
        }
        auto gload_plane = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                rimg[i] = *pimg[i];
                pimg[i] += OBS_BYTES / 16;
            }
        };
        auto stage_plane = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int idx = lane + 64 * i;
                if (idx < PLANE_U4) {
                    s_img[2 * (wave * PLANE_U4 + idx)] = u8x8_to_bf16x8(rimg[i].x, rimg[i].y);
                    s_img[2 * (wave * PLANE_U4 + idx) + 1] = u8x8_to_bf16x8(rimg[i].z, rimg[i].w);
                }
            }
        };
        gload_plane();
        const int o = lane & 15, Gq = lane >> 4;
        const int row_in_step = 8 * (Gq >> 1) + (o >> 2);          // + 4 for the second read
        const int ycol_off = (16 * (Gq & 1) + 4 * (o & 3)) * 2;    // byte offset inside a d(pre1) row
        // rows 16 ks + row_in_step (+ 4): a step of 16 rows is four blocks, so the rotation alternates between
        // two values with the parity of ks -- granule index + 4, i.e. bit 7 of the byte offset flipped
        const int ya = dy1_offset(row_in_step, ycol_off), yb = dy1_offset(row_in_step + 4, ycol_off);
        const int ky_lane = 2 * (Gq & 1) + ((o & 3) >> 1), kx0 = 4 * (o & 1);
        // byte offset of (ci, ky, kx0) for column tile t = ci*2 + upper/lower four kernel rows
        int xoff[TX];
#pragma unroll
        for (int b = 0; b < TX; ++b) xoff[b] = ((wave * IN_H + b * 4 + ky_lane) * IN_W + kx0) * 2;

        __syncthreads();                              // zero fill and window table done
        stage_plane();                                // nobody else touches this plane
        __syncthreads();
        if (s_begin + 1 < s_end) gload_plane();
        int cur = 0;
        for (int s = s_begin; s < s_end; ++s) {
            __syncthreads();                          // d(pre1) of s is complete
            __syncthreads();                          // (the producers' staging barrier)
            const char *src = dyl + cur * DYB;
#pragma unroll 5
            for (int ks = 0; ks < KSTEPS; ++ks) {
                const int ma = 16 * ks + row_in_step, mb = ma + 4;
                const int pa = TABLE ? s_win[ma] : window(ma), pb = TABLE ? s_win[mb] : window(mb);
                const int flip = (ks & 1) << 7;
                const bf16x8 fy = tr_pair(src, ks * (16 * C1 * 2) + (ya ^ flip), ks * (16 * C1 * 2) + (yb ^ flip));
#pragma unroll
                for (int b = 0; b < TX; ++b) {
                    const bf16x8 fx = tr_pair(img, pa + xoff[b], pb + xoff[b]);
                    acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fy, fx, acc[b], 0, 0, 0);
                }
            }
            if (s + 1 < s_end) stage_plane();         // the plane of s+1: this wavefront's reads of s are done
            if (s + 2 < s_end) gload_plane();
            cur ^= 1;
        }
        __syncthreads();
        const int fr = lane & 31, fg = lane >> 5;
#pragma unroll
        for (int b = 0; b < TX; ++b) {
            const int k = (wave * TX + b) * 32 + fr;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int n = 8 * (r >> 2) + 4 * fg + (r & 3);
                out[n * KW1 + k] = acc[b][r];
            }
        }
        __syncthreads();
    }
    // bias gradient: the producers' lane sums, added in a fixed order
    if (tid < C1) {
        float t = red[tid];
        for (int g = 1; g < 4 * 16; ++g) t += red[g * C1 + tid];
        out[C1 * KW1 + tid] = t;
    }
}

}  // namespace arn
