// Convolutions (forward and input-gradient) with the input of a few samples
// resident in LDS and the layer's weights resident in registers.
//
// One workgroup (4 wavefronts) walks over a fixed range of samples.  For each
// group of G samples the input image (bf16, plus its low part in the
// three-product inference/forward precision) is copied once, contiguously, into
// a padded LDS image; the MFMA activation fragments are then read straight from
// that image at (position, tap) addresses -- no im2col tile is ever built, so
// each input element crosses the global-memory/LDS boundary once instead of once
// per overlapping window.  Every wavefront owns CO/4 output channels and keeps
// all K of their weights in registers for the whole kernel, so the only LDS
// traffic in the inner loop is one activation fragment per MFMA group.
// v_mfma_f32_16x16x32_bf16 is used because the 16-row position tile wastes
// least on the odd spatial sizes (81, 49, 100 positions per sample).
//
// LDS images are double buffered by sample group and the next group is
// prefetched into registers while the current one is multiplied.
//
// MFMA 16x16x32 layout (checked on hardware):
//   A (16 x 32): lane l holds row l%16, k = 8*(l/16) .. +7     -> weights, row = channel
//   B (32 x 16): lane l holds col l%16, k = 8*(l/16) .. +7     -> activations, col = position
//   D (16 x 16): lane l holds col l%16, rows 4*(l/16) + r, r = 0..3
#pragma once
#include <type_traits>

#include "arn_gemm.h"
#include "arn_layout.h"

namespace arn {

// Conv description C supplies (all static):
//   CI           input channels (32 or 64); a pixel is CI bf16, padded by 32 bytes in LDS
//   SRC_PIX      pixels per sample in global memory;  IMG  bytes of one sample's image in LDS
//   P, HO        output positions per sample (HO x HO)
//   CO, K        output channels (64 or 128) and contraction length (taps * CI)
//   G            samples per iteration;  SPLIT  three-product precision
//   ZERO_FILL    LDS image has a zero border (input-gradient problems)
//   dst_off(p)   LDS byte offset (within the sample's image) of source pixel p
//   base_off(pos) LDS byte offset of tap (0,0) of output position pos
//   tap_off(t)   LDS byte offset of tap t relative to tap (0,0)
//                LDS bank rule for the fragment reads (ds_read_b128, measured): the 64 lanes are served
//                in four groups of 16 -- lanes {0-3, 12-15, 20-23, 24-27}, {4-7, 8-11, 16-19, 28-31}
//                and the same plus 32 -- and a group is conflict-free when its 16-byte words fall in
//                16 different 16-byte slots modulo 256 bytes.  A fragment read has lane (li, lg) at
//                base_off(position li of the tile) + 16 lg; with a pixel stride of 32 mod 64 bytes it is
//                conflict-free as long as base_off advances by exactly one pixel stride (mod 256) from
//                every position to the next, also across the end of an output row and from one
//                sample of the group to the next.  The images therefore pad every row (and the
//                image) by the few 16-byte words that make those steps come out right.
//   NBUF         LDS image buffers: 2 = double buffered by sample group (one barrier per
//                group); 1 = single (two barriers) so that two or three workgroups share a CU
//                and fill each other's staging and latency gaps
//   PIPE         explicit half-tile software pipelining of the LDS fragment reads (needs
//                registers for two half-tiles of fragments on top of the weights)
//   MASK_ELEMS   0, or elements per sample of the tensor whose sign masks the output
//                (ReLU derivative); its sign bits (written by the forward kernels, one bit
//                per element) are staged to LDS with the image so that the epilogue needs
//                no dependent global load
// and an Args struct with in, in_lo (SPLIT), w, w_lo (SPLIT), mask (MASK_ELEMS > 0),
//   Lane lane(n)                      per-lane constants for channels n..n+3 (e.g. the bias)
//   store(sample, pos, n, v, lane, maskbits)   epilogue for channels n..n+3 of one position;
//                                     maskbits = LDS bytes, bit e&7 of byte e>>3 for element e
//                                     of the G samples' mask tensors.
// Threads per workgroup of the sample-resident kernels.  resident_conv_kernel uses four wavefronts
// (one per SIMD); each keeps its share of the weights in registers.
constexpr int RES_THREADS = 512;    // conv1 forward

// true if base_off advances by the pixel stride (mod 256 bytes) between all consecutive rows of a sample group
template <class C>
constexpr bool layout_is_uniform() {
    int prev = 0;
    for (int row = 0; row < C::G * C::P; ++row) {
        const int g = row / C::P, pos = row - g * C::P;
        const int at = g * C::IMG + C::base_off(pos);
        if (row > 0 && ((at - prev - C::PSB) & 255) != 0) return false;
        prev = at;
    }
    return true;
}

// Configurations with a static member WAVES = 8 run eight wavefronts per workgroup and one workgroup per CU
// (for images too large for two workgroups to share the LDS): wavefronts w and w + 4 own the same channel
// group and take alternate position tiles.
template <class C, class = void>
struct ResWaves {
    static constexpr int value = 4;
};
template <class C>
struct ResWaves<C, decltype((void)C::WAVES)> {
    static constexpr int value = C::WAVES;
};

template <class C>
__global__ __launch_bounds__(64 * ResWaves<C>::value, ResWaves<C>::value == 4 ? 2 : 1) void resident_conv_kernel(
    const typename C::Args a, int B, int spw) {
    constexpr int RESC_THREADS = 64 * ResWaves<C>::value;
    constexpr int WPARTS = ResWaves<C>::value / 4;       // wavefronts that share a channel group
    constexpr int CI = C::CI, PS = CI * 2 + 32, NCH = CI / 8;   // pixel stride = 32 mod 64 bytes: conflict-free 16-position x 4-chunk reads (measured)
    constexpr int IMG = C::IMG;                          // bytes of one sample's LDS image (rows padded, see below)
    constexpr int PARTS = C::SPLIT ? 2 : 1;              // hi (+ lo)
    constexpr int BUF = C::G * IMG * PARTS;              // one buffer: G samples, hi then lo
    constexpr int NQ = C::G * C::SRC_PIX * NCH;          // 16-byte chunks per part per iteration
    constexpr int NL = (NQ + RESC_THREADS - 1) / RESC_THREADS;
    constexpr int R = C::G * C::P, NT = (R + 15) / 16;
    constexpr int CT = C::CO / 64;                       // 16-channel tiles per wavefront
    constexpr int KS = C::K / 32, KH = KS / 2;           // k-steps per tile and per half-tile
    constexpr int MSB = C::MASK_ELEMS / 8;               // mask bytes per sample (1 bit per element)
    constexpr int MW = MSB % 8 == 0 ? 8 : 4;             // mask bytes are copied in 8-byte words where a sample's share allows
    typedef typename std::conditional<MW == 8, u32x2, uint32_t>::type MWord;
    constexpr int NMQ = C::G * MSB / MW;                 // mask words per iteration
    constexpr int NML = (NMQ + RESC_THREADS - 1) / RESC_THREADS;
    constexpr int MBUF = (NMQ * MW + 15) / 16 * 16;
    static_assert(C::MASK_ELEMS % 8 == 0 && MSB % MW == 0, "mask bytes per sample in whole words");
    static_assert(KS % 2 == 0, "k-steps split into two halves");
    constexpr int NBUF = C::NBUF;
    static_assert((BUF + MBUF) * NBUF <= 160 * 1024, "LDS budget");
    static_assert(C::PSB == PS && IMG % 16 == 0, "pixel stride / image alignment");
    static_assert(layout_is_uniform<C>(), "fragment rows must advance by one pixel stride modulo 256 bytes");

    __shared__ u32x4 lds[NBUF * BUF / 16];
    __shared__ MWord lds_mask8[NMQ ? NBUF * MBUF / MW : 2];
    uint8_t *const lds_mask = reinterpret_cast<uint8_t *>(lds_mask8);
    char *const lds_b = reinterpret_cast<char *>(lds);

    const int tid = threadIdx.x, lane = tid & 63, wave = (tid >> 6) & 3;
    const int li = lane & 15, lg = lane >> 4;
    const int s_begin = blockIdx.x * spw;
    const int s_end = s_begin + spw < B ? s_begin + spw : B;
    if (s_begin >= s_end) return;
    // small batches: gridDim.y workgroups share a sample group, each taking every gridDim.y-th position tile
    // (and the wavefronts that share a channel group split those again)
    const int t_first = blockIdx.y * WPARTS + (tid >> 8), t_step = gridDim.y * WPARTS;

    // weights of this wavefront's channels, all k, as A-operand fragments (loaded below, after the
    // first image loads have been issued, so that staging does not wait for them)
    bf16x8 wh[CT][KS], wl[C::SPLIT ? CT : 1][C::SPLIT ? KS : 1];

    typename C::Args::Lane lane_state[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) lane_state[ct] = a.lane(wave * (16 * CT) + ct * 16 + 4 * lg);

    u32x4 rh[NL], rl[C::SPLIT ? NL : 1];
    MWord rm[NML ? NML : 1];
    auto gload = [&](int s) __attribute__((always_inline)) {   // samples s .. s+G-1 (clamped to the last valid one)
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            int q = tid + RESC_THREADS * i;
            q = q < NQ ? q : NQ - 1;
            const int g = q / (C::SRC_PIX * NCH), rem = q - g * (C::SRC_PIX * NCH);
            const int sg = s + g < s_end ? s + g : s_end - 1;
            const size_t at = (size_t)sg * C::SRC_PIX * CI + (size_t)rem * 8;
            rh[i] = *reinterpret_cast<const u32x4 *>(a.in + at);
            if constexpr (C::SPLIT) rl[i] = *reinterpret_cast<const u32x4 *>(a.in_lo + at);
        }
        if constexpr (NMQ > 0) {
#pragma unroll
            for (int i = 0; i < NML; ++i) {
                int q = tid + RESC_THREADS * i;
                q = q < NMQ ? q : NMQ - 1;
                const int g = q / (MSB / MW), rem = q - g * (MSB / MW);
                const int sg = s + g < s_end ? s + g : s_end - 1;
                rm[i] = *reinterpret_cast<const MWord *>(a.mask + (size_t)sg * MSB + (size_t)rem * MW);
            }
        }
    };
    auto stage = [&](int buf) __attribute__((always_inline)) {
        char *dst = lds_b + buf * BUF;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int q = tid + RESC_THREADS * i;
            if (q < NQ) {
                const int p = q / NCH, c = q - p * NCH;          // p = g * SRC_PIX + source pixel
                const int g = p / C::SRC_PIX, sp = p - g * C::SRC_PIX;
                const int off = g * IMG + C::dst_off(sp) + c * 16;
                *reinterpret_cast<u32x4 *>(dst + off) = rh[i];
                if constexpr (C::SPLIT) *reinterpret_cast<u32x4 *>(dst + C::G * IMG + off) = rl[i];
            }
        }
        if constexpr (NMQ > 0) {
#pragma unroll
            for (int i = 0; i < NML; ++i) {
                const int q = tid + RESC_THREADS * i;
                if (q < NMQ) lds_mask8[buf * (MBUF / MW) + q] = rm[i];
            }
        }
    };

    // activation fragments of one half-tile (k-steps half*KH .. +KH-1) of position tile t
    auto load_half = [&](const char *img, int t, int half, bf16x8 (&fh)[KH], bf16x8 (&fl)[C::SPLIT ? KH : 1])
                         __attribute__((always_inline)) {
        int row = t * 16 + li;
        row = row < R ? row : R - 1;                     // padded rows recompute the last one; never stored
        const int g = row / C::P, pos = row - g * C::P;
        const int base = g * IMG + C::base_off(pos) + 16 * lg;
#pragma unroll
        for (int j = 0; j < KH; ++j) {
            const int ks = half * KH + j;
            const int tap = (32 * ks) / CI, ci0 = (32 * ks) % CI;
            const int off = base + C::tap_off(tap) + ci0 * 2;
            fh[j] = as_bf16x8(*reinterpret_cast<const u32x4 *>(img + off));
            if constexpr (C::SPLIT) fl[j] = as_bf16x8(*reinterpret_cast<const u32x4 *>(img + C::G * IMG + off));
        }
    };
    auto mfma_half = [&](int half, const bf16x8 (&fh)[KH], const bf16x8 (&fl)[C::SPLIT ? KH : 1], f32x4 (&acc)[CT])
                         __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < KH; ++j) {
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                if (half == 0) {
                    if constexpr (C::SPLIT) {
                        acc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wl[ct][j], fh[j], acc[ct], 0, 0, 0);
                        acc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[ct][j], fl[j], acc[ct], 0, 0, 0);
                    }
                    acc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[ct][j], fh[j], acc[ct], 0, 0, 0);
                } else {
                    if constexpr (C::SPLIT) {
                        acc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wl[ct][KH + j], fh[j], acc[ct], 0, 0, 0);
                        acc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[ct][KH + j], fl[j], acc[ct], 0, 0, 0);
                    }
                    acc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[ct][KH + j], fh[j], acc[ct], 0, 0, 0);
                }
            }
        }
    };

    auto tile_store = [&](int t, const f32x4 (&acc)[CT], int s, const uint8_t *mbits) __attribute__((always_inline)) {
        const int orow = t * 16 + li;
        const int rowc = orow < R ? orow : R - 1;
        const int g = rowc / C::P, pos = rowc - g * C::P;
        if (orow < R && s + g < s_end) {
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
                a.store(s + g, g, pos, wave * (16 * CT) + ct * 16 + 4 * lg, acc[ct], lane_state[ct], mbits);
        }
    };

    gload(s_begin);
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        const size_t row = frag_base(wave * CT + ct, C::K, lane);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            wh[ct][ks] = as_bf16x8(*reinterpret_cast<const u32x4 *>(a.w + row + FRAG_STEP * ks));
            if constexpr (C::SPLIT) wl[ct][ks] = as_bf16x8(*reinterpret_cast<const u32x4 *>(a.w_lo + row + FRAG_STEP * ks));
        }
    }
    if constexpr (C::ZERO_FILL) {   // the zero border is written while the first image and the weights are on their way
        for (int i = tid; i < NBUF * BUF / 16; i += RESC_THREADS) lds[i] = zero_u4();
        __syncthreads();
    }
    wait_global_loads();
    int buf = 0;
    for (int s = s_begin; s < s_end; s += C::G) {
        stage(buf);
        __syncthreads();
        if (s + C::G < s_end) gload(s + C::G);
        const char *img = lds_b + buf * BUF;
        const uint8_t *mbits = lds_mask + buf * MBUF;

        if constexpr (C::PIPE) {
            bf16x8 fa_h[KH], fa_l[C::SPLIT ? KH : 1], fb_h[KH], fb_l[C::SPLIT ? KH : 1];
            load_half(img, t_first < NT ? t_first : 0, 0, fa_h, fa_l);
#pragma unroll 1
            for (int t = t_first; t < NT; t += t_step) {
                f32x4 acc[CT];
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) acc[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
                load_half(img, t, 1, fb_h, fb_l);            // in flight during the first half's MFMAs
                __builtin_amdgcn_sched_barrier(0);
                mfma_half(0, fa_h, fa_l, acc);
                __builtin_amdgcn_sched_barrier(0);
                load_half(img, t + t_step < NT ? t + t_step : t, 0, fa_h, fa_l);   // next tile's first half
                __builtin_amdgcn_sched_barrier(0);
                mfma_half(1, fb_h, fb_l, acc);
                __builtin_amdgcn_sched_barrier(0);
                tile_store(t, acc, s, mbits);
            }
        } else {
#pragma unroll 1
            for (int t = t_first; t < NT; t += t_step) {
                f32x4 acc[CT];
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) acc[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
                bf16x8 fh[KH], fl[C::SPLIT ? KH : 1];
                load_half(img, t, 0, fh, fl);
                mfma_half(0, fh, fl, acc);
                load_half(img, t, 1, fh, fl);
                mfma_half(1, fh, fl, acc);
                tile_store(t, acc, s, mbits);
            }
        }
        if constexpr (NBUF == 1) __syncthreads();    // everyone is done reading before the next group is staged
        if constexpr (NBUF == 2) buf ^= 1;
    }
}

// ---------------------------------------------------------------------------
// conv1 forward: uint8 observation [4][IN_H][IN_W] -> act1 [H1][W1][32] (84x84 -> 20x20), 8x8 stride 4,
// fused with the uint8 -> bf16 unpack (exact) and the 1/255 scale (fp32 epilogue).
// The sample is converted to a bf16 image in LDS once (each pixel is used by up
// to four windows); a 32-wide k-step is four rows (ky) of eight pixels (kx) of
// one input channel, so an activation fragment is 16 contiguous bytes of the
// image.  A wavefront keeps one 16-channel tile of W1 (hi and lo parts) in registers;
// the position tiles of a sample (25 at 84x84; the last one may be ragged) are dealt round-robin to the four
// wavefront pairs.  Three-product precision with an exact activation operand needs
// two MFMAs per fragment (W_hi x, W_lo x).
// The work of workgroup (block_x, block_y) of a grid with grid_y workgroups per sample range, in the caller's LDS
// buffer of conv1_fwd_lds_bytes<Geo>() bytes.
template <class Geo>
constexpr int conv1_fwd_lds_bytes() { return 4 * Geo::OBS_BYTES; }   // two bf16 images

// FULL: the lo part and the sign bits are always written (the gradient step's forward).  As a compile-time fact the
// stores are unconditional, and the compiler's count of memory operations behind the frame prefetch -- which sets how
// many of them may still be in flight when the prefetched frame is needed (s_waitcnt vmcnt counts in order) -- is the
// real one instead of the fewest over all branches.
template <class Geo, bool FULL = false>
__device__ __forceinline__ void conv1_fwd_resident_body(
    u32x4 *lds, int block_x, int block_y, int grid_y, const uint8_t *__restrict__ obs, const __bf16 *__restrict__ w,
    const __bf16 *__restrict__ w_lo, const float *__restrict__ bias, __bf16 *__restrict__ out,
    __bf16 *__restrict__ out_lo, uint8_t *__restrict__ mask_out, int B, int spw) {
    constexpr int IN_H = Geo::IN_H, IN_W = Geo::IN_W, W1 = Geo::W1, P1 = Geo::P1, OBS_BYTES = Geo::OBS_BYTES;
    static_assert(OBS_BYTES % 16 == 0, "a sample is copied in 16-byte words");
    constexpr int IMG_U4 = OBS_BYTES / 16;                           // sixteen-pixel groups (1764 at 84x84)
    constexpr int NL = (IMG_U4 + RES_THREADS - 1) / RES_THREADS;     // 4
    constexpr int KS = KW1 / 32;                                     // 8
    constexpr int NT = (P1 + 15) / 16;                               // position tiles (25 at 84x84, no remainder)
    constexpr bool RAGGED = P1 % 16 != 0;
    u32x4(*const s_img)[2 * IMG_U4] = reinterpret_cast<u32x4(*)[2 * IMG_U4]>(lds);   // bf16 [4][IN_H][IN_W], double buffered
    static_assert(sizeof(u32x4) * 4 * IMG_U4 == conv1_fwd_lds_bytes<Geo>() && conv1_fwd_lds_bytes<Geo>() <= 160 * 1024, "LDS budget");

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, lg = lane >> 4;
    const int s_begin = block_x * spw;
    const int s_end = s_begin + spw < B ? s_begin + spw : B;
    if (s_begin >= s_end) return;

    // wavefront w owns channel tile w & 1 and position tiles (w >> 1) + 4j
    const int ct = wave & 1, t0 = wave >> 1;
    bf16x8 wh[KS], wl[KS];
    const float4 bs = *reinterpret_cast<const float4 *>(bias + ct * 16 + 4 * lg);

    u32x4 rimg[NL];
    // One persistent pointer per load, advanced by a sample after each use: with addresses computed per sample the
    // temporaries were allocated in registers that the previous prefetch had filled, and the wait that protects them
    // (s_waitcnt vmcnt, in order) also waited for most of the stores of the sample before.
    const u32x4 *pimg[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int idx = tid + RES_THREADS * i;
        pimg[i] = reinterpret_cast<const u32x4 *>(obs + (size_t)s_begin * OBS_BYTES) + (idx < IMG_U4 ? idx : IMG_U4 - 1);
    }
    auto gload = [&](int) __attribute__((always_inline)) {      // samples in order, starting at s_begin
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            rimg[i] = *pimg[i];
            pimg[i] += IMG_U4;
        }
    };

    // activation fragments of position tile t: for each k-step, 16 bytes of the image (8 pixels of a row)
    auto frag_load = [&](const char *img, int t, u32x2 (&f)[2 * KS]) __attribute__((always_inline)) {
        int pos = t * 16 + li;
        if constexpr (RAGGED) pos = pos < P1 ? pos : P1 - 1;       // rows past the last position recompute it; never stored
        const int oy = pos / W1, ox = pos - oy * W1;
        const int base = ((S1 * oy + lg) * IN_W + S1 * ox) * 2;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int off = base + ((ks >> 1) * (IN_H * IN_W) + (ks & 1) * 4 * IN_W) * 2;
            f[2 * ks] = *reinterpret_cast<const u32x2 *>(img + off);
            f[2 * ks + 1] = *reinterpret_cast<const u32x2 *>(img + off + 8);
        }
    };
    auto unit = [&](int s, int t, const u32x2 (&f)[2 * KS]) __attribute__((always_inline)) {
        const int pos = t * 16 + li;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 b = as_bf16x8(u32x4{f[2 * ks].x, f[2 * ks].y, f[2 * ks + 1].x, f[2 * ks + 1].y});
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wl[ks], b, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[ks], b, acc, 0, 0, 0);
        }
        constexpr float sc = 1.0f / 255.0f;
        const float r0 = fmaxf(acc[0] * sc + bs.x, 0.f), r1 = fmaxf(acc[1] * sc + bs.y, 0.f);
        const float r2 = fmaxf(acc[2] * sc + bs.z, 0.f), r3 = fmaxf(acc[3] * sc + bs.w, 0.f);
        const size_t at = ((size_t)s * P1 + pos) * C1 + ct * 16;
        const bool live = !RAGGED || pos < P1;
        if (live) store_bf16x4_split(out, out_lo, at + 4 * lg, r0, r1, r2, r3, std::integral_constant<bool, FULL>());
        if (FULL || mask_out) {
            const uint32_t bits = sign_bits16(r0, r1, r2, r3, lg);     // all lanes take part
            if (lg == 0 && live) *reinterpret_cast<uint16_t *>(mask_out + (at >> 3)) = (uint16_t)bits;
        }
    };

    gload(s_begin);
    const size_t wrow = frag_base(ct, KW1, lane);   // after the first image loads: staging does not wait for the weights
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        wh[ks] = as_bf16x8(*reinterpret_cast<const u32x4 *>(w + wrow + FRAG_STEP * ks));
        wl[ks] = as_bf16x8(*reinterpret_cast<const u32x4 *>(w_lo + wrow + FRAG_STEP * ks));
    }
    wait_global_loads();
    int buf = 0;
    for (int s = s_begin; s < s_end; ++s) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int idx = tid + RES_THREADS * i;
            if (idx < IMG_U4) {
                s_img[buf][2 * idx] = u8x8_to_bf16x8(rimg[i].x, rimg[i].y);
                s_img[buf][2 * idx + 1] = u8x8_to_bf16x8(rimg[i].z, rimg[i].w);
            }
        }
        __syncthreads();
        if (s + 1 < s_end) gload(s + 1);
        const char *img = reinterpret_cast<const char *>(s_img[buf]);
        // The fragments of the next position tile are read from LDS while the MFMAs of the current one
        // run (two register sets, statically alternated).  Tiles t0 + 4j, j = 0..5, exist for every
        // wavefront; tile 24 (j = 6) only for t0 = 0.
        u32x2 fa[2 * KS], fb[2 * KS];
        if constexpr (NT != 25) {
            // any tile count: this wavefront's tiles t0, t0 + 4, ... in pairs, then the odd one
            const int nj = (NT - t0 + 3) / 4;
            frag_load(img, t0, fa);
            int j = 0;
#pragma unroll 1
            for (; j + 1 < nj; j += 2) {
                frag_load(img, t0 + 4 * (j + 1), fb);
                unit(s, t0 + 4 * j, fa);
                if (j + 2 < nj) frag_load(img, t0 + 4 * (j + 2), fa);
                unit(s, t0 + 4 * (j + 1), fb);
            }
            if (j < nj) unit(s, t0 + 4 * j, fa);
        } else if (grid_y == 1) {
            frag_load(img, t0, fa);
#pragma unroll
            for (int j = 0; j < 6; j += 2) {
                frag_load(img, t0 + 4 * (j + 1), fb);
                unit(s, t0 + 4 * j, fa);
                if (j + 2 < 6 || t0 == 0) frag_load(img, t0 + 4 * (j + 2), fa);
                unit(s, t0 + 4 * (j + 1), fb);
            }
            if (t0 == 0) unit(s, NT - 1, fa);
        } else {
            // small batches: three workgroups per sample, each taking one pair of this wavefront's tiles
            // (the last one also tile 24)
            const int j = 2 * block_y;
            const bool tail = j == 4 && t0 == 0;
            frag_load(img, t0 + 4 * j, fa);
            frag_load(img, t0 + 4 * (j + 1), fb);
            unit(s, t0 + 4 * j, fa);
            if (tail) frag_load(img, NT - 1, fa);
            unit(s, t0 + 4 * (j + 1), fb);
            if (tail) unit(s, NT - 1, fa);
        }
        buf ^= 1;
    }
}

template <class Geo>
__global__ __launch_bounds__(RES_THREADS) void conv1_fwd_resident_kernel(
    const uint8_t *__restrict__ obs, const __bf16 *__restrict__ w, const __bf16 *__restrict__ w_lo,
    const float *__restrict__ bias, __bf16 *__restrict__ out, __bf16 *__restrict__ out_lo,
    uint8_t *__restrict__ mask_out, int B, int spw) {
    __shared__ u32x4 lds[conv1_fwd_lds_bytes<Geo>() / 16];
    conv1_fwd_resident_body<Geo>(lds, blockIdx.x, blockIdx.y, gridDim.y, obs, w, w_lo, bias, out, out_lo, mask_out, B, spw);
}

// ---------------------------------------------------------------------------
// conv2 forward: act1 [20][20][32] -> act2 [9][9][64], 4x4 stride 2.  The LDS
// image keeps even and odd columns in separate planes so that the stride-2
// windows of neighbouring positions are neighbouring LDS pixels.
struct ResConv2Fwd {
    static constexpr int CI = C1, SRC_PIX = P1, P = P2, HO = H2, CO = C2, K = KW2, G = 1;
    static constexpr bool SPLIT = true, ZERO_FILL = false, PIPE = false;
    static constexpr int MASK_ELEMS = 0, NBUF = 1;
    // image rows 2r and 2r+1 form one block of four planes (row parity x column parity, 10 pixels each)
    // plus one pixel of padding: 41 pixels, so that the first position of an output row follows the
    // last of the row before at one pixel stride modulo 256 bytes
    static constexpr int PSB = C1 * 2 + 32, PAIR = 41, IMG = (H1 / 2) * PAIR * PSB;
    __device__ static constexpr int plane_pix(int y, int x) {
        return (y >> 1) * PAIR + (y & 1) * H1 + (x & 1) * (H1 / 2) + (x >> 1);
    }
    __device__ static constexpr int dst_off(int p) { return plane_pix(p / H1, p % H1) * PSB; }
    __device__ static constexpr int base_off(int pos) { return plane_pix(2 * (pos / H2), 2 * (pos % H2)) * PSB; }
    __device__ static constexpr int tap_off(int t) { return plane_pix(t / K2, t % K2) * PSB; }
    struct Args {
        const __bf16 *in, *in_lo, *w, *w_lo;
        const uint8_t *mask;
        const float *bias;
        __bf16 *out, *out_lo;
        uint8_t *mask_out;     // sign bits of the output for the backward pass, or null
        typedef float4 Lane;
        __device__ __forceinline__ Lane lane(int n) const { return *reinterpret_cast<const float4 *>(bias + n); }
        __device__ __forceinline__ void store(int s, int, int pos, int n, f32x4 v, const Lane &b,
                                              const uint8_t *) const {
            const float r0 = fmaxf(v[0] + b.x, 0.f), r1 = fmaxf(v[1] + b.y, 0.f), r2 = fmaxf(v[2] + b.z, 0.f),
                        r3 = fmaxf(v[3] + b.w, 0.f);
            const size_t at = ((size_t)s * P2 + pos) * C2 + n;
            store_bf16x4_split(out, out_lo, at, r0, r1, r2, r3);
            if (mask_out) {
                const int lg = (n >> 2) & 3;
                const uint32_t bits = sign_bits16(r0, r1, r2, r3, lg);
                if (lg == 0) *reinterpret_cast<uint16_t *>(mask_out + (at >> 3)) = (uint16_t)bits;
            }
        }
    };
};

// conv3 forward: act2 [9][9][64] -> act3 [7][7][64], 3x3 stride 1
struct ResConv3Fwd {
    static constexpr int CI = C2, SRC_PIX = P2, P = P3, HO = H3, CO = C3, K = KW3, G = 2;
    static constexpr bool SPLIT = true, ZERO_FILL = false, PIPE = false;
    static constexpr int MASK_ELEMS = 0, NBUF = 1;
    // 9 pixels of 160 bytes per row + 192 bytes: position (oy+1, 0) then follows (oy, 6) at one pixel
    // stride mod 256; the image is padded likewise for the step from sample g to g+1
    static constexpr int PSB = C2 * 2 + 32, ROWB = H2 * PSB + 192, IMG = H2 * ROWB + 64;
    __device__ static constexpr int dst_off(int p) { return (p / H2) * ROWB + (p % H2) * PSB; }
    __device__ static constexpr int base_off(int pos) { return (pos / H3) * ROWB + (pos % H3) * PSB; }
    __device__ static constexpr int tap_off(int t) { return (t / K3) * ROWB + (t % K3) * PSB; }
    struct Args {
        const __bf16 *in, *in_lo, *w, *w_lo;
        const uint8_t *mask;
        const float *bias;
        __bf16 *out, *out_lo;
        uint8_t *mask_out;     // sign bits of the output for the backward pass, or null
        typedef float4 Lane;
        __device__ __forceinline__ Lane lane(int n) const { return *reinterpret_cast<const float4 *>(bias + n); }
        __device__ __forceinline__ void store(int s, int, int pos, int n, f32x4 v, const Lane &b,
                                              const uint8_t *) const {
            const float r0 = fmaxf(v[0] + b.x, 0.f), r1 = fmaxf(v[1] + b.y, 0.f), r2 = fmaxf(v[2] + b.z, 0.f),
                        r3 = fmaxf(v[3] + b.w, 0.f);
            const size_t at = ((size_t)s * P3 + pos) * C3 + n;
            store_bf16x4_split(out, out_lo, at, r0, r1, r2, r3);
            if (mask_out) {
                const int lg = (n >> 2) & 3;
                const uint32_t bits = sign_bits16(r0, r1, r2, r3, lg);
                if (lg == 0) *reinterpret_cast<uint16_t *>(mask_out + (at >> 3)) = (uint16_t)bits;
            }
        }
    };
};

// conv3 input gradient: d(pre3) [7][7][64] zero-padded by 2 to 11x11, 3x3 taps
// (ty,tx) reading padded (y+ty, x+tx) against W3[co][ci][2-ty][2-tx]; output
// d(pre2) [9][9][64] masked by act2 > 0.
struct ResConv3Dgrad {
    static constexpr int PADW = H3 + 4;   // 11
    static constexpr int CI = C3, SRC_PIX = P3, P = P2, HO = H2, CO = C2, K = 9 * C3, G = 2;
    static constexpr bool SPLIT = false, ZERO_FILL = true, PIPE = true;
    static constexpr int MASK_ELEMS = P2 * C2, NBUF = 1;
    // row and image padding as in the forward kernels (9 positions per output row over 11-pixel rows)
    static constexpr int PSB = C3 * 2 + 32, ROWB = PADW * PSB + 192, IMG = 21664;
    __device__ static constexpr int dst_off(int p) { return (p / H3 + 2) * ROWB + (p % H3 + 2) * PSB; }
    __device__ static constexpr int base_off(int pos) { return (pos / H2) * ROWB + (pos % H2) * PSB; }
    __device__ static constexpr int tap_off(int t) { return (t / 3) * ROWB + (t % 3) * PSB; }
    struct Args {
        const __bf16 *in, *in_lo, *w, *w_lo;
        const uint8_t *mask;   // sign bits of act2
        __bf16 *out;
        struct Lane {};
        __device__ __forceinline__ Lane lane(int) const { return Lane{}; }
        __device__ __forceinline__ void store(int s, int g, int pos, int n, f32x4 v, const Lane &,
                                              const uint8_t *mbits) const {
            const int e = (g * P2 + pos) * C2 + n;
            const uint32_t m = (uint32_t)mbits[e >> 3] >> (e & 7);
            *reinterpret_cast<u32x2 *>(out + ((size_t)s * P2 + pos) * C2 + n) =
                pack_bf16x4(m & 1 ? v[0] : 0.f, m & 2 ? v[1] : 0.f, m & 4 ? v[2] : 0.f, m & 8 ? v[3] : 0.f);
        }
    };
};

// conv2 input gradient (stride 2): d(pre2) [9][9][64] zero-padded by 1 to 11x11.
// The four output phases (y%2, x%2) share their activation fragments, so they
// are the 4 x 32 "channels" of one 2x2 stride-1 convolution over the padded
// image with 10x10 positions (u,v); channel n = phase*32 + ci lands at act1
// pixel (2u + phase/2, 2v + phase%2).  This is the image description only: the kernel that uses it
// (conv1_bwd_fused_body) feeds d(pre1) straight into conv1's weight gradient, one sample per iteration.
struct ResConv2Dgrad {
    static constexpr int PADW = H2 + 2;   // 11
    static constexpr int CI = C2, SRC_PIX = P2, P = 100, HO = 10, CO = 4 * C1, K = 4 * C2, G = 1;
    static constexpr bool SPLIT = false, ZERO_FILL = true;
    // row padding as in the forward kernels (10 positions per output row over 11-pixel rows)
    static constexpr int PSB = C2 * 2 + 32, ROWB = PADW * PSB + 96, IMG = 20608;
    __device__ static constexpr int dst_off(int p) { return (p / H2 + 1) * ROWB + (p % H2 + 1) * PSB; }
    __device__ static constexpr int base_off(int pos) { return (pos / 10) * ROWB + (pos % 10) * PSB; }
    __device__ static constexpr int tap_off(int t) { return (t / 2) * ROWB + (t % 2) * PSB; }
    // act1 pixel that channel group `phase` of position pos lands on (always inside the map here)
    __device__ static constexpr int out_pixel(int pos, int phase) {
        return (2 * (pos / 10) + (phase >> 1)) * H1 + 2 * (pos % 10) + (phase & 1);
    }
};

// ---------------------------------------------------------------------------
// Input gradients for any geometry Geo (arn_layout.h), used by the padded 104x80 network.  Same kernel and the
// same LDS bank rule as above; the row and image padding that makes the fragment reads conflict free is
// computed from the map sizes.

constexpr int pad_to_step(int have, int want) { return (((want - have) % 256) + 256) % 256; }

// conv2 forward (4x4, stride 2, padding PAD2 > 0): act1 [H1][W1][32] with a zero border, act2 [H2][W2][64];
// three products.  As in ResConv2Fwd the bordered image keeps even and odd columns in separate planes (so that
// the stride-2 windows of neighbouring positions are neighbouring LDS pixels) and two image rows form one
// block of PAIR pixels; PAIR is the next size for which the first position of an output row follows the last
// of the row before at one pixel stride modulo 256 bytes.  The image (hi and lo) fills most of a CU's LDS, so
// one workgroup of eight wavefronts runs per CU.
template <class Geo>
struct ResConv2FwdGeo {
    static_assert(Geo::PAD2 > 0, "the unpadded case has a layout of its own (ResConv2Fwd)");
    static constexpr int PADH = Geo::H1 + 2 * Geo::PAD2, PADW = Geo::W1 + 2 * Geo::PAD2;
    static constexpr int EVENW = (PADW + 1) / 2;                       // pixels in the even-column plane of a row
    static constexpr int CI = C1, SRC_PIX = Geo::P1, P = Geo::P2, CO = C2, K = KW2, G = 1, WAVES = 8;
    static constexpr bool SPLIT = true, ZERO_FILL = true, PIPE = false;
    static constexpr int MASK_ELEMS = 0, NBUF = 1;
    static constexpr int PSB = C1 * 2 + 32;
    static constexpr int pair_pixels() {
        int p = 2 * PADW;
        while (((p - Geo::W2) * PSB) % 256 != 0) ++p;
        return p;
    }
    static constexpr int PAIR = pair_pixels(), IMG = ((PADH + 1) / 2) * PAIR * PSB;
    __device__ static constexpr int plane_pix(int y, int x) {
        return (y >> 1) * PAIR + (y & 1) * PADW + (x & 1) * EVENW + (x >> 1);
    }
    __device__ static constexpr int dst_off(int p) {
        return plane_pix(p / Geo::W1 + Geo::PAD2, p % Geo::W1 + Geo::PAD2) * PSB;
    }
    __device__ static constexpr int base_off(int pos) { return plane_pix(2 * (pos / Geo::W2), 2 * (pos % Geo::W2)) * PSB; }
    __device__ static constexpr int tap_off(int t) { return plane_pix(t / K2, t % K2) * PSB; }
    struct Args {
        const __bf16 *in, *in_lo, *w, *w_lo;
        const uint8_t *mask;
        const float *bias;
        __bf16 *out, *out_lo;
        uint8_t *mask_out;     // sign bits of the output for the backward pass, or null
        typedef float4 Lane;
        __device__ __forceinline__ Lane lane(int n) const { return *reinterpret_cast<const float4 *>(bias + n); }
        __device__ __forceinline__ void store(int s, int, int pos, int n, f32x4 v, const Lane &b,
                                              const uint8_t *) const {
            const float r0 = fmaxf(v[0] + b.x, 0.f), r1 = fmaxf(v[1] + b.y, 0.f), r2 = fmaxf(v[2] + b.z, 0.f),
                        r3 = fmaxf(v[3] + b.w, 0.f);
            const size_t at = ((size_t)s * Geo::P2 + pos) * C2 + n;
            store_bf16x4_split(out, out_lo, at, r0, r1, r2, r3);
            if (mask_out) {
                const int lg = (n >> 2) & 3;
                const uint32_t bits = sign_bits16(r0, r1, r2, r3, lg);
                if (lg == 0) *reinterpret_cast<uint16_t *>(mask_out + (at >> 3)) = (uint16_t)bits;
            }
        }
    };
};

// conv3 forward (3x3, stride 1, padding PAD3 > 0): act2 [H2][W2][64] with a zero border of PAD3 pixels,
// act3 [H3][W3][64]; three products.
template <class Geo>
struct ResConv3FwdGeo {
    static_assert(Geo::PAD3 > 0, "the unpadded case has a layout of its own (ResConv3Fwd)");
    static constexpr int PADH = Geo::H2 + 2 * Geo::PAD3, PADW = Geo::W2 + 2 * Geo::PAD3;
    static constexpr int CI = C2, SRC_PIX = Geo::P2, P = Geo::P3, CO = C3, K = KW3, G = 1;
    static constexpr bool SPLIT = true, ZERO_FILL = true, PIPE = false;
    static constexpr int MASK_ELEMS = 0, NBUF = 1;
    static constexpr int PSB = C2 * 2 + 32;
    static constexpr int ROWB = PADW * PSB + pad_to_step(PADW * PSB, Geo::W3 * PSB);
    static constexpr int IMG = PADH * ROWB;
    __device__ static constexpr int dst_off(int p) {
        return (p / Geo::W2 + Geo::PAD3) * ROWB + (p % Geo::W2 + Geo::PAD3) * PSB;
    }
    __device__ static constexpr int base_off(int pos) { return (pos / Geo::W3) * ROWB + (pos % Geo::W3) * PSB; }
    __device__ static constexpr int tap_off(int t) { return (t / K3) * ROWB + (t % K3) * PSB; }
    struct Args {
        const __bf16 *in, *in_lo, *w, *w_lo;
        const uint8_t *mask;
        const float *bias;
        __bf16 *out, *out_lo;
        uint8_t *mask_out;     // sign bits of the output for the backward pass, or null
        typedef float4 Lane;
        __device__ __forceinline__ Lane lane(int n) const { return *reinterpret_cast<const float4 *>(bias + n); }
        __device__ __forceinline__ void store(int s, int, int pos, int n, f32x4 v, const Lane &b,
                                              const uint8_t *) const {
            const float r0 = fmaxf(v[0] + b.x, 0.f), r1 = fmaxf(v[1] + b.y, 0.f), r2 = fmaxf(v[2] + b.z, 0.f),
                        r3 = fmaxf(v[3] + b.w, 0.f);
            const size_t at = ((size_t)s * Geo::P3 + pos) * C3 + n;
            store_bf16x4_split(out, out_lo, at, r0, r1, r2, r3);
            if (mask_out) {
                const int lg = (n >> 2) & 3;
                const uint32_t bits = sign_bits16(r0, r1, r2, r3, lg);
                if (lg == 0) *reinterpret_cast<uint16_t *>(mask_out + (at >> 3)) = (uint16_t)bits;
            }
        }
    };
};

// conv3 (3x3, stride 1, padding PAD3): d(pre3) [H3][W3][64] zero-padded by OFF = 2 - PAD3 on every side;
// tap (ty,tx) reads padded (y+ty, x+tx) against W3[co][ci][2-ty][2-tx]; output d(pre2) [H2][W2][64].
template <class Geo>
struct ResConv3DgradGeo {
    static constexpr int OFF = K3 - 1 - Geo::PAD3, PADH = Geo::H3 + 2 * OFF, PADW = Geo::W3 + 2 * OFF;
    static_assert(PADH - 2 == Geo::H2 && PADW - 2 == Geo::W2, "stride-1 3x3 correlation over the padded gradient");
    static constexpr int CI = C3, SRC_PIX = Geo::P3, P = Geo::P2, CO = C2, K = 9 * C3, G = 2;
    static constexpr bool SPLIT = false, ZERO_FILL = true, PIPE = true;
    static constexpr int MASK_ELEMS = Geo::P2 * C2, NBUF = 1;
    static constexpr int PSB = C3 * 2 + 32;
    // W2 positions per output row: the first position of the next row must follow at one pixel stride mod 256
    static constexpr int ROWB = PADW * PSB + pad_to_step(PADW * PSB, Geo::W2 * PSB);
    static constexpr int LAST = (Geo::H2 - 1) * ROWB + (Geo::W2 - 1) * PSB;
    static constexpr int IMG = PADH * ROWB + pad_to_step(PADH * ROWB, LAST + PSB);
    __device__ static constexpr int dst_off(int p) { return (p / Geo::W3 + OFF) * ROWB + (p % Geo::W3 + OFF) * PSB; }
    __device__ static constexpr int base_off(int pos) { return (pos / Geo::W2) * ROWB + (pos % Geo::W2) * PSB; }
    __device__ static constexpr int tap_off(int t) { return (t / 3) * ROWB + (t % 3) * PSB; }
    struct Args {
        const __bf16 *in, *in_lo, *w, *w_lo;
        const uint8_t *mask;   // sign bits of act2
        __bf16 *out;
        struct Lane {};
        __device__ __forceinline__ Lane lane(int) const { return Lane{}; }
        __device__ __forceinline__ void store(int s, int g, int pos, int n, f32x4 v, const Lane &,
                                              const uint8_t *mbits) const {
            const int e = (g * Geo::P2 + pos) * C2 + n;
            const uint32_t m = (uint32_t)mbits[e >> 3] >> (e & 7);
            *reinterpret_cast<u32x2 *>(out + ((size_t)s * Geo::P2 + pos) * C2 + n) =
                pack_bf16x4(m & 1 ? v[0] : 0.f, m & 2 ? v[1] : 0.f, m & 4 ? v[2] : 0.f, m & 8 ? v[3] : 0.f);
        }
    };
};

// conv2 (4x4, stride 2, padding PAD2): d(pre2) [H2][W2][64] zero-padded by 1.  In coordinates of the padded
// input, (y + PAD2, x + PAD2) = (2u + py, 2v + px); the four phases (py,px) share their fragments, so they are
// the 4 x 32 channels of one 2x2 stride-1 correlation over positions (u,v); channel n = phase*32 + ci lands at
// act1 pixel (2u + py - PAD2, 2v + px - PAD2) if that is inside the map.  Image description for
// conv1_bwd_fused_body, as ResConv2Dgrad.
template <class Geo>
struct ResConv2DgradGeo {
    static constexpr int U = ((Geo::H1 - 1 + Geo::PAD2) >> 1) + 1, V = ((Geo::W1 - 1 + Geo::PAD2) >> 1) + 1;
    static constexpr int PADH = Geo::H2 + 2, PADW = Geo::W2 + 2;
    static_assert(U <= PADH - 1 && V <= PADW - 1, "every 2x2 window lies inside the padded gradient");
    static constexpr int CI = C2, SRC_PIX = Geo::P2, P = U * V, CO = 4 * C1, K = 4 * C2, G = 1;
    static constexpr bool SPLIT = false, ZERO_FILL = true;
    static constexpr int PSB = C2 * 2 + 32;
    static constexpr int ROWB = PADW * PSB + pad_to_step(PADW * PSB, V * PSB);
    static constexpr int IMG = (PADH * ROWB + 15) / 16 * 16;
    __device__ static constexpr int dst_off(int p) { return (p / Geo::W2 + 1) * ROWB + (p % Geo::W2 + 1) * PSB; }
    __device__ static constexpr int base_off(int pos) { return (pos / V) * ROWB + (pos % V) * PSB; }
    __device__ static constexpr int tap_off(int t) { return (t / 2) * ROWB + (t % 2) * PSB; }
    // act1 pixel that channel group `phase` of position pos lands on, or -1 if that is outside the map
    __device__ static constexpr int out_pixel(int pos, int phase) {
        const int y = 2 * (pos / V) + (phase >> 1) - Geo::PAD2, x = 2 * (pos % V) + (phase & 1) - Geo::PAD2;
        return (unsigned)y < (unsigned)Geo::H1 && (unsigned)x < (unsigned)Geo::W1 ? y * Geo::W1 + x : -1;
    }
};

}  // namespace arn
