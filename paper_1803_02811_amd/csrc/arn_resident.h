// Weight gradient of conv2 / conv3 with a few samples' operands resident in LDS (a workgroup body, launched by
// conv_backward_kernel); conv1's weight gradient uses the same contraction inside conv1_bwd_fused_body.
//
// dW[co][k'] = sum over samples and output positions m of dY[m][co] * x(m,k').
// The contraction index m is the slow index of both operands in memory, so both
// MFMA fragments are taken with the transposing LDS read.  Unlike the generic
// gemm_tn_kernel no im2col tile is built: a sample's input (converted to bf16
// once) and its dY rows are copied to LDS with contiguous 16-byte loads, and the
// transposing reads address the overlapping windows inside that image directly.
// Each workgroup owns a fixed, contiguous range of samples and accumulates in
// registers; partial results go to part[workgroup][...] and are summed in
// workgroup order by conv_reduce_kernel, so dW is bit-reproducible.
#pragma once
#include <type_traits>

#include "arn_gemm.h"
#include "arn_layout.h"

namespace arn {

// two transposing 8-byte reads -> one MFMA fragment (k = rows a..a+3, b..b+3)
__device__ __forceinline__ bf16x8 tr_pair(const char *lds_base, int off_a, int off_b) {
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(lds_base + off_a));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(lds_base + off_b));
    s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
}

// conv2 / conv3: x = NHWC bf16 activations [HIN][WIN][CIN] of G samples per
// iteration (k' = (ky*KS + kx)*CIN + ci), dY = d(pre) rows [G*HOUT*WOUT][COUT].
// With PAD > 0 the LDS image of a sample has a zero border of PAD pixels (cleared once; only the
// interior is restaged), so windows that reach into the padding read zeros.
// WAVES_Y wavefronts split the COUT/32 row tiles, the others split the column tiles.
//
// LDS layout.  One transposing read takes, for each of four consecutive contraction rows m, 64 contiguous bytes
// (32 lanes x 8 bytes, two such reads per fragment).  It is free of bank conflicts when consecutive rows lie
// 64 bytes apart modulo 256 (measured on the dense weight-gradient kernel: conflict cycles 54 % of the LDS-active
// cycles with rows 16 bytes apart modulo 256, 33 % with 32, none with 64).  Hence
//   YS  dY row stride:      the smallest multiple of 16 >= 2 COUT that is 64 or 192 modulo 256;
//   PS  pixel stride of x:  the same with STRIDE * PS (consecutive output positions are STRIDE pixels apart);
//   RS  image row stride:   WP * PS plus a gap chosen so that the step from the last window of an output row to
//                           the first of the next is STRIDE * PS modulo 256 as well
// when that fits the 160 KB; otherwise (the padded 12x9 layer with four samples) the compact layout with
// 16 bytes of padding per pixel and row, which is conflict-free within 16 lanes only.
constexpr int CW_THREADS = 512;   // eight wavefronts, two per SIMD: one hides the other's LDS latency

constexpr int wgrad_stride_for(int data_bytes, int step) {   // smallest s >= data_bytes, multiple of 16, with step*s = 64 or 192 mod 256
    for (int s = data_bytes;; s += 16)
        if ((step * s) % 256 == 64 || (step * s) % 256 == 192) return s;
}
template <int CIN, int HIN, int WIN, int KS, int STRIDE, int PAD, int HOUT, int WOUT, int COUT, int G>
struct WgradLayout {
    static constexpr int P = HOUT * WOUT, R = G * P, KSTEPS = (R + 15) / 16, RPAD = KSTEPS * 16;
    static constexpr int HP = HIN + 2 * PAD, WP = WIN + 2 * PAD;
    static constexpr int PS_WIDE = wgrad_stride_for(CIN * 2, STRIDE), YS_WIDE = wgrad_stride_for(COUT * 2, 1);
    static constexpr int row_gap(int ps) {   // STRIDE * (WP * ps + gap - WOUT * ps) = 0 mod 256
        for (int g = 0;; g += 16)
            if ((STRIDE * ((WP - WOUT) * ps + g)) % 256 == 0) return g;
    }
    static constexpr int RS_WIDE = WP * PS_WIDE + row_gap(PS_WIDE);
    static constexpr int WIN_BYTES = (RPAD + 16) * 4;   // window-origin table, one step of look-ahead past the end
    static constexpr bool WIDE = G * HP * RS_WIDE + RPAD * YS_WIDE + WIN_BYTES <= 160 * 1024;
    static constexpr int PS = WIDE ? PS_WIDE : CIN * 2 + 16, YS = WIDE ? YS_WIDE : COUT * 2 + 16;
    static constexpr int RS = WIDE ? RS_WIDE : WP * PS;              // bytes per image row
    static constexpr int IMG = HP * RS;                              // bytes per sample image
    static constexpr int X_BYTES = G * IMG, Y_BYTES = RPAD * YS, BYTES = X_BYTES + Y_BYTES + WIN_BYTES;
    static_assert(PS % 16 == 0 && YS % 16 == 0 && RS % 16 == 0 && BYTES <= 160 * 1024, "LDS budget");
};

// LDS bytes of conv_wgrad_resident_body with the same parameters
template <int CIN, int HIN, int WIN, int KS, int STRIDE, int PAD, int HOUT, int WOUT, int COUT, int G>
constexpr int conv_wgrad_lds_bytes() {
    return WgradLayout<CIN, HIN, WIN, KS, STRIDE, PAD, HOUT, WOUT, COUT, G>::BYTES;
}

// The work of workgroup `block` (of 512 threads) in the caller's LDS buffer `lds`.
template <int CIN, int HIN, int WIN, int KS, int STRIDE, int PAD, int HOUT, int WOUT, int COUT, int G, int WAVES_Y>
__device__ __forceinline__ void conv_wgrad_resident_body(u32x4 *lds, int block, const __bf16 *__restrict__ x,
                                                         const __bf16 *__restrict__ dy, float *__restrict__ part, int B,
                                                         int spw) {
    typedef WgradLayout<CIN, HIN, WIN, KS, STRIDE, PAD, HOUT, WOUT, COUT, G> L;
    constexpr int PIX = HIN * WIN, P = L::P, KP = KS * KS * CIN;
    constexpr int PS = L::PS, YS = L::YS, RS = L::RS, IMG = L::IMG;
    constexpr int R = L::R, KSTEPS = L::KSTEPS, RPAD = L::RPAD;
    constexpr int XCH = CIN / 8, YCH = COUT / 8;                     // 16-byte chunks per pixel / per dY row
    constexpr int NXC = G * PIX * XCH, NYC = G * P * YCH;
    constexpr int NT = CW_THREADS;
    constexpr int NI = (NXC + NT - 1) / NT, ND = (NYC + NT - 1) / NT;
    constexpr int NY = COUT / 32, NX = KP / 32, WAVES_X = (NT / 64) / WAVES_Y;
    constexpr int TY = NY / WAVES_Y, TX = (NX + WAVES_X - 1) / WAVES_X;   // the last wavefront along x may own fewer column tiles
    static_assert(NY % WAVES_Y == 0, "tile split");
    static_assert(NT % YCH == 0 && (NT / YCH) * COUT * 4 <= L::Y_BYTES, "bias-gradient scratch");

    u32x4 *const s_x = lds;                              // G images of IMG bytes
    u32x4 *const s_dy = lds + L::X_BYTES / 16;           // [RPAD] rows of YS bytes

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wy = wave % WAVES_Y, wx = wave / WAVES_Y;
    const int s_begin = block * spw;
    const int s_end = s_begin + spw < B ? s_begin + spw : B;

    // rows R..RPAD of dY stay zero for the whole kernel, and so does the border of the images
    for (int i = tid; i < (RPAD - R) * YS / 16; i += NT) s_dy[R * YS / 16 + i] = zero_u4();
    if constexpr (PAD > 0)
        for (int i = tid; i < L::X_BYTES / 16; i += NT) s_x[i] = zero_u4();

    // Staging registers: the global loads of the next iteration's samples are in flight while one iteration
    // computes.  (A second set, two iterations ahead, was measured: no faster for conv2, and with conv3's 80
    // accumulator registers it spills.)
    u32x4 rxa[NI], rya[ND];
    // The G samples of an iteration are contiguous in memory, so chunk idx of the iteration is 16 idx bytes past
    // sample s: a wavefront-uniform base and one 32-bit offset per load (no per-load address registers).  Chunks of
    // samples at or beyond s_end are read from the last 16 bytes of sample s_end - 1 instead (in bounds) and are
    // zeroed on store.
    auto gload = [&](int s, u32x4 (&rx)[NI], u32x4 (&ry)[ND]) __attribute__((always_inline)) {
        const int live = s_end - s < G ? s_end - s : G;
        const char *xb = reinterpret_cast<const char *>(x + (size_t)s * PIX * CIN);
        const char *yb = reinterpret_cast<const char *>(dy + (size_t)s * P * COUT);
        const uint32_t xlim = (uint32_t)live * (PIX * CIN * 2) - 16, ylim = (uint32_t)live * (P * COUT * 2) - 16;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const uint32_t off = (uint32_t)(tid + NT * i) * 16;
            rx[i] = *reinterpret_cast<const u32x4 *>(xb + (off < xlim ? off : xlim));
        }
#pragma unroll
        for (int i = 0; i < ND; ++i) {
            const uint32_t off = (uint32_t)(tid + NT * i) * 16;
            ry[i] = *reinterpret_cast<const u32x4 *>(yb + (off < ylim ? off : ylim));
        }
    };

    f32x16 acc[TY][TX];
#pragma unroll
    for (int a = 0; a < TY; ++a)
#pragma unroll
        for (int b = 0; b < TX; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
    float bs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};   // bias gradient of the thread's eight dY channels (chunk tid % YCH)

    const int o = lane & 15, Gq = lane >> 4;
    const int row_in_step = 8 * (Gq >> 1) + (o >> 2);
    const int col_lane = (16 * (Gq & 1) + 4 * (o & 3)) * 2;         // byte offset of the lane's 4 columns in a 32-column tile
    char *const xl = reinterpret_cast<char *>(s_x);
    char *const yl = reinterpret_cast<char *>(s_dy);

    // byte offset in s_x of the window origin of contraction row m: does not depend on the sample, tabulated once
    // (padded rows: any in-range window, their dY is zero)
    int *const s_win = reinterpret_cast<int *>(lds + (L::X_BYTES + L::Y_BYTES) / 16);
    for (int m = tid; m < RPAD + 16; m += NT) {
        const int mm = m < R ? m : R - 1;
        const int g = mm / P, rem = mm - g * P, oy = rem / WOUT, ox = rem - oy * WOUT;
        s_win[m] = g * IMG + STRIDE * oy * RS + STRIDE * ox * PS;
    }

    // The contraction over the staged rows, 16 per step, for a wavefront that owns T column tiles (the last
    // wavefront along x may own fewer than TX: the tile count is a template argument so that the loop body has no
    // branches).  Rolling software pipeline with one set of fragment registers: as soon as the MFMAs on column
    // tile b of step ks are issued, the reads of tile b of step ks + 1 are issued into the same registers, so
    // every read has the other tiles' MFMAs to return behind; the dY fragments and the window origins run one
    // and two steps ahead in registers of their own.  LDS reads return in order.
    auto contract_rows = [&](auto tiles) __attribute__((always_inline)) {
        constexpr int T = decltype(tiles)::value;
        int toff[T];
#pragma unroll
        for (int b = 0; b < T; ++b) {
            const int k0 = (wx * TX + b) * 32, tap = k0 / CIN, ci0 = k0 - tap * CIN;
            const int ky = tap / KS, kx = tap - ky * KS;
            toff[b] = ky * RS + kx * PS + ci0 * 2 + col_lane;
        }
        const int ycol = wy * TY * 64 + col_lane;
        auto origins = [&](int ks, int &wa, int &wb) __attribute__((always_inline)) {
            wa = s_win[16 * ks + row_in_step];
            wb = s_win[16 * ks + row_in_step + 4];
        };
        auto fetch_y = [&](int ks, bf16x8 (&fy)[TY]) __attribute__((always_inline)) {
            const int ya = (16 * ks + row_in_step) * YS + ycol;
#pragma unroll
            for (int a = 0; a < TY; ++a) fy[a] = tr_pair(yl, ya + a * 64, ya + 4 * YS + a * 64);
        };
        bf16x8 fy[TY], fyn[TY], fx[T];
        int wa, wb, wan, wbn;       // origins of the step being fetched, and of the one after
        origins(0, wa, wb);
        origins(1, wan, wbn);
        fetch_y(0, fy);
#pragma unroll
        for (int b = 0; b < T; ++b) fx[b] = tr_pair(xl, wa + toff[b], wb + toff[b]);
        wa = wan, wb = wbn;
#pragma unroll 1
        for (int ks = 0; ks + 1 < KSTEPS; ++ks) {
            origins(ks + 2, wan, wbn);      // at most step KSTEPS: inside the table's look-ahead rows
            fetch_y(ks + 1, fyn);
#pragma unroll
            for (int b = 0; b < T; ++b) {
                __builtin_amdgcn_sched_barrier(0);   // keeps the compiler from gathering the reads behind the MFMAs
#pragma unroll
                for (int a = 0; a < TY; ++a)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fy[a], fx[b], acc[a][b], 0, 0, 0);
                fx[b] = tr_pair(xl, wa + toff[b], wb + toff[b]);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int a = 0; a < TY; ++a) fy[a] = fyn[a];
            wa = wan, wb = wbn;
        }
#pragma unroll
        for (int b = 0; b < T; ++b)
#pragma unroll
            for (int a = 0; a < TY; ++a)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fy[a], fx[b], acc[a][b], 0, 0, 0);
    };

    // one iteration: the staged registers of samples s .. s+G-1 go to LDS, they are refilled with the next
    // iteration's samples, then the contraction
    auto iteration = [&](int s, u32x4 (&rx)[NI], u32x4 (&ry)[ND]) __attribute__((always_inline)) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int idx = tid + NT * i;
            if (idx < NXC) {
                const int pix = idx / XCH, c = idx - pix * XCH;
                const int g = pix / PIX, rem = pix - g * PIX, yy = rem / WIN, xx = rem - yy * WIN;
                const bool live = s + g < s_end;
                *reinterpret_cast<u32x4 *>(xl + g * IMG + (yy + PAD) * RS + (xx + PAD) * PS + c * 16) =
                    live ? rx[i] : zero_u4();
            }
        }
#pragma unroll
        for (int i = 0; i < ND; ++i) {
            const int idx = tid + NT * i;
            if (idx < NYC) {
                const int row = idx / YCH, c = idx - row * YCH;
                const bool live = s + row / P < s_end;
                *reinterpret_cast<u32x4 *>(yl + row * YS + c * 16) = live ? ry[i] : zero_u4();
                if (live) {
                    const bf16x8 f = as_bf16x8(ry[i]);
#pragma unroll
                    for (int e = 0; e < 8; ++e) bs[e] += (float)f[e];
                }
            }
        }
        __syncthreads();
        if (s + G < s_end) gload(s + G, rx, ry);

        constexpr int T_LAST = NX - (WAVES_X - 1) * TX;
        static_assert(T_LAST >= 1 && T_LAST <= TX, "column tiles of the last wavefront");
        if (T_LAST == TX || wx < WAVES_X - 1) contract_rows(std::integral_constant<int, TX>());
        else contract_rows(std::integral_constant<int, T_LAST>());
    };
    if (s_begin < s_end) gload(s_begin, rxa, rya);
    for (int s = s_begin; s < s_end; s += G) iteration(s, rxa, rya);

    float *out = part + (size_t)block * (COUT * KP + COUT);
    const int fr = lane & 31, fg = lane >> 5;
#pragma unroll
    for (int a = 0; a < TY; ++a)
#pragma unroll
        for (int b = 0; b < TX; ++b) {
            if (wx * TX + b >= NX) break;
            const int k = (wx * TX + b) * 32 + fr;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int n = (wy * TY + a) * 32 + 8 * (r >> 2) + 4 * fg + (r & 3);
                out[(size_t)n * KP + k] = acc[a][b][r];
            }
        }
    __syncthreads();
    float *red = reinterpret_cast<float *>(s_dy);
#pragma unroll
    for (int e = 0; e < 8; ++e) red[(tid / YCH) * COUT + (tid % YCH) * 8 + e] = bs[e];
    __syncthreads();
    if (tid < COUT) {
        float t = red[tid];
        for (int g = 1; g < NT / YCH; ++g) t += red[g * COUT + tid];
        out[COUT * KP + tid] = t;
    }
}

}  // namespace arn
