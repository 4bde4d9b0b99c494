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
// LDS pixels and dY rows are padded (PS, YS bytes) so that the four rows touched
// by one transposing read fall into different banks.  WAVES_Y wavefronts split
// the COUT/32 row tiles, the others split the column tiles.
constexpr int CW_THREADS = 512;   // eight wavefronts, two per SIMD: one hides the other's LDS latency

// LDS bytes of conv_wgrad_resident_body with the same parameters
template <int CIN, int HIN, int WIN, int KS, int STRIDE, int PAD, int HOUT, int WOUT, int COUT, int G>
constexpr int conv_wgrad_lds_bytes() {
    constexpr int RPAD = (G * HOUT * WOUT + 15) / 16 * 16;
    return G * (HIN + 2 * PAD) * (WIN + 2 * PAD) * (CIN * 2 + 16) + RPAD * (COUT * 2 + 16) + RPAD * 4;
}

// The work of workgroup `block` (of 512 threads) in the caller's LDS buffer `lds`.
template <int CIN, int HIN, int WIN, int KS, int STRIDE, int PAD, int HOUT, int WOUT, int COUT, int G, int WAVES_Y>
__device__ __forceinline__ void conv_wgrad_resident_body(u32x4 *lds, int block, const __bf16 *__restrict__ x,
                                                         const __bf16 *__restrict__ dy, float *__restrict__ part, int B,
                                                         int spw) {
    constexpr int PIX = HIN * WIN, P = HOUT * WOUT, KP = KS * KS * CIN;
    constexpr int HP = HIN + 2 * PAD, WP = WIN + 2 * PAD, PIXP = HP * WP;   // LDS image with its zero border
    constexpr int PS = CIN * 2 + 16, YS = COUT * 2 + 16;            // padded strides in bytes
    constexpr int R = G * P, KSTEPS = (R + 15) / 16, RPAD = KSTEPS * 16;
    constexpr int XCH = CIN / 8, YCH = COUT / 8;                     // 16-byte chunks per pixel / per dY row
    constexpr int NXC = G * PIX * XCH, NYC = G * P * YCH;
    constexpr int NT = CW_THREADS;
    constexpr int NI = (NXC + NT - 1) / NT, ND = (NYC + NT - 1) / NT;
    constexpr int NY = COUT / 32, NX = KP / 32, WAVES_X = (NT / 64) / WAVES_Y;
    constexpr int TY = NY / WAVES_Y, TX = (NX + WAVES_X - 1) / WAVES_X;   // the last wavefront along x may own fewer column tiles
    static_assert(NY % WAVES_Y == 0, "tile split");
    static_assert(NT % YCH == 0 && (NT / YCH) * COUT * 4 <= RPAD * YS, "bias-gradient scratch");
    static_assert((G * PIXP * PS) % 16 == 0 && (RPAD * YS) % 16 == 0, "16-byte aligned LDS regions");
    static_assert(conv_wgrad_lds_bytes<CIN, HIN, WIN, KS, STRIDE, PAD, HOUT, WOUT, COUT, G>() == G * PIXP * PS + RPAD * YS + RPAD * 4 &&
                      G * PIXP * PS + RPAD * YS + RPAD * 4 <= 160 * 1024, "LDS budget");

    u32x4 *const s_x = lds;                              // [G * PIXP] pixels of PS bytes
    u32x4 *const s_dy = lds + G * PIXP * PS / 16;        // [RPAD] rows of YS bytes
    int *const s_win = reinterpret_cast<int *>(lds + (G * PIXP * PS + RPAD * YS) / 16);   // [RPAD]: byte offset of the window origin of contraction row m in s_x

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wy = wave % WAVES_Y, wx = wave / WAVES_Y;
    const int s_begin = block * spw;
    const int s_end = s_begin + spw < B ? s_begin + spw : B;

    // window origins do not depend on the sample: tabulated once instead of two divisions per row and k-step
    for (int m = tid; m < RPAD; m += NT) {
        const int mm = m < R ? m : R - 1;                    // padded rows: any in-range window (their dY is zero)
        const int g = mm / P, rem = mm - g * P, oy = rem / WOUT, ox = rem - oy * WOUT;
        s_win[m] = (g * PIXP + STRIDE * oy * WP + STRIDE * ox) * PS;
    }
    // rows R..RPAD of dY stay zero for the whole kernel, and so does the border of the images
    for (int i = tid; i < (RPAD - R) * YS / 16; i += NT) s_dy[R * YS / 16 + i] = zero_u4();
    if constexpr (PAD > 0)
        for (int i = tid; i < G * PIXP * PS / 16; i += NT) s_x[i] = zero_u4();

    u32x4 rx[NI], ry[ND];
    auto gload = [&](int s) __attribute__((always_inline)) {   // samples s .. s+G-1; those at or beyond s_end are read from s_end-1 and zeroed on store
        const int last = s_end - 1;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            int idx = tid + NT * i;
            idx = idx < NXC ? idx : NXC - 1;
            const int g = idx / (PIX * XCH), rem = idx - g * (PIX * XCH);
            const int sg = s + g < s_end ? s + g : last;
            rx[i] = reinterpret_cast<const u32x4 *>(x + (size_t)sg * PIX * CIN)[rem];
        }
#pragma unroll
        for (int i = 0; i < ND; ++i) {
            int idx = tid + NT * i;
            idx = idx < NYC ? idx : NYC - 1;
            const int g = idx / (P * YCH), rem = idx - g * (P * YCH);
            const int sg = s + g < s_end ? s + g : last;
            ry[i] = reinterpret_cast<const u32x4 *>(dy + (size_t)sg * P * COUT)[rem];
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

    if (s_begin < s_end) gload(s_begin);
    for (int s = s_begin; s < s_end; s += G) {
        __syncthreads();
        char *xl = reinterpret_cast<char *>(s_x);
        char *yl = reinterpret_cast<char *>(s_dy);
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int idx = tid + NT * i;
            if (idx < NXC) {
                const int pix = idx / XCH, c = idx - pix * XCH;
                const int g = pix / PIX, rem = pix - g * PIX, yy = rem / WIN, xx = rem - yy * WIN;
                const bool live = s + g < s_end;
                *reinterpret_cast<u32x4 *>(xl + (g * PIXP + (yy + PAD) * WP + xx + PAD) * PS + c * 16) =
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
        if (s + G < s_end) gload(s + G);

#pragma unroll 1
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const int ma = 16 * ks + row_in_step, mb = ma + 4;
            const int base[2] = {s_win[ma] + col_lane, s_win[mb] + col_lane};   // window origins in the bordered image
            bf16x8 fy[TY];
#pragma unroll
            for (int a = 0; a < TY; ++a) {
                const int c0 = (wy * TY + a) * 64 + col_lane;
                fy[a] = tr_pair(yl, ma * YS + c0, mb * YS + c0);
            }
#pragma unroll
            for (int b = 0; b < TX; ++b) {
                if (wx * TX + b >= NX) break;                // wavefront-uniform
                const int k0 = (wx * TX + b) * 32, tap = k0 / CIN, ci0 = k0 - tap * CIN;
                const int ky = tap / KS, kx = tap - ky * KS;
                const int toff = (ky * WP + kx) * PS + ci0 * 2;
                const bf16x8 fx = tr_pair(xl, base[0] + toff, base[1] + toff);
#pragma unroll
                for (int a = 0; a < TY; ++a)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fy[a], fx, acc[a][b], 0, 0, 0);
            }
        }
    }

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
