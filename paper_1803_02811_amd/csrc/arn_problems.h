// The layers of the Nature CNN written as instances of the two contraction
// kernels in arn_gemm.h: how each one gathers its activation operand, where its
// packed weights live and what its epilogue does.
//
// Activations are NHWC bf16: act1 [B,20,20,32], act2 [B,9,9,64], act3 [B,7,7,64]
// (= the fc input with index (y*7+x)*64 + c; the packed fc weights are permuted
// to match), h [B,512].  Gradients at pre-activations use the same layouts.
#pragma once
#include "arn_gemm.h"
#include "arn_layout.h"

namespace arn {

// ------------------------------ gathers ----------------------------------
// conv1: rows are output positions (n,oy,ox); k = ci*64 + ky*8 + kx indexes the
// uint8 observation window.  Pixels 0..255 are exact in bf16; the 1/255 scale
// is applied in fp32 by the epilogue.
struct ObsGather {
    const uint8_t *obs;
    int M;   // B*400
    struct Row {
        const uint8_t *base;
        bool ok;
    };
    __device__ __forceinline__ Row row_at(long m) const {
        Row r;
        r.ok = m < M;
        const int mm = r.ok ? (int)m : 0;
        const int n = mm / P1, rem = mm - n * P1, oy = rem / H1, ox = rem - oy * H1;
        r.base = obs + (size_t)n * OBS_BYTES + oy * (S1 * IN_W) + ox * S1;
        return r;
    }
    // Loads are unconditional (out-of-range rows read sample 0 and are zeroed
    // afterwards) so that several can be in flight at once.
    __device__ __forceinline__ u32x4 load_at(const Row &r, int k) const {
        const int ci = k >> 6, ky = (k >> 3) & 7;
        const uint32_t *q = reinterpret_cast<const uint32_t *>(r.base + ci * (IN_H * IN_W) + ky * IN_W);
        const uint32_t lo = q[0], hi = q[1];
        return keep_or_zero(u8x8_to_bf16x8(lo, hi), r.ok);
    }
};

// conv2 / conv3 forward: rows are output positions; k = (ky*KS + kx)*CIN + ci,
// so for fixed ky the KS*CIN values are contiguous in the NHWC input.
template <int CIN, int HIN, int KS, int STRIDE, int HOUT>
struct ConvGather {
    const __bf16 *in;
    long lo_off = 0;   // element distance from `in` to the low-part tensor (split precision only)
    int M;   // B*HOUT*HOUT
    struct Row {
        const __bf16 *base;
        bool ok;
    };
    __device__ __forceinline__ Row row_at(long m) const {
        Row r;
        r.ok = m < M;
        const int mm = r.ok ? (int)m : 0;
        const int n = mm / (HOUT * HOUT), rem = mm - n * (HOUT * HOUT), oy = rem / HOUT, ox = rem - oy * HOUT;
        r.base = in + ((size_t)(n * HIN + oy * STRIDE) * HIN + ox * STRIDE) * CIN;
        return r;
    }
    __device__ __forceinline__ u32x4 load_at(const Row &r, int k) const {
        constexpr int SEG = KS * CIN;
        const int ky = k / SEG, within = k - ky * SEG;
        const u32x4 v = *reinterpret_cast<const u32x4 *>(r.base + ky * (HIN * CIN) + within);
        return keep_or_zero(v, r.ok);
    }
    __device__ __forceinline__ u32x4 load_lo_at(const Row &r, int k) const {
        constexpr int SEG = KS * CIN;
        const int ky = k / SEG, within = k - ky * SEG;
        const u32x4 v = *reinterpret_cast<const u32x4 *>(r.base + lo_off + ky * (HIN * CIN) + within);
        return keep_or_zero(v, r.ok);
    }
};
typedef ConvGather<C1, H1, K2, S2, H2> Conv2Gather;
typedef ConvGather<C2, H2, K3, S3, H3> Conv3Gather;

// dense rows: act [M][K]
template <int K_>
struct DenseGather {
    const __bf16 *in;
    long lo_off = 0;
    int M;
    struct Row {
        const __bf16 *base;
        bool ok;
    };
    __device__ __forceinline__ Row row_at(long m) const {
        Row r;
        r.ok = m < M;
        r.base = in + (size_t)(r.ok ? m : 0) * K_;
        return r;
    }
    __device__ __forceinline__ u32x4 load_at(const Row &r, int k) const {
        const u32x4 v = *reinterpret_cast<const u32x4 *>(r.base + k);
        return keep_or_zero(v, r.ok);
    }
    __device__ __forceinline__ u32x4 load_lo_at(const Row &r, int k) const {
        const u32x4 v = *reinterpret_cast<const u32x4 *>(r.base + lo_off + k);
        return keep_or_zero(v, r.ok);
    }
};
// dense rows with a run-time row length (head gradients: K = padded head width)
struct DenseGatherRt {
    const __bf16 *in;
    int M, K;
    struct Row {
        const __bf16 *base;
        bool ok;
    };
    __device__ __forceinline__ Row row_at(long m) const {
        Row r;
        r.ok = m < M;
        r.base = in + (size_t)(r.ok ? m : 0) * K;
        return r;
    }
    __device__ __forceinline__ u32x4 load_at(const Row &r, int k) const {
        const u32x4 v = *reinterpret_cast<const u32x4 *>(r.base + k);
        return keep_or_zero(v, r.ok);
    }
};

// ------------------------------ forward ----------------------------------
struct Conv1Fwd : ObsGather {
    static constexpr int BM = 128, BN = 32, WAVES_N = 1, K = KW1;
    static constexpr bool ACT_LO = false;   // pixels are exact in bf16
    const __bf16 *w, *w_lo = nullptr;
    const float *bias;
    __bf16 *out, *out_lo = nullptr;
    __device__ __forceinline__ Row row(int m, int) const { return row_at(m); }
    __device__ __forceinline__ u32x4 load(const Row &r, int k) const { return load_at(r, k); }
    __device__ __forceinline__ u32x4 load_lo(const Row &, int) const { return zero_u4(); }
    __device__ __forceinline__ const __bf16 *weights(int) const { return w; }
    __device__ __forceinline__ const __bf16 *weights_lo(int) const { return w_lo; }
    __device__ __forceinline__ void store(int m, int n, f32x4 v, int) const {
        if (m >= M) return;
        const float4 b = *reinterpret_cast<const float4 *>(bias + n);
        constexpr float s = 1.0f / 255.0f;
        store_bf16x4_split(out, out_lo, (size_t)m * C1 + n, fmaxf(v[0] * s + b.x, 0.f), fmaxf(v[1] * s + b.y, 0.f),
                           fmaxf(v[2] * s + b.z, 0.f), fmaxf(v[3] * s + b.w, 0.f));
    }
};

template <class Gather, int COUT, int K_>
struct ConvFwd : Gather {
    static constexpr int BM = 128, BN = COUT, WAVES_N = 2, K = K_;
    static constexpr bool ACT_LO = true;
    const __bf16 *w, *w_lo = nullptr;
    const float *bias;
    __bf16 *out, *out_lo = nullptr;
    __device__ __forceinline__ typename Gather::Row row(int m, int) const { return this->row_at(m); }
    __device__ __forceinline__ u32x4 load(const typename Gather::Row &r, int k) const { return this->load_at(r, k); }
    __device__ __forceinline__ u32x4 load_lo(const typename Gather::Row &r, int k) const {
        return this->load_lo_at(r, k);
    }
    __device__ __forceinline__ const __bf16 *weights(int) const { return w; }
    __device__ __forceinline__ const __bf16 *weights_lo(int) const { return w_lo; }
    __device__ __forceinline__ void store(int m, int n, f32x4 v, int) const {
        if (m >= this->M) return;
        const float4 b = *reinterpret_cast<const float4 *>(bias + n);
        store_bf16x4_split(out, out_lo, (size_t)m * COUT + n, fmaxf(v[0] + b.x, 0.f), fmaxf(v[1] + b.y, 0.f),
                           fmaxf(v[2] + b.z, 0.f), fmaxf(v[3] + b.w, 0.f));
    }
};
typedef ConvFwd<Conv2Gather, C2, KW2> Conv2Fwd;
typedef ConvFwd<Conv3Gather, C3, KW3> Conv3Fwd;

// fc: h = relu(act3 Wfc^T + b).  With ksplit > 1 each blockIdx.z covers a range
// of k-tiles and writes an fp32 partial [z][M][512]; fc_finish_kernel adds the
// partials in z order and applies bias, ReLU and the hi/lo split.  With
// ksplit == 1 the epilogue does that directly.
struct FcFwd : DenseGather<FEAT> {
    static constexpr int BM = 128, BN = 128, WAVES_N = 2, K = FEAT, STAGES = 2;
    static constexpr bool ACT_LO = true;
    int ksplit;
    bool to_partial;     // write fp32 partial sums even with ksplit == 1 (the consumer finishes the layer)
    const __bf16 *w, *w_lo = nullptr;
    const float *bias;
    __bf16 *out, *out_lo = nullptr;
    float *partial;
    __device__ __forceinline__ Row row(int m, int) const { return row_at(m); }
    __device__ __forceinline__ u32x4 load(const Row &r, int k) const { return load_at(r, k); }
    __device__ __forceinline__ u32x4 load_lo(const Row &r, int k) const { return load_lo_at(r, k); }
    __device__ __forceinline__ const __bf16 *weights(int) const { return w; }
    __device__ __forceinline__ const __bf16 *weights_lo(int) const { return w_lo; }
    __device__ __forceinline__ void store(int m, int n, f32x4 v, int z) const {
        if (m >= M) return;
        if (to_partial) {
            *reinterpret_cast<float4 *>(partial + ((size_t)z * M + m) * HID + n) = make_float4(v[0], v[1], v[2], v[3]);
            return;
        }
        const float4 b = *reinterpret_cast<const float4 *>(bias + n);
        store_bf16x4_split(out, out_lo, (size_t)m * HID + n, fmaxf(v[0] + b.x, 0.f), fmaxf(v[1] + b.y, 0.f),
                           fmaxf(v[2] + b.z, 0.f), fmaxf(v[3] + b.w, 0.f));
    }
};

// heads: rows of the packed head matrix are the A policy rows then the value
// row (PV), or the A*atoms categorical rows (C51).
// PV: N = 32 columns, k cut into HEAD_KSPLIT ranges; fp32 partials [z][M][32]
// (bias and the split into logits / value are applied by the consumer).
struct HeadFwdPV : DenseGather<HID> {
    static constexpr int BM = 128, BN = 32, WAVES_N = 1, K = HID;
    static constexpr bool ACT_LO = true;
    int ksplit;
    const __bf16 *w, *w_lo = nullptr;
    float *partial;
    __device__ __forceinline__ Row row(int m, int) const { return row_at(m); }
    __device__ __forceinline__ u32x4 load(const Row &r, int k) const { return load_at(r, k); }
    __device__ __forceinline__ u32x4 load_lo(const Row &r, int k) const { return load_lo_at(r, k); }
    __device__ __forceinline__ const __bf16 *weights(int) const { return w; }
    __device__ __forceinline__ const __bf16 *weights_lo(int) const { return w_lo; }
    __device__ __forceinline__ void store(int m, int n, f32x4 v, int z) const {
        if (m >= M) return;
        *reinterpret_cast<float4 *>(partial + ((size_t)z * M + m) * 32 + n) = make_float4(v[0], v[1], v[2], v[3]);
    }
};
// C51: atom logits fp32 [M][A*atoms] with bias.
struct HeadFwdC51 : DenseGather<HID> {
    static constexpr int BM = 128, BN = 64, WAVES_N = 1, K = HID;
    static constexpr bool ACT_LO = true;
    const __bf16 *w, *w_lo = nullptr;
    const float *bias;
    float *z;       // [M][ZW]
    int ZW;         // A*atoms
    __device__ __forceinline__ Row row(int m, int) const { return row_at(m); }
    __device__ __forceinline__ u32x4 load(const Row &r, int k) const { return load_at(r, k); }
    __device__ __forceinline__ u32x4 load_lo(const Row &r, int k) const { return load_lo_at(r, k); }
    __device__ __forceinline__ const __bf16 *weights(int) const { return w; }
    __device__ __forceinline__ const __bf16 *weights_lo(int) const { return w_lo; }
    __device__ __forceinline__ void store(int m, int n, f32x4 v, int) const {
        if (m >= M) return;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int c = n + e;
            if (c < ZW) z[(size_t)m * ZW + c] = v[e] + bias[c];
        }
    }
};

// --------------------------- input gradients ------------------------------
// d(pre_fc) = (dz W_head) * [h > 0]; the contraction length is the padded head width
struct HeadDgrad : DenseGatherRt {
    static constexpr int BM = 64, BN = 64, WAVES_N = 2;
    const __bf16 *w;     // [512][K]
    const __bf16 *h;
    __bf16 *out;         // [M][512]
    __device__ __forceinline__ Row row(int m, int) const { return row_at(m); }
    __device__ __forceinline__ u32x4 load(const Row &r, int k) const { return load_at(r, k); }
    __device__ __forceinline__ const __bf16 *weights(int) const { return w; }
    __device__ __forceinline__ void store(int m, int n, f32x4 v, int) const {
        if (m >= M) return;
        const size_t at = (size_t)m * HID + n;
        const f32x4 a = unpack_bf16x4(*reinterpret_cast<const u32x2 *>(h + at));
        *reinterpret_cast<u32x2 *>(out + at) = pack_bf16x4(a[0] > 0.f ? v[0] : 0.f, a[1] > 0.f ? v[1] : 0.f,
                                                          a[2] > 0.f ? v[2] : 0.f, a[3] > 0.f ? v[3] : 0.f);
    }
};

// d(pre3) = (d(pre_fc) W_fc) * [act3 > 0]      [B][3136], NHWC index
struct FcDgrad : DenseGather<HID> {
    static constexpr int BM = 128, BN = 64, WAVES_N = 2, K = HID, STAGES = 2;
    const __bf16 *w;          // [3136][512]
    const uint8_t *maskbits;  // sign bits of act3, bit e&7 of byte e>>3 for element e = m*3136 + n
    __bf16 *out;
    __device__ __forceinline__ Row row(int m, int) const { return row_at(m); }
    __device__ __forceinline__ u32x4 load(const Row &r, int k) const { return load_at(r, k); }
    __device__ __forceinline__ const __bf16 *weights(int) const { return w; }
    __device__ __forceinline__ void store(int m, int n, f32x4 v, int) const {
        if (m >= M) return;
        const size_t at = (size_t)m * FEAT + n;
        const uint32_t mb = (uint32_t)maskbits[at >> 3] >> (at & 7);
        *reinterpret_cast<u32x2 *>(out + at) =
            pack_bf16x4(mb & 1 ? v[0] : 0.f, mb & 2 ? v[1] : 0.f, mb & 4 ? v[2] : 0.f, mb & 8 ? v[3] : 0.f);
    }
};

// conv3 input gradient as a gather: rows are act2 positions (n,y,x), k =
// (ty*3+tx)*64 + co reads d(pre3)[n, y-2+ty, x-2+tx, co] (zero outside the 7x7
// map) against W3[co][ci][2-ty][2-tx]; epilogue applies act2's ReLU mask.
struct Conv3Dgrad {
    static constexpr int BM = 128, BN = 64, WAVES_N = 2, K = 9 * C3;
    const __bf16 *dpre;  // d(pre3) [B,7,7,64]
    const __bf16 *w;     // [64 ci][9*64]
    const __bf16 *act;   // act2
    __bf16 *out;         // d(pre2) [B,9,9,64]
    int M;               // B*81
    struct Row {
        long base;
        int y, x;
        bool ok;
    };
    __device__ __forceinline__ Row row(int m, int) const {
        Row r;
        r.ok = m < M;
        const int mm = r.ok ? m : 0;
        const int n = mm / P2, rem = mm - n * P2;
        r.y = rem / H2;
        r.x = rem - r.y * H2;
        r.base = ((long)(n * H3 + r.y) * H3 + r.x) * C3;
        return r;
    }
    __device__ __forceinline__ u32x4 load(const Row &r, int k) const {
        const int tap = k >> 6, ty = tap / 3, tx = tap - ty * 3;
        const int sy = r.y - 2 + ty, sx = r.x - 2 + tx;
        const bool ok = r.ok && sy >= 0 && sy < H3 && sx >= 0 && sx < H3;
        const long at = ok ? r.base + ((ty - 2) * H3 + (tx - 2)) * C3 + (k & 63) : 0;   // clamp, load, then zero
        const u32x4 v = *reinterpret_cast<const u32x4 *>(dpre + at);
        return keep_or_zero(v, ok);
    }
    __device__ __forceinline__ const __bf16 *weights(int) const { return w; }
    __device__ __forceinline__ void store(int m, int n, f32x4 v, int) const {
        if (m >= M) return;
        const size_t at = (size_t)m * C2 + n;
        const f32x4 a = unpack_bf16x4(*reinterpret_cast<const u32x2 *>(act + at));
        *reinterpret_cast<u32x2 *>(out + at) = pack_bf16x4(a[0] > 0.f ? v[0] : 0.f, a[1] > 0.f ? v[1] : 0.f,
                                                          a[2] > 0.f ? v[2] : 0.f, a[3] > 0.f ? v[3] : 0.f);
    }
};

// conv2 input gradient (stride 2) as four phase problems, z = 2*py + px:
// rows are (n,u,v) with the act1 position (2u+py, 2v+px); k = (ty*2+tx)*64 + co
// reads d(pre2)[n, u-1+ty, v-1+tx, co] against W2[co][ci][py+2(1-ty)][px+2(1-tx)].
struct Conv2Dgrad {
    static constexpr int BM = 128, BN = 32, WAVES_N = 1, K = 4 * C2;
    const __bf16 *dpre;  // d(pre2) [B,9,9,64]
    const __bf16 *w;     // [4][32 ci][4*64]
    const __bf16 *act;   // act1
    __bf16 *out;         // d(pre1) [B,20,20,32]
    int M;               // B*100
    struct Row {
        long base;
        int u, v;
        bool ok;
    };
    __device__ __forceinline__ Row row(int m, int) const {
        Row r;
        r.ok = m < M;
        const int mm = r.ok ? m : 0;
        const int n = mm / 100, rem = mm - n * 100;
        r.u = rem / 10;
        r.v = rem - r.u * 10;
        r.base = ((long)(n * H2 + r.u) * H2 + r.v) * C2;
        return r;
    }
    __device__ __forceinline__ u32x4 load(const Row &r, int k) const {
        const int tap = k >> 6, ty = tap >> 1, tx = tap & 1;
        const int sy = r.u - 1 + ty, sx = r.v - 1 + tx;
        const bool ok = r.ok && sy >= 0 && sy < H2 && sx >= 0 && sx < H2;
        const long at = ok ? r.base + ((ty - 1) * H2 + (tx - 1)) * C2 + (k & 63) : 0;
        const u32x4 v = *reinterpret_cast<const u32x4 *>(dpre + at);
        return keep_or_zero(v, ok);
    }
    __device__ __forceinline__ const __bf16 *weights(int z) const { return w + (size_t)z * C1 * K; }
    __device__ __forceinline__ void store(int m, int n, f32x4 v, int z) const {
        if (m >= M) return;
        const int s = m / 100, rem = m - s * 100, u = rem / 10, vv = rem - u * 10;
        const int y = 2 * u + (z >> 1), x = 2 * vv + (z & 1);
        const size_t at = ((size_t)(s * H1 + y) * H1 + x) * C1 + n;
        const f32x4 a = unpack_bf16x4(*reinterpret_cast<const u32x2 *>(act + at));
        *reinterpret_cast<u32x2 *>(out + at) = pack_bf16x4(a[0] > 0.f ? v[0] : 0.f, a[1] > 0.f ? v[1] : 0.f,
                                                          a[2] > 0.f ? v[2] : 0.f, a[3] > 0.f ? v[3] : 0.f);
    }
};

// --------------------------- weight gradients -----------------------------
// part[n][k] = sum_m dY[m][n] act(m,k); dY is a dense [M][N1] bf16 matrix.
template <class Gather, int BN1_, int BK2_, int WAVES_X_, int N1_, int KP_>
struct Wgrad : Gather {
    static constexpr int BN1 = BN1_, BK2 = BK2_, WAVES_X = WAVES_X_, N1 = N1_, KP = KP_;
    const __bf16 *dy;
    __device__ __forceinline__ typename Gather::Row xrow(long m) const { return this->row_at(m); }
    __device__ __forceinline__ u32x4 loadx(const typename Gather::Row &r, int k) const { return this->load_at(r, k); }
    __device__ __forceinline__ u32x4 loady(long m, int n) const {
        return *reinterpret_cast<const u32x4 *>(dy + (size_t)m * N1 + n);
    }
};
typedef Wgrad<ObsGather, 32, 128, 4, C1, KW1> Conv1Wgrad;
typedef Wgrad<Conv2Gather, 64, 128, 4, C2, KW2> Conv2Wgrad;
typedef Wgrad<Conv3Gather, 64, 64, 2, C3, KW3> Conv3Wgrad;
typedef Wgrad<DenseGather<FEAT>, 128, 64, 2, HID, FEAT> FcWgrad;
// heads: N1 (padded head rows) is a run-time value
struct HeadWgrad : DenseGather<HID> {
    static constexpr int BN1 = 64, BK2 = 128, WAVES_X = 4, KP = HID;
    int N1;
    const __bf16 *dy;
    __device__ __forceinline__ Row xrow(long m) const { return row_at(m); }
    __device__ __forceinline__ u32x4 loadx(const Row &r, int k) const { return load_at(r, k); }
    __device__ __forceinline__ u32x4 loady(long m, int n) const {
        return *reinterpret_cast<const u32x4 *>(dy + (size_t)m * N1 + n);
    }
};

}  // namespace arn
