// The convolution layers for any frame size and padding (template parameter G, a Geometry from
// arn_layout.h) as instances of the two contraction kernels in arn_gemm.h: the activation operand is
// gathered on the fly (implicit im2col) with zeros where a window reaches into the padding.  This is the
// path of the appendix's own setting (104x80 frames, padding 1 on conv2 and conv3) for the forward
// convolutions and the weight gradients; the 84x84 network has sample-resident kernels of its own
// (arn_resident_conv.h, arn_resident.h) and does not come through here.
//
// Activations are NHWC bf16: act1 [B,H1,W1,32], act2 [B,H2,W2,64], act3 [B,H3,W3,64] (= the fc input with
// index (y*W3+x)*64 + c; the packed fc weights are permuted to match).  Gradients at pre-activations use
// the same layouts.  Packed weight layouts are those of the 84x84 path (they do not depend on G).
#pragma once
#include "arn_gemm.h"
#include "arn_layout.h"
#include "arn_problems.h"

namespace arn {

// ------------------------------ gathers ----------------------------------
// conv1: rows are output positions (n,oy,ox); k = ci*64 + ky*8 + kx indexes the uint8 observation window
// (no padding).  Pixels 0..255 are exact in bf16; the 1/255 scale is applied in fp32 by the epilogue.
template <class G>
struct ObsGatherG {
    static_assert(G::IN_W % 4 == 0, "window rows are read as aligned 32-bit words");
    const uint8_t *obs;
    int M;   // B * P1
    struct Row {
        const uint8_t *base;
        bool ok;
    };
    __device__ __forceinline__ Row row_at(long m) const {
        Row r;
        r.ok = m < M;
        const int mm = r.ok ? (int)m : 0;
        const int n = mm / G::P1, rem = mm - n * G::P1, oy = rem / G::W1, ox = rem - oy * G::W1;
        r.base = obs + (size_t)n * G::OBS_BYTES + oy * (S1 * G::IN_W) + ox * S1;
        return r;
    }
    // Loads are unconditional (out-of-range rows read sample 0 and are zeroed afterwards) so that several
    // can be in flight at once.
    __device__ __forceinline__ u32x4 load_at(const Row &r, int k) const {
        const int ci = k >> 6, ky = (k >> 3) & 7;
        const uint32_t *q = reinterpret_cast<const uint32_t *>(r.base + ci * (G::IN_H * G::IN_W) + ky * G::IN_W);
        const uint32_t lo = q[0], hi = q[1];
        return keep_or_zero(u8x8_to_bf16x8(lo, hi), r.ok);
    }
};

// conv2 / conv3: rows are output positions; k = (ky*KS + kx)*CIN + ci.  A 16-byte chunk is eight channels
// of one tap, so it is either wholly inside the input or wholly in the padding.
template <int CIN, int HIN, int WIN, int KS, int STRIDE, int PAD, int HOUT, int WOUT>
struct ConvGatherG {
    const __bf16 *in;
    long lo_off = 0;   // element distance from `in` to the low-part tensor (three-product forward only)
    int M;             // B * HOUT * WOUT
    struct Row {
        long base;     // element offset of tap (0,0); may point into the padding (never dereferenced there)
        int y0, x0;
        bool ok;
    };
    __device__ __forceinline__ Row row_at(long m) const {
        Row r;
        r.ok = m < M;
        const int mm = r.ok ? (int)m : 0;
        const int n = mm / (HOUT * WOUT), rem = mm - n * (HOUT * WOUT), oy = rem / WOUT, ox = rem - oy * WOUT;
        r.y0 = oy * STRIDE - PAD;
        r.x0 = ox * STRIDE - PAD;
        r.base = (((long)n * HIN + r.y0) * WIN + r.x0) * CIN;
        return r;
    }
    __device__ __forceinline__ long at(const Row &r, int k, bool &ok) const {
        const int tap = k / CIN, ci0 = k - tap * CIN, ky = tap / KS, kx = tap - ky * KS;
        ok = r.ok && (unsigned)(r.y0 + ky) < (unsigned)HIN && (unsigned)(r.x0 + kx) < (unsigned)WIN;
        return ok ? r.base + (ky * WIN + kx) * CIN + ci0 : 0;   // clamp, load, then zero
    }
    __device__ __forceinline__ u32x4 load_at(const Row &r, int k) const {
        bool ok;
        const long a = at(r, k, ok);
        return keep_or_zero(*reinterpret_cast<const u32x4 *>(in + a), ok);
    }
    __device__ __forceinline__ u32x4 load_lo_at(const Row &r, int k) const {
        bool ok;
        const long a = at(r, k, ok);
        return keep_or_zero(*reinterpret_cast<const u32x4 *>(in + lo_off + a), ok);
    }
};
template <class G>
using Conv2GatherG = ConvGatherG<C1, G::H1, G::W1, K2, S2, G::PAD2, G::H2, G::W2>;
template <class G>
using Conv3GatherG = ConvGatherG<C2, G::H2, G::W2, K3, S3, G::PAD3, G::H3, G::W3>;

// ------------------------------ forward ----------------------------------
// (conv1 forward: conv1_fwd_resident_kernel<G> in arn_resident_conv.h)

template <class Gather, int COUT, int K_>
struct ConvFwdG : Gather {
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
template <class G>
using Conv2FwdG = ConvFwdG<Conv2GatherG<G>, C2, KW2>;
template <class G>
using Conv3FwdG = ConvFwdG<Conv3GatherG<G>, C3, KW3>;

// --------------------------- input gradients ------------------------------
// ReLU derivative taken from the stored activation (act > 0  <=>  pre > 0)
__device__ __forceinline__ void store_masked_by_act(__bf16 *out, const __bf16 *act, size_t at, f32x4 v) {
    const f32x4 a = unpack_bf16x4(*reinterpret_cast<const u32x2 *>(act + at));
    *reinterpret_cast<u32x2 *>(out + at) = pack_bf16x4(a[0] > 0.f ? v[0] : 0.f, a[1] > 0.f ? v[1] : 0.f,
                                                      a[2] > 0.f ? v[2] : 0.f, a[3] > 0.f ? v[3] : 0.f);
}

// d(pre3) = (d(pre_fc) W_fc) * [act3 > 0]      [B][FEAT], NHWC index
template <int FEAT_>
struct FcDgradAct : DenseGather<HID> {
    static constexpr int BM = 128, BN = 64, WAVES_N = 2, K = HID, STAGES = 2;
    const __bf16 *w;     // [FEAT][512]
    const __bf16 *act;   // act3
    __bf16 *out;
    __device__ __forceinline__ Row row(int m, int) const { return row_at(m); }
    __device__ __forceinline__ u32x4 load(const Row &r, int k) const { return load_at(r, k); }
    __device__ __forceinline__ const __bf16 *weights(int) const { return w; }
    __device__ __forceinline__ void store(int m, int n, f32x4 v, int) const {
        if (m >= M) return;
        store_masked_by_act(out, act, (size_t)m * FEAT_ + n, v);
    }
};

// (conv3 / conv2 input gradients: ResConv3DgradGeo / ResConv2DgradGeo in arn_resident_conv.h)

// --------------------------- weight gradients -----------------------------
// (conv1 weight gradient: conv1_wgrad_resident_kernel<G> in arn_resident.h)
// (conv2 / conv3 weight gradients: conv_wgrad_resident_kernel in arn_resident.h)

}  // namespace arn
