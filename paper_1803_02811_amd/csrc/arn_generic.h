// Convolution forward passes for any frame size and padding (template parameter G, a Geometry from
// arn_layout.h) as instances of the two contraction kernels in arn_gemm.h: the activation operand is
// gathered on the fly (implicit im2col) with zeros where a window reaches into the padding.  This is the
// path of the conv2 and conv3 forward passes of the appendix's own setting (104x80 frames, padding 1 on
// conv2 and conv3); everything else of that setting, and all of the 84x84 network, runs on the
// sample-resident kernels (arn_resident_conv.h, arn_resident.h).
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
    uint8_t *mask_out = nullptr;   // sign bits of the output (bit e&7 of byte e>>3, NHWC element e) for the backward pass, or null
    __device__ __forceinline__ typename Gather::Row row(int m, int) const { return this->row_at(m); }
    __device__ __forceinline__ u32x4 load(const typename Gather::Row &r, int k) const { return this->load_at(r, k); }
    __device__ __forceinline__ u32x4 load_lo(const typename Gather::Row &r, int k) const {
        return this->load_lo_at(r, k);
    }
    __device__ __forceinline__ const __bf16 *weights(int) const { return w; }
    __device__ __forceinline__ const __bf16 *weights_lo(int) const { return w_lo; }
    // called by all 64 lanes together: lanes l and l+32 hold channels n..n+3 and n+4..n+7 of the same position
    __device__ __forceinline__ void store(int m, int n, f32x4 v, int) const {
        const float4 b = *reinterpret_cast<const float4 *>(bias + n);
        const float r0 = fmaxf(v[0] + b.x, 0.f), r1 = fmaxf(v[1] + b.y, 0.f), r2 = fmaxf(v[2] + b.z, 0.f),
                    r3 = fmaxf(v[3] + b.w, 0.f);
        const bool live = m < this->M;
        if (mask_out) {
            const int half = (n >> 2) & 1;
            const uint32_t t = ((r0 > 0.f ? 1u : 0u) | (r1 > 0.f ? 2u : 0u) | (r2 > 0.f ? 4u : 0u) | (r3 > 0.f ? 8u : 0u))
                               << (4 * half);
            const auto both = __builtin_amdgcn_permlane32_swap(t, t, false, false);   // own nibble and the other lane's
            if (live && half == 0) mask_out[((size_t)m * COUT + n) >> 3] = (uint8_t)(both[0] | both[1]);
        }
        if (live) store_bf16x4_split(out, out_lo, (size_t)m * COUT + n, r0, r1, r2, r3);
    }
};
template <class G>
using Conv2FwdG = ConvFwdG<Conv2GatherG<G>, C2, KW2>;
template <class G>
using Conv3FwdG = ConvFwdG<Conv3GatherG<G>, C3, KW3>;

// --------------------------- input gradients ------------------------------
// (conv3 / conv2 input gradients: ResConv3DgradGeo / ResConv2DgradGeo in arn_resident_conv.h)

// --------------------------- weight gradients -----------------------------
// (conv1 weight gradient: conv1_wgrad_resident_kernel<G> in arn_resident.h)
// (conv2 / conv3 weight gradients: conv_wgrad_resident_kernel in arn_resident.h)

}  // namespace arn
