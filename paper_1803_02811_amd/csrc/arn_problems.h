// The dense layers of the Nature CNN (fc and heads) written as instances of the two
// contraction kernels in arn_gemm.h: how each one gathers its activation operand,
// where its packed weights live and what its epilogue does.  (The convolutions have
// their own sample-resident kernels in arn_resident_conv.h / arn_resident.h.)
//
// Activations are NHWC bf16: act1 [B,20,20,32], act2 [B,9,9,64], act3 [B,7,7,64]
// (= the fc input with index (y*7+x)*64 + c; the packed fc weights are permuted
// to match), h [B,512]; with the 104x80 geometry [B,25,19,32], [B,12,9,64], [B,12,9,64].
// Gradients at pre-activations use the same layouts.  The fc problems are templates on
// the fc input size (3136 or 6912).
#pragma once
#include "arn_gemm.h"
#include "arn_layout.h"

namespace arn {

// ------------------------------ gathers ----------------------------------
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
    // rows past M read row 0 (in bounds); the kernels zero them when they stage the registers into LDS
    __device__ __forceinline__ u32x4 load_at(const Row &r, int k) const {
        return *reinterpret_cast<const u32x4 *>(r.base + k);
    }
    __device__ __forceinline__ u32x4 load_lo_at(const Row &r, int k) const {
        return *reinterpret_cast<const u32x4 *>(r.base + lo_off + k);
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
        return *reinterpret_cast<const u32x4 *>(r.base + k);
    }
};


// fc: h = relu(act3 Wfc^T + b).  With ksplit > 1 each blockIdx.z covers a range
// of k-tiles and writes an fp32 partial [z][M][512]; fc_finish_kernel adds the
// partials in z order and applies bias, ReLU and the hi/lo split.  With
// ksplit == 1 the epilogue does that directly.
template <int FEAT_>
struct FcFwdT : DenseGather<FEAT_> {
    typedef typename DenseGather<FEAT_>::Row Row;
    static constexpr int BM = 128, BN = 128, WAVES_N = 2, K = FEAT_, STAGES = 2, THREADS = 512;
    static constexpr bool ACT_LO = true;
    int ksplit;
    bool to_partial;     // write fp32 partial sums even with ksplit == 1 (the consumer finishes the layer)
    const __bf16 *w, *w_lo = nullptr;
    const float *bias;
    __bf16 *out, *out_lo = nullptr;
    float *partial;
    __device__ __forceinline__ Row row(int m, int) const { return this->row_at(m); }
    __device__ __forceinline__ u32x4 load(const Row &r, int k) const { return this->load_at(r, k); }
    __device__ __forceinline__ u32x4 load_lo(const Row &r, int k) const { return this->load_lo_at(r, k); }
    __device__ __forceinline__ const __bf16 *weights(int) const { return w; }
    __device__ __forceinline__ const __bf16 *weights_lo(int) const { return w_lo; }
    __device__ __forceinline__ void store(int m, int n, f32x4 v, int z) const {
        const int M = this->M;
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
typedef FcFwdT<FEAT> FcFwd;
// The same layer with fp16 activations and weights in one product (no-gradient forward): `in` and `w` point at
// fp16 data of the same layouts; the outputs are the fp32 partial sums or the (hi, lo) bf16 hidden layer as above.
template <int FEAT_>
struct FcFwdF16T : FcFwdT<FEAT_> {
    static constexpr bool F16 = true;
};

// categorical head: rows of the packed head matrix are the A*atoms categorical rows
// C51: atom logits fp32 [M][ZS] with bias; ZS = ZW (dense, the inference output) or the padded head width
// (the gradient step's own buffers: 16-byte stores).
struct HeadFwdC51 : DenseGather<HID> {
    static constexpr int BM = 128, BN = 64, WAVES_N = 1, K = HID;
    static constexpr bool ACT_LO = true;
    const __bf16 *w, *w_lo = nullptr;
    const float *bias;   // padded head width entries (zeros past ZW)
    float *z;       // [M][ZS]
    int ZW;         // A*atoms
    int ZS;         // row stride in floats: ZW, or a multiple of 64 >= ZW
    __device__ __forceinline__ Row row(int m, int) const { return row_at(m); }
    __device__ __forceinline__ u32x4 load(const Row &r, int k) const { return load_at(r, k); }
    __device__ __forceinline__ u32x4 load_lo(const Row &r, int k) const { return load_lo_at(r, k); }
    __device__ __forceinline__ const __bf16 *weights(int) const { return w; }
    __device__ __forceinline__ const __bf16 *weights_lo(int) const { return w_lo; }
    __device__ __forceinline__ void store(int m, int n, f32x4 v, int) const {
        if (m >= M) return;
        const float4 b = *reinterpret_cast<const float4 *>(bias + n);
        float *dst = z + (size_t)m * ZS + n;
        if (ZS != ZW) {                        // padded rows: every column exists
            *reinterpret_cast<float4 *>(dst) = make_float4(v[0] + b.x, v[1] + b.y, v[2] + b.z, v[3] + b.w);
        } else if ((ZW & 1) == 0) {            // dense rows of even length: n and m*ZW are even, 8-byte stores
            if (n + 1 < ZW) *reinterpret_cast<float2 *>(dst) = make_float2(v[0] + b.x, v[1] + b.y);
            if (n + 3 < ZW) *reinterpret_cast<float2 *>(dst + 2) = make_float2(v[2] + b.z, v[3] + b.w);
        } else {
            const float r[4] = {v[0] + b.x, v[1] + b.y, v[2] + b.z, v[3] + b.w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (n + e < ZW) dst[e] = r[e];
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

// d(pre3) = (d(pre_fc) W_fc) * [act3 > 0]      [B][FEAT], NHWC index.  BN_ = 64, or 128 for large batches (a third
// less operand traffic from the L2 per flop; FEAT need not be a multiple of it: N_ROWS).
template <int FEAT_, int BN_ = 64>
struct FcDgradT : DenseGather<HID> {
    static constexpr int BM = 128, BN = BN_, WAVES_N = 2, K = HID, STAGES = 1, FEAT = FEAT_, N_ROWS = FEAT_;
    const __bf16 *w;          // [FEAT][512]
    const uint8_t *maskbits;  // sign bits of act3, bit e&7 of byte e>>3 for element e = m*FEAT + n
    __bf16 *out;
    __device__ __forceinline__ Row row(int m, int) const { return row_at(m); }
    __device__ __forceinline__ u32x4 load(const Row &r, int k) const { return load_at(r, k); }
    __device__ __forceinline__ const __bf16 *weights(int) const { return w; }
    // the four ReLU-derivative bits of output quad (m, n..n+3), fetched before the k loop
    __device__ __forceinline__ uint32_t prefetch(int m, int n) const {
        const size_t at = (size_t)(m < M ? m : 0) * FEAT + (n < FEAT ? n : 0);
        return (uint32_t)maskbits[at >> 3] >> (at & 7);
    }
    __device__ __forceinline__ void store(int m, int n, f32x4 v, int, uint32_t mb) const {
        if (m >= M || n >= FEAT) return;
        const size_t at = (size_t)m * FEAT + n;
        *reinterpret_cast<u32x2 *>(out + at) =
            pack_bf16x4(mb & 1 ? v[0] : 0.f, mb & 2 ? v[1] : 0.f, mb & 4 ? v[2] : 0.f, mb & 8 ? v[3] : 0.f);
    }
};
typedef FcDgradT<FEAT> FcDgrad;

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
