// MFMA building blocks for gfx950: two workgroup-level contraction kernels that
// the dense layers (fc, categorical head) are instances of.
//
//   gemm_nt_kernel : out[m][n] = sum_k act(m,k) * W[n][k]
//       forward layers and input gradients.  `act` is gathered on the fly by the
//       problem struct; W is a packed bf16 matrix with k contiguous.
//   gemm_tn_kernel : out[n][k] = sum_m dY[m][n] * act(m,k)
//       weight gradients: the contraction runs over the batch/position index,
//       which is the slow index of both operands in memory, so fragments are
//       taken from LDS with the transposing read ds_read_b64_tr_b16.
//
// Both use v_mfma_f32_32x32x16_bf16 (fp32 accumulate), 4 (or, for the NT kernel, 8)
// wavefronts of 64 lanes, and 64-element k-tiles staged through LDS (optionally two
// stages in the NT kernel) with a register prefetch of the tile after next.
//
// MFMA operand layout used throughout (checked on hardware):
//   A (32 x 16): lane l holds row l%32,  k = 8*(l/32) .. +7
//   B (16 x 32): lane l holds col l%32,  k = 8*(l/32) .. +7
//   D (32 x 32): lane l holds col l%32,  rows 8*(r/4) + 4*(l/32) + r%4, r = 0..15
// The weights (or dY) go in as A and the activations as B, so a lane ends up
// with 4 consecutive channels of one position: one 8-byte NHWC store.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace arn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
// 16- and 8-byte register/LDS words as native vectors (plain loads and stores, kept in registers)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

constexpr int LDS_ROW = 9;   // u32x4 per staged row: 8 of data (64 bf16) + 1 of padding

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ f16x8 as_f16x8(u32x4 v) { return __builtin_bit_cast(f16x8, v); }

__device__ __forceinline__ u32x2 pack_bf16x4(float a, float b, float c, float d) {
    bf16x4 v = {(__bf16)a, (__bf16)b, (__bf16)c, (__bf16)d};
    return __builtin_bit_cast(u32x2, v);
}

// v -> (hi, lo) with hi = bf16(v), lo = bf16(v - hi)
template <bool ALWAYS_LO = false>
__device__ __forceinline__ void store_bf16x4_split(__bf16 *hi, __bf16 *lo, size_t at, float a, float b, float c,
                                                   float d, std::integral_constant<bool, ALWAYS_LO> = {}) {
    const bf16x4 h = {(__bf16)a, (__bf16)b, (__bf16)c, (__bf16)d};
    *reinterpret_cast<u32x2 *>(hi + at) = __builtin_bit_cast(u32x2, h);
    if (ALWAYS_LO || lo) {
        const bf16x4 l = {(__bf16)(a - (float)h[0]), (__bf16)(b - (float)h[1]), (__bf16)(c - (float)h[2]),
                          (__bf16)(d - (float)h[3])};
        *reinterpret_cast<u32x2 *>(lo + at) = __builtin_bit_cast(u32x2, l);
    }
}

// ReLU sign bits of a 16x16 MFMA tile: lane (li = l%16, lg = l/16) holds channels 4*lg..4*lg+3
// of position li; the four lanes of a position combine their nibbles into one 16-bit word
// (bit c = value of channel c > 0), valid in every participating lane.
__device__ __forceinline__ uint32_t sign_bits16(float a, float b, float c, float d, int lg) {
    uint32_t t = ((a > 0.f ? 1u : 0u) | (b > 0.f ? 2u : 0u) | (c > 0.f ? 4u : 0u) | (d > 0.f ? 8u : 0u)) << (4 * lg);
    // v_permlane16_swap / v_permlane32_swap (VALU, no LDS traffic): with both operands equal, the two
    // results are the lane's own value and that of the lane 16 (32) away (checked on hardware)
    const auto a16 = __builtin_amdgcn_permlane16_swap(t, t, false, false);
    t = a16[0] | a16[1];
    const auto a32 = __builtin_amdgcn_permlane32_swap(t, t, false, false);
    return a32[0] | a32[1];
}

__device__ __forceinline__ f32x4 unpack_bf16x4(u32x2 u) {
    bf16x4 v = __builtin_bit_cast(bf16x4, u);
    f32x4 r = {(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
    return r;
}

// eight uint8 (two little-endian words) -> eight bf16, exact
__device__ __forceinline__ u32x4 u8x8_to_bf16x8(uint32_t lo, uint32_t hi) {
    auto two = [](uint32_t b0, uint32_t b1) -> uint32_t {
        return (__float_as_uint((float)b0) >> 16) | (__float_as_uint((float)b1) & 0xffff0000u);
    };
    u32x4 r;
    r.x = two(lo & 0xff, (lo >> 8) & 0xff);
    r.y = two((lo >> 16) & 0xff, lo >> 24);
    r.z = two(hi & 0xff, (hi >> 8) & 0xff);
    r.w = two((hi >> 16) & 0xff, hi >> 24);
    return r;
}

// Weights that a wavefront keeps in registers as MFMA A-operand fragments (16 rows x 32 k) are packed in fragment
// order: the eight values of lane l for (16-row tile t, k-step ks) of a [rows][K] matrix are the 16 contiguous
// bytes at element ((t * K/32 + ks) * 64 + l) * 8.  A wavefront's load of one fragment is then one contiguous
// kilobyte; read from the row-major matrix it was sixteen 64-byte pieces a row apart, and a workgroup's
// 300 KB of such loads took 8 us before the first MFMA (measured).  frag_base + FRAG_STEP * ks addresses it.
constexpr int FRAG_STEP = 512;
__device__ __forceinline__ size_t frag_base(int tile, int K, int lane) { return (size_t)tile * K * 16 + (size_t)lane * 8; }
// the same index for the packing side: element (row, k) of the [rows][K] matrix
__host__ __device__ constexpr long frag_index(long row, long k, long K) {
    return ((row >> 4) * (K >> 5) + (k >> 5)) * 512 + ((((k & 31) >> 3) << 4) + (row & 15)) * 8 + (k & 7);
}

__device__ __forceinline__ u32x4 zero_u4() { return u32x4{0u, 0u, 0u, 0u}; }

// Waits until every global load of this wavefront has returned (s_waitcnt vmcnt(0), other counters unchanged).
// Kernels that keep weights in registers call it once after loading them: otherwise the compiler places the
// wait for those loads at their first use inside the sample loop, where it cannot tell them from the prefetch
// of the next sample issued just before -- and every iteration would wait for its own prefetch.
__device__ __forceinline__ void wait_global_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// v if keep else 0, through a mask the optimiser cannot see through: a gather
// written as `ok ? *p : 0` is compiled to a branch around the load with a wait
// right behind it, which serialises the loads of one k-tile.  With the mask the
// (always in-bounds, clamped) loads are issued back to back.  The mask is applied where
// the registers are written to LDS, not where they are loaded: applied at the load it sits
// in the same basic block as the prefetch, and the wavefront waits for the next tile's
// loads before it starts the MFMAs of the current one.
__device__ __forceinline__ u32x4 keep_or_zero(u32x4 v, bool keep) {
    uint32_t mask = keep ? 0xffffffffu : 0u;
    asm volatile("" : "+v"(mask));
    return u32x4{v.x & mask, v.y & mask, v.z & mask, v.w & mask};
}

// ---------------------------------------------------------------------------
// out[m][n] = sum_k act(m,k) W[n][k]
//
// Problem P supplies
//   BM, BN           workgroup tile (positions x channels), multiples of 32
//   WAVES_N          wavefronts along channels (1, 2 or 4)
//   K                contraction length, multiple of 64 (static or a data member)
//   Row row(m, z)    per-row gather state for position m (z = blockIdx.z)
//   u32x4 load(row, k)   eight bf16 of act(m, k..k+7); zeros where out of range
//   const __bf16* weights(z)   W, at least gridDim.y*BN rows of K
//   store(m, n, v, z)    epilogue for channels n..n+3 of position m
// Grid: x = position tiles, y = channel tiles, z = problem-defined.
//
// SPLIT = true is the three-product bf16 scheme used for action-selection
// inference: each operand is a pair (hi, lo) of bf16 with hi + lo carrying ~16
// mantissa bits, and the product is accumulated as hi*hi + lo_w*hi_a + hi_w*lo_a
// in fp32.  P then also supplies weights_lo(z), load_lo(row, k) and the flag
// ACT_LO (false when the activation operand is exact in one bf16, as for uint8
// pixels, which drops the third product).
// ---------------------------------------------------------------------------
template <class P, bool SPLIT>
struct ActLo {
    static constexpr bool value = false;
};
template <class P>
struct ActLo<P, true> {
    static constexpr bool value = P::ACT_LO;
};

// Problems with a data member `ksplit` cut the contraction into that many
// ranges of k-tiles, one per blockIdx.z; their store() receives z and writes a
// partial sum that a later kernel adds up in z order.
template <class P, class = void>
struct HasKSplit {
    static constexpr bool value = false;
};
template <class P>
struct HasKSplit<P, decltype((void)P::ksplit)> {
    static constexpr bool value = true;
};

// Problems with a static member STAGES = 2 double-buffer their LDS tiles (one
// barrier per k-tile, staging of the next tile overlaps the MFMAs); the default
// of one stage halves the LDS footprint, which matters more when several
// workgroups can share a CU.
template <class P, class = void>
struct StagesOf {
    static constexpr int value = 1;
};
template <class P>
struct StagesOf<P, decltype((void)P::STAGES)> {
    static constexpr int value = P::STAGES;
};

// Problems with a static member THREADS = 512 run eight wavefronts per workgroup (two per SIMD, so that one
// wavefront's LDS waits overlap the other's MFMAs); the default is 256.
template <class P, class = void>
struct ThreadsOf {
    static constexpr int value = 256;
};
template <class P>
struct ThreadsOf<P, decltype((void)P::THREADS)> {
    static constexpr int value = P::THREADS;
};
// Problems with a static member F16 = true hold fp16 operands (same 16-byte fragments, the fp16 MFMA): the single
// product of the forward passes that carry no gradient.
template <class P, class = void>
struct IsF16 {
    static constexpr bool value = false;
};
template <class P>
struct IsF16<P, decltype((void)P::F16)> {
    static constexpr bool value = P::F16;
};
// one 32x32x16 MFMA on fragments held as eight 16-bit lanes: bf16, or fp16 when F16
template <bool F16>
__device__ __forceinline__ f32x16 mfma_32x32x16(bf16x8 a, bf16x8 b, f32x16 c) {
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// Problems with a member function prefetch(m, n) have it called for every output quad before the k loop;
// its result (for example the ReLU-derivative bits of the quad) is handed to store(), which then needs no
// dependent load in the epilogue.
template <class P, class = void>
struct HasPrefetch {
    static constexpr bool value = false;
};
template <class P>
struct HasPrefetch<P, decltype((void)&P::prefetch)> {
    static constexpr bool value = true;
};

// Problems whose number of weight rows N_ROWS is not a multiple of BN: the last tile's rows past the end are read from
// the last row (and the problem's epilogue drops their columns).
template <class P, class = void>
struct WeightRows {
    static constexpr int value = 1 << 30;
};
template <class P>
struct WeightRows<P, decltype((void)P::N_ROWS)> {
    static constexpr int value = P::N_ROWS;
};

template <class P, bool SPLIT = false>
__global__ __launch_bounds__(ThreadsOf<P>::value) void gemm_nt_kernel(const P p) {
    constexpr int NT = ThreadsOf<P>::value, NW = NT / 64, RS = NT / 8;   // threads, wavefronts, rows staged per pass
    constexpr int BM = P::BM, BN = P::BN, WN = P::WAVES_N, WM = NW / WN;
    constexpr int TN = BN / (32 * WN), TM = BM / (32 * WM);
    constexpr int A_CH = BM / RS, W_CH = BN / RS;     // 16-byte chunks staged per thread and k-tile
    static_assert(BM % RS == 0 && BN % RS == 0, "staging passes");
    constexpr bool ALO = ActLo<P, SPLIT>::value;
    int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
    int kt_begin = 0, KT = p.K / 64;
    if constexpr (HasKSplit<P>::value) {
        // Split-k launches: workgroups go to the eight XCDs round robin in linear order (x fastest), and each XCD has
        // an L2 of its own.  With the plain mapping an XCD sees every k range of its position tiles and all of W;
        // remapped, an XCD works on one k range (or a few) of a band of position tiles, so what its L2 fetches from
        // memory is halved (measured: 77.2 -> 38.6 MB per launch of the fc layer at 2048 samples; the launch itself
        // 26.9 -> 26.5 us, 17.0 -> 15.2 us at 1024 samples).  Only for grids that split evenly; otherwise the plain
        // mapping.
        const int gx = gridDim.x, gy = gridDim.y, gz = gridDim.z;
        const bool pow2 = (gz & (gz - 1)) == 0;
        if (pow2 && gz >= 8) {
            const int L = bx + gx * (by + gy * bz), c = L & 7, zpc = gz >> 3;
            int r = L >> 3;
            bz = c * zpc + r % zpc;
            r /= zpc;
            bx = r % gx;
            by = r / gx;
        } else if (pow2 && gz > 1 && gx % (8 / gz) == 0) {
            const int L = bx + gx * (by + gy * bz), c = L & 7, g = 8 / gz, xs = gx / g, r = L >> 3;
            bz = c / g;
            bx = (c % g) * xs + r % xs;
            by = r / xs;
        }
        const int total = KT;
        kt_begin = bz * total / p.ksplit;
        KT = (bz + 1) * total / p.ksplit;
    }
    static_assert(TN >= 1 && TM >= 1, "tile shape");

    // with two LDS stages tile kt is consumed from stage kt&1 while tile kt+1 is written to the other
    constexpr int NST = StagesOf<P>::value;
    constexpr int SA = BM * LDS_ROW, SW = BN * LDS_ROW;
    __shared__ u32x4 sA[NST * SA];
    __shared__ u32x4 sW[NST * SW];
    __shared__ u32x4 sA2[ALO ? NST * SA : 1];
    __shared__ u32x4 sW2[SPLIT ? NST * SW : 1];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave % WN, wm = wave / WN;
    const int m0 = bx * BM, n0 = by * BN, z = bz;
    const int kc = tid & 7;      // which 16-byte chunk of the 128-byte k-tile row
    const int r0 = tid >> 3;     // first staged row; this thread also stages r0+RS, r0+2RS, ...

    typename P::Row rows[A_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) rows[i] = p.row(m0 + r0 + RS * i, z);
    const u32x4 *wsrc[W_CH];
    const u32x4 *wsrc2[W_CH];
#pragma unroll
    for (int i = 0; i < W_CH; ++i) {
        const int nrow = n0 + r0 + RS * i;
        const size_t at = (size_t)(nrow < WeightRows<P>::value ? nrow : WeightRows<P>::value - 1) * p.K;
        wsrc[i] = reinterpret_cast<const u32x4 *>(p.weights(z) + at) + kc;
        if constexpr (SPLIT) wsrc2[i] = reinterpret_cast<const u32x4 *>(p.weights_lo(z) + at) + kc;
    }

    u32x4 ra[A_CH], rw[W_CH], ra2[ALO ? A_CH : 1], rw2[SPLIT ? W_CH : 1];
    auto gload = [&](int kt) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            ra[i] = p.load(rows[i], kt * 64 + kc * 8);
            if constexpr (ALO) ra2[i] = p.load_lo(rows[i], kt * 64 + kc * 8);
        }
#pragma unroll
        for (int i = 0; i < W_CH; ++i) {
            rw[i] = wsrc[i][kt * 8];
            if constexpr (SPLIT) rw2[i] = wsrc2[i][kt * 8];
        }
    };

    f32x16 acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    auto stage = [&](int st) __attribute__((always_inline)) {   // registers -> LDS stage st
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {       // rows past M were read from row 0: zeroed here
            sA[st * SA + (r0 + RS * i) * LDS_ROW + kc] = keep_or_zero(ra[i], rows[i].ok);
            if constexpr (ALO) sA2[st * SA + (r0 + RS * i) * LDS_ROW + kc] = keep_or_zero(ra2[i], rows[i].ok);
        }
#pragma unroll
        for (int i = 0; i < W_CH; ++i) {
            sW[st * SW + (r0 + RS * i) * LDS_ROW + kc] = rw[i];
            if constexpr (SPLIT) sW2[st * SW + (r0 + RS * i) * LDS_ROW + kc] = rw2[i];
        }
    };

    const int fr = lane & 31, fg = lane >> 5;
    uint32_t pre[HasPrefetch<P>::value ? TN : 1][HasPrefetch<P>::value ? TM : 1][4];
    if constexpr (HasPrefetch<P>::value) {
#pragma unroll
        for (int a = 0; a < TN; ++a)
#pragma unroll
            for (int b = 0; b < TM; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    pre[a][b][q] = p.prefetch(m0 + (wm * TM + b) * 32 + fr, n0 + (wn * TN + a) * 32 + 8 * q + 4 * fg);
    }
    gload(kt_begin);
    stage(0);
    if (kt_begin + 1 < KT) gload(kt_begin + 1);
    __syncthreads();
    for (int kt = kt_begin; kt < KT; ++kt) {
        const int st = NST == 2 ? (kt - kt_begin) & 1 : 0;
        if constexpr (NST == 2) {
            // tile kt+1 (in registers since the previous iteration) goes to the free stage,
            // then the loads of tile kt+2 are issued; both overlap the MFMAs on tile kt
            if (kt + 1 < KT) stage(st ^ 1);
            if (kt + 2 < KT) gload(kt + 2);
        }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 fw[TN], fa[TM], fw2[SPLIT ? TN : 1], fa2[ALO ? TM : 1];
#pragma unroll
            for (int a = 0; a < TN; ++a) {
                const int at = st * SW + ((wn * TN + a) * 32 + fr) * LDS_ROW + kk * 2 + fg;
                fw[a] = as_bf16x8(sW[at]);
                if constexpr (SPLIT) fw2[a] = as_bf16x8(sW2[at]);
            }
#pragma unroll
            for (int b = 0; b < TM; ++b) {
                const int at = st * SA + ((wm * TM + b) * 32 + fr) * LDS_ROW + kk * 2 + fg;
                fa[b] = as_bf16x8(sA[at]);
                if constexpr (ALO) fa2[b] = as_bf16x8(sA2[at]);
            }
#pragma unroll
            for (int a = 0; a < TN; ++a)
#pragma unroll
                for (int b = 0; b < TM; ++b) {
                    if constexpr (SPLIT)
                        acc[a][b] = mfma_32x32x16<IsF16<P>::value>(fw2[a], fa[b], acc[a][b]);
                    if constexpr (ALO)
                        acc[a][b] = mfma_32x32x16<IsF16<P>::value>(fw[a], fa2[b], acc[a][b]);
                    acc[a][b] = mfma_32x32x16<IsF16<P>::value>(fw[a], fa[b], acc[a][b]);
                }
        }
        __syncthreads();
        if constexpr (NST == 1) {
            if (kt + 1 < KT) {
                stage(0);
                if (kt + 2 < KT) gload(kt + 2);
                __syncthreads();
            }
        }
    }

#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b) {
            const int m = m0 + (wm * TM + b) * 32 + fr;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + (wn * TN + a) * 32 + 8 * q + 4 * fg;
                f32x4 v = {acc[a][b][4 * q], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]};
                if constexpr (HasPrefetch<P>::value) p.store(m, n, v, z, pre[a][b][q]);
                else p.store(m, n, v, z);
            }
        }
}

// ---------------------------------------------------------------------------
// Transposing LDS fragment read.
//
// `tile` holds 64 rows (contraction index m) of `row_u4` u32x4 each, columns
// contiguous.  Returns, for MFMA lane l, the eight values
//   tile[mbase + 8*(l/32) + e][col0 + l%32],  e = 0..7
// i.e. an A- or B-operand fragment whose k index is the tile's row index.
// ds_read_b64_tr_b16 works on groups of 16 lanes: lane 4q+e of a group receives
// element e of the four 8-byte rows addressed by lanes q, q+4, q+8, q+12.
// ---------------------------------------------------------------------------
__device__ __forceinline__ bf16x8 tr_fragment(const u32x4 *tile, int row_u4, int mbase, int col0, int lane) {
    const int o = lane & 15, G = lane >> 4;
    const int row = mbase + 8 * (G >> 1) + (o >> 2);
    const int col = col0 + 16 * (G & 1) + 4 * (o & 3);
    const char *addr = reinterpret_cast<const char *>(tile) + (size_t)row * row_u4 * 16 + col * 2;
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(addr));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(addr + (size_t)4 * row_u4 * 16));
    s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
}

// ---------------------------------------------------------------------------
// part[split][n][k] = sum_{m in split} dY[m][n] * act(m,k)       (fp32)
// part[split][N1*KP + n] = sum_{m in split} dY[m][n]             (bias gradient)
//
// Problem P supplies
//   BN1, BK2         output tile (dY channels x act columns), multiples of 32
//   WAVES_X          wavefronts along act columns (1, 2 or 4)
//   N1, KP           full output shape (rows, columns; static or data members)
//   XRow xrow(m), u32x4 loadx(xrow, k)    gather of act(m, k..k+7)
//   u32x4 loady(m, n)                     eight bf16 of dY[m][n..n+7]
//   int M                                  number of contraction rows
// Grid: x = column tiles, y = row tiles, z = batch split.  Each split covers
// `rows_per_split` (a multiple of 64) consecutive m; partials are summed by
// reduce_partials_kernel in split order, which fixes the rounding order.
// ---------------------------------------------------------------------------
template <class P>
__global__ __launch_bounds__(256) void gemm_tn_kernel(const P p, float *__restrict__ part, int rows_per_split) {
    constexpr int BN1 = P::BN1, BK2 = P::BK2, WX = P::WAVES_X, WY = 4 / WX;
    constexpr int TY = BN1 / (32 * WY), TX = BK2 / (32 * WX);
    constexpr int YC = BN1 / 8, XC = BK2 / 8;          // 16-byte chunks per staged row
    // Padding of a staged row: 64 bytes, which puts consecutive rows 64 bytes apart modulo 256 (rows are multiples of
    // 128 bytes).  A transposing read takes 64 contiguous bytes of each of four consecutive rows: with 16 bytes of
    // padding 54 % of the LDS-active cycles were bank conflicts, with 32 bytes 33 %, with 64 none (measured).
    constexpr int TN_PAD = 4;
    constexpr int YROW = YC + TN_PAD, XROW = XC + TN_PAD;        // padded LDS row, in u32x4
    static_assert(YC % 8 == 0 && XC % 8 == 0, "rows of whole 128 bytes");
    constexpr int Y_CH = 64 * YC / 256, X_CH = 64 * XC / 256;
    static_assert(TY >= 1 && TX >= 1 && Y_CH >= 1 && X_CH >= 1, "tile shape");
    constexpr int BIAS_SCRATCH = (256 / YC) * BN1 * 4;   // bytes: one partial bias sum per thread and column
    constexpr bool SCRATCH_IN_Y = BIAS_SCRATCH <= 64 * YROW * 16;
    static_assert(256 % YC == 0 && (SCRATCH_IN_Y || BIAS_SCRATCH <= 64 * XROW * 16), "bias-gradient scratch");

    __shared__ u32x4 sY[64 * YROW];
    __shared__ u32x4 sX[64 * XROW];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wx = wave % WX, wy = wave / WX;
    const int x0 = blockIdx.x * BK2, y0 = blockIdx.y * BN1, split = blockIdx.z;
    const long m_begin = (long)split * rows_per_split;
    long m_end = m_begin + rows_per_split;
    if (m_end > p.M) m_end = p.M;

    u32x4 ry[Y_CH], rx[X_CH];
    auto gload = [&](long mt) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < Y_CH; ++i) {
            const int c = tid + 256 * i, r = c / YC, cc = c % YC;
            const long m = mt + r;
            ry[i] = p.loady(m < m_end ? m : m_begin, y0 + cc * 8);   // clamped; zeroed when staged
        }
#pragma unroll
        for (int i = 0; i < X_CH; ++i) {
            const int c = tid + 256 * i, r = c / XC, cc = c % XC;
            const long m = mt + r;
            rx[i] = p.loadx(p.xrow(m < m_end ? m : m_begin), x0 + cc * 8);
        }
    };

    f32x16 acc[TY][TX];
#pragma unroll
    for (int a = 0; a < TY; ++a)
#pragma unroll
        for (int b = 0; b < TX; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
    // bias gradient (column sums of dY), kept by the workgroups of the first tile column: a thread always
    // stages the same eight dY columns (256 is a multiple of YC), so it adds what it stages, in fp32
    float bs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const bool keeps_bias = blockIdx.x == 0;

    if (m_begin < m_end) gload(m_begin);
    for (long mt = m_begin; mt < m_end; mt += 64) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < Y_CH; ++i) {
            const int c = tid + 256 * i;
            const u32x4 v = keep_or_zero(ry[i], mt + c / YC < m_end);   // rows past the end of the range: zero
            sY[(c / YC) * YROW + c % YC] = v;
            if (keeps_bias) {
                const bf16x8 f = as_bf16x8(v);
#pragma unroll
                for (int e = 0; e < 8; ++e) bs[e] += (float)f[e];
            }
        }
#pragma unroll
        for (int i = 0; i < X_CH; ++i) {
            const int c = tid + 256 * i;
            sX[(c / XC) * XROW + c % XC] = keep_or_zero(rx[i], mt + c / XC < m_end);
        }
        __syncthreads();
        if (mt + 64 < m_end) gload(mt + 64);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 fy[TY], fx[TX];
#pragma unroll
            for (int a = 0; a < TY; ++a) fy[a] = tr_fragment(sY, YROW, kk * 16, (wy * TY + a) * 32, lane);
#pragma unroll
            for (int b = 0; b < TX; ++b) fx[b] = tr_fragment(sX, XROW, kk * 16, (wx * TX + b) * 32, lane);
#pragma unroll
            for (int a = 0; a < TY; ++a)
#pragma unroll
                for (int b = 0; b < TX; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fy[a], fx[b], acc[a][b], 0, 0, 0);
        }
    }

    float *out = part + (size_t)split * ((size_t)p.N1 * p.KP + p.N1);
    const int fr = lane & 31, fg = lane >> 5;
#pragma unroll
    for (int a = 0; a < TY; ++a)
#pragma unroll
        for (int b = 0; b < TX; ++b) {
            const int k = x0 + (wx * TX + b) * 32 + fr;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int n = y0 + (wy * TY + a) * 32 + 8 * (r >> 2) + 4 * fg + (r & 3);
                out[(size_t)n * p.KP + k] = acc[a][b][r];
            }
        }
    if (keeps_bias) {
        // the 256/YC threads that share a column add their sums in thread order
        __syncthreads();
        float *scr = reinterpret_cast<float *>(SCRATCH_IN_Y ? sY : sX);
#pragma unroll
        for (int e = 0; e < 8; ++e) scr[(tid / YC) * BN1 + (tid % YC) * 8 + e] = bs[e];
        __syncthreads();
        if (tid < BN1) {
            float t = scr[tid];
            for (int g = 1; g < 256 / YC; ++g) t += scr[g * BN1 + tid];
            out[(size_t)p.N1 * p.KP + y0 + tid] = t;
        }
    }
}

}  // namespace arn
