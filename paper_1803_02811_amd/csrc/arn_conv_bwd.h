// The convolutions' backward pass below d(pre3) and d(pre2) in one launch.
//
// Once conv3's input gradient has produced d(pre2), three pieces of work are independent of each other: conv2's
// input gradient with conv1's weight gradient (conv1_bwd_fused_body), conv2's weight gradient and conv3's weight
// gradient (conv_wgrad_resident_body).  Each wants one 512-thread workgroup per CU at a time, so as separate
// kernels they ran one after the other, each with its own ramp-up and drain; here they are three ranges of
// workgroups of one grid, longest first, and a CU picks up a workgroup of the next range as soon as its
// workgroup of the previous one is done.  The LDS buffer is shared (sized for the largest of the three).
#pragma once
#include "arn_conv1_bwd.h"
#include "arn_resident.h"

namespace arn {

struct ConvBackwardArgs {
    // conv2 input gradient + conv1 weight gradient
    const uint8_t *obs;
    const __bf16 *dp2, *w2d;
    const uint8_t *mask1;
    float *part1;
    // conv2 weight gradient (x = act1, dY = d(pre2)), conv3 weight gradient (x = act2, dY = d(pre3))
    const __bf16 *a1, *a2, *dp3;
    float *part2, *part3;
    int B;
    int n1, n2;               // workgroups of the first two ranges (the third is the rest of the grid)
    int spw1, spw2, spw3;     // samples per workgroup of each range
};

template <class Geo, class D2>
struct ConvBackward {
    static_assert(C1B_THREADS == CW_THREADS, "one block size for all three ranges");
    static constexpr int THREADS = C1B_THREADS;
    static constexpr int L1 = conv1_bwd_lds_bytes<Geo, D2>();
    static constexpr int L2 = conv_wgrad_lds_bytes<C1, Geo::H1, Geo::W1, K2, S2, Geo::PAD2, Geo::H2, Geo::W2, C2, CONV2_WG_G>();
    static constexpr int L3 = conv_wgrad_lds_bytes<C2, Geo::H2, Geo::W2, K3, S3, Geo::PAD3, Geo::H3, Geo::W3, C3, CONV3_WG_G>();
    static constexpr int L12 = L1 > L2 ? L1 : L2;
    static constexpr int LDS_BYTES = ((L12 > L3 ? L12 : L3) + 15) / 16 * 16;
};

template <class Geo, class D2>
__global__ __launch_bounds__(C1B_THREADS) void conv_backward_kernel(const ConvBackwardArgs a) {
    __shared__ u32x4 lds[ConvBackward<Geo, D2>::LDS_BYTES / 16];
    const int b = blockIdx.x;
    if (b < a.n1) {
        conv1_bwd_fused_body<Geo, D2>(lds, b, a.obs, a.dp2, a.w2d, a.mask1, a.part1, a.B, a.spw1);
    } else if (b < a.n1 + a.n2) {
        conv_wgrad_resident_body<C1, Geo::H1, Geo::W1, K2, S2, Geo::PAD2, Geo::H2, Geo::W2, C2, CONV2_WG_G, 2>(
            lds, b - a.n1, a.a1, a.dp2, a.part2, a.B, a.spw2);
    } else {
        conv_wgrad_resident_body<C2, Geo::H2, Geo::W2, K3, S3, Geo::PAD3, Geo::H3, Geo::W3, C3, CONV3_WG_G, 2>(
            lds, b - a.n1 - a.n2, a.a2, a.dp3, a.part3, a.B, a.spw3);
    }
}

}  // namespace arn
