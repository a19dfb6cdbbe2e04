// Pieces shared by the attention code of the phase kernels and of the stream
// kernel: how a wavefront maps onto cache positions, and the lane reductions.
#pragma once
#include <type_traits>
#include "device_utils.h"

namespace cfpp {

template <int D> struct AttnShape {
    static constexpr int LPP = D >= 128 ? 4 : 2;
    static constexpr int PPW = 64 / LPP;
    static constexpr int NP = D / 8 / LPP;     // pieces per lane
    static constexpr int NV = NP * 8;          // accumulators per lane
    // values a lane still holds after the butterfly reduce-scatter over positions
    static constexpr int NLEFT = LPP == 2 ? (((((NV + 1) / 2 + 1) / 2 + 1) / 2 + 1) / 2 + 1) / 2
                                          : ((((NV + 1) / 2 + 1) / 2 + 1) / 2 + 1) / 2;
};

template <int M>
__device__ __forceinline__ float lane_xor(float v)
{
    if constexpr (M == 1) return dpp_mov<kDppXor1>(v);
    else if constexpr (M == 2) return dpp_mov<kDppXor2>(v);
    else return __shfl_xor(v, M, 64);
}

// Butterfly reduce-scatter of vals[0..NV) over the lanes that differ in the bits
// M0, 2*M0, ..., 32: at each step a lane keeps one half of its list and adds
// the partner's copy of it.  On return the lane holds `cnt` finished sums, for
// original indices off .. off+cnt-1, in vals[0..cnt).
template <int NV, int M0>
__device__ __forceinline__ void reduce_scatter(float (&vals)[NV], int lane, int &off, int &cnt)
{
    off = 0;
    cnt = NV;
    auto step = [&](auto mtag, auto ntag) {
        constexpr int M = decltype(mtag)::value, N = decltype(ntag)::value;
        constexpr int HALF = (N + 1) / 2;
        const bool high = (lane & M) != 0;
#pragma unroll
        for (int i = 0; i < HALF; ++i) {
            const float lo = vals[i];
            const float hi = (i + HALF < N) ? vals[i + HALF] : 0.f;
            const float recv = lane_xor<M>(high ? lo : hi);
            vals[i] = (high ? hi : lo) + recv;
        }
        off += high ? HALF : 0;
        cnt = high ? max(0, cnt - HALF) : min(cnt, HALF);
    };
    using std::integral_constant;
    constexpr int N0 = NV, N1 = (N0 + 1) / 2, N2 = (N1 + 1) / 2, N3 = (N2 + 1) / 2, N4 = (N3 + 1) / 2;
    if constexpr (M0 == 2) {
        step(integral_constant<int, 2>{}, integral_constant<int, N0>{});
        step(integral_constant<int, 4>{}, integral_constant<int, N1>{});
        step(integral_constant<int, 8>{}, integral_constant<int, N2>{});
        step(integral_constant<int, 16>{}, integral_constant<int, N3>{});
        step(integral_constant<int, 32>{}, integral_constant<int, N4>{});
    } else {
        static_assert(M0 == 4, "lanes per position must be 2 or 4");
        step(integral_constant<int, 4>{}, integral_constant<int, N0>{});
        step(integral_constant<int, 8>{}, integral_constant<int, N1>{});
        step(integral_constant<int, 16>{}, integral_constant<int, N2>{});
        step(integral_constant<int, 32>{}, integral_constant<int, N3>{});
    }
}

}  // namespace cfpp
