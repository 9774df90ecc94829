// Cross-lane helpers shared by the apply kernels (wave64).
#ifndef MLORA_WAVE_OPS_H
#define MLORA_WAVE_OPS_H
#include "internal.h"

namespace mlora {

// Value of lane (l ^ D).  D = 1, 2, 4, 8 are DPP moves inside a row of 16 lanes, 16 is an LDS
// crossbar swizzle inside each half wave, 32 goes through ds_bpermute.
template <int D>
__device__ __forceinline__ float lane_xor(float v)
{
    const int x = __float_as_int(v);
    int r;
    if constexpr (D == 1) r = __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xf, 0xf, true);          // quad_perm [1,0,3,2]
    else if constexpr (D == 2) r = __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xf, 0xf, true);     // quad_perm [2,3,0,1]
    else if constexpr (D == 4) {
        r = __builtin_amdgcn_update_dpp(0, x, 0x104, 0xf, 0x5, false);                          // row_shl:4, lanes with bit 2 clear
        r = __builtin_amdgcn_update_dpp(r, x, 0x114, 0xf, 0xa, false);                          // row_shr:4, lanes with bit 2 set
    } else if constexpr (D == 8) r = __builtin_amdgcn_update_dpp(0, x, 0x128, 0xf, 0xf, true);  // row_ror:8
    else if constexpr (D == 16) r = __builtin_amdgcn_ds_swizzle(x, 0x401F);                     // xor 16 in groups of 32
    else r = __shfl_xor(x, 32, 64);
    return __int_as_float(r);
}

// Sum each of the N per-lane values over the 64 lanes of the wave.  On return lane L holds in
// v[0] the total of original index bitreverse(L mod N): each step a lane hands half of its
// values to its partner and keeps the other half, so the work halves every step.
template <int N, int H, int D>
struct TransposeStep {
    static __device__ __forceinline__ void run(float (&v)[N], int lane)
    {
        const bool up = (lane & D) != 0;
#pragma unroll
        for (int i = 0; i < H; ++i) {
            const float send = up ? v[i] : v[i + H];
            const float keep = up ? v[i + H] : v[i];
            v[i] = keep + lane_xor<D>(send);
        }
        TransposeStep<N, H / 2, D * 2>::run(v, lane);
    }
};
template <int N, int D>
struct TransposeStep<N, 0, D> {
    static __device__ __forceinline__ void run(float (&v)[N], int lane)
    {
        if constexpr (D < 64) {
            v[0] += lane_xor<D>(v[0]);
            TransposeStep<N, 0, D * 2>::run(v, lane);
        }
    }
};
template <int N>
__device__ __forceinline__ void wave_sum_transpose(float (&v)[N], int lane)
{
    TransposeStep<N, N / 2, 1>::run(v, lane);
}

template <int BITS>
__device__ __forceinline__ int bitrev(int x)
{
    int r = 0;
#pragma unroll
    for (int b = 0; b < BITS; ++b) r |= ((x >> b) & 1) << (BITS - 1 - b);
    return r;
}

template <int N> struct Log2 { static constexpr int v = 1 + Log2<N / 2>::v; };
template <> struct Log2<1> { static constexpr int v = 0; };

}  // namespace mlora
#endif
