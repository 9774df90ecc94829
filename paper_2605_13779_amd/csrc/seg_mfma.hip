// Rank-64 segmented (prefill) LoRA apply on the gfx950 matrix cores.
//
// A workgroup owns a tile of up to 32 consecutive rows of one segment (all rows of a segment use
// one adapter: a request's prompt is one contiguous run).  Both halves are dense contractions:
//   shrink  h[32 x 64]    = X[32 x d_in] * A_s^T[d_in x 64]   v_mfma_f32_32x32x16_bf16, the four
//                                                              waves split d_in, partials summed in LDS
//   scale   h *= alpha / r (fp32), then h is split into bf16 hi + lo so that the expand sees h
//           to ~16 mantissa bits (the shrink result is not rounded to bf16)
//   expand  Y[32 x d_out] += h * B_s^T[64 x d_out]             two MFMAs (hi, lo) per 16 ranks,
//                                                              staged through LDS so that the
//                                                              in-place bf16 add on y is coalesced
// h never leaves the workgroup.
#include "internal.h"

namespace mlora {

namespace {
constexpr int TM = 32;          // rows per tile
constexpr int NB = 256;         // outputs per expand iteration (64 per wave)
constexpr int ST_LD = NB + 4;   // padded row stride of the staging tile, in floats
constexpr int H_LD = 72;        // padded row stride of the bf16 h tiles, in elements
}

__device__ __forceinline__ f32x16_t mfma32(const uint4 &a, const uint4 &b, f32x16_t c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// Accumulator register i of lane l holds row (i/4)*8 + (l/32)*4 + i%4, column l%32.
__device__ __forceinline__ int acc_row(int i, int kh) { return (i >> 2) * 8 + kh * 4 + (i & 3); }

namespace {
constexpr int KG = 4;            // k steps (of 16) per prefetch group: one 128-byte line per row
struct KGroup { uint4 x[KG], v0[KG], v1[KG]; };
struct ExpStage { uint4 b[2][4]; uint4 y[4]; };
}

__global__ __launch_bounds__(256)
void seg_mfma_kernel(const SegArgs a)
{
    __shared__ __attribute__((aligned(16))) float buf[2][TM * ST_LD];   // partials, then staging (double-buffered)
    __shared__ __attribute__((aligned(16))) uint16_t hh[TM * H_LD];
    __shared__ __attribute__((aligned(16))) uint16_t hl[TM * H_LD];

    const int per_xcd = gridDim.x >> 3;
    const int v = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (v >= a.n_tiles) return;
    const int slot = a.tiles[3 * v], row0 = a.tiles[3 * v + 1], nrows = a.tiles[3 * v + 2];
    if (slot < 0 || a.meta.rank[slot] <= 0) return;
    const float scale = a.meta.scale[slot];

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, m = lane & 31, kh = lane >> 5;

    // ---------------- shrink: each wave owns a contiguous quarter of d_in ----------------
    {
        const uint16_t *xp = a.x + (int64_t)(row0 + min(m, nrows - 1)) * a.ldx + kh * 8;
        const uint16_t *Ag = a.a_tab + (int64_t)slot * 64 * a.d_in;
        const uint16_t *a0 = Ag + (int64_t)m * a.d_in + kh * 8;
        const uint16_t *a1 = Ag + (int64_t)(32 + m) * a.d_in + kh * 8;
        f32x16_t acc0 = {0}, acc1 = {0};
        const int steps = a.d_in >> 4;
        const int steps_w = (steps + 3) >> 2;
        const int s_lo = w * steps_w, s_hi = min(steps, s_lo + steps_w);
        const int n_grp = (steps_w + KG - 1) / KG;
        auto load = [&](int g, KGroup &kg) {
#pragma unroll
            for (int i = 0; i < KG; ++i) {
                const int s = s_lo + g * KG + i;
                const bool in = s < s_hi;
                const int sc = in ? s : 0;
                kg.x[i] = *(const uint4 *)(xp + sc * 16);
                kg.v0[i] = *(const uint4 *)(a0 + sc * 16);
                kg.v1[i] = *(const uint4 *)(a1 + sc * 16);
                if (!in) kg.x[i] = make_uint4(0, 0, 0, 0);
            }
        };
        auto mma = [&](const KGroup &kg) {
#pragma unroll
            for (int i = 0; i < KG; ++i) {
                acc0 = mfma32(kg.x[i], kg.v0[i], acc0);
                acc1 = mfma32(kg.x[i], kg.v1[i], acc1);
            }
        };
        KGroup g0, g1;
        load(0, g0);
        for (int g = 0; g < n_grp; g += 2) {
            if (g + 1 < n_grp) load(g + 1, g1);
            mma(g0);
            if (g + 1 < n_grp) {
                if (g + 2 < n_grp) load(g + 2, g0);
                mma(g1);
            }
        }
        float *red = &buf[0][0] + w * (TM * 64);          // 4 * 32 * 64 floats fit in buf[0..1]
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            red[acc_row(i, kh) * 64 + m] = acc0[i];
            red[acc_row(i, kh) * 64 + 32 + m] = acc1[i];
        }
    }
    __syncthreads();
    {
        const float *red = &buf[0][0];
        for (int e = tid; e < TM * 64; e += 256) {
            float s = (red[e] + red[e + TM * 64]) + (red[e + 2 * TM * 64] + red[e + 3 * TM * 64]);
            s *= scale;
            const uint32_t hi = f2bf(s);
            const uint32_t lo = f2bf(s - __uint_as_float(hi << 16));
            const int tok = e >> 6, j = e & 63;
            hh[tok * H_LD + j] = (uint16_t)hi;
            hl[tok * H_LD + j] = (uint16_t)lo;
        }
    }
    __syncthreads();
    uint4 hA[4], lA[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        hA[ks] = *(const uint4 *)(hh + m * H_LD + ks * 16 + kh * 8);
        lA[ks] = *(const uint4 *)(hl + m * H_LD + ks * 16 + kh * 8);
    }

    // ---------------- expand + in-place add ----------------
    const uint16_t *Bg = a.b_tab + (int64_t)slot * a.d_out * 64;
    const int og = tid & 31, tr = tid >> 5;
    auto load_exp = [&](int n0, ExpStage &st) {
        const int oc = n0 + og * 8;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int tok = tr + 8 * q;
            if (tok < nrows && oc < a.d_out) st.y[q] = *(const uint4 *)(a.y + (int64_t)(row0 + tok) * a.ldy + oc);
        }
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            const int ob = n0 + w * 64 + nb * 32;
            const uint16_t *bp = Bg + (int64_t)min(ob + m, a.d_out - 1) * 64 + kh * 8;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) st.b[nb][ks] = *(const uint4 *)(bp + ks * 16);
        }
    };
    ExpStage cur, nxt;
    load_exp(0, cur);
    int par = 0;
    for (int n0 = 0; n0 < a.d_out; n0 += NB, par ^= 1) {
        if (n0 + NB < a.d_out) load_exp(n0 + NB, nxt);
        float *stg = &buf[par][0];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            f32x16_t acc = {0};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                acc = mfma32(hA[ks], cur.b[nb][ks], acc);
                acc = mfma32(lA[ks], cur.b[nb][ks], acc);
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) stg[acc_row(i, kh) * ST_LD + w * 64 + nb * 32 + m] = acc[i];
        }
        __syncthreads();     // one barrier per pass: the other staging buffer is written next pass
        const int oc = n0 + og * 8;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int tok = tr + 8 * q;
            if (tok < nrows && oc < a.d_out) {
                const float4 d0 = *(const float4 *)(stg + tok * ST_LD + og * 8);
                const float4 d1 = *(const float4 *)(stg + tok * ST_LD + og * 8 + 4);
                const uint4 yv = cur.y[q];
                uint4 o;
                o.x = pack_bf2(bf_lo(yv.x) + d0.x, bf_hi(yv.x) + d0.y);
                o.y = pack_bf2(bf_lo(yv.y) + d0.z, bf_hi(yv.y) + d0.w);
                o.z = pack_bf2(bf_lo(yv.z) + d1.x, bf_hi(yv.z) + d1.y);
                o.w = pack_bf2(bf_lo(yv.w) + d1.z, bf_hi(yv.w) + d1.w);
                *(uint4 *)(a.y + (int64_t)(row0 + tok) * a.ldy + oc) = o;
            }
        }
        cur = nxt;
    }
}

hipError_t launch_seg_mfma(const SegArgs &a, hipStream_t st)
{
    if (a.n_tiles <= 0) return hipSuccess;
    const unsigned grid = (unsigned)((a.n_tiles + 7) / 8 * 8);
    seg_mfma_kernel<<<dim3(grid), dim3(256), 0, st>>>(a);
    return hipGetLastError();
}

}  // namespace mlora
