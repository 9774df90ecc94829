// Vector-ALU LoRA apply over plan chunks: decode (gather by slot index), packed MoE pairs and
// small-rank segments.  One workgroup handles up to MLORA_CHUNK rows that share one adapter
// (and one expert) and one tile of d_out:
//   shrink  h[c][j] = sum_i x[row_c, i] * A[j, i]   -- wavefront reduction, packed-bf16 dot2,
//                                                      fp32 accumulate, h kept in LDS as fp32
//   scale   h *= alpha / r
//   expand  y[row_c, o] = bf16_rne(float(y[row_c, o]) + sum_j h[c][j] * B[o, j])   in place
// The shrink result never leaves the workgroup.  Adapter rows beyond the slot's true rank are
// zero in the tables (padded slots), so the loops run to the padded rank.
#include "internal.h"

namespace mlora {

template <int RP, int NW>
struct RowsCfg {
    static constexpr int NT  = NW * 64;
    static constexpr int JG  = RP < NW ? RP : NW;        // groups of A rows across waves
    static constexpr int KS  = NW / JG;                  // d_in slices across waves
    static constexpr int JPW = RP / JG;                  // A rows per wave
    static constexpr int CS  = (32 / JPW) < kChunk ? (32 / JPW) : kChunk;   // rows per shrink pass
    static constexpr int NV  = CS * JPW;                 // accumulators per lane (power of two)
    static constexpr int OPL = RP >= 8 ? 1 : 8 / RP;     // outputs per lane in the expand
    static constexpr int BV  = RP >= 8 ? RP / 8 : 1;     // 16-byte loads of B per lane
};

// Sum each of the N per-lane values over the 64 lanes of the wave.  On return lane L holds in
// v[0] the total of original index bitreverse(L mod N): each step a lane hands half of its
// values to its partner and keeps the other half, so the work halves every step.
template <int N>
__device__ __forceinline__ void wave_sum_transpose(float (&v)[N], int lane)
{
    int d = 1;
#pragma unroll
    for (int h = N / 2; h >= 1; h >>= 1, d <<= 1) {
        const bool up = (lane & d) != 0;
#pragma unroll
        for (int i = 0; i < h; ++i) {
            float send = up ? v[i] : v[i + h];
            float keep = up ? v[i + h] : v[i];
            v[i] = keep + __shfl_xor(send, d, 64);
        }
    }
#pragma unroll
    for (; d < 64; d <<= 1) v[0] += __shfl_xor(v[0], d, 64);
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

template <int OPL> struct YVec;
template <> struct YVec<1> { typedef uint16_t T; };
template <> struct YVec<2> { typedef uint32_t T; };
template <> struct YVec<4> { typedef uint2 T; };
template <> struct YVec<8> { typedef uint4 T; };

__device__ __forceinline__ void y_unpack(uint16_t r, float *f) { f[0] = bf_lo(r); }
__device__ __forceinline__ void y_unpack(uint32_t r, float *f) { f[0] = bf_lo(r); f[1] = bf_hi(r); }
__device__ __forceinline__ void y_unpack(uint2 r, float *f)
{ f[0] = bf_lo(r.x); f[1] = bf_hi(r.x); f[2] = bf_lo(r.y); f[3] = bf_hi(r.y); }
__device__ __forceinline__ void y_unpack(uint4 r, float *f)
{
    f[0] = bf_lo(r.x); f[1] = bf_hi(r.x); f[2] = bf_lo(r.y); f[3] = bf_hi(r.y);
    f[4] = bf_lo(r.z); f[5] = bf_hi(r.z); f[6] = bf_lo(r.w); f[7] = bf_hi(r.w);
}
__device__ __forceinline__ void y_pack(const float *f, uint16_t &r) { r = (uint16_t)f2bf(f[0]); }
__device__ __forceinline__ void y_pack(const float *f, uint32_t &r) { r = pack_bf2(f[0], f[1]); }
__device__ __forceinline__ void y_pack(const float *f, uint2 &r)
{ r.x = pack_bf2(f[0], f[1]); r.y = pack_bf2(f[2], f[3]); }
__device__ __forceinline__ void y_pack(const float *f, uint4 &r)
{
    r.x = pack_bf2(f[0], f[1]); r.y = pack_bf2(f[2], f[3]);
    r.z = pack_bf2(f[4], f[5]); r.w = pack_bf2(f[6], f[7]);
}

template <int RP, int NW>
__global__ __launch_bounds__(NW * 64)
void rows_kernel(const RowsArgs a)
{
    using C = RowsCfg<RP, NW>;
    __shared__ float hs[kChunk][RP];
    __shared__ float part[C::KS > 1 ? C::KS : 1][kChunk][RP];
    __shared__ int32_t s_item[kChunk];

    // Workgroups are dealt round-robin to the 8 XCDs; undo that so that neighbouring work ids
    // (the tiles of one chunk, the chunks of one adapter) share an XCD and its L2.
    const int per_xcd = gridDim.x >> 3;
    const int v = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    const int chunk = v / a.n_tiles, tile = v - chunk * a.n_tiles;
    if (chunk >= a.grid_chunks || chunk >= a.hdr[0]) return;
    const int key = a.chunks[3 * chunk], start = a.chunks[3 * chunk + 1], cnt = a.chunks[3 * chunk + 2];
    const int slot = key / a.n_experts;
    if (a.meta.rank[slot] <= 0) return;
    const float scale = a.meta.scale[slot];

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    if (tid < kChunk) {
        int c = tid < cnt ? tid : cnt - 1;
        s_item[tid] = a.sorted ? a.sorted[start + c] : start + c;
    }
    __syncthreads();

    // ---------------- shrink ----------------
    const int jg = w % C::JG, ks = w / C::JG;
    const uint16_t *Ag = a.a_tab + (int64_t)key * RP * a.d_in + (int64_t)(jg * C::JPW) * a.d_in;
    const int U = a.d_in >> 3;
    for (int c0 = 0; c0 < cnt; c0 += C::CS) {
        const int n = min(C::CS, cnt - c0);
        float acc[C::NV];
#pragma unroll
        for (int i = 0; i < C::NV; ++i) acc[i] = 0.f;
        const uint4 *xp[C::CS];
#pragma unroll
        for (int c = 0; c < C::CS; ++c) {
            int row = s_item[min(c0 + c, kChunk - 1)] / a.top_k;
            xp[c] = (const uint4 *)(a.x + (int64_t)row * a.ldx);
        }
#pragma unroll 2
        for (int u = ks * 64 + lane; u < U; u += C::KS * 64) {
            uint4 av[C::JPW];
#pragma unroll
            for (int jj = 0; jj < C::JPW; ++jj) av[jj] = ((const uint4 *)(Ag + (int64_t)jj * a.d_in))[u];
#pragma unroll
            for (int c = 0; c < C::CS; ++c) {
                if (c < n) {
                    const uint4 xv = xp[c][u];
#pragma unroll
                    for (int jj = 0; jj < C::JPW; ++jj) acc[c * C::JPW + jj] = dot8(xv, av[jj], acc[c * C::JPW + jj]);
                }
            }
        }
        wave_sum_transpose<C::NV>(acc, lane);
        if (lane < C::NV) {
            const int idx = bitrev<Log2<C::NV>::v>(lane);
            const int c = idx / C::JPW, jj = idx % C::JPW;
            if (c0 + c < kChunk) {
                if (C::KS > 1) part[ks][c0 + c][jg * C::JPW + jj] = acc[0];
                else           hs[c0 + c][jg * C::JPW + jj] = acc[0] * scale;
            }
        }
    }
    __syncthreads();
    if (C::KS > 1) {
        for (int i = tid; i < kChunk * RP; i += C::NT) {
            float s = 0.f;
#pragma unroll
            for (int k = 0; k < C::KS; ++k) s += (&part[k][0][0])[i];
            (&hs[0][0])[i] = s * scale;
        }
        __syncthreads();
    }

    // ---------------- expand + in-place add ----------------
    typedef typename YVec<C::OPL>::T yvec_t;
    const uint16_t *Bg = a.b_tab + (int64_t)key * a.d_out * RP;
    const int tile_sz = (((a.d_out + a.n_tiles - 1) / a.n_tiles) + 7) & ~7;
    const int lo = tile * tile_sz, hi = min(a.d_out, lo + tile_sz);
    for (int o = lo + tid * C::OPL; o < hi; o += C::NT * C::OPL) {
        uint4 braw[C::BV];
#pragma unroll
        for (int q = 0; q < C::BV; ++q) braw[q] = ((const uint4 *)(Bg + (int64_t)o * RP))[q];
        yvec_t yraw[kChunk];
#pragma unroll
        for (int c = 0; c < kChunk; ++c)
            if (c < cnt) yraw[c] = *(const yvec_t *)(a.y + (int64_t)s_item[c] * a.ldy + o);
        // b[q*RP + j] for output q of this lane; for RP >= 8 there is one output and RP values
        float b[C::BV * 8];
#pragma unroll
        for (int q = 0; q < C::BV; ++q) {
            b[q * 8 + 0] = bf_lo(braw[q].x); b[q * 8 + 1] = bf_hi(braw[q].x);
            b[q * 8 + 2] = bf_lo(braw[q].y); b[q * 8 + 3] = bf_hi(braw[q].y);
            b[q * 8 + 4] = bf_lo(braw[q].z); b[q * 8 + 5] = bf_hi(braw[q].z);
            b[q * 8 + 6] = bf_lo(braw[q].w); b[q * 8 + 7] = bf_hi(braw[q].w);
        }
#pragma unroll
        for (int c = 0; c < kChunk; ++c) {
            if (c < cnt) {
                float yf[C::OPL];
                y_unpack(yraw[c], yf);
#pragma unroll
                for (int q = 0; q < C::OPL; ++q) {
                    float d = 0.f;
#pragma unroll
                    for (int j = 0; j < RP; ++j) d = fmaf(hs[c][j], b[q * RP + j], d);
                    yf[q] += d;
                }
                yvec_t out;
                y_pack(yf, out);
                *(yvec_t *)(a.y + (int64_t)s_item[c] * a.ldy + o) = out;
            }
        }
    }
}

template <int RP>
static hipError_t launch_rp(const RowsArgs &a, hipStream_t st)
{
    const int total = a.grid_chunks * a.n_tiles;
    const unsigned grid = (unsigned)((total + 7) / 8 * 8);
    rows_kernel<RP, 4><<<dim3(grid), dim3(256), 0, st>>>(a);
    return hipGetLastError();
}

hipError_t launch_rows(const RowsArgs &a, hipStream_t st)
{
    if (a.grid_chunks <= 0) return hipSuccess;
    switch (a.r_pad) {
        case 1:  return launch_rp<1>(a, st);
        case 2:  return launch_rp<2>(a, st);
        case 4:  return launch_rp<4>(a, st);
        case 8:  return launch_rp<8>(a, st);
        case 16: return launch_rp<16>(a, st);
        case 32: return launch_rp<32>(a, st);
        case 64: return launch_rp<64>(a, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace mlora
