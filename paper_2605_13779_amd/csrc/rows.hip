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
template <int N, int H, int D>
struct TransposeStep {
    static __device__ __forceinline__ void run(float (&v)[N], int lane)
    {
        const bool up = (lane & D) != 0;
#pragma unroll
        for (int i = 0; i < H; ++i) {
            const float send = up ? v[i] : v[i + H];
            const float keep = up ? v[i + H] : v[i];
            v[i] = keep + __shfl_xor(send, D, 64);
        }
        TransposeStep<N, H / 2, D * 2>::run(v, lane);
    }
};
template <int N, int D>
struct TransposeStep<N, 0, D> {
    static __device__ __forceinline__ void run(float (&v)[N], int lane)
    {
        if constexpr (D < 64) {
            v[0] += __shfl_xor(v[0], D, 64);
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

// One pipeline stage of the shrink: for one 16-byte unit of d_in per lane, the wave's JPW rows
// of A and the same unit of every row of the chunk.  All loads of a stage are issued together.
template <int JPW, int CS>
struct ShrinkStage {
    uint4 av[JPW];
    uint4 xv[CS];
};

template <int RP, int NW>
__global__ __launch_bounds__(NW * 64)
void rows_kernel(const RowsArgs a)
{
    using C = RowsCfg<RP, NW>;
    __shared__ float hs[kChunk][RP];
    __shared__ float part[C::KS > 1 ? C::KS : 1][kChunk][RP];

    // Workgroups are dealt round-robin to the 8 XCDs; undo that so that neighbouring work ids
    // (the tiles of one chunk, the chunks of one adapter) share an XCD and its L2.
    const int per_xcd = gridDim.x >> 3;
    const int v = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    const int chunk = v / a.n_tiles, tile = v - chunk * a.n_tiles;
    uint64_t *prof = a.prof ? a.prof + (int64_t)blockIdx.x * 8 : nullptr;
    if (prof && threadIdx.x == 0) { prof[0] = wall_clock64(); prof[7] = 0; }
    if (chunk >= a.grid_chunks || chunk >= a.hdr[0]) return;
    const int32_t *rec = a.chunks + (int64_t)chunk * kRec;
    const int key = rec[0], cnt = rec[1];
    int item[kChunk];
#pragma unroll
    for (int c = 0; c < kChunk; ++c) item[c] = rec[4 + (c < cnt ? c : cnt - 1)];
    const int slot = key / a.n_experts;
    if (a.meta.rank[slot] <= 0) return;
    const float scale = a.meta.scale[slot];

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    if (prof && tid == 0) { prof[1] = wall_clock64(); prof[7] = cnt; }

    // ---------------- shrink ----------------
    const int jg = w % C::JG, ks = w / C::JG;
    const uint4 *Ag = (const uint4 *)(a.a_tab + (int64_t)key * RP * a.d_in + (int64_t)(jg * C::JPW) * a.d_in);
    const int U = a.d_in >> 3;                       // 16-byte units per row
    const int n_it = (U + C::KS * 64 - 1) / (C::KS * 64);
    typedef ShrinkStage<C::JPW, C::CS> Stage;
#pragma unroll
    for (int c0 = 0; c0 < kChunk; c0 += C::CS) {
        if (c0 >= cnt) break;
        const int n = min(C::CS, cnt - c0);
        float acc[C::NV];
#pragma unroll
        for (int i = 0; i < C::NV; ++i) acc[i] = 0.f;
        const uint4 *xp[C::CS];
#pragma unroll
        for (int c = 0; c < C::CS; ++c)
            xp[c] = (const uint4 *)(a.x + (int64_t)(item[c0 + c] / a.top_k) * a.ldx);

        auto load = [&](int it, Stage &st) {
            const int u = (it * C::KS + ks) * 64 + lane;
            const bool in = u < U;
            const int uc = in ? u : 0;
#pragma unroll
            for (int jj = 0; jj < C::JPW; ++jj) st.av[jj] = Ag[(int64_t)jj * U + uc];
#pragma unroll
            for (int c = 0; c < C::CS; ++c) {
                if (c < n) {
                    st.xv[c] = xp[c][uc];
                    if (!in) st.xv[c] = make_uint4(0, 0, 0, 0);
                }
            }
        };
        auto fma_stage = [&](const Stage &st) {
#pragma unroll
            for (int c = 0; c < C::CS; ++c) {
                if (c < n) {
#pragma unroll
                    for (int jj = 0; jj < C::JPW; ++jj)
                        acc[c * C::JPW + jj] = dot8(st.xv[c], st.av[jj], acc[c * C::JPW + jj]);
                }
            }
        };
        Stage s0, s1;
        load(0, s0);
        for (int it = 0; it < n_it; it += 2) {
            if (it + 1 < n_it) load(it + 1, s1);
            fma_stage(s0);
            if (it + 1 < n_it) {
                if (it + 2 < n_it) load(it + 2, s0);
                fma_stage(s1);
            }
        }
        if (prof && tid == 0) prof[2] = wall_clock64();
        wave_sum_transpose<C::NV>(acc, lane);
        if (lane < C::NV) {
            const int idx = bitrev<Log2<C::NV>::v>(lane);
            const int c = idx / C::JPW, jj = idx % C::JPW;
            if (C::KS > 1) part[ks][c0 + c][jg * C::JPW + jj] = acc[0];
            else           hs[c0 + c][jg * C::JPW + jj] = acc[0] * scale;
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

    if (prof && tid == 0) prof[3] = wall_clock64();
    // ---------------- expand + in-place add ----------------
    // Each pass covers EU * NT * OPL outputs; all of its loads (B rows and the y values of every
    // row of the chunk) are issued before the first use.
    typedef typename YVec<C::OPL>::T yvec_t;
    constexpr int EU = RP <= 16 ? 4 : (RP == 32 ? 2 : 1);
    const uint16_t *Bg = a.b_tab + (int64_t)key * a.d_out * RP;
    const int tile_sz = (((a.d_out + a.n_tiles - 1) / a.n_tiles) + 7) & ~7;
    const int lo = tile * tile_sz, hi = min(a.d_out, lo + tile_sz);
    uint16_t *yrow[kChunk];
#pragma unroll
    for (int c = 0; c < kChunk; ++c) yrow[c] = a.y + (int64_t)item[c] * a.ldy;
    for (int o0 = lo + tid * C::OPL; o0 < hi; o0 += EU * C::NT * C::OPL) {
        uint4 braw[EU][C::BV];
        yvec_t yraw[EU][kChunk];
#pragma unroll
        for (int e = 0; e < EU; ++e) {
            const int o = o0 + e * C::NT * C::OPL;
            const int oc = o < hi ? o : lo;              // clamped address, result discarded
#pragma unroll
            for (int q = 0; q < C::BV; ++q) braw[e][q] = ((const uint4 *)(Bg + (int64_t)oc * RP))[q];
#pragma unroll
            for (int c = 0; c < kChunk; ++c)
                if (c < cnt) yraw[e][c] = *(const yvec_t *)(yrow[c] + oc);
        }
#pragma unroll
        for (int e = 0; e < EU; ++e) {
            const int o = o0 + e * C::NT * C::OPL;
            if (o < hi) {
                // b[q*RP + j] for output q of this lane; for RP >= 8 there is one output and RP values
                float b[C::BV * 8];
#pragma unroll
                for (int q = 0; q < C::BV; ++q) {
                    b[q * 8 + 0] = bf_lo(braw[e][q].x); b[q * 8 + 1] = bf_hi(braw[e][q].x);
                    b[q * 8 + 2] = bf_lo(braw[e][q].y); b[q * 8 + 3] = bf_hi(braw[e][q].y);
                    b[q * 8 + 4] = bf_lo(braw[e][q].z); b[q * 8 + 5] = bf_hi(braw[e][q].z);
                    b[q * 8 + 6] = bf_lo(braw[e][q].w); b[q * 8 + 7] = bf_hi(braw[e][q].w);
                }
#pragma unroll
                for (int c = 0; c < kChunk; ++c) {
                    if (c < cnt) {
                        float yf[C::OPL];
                        y_unpack(yraw[e][c], yf);
#pragma unroll
                        for (int q = 0; q < C::OPL; ++q) {
                            float d = 0.f;
#pragma unroll
                            for (int j = 0; j < RP; ++j) d = fmaf(hs[c][j], b[q * RP + j], d);
                            yf[q] += d;
                        }
                        yvec_t out;
                        y_pack(yf, out);
                        *(yvec_t *)(yrow[c] + o) = out;
                    }
                }
            }
        }
    }
    if (prof && tid == 0) prof[4] = wall_clock64();
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
