// Rank-64 segmented (prefill) LoRA apply on the gfx950 matrix cores.
//
// A workgroup owns a tile of up to 32 consecutive rows of one segment (all rows of a segment use
// one adapter: a request's prompt is one contiguous run).  Both halves are dense contractions:
//   shrink  h[32 x 64]    = X[32 x d_in] * A_s^T[d_in x 64]   v_mfma_f32_32x32x16_bf16, the eight
//                                                              waves split d_in, partials summed in LDS
//   scale   h *= alpha / r (fp32), then h is split into bf16 hi + lo so that the expand sees h
//           to ~16 mantissa bits (the shrink result is not rounded to bf16)
//   expand  Y[32 x d_out] += h * B_s^T[64 x d_out]             two MFMAs (hi, lo) per 16 ranks; every
//                                                              wave walks its own 64-wide passes and
//                                                              stages them in a private LDS tile so
//                                                              that the in-place bf16 add on y moves
//                                                              whole 128-byte row segments
// h never leaves the workgroup.
#include "internal.h"

namespace mlora {

namespace {
constexpr int TM = 32;            // rows per tile
constexpr int NW = 8;             // waves per workgroup
constexpr int NT = NW * 64;
constexpr int KT = 256;           // elements of d_in per staged k tile (16 MFMA k steps, two per wave)
constexpr int TROW = KT * 2 + 16; // padded byte stride of a staged row (x or A)
constexpr int TILE_BYTES = (TM + 64) * TROW;
constexpr int WB = 64;            // outputs per wave per expand pass (two 32-wide MFMA blocks)
constexpr int BROW = 64 * 2 + 16; // padded byte stride of a staged B row (64 ranks)
constexpr int ST_LD = WB + 4;     // padded row stride of a wave's staging tile, in floats
constexpr int WAVE_BYTES = WB * BROW > TM * ST_LD * 4 ? WB * BROW : TM * ST_LD * 4;
constexpr int RED_BYTES = NW * TM * 64 * 4;              // k-slice partials of the shrink
constexpr int H_LD = 64;          // row stride of the bf16 h tiles, in elements
constexpr int cmax(int a, int b) { return a > b ? a : b; }
constexpr int BUF_BYTES = cmax(cmax(TILE_BYTES, RED_BYTES), NW * WAVE_BYTES);
}

__device__ __forceinline__ f32x16_t mfma32(const uint4 &a, const uint4 &b, f32x16_t c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// Accumulator register i of lane l holds row (i/4)*8 + (l/32)*4 + i%4, column l%32.
__device__ __forceinline__ int acc_row(int i, int kh) { return (i >> 2) * 8 + kh * 4 + (i & 3); }

// Every global access is a whole 16 bytes per lane with neighbouring lanes on neighbouring
// addresses (full 128-byte lines per row segment); LDS turns those row-major pieces into the
// MFMA operand layout, where a lane owns eight consecutive k of one row.  Loading operands
// straight from global memory in that layout touches 32 different lines per instruction and
// thrashes the small L1.
__global__ __launch_bounds__(NT, 4)
void seg_mfma_kernel(const SegArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char buf[BUF_BYTES];   // k tiles, then partials + h, then per-wave tiles
    static_assert(RED_BYTES + 2 * TM * H_LD * 2 <= BUF_BYTES, "the bf16 h tiles sit behind the partials");
    uint16_t *hh = (uint16_t *)(buf + RED_BYTES);
    uint16_t *hl = hh + TM * H_LD;

    __shared__ uint32_t s_tag;
    __shared__ int s_fail;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, m = lane & 31, kh = lane >> 5;
    const int G = a.cluster;                  // workgroups that share one tile: k-slices of the shrink, output slices of the expand
    const int n_wg = (int)gridDim.x;
    const bool last_wg = (int)blockIdx.x == n_wg - 1;
    uint32_t tag = 0;
    if (G > 1) {
        if (tid == 0) { tag = tag_read(a.ctrl); s_tag = tag; s_fail = 0; tag_sign_in(a.ctrl, (int)blockIdx.x, tag); }
        __syncthreads();
        tag = s_tag;
    }
    // neighbouring work ids share an XCD (workgroups are dealt round-robin to 8 XCDs): the tiles of one
    // segment reuse its adapter in L2, and the members of a cluster sit next to each other in dispatch order
    const int per_xcd = n_wg >> 3;
    const int v = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    const int tile = v / G, g = v - tile * G;
    bool live = tile < a.n_tiles;
    int slot = -1, row0 = 0, nrows = 1;
    if (live) { slot = a.tiles[3 * tile]; row0 = a.tiles[3 * tile + 1]; nrows = a.tiles[3 * tile + 2]; }
    live = live && slot >= 0 && a.meta.rank[slot] > 0;
    if (!live) {
        if (G > 1 && last_wg && w == 0) tag_advance(a.ctrl, n_wg, tag, lane);
        return;
    }
    const float scale = a.meta.scale[slot];

    // ---------------- shrink: k tiles of [32 x rows + 64 A rows] x 256 staged through LDS ----------------
    {
        // staged row r (0..31 = x rows of the tile, 32..95 = A rows); thread handles rows srow + 16 q, 16-byte segment sseg
        const int srow = tid >> 5, sseg = tid & 31;
        const uint16_t *gp[6];
#pragma unroll
        for (int q = 0; q < 6; ++q) {
            const int r = srow + 16 * q;
            gp[q] = (q < 2) ? a.x + (int64_t)(row0 + min(r, nrows - 1)) * a.ldx + sseg * 8
                            : a.a_tab + ((int64_t)slot * 64 + (r - 32)) * a.d_in + sseg * 8;
        }
        f32x16_t acc0 = {0}, acc1 = {0};
        const int n_kt_all = (a.d_in + KT - 1) / KT;
        const int kt_per = (n_kt_all + G - 1) / G;
        const int kt0 = g * kt_per;                            // this member's k tiles: [kt0, kt0 + n_kt)
        const int n_kt = max(0, min(n_kt_all, kt0 + kt_per) - kt0);
        auto fetch = [&](int t, uint4 (&stage)[6]) {
            const int k0 = (kt0 + t) * KT;
            const bool in = t < n_kt && k0 + sseg * 8 < a.d_in;   // d_in is a multiple of 16: a segment is in or out as a whole
#pragma unroll
            for (int q = 0; q < 6; ++q) {
                stage[q] = make_uint4(0, 0, 0, 0);
                if (in) stage[q] = q < 2 ? ld_stream(gp[q] + k0) : *(const uint4 *)(gp[q] + k0);
            }
        };
        auto consume = [&](const uint4 (&stage)[6]) {
            __syncthreads();                                  // the previous tile has been read by every wave
#pragma unroll
            for (int q = 0; q < 6; ++q) *(uint4 *)(buf + (srow + 16 * q) * TROW + sseg * 16) = stage[q];
            __syncthreads();
        };
        auto mma_tile = [&]() {
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const int kb = (2 * w + s2) * 32 + kh * 16;   // byte offset of this lane's 8 k values
                const uint4 xv = *(const uint4 *)(buf + m * TROW + kb);
                const uint4 v0 = *(const uint4 *)(buf + (32 + m) * TROW + kb);
                const uint4 v1 = *(const uint4 *)(buf + (64 + m) * TROW + kb);
                acc0 = mfma32(xv, v0, acc0);
                acc1 = mfma32(xv, v1, acc1);
            }
        };
        // two k tiles are in flight while a third is being multiplied
        uint4 sa[6], sb[6];
        fetch(0, sa);
        fetch(1, sb);
        for (int t = 0; t < n_kt; t += 2) {
            consume(sa);
            fetch(t + 2, sa);
            mma_tile();
            if (t + 1 < n_kt) {
                consume(sb);
                fetch(t + 3, sb);
                mma_tile();
            }
        }
        __syncthreads();
        float *red = (float *)buf + w * (TM * 64);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            red[acc_row(i, kh) * 64 + m] = acc0[i];
            red[acc_row(i, kh) * 64 + 32 + m] = acc1[i];
        }
    }
    __syncthreads();
    {
        float part[4];                                           // TM * 64 / NT elements per thread
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = tid + q * NT;
            float s = 0.f;
#pragma unroll
            for (int k = 0; k < NW; ++k) s += ((const float *)buf)[e + k * TM * 64];
            part[q] = s;
        }
        bool ok = true;
        if (G > 1) {
            // publish this member's partial, then add the members' partials in member order, so that
            // every member of the cluster ends up with bit-identical h
            uint64_t *mine = a.xch + ((int64_t)tile * G + g) * (TM * 64);
#pragma unroll
            for (int q = 0; q < 4; ++q) xch_put(mine + tid + q * NT, part[q], tag);
            float tot[4] = {0.f, 0.f, 0.f, 0.f};
            for (int gg = 0; gg < G; ++gg) {
                if (gg == g) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) tot[q] += part[q];
                    continue;
                }
                const uint64_t *src = a.xch + ((int64_t)tile * G + gg) * (TM * 64);
                uint64_t wv[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) wv[q] = xch_get(src + tid + q * NT);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    int spins = 0;
                    while ((uint32_t)(wv[q] >> 32) != tag) {
                        if (++spins > kSpinLimit) { ok = false; break; }
                        __builtin_amdgcn_s_sleep(1);
                        wv[q] = xch_get(src + tid + q * NT);
                    }
                    tot[q] += __uint_as_float((uint32_t)wv[q]);
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) part[q] = tot[q];
        }
        if (!ok) s_fail = 1;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = tid + q * NT;
            const float s = part[q] * scale;
            const uint32_t hi = f2bf(s);
            const uint32_t lo = f2bf(s - __uint_as_float(hi << 16));
            const int tok = e >> 6, j = e & 63;
            hh[tok * H_LD + j] = (uint16_t)hi;
            hl[tok * H_LD + j] = (uint16_t)lo;
        }
    }
    __syncthreads();
    if (G > 1 && s_fail) {                       // a member never showed up (not expected): leave y alone, raise the flag
        if (tid == 0) __hip_atomic_store(a.ctrl + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (last_wg && w == 0) tag_advance(a.ctrl, n_wg, tag, lane);
        return;
    }
    uint4 hA[4], lA[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        hA[ks] = *(const uint4 *)(hh + m * H_LD + ks * 16 + kh * 8);
        lA[ks] = *(const uint4 *)(hl + m * H_LD + ks * 16 + kh * 8);
    }
    __syncthreads();                 // buf turns from partials into the waves' private tiles

    // ---------------- expand + in-place add: every wave walks its own 64-wide passes ----------------
    // A pass stages its 64 B rows in the wave's LDS tile, reads them back as MFMA operands, then
    // reuses the same tile to turn the accumulators into row-contiguous pieces for the add on y.
    // The tile is private to the wave and LDS serves a wave's requests in order, so compiler-level
    // fences are all that is needed between the phases.
    const uint16_t *Bg = a.b_tab + (int64_t)slot * a.d_out * 64;
    unsigned char *wt = buf + w * WAVE_BYTES;
    float *stg = (float *)wt;
    const int og = lane & 7, tr = lane >> 3;          // 8 lanes cover 128 bytes of one row
    const int out_per = ((a.d_out + WB * G - 1) / (WB * G)) * WB;      // outputs per member, a multiple of a pass
    const int out_lo = g * out_per, out_hi = min(a.d_out, out_lo + out_per);
    for (int n0 = out_lo + w * WB; n0 < out_hi; n0 += NW * WB) {
        const int oc = n0 + og * 8;
        uint4 yv[4], braw[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {                 // B rows n0 + 8 i + lane / 8, 16-byte piece lane % 8
            const int o = min(n0 + 8 * i + tr, a.d_out - 1);
            braw[i] = *(const uint4 *)(Bg + (int64_t)o * 64 + og * 8);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int tok = tr + 8 * q;
            if (tok < nrows && oc < a.d_out) yv[q] = ld_stream(a.y + (int64_t)(row0 + tok) * a.ldy + oc);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) *(uint4 *)(wt + (8 * i + tr) * BROW + og * 16) = braw[i];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        f32x16_t acc[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            uint4 bv[4];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bv[ks] = *(const uint4 *)(wt + (nb * 32 + m) * BROW + ks * 32 + kh * 16);
            acc[nb] = f32x16_t{0};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                acc[nb] = mfma32(hA[ks], bv[ks], acc[nb]);
                acc[nb] = mfma32(lA[ks], bv[ks], acc[nb]);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");     // all operand reads precede the reuse of the tile
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) stg[acc_row(i, kh) * ST_LD + nb * 32 + m] = acc[nb][i];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int tok = tr + 8 * q;
            if (tok < nrows && oc < a.d_out) {
                const float4 d0 = *(const float4 *)(stg + tok * ST_LD + og * 8);
                const float4 d1 = *(const float4 *)(stg + tok * ST_LD + og * 8 + 4);
                uint4 o;
                o.x = pack_bf2(bf_lo(yv[q].x) + d0.x, bf_hi(yv[q].x) + d0.y);
                o.y = pack_bf2(bf_lo(yv[q].y) + d0.z, bf_hi(yv[q].y) + d0.w);
                o.z = pack_bf2(bf_lo(yv[q].z) + d1.x, bf_hi(yv[q].z) + d1.y);
                o.w = pack_bf2(bf_lo(yv[q].w) + d1.z, bf_hi(yv[q].w) + d1.w);
                st_stream(a.y + (int64_t)(row0 + tok) * a.ldy + oc, o);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
    if (G > 1 && last_wg && w == 0) tag_advance(a.ctrl, n_wg, tag, lane);
}

hipError_t launch_seg_mfma(const SegArgs &a_in, hipStream_t st)
{
    if (a_in.n_tiles <= 0) return hipSuccess;
    SegArgs a = a_in;
    // Cluster size: more workgroups than CUs evens out the load (tiles are cut per segment, so their
    // number is rarely a multiple of the CU count) and halves each workgroup's chain of dependent
    // passes.  Members of a cluster are neighbours in dispatch order, so a member that is not resident
    // yet gets its slot as soon as any complete cluster retires; waits are bounded anyway.
    static int cap = 0;
    if (cap == 0) {
        int per_cu = 0, cus = 0, dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return hipErrorUnknown;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, seg_mfma_kernel, NT, 0) != hipSuccess) return hipErrorUnknown;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return hipErrorUnknown;
        cap = per_cu * cus;
    }
    int g = tuning("seg_cluster");                        // 0 auto, 1 / 2 / 4 forced
    if (g != 1 && g != 2 && g != 4) g = a.n_tiles * 2 <= cap + cap / 8 ? 2 : 1;
    while (g > 1 && (!a.xch || !a.ctrl || (int64_t)a.n_tiles * g > a.xch_blocks || (int64_t)a.n_tiles * g > 2 * (int64_t)cap)) g >>= 1;
    a.cluster = g;
    const unsigned grid = (unsigned)(((int64_t)a.n_tiles * g + 7) / 8 * 8);
    seg_mfma_kernel<<<dim3(grid), dim3(NT), 0, st>>>(a);
    return hipGetLastError();
}

}  // namespace mlora
