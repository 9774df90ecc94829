// Vector-ALU LoRA apply over plan chunks: decode (gather by slot index), packed MoE pairs and
// small-rank segments.  A chunk is up to MLORA_CHUNK rows that share one adapter (and expert):
//   shrink  h[c][j] = sum_i x[row_c, i] * A[j, i]   -- wavefront reduction, packed-bf16 dot2,
//                                                      fp32 accumulate
//   scale   h *= alpha / r
//   expand  y[row_c, o] = bf16_rne(float(y[row_c, o]) + sum_j h[c][j] * B[o, j])   in place
// Adapter rows beyond the slot's true rank are zero in the tables (padded slots), so the loops
// run to the padded rank.
//
// These launches last microseconds, so what matters is how few dependent memory round trips a
// workgroup makes: every work item issues all of its loads in one flight.  Two shapes of launch:
//   fused  one item per chunk: shrink, then expand, h stays in LDS (MoE sites, small d_in*d_out).
//   split  the chunk's work is cut into k-slices of the shrink and tiles of the expand, all in
//          ONE launch.  Shrink items publish their partial h (fp32, a few hundred bytes) through
//          a small L2-resident exchange buffer; expand items prefetch their B rows and y values,
//          then pick the partials up.  No adapter byte is read twice and a big d_in or d_out
//          spreads over many CUs.  Each word of the exchange carries value and launch tag in one
//          64-bit store, so no fences are needed; the launch grid never exceeds what the GPU
//          keeps resident and every workgroup runs its shrink items before its expand items,
//          so a waiting expand item always waits for a workgroup that is running and not waiting.
#include "internal.h"

namespace mlora {

template <int RP, int NW>
struct RowsCfg {
    static constexpr int NT  = NW * 64;
    static constexpr int JPW = RP < 8 ? RP : 8;          // A rows per wave
    static constexpr int JG  = RP / JPW;                 // groups of A rows across waves
    static constexpr int KS  = NW / JG;                  // d_in slices across waves
    static constexpr int FLU = KS * 64;                  // 16-byte units of d_in per flight
    static constexpr int CS  = JPW >= 8 ? 1 : (8 / JPW < kChunk ? 8 / JPW : kChunk);   // rows per reduction pass
    static constexpr int NV  = CS * JPW;                 // values per lane per pass (8)
    static constexpr int OPL = RP >= 8 ? 1 : 8 / RP;     // outputs per lane in the expand
    static constexpr int BV  = RP >= 8 ? RP / 8 : 1;     // 16-byte loads of B per lane
    static constexpr int TILE = RP <= 4 ? NT * OPL : (RP <= 16 ? (NW == 16 ? 2048 : 1024) : (NW == 16 ? 1024 : 512));   // outputs per expand flight
    static constexpr int EU  = TILE / (NT * OPL);        // outputs groups per lane per flight
    static_assert(JG * KS == NW && EU >= 1, "wave layout");
};

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

// Work of workgroup `wg` out of `n_wg` on one site (one launch may cover several sites).
template <int RP, int NW, bool SPLIT>
__device__ __forceinline__ void rows_body(const RowsArgs &a, const int wg, const int n_wg)
{
    using C = RowsCfg<RP, NW>;
    typedef typename YVec<C::OPL>::T yvec_t;
    __shared__ float hs[kChunk][RP];
    __shared__ float part[C::KS][kChunk][RP];
    __shared__ uint32_t s_tag;
    __shared__ int s_fail;

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int jg = w % C::JG, ks = w / C::JG;
    const int U = a.d_in >> 3;                               // 16-byte units per row of x / A
    uint64_t *prof = a.prof ? a.prof + (int64_t)wg * 8 : nullptr;
    if (prof && tid == 0) { prof[0] = wall_clock64(); prof[7] = 0; }

    // Items are numbered over the upper bound of chunks, so an item's chunk record can be fetched
    // together with the live chunk count (and the launch tag) in one round trip.
    const int n_shr = SPLIT ? a.grid_chunks * a.ksplit : 0;
    const int n_items = SPLIT ? n_shr + a.grid_chunks * a.ntiles
                              : (a.tile_par > 1 ? ((a.grid_chunks + 7) & ~7) * a.tile_par : ((a.grid_chunks + 63) & ~63));

    // Split launches carry a tag that must differ from launch to launch, also when a captured
    // graph replays the same kernel arguments, so it lives in device memory: every workgroup
    // reads it, then signs in (fire-and-forget add on one of 64 counters); the last workgroup of
    // the grid, when its own items are done, sees all sign-ins and advances the tag for the
    // next launch.  Nobody waits for an atomic's return value on the way in.
    uint32_t tag = 0;
    if (SPLIT && tid == 0) {
        s_fail = 0;
        tag = tag_read(a.ctrl);
    }
    bool first_item = true;

    for (int item = wg; item < n_items; item += n_wg) {
        // ---- which chunk, which part of it ----
        int chunk, kslice = 0, tile0 = 0, tile1 = a.ntiles;
        bool do_shrink = true, do_expand = true;
        if (SPLIT) {
            if (item < n_shr) { chunk = item / a.ksplit; kslice = item - chunk * a.ksplit; do_expand = false; }
            else { const int e = item - n_shr; chunk = e / a.ntiles; tile0 = e - chunk * a.ntiles; tile1 = tile0 + 1; do_shrink = false; }
        } else if (a.tile_par > 1) {
            // workgroups are dealt round-robin to the 8 XCDs: keep the tiles of one chunk (they all
            // read the chunk's A rows) on one XCD and its L2, and deal the chunks over the XCDs
            const int idx = item >> 3, grp8 = idx / a.tile_par;
            chunk = grp8 * 8 + (item & 7); tile0 = idx - grp8 * a.tile_par; tile1 = tile0 + 1;
            if (chunk >= a.grid_chunks) continue;
        } else {
            // neighbouring chunks can belong to one adapter (and expert): keep them on one XCD, where
            // the second chunk finds the adapter rows in L2 (workgroups are dealt round-robin to 8 XCDs)
            // (runs of 8 chunks per XCD, dealt cyclically, so the unused tail of the records spreads evenly)
            const int idx = item >> 3;
            chunk = ((idx >> 3) * 8 + (item & 7)) * 8 + (idx & 7);
            if (chunk >= a.grid_chunks) continue;
        }
        // The whole record is fetched before its count is looked at (one round trip, not two).
        const int4 *rec = (const int4 *)(a.chunks + (int64_t)chunk * kRec);
        int4 r0 = rec[0], r1 = rec[1];
        asm volatile("" : "+v"(r0.x), "+v"(r0.y), "+v"(r1.x), "+v"(r1.y), "+v"(r1.z), "+v"(r1.w));
        const int key = __builtin_amdgcn_readfirstlane(r0.x), cnt = __builtin_amdgcn_readfirstlane(r0.y);
        int row[kChunk];
        row[0] = __builtin_amdgcn_readfirstlane(r1.x); row[1] = __builtin_amdgcn_readfirstlane(r1.y);
        row[2] = __builtin_amdgcn_readfirstlane(r1.z); row[3] = __builtin_amdgcn_readfirstlane(r1.w);
        if (SPLIT && first_item) {
            if (tid == 0) {
                s_tag = tag;
                tag_sign_in(a.ctrl, wg, tag);
            }
            __syncthreads();
            tag = s_tag;
        }
        if (cnt <= 0) { first_item = false; continue; }            // record past the live chunks of this batch
#pragma unroll
        for (int c = 1; c < kChunk; ++c) row[c] = c < cnt ? row[c] : row[0];
        static_assert(kChunk == 4 && kRec == 8, "record layout: two 16-byte loads");
        const int slot = key / a.n_experts;
        // rank and scale are only consumed after the flight has landed (an early exit on an empty
        // slot would let the compiler order every load of the item behind these two reads)
        // They are fetched as per-lane data (the lane offset is an opaque zero): a value the
        // compiler knows to be wave-uniform is moved to a scalar register as soon as it is loaded,
        // which would put a wait for these two reads in front of the flight.
        int lane_zero;
        asm volatile("v_mov_b32 %0, 0" : "=v"(lane_zero));
        const int rank = a.meta.rank[slot + lane_zero];
        const float scale = a.meta.scale[slot + lane_zero];

        // ---- one flight: every load of this item is issued here ----
        const uint16_t *Bg = a.b_tab + (int64_t)key * a.d_out * RP;
        uint16_t *yrow[kChunk];
#pragma unroll
        for (int c = 0; c < kChunk; ++c) yrow[c] = a.y + (int64_t)row[c] * a.ldy;
        uint4 braw[C::EU][C::BV];
        yvec_t yraw[C::EU][kChunk];
        auto load_tile = [&](int t) {
            const int lo = t * C::TILE;
#pragma unroll
            for (int e = 0; e < C::EU; ++e) {
                const int o = lo + (e * C::NT + tid) * C::OPL;
                const int oc = o < a.d_out ? o : 0;               // clamped address, result unused
#pragma unroll
                for (int q = 0; q < C::BV; ++q) braw[e][q] = ((const uint4 *)(Bg + (int64_t)oc * RP))[q];
#pragma unroll
                for (int c = 0; c < kChunk; ++c)
                    if (c < cnt) yraw[e][c] = *(const yvec_t *)(yrow[c] + oc);
            }
        };
        const int u_lo = SPLIT ? kslice * a.kslice_units : 0;
        const int u_hi = SPLIT ? min(U, u_lo + a.kslice_units) : U;
        const uint4 *Ag = (const uint4 *)(a.a_tab + (int64_t)key * RP * a.d_in + (int64_t)(jg * C::JPW) * a.d_in);
        const uint4 *xp[kChunk];
#pragma unroll
        for (int c = 0; c < kChunk; ++c) xp[c] = (const uint4 *)(a.x + (int64_t)(row[c] / a.top_k) * a.ldx);
        uint4 av[C::JPW], xv[kChunk];
        auto load_flight = [&](int f) {
            const int u = f + ks * 64 + lane;
            const int uc = u < u_hi ? u : u_lo;
#pragma unroll
            for (int jj = 0; jj < C::JPW; ++jj) av[jj] = Ag[(int64_t)jj * U + uc];
#pragma unroll
            for (int c = 0; c < kChunk; ++c)
                if (c < cnt) xv[c] = xp[c][uc];
        };
        if (do_shrink) load_flight(u_lo);
        if (do_expand) load_tile(tile0);
        if (prof && tid == 0 && first_item) { prof[1] = wall_clock64(); prof[7] = cnt + 100 * (do_shrink ? 1 : 0) + 1000 * (do_expand ? 1 : 0); }

        // ---- shrink over this item's range of d_in ----
        if (do_shrink) {
            bool first = true;
            for (int f = u_lo; f < u_hi; f += C::FLU) {
                if (f > u_lo) load_flight(f);
                const bool in = f + ks * 64 + lane < u_hi;
#pragma unroll
                for (int c0 = 0; c0 < kChunk; c0 += C::CS) {
                    if (c0 >= cnt) break;
                    float acc[C::NV];
#pragma unroll
                    for (int i = 0; i < C::NV; ++i) acc[i] = 0.f;
#pragma unroll
                    for (int c = 0; c < C::CS; ++c) {
                        if (c0 + c < cnt) {
                            const uint4 xz = in ? xv[c0 + c] : make_uint4(0, 0, 0, 0);
#pragma unroll
                            for (int jj = 0; jj < C::JPW; ++jj) acc[c * C::JPW + jj] = dot8(xz, av[jj], 0.f);
                        }
                    }
                    wave_sum_transpose<C::NV>(acc, lane);
                    if (lane < C::NV) {
                        const int idx = bitrev<Log2<C::NV>::v>(lane);
                        const int c = c0 + idx / C::JPW, j = jg * C::JPW + idx % C::JPW;
                        part[ks][c][j] = first ? acc[0] : part[ks][c][j] + acc[0];
                    }
                }
                first = false;
            }
            if (prof && tid == 0 && first_item) prof[2] = wall_clock64();
            __syncthreads();
            if (tid < kChunk * RP) {
                const int c = tid / RP, j = tid % RP;
                float s = 0.f;
#pragma unroll
                for (int k = 0; k < C::KS; ++k) s += part[k][c][j];
                if (SPLIT) {
                    if (c < cnt) xch_put(a.xch + ((int64_t)(chunk * a.ksplit + kslice) * kChunk + c) * RP + j, s, tag);
                } else {
                    hs[c][j] = s * scale;
                }
            }
            __syncthreads();
        } else {
            // ---- pick up the partial shrink results of every k-slice, summed in slice order ----
            bool ok = true;
            if (tid < kChunk * RP) {
                const int c = tid / RP, j = tid % RP;
                float s = 0.f;
                if (c < cnt) {
                    const uint64_t *src = a.xch + ((int64_t)(chunk * a.ksplit) * kChunk + c) * RP + j;
                    for (int k0 = 0; k0 < a.ksplit; k0 += 4) {        // four words in flight at a time
                        uint64_t wv[4];
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            if (k0 + k < a.ksplit) wv[k] = xch_get(src + (int64_t)(k0 + k) * kChunk * RP);
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            if (k0 + k < a.ksplit) {
                                int spins = 0;
                                while ((uint32_t)(wv[k] >> 32) != tag) {
                                    if (++spins > kSpinLimit) { ok = false; break; }
                                    __builtin_amdgcn_s_sleep(1);
                                    wv[k] = xch_get(src + (int64_t)(k0 + k) * kChunk * RP);
                                }
                                s += __uint_as_float((uint32_t)wv[k]);
                            }
                        }
                    }
                }
                hs[c][j] = s * scale;
            }
            if (!ok) s_fail = 1;
            __syncthreads();
            if (s_fail) {                                         // never seen in a healthy launch
                if (tid == 0) __hip_atomic_store(a.ctrl + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
        }
        if (prof && tid == 0 && first_item) prof[3] = wall_clock64();

        // ---- expand + in-place add ----
        if (do_expand) {
            for (int t = tile0; t < tile1; ++t) {
                if (t > tile0) load_tile(t);
                const int lo = t * C::TILE;
#pragma unroll
                for (int e = 0; e < C::EU; ++e) {
                    // hs is re-read for every output group: keeping all of it in registers across
                    // groups costs more registers than the LDS reads cost time
                    asm volatile("" ::: "memory");
                    const int o = lo + (e * C::NT + tid) * C::OPL;
                    // bf[q*RP + j]: B value of output q of this lane; for RP >= 8 there is one output
                    float bf[C::BV * 8];
#pragma unroll
                    for (int q = 0; q < C::BV; ++q) {
                        bf[q * 8 + 0] = bf_lo(braw[e][q].x); bf[q * 8 + 1] = bf_hi(braw[e][q].x);
                        bf[q * 8 + 2] = bf_lo(braw[e][q].y); bf[q * 8 + 3] = bf_hi(braw[e][q].y);
                        bf[q * 8 + 4] = bf_lo(braw[e][q].z); bf[q * 8 + 5] = bf_hi(braw[e][q].z);
                        bf[q * 8 + 6] = bf_lo(braw[e][q].w); bf[q * 8 + 7] = bf_hi(braw[e][q].w);
                    }
#pragma unroll
                    for (int c = 0; c < kChunk; ++c) {
                        if (c < cnt && o < a.d_out && rank > 0) {     // empty slot: rows stay untouched
                            float yf[C::OPL];
                            y_unpack(yraw[e][c], yf);
#pragma unroll
                            for (int q = 0; q < C::OPL; ++q) {
                                float d = 0.f;
#pragma unroll
                                for (int j = 0; j < RP; ++j) d = fmaf(hs[c][j], bf[q * RP + j], d);
                                yf[q] += d;
                            }
                            yvec_t out;
                            y_pack(yf, out);
                            *(yvec_t *)(yrow[c] + o) = out;
                        }
                    }
                }
            }
            __syncthreads();                                      // hs is rewritten by the next item
        }
        if (prof && tid == 0 && first_item) prof[4] = wall_clock64();
        first_item = false;
    }

    // ---- tag bookkeeping ----
    if (SPLIT) {
        if (first_item && tid == 0) tag_sign_in(a.ctrl, wg, tag);   // a workgroup without items still signs in
        if (wg == n_wg - 1 && w == 0) {
            if (!first_item) tag = s_tag;
            else tag = __shfl(tag, 0, 64);
            tag_advance(a.ctrl, n_wg, tag, lane);
        }
    }
}

template <int RP, int NW, bool SPLIT>
__global__ __launch_bounds__(NW * 64, (NW >= 8 && RP <= 16) ? 4 : 1)
void rows_kernel(const RowsArgs a)
{
    rows_body<RP, NW, SPLIT>(a, (int)blockIdx.x, (int)gridDim.x);
}

// Several sites that share a batch plan in one launch (q/k/v of one layer, or gate/up): site s owns
// workgroups [first[s], first[s + 1]).  Only fused launches are grouped; nothing crosses workgroups.
struct MultiArgs {
    int32_t n;
    int32_t first[kMaxMulti + 1];
    RowsArgs site[kMaxMulti];
};

template <int RP, int NW>
__global__ __launch_bounds__(NW * 64, (NW >= 8 && RP <= 16) ? 4 : 1)
void rows_multi_kernel(const MultiArgs m)
{
    const int b = (int)blockIdx.x;
    int s = 0;
#pragma unroll
    for (int k = 1; k < kMaxMulti; ++k) s += (k < m.n && b >= m.first[k]) ? 1 : 0;
    rows_body<RP, NW, false>(m.site[s], b - m.first[s], m.first[s + 1] - m.first[s]);
}

template <int RP, int NW, bool SPLIT>
static int rows_capacity()
{
    static int cap = 0;
    if (cap == 0) {
        int per_cu = 0, cus = 0, dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, rows_kernel<RP, NW, SPLIT>, NW * 64, 0) != hipSuccess) return 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cap = per_cu * cus;
    }
    return cap;
}

template <int RP, int NW>
static hipError_t launch_rp(RowsArgs a, hipStream_t st)
{
    using C = RowsCfg<RP, NW>;
    const int U = a.d_in >> 3;
    const int ntiles = (a.d_out + C::TILE - 1) / C::TILE;
    const int ksplit = (U + C::FLU - 1) / C::FLU;
    a.ntiles = ntiles;
    const bool can_split = a.xch && a.ctrl && a.grid_chunks <= a.xch_chunks && ksplit <= 8 && ksplit * RP <= 128;
    const int mode = tuning("rows_mode");                 // 0 auto, 1 fused, 2 split, 3 fused with one tile per item
    bool split = can_split && ksplit > 1;                 // d_in needs several flights: cut it across workgroups
    if (mode == 1 || mode == 3) split = false;
    if (mode == 2) split = can_split;
    if (split) {
        const int cap = rows_capacity<RP, NW, true>();
        if (cap <= 0) return hipErrorUnknown;
        a.mode = 1;
        a.ksplit = ksplit;
        a.kslice_units = (U + ksplit - 1) / ksplit;
        int64_t items = (int64_t)a.grid_chunks * (ksplit + ntiles);
        if (items > cap) items = cap;                     // every workgroup resident: waits always end
        rows_kernel<RP, NW, true><<<dim3((unsigned)items), dim3(NW * 64), 0, st>>>(a);
    } else {
        a.mode = 0; a.ksplit = 1; a.kslice_units = U;
        a.tile_par = (mode == 3 || (mode == 0 && ksplit == 1 && a.n_experts == 1)) ? ntiles : 1;
        const unsigned grid = a.tile_par > 1 ? (unsigned)(((a.grid_chunks + 7) & ~7) * a.tile_par) : (unsigned)((a.grid_chunks + 63) & ~63);
        rows_kernel<RP, NW, false><<<dim3(grid), dim3(NW * 64), 0, st>>>(a);
    }
    return hipGetLastError();
}

template <int RP>
static hipError_t launch_nw(const RowsArgs &a, hipStream_t st)
{
    const int U = a.d_in >> 3;
    int nw = tuning("rows_waves");
    if (nw != 4 && nw != 8 && nw != 16) {
        // 16 waves when one flight of them covers all of d_in (then every item is shrink + one tile,
        // nothing crosses workgroups); else 8, or 4 when 8 would be mostly idle lanes
        nw = U >= RowsCfg<RP, 8>::FLU * 3 / 4 ? 8 : 4;
        if constexpr (RP >= 8 && RP <= 16) {
            if (a.n_experts == 1 && U > RowsCfg<RP, 8>::FLU && U <= RowsCfg<RP, 16>::FLU) nw = 16;
        }
    }
    if constexpr (RP >= 64) nw = 8;
    if constexpr (RP >= 8 && RP <= 16) { if (nw == 16) return launch_rp<RP, 16>(a, st); }
    if (nw >= 8) return launch_rp<RP, 8>(a, st);
    if constexpr (RP < 64) return launch_rp<RP, 4>(a, st);
    return hipErrorInvalidValue;
}

// Fill in the fused-launch fields of one site; returns its number of workgroups.
template <int RP, int NW>
static int prepare_fused(RowsArgs &a)
{
    using C = RowsCfg<RP, NW>;
    const int U = a.d_in >> 3;
    a.ntiles = (a.d_out + C::TILE - 1) / C::TILE;
    a.mode = 0; a.ksplit = 1; a.kslice_units = U;
    a.tile_par = a.n_experts == 1 ? a.ntiles : 1;
    return a.tile_par > 1 ? ((a.grid_chunks + 7) & ~7) * a.tile_par : ((a.grid_chunks + 63) & ~63);
}

template <int RP>
static hipError_t launch_multi_rp(const RowsArgs *sites, int n, hipStream_t st)
{
    MultiArgs m;
    m.n = n;
    m.first[0] = 0;
    for (int k = 0; k < n; ++k) {
        m.site[k] = sites[k];
        m.first[k + 1] = m.first[k] + prepare_fused<RP, 16>(m.site[k]);
    }
    for (int k = n; k < kMaxMulti; ++k) { m.site[k] = sites[0]; m.first[k + 1] = m.first[n]; }
    rows_multi_kernel<RP, 16><<<dim3((unsigned)m.first[n]), dim3(16 * 64), 0, st>>>(m);
    return hipGetLastError();
}

// Sites can share a launch when each of them alone would run the 16-wave fused shape.
bool rows_can_group(const RowsArgs &a)
{
    if (a.r_pad != 8 && a.r_pad != 16) return false;
    const int U = a.d_in >> 3;
    const int flu8 = a.r_pad == 8 ? RowsCfg<8, 8>::FLU : RowsCfg<16, 8>::FLU;
    const int flu16 = a.r_pad == 8 ? RowsCfg<8, 16>::FLU : RowsCfg<16, 16>::FLU;
    return a.n_experts == 1 && U > flu8 && U <= flu16 && !tuning("rows_mode") && !tuning("rows_waves");
}

hipError_t launch_rows_multi(const RowsArgs *sites, int n, hipStream_t st)
{
    if (n < 1 || n > kMaxMulti) return hipErrorInvalidValue;
    for (int k = 0; k < n; ++k)
        if (sites[k].r_pad != sites[0].r_pad || !rows_can_group(sites[k])) return hipErrorInvalidValue;
    if (sites[0].grid_chunks <= 0) return hipSuccess;
    return sites[0].r_pad == 8 ? launch_multi_rp<8>(sites, n, st) : launch_multi_rp<16>(sites, n, st);
}

hipError_t launch_rows(const RowsArgs &a, hipStream_t st)
{
    if (a.grid_chunks <= 0) return hipSuccess;
    switch (a.r_pad) {
        case 1:  return launch_nw<1>(a, st);
        case 2:  return launch_nw<2>(a, st);
        case 4:  return launch_nw<4>(a, st);
        case 8:  return launch_nw<8>(a, st);
        case 16: return launch_nw<16>(a, st);
        case 32: return launch_nw<32>(a, st);
        case 64: return launch_nw<64>(a, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace mlora
