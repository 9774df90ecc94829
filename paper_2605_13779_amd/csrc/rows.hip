// LoRA apply over plan chunks: decode (gather by slot index), packed MoE pairs and small-rank
// segments.  Vector ALU, with the expand of padded ranks 8 and 16 on 4x4x4 matrix-core blocks.  A chunk is up to MLORA_CHUNK rows that share one adapter (and expert):
//   shrink  h[c][j] = sum_i x[row_c, i] * A[j, i]   -- wavefront reduction, packed-bf16 dot2,
//                                                      fp32 accumulate
//   scale   h *= alpha / r
//   expand  y[row_c, o] = bf16_rne(float(y[row_c, o]) + sum_j h[c][j] * B[o, j])   in place
// Adapter rows beyond the slot's true rank are zero in the tables (padded slots), so the loops
// run to the padded rank; big launches over tables with padded slots skip the reads of those rows of A.
//
// These launches last microseconds, so what matters is how few dependent memory round trips a
// workgroup makes: every work item issues its loads in one flight.  Two shapes of launch:
//   one item per chunk   shrink, then expand, h stays in LDS (MoE sites, rank-1 sites, and dense
//                        launches that have enough chunks to fill the GPU).
//   chunk parts          a dense launch with fewer chunks than the GPU has CUs cuts every chunk
//                        into parts.  Part p shrinks k-slice p of d_in and expands its own range of
//                        outputs; the parts trade their partial h (fp32, a few hundred bytes)
//                        through a small L2-resident exchange buffer, while the B rows and y
//                        values of the expand are already on their way.  No adapter byte is read
//                        twice and a big d_in or d_out spreads over many CUs.  Each word of the
//                        exchange carries value and launch tag in one 64-bit store, so no fences
//                        are needed; a part whose partners have not published after a bounded
//                        number of polls takes its item again on its own, with the whole shrink.
#include "plan_device.h"
#include "wave_ops.h"

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
    static constexpr bool MX0 = (RP == 8 || RP == 16) && kChunk == 4;
    static constexpr int TILE = RP <= 4 ? NT * OPL : (RP <= 16 ? ((MX0 && NW == 8) ? 512 : 1024) : 512);   // outputs per expand tile
    static constexpr int DEPTH = (MX0 && NW == 8) ? 2 : 1;   // expand tiles kept in flight by an item that walks several
    static constexpr int EU  = TILE / (NT * OPL);        // outputs groups per lane per flight
    // The expand of a 4-row chunk is a small dense contraction (4 x RP times RP x 64 per wave and
    // output group); on the vector ALU it costs 4 * RP multiply-adds per lane and was what bounded
    // these kernels.  For RP = 8 and 16 it runs on the matrix cores instead: the 4x4x4 bf16 MFMA
    // works on 16 independent 4x4 blocks, lane l = (block l/4, column l%4), so lane l's result
    // column is its own output and its four accumulator registers are the chunk's four rows.
    static constexpr bool MX = (RP == 8 || RP == 16) && kChunk == 4;
    // Every row of x (and y) of a chunk is loaded whatever its count: fewer, emptier loads lost time in
    // the 8-wave decode kernels of rank 8 / 16 and won it everywhere else (load issue is what they save).
    static constexpr bool ALLROWS = MX && NW == 8;
    static_assert(JG * KS == NW && EU >= 1, "wave layout");
};

// Calls f(std::integral_constant<int, 0>) ... f(std::integral_constant<int, N - 1>): a loop whose
// index is a compile-time constant inside the body (register arrays stay in registers).
template <int N, int I = 0, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(IntC<I>{});
        static_for<N, I + 1>(f);
    }
}

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
// XCH: the kernel can pass partial shrink results between workgroups (a.mode 2).
// RI: the launch has no plan; item i is row i and its slot is a.row_slot[i] (rank 1 and 2 only).
// RUN: one item per chunk -- 1 << RUN consecutive chunks go to one XCD (3 everywhere; one instantiation
// with longer runs exists for measurements, see rows_multi_kernel).
template <int RP, int NW, bool XCH, bool RI = false, int RUN = 3>
__device__ __forceinline__ void rows_body(const RowsArgs &a, const int wg, const int n_wg, const int32_t *lrec = nullptr)
{
    static_assert(!RI || (!XCH && RP <= 2), "row items: small ranks, nothing traded");
    using C = RowsCfg<RP, NW>;
    typedef typename YVec<C::OPL>::T yvec_t;
    __shared__ __attribute__((aligned(16))) float hs[kChunk][RP];
    __shared__ float part[C::KS][kChunk][RP];
    __shared__ uint32_t s_tag;
    __shared__ uint32_t s_missing;

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int jg = w % C::JG, ks = w / C::JG;
    const int U = a.d_in >> 3;                               // 16-byte units per row of x / A
#ifdef MLORA_PROF
    uint64_t *prof = a.prof ? a.prof + (int64_t)wg * 8 : nullptr;     // per-phase timestamps (profiling builds)
#else
    constexpr uint64_t *prof = nullptr;                              // the stamps below compile away
#endif
    if (prof && tid == 0) { prof[0] = wall_clock64(); prof[7] = 0; }

    const bool use_x = XCH && a.mode != 0;                   // this site's items exchange partial results
    // Items are numbered over the upper bound of chunks, so an item's chunk record can be fetched
    // together with the live chunk count (and the launch tag) in one round trip.
    constexpr int kRunMask = (8 << RUN) - 1;                   // chunks per XCD run times 8 XCDs, minus one
    const int n_items = a.tile_par > 1 ? ((a.grid_chunks + 7) & ~7) * a.tile_par : ((a.grid_chunks + kRunMask) & ~kRunMask);

    // Launches that exchange carry a tag that must differ from launch to launch, also when a
    // captured graph replays the same kernel arguments, so it lives in device memory: every
    // workgroup reads it, then signs in (fire-and-forget add on one of 64 counters); the last
    // workgroup of the grid, when its own items are done, sees all sign-ins and advances the tag
    // for the next launch.  Nobody waits for an atomic's return value on the way in.
    uint32_t tag = 0;
    if (XCH && tid == 0) {
        s_missing = 0;
        if (use_x) tag = tag_read(a.ctrl);
    }
    bool first_item = true;
    // An item is taken a second time only after a bounded wait for another workgroup's partial sums
    // has given up: it then runs on its own, with the whole shrink.
    bool solo_next = false;

    for (int item = wg; item < n_items; item += n_wg) {
        // Per-item copies of the thread's coordinates: what is derived from them (LDS addresses, lane
        // masks) is recomputed in each item instead of being kept, and spilled, across the whole loop;
        // a reload of such a spill would wait for every load of the item that is still in flight.
        int tid_item = (int)threadIdx.x;
        asm volatile("" : "+v"(tid_item));
        const int tid = tid_item, w = tid >> 6, lane = tid & 63;
        const int jg = w % C::JG, ks = w / C::JG;
        // ---- which chunk, which part of it ----
        int chunk, kslice = 0, out0 = 0, out1 = a.d_out;
        // The first launch of the MoE down projection only shrinks (a.h_out); it comes here for padded ranks
        // above 16 only, so the kernels of the smaller ranks do not carry that mode.
        constexpr bool HMODE = RP >= 32 && !XCH && !RI;
        const bool h_only = HMODE && a.h_out != nullptr;
        bool do_shrink = true, do_expand = !h_only;
        int part_i = 0;
        if (a.tile_par > 1) {
            // workgroups are dealt round-robin to the 8 XCDs: keep the parts of one chunk (they share
            // the chunk's rows of x and its exchange words) on one XCD and its L2, and deal the chunks
            // over the XCDs
            const int idx = item >> 3, grp8 = idx / a.tile_par;
            part_i = idx - grp8 * a.tile_par;
            chunk = grp8 * 8 + (item & 7);
            out0 = part_i * a.out_per_part; out1 = min(a.d_out, out0 + a.out_per_part);
            do_expand = out0 < out1 && !h_only;
            if (chunk >= a.grid_chunks) continue;
        } else {
            // neighbouring chunks can belong to one adapter (and expert): keep them on one XCD, where
            // the second chunk finds the adapter rows in L2 (workgroups are dealt round-robin to 8 XCDs)
            // (runs of 8 chunks per XCD, dealt cyclically, so the unused tail of the records spreads evenly)
            const int idx = item >> 3;
            chunk = ((idx >> RUN) * 8 + (item & 7)) * (1 << RUN) + (idx & ((1 << RUN) - 1));
            if (chunk >= a.grid_chunks) continue;
        }
        // The whole record is fetched before its count is looked at (one round trip, not two).
        // (a launch that planned for itself has the records in LDS)
        int4 r0, r1;
        uint4 x_early = make_uint4(0, 0, 0, 0);
        if constexpr (RI) {
            // Ungrouped launch of a rank-1 / rank-2 site: item = row, no plan.  Grouping rows by slot
            // saves at most one or two adapter rows per row there, less than a planner launch costs.
            const int sl = a.row_slot[chunk];
            // The row's x does not depend on its slot: it is requested behind the slot read, before its
            // value is looked at, and travels while it is awaited.  (y does not depend on it either, but
            // is needed last: requested early as well it only queues in front of the adapter's rows --
            // 7.05 us per launch at 512 rows of 4096 against 6.88 us; with x late too 7.53 us.)
            const int u = ks * 64 + lane;                    // this lane's unit of the first shrink flight
            x_early = *(const uint4 *)((const char *)(a.x + (int64_t)chunk * a.ldx) + (uint32_t)(u < U ? u : 0) * 16u);
            r0 = make_int4(sl, (sl >= 0 && sl < a.row_slots) ? 1 : 0, 0, 0);
            r1 = make_int4(chunk, chunk, chunk, chunk);
        } else {
            const int4 *rec = lrec ? (const int4 *)(lrec + chunk * kRec) : (const int4 *)(a.chunks + (int64_t)chunk * kRec);
            r0 = rec[0]; r1 = rec[1];
        }
        asm volatile("" : "+v"(r0.x), "+v"(r0.y), "+v"(r1.x), "+v"(r1.y), "+v"(r1.z), "+v"(r1.w));
        const int key = __builtin_amdgcn_readfirstlane(r0.x), cnt = __builtin_amdgcn_readfirstlane(r0.y);
        int row[kChunk];
        row[0] = __builtin_amdgcn_readfirstlane(r1.x); row[1] = __builtin_amdgcn_readfirstlane(r1.y);
        row[2] = __builtin_amdgcn_readfirstlane(r1.z); row[3] = __builtin_amdgcn_readfirstlane(r1.w);
        if (prof && tid == 0 && first_item) prof[5] = wall_clock64();      // the chunk record has arrived
        if (XCH && first_item) {
            if (tid == 0) {
                s_tag = tag;
                if (use_x) tag_sign_in(a.ctrl, wg, tag);
            }
            __syncthreads();
            tag = s_tag;
        }
        if (prof && tid == 0 && first_item) prof[6] = wall_clock64();      // ... and the launch tag
        if (cnt <= 0) { first_item = false; continue; }            // record past the live chunks of this batch
        // An item runs on its own (whole shrink, nothing published or awaited) when its bounded wait
        // has just given up, or when an earlier launch's give-up has switched the exchange off.
        const bool solo = solo_next || (XCH && tag == kTagPoison);
        solo_next = false;
        if (a.tile_par > 1 && use_x && !solo) { kslice = part_i; do_shrink = part_i < a.ksplit; }   // else every part does the whole shrink
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
        int rank;                  // (requested behind the shrink's operands, which are wanted first)
        float scale;

        const bool xitem = use_x && !solo;
        // ---- one flight: every load of this item is issued here ----
        const uint16_t *Bg = a.b_tab + (int64_t)key * a.d_out * RP;
        // MoE down projection, first launch: no expand here; the chunk's scaled h, times the row's
        // routing weight, goes to a.h_out (the weights travel with the flight)
        uint16_t *yrow[kChunk];
        float wrow[kChunk];
#pragma unroll
        for (int c = 0; c < kChunk; ++c) {
            yrow[c] = a.y + (int64_t)row[c] * a.ldy;
            if constexpr (HMODE) wrow[c] = h_only ? a.row_w[row[c] + lane_zero] : 1.f;
        }
        // Matrix-core expand: the result comes out with lane l holding row l%4 of the chunk and the four
        // outputs of its block (see below), so a lane reads and writes 8 contiguous bytes of its own row:
        // one 64-lane access covers 128 contiguous bytes of each of the four rows.
        const int r4 = lane & 3;
        const int my_row = r4 == 0 ? row[0] : (r4 == 1 ? row[1] : (r4 == 2 ? row[2] : row[3]));
        char *const y_lane = (char *)(a.y + (int64_t)my_row * a.ldy);
        uint4 braw[C::DEPTH][C::EU][C::BV];
        yvec_t yraw[C::DEPTH][C::EU][C::MX ? 1 : kChunk];
        uint2 yq[C::DEPTH][C::EU];
        auto load_tile = [&](int lo, auto dconst, auto first_c) {      // first_c: the item's first tile
            constexpr int d = decltype(dconst)::value;
            (void)first_c;
#pragma unroll
            for (int e = 0; e < C::EU; ++e) {
                const int o = lo + (e * C::NT + tid) * C::OPL;
                const uint32_t oc = o < out1 ? (uint32_t)o : 0u;  // clamped address, result unused
                // uniform 64-bit base + 32-bit per-lane byte offset: no 64-bit address registers per lane
#pragma unroll
                for (int q = 0; q < C::BV; ++q) braw[d][e][q] = *(const uint4 *)((const char *)Bg + (oc * (uint32_t)(RP * 2) + (uint32_t)(q * 16)));
                {
                    if constexpr (C::MX) {
                        yq[d][e] = *(const uint2 *)(y_lane + (oc & ~3u) * 2u);
                    } else {
#pragma unroll
                        for (int c = 0; c < kChunk; ++c) {  // rows past the chunk's count are not fetched
                            if (C::ALLROWS || c == 0 || c < cnt) yraw[d][e][c] = *(const yvec_t *)((const char *)yrow[c] + oc * 2u);
                        }
                    }
                }
            }
        };
        const uint32_t a_row_bytes = (uint32_t)a.d_in * 2u;
        const char *Ag = (const char *)(a.a_tab + (int64_t)key * RP * a.d_in);
        uint32_t a_row_off[C::JPW];
        if constexpr (XCH) {
            Ag += (int64_t)(jg * C::JPW) * a_row_bytes;
#pragma unroll
            for (int jj = 0; jj < C::JPW; ++jj) a_row_off[jj] = (uint32_t)jj * a_row_bytes;
        } else {
            // Rank-bounded reads (slots of different true rank in one padded table): rows of A past
            // the slot's rank are not fetched.  The wave that would have read them reads the slot's
            // last real row again (a cache hit, every load is still issued), and what it computes
            // from that row meets the zero columns of B in the expand.
            int a_last = RP - 1;
            if (a.rank_bound) a_last = min(max(__builtin_amdgcn_readfirstlane(a.meta.rank[slot]), 1), RP) - 1;
            const int a_j0 = __builtin_amdgcn_readfirstlane(jg * C::JPW);
#pragma unroll
            for (int jj = 0; jj < C::JPW; ++jj) a_row_off[jj] = (uint32_t)min(a_j0 + jj, a_last) * a_row_bytes;
        }
        const uint4 *xp[kChunk];
#pragma unroll
        for (int c = 0; c < kChunk; ++c) xp[c] = (const uint4 *)(a.x + (int64_t)(row[c] / a.top_k) * a.ldx);
        uint4 av[C::JPW], xv[kChunk];
        auto load_flight = [&](int f, int ul, int uh, auto first_c) {  // first_c: the item's first flight (row items have its x already)
            constexpr bool early = RI && decltype(first_c)::value != 0;
            const int u = f + ks * 64 + lane;
            const uint32_t ub = (uint32_t)(u < uh ? u : ul) * 16u;
            // The waves past the end of the range issue nothing (a k-slice of an exchange item is often
            // one wave wide, and the last flight of a long shrink is partial).  A CU accepts one 64-lane
            // 16-byte load per 16 cycles whatever the lanes fetch, and clamped loads took more of that
            // than the item's real bytes.  (Not in the 4-wave kernels: their ranges fill the workgroup,
            // and the branch alone measured slower there.)
            if constexpr (XCH || NW == 8) {
                if (__builtin_amdgcn_readfirstlane(f + ks * 64) >= uh) {
#pragma unroll
                    for (int jj = 0; jj < C::JPW; ++jj) av[jj] = make_uint4(0, 0, 0, 0);
#pragma unroll
                    for (int c = 0; c < kChunk; ++c) xv[c] = make_uint4(0, 0, 0, 0);
                    return;
                }
            }
#pragma unroll
            for (int jj = 0; jj < C::JPW; ++jj) av[jj] = *(const uint4 *)(Ag + (size_t)a_row_off[jj] + ub);
            // Rows past the chunk's count are not fetched, except in the 8-wave matrix-core kernels (ALLROWS;
            // measured).  The count is wave-uniform and the tile loads that follow are unconditional, so
            // the waits for these loads keep a known number in flight.
#pragma unroll
            for (int c = 0; c < kChunk; ++c) {
                if (early && c == 0) xv[c] = x_early;
                else if (C::ALLROWS || c == 0 || c < cnt) xv[c] = *(const uint4 *)((const char *)xp[c] + ub);
            }
        };
        // Tiles 1 .. DEPTH-1 of the expand are requested once the shrink's operands have been consumed
        // (their registers are free then) and travel while the partial sums are reduced and traded.
        auto load_more_tiles = [&]() {
            static_for<C::DEPTH>([&](auto dc) {
                if constexpr (decltype(dc)::value >= 1) { if (out0 + dc.value * C::TILE < out1) load_tile(out0 + dc.value * C::TILE, dc, IntC<0>{}); }
            });
        };
        // Shrink over the units [ul, uh) of d_in.  Returns, in thread c * RP + j, the sum for row c
        // of the chunk and adapter row j (other threads: 0).
        auto shrink_units = [&](int ul, int uh, bool then_tiles) -> float {
            bool first = true;
            for (int f = ul; f < uh; f += C::FLU) {
                if (f > ul) load_flight(f, ul, uh, IntC<0>{});
                const bool in = f + ks * 64 + lane < uh;
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
            if (then_tiles) {
                if constexpr (C::MX) load_tile(out0, IntC<0>{}, IntC<1>{});            // (see kTilesBehindShrink)
                load_more_tiles();
            }
            __syncthreads();
            float s = 0.f;
            if (tid < kChunk * RP && tid / RP < cnt) {
#pragma unroll
                for (int k = 0; k < C::KS; ++k) s += part[k][tid / RP][tid % RP];
            }
            __syncthreads();                                      // part may be written again
            return s;
        };
        const int u_lo = solo ? 0 : kslice * a.kslice_units, u_hi = solo ? U : min(U, u_lo + a.kslice_units);
        if (do_shrink) load_flight(u_lo, u_lo, u_hi, IntC<1>{});
        rank = a.meta.rank[slot + lane_zero];
        scale = a.meta.scale[slot + lane_zero];
        // The first expand tile travels with the shrink operands -- except in the kernels of ranks 8 and
        // 16 (matrix-core expand), where it leaves with the later tiles once the shrink's operands have
        // been consumed: the item's first flight is what its whole chain waits for, a wave gets its loads
        // back in the order it issued them, and the tile's rows of B and y are not needed before the
        // partial sums have been reduced (and traded) (c2 layer step 65.05 -> 64.0 us; packed MoE gate+up
        // 97.9 -> 97.3 us).
        constexpr bool kTilesBehindShrink = C::MX;
        if (do_expand && !(kTilesBehindShrink && do_shrink)) {
            load_tile(out0, IntC<0>{}, IntC<1>{});
            if (!do_shrink) load_more_tiles();
        }
        if (prof && tid == 0 && first_item) { prof[1] = wall_clock64(); prof[7] = cnt + 100 * (do_shrink ? 1 : 0) + 1000 * (do_expand ? 1 : 0); }

        // ---- shrink over this item's range of d_in ----
        float own = 0.f;
        if (do_shrink) own = shrink_units(u_lo, u_hi, do_expand);
        if (prof && tid == 0 && first_item) prof[2] = wall_clock64();
        const int hc = tid / RP, hj = tid % RP;                   // this thread's element of h (tid < kChunk * RP)
        const bool h_thread = tid < kChunk * RP && hc < cnt;
        if (!xitem) {
            if (tid < kChunk * RP) hs[hc][hj] = own * scale;
            if constexpr (HMODE) if (h_only) {
                // weighted, scaled h of row hc as a bf16 head (truncated) and tail (rounded) in one word:
                // 16 bits of it reach the matrix cores of the second launch; rows of an empty slot are skipped there too
                if (h_thread && rank > 0) {
                    const float f = own * scale * (hc == 0 ? wrow[0] : (hc == 1 ? wrow[1] : (hc == 2 ? wrow[2] : wrow[3])));
                    const int hrow = hc == 0 ? row[0] : (hc == 1 ? row[1] : (hc == 2 ? row[2] : row[3]));
                    const uint32_t hi = __float_as_uint(f) & 0xffff0000u;
                    a.h_out[(int64_t)hrow * RP + hj] = (hi >> 16) | (f2bf(f - __uint_as_float(hi)) << 16);
                }
            }
            __syncthreads();
        } else {
            uint64_t *xw = a.xch + ((int64_t)(chunk * a.ksplit) * kChunk + hc) * RP + hj;   // + k * kChunk * RP: slice k
            if (do_shrink && h_thread) xch_put(xw + (int64_t)kslice * kChunk * RP, own, tag);
            if (do_expand) {
                // ---- the partial sums of every k-slice, added in slice order ----
                // The workgroups that produce them belong to this launch and publish before they wait
                // for anything, so they arrive within microseconds when those workgroups are running.
                // Should one not be running yet (more live items than the GPU holds at once), the
                // bounded wait ends and this workgroup starts the item again on its own.
                float s = 0.f;
                bool gave_up = false;
                if (h_thread) {
                    for (int k0 = 0; k0 < a.ksplit; k0 += 4) {    // four words in flight at a time
                        uint64_t wv[4];
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            if (k0 + k < a.ksplit) wv[k] = xch_get(xw + (int64_t)(k0 + k) * kChunk * RP);
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            if (k0 + k < a.ksplit) {
                                if (do_shrink && k0 + k == kslice) { s += own; continue; }
                                int spins = 0;
                                while ((uint32_t)(wv[k] >> 32) != tag) {
                                    if (++spins > a.poll_limit) { gave_up = true; break; }
                                    __builtin_amdgcn_s_sleep(1);
                                    wv[k] = xch_get(xw + (int64_t)(k0 + k) * kChunk * RP);
                                }
                                s += __uint_as_float((uint32_t)wv[k]);
                            }
                        }
                    }
                    if (gave_up) atomicOr(&s_missing, 1u);
                }
                __syncthreads();
                if (s_missing) {                                  // rare
                    __syncthreads();
                    if (tid == 0) s_missing = 0;                  // next use is behind the shrink's barriers
                    solo_next = true; first_item = false;
                    item -= n_wg;
                    continue;
                }
                if (tid < kChunk * RP) hs[hc][hj] = s * scale;
                __syncthreads();
            }
        }
        if (prof && tid == 0 && first_item) prof[3] = wall_clock64();

        // ---- expand + in-place add ----
        if (do_expand) {
            // Matrix-core operands of h: lane l supplies row l%4 of the chunk, four ranks per step.
            // h is fp32; it goes in as a bf16 head (truncated) plus a bf16 tail (rounded), which
            // together carry 16 bits of h, far inside the output's own bf16 rounding.
            s16x4_t ahi[C::MX ? RP / 4 : 1], alo[C::MX ? RP / 4 : 1];
            if constexpr (C::MX) {
                const float *hrow = hs[lane & 3];
#pragma unroll
                for (int s4 = 0; s4 < RP / 4; ++s4) {
                    const float4 v = *(const float4 *)(hrow + 4 * s4);
                    const float f[4] = {v.x, v.y, v.z, v.w};
                    uint32_t hi[4], lo[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        hi[k] = __float_as_uint(f[k]) & 0xffff0000u;
                        lo[k] = f2bf(f[k] - __uint_as_float(hi[k]));
                    }
                    ahi[s4] = __builtin_bit_cast(s16x4_t, make_uint2((hi[0] >> 16) | hi[1], (hi[2] >> 16) | hi[3]));
                    alo[s4] = __builtin_bit_cast(s16x4_t, make_uint2(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16)));
                }
            }
            // an item that walks several tiles keeps DEPTH of them in flight: tile t + DEPTH is requested
            // as soon as tile t has been written back
            for (int l0 = out0; l0 < out1; l0 += C::DEPTH * C::TILE) {
                static_for<C::DEPTH>([&](auto dc) {
                    constexpr int d = decltype(dc)::value;
                    const int lo = l0 + d * C::TILE;
                    if (lo < out1) {
#pragma unroll
                        for (int e = 0; e < C::EU; ++e) {
                            const int o = lo + (e * C::NT + tid) * C::OPL;
                            if constexpr (C::MX) {
                                // Operand order: the adapter's B rows are the "row" operand (lane l supplies
                                // output l of the wave's 64), h the "column" operand (lane l supplies chunk row
                                // l%4), so accumulator register i of lane l is output 4*(l/4) + i of row l%4.
                                f32x4_t d0 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                                for (int s4 = 0; s4 < RP / 4; ++s4) {
                                    const uint4 bq = braw[d][e][s4 / 2];
                                    const s16x4_t bop = __builtin_bit_cast(s16x4_t, (s4 & 1) ? make_uint2(bq.z, bq.w) : make_uint2(bq.x, bq.y));
                                    d0 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(bop, ahi[s4], d0, 0, 0, 0);
                                    d1 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(bop, alo[s4], d1, 0, 0, 0);
                                }
                                const int ob = o & ~3;                            // first output of this lane's block
                                if (r4 < cnt && ob < out1 && rank > 0) {          // empty slot: rows stay untouched
                                    const uint2 yv = yq[d][e];
                                    st_quiet(y_lane + (uint32_t)ob * 2u,
                                             make_uint2(pack_bf2(bf_lo(yv.x) + (d0[0] + d1[0]), bf_hi(yv.x) + (d0[1] + d1[1])),
                                                        pack_bf2(bf_lo(yv.y) + (d0[2] + d1[2]), bf_hi(yv.y) + (d0[3] + d1[3]))));
                                }
                            } else {
                                // hs is re-read for every output group: keeping all of it in registers across
                                // groups costs more registers than the LDS reads cost time
                                asm volatile("" ::: "memory");
                                // bf[q*RP + j]: B value of output q of this lane; for RP >= 8 there is one output
                                float bf[C::BV * 8];
#pragma unroll
                                for (int q = 0; q < C::BV; ++q) {
                                    bf[q * 8 + 0] = bf_lo(braw[d][e][q].x); bf[q * 8 + 1] = bf_hi(braw[d][e][q].x);
                                    bf[q * 8 + 2] = bf_lo(braw[d][e][q].y); bf[q * 8 + 3] = bf_hi(braw[d][e][q].y);
                                    bf[q * 8 + 4] = bf_lo(braw[d][e][q].z); bf[q * 8 + 5] = bf_hi(braw[d][e][q].z);
                                    bf[q * 8 + 6] = bf_lo(braw[d][e][q].w); bf[q * 8 + 7] = bf_hi(braw[d][e][q].w);
                                }
#pragma unroll
                                for (int c = 0; c < kChunk; ++c) {
                                    if (c < cnt && o < out1 && rank > 0) {        // empty slot: rows stay untouched
                                        float yf[C::OPL];
                                        y_unpack(yraw[d][e][c], yf);
#pragma unroll
                                        for (int q = 0; q < C::OPL; ++q) {
                                            float dlt = 0.f;
#pragma unroll
                                            for (int j = 0; j < RP; ++j) dlt = fmaf(hs[c][j], bf[q * RP + j], dlt);
                                            yf[q] += dlt;
                                        }
                                        yvec_t out;
                                        y_pack(yf, out);
                                        st_quiet(yrow[c] + o, out);
                                    }
                                }
                            }
                        }
                        if (lo + C::DEPTH * C::TILE < out1) load_tile(lo + C::DEPTH * C::TILE, dc, IntC<0>{});
                    }
                });
            }
            __syncthreads();                                      // hs is rewritten by the next item
        }
        if (prof && tid == 0 && first_item) prof[4] = wall_clock64();
        first_item = false;
    }

    // ---- tag bookkeeping ----
    if (use_x) {
        if (first_item && tid == 0) tag_sign_in(a.ctrl, wg, tag);   // a workgroup without items still signs in
        if (wg == n_wg - 1 && w == 0) {
            if (!first_item) tag = s_tag;
            else tag = __shfl(tag, 0, 64);
            if (tag != kTagPoison) tag_advance(a.ctrl, n_wg, tag, lane);
        }
    }
}

// Waves per SIMD the kernels are compiled for (the register budget follows): 4 for the 8-wave kernels
// of ranks up to 16, and 5 for the 4-wave rank-8 kernel without exchange -- the packed MoE launches,
// which stream at the memory system's rate and gained 3.6 % from the fifth workgroup per CU (94
// registers, no spills; compiled for 6 it spills and takes 40 % longer).
template <int RP, int NW, bool XCH>
constexpr int rows_waves_per_simd() { return (NW >= 8 && RP <= 16) ? 4 : ((NW == 4 && RP == 8 && !XCH) ? 5 : 1); }

template <int RP, int NW, bool XCH>
__global__ __launch_bounds__(NW * 64, (rows_waves_per_simd<RP, NW, XCH>()))
void rows_kernel(const RowsArgs a)
{
    rows_body<RP, NW, XCH>(a, (int)blockIdx.x, (int)gridDim.x);
}

// The launch without a plan: item i is row i (rank 1 and 2).
template <int RP, int NW>
__global__ __launch_bounds__(NW * 64, NW >= 8 ? 4 : 1)
void rows_items_kernel(const RowsArgs a)
{
    rows_body<RP, NW, false, true>(a, (int)blockIdx.x, (int)gridDim.x);
}

// Several sites that share a batch plan in one launch (q/k/v of one layer, or gate/up): site s owns
// workgroups [first[s], first[s + 1]).  Workgroups of different sites never talk to each other.
struct MultiArgs {
    int32_t n;
    int32_t first[kMaxMulti + 1];
    RowsArgs site[kMaxMulti];
};

template <int RP, int NW, bool XCH, int RUN = 3>
__global__ __launch_bounds__(NW * 64, (rows_waves_per_simd<RP, NW, XCH>()))
void rows_multi_kernel(const MultiArgs m)
{
    const int b = (int)blockIdx.x;
    int s = 0;
#pragma unroll
    for (int k = 1; k < kMaxMulti; ++k) s += (k < m.n && b >= m.first[k]) ? 1 : 0;
    rows_body<RP, NW, XCH, false, RUN>(m.site[s], b - m.first[s], m.first[s + 1] - m.first[s]);
}

// The first launch of a decode step can plan for itself: every workgroup sorts the batch's
// (slot, row) keys in LDS (what the one-workgroup planner kernel does, a microsecond of work) instead
// of waiting for a planner launch and then fetching its chunk record; workgroup 0 also leaves the
// plan in global memory for the launches that follow.  Batches of up to kLocalPlanRows rows over up
// to kLocalPlanSlots slots.
constexpr int kLocalPlanRows = 256;   // more rows mean more distinct slots per wave, and every workgroup pays for them
struct PlanLocalArgs {
    const int32_t *token_slot;
    const int32_t *ready_rank;
    int32_t T, n_slots, rec_bound;
    PlanView pv;
};

template <int RP, int NW, bool XCH>
__global__ __launch_bounds__(NW * 64, (rows_waves_per_simd<RP, NW, XCH>()))
void rows_multi_plan_kernel(const MultiArgs m, const PlanLocalArgs pl)
{
    __shared__ PlanLocalLds p_lds;
    __shared__ __attribute__((aligned(16))) int32_t p_rec[kLocalPlanRows * kRec];
    const int b = (int)blockIdx.x;
    plan_dense_local(pl.token_slot, pl.T, pl.n_slots, pl.ready_rank, pl.rec_bound, (int)threadIdx.x, NW * 64,
                     p_lds, p_rec, b == 0, pl.pv);
    int s = 0;
#pragma unroll
    for (int k = 1; k < kMaxMulti; ++k) s += (k < m.n && b >= m.first[k]) ? 1 : 0;
    rows_body<RP, NW, XCH>(m.site[s], b - m.first[s], m.first[s + 1] - m.first[s], p_rec);
}

template <int RP, int NW, bool XCH>
static int rows_capacity()
{
    static int cap = 0;
    if (cap == 0) {
        int per_cu = 0, cus = 0, dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, rows_kernel<RP, NW, XCH>, NW * 64, 0) != hipSuccess) return 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cap = per_cu * cus;
    }
    return cap;
}

// Bytes one chunk of a site moves: adapter rows and x for the shrink, B rows and y (read + write)
// for the expand.
static double chunk_bytes(const RowsArgs &a)
{
    return 2.0 * a.d_in * (a.r_pad + kChunk) + (double)a.d_out * (2.0 * a.r_pad + 4.0 * kChunk);
}

static bool can_exchange(const RowsArgs &a)
{
    return a.xch && a.ctrl && a.n_experts == 1 && a.grid_chunks <= a.xch_chunks;
}

// Cuts a chunk of a dense site into `parts` items.  A CU pulls only so many bytes per microsecond,
// so a launch with fewer chunks than the GPU has CUs spreads each chunk over several workgroups:
// part p expands outputs [p * out_per_part, ...) and, where the site has an exchange area, shrinks
// k-slice p of d_in and trades the partial sums with the other parts of its chunk (no adapter byte
// is read twice); without an exchange area every part redoes the whole shrink.
static void set_parts(RowsArgs &a, int parts, bool exchange)
{
    const int U = a.d_in >> 3;
    const int groups = (a.d_out + 63) / 64;
    if (exchange) {
        if (parts > 8) parts = 8;
        if (parts * a.r_pad > 128) parts = 128 / a.r_pad;
    }
    if (parts > groups) parts = groups;
    if (parts < 1 || a.n_experts != 1 || a.h_out) parts = 1;       // (a launch that only shrinks has no outputs to divide)
    const int gpp = (groups + parts - 1) / parts;
    a.out_per_part = gpp * 64;
    a.tile_par = (groups + gpp - 1) / gpp;
    a.mode = 0; a.ksplit = 1; a.kslice_units = U;
    // "rows_poll_limit" (testing): a negative value makes every reader give up at once, so that each
    // item runs the path that does not depend on other workgroups
    const int pl = tuning(kRowsPollLimit);
    a.poll_limit = pl < 0 ? 0 : (pl > 0 ? pl : kPollLimit);
    if (exchange && a.tile_par > 1) {
        int ku = (U + a.tile_par - 1) / a.tile_par;
        ku = (ku + 63) & ~63;
        a.mode = 2;
        a.kslice_units = ku;
        a.ksplit = (U + ku - 1) / ku;
    }
}

static int fused_grid(const RowsArgs &a, int run_log2 = 3)
{
    const int run_mask = (8 << run_log2) - 1;
    return a.tile_par > 1 ? ((a.grid_chunks + 7) & ~7) * a.tile_par : ((a.grid_chunks + run_mask) & ~run_mask);
}

// Rank-bounded reads of A cost one dependent read of the slot's rank in front of the item's loads:
// worth it where a launch runs several rounds of items per CU (the read hides behind the other
// items), not where the launch is one short chain.  "rows_rank_bound": 1 always, -1 never.
static int use_rank_bound(const RowsArgs &a, int cap)
{
    const int t = tuning(kRowsRankBound);
    if (t) return t > 0 ? 1 : 0;
    return a.rank_bound && a.mode != 2 && (int64_t)a.grid_chunks * 2 >= cap;
}

static int items_target(int cap)
{
    // the chunk count used for the division is an upper bound; live chunks are fewer, and a launch
    // whose live items all fit on the GPU at once finishes in one round (measured best at 3/4)
    const int t = tuning(kRowsItemsTarget);
    return t > 0 ? t : cap * 3 / 4;
}

template <int RP, int NW>
static hipError_t launch_rp(RowsArgs a, hipStream_t st)
{
    const int mode = tuning(kRowsMode);     // 0 auto, 1 parts that redo the shrink, 3 one item per chunk
    const int cap = rows_capacity<RP, NW, true>();
    if (cap <= 0) return hipErrorUnknown;
    const bool exchange = can_exchange(a) && mode == 0 && !a.row_slot;
    set_parts(a, mode == 3 ? 1 : items_target(cap) / a.grid_chunks, exchange);
    a.rank_bound = use_rank_bound(a, cap);
    if (a.row_slot) {
        if constexpr (RP <= 2) rows_items_kernel<RP, NW><<<dim3((unsigned)fused_grid(a)), dim3(NW * 64), 0, st>>>(a);
        else return hipErrorInvalidValue;
    } else if (a.mode == 2) rows_kernel<RP, NW, true><<<dim3((unsigned)fused_grid(a)), dim3(NW * 64), 0, st>>>(a);
    else rows_kernel<RP, NW, false><<<dim3((unsigned)fused_grid(a)), dim3(NW * 64), 0, st>>>(a);
    return hipGetLastError();
}

template <int RP>
static hipError_t launch_nw(const RowsArgs &a, hipStream_t st)
{
    const int U = a.d_in >> 3;
    int nw = tuning(kRowsWaves);
    if (nw != 4 && nw != 8) nw = U >= RowsCfg<RP, 8>::FLU * 3 / 4 ? 8 : 4;   // 4 when 8 would be mostly idle lanes
    if constexpr (RP >= 64) nw = 8;
    if (nw >= 8) return launch_rp<RP, 8>(a, st);
    if constexpr (RP < 64) return launch_rp<RP, 4>(a, st);
    return hipErrorInvalidValue;
}

template <int RP, int NW>
static hipError_t launch_multi_rp(const RowsArgs *sites, int n, hipStream_t st, const PlanLocalArgs *pl = nullptr)
{
    const int cap = rows_capacity<RP, NW, true>();
    if (cap <= 0) return hipErrorUnknown;
    MultiArgs m;
    m.n = n;
    m.first[0] = 0;
    // every item of the launch should move about the same number of bytes
    double total = 0.0;
    bool exchange = tuning(kRowsMode) == 0;
    for (int k = 0; k < n; ++k) { total += chunk_bytes(sites[k]); exchange = exchange && can_exchange(sites[k]); }
    const double per_item = total * sites[0].grid_chunks / items_target(cap);
    bool any_x = false;
    for (int k = 0; k < n; ++k) {
        m.site[k] = sites[k];
        // (one site alone gets the parts its own launch would get, so that the results are the same bits)
        set_parts(m.site[k], n == 1 ? items_target(cap) / sites[0].grid_chunks : (int)(chunk_bytes(sites[k]) / per_item + 0.5), exchange);
        m.site[k].rank_bound = use_rank_bound(m.site[k], cap);
        any_x = any_x || m.site[k].mode == 2;
        m.first[k + 1] = m.first[k] + fused_grid(m.site[k]);
    }
    // "rows_chunk_run" = 256 (measurements; the rank-8 four-wave launch without parts, i.e. the packed MoE
    // sites): runs of 256 chunks per XCD instead of 8, so that all chunks of a slot's experts, and with
    // them the rows of x they share, mostly meet in one L2
    constexpr int kLongRun = 8;
    bool long_run = false;
    if constexpr (RP == 8 && NW == 4) {
        if (!any_x && !pl && tuning(kRowsChunkRun) == (1 << kLongRun)) {
            long_run = true;
            for (int k = 0; k < n; ++k) long_run = long_run && m.site[k].tile_par == 1;
            if (long_run)
                for (int k = 0; k < n; ++k) m.first[k + 1] = m.first[k] + fused_grid(m.site[k], kLongRun);
        }
    }
    for (int k = n; k < kMaxMulti; ++k) { m.site[k] = m.site[0]; m.first[k + 1] = m.first[n]; }
    if constexpr (NW == 8) {
        if (pl) {
            if (any_x) rows_multi_plan_kernel<RP, NW, true><<<dim3((unsigned)m.first[n]), dim3(NW * 64), 0, st>>>(m, *pl);
            else rows_multi_plan_kernel<RP, NW, false><<<dim3((unsigned)m.first[n]), dim3(NW * 64), 0, st>>>(m, *pl);
            return hipGetLastError();
        }
    }
    if (pl) return hipErrorInvalidValue;
    if constexpr (RP == 8 && NW == 4) {
        if (long_run) {
            rows_multi_kernel<RP, NW, false, kLongRun><<<dim3((unsigned)m.first[n]), dim3(NW * 64), 0, st>>>(m);
            return hipGetLastError();
        }
    }
    if (any_x) rows_multi_kernel<RP, NW, true><<<dim3((unsigned)m.first[n]), dim3(NW * 64), 0, st>>>(m);
    else rows_multi_kernel<RP, NW, false><<<dim3((unsigned)m.first[n]), dim3(NW * 64), 0, st>>>(m);
    return hipGetLastError();
}

// Waves per workgroup a site would run with in a shared launch (4 or 8), or 0 if it needs a launch
// of its own.  Sites of rank 8 or 16 can share one; a dense site must also keep most lanes of an
// 8-wave shrink busy, a packed MoE site takes 4 waves when 8 would be mostly idle.
int rows_group_waves(const RowsArgs &a)
{
    if ((a.r_pad != 8 && a.r_pad != 16) || a.h_out || tuning(kRowsWaves)) return 0;
    const int U = a.d_in >> 3;
    const int flu8 = a.r_pad == 8 ? RowsCfg<8, 8>::FLU : RowsCfg<16, 8>::FLU;
    if (U >= flu8 * 3 / 4) return 8;
    return a.n_experts > 1 ? 4 : 0;
}

hipError_t launch_rows_multi(const RowsArgs *sites, int n, hipStream_t st)
{
    if (n < 1 || n > kMaxMulti) return hipErrorInvalidValue;
    const int nw = rows_group_waves(sites[0]);
    if (nw == 0) return hipErrorInvalidValue;
    for (int k = 0; k < n; ++k)
        if (sites[k].r_pad != sites[0].r_pad || rows_group_waves(sites[k]) != nw) return hipErrorInvalidValue;
    if (sites[0].grid_chunks <= 0) return hipSuccess;
    if (nw == 8) return sites[0].r_pad == 8 ? launch_multi_rp<8, 8>(sites, n, st) : launch_multi_rp<16, 8>(sites, n, st);
    return sites[0].r_pad == 8 ? launch_multi_rp<8, 4>(sites, n, st) : launch_multi_rp<16, 4>(sites, n, st);
}

// A dense site whose own launch would run the 8-wave kernel can plan inside that launch.
template <int RP>
static bool wide_enough_for_8_waves(int U) { return RP >= 64 || U >= RowsCfg<RP, 8>::FLU * 3 / 4; }

bool rows_plans_alone(const RowsArgs &a)
{
    if (a.n_experts != 1 || a.h_out || tuning(kRowsWaves)) return false;
    const int U = a.d_in >> 3;
    switch (a.r_pad) {
        case 1:  return wide_enough_for_8_waves<1>(U);
        case 2:  return wide_enough_for_8_waves<2>(U);
        case 4:  return wide_enough_for_8_waves<4>(U);
        case 8:  return wide_enough_for_8_waves<8>(U);
        case 16: return wide_enough_for_8_waves<16>(U);
        case 32: return wide_enough_for_8_waves<32>(U);
        case 64: return true;
    }
    return false;
}

// Plans the dense batch inside the launch of `sites` (8-wave sites of one rank, see rows_group_waves)
// and leaves the plan in pv.  T <= rows_local_plan_rows().
int rows_local_plan_rows() { return kLocalPlanRows; }
int rows_local_plan_slots() { return kLocalPlanSlots; }

hipError_t launch_rows_multi_plan(const RowsArgs *sites, int n, const PlanView &pv, const int32_t *token_slot, int T,
                                  int n_slots, const int32_t *ready_rank, hipStream_t st)
{
    if (n < 1 || n > kMaxMulti || T < 1 || T > kLocalPlanRows || n_slots > kLocalPlanSlots) return hipErrorInvalidValue;
    if (n == 1) {
        if (!rows_plans_alone(sites[0])) return hipErrorInvalidValue;
    } else {
        for (int k = 0; k < n; ++k)
            if (sites[k].r_pad != sites[0].r_pad || rows_group_waves(sites[k]) != 8) return hipErrorInvalidValue;
    }
    PlanLocalArgs pl;
    pl.token_slot = token_slot; pl.ready_rank = ready_rank; pl.T = T; pl.n_slots = n_slots;
    pl.rec_bound = (int)max_chunks(T, n_slots);
    if (pl.rec_bound > kLocalPlanRows) return hipErrorInvalidValue;
    pl.pv = pv;
    switch (sites[0].r_pad) {
        case 1:  return launch_multi_rp<1, 8>(sites, n, st, &pl);
        case 2:  return launch_multi_rp<2, 8>(sites, n, st, &pl);
        case 4:  return launch_multi_rp<4, 8>(sites, n, st, &pl);
        case 8:  return launch_multi_rp<8, 8>(sites, n, st, &pl);
        case 16: return launch_multi_rp<16, 8>(sites, n, st, &pl);
        case 32: return launch_multi_rp<32, 8>(sites, n, st, &pl);
        case 64: return launch_multi_rp<64, 8>(sites, n, st, &pl);
    }
    return hipErrorInvalidValue;
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
