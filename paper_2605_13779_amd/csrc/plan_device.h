// Device-side pieces of the one-workgroup dense planner (bitonic sort of (slot, row) keys, scans),
// shared by the planner kernel and by the decode launch that plans for itself.
#pragma once
#include "internal.h"

namespace mlora {

constexpr int kSortMax = 1024;

template <int D>
__device__ __forceinline__ uint32_t lane_xor_u32(uint32_t x)
{
    int r;
    if constexpr (D == 1) r = __builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xf, 0xf, true);
    else if constexpr (D == 2) r = __builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xf, 0xf, true);
    else if constexpr (D == 4) {
        r = __builtin_amdgcn_update_dpp(0, (int)x, 0x104, 0xf, 0x5, false);
        r = __builtin_amdgcn_update_dpp(r, (int)x, 0x114, 0xf, 0xa, false);
    } else if constexpr (D == 8) r = __builtin_amdgcn_update_dpp(0, (int)x, 0x128, 0xf, 0xf, true);
    else if constexpr (D == 16) r = __builtin_amdgcn_ds_swizzle((int)x, 0x401F);
    else r = __shfl_xor((int)x, 32, 64);
    return (uint32_t)r;
}

// One compare-exchange step of the network for the key held by thread i (partner i ^ J, merge size K).
template <int K, int J>
__device__ __forceinline__ void bitonic_step(uint32_t &ks, uint32_t &kt, int i, uint2 *xch)
{
    uint32_t ps, pt;
    if constexpr (J < 64) {
        ps = lane_xor_u32<J>(ks);
        pt = lane_xor_u32<J>(kt);
    } else {
        xch[i] = make_uint2(ks, kt);
        __syncthreads();
        const uint2 p = xch[i ^ J];
        __syncthreads();
        ps = p.x; pt = p.y;
    }
    const bool self_less = ks < ps || (ks == ps && kt < pt);
    const bool up = (i & K) == 0, lower = (i & J) == 0;
    const bool keep_self = (lower == up) == self_less;      // lower lane of an ascending pair keeps the smaller key
    if (!keep_self) { ks = ps; kt = pt; }
}

template <int K, int J>
struct BitonicMerge {
    static __device__ __forceinline__ void run(uint32_t &ks, uint32_t &kt, int i, uint2 *xch)
    {
        bitonic_step<K, J>(ks, kt, i, xch);
        if constexpr (J > 1) BitonicMerge<K, J / 2>::run(ks, kt, i, xch);
    }
};

template <int K>
struct BitonicSort {
    static __device__ __forceinline__ void run(uint32_t &ks, uint32_t &kt, int i, int N, uint2 *xch)
    {
        if constexpr (K > 2) BitonicSort<K / 2>::run(ks, kt, i, N, xch);
        if (K <= N) BitonicMerge<K, K / 2>::run(ks, kt, i, xch);      // N is uniform over the workgroup
    }
};

// Inclusive scan over the 64 lanes of a wave with data-parallel-primitive moves (values >= 0, so 0
// is the identity of both operations): shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the
// last lane of row 0 / 2 is broadcast into row 1 / 3 and the last lane of the lower half into the
// upper half.  Lanes without a source keep the identity.
template <bool IS_MAX>
__device__ __forceinline__ int wave_scan(int v)
{
    auto op = [](int a, int b) { return IS_MAX ? max(a, b) : a + b; };
    v = op(v, __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false));     // row_shr:1
    v = op(v, __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false));     // row_shr:2
    v = op(v, __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false));     // row_shr:4
    v = op(v, __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false));     // row_shr:8
    v = op(v, __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false));     // row_bcast:15 into rows 1 and 3
    v = op(v, __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false));     // row_bcast:31 into rows 2 and 3
    return v;
}

// Inclusive scan over the workgroup (one value per thread); IS_MAX selects max instead of plus.
template <bool IS_MAX>
__device__ __forceinline__ int block_scan(int v, int tid, int nw, int32_t *wave_tot)
{
    const int lane = tid & 63, w = tid >> 6;
    v = wave_scan<IS_MAX>(v);
    if (lane == 63) wave_tot[w] = v;
    __syncthreads();
    // the totals of the waves in front of this one: all sixteen words in four reads (a loop over
    // k < w is a chain of dependent LDS reads); words of waves that do not exist are never selected
    int base = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int4 t = ((const int4 *)wave_tot)[q];
        const int e[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int v = 4 * q + k < w ? e[k] : 0;
            base = IS_MAX ? max(base, v) : base + v;
        }
    }
    __syncthreads();
    (void)nw;
    return IS_MAX ? max(v, base) : v + base;
}

// The planner inside a workgroup of an apply kernel: every thread calls it (i = thread index,
// nthreads a multiple of 64, 256..512, T <= 256 rows (waves 0..3), n_slots <= kLocalPlanSlots).  token_slot[0..T) ->
// the batch's chunk records in LDS (lrec, kRec ints per chunk, rec_bound of them, the ones past the
// live chunks with count 0), the same records the planner kernel writes: rows grouped by slot,
// ascending row inside a slot, groups in slot order, cut into chunks of kChunk rows.  With write_pv
// the workgroup also leaves the plan in global memory for the launches that follow.
//
// No sort here: a row's place is (rows of smaller slots) + (earlier rows of its own slot).  Inside a
// wave the second term comes from ballots, one per distinct slot of the wave; across waves from a
// small table of per-wave counts; the first term from one scan over the slots.  Five barriers,
// against fifteen of the sorting network, which is what a 512-thread workgroup feels.
constexpr int kLocalPlanSlots = 1024;
struct PlanLocalLds {
    int32_t cntw[4][kLocalPlanSlots];      // rows of slot s in wave w (the rows sit in the first 4 waves)
    __attribute__((aligned(16))) int32_t srow[2][256];   // usable slot of each row (-1: none), one copy per half
    int32_t prt[256];                      // the upper half's counts for each row (same << 16 | earlier)
    int32_t off[kLocalPlanSlots + 1];      // rows of smaller slots
    int32_t cbase[kLocalPlanSlots + 1];    // chunks of smaller slots
    __attribute__((aligned(16))) int32_t wave_tot[16];
};

__device__ __forceinline__ void plan_dense_local(const int32_t *__restrict__ token_slot, int T, int n_slots,
                                                 const int32_t *__restrict__ ready_rank, int rec_bound,
                                                 int i, int nthreads, PlanLocalLds &L,
                                                 int32_t *lrec, bool write_pv, const PlanView &pv)
{
    const int lane = i & 63, w = i >> 6, nw = nthreads >> 6;
    constexpr int kRowWaves = 4;
    // The rows sit in waves 0..3.  A workgroup of eight waves lets wave w + 4 do the upper half of
    // wave w's compares (below): it fetches the same 64 slots and hands its counts over through LDS.
    const bool split = nw >= 2 * kRowWaves;
    const int hw = split ? (w & (kRowWaves - 1)) : w, half = split ? w / kRowWaves : 0;
    const int hrow = hw * 64 + lane;
    int sh = -1;
    if (hw < kRowWaves && hrow < T) {
        const int v = token_slot[hrow];
        if (v >= 0 && v < n_slots && !(ready_rank && ready_rank[v] <= 0)) sh = v;
    }
    const int s = w < kRowWaves ? sh : -1;       // a row's own thread: i == hrow
    // Earlier rows of the same slot inside the wave, and the wave's count per slot: every lane
    // compares its slot with the wave's 64 slots, read back from LDS four at a time (all lanes read
    // the same address: a broadcast).  A loop over the distinct slots with ballots is shorter on
    // paper, but each of its 30 to 40 rounds (64 slots, Zipf popularity) is a chain of scalar /
    // vector hand-overs and took 1.9 us.  Every row wave clears and fills its own line of the count
    // table (LDS operations of a wave stay in order).
    int rank = 0, same = 0;
    if (hw < kRowWaves) {
        if (w < kRowWaves)
            for (int k = lane; k < n_slots; k += 64) L.cntw[w][k] = 0;
        int32_t *mine = L.srow[half] + 64 * hw;   // this wave's own copy of the 64 slots
        mine[lane] = sh;
        const int j_lo = split ? 32 * half : 0, n4 = split ? 8 : 16;
#pragma unroll 4
        for (int q = 0; q < n4; ++q) {
            const int j = j_lo + 4 * q;
            const int4 v = *(const int4 *)(mine + j);
            same += (v.x == sh) + (v.y == sh) + (v.z == sh) + (v.w == sh);
            rank += (v.x == sh && j < lane) + (v.y == sh && j + 1 < lane) + (v.z == sh && j + 2 < lane) + (v.w == sh && j + 3 < lane);
        }
        if (w >= kRowWaves) L.prt[hrow] = same << 16 | rank;
    }
    if (split) {
        __syncthreads();
        if (w < kRowWaves) { const int p = L.prt[i]; rank += p & 0xffff; same += p >> 16; }
    }
    if (s >= 0 && rank == 0) L.cntw[w][s] = same;
    __syncthreads();
    // per slot: size and chunks, a run of slots per thread; one scan carries both sums (each total is
    // at most 256)
    const int per = (n_slots + nthreads - 1) / nthreads;
    const int k_lo = min(n_slots, i * per), k_hi = min(n_slots, k_lo + per);
    int size = 0, chunks = 0;
    for (int k = k_lo; k < k_hi; ++k) {
        int c = 0;
        for (int v = 0; v < kRowWaves; ++v) c += L.cntw[v][k];
        size += c;
        chunks += (c + kChunk - 1) / kChunk;
    }
    const int inc = block_scan<false>(chunks << 16 | size, i, nw, L.wave_tot);
    int run_s = (inc & 0xffff) - size, run_c = (inc >> 16) - chunks;
    for (int k = k_lo; k < k_hi; ++k) {
        int c = 0;
        for (int v = 0; v < kRowWaves; ++v) c += L.cntw[v][k];
        L.off[k] = run_s; L.cbase[k] = run_c;
        run_s += c;
        run_c += (c + kChunk - 1) / kChunk;
    }
    if (i == nthreads - 1) { L.off[kLocalPlanSlots] = inc & 0xffff; L.cbase[kLocalPlanSlots] = inc >> 16; }
    __syncthreads();
    const int n_rows = L.off[kLocalPlanSlots], n_chunks = L.cbase[kLocalPlanSlots];
    if (s >= 0) {
        int n = 0;
        for (int k = 0; k < kRowWaves; ++k) { const int c = L.cntw[k][s]; n += c; rank += k < w ? c : 0; }
        const int pos = L.off[s] + rank, c = L.cbase[s] + rank / kChunk;
        int32_t *rec = lrec + c * kRec;
        rec[4 + (rank % kChunk)] = i;
        if (rank % kChunk == 0) { rec[0] = s; rec[1] = min(kChunk, n - rank); rec[2] = pos; rec[3] = 0; }
        if (write_pv) {
            pv.sorted[pos] = i;
            int32_t *g = pv.chunks + (int64_t)c * kRec;
            g[4 + (rank % kChunk)] = i;
            if (rank % kChunk == 0) { g[0] = s; g[1] = min(kChunk, n - rank); g[2] = pos; g[3] = 0; }
        }
    }
    if (write_pv && i == 0) { pv.hdr[0] = n_chunks; pv.hdr[1] = n_rows; }
    for (int d = n_chunks + i; d < rec_bound; d += nthreads) {
        lrec[d * kRec + 1] = 0;
        if (write_pv) pv.chunks[(int64_t)d * kRec + 1] = 0;
    }
    __syncthreads();
}

}  // namespace mlora
