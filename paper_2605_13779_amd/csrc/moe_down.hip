// MoE down projection: shrink per chunk of a (slot, expert) group, then expand + routing-weight combine
// on the matrix cores.
//
// Per-expert LoRA tensors sit on the expert down projection too (Sections 3.4 and 4.4): pair
// p = (t, k) has its own input row and its delta is added, times the routing weight, into the ONE
// output row of token t.  The first launch (one wave per chunk of up to four pairs of a (slot, expert)
// group; ranks above 16 go through the chunk kernels of rows.hip) leaves,
// per pair, the rank-r vector  h[p] = w[p] * (alpha / r) * A_{s,e} x[p]  (fp32 split into a bf16
// head and tail).  What is left is, per slot s,
//
//     Y_s [tokens of s, d_out]  +=  H_s [tokens of s, E * r]  x  Bcat_s [E * r, d_out]
//
// where row t of H_s holds h[(t, k)] in the r columns of expert e(t, k) and zeros elsewhere, and
// Bcat_s stacks the slot's per-expert B tensors along the contraction axis -- exactly how the packed
// tables store them.  That is a dense contraction per slot (H_s is block sparse, but with a few
// tokens per (slot, expert) group nearly every expert's block is touched), so it runs on
// v_mfma_f32_32x32x16_bf16, and it has what the row-by-row form lacks: every output row has ONE
// writer (no fp32 [pairs, d_out] workspace to write and read back, no atomics, a fixed summation
// order), and a slot's B tensors are streamed once per 96 tokens.  Contraction steps whose experts
// received no pair of the slot are skipped (their B rows are not fetched), so sparse routing does not
// pay for the dense form.
//
// A workgroup owns a tile of up to 96 tokens of one slot and 128 outputs; each of its 4 waves owns
// 32 outputs and streams its rows of B straight from the tables in operand layout (lane = output,
// 8 consecutive ranks: one 16-byte load), one chunk of 8 contraction steps ahead (two ahead measured
// slower: more of B in flight than the memory system serves only queues in front of the rest).  H is never
// written out densely.  The tile's h vectors are fetched once into LDS, split into bf16 head and
// tail in operand layout (K vectors per token, plus one vector of zeros), beside a byte table
// inv[token][expert] = which of the token's K pairs went to that expert (0xff: none).  A lane's
// operand for a contraction step is then one table byte and two 16-byte LDS reads -- the pair's
// vector or the zeros -- so that after the prologue the waves run without a barrier until the
// epilogue.  Ranks below 8 are padded to 8 in the contraction (zeros in both operands; the loads
// fetch the real ranks only).
#include <atomic>
#include "plan_device.h"
#include "wave_ops.h"

namespace mlora {

namespace {
constexpr int TN = 128;            // outputs per tile
constexpr int NWD = 4;             // waves: 32 outputs each
constexpr int NTD = NWD * 64;
constexpr int CHK = 128;           // contraction values per chunk (8 steps of 16)
constexpr int NST = CHK / 16;
constexpr int KMAX = 16;           // largest top-k (a pair's index fits the table byte)
constexpr int STG_LD = TN + 4;     // padded row stride of the output staging block, in floats
constexpr int kStageBytes = 32 * STG_LD * 4;
constexpr int kLdsTwo = 80 * 1024 - 1024;     // dynamic LDS that leaves room for two workgroups per CU
constexpr int kLdsOne = 160 * 1024 - 2048;    // ... for one

// Where the tile's tables sit in dynamic LDS (byte offsets), for a padded rank rpe >= 8 and tm tokens.
struct DownLayout {
    int n_chunks;      // chunks of the padded contraction axis E * rpe
    int inv_half;      // rank 8: a step holds two experts, one per lane half; odd experts start here in a row
    int inv_ld;        // bytes per token row of inv
    int lo_off, inv_off, live_off, total;
};

__host__ __device__ inline DownLayout down_layout(int rpe, int tm, int K, int E)
{
    DownLayout L;
    L.n_chunks = (E * rpe + CHK - 1) / CHK;
    L.inv_half = rpe == 8 ? L.n_chunks * 8 : 0;
    const int row = L.n_chunks * (CHK / rpe);
    L.inv_ld = ((row + 7) & ~7) + 8;                         // (+8: rows do not start on the same banks)
    const int hb = ((tm * K + 1) * rpe * 2 + 15) & ~15;      // the vectors, one of zeros behind them
    L.lo_off = hb;
    L.inv_off = 2 * hb;
    L.live_off = (L.inv_off + tm * L.inv_ld + 15) & ~15;
    L.total = L.live_off + ((L.n_chunks + 15) & ~15);
    return L;
}

inline int down_dyn_bytes(int rpe, int tm, int K, int E)
{
    const int t = down_layout(rpe, tm, K, E).total;
    return t > kStageBytes ? t : kStageBytes;
}

// 32-row blocks per tile: the most that leaves two workgroups per CU, else the most that fits at all (0: none).
inline int down_blocks(int r_pad, int K, int E)
{
    const int rpe = r_pad < 8 ? 8 : r_pad;
    if ((int64_t)E * rpe > (1 << 21)) return 0;
    for (int mb = 3; mb >= 1; --mb) if (down_dyn_bytes(rpe, 32 * mb, K, E) <= kLdsTwo) return mb;
    for (int mb = 3; mb >= 1; --mb) if (down_dyn_bytes(rpe, 32 * mb, K, E) <= kLdsOne) return mb;
    return 0;
}
}  // namespace

__device__ __forceinline__ f32x16_t mfma32d(const uint4 &a, const uint4 &b, f32x16_t c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

template <int RP, int MB>
__global__ __launch_bounds__(NTD, 2)
void moe_down_kernel(const MoeDownArgs a)
{
    constexpr int RPE = RP < 8 ? 8 : RP, TM = 32 * MB;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ int32_t tokM[TM];                  // the tile's tokens

    const int tid = (int)threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = (int)blockIdx.x / a.n_ntiles, nt = (int)blockIdx.x - g * a.n_ntiles;

    // ---- which slot, which tile of its tokens: tile g of the list of all slots' tiles (every wave
    //      finds it by itself: 64 slots per step, no barrier) ----
    int s = -1, t_lo = 0, rows = 0, r_s = 0;
    for (int s0 = 0, base = 0; s0 < a.n_slots; s0 += 64) {
        const int si = s0 + lane;
        const int lo = si < a.n_slots ? a.tok_off[si] : 0, hi = si < a.n_slots ? a.tok_off[si + 1] : 0;
        const int r_i = si < a.n_slots ? a.rank[si] : 0;
        const int tiles = (hi - lo + TM - 1) / TM;
        const int inc = wave_scan<false>(tiles), excl = base + inc - tiles;
        const uint64_t hit = __ballot(tiles > 0 && g >= excl && g < excl + tiles);
        if (hit) {
            const int l = __ffsll((long long)hit) - 1;
            s = s0 + l;
            r_s = __shfl(r_i, l, 64);
            t_lo = __shfl(lo, l, 64) + (g - __shfl(excl, l, 64)) * TM;
            rows = min(TM, __shfl(hi, l, 64) - t_lo);
            break;
        }
        base += __shfl(inc, 63, 64);
        if (g < base) break;
    }
    s = __builtin_amdgcn_readfirstlane(s);
    if (s < 0 || __builtin_amdgcn_readfirstlane(r_s) <= 0) return;   // no such tile, or the slot holds no adapter at this site
    t_lo = __builtin_amdgcn_readfirstlane(t_lo);
    rows = __builtin_amdgcn_readfirstlane(rows);

    const int E = a.E, K = a.K;
    const DownLayout L = down_layout(RPE, TM, K, E);
    uint16_t *const hch = (uint16_t *)lds, *const hcl = (uint16_t *)(lds + L.lo_off);
    uint8_t *const inv = lds + L.inv_off, *const live_l = lds + L.live_off;
    const int n_chunks = L.n_chunks, zero_row = TM * K;
    const char *Bs = (const char *)(a.b_tab + (int64_t)s * E * a.d_out * RP);
    const int am = lane & 31, kg = lane >> 5;
    const uint32_t o_b = (uint32_t)min(nt * TN + w * 32 + am, a.d_out - 1);   // this lane's output as B operand

    // B rows of one contraction step: ranks [j0, j0 + 8) of expert e (the real ranks when there are fewer)
    auto load_b = [&](int c, int st, bool live) __attribute__((always_inline)) -> uint4 {
        const int kv0 = live ? c * CHK + st * 16 + kg * 8 : 0;           // (dead steps: the slot's first rows again, a cache hit)
        const uint32_t e = (uint32_t)min(kv0 / RPE, E - 1), j0 = (uint32_t)(kv0 % RPE);
        const char *src = Bs + ((e * (uint32_t)a.d_out + o_b) * (uint32_t)RP + (RP >= 8 ? j0 : 0u)) * 2u;
        if constexpr (RP >= 8) return *(const uint4 *)src;
        else if constexpr (RP == 4) { const uint2 v = *(const uint2 *)src; return make_uint4(v.x, v.y, 0u, 0u); }
        else if constexpr (RP == 2) return make_uint4(*(const uint32_t *)src, 0u, 0u, 0u);
        else return make_uint4(*(const uint16_t *)src, 0u, 0u, 0u);
    };
    uint4 bq[2][NST];
    auto load_chunk_b = [&](int c, auto bufc, uint32_t mask) __attribute__((always_inline)) {
        constexpr int bi = decltype(bufc)::value;
#pragma unroll
        for (int st = 0; st < NST; ++st) bq[bi][st] = load_b(c, st, (mask >> st & 1u) != 0);   // (every load is issued: the waits count them)
    };
    auto range_mask = [&](int c) { const int left = E * RPE - c * CHK; return left >= CHK ? 0xffu : (left <= 0 ? 0u : (1u << ((left + 15) >> 4)) - 1u); };

    // ---- the tile's tokens; live contraction steps per chunk (bit st: some expert of step st received
    //      a pair of this slot), from the slot's group offsets; inv cleared ----
    if (tid < TM) tokM[tid] = tid < rows ? a.tok_sorted[t_lo + tid] : -1;
    const int32_t *goff = a.group_off + (int64_t)s * E;
    for (int i0 = w * 64; i0 < n_chunks * NST; i0 += NTD) {
        const int i = i0 + lane, c = i >> 3, st = i & 7;
        bool live = false;
        if (c < n_chunks) {
            const int kv = c * CHK + st * 16;
            const int e0 = kv / RPE, e1 = min(E, (kv + 15) / RPE + 1);
            live = e0 < E && goff[e1] > goff[e0];
        }
        const uint64_t bits = __ballot(live);
        if (st == 0 && c < n_chunks) live_l[c] = (uint8_t)(bits >> (lane & 56));
    }
    load_chunk_b(0, IntC<0>{}, range_mask(0));     // on their way while the tile's tables are built
    for (int i = tid; i < TM * L.inv_ld / 8; i += NTD) ((uint2 *)inv)[i] = make_uint2(0xffffffffu, 0xffffffffu);
    if (tid < RPE / 8) { ((uint4 *)(hch + zero_row * RPE))[tid] = make_uint4(0, 0, 0, 0); ((uint4 *)(hcl + zero_row * RPE))[tid] = make_uint4(0, 0, 0, 0); }
    __syncthreads();

    // ---- this thread's pieces of the tile's y rows (16 bytes each): on their way until the epilogue ----
    constexpr int YP = 32 * (TN / 8) / NTD;                          // pieces per thread and block of 32 rows
    uint4 yv[MB][YP];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int i = 0; i < YP; ++i) {
            const int q = tid + i * NTD, m = mb * 32 + q / (TN / 8), o = nt * TN + (q % (TN / 8)) * 8;
            const int t = tokM[m];
            yv[mb][i] = make_uint4(0, 0, 0, 0);
            if (t >= 0 && o < a.d_out) yv[mb][i] = *(const uint4 *)(a.y + (int64_t)t * a.ldy + o);
        }

    // ---- the tile's pairs: which expert (as the plan saw it) -> inv; the h vector -> head and tail.
    //      Several pairs per thread at a time, so that their loads travel together. ----
    constexpr int NB = RP <= 16 ? 4 : (RP == 32 ? 2 : 1);
    for (int q0 = tid; q0 < TM * K; q0 += NB * NTD) {
        int key[NB];
        uint32_t hv[NB][RP];
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int q = q0 + i * NTD;
            const int t = q < TM * K ? tokM[q / K] : -1;
            key[i] = -1;
            if (t < 0) continue;
            const int64_t p = (int64_t)t * K + (q - (q / K) * K);
            key[i] = a.key_of[p];                                       // (-1: not in the plan)
            const uint32_t *hp = a.h + p * RP;
            if constexpr (RP >= 4) {
#pragma unroll
                for (int u = 0; u < RP / 4; ++u) { const uint4 v = ((const uint4 *)hp)[u]; hv[i][4 * u] = v.x; hv[i][4 * u + 1] = v.y; hv[i][4 * u + 2] = v.z; hv[i][4 * u + 3] = v.w; }
            } else {
#pragma unroll
                for (int j = 0; j < RP; ++j) hv[i][j] = hp[j];
            }
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int q = q0 + i * NTD, m = q / K, k = q - m * K;
            const int e = key[i] - s * E;
            if (key[i] < 0 || e < 0 || e >= E) continue;                // (its vector is never looked at)
            inv[m * L.inv_ld + (RPE == 8 ? (e & 1) * L.inv_half + (e >> 1) : e)] = (uint8_t)k;
            uint16_t *dh = hch + q * RPE, *dl = hcl + q * RPE;
            if constexpr (RP >= 8) {
#pragma unroll
                for (int u = 0; u < RP / 8; ++u) {
                    const uint32_t *v = hv[i] + 8 * u;
                    ((uint4 *)dh)[u] = make_uint4((v[0] & 0xffffu) | (v[1] << 16), (v[2] & 0xffffu) | (v[3] << 16),
                                                  (v[4] & 0xffffu) | (v[5] << 16), (v[6] & 0xffffu) | (v[7] << 16));
                    ((uint4 *)dl)[u] = make_uint4((v[0] >> 16) | (v[1] & 0xffff0000u), (v[2] >> 16) | (v[3] & 0xffff0000u),
                                                  (v[4] >> 16) | (v[5] & 0xffff0000u), (v[6] >> 16) | (v[7] & 0xffff0000u));
                }
            } else {
                uint32_t ph[4] = {0u, 0u, 0u, 0u}, pl[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int j = 0; j < RP; ++j) { ph[j >> 1] |= (hv[i][j] & 0xffffu) << (16 * (j & 1)); pl[j >> 1] |= (hv[i][j] >> 16) << (16 * (j & 1)); }
                *(uint4 *)dh = make_uint4(ph[0], ph[1], ph[2], ph[3]);
                *(uint4 *)dl = make_uint4(pl[0], pl[1], pl[2], pl[3]);
            }
        }
    }
    __syncthreads();

    // ---- the contraction: no barrier from here to the epilogue ----
    f32x16_t acc[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc[mb] = f32x16_t{0};
    const uint8_t *inv_lane = inv + am * L.inv_ld + (RPE == 8 ? kg * L.inv_half : 0);
    auto chunk = [&](int c, auto bufc) __attribute__((always_inline)) {
        constexpr int bi = decltype(bufc)::value;
        {
            const int c2 = c + 1;
            const uint32_t m2 = __builtin_amdgcn_readfirstlane(c2 < n_chunks ? (uint32_t)live_l[c2] : 0u);
            load_chunk_b(c2, IntC<(bi + 1) % 2>{}, m2);
        }
        const uint32_t mask = __builtin_amdgcn_readfirstlane((uint32_t)live_l[c]);
        if (mask == 0u) return;
        // which of the token's pairs each step's expert is, for this lane's token of every block
        uint64_t sel[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const uint8_t *p = inv_lane + mb * 32 * L.inv_ld;
            if constexpr (RPE <= 16) { const uint2 v = *(const uint2 *)(p + 8 * c); sel[mb] = (uint64_t)v.y << 32 | v.x; }
            else if constexpr (RPE == 32) sel[mb] = *(const uint32_t *)(p + 4 * c);
            else sel[mb] = *(const uint16_t *)(p + 2 * c);
        }
#pragma unroll
        for (int st = 0; st < NST; ++st) {
            if (!(mask >> st & 1u)) continue;
            constexpr int per = RPE <= 16 ? 1 : RPE / 16;                     // steps per expert
            const int j0 = RPE == 8 ? 0 : (RPE == 16 ? kg * 8 : (st % per) * 16 + kg * 8);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                if (mb * 32 >= rows) continue;
                const uint32_t kb = (uint32_t)(sel[mb] >> (8 * (st / per))) & 0xffu;
                const int row = kb == 0xffu ? zero_row : (mb * 32 + am) * K + (int)kb;
                const uint4 ah = *(const uint4 *)(hch + row * RPE + j0);
                const uint4 al = *(const uint4 *)(hcl + row * RPE + j0);
                acc[mb] = mfma32d(ah, bq[bi][st], acc[mb]);
                acc[mb] = mfma32d(al, bq[bi][st], acc[mb]);
            }
        }
    };
    for (int c = 0; c < n_chunks; c += 2) {
        chunk(c, IntC<0>{});
        if (c + 1 < n_chunks) chunk(c + 1, IntC<1>{});
    }

    // ---- accumulators -> staging block (the tables are dead) -> y, whole 16-byte row pieces ----
    float *stg = (float *)lds;
    __syncthreads();
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        if (mb * 32 >= rows) break;
#pragma unroll
        for (int i = 0; i < 16; ++i) stg[((i >> 2) * 8 + kg * 4 + (i & 3)) * STG_LD + w * 32 + am] = acc[mb][i];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < YP; ++i) {
            const int q = tid + i * NTD, m = q / (TN / 8), oc = (q - m * (TN / 8)) * 8, o = nt * TN + oc;
            if (mb * 32 + m >= rows || o >= a.d_out) continue;
            const uint4 y0 = yv[mb][i];
            const float4 d0 = *(const float4 *)(stg + m * STG_LD + oc), d1 = *(const float4 *)(stg + m * STG_LD + oc + 4);
            uint4 out;
            out.x = pack_bf2(bf_lo(y0.x) + d0.x, bf_hi(y0.x) + d0.y);
            out.y = pack_bf2(bf_lo(y0.y) + d0.z, bf_hi(y0.y) + d0.w);
            out.z = pack_bf2(bf_lo(y0.z) + d1.x, bf_hi(y0.z) + d1.y);
            out.w = pack_bf2(bf_lo(y0.w) + d1.z, bf_hi(y0.w) + d1.w);
            *(uint4 *)(a.y + (int64_t)tokM[mb * 32 + m] * a.ldy + o) = out;
        }
        __syncthreads();
    }
}

// First launch for padded ranks up to 16: one wave per chunk record of the plan (up to four pairs of
// one (slot, expert) group, their ids inside the record).  The lanes split d_in in 16-byte units; the
// chunk's x rows go against the adapter's A rows (fp32 sums per lane, one transposing reduction over
// the wave), and pair p's  h = w[p] * (alpha / r) * A x[p]  is left as bf16 head | tail words.  What a
// wave costs is its dependent round trips (record -> rows; a second flight when d_in is above 512);
// with a wave per chunk they all travel at once and the launch runs at the memory system's rate.
// A group of more than four pairs is several neighbouring records, hence neighbouring waves that run
// at the same time and find the adapter's rows in L2 after the first of them.  (One wave per GROUP,
// walking the group's pairs four at a time, came back for A a few microseconds later, when the rows
// had left L2 again: 18 MB of 94 MB fetched at the c4 shapes, 21.3 against 17.5 us.)
// Workgroup b sits on XCD b % 8: two workgroups of an XCD share a run of 8 records.
template <int RP>
__global__ __launch_bounds__(256)
void moe_down_shrink_kernel(const MoeDownArgs a)
{
    constexpr int CB = kChunk, NV = CB * RP;
    static_assert(kChunk == 4 && kRec == 8, "record layout: two 16-byte loads");
    const int lane = (int)threadIdx.x & 63;
    const int b = (int)blockIdx.x, q = b >> 3;
    const int c = __builtin_amdgcn_readfirstlane((((q >> 1) * 8 + (b & 7)) * 2 + (q & 1)) * 4 + ((int)threadIdx.x >> 6));
    if (c >= a.chunk_bound) return;
    const int4 *rec = (const int4 *)(a.chunks + (int64_t)c * kRec);
    const int4 r0 = rec[0], r1 = rec[1];
    const int key = __builtin_amdgcn_readfirstlane(r0.x), cnt = __builtin_amdgcn_readfirstlane(r0.y);
    if (cnt <= 0) return;                                                 // past the live chunks
    int p[CB];
    p[0] = __builtin_amdgcn_readfirstlane(r1.x); p[1] = __builtin_amdgcn_readfirstlane(r1.y);
    p[2] = __builtin_amdgcn_readfirstlane(r1.z); p[3] = __builtin_amdgcn_readfirstlane(r1.w);
#pragma unroll
    for (int i = 1; i < CB; ++i) p[i] = i < cnt ? p[i] : p[0];
    const int U = a.d_in >> 3;
    const int s = key / a.E;
    const uint4 *Ag = (const uint4 *)(a.a_tab + (int64_t)key * RP * a.d_in);
    const uint4 *xp[CB];
#pragma unroll
    for (int i = 0; i < CB; ++i) xp[i] = (const uint4 *)(a.x + (int64_t)p[i] * a.ldx);
    uint4 av[RP], xv[CB];
    auto load_flight = [&](int u0) __attribute__((always_inline)) {
        const int u = u0 + lane, uc = u < U ? u : 0;
#pragma unroll
        for (int j = 0; j < RP; ++j) av[j] = Ag[(int64_t)j * U + uc];
#pragma unroll
        for (int i = 0; i < CB; ++i) if (i < cnt) xv[i] = xp[i][uc];
    };
    load_flight(0);
    const int p_l = lane == 1 ? p[1] : (lane == 2 ? p[2] : (lane == 3 ? p[3] : p[0]));
    const float w_l = lane < cnt ? a.pair_w[p_l] : 0.f;
    const int r_s = a.rank[s];
    const float scale = a.scale[s];
    float acc[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) acc[i] = 0.f;
    for (int u0 = 0; u0 < U; u0 += 64) {
        if (u0 > 0) load_flight(u0);
        const bool in = u0 + lane < U;
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            if (i >= cnt) continue;
            const uint4 xz = in ? xv[i] : make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int j = 0; j < RP; ++j) acc[i * RP + j] = dot8(xz, av[j], acc[i * RP + j]);
        }
    }
    if (r_s <= 0) return;                                                 // the slot holds no adapter at this site
    wave_sum_transpose<NV>(acc, lane);
    const int idx = bitrev<Log2<NV>::v>(lane & (NV - 1)), ci = idx / RP, j = idx - ci * RP;
    const int pc = __shfl(p_l, ci, 64);
    const float wc = __shfl(w_l, ci, 64);
    if (lane < NV && ci < cnt) {
        const float f = acc[0] * scale * wc;
        const uint32_t hi = __float_as_uint(f) & 0xffff0000u;                 // head truncated, tail rounded
        a.h[(int64_t)pc * RP + j] = (hi >> 16) | (f2bf(f - __uint_as_float(hi)) << 16);
    }
}

bool moe_down_shrinks_by_wave(int r_pad) { return r_pad <= 16; }

hipError_t launch_moe_down_shrink(const MoeDownArgs &a, hipStream_t st)
{
    const int64_t groups = (int64_t)a.n_slots * a.E;
    if (groups <= 0 || a.T <= 0) return hipSuccess;
    if (!a.chunks || a.chunk_bound <= 0) return hipErrorInvalidValue;
    // 64 records per round of the eight XCDs (two workgroups of four waves each per XCD)
    const dim3 grid((unsigned)(((int64_t)a.chunk_bound + 63) / 64 * 16)), block(256);
    switch (a.r_pad) {
        case 1:  moe_down_shrink_kernel<1><<<grid, block, 0, st>>>(a); break;
        case 2:  moe_down_shrink_kernel<2><<<grid, block, 0, st>>>(a); break;
        case 4:  moe_down_shrink_kernel<4><<<grid, block, 0, st>>>(a); break;
        case 8:  moe_down_shrink_kernel<8><<<grid, block, 0, st>>>(a); break;
        case 16: moe_down_shrink_kernel<16><<<grid, block, 0, st>>>(a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

int moe_down_tile_rows(int r_pad, int K, int E) { return 32 * down_blocks(r_pad, K, E); }
int moe_down_tile_cols() { return TN; }
int moe_down_max_k() { return KMAX; }

template <int RP, int MB>
static hipError_t launch_moe_down_mb(const MoeDownArgs &a, hipStream_t st)
{
    const int dyn = down_dyn_bytes(RP < 8 ? 8 : RP, 32 * MB, a.K, a.E);
    // (a kernel may use more than 64 KB of dynamic LDS only after this call, per device; devices are few)
    static std::atomic<uint64_t> allowed{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!(allowed.load(std::memory_order_acquire) >> dev & 1u)) {
        if (hipFuncSetAttribute((const void *)moe_down_kernel<RP, MB>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsOne) != hipSuccess)
            return hipErrorUnknown;
        allowed.fetch_or(1ull << dev, std::memory_order_release);
    }
    const dim3 grid((unsigned)((int64_t)a.n_mtiles * a.n_ntiles)), block(NTD);
    moe_down_kernel<RP, MB><<<grid, block, (size_t)dyn, st>>>(a);
    return hipGetLastError();
}

template <int RP>
static hipError_t launch_moe_down_rp(const MoeDownArgs &a, hipStream_t st)
{
    switch (down_blocks(RP, a.K, a.E)) {
        case 3: return launch_moe_down_mb<RP, 3>(a, st);
        case 2: return launch_moe_down_mb<RP, 2>(a, st);
        case 1: return launch_moe_down_mb<RP, 1>(a, st);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_moe_down(const MoeDownArgs &a, hipStream_t st)
{
    if (a.T <= 0) return hipSuccess;
    if (a.K > KMAX || a.n_ntiles != (a.d_out + TN - 1) / TN) return hipErrorInvalidValue;
    if ((int64_t)a.E * a.d_out * a.r_pad * 2 >= ((int64_t)1 << 32)) return hipErrorInvalidValue;   // 32-bit offsets inside a slot's B
    switch (a.r_pad) {
        case 1:  return launch_moe_down_rp<1>(a, st);
        case 2:  return launch_moe_down_rp<2>(a, st);
        case 4:  return launch_moe_down_rp<4>(a, st);
        case 8:  return launch_moe_down_rp<8>(a, st);
        case 16: return launch_moe_down_rp<16>(a, st);
        case 32: return launch_moe_down_rp<32>(a, st);
        case 64: return launch_moe_down_rp<64>(a, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace mlora
