// Internal declarations shared by the mlora translation units (host launchers + device helpers).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/mlora.h"

namespace mlora {

constexpr int kChunk = MLORA_CHUNK;
constexpr int kRec = 4 + kChunk;

// Device view of a site's metadata block: rank | scale | catalog_id.
struct MetaView {
    const int32_t *rank;
    const float   *scale;
};

// Device view of a plan buffer (all int32).  A chunk record is kRec ints:
//   [0] key (dense: slot; MoE: slot*E + expert)  [1] count (1..kChunk)  [2] start in `sorted`
//   [3] unused  [4 .. 4+kChunk) the row ids of the chunk, ascending
// Records past the live chunks of a batch have count 0.
// so that a workgroup learns everything about its chunk from one 48-byte read.
struct PlanView {
    int32_t *hdr;         // [8]  hdr[0] = number of chunks, hdr[1] = number of usable rows
    int32_t *count;       // [n_keys + 1]  zero between calls
    int32_t *group_off;   // [n_keys + 1]
    int32_t *chunk_base;  // [n_keys + 1]
    int32_t *key_of;      // [max_items]
    int32_t *ticket;      // [max_items]
    int32_t *tmp;         // [max_items]
    int32_t *sorted;      // [max_items]
    int32_t *chunks;      // [kRec * max_chunks]
    // Route plans also group the batch's TOKENS by slot (the MoE down projection sums a token's pairs
    // into one output row and works per slot): tok_hdr[1] = usable tokens, tok_off = exclusive prefix
    // of the slots' token counts, tok_sorted = tokens grouped by slot, ascending inside a slot; the
    // rest is the planner's working space for that grouping.
    int32_t *tok_hdr;     // [8]
    int32_t *tok_count;   // [n_keys + 1]  zero between calls
    int32_t *tok_off;     // [n_keys + 1]
    int32_t *tok_key_of;  // [max_items]
    int32_t *tok_ticket;  // [max_items]
    int32_t *tok_tmp;     // [max_items]
    int32_t *tok_sorted;  // [max_items]
};
// The view the planner kernels take for the token-level grouping (no chunk records).
__host__ __device__ inline PlanView plan_token_view(const PlanView &v)
{
    PlanView t{};
    t.hdr = v.tok_hdr; t.count = v.tok_count; t.group_off = v.tok_off; t.chunk_base = nullptr;
    t.key_of = v.tok_key_of; t.ticket = v.tok_ticket; t.tmp = v.tok_tmp; t.sorted = v.tok_sorted; t.chunks = nullptr;
    return t;
}

size_t plan_words(int64_t max_items, int64_t n_keys);
PlanView plan_view(void *base, int64_t max_items, int64_t n_keys);
inline int64_t max_chunks(int64_t items, int64_t n_keys)
{
    // sum over groups of ceil(n_g / kChunk) <= (items + (kChunk - 1) * groups) / kChunk
    int64_t touched = n_keys < items ? n_keys : items;
    return (items + (kChunk - 1) * touched) / kChunk;
}

// plan.hip
hipError_t launch_plan_dense_small(const PlanView &pv, const int32_t *token_slot, int T, int n_slots,
                                   const int32_t *ready_rank, hipStream_t st);
hipError_t launch_plan_general(const PlanView &pv, const int32_t *topk, const int32_t *token_slot,
                               int T, int K, int E, int n_slots, const int32_t *ready_rank,
                               int32_t *out_sorted, int32_t *out_group_off, hipStream_t st);
hipError_t launch_fill_i32(int32_t *p, int32_t v, int64_t n, hipStream_t st);

// rows.hip: vector-ALU apply over plan chunks (decode, MoE, small-rank segmented)
struct RowsArgs {
    const uint16_t *x; int64_t ldx;
    uint16_t *y;       int64_t ldy;
    const uint16_t *a_tab; const uint16_t *b_tab;
    MetaView meta;
    const int32_t *chunks;   // kRec ints per chunk
    int32_t d_in, d_out, r_pad;
    int32_t n_experts;       // >= 1: key / n_experts = slot
    int32_t top_k;           // x row = item / top_k
    int32_t grid_chunks;     // upper bound on the number of chunks
    // exchange area of the site (null on sites that only run fused launches)
    uint64_t *xch;           // [xch_chunks][<= 128 values][kChunk] words
    uint32_t *ctrl;          // [0] launch tag, [1] error flag, [8..72) sign-ins
    int32_t xch_chunks;
    // filled in by the launcher
    int32_t mode;            // 0 nothing crosses workgroups; 2 parts that trade k-slices
    int32_t ksplit, kslice_units;
    int32_t tile_par;        // parts a chunk is cut into (one item each; 1 = one item per chunk): part p expands
    int32_t out_per_part;    // outputs [p * out_per_part, ...) and, in mode 2, shrinks k-slice p
    int32_t poll_limit;      // polls of an exchange word before a reader takes the item on its own
    int32_t rank_bound;      // 1: read the slot's rank first and fetch only that many rows of A
    // ungrouped launch (ranks 1 and 2 only): item i is row i with slot row_slot[i]; `chunks` is not read
    const int32_t *row_slot;
    int32_t row_slots;       // slots the site holds (indices outside [0, row_slots) leave the row untouched)
    // MoE down projection, first launch: no expand; row p's scaled h times row_w[p] goes to
    // h_out[p][r_pad], one word per value (bf16 head | bf16 tail << 16); the second launch
    // (moe_down.hip) multiplies it with the B tables on the matrix cores, token by token
    uint32_t *h_out;
    const float *row_w;
#ifdef MLORA_PROF
    uint64_t *prof;          // per-workgroup phase timestamps (builds with -DMLORA_PROF only)
#endif
};
hipError_t launch_rows(const RowsArgs &a, hipStream_t st);
constexpr int kMaxMulti = 4;     // sites per grouped launch
int rows_group_waves(const RowsArgs &a);
bool rows_plans_alone(const RowsArgs &a);
int rows_local_plan_rows();
int rows_local_plan_slots();
hipError_t launch_rows_multi_plan(const RowsArgs *sites, int n, const PlanView &pv, const int32_t *token_slot, int T,
                                  int n_slots, const int32_t *ready_rank, hipStream_t st);
hipError_t launch_rows_multi(const RowsArgs *sites, int n, hipStream_t st);

// moe_down.hip: second launch of the MoE down projection (expand + routing-weight combine on the matrix cores)
struct MoeDownArgs {
    uint16_t *y; int64_t ldy;
    const uint16_t *b_tab;       // [n_slots][E][d_out][r_pad]
    const int32_t *rank;         // [n_slots]
    uint32_t *h;                 // [T*K][r_pad]: written by the first launch, read by the second
    const int32_t *key_of;       // [T*K] the plan's key of each pair (slot * E + expert, -1: not in the plan)
    const int32_t *sorted;       // the plan's pairs grouped by (slot, expert)
    const int32_t *group_off;    // [n_slots*E + 1]
    const int32_t *tok_sorted;   // the plan's tokens grouped by slot
    const int32_t *tok_off;      // [n_slots + 1]
    int32_t T, K, E, n_slots, d_out, r_pad;
    int32_t n_mtiles;            // upper bound on the number of token tiles: T / tile + n_slots
    int32_t n_ntiles;            // output tiles per token tile
    // first launch (one wave per chunk record) only:
    const uint16_t *x; int64_t ldx;   // one input row per pair
    const uint16_t *a_tab;            // [n_slots][E][r_pad][d_in]
    const float *scale;               // [n_slots] alpha / r
    const float *pair_w;              // [T*K] routing weights
    int32_t d_in;
    const int32_t *chunks;            // the plan's chunk records (kRec ints: key, count, -, -, the chunk's pairs)
    int32_t chunk_bound;              // records to look at (those past the live chunks have count 0)
};
bool moe_down_shrinks_by_wave(int r_pad);
hipError_t launch_moe_down_shrink(const MoeDownArgs &a, hipStream_t st);
hipError_t launch_moe_down(const MoeDownArgs &a, hipStream_t st);
int moe_down_tile_rows(int r_pad, int K, int E);   // 0: this shape does not fit
int moe_down_tile_cols();
int moe_down_max_k();

// seg_mfma.hip: rank-64 segmented apply on the matrix cores (a shrink launch, then an expand launch)
constexpr int kSegInline = 832;   // words of tables inside the kernel arguments (the whole argument block stays below 4 KB)
struct SegArgs {
    const uint16_t *x; int64_t ldx;
    uint16_t *y;       int64_t ldy;
    const uint16_t *a_tab; const uint16_t *b_tab;
    MetaView meta;
    const int32_t *tiles;    // [4 * n_tiles]: slot, first row, rows (<= 64), 0 -- consecutive pieces of the segments
    int32_t n_tiles;
    // Expand work: a piece is a run of rows of one segment (slot, first row, rows, row of hfin that
    // holds its first row's h); it starts on a 32-row block of a tile.  Workgroup group g owns the
    // pieces [groups[g], groups[g + 1]): every group has the same number of 32-row blocks (+-1).
    const int32_t *ranges;   // [4 * n_ranges] pieces
    int32_t n_ranges;
    const int32_t *groups;   // [n_groups + 1]
    int32_t n_groups;
    int32_t d_in, d_out;
    float *hpart;            // [n_swg + n_tiles][64 rows][64] fp32 partial shrink results, one block per (workgroup, tile) piece
    uint16_t *hfin;          // [n_tiles][64 rows][64 bf16 heads | 64 bf16 tails] scaled shrink result
    int32_t *hcount;         // [n_tiles] pieces that have arrived; zero between launches
    uint32_t *hctrl;         // one-launch form: [0] epoch, [1] error word, [8..72) sign-ins
    uint32_t *hflag;         // one-launch form: [n_tiles] epoch of the launch that completed the tile's h
    int32_t upt;             // units of d_in per tile (a unit is seg_unit() elements)
    int32_t n_swg;           // workgroups of the shrink launch; n_swg * 3 <= n_tiles * upt
    int32_t n_slices;        // output slices of 512
    // Small batches carry both tables inside the kernel arguments (no table copy in front of the
    // launches): tile i = words 2i (first row) and 2i + 1 (slot | rows << 16), piece j = words
    // 2 * n_tiles + 3j (first row), + 1 (slot | rows << 16), + 2 (hfin row), then n_groups + 1 words
    // of group offsets.  inl_on = 0: read tiles / ranges / groups.
    int32_t inl_on;
    uint32_t inl[kSegInline];
};
hipError_t launch_seg_shrink(const SegArgs &a, hipStream_t st);
hipError_t launch_seg_expand(const SegArgs &a, hipStream_t st);
hipError_t launch_seg_fused(const SegArgs &a, hipStream_t st);
int seg_fused_capacity();
int seg_unit();
int seg_shrink_capacity();
int seg_expand_capacity();

// Launch-shape overrides (mlora_set_tuning): one relaxed atomic per knob, 0 = automatic.  Sweeps and
// tests set them; the launch code reads each knob it needs once per call.
enum Knob {
    kRowsPollLimit, kRowsRankBound, kRowsItemsTarget, kRowsMode, kRowsWaves, kPlanGeneral, kPlanSeparate,
    kPlanPipeline, kSegExpandGroups, kSegTableCopy, kSegShrinkWgs, kSegNoMfma, kSegOverlap, kUploadPieceKb, kSegFused,
    kRowsChunkRun, kKnobCount
};
int tuning(Knob k);             // api.hip
#ifdef MLORA_PROF
uint64_t *debug_prof();         // api.hip (builds with -DMLORA_PROF only)
#endif

}  // namespace mlora

#ifdef __HIPCC__
namespace mlora {

// a compile-time integer as a function argument (static loops over register arrays)
template <int I> struct IntC { static constexpr int value = I; };

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;

// ---- exchange of partial results between workgroups of ONE launch ----------------------------
// A word is (launch tag << 32) | fp32 bits, written and read with single relaxed device-scope
// 64-bit accesses, so a reader that sees the tag also sees the value and no fences are needed.
// The tag must differ from launch to launch, also when a captured graph replays the same kernel
// arguments, so it lives in device memory (ctrl[0]): every workgroup reads it, then signs in with a
// fire-and-forget add on one of 64 counters (ctrl[8..72)); the last workgroup of the grid, once its
// own work is done, sees all sign-ins, clears the counters and advances the tag.  ctrl[1] is an
// error flag raised when a bounded wait gives up.
constexpr int kSpinLimit = 1 << 18;
constexpr uint32_t kTagPoison = 0xffffffffu;   // exchange switched off after a bounded wait gave up (see tag_advance)
// Polls of an exchange word before a reader computes the value itself (a partner can start late).
// The two ways of getting the value add the same terms in a different order, so an output can differ
// by one rounding step between them; both are within the tolerance of the result.
constexpr int kPollLimit = 4096;

__device__ __forceinline__ void xch_put(uint64_t *p, float v, uint32_t tag)
{
    __hip_atomic_store(p, ((uint64_t)tag << 32) | __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t xch_get(const uint64_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t tag_read(const uint32_t *ctrl)
{
    return __hip_atomic_load(ctrl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// One thread per workgroup, after its tag_read has returned (the branch makes the add depend on it).
__device__ __forceinline__ void tag_sign_in(uint32_t *ctrl, int wg, uint32_t tag)
{
    if (tag != kTagPoison)
        (void)__hip_atomic_fetch_add(ctrl + 8 + (wg & 63), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Called by one full wave of the last workgroup of the grid when its work is done.
__device__ __forceinline__ void tag_advance(uint32_t *ctrl, int n_wg, uint32_t tag, int lane)
{
    uint32_t total = 0;
    for (int spins = 0; spins < kSpinLimit; ++spins) {
        int c = (int)__hip_atomic_load(ctrl + 8 + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) c += __shfl_xor(c, d, 64);
        total = (uint32_t)c;
        if (total >= (uint32_t)n_wg) break;
        __builtin_amdgcn_s_sleep(2);
    }
    if (total >= (uint32_t)n_wg) {
        __hip_atomic_store(ctrl + 8 + lane, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (lane == 0) {
            uint32_t nt = tag + 1;
            if (nt == 0 || nt == kTagPoison) nt = 1;
            __hip_atomic_store(ctrl, nt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    } else if (lane == 0) {
        // Never expected.  The sign-in count can no longer be trusted, so no later launch may take a
        // word of the exchange area for current: the tag is set to a value under which every item runs
        // on its own (whole shrink, nothing published, nothing awaited; results stay right) until
        // mlora_site_check has reported the flag and reset the control block.
        __hip_atomic_store(ctrl, kTagPoison, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(ctrl + 1, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Streaming accesses (touched once per launch): the non-temporal hint keeps them from pushing
// the adapter tables, which are re-read by many workgroups, out of L2.
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
__device__ __forceinline__ uint4 ld_stream(const void *p)
{
    const u32x4_t v = __builtin_nontemporal_load((const u32x4_t *)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st_stream(void *p, const uint4 &v)
{
    u32x4_t t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, (u32x4_t *)p);
}

// Stores the compiler's wait-count bookkeeping does not see.  With a store it knows of still in
// flight, the compiler can only wait for a load result by draining every outstanding memory
// operation (loads and stores retire in order among themselves, not against each other), which
// ends any prefetch of the next tile.  Issued this way, a store only makes a later wait a little
// longer while it is unacknowledged: the hardware counter still includes it.  The data registers
// are read when the instruction issues; they may be reused right away.
__device__ __forceinline__ void st_quiet(void *p, const uint4 &v)
{
    u32x4_t t = {v.x, v.y, v.z, v.w};
    asm volatile("global_store_dwordx4 %0, %1, off" : : "v"(p), "v"(t) : "memory");
}
__device__ __forceinline__ void st_quiet_stream(void *p, const uint4 &v)
{
    u32x4_t t = {v.x, v.y, v.z, v.w};
    asm volatile("global_store_dwordx4 %0, %1, off nt" : : "v"(p), "v"(t) : "memory");
}
__device__ __forceinline__ void st_quiet(void *p, uint2 v)
{
    asm volatile("global_store_dwordx2 %0, %1, off" : : "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void st_quiet(void *p, uint32_t v)
{
    asm volatile("global_store_dword %0, %1, off" : : "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void st_quiet(void *p, uint16_t v)
{
    const uint32_t t = v;
    asm volatile("global_store_short %0, %1, off" : : "v"(p), "v"(t) : "memory");
}

__device__ __forceinline__ float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even; NaN stays NaN.
__device__ __forceinline__ uint32_t f2bf(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
// Two fp32 -> packed bf16 in one instruction (v_cvt_pk_bf16_f32: round to nearest even, NaN kept);
// bit-identical to f2bf on every input.
__device__ __forceinline__ uint32_t pack_bf2(float lo, float hi)
{
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// a.lo*b.lo + a.hi*b.hi + c on packed bf16 pairs, fp32 accumulate (v_dot2c_f32_bf16).
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a),
                                           __builtin_bit_cast(bf16x2_t, b), c, false);
}
__device__ __forceinline__ float dot8(const uint4 &a, const uint4 &b, float c)
{
    c = dot2(a.x, b.x, c); c = dot2(a.y, b.y, c); c = dot2(a.z, b.z, c); c = dot2(a.w, b.w, c);
    return c;
}

}  // namespace mlora
#endif
