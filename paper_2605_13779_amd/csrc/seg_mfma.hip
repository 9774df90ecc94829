// Rank-64 segmented (prefill) LoRA apply on the gfx950 matrix cores: a shrink half and an expand half, run
// as one launch (seg_fused_kernel, the default) or as two.
//
// All rows of a segment use one adapter (a request's prompt is one contiguous run), so both halves
// are dense contractions on the matrix cores (v_mfma_f32_32x32x16_bf16 in the shrink,
// v_mfma_f32_16x16x32_bf16 in the expand):
//
//   shrink  hp[j][64 rows x 64]  = X[64 rows x k-slice j] * A_s^T[k-slice j x 64]
//           A workgroup owns a tile of up to 64 consecutive rows of one segment and one k-slice of
//           d_in; x and A_s pieces are staged through LDS (coalesced 16-byte loads in, MFMA operand
//           layout out), so the adapter rows are read once per 64 rows.  The fp32 partial sums go to
//           a small device buffer (16 KB per tile and k-slice; it stays in L2).  The workgroup that
//           finishes a tile's last k-slice adds the slices in slice order, scales in fp32 and writes
//           h as bf16 head + tail (16 mantissa bits reach the expand's MFMA; the shrink result is
//           never rounded to bf16).  Nobody waits: whoever arrives last does the sum.
//   expand  Y[rows x 512 outputs] += h * B_s^T
//           A workgroup owns a slice of 512 outputs of a group of rows; every group is the same
//           number of 32-row blocks (cut wherever that falls, inside or across segments), so the
//           launch is one round of equal items.  Every wave keeps its 64 rows of B_s in registers
//           (fetched again where the adapter changes inside the group) and walks the rows 32 at a
//           time, with the next block's h and y already requested.  The accumulators pass
//           through a wave-private LDS tile so that the in-place bf16 add on y moves row-contiguous
//           16-byte pieces.
//
// As two launches, the stream order between them is the only dependency between workgroups that anyone
// waits for; in the one-launch form the expand's workgroups wait for per-tile flags instead (see
// seg_fused_kernel).  What the tiling buys: per 64 rows the shrink pulls one copy of the adapter's A rows
// through the CU's L1, and the expand pulls B_s once per run instead of once per 32 rows; with
// 32-row tiles that re-read both, adapter bytes were more than half of all L1 traffic.
#include "internal.h"
#include <type_traits>

namespace mlora {

namespace {
constexpr int TM = 64;            // rows per shrink tile
constexpr int NW = 8;             // waves per workgroup
constexpr int NT = NW * 64;
constexpr int KU = 128;           // elements of d_in per unit of the shrink (8 MFMA k steps)
constexpr int UROW = KU * 2 + 16; // padded byte stride of a staged row (x or A)
constexpr int STAGE_BYTES = (TM + 64) * UROW;
constexpr int RED_BYTES = 2 * TM * 64 * 4;                // the two k halves of a unit
constexpr int kWaitVm0 = 0x0F70; // s_waitcnt vmcnt(0) with the other counters left alone (gfx9 encoding)
constexpr int ES = 512;           // outputs per expand slice (64 per wave)
constexpr int H_LD = 72;          // padded row stride of the bf16 h tiles, in elements
constexpr int ST_LD = 68;         // padded row stride of a wave's 16 x 64 staging tile, in floats
constexpr int SHRINK_LDS = 2 * STAGE_BYTES;                          // two stage buffers, used in turn
constexpr int EXPAND_H_BYTES = 2 * 2 * 32 * H_LD * 2;                // two buffers of bf16 heads and tails of a 32-row block
constexpr int EXPAND_LDS = EXPAND_H_BYTES + NW * 16 * ST_LD * 4;    // ... and a staging tile per wave
constexpr int kFlagSpin = 1 << 20;                                  // polls of a tile's flag (one launch: never reached)
static_assert(RED_BYTES <= STAGE_BYTES, "partials reuse the staging area");
static_assert(sizeof(SegArgs) + 8 <= 4096, "kernel arguments (with the one-launch form's block count) stay within 4 KB");
}

__device__ __forceinline__ f32x16_t mfma32(const uint4 &a, const uint4 &b, f32x16_t c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// 16 x 16 x 32: lane l supplies 8 consecutive k (at 8 * (l / 16)) of row / column l % 16; accumulator
// register i of lane l is row 4 * (l / 16) + i, column l % 16.
__device__ __forceinline__ f32x4_t mfma16(const uint4 &a, const uint4 &b, f32x4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// 32 x 32 x 16: accumulator register i of lane l holds row (i/4)*8 + (l/32)*4 + i%4, column l%32.
__device__ __forceinline__ int acc_row(int i, int kh) { return (i >> 2) * 8 + kh * 4 + (i & 3); }

template <typename F>
__device__ __forceinline__ void static_for2(F &&f)
{
    f(std::integral_constant<int, 0>{});
    f(std::integral_constant<int, 1>{});
}

// Table records, from the kernel arguments when the batch is small enough to carry them there.
struct SegRec { int slot, row0, rows, tile0; };
__device__ __forceinline__ SegRec seg_tile(const SegArgs &a, int i)
{
    if (a.inl_on) {
        const uint32_t w0 = a.inl[2 * i], w1 = a.inl[2 * i + 1];
        return {(int)(w1 & 0xffffu), (int)w0, (int)(w1 >> 16), 0};
    }
    return {a.tiles[4 * i], a.tiles[4 * i + 1], a.tiles[4 * i + 2], 0};
}
__device__ __forceinline__ SegRec seg_range(const SegArgs &a, int j)
{
    if (a.inl_on) {
        const uint32_t *r = a.inl + 2 * a.n_tiles + 3 * j;
        return {(int)(r[1] & 0xffffu), (int)r[0], (int)(r[1] >> 16), (int)r[2]};
    }
    return {a.ranges[4 * j], a.ranges[4 * j + 1], a.ranges[4 * j + 2], a.ranges[4 * j + 3]};
}
__device__ __forceinline__ int seg_group_off(const SegArgs &a, int g)
{
    return a.inl_on ? (int)a.inl[2 * a.n_tiles + 3 * a.n_ranges + g] : a.groups[g];
}

// Workgroups are dealt round-robin to the 8 XCDs; work ids are laid out so that an XCD gets a
// contiguous range of them (neighbouring ids share adapter bytes, which then sit in that XCD's L2).
__device__ __forceinline__ int xcd_contiguous_id(int block, int n_blocks)
{
    return (block & 7) * (n_blocks >> 3) + (block >> 3);
}

// Shrink.  The work is the list of all (tile, k-unit) pairs, tile-major (a k-unit is KU elements of
// d_in); workgroup b of n takes the contiguous share [b*U/n, (b+1)*U/n) of it, so every workgroup
// moves the same number of bytes whatever the segment lengths are.  A share usually covers the end
// of one tile and the start of the next; each piece is a partial sum, and the workgroup that delivers
// a tile's last piece adds the pieces in share order (a fixed order: the result does not depend on
// who is last) and writes h.
//
// Every global access is a whole 16 bytes per lane with neighbouring lanes on neighbouring
// addresses; LDS turns those row-major pieces into the MFMA operand layout, where a lane owns
// eight consecutive k of one row.  (Loading operands straight from global memory in that layout
// touches 32 different lines per instruction and thrashes the small L1.)  Three units are in flight
// in registers while a fourth is multiplied; their loads are unconditional, so that the compiler can
// wait for the oldest and leave the others in flight.
struct ShrinkShare {
    int64_t U;        // all units
    int32_t n;        // workgroups
    // workgroup that owns unit u: the smallest b with (b + 1) * U / n > u
    __device__ int owner(int64_t u) const { return (int)(((u + 1) * n + U - 1) / U) - 1; }
};

// FUSED: the expand runs in the same launch, on other XCDs too, so h is written with device-scope stores
// and each tile's flag is set to the launch's epoch once its h is complete.
template <bool FUSED>
__device__ __forceinline__ void seg_shrink_body(const SegArgs &a, const int b, unsigned char *buf2, const uint32_t epoch)
{
    __shared__ int s_last;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, m = lane & 31, kh = lane >> 5;
    if (b >= a.n_swg) return;
    const ShrinkShare sh{(int64_t)a.n_tiles * a.upt, a.n_swg};
    const int64_t u0 = (int64_t)b * sh.U / sh.n, u1 = (int64_t)(b + 1) * sh.U / sh.n;
    const int n = (int)(u1 - u0);
    if (n <= 0) return;

    // staged row r: 0..63 = x rows of the tile, 64..127 = A rows; this thread moves rows srow + 32 q
    const int srow = tid >> 4, sseg = tid & 15;
    // ---- fetch side: walks the share unit by unit ----
    int f_tile = (int)(u0 / a.upt), f_ku = (int)(u0 - (int64_t)f_tile * a.upt), f_left = n;
    const char *f_a = nullptr;
    int64_t f_x[2];
    auto f_open = [&]() {                              // addresses for the tile the fetch side is in
        const SegRec t = seg_tile(a, f_tile);
        const int slot = max(t.slot, 0), row0 = t.row0, nrows = t.rows;
        f_a = (const char *)(a.a_tab + (int64_t)slot * 64 * a.d_in);
#pragma unroll
        for (int q = 0; q < 2; ++q) f_x[q] = (int64_t)(row0 + min(srow + 32 * q, nrows - 1)) * a.ldx * 2;
    };
    f_open();
    auto fetch = [&](uint4 (&st)[4]) {                 // unconditional; past the share it repeats the last unit
        const int k = min(f_ku * KU + sseg * 8, a.d_in - 8);
#pragma unroll
        for (int q = 0; q < 2; ++q) st[q] = ld_stream((const char *)a.x + f_x[q] + (int64_t)k * 2);
#pragma unroll
        for (int q = 0; q < 2; ++q) st[2 + q] = *(const uint4 *)(f_a + ((int64_t)(srow + 32 * q) * a.d_in + k) * 2);
        if (--f_left > 0) {
            if (++f_ku == a.upt) { f_ku = 0; ++f_tile; f_open(); }
        }
    };
    // ---- multiply side ----
    // wave w: row block rb against adapter-row block cb, k steps kh2*4 .. kh2*4+3 of each unit
    const int rb = w & 1, cb = (w >> 1) & 1, kh2 = w >> 2;
    int c_tile = (int)(u0 / a.upt), c_ku = (int)(u0 - (int64_t)c_tile * a.upt);
    f32x16_t acc = {0};
    // this share's piece of tile c_tile is complete; buf is the stage buffer that was multiplied last
    auto finish_tile = [&](unsigned char *buf) {
        const SegRec ct = seg_tile(a, c_tile);
        const int slot = ct.slot, nrows = ct.rows;
        __syncthreads();                               // the staged unit has been read by every wave
        float *red = (float *)buf;                     // [k half][64 rows][64 adapter rows]
#pragma unroll
        for (int i = 0; i < 16; ++i) red[((kh2 * TM) + rb * 32 + acc_row(i, kh)) * 64 + cb * 32 + m] = acc[i];
        acc = f32x16_t{0};
        __syncthreads();
        const bool live = slot >= 0 && a.meta.rank[slot] > 0;     // the expand skips the same tiles
        const int first = sh.owner((int64_t)c_tile * a.upt), pieces = sh.owner((int64_t)c_tile * a.upt + a.upt - 1) - first + 1;
        float4 mine[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int e4 = tid + NT * q, row = e4 >> 4, c4 = e4 & 15;
            const float4 p0 = *(const float4 *)(red + row * 64 + c4 * 4);
            const float4 p1 = *(const float4 *)(red + (TM + row) * 64 + c4 * 4);
            mine[q] = make_float4(p0.x + p1.x, p0.y + p1.y, p0.z + p1.z, p0.w + p1.w);
        }
        bool last = true;
        if (live && pieces > 1) {
            // piece ids are unique: workgroup + tile grows from one piece to the next
            uint64_t *part = (uint64_t *)(a.hpart + (int64_t)(b + c_tile) * (TM * 64));
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int e4 = tid + NT * q;
                if ((e4 >> 4) < nrows) {
                    __hip_atomic_store(part + e4 * 2, ((uint64_t)__float_as_uint(mine[q].y) << 32) | __float_as_uint(mine[q].x), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(part + e4 * 2 + 1, ((uint64_t)__float_as_uint(mine[q].w) << 32) | __float_as_uint(mine[q].z), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            // Every thread's words have been acknowledged at device scope before the tile's counter
            // moves, and the last arriver reads them with device-scope loads after it has seen the
            // count.  (Release and acquire fences would do the same by writing back and invalidating
            // the whole L2, which holds the adapter rows everybody is reading.)  The wait also drains
            // the units in flight; it happens once or twice per workgroup.
            __builtin_amdgcn_s_waitcnt(kWaitVm0);
            __syncthreads();
            if (tid == 0) {
                const int old = __hip_atomic_fetch_add(a.hcount + c_tile, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                s_last = old == pieces - 1;
                if (s_last) __hip_atomic_store(a.hcount + c_tile, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
            }
            __syncthreads();
            last = s_last != 0;
        }
        if (live && last) {
            const float scale = a.meta.scale[slot];
            uint16_t *hf = a.hfin + (int64_t)c_tile * (TM * 128);  // per row: 64 heads, then 64 tails
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int e4 = tid + NT * q, row = e4 >> 4, c4 = e4 & 15;
                if (row >= nrows) continue;
                float4 s = mine[q];
                if (pieces > 1) {
                    s = make_float4(0.f, 0.f, 0.f, 0.f);
                    const uint64_t *src = (const uint64_t *)(a.hpart + (int64_t)(first + c_tile) * (TM * 64)) + e4 * 2;
                    for (int k0 = 0; k0 < pieces; k0 += 4) {       // four pieces in flight at a time, added in order
                        uint64_t w0[4], w1[4];
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            const int kk = min(k0 + k, pieces - 1);
                            w0[k] = __hip_atomic_load(src + (int64_t)kk * (TM * 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            w1[k] = __hip_atomic_load(src + (int64_t)kk * (TM * 32) + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            if (k0 + k < pieces) {
                                s.x += __uint_as_float((uint32_t)w0[k]); s.y += __uint_as_float((uint32_t)(w0[k] >> 32));
                                s.z += __uint_as_float((uint32_t)w1[k]); s.w += __uint_as_float((uint32_t)(w1[k] >> 32));
                            }
                        }
                    }
                }
                const float f[4] = {s.x * scale, s.y * scale, s.z * scale, s.w * scale};
                uint32_t hi[4], lo[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    hi[k] = f2bf(f[k]);
                    lo[k] = f2bf(f[k] - __uint_as_float(hi[k] << 16));
                }
                const uint64_t hw = (uint64_t)(hi[2] | (hi[3] << 16)) << 32 | (hi[0] | (hi[1] << 16));
                const uint64_t lw = (uint64_t)(lo[2] | (lo[3] << 16)) << 32 | (lo[0] | (lo[1] << 16));
                if constexpr (FUSED) {
                    __hip_atomic_store((uint64_t *)(hf + row * 128 + c4 * 4), hw, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store((uint64_t *)(hf + row * 128 + 64 + c4 * 4), lw, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    *(uint64_t *)(hf + row * 128 + c4 * 4) = hw;
                    *(uint64_t *)(hf + row * 128 + 64 + c4 * 4) = lw;
                }
            }
        }
        if constexpr (FUSED) {
            // the tile's h has been acknowledged at device scope before its flag shows the epoch
            // (tiles without adapter get their flag too: nobody reads their h, but nobody waits in vain)
            if (last) {
                __builtin_amdgcn_s_waitcnt(kWaitVm0);
                __syncthreads();
                if (tid == 0) __hip_atomic_store(a.hflag + c_tile, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        // Every path through here ends with nothing in flight, and the compiler is told so (a wait it
        // can see, not inline assembly): otherwise it assumes that loads of this block may still be
        // pending where the paths join again and drains the prefetched units in front of every fetch.
        __builtin_amdgcn_s_waitcnt(kWaitVm0);
        __syncthreads();                               // the partials' LDS is staged into again
    };
    int c_left = n;
    // One barrier per unit: a unit is written into the buffer that was multiplied two units ago, and
    // every wave has passed the barrier in between.
    int c_par = 0;
    auto consume = [&](uint4 (&st)[4]) {
        const bool in = c_ku * KU + sseg * 8 < a.d_in; // d_in is a multiple of 16: a 16-byte piece is in or out as a whole
        unsigned char *buf = buf2 + c_par * STAGE_BYTES;
        c_par ^= 1;
#pragma unroll
        for (int q = 0; q < 4; ++q) *(uint4 *)(buf + (srow + 32 * q) * UROW + sseg * 16) = in ? st[q] : make_uint4(0, 0, 0, 0);
        __syncthreads();
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int kb = (kh2 * 4 + s) * 32 + kh * 16;   // byte offset of this lane's 8 k values
            const uint4 xv = *(const uint4 *)(buf + (rb * 32 + m) * UROW + kb);
            const uint4 av = *(const uint4 *)(buf + (64 + cb * 32 + m) * UROW + kb);
            acc = mfma32(xv, av, acc);
        }
        --c_left;
        if (++c_ku == a.upt || c_left == 0) {
            finish_tile(buf);
            c_ku = 0; ++c_tile;
        }
    };

    uint4 s0[4], s1[4], s2[4];
    fetch(s0); fetch(s1); fetch(s2);
    const int rounds = n / 3, rest = n - rounds * 3;
    for (int r = 0; r + 1 < rounds; ++r) {
        consume(s0); fetch(s0);
        consume(s1); fetch(s1);
        consume(s2); fetch(s2);
    }
    if (rounds > 0) {                                  // last full round: refill only what the rest needs
        consume(s0); if (rest > 0) fetch(s0);
        consume(s1); if (rest > 1) fetch(s1);
        consume(s2);
    }
    if (rest > 0) consume(s0);
    if (rest > 1) consume(s1);
}

__global__ __launch_bounds__(NT, 4)
void seg_shrink_kernel(const SegArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[SHRINK_LDS];
    seg_shrink_body<false>(a, xcd_contiguous_id((int)blockIdx.x, (int)gridDim.x), lds, 0u);
}

// Loads are issued unconditionally (clamped addresses): the compiler can wait for one load while
// younger ones stay in flight only if it knows how many were issued after it; a load under a
// run-time condition turns every later wait into a full drain.
// FUSED: the shrink runs in the same launch; a piece's rows are worked on once the flags of the tiles
// they lie in show the launch's epoch (B_s and the first y pieces are requested before the wait), and h
// is read with device-scope loads.
template <bool FUSED>
__device__ __forceinline__ void seg_expand_body(const SegArgs &a, const int id, unsigned char *lds, const uint32_t epoch)
{
    uint16_t *const hh0 = (uint16_t *)lds, *const hl0 = hh0 + 2 * 32 * H_LD;
    float *const stg_all0 = (float *)(lds + EXPAND_H_BYTES);
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, m = lane & 31, kh = lane >> 5;
    if (id >= a.n_groups * a.n_slices) return;
    // The output slices of one group of rows are neighbours (same XCD, started together): between
    // them they sweep whole rows of y, which the memory side serves better than the same slice of
    // many row ranges (1 KB pieces 14 KB apart per workgroup either way), and they share the rows' h.
    const int grp = id / a.n_slices, sl = id - grp * a.n_slices;
    const int p_end = seg_group_off(a, grp + 1);
    int slot = -1, row0 = 0, nrows = 0;

    // this wave's 64 rows of B_s, as operands of the 16 x 16 x 32 MFMA: bv[cb][ks] = ranks
    // ks*32 + kq*8 .. +7 of row o_w + cb*16 + mm
    const int mm = lane & 15, kq = lane >> 4;
    const int o_w = sl * ES + w * 64;
    uint4 bv[4][2];
    auto b_load = [&]() {
        const uint16_t *Bg = a.b_tab + (int64_t)slot * a.d_out * 64;
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) {
            const int o = min(o_w + cb * 16 + mm, a.d_out - 1);
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) bv[cb][ks] = *(const uint4 *)(Bg + (int64_t)o * 64 + ks * 32 + kq * 8);
        }
    };
    // h of a 32-row block is 32 x 256 bytes (64 heads, 64 tails per row): one 16-byte piece per thread
    const int hrow = tid >> 4, hpc = tid & 15;
    const uint16_t *hf0 = a.hfin + hpc * 8;            // + (hfin row of the piece's first row) * 128, per piece
    uint4 hv;
    auto h_fetch = [&](int blk) {
        const int r = min(blk * 32 + hrow, nrows - 1);
        if constexpr (FUSED) {
            const uint64_t *src = (const uint64_t *)(hf0 + (int64_t)r * 128);
            const uint64_t v0 = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint64_t v1 = __hip_atomic_load(src + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            hv = make_uint4((uint32_t)v0, (uint32_t)(v0 >> 32), (uint32_t)v1, (uint32_t)(v1 >> 32));
        } else {
            hv = *(const uint4 *)(hf0 + (int64_t)r * 128);
        }
    };
    auto h_store = [&](int buf_i) {
        uint16_t *dst = hpc < 8 ? hh0 + buf_i * (32 * H_LD) + hrow * H_LD + hpc * 8 : hl0 + buf_i * (32 * H_LD) + hrow * H_LD + (hpc - 8) * 8;
        *(uint4 *)dst = hv;
    };

    // y pieces: 8 lanes cover the 128 bytes (64 outputs) of one row, 8 rows per round; a block is
    // handled as two halves of 16 rows so that the wave's staging tile stays small
    const int og = lane & 7, tr = lane >> 3;
    const int oc = min(o_w + og * 8, a.d_out - 8);
    const bool col_ok = o_w + og * 8 < a.d_out;
    float *stg = stg_all0 + w * (16 * ST_LD);
    uint4 yv[2][2];
    auto y_fetch = [&](int blk, auto half_c) {
        constexpr int half = decltype(half_c)::value;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int tok = min(blk * 32 + half * 16 + tr + 8 * q, nrows - 1);
            yv[half][q] = *(const uint4 *)(a.y + (int64_t)(row0 + tok) * a.ldy + oc);
        }
    };

    // One 32-row block: MORE = a next block exists; its h and y pieces are requested while this block
    // is worked on (unconditionally, so that the waits can leave them in flight).
    auto block = [&](int blk, auto more_c) {
        constexpr bool MORE = decltype(more_c)::value;
        const int cur = blk & 1;
        if constexpr (MORE) h_fetch(blk + 1);
        static_for2([&](auto half_c) {
            constexpr int half = decltype(half_c)::value;
            // 16 rows x 64 outputs: four 16-wide blocks, two k steps of 32 ranks, head and tail of h
            f32x4_t acc[4];
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) acc[cb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const uint4 hA = *(const uint4 *)(hh0 + cur * (32 * H_LD) + (half * 16 + mm) * H_LD + ks * 32 + kq * 8);
                const uint4 lA = *(const uint4 *)(hl0 + cur * (32 * H_LD) + (half * 16 + mm) * H_LD + ks * 32 + kq * 8);
#pragma unroll
                for (int cb = 0; cb < 4; ++cb) {
                    acc[cb] = mfma16(hA, bv[cb][ks], acc[cb]);
                    acc[cb] = mfma16(lA, bv[cb][ks], acc[cb]);
                }
            }
            // The staging tile is private to the wave and LDS serves a wave's requests in order, so
            // compiler-level fences are all that is needed between its phases.
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                for (int i = 0; i < 4; ++i) stg[(4 * kq + i) * ST_LD + cb * 16 + mm] = acc[cb][i];
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int trow = tr + 8 * q, tok = blk * 32 + half * 16 + trow;
                const float4 d0 = *(const float4 *)(stg + trow * ST_LD + og * 8);
                const float4 d1 = *(const float4 *)(stg + trow * ST_LD + og * 8 + 4);
                const uint4 yo = yv[half][q];
                uint4 o;
                o.x = pack_bf2(bf_lo(yo.x) + d0.x, bf_hi(yo.x) + d0.y);
                o.y = pack_bf2(bf_lo(yo.y) + d0.z, bf_hi(yo.y) + d0.w);
                o.z = pack_bf2(bf_lo(yo.z) + d1.x, bf_hi(yo.z) + d1.y);
                o.w = pack_bf2(bf_lo(yo.w) + d1.z, bf_hi(yo.w) + d1.w);
                if (tok < nrows && col_ok) st_quiet(a.y + (int64_t)(row0 + tok) * a.ldy + oc, o);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");     // reads of the tile precede its reuse
            if constexpr (MORE) y_fetch(blk + 1, half_c);              // into the registers just used
        });
        if constexpr (MORE) {
            h_store(cur ^ 1);
            __syncthreads();                           // h tile cur has been read by all; tile cur^1 is complete
        }
    };
    // The group's pieces in turn; B_s is fetched again only where the adapter changes (a segment
    // boundary inside the group).
    bool first = true;
    for (int p = seg_group_off(a, grp); p < p_end; ++p) {
        const SegRec rr = seg_range(a, p);
        if (rr.slot < 0 || a.meta.rank[rr.slot] <= 0) continue;      // the shrink skips the same rows
        if (!first) __syncthreads();                   // the last h tile of the piece before has been read by all
        first = false;
        if (rr.slot != slot) { slot = rr.slot; b_load(); }
        row0 = rr.row0; nrows = rr.rows;
        hf0 = a.hfin + (int64_t)rr.tile0 * 128 + hpc * 8;
        const int n_blk = (nrows + 31) >> 5;
        if constexpr (FUSED) {
            if (tid == 0) {                        // the tiles these rows lie in: h complete?
                int spins = 0;
                for (int ti = rr.tile0 >> 6; ti <= (rr.tile0 + nrows - 1) >> 6; ++ti)
                    while (__hip_atomic_load(a.hflag + ti, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != epoch) {
                        if (++spins > kFlagSpin) { __hip_atomic_store(a.hctrl + 1, 3u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); break; }
                        __builtin_amdgcn_s_sleep(8);
                    }
            }
            __syncthreads();
            // (h, which is wanted first, is requested first: with the first y pieces on their way from in
            // front of the wait for the flags, h came back behind them -- 2 us per call at 7168 outputs)
            h_fetch(0);
            y_fetch(0, std::integral_constant<int, 0>{});
            y_fetch(0, std::integral_constant<int, 1>{});
        } else {
            h_fetch(0);
            y_fetch(0, std::integral_constant<int, 0>{});
            y_fetch(0, std::integral_constant<int, 1>{});
        }
        h_store(0);
        __syncthreads();
        for (int blk = 0; blk + 1 < n_blk; ++blk) block(blk, std::true_type{});
        block(n_blk - 1, std::false_type{});
    }
}

__global__ __launch_bounds__(NT, 4)
void seg_expand_kernel(const SegArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[EXPAND_LDS];
    seg_expand_body<false>(a, xcd_contiguous_id((int)blockIdx.x, (int)gridDim.x), lds, 0u);
}

// Both halves in one launch: the first n_sblocks workgroups shrink, the others expand.  All shrink
// workgroups are resident from the start (the host keeps their number within what the GPU holds), they
// never wait for anybody, and an expand workgroup waits only for flags that they set: nothing can
// deadlock, and the waits are bounded all the same (on giving up a workgroup raises the site's error
// word and goes on).  The epoch that the flags carry lives in device memory and is advanced by the
// launch's last workgroup (as the exchange tag of the decode launches is), so that a replayed graph,
// which repeats the kernel arguments, still gets a fresh one.
__global__ __launch_bounds__(NT, 4)
void seg_fused_kernel(const SegArgs a, const int n_sblocks)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[SHRINK_LDS > EXPAND_LDS ? SHRINK_LDS : EXPAND_LDS];
    __shared__ uint32_t s_epoch;
    const int blk = (int)blockIdx.x, n_blk = (int)gridDim.x;
    if (threadIdx.x == 0) {
        const uint32_t e = tag_read(a.hctrl);
        s_epoch = e;
        (void)__hip_atomic_fetch_add(a.hctrl + 8 + (blk & 63), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    const uint32_t epoch = s_epoch;
    if (blk < n_sblocks) seg_shrink_body<true>(a, xcd_contiguous_id(blk, n_sblocks), lds, epoch);
    else seg_expand_body<true>(a, xcd_contiguous_id(blk - n_sblocks, n_blk - n_sblocks), lds, epoch);
    if (blk == n_blk - 1 && threadIdx.x < 64) {
        // every workgroup has signed in (all are past their first instructions or done): next epoch
        const int lane = (int)threadIdx.x;
        uint32_t total = 0;
        for (int spins = 0; spins < kSpinLimit; ++spins) {
            int c = (int)__hip_atomic_load(a.hctrl + 8 + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) c += __shfl_xor(c, d, 64);
            total = (uint32_t)c;
            if (total >= (uint32_t)n_blk) break;
            __builtin_amdgcn_s_sleep(2);
        }
        __hip_atomic_store(a.hctrl + 8 + lane, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (lane == 0) {
            if (total < (uint32_t)n_blk) __hip_atomic_store(a.hctrl + 1, 3u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // never expected
            __hip_atomic_store(a.hctrl, epoch + 1 == 0u ? 1u : epoch + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

int seg_unit() { return KU; }

int seg_shrink_capacity()
{
    static int cap = 0;
    if (cap == 0) {
        int per_cu = 0, cus = 0, dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, seg_shrink_kernel, NT, 0) != hipSuccess) return 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cap = per_cu * cus;
    }
    return cap;
}

int seg_expand_capacity()
{
    static int cap = 0;
    if (cap == 0) {
        int per_cu = 0, cus = 0, dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, seg_expand_kernel, NT, 0) != hipSuccess) return 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cap = per_cu * cus;
    }
    return cap;
}

int seg_fused_capacity()
{
    static int cap = 0;
    if (cap == 0) {
        int per_cu = 0, cus = 0, dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, seg_fused_kernel, NT, 0) != hipSuccess) return 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cap = per_cu * cus;
    }
    return cap;
}

// Shrink and expand of one batch in one launch (a.hctrl / a.hflag set; a.n_swg within seg_fused_capacity()).
hipError_t launch_seg_fused(const SegArgs &a, hipStream_t st)
{
    if (a.n_tiles <= 0 || a.n_ranges <= 0 || a.n_groups <= 0) return hipSuccess;
    if (a.n_swg < 1 || a.upt != (a.d_in + KU - 1) / KU || !a.hctrl || !a.hflag) return hipErrorInvalidValue;
    const int gs = (a.n_swg + 7) / 8 * 8;
    if (gs > seg_fused_capacity()) return hipErrorInvalidValue;
    const int ge = (int)(((int64_t)a.n_groups * a.n_slices + 7) / 8 * 8);
    seg_fused_kernel<<<dim3((unsigned)(gs + ge)), dim3(NT), 0, st>>>(a, gs);
    return hipGetLastError();
}

hipError_t launch_seg_shrink(const SegArgs &a, hipStream_t st)
{
    if (a.n_tiles <= 0 || a.n_ranges <= 0 || a.n_groups <= 0) return hipSuccess;
    if (a.n_swg < 1 || a.upt != (a.d_in + KU - 1) / KU) return hipErrorInvalidValue;
    const unsigned gs = (unsigned)((a.n_swg + 7) / 8 * 8);
    seg_shrink_kernel<<<dim3(gs), dim3(NT), 0, st>>>(a);
    return hipGetLastError();
}

hipError_t launch_seg_expand(const SegArgs &a, hipStream_t st)
{
    if (a.n_tiles <= 0 || a.n_ranges <= 0 || a.n_groups <= 0) return hipSuccess;
    const unsigned ge = (unsigned)(((int64_t)a.n_groups * a.n_slices + 7) / 8 * 8);
    seg_expand_kernel<<<dim3(ge), dim3(NT), 0, st>>>(a);
    return hipGetLastError();
}

}  // namespace mlora
