// C-ABI entry points: validation, slot bookkeeping and launch configuration.  All arithmetic of
// the LoRA apply runs in the kernels of rows.hip / seg_mfma.hip / plan.hip.
#include "internal.h"

#include <algorithm>
#include <cstring>
#include <atomic>
#include <mutex>
#include <new>
#include <vector>

using namespace mlora;

struct mlora_plan {
    int32_t max_items, n_keys, device;
    PlanView pv;
    // what the last planning call put in it (host-side knowledge only)
    int32_t items, top_k, n_experts, n_slots, grid_chunks;
    bool moe;
};

struct mlora_site {
    mlora_site_desc d;
    int32_t r_pad, E;
    uint16_t *a_tab, *b_tab;
    int32_t *rank;
    float *scale;
    int64_t *catalog;
    mlora_plan priv;            // private plan living in the caller-provided scratch
    uint32_t *ctrl;             // dense sites: launch tag / sign-in counters of launches whose workgroups trade partial sums
    uint64_t *xch;              // dense sites: partial shrink results in flight between workgroups
    int32_t *seg_dev;           // device area for segment tiles / chunks
    int32_t seg_cap;            // in entries of 3 ints
    int32_t *stage[2];          // pinned host staging for the segment tables (lazy)
    hipEvent_t stage_ev[2];
    bool stage_busy[2];
    int stage_next;
    hipStream_t seg_side = nullptr;   // rank-64 prefill with batches in flight: the shrinks' stream and its events (lazy)
    hipEvent_t seg_ev[5] = {};
    std::vector<int32_t> host_rank;   // what the uploads asked for, per slot (0 = empty): a hint for the launch shape only
    int32_t n_short = 0;        // slots whose rank is below the padded rank of the tables
    void *pack;                 // pinned host image of one slot (A part, then B part) for uploads from per-expert tensors (lazy)
    hipEvent_t pack_ev;
    bool pack_busy;
};

namespace {

constexpr int32_t kDensePrivItems = 1024;      // rows per private dense plan (one-workgroup planner)
constexpr int32_t kMoePrivItems = 131072;      // pairs per private MoE plan
constexpr int32_t kSegCap = 65536;             // segment tiles / chunks per call
constexpr int32_t kXchChunks = 256;            // chunks per launch whose parts may trade partial sums
constexpr size_t kCtrlBytes = 1024;
constexpr size_t kXchBytes = (size_t)kXchChunks * 128 * kChunk * 8;   // <= 128 values per row of a chunk
constexpr size_t kSegXchBytes = (size_t)24 << 20;   // rank-64 sites: exchange words, then the prefill's partial shrink results
// behind the exchange words: tile counters (16 KB), then per tile 16 KB of h (bf16 head + tail), then the
// fp32 partials of the k-slices
constexpr int32_t kSegMaxTiles = 256;              // tiles of 64 rows per batch of launches
constexpr size_t kSegCountBytes = 16384;
constexpr int32_t kSegHpBlocks = (int32_t)((kSegXchBytes - kXchBytes - kSegCountBytes - (size_t)kSegMaxTiles * 16384) / 16384);

std::atomic<int32_t> g_knob[kKnobCount];
const char *const kKnobName[kKnobCount] = {
    "rows_poll_limit", "rows_rank_bound", "rows_items_target", "rows_mode", "rows_waves", "plan_general",
    "plan_separate", "plan_pipeline", "seg_expand_groups", "seg_table_copy", "seg_shrink_wgs", "seg_no_mfma", "seg_overlap",
    "upload_piece_kb", "seg_fused", "rows_chunk_run"};

// Host-side record of a slot's rank (the kernels read the device table; this only tells the launch
// code whether any slot is padded, i.e. whether rank-bounded reads of A can save traffic).
void note_rank(mlora_site *s, int32_t slot, int32_t r)
{
    int32_t &h = s->host_rank[(size_t)slot];
    s->n_short += (int32_t)(r > 0 && r < s->r_pad) - (int32_t)(h > 0 && h < s->r_pad);
    h = r;
}

int32_t round_pow2(int32_t r)
{
    int32_t p = 1;
    while (p < r) p <<= 1;
    return p;
}

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

int32_t check_desc(const mlora_site_desc *d)
{
    if (!d) return MLORA_E_INVALID;
    if (d->d_in <= 0 || d->d_out <= 0 || d->n_slots <= 0 || d->n_experts < 0 || d->device < 0) return MLORA_E_INVALID;
    if (d->r_max < 1 || d->r_max > MLORA_MAX_RANK) return MLORA_E_SHAPE;
    if ((d->d_in & 7) || (d->d_out & 7)) return MLORA_E_SHAPE;
    int64_t keys = (int64_t)d->n_slots * (d->n_experts > 0 ? d->n_experts : 1);
    if (keys > (1 << 24)) return MLORA_E_UNSUPPORTED;
    return MLORA_OK;
}

int32_t priv_items(const mlora_site_desc *d) { return d->n_experts > 0 ? kMoePrivItems : kDensePrivItems; }

__global__ void meta_set_kernel(int32_t *rank, float *scale, int64_t *catalog, int slot, int r, float s, int64_t id)
{
    rank[slot] = r; scale[slot] = s; catalog[slot] = id;
}

// token -> slot through the catalog ids the slots hold: the lowest ready slot whose id matches, else -1.
// One workgroup per 256 tokens; the id table (<= a few KB) is staged in LDS in pieces.
__global__ __launch_bounds__(256)
void slot_lookup_kernel(const int64_t *token_id, int T, const int64_t *catalog, const int32_t *rank, int n_slots,
                        int32_t *token_slot)
{
    __shared__ int64_t ids[1024];
    const int t = (int)(blockIdx.x * 256 + threadIdx.x);
    const int64_t want = t < T ? token_id[t] : -1;
    int found = -1;
    for (int base = 0; base < n_slots; base += 1024) {
        const int n = min(1024, n_slots - base);
        __syncthreads();
        for (int k = (int)threadIdx.x; k < n; k += 256) ids[k] = rank[base + k] > 0 ? catalog[base + k] : -1;
        __syncthreads();
        if (want >= 0 && found < 0)
            for (int k = 0; k < n; ++k)
                if (ids[k] == want) { found = base + k; break; }
    }
    if (t < T) token_slot[t] = found;
}

__global__ void meta_clear_kernel(int32_t *rank, float *scale, int64_t *catalog, int n)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) { rank[i] = 0; scale[i] = 0.f; catalog[i] = -1; }
}

// Zero the padding of one slot: A rows r..r_pad-1 and B columns r..r_pad-1, for every expert.
__global__ void pad_zero_kernel(uint16_t *a_slot, uint16_t *b_slot, int E, int r, int r_pad, int d_in, int d_out)
{
    const int64_t na = (int64_t)E * (r_pad - r) * d_in, nb = (int64_t)E * d_out * (r_pad - r);
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < na + nb; i += (int64_t)gridDim.x * blockDim.x) {
        if (i < na) {
            int64_t e = i / ((int64_t)(r_pad - r) * d_in), rem = i % ((int64_t)(r_pad - r) * d_in);
            a_slot[e * r_pad * d_in + (int64_t)r * d_in + rem] = 0;
        } else {
            int64_t k = i - na;
            int64_t row = k / (r_pad - r), col = k % (r_pad - r);
            b_slot[row * r_pad + r + col] = 0;
        }
    }
}

bool ok(hipError_t e) { return e == hipSuccess; }

struct DeviceGuard {
    int prev = -1;
    bool good = true;
    explicit DeviceGuard(int dev)
    {
        if (!ok(hipGetDevice(&prev))) { good = false; return; }
        if (prev != dev && !ok(hipSetDevice(dev))) good = false;
        cur = dev;
    }
    ~DeviceGuard() { if (good && prev != cur) (void)hipSetDevice(prev); }
    int cur = -1;
};

int32_t check_xy(const mlora_site *s, const void *x, int64_t ldx, const void *y, int64_t ldy)
{
    if (!s || !x || !y) return MLORA_E_INVALID;
    if (ldx < s->d.d_in || ldy < s->d.d_out || (ldx & 7) || (ldy & 7)) return MLORA_E_SHAPE;
    if (!aligned16(x) || !aligned16(y)) return MLORA_E_SHAPE;
    return MLORA_OK;
}

RowsArgs rows_args(const mlora_site *s, const void *x, int64_t ldx, void *y, int64_t ldy)
{
    RowsArgs a{};
    a.x = (const uint16_t *)x; a.ldx = ldx; a.y = (uint16_t *)y; a.ldy = ldy;
    a.a_tab = s->a_tab; a.b_tab = s->b_tab;
    a.meta.rank = s->rank; a.meta.scale = s->scale;
    a.d_in = s->d.d_in; a.d_out = s->d.d_out; a.r_pad = s->r_pad;
    a.n_experts = s->E; a.top_k = 1;
    a.xch = s->xch; a.ctrl = s->ctrl; a.xch_chunks = s->xch ? kXchChunks : 0;   // a rank-64 site's larger area holds these too
    a.rank_bound = s->n_short > 0 ? 1 : 0;      // the launch code keeps it only where it pays
#ifdef MLORA_PROF
    a.prof = debug_prof();
#endif
    return a;
}

void init_plan(mlora_plan *p, int32_t max_items, int32_t n_keys, int32_t device, void *base)
{
    p->max_items = max_items; p->n_keys = n_keys; p->device = device;
    p->pv = plan_view(base, max_items, n_keys);
    p->items = 0; p->top_k = 1; p->n_experts = 1; p->n_slots = 0; p->grid_chunks = 0; p->moe = false;
}

int32_t plan_decode_impl(mlora_plan *plan, const int32_t *token_slot, int32_t T, int32_t n_slots,
                         const int32_t *ready_rank, hipStream_t st)
{
    if (T > plan->max_items || n_slots > plan->n_keys) return MLORA_E_UNSUPPORTED;
    plan->items = T; plan->top_k = 1; plan->n_experts = 1; plan->n_slots = n_slots; plan->moe = false;
    plan->grid_chunks = (int32_t)max_chunks(T, n_slots);
    hipError_t e;
    if (T <= kDensePrivItems && !tuning(kPlanGeneral))
        e = launch_plan_dense_small(plan->pv, token_slot, T, n_slots, ready_rank, st);
    else
        e = launch_plan_general(plan->pv, nullptr, token_slot, T, 1, 1, n_slots, ready_rank, nullptr, nullptr, st);
    return ok(e) ? MLORA_OK : MLORA_E_HIP;
}

int32_t plan_route_impl(mlora_plan *plan, const int32_t *topk, const int32_t *token_slot, int32_t T, int32_t K,
                        int32_t n_slots, int32_t E, const int32_t *ready_rank,
                        int32_t *out_sorted, int32_t *out_off, hipStream_t st)
{
    const int64_t P = (int64_t)T * K, NK = (int64_t)n_slots * E;
    if (P > plan->max_items || NK > plan->n_keys) return MLORA_E_UNSUPPORTED;
    plan->items = (int32_t)P; plan->top_k = K; plan->n_experts = E; plan->n_slots = n_slots; plan->moe = true;
    plan->grid_chunks = (int32_t)max_chunks(P, NK);
    hipError_t e = launch_plan_general(plan->pv, topk, token_slot, T, K, E, n_slots, ready_rank, out_sorted, out_off, st);
    return ok(e) ? MLORA_OK : MLORA_E_HIP;
}

int32_t apply_planned_impl(mlora_site *s, const mlora_plan *plan, const void *x, int64_t ldx,
                           void *y, int64_t ldy, hipStream_t st)
{
    if (plan->items == 0) return MLORA_OK;
    RowsArgs a = rows_args(s, x, ldx, y, ldy);
    a.chunks = plan->pv.chunks;
    a.top_k = plan->top_k;
    a.grid_chunks = plan->grid_chunks;
    return ok(launch_rows(a, st)) ? MLORA_OK : MLORA_E_HIP;
}

// Copy a small host table to the site's device area through pinned staging (two buffers in turn).
int32_t stage_table(mlora_site *s, const std::vector<int32_t> &tab, hipStream_t st)
{
    const size_t bytes = tab.size() * sizeof(int32_t);
    const int k = s->stage_next;
    if (!s->stage[k]) {
        if (!ok(hipHostMalloc((void **)&s->stage[k], (size_t)kSegCap * 3 * sizeof(int32_t), hipHostMallocDefault))) return MLORA_E_HIP;
        if (!ok(hipEventCreateWithFlags(&s->stage_ev[k], hipEventDisableTiming))) return MLORA_E_HIP;
    }
    if (s->stage_busy[k] && !ok(hipEventSynchronize(s->stage_ev[k]))) return MLORA_E_HIP;
    std::memcpy(s->stage[k], tab.data(), bytes);
    if (!ok(hipMemcpyAsync(s->seg_dev, s->stage[k], bytes, hipMemcpyHostToDevice, st))) return MLORA_E_HIP;
    if (!ok(hipEventRecord(s->stage_ev[k], st))) return MLORA_E_HIP;
    s->stage_busy[k] = true;
    s->stage_next = k ^ 1;
    return MLORA_OK;
}

// The last quarter of the tile-counter block holds what the one-launch form of the prefill needs: 128
// words of control (epoch, error word, sign-in counters), then one flag per tile of a batch.
uint32_t *seg_ctrl_of(const mlora_site *s)
{
    return (uint32_t *)((char *)s->xch + kXchBytes) + (kSegCountBytes / 4 - 1024 - 128);
}
static_assert(kSegMaxTiles <= 1024 && kSegMaxTiles * 4 + (1024 + 128) * 4 <= (int)kSegCountBytes, "counters, control words and flags share the block");

// Batches of the rank-64 prefill with their shrinks on the site's second stream, one batch ahead of the
// expands on the caller's stream.  Batch i uses half i % 2 of the partial-result buffers, so shrink
// i + 2 waits for expand i.  The second stream forks from the caller's stream and is joined back into it
// (the last expand waits for the last shrink), so the call behaves like work on `st` alone, also
// under stream capture.
int32_t launch_seg_overlapped(mlora_site *s, const std::vector<SegArgs> &subs, hipStream_t st)
{
    if (!s->seg_side) {
        if (!ok(hipStreamCreateWithFlags(&s->seg_side, hipStreamNonBlocking))) return MLORA_E_HIP;
        for (int k = 0; k < 5; ++k)
            if (!ok(hipEventCreateWithFlags(&s->seg_ev[k], hipEventDisableTiming))) return MLORA_E_HIP;
    }
    hipEvent_t fork = s->seg_ev[0], *shrunk = s->seg_ev + 1, *expanded = s->seg_ev + 3;
    if (!ok(hipEventRecord(fork, st)) || !ok(hipStreamWaitEvent(s->seg_side, fork, 0))) return MLORA_E_HIP;
    const int n = (int)subs.size();
    for (int i = 0; i < n; ++i) {
        if (i >= 2 && !ok(hipStreamWaitEvent(s->seg_side, expanded[i & 1], 0))) return MLORA_E_HIP;
        if (!ok(launch_seg_shrink(subs[i], s->seg_side)) || !ok(hipEventRecord(shrunk[i & 1], s->seg_side))) return MLORA_E_HIP;
        if (!ok(hipStreamWaitEvent(st, shrunk[i & 1], 0)) || !ok(launch_seg_expand(subs[i], st))) return MLORA_E_HIP;
        if (i + 2 < n && !ok(hipEventRecord(expanded[i & 1], st))) return MLORA_E_HIP;
    }
    return MLORA_OK;
}

// Rank-64 prefill: cut the segments into tiles of 64 rows (shrink items) and into equal groups of
// 32-row blocks (expand items), in batches that fit the partial-result buffer, and launch shrink +
// expand per batch.
int32_t segmented_mfma(mlora_site *s, const void *x, int64_t ldx, void *y, int64_t ldy,
                       const int32_t *seg_off, const int32_t *seg_slot, int32_t S, hipStream_t st)
{
    struct Tile { int32_t slot, row0, rows, seg; };
    std::vector<Tile> tiles;
    for (int32_t k = 0; k < S; ++k) {
        if (seg_slot[k] < 0) continue;
        for (int32_t r0 = seg_off[k]; r0 < seg_off[k + 1]; r0 += 64)
            tiles.push_back({seg_slot[k], r0, seg_off[k + 1] - r0 < 64 ? seg_off[k + 1] - r0 : 64, k});
    }
    if (tiles.empty()) return MLORA_OK;
    const int32_t d_in = s->d.d_in, d_out = s->d.d_out;
    const int32_t n_slices = (d_out + 511) / 512;
    const int64_t n_all = (int64_t)tiles.size();
    const int32_t upt = (d_in + seg_unit() - 1) / seg_unit();
    const int32_t cap = seg_shrink_capacity();
    if (cap <= 0) return MLORA_E_HIP;
    // a batch of launches covers at most kSegMaxTiles tiles, and its shrink pieces fit the buffer
    int64_t batch_tiles = kSegMaxTiles;
    if (batch_tiles > kSegHpBlocks - cap) batch_tiles = kSegHpBlocks - cap;
    if (batch_tiles < 1) return MLORA_E_UNSUPPORTED;
    // The expand's workgroups come in groups of n_slices (one per output slice) that own the same
    // rows.  Every group gets the same number of 32-row blocks (+-1), cut out of the batch's block
    // list wherever that falls -- also inside a segment or across segments (a workgroup then fetches
    // the next adapter's B rows and goes on).  With whole tile runs of single segments as items, the
    // launch ran in two to three rounds of uneven items and its time moved by 15 % with the run length.
    const int32_t cap_e = seg_expand_capacity();
    if (cap_e <= 0) return MLORA_E_HIP;
    int32_t groups_wanted = tuning(kSegExpandGroups);
    if (groups_wanted < 1) groups_wanted = cap_e / n_slices > 0 ? cap_e / n_slices : 1;
    // One batch of launches: tiles [t0, t0 + nt) of the call; `half` selects which half of the partial-result
    // buffers it uses (0: the whole buffers).  Returns the launch arguments in `a` and the tables in `tab`
    // (the caller stages them if they did not fit the kernel arguments).
    auto build_batch = [&](int64_t t0, int32_t nt, int32_t halves, int32_t half, SegArgs &a, std::vector<int32_t> &tab) -> int32_t {
        tab.clear();
        tab.reserve((size_t)nt * 8);
        for (int32_t i = 0; i < nt; ++i) {
            const Tile &t = tiles[t0 + i];
            tab.push_back(t.slot); tab.push_back(t.row0); tab.push_back(t.rows); tab.push_back(0);
        }
        // pieces of the groups: walk the batch's 32-row blocks (tile i has one or two)
        int64_t n_blocks = 0;
        for (int32_t i = 0; i < nt; ++i) n_blocks += tiles[t0 + i].rows > 32 ? 2 : 1;
        const int32_t n_groups = (int32_t)(n_blocks < groups_wanted ? n_blocks : groups_wanted);
        std::vector<int32_t> group_off;
        group_off.reserve((size_t)n_groups + 1);
        int32_t n_ranges = 0;
        {
            int32_t ti = 0, half = 0;                  // next block: half `half` of tile ti
            int64_t b = 0;
            for (int32_t g = 0; g < n_groups; ++g) {
                const int64_t b_end = (int64_t)(g + 1) * n_blocks / n_groups;
                group_off.push_back(n_ranges);
                int32_t cur_seg = -1;
                while (b < b_end) {
                    const Tile &t = tiles[t0 + ti];
                    const int32_t r_off = half * 32;
                    const int32_t rows = (t.rows - r_off) < 32 ? (t.rows - r_off) : 32;
                    const size_t last = tab.size();
                    if (t.seg == cur_seg && tab[last - 3] + tab[last - 2] == t.row0 + r_off) {
                        tab[last - 2] += rows;         // the piece goes on
                    } else {
                        tab.push_back(t.slot); tab.push_back(t.row0 + r_off); tab.push_back(rows); tab.push_back(ti * 64 + r_off);
                        ++n_ranges;
                        cur_seg = t.seg;
                    }
                    ++b;
                    if (half == 0 && t.rows > 32) half = 1; else { half = 0; ++ti; }
                }
            }
            group_off.push_back(n_ranges);
        }
        const size_t groups_at = tab.size();
        tab.insert(tab.end(), group_off.begin(), group_off.end());
        if ((int64_t)tab.size() > (int64_t)s->seg_cap * 3) return MLORA_E_UNSUPPORTED;
        a = SegArgs{};
        // a batch whose tables fit the kernel arguments needs no copy in front of its launches
        bool rows_fit = true;                          // a piece's row count shares a word with its slot
        for (int32_t j = 0; j < n_ranges; ++j) rows_fit = rows_fit && tab[4 * (nt + j) + 2] <= 0xffff;
        a.inl_on = 2 * nt + 3 * n_ranges + n_groups + 1 <= kSegInline && s->d.n_slots <= 0xffff && rows_fit &&
                   !tuning(kSegTableCopy);
        if (a.inl_on) {
            for (int32_t i = 0; i < nt; ++i) {
                a.inl[2 * i] = (uint32_t)tab[4 * i + 1];
                a.inl[2 * i + 1] = (uint32_t)tab[4 * i] | (uint32_t)tab[4 * i + 2] << 16;
            }
            for (int32_t j = 0; j < n_ranges; ++j) {
                const int32_t *r = tab.data() + 4 * (nt + j);
                uint32_t *o = a.inl + 2 * nt + 3 * j;
                o[0] = (uint32_t)r[1]; o[1] = (uint32_t)r[0] | (uint32_t)r[2] << 16; o[2] = (uint32_t)r[3];
            }
            for (int32_t g = 0; g <= n_groups; ++g) a.inl[2 * nt + 3 * n_ranges + g] = (uint32_t)group_off[g];
        }
        a.x = (const uint16_t *)x; a.ldx = ldx; a.y = (uint16_t *)y; a.ldy = ldy;
        a.a_tab = s->a_tab; a.b_tab = s->b_tab; a.meta.rank = s->rank; a.meta.scale = s->scale;
        a.tiles = s->seg_dev; a.n_tiles = nt;
        a.ranges = s->seg_dev + (int64_t)nt * 4; a.n_ranges = n_ranges;
        a.groups = s->seg_dev + (int64_t)groups_at; a.n_groups = n_groups;
        a.d_in = d_in; a.d_out = d_out;
        const int32_t hp_blocks = kSegHpBlocks / halves;
        a.hcount = (int32_t *)((char *)s->xch + kXchBytes);
        a.hfin = (uint16_t *)((char *)a.hcount + kSegCountBytes);
        a.hpart = (float *)((char *)a.hfin + (size_t)kSegMaxTiles * 16384);
        a.hctrl = seg_ctrl_of(s);                      // (one-launch form: epoch, error word, sign-ins; then a flag per tile)
        a.hflag = a.hctrl + 128;
        a.hcount += (size_t)half * (kSegCountBytes / 4 / halves);
        a.hfin += (size_t)half * (kSegMaxTiles / halves) * 8192;
        a.hpart += (size_t)half * hp_blocks * 4096;
        a.upt = upt; a.n_slices = n_slices;
        int64_t swg = (int64_t)nt * upt / 3;               // every workgroup keeps three units in flight
        const int tuned = tuning(kSegShrinkWgs);
        // As many workgroups as the GPU holds at once; a whole number per tile instead, where that
        // still fills three quarters of it: no share then crosses a tile boundary, and a share that
        // does pays a hand-over in the middle of its stream (c5: 405 workgroups, three per tile,
        // 95.2 us per call against 97.3 us with 512).
        int64_t fit = cap;
        if (nt > 0 && cap / nt >= 2 && (int64_t)(cap / nt) * nt * 4 >= (int64_t)cap * 3) fit = (int64_t)(cap / nt) * nt;
        if (swg > (tuned > 0 ? tuned : fit)) swg = tuned > 0 ? tuned : fit;
        if (swg > hp_blocks - nt) swg = hp_blocks - nt;           // one partial block per (workgroup, tile) piece
        a.n_swg = (int32_t)(swg < 1 ? 1 : swg);
        return MLORA_OK;
    };
    SegArgs a;
    std::vector<int32_t> tab;
    // Several batches in flight: the shrinks run on a second stream, one batch ahead of the expands
    // (two halves of the partial-result buffers in turn), so that one batch's hand-over -- the end of
    // its shrink, the start of its expand -- overlaps the neighbouring batches' streams.  Only for
    // batches whose tables travel in the kernel arguments.
    const int32_t n_sub = tuning(kSegOverlap);
    if (n_sub >= 2 && n_all >= 2 * n_sub) {
        int64_t sub_tiles = (n_all + n_sub - 1) / n_sub;
        if (sub_tiles > kSegMaxTiles / 2) sub_tiles = kSegMaxTiles / 2;
        if (sub_tiles > kSegHpBlocks / 2 - cap) sub_tiles = kSegHpBlocks / 2 - cap;
        if (sub_tiles >= 1) {
            std::vector<SegArgs> subs;
            bool all_inline = true;
            int32_t i = 0;
            for (int64_t t0 = 0; t0 < n_all && all_inline; t0 += sub_tiles, ++i) {
                const int32_t nt = (int32_t)(n_all - t0 < sub_tiles ? n_all - t0 : sub_tiles);
                int32_t rc = build_batch(t0, nt, 2, i & 1, a, tab);
                if (rc) return rc;
                all_inline = a.inl_on != 0;
                subs.push_back(a);
            }
            if (all_inline) return launch_seg_overlapped(s, subs, st);
        }
    }
    for (int64_t t0 = 0; t0 < n_all; t0 += batch_tiles) {
        const int32_t nt = (int32_t)(n_all - t0 < batch_tiles ? n_all - t0 : batch_tiles);
        int32_t rc = build_batch(t0, nt, 1, 0, a, tab);
        if (rc) return rc;
        if (!a.inl_on) {
            rc = stage_table(s, tab, st);
            if (rc) return rc;
        }
        // both halves in one launch (the expand's workgroups wait for the flags of their tiles); "seg_fused" = -1:
        // the pair of launches
        if (tuning(kSegFused) >= 0 && (a.n_swg + 7) / 8 * 8 <= seg_fused_capacity()) {
            if (!ok(launch_seg_fused(a, st))) return MLORA_E_HIP;
        } else if (!ok(launch_seg_shrink(a, st)) || !ok(launch_seg_expand(a, st))) return MLORA_E_HIP;
    }
    return MLORA_OK;
}

}  // namespace

#ifdef MLORA_PROF
static uint64_t *g_prof = nullptr;
#endif
namespace mlora {
#ifdef MLORA_PROF
uint64_t *debug_prof() { return g_prof; }
#endif
int tuning(Knob k) { return g_knob[k].load(std::memory_order_relaxed); }
}  // namespace mlora

extern "C" {

#ifdef MLORA_PROF
// Profiling builds only (-DMLORA_PROF; not in the default library, not in the public header): device
// buffer that receives per-workgroup phase timestamps of the vector kernel, 8 x uint64 per
// workgroup; null switches it off.
void mlora_debug_set_prof(void *dev) { g_prof = (uint64_t *)dev; }
#endif

const char *mlora_status_str(int32_t st)
{
    switch (st) {
        case MLORA_OK: return "ok";
        case MLORA_E_INVALID: return "invalid argument";
        case MLORA_E_SHAPE: return "shape, rank or alignment not supported";
        case MLORA_E_SLOT: return "slot index out of range";
        case MLORA_E_SEGMENTS: return "segment offsets malformed";
        case MLORA_E_HIP: return "HIP runtime error";
        case MLORA_E_UNSUPPORTED: return "unsupported call for this site or size";
    }
    return "unknown status";
}

int32_t mlora_set_tuning(const char *name, int32_t value)
{
    if (!name) return MLORA_E_INVALID;
    for (int k = 0; k < kKnobCount; ++k)
        if (std::strcmp(name, kKnobName[k]) == 0) {
            g_knob[k].store(value, std::memory_order_relaxed);
            return MLORA_OK;
        }
    return MLORA_E_INVALID;                        // unknown knob
}

int32_t mlora_site_bytes(const mlora_site_desc *d, size_t *a_tab, size_t *b_tab, size_t *meta, size_t *scratch)
{
    int32_t rc = check_desc(d);
    if (rc) return rc;
    if (!a_tab || !b_tab || !meta || !scratch) return MLORA_E_INVALID;
    const int64_t E = d->n_experts > 0 ? d->n_experts : 1, rp = round_pow2(d->r_max);
    *a_tab = align256((size_t)d->n_slots * E * rp * d->d_in * 2);
    *b_tab = align256((size_t)d->n_slots * E * d->d_out * rp * 2);
    *meta = align256((size_t)d->n_slots * 16);
    *scratch = align256(plan_words(priv_items(d), (int64_t)d->n_slots * E) * 4) + align256((size_t)kSegCap * 3 * 4)
             + (d->n_experts > 0 ? 0 : kCtrlBytes + (round_pow2(d->r_max) == 64 ? kSegXchBytes : kXchBytes));
    return MLORA_OK;
}

int32_t mlora_site_create(const mlora_site_desc *d, void *a_tab, void *b_tab, void *meta, void *scratch, mlora_site **out)
{
    int32_t rc = check_desc(d);
    if (rc) return rc;
    if (!a_tab || !b_tab || !meta || !scratch || !out) return MLORA_E_INVALID;
    if (((uintptr_t)a_tab | (uintptr_t)b_tab | (uintptr_t)meta | (uintptr_t)scratch) & 255) return MLORA_E_SHAPE;
    mlora_site *s = new (std::nothrow) mlora_site();
    if (!s) return MLORA_E_INVALID;
    s->d = *d;
    s->E = d->n_experts > 0 ? d->n_experts : 1;
    s->r_pad = round_pow2(d->r_max);
    s->host_rank.assign((size_t)d->n_slots, 0);
    s->a_tab = (uint16_t *)a_tab; s->b_tab = (uint16_t *)b_tab;
    s->rank = (int32_t *)meta;
    s->scale = (float *)((char *)meta + (size_t)d->n_slots * 4);
    s->catalog = (int64_t *)((char *)meta + (size_t)d->n_slots * 8);
    const int64_t NK = (int64_t)d->n_slots * s->E;
    init_plan(&s->priv, priv_items(d), (int32_t)NK, d->device, scratch);
    s->seg_dev = (int32_t *)((char *)scratch + align256(plan_words(priv_items(d), NK) * 4));
    s->seg_cap = kSegCap;
    s->ctrl = nullptr; s->xch = nullptr;
    if (d->n_experts == 0) {
        s->ctrl = (uint32_t *)((char *)s->seg_dev + align256((size_t)kSegCap * 3 * 4));
        s->xch = (uint64_t *)((char *)s->ctrl + kCtrlBytes);
    }
    s->stage[0] = s->stage[1] = nullptr;
    s->stage_busy[0] = s->stage_busy[1] = false;
    s->stage_next = 0;
    s->pack = nullptr; s->pack_busy = false;
    DeviceGuard g(d->device);
    if (!g.good) { delete s; return MLORA_E_HIP; }
    meta_clear_kernel<<<dim3((d->n_slots + 255) / 256), dim3(256), 0, 0>>>(s->rank, s->scale, s->catalog, d->n_slots);
    hipError_t e = launch_fill_i32(s->priv.pv.hdr, 0, 8 + 3 * (NK + 1), 0);
    if (ok(e)) e = launch_fill_i32(s->priv.pv.tok_hdr, 0, 8 + 2 * (NK + 1), 0);
    if (ok(e) && s->ctrl) {
        e = launch_fill_i32((int32_t *)s->ctrl, 0, (int64_t)((kCtrlBytes + (s->r_pad == 64 ? kSegXchBytes : kXchBytes)) / 4), 0);   // tag 0 = never written
        if (ok(e)) e = launch_fill_i32((int32_t *)s->ctrl, 1, 1, 0);                               // first launch tag
        if (ok(e) && s->r_pad == 64) e = launch_fill_i32((int32_t *)seg_ctrl_of(s), 1, 1, 0);      // ... and the prefill's first epoch
    }
    if (!ok(e) || !ok(hipGetLastError()) || !ok(hipStreamSynchronize(0))) { delete s; return MLORA_E_HIP; }
    *out = s;
    return MLORA_OK;
}

void mlora_site_destroy(mlora_site *s)
{
    if (!s) return;
    for (int k = 0; k < 2; ++k)
        if (s->stage[k]) {
            if (s->stage_busy[k]) (void)hipEventSynchronize(s->stage_ev[k]);
            (void)hipEventDestroy(s->stage_ev[k]);
            (void)hipHostFree(s->stage[k]);
        }
    if (s->seg_side) {
        (void)hipStreamSynchronize(s->seg_side);
        for (int k = 0; k < 5; ++k) if (s->seg_ev[k]) (void)hipEventDestroy(s->seg_ev[k]);
        (void)hipStreamDestroy(s->seg_side);
    }
    if (s->pack) {
        if (s->pack_busy) (void)hipEventSynchronize(s->pack_ev);
        (void)hipEventDestroy(s->pack_ev);
        (void)hipHostFree(s->pack);
    }
    delete s;
}

int32_t lora_slots_upload(mlora_site *s, int32_t slot, int64_t catalog_id, const void *A, const void *B,
                          int32_t r, float alpha, int32_t src_on_device, void *stream)
{
    if (!s || !A || !B) return MLORA_E_INVALID;
    if (slot < 0 || slot >= s->d.n_slots) return MLORA_E_SLOT;
    if (r < 1 || r > s->d.r_max) return MLORA_E_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    DeviceGuard g(s->d.device);
    if (!g.good) return MLORA_E_HIP;
    const int64_t E = s->E, rp = s->r_pad, d_in = s->d.d_in, d_out = s->d.d_out;
    uint16_t *a_slot = s->a_tab + (int64_t)slot * E * rp * d_in;
    uint16_t *b_slot = s->b_tab + (int64_t)slot * E * d_out * rp;
    const hipMemcpyKind kind = src_on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
    // take the slot out of service while its bytes change
    meta_set_kernel<<<dim3(1), dim3(1), 0, st>>>(s->rank, s->scale, s->catalog, slot, 0, 0.f, -1);
    if (r < rp) {
        int64_t n = E * (rp - r) * (d_in + d_out);
        unsigned blocks = (unsigned)((n + 255) / 256);
        if (blocks > 4096) blocks = 4096;
        pad_zero_kernel<<<dim3(blocks), dim3(256), 0, st>>>(a_slot, b_slot, (int)E, r, (int)rp, (int)d_in, (int)d_out);
    }
    hipError_t e;
    if (r == rp) {
        e = hipMemcpyAsync(a_slot, A, (size_t)E * r * d_in * 2, kind, st);
        if (ok(e)) e = hipMemcpyAsync(b_slot, B, (size_t)E * d_out * r * 2, kind, st);
    } else {
        e = hipMemcpy2DAsync(a_slot, (size_t)rp * d_in * 2, A, (size_t)r * d_in * 2, (size_t)r * d_in * 2, (size_t)E, kind, st);
        if (ok(e)) e = hipMemcpy2DAsync(b_slot, (size_t)rp * 2, B, (size_t)r * 2, (size_t)r * 2, (size_t)(E * d_out), kind, st);
    }
    if (!ok(e)) return MLORA_E_HIP;
    meta_set_kernel<<<dim3(1), dim3(1), 0, st>>>(s->rank, s->scale, s->catalog, slot, r, alpha / (float)r, catalog_id);
    note_rank(s, slot, r);
    return ok(hipGetLastError()) ? MLORA_OK : MLORA_E_HIP;
}

int32_t mlora_slot_image_bytes(const mlora_site_desc *d, size_t *a_bytes, size_t *b_bytes)
{
    int32_t rc = check_desc(d);
    if (rc) return rc;
    if (!a_bytes || !b_bytes) return MLORA_E_INVALID;
    const int64_t E = d->n_experts > 0 ? d->n_experts : 1, rp = round_pow2(d->r_max);
    *a_bytes = (size_t)E * rp * d->d_in * 2;
    *b_bytes = (size_t)E * d->d_out * rp * 2;
    return MLORA_OK;
}

// Experts [e0, e1) of one table of the slot image.
// A_e [r, d_in] -> rows 0..r-1 of the expert's [r_pad, d_in] block, the rest zero
static void pack_a_range(char *ai, const void *const *A_e, int64_t e0, int64_t e1, int64_t r, int64_t rp, int64_t d_in)
{
    for (int64_t e = e0; e < e1; ++e) {
        std::memcpy(ai + e * rp * d_in * 2, A_e[e], (size_t)r * d_in * 2);
        if (r < rp) std::memset(ai + (e * rp + r) * d_in * 2, 0, (size_t)(rp - r) * d_in * 2);
    }
}

// B_e [d_out, r] -> columns 0..r-1 of the expert's [d_out, r_pad] block, the rest zero
static void pack_b_range(char *bi, const void *const *B_e, int64_t e0, int64_t e1, int64_t r, int64_t rp, int64_t d_out)
{
    for (int64_t e = e0; e < e1; ++e) {
        if (r == rp) {
            std::memcpy(bi + e * d_out * rp * 2, B_e[e], (size_t)d_out * rp * 2);
            continue;
        }
        const char *src = (const char *)B_e[e];
        char *dst = bi + e * d_out * rp * 2;
        for (int64_t o = 0; o < d_out; ++o) {
            std::memcpy(dst + o * rp * 2, src + o * r * 2, (size_t)r * 2);
            std::memset(dst + (o * rp + r) * 2, 0, (size_t)(rp - r) * 2);
        }
    }
}

int32_t mlora_pack_experts(const mlora_site_desc *d, const void *const *A_e, const void *const *B_e, int32_t r,
                           void *a_img, void *b_img)
{
    int32_t rc = check_desc(d);
    if (rc) return rc;
    if (!A_e || !B_e || !a_img || !b_img) return MLORA_E_INVALID;
    if (r < 1 || r > d->r_max) return MLORA_E_SHAPE;
    const int64_t E = d->n_experts > 0 ? d->n_experts : 1, rp = round_pow2(d->r_max);
    for (int64_t e = 0; e < E; ++e)
        if (!A_e[e] || !B_e[e]) return MLORA_E_INVALID;
    pack_a_range((char *)a_img, A_e, 0, E, r, rp, d->d_in);
    pack_b_range((char *)b_img, B_e, 0, E, r, rp, d->d_out);
    return MLORA_OK;
}

int32_t lora_slots_upload_experts(mlora_site *s, int32_t slot, int64_t catalog_id, const void *const *A_e,
                                  const void *const *B_e, int32_t r, float alpha, void *stream)
{
    if (!s || !A_e || !B_e) return MLORA_E_INVALID;
    if (slot < 0 || slot >= s->d.n_slots) return MLORA_E_SLOT;
    if (r < 1 || r > s->d.r_max) return MLORA_E_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    DeviceGuard g(s->d.device);
    if (!g.good) return MLORA_E_HIP;
    size_t ab = 0, bb = 0;
    int32_t rc = mlora_slot_image_bytes(&s->d, &ab, &bb);
    if (rc) return rc;
    if (!s->pack) {
        if (!ok(hipHostMalloc(&s->pack, ab + bb, hipHostMallocDefault))) return MLORA_E_HIP;
        if (!ok(hipEventCreateWithFlags(&s->pack_ev, hipEventDisableTiming))) return MLORA_E_HIP;
    }
    if (s->pack_busy && !ok(hipEventSynchronize(s->pack_ev))) return MLORA_E_HIP;   // the previous image has left the host
    const int64_t E = s->E, rp = s->r_pad;
    for (int64_t e = 0; e < E; ++e)
        if (!A_e[e] || !B_e[e]) return MLORA_E_INVALID;
    // The image is the slot's bytes, padding included: no zero-fill launch.  It leaves the host in
    // pieces of about 2 MB ("upload_piece_kb"; measured best among 256 KB .. whole table), each copied
    // as soon as it is packed, so that the copies of the earlier pieces run while the host packs the
    // later ones.
    meta_set_kernel<<<dim3(1), dim3(1), 0, st>>>(s->rank, s->scale, s->catalog, slot, 0, 0.f, -1);
    char *ai = (char *)s->pack, *bi = ai + ab;
    // after a failed copy the earlier pieces may still be leaving the image: wait before it can be reused
    auto drain = [&]() { (void)hipStreamSynchronize(st); return (int32_t)MLORA_E_HIP; };
    const int64_t a_exp = rp * s->d.d_in * 2, b_exp = (int64_t)s->d.d_out * rp * 2;       // bytes per expert
    const int64_t piece = (int64_t)(tuning(kUploadPieceKb) > 0 ? tuning(kUploadPieceKb) : 2048) << 10;
    const int64_t a_step = std::max<int64_t>(1, piece / a_exp), b_step = std::max<int64_t>(1, piece / b_exp);
    for (int64_t e0 = 0; e0 < E; e0 += a_step) {
        const int64_t e1 = std::min(E, e0 + a_step);
        pack_a_range(ai, A_e, e0, e1, r, rp, s->d.d_in);
        if (!ok(hipMemcpyAsync((char *)s->a_tab + (size_t)slot * ab + e0 * a_exp, ai + e0 * a_exp, (size_t)((e1 - e0) * a_exp), hipMemcpyHostToDevice, st))) return drain();
    }
    for (int64_t e0 = 0; e0 < E; e0 += b_step) {
        const int64_t e1 = std::min(E, e0 + b_step);
        pack_b_range(bi, B_e, e0, e1, r, rp, s->d.d_out);
        if (!ok(hipMemcpyAsync((char *)s->b_tab + (size_t)slot * bb + e0 * b_exp, bi + e0 * b_exp, (size_t)((e1 - e0) * b_exp), hipMemcpyHostToDevice, st))) return drain();
    }
    meta_set_kernel<<<dim3(1), dim3(1), 0, st>>>(s->rank, s->scale, s->catalog, slot, r, alpha / (float)r, catalog_id);
    if (!ok(hipEventRecord(s->pack_ev, st))) return MLORA_E_HIP;
    s->pack_busy = true;
    note_rank(s, slot, r);
    return ok(hipGetLastError()) ? MLORA_OK : MLORA_E_HIP;
}

int32_t mlora_site_check(mlora_site *s, void *stream)
{
    if (!s) return MLORA_E_INVALID;
    DeviceGuard g(s->d.device);
    if (!g.good) return MLORA_E_HIP;
    if (!ok(hipStreamSynchronize((hipStream_t)stream))) return MLORA_E_HIP;
    if (!s->ctrl) return MLORA_OK;
    uint32_t flag = 0;
    if (!ok(hipMemcpy(&flag, s->ctrl + 1, sizeof flag, hipMemcpyDeviceToHost))) return MLORA_E_HIP;
    if (flag) {
        // back to a working exchange: counters and flag cleared, a fresh tag
        (void)launch_fill_i32((int32_t *)s->ctrl, 0, (int64_t)(kCtrlBytes / 4), (hipStream_t)stream);
        (void)launch_fill_i32((int32_t *)s->ctrl, 1, 1, (hipStream_t)stream);
        return MLORA_E_HIP;
    }
    if (s->r_pad == 64 && s->xch) {
        // the one-launch prefill keeps its own control words (a wait for a tile's flag that gave up)
        uint32_t *sc = seg_ctrl_of(s);
        if (!ok(hipMemcpy(&flag, sc + 1, sizeof flag, hipMemcpyDeviceToHost))) return MLORA_E_HIP;
        if (flag) {
            (void)launch_fill_i32((int32_t *)sc + 1, 0, 127, (hipStream_t)stream);   // error word and sign-ins; the epoch goes on
            return MLORA_E_HIP;
        }
    }
    return MLORA_OK;
}

int32_t lora_slot_lookup(mlora_site *s, const int64_t *token_catalog_id, int32_t T, int32_t *token_slot, void *stream)
{
    if (!s || T < 0) return MLORA_E_INVALID;
    if (T == 0) return MLORA_OK;
    if (!token_catalog_id || !token_slot) return MLORA_E_INVALID;
    DeviceGuard g(s->d.device);
    if (!g.good) return MLORA_E_HIP;
    slot_lookup_kernel<<<dim3((unsigned)((T + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>(
        token_catalog_id, T, s->catalog, s->rank, s->d.n_slots, token_slot);
    return ok(hipGetLastError()) ? MLORA_OK : MLORA_E_HIP;
}

int32_t lora_slots_evict(mlora_site *s, int32_t slot, void *stream)
{
    if (!s) return MLORA_E_INVALID;
    if (slot < 0 || slot >= s->d.n_slots) return MLORA_E_SLOT;
    DeviceGuard g(s->d.device);
    if (!g.good) return MLORA_E_HIP;
    meta_set_kernel<<<dim3(1), dim3(1), 0, (hipStream_t)stream>>>(s->rank, s->scale, s->catalog, slot, 0, 0.f, -1);
    note_rank(s, slot, 0);
    return ok(hipGetLastError()) ? MLORA_OK : MLORA_E_HIP;
}

int32_t mlora_plan_bytes(int32_t max_items, int32_t n_keys, size_t *bytes)
{
    if (!bytes || max_items <= 0 || n_keys <= 0) return MLORA_E_INVALID;
    *bytes = align256(plan_words(max_items, n_keys) * 4);
    return MLORA_OK;
}

int32_t mlora_plan_create(int32_t max_items, int32_t n_keys, int32_t device, void *plan_dev, mlora_plan **out)
{
    if (!plan_dev || !out || max_items <= 0 || n_keys <= 0 || device < 0) return MLORA_E_INVALID;
    if ((uintptr_t)plan_dev & 255) return MLORA_E_SHAPE;
    mlora_plan *p = new (std::nothrow) mlora_plan();
    if (!p) return MLORA_E_INVALID;
    init_plan(p, max_items, n_keys, device, plan_dev);
    DeviceGuard g(device);
    if (!g.good) { delete p; return MLORA_E_HIP; }
    hipError_t e = launch_fill_i32(p->pv.hdr, 0, 8 + 3 * ((int64_t)n_keys + 1), 0);
    if (ok(e)) e = launch_fill_i32(p->pv.tok_hdr, 0, 8 + 2 * ((int64_t)n_keys + 1), 0);
    if (!ok(e) || !ok(hipStreamSynchronize(0))) { delete p; return MLORA_E_HIP; }
    *out = p;
    return MLORA_OK;
}

void mlora_plan_destroy(mlora_plan *p) { delete p; }

int32_t lora_plan_decode(mlora_plan *plan, const int32_t *token_slot, int32_t T, int32_t n_slots,
                         const mlora_site *ready_from, void *stream)
{
    if (!plan || T < 0 || n_slots <= 0 || (T > 0 && !token_slot)) return MLORA_E_INVALID;
    if (ready_from && ready_from->d.n_slots < n_slots) return MLORA_E_SLOT;
    if (T == 0) { plan->items = 0; plan->grid_chunks = 0; plan->moe = false; return MLORA_OK; }
    DeviceGuard g(plan->device);
    if (!g.good) return MLORA_E_HIP;
    return plan_decode_impl(plan, token_slot, T, n_slots, ready_from ? ready_from->rank : nullptr, (hipStream_t)stream);
}

int32_t lora_apply_decode_planned(mlora_site *s, const mlora_plan *plan, const void *x, int64_t ldx,
                                  void *y, int64_t ldy, void *stream)
{
    if (!s || !plan) return MLORA_E_INVALID;
    if (s->d.n_experts > 0 || plan->moe) return MLORA_E_UNSUPPORTED;
    if (plan->items == 0) return MLORA_OK;
    int32_t rc = check_xy(s, x, ldx, y, ldy);
    if (rc) return rc;
    if (plan->n_slots > s->d.n_slots) return MLORA_E_SLOT;
    DeviceGuard g(s->d.device);
    if (!g.good) return MLORA_E_HIP;
    return apply_planned_impl(s, plan, x, ldx, y, ldy, (hipStream_t)stream);
}

// Neighbouring sites that can share a launch are grouped; the others get a launch of their own.
static int32_t apply_multi_impl(mlora_site *const *sites, int32_t n_sites, const mlora_plan *plan,
                                const void *const *xs, const int64_t *ldxs, void *const *ys, const int64_t *ldys,
                                hipStream_t st)
{
    int32_t k = 0;
    while (k < n_sites) {
        RowsArgs grp[kMaxMulti];
        int32_t n = 0, nw = 0;
        while (k + n < n_sites && n < kMaxMulti) {
            RowsArgs a = rows_args(sites[k + n], xs[k + n], ldxs[k + n], ys[k + n], ldys[k + n]);
            a.chunks = plan->pv.chunks; a.top_k = plan->top_k; a.grid_chunks = plan->grid_chunks;
            const int w = rows_group_waves(a);
            if (w == 0 || (n > 0 && (a.r_pad != grp[0].r_pad || w != nw))) break;
            nw = w;
            grp[n++] = a;
        }
        if (n >= 2) {
            if (!ok(launch_rows_multi(grp, n, st))) return MLORA_E_HIP;
            k += n;
        } else {
            int32_t rc = apply_planned_impl(sites[k], plan, xs[k], ldxs[k], ys[k], ldys[k], st);
            if (rc) return rc;
            k += 1;
        }
    }
    return MLORA_OK;
}

int32_t lora_apply_decode_multi(mlora_site *const *sites, int32_t n_sites, const mlora_plan *plan,
                                const void *const *xs, const int64_t *ldxs, void *const *ys, const int64_t *ldys,
                                void *stream)
{
    if (!sites || !plan || !xs || !ldxs || !ys || !ldys || n_sites < 1) return MLORA_E_INVALID;
    if (plan->moe) return MLORA_E_UNSUPPORTED;
    for (int32_t k = 0; k < n_sites; ++k) {
        if (!sites[k]) return MLORA_E_INVALID;
        if (sites[k]->d.n_experts > 0) return MLORA_E_UNSUPPORTED;
        if (sites[k]->d.device != sites[0]->d.device) return MLORA_E_INVALID;
        if (plan->n_slots > sites[k]->d.n_slots) return MLORA_E_SLOT;
        int32_t rc = check_xy(sites[k], xs[k], ldxs[k], ys[k], ldys[k]);
        if (rc) return rc;
    }
    if (plan->items == 0) return MLORA_OK;
    DeviceGuard g(sites[0]->d.device);
    if (!g.good) return MLORA_E_HIP;
    return apply_multi_impl(sites, n_sites, plan, xs, ldxs, ys, ldys, (hipStream_t)stream);
}

int32_t lora_plan_apply_decode_multi(mlora_site *const *sites, int32_t n_sites, mlora_plan *plan,
                                     const int32_t *token_slot, int32_t T, int32_t n_slots, const mlora_site *ready_from,
                                     const void *const *xs, const int64_t *ldxs, void *const *ys, const int64_t *ldys,
                                     void *stream)
{
    if (!sites || !plan || !xs || !ldxs || !ys || !ldys || n_sites < 1 || T < 0 || n_slots <= 0) return MLORA_E_INVALID;
    if (T > 0 && !token_slot) return MLORA_E_INVALID;
    if (ready_from && ready_from->d.n_slots < n_slots) return MLORA_E_SLOT;
    if (T > plan->max_items || n_slots > plan->n_keys) return MLORA_E_UNSUPPORTED;
    for (int32_t k = 0; k < n_sites; ++k) {
        if (!sites[k]) return MLORA_E_INVALID;
        if (sites[k]->d.n_experts > 0) return MLORA_E_UNSUPPORTED;
        if (sites[k]->d.device != sites[0]->d.device || sites[k]->d.device != plan->device) return MLORA_E_INVALID;
        if (n_slots > sites[k]->d.n_slots) return MLORA_E_SLOT;
        int32_t rc = check_xy(sites[k], xs[k], ldxs[k], ys[k], ldys[k]);
        if (rc) return rc;
    }
    DeviceGuard g(plan->device);
    if (!g.good) return MLORA_E_HIP;
    hipStream_t st = (hipStream_t)stream;
    if (T == 0) { plan->items = 0; plan->grid_chunks = 0; plan->moe = false; return MLORA_OK; }
    const int32_t *ready_rank = ready_from ? ready_from->rank : nullptr;
    // the leading sites that can share a launch plan inside it; everything else as two calls would do
    RowsArgs grp[kMaxMulti];
    int32_t n = 0;
    if (T <= rows_local_plan_rows() && n_slots <= rows_local_plan_slots() && max_chunks(T, n_slots) <= rows_local_plan_rows() &&
        !tuning(kPlanGeneral) &&
        !tuning(kPlanSeparate)) {
        while (n < n_sites && n < kMaxMulti) {
            RowsArgs a = rows_args(sites[n], xs[n], ldxs[n], ys[n], ldys[n]);
            a.chunks = plan->pv.chunks; a.top_k = 1; a.grid_chunks = (int32_t)max_chunks(T, n_slots);
            if (rows_group_waves(a) != 8 || (n > 0 && a.r_pad != grp[0].r_pad)) {
                if (n == 0 && rows_plans_alone(a)) grp[n++] = a;       // a launch of its own, planned inside
                break;
            }
            grp[n++] = a;
        }
        if (n == 1 && !rows_plans_alone(grp[0])) n = 0;
    }
    if (n == 0) {
        int32_t rc = plan_decode_impl(plan, token_slot, T, n_slots, ready_rank, st);
        if (rc) return rc;
        return apply_multi_impl(sites, n_sites, plan, xs, ldxs, ys, ldys, st);
    }
    plan->items = T; plan->top_k = 1; plan->n_experts = 1; plan->n_slots = n_slots; plan->moe = false;
    plan->grid_chunks = (int32_t)max_chunks(T, n_slots);
    if (!ok(launch_rows_multi_plan(grp, n, plan->pv, token_slot, T, n_slots, ready_rank, st))) return MLORA_E_HIP;
    if (n == n_sites) return MLORA_OK;
    return apply_multi_impl(sites + n, n_sites - n, plan, xs + n, ldxs + n, ys + n, ldys + n, st);
}

int32_t moe_plan_route(mlora_plan *plan, const int32_t *topk_ids, const int32_t *token_slot, int32_t T, int32_t K,
                       int32_t n_slots, int32_t n_experts, const mlora_site *ready_from,
                       int32_t *out_sorted_pair, int32_t *out_group_off, void *stream)
{
    if (!plan || T < 0 || K <= 0 || n_slots <= 0 || n_experts <= 0) return MLORA_E_INVALID;
    if (T > 0 && (!topk_ids || !token_slot)) return MLORA_E_INVALID;
    if (ready_from && ready_from->d.n_slots < n_slots) return MLORA_E_SLOT;
    DeviceGuard g(plan->device);
    if (!g.good) return MLORA_E_HIP;
    hipStream_t st = (hipStream_t)stream;
    if (T == 0) {
        plan->items = 0; plan->grid_chunks = 0; plan->moe = true;
        if (out_group_off && !ok(launch_fill_i32(out_group_off, 0, (int64_t)n_slots * n_experts + 1, st))) return MLORA_E_HIP;
        return MLORA_OK;
    }
    return plan_route_impl(plan, topk_ids, token_slot, T, K, n_slots, n_experts,
                           ready_from ? ready_from->rank : nullptr, out_sorted_pair, out_group_off, st);
}

int32_t moe_lora_apply_planned(mlora_site *s, const mlora_plan *plan, const void *x, int64_t ldx,
                               void *y, int64_t ldy, void *stream)
{
    if (!s || !plan) return MLORA_E_INVALID;
    if (s->d.n_experts <= 0 || !plan->moe) return MLORA_E_UNSUPPORTED;
    if (plan->items == 0) return MLORA_OK;
    if (plan->n_experts != s->d.n_experts || plan->n_slots > s->d.n_slots) return MLORA_E_SHAPE;
    int32_t rc = check_xy(s, x, ldx, y, ldy);
    if (rc) return rc;
    DeviceGuard g(s->d.device);
    if (!g.good) return MLORA_E_HIP;
    return apply_planned_impl(s, plan, x, ldx, y, ldy, (hipStream_t)stream);
}

int32_t moe_lora_apply_multi(mlora_site *const *sites, int32_t n_sites, const mlora_plan *plan,
                             const void *const *xs, const int64_t *ldxs, void *const *ys, const int64_t *ldys,
                             void *stream)
{
    if (!sites || !plan || !xs || !ldxs || !ys || !ldys || n_sites < 1) return MLORA_E_INVALID;
    if (!plan->moe) return MLORA_E_UNSUPPORTED;
    for (int32_t k = 0; k < n_sites; ++k) {
        if (!sites[k]) return MLORA_E_INVALID;
        if (sites[k]->d.n_experts <= 0) return MLORA_E_UNSUPPORTED;
        if (sites[k]->d.device != sites[0]->d.device) return MLORA_E_INVALID;
        if (plan->items > 0 && (plan->n_experts != sites[k]->d.n_experts || plan->n_slots > sites[k]->d.n_slots)) return MLORA_E_SHAPE;
        int32_t rc = check_xy(sites[k], xs[k], ldxs[k], ys[k], ldys[k]);
        if (rc) return rc;
    }
    if (plan->items == 0) return MLORA_OK;
    DeviceGuard g(sites[0]->d.device);
    if (!g.good) return MLORA_E_HIP;
    return apply_multi_impl(sites, n_sites, plan, xs, ldxs, ys, ldys, (hipStream_t)stream);
}

int32_t moe_down_workspace_bytes(int32_t T, int32_t K, int32_t d_out, size_t *bytes)
{
    if (!bytes || T < 0 || K <= 0 || d_out <= 0 || (d_out & 7)) return MLORA_E_INVALID;
    // one 32-bit word per pair and (padded) rank value: the first launch's h, whatever the site's rank
    *bytes = align256((size_t)T * K * MLORA_MAX_RANK * sizeof(uint32_t));
    return MLORA_OK;
}

int32_t moe_lora_apply_down(mlora_site *s, const mlora_plan *plan, const void *x, int64_t ldx,
                            const float *pair_w, const int32_t *token_slot, void *workspace,
                            void *y, int64_t ldy, void *stream)
{
    if (!s || !plan) return MLORA_E_INVALID;
    if (s->d.n_experts <= 0 || !plan->moe) return MLORA_E_UNSUPPORTED;
    if (plan->items == 0) return MLORA_OK;
    if (plan->n_experts != s->d.n_experts || plan->n_slots > s->d.n_slots) return MLORA_E_SHAPE;
    if (!pair_w || !token_slot || !workspace || !aligned16(workspace)) return MLORA_E_INVALID;
    const int tile_rows = moe_down_tile_rows(s->r_pad, plan->top_k, s->E);
    if (plan->top_k > moe_down_max_k() || tile_rows <= 0 || (int64_t)s->E * s->d.d_out * s->r_pad * 2 >= ((int64_t)1 << 32)) return MLORA_E_UNSUPPORTED;
    int32_t rc = check_xy(s, x, ldx, y, ldy);
    if (rc) return rc;
    DeviceGuard g(s->d.device);
    if (!g.good) return MLORA_E_HIP;
    hipStream_t st = (hipStream_t)stream;
    const int32_t T = plan->items / plan->top_k;
    MoeDownArgs d{};
    d.y = (uint16_t *)y; d.ldy = ldy; d.b_tab = s->b_tab; d.rank = s->rank; d.h = (uint32_t *)workspace;
    d.key_of = plan->pv.key_of; d.sorted = plan->pv.sorted; d.group_off = plan->pv.group_off;
    d.tok_sorted = plan->pv.tok_sorted; d.tok_off = plan->pv.tok_off;
    d.T = T; d.K = plan->top_k; d.E = s->E; d.n_slots = plan->n_slots; d.d_out = s->d.d_out; d.r_pad = s->r_pad;
    d.x = (const uint16_t *)x; d.ldx = ldx; d.a_tab = s->a_tab; d.scale = s->scale; d.pair_w = pair_w; d.d_in = s->d.d_in;
    d.chunks = plan->pv.chunks; d.chunk_bound = plan->grid_chunks;
    // first launch: per chunk of a (slot, expert) group, h = w * (alpha / r) * A x for the chunk's pairs
    if (moe_down_shrinks_by_wave(s->r_pad)) {
        if (!ok(launch_moe_down_shrink(d, st))) return MLORA_E_HIP;
    } else {
        RowsArgs a = rows_args(s, x, ldx, y, ldy);
        a.chunks = plan->pv.chunks;
        a.top_k = 1;                                   // one input row per pair
        a.grid_chunks = plan->grid_chunks;
        a.h_out = (uint32_t *)workspace; a.row_w = pair_w;
        if (!ok(launch_rows(a, st))) return MLORA_E_HIP;
    }
    // second launch: per slot and tile of its tokens, y += H x Bcat on the matrix cores
    d.n_mtiles = T / tile_rows + plan->n_slots;
    d.n_ntiles = (s->d.d_out + moe_down_tile_cols() - 1) / moe_down_tile_cols();
    return ok(launch_moe_down(d, st)) ? MLORA_OK : MLORA_E_HIP;
}

// Where a decode call keeps what lives beyond its inputs and outputs: the batch plan and, for
// launches whose workgroups trade partial sums, the control block and the exchange words.
struct DecodeScratch {
    mlora_plan *plan;
    uint32_t *ctrl;
    uint64_t *xch;
};

static int32_t apply_decode_impl(mlora_site *s, const void *x, int64_t ldx, void *y, int64_t ldy,
                                 const int32_t *token_slot, int32_t T, hipStream_t st, const DecodeScratch &sc)
{
    auto args = [&](const void *xp, void *yp) {
        RowsArgs a = rows_args(s, xp, ldx, yp, ldy);
        a.xch = sc.xch; a.ctrl = sc.ctrl; a.xch_chunks = sc.xch ? kXchChunks : 0;
        return a;
    };
    if (s->r_pad <= 2 && !tuning(kPlanGeneral) && !tuning(kPlanSeparate)) {
        // Tiny adapters (the compact rank-1 catalog of Section 4): rows are applied one by one, without
        // a plan -- grouping would save at most two adapter rows per row, a planner launch costs more.
        RowsArgs a = args(x, y);
        a.row_slot = token_slot; a.row_slots = s->d.n_slots; a.top_k = 1; a.grid_chunks = T;
        return ok(launch_rows(a, st)) ? MLORA_OK : MLORA_E_HIP;
    }
    mlora_plan *plan = sc.plan;
    // batches beyond the private plan are processed in slices; rows are independent
    for (int32_t t0 = 0; t0 < T; t0 += plan->max_items) {
        const int32_t n = T - t0 < plan->max_items ? T - t0 : plan->max_items;
        const uint16_t *xs = (const uint16_t *)x + (int64_t)t0 * ldx;
        uint16_t *ys = (uint16_t *)y + (int64_t)t0 * ldy;
        // a small batch on a site whose launch can plan for itself needs no planner launch (same plan,
        // same bits; see lora_plan_apply_decode_multi)
        if (n <= rows_local_plan_rows() && s->d.n_slots <= rows_local_plan_slots() &&
            max_chunks(n, s->d.n_slots) <= rows_local_plan_rows() && !tuning(kPlanGeneral) && !tuning(kPlanSeparate)) {
            RowsArgs a = args(xs, ys);
            a.chunks = plan->pv.chunks; a.top_k = 1; a.grid_chunks = (int32_t)max_chunks(n, s->d.n_slots);
            if (rows_plans_alone(a)) {
                plan->items = n; plan->top_k = 1; plan->n_experts = 1; plan->n_slots = s->d.n_slots; plan->moe = false;
                plan->grid_chunks = a.grid_chunks;
                if (!ok(launch_rows_multi_plan(&a, 1, plan->pv, token_slot + t0, n, s->d.n_slots, s->rank, st))) return MLORA_E_HIP;
                continue;
            }
        }
        int32_t rc = plan_decode_impl(plan, token_slot + t0, n, s->d.n_slots, s->rank, st);
        if (rc) return rc;
        RowsArgs a = args(xs, ys);
        a.chunks = plan->pv.chunks; a.top_k = plan->top_k; a.grid_chunks = plan->grid_chunks;
        if (!ok(launch_rows(a, st))) return MLORA_E_HIP;
    }
    return MLORA_OK;
}

static int32_t check_decode_call(mlora_site *s, const void *x, int64_t ldx, void *y, int64_t ldy,
                                 const int32_t *token_slot, int32_t T)
{
    if (!s || T < 0) return MLORA_E_INVALID;
    if (s->d.n_experts > 0) return MLORA_E_UNSUPPORTED;
    if (T == 0) return MLORA_OK;
    if (!token_slot) return MLORA_E_INVALID;
    return check_xy(s, x, ldx, y, ldy);
}

int32_t lora_apply_decode(mlora_site *s, const void *x, int64_t ldx, void *y, int64_t ldy,
                          const int32_t *token_slot, int32_t T, void *stream)
{
    int32_t rc = check_decode_call(s, x, ldx, y, ldy, token_slot, T);
    if (rc || T == 0) return rc;
    DeviceGuard g(s->d.device);
    if (!g.good) return MLORA_E_HIP;
    return apply_decode_impl(s, x, ldx, y, ldy, token_slot, T, (hipStream_t)stream, DecodeScratch{&s->priv, s->ctrl, s->xch});
}

// ---- the decode call for callers that cannot allocate ----------------------------------------
// What lora_apply_decode keeps in the site's caller-allocated scratch buffer (the batch plan, the
// control block and the exchange words of launches whose workgroups trade partial sums) lives here
// in a file-scope device array of fixed size, one copy per GPU, held until the process ends.
constexpr int32_t kNoAllocRows = 1024;             // largest batch (rows) and slot count the array is sized for
constexpr int32_t kNoAllocSlots = 1024;
constexpr size_t kNoAllocPlanBytes = 98304;        // >= plan_words(kNoAllocRows, kNoAllocSlots) * 4, checked at set-up
constexpr size_t kNoAllocBytes = kNoAllocPlanBytes + kCtrlBytes + kXchBytes;      // 1.1 MB
static __device__ __align__(256) unsigned char scratch[kNoAllocBytes];

constexpr int kNoAllocDevices = 64;
struct NoAllocState {
    bool ready = false;
    mlora_plan plan;                               // view into this device's copy of the array
    uint32_t *ctrl = nullptr;
    uint64_t *xch = nullptr;
};
static NoAllocState g_noalloc[kNoAllocDevices];
static std::mutex g_noalloc_mu;

// The device's copy of the array, set up on the first call on that device (which must be current).
// `scratch` itself is only a host-side handle; the device address comes from hipGetSymbolAddress.
static int32_t noalloc_state(int device, hipStream_t st, NoAllocState **out)
{
    if (device < 0 || device >= kNoAllocDevices) return MLORA_E_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_noalloc_mu);
    NoAllocState &n = g_noalloc[device];
    if (!n.ready) {
        if (plan_words(kNoAllocRows, kNoAllocSlots) * 4 > kNoAllocPlanBytes) return MLORA_E_UNSUPPORTED;
        void *ptr = nullptr;
        if (!ok(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))) || !ptr) return MLORA_E_HIP;
        if ((uintptr_t)ptr & 255) return MLORA_E_HIP;
        init_plan(&n.plan, kNoAllocRows, kNoAllocSlots, device, ptr);
        n.ctrl = (uint32_t *)((char *)ptr + kNoAllocPlanBytes);
        n.xch = (uint64_t *)((char *)n.ctrl + kCtrlBytes);
        // What must start at zero: the plan's header and counters, the control block, the exchange
        // words (tag 0 = never written); the first launch tag is 1.  Fill kernels on the caller's
        // stream, waited for once, so that later calls on any stream find the array set up.
        hipError_t e = launch_fill_i32(n.plan.pv.hdr, 0, 8 + 3 * ((int64_t)kNoAllocSlots + 1), st);
        if (ok(e)) e = launch_fill_i32(n.plan.pv.tok_hdr, 0, 8 + 2 * ((int64_t)kNoAllocSlots + 1), st);
        if (ok(e)) e = launch_fill_i32((int32_t *)n.ctrl, 0, (int64_t)((kCtrlBytes + kXchBytes) / 4), st);
        if (ok(e)) e = launch_fill_i32((int32_t *)n.ctrl, 1, 1, st);
        if (!ok(e) || !ok(hipStreamSynchronize(st))) return MLORA_E_HIP;
        n.ready = true;
    }
    *out = &n;
    return MLORA_OK;
}

int32_t lora_apply_decode_noalloc(mlora_site *s, const void *x, int64_t ldx, void *y, int64_t ldy,
                                  const int32_t *token_slot, int32_t T, void *stream)
{
    int32_t rc = check_decode_call(s, x, ldx, y, ldy, token_slot, T);
    if (rc) return rc;
    if (T > kNoAllocRows || s->d.n_slots > kNoAllocSlots) return MLORA_E_UNSUPPORTED;   // beyond what the array holds
    if (T == 0) return MLORA_OK;
    DeviceGuard g(s->d.device);
    if (!g.good) return MLORA_E_HIP;
    NoAllocState *n = nullptr;
    rc = noalloc_state(s->d.device, (hipStream_t)stream, &n);
    if (rc) return rc;
    return apply_decode_impl(s, x, ldx, y, ldy, token_slot, T, (hipStream_t)stream, DecodeScratch{&n->plan, n->ctrl, n->xch});
}

int32_t lora_apply_segmented(mlora_site *s, const void *x, int64_t ldx, void *y, int64_t ldy,
                             const int32_t *seg_off, const int32_t *seg_slot, int32_t S, int32_t T, void *stream)
{
    if (!s || S < 0 || T < 0) return MLORA_E_INVALID;
    if (s->d.n_experts > 0) return MLORA_E_UNSUPPORTED;
    if (S == 0) return T == 0 ? MLORA_OK : MLORA_E_SEGMENTS;
    if (!seg_off || !seg_slot) return MLORA_E_INVALID;
    if (seg_off[0] != 0 || seg_off[S] != T) return MLORA_E_SEGMENTS;
    for (int32_t k = 0; k < S; ++k) {
        if (seg_off[k + 1] < seg_off[k]) return MLORA_E_SEGMENTS;
        if (seg_slot[k] < -1 || seg_slot[k] >= s->d.n_slots) return MLORA_E_SLOT;
    }
    if (T == 0) return MLORA_OK;
    int32_t rc = check_xy(s, x, ldx, y, ldy);
    if (rc) return rc;
    DeviceGuard g(s->d.device);
    if (!g.good) return MLORA_E_HIP;
    hipStream_t st = (hipStream_t)stream;

    const bool mfma = s->r_pad == 64 && (s->d.d_in & 15) == 0 && s->xch && !tuning(kSegNoMfma);
    if (mfma) return segmented_mfma(s, x, ldx, y, ldy, seg_off, seg_slot, S, st);
    std::vector<int32_t> tab;
    for (int32_t k = 0; k < S; ++k) {
        if (seg_slot[k] < 0) continue;
        for (int32_t r0 = seg_off[k]; r0 < seg_off[k + 1]; r0 += kChunk) {
            const int32_t n = seg_off[k + 1] - r0 < kChunk ? seg_off[k + 1] - r0 : kChunk;
            tab.push_back(seg_slot[k]); tab.push_back(n); tab.push_back(r0); tab.push_back(0);
            for (int32_t c = 0; c < kChunk; ++c) tab.push_back(r0 + (c < n ? c : n - 1));
        }
    }
    const int64_t n_units = (int64_t)(tab.size() / kRec);
    if (n_units == 0) return MLORA_OK;
    // the records go to the site's device area in batches that fit it (one copy + one launch each; the
    // stream orders a batch's copy behind the launch that read the batch before it)
    const int64_t per_batch = (int64_t)s->seg_cap * 3 / kRec - 1;
    if (per_batch < 1) return MLORA_E_UNSUPPORTED;
    std::vector<int32_t> piece;
    for (int64_t u0 = 0; u0 < n_units; u0 += per_batch) {
        const int64_t n = n_units - u0 < per_batch ? n_units - u0 : per_batch;
        if (n < n_units) piece.assign(tab.begin() + u0 * kRec, tab.begin() + (u0 + n) * kRec);
        rc = stage_table(s, n < n_units ? piece : tab, st);
        if (rc) return rc;
        RowsArgs a = rows_args(s, x, ldx, y, ldy);
        a.chunks = s->seg_dev;
        a.grid_chunks = (int32_t)n;
        if (!ok(launch_rows(a, st))) return MLORA_E_HIP;
    }
    return MLORA_OK;
}

int32_t moe_lora_apply_packed(mlora_site *s, const void *x, int64_t ldx, void *y, int64_t ldy,
                              const int32_t *topk_ids, const int32_t *token_slot, int32_t T, int32_t K,
                              int32_t *out_sorted_pair, int32_t *out_group_off, void *stream)
{
    if (!s || T < 0 || K <= 0) return MLORA_E_INVALID;
    if (s->d.n_experts <= 0) return MLORA_E_UNSUPPORTED;
    DeviceGuard g(s->d.device);
    if (!g.good) return MLORA_E_HIP;
    hipStream_t st = (hipStream_t)stream;
    if (T == 0) {
        if (out_group_off && !ok(launch_fill_i32(out_group_off, 0, (int64_t)s->d.n_slots * s->E + 1, st))) return MLORA_E_HIP;
        return MLORA_OK;
    }
    if (!topk_ids || !token_slot) return MLORA_E_INVALID;
    int32_t rc = check_xy(s, x, ldx, y, ldy);
    if (rc) return rc;
    const int64_t P = (int64_t)T * K;
    if (P > s->priv.max_items) {
        if (out_sorted_pair || out_group_off) return MLORA_E_UNSUPPORTED;   // indices are per call, not per slice
        const int32_t tok_per = s->priv.max_items / K;
        if (tok_per < 1) return MLORA_E_UNSUPPORTED;
        for (int32_t t0 = 0; t0 < T; t0 += tok_per) {
            const int32_t n = T - t0 < tok_per ? T - t0 : tok_per;
            rc = plan_route_impl(&s->priv, topk_ids + (int64_t)t0 * K, token_slot + t0, n, K, s->d.n_slots, s->E,
                                 s->rank, nullptr, nullptr, st);
            if (rc) return rc;
            rc = apply_planned_impl(s, &s->priv, (const uint16_t *)x + (int64_t)t0 * ldx, ldx,
                                    (uint16_t *)y + (int64_t)t0 * K * ldy, ldy, st);
            if (rc) return rc;
        }
        return MLORA_OK;
    }
    rc = plan_route_impl(&s->priv, topk_ids, token_slot, T, K, s->d.n_slots, s->E, s->rank,
                         out_sorted_pair, out_group_off, st);
    if (rc) return rc;
    return apply_planned_impl(s, &s->priv, x, ldx, y, ldy, st);
}

}  // extern "C"
