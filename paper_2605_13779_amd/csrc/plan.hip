// Batch grouping kernels: which rows use which adapter.
//
// Dense decode (at most 64 distinct adapters share one decoding step, Section 4 cache-tier
// table) and the packed-MoE route index build (per-expert LoRA tensors keyed by expert id,
// Section 3.4).  All integer work; every output is uniquely determined by the inputs.
#include "plan_device.h"

namespace mlora {

size_t plan_words(int64_t M, int64_t NK)
{
    return 8 + 3 * (NK + 1) + 4 * M + kRec * max_chunks(M, NK) + 64      // the grouping of the items and its chunk records
         + 8 + 2 * (NK + 1) + 4 * M;                                       // the grouping of the tokens (route plans)
}

PlanView plan_view(void *base, int64_t M, int64_t NK)
{
    PlanView v;
    int32_t *p = (int32_t *)base;
    v.hdr = p;            p += 8;
    v.count = p;          p += NK + 1;
    v.group_off = p;      p += NK + 1;
    v.chunk_base = p;     p += NK + 1;
    v.key_of = p;         p += M;
    v.ticket = p;         p += M;
    v.tmp = p;            p += M;
    v.sorted = p;         p += M;
    v.chunks = p;         p += kRec * max_chunks(M, NK) + 64;
    v.tok_hdr = p;        p += 8;
    v.tok_count = p;      p += NK + 1;
    v.tok_off = p;        p += NK + 1;
    v.tok_key_of = p;     p += M;
    v.tok_ticket = p;     p += M;
    v.tok_tmp = p;        p += M;
    v.tok_sorted = p;
    return v;
}

__global__ void fill_i32_kernel(int32_t *p, int32_t v, int64_t n)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

hipError_t launch_fill_i32(int32_t *p, int32_t v, int64_t n, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    fill_i32_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>(p, v, n);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Small dense batches (up to kSortMax rows): one workgroup, one key (slot, row) per thread, sorted
// with a bitonic network -- keys are distinct, so the result is the stable sort by slot.  Exchanges
// at distance < 64 stay inside a wave (DPP / swizzle), only the few longer ones go through LDS.
// Group starts and chunk numbers then come from two scans, and the chunk records are written.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024)
void plan_dense_small_kernel(PlanView pv, const int32_t *__restrict__ token_slot, int T, int n_slots,
                             const int32_t *__restrict__ ready_rank, int rec_bound, int N)
{
    __shared__ uint2 xch[kSortMax];              // long-distance exchanges, then sorted slots / chunk starts
    __shared__ __attribute__((aligned(16))) int32_t wave_tot[16];
    __shared__ int32_t s_rows, s_chunks;
    const int i = threadIdx.x;                   // blockDim.x == N, a power of two in [64, 1024]
    const uint32_t kNone = 0xffffffffu;
    if (i == 0) { s_rows = 0; s_chunks = 0; }
    uint32_t ks = kNone, kt = (uint32_t)i;
    if (i < T) {
        const int s = token_slot[i];
        if (s >= 0 && s < n_slots && !(ready_rank && ready_rank[s] <= 0)) ks = (uint32_t)s;
    }
    BitonicSort<kSortMax>::run(ks, kt, i, N, xch);

    // neighbours' slots through LDS: group starts, number of usable rows
    int32_t *ss = (int32_t *)xch;
    ss[i] = (int32_t)ks;
    __syncthreads();
    const bool live = ks != kNone;
    const bool start = live && (i == 0 || (uint32_t)ss[i - 1] != ks);
    if (live && (i == N - 1 || (uint32_t)ss[i + 1] == kNone)) s_rows = i + 1;
    __syncthreads();
    const int n_rows = s_rows;
    const int gs = block_scan<true>(start ? i : 0, i, N >> 6, wave_tot);
    const int r = i - gs;
    const bool cstart = live && (r % kChunk) == 0;
    const int c = block_scan<false>(cstart ? 1 : 0, i, N >> 6, wave_tot) - 1;     // chunk of this row
    if (live && i == n_rows - 1) s_chunks = c + 1;
    int32_t *cs = (int32_t *)xch;                // chunk c starts at sorted position cs[c]
    __syncthreads();
    const int n_chunks = s_chunks;
    if (cstart) cs[c] = i;
    if (i == 0) cs[n_chunks] = n_rows;
    __syncthreads();
    if (live) {
        pv.sorted[i] = (int32_t)kt;
        int32_t *rec = pv.chunks + (int64_t)c * kRec;
        rec[4 + (r % kChunk)] = (int32_t)kt;
        if (cstart) { rec[0] = (int32_t)ks; rec[1] = cs[c + 1] - cs[c]; rec[2] = i; rec[3] = 0; }
    }
    if (i == 0) { pv.hdr[0] = n_chunks; pv.hdr[1] = n_rows; }
    // records past the live chunks are marked empty (count 0): the apply kernels read only records
    for (int d = n_chunks + i; d < rec_bound; d += N) pv.chunks[(int64_t)d * kRec + 1] = 0;
}

hipError_t launch_plan_dense_small(const PlanView &pv, const int32_t *token_slot, int T, int n_slots,
                                   const int32_t *ready_rank, hipStream_t st)
{
    int N = 64;
    while (N < T) N <<= 1;
    if (N > kSortMax) return hipErrorInvalidValue;
    plan_dense_small_kernel<<<dim3(1), dim3(N), 0, st>>>(pv, token_slot, T, n_slots, ready_rank,
                                                         (int)max_chunks(T, n_slots), N);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// General pipeline (MoE pairs, large dense batches): histogram with tickets, scan, scatter, and
// an in-group rank that restores ascending order, so the result is the stable counting sort.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256)
void plan_hist_kernel(PlanView pv, const int32_t *__restrict__ topk, const int32_t *__restrict__ token_slot,
                      int P, int K, int E, int n_slots, const int32_t *__restrict__ ready_rank)
{
    int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= P) return;
    int t = p / K;
    int s = token_slot[t];
    int e = topk ? topk[p] : 0;
    int key = -1;
    if (s >= 0 && s < n_slots && e >= 0 && e < E && !(ready_rank && ready_rank[s] <= 0)) key = s * E + e;
    pv.key_of[p] = key;
    if (key >= 0) pv.ticket[p] = atomicAdd(&pv.count[key], 1);
}

// One workgroup: exclusive scans of the group sizes and of the per-group chunk counts.
__global__ __launch_bounds__(1024)
void plan_scan_kernel(PlanView pv, int NK, int32_t *__restrict__ out_group_off)
{
    __shared__ __attribute__((aligned(16))) int32_t wave_tot[16];
    const int tid = threadIdx.x;
    const int per = (NK + 1023) / 1024;
    const int lo = min(NK, tid * per), hi = min(NK, lo + per);
    int items = 0, chunks = 0;
    for (int k = lo; k < hi; ++k) {
        int c = pv.count[k];
        items += c;
        chunks += (c + kChunk - 1) / kChunk;
    }
    const int inc_i = block_scan<false>(items, tid, 16, wave_tot);
    const int inc_c = block_scan<false>(chunks, tid, 16, wave_tot);
    int run_i = inc_i - items, run_c = inc_c - chunks;
    for (int k = lo; k < hi; ++k) {
        int c = pv.count[k];
        pv.group_off[k] = run_i;
        if (out_group_off) out_group_off[k] = run_i;
        if (pv.chunk_base) pv.chunk_base[k] = run_c;
        pv.count[k] = 0;                           // leave the histogram clean for the next call
        run_i += c;
        run_c += (c + kChunk - 1) / kChunk;
    }
    if (tid == 1023) {
        pv.group_off[NK] = inc_i;
        if (out_group_off) out_group_off[NK] = inc_i;
        if (pv.chunk_base) pv.chunk_base[NK] = inc_c;
        pv.hdr[0] = inc_c;
        pv.hdr[1] = inc_i;
    }
}

__global__ __launch_bounds__(256)
void plan_scatter_kernel(PlanView pv, int P)
{
    int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= P) return;
    int key = pv.key_of[p];
    if (key >= 0) pv.tmp[pv.group_off[key] + pv.ticket[p]] = p;
}

__global__ __launch_bounds__(256)
void plan_fix_kernel(PlanView pv, int P, int32_t *__restrict__ out_sorted, int rec_bound)
{
    int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= P) return;
    const int n_rows = pv.hdr[1];
    const bool records = pv.chunks != nullptr;            // (the token-level grouping of a route plan has none)
    if (records && j >= pv.hdr[0] && j < rec_bound) pv.chunks[(int64_t)j * kRec + 1] = 0;   // empty record past the live chunks
    if (j >= n_rows) {
        pv.sorted[j] = -1;
        if (out_sorted) out_sorted[j] = -1;
        return;
    }
    int p = pv.tmp[j];
    int key = pv.key_of[p];
    int off = pv.group_off[key], n = pv.group_off[key + 1] - off;
    int r = 0;
    for (int m = 0; m < n; ++m) r += (pv.tmp[off + m] < p);
    pv.sorted[off + r] = p;
    if (out_sorted) out_sorted[off + r] = p;
    if (!records) return;
    int32_t *rec = pv.chunks + (int64_t)(pv.chunk_base[key] + r / kChunk) * kRec;
    rec[4 + (r % kChunk)] = p;
    if (r % kChunk == 0) { rec[0] = key; rec[1] = min(kChunk, n - r); rec[2] = off + r; rec[3] = 0; }
}

// ---------------------------------------------------------------------------------------------
// The same result in one launch, for batches of moderate size (MoE decode / prefill steps of a
// few thousand tokens).  Every workgroup owns kOneRange consecutive pairs and builds, in LDS, the
// histogram of ALL pairs and the histogram of the pairs in front of its range; a scan of the first
// gives the group starts and chunk numbers, the second is the stable rank of the range's first
// member of each group.  Position of pair p = group start + pairs of its key in front of the
// range + pairs of its key in front of it inside the range.  Every workgroup reads all keys
// (P * 4 bytes from L2 each), which is what replaces the three dependent launches and the global
// atomics of the pipeline above; the result is the unique stable counting sort either way.
// ---------------------------------------------------------------------------------------------
constexpr int kOneRange = 256;     // pairs owned by a workgroup
constexpr int kOneKeys = 4096;     // largest key space (LDS: three int32 tables of this size)
constexpr int kOnePairs = 32768;   // largest batch (each workgroup walks all of it)
constexpr int kOneThreads = 1024;

// k_magic = ceil(2^32 / K) (0 for K = 1): p / K is then the high word of p * k_magic, exact while
// p * K < 2^32.  A wave instruction takes four cycles on the 16-lane SIMDs, every workgroup walks
// all pairs, and the general division is some forty instructions per pair.
__device__ __forceinline__ int route_key(const int32_t *__restrict__ topk, const int32_t *__restrict__ token_slot,
                                         const int32_t *__restrict__ ready_rank, int p, uint32_t k_magic, int E, int n_slots)
{
    const int s = token_slot[k_magic ? (int)__umulhi((uint32_t)p, k_magic) : p];
    const int e = topk ? topk[p] : 0;
    if (s >= 0 && s < n_slots && e >= 0 && e < E && !(ready_rank && ready_rank[s] <= 0)) return s * E + e;
    return -1;
}

__device__ __forceinline__
void plan_route_one_body(const PlanView &pv, const int32_t *__restrict__ topk, const int32_t *__restrict__ token_slot,
                         int P, int K, uint32_t k_magic, int E, int n_slots, const int32_t *__restrict__ ready_rank,
                         int32_t *__restrict__ out_sorted, int32_t *__restrict__ out_group_off, int rec_bound, const int block)
{
    __shared__ int32_t goff[kOneKeys + 1];       // exclusive group starts
    __shared__ uint32_t cnt2[kOneKeys];          // per key: pairs in the batch (low half) | pairs in front of this range (high half)
    __shared__ int32_t cbase[kOneKeys + 1];      // first chunk of each group
    __shared__ __attribute__((aligned(16))) int32_t lkey[kOneRange];
    __shared__ int32_t lrank[kOneRange];
    __shared__ __attribute__((aligned(16))) int32_t wave_tot[16];
    static_assert(kOneThreads == 4 * kOneRange, "four threads per pair in the in-range rank");
    static_assert(kOnePairs <= 32768, "two 16-bit counts per word");
    const int tid = threadIdx.x, NK = n_slots * E;
    const int p0 = block * kOneRange;
    const bool records = pv.chunks != nullptr;   // (the token-level grouping of a route plan has none)
    for (int k = tid; k < NK; k += kOneThreads) cnt2[k] = 0u;
    if (tid < kOneRange) lkey[tid] = -1;         // positions past the batch
    __syncthreads();
    // one visit per pair: both counts in one LDS add, and the keys of this range kept
    auto visit = [&](int q, int key) __attribute__((always_inline)) {
        if (key >= 0) atomicAdd(&cnt2[key], q < p0 ? 0x10001u : 1u);
        if (q >= p0 && q < p0 + kOneRange) lkey[q - p0] = key;
    };
    if (topk && K > 1) {
        // a thread takes whole tokens: the slot (and whether it is ready) once, the token's K experts
        // as 16-byte pieces where K allows -- an eighth of the loads of a pair-by-pair walk at K = 8
        const int T = P / K;
        const bool vec = K <= 16 && !(K & 3) && !((uintptr_t)topk & 15);    // a token's experts as 16-byte pieces
        constexpr int kT = 2;                                   // tokens per thread in flight
        for (int t0 = 0; t0 < T; t0 += kT * kOneThreads) {
            int sl[kT];
            int4 ex[kT][4];
#pragma unroll
            for (int u = 0; u < kT; ++u) {
                const int t = t0 + u * kOneThreads + tid;
                sl[u] = t < T ? token_slot[t] : -1;
                if (t < T && vec) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) if (4 * v < K) ex[u][v] = *(const int4 *)(topk + (int64_t)t * K + 4 * v);
                }
            }
#pragma unroll
            for (int u = 0; u < kT; ++u) {
                const int t = t0 + u * kOneThreads + tid;
                if (t >= T) continue;
                const int s = sl[u];
                const bool ok = s >= 0 && s < n_slots && !(ready_rank && ready_rank[s] <= 0);
                if (vec) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        if (4 * v >= K) break;
                        const int e4[4] = {ex[u][v].x, ex[u][v].y, ex[u][v].z, ex[u][v].w};
#pragma unroll
                        for (int i = 0; i < 4; ++i) visit(t * K + 4 * v + i, ok && e4[i] >= 0 && e4[i] < E ? s * E + e4[i] : -1);
                    }
                } else {
                    for (int k = 0; k < K; ++k) {
                        const int e = topk[(int64_t)t * K + k];
                        visit(t * K + k, ok && e >= 0 && e < E ? s * E + e : -1);
                    }
                }
            }
        }
    } else {
        constexpr int kU = 16;                                  // keys per thread in flight
        for (int q0 = 0; q0 < P; q0 += kU * kOneThreads) {
            int key[kU];
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                const int q = q0 + u * kOneThreads + tid;
                key[u] = q < P ? route_key(topk, token_slot, ready_rank, q, k_magic, E, n_slots) : -1;
            }
#pragma unroll
            for (int u = 0; u < kU; ++u) visit(q0 + u * kOneThreads + tid, key[u]);
        }
    }
    if (tid < kOneRange) lrank[tid] = 0;
    __syncthreads();
    // Members of the same group in front of a pair inside the range: pair i = tid % 256 against the
    // quarter tid / 256 of the range, four keys per LDS read; the quarters' counts meet in lrank.
    {
        const int i = tid & (kOneRange - 1), m0 = (tid / kOneRange) * (kOneRange / 4);
        const int key = lkey[i];
        int r = 0;
        if (key >= 0) {
#pragma unroll 4
            for (int m = m0; m < m0 + kOneRange / 4; m += 4) {
                const int4 k4 = *(const int4 *)(lkey + m);
                r += (m < i && k4.x == key) + (m + 1 < i && k4.y == key) + (m + 2 < i && k4.z == key) + (m + 3 < i && k4.w == key);
            }
            if (r) atomicAdd(&lrank[i], r);
        }
    }
    // exclusive scans of the group sizes and of the groups' chunk counts: one scan of both, 16 bits
    // each (at most kOnePairs = 2^15 pairs, and no more chunks than pairs)
    const int per = (NK + kOneThreads - 1) / kOneThreads;       // <= 4
    const int lo = min(NK, tid * per), hi = min(NK, lo + per);
    int cnt[kOneKeys / kOneThreads], both = 0;
#pragma unroll
    for (int u = 0; u < kOneKeys / kOneThreads; ++u) {
        cnt[u] = lo + u < hi ? (int)(cnt2[lo + u] & 0xffffu) : 0;
        both += cnt[u] | ((cnt[u] + kChunk - 1) / kChunk) << 16;
    }
    const int inc = block_scan<false>(both, tid, 16, wave_tot);
    const int inc_i = inc & 0xffff, inc_c = (int)((uint32_t)inc >> 16);
    int run_i = inc_i - (both & 0xffff), run_c = inc_c - (int)((uint32_t)both >> 16);
#pragma unroll
    for (int u = 0; u < kOneKeys / kOneThreads; ++u) {
        if (lo + u < hi) {
            goff[lo + u] = run_i;
            cbase[lo + u] = run_c;
            run_i += cnt[u];
            run_c += (cnt[u] + kChunk - 1) / kChunk;
        }
    }
    if (tid == kOneThreads - 1) { goff[NK] = inc_i; cbase[NK] = inc_c; }
    __syncthreads();
    const int n_rows = goff[NK], n_chunks = cbase[NK];
    if (block == 0) {
        for (int k = tid; k <= NK; k += kOneThreads) {
            pv.group_off[k] = goff[k];
            if (out_group_off) out_group_off[k] = goff[k];
            if (records) pv.chunk_base[k] = cbase[k];
        }
        if (tid == 0) { pv.hdr[0] = n_chunks; pv.hdr[1] = n_rows; }
    }
    if (tid < kOneRange) {
        const int j = p0 + tid;                  // this range also owns positions / records [p0, p0 + kOneRange)
        if (j < P) {
            if (records && j >= n_chunks && j < rec_bound) pv.chunks[(int64_t)j * kRec + 1] = 0;   // empty record past the live chunks
            if (j >= n_rows) {
                pv.sorted[j] = -1;
                if (out_sorted) out_sorted[j] = -1;
            }
            const int key = lkey[tid];
            pv.key_of[j] = key;                      // (the key as this plan saw it: the MoE down projection asks per pair)
            if (key >= 0) {
                const int r = (int)(cnt2[key] >> 16) + lrank[tid];
                const int off = goff[key], n = goff[key + 1] - off;
                pv.sorted[off + r] = j;
                if (out_sorted) out_sorted[off + r] = j;
                if (records) {
                    int32_t *rec = pv.chunks + (int64_t)(cbase[key] + r / kChunk) * kRec;
                    rec[4 + (r % kChunk)] = j;
                    if (r % kChunk == 0) { rec[0] = key; rec[1] = min(kChunk, n - r); rec[2] = off + r; rec[3] = 0; }
                }
            }
        }
    }
}

// Workgroups [0, pair_blocks) group the routed pairs by (slot, expert); the workgroups behind them
// (route plans only) group the tokens by slot with the same code: key = slot, one item per token.
__global__ __launch_bounds__(kOneThreads)
void plan_route_one_kernel(PlanView pv, const int32_t *__restrict__ topk, const int32_t *__restrict__ token_slot,
                           int P, int K, uint32_t k_magic, int E, int n_slots, const int32_t *__restrict__ ready_rank,
                           int32_t *__restrict__ out_sorted, int32_t *__restrict__ out_group_off, int rec_bound,
                           int pair_blocks, int T)
{
    const int b = (int)blockIdx.x;
    if (b < pair_blocks) {
        plan_route_one_body(pv, topk, token_slot, P, K, k_magic, E, n_slots, ready_rank, out_sorted, out_group_off, rec_bound, b);
    } else {
        const PlanView tv = plan_token_view(pv);
        plan_route_one_body(tv, nullptr, token_slot, T, 1, 0u, 1, n_slots, ready_rank, nullptr, nullptr, 0, b - pair_blocks);
    }
}

bool plan_route_in_one_launch(int64_t P, int64_t NK)
{
    return P <= kOnePairs && NK <= kOneKeys && !tuning(kPlanPipeline);
}

hipError_t launch_plan_general(const PlanView &pv, const int32_t *topk, const int32_t *token_slot,
                               int T, int K, int E, int n_slots, const int32_t *ready_rank,
                               int32_t *out_sorted, int32_t *out_group_off, hipStream_t st)
{
    const int P = T * K, NK = n_slots * E;
    const bool route = topk != nullptr;            // a route plan also groups the tokens by slot
    if (plan_route_in_one_launch(P, NK)) {
        const int pair_blocks = (P + kOneRange - 1) / kOneRange, tok_blocks = route ? (T + kOneRange - 1) / kOneRange : 0;
        plan_route_one_kernel<<<dim3((unsigned)(pair_blocks + tok_blocks)), dim3(kOneThreads), 0, st>>>(
            pv, topk, token_slot, P, K, K > 1 ? (uint32_t)((0x100000000ull + (uint64_t)K - 1) / (uint64_t)K) : 0u, E, n_slots,
            ready_rank, out_sorted, out_group_off, (int)max_chunks(P, NK), pair_blocks, T);
        return hipGetLastError();
    }
    const unsigned nb = (unsigned)((P + 255) / 256);
    plan_hist_kernel<<<dim3(nb), dim3(256), 0, st>>>(pv, topk, token_slot, P, K, E, n_slots, ready_rank);
    plan_scan_kernel<<<dim3(1), dim3(1024), 0, st>>>(pv, NK, out_group_off);
    plan_scatter_kernel<<<dim3(nb), dim3(256), 0, st>>>(pv, P);
    plan_fix_kernel<<<dim3(nb), dim3(256), 0, st>>>(pv, P, out_sorted, (int)max_chunks(P, NK));
    if (route) {
        const PlanView tv = plan_token_view(pv);
        const unsigned tb = (unsigned)((T + 255) / 256);
        plan_hist_kernel<<<dim3(tb), dim3(256), 0, st>>>(tv, nullptr, token_slot, T, 1, 1, n_slots, ready_rank);
        plan_scan_kernel<<<dim3(1), dim3(1024), 0, st>>>(tv, n_slots, nullptr);
        plan_scatter_kernel<<<dim3(tb), dim3(256), 0, st>>>(tv, T);
        plan_fix_kernel<<<dim3(tb), dim3(256), 0, st>>>(tv, T, nullptr, 0);
    }
    return hipGetLastError();
}

}  // namespace mlora
