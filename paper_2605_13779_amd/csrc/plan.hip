// Batch grouping kernels: which rows use which adapter.
//
// Dense decode (at most 64 distinct adapters share one decoding step, Section 4 cache-tier
// table) and the packed-MoE route index build (per-expert LoRA tensors keyed by expert id,
// Section 3.4).  All integer work; every output is uniquely determined by the inputs.
#include "internal.h"

namespace mlora {

size_t plan_words(int64_t M, int64_t NK)
{
    return 8 + 3 * (NK + 1) + 4 * M + kRec * max_chunks(M, NK) + 64;
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
    v.chunks = p;
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
// Small dense batches: one workgroup, comparison counting in LDS.  Row t lands at position
// #{t' usable : (slot', t') < (slot, t)}, which is the stable sort by slot.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024)
void plan_dense_small_kernel(PlanView pv, const int32_t *__restrict__ token_slot, int T, int n_slots,
                             const int32_t *__restrict__ ready_rank, int rec_bound)
{
    extern __shared__ int4 sm4[];
    const int Tp = (T + 3) & ~3;
    int32_t *ss = (int32_t *)sm4;      // usable slot or -1 (padded to a multiple of 4 with -1)
    int32_t *rk = ss + Tp;             // rank of the row inside its slot group
    const int4 *ss4 = (const int4 *)ss, *rk4 = (const int4 *)rk;
    __shared__ int32_t n_chunks, n_rows;
    const int tid = threadIdx.x, nt = blockDim.x;
    if (tid == 0) { n_chunks = 0; n_rows = 0; }
    for (int t = tid; t < Tp; t += nt) {
        int s = -1;
        if (t < T) {
            s = token_slot[t];
            if (s < 0 || s >= n_slots || (ready_rank && ready_rank[s] <= 0)) s = -1;
        }
        ss[t] = s;
    }
    __syncthreads();
    for (int t = tid; t < Tp; t += nt) {
        const int s = ss[t];
        int r = -1;
        if (s >= 0) {
            r = 0;
#pragma unroll 4
            for (int q = 0; q * 4 < t; ++q) {
                const int4 v = ss4[q];
                const int u = q * 4;
                r += (v.x == s) + ((v.y == s) & (u + 1 < t)) + ((v.z == s) & (u + 2 < t)) + ((v.w == s) & (u + 3 < t));
            }
        }
        rk[t] = r;
    }
    __syncthreads();
    int my_chunks = 0, my_rows = 0;
    for (int t = tid; t < T; t += nt) {
        const int s = ss[t];
        if (s < 0) continue;
        int less = 0, n = 0, cb = 0;
#pragma unroll 4
        for (int q = 0; q * 4 < Tp; ++q) {
            const int4 v = ss4[q], k = rk4[q];
            // padding and unusable rows carry slot -1 and never compare below a usable slot here
            const bool l0 = (unsigned)v.x < (unsigned)s, l1 = (unsigned)v.y < (unsigned)s;
            const bool l2 = (unsigned)v.z < (unsigned)s, l3 = (unsigned)v.w < (unsigned)s;
            less += l0 + l1 + l2 + l3;
            n += (v.x == s) + (v.y == s) + (v.z == s) + (v.w == s);
            cb += (l0 & ((k.x % kChunk) == 0)) + (l1 & ((k.y % kChunk) == 0))
                + (l2 & ((k.z % kChunk) == 0)) + (l3 & ((k.w % kChunk) == 0));
        }
        const int r = rk[t], pos = less + r;
        pv.sorted[pos] = t;
        my_rows += 1;
        const int c = cb + r / kChunk;
        int32_t *rec = pv.chunks + (int64_t)c * kRec;
        rec[4 + (r % kChunk)] = t;
        if (r % kChunk == 0) {
            rec[0] = s; rec[1] = min(kChunk, n - r); rec[2] = pos; rec[3] = 0;
            my_chunks += 1;
        }
    }
    if (my_chunks) atomicAdd(&n_chunks, my_chunks);
    if (my_rows) atomicAdd(&n_rows, my_rows);
    __syncthreads();
    if (tid == 0) { pv.hdr[0] = n_chunks; pv.hdr[1] = n_rows; }
    // records past the live chunks are marked empty (count 0): the apply kernels read only records
    for (int c = n_chunks + tid; c < rec_bound; c += nt) pv.chunks[(int64_t)c * kRec + 1] = 0;
}

hipError_t launch_plan_dense_small(const PlanView &pv, const int32_t *token_slot, int T, int n_slots,
                                   const int32_t *ready_rank, hipStream_t st)
{
    int nt = T <= 256 ? 256 : (T <= 512 ? 512 : 1024);
    size_t lds = (size_t)2 * ((T + 3) & ~3) * sizeof(int32_t);
    plan_dense_small_kernel<<<dim3(1), dim3(nt), lds, st>>>(pv, token_slot, T, n_slots, ready_rank,
                                                            (int)max_chunks(T, n_slots));
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
    __shared__ int32_t s_items[1024], s_chunks[1024];
    const int tid = threadIdx.x;
    const int per = (NK + 1023) / 1024;
    const int lo = min(NK, tid * per), hi = min(NK, lo + per);
    int items = 0, chunks = 0;
    for (int k = lo; k < hi; ++k) {
        int c = pv.count[k];
        items += c;
        chunks += (c + kChunk - 1) / kChunk;
    }
    s_items[tid] = items; s_chunks[tid] = chunks;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {          // Hillis-Steele inclusive scan
        int a = 0, b = 0;
        if (tid >= d) { a = s_items[tid - d]; b = s_chunks[tid - d]; }
        __syncthreads();
        s_items[tid] += a; s_chunks[tid] += b;
        __syncthreads();
    }
    int run_i = s_items[tid] - items, run_c = s_chunks[tid] - chunks;
    for (int k = lo; k < hi; ++k) {
        int c = pv.count[k];
        pv.group_off[k] = run_i;
        if (out_group_off) out_group_off[k] = run_i;
        pv.chunk_base[k] = run_c;
        pv.count[k] = 0;                           // leave the histogram clean for the next call
        run_i += c;
        run_c += (c + kChunk - 1) / kChunk;
    }
    if (tid == 1023) {
        pv.group_off[NK] = s_items[1023];
        if (out_group_off) out_group_off[NK] = s_items[1023];
        pv.chunk_base[NK] = s_chunks[1023];
        pv.hdr[0] = s_chunks[1023];
        pv.hdr[1] = s_items[1023];
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
    if (j >= pv.hdr[0] && j < rec_bound) pv.chunks[(int64_t)j * kRec + 1] = 0;   // empty record past the live chunks
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
    int32_t *rec = pv.chunks + (int64_t)(pv.chunk_base[key] + r / kChunk) * kRec;
    rec[4 + (r % kChunk)] = p;
    if (r % kChunk == 0) { rec[0] = key; rec[1] = min(kChunk, n - r); rec[2] = off + r; rec[3] = 0; }
}

hipError_t launch_plan_general(const PlanView &pv, const int32_t *topk, const int32_t *token_slot,
                               int T, int K, int E, int n_slots, const int32_t *ready_rank,
                               int32_t *out_sorted, int32_t *out_group_off, hipStream_t st)
{
    const int P = T * K, NK = n_slots * E;
    const unsigned nb = (unsigned)((P + 255) / 256);
    plan_hist_kernel<<<dim3(nb), dim3(256), 0, st>>>(pv, topk, token_slot, P, K, E, n_slots, ready_rank);
    plan_scan_kernel<<<dim3(1), dim3(1024), 0, st>>>(pv, NK, out_group_off);
    plan_scatter_kernel<<<dim3(nb), dim3(256), 0, st>>>(pv, P);
    plan_fix_kernel<<<dim3(nb), dim3(256), 0, st>>>(pv, P, out_sorted, (int)max_chunks(P, NK));
    return hipGetLastError();
}

}  // namespace mlora
