/*
 * Oracle for the batched multi-adapter LoRA apply.  TEST INFRASTRUCTURE ONLY:
 * it exists so that tests, the smoke check and the benchmark's cpu_baseline leg
 * have an independent, slow, obviously-correct answer.  The product path never
 * calls it and shares no code with it.
 *
 * What it computes (the standard LoRA update the paper builds on via its LoRA
 * citation in Section 1 and Related Work, with the per-token slot rule of the
 * serving path in Sections 3.4 and 4: a request decodes with the adapter that is
 * resident in its GPU batch slot; at most a bounded number of distinct adapters
 * share one batch):
 *
 *     for every row t whose slot s = a(t) is >= 0 and whose slot holds rank r >= 1
 *         h[j]    = sum_i x[t,i] * A_s[j,i]                       j = 0..r-1
 *         y'[t,o] = y[t,o] + (alpha_s / r) * sum_j h[j] * B_s[o,j]
 *     every other row is returned unchanged.
 *
 * A_s is [r, d_in] and B_s is [d_out, r] (the PEFT export layout of Section 3.3),
 * stored in slot tables padded to a maximum rank (Section 3.2: adapters are padded
 * into max-shape slots and the inactive rows masked) -- the oracle simply never
 * reads rows j >= r.  All arithmetic is fp64 over the bf16-valued inputs with no
 * intermediate rounding; loops are in the order written above, no blocking.
 *
 * MoE variant (Section 3.4 / Section 4 packed per-expert tensors, keyed by expert
 * id): routed pair p = t*K + k uses expert e = topk[t,k] and tables indexed
 * [slot, expert]; it updates row p of a pair-major y.
 *
 * Route index build: stable counting sort of the eligible pairs by
 * key = slot*E + expert, ties in ascending p.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* bf16 is the upper half of an IEEE binary32. */
double oracle_bf16_to_f64(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* fp64 -> bf16, round to nearest, ties to even, done directly on the double so
 * that there is no double rounding through binary32.  Finite inputs in the
 * normal bf16 range are what the tests use; overflow goes to infinity, NaN stays
 * NaN, results below the smallest normal are handled through the binary32
 * conversion (exact for those magnitudes because the spacing is coarser). */
uint16_t oracle_f64_to_bf16(double v)
{
    if (isnan(v)) return 0x7fc0;
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs(v);
    if (a == 0.0) return sign;
    if (isinf(a)) return sign | 0x7f80;
    int e;
    double m = frexp(a, &e);            /* a = m * 2^e, m in [0.5,1) */
    int E = e - 1;                      /* a = (2m) * 2^E, 2m in [1,2) */
    if (E < -126) {
        /* subnormal bf16: quantum is 2^-133 */
        double q = ldexp(a, 133);
        double fl = floor(q);
        double rem = q - fl;
        uint32_t n = (uint32_t)fl;
        if (rem > 0.5 || (rem == 0.5 && (n & 1))) n += 1;
        return sign | (uint16_t)n;      /* n == 128 rolls into the smallest normal */
    }
    double q = ldexp(2.0 * m, 7);       /* in [128, 256) */
    double fl = floor(q);
    double rem = q - fl;
    uint32_t n = (uint32_t)fl;          /* 128..255, implicit bit included */
    if (rem > 0.5 || (rem == 0.5 && (n & 1))) n += 1;
    if (n == 256) { n = 128; E += 1; }
    if (E > 127) return sign | 0x7f80;
    uint32_t bits = ((uint32_t)(E + 127) << 7) | (n - 128);
    return sign | (uint16_t)bits;
}

void oracle_round_to_bf16(const double *src, uint16_t *dst, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) dst[i] = oracle_f64_to_bf16(src[i]);
}

void oracle_widen_bf16(const uint16_t *src, double *dst, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) dst[i] = oracle_bf16_to_f64(src[i]);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* One row: y_out[o] = y_in[o] + (alpha/r) * sum_j (sum_i x[i] A[j,i]) B[o,j]. */
static void one_row(const uint16_t *x, const uint16_t *y_in, double *y_out,
                    const uint16_t *A, const uint16_t *B,
                    int64_t d_in, int64_t d_out, int64_t r_max, int r, double alpha)
{
    double h[r > 0 ? r : 1];
    for (int j = 0; j < r; ++j) {
        double acc = 0.0;
        for (int64_t i = 0; i < d_in; ++i)
            acc += oracle_bf16_to_f64(x[i]) * oracle_bf16_to_f64(A[(int64_t)j * d_in + i]);
        h[j] = acc;
    }
    double scale = alpha / (double)r;
    for (int64_t o = 0; o < d_out; ++o) {
        double acc = 0.0;
        for (int j = 0; j < r; ++j)
            acc += h[j] * oracle_bf16_to_f64(B[o * r_max + j]);
        y_out[o] = oracle_bf16_to_f64(y_in[o]) + scale * acc;
    }
}

static void copy_row(const uint16_t *y_in, double *y_out, int64_t d_out)
{
    for (int64_t o = 0; o < d_out; ++o) y_out[o] = oracle_bf16_to_f64(y_in[o]);
}

/*
 * Decode shape: one token per row, each with its own slot index.
 *   x        [T, d_in]  bf16 bits        y_in [T, d_out] bf16 bits
 *   A_tab    [n_slots, r_max, d_in]      B_tab [n_slots, d_out, r_max]
 *   rank     [n_slots]  (0 = empty slot) alpha [n_slots]
 *   token_slot [T] in {-1, 0..n_slots-1}
 *   y_out    [T, d_out] fp64
 * Returns 0, or -1 if a slot index is outside [-1, n_slots).
 */
int oracle_apply_decode(const uint16_t *x, const uint16_t *y_in, double *y_out,
                        const uint16_t *A_tab, const uint16_t *B_tab,
                        const int32_t *rank, const double *alpha,
                        const int32_t *token_slot,
                        int64_t T, int64_t d_in, int64_t d_out,
                        int64_t n_slots, int64_t r_max)
{
    for (int64_t t = 0; t < T; ++t)
        if (token_slot[t] < -1 || token_slot[t] >= n_slots) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < T; ++t) {
        int32_t s = token_slot[t];
        if (s < 0 || rank[s] <= 0) { copy_row(y_in + t * d_out, y_out + t * d_out, d_out); continue; }
        one_row(x + t * d_in, y_in + t * d_out, y_out + t * d_out,
                A_tab + (int64_t)s * r_max * d_in, B_tab + (int64_t)s * d_out * r_max,
                d_in, d_out, r_max, rank[s], alpha[s]);
    }
    return 0;
}

/*
 * Segmented (prefill) shape: rows [seg_off[k], seg_off[k+1]) all use seg_slot[k].
 * Same arithmetic as the decode shape, row by row.
 * Returns -2 if the offsets are not monotone from 0 to T.
 */
int oracle_apply_segmented(const uint16_t *x, const uint16_t *y_in, double *y_out,
                           const uint16_t *A_tab, const uint16_t *B_tab,
                           const int32_t *rank, const double *alpha,
                           const int32_t *seg_off, const int32_t *seg_slot, int64_t S,
                           int64_t T, int64_t d_in, int64_t d_out,
                           int64_t n_slots, int64_t r_max)
{
    if (S > 0 && (seg_off[0] != 0 || seg_off[S] != T)) return -2;
    if (S == 0 && T != 0) return -2;
    for (int64_t k = 0; k < S; ++k) {
        if (seg_off[k + 1] < seg_off[k]) return -2;
        if (seg_slot[k] < -1 || seg_slot[k] >= n_slots) return -1;
    }
    for (int64_t k = 0; k < S; ++k) {
        int32_t s = seg_slot[k];
#pragma omp parallel for schedule(dynamic, 1)
        for (int64_t t = seg_off[k]; t < seg_off[k + 1]; ++t) {
            if (s < 0 || rank[s] <= 0) { copy_row(y_in + t * d_out, y_out + t * d_out, d_out); continue; }
            one_row(x + t * d_in, y_in + t * d_out, y_out + t * d_out,
                    A_tab + (int64_t)s * r_max * d_in, B_tab + (int64_t)s * d_out * r_max,
                    d_in, d_out, r_max, rank[s], alpha[s]);
        }
    }
    return 0;
}

/*
 * Packed MoE shape.  x [T, d_in]; y [T*K, d_out] pair-major (p = t*K + k);
 * A_tab [n_slots, E, r_max, d_in]; B_tab [n_slots, E, d_out, r_max];
 * topk [T, K] expert ids.  Returns -3 on an expert id outside [0, E).
 */
int oracle_apply_moe(const uint16_t *x, const uint16_t *y_in, double *y_out,
                     const uint16_t *A_tab, const uint16_t *B_tab,
                     const int32_t *rank, const double *alpha,
                     const int32_t *topk, const int32_t *token_slot,
                     int64_t T, int64_t K, int64_t E,
                     int64_t d_in, int64_t d_out, int64_t n_slots, int64_t r_max)
{
    for (int64_t t = 0; t < T; ++t) {
        if (token_slot[t] < -1 || token_slot[t] >= n_slots) return -1;
        for (int64_t k = 0; k < K; ++k)
            if (topk[t * K + k] < 0 || topk[t * K + k] >= E) return -3;
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t p = 0; p < T * K; ++p) {
        int64_t t = p / K;
        int32_t s = token_slot[t];
        if (s < 0 || rank[s] <= 0) { copy_row(y_in + p * d_out, y_out + p * d_out, d_out); continue; }
        int64_t g = (int64_t)s * E + topk[p];
        one_row(x + t * d_in, y_in + p * d_out, y_out + p * d_out,
                A_tab + g * r_max * d_in, B_tab + g * d_out * r_max,
                d_in, d_out, r_max, rank[s], alpha[s]);
    }
    return 0;
}

/*
 * MoE down projection with the routing-weight combine (the per-expert LoRA tensors of Section 3.4
 * on the expert down projection; the packed adapter of Section 4.4 stacks them per expert like the
 * gate and up ones).  Pair p = t*K + k has its own input row (the expert's intermediate
 * activation) and the K pairs of a token add into ONE output row, each times its routing weight:
 *
 *   y_out[t, :] = y_in[t, :] + sum_{k=0..K-1} w[t,k] * (alpha_s / r_s) * B_{s,e(t,k)} * (A_{s,e(t,k)} * x[t*K+k, :])
 *
 *   x [T*K, d_in] bf16 bits; y_in [T, d_out] bf16 bits; w [T, K] fp64 (fp32 values widened);
 *   A_tab [n_slots, E, r_max, d_in]; B_tab [n_slots, E, d_out, r_max]; topk [T, K].
 * k runs upwards.  Tokens without a usable slot are copied.  Return codes as oracle_apply_moe.
 */
int oracle_apply_moe_down(const uint16_t *x, const uint16_t *y_in, double *y_out,
                          const uint16_t *A_tab, const uint16_t *B_tab,
                          const int32_t *rank, const double *alpha,
                          const int32_t *topk, const double *w, const int32_t *token_slot,
                          int64_t T, int64_t K, int64_t E,
                          int64_t d_in, int64_t d_out, int64_t n_slots, int64_t r_max)
{
    for (int64_t t = 0; t < T; ++t) {
        if (token_slot[t] < -1 || token_slot[t] >= n_slots) return -1;
        for (int64_t k = 0; k < K; ++k)
            if (topk[t * K + k] < 0 || topk[t * K + k] >= E) return -3;
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < T; ++t) {
        int32_t s = token_slot[t];
        copy_row(y_in + t * d_out, y_out + t * d_out, d_out);
        if (s < 0 || rank[s] <= 0) continue;
        int r = rank[s];
        double scale = alpha[s] / (double)r;
        for (int64_t k = 0; k < K; ++k) {
            int64_t p = t * K + k;
            int64_t g = (int64_t)s * E + topk[p];
            const uint16_t *A = A_tab + g * r_max * d_in, *B = B_tab + g * d_out * r_max;
            double h[r];
            for (int j = 0; j < r; ++j) {
                double acc = 0.0;
                for (int64_t i = 0; i < d_in; ++i)
                    acc += oracle_bf16_to_f64(x[p * d_in + i]) * oracle_bf16_to_f64(A[(int64_t)j * d_in + i]);
                h[j] = acc;
            }
            for (int64_t o = 0; o < d_out; ++o) {
                double acc = 0.0;
                for (int j = 0; j < r; ++j) acc += h[j] * oracle_bf16_to_f64(B[o * r_max + j]);
                y_out[t * d_out + o] += w[p] * (scale * acc);
            }
        }
    }
    return 0;
}

/*
 * Route index build.  Eligible pairs (slot >= 0 and rank[slot] > 0) are sorted by
 * key = slot*E + expert with a stable counting sort, so ties keep ascending p.
 *   sorted_pair [T*K]  (first group_off[n_slots*E] entries valid, rest set to -1)
 *   group_off   [n_slots*E + 1] exclusive prefix sum of the key counts
 */
int oracle_route_sort(const int32_t *topk, const int32_t *token_slot, const int32_t *rank,
                      int64_t T, int64_t K, int64_t E, int64_t n_slots,
                      int32_t *sorted_pair, int32_t *group_off)
{
    int64_t NK = n_slots * E;
    for (int64_t g = 0; g <= NK; ++g) group_off[g] = 0;
    for (int64_t p = 0; p < T * K; ++p) {
        int32_t s = token_slot[p / K];
        if (s < -1 || s >= n_slots) return -1;
        if (topk[p] < 0 || topk[p] >= E) return -3;
        if (s < 0 || rank[s] <= 0) continue;
        group_off[(int64_t)s * E + topk[p] + 1] += 1;
    }
    for (int64_t g = 0; g < NK; ++g) group_off[g + 1] += group_off[g];
    int32_t *cursor = (int32_t *)malloc(sizeof(int32_t) * (size_t)(NK > 0 ? NK : 1));
    if (!cursor) return -9;
    for (int64_t g = 0; g < NK; ++g) cursor[g] = group_off[g];
    for (int64_t p = 0; p < T * K; ++p) sorted_pair[p] = -1;
    for (int64_t p = 0; p < T * K; ++p) {
        int32_t s = token_slot[p / K];
        if (s < 0 || rank[s] <= 0) continue;
        int64_t g = (int64_t)s * E + topk[p];
        sorted_pair[cursor[g]++] = (int32_t)p;
    }
    free(cursor);
    return 0;
}
