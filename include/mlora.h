/*
 * mlora -- batched multi-adapter LoRA apply for one MI355X (gfx950).
 *
 * The operation (standard LoRA update, which the paper adopts through its LoRA citation in
 * Section 1 and Related Work; per-token adapter choice from the serving path of Sections 3.4
 * and 4, where a request decodes with the adapter resident in its GPU batch slot):
 *
 *     y[t, :] += (alpha_s / r_s) * B_s * (A_s * x[t, :])          s = a(t) >= 0
 *
 * with A_s [r_s, d_in] and B_s [d_out, r_s] in the PEFT export layout (Section 3.3), kept in
 * slot tables allocated at a configured maximum rank into which smaller adapters are padded
 * (Section 3.2).  bf16 in, fp32 accumulate, one round-to-nearest-even back to bf16.
 *
 * Conventions for every entry point
 *   - extern "C"; returns an int32 status (0 = MLORA_OK, negative = error); never throws.
 *   - Pointers named *_dev / x / y / token_slot / topk_ids are DEVICE pointers owned by the
 *     caller; everything else is a HOST pointer.  `stream` is a hipStream_t passed as void*
 *     (NULL = the default stream).  Calls only enqueue work; they do not synchronise the
 *     stream (lora_apply_segmented may wait for its own previous small host-to-device copy).
 *   - bf16 tensors are row-major with 16-byte aligned rows; d_in and d_out are multiples of 8;
 *     ldx / ldy are row strides in elements (multiples of 8).
 *   - A slot index of -1, an index outside [0, n_slots), or a slot that holds no adapter
 *     (never uploaded, or evicted) leaves the row bit-identical.
 *   - A site serves applies on one stream at a time: its scratch (private plan, exchange words,
 *     prefill partial sums) is shared by all of its calls, so two applies of one site that overlap
 *     on different streams race; uploading into a slot that an unfinished apply on another stream
 *     reads is a caller error.  Different sites are independent.
 */
#ifndef MLORA_H
#define MLORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MLORA_OK            =  0,
    MLORA_E_INVALID     = -1,   /* null pointer, negative size, bad descriptor            */
    MLORA_E_SHAPE       = -2,   /* rank outside [1, r_max], misaligned strides or widths  */
    MLORA_E_SLOT        = -3,   /* slot outside [0, n_slots)                              */
    MLORA_E_SEGMENTS    = -4,   /* offsets not monotone, not starting at 0 or ending at T */
    MLORA_E_HIP         = -5,   /* a HIP runtime call or launch failed                    */
    MLORA_E_UNSUPPORTED = -6    /* e.g. MoE call on a dense site, batch larger than plan  */
};

#define MLORA_MAX_RANK 64       /* r_max is rounded up to a power of two <= 64 in the tables */
#define MLORA_CHUNK     4       /* rows of one adapter handled together by one workgroup   */

/* One LoRA-targeted projection (a "site"): its slot tables and their shape limits
 * (Section 3.2: a worker advertises adapter-shape limits and allocates slots at them). */
typedef struct {
    int32_t d_in, d_out;
    int32_t r_max;              /* largest rank a slot can hold, 1..64                     */
    int32_t n_slots;            /* resident adapters (the same-batch window is <= 64)      */
    int32_t n_experts;          /* 0 = dense site; > 0 = packed per-expert tables          */
    int32_t device;             /* HIP device ordinal                                      */
} mlora_site_desc;

typedef struct mlora_site mlora_site;   /* opaque, host-side handle                        */
typedef struct mlora_plan mlora_plan;   /* opaque: one batch's rows grouped by adapter     */

const char *mlora_status_str(int32_t status);

/* Sizes in bytes of the four device buffers a site needs.
 *   a_tab: [n_slots, max(n_experts,1), r_pad, d_in]  bf16   (r_pad = r_max rounded to 2^k)
 *   b_tab: [n_slots, max(n_experts,1), d_out, r_pad] bf16
 *   meta : rank int32[n_slots] | scale fp32[n_slots] | catalog_id int64[n_slots]
 *   scratch: private grouping buffers for the entry points that take no explicit plan.
 * Errors: MLORA_E_INVALID (null, non-positive sizes), MLORA_E_SHAPE (d_in/d_out not a
 * multiple of 8, r_max outside 1..64). */
int32_t mlora_site_bytes(const mlora_site_desc *desc, size_t *a_tab, size_t *b_tab,
                         size_t *meta, size_t *scratch);

/* Binds caller-allocated device buffers (256-byte aligned, sizes from mlora_site_bytes) to a
 * new site and marks every slot empty (enqueued on the default stream, then synchronised once).
 * The caller keeps ownership of the buffers and must keep them alive until destroy. */
int32_t mlora_site_create(const mlora_site_desc *desc, void *a_tab_dev, void *b_tab_dev,
                          void *meta_dev, void *scratch_dev, mlora_site **out);
void    mlora_site_destroy(mlora_site *site);   /* frees host state only */
/* Synchronises `stream`, then returns MLORA_E_HIP if a launch on this site gave up waiting for
 * an intermediate result of its own launch (bounded wait; not expected to happen) and clears
 * that flag; MLORA_OK otherwise. */
int32_t mlora_site_check(mlora_site *site, void *stream);

/* Copies one adapter into slot `slot` (the last hop of an adapter load, Sections 3.4 and 4:
 * an exported revision becomes an engine-local adapter in a GPU slot).
 *   A: [r, d_in] (MoE site: [n_experts, r, d_in]); B: [d_out, r] (MoE: [n_experts, d_out, r]),
 *   bf16, contiguous, host memory if src_on_device == 0 else device memory.
 * Rows/columns r..r_pad-1 are zero-filled; rank[slot] = r, scale[slot] = alpha / r,
 * catalog_id[slot] = catalog_id.  Asynchronous on `stream`; a host source must stay valid
 * until the stream has passed this point.
 * Errors: MLORA_E_SLOT, MLORA_E_SHAPE (r < 1 or r > r_max), MLORA_E_INVALID, MLORA_E_HIP. */
int32_t lora_slots_upload(mlora_site *site, int32_t slot, int64_t catalog_id,
                          const void *A, const void *B, int32_t r, float alpha,
                          int32_t src_on_device, void *stream);
/* The same upload from per-expert tensors (the fragmented form an adapter is exported in before
 * packing, Section 4.4: one [r, d_in] and one [d_out, r] tensor per expert and projection).
 *   A_e, B_e: HOST arrays of max(n_experts, 1) HOST pointers to contiguous bf16 tensors.
 * The tensors are stacked along the expert axis, zero padded to r_pad, into a pinned host image of
 * the slot that the site keeps, and leave the host in a few large copies (about 2 MB each, issued
 * while the host packs the next piece) instead of one copy per tensor.  The call returns when the
 * image is packed and every copy is enqueued; the caller's tensors may be released then.  A second call on the same
 * site waits until the previous image has been copied.
 * mlora_pack_experts is the host-only packing step (a_img / b_img: mlora_slot_image_bytes bytes);
 * it needs no GPU. */
int32_t mlora_slot_image_bytes(const mlora_site_desc *desc, size_t *a_bytes, size_t *b_bytes);
int32_t mlora_pack_experts(const mlora_site_desc *desc, const void *const *A_e, const void *const *B_e,
                           int32_t r, void *a_img, void *b_img);
int32_t lora_slots_upload_experts(mlora_site *site, int32_t slot, int64_t catalog_id,
                                  const void *const *A_e, const void *const *B_e, int32_t r, float alpha,
                                  void *stream);
/* Marks the slot empty (rank 0): rows that point at it are left untouched (an adapter is
 * visible to traffic only while it is ready, Section 4). */
int32_t lora_slots_evict(mlora_site *site, int32_t slot, void *stream);

/* Device-side catalog id -> slot: token_slot[t] = the lowest slot that is ready (rank > 0) and whose
 * catalog_id equals token_catalog_id[t], else -1 (ids < 0 map to -1).  Both arrays are DEVICE memory
 * (int64[T] in, int32[T] out).  Lets a batch carry the adapter names of the catalog (Section 4:
 * the actor maps a revision to a local adapter id) and resolve them without a host round trip; the
 * result feeds lora_plan_decode / lora_apply_decode / moe_plan_route. */
int32_t lora_slot_lookup(mlora_site *site, const int64_t *token_catalog_id, int32_t T, int32_t *token_slot,
                         void *stream);

/* ---- explicit plans: group a batch once, reuse it for every site of every layer ------------ */

/* Device bytes for a plan that can hold up to max_items rows (dense: tokens; MoE: token-expert
 * pairs) over n_keys groups (dense: n_slots; MoE: n_slots * n_experts). */
int32_t mlora_plan_bytes(int32_t max_items, int32_t n_keys, size_t *bytes);
int32_t mlora_plan_create(int32_t max_items, int32_t n_keys, int32_t device, void *plan_dev,
                          mlora_plan **out);
void    mlora_plan_destroy(mlora_plan *plan);

/* Groups the T rows of a decode batch by slot (stable: ascending row inside a slot) and cuts
 * each group into chunks of MLORA_CHUNK rows.  token_slot: DEVICE int32[T].  If ready_from is
 * non-NULL, rows whose slot is empty at that site are dropped here; the apply re-checks anyway.
 * Errors: MLORA_E_UNSUPPORTED if T > max_items or n_slots > n_keys. */
int32_t lora_plan_decode(mlora_plan *plan, const int32_t *token_slot, int32_t T, int32_t n_slots,
                         const mlora_site *ready_from, void *stream);
/* y[T, d_out] += per-row LoRA delta using a plan built by lora_plan_decode on the same stream
 * (or otherwise ordered before this call).  x: [T, d_in] bf16, y: [T, d_out] bf16 in place. */
int32_t lora_apply_decode_planned(mlora_site *site, const mlora_plan *plan,
                                  const void *x, int64_t ldx, void *y, int64_t ldy, void *stream);

/* Several dense sites that take the same batch plan, applied with as few launches as possible
 * (q/k/v of one layer, or gate/up, are independent of each other and can share one launch; sites
 * of another rank, MoE sites and sites with a small d_in get a launch of their own).  sites, xs, ldxs, ys, ldys are HOST
 * arrays of length n_sites; each (site, x, y) triple follows the rules of
 * lora_apply_decode_planned.  The result is that of n_sites separate calls up to the order in which
 * the fp32 partial sums of the shrink are added (a launch may cut d_in into more or fewer slices). */
int32_t lora_apply_decode_multi(mlora_site *const *sites, int32_t n_sites, const mlora_plan *plan,
                                const void *const *xs, const int64_t *ldxs,
                                void *const *ys, const int64_t *ldys, void *stream);
/* lora_plan_decode followed by lora_apply_decode_multi, for the first sites of a decode step (q/k/v
 * of the first layer): the batch is grouped by slot (Section 4: the requests of one decoding step
 * name at most 64 distinct resident adapters) and the plan is left in `plan` for every later
 * planned apply of the step.  For batches of up to 256 rows the leading sites that can share a
 * launch build the plan inside that launch (every workgroup sorts the batch's keys itself instead
 * of waiting for a planner launch; workgroup 0 writes the plan out), which saves the planner
 * launch; otherwise this is exactly the two calls.  Plan and results are those of the two calls,
 * bit for bit.  Arguments and errors as for those two calls. */
int32_t lora_plan_apply_decode_multi(mlora_site *const *sites, int32_t n_sites, mlora_plan *plan,
                                     const int32_t *token_slot, int32_t T, int32_t n_slots,
                                     const mlora_site *ready_from,
                                     const void *const *xs, const int64_t *ldxs,
                                     void *const *ys, const int64_t *ldys, void *stream);

/* Route index build for packed MoE LoRA (per-expert LoRA tensors are keyed by expert id,
 * Section 3.4): pair p = t*K + k has key = token_slot[t] * n_experts + topk_ids[t, k]; pairs
 * with a usable slot are sorted by key with a stable counting sort (ties ascending p).
 *   topk_ids: DEVICE int32[T, K] with distinct experts per token; token_slot: DEVICE int32[T].
 *   out_sorted_pair: nullable DEVICE int32[T*K]; entries past the number of usable pairs = -1.
 *   out_group_off : nullable DEVICE int32[n_slots*n_experts + 1], exclusive prefix of counts.
 * Both outputs are exactly determined by the inputs (bit-exact against a CPU counting sort). */
int32_t moe_plan_route(mlora_plan *plan, const int32_t *topk_ids, const int32_t *token_slot,
                       int32_t T, int32_t K, int32_t n_slots, int32_t n_experts,
                       const mlora_site *ready_from,
                       int32_t *out_sorted_pair, int32_t *out_group_off, void *stream);
/* y[T*K, d_out] (pair-major) += per-pair LoRA delta with the (slot, expert) tables of a packed
 * MoE site, using a plan from moe_plan_route.  x: [T, d_in]. */
int32_t moe_lora_apply_planned(mlora_site *site, const mlora_plan *plan,
                               const void *x, int64_t ldx, void *y, int64_t ldy, void *stream);
/* Several packed MoE sites that take the same route plan, applied with as few launches as possible:
 * the gate and up projections of an expert layer read the same x with the same routing (per-expert
 * LoRA tensors on gate, up and down, Section 3.4) and are independent of each other, so sites of
 * rank 8 or 16 with the same rank share one launch; others get a launch of their own.  sites, xs,
 * ldxs, ys, ldys are HOST arrays of length n_sites; each (site, x, y) triple follows the rules of
 * moe_lora_apply_planned, and the result is bit-identical to n_sites such calls. */
int32_t moe_lora_apply_multi(mlora_site *const *sites, int32_t n_sites, const mlora_plan *plan,
                             const void *const *xs, const int64_t *ldxs, void *const *ys,
                             const int64_t *ldys, void *stream);

/* MoE down projection with the routing-weight combine (per-expert LoRA tensors on the expert down
 * projection, Sections 3.4 and 4.4): pair p = t*K + k has its own input row x[p, :] (the expert's
 * intermediate activation) and the K pairs of a token add into one output row,
 *
 *     y[t, :] += sum_{k = 0..K-1} pair_w[t, k] * (alpha_s / r_s) * B_{s,e(t,k)} * (A_{s,e(t,k)} * x[p, :])
 *
 * summed in fp32 and rounded to bf16 once: every output row has one writer, no atomics, and the
 * summation order is fixed (by expert id), so the result is deterministic.
 *   plan: from moe_plan_route on the same topk_ids / token_slot;  x: [T*K, d_in];  y: [T, d_out];
 *   pair_w: DEVICE fp32 [T, K];  token_slot: DEVICE int32[T], the array given to moe_plan_route
 *   (the plan already holds the grouping of the tokens by slot; the argument is checked, not read);
 *   workspace: DEVICE, moe_down_workspace_bytes(T, K, d_out) bytes (T * K * MLORA_MAX_RANK 32-bit
 *   words), 16-byte aligned, overwritten.
 * Two launches.  The first leaves in the workspace, for every pair of the plan, the rank-r vector
 * h[p] = pair_w[p] * (alpha / r) * A x[p] as bf16 head and tail (one wave per chunk of up to four
 * pairs of a (slot, expert) group; the chunks of a group run side by side, so an adapter's A rows
 * leave memory once).  The second is, per slot, the dense contraction
 * Y_s += H_s * Bcat_s on the matrix cores: H_s holds h[(t, k)] in the r columns of expert e(t, k)
 * of row t, Bcat_s is the slot's per-expert B tensors stacked along the contraction axis, as the
 * packed tables store them.  Pairs that the plan left out (expert ids outside [0, n_experts), slots
 * not ready when the plan was built) add nothing, whatever the workspace holds.
 * A token's K expert ids must be distinct (as a top-k routing gives them): of two pairs of one token
 * on the same expert only one would be added.
 * Limits: K <= 16, and 32 * (n_experts + 4 * K * max(r_pad, 8)) bytes of tables must fit the LDS
 * of a compute unit (n_experts = 1024 at rank 8 and K = 8 does; MLORA_E_UNSUPPORTED otherwise).
 * Errors: as moe_lora_apply_planned; MLORA_E_INVALID on null pointers. */
int32_t moe_down_workspace_bytes(int32_t T, int32_t K, int32_t d_out, size_t *bytes);
int32_t moe_lora_apply_down(mlora_site *site, const mlora_plan *plan, const void *x, int64_t ldx,
                            const float *pair_w, const int32_t *token_slot, void *workspace,
                            void *y, int64_t ldy, void *stream);

/* ---- the four calls of the problem statement ------------------------------------------------ */

/* Decode: one token per row, gather-by-index.  Equivalent to lora_plan_decode on the site's
 * private scratch followed by lora_apply_decode_planned (for batches of up to 256 rows on sites
 * whose d_in is wide enough for the 8-wave kernel the plan is built inside the apply launch: same
 * plan, same bits, one launch).  Sites of rank 1 and 2 (compact catalogs of tiny adapters, Section 4)
 * are applied row by row without any plan: grouping rows by slot would save at most two adapter
 * rows per row, less than a planner launch costs; the result equals the planned one up to the order
 * in which the fp32 partial sums of the shrink are added.  T = 0 is MLORA_OK and launches nothing.
 * Errors: MLORA_E_UNSUPPORTED on a MoE site, MLORA_E_SHAPE on bad strides. */
int32_t lora_apply_decode(mlora_site *site, const void *x, int64_t ldx, void *y, int64_t ldy,
                          const int32_t *token_slot, int32_t T, void *stream);

/* lora_apply_decode for callers that cannot allocate device memory, and cannot let a library do it:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same result bit for bit; it allocates nothing (no hipMalloc / hipFree, no allocating
 * library call).  What lora_apply_decode keeps in the site's scratch buffer -- the batch plan, the
 * control block and the exchange words of launches whose workgroups trade partial sums -- lives in a
 * device array inside the library: 1,147,904 bytes per GPU the library runs on, held until the process ends
 * and set up by the first call on that GPU (a few small fill launches on `stream`, waited for once;
 * make that first call outside any graph capture).
 * Limits: T <= 1024 rows and a site of at most 1024 slots, else MLORA_E_UNSUPPORTED (nothing is
 * launched).  Every call on a GPU shares that GPU's array, whatever the site: calls that overlap on
 * one GPU (different streams) race; calls on one stream, or otherwise ordered, are safe.  The array
 * keeps the last call's contents; what has to start clean is cleared by the kernels themselves. */
int32_t lora_apply_decode_noalloc(mlora_site *site, const void *x, int64_t ldx, void *y, int64_t ldy,
                                  const int32_t *token_slot, int32_t T, void *stream);

/* Segmented prefill: rows [seg_off[k], seg_off[k+1]) all use slot seg_slot[k] (a request's
 * prompt is one contiguous run).  seg_off (int32[S+1]) and seg_slot (int32[S]) are HOST arrays;
 * they are validated here (MLORA_E_SEGMENTS / MLORA_E_SLOT) and copied to the device.  Sites
 * with r_pad == 64 and d_in a multiple of 16 run the MFMA kernel; others run the
 * vector kernel over runs of MLORA_CHUNK rows. */
int32_t lora_apply_segmented(mlora_site *site, const void *x, int64_t ldx, void *y, int64_t ldy,
                             const int32_t *seg_off, const int32_t *seg_slot, int32_t S,
                             int32_t T, void *stream);

/* Packed MoE: moe_plan_route on the site's private scratch followed by moe_lora_apply_planned.
 * y is [T*K, d_out] pair-major. */
int32_t moe_lora_apply_packed(mlora_site *site, const void *x, int64_t ldx, void *y, int64_t ldy,
                              const int32_t *topk_ids, const int32_t *token_slot,
                              int32_t T, int32_t K,
                              int32_t *out_sorted_pair, int32_t *out_group_off, void *stream);

/* ---- which adapter sits in which slot (host-side state only; moves no bytes) ------------------ */

/* The GPU-batch tier of the paper's serving section (Section 4: cache tiers, cold loading as
 * scheduled service work, registered / prewarming / ready): catalog id -> slot, least-recently-used
 * eviction among ready slots that are not pinned, one shared load per missing adapter, at most
 * max_in_flight load jobs with at most max_queue waiting behind them, retryable rejection beyond. */
typedef struct mlora_resident mlora_resident;

enum {                          /* results of mlora_resident_request (>= 0; errors are negative)        */
    MLORA_R_READY    = 0,       /* *slot holds the adapter; it becomes the most recently used             */
    MLORA_R_LOAD     = 1,       /* a load job starts: upload into *slot, then mlora_resident_complete     */
    MLORA_R_PENDING  = 2,       /* a load of the same adapter is already running or queued: wait for it   */
    MLORA_R_QUEUED   = 3,       /* waits for a load job; mlora_resident_complete of another job starts it */
    MLORA_R_REJECTED = 4        /* jobs and queue are full: nothing changed, retry later                  */
};
enum {                          /* indices into mlora_resident_stats                                      */
    MLORA_STAT_HITS = 0, MLORA_STAT_LOADS = 1, MLORA_STAT_SHARED = 2, MLORA_STAT_REJECTS = 3,
    MLORA_STAT_EVICTIONS = 4, MLORA_RESIDENT_STATS = 5
};

int32_t mlora_resident_create(int32_t n_slots, int32_t max_in_flight, int32_t max_queue, mlora_resident **out);
void    mlora_resident_destroy(mlora_resident *r);
/* Makes catalog_id (>= 0) known; it is not visible to mlora_resident_lookup before a load completes. */
int32_t mlora_resident_register(mlora_resident *r, int64_t catalog_id);
/* Slot of a READY adapter, else -1 (registered, queued and prewarming adapters are not exposed). */
int32_t mlora_resident_lookup(mlora_resident *r, int64_t catalog_id);
/* See the MLORA_R_* values.  *evicted_id = the adapter that lost *slot to this load, or -1.
 * MLORA_E_INVALID if catalog_id was never registered. */
int32_t mlora_resident_request(mlora_resident *r, int64_t catalog_id, int32_t *slot, int64_t *evicted_id);
/* Ends the load job of catalog_id: ok != 0 -> READY, ok == 0 -> back to registered, its slot free.
 * If a queued job can start now, *next_id / *next_slot name it (the caller uploads it next) and
 * *evicted_id the adapter it displaced; otherwise they are -1. */
int32_t mlora_resident_complete(mlora_resident *r, int64_t catalog_id, int32_t ok, int64_t *next_id,
                                int32_t *next_slot, int64_t *evicted_id);
/* Slots used by the batch that is being built or run are pinned: they are never evicted. */
int32_t mlora_resident_pin(mlora_resident *r, int32_t slot, int32_t pinned);
int32_t mlora_resident_stats(mlora_resident *r, int64_t *out /* [MLORA_RESIDENT_STATS] */);

/* Switches read where a launch is shaped (0 = automatic / default).  Host-side, process-wide; meant for
 * sweeps and for tests that force a path.  Names: rows_poll_limit, rows_rank_bound, rows_items_target,
 * rows_mode, rows_waves, rows_chunk_run (decode / MoE launches); plan_general, plan_separate, plan_pipeline (planners);
 * seg_expand_groups, seg_table_copy, seg_shrink_wgs, seg_no_mfma, seg_overlap (batches of the rank-64
 * prefill in flight on a second stream), seg_fused (-1: that prefill as two launches instead of one);
 * upload_piece_kb.
 * MLORA_E_INVALID for any other name. */
int32_t mlora_set_tuning(const char *name, int32_t value);

#ifdef __cplusplus
}
#endif
#endif /* MLORA_H */
