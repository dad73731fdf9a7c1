/*
 * heatkv.h - C ABI of the MI355X-native HeatKV hot path.
 *
 * HeatKV (head-tuned KV-cache compression for next-scale image generation)
 * keeps, for every attention head, an arbitrary subset of the previously
 * generated scales in the KV cache.  An offline calibration pass measures how
 * much attention mass each head puts on each prior scale (Sec. 3.1, Eq. 2), a
 * ranking of the heads per source scale (Eq. 4) and a budget rule (Eq. 5) are
 * turned into a static pruning schedule (Alg. 1, Alg. 2), and at generation
 * time the queries of the current scale attend over the ragged per-head cache.
 *
 * Conventions
 *  - All indices are 0-based: scales k, i in [0,K), layers in [0,L), heads in
 *    [0,H).  The paper's scale k is k-1 here; "sinks" = s counts the leading
 *    scales 0..s-1 that are never pruned.
 *  - Tensors are dense row-major.  dtype 0 = fp32, 1 = bf16; a "row" is one
 *    token of one head, d elements.  Pointers named dev_* / documented "device"
 *    are HIP device memory owned by the caller; "host" pointers are ordinary
 *    host memory owned by the caller.  The library owns only heatkv_plan
 *    objects (host tables plus small device tables).
 *  - Device work is enqueued on the hipStream_t passed as `stream` (void*, may
 *    be null for the default stream) and returns without waiting for it.
 *  - Every function returns HEATKV_OK (0) or a negative HEATKV_E* code and
 *    never throws; heatkv_last_error() returns a thread-local description of
 *    the last failure.
 *  - KV cache storage ("arena"): one K arena and one V arena, each
 *    [batch][capacity_tokens][d], capacity from heatkv_plan_arena_tokens().
 *    Inside an arena every (layer, head) owns one contiguous run of rows
 *    holding its retained prior scales in ascending scale order; run offsets
 *    are prefix sums fixed by the static schedule.  Each append rewrites one
 *    layer's runs into free space of the same arena (a FIFO of layer regions),
 *    so calls must be issued in generation order: for k = 0..K-1, for
 *    layer = 0..L-1: attend_scale(layer,k) and append_scale(layer,k) in either
 *    order, all on one stream (or otherwise ordered by the caller).
 */
#ifndef HEATKV_H
#define HEATKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HEATKV_OK 0
#define HEATKV_EINVAL (-1)  /* null pointer, bad shape, index out of range, workspace too small */
#define HEATKV_EBUDGET (-2) /* budget smaller than the sink scales (Eq. 5 would exceed the head count) */
#define HEATKV_ENOMEM (-3)  /* host or device allocation failed */
#define HEATKV_EHIP (-4)    /* a HIP runtime call failed; text in heatkv_last_error() */

#define HEATKV_F32 0
#define HEATKV_BF16 1

/* Schedule variants (Alg. 1 and Sec. 4.2 "Pruning Algorithm"). */
#define HEATKV_VARIANT_HEATKV 0       /* per-source-scale orders from S-CAS, greedy early pruning   */
#define HEATKV_VARIANT_BINARY 1       /* one order from CAS, a head keeps all or only the sinks      */
#define HEATKV_VARIANT_NAIVE 2        /* scale-dependent sets, E_k = G_k \ G_{k-1}                   */
#define HEATKV_VARIANT_BINARY_NAIVE 3 /* binary sets, E_k = G_k \ G_{k-1}                            */

#define HEATKV_SET_G 0
#define HEATKV_SET_E 1
#define HEATKV_SET_A 2

#define HEATKV_MAX_SCALES 31

/* Storage format of the cache rows in the arenas.  NATIVE: the shape's dtype.  FP8_E4M3 (bf16 shapes with d = 128
 * only): every retained K and V element is stored as one OCP FP8 E4M3 code (1 sign, 4 exponent bits with bias 7,
 * 3 mantissa bits, subnormals, no infinities, largest magnitude 448), rounded to nearest with ties to even and
 * saturating at +-448 when a scale is appended (a NaN stays a NaN); no scale factors.  The paper leaves
 * quantisation of the cache to future work (Sec. 5) and fixes no format; this one halves the bytes of a cached
 * token (2*d instead of 4*d for K and V together).  Rows are converted once, when they enter the cache; later
 * cache updates move the codes unchanged.  Attention reads them back exactly (every E4M3 value is a bf16 value);
 * the current scale's K/V, which come from the caller's tensors, keep their precision. */
#define HEATKV_KV_NATIVE 0
#define HEATKV_KV_FP8_E4M3 1

/* Problem shape (Sec. 3.1 notation): L layers, H heads per layer, head dimension d,
 * K scales with t[k] tokens each, `batch` independent sequences processed together. */
typedef struct {
  int32_t L, H, d, K, batch, dtype;
  const int32_t* t; /* host, [K]; copied by the functions that take a shape */
} heatkv_shape;

typedef struct heatkv_plan heatkv_plan;

const char* heatkv_last_error(void);

/* ---------------------------------------------------------------------------
 * Calibration (Sec. 3.1, Eq. 2).  For the queries of scale k1 and the
 * uncompressed keys of scales 0..k1 it forms the softmax-normalised attention
 * rows, sums each row inside every key block k2 <= k1, and averages over the
 * t[k1] query rows:
 *     mass[b][h][k2] = 1/t[k1] * sum_n sum_{m in scale k2} alpha[n][m],  0 for k2 > k1.
 * q      device [batch][H][t[k1]][d]
 * k_all  device [batch][H][c[k1]][d], c[k1] = t[0]+..+t[k1], scale blocks in order
 * mass   device fp32 [batch][H][K], fully overwritten
 * ws     device scratch of at least heatkv_calibrate_workspace_bytes(shape,k1) bytes
 * The result is deterministic (fixed reduction order, no floating-point atomics).
 * `layer` is not used by the arithmetic (every layer has the same shape); it is
 * range-checked only.
 */
size_t heatkv_calibrate_workspace_bytes(const heatkv_shape* shape, int k1);
int heatkv_calibrate(const heatkv_shape* shape, int layer, int k1, const void* q, const void* k_all,
                     float sm_scale, float* mass, void* ws, size_t ws_bytes, void* stream);

/* heatkv_calibrate for callers that cannot allocate device memory or pass a workspace: code running under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same arithmetic and the
 * same bits in `mass` as heatkv_calibrate; the per-tile partial sums go to a 1 MiB array that the library holds
 * in static device memory (one copy per GPU, for the life of the process) instead of `ws`.  The call allocates
 * nothing.  HEATKV_EINVAL, before any GPU work, if heatkv_calibrate_workspace_bytes(shape, k1) exceeds 1 MiB
 * (1048576 bytes; e.g. batch 32 x 16 heads x 13 scales fits up to t[k1] = 4992).  All calls on one GPU share
 * the array: two such calls that overlap in time on the same GPU (different streams, different threads) race;
 * issue them on one stream or order them otherwise.  Nothing in the array has to start at zero (every partial
 * that is read was written by the same call first). */
int heatkv_calibrate_static(const heatkv_shape* shape, int layer, int k1, const void* q, const void* k_all,
                            float sm_scale, float* mass, void* stream);

/* Dataset average of Eq. 2 (Sec. 3.1: beta is the mean of beta^d over the
 * calibration set; every batch row is one data point):
 *     beta[layer][h][k1][k2] += weight * sum_b mass[b][h][k2]
 * with weight = 1 / (number of data points).  Batch rows are added in index
 * order by one thread per entry, so the result is reproducible.
 * mass  device fp32 [batch][H][K] as written by heatkv_calibrate
 * beta  device fp32 [L][H][K][K], zero-initialised by the caller before the first call
 */
int heatkv_accumulate_beta(const heatkv_shape* shape, int layer, int k1, const float* mass, float weight,
                           float* beta, void* stream);

/* heatkv_calibrate followed by heatkv_accumulate_beta with one launch fewer (Sec. 3.1, Eq. 2 and the dataset
 * average): same arithmetic in the same order, hence the same bits.  mass may be null when the per-row masses
 * are not wanted. */
int heatkv_calibrate_accumulate(const heatkv_shape* shape, int layer, int k1, const void* q, const void* k_all,
                                float sm_scale, float weight, float* beta, float* mass, void* ws, size_t ws_bytes,
                                void* stream);

/* The same for several query scales in one launch (Sec. 3.1: the calibration set is processed offline, so the
 * activations of all scales of a data point are available together, unlike during generation; one launch
 * keeps the chip full where the short scales alone cannot).  Arithmetic and summation order per scale are
 * those of heatkv_calibrate_accumulate, hence the same bits.
 * n_scales  1..K; k1: host [n_scales], distinct scale indices in any order
 * q, k_all  host arrays of n_scales device pointers, entry i laid out as for heatkv_calibrate with k1[i]
 * mass      null, or a host array of n_scales device pointers (each fp32 [batch][H][K] or null)
 * ws        device scratch of at least heatkv_calibrate_scales_workspace_bytes(shape, n_scales, k1) bytes
 * The host arrays are read during the call only. */
size_t heatkv_calibrate_scales_workspace_bytes(const heatkv_shape* shape, int n_scales, const int32_t* k1);
int heatkv_calibrate_scales_accumulate(const heatkv_shape* shape, int layer, int n_scales, const int32_t* k1,
                                       const void* const* q, const void* const* k_all, float sm_scale, float weight,
                                       float* beta, float* const* mass, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * Schedule construction (Sec. 3.1 Eq. 3-4, Sec. 3.2 Eq. 5, Sec. 3.3 Alg. 1, App. A Alg. 2).
 * Host only, integer arithmetic except for the fp64 sums that rank the heads.
 * beta   host fp32 [L][H][K][K]: beta[l][h][k1][k2], the Eq. 2 masses averaged
 *        over the calibration set (every batch row of every set is one data point).
 * budget_bytes_per_seq: KV bytes one sequence may hold over all layers and
 *        heads; the token budget is B = floor(bytes / (2*d*elem_size)), the
 *        paper's b*T*c_{K-1} in its 1-based numbering (Alg. 1, first line).
 * Ranking: for each source scale i in [sinks, K-1) heads are sorted ascending
 * by sum_{tau>i} beta[tau][i] (fp64, tau ascending); ties keep ascending flat
 * head id l*H+h.  Binary variants sort by sum_{tau in [sinks,K-1)} beta[K-1][tau].
 * N_k = clamp(ceil((T*c[k] - B) / (c[k] - c[sinks-1])), 0, ..) for k in [sinks, K-1);
 * HEATKV_EBUDGET if it exceeds T = L*H.  sinks must be in [0, K-2].
 * On success *out is a new plan to be released with heatkv_plan_destroy().
 */
int heatkv_build_schedule(const heatkv_shape* shape, const float* beta, uint64_t budget_bytes_per_seq,
                          int sinks, int variant, heatkv_plan** out);

/* heatkv_build_schedule with a storage format for the cache rows (HEATKV_KV_*).  The token budget follows the
 * format: B = floor(bytes / (2*d*kv_elem_size)), kv_elem_size = 1 for HEATKV_KV_FP8_E4M3, so the same byte budget
 * holds twice the tokens.  heatkv_build_schedule is this call with HEATKV_KV_NATIVE.  HEATKV_EINVAL for an
 * unknown format or one the shape does not support. */
int heatkv_build_schedule_kv(const heatkv_shape* shape, const float* beta, uint64_t budget_bytes_per_seq,
                             int sinks, int variant, int kv_format, heatkv_plan** out);

/* Plan from an explicit retention pattern instead of Alg. 1.
 * present host uint8 [K][L][H][K]: present[k][l][h][i] != 0 iff prior scale i
 * is in head (l,h)'s cache when scale k is generated.  Requirements, else
 * HEATKV_EINVAL: present[k][..][i] == 0 for i >= k; a scale that is absent at
 * scale k stays absent at k+1.  No G/E/A sets, orders or N_k are defined for
 * such a plan (the accessors return HEATKV_EINVAL). */
int heatkv_load_schedule(const heatkv_shape* shape, const uint8_t* present, heatkv_plan** out);
/* The same with a storage format for the cache rows (HEATKV_KV_*). */
int heatkv_load_schedule_kv(const heatkv_shape* shape, const uint8_t* present, int kv_format, heatkv_plan** out);

void heatkv_plan_destroy(heatkv_plan* plan);

/* Copies the plan's tables to the current HIP device (synchronous, allocates
 * device memory).  attend/append call it on first use if it has not run. */
int heatkv_plan_upload(heatkv_plan* plan);

/* --- plan inspection (host, no GPU needed) -------------------------------- */
/* B in tokens (0 for a loaded plan). */
int64_t heatkv_plan_budget_tokens(const heatkv_plan* plan);
/* N_k for k in [0,K-1): out host int32 [K-1]. */
int heatkv_plan_N(const heatkv_plan* plan, int32_t* out);
/* O_i, i in [sinks, K-1): out host int32 [T] flat head ids, least dependent first.
 * Binary variants hold one order, returned for every valid i. */
int heatkv_plan_order(const heatkv_plan* plan, int i, int32_t* heads_out);
/* G_k / E_k for k in [0,K-1), A_k for k in [0,K): bitmap host uint8 [K][T],
 * bitmap[i][l*H+h] = 1 iff head-scale (i,l,h) is in the set.  Binary variants
 * report a pruned head as all of its non-sink source scales i <= min(k, K-2). */
int heatkv_plan_sets(const heatkv_plan* plan, int k, int which, uint8_t* bitmap);
/* Token positions (in the full c[K-1]-token sequence) of the prior scales that
 * head (layer,head) holds when scale k is generated, ascending.  token_idx may
 * be null to query the count; *n receives the count. */
int heatkv_plan_retained(const heatkv_plan* plan, int k, int layer, int head, int32_t* token_idx, int32_t* n);
/* Storage format of the plan's cache rows (HEATKV_KV_*). */
int heatkv_plan_kv_format(const heatkv_plan* plan);
/* Rows per batch entry of each arena. */
int64_t heatkv_plan_arena_tokens(const heatkv_plan* plan);
/* Bytes of one arena (K or V): batch * arena_tokens * d * (size of a stored element: that of the dtype, or 1 for
 * HEATKV_KV_FP8_E4M3). */
size_t heatkv_plan_arena_bytes(const heatkv_plan* plan);
/* Run table seen by attend_scale(layer,k): for each head the first arena row
 * (within one batch entry) and the number of retained prior tokens.
 * row_out, len_out host int32 [H]. */
int heatkv_plan_runs(const heatkv_plan* plan, int k, int layer, int32_t* row_out, int32_t* len_out);
/* Cache rows (per sequence, all layers) that are live once append_scale(layer,k)
 * has completed: layers <= layer hold their scale-(k+1) runs, later layers
 * their scale-k runs. */
int64_t heatkv_plan_live_tokens(const heatkv_plan* plan, int k, int layer);

/* ---------------------------------------------------------------------------
 * Cache update after layer `layer` has run at scale k (Sec. 3.3: elements of
 * G_k \ A_k leave right after their layer has executed; E_{k+1} before the next
 * scale).  Rewrites the layer's runs into the form attend_scale(layer,k+1)
 * reads: each head keeps the prior scales not in A_{k+1} and gains the t[k]
 * rows of scale k unless (k,layer,head) is in A_{k+1}.  k = K-1 is a no-op
 * (the last scale is never cached).
 * k_new, v_new  device [batch][H][t[k]][d]
 * k_arena, v_arena device, heatkv_plan_arena_bytes() each; updated in place.
 */
int heatkv_append_scale(heatkv_plan* plan, int layer, int k, const void* k_new, const void* v_new,
                        void* k_arena, void* v_arena, void* stream);

/* ---------------------------------------------------------------------------
 * Next-scale attention over the compressed cache (Sec. 3.1 for the attention
 * rows, Sec. 3.3 for which prior scales are present):
 *     out[b][h] = softmax(q[b][h] * [K_R ; k_cur[b][h]]^T * sm_scale) * [V_R ; v_cur[b][h]]
 * where K_R, V_R are head (layer,h)'s retained rows in the arenas.  The current
 * scale is always read from k_cur/v_cur, so the result does not depend on
 * whether append_scale(layer,k) already ran.
 * q, k_cur, v_cur, out  device [batch][H][t[k]][d] (out has the input dtype)
 * ws  device scratch of at least heatkv_attend_workspace_bytes(plan,layer,k) bytes
 *     (may be null when that is 0).
 * Softmax statistics and accumulation are fp32; bf16 inputs are multiplied on
 * the matrix cores with fp32 accumulation, probabilities are rounded to bf16
 * before the second product.
 */
size_t heatkv_attend_workspace_bytes(const heatkv_plan* plan, int layer, int k);
int heatkv_attend_scale(heatkv_plan* plan, int layer, int k, const void* q, const void* k_cur,
                        const void* v_cur, const void* k_arena, const void* v_arena, float sm_scale,
                        void* out, void* ws, size_t ws_bytes, void* stream);

/* attend_scale(layer,k) and append_scale(layer,k) in one launch (Sec. 3.3: the cache update that follows a
 * layer's attention).  Same arguments and results as the two calls made one after the other; the row copies of
 * the cache update run as extra workgroups next to the attention workgroups, which saves one kernel's start
 * and finish latency per layer and scale.  Legal because the update only writes the layer's next region, which
 * the attention of this scale never reads.  k = K-1 is attention only.
 */
int heatkv_attend_append_scale(heatkv_plan* plan, int layer, int k, const void* q, const void* k_cur,
                               const void* v_cur, void* k_arena, void* v_arena, float sm_scale, void* out,
                               void* ws, size_t ws_bytes, void* stream);

/*
 * Head scores behind the orders O_i (Sec. 3.2): scores[i*T + head] for source scale i in [sinks, K-1) is the
 * un-normalised sum of Eq. 4, sum over tau in (i, K) of beta[head][tau][i] (variants HEATKV and NAIVE), or of
 * Eq. 3, sum over tau in [sinks, K-1) of beta[head][K-1][tau], the same for every i (binary variants); fp64,
 * tau ascending, on the fp32 table handed in.  Sorting a row ascending, ties by head id, gives
 * heatkv_plan_order.  Rows outside [sinks, K-1) are zero.  beta: host [L][H][K][K]; scores: host [K][T].
 * Host only.  HEATKV_EINVAL for null pointers, sinks outside [0, K-2] or an unknown variant.
 */
int heatkv_head_scores(const heatkv_shape* shape, const float* beta, int sinks, int variant, double* scores);

/*
 * Stability of the head orders over calibration runs (App. C, S-CAS stability).  betas: host
 * [runs][L][H][K][K], one table per run.  For every source scale i in [sinks, K-1): each run's order O_i
 * gives each head a rank position (0 = pruned first); per head, the standard deviation of its positions
 * around the head's own mean position (population form, divided by `runs`; the appendix does not say which);
 * dispersion[i] = mean over the T heads.  Entries outside [sinks, K-1) are zero.  dispersion: host [K].
 * Host only.  HEATKV_EINVAL for null pointers, runs < 1, sinks outside [0, K-2] or an unknown variant.
 */
int heatkv_rank_dispersion(const heatkv_shape* shape, const float* betas, int runs, int sinks, int variant,
                           double* dispersion);

#ifdef __cplusplus
}
#endif
#endif /* HEATKV_H */
