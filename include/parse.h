/*
 * parse.h -- C ABI of the MI355X (gfx950) routed low-rank linear layer.
 *
 * The layer computes, per prompt p with rank subset S_p (Sec. 4.1, Eq. 4),
 *
 *        y = sum_{i in S_p} sigma_i u_i (v_i^T x) = A_S (B_S^T x)        (Sec. 4.4, Eq. 10)
 *
 * where A = U Sigma and B^T = V are stored offline with Sigma (and any whitening) absorbed,
 * the rank experts are grouped into G groups of gs = R/G consecutive ranks, a linear router
 * scores the groups for each prompt and keeps the top k (Sec. 4.1, Eq. 5), a pattern cache
 * answers for similar prompts without running the router (Sec. 4.3), the selected groups are
 * aggregated into contiguous memory (Sec. 4.4, "Expert Memory Aggregation") and the subset
 * chosen at prefill is reused for every decode step (Sec. 4.3, "Rank Reuse for Decoding").
 *
 * Conventions that hold for every entry point unless stated otherwise
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *     ordinary host memory.  The library never frees or keeps a caller's pointer beyond
 *     the call (the kernels it enqueued still read/write them until the stream drains).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work and return; they do not synchronise unless the comment says so.
 *   - return value: PARSE_OK (0) or a negative parse_status.  Arguments are checked on the
 *     host before anything is enqueued; on an error nothing was launched and no output
 *     was written.  Contents of device-resident index arrays cannot be checked on the
 *     host: every kernel bounds-checks what it reads from them and skips an invalid
 *     entry (documented per call); parse_check_offsets / parse_check_subset validate
 *     host copies.
 *   - device pointers must be 16-byte aligned; bf16 buffers hold raw bfloat16 bit patterns.
 *   - same inputs give the same bits on every run (no floating-point atomics anywhere).
 */
#ifndef PARSE_H_
#define PARSE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void *parse_stream; /* a hipStream_t */

typedef enum { PARSE_F32 = 0, PARSE_BF16 = 1 } parse_dtype;

typedef enum {
  PARSE_OK = 0,
  PARSE_EINVAL = -1,     /* NULL pointer, bad enum, non-positive size */
  PARSE_ESHAPE = -2,     /* sizes inconsistent with each other or with a kernel's limits */
  PARSE_EALIGN = -3,     /* pointer or leading dimension not aligned as required */
  PARSE_ECAPACITY = -4,  /* pattern cache is full */
  PARSE_EWORKSPACE = -5, /* workspace missing or smaller than the *_workspace_bytes query */
  PARSE_EHIP = -6,       /* a HIP runtime call failed; text via parse_last_hip_error() */
  PARSE_ELAYOUT = -7     /* factor layout not supported by this call */
} parse_status;

/* How a factor matrix is laid out in device memory.
 *
 * PARSE_ROWMAJOR   Vt[R][n] and Ut[R][m], rank-major: row r of Vt is v_r^T (row r of B^T),
 *                  row r of Ut is sigma_r u_r^T (column r of A).  A rank group is gs
 *                  consecutive rows = one contiguous slab.
 * PARSE_MFMA16     bf16 only; the same numbers reordered into the operand order of the
 *                  32x32x16 bf16 matrix instruction, so that a wavefront fetches one 1 KiB
 *                  operand (32 rows x 16 reduction indices) with a single fully coalesced
 *                  16-byte-per-lane load.  With e = 8 bf16 held by one lane:
 *                    Vt element (r, i):  rb=r/32 j=r%32 kb=i/16 q=(i%16)/8 e=i%8
 *                        offset = (((rb*(n/16) + kb)*2 + q)*32 + j)*8 + e
 *                    Ut element (r, c):  kb=r/16 q=(r%16)/8 e=r%8 cb=c/32 j=c%32
 *                        offset = (((kb*(m/32) + cb)*2 + q)*32 + j)*8 + e
 *                  Needs n % 16 == 0, m % 32 == 0, gs % 32 == 0.  A rank group is still one
 *                  contiguous slab of gs*n (resp. gs*m) elements in both matrices, so
 *                  aggregation stays a plain slab copy.
 */
typedef enum { PARSE_ROWMAJOR = 0, PARSE_MFMA16 = 1 } parse_layout;

/* One routed low-rank linear (Sec. 4.4, Eq. 10).  Host struct; Vt/Ut are device pointers. */
typedef struct {
  int32_t n;      /* d_in  */
  int32_t m;      /* d_out */
  int32_t R;      /* stored rank */
  int32_t G;      /* rank groups; gs = R / G, R % G == 0 */
  int32_t dtype;  /* parse_dtype of Vt, Ut and of the activations */
  int32_t layout; /* parse_layout of Vt and Ut */
  const void *Vt; /* B^T           : R x n */
  const void *Ut; /* A^T = (U Sigma)^T : R x m */
} parse_layer;

/* Text for a status code (static storage). */
const char *parse_status_string(int status);
/* Text of the HIP error behind the last PARSE_EHIP on this thread (static storage). */
const char *parse_last_hip_error(void);
/* Library version: major*10000 + minor*100 + patch. */
int parse_version(void);

/* Host-side validators for arrays that the other calls take as device pointers.
 * parse_check_offsets: tok_offsets_host[P+1] must start at 0, be strictly increasing (no empty
 *   prompt) and end at `rows`.  parse_check_subset: k group ids, strictly ascending, each in [0, G).
 * Return PARSE_OK, PARSE_EINVAL (NULL / non-positive sizes) or PARSE_ESHAPE. */
int parse_check_offsets(const int32_t *tok_offsets_host, int32_t P, int32_t rows);
int parse_check_subset(const int32_t *subset_host, int32_t k, int32_t G);

/* ---- offline preparation (Sec. 4.4: factors are reorganised once, offline) -------------
 * Reorders a PARSE_ROWMAJOR bf16 layer into PARSE_MFMA16.  Vt_out / Ut_out: device buffers of
 * R*n and R*m bf16.  PARSE_ELAYOUT if src is not row-major bf16, PARSE_ESHAPE if the divisibility
 * rules above fail. */
int parse_layer_to_mfma16(const parse_layer *src, void *Vt_out, void *Ut_out, parse_stream stream);

/* ---- a1 + a2: pool and route (Sec. 4.1, Eq. 5; prompt-level embedding, end of Sec. 4.1) ----
 * e_p = mean of prompt p's token rows of X (fp32 accumulation); s_p = Wr e_p; subset_out[p] = the
 * k groups with the largest scores, ties to the lower id, written in ascending id order.
 *   X            device [rows][d], dtype xdtype, row-major.  A ready-made embedding is a prompt of length 1.
 *   tok_offsets  device int32 [P+1], prompt p owns rows [tok_offsets[p], tok_offsets[p+1]).  Rows are
 *                clamped to [0, rows]; a prompt that ends up empty gets e_p = 0.
 *   Wr           device float [G][d], bias-free router.      1 <= k <= G <= 64, d % 8 == 0, d <= 16384.
 *   subset_out   device int32 [P][subset_stride] (k ids per row; subset_stride >= k lets a caller
 *                interleave several layers' subsets), scores_out device float [P][G] or NULL,
 *                emb_out device float [P][d] or NULL.
 *   workspace    device, at least parse_route_workspace_bytes(rows, P, d) bytes. */
size_t parse_route_workspace_bytes(int32_t rows, int32_t P, int32_t d);
/* The prompt embedding alone (end of Sec. 4.1), for callers that ask the pattern cache first and run the router only on
 * a miss (Sec. 4.3; parse_cache_lookup_or_route does that): emb_out [P][d] equals parse_route's emb_out bit for bit.
 * Arguments, limits, workspace and errors as for parse_route. */
int parse_pool(const void *X, int32_t xdtype, int32_t rows, const int32_t *tok_offsets, int32_t P, int32_t d,
               float *emb_out, void *workspace, size_t workspace_bytes, parse_stream stream);
int parse_route(const void *X, int32_t xdtype, int32_t rows, const int32_t *tok_offsets, int32_t P,
                int32_t d, const float *Wr, int32_t G, int32_t k, int32_t *subset_out,
                int32_t subset_stride, float *scores_out, float *emb_out, void *workspace,
                size_t workspace_bytes, parse_stream stream);
/* The same with a shared head (Sec. 4.4, expert memory aggregation: the components with the largest singular
 * values are used by nearly all prompts and sit at the head of memory): groups 0..n_shared-1 are in every
 * subset, the router picks the k - n_shared best of the groups n_shared..G-1.  0 <= n_shared <= k;
 * n_shared = 0 is parse_route. */
int parse_route_shared(const void *X, int32_t xdtype, int32_t rows, const int32_t *tok_offsets, int32_t P,
                       int32_t d, const float *Wr, int32_t G, int32_t k, int32_t n_shared,
                       int32_t *subset_out, int32_t subset_stride, float *scores_out, float *emb_out,
                       void *workspace, size_t workspace_bytes, parse_stream stream);

/* ---- a3: pattern cache (Sec. 4.3, "Rank Retrieval for Prefilling") -------------------------
 * Maps prompt embeddings to the rank subsets of all L routed matrices of a model.  The only
 * library-owned state: keys float [capacity][d], values int32 [capacity][L][k], a device-side
 * entry count, and scratch for one batch of at most max_batch prompts.  A lookup answers with
 * the nearest key by cosine similarity (smallest entry index on equal similarity); it is a hit
 * when the similarity is >= tau.  Calls on one cache must be issued on one stream (or be ordered
 * by the caller); calls that overlap on one cache race.
 * create, destroy and count synchronise (count copies to the host); everything else only enqueues, so a whole batch
 * -- explicit inserts included -- can be recorded into a HIP graph. */
typedef struct parse_cache parse_cache;
int parse_cache_create(parse_cache **cache, int32_t capacity, int32_t d, int32_t L, int32_t k,
                       int32_t max_batch);
int parse_cache_destroy(parse_cache *cache);
int parse_cache_clear(parse_cache *cache, parse_stream stream);
/* Routing on a miss (parse_cache_lookup_or_route) keeps groups 0..n_shared-1 in every subset, as
 * parse_route_shared does.  Host-side setting, 0 by default; 0 <= n_shared <= k. */
int parse_cache_set_shared(parse_cache *cache, int32_t n_shared);
/* count_out: host int32, the number of entries.  dropped_out: host int32 or NULL, the number of parse_cache_insert
 * calls since create / clear whose entry was dropped because the cache was full. */
int parse_cache_count(parse_cache *cache, int32_t *count_out, int32_t *dropped_out, parse_stream stream);
/* Appends one entry (only enqueues).  emb device float [d]; subsets device int32 [L][k].  The capacity check happens on the
 * device: an entry that finds the cache full is dropped and counted; parse_cache_count reports how many were. */
int parse_cache_insert(parse_cache *cache, const float *emb, const int32_t *subsets,
                       parse_stream stream);
/* Pure lookup for P <= max_batch embeddings (device float [P][d]).
 *   entry_out  device int32 [P]: the entry that answered, -1 on a miss (also when the cache is empty)
 *   sim_out    device float [P] or NULL: best cosine similarity (-inf if the cache is empty)
 *   subset_out device int32 [P][L][k] or NULL: stored subsets on a hit, untouched on a miss */
int parse_cache_lookup(parse_cache *cache, const float *emb, int32_t P, float tau,
                       int32_t *entry_out, float *sim_out, int32_t *subset_out,
                       parse_stream stream);
/* Lookup with sequential semantics in arrival order: prompt i that misses is routed with
 * Wr (device float [L][G][d], G <= 64) for every layer and, while there is room, appended at once,
 * so that prompt i+1 of the same batch can hit it.
 *   entry_out  device int32 [P]: hit entry, or the new entry's index, or -1 (miss, cache full)
 *   hit_out    device uint8 [P]: 1 = hit, 0 = miss
 *   sim_out    device float [P] or NULL;   subset_out device int32 [P][L][k] (always written) */
int parse_cache_lookup_or_route(parse_cache *cache, const float *emb, int32_t P, float tau,
                                const float *Wr, int32_t G, int32_t *entry_out, uint8_t *hit_out,
                                float *sim_out, int32_t *subset_out, parse_stream stream);

/* ---- a5: bucket prompts by identical subset ---------------------------------------------
 * Patterns are numbered by first appearance in arrival order.
 *   subset      device int32, prompt p's k ids at subset[p*subset_stride .. +k)
 *   pattern_id  device int32 [P];  perm device int32 [P]: prompts ordered by (pattern id, arrival);
 *   bucket_off  device int32 [P+1]: bucket j is perm[bucket_off[j] .. bucket_off[j+1]), entries past
 *               n_patterns repeat P;  n_patterns device int32 [1];  rep device int32 [P]: first prompt
 *               of pattern j for j < n_patterns, -1 after.            1 <= P <= 1024, 1 <= k <= 64. */
int parse_bucket_patterns(const int32_t *subset, int32_t P, int32_t k, int32_t subset_stride,
                          int32_t *pattern_id, int32_t *perm, int32_t *bucket_off,
                          int32_t *n_patterns, int32_t *rep, parse_stream stream);

/* ---- a4: expert memory aggregation (Sec. 4.4) ---------------------------------------------
 * Copies the k selected group slabs of Vt and Ut, in the order the ids are stored (ascending by
 * contract), into Vt_S [k*gs][n] and Ut_S [k*gs][m]; the result has the source's dtype and layout
 * (in both layouts a rank group is one contiguous slab, so this is 2k coalesced slab copies).
 * An id outside [0, G) leaves its slab of the destination untouched.
 *   subset  device int32 [k] */
int parse_pack_experts(const parse_layer *layer, const int32_t *subset, int32_t k, void *Vt_S,
                       void *Ut_S, parse_stream stream);
/* The same for every pattern of a batch without a host round trip: pattern j < *n_patterns is taken
 * from prompt rep[j]'s subset (subset[rep[j]*subset_stride .. +k)) and written to
 * Vt_S + j*k*gs*n and Ut_S + j*k*gs*m elements; j >= *n_patterns (device value) is skipped.
 * Destinations must hold max_patterns patterns.  rep == NULL means pattern j = row j. */
int parse_pack_patterns(const parse_layer *layer, const int32_t *subset, int32_t subset_stride,
                        int32_t k, const int32_t *rep, const int32_t *n_patterns,
                        int32_t max_patterns, void *Vt_S, void *Ut_S, parse_stream stream);

/* Aggregation keyed by pattern-cache entry (the aggregated copy of a pattern is made once, when the pattern
 * enters the cache, and reused by every later hit and every decode step): for each of the P prompts of a
 * parse_cache_lookup_or_route batch with hit[p] == 0 and 0 <= entry[p] < n_slots, prompt p's subset
 * (subset[p*subset_stride .. +k)) is packed into slot entry[p] of Vt_S [n_slots][k*gs][n] and
 * Ut_S [n_slots][k*gs][m].  Hits and misses that found the cache full (entry -1) are skipped; the forward
 * call then takes pattern_id = entry.  entry device int32 [P], hit device uint8 [P]. */
int parse_pack_new_entries(const parse_layer *layer, const int32_t *subset, int32_t subset_stride,
                           int32_t k, int32_t P, const int32_t *entry, const uint8_t *hit,
                           int32_t n_slots, void *Vt_S, void *Ut_S, parse_stream stream);

/* ---- a6 / a7: the routed product ------------------------------------------------------------
 * Patterns of one call.  All patterns of a layer have the same active rank r_S = k*gs.
 * Shared head (Sec. 4.4): with n_shared > 0 the first n_shared groups of every pattern are the layer's
 * groups 0..n_shared-1; they are stored ONCE (Vt_shared, Ut_shared = parse_pack_experts of the ids
 * 0..n_shared-1) and the per-pattern blocks hold only the other k - n_shared groups (parse_pack_patterns /
 * parse_pack_new_entries on `subset + n_shared` with k - n_shared ids and the full row stride), so a prompt
 * reads two contiguous blocks.  bf16 prefill in the planned and two-launch schedules (a workspace is then required;
 * the head must be whole 32-rank blocks for the planned one; the fused kernel reads one block per pattern and
 * answers PARSE_ELAYOUT); decode reads the layer's own store by group id and ignores these three fields -- there the
 * shared groups are simply groups that every sequence selected: streamed once per step, applied to all. */
typedef struct {
  const void *Vt_S;       /* device, packed [n_patterns][(k-n_shared)*gs][n] in the layer's layout; prefill only */
  const void *Ut_S;       /* device, packed [n_patterns][(k-n_shared)*gs][m];                       prefill only */
  const int32_t *subsets; /* device int32, pattern j's ids at subsets[j*subset_stride .. +k); decode only */
  int32_t subset_stride;
  int32_t n_patterns;     /* capacity of the arrays above; pattern ids outside [0, n_patterns) give zero rows */
  int32_t k;
  const void *Vt_shared;  /* device [n_shared*gs][n], or NULL when n_shared == 0 */
  const void *Ut_shared;  /* device [n_shared*gs][m], or NULL when n_shared == 0 */
  int32_t n_shared;
  int32_t schedule;       /* parse_prefill_schedule for bf16 prefill; 0 = chosen by the library */
} parse_patterns;

/* How the bf16 prefill product of a call is scheduled (field `schedule` of parse_patterns; there is no process-wide
 * setting).  PARSE_SCHED_AUTO: planned when the workspace allows it, else two-launch, else fused.
 * PARSE_SCHED_FUSED: ONE kernel, a workgroup owns 64 token rows and keeps the r_S-wide intermediate in LDS (no
 *   workspace needed; few workgroups on short batches).
 * PARSE_SCHED_TILES: two launches of a tile kernel that takes factor operands straight from memory into registers;
 *   the intermediate goes through the workspace; a tile that spans several prompts is redone per prompt.
 * PARSE_SCHED_PLANNED: a prefill plan (parse_prefill_plan) renumbers the token rows by pattern, then two launches of
 *   an LDS-staged tile kernel over 256- or 128-row tiles that each belong to one pattern.
 * A forced schedule that the shapes or the workspace do not allow gives PARSE_ESHAPE / PARSE_EWORKSPACE. */
typedef enum { PARSE_SCHED_AUTO = 0, PARSE_SCHED_FUSED = 1, PARSE_SCHED_TILES = 2, PARSE_SCHED_PLANNED = 3 } parse_prefill_schedule;

typedef enum { PARSE_PREFILL = 0, PARSE_DECODE = 1 } parse_mode;

/* Workspace of parse_lowrank_forward.  P and n_patterns size the planned prefill schedule (its plan and its padded
 * intermediate); with P == 0 or n_patterns == 0 the answer covers the other schedules only (the forward call then
 * does not use the planned one). */
size_t parse_lowrank_workspace_bytes(int32_t mode, const parse_layer *layer, int32_t rows, int32_t k,
                                     int32_t P, int32_t n_patterns);
/* PARSE_PREFILL  Y[t] = A_S (B_S^T x_t) for every token t of prompt p, S = pattern pattern_id[p]
 *                (Eq. 4 / Eq. 10), read from the packed factors.  bf16 layers must be PARSE_MFMA16:
 *                both products on the bf16 matrix cores with fp32 accumulation, the r_S-wide
 *                intermediate rounded to bf16.  Schedules: see parse_prefill_schedule (patterns->schedule).
 *                With workspace == NULL the fused kernel is used.  The planned schedule builds its plan inside the
 *                call (one extra small launch); parse_lowrank_prefill_planned takes a ready plan instead.  f32
 *                layers must be PARSE_ROWMAJOR (plain fp32 kernels, intermediate in the workspace).
 *                  X device [rows][n], Y device [rows][m] (layer dtype), tok_offsets device int32 [P+1],
 *                  pattern_id device int32 [P].
 * PARSE_DECODE   one token per sequence (rows == P, tok_offsets ignored, may be NULL), bf16 PARSE_MFMA16
 *                layers only.  Sequences are taken in panels of 32 (the N side of the matrix instruction): rows > 32
 *                costs one pass over the selected groups per panel, and a group is streamed for a panel only if one
 *                of that panel's sequences selected it.  Per panel: streams every group that some sequence selected exactly
 *                once from the layer's own store (layer->Vt / layer->Ut, not the packed copies) and applies
 *                it to the sequences whose pattern holds it (Sec. 4.3, rank reuse: pattern_id is fixed
 *                at prefill).  Bandwidth-bound.  A panel of one to four sequences is computed on the vector
 *                units with a finer split of the work (same rounding points: z and y to bf16, fp32 sums); a
 *                sequence's result may therefore differ in rounding between a small and a large panel.
 * workspace: device, >= parse_lowrank_workspace_bytes(mode, layer, rows, k, P, n_patterns) bytes (optional for
 *            bf16 prefill). */
int parse_lowrank_forward(int32_t mode, const parse_layer *layer, const parse_patterns *patterns,
                          const void *X, int32_t rows, const int32_t *tok_offsets,
                          const int32_t *pattern_id, int32_t P, void *Y, void *workspace,
                          size_t workspace_bytes, parse_stream stream);

/* ---- prefill plan (Sec. 4.3: prompts that share a pattern are executed together) -----------------------------
 * Renumbers the token rows of a batch so that the rows of one pattern are consecutive (prompts in arrival order)
 * and every pattern starts on a 256-row boundary; a tile of such "virtual rows" belongs to one pattern whatever the
 * prompt lengths are.  The plan depends only on (tok_offsets, pattern_id): one plan serves every layer of the batch.
 *   tok_offsets device int32 [P+1], ascending, tok_offsets[0] = 0, tok_offsets[P] = rows (rows outside every prompt
 *               are in no tile: their output rows are not written)
 *   pattern_id  device int32 [P]; ids outside [0, n_patterns) mark prompts whose output rows become zero
 *   plan        device, >= parse_prefill_plan_bytes(rows, P, n_patterns) bytes, 16-byte aligned, caller-owned.
 *               int32 words: [0] virtual tiles of 256 rows, [1] virtual rows, [2] 256, [3] capacity in tiles,
 *               [16 ..) pattern of each tile (-1 = zero rows), then (from word 16 + capacity rounded up to 16)
 *               the actual row of each virtual row, -1 for padding.
 * 1 <= P <= 2048, n_patterns <= 2048.  Only enqueues. */
size_t parse_prefill_plan_bytes(int32_t rows, int32_t P, int32_t n_patterns);
int parse_prefill_plan(const int32_t *tok_offsets, const int32_t *pattern_id, int32_t P, int32_t rows,
                       int32_t n_patterns, void *plan, size_t plan_bytes, parse_stream stream);
/* parse_bucket_patterns and parse_prefill_plan of the same batch in ONE launch (Sec. 4.3: both group the prompts of a
 * batch by pattern, from the same probe results, and neither needs the other's output).  The first nine arguments are
 * parse_bucket_patterns' (pattern_id_out .. rep are its outputs), the rest parse_prefill_plan's (plan_pattern_id is the
 * id the plan groups by, e.g. the cache entry of each prompt); every output equals the separate calls', and so do the
 * limits and the errors.  P <= 256 takes one launch, a larger batch the two launches of the separate calls.  Only
 * enqueues. */
int parse_bucket_and_plan(const int32_t *subset, int32_t P, int32_t k, int32_t subset_stride, int32_t *pattern_id_out,
                          int32_t *perm, int32_t *bucket_off, int32_t *n_patterns_out, int32_t *rep,
                          const int32_t *tok_offsets, const int32_t *plan_pattern_id, int32_t rows, int32_t n_patterns,
                          void *plan, size_t plan_bytes, parse_stream stream);
/* The bf16 prefill product (Eq. 10) of one layer over a ready plan: two launches, no prompt-dependent work on the
 * host.  layer bf16 PARSE_MFMA16 with n % 64 == 0; patterns as for PARSE_PREFILL (a shared head must be whole 32-rank
 * blocks); the plan must
 * have been built from the same tok_offsets, pattern_id, rows, P and patterns->n_patterns (the two arrays are checked
 * for presence only: everything the kernels need from them is in the plan).
 *   workspace  device, >= parse_lowrank_prefill_planned_workspace_bytes(layer, rows, P, k, n_patterns): the
 *              intermediate of the padded virtual rows, in operand order; for batches of at most 1024 token rows
 *              (n >= 1024) also the fp32 partial sums of the first product, whose reduction over n is then cut in
 *              2..8 slices (one more small launch adds them in slice order; the count depends on rows and n only,
 *              so fused and single-layer calls agree bit for bit). */
size_t parse_lowrank_prefill_planned_workspace_bytes(const parse_layer *layer, int32_t rows, int32_t P, int32_t k,
                                                     int32_t n_patterns);
int parse_lowrank_prefill_planned(const parse_layer *layer, const parse_patterns *patterns, const void *X,
                                  int32_t rows, const int32_t *tok_offsets, const int32_t *pattern_id, int32_t P,
                                  const void *plan, void *Y, void *workspace, size_t workspace_bytes,
                                  parse_stream stream);

/* ---- rank-granular routing (Sec. 4.1, Eq. 4-5 as written: one expert per rank component) ----------------
 * The router maps the prompt embedding to one score per rank, R^d -> R^G with G = the stored rank (up to 8192),
 * and the K best ranks are active.  parse_route_ranks = pool -> scores = Wr e -> exact top-K (ties to the lower
 * rank id), ids ascending in subset_out[p][0..K).  Arguments as parse_route, with
 *   Wr device float [G][d];  1 <= K <= G <= 8192;  scores_out device float [P][G] or NULL (16-byte aligned);
 *   workspace >= parse_route_ranks_workspace_bytes(rows, P, d, G).
 * parse_pack_ranks = the memory aggregation of Sec. 4.4 for single ranks: the K selected rank rows of a
 * ROW-MAJOR bf16 layer are gathered into one contiguous block per pattern, written directly in PARSE_MFMA16
 * operand order (K % 32 == 0, n % 16 == 0, m % 32 == 0):
 *   subset device int32 [n_patterns][subset_stride] (K ids per row; ids outside [0, R) give zero rows),
 *   Vt_S device [n_patterns][K][n], Ut_S device [n_patterns][K][m].
 * The packed blocks feed parse_lowrank_forward(PARSE_PREFILL) unchanged: describe the layer to it with
 * PARSE_MFMA16 layout and G = R/32 (32-rank units) and the patterns with k = K/32. */
size_t parse_route_ranks_workspace_bytes(int32_t rows, int32_t P, int32_t d, int32_t G);
int parse_route_ranks(const void *X, int32_t xdtype, int32_t rows, const int32_t *tok_offsets, int32_t P,
                      int32_t d, const float *Wr, int32_t G, int32_t K, int32_t *subset_out,
                      int32_t subset_stride, float *scores_out, float *emb_out, void *workspace,
                      size_t workspace_bytes, parse_stream stream);
int parse_pack_ranks(const parse_layer *layer, const int32_t *subset, int32_t subset_stride, int32_t K,
                     int32_t n_patterns, void *Vt_S, void *Ut_S, parse_stream stream);

/* ---- router training step (Sec. 4.2, Eq. 6-9) ---------------------------------------------------------------
 * The factors stay fixed; the router matrix Wr is trained against the dense model's output.  For one batch:
 *   loss_p   = sum over prompt p's tokens of || y_hat - y_dense ||^2                         (Eq. 6)
 *   y_hat    = the routed output with the hard top-k mask (parse_lowrank_forward)              (Eq. 7)
 *   backward = straight-through: the mask's derivative is that of the K-normalised sigmoid mask
 *              m_g = k sigmoid(s_g / temperature) / (sum_j sigmoid(s_j / temperature) + eps)    (Eq. 8-9)
 *   grad_Wr[j][:] = sum_p dL/ds_j(p) e_p,  s = Wr e_p (groups as experts, one embedding per prompt).
 * layer          bf16 PARSE_MFMA16, n % 128 == 0, m % 128 == 0, G <= 64, P*G <= 8192
 * Ut_rankmajor   device: the layer's Ut ([R][m] row-major) reordered like a RIGHT factor, i.e. the Vt output of
 *                parse_layer_to_mfma16 for a row-major layer whose Vt is that Ut and whose n is m
 * X [rows][n], Y_hat, Y_dense [rows][m]  device bf16;  tok_offsets device int32 [P+1]
 * emb [P][d], scores [P][G]             device float, as written by parse_route (emb_out, scores_out)
 * loss_out       device float [P] or NULL;  grad_Wr device float [G][d] (overwritten)
 * workspace      device, >= parse_router_grad_workspace_bytes(layer, rows, P) */
size_t parse_router_grad_workspace_bytes(const parse_layer *layer, int32_t rows, int32_t P);
int parse_router_grad(const parse_layer *layer, const void *Ut_rankmajor, const void *X, int32_t rows,
                      const int32_t *tok_offsets, int32_t P, const void *Y_hat, const void *Y_dense,
                      const float *emb, const float *scores, int32_t d, int32_t k, float temperature,
                      float eps, float *loss_out, float *grad_Wr, void *workspace, size_t workspace_bytes,
                      parse_stream stream);

/* Horizontal fusion for decode (Sec. 4.4, Eq. 11-12: projections that share their input run as one stacked
 * first product and one batched second product).  n_layers (1..4) layers that read the SAME token rows X
 * (equal n; m, R, G and the patterns may differ per layer) take ONE decode step together: the result equals
 * n_layers separate PARSE_DECODE calls, at the launch count of one.
 *   layers, patterns  host arrays [n_layers]; layer l uses patterns[l] (its own subsets, k, n_patterns)
 *   X                 device [rows][n] bf16, one token per sequence (panels of 32 as for PARSE_DECODE)
 *   pattern_id        device int32 [rows], shared by all layers (a sequence's cache entry)
 *   Y                 host array [n_layers] of device pointers, Y[l] = [rows][layers[l].m] bf16
 *   workspace         device, >= parse_lowrank_decode_multi_workspace_bytes(layers, n_layers), caller-owned
 * Errors as parse_lowrank_forward; nothing is launched on error.  Same inputs, same bits.  (A result may differ in
 * rounding from the single-layer call's: the reduction over n is cut into slices by the size of the whole call.) */
size_t parse_lowrank_decode_multi_workspace_bytes(const parse_layer *layers, int32_t n_layers);
int parse_lowrank_decode_multi(const parse_layer *layers, const parse_patterns *patterns, int32_t n_layers,
                               const void *X, int32_t rows, const int32_t *pattern_id, void *const *Y,
                               void *workspace, size_t workspace_bytes, parse_stream stream);

/* ---- decode plan (Sec. 4.3, rank reuse: the subsets are fixed after prefill) -------------------------------------
 * Everything the decode kernels derive from the subsets -- per layer the sequence mask of every group, the ascending
 * list of groups that at least one sequence selected, their count -- computed ONCE per batch instead of in every step.
 *   layers, patterns  host arrays [n_layers] (1..4 layers that share their input; patterns[l].subsets is used)
 *   pattern_id        device int32 [rows], a sequence's pattern (cache entry); rows <= 32
 *   plan              device, >= parse_decode_plan_bytes(n_layers) bytes, 16-byte aligned, caller-owned
 * parse_lowrank_decode_planned is the decode step of those layers over a ready plan: TWO launches (the intermediate of
 * every used rank block, then the output columns), nothing derived from the subsets at run time.  Results are
 * bit-identical to parse_lowrank_forward(PARSE_DECODE) / parse_lowrank_decode_multi, which build the same plan inside
 * the call (one more small launch), and the same from run to run (no floating-point atomics: partial sums are added in
 * a fixed order).
 * The plan also holds the arrival counters with which the workgroups that share a rank block's reduction find out
 * which of them finishes it (zero after parse_decode_plan and again after every call): the decode call WRITES the
 * plan, so a plan serves one decode call at a time -- calls that share a plan go on one stream or are ordered by the
 * caller; concurrent calls need a plan each.
 *   X device [rows][n] bf16;  Y host array [n_layers] of device pointers [rows][layers[l].m] bf16
 *   workspace device, >= parse_lowrank_decode_planned_workspace_bytes(layers, n_layers) (the intermediates and the
 *             partial sums of the split reduction; contents irrelevant before, undefined after) */
size_t parse_decode_plan_bytes(int32_t n_layers);
int parse_decode_plan(const parse_layer *layers, const parse_patterns *patterns, int32_t n_layers,
                      const int32_t *pattern_id, int32_t rows, void *plan, size_t plan_bytes, parse_stream stream);
size_t parse_lowrank_decode_planned_workspace_bytes(const parse_layer *layers, int32_t n_layers);
int parse_lowrank_decode_planned(const parse_layer *layers, int32_t n_layers, const void *X, int32_t rows,
                                 void *plan, void *const *Y, void *workspace, size_t workspace_bytes,
                                 parse_stream stream);

/* ---- decode without allocation ---------------------------------------------------------------------------
 * For callers that cannot allocate device memory: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  The same step as parse_lowrank_forward(PARSE_DECODE, ...) -- same kernels, same bits --
 * but the memory the kernels need beyond inputs and outputs (the rounded intermediate in operand order, the partial
 * sums of its split reduction and the decode plan: group masks, list of used groups, arrival counters) is a fixed
 * array of PARSE_DECODE_STATIC_SCRATCH_BYTES inside the library's
 * device image instead of a caller's workspace.  The call allocates and frees nothing, on any call, and calls no
 * allocating routine; every GPU the library runs on holds its own copy of the array until the process ends.
 *   layer, patterns, X, rows, pattern_id, Y   as for PARSE_DECODE (device pointers, rows <= 32, bf16 PARSE_MFMA16)
 * PARSE_EWORKSPACE when the layer needs more than the array holds: parse_lowrank_workspace_bytes(PARSE_DECODE, layer,
 * rows, k, 0, 0) is what it needs (64 bytes per stored rank, 128 more per stored rank and slice when the reduction
 * over n is split in slices, about 2 KiB of plan: 2.1 MiB for R = 2560, n = 11008); other errors as
 * parse_lowrank_forward.  Nothing is launched on error.
 * All calls on one GPU share that GPU's array: calls that overlap on one GPU (two streams, two threads) race;
 * issue them on one stream or order them.  The array keeps the last call's contents; the kernels read only what
 * the same call wrote, so nothing needs clearing between calls. */
#define PARSE_DECODE_STATIC_SCRATCH_BYTES (4u << 20)
size_t parse_lowrank_decode_static_capacity(void);
int parse_lowrank_decode_static(const parse_layer *layer, const parse_patterns *patterns, const void *X,
                                int32_t rows, const int32_t *pattern_id, void *Y, parse_stream stream);

/* Horizontal fusion for prefill (Sec. 4.4, Eq. 11-12): n_layers (1..4) bf16 PARSE_MFMA16 layers that read the
 * SAME token rows X (equal n) in two launches for all of them -- one stacked first product over the selected
 * ranks of every layer, one batched second product.  patterns[0].schedule chooses for the call:
 *   PARSE_SCHED_AUTO / PARSE_SCHED_PLANNED  the planned tile kernels over one prefill plan built inside the call (one
 *     more small launch; every layer needs the same n_patterns, n % 64 == 0, k*gs % 32 == 0, m % 32 == 0); AUTO falls
 *     back to the two-launch schedule when the shapes or the workspace do not allow it;
 *   PARSE_SCHED_TILES  the two-launch tile kernels on prompt-order tiles (n and k*gs multiples of 128);
 *   PARSE_SCHED_FUSED  PARSE_EINVAL (the single-launch kernel takes one layer).
 * The result equals n_layers separate PARSE_PREFILL calls under the same schedule, bit for bit.
 *   layers, patterns  host arrays [n_layers]; patterns[l] holds layer l's packed factors (Vt_S, Ut_S, k; shared head
 *                     allowed)
 *   X                 device [rows][n] bf16; tok_offsets device int32 [P+1]; pattern_id device int32 [P]
 *   Y                 host array [n_layers] of device pointers, Y[l] = [rows][layers[l].m] bf16
 *   workspace         device, >= parse_lowrank_prefill_multi_workspace_bytes(...) (the intermediates and, for the
 *                     planned schedule, the plan: sized for any number of prompts up to 2048), required
 * PARSE_ESHAPE when no schedule takes the shapes (use separate calls then). */
size_t parse_lowrank_prefill_multi_workspace_bytes(const parse_layer *layers, const parse_patterns *patterns,
                                                   int32_t n_layers, int32_t rows);
int parse_lowrank_prefill_multi(const parse_layer *layers, const parse_patterns *patterns, int32_t n_layers,
                                const void *X, int32_t rows, const int32_t *tok_offsets,
                                const int32_t *pattern_id, int32_t P, void *const *Y, void *workspace,
                                size_t workspace_bytes, parse_stream stream);

/* ---- achievable-peak probes (measurement only) ---------------------------------------------------------------
 * Kernels with nothing but the resource a roofline prices: the caller times them with HIP events on its stream and
 * reports the rates beside the nominal peaks (MI355X: 2.5 PFLOP/s dense bf16, 8 TB/s HBM).  They only enqueue.
 * parse_probe_mfma_bf16  register-resident loop of 32x32x16 bf16 matrix instructions: `workgroups` x 4 wavefronts x
 *                        `iters` x 8 instructions of 32768 flop each, operands taken once from `data` (device, >= 24 KiB,
 *                        the caller chooses the values: the rate depends on them); out: device float [workgroups*256].
 * parse_probe_read       read-only stream of `bytes` from src (device) by `workgroups` workgroups, contiguous shares;
 *                        bytes must be a multiple of workgroups * 64 KiB; sink: device uint32 [1] or NULL.
 * parse_probe_copy       dst[i] = src[i], 16 bytes per lane; bytes % 16 == 0. */
int parse_probe_mfma_bf16(const void *data, int32_t workgroups, int32_t iters, float *out, parse_stream stream);
int parse_probe_read(const void *src, size_t bytes, int32_t workgroups, void *sink, parse_stream stream);
int parse_probe_copy(const void *src, void *dst, size_t bytes, parse_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* PARSE_H_ */
