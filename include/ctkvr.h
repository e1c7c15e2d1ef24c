/*
 * ctkvr.h -- C ABI of the MI355X (gfx950) implementation of CTkvr's data-parallel
 * hot path: the query-centroid inverted file built at prefill (Algorithm 1,
 * lines 1-4 of the paper) and the per-decode-step centroid-then-token retrieval
 * followed by sparse attention (Algorithm 2, lines 1-9).
 *
 * Notation (the paper's): b batch, h query heads, g KV heads, G = h/g, d head
 * dimension, s context length, C query centroids per head, C' probed centroids
 * (n_probe), rho keys per inverted list (list_len), rho' sparsity budget (top_k).
 * Query heads i*G .. (i+1)*G-1 share KV head i (Section 3.1.1, footnote on
 * grouped-query attention).
 *
 * Conventions
 *   - Every tensor pointer is a DEVICE pointer owned by the caller unless the
 *     comment says HOST.  The library never frees caller memory and keeps no
 *     reference to it after a call returns, except where stated.
 *   - Work is enqueued on the HIP stream passed as `hip_stream` (a hipStream_t
 *     cast to void*; NULL = the default stream).  ctkvr_decode_step does not
 *     synchronise and does not allocate.
 *   - Functions return CTKVR_OK (0) or a negative ctkvr_status; nothing is thrown
 *     across the boundary.  ctkvr_last_error() gives a thread-local message for
 *     the last non-OK return.  Argument errors are detected on the host before
 *     anything is launched.
 *   - The KV cache is paged: k_pages / v_pages are
 *     [num_pages][g][page_size][d] elements of `dtype`; token t of sequence i
 *     lives in page block_table[i*max_pages + t/page_size], slot t%page_size.
 *   - head_dim must be 128 and G one of 1, 2, 4, 8, else CTKVR_EUNSUPPORTED.
 *   - Selections break ties towards the lowest id and are reported in ascending
 *     id order.
 */
#ifndef CTKVR_H
#define CTKVR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ctkvr_index ctkvr_index;   /* opaque: centroids, their inverse norms, inverted lists, workspace */

typedef enum {
    CTKVR_OK = 0,
    CTKVR_EINVAL = -1,        /* bad argument (null pointer, C' > C, rho > s, h % g != 0, ...) */
    CTKVR_ENOMEM = -2,        /* device or host allocation failed */
    CTKVR_EHIP = -3,          /* a HIP runtime call failed */
    CTKVR_EUNSUPPORTED = -4   /* valid in the paper, not supported by this build (head_dim != 128, ...) */
} ctkvr_status;

typedef enum { CTKVR_F32 = 0, CTKVR_BF16 = 1 } ctkvr_dtype;

typedef enum {
    CTKVR_CENTROID_LAST_C = 0,   /* Algorithm 1 line 1: the last C prompt queries */
    CTKVR_CENTROID_KMEANS = 1    /* Lloyd iterations over the prompt queries replace line 1 only */
} ctkvr_centroid_mode;

typedef enum {
    CTKVR_BUILD_EXACT = 0,   /* list scores in the fixed fp32 arithmetic of the decode path (bit-reproducible) */
    CTKVR_BUILD_MFMA = 1     /* list scores on the matrix cores (bf16 inputs only); lists may differ from
                                EXACT only for keys whose score ties the rho-th within rounding */
} ctkvr_build_algo;

typedef struct {
    int32_t batch;           /* b */
    int32_t n_q_heads;       /* h */
    int32_t n_kv_heads;      /* g */
    int32_t head_dim;        /* d, must be 128 */
    int32_t page_size;       /* tokens per KV page (16 in the benchmark workloads) */
    int32_t dtype;           /* ctkvr_dtype of q, K, V and the centroid table */
    int32_t n_centroids;     /* C; 0 => per sequence C_i = ctx_len_i / centroid_div */
    int32_t centroid_div;    /* used when n_centroids == 0 */
    int32_t list_len;        /* rho  (Algorithm 1 line 4) */
    int32_t n_probe;         /* C'   (Algorithm 2 line 3) */
    int32_t top_k;           /* rho' (Algorithm 2 line 6) */
    float   sm_scale;        /* softmax scale applied to q.k; 0 => 1/sqrt(head_dim) */
    int32_t centroid_mode;   /* ctkvr_centroid_mode */
    int32_t kmeans_iters;    /* Lloyd iterations when centroid_mode == KMEANS */
    int32_t build_algo;      /* ctkvr_build_algo */
    int32_t n_init;          /* L_init: the first n_init keys stay with the attention (Algorithm 1 lines 5-6) */
    int32_t n_local;         /* L_local: so do the last n_local keys of the prompt; neither enters a list */
} ctkvr_params;

/*
 * Index construction at prefill (Algorithm 1, lines 1-4).
 *   q_prefill   post-RoPE prompt queries, [total_rows][h][d] of `dtype`, sequences
 *               concatenated; cu_seqlens (HOST, batch+1 entries) gives each
 *               sequence's row range.  With q_is_tail = 1 a sequence contributes
 *               only the queries of its last C_i prompt positions (all LAST_C needs);
 *               with q_is_tail = 0 it contributes all ctx_len_i of them.
 *   k_pages, block_table, max_pages   the paged key cache (see above).
 *   ctx_lens    HOST, [batch]: s of every sequence.  The index is built over keys
 *               0 .. s-1 and stays valid for decode steps over that frozen prefix.
 *   init_pos    KMEANS only, DEVICE int32 [batch][g][C]: prompt positions whose
 *               queries seed the centres (e.g. from k-means++ run by the caller).
 * For every sequence, KV head and centroid j the list holds the rho keys with the
 * largest max over the group's query heads of softmax_t(c_{h,j} . k_t * sm_scale)
 * taken over all s keys (lines 2-4), ascending; with n_init, n_local > 0 the rho keys are
 * chosen among keys n_init .. s - n_local - 1 only (the scores are unchanged).
 * On success *out_index owns device memory until ctkvr_free.  The call
 * synchronises the stream before returning.
 * Errors: EINVAL for null/inconsistent arguments (C_i < n_probe, rho > s_i - n_init - n_local, ...);
 * EUNSUPPORTED for head_dim != 128, G not in {1,2,4,8}, MFMA build with f32 data.
 */
int ctkvr_build_index(const ctkvr_params *p, const void *q_prefill, const int32_t *cu_seqlens, int32_t q_is_tail,
                      const void *k_pages, const int32_t *block_table, int32_t max_pages, const int32_t *ctx_lens,
                      const int32_t *init_pos, void *hip_stream, ctkvr_index **out_index);

/*
 * Wrap an index built elsewhere (Algorithm 1's outputs) so that decode steps can
 * run on it.  All pointers HOST: centroids [batch][h][C_max][d] of `dtype`
 * (C_max = max_i C_i; rows j >= C_i unused), lists int32 [batch][g][C_max][rho]
 * ascending key ids, ctx_lens [batch].  The data is copied; inverse centroid
 * norms are recomputed on the device.
 */
int ctkvr_index_load(const ctkvr_params *p, const int32_t *ctx_lens, const void *centroids, const int32_t *lists,
                     void *hip_stream, ctkvr_index **out_index);

/*
 * One decode step of retrieval + sparse attention for every sequence of the
 * batch (Algorithm 2, lines 1-9):
 *   lines 1-3  cosine of q_h to every centroid of head h, max over the group,
 *              top-C' centroids per KV head;
 *   line  4    union of their lists, deduplicated -> L recalled key ids;
 *   lines 5-6  max over the group of softmax(q . K^Recall * sm_scale) over the
 *              recalled keys, top-rho' key ids;
 *   lines 7-9  softmax(q . K^sparse * sm_scale) V^sparse per query head.
 *   q          [batch][h][d] post-RoPE, `dtype`.
 *   out        fp32 [batch][h][d].
 * Optional outputs (NULL to skip):
 *   out_lse    fp32 [batch][h]: natural-log sum of exp of the scaled logits over
 *              the selected keys (lets a caller merge a resident window later);
 *   out_sel    int32 [batch][g][rho'] selected key ids ascending, -1 padded when L < rho';
 *   out_ncand  int32 [batch][g]: L;
 *   out_probe  int32 [batch][g][C'] probed centroid ids ascending.
 * The KV cache must hold the same first ctx_len_i keys the index was built on.
 * Asynchronous on hip_stream; uses the index's workspace, so steps on one index
 * must not overlap.  Errors: EINVAL (null required pointer, max_pages too small).
 */
int ctkvr_decode_step(ctkvr_index *idx, const void *q, const void *k_pages, const void *v_pages,
                      const int32_t *block_table, int32_t max_pages, float *out, float *out_lse, int32_t *out_sel,
                      int32_t *out_ncand, int32_t *out_probe, void *hip_stream);

/*
 * The decode step with the resident window (Algorithm 2 lines 1-11; Section 3.2): as
 * ctkvr_decode_step, and in addition every query head attends over the first n_init keys and
 * over the keys from ctx_len_i - n_local to cur_lens[i] - 1, and the two attention outputs are
 * merged through their log-sum-exps (line 11), which equals attention over the union.
 *   cur_lens   DEVICE int32 [batch] or NULL: tokens of each sequence now in the KV cache,
 *              cur_lens[i] >= ctx_len_i.  The tokens decoded since the index was built belong
 *              to the local window; the caller appends their keys and values to the paged cache.
 *              NULL means cur_lens[i] = ctx_len_i.  Values are clamped to
 *              [ctx_len_i, max_pages * page_size].
 * The lists of an index built with n_init, n_local > 0 hold no window key, so nothing is
 * counted twice.  out_lse is the log-sum-exp over selected and window keys together.
 * ctkvr_decode_step on such an index is this call with cur_lens = NULL.
 * Errors: as ctkvr_decode_step.
 */
int ctkvr_decode_step_window(ctkvr_index *idx, const void *q, const void *k_pages, const void *v_pages,
                             const int32_t *block_table, int32_t max_pages, const int32_t *cur_lens, float *out,
                             float *out_lse, int32_t *out_sel, int32_t *out_ncand, int32_t *out_probe, void *hip_stream);

/*
 * ctkvr_decode_step for callers that cannot allocate device memory or tolerate a call that
 * does (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * the same step with the same arguments, results and errors, but every intermediate buffer of
 * the step (cosines, recall bitmap, recalled ids and rows, logits, ranking keys and their
 * histogram, the selection's bitmap and list, the selected rows and logits) lives in a static
 * device array of the library, 32 MiB per GPU, instead of the workspace `idx` owns.  The call
 * allocates and frees nothing, on the host side of HIP or through it; the array's device
 * address is looked up on the first call on each device.
 *   - The step's buffers must fit: about
 *       units * (l_stride * (16 + 4 G) + 4 C_max + s_max / 8 + top_k * (8 + 4 G) + 30 KiB)
 *     bytes, units = batch * g, plus, on geometries that allow the single-launch form (units at most
 *     the number of compute units), units * 32 * (4 top_k + 21 KiB) for its per-block slots (the 32K
 *     benchmark workload takes about 15 MiB).  Larger geometries return CTKVR_EUNSUPPORTED before
 *     anything is launched.
 *   - Every call on a GPU shares that GPU's array, whichever index it serves: calls that
 *     overlap on one GPU (different streams, different threads) race.  The call clears what a
 *     step expects to find zero, so it may follow a call for any other index.
 *   - ctkvr_centroid_update and ctkvr_index_last_candidates read the workspace `idx` owns: they
 *     follow ctkvr_decode_step, not this call.
 */
int ctkvr_decode_step_static(ctkvr_index *idx, const void *q, const void *k_pages, const void *v_pages,
                             const int32_t *block_table, int32_t max_pages, float *out, float *out_lse, int32_t *out_sel,
                             int32_t *out_ncand, int32_t *out_probe, void *hip_stream);

/*
 * Dynamic centroid update (Algorithm 2 line 12; Section 3.1.2, "Dynamic Centroid Update"),
 * to be called after ctkvr_decode_step with the same q, on the same stream, before the next
 * step: for every sequence and KV head the query vectors of the group's heads replace the
 * centroids of one slot of the index, and that slot's list becomes the rho keys with the
 * largest rerank score of the step (the quantity line 6 ranks by, over the recalled keys),
 * ties to the lowest id, ascending.  Slots are taken first in, first out: update number n
 * (counted from 0 since the build) writes slot n mod C_i, so the earliest prompt query goes
 * first.  With rho = rho' the list is the step's selection; otherwise the ranking is run
 * once more with budget rho.  Should fewer than rho keys have been recalled the last one is
 * repeated.  Asynchronous, allocates nothing, uses the index's workspace like a step.
 * Errors: EINVAL (null pointer; no decode step since the build or the last update).
 */
int ctkvr_centroid_update(ctkvr_index *idx, const void *q, void *hip_stream);

/* Release an index (NULL is allowed).  Synchronises the device first. */
void ctkvr_free(ctkvr_index *idx);

/* Thread-local description of the last non-OK return of this library. */
const char *ctkvr_last_error(void);

/* ---- inspection (tests, tooling); each synchronises ----------------------- */
typedef struct {
    int32_t batch, n_q_heads, n_kv_heads, head_dim, dtype;
    int32_t c_max;           /* centroid rows allocated per head */
    int32_t list_len, n_probe, top_k;
    int32_t l_stride;        /* candidate slots per (sequence, KV head): max_i min(s_i, C' * rho) */
    int64_t index_bytes;     /* bytes of the inverted lists: b * g * C_max * rho * 4 */
    int64_t device_bytes;    /* everything the index holds on the device */
} ctkvr_index_info_t;

int ctkvr_index_info(const ctkvr_index *idx, ctkvr_index_info_t *out);
/* Copy out the inverted lists, int32 [batch][g][C_max][rho], to HOST memory. */
int ctkvr_index_lists(const ctkvr_index *idx, int32_t *dst_host);
/* Copy out the centroid table, [batch][h][C_max][d] of `dtype`, to HOST memory. */
int ctkvr_index_centroids(const ctkvr_index *idx, void *dst_host);
/* Recalled key ids of the last decode step, int32 [batch][g][l_stride] (first L valid), to HOST memory. */
int ctkvr_index_last_candidates(const ctkvr_index *idx, int32_t *dst_host);

/* ---- per-kernel timing (measurement aid) ----------------------------------- */
/* The decode step runs these kernels in order: 0 centroid cosine, 1 probe select + list
 * gather into a bitmap, 2 bitmap expansion into the recalled id list fused with key scoring,
 * 3 softmax denominators, 4 ranking keys + their histogram, 5 chip-wide pass over the
 * ranking keys (bitmap + deciding bucket's list), 6 rerank select, 7 sparse attention.  For
 * small batches 6 and 7 are one launch, timed as stage 7 (stage 6 then reads as the cost of
 * an event pair).  While timing is enabled a ninth, empty kernel follows (stage 8): its
 * figure is what a pair of events costs around a kernel that does nothing. */
#define CTKVR_N_STAGES 9
/* After this call every decode step on `idx` records a HIP event before its first
 * kernel and after each kernel, for up to max_steps steps (0 disables and frees
 * the events).  Recording adds work to the stream: use it for the breakdown, not
 * for the headline step time. */
int ctkvr_profile_enable(ctkvr_index *idx, int32_t max_steps);
/* Synchronises, writes ms_host[step][stage] (fp32, CTKVR_N_STAGES per step) for
 * the steps recorded since the last collect (at most capacity_steps), stores
 * their number in *n_steps and restarts recording at step 0. */
int ctkvr_profile_collect(ctkvr_index *idx, float *ms_host, int32_t capacity_steps, int32_t *n_steps);

/* ---- environment variables ------------------------------------------------------------- */
/* Read when an index is created (ctkvr_build_index, ctkvr_index_load); none changes a result, all
 * exist so that each form of a launch can be measured and tested against the other:
 *   CTKVR_DECODE_PATH        = staged | fused | auto   default of ctkvr_index_set_decode_path
 *   CTKVR_DECODE_GROUPS      = n   sequences stepped as n forked groups (default 1)
 *   CTKVR_XCD_UNITS          = 0|1 the blocks of a (sequence, KV head) unit spread over the XCDs / all on one XCD in
 *                                  every kernel of a step (needs a multiple of 8 units; default: one XCD, except, for
 *                                  large batches, in the two bandwidth-bound launches)
 *   CTKVR_SCORE_BY_RANK      = 0|1 recalled ids split over a unit's blocks by id range / by rank
 *                                  (default: by rank for small batches)
 *   CTKVR_KEYCLASS           = 0|1 ranking-key histogram and classification as two launches / one
 *                                  (default: one for small batches)
 *   CTKVR_FUSED_THREADS      = 256|1024  block size of the single-launch step
 *   CTKVR_BUILD_CANDIDATES   = 0|1 see ctkvr_index_build_route
 *   CTKVR_BUILD_CANDIDATES_REDO    (set: the candidate route also hands every chunk back; tests)
 *   CTKVR_BUILD_SCRATCH_CACHE = 0|1 see ctkvr_release_scratch (read at every build) */

/* ---- how the matrix-core list build chose a unit's top-rho (Algorithm 1 line 4) ---------- */
/* CTKVR_BUILD_MFMA ranks either all s keys of a (KV head, centroid) unit (their 4-byte ranking keys
 * written once, read for a histogram and read again for the selection) or only the keys at or above
 * a per-unit threshold taken from a 1-in-16 sample of the positions (a few thousand candidates per
 * unit; taken when every sequence is at least 32 rho long, rho is 256..2730 and the selection's
 * shared memory holds a bitmap of the context, i.e. up to about 2^19 tokens).  The second route
 * yields exactly the same lists: a chunk of units in which a unit ends with fewer than rho
 * candidates, more than fit, or hundreds of candidates exactly equal to its rho-th key, is redone
 * by the first route.
 * by_candidates_host: 1 if the index was built by the candidate route; chunks_redone_host: how many
 * chunks it handed back.  Both HOST, either may be NULL.  The environment variable
 * CTKVR_BUILD_CANDIDATES = 0 | 1, read at build time, forces the choice where the geometry allows it. */
int ctkvr_index_build_route(const ctkvr_index *idx, int32_t *by_candidates_host, int32_t *chunks_redone_host);

/* ---- scratch kept between index builds (Algorithm 1 runs once per prompt) ----------------- */
/* The candidate route of CTKVR_BUILD_MFMA keeps its device scratch (about 1.1 GB for a 128K context,
 * 32/8 heads, C = rho = 2048; never more than 2 GiB -- a build that needs more, or that finds the
 * scratch in use by a build on another host thread, allocates and frees its own) in one allocation per
 * device until this call, so that the next build neither allocates nor frees (0.75 ms of an 8 ms build).
 * Frees the current device's scratch; an error if a build is using it.  The environment variable
 * CTKVR_BUILD_SCRATCH_CACHE = 0, read at build time, switches the keeping off. */
int ctkvr_release_scratch(void);

/* ---- how a decode step is launched ----------------------------------------- */
/* Algorithm 2 lines 1-9 run either as a sequence of launches (one per stage; any geometry) or as
 * ONE launch whose blocks walk the stages together, a fixed group of co-resident blocks per
 * (sequence, KV head) separated by barriers in device memory (batch * g at most the number of
 * compute units, and a shared-memory plan that fits).  Both give the same integers bit for bit;
 * outputs agree within rounding.  AUTO takes the staged launches, which measure faster on every
 * benchmark geometry of this part (an empty launch behind another costs 1.6 us in a graph, a
 * barrier among 32 blocks with what it has to wait for 1.5-2.5 us); FUSED is there to be measured.
 * The single launch needs all its blocks resident at once: two such steps (two indexes, two
 * streams) must not run on one GPU at the same time -- their waits are bounded, and an expired
 * wait is reported by ctkvr_index_check.  The environment variable CTKVR_DECODE_PATH = staged |
 * fused | auto sets the default of indexes created afterwards. */
typedef enum { CTKVR_PATH_AUTO = 0, CTKVR_PATH_STAGED = 1, CTKVR_PATH_FUSED = 2 } ctkvr_decode_path;
/* Errors: EINVAL (unknown path), EUNSUPPORTED (FUSED on a geometry that does not allow it). */
int ctkvr_index_set_decode_path(ctkvr_index *idx, int32_t path);
/* The path the next step will take: CTKVR_PATH_STAGED or CTKVR_PATH_FUSED (negative: error). */
int ctkvr_index_decode_path(const ctkvr_index *idx);
/* Synchronises the device and reports whether any single-launch step on `idx` gave up a wait
 * (CTKVR_EHIP; the index must then be freed) -- CTKVR_OK otherwise. */
int ctkvr_index_check(ctkvr_index *idx);
/* Measurement aid for the single launch: with enable != 0 the first block of the first unit
 * stamps the 100 MHz wall clock at kernel entry and after each of its phases (entries 0-7: when it
 * leaves the phase's barrier), when its own work of each phase is done (entries 8-13: when it
 * arrives at the barrier) and at points inside the phases (entries 16 and up; 0 = not stamped); the
 * call synchronises and copies the 64 entries of the last step to ticks_host (HOST, 64 values, may
 * be NULL). */
int ctkvr_profile_phases(ctkvr_index *idx, int32_t enable, long long *ticks_host);

/* Measurement aid: what a launch costs when the kernel does nothing.  Captures n_launches empty
 * kernels, one behind the other, in a HIP graph on a stream of its own, replays it once untimed and
 * once between two events, and stores the microseconds per launch in *us_per_launch_host (HOST).
 * Creates and destroys a stream, a graph and two events; synchronises that stream only. */
int ctkvr_measure_dispatch_floor(int32_t n_launches, float *us_per_launch_host, void *hip_stream);

/* Self-check of the fixed-point exponential that the softmax denominators are summed in (the
 * integer S of the score normalisation, Algorithm 1 line 2 and Algorithm 2 line 6): the library
 * holds it in two forms, one written out step by step after its definition and the straight-line
 * one its kernels use, which must agree bit for bit.  Evaluates both on the device for EVERY fp32 value in [-32, 0] (about
 * 1.1e9 inputs, -0 and +0 included), synchronises, and stores the number of inputs on which they
 * differ in *mismatches_host (HOST; 0 is the only acceptable value).  Allocates and frees 8 bytes
 * of device memory.  Returns a status code. */
int ctkvr_selftest_exp(uint64_t *mismatches_host, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CTKVR_H */
