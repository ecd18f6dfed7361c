/*
 * icecache.h - C ABI of the MI355X (gfx950) implementation of the IceCache hot path.
 *
 * One ice_index_t holds one attention layer's clustered, paged KV cache for
 * U = batch * n_kv_heads independent units (one unit = one (sequence, KV head) pair; the
 * paper keeps one index per head, Sec. 4.1).  Keys with similar embeddings share a page
 * (Sec. 4.1); a decode query scores one representative per page, picks the best pages under a
 * token budget (Sec. 4.3-4.4, Alg. 3) and attends only to the tokens in them (Eq. 1).
 *
 * Conventions
 *   Pointers  Every tensor pointer is a DEVICE pointer owned by the caller, 16-byte aligned,
 *             contiguous and row-major as annotated.  bf16 = upper 16 bits of an IEEE fp32.
 *             The only host pointers are ice_config_t*, ice_index_view_t*, ice_index_t** and
 *             the flop count written by ice_debug_peak_mfma.
 *   Memory    The library never allocates device memory.  The caller passes one workspace of
 *             ice_workspace_bytes() bytes (256-byte aligned) to ice_create(); page pools,
 *             tables, representatives, centroids and scratch all live inside it.
 *             ice_build_index COPIES K and V into page tiles; the originals may be freed.
 *   Streams   `stream` is a hipStream_t (NULL = default stream).  Every call only enqueues
 *             work; no call synchronises or reads device memory on the host.  Calls on one
 *             index must be issued in order on one stream (or be ordered by the caller).
 *   Errors    Every call returns an ice_status_t and never throws or aborts.  All errors are
 *             detected on the host from the arguments and host-side counters BEFORE anything is
 *             enqueued; ice_last_error() returns a thread-local description of the last failure.
 *   Units     unit u = b * n_kv_heads + h_kv; query head h_q belongs to KV head
 *             h_q / group_size.  Page ids are local to a unit: 0 <= id < n_pages[u].
 */
#ifndef ICECACHE_H
#define ICECACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ice_index ice_index_t;

typedef enum {
    ICE_OK = 0,
    ICE_ERR_INVALID_ARG = 1, /* null or misaligned pointer, non-positive size                  */
    ICE_ERR_SHAPE = 2,       /* sizes inconsistent with each other or with the configuration   */
    ICE_ERR_STATE = 3,       /* call made before ice_build_index / ice_import_index            */
    ICE_ERR_CAPACITY = 4,    /* would exceed max_tokens, or the workspace is too small         */
    ICE_ERR_UNSUPPORTED = 5, /* head_dim != 128, page_size not in {16,32,64}, group_size not in
                                {1,2,4,8}                                                       */
    ICE_ERR_DEVICE = 6       /* a HIP call failed (text in ice_last_error)                      */
} ice_status_t;

typedef struct {
    int32_t batch;        /* B  >= 1                                                            */
    int32_t n_kv_heads;   /* H_kv >= 1                                                          */
    int32_t group_size;   /* G = query heads per KV head (GQA, Sec. 4.3): 1, 2, 4 or 8          */
    int32_t head_dim;     /* d: 128 only                                                        */
    int32_t max_tokens;   /* per unit: prefill tokens plus every later ice_insert               */
    int32_t kmeans_iters; /* T >= 1 Lloyd rounds, fixed count (no convergence test)             */
    uint64_t seed;        /* selects the promoted keys when init_idx is NULL                    */
    const int32_t *init_idx; /* optional DEVICE int32 [B,H_kv,n_clusters]: token index of each
                                promoted key (the initial centroids, Alg. 2 "random promotion");
                                entries should be distinct; read during ice_build_index         */
} ice_config_t;

/* Device-pointer view of an index (export) or of caller arrays to copy in (import).
 * Per-unit arrays are laid out [U][...] with the element strides given below.
 *   Kp, Vp        bf16  [U][max_pages][page_size][d]   page tiles (4 KiB each at page_size 16)
 *   page_cluster  int32 [U][max_pages]                 owning cluster, -1 for unused pages
 *   page_fill     int32 [U][max_pages]                 tokens in the page, 0..page_size
 *   page_pos      int32 [U][max_pages][page_size]      original token position, -1 = empty slot
 *   cluster_tail  int32 [U][n_clusters]                last page of the cluster or -1
 *   cluster_cnt   int32 [U][n_clusters]
 *   cluster_sum   fp32  [U][n_clusters][d]
 *   centroid      fp32  [U][n_clusters][d]
 *   page_sum      fp32  [U][max_pages][d]              slot-ordered fp32 sum of the page's keys
 *   rep           bf16  [U][max_pages][d]              representative = bf16(page_sum / fill)
 *   n_pages       int32 [U]                            live pages per unit
 *   assign        int32 [U][max_tokens]  (export only) cluster of every prefill token after the
 *                                                      last Lloyd round
 *   assign_centroid_bf16 bf16 [U][cpad][d] (export only) the bf16 centroids that `assign` was
 *                                                      computed against (cpad = n_clusters
 *                                                      rounded up to 32)
 *   init_idx      int32 [U][n_clusters]  (export only) promoted token indices actually used
 */
typedef struct {
    int32_t n_units, group_size, head_dim, page_size, n_clusters, cpad;
    int32_t max_pages;   /* floor(max_tokens / page_size) + n_clusters                          */
    int32_t max_tokens;
    int32_t n_tokens;    /* tokens per unit so far (host-side counter; equal for all units)     */
    int32_t reserved;
    void *Kp, *Vp;
    int32_t *page_cluster, *page_fill, *page_pos, *cluster_tail, *cluster_cnt;
    float *cluster_sum, *centroid, *page_sum;
    void *rep;
    int32_t *n_pages;
    int32_t *assign;
    void *assign_centroid_bf16;
    int32_t *init_idx;
} ice_index_view_t;

/* Bytes of device workspace an index with this configuration needs.  0 on invalid arguments. */
size_t ice_workspace_bytes(const ice_config_t *cfg, int32_t page_size, int32_t n_clusters);

/* Creates the host-side object over a caller-owned device workspace (not touched here).
 * The workspace must stay alive until ice_destroy.  cfg is copied (init_idx pointer included). */
ice_status_t ice_create(const ice_config_t *cfg, void *workspace, size_t workspace_bytes,
                        ice_index_t **out);
/* Frees the host-side object only. */
ice_status_t ice_destroy(ice_index_t *idx);

/* Index build at prefill (Sec. 4.1-4.2, Alg. 2 restricted to two levels, iterated):
 * n_clusters keys per unit are promoted to initial centroids; kmeans_iters rounds of
 * (nearest centroid by squared Euclidean distance on bf16 centroids, lowest id on ties ->
 * member means); each cluster's tokens, in ascending position, are cut into pages of page_size
 * (a node owns a list of pages, Sec. 4.1); every page gets a representative (mean key).
 *   K, V: bf16 [B, H_kv, n_tokens, d].
 * Errors: SHAPE if n_clusters > n_tokens or n_tokens > max_tokens; UNSUPPORTED page_size;
 * CAPACITY if the workspace is too small for (page_size, n_clusters).  Rebuilding is allowed. */
ice_status_t ice_build_index(ice_index_t *idx, const void *K, const void *V, int32_t n_tokens,
                             int32_t page_size, int32_t n_clusters, void *stream);

/* Inserts one decode token per unit (Sec. 4.2 last paragraph, Alg. 1 insertion loop): nearest
 * centroid, append to that cluster's tail page (a new page when it is full or absent, Sec. 4.1),
 * update the page representative and the cluster's running mean.
 *   k, v: bf16 [B, H_kv, d].   CAPACITY when n_tokens == max_tokens; STATE before a build. */
ice_status_t ice_insert(ice_index_t *idx, const void *k, const void *v, void *stream);

/* The same for m tokens per (sequence, KV head), inserted one after the other in the order given
 * (each sees the centroid the previous one moved): the state afterwards is bit for bit that of m
 * ice_insert calls.  This is how tokens that leave the recent window enter the index a page at a
 * time (Alg. 1, insertion loop).  k, v: bf16 [B, H_kv, m, d].  SHAPE for m < 1; CAPACITY when
 * the index would hold more than max_tokens tokens per unit (nothing is inserted then). */
ice_status_t ice_insert_batch(ice_index_t *idx, const void *k, const void *v, int32_t m, void *stream);

/* Page selection for one decode query (Sec. 4.3-4.4, Alg. 3): P = floor(token_budget/page_size);
 * score(p) = max over the G query heads of (q_h . rep_p) / ||q_h||; the min(P, n_pages) best
 * pages by (score descending, id ascending) are returned with ids ascending, padded with -1.
 *   q: bf16 [B, H_q, d];  page_ids: int32 [B, H_kv, P];  n_selected: int32 [B, H_kv];
 *   scores_or_null: fp32 [B, H_kv, P] group score of each returned page (0 in the padding).
 * SHAPE if token_budget < page_size; UNSUPPORTED if the index can hold more than 32768 pages per
 * unit (the scores of a unit are ranked from one workgroup's registers: 524 288 tokens per KV head
 * at page size 16 less one page per cluster), or if the budget's winner lists (12 bytes per page
 * of the budget) do not fit a CU's LDS; a budget that covers every page is always accepted.
 * n_selected[u] = -1 (ids -1, zero attention output) reports a unit whose workgroups could not hand
 * their scores over within the bounded wait (see ice_debug_select_fault); never expected in use. */
ice_status_t ice_select(ice_index_t *idx, const void *q, int32_t token_budget, int32_t *page_ids,
                        int32_t *n_selected, float *scores_or_null, void *stream);

/* Sparse attention over the listed pages (Eq. 1 with the mask set on the tokens of those
 * pages): softmax(q_h . k / sqrt(d)) . v over every filled slot, fp32 accumulation and output.
 *   page_ids: int32 [B, H_kv, P] with P = n_ids_per_unit; the first n_selected[u] entries of
 *   each row are used and must be distinct live page ids;  out: fp32 [B, H_q, d].
 * A unit with n_selected == 0 gets zeros. */
ice_status_t ice_attend(ice_index_t *idx, const void *q, const int32_t *page_ids,
                        const int32_t *n_selected, int32_t n_ids_per_unit, float *out, void *stream);

/* ice_attend for callers that cannot allocate device memory and have no scratch to lend: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * result (to the rounding of a different split of the page list), but the partial sums of the page
 * list's shares do not go through the workspace: they live in a static device array of the library
 * (1 065 984 bytes per GPU the library runs on, held until the process ends), whose address is
 * looked up once per device at the first call there.  The call itself allocates nothing and calls
 * no allocating routine.
 * Limit: at most 256 units (batch * n_kv_heads); UNSUPPORTED beyond.  Every call on one GPU shares
 * that GPU's array: calls that overlap in time on one GPU (different streams or threads) race;
 * calls issued in order on one stream are safe.  DEVICE if the array's address cannot be found. */
ice_status_t ice_attend_noalloc(ice_index_t *idx, const void *q, const int32_t *page_ids,
                                const int32_t *n_selected, int32_t n_ids_per_unit, float *out, void *stream);

/* ice_select followed by ice_attend on the same stream; the ids never leave the device. */
ice_status_t ice_select_attend(ice_index_t *idx, const void *q, int32_t token_budget,
                               int32_t *page_ids, int32_t *n_selected, float *out, void *stream);

/* Attention with resident tokens: the decode loop of the paper (Alg. 1, App. A) always attends to
 * the sink tokens at the start of the sequence and to a window of the most recent tokens, which
 * are not (yet) in the index.  The caller keeps them as one dense run per (sequence, KV head),
 *   resident_k, resident_v bf16 [B, H_kv, n_resident, d]   (device, caller-owned, 16-byte aligned),
 * and these calls put them in the same softmax as the tokens of the pages (Eq. 1 with the mask on
 * the union).  n_resident = 0 gives ice_attend / ice_select_attend exactly (the pointers are then
 * not read).  SHAPE for n_resident outside [0, 2^20]; otherwise the errors of the plain calls.
 * Tokens leave the window into the index with ice_insert_batch. */
ice_status_t ice_attend_resident(ice_index_t *idx, const void *q, const int32_t *page_ids,
                                 const int32_t *n_selected, int32_t n_ids_per_unit, const void *resident_k,
                                 const void *resident_v, int32_t n_resident, float *out, void *stream);
ice_status_t ice_select_attend_resident(ice_index_t *idx, const void *q, int32_t token_budget,
                                        const void *resident_k, const void *resident_v, int32_t n_resident,
                                        int32_t *page_ids, int32_t *n_selected, float *out, void *stream);

/* Reuse of a selection by other layers (App. B: the layers after an anchor layer attend to the
 * tokens the anchor layer selected).  Page ids are local to one layer's index, token positions
 * are not:
 *   ice_selected_tokens  writes the sequence positions of the tokens of the listed pages, in list
 *       and slot order: token_pos int32 [B, H_kv, n_ids_per_unit * page_size] padded with -1,
 *       n_tok int32 [B, H_kv].  n_ids_per_unit in [1, 1024].
 *   ice_attend_tokens    attention (Eq. 1) of q over rows token_pos[b, h, 0 .. n_tok[b, h]) of a
 *       dense cache K, V bf16 [B, H_kv, n_rows, d] (any layer's; caller-owned device memory);
 *       max_tok = length of a unit's position list.  The index only supplies B, H_kv and the group
 *       size (STATE before a build or import).  Positions must lie in [0, n_rows) (others are
 *       clamped into the cache, not skipped).
 * With the cache the index was built from, ice_attend_tokens over ice_selected_tokens' positions
 * gives ice_attend's result over those pages. */
ice_status_t ice_selected_tokens(ice_index_t *idx, const int32_t *page_ids, const int32_t *n_selected,
                                 int32_t n_ids_per_unit, int32_t *token_pos, int32_t *n_tok, void *stream);
ice_status_t ice_attend_tokens(ice_index_t *idx, const void *q, const void *K, const void *V, int32_t n_rows,
                               const int32_t *token_pos, const int32_t *n_tok, int32_t max_tok, float *out,
                               void *stream);

/* Hierarchical selection: the two-level form of the paper's top-down search (Sec. 3.3, Alg. 4: level
 * by level from the best parents to their children; page selection, Alg. 3, calls it).
 * Stage 1 ranks the n_clusters centroids (as stored, rounded to bf16) by the same normalised GQA
 * score as pages and keeps the min(n_probe, n_clusters) best, lower id first on ties; every
 * cluster is eligible, one without pages contributes none.  Stage 2 ranks only the live pages of
 * the kept clusters and returns the best min(P, number of such pages), P = floor(budget / page_size),
 * ids ascending, padded with -1; with n_probe >= n_clusters the result is ice_select's.
 * Stage 3, when n_refine > 0 (the paper ranks keys and loads the pages that hold them): stage 2 keeps
 * min(n_refine, candidates) pages instead, each is re-scored by its best key (max over its tokens
 * and the group's heads of q_h . k / ||q_h||), and the best min(P, kept) by that score, lower id
 * first on ties, are returned; scores then holds these key scores.  n_refine must be 0 or >= P.
 *   q bf16 [B, H_q, d]; page_ids int32 [B, H_kv, P]; n_selected int32 [B, H_kv];
 *   scores_or_null fp32 [B, H_kv, P] (group scores of the returned pages);
 *   clusters_or_null int32 [B, H_kv, n_probe] (kept cluster ids ascending, -1 padded; n_probe may
 *   exceed n_clusters, the lists inside the kernel are as long as what can be kept);
 *   out_or_null fp32 [B, H_q, d]: when given, attention over the returned pages (as ice_attend)
 *   runs in the same launch.
 * All device pointers, caller-owned; only enqueues.  Errors as ice_select, plus SHAPE for
 * n_probe < 1 or 0 < n_refine < P, and UNSUPPORTED for more than 16384 pages per unit or when the
 * candidate lists (8 bytes per page the index can hold) do not fit a CU's LDS. */
ice_status_t ice_select_hier(ice_index_t *idx, const void *q, int32_t token_budget, int32_t n_probe, int32_t n_refine,
                             int32_t *page_ids, int32_t *n_selected, float *scores_or_null,
                             int32_t *clusters_or_null, float *out_or_null, void *stream);

/* A third level (Sec. 3.3: the tree has levels L..1, every point's parent is a point one level up;
 * Alg. 4 searches it top-down).  ice_build_top_level puts n_top nodes per unit above the clusters:
 * n_top clusters are promoted (evenly spaced cluster ids), then `iters` rounds of (every cluster goes
 * to the nearest top node by squared Euclidean distance between its bf16 centroid and the node's bf16
 * rounding, lowest id on ties -> every node moves to the mean of its clusters' bf16 centroids); the
 * state kept is the last assignment and the means of that assignment.  Built from the centroids as
 * they are at the call (after ice_build_index, or after insertions); it does not follow later
 * insertions (a new key gets a parent, the levels above stay as they are, Sec. 4.2), and
 * ice_build_index / ice_import_index drop it.  n_top in [1, min(256, n_clusters)]; 0 drops it.
 *
 * ice_select_hier3 is ice_select_hier with one stage in front: the n_top nodes are ranked by the
 * same normalised GQA score, the min(n_probe_top, n_top) best are kept (lower id first on ties), and
 * stage 1 ranks only the clusters hanging under them (it keeps min(n_probe, their number)).  With
 * n_probe_top >= n_top the result is ice_select_hier's.
 *   tops_or_null int32 [B, H_kv, n_probe_top]: kept top nodes ascending, -1 padded.
 * STATE before ice_build_top_level; SHAPE for n_probe_top < 1; otherwise as ice_select_hier.
 * ice_export_top_level gives device pointers into the workspace:
 *   top_centroid fp32 [U][n_top_max][d], top_centroid_bf16 bf16 [U][n_top_max][d] (rows >= n_top zero),
 *   top_of int32 [U][n_clusters], top_count int32 [U][n_top_max], top_init int32 [U][n_top_max] (the
 *   cluster each node was promoted from). */
typedef struct {
    int32_t n_top, n_top_max;
    float *top_centroid;
    void *top_centroid_bf16;
    int32_t *top_of, *top_count, *top_init;
} ice_top_view_t;
ice_status_t ice_build_top_level(ice_index_t *idx, int32_t n_top, int32_t iters, void *stream);
ice_status_t ice_export_top_level(ice_index_t *idx, ice_top_view_t *view);
ice_status_t ice_select_hier3(ice_index_t *idx, const void *q, int32_t token_budget, int32_t n_probe_top, int32_t n_probe,
                              int32_t n_refine, int32_t *page_ids, int32_t *n_selected, float *scores_or_null,
                              int32_t *clusters_or_null, int32_t *tops_or_null, float *out_or_null, void *stream);

/* Geometry of the clustering (Sec. 4.2, Eq. 2).  The paper measures key-key distances between
 * transformed keys T_K(k) = [k / c, sqrt(1 - ||k||^2 / c^2)], c >= the largest key norm.  With
 * ICE_GEOMETRY_TRANSFORMED the next ice_build_index (and every later insertion) does the same,
 * kept times c: every key and every centroid carries ONE more coordinate, a(k) = sqrt(c^2 - ||k||^2)
 * rounded to bf16 resp. the mean of its members' a, c^2 = the largest squared norm among the
 * unit's prefill keys (a later key with a larger norm gets a = 0).  Page tiles, representatives,
 * selection and attention are unchanged (the transformed query has 0 in that coordinate, Eq. 3).
 * ICE_GEOMETRY_RAW (the default) clusters on the keys as they are.  An imported index is raw.
 * ice_export_geometry gives device pointers into the workspace (null when raw):
 *   key_extra bf16 [U][max_tokens] by token position; centroid_extra, cluster_sum_extra fp32
 *   [U][n_clusters]; radius_sq fp32 [U]; assign_centroid_extra_bf16 bf16 [U][cpad], the extra
 *   coordinate of the centroids that the exported `assign` was computed against. */
enum { ICE_GEOMETRY_RAW = 0, ICE_GEOMETRY_TRANSFORMED = 1 };
typedef struct {
    int32_t geometry, reserved;
    void *key_extra;
    float *centroid_extra, *cluster_sum_extra, *radius_sq;
    void *assign_centroid_extra_bf16;
} ice_geometry_view_t;
ice_status_t ice_set_geometry(ice_index_t *idx, int32_t geometry);
ice_status_t ice_export_geometry(ice_index_t *idx, ice_geometry_view_t *view);

/* Test and snapshot surface.  Export fills `view` with pointers INTO the workspace (no copy).
 * Import copies caller arrays (device pointers, same layout; the export-only fields are
 * ignored; n_tokens, page_size, n_clusters, max_pages must fit the workspace) into the index and
 * recomputes only what is derived from the centroids (their bf16 rounding and squared norms);
 * every other bit is used as given. */
ice_status_t ice_export_index(ice_index_t *idx, ice_index_view_t *view);
ice_status_t ice_import_index(ice_index_t *idx, const ice_index_view_t *view, void *stream);

/* The assignment step alone (one Lloyd round's first half, Sec. 4.2: every key gets its nearest
 * promoted point) on caller data, for parity tests:
 *   K bf16 [n_units, n, d]; centroids_bf16 bf16 [n_units, n_clusters, d] ->
 *   assign_out int32 [n_units, n]; best_out_or_null fp32 [n_units, n] = min_c(||mu_c||^2 - 2 k.mu_c).
 * With assign_out NULL only the assignment kernel is enqueued (its packed winners stay in the
 * workspace): the form the benchmark times.  Uses the index's workspace as scratch and invalidates a
 * built index (STATE afterwards). */
ice_status_t ice_debug_assign(ice_index_t *idx, const void *K, int32_t n, const void *centroids_bf16,
                              int32_t n_clusters, int32_t *assign_out_or_null, float *best_out_or_null,
                              void *stream);

/* Measurement hook: enqueues ONE stage of the last ice_build_index again, on the state that build
 * left and the same K, V (bf16 [B, H_kv, n_tokens, d] as given to the build): the assignment of the
 * last Lloyd round, the counting sort by cluster, the member means, or the page layout (Sec. 4.1-4.2).
 * Every stage reproduces what it wrote before, so the index is unchanged; the benchmark brackets
 * such calls with events to time each kernel by itself.  STATE unless the index is fresh from
 * ice_build_index (no insertion since, not imported). */
enum { ICE_STAGE_ASSIGN = 0, ICE_STAGE_SORT = 1, ICE_STAGE_MEANS = 2, ICE_STAGE_PAGINATE = 3 };
ice_status_t ice_debug_rerun_stage(ice_index_t *idx, const void *K, const void *V, int32_t stage, void *stream);

/* Test hook for the failure path of ice_select / ice_select_attend when a unit is served by several
 * workgroups (fewer than 256 units): those workgroups hand their page scores to the last one of
 * them through device memory, and that one waits for a missing score only a bounded number of
 * re-reads.  This call is ice_select_attend (out_or_null: ice_select) with the score stores of
 * workgroup `muted_chunk` of every unit left out and the wait cut to 2^wait_log2 re-reads, so the
 * wait expires with every wave running to its end.  What an expired wait does, here and in the
 * product calls: the unit is not ranked; n_selected[u] = -1, its page ids are -1, its output rows
 * are 0, and every later selection call reports the same for that unit until ice_build_index or
 * ice_import_index re-arms it.  UNSUPPORTED when units have one workgroup each (nothing is handed
 * over); SHAPE for muted_chunk outside the launch's workgroups per unit or wait_log2 outside [0, 20]. */
ice_status_t ice_debug_select_fault(ice_index_t *idx, const void *q, int32_t token_budget, int32_t *page_ids,
                                    int32_t *n_selected, float *out_or_null, int32_t muted_chunk, int32_t wait_log2,
                                    void *stream);

/* Measured-peak microbenchmarks for the benchmark's roofline context (no method arithmetic):
 *   ice_debug_peak_read  streams `bytes` (multiple of 16, 16-byte aligned device pointer) once with
 *                        16-byte non-temporal loads; achieved bytes/s = bytes / kernel time.
 *   ice_debug_peak_mfma  runs `iters` rounds of four independent v_mfma_f32_32x32x16_bf16 chains per
 *                        wave on register operands and writes the flop count of the launch to the
 *                        HOST double *flops_out (may be null).
 * `sink` is a device buffer of at least 524288 floats that keeps the results alive.  Both only
 * enqueue on `stream`.  INVALID_ARG for null / misaligned pointers or iters < 1. */
ice_status_t ice_debug_peak_read(const void *buf, size_t bytes, float *sink, void *stream);
ice_status_t ice_debug_peak_mfma(float *sink, int32_t iters, double *flops_out, void *stream);

const char *ice_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ICECACHE_H */
