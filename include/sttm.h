/*
 * libsttm -- spatio-temporal token merging for video token tensors on one AMD GPU (gfx950).
 *
 * The library turns a video's visual tokens Z_V in R^{T x H x W x C} into the reduced sequence
 * Z_ST in R^{N_ST x C} (Sec. 3.1 of the STTM paper) in three stages:
 *
 *   1. spatial:  per frame, a coarse-to-fine search over a dense quadtree keeps a node when the cosine
 *                similarity between its mean and each child's mean exceeds tau_S, else descends (Sec. 3.2);
 *   2. temporal: every kept node of frame t is linked to an overlapping kept node of frame t-1 when their
 *                cosine similarity exceeds tau_T (top-left-most passing destination wins); chains of links
 *                are resolved to their common root, the earliest occurrence (Sec. 3.3);
 *   3. reduce:   every connected graph becomes one token, the average of its member tokens, emitted in
 *                order of the root's (video, frame, y, x) (Sec. 3.1, 3.3, 3.4).
 * A fourth call picks tau_S / tau_T from a token budget (the paper sets them by hand, Sec. 4.1, and names an
 * automatic rule as future work, Sec. 5; the rule here is defined below).
 *
 * Conventions
 *   - plain C ABI; every function returns an sttm_status (0 = ok) unless stated otherwise and never throws
 *     or aborts; sttm_last_error() gives the message of the last failure on that context.
 *   - "device" pointers are HIP device memory on the context's device, owned by the caller; the library
 *     never allocates or frees device memory: all intermediate tables live in a caller-provided workspace.
 *   - "host" pointers are ordinary host memory, read or written before the call returns.
 *   - all work is enqueued on the context's stream; calls return before the GPU finishes unless they
 *     hand a value back through a host pointer (documented per call), in which case they synchronise the stream.
 *   - feats is contiguous [B, T, H, W, D] (D fastest), B independent videos; tokens are addressed by the
 *     flat cell index i = ((b*T + t)*H + y)*W + x.  Requirements: 1 <= H, W <= 32; D % 8 == 0;
 *     B*T <= 65535 frames; B*T*H*W < 2^31; root_grid a power of two <= P, P = smallest power of two >= max(H, W).
 *   - a grid that is not a power of two is embedded top-left in the P x P grid; padded cells take no part.
 *   - quadtree level 0 is the finest (single cells), level log2(P/root_grid) holds the roots.
 *   - similarities are clamped to <= 1 and compared strictly (">"): a threshold >= 1 merges nothing.
 *     A zero-norm vector has similarity 0 to everything; NaN never passes a threshold.
 */
#ifndef STTM_H_
#define STTM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sttm_ctx sttm_ctx; /* opaque; bound to one device and one stream */

typedef enum {
  STTM_OK = 0,
  STTM_ERR_NULL = 1,      /* a required pointer is NULL */
  STTM_ERR_SHAPE = 2,     /* a dimension or root_grid violates the requirements above */
  STTM_ERR_DTYPE = 3,     /* unknown sttm_dtype */
  STTM_ERR_ARG = 4,       /* any other bad argument (e.g. target_keep outside (0, 1]) */
  STTM_ERR_WORKSPACE = 5, /* no workspace set, or it is smaller than sttm_workspace_bytes() */
  STTM_ERR_STATE = 6,     /* stage called before the stage it depends on */
  STTM_ERR_CAPACITY = 7,  /* more output tokens than the caller's capacity */
  STTM_ERR_HIP = 8        /* a HIP runtime call failed; message holds hipGetErrorString */
} sttm_status;

typedef enum { STTM_F32 = 0, STTM_BF16 = 1, STTM_F16 = 2 } sttm_dtype;
typedef enum { STTM_STAGE_SPATIAL = 0, STTM_STAGE_TEMPORAL = 1 } sttm_stage;

/* Which destination a node of frame t takes when it overlaps several kept nodes of frame t-1 (Sec. 3.3; the
 * "Approximated Temporal Matching" ablation of Sec. 4.3 compares the top-left rule with the most similar one). */
typedef enum {
  STTM_MATCH_FIRST_PASSING = 0, /* every overlapping destination is tested; of those above tau_T the one towards
                                   the top-left (smallest raster index) wins -- the rule of Sec. 3.3, the default */
  STTM_MATCH_TOPLEFT_ONLY = 1,  /* only the destination under the node's own top-left cell is tested */
  STTM_MATCH_MOST_SIMILAR = 2   /* of those above tau_T the most similar wins (ties: towards the top-left) */
} sttm_match;

/* Linear order of the output rows (Sec. 3.4): earlier frames first; inside a frame by the root's top-left cell. */
typedef enum {
  STTM_ORDER_RASTER = 0, /* (y0, x0) row by row = ascending cluster id; the default */
  STTM_ORDER_ZSCAN = 1   /* Z-shaped scan: quadrants top-left, top-right, bottom-left, bottom-right, recursively */
} sttm_order;

/* Tables sttm_export() can copy out (parity tests compare them with the CPU oracle). F = B*T frames,
 * NN = nodes per frame over all levels of the P x P pyramid (see sttm_nodes_per_frame). */
typedef enum {
  STTM_TBL_CHILD_SIM = 0,  /* float [F, NN]: sigma(parent(n), n) for every node below the root level (Sec. 3.2) */
  STTM_TBL_MIN_SIM = 1,    /* float [F, NN]: m_n = min over n's existing children; levels >= 1 */
  STTM_TBL_NORM2 = 2,      /* float [F, NN]: squared norm of the sum of n's valid cells */
  STTM_TBL_PAIR_SIM = 3,   /* float [F, H*W]: for frame f (t >= 1) and cell q that is the top-left cell of the finer
                              of the two overlapping nodes (frame t vs t-1): their cosine similarity (Sec. 3.3) */
  STTM_TBL_BEST_SIM = 4,   /* float [F, H*W]: at the top-left cell of every kept node of a frame t >= 1:
                              e_n = max similarity over its overlapping nodes of frame t-1 */
  STTM_TBL_PARENT = 5      /* int32 [F, H*W]: at the top-left cell of every kept node: flat index of the top-left
                              cell of its destination node in frame t-1, or -1 (no edge; also all other cells) */
} sttm_table;

/* ---- context ---------------------------------------------------------------------------------------- */

/* Creates a context on HIP device `device`. `hip_stream` is a hipStream_t owned by the caller (NULL = the
 * default stream); every kernel and copy of this context is enqueued on it. Host memory only is allocated. */
int sttm_create(sttm_ctx** out, int device, void* hip_stream);
int sttm_destroy(sttm_ctx* ctx);
/* Message of the last failing call on ctx (static text if ctx is NULL). Owned by the context. */
const char* sttm_last_error(const sttm_ctx* ctx);
/* Number of pyramid nodes per frame (all levels, padded P x P grid), or 0 for an invalid shape. */
int sttm_nodes_per_frame(int H, int W, int root_grid);
/* Index of node (level, by, bx) inside a frame's NN-entry table, or -1. */
int sttm_node_index(int H, int W, int root_grid, int level, int by, int bx);

/* Bytes of device workspace the four stages need for this shape (0 for an invalid shape). */
size_t sttm_workspace_bytes(int B, int T, int H, int W, int D, int dtype, int root_grid);
/* Hands the library a device buffer (256-byte aligned) it may overwrite at will until the next
 * sttm_set_workspace / sttm_destroy. Tables of earlier stages live there between calls. */
int sttm_set_workspace(sttm_ctx* ctx, void* workspace_dev, size_t bytes);

/* The library recognises "the same features / node map as before" by the device pointer alone: it cannot see a
 * buffer being rewritten in place. A caller that overwrites feats, node_map or cluster_ids in place between two
 * calls of one pass over a video calls sttm_invalidate() first: every table a later stage would reuse (statistics,
 * thresholds, node sums, the reduce call's lists) is then treated as absent, and the stages that need them return
 * STTM_ERR_STATE until they are computed again. Host-side only; the workspace itself is left alone. */
int sttm_invalidate(sttm_ctx* ctx);

/* Destination rule of the temporal stage (sttm_match); applies to the temporal calls that follow. With
 * STTM_MATCH_TOPLEFT_ONLY the table BEST_SIM and the temporal budget use the similarity to that one destination. */
int sttm_set_match_mode(sttm_ctx* ctx, int mode);
/* Row order of sttm_reduce and sttm_positions (sttm_order); applies to the calls that follow. */
int sttm_set_output_order(sttm_ctx* ctx, int order);
/* level = 1 (the default): the spatial statistics pass also computes x_c(t) . x_c(t+1) for every cell c and frame t
 * (Sec. 3.3 compares the features of overlapping nodes of consecutive frames; where both nodes are single cells
 * that is this dot product), and the temporal pass leaves those pairs out instead of reading both rows again.
 * level = 2: the same also for every 2x2 and 4x4 block (S_n(t) . S_n(t+1), used where both frames keep the same
 * node n at level 1 or 2). level = 0 keeps the two passes separate. Each level makes the statistics pass slower
 * and the temporal pass faster: 1 pays wherever many tokens stay unmerged in space, 2 where many of them merge
 * spatially (measured on a 512-frame video: from budgets of about a third of the tokens downwards; at a half it costs
 * the statistics pass slightly more than the temporal pass gains), 0 never did on the workloads measured. Results
 * agree to rounding. Takes effect with the next
 * statistics pass (sttm_spatial_stats / sttm_spatial_quadtree with thresholds). */
int sttm_set_cell_dots(sttm_ctx* ctx, int level);

/* ---- stage 1: spatial quadtree (Sec. 3.2) ------------------------------------------------------------- */

/* Pyramid statistics only: block sums at every level, squared norms, parent-child cosine similarities and
 * m_n = min over children, into the workspace. Binds the context to this shape. Asynchronous. */
int sttm_spatial_stats(sttm_ctx* ctx, const void* feats_dev, int dtype, int B, int T, int H, int W, int D,
                       int root_grid);

/* Granularity decision. tau_s: host array of B thresholds (one per video), or NULL = use the thresholds last
 * chosen by sttm_budget_threshold(STTM_STAGE_SPATIAL). With tau_s != NULL the statistics are (re)computed from
 * feats first; with NULL they must already be in the workspace (STTM_ERR_STATE otherwise) and feats is not read.
 * Outputs (device): node_map int32 [B,T,H,W] = flat index of the top-left cell of the kept node covering the
 * cell; node_level uint8 [B,T,H,W] = that node's level (may be NULL). Asynchronous. */
int sttm_spatial_quadtree(sttm_ctx* ctx, const void* feats_dev, int dtype, int B, int T, int H, int W, int D,
                          int root_grid, const float* tau_s_host, int32_t* node_map_dev, uint8_t* node_level_dev);

/* ---- stage 2: temporal merging (Sec. 3.3) ------------------------------------------------------------- */

/* Similarities between every kept node of frame t >= 1 and each overlapping kept node of frame t-1, and the best
 * one per node (tables PAIR_SIM, BEST_SIM). node_map / node_level as produced by stage 1 (any valid quadtree
 * partition per frame is accepted). Needs the stage-1 statistics of the same feats in the workspace: feats_dev must
 * be the buffer the last statistics pass read (STTM_ERR_STATE otherwise; the norms, the sums of large nodes and the
 * cell-to-cell dot products come from that pass). Asynchronous. */
int sttm_temporal_stats(sttm_ctx* ctx, const void* feats_dev, const int32_t* node_map_dev,
                        const uint8_t* node_level_dev);

/* Directed edges (similarity > tau_T, top-left-most passing destination), then the common root of every chain.
 * tau_t: host array of B thresholds, or NULL = those chosen by sttm_budget_threshold(STTM_STAGE_TEMPORAL).
 * With tau_t != NULL the temporal statistics are (re)computed first; with NULL they must be in the workspace and
 * node_map_dev must be the node map they were computed for (STTM_ERR_STATE otherwise). A new statistics pass
 * (sttm_temporal_stats) discards the threshold of an earlier budget search.
 * Output (device): cluster_ids int32 [B,T,H,W] = flat index of the top-left cell of the root node of the cell's
 * cluster (= the smallest flat index in the cluster). Asynchronous. */
int sttm_temporal_merge(sttm_ctx* ctx, const void* feats_dev, const int32_t* node_map_dev,
                        const uint8_t* node_level_dev, const float* tau_t_host, int32_t* cluster_ids_dev);

/* ---- thresholds from a token budget (Sec. 4.1 / Sec. 5) ------------------------------------------------ */

/* target_keep: host array [B], each in (0, 1]: the fraction of that video's T*H*W tokens the whole path should
 * keep. The spatial stage aims at floor(sqrt(keep)*T*H*W) nodes, the temporal stage at floor(keep*T*H*W) tokens.
 * Token count as a function of the threshold is a step function K(tau) = base + sum_j w_j [v_j <= tau] (spatial:
 * v = max of m over the path from the root to the node, w = children - 1; temporal: v = e_n, w = 1). The threshold
 * chosen is the midpoint of the last interval between consecutive distinct v on which K <= target (1 if K never
 * exceeds it, -2 if even merging everything exceeds it). Requires the stage's statistics in the workspace; stores
 * the thresholds on the device for the following sttm_spatial_quadtree / sttm_temporal_merge call with NULL
 * thresholds. tau_out: host array [B] or NULL; when non-NULL the stream is synchronised and the values copied out
 * (with NULL the last step of the search is left to that following call, which saves a kernel launch). */
int sttm_budget_threshold(sttm_ctx* ctx, int stage, const double* target_keep_host, float* tau_out_host);

/* ---- stage 3: gather / average (Sec. 3.1, 3.3, 3.4) ---------------------------------------------------- */

/* One output row per cluster, in ascending cluster id (or, with STTM_ORDER_ZSCAN, the rows of a frame in the
 * Z-shaped scan of their roots; see sttm_set_output_order): merged [capacity, D] of out_dtype = mean of the member
 * cells' features (fp32 accumulation in a fixed order); counts int32 [capacity] = members; out_ids int32 [capacity]
 * = cluster id; offsets int64 [B+1] = first row of each video, offsets[B] = K (all device, counts/out_ids may be
 * NULL). out_dtype: any sttm_dtype for fp32 input; the input's own type or fp32 for bf16 / fp16 input
 * (STTM_ERR_DTYPE otherwise). Rows beyond capacity are not written. n_out: host pointer or NULL; when non-NULL
 * the stream is synchronised, *n_out = K and STTM_ERR_CAPACITY is returned if K > capacity. Uses the shape bound
 * by stage 1; cluster_ids may be any labelling in which a cluster's id is its smallest member's flat index.
 * node_map / node_level (device, both or neither): the stage-1 partition the cluster ids were built on, as
 * sttm_temporal_merge received it -- all cells of a node must carry the same cluster id, and the workspace must
 * still hold the stage-1 statistics of these (unchanged) feats (STTM_ERR_STATE otherwise). Nodes at level >= 3 are
 * then added from the per-node sums stage 1 left in the workspace instead of being read again cell by cell; the
 * result differs from the NULL call only in the order of the fp32 additions. */
int sttm_reduce(sttm_ctx* ctx, const void* feats_dev, const int32_t* cluster_ids_dev,
                const int32_t* node_map_dev, const uint8_t* node_level_dev, int out_dtype, int64_t capacity,
                void* merged_dev, int32_t* counts_dev, int32_t* out_ids_dev, int64_t* offsets_dev,
                int64_t* n_out_host);

/* For callers that cannot allocate (code under HIP graph capture, serving loops and harnesses in which device
 * allocation is forbidden): sttm_reduce without a workspace and without the stage-1 partition. Same result as
 * sttm_reduce(ctx, feats, cluster_ids, NULL, NULL, ...) bit for bit (same kernels); the shape is passed here because
 * no stage-1 call need have bound one. Its tables (ranks, sort buffers, member lists, partial sums of large clusters)
 * live in a fixed array of sttm_reduce_noalloc_max_bytes() = 32 MiB inside the library's device image, held by every
 * GPU the library runs on until the process ends; the call allocates nothing, on the device or through a library
 * that would, never synchronises and copies nothing to the host, so K is read from offsets[B] (rows beyond
 * capacity are not written). A shape whose tables need more (sttm_reduce_noalloc_bytes(), about 44 bytes per token
 * plus D/2 bytes per token plus 2 MiB) is refused with STTM_ERR_WORKSPACE. All calls on one GPU share the one
 * array: two calls that overlap in time on the same GPU (different streams or contexts) race; calls on one stream
 * do not. The context's workspace, bound shape and cached tables are left untouched; sttm_positions does not
 * follow this call. Row order as set by sttm_set_output_order. */
int sttm_reduce_noalloc(sttm_ctx* ctx, const void* feats_dev, int dtype, int B, int T, int H, int W, int D,
                        const int32_t* cluster_ids_dev, int out_dtype, int64_t capacity, void* merged_dev,
                        int32_t* counts_dev, int32_t* out_ids_dev, int64_t* offsets_dev);
size_t sttm_reduce_noalloc_max_bytes(void);
size_t sttm_reduce_noalloc_bytes(int B, int T, int H, int W, int D, int dtype);

/* ---- position indices of the output rows (Sec. 3.4) ---------------------------------------------------------- */

/* For the rows the preceding sttm_reduce call on the same cluster_ids produced (same order), all device, each may
 * be NULL, rows beyond capacity are not written:
 *   survived   int32 [capacity]: index, within its video, of the surviving (root) token: t*H*W + y0*W + x0
 *                                ("survived" strategy: the root keeps its original position);
 *   reassigned int32 [capacity]: index of the row within its video's output sequence ("reassigned" strategy);
 *   merged_pos float [capacity]: mean of the member tokens' original indices (the index-level form of the
 *                                "merged" strategy, which averages the members' rotary embeddings);
 *   root_tyxl  int32 [capacity, 4]: (t, y0, x0, level) of the root node, for encodings built on (t, y, x);
 *                                level is -1 when node_level is NULL.
 * cluster_ids / node_map / node_level as given to sttm_temporal_merge (node_map and node_level may be NULL; with
 * both, every node is counted in one step instead of cell by cell); offsets as written by sttm_reduce.
 * Asynchronous. STTM_ERR_STATE unless sttm_reduce ran last on this context with these cluster_ids. */
int sttm_positions(sttm_ctx* ctx, const int32_t* cluster_ids_dev, const int32_t* node_map_dev,
                   const uint8_t* node_level_dev, const int64_t* offsets_dev, int64_t capacity, int32_t* survived_dev, int32_t* reassigned_dev,
                   float* merged_pos_dev, int32_t* root_tyxl_dev);

/* ---- inspection ---------------------------------------------------------------------------------------- */

/* Copies an internal table (device to device, asynchronous) into dst_dev; bytes must equal the table's size. */
int sttm_export(sttm_ctx* ctx, int table, void* dst_dev, size_t bytes);

/* The three kernels that read the features (one per stage); everything else touches O(1) scalars per token. */
typedef enum {
  STTM_KERNEL_PYRAMID_STATS = 0, /* stage 1: block sums, norms, parent-child dot products */
  STTM_KERNEL_TEMPORAL_DOTS = 1, /* stage 2: dot products of overlapping nodes of consecutive frames (the timed
                                    region is the planner that lists the work plus the pass over the features) */
  STTM_KERNEL_REDUCE_GATHER = 2, /* stage 3: gather and average the member rows */
  STTM_KERNEL_COUNT = 3
} sttm_kernel;

/* Benchmark aid: with every > 0, every `every`-th launch of each of the three feature kernels (the first one
 * included) is bracketed by HIP events on the context's stream; 0 turns it off; either call resets the record.
 * An event pair costs a few microseconds of stream time, hence the option to sample. sttm_profile_read
 * synchronises the stream and returns the summed device time in milliseconds and the number of launches
 * recorded for one kernel. */
int sttm_profile_enable(sttm_ctx* ctx, int every);
int sttm_profile_read(sttm_ctx* ctx, int kernel, double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* STTM_H_ */
