/*
 * revive.h - C ABI of the failure-remapped MoE layer for AMD MI355X (gfx950).
 *
 * The library implements the MoE layer as it runs after failed expert ranks
 * have been removed from service (ReviveMoE, arXiv 2602.21140):
 *
 *   - Sec. 3.4 "Redundant experts": recovery removes the failed replicas from
 *     the logical-to-physical expert map; weights do not move.
 *   - Sec. 3.4 "Missing experts" / Sec. 4.2: an expert with no replica left is
 *     masked to -inf immediately before the top-k, so the next-best live
 *     experts take its place.
 *   - Sec. 2.1 / 2.3: gating scores -> top-k -> dispatch (A2E) of tokens to
 *     their experts -> expert FFN -> combine (E2A) weighted by the scores.
 *   - Sec. 3.6: the forward runs as a captured graph; here the map and the
 *     mask are device-resident *data*, so a recovery is one small table copy
 *     followed by a replay of the same graph executable.
 *
 * Expert-parallel ranks are simulated on one GPU: rank r owns the physical
 * expert slots [r*S, (r+1)*S) and the rows [slot_offsets[r*S],
 * slot_offsets[(r+1)*S)) of the permuted activation buffer.  A failed rank
 * receives no rows and its slots' weights are never read (Sec. 3.5: a failed
 * device still exists but is never touched).
 *
 * Conventions
 *   - Every function returns REVIVE_OK (0) or a negative revive_status; no
 *     exception or abort crosses this boundary.  revive_last_error() gives
 *     the text of the last failure on a context.
 *   - "dev" pointers are device (HBM) pointers owned by the caller, "host"
 *     pointers are ordinary host memory.  The library owns only its context,
 *     its small device tables and what it places in the bound workspace.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - The four data-path calls (route, dispatch, expert_ffn, combine) are
 *     asynchronous on `stream`; they allocate nothing, never synchronise,
 *     never read device data on the host, and launch the same grids for the
 *     same T, so they may be recorded with hipStreamBeginCapture.
 *   - Element type `dtype`: 0 = fp32, 1 = bf16.  It is the type of x, of all
 *     weights and of x_perm / y_perm / y_shared / out.  Products accumulate in
 *     fp32; bf16 results are rounded to nearest-even once per stored tensor.
 *   - Matrices are row-major.  Weights are "output-major", i.e. the transposes
 *     of the matrices in y = (silu(x G) * (x U)) D:
 *       w_router      [E, H]      row e  = router column of expert e
 *       gate / up     [I, H]      row i  = the H weights producing intermediate i
 *       down          [H, I]      row h  = the I weights producing output h
 *     fp32 layers take them plainly: w_gate_up[p] = [gate; up] as [2I, H],
 *     w_down[p] = [H, I].  bf16 layers take gate, up and down in a TILED layout
 *     that makes every block a workgroup fetches contiguous in HBM: a [rows, K]
 *     matrix is stored as [ceil(rows/128)][K/32][128][32] elements (rows
 *     zero-padded to a multiple of 128; element (r, k) sits at
 *     ((r/128 * K/32 + k/32) * 128 + r%128) * 32 + k%32).  w_gate_up[p] is the
 *     tiled gate matrix followed by the tiled up matrix; w_down[p] the tiled
 *     down matrix; the shared expert's matrices likewise.  The router matrix is
 *     always plain.  The Python binding's pack_expert / unpack_expert convert
 *     from and to the math layout.
 *   - Limits: E <= 512, P = n_ranks*slots_per_rank <= 1024, k <= 32,
 *     H % 8 == 0; for bf16 additionally H % 64 == 0, I % 64 == 0 and
 *     I_shared % 64 == 0, and one expert matrix (2*I*H or H*I elements, rows
 *     padded to 128) must stay below 2 GiB.  T_max * k < 2^30, and T_max * k
 *     must stay below 32768 row-tiles (256 rows for bf16, 64 rows for fp32),
 *     the most one slot can be handed when every token picks it.
 */
#ifndef REVIVE_H
#define REVIVE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct revive_ctx revive_ctx;
typedef struct revive_graph revive_graph;
typedef void* revive_stream; /* hipStream_t */

typedef enum revive_status {
  REVIVE_OK = 0,
  REVIVE_EINVAL = -1,               /* bad argument or unsupported shape   */
  REVIVE_ENOMEM = -2,               /* allocation failed / workspace small */
  REVIVE_ESTATE = -3,               /* call made in the wrong order        */
  REVIVE_EINSUFFICIENT_EXPERTS = -4,/* fewer than k live experts reachable */
  REVIVE_EHIP = -5                  /* a HIP runtime call failed           */
} revive_status;

enum { REVIVE_SCORE_SOFTMAX = 0, REVIVE_SCORE_SIGMOID = 1 };
enum { REVIVE_DTYPE_F32 = 0, REVIVE_DTYPE_BF16 = 1 };

typedef struct revive_config {
  int32_t T_max;          /* largest token count of any call                     */
  int32_t H;              /* hidden size                                         */
  int32_t E;              /* logical routed experts                              */
  int32_t k;              /* experts per token                                   */
  int32_t I;              /* routed expert intermediate width                    */
  int32_t I_shared;       /* shared expert width, 0 = no shared expert           */
  int32_t n_ranks;        /* simulated expert-parallel ranks R                   */
  int32_t slots_per_rank; /* physical expert slots per rank S                    */
  int32_t max_replicas;   /* upper bound on replicas of one logical expert       */
  int32_t score_fn;       /* REVIVE_SCORE_*                                      */
  int32_t n_group;        /* contiguous expert groups; 1 = ungrouped             */
  int32_t topk_group;     /* groups kept per token (1 when ungrouped)            */
  int32_t dtype;          /* REVIVE_DTYPE_*                                      */
  float route_scale;      /* multiplies the renormalised top-k weights           */
} revive_config;

typedef struct revive_map_stats {
  int32_t n_live_slots;       /* slots holding an expert on a live rank         */
  int32_t n_live_experts;     /* experts with at least one surviving replica    */
  int32_t n_lost_experts;     /* experts with none: masked in the gate          */
  int32_t n_degraded_experts; /* experts that lost some but not all replicas    */
} revive_map_stats;

/* ---- context ------------------------------------------------------------ */

/* Validate `cfg`, allocate the context, its device tables (<= a few hundred KB)
 * and pinned staging on the current device.  *out is NULL on failure. */
int revive_create(const revive_config* cfg /*host*/, revive_ctx** out);
int revive_destroy(revive_ctx* ctx);

/* Size of the scratch workspace the data-path calls need (block histograms,
 * GEMM tile lists, the FFN's intermediate activations), and binding of a
 * caller-owned device buffer of at least that size (256-byte aligned).  The
 * buffer must stay valid until the context is destroyed or another is bound.
 * Binding writes a few bytes of the buffer (synchronously); the data-path
 * calls of one context share the workspace, so calls that overlap in time on
 * different streams race. */
int revive_workspace_bytes(const revive_ctx* ctx, size_t* bytes /*host*/);
int revive_bind_workspace(revive_ctx* ctx, void* dev, size_t bytes);

/* Static placement (Sec. 3.4): phys_to_logical[p] is the logical expert whose
 * weights slot p holds, or -1 for an empty slot.  host int32[P].  Fixed for the
 * life of the weights; failures never change it.  Must precede update_map. */
int revive_set_placement(revive_ctx* ctx, const int32_t* phys_to_logical /*host*/);

/* a0 - Recovery step (Sec. 3.4, Sec. 4.1 "update to gating mechanisms").
 * rank_failed: host uint8[R], 1 = failed.  Rebuilds, on the host, for every
 * logical expert the ascending list of surviving slots; an expert with none
 * becomes masked.  Validates first: bytes must be 0/1 and every token must
 * still be able to reach k live experts (else REVIVE_EINSUFFICIENT_EXPERTS);
 * on any error the device tables are left untouched.  On success enqueues one
 * host-to-device copy into the fixed-address tables on `stream`; work queued
 * on that stream afterwards (including replays of a captured graph) sees the
 * new map.  Not capturable.  stats may be NULL. */
int revive_update_map(revive_ctx* ctx, const uint8_t* rank_failed /*host*/, revive_stream stream,
                      revive_map_stats* stats /*host, nullable*/);

/* As revive_update_map, with experts that are failed individually as well
 * (Sec. 4.2: a failed expert is treated as failed wherever it is chosen and is
 * masked to -inf before the top-k).  expert_failed: host uint8[E], 1 = every
 * replica of that expert is removed; NULL = none.  Rank and expert failures
 * compose. */
int revive_update_map_experts(revive_ctx* ctx, const uint8_t* rank_failed /*host*/,
                              const uint8_t* expert_failed /*host, nullable*/, revive_stream stream,
                              revive_map_stats* stats /*host, nullable*/);

/* Copies of the current host-side tables (for tests): l2p_table int32
 * [E*max_replicas] (-1 padded), l2p_count int32[E], slot_alive uint8[P]. */
int revive_get_map(const revive_ctx* ctx, int32_t* l2p_table /*host*/, int32_t* l2p_count /*host*/,
                   uint8_t* slot_alive /*host*/);

/* The host computation of revive_update_map alone, without a context or a
 * GPU: builds the three tables (same layouts as revive_get_map) from a
 * placement and a failed-rank mask.  Same validation and return codes; stats
 * is filled even when REVIVE_EINSUFFICIENT_EXPERTS is returned.  With
 * ctx == NULL the error text is read with revive_last_error(NULL). */
int revive_build_map(const revive_config* cfg /*host*/, const int32_t* phys_to_logical /*host,[P]*/,
                     const uint8_t* rank_failed /*host,[R]*/, int32_t* l2p_table /*host*/,
                     int32_t* l2p_count /*host*/, uint8_t* slot_alive /*host*/,
                     revive_map_stats* stats /*host, nullable*/);

int revive_build_map_experts(const revive_config* cfg /*host*/, const int32_t* phys_to_logical /*host,[P]*/,
                             const uint8_t* rank_failed /*host,[R]*/, const uint8_t* expert_failed /*host,[E],nullable*/,
                             int32_t* l2p_table /*host*/, int32_t* l2p_count /*host*/, uint8_t* slot_alive /*host*/,
                             revive_map_stats* stats /*host, nullable*/);

/* ---- lost-expert study (Sec. 4.2) ---------------------------------------- */

/* "Every nth": mask[e] = 1 for the experts whose index is a multiple of n (n = 2
 * fails every even-indexed expert), a fraction 1/n of them.  mask: host uint8[E]. */
int revive_mask_every_nth(int32_t E, int32_t n, uint8_t* mask /*host*/);

/* "Task-based": mask[e] = 1 for the n_fail most frequently activated experts
 * (descending count, equal counts by ascending id).  counts: host int64[E]. */
int revive_mask_most_activated(const int64_t* counts /*host*/, int32_t E, int32_t n_fail, uint8_t* mask /*host*/);

/* Activation counting: counts[e] += number of times e appears in topk_logical
 * [T, k].  counts: dev int64[E], accumulated (the caller zeroes it once; calls
 * for several batches or layers add up).  Integer adds: order-independent. */
int revive_expert_counts(revive_ctx* ctx, const int32_t* topk_logical, int32_t T, int64_t* counts, revive_stream stream);

/* ---- logical-rank compaction (Sec. 3.5) ----------------------------------- */

/* New logical ranks of a communication domain after device `failed_device`
 * fails.  logical_rank: host int32[n], in/out, -1 = device not in the domain.
 * Without a role switch (switched_device < 0) the device holding the next rank
 * takes the failed one's rank and every later rank is decremented.  With a role
 * switch, switched_device takes the failed device's rank and the gap it leaves
 * behind (if it had a rank) is closed the same way.  Pure host function, one
 * failure at a time, for a caller that renumbers a communicator. */
int revive_compact_ranks(int32_t* logical_rank /*host*/, int32_t n, int32_t failed_device, int32_t switched_device);

/* The same renumbering for the simulated ranks of a context, as device-resident
 * data: revive_update_map keeps, next to the expert map and updated by the same
 * copy, logical_rank[R] (compacted logical rank of each rank, -1 = failed; the
 * survivors keep their order, which is what removing the failed ranks one at a
 * time gives) and the number of live ranks.  A rank that comes back (role
 * switch into a failed rank's place: its slots are refilled and the rank is
 * un-failed) takes the failed rank's logical rank again.  revive_get_rank_map
 * copies the host-side table: logical_rank host int32[R], n_live_ranks host
 * int32[1]; either may be NULL. */
int revive_get_rank_map(const revive_ctx* ctx, int32_t* logical_rank /*host*/, int32_t* n_live_ranks /*host*/);

/* Compacted rank segments of a dispatched buffer (Sec. 3.5: after recovery the
 * failed ranks are no part of the layout).  slot_offsets: dev int32[P+1] as
 * written by revive_dispatch.  rank_offsets: dev int32[R+1]; for l < n_live,
 * rank_offsets[l] is the first row of the rank that holds logical rank l, so
 * that segment l is rows [rank_offsets[l], rank_offsets[l+1]); entries n_live
 * .. R hold N.  Failed ranks receive no rows, so the segments tile [0, N).
 * Reads the device-resident rank table: asynchronous on `stream`, allocates
 * nothing, capturable; a replay after revive_update_map sees the new table. */
int revive_rank_offsets(revive_ctx* ctx, const int32_t* slot_offsets, int32_t* rank_offsets, revive_stream stream);

/* ---- data path ---------------------------------------------------------- */

/* a1..a5 - Gate (Sec. 2.1), failure mask (Sec. 3.4 "Missing experts", Sec. 4.2)
 * and logical->physical remap (Sec. 3.4 "Redundant experts").
 *   x          dev [T, H] dtype
 *   w_router   dev [E, H] dtype
 *   logits     dev [T, E] fp32.  logits_given == 0: written with x * w_router^T
 *              (fp32 accumulate) and then used; != 0: read as given, x and
 *              w_router are ignored (may be NULL).
 *   topk_logical dev int32 [T, k]: chosen experts, best first; ties to the
 *              lower expert id; masked experts never appear.
 *   topk_weight  dev fp32  [T, k]: score of the chosen expert over the sum of
 *              the chosen scores, times route_scale.
 *   topk_phys    dev int32 [T, k]: slot serving the choice: the
 *              (t mod count[e])-th surviving replica of e, ascending slot id.
 * Scores: softmax over all E logits, or elementwise sigmoid.  With n_group > 1
 * the experts are split into contiguous groups, a group scores the sum of its
 * two best live scores, the topk_group best groups are kept (ties to the lower
 * group id) and the top-k is taken inside them.  Group scores are evaluated in
 * fp64; expert order is decided on the fp32 logits. */
int revive_route(revive_ctx* ctx, const void* x, const void* w_router, float* logits,
                 int32_t logits_given, int32_t T, int32_t* topk_logical, float* topk_weight,
                 int32_t* topk_phys, revive_stream stream);

/* Microbatches (Sec. 2.2): when x holds rows [first_token, first_token + T) of a
 * larger batch, the replica rule of revive_route uses the token's index in the
 * whole batch, (first_token + t) mod count[e], so that the microbatches choose
 * the very slots the undivided batch would.  Host state of the context, read
 * when revive_route is called (or recorded); default 0. */
int revive_set_token_offset(revive_ctx* ctx, int64_t first_token);

/* a6/a7 - Dispatch / A2E (Sec. 2.3): stable counting sort of the N = T*k routed
 * rows i = t*k + j by physical slot, and the row permutation.
 *   slot_offsets dev int32 [P+1]: exclusive prefix sum of rows per slot;
 *                slot_offsets[P] = N.  Slot order is rank order.
 *   dst_row      dev int32 [N]: row of x_perm that receives routed row i.
 *   src_of       dev int32 [N]: inverse (src_of[dst_row[i]] = i); ascending
 *                inside every slot.
 *   x_perm       dev [N, H] dtype: x_perm[dst_row[i], :] = x[i / k, :].
 * Deterministic: the same input gives the same indices on every call. */
int revive_dispatch(revive_ctx* ctx, const void* x, const int32_t* topk_phys, int32_t T,
                    void* x_perm, int32_t* slot_offsets, int32_t* dst_row, int32_t* src_of,
                    revive_stream stream);

/* revive_dispatch for callers that cannot allocate or bind device memory (code
 * under graph capture set up by someone else, serving loops and harnesses that
 * forbid hipMalloc): same arguments, same results, but the kernels' scratch
 * (chunk histograms and the finished-workgroup counter) is a static device
 * array inside the library instead of the bound workspace, so no workspace
 * is needed and the call allocates nothing.  The array is 256 KiB + 256 B, is
 * held by every GPU the library is loaded on until the process ends, and bounds
 * the call to T * k <= 65536 routed rows (REVIVE_EINVAL beyond that; P <= 1024
 * as everywhere).  All contexts of a device share the one array: calls of this
 * entry point that overlap in time on one GPU race, whatever their streams.
 * Capturable like revive_dispatch. */
int revive_dispatch_static(revive_ctx* ctx, const void* x, const int32_t* topk_phys, int32_t T,
                           void* x_perm, int32_t* slot_offsets, int32_t* dst_row, int32_t* src_of,
                           revive_stream stream);

/* a8 - Expert FFN (Sec. 2.1): for every slot p with rows [slot_offsets[p],
 * slot_offsets[p+1]):  y = (silu(X G_p) * (X U_p)) D_p, and the same on all T
 * rows of x for the shared expert when y_shared != NULL.
 *   w_gate_up  dev table of P dev pointers, entry p -> gate and up matrices of slot p
 *   w_down     dev table of P dev pointers, entry p -> down matrix of slot p
 *              (layouts: see the conventions at the top)
 *              entries of slots that receive no rows are never dereferenced.
 *   y_perm     dev [N, H] dtype
 *   x, w_sh_gate_up, w_sh_down (same layouts, width I_shared), y_shared [T, H]:
 *              shared expert; all four may be NULL when I_shared == 0 or the
 *              caller skips it.
 * The intermediate activation is rounded to dtype once. */
int revive_expert_ffn(revive_ctx* ctx, const void* x_perm, const int32_t* slot_offsets,
                      const void* const* w_gate_up, const void* const* w_down, void* y_perm,
                      const void* x, const void* w_sh_gate_up, const void* w_sh_down,
                      void* y_shared, int32_t T, revive_stream stream);

/* a8' - The shared expert alone: y_shared = (silu(x G_s) * (x U_s)) D_s on all T
 * rows of x.  It depends on nothing that routing produces, so a caller may
 * enqueue it on a second stream next to route/dispatch and pass y_shared = NULL
 * to revive_expert_ffn; revive_combine must then be ordered after both streams.
 * Uses its own part of the workspace (no overlap with revive_expert_ffn's). */
int revive_shared_ffn(revive_ctx* ctx, const void* x, const void* w_sh_gate_up,
                      const void* w_sh_down, void* y_shared, int32_t T, revive_stream stream);

/* a9 - Combine / E2A (Sec. 2.3): out[t, :] = sum_j topk_weight[t, j] *
 * y_perm[dst_row[t*k + j], :] (+ y_shared[t, :]); fp32 accumulation in
 * ascending j, shared expert last, one rounding to dtype.
 *   out dev [T, H] dtype;  y_shared may be NULL. */
int revive_combine(revive_ctx* ctx, const void* y_perm, const int32_t* dst_row,
                   const float* topk_weight, const void* y_shared, int32_t T, void* out,
                   revive_stream stream);

/* ---- graph replay (Sec. 3.6) -------------------------------------------- */

/* Record whatever the caller enqueues on `stream` between begin and end into a
 * graph and instantiate it once.  revive_graph_launch replays that same
 * executable; revive_update_map never invalidates it.  revive_graph_exec_id
 * returns the executable's handle value so a caller can check it is unchanged. */
int revive_graph_begin(revive_ctx* ctx, revive_stream stream);
int revive_graph_end(revive_ctx* ctx, revive_stream stream, revive_graph** out);
int revive_graph_launch(revive_graph* g, revive_stream stream);
uintptr_t revive_graph_exec_id(const revive_graph* g);
int revive_graph_destroy(revive_graph* g);

/* ---- per-kernel timing --------------------------------------------------- */

/* Kernels the library launches, for revive_kernel_time(). */
enum {
  REVIVE_K_ROUTER_GEMM = 0,
  REVIVE_K_ROUTE_TOPK,
  REVIVE_K_DISPATCH_INDEX,
  REVIVE_K_DISPATCH_PERMUTE,
  REVIVE_K_FFN_TILES,
  REVIVE_K_FFN_GATE_UP,
  REVIVE_K_FFN_DOWN,
  REVIVE_K_FFN_SHARED_GATE_UP,
  REVIVE_K_FFN_SHARED_DOWN,
  REVIVE_K_COMBINE,
  REVIVE_K_EXPERT_COUNTS,
  REVIVE_K_COUNT
};

/* With timing enabled every kernel launch outside a stream capture is
 * bracketed by a pair of HIP events on its stream.  revive_kernel_time waits
 * for the recorded events and returns the accumulated milliseconds and launch
 * count of one kernel since the last reset.  Off by default. */
int revive_set_kernel_timing(revive_ctx* ctx, int32_t enabled);
int revive_kernel_time(revive_ctx* ctx, int32_t kernel, double* total_ms /*host*/,
                       int64_t* launches /*host*/);
int revive_reset_kernel_times(revive_ctx* ctx);
const char* revive_kernel_name(int32_t kernel);

/* ---- errors ------------------------------------------------------------- */
const char* revive_last_error(const revive_ctx* ctx);
const char* revive_status_name(int status);

#ifdef __cplusplus
}
#endif
#endif /* REVIVE_H */
