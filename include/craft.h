/*
 * craft.h -- C ABI of libcraft: one expert-parallel rank's MoE layer under a CRAFT
 * replication plan, on one MI355X (gfx950).
 *
 * The calls follow the paper's statement of the problem:
 *   load profiling  (Sec. 2.3, Sec. 3.1 "expert load", Alg. 1 input W[B][L][E])
 *   planning        (Sec. 4.2 workflow steps 3-5, Alg. 1 cost model, Alg. 2, Alg. 3)
 *   execution       (Sec. 2.1: router top-K, expert FFN, weighted sum; Sec. 1: a
 *                    replicated expert's tokens are spread over its copies)
 *
 * Conventions
 *   - Plain C types only.  Every pointer is marked HOST or DEVICE.  The caller owns
 *     every buffer; the library allocates only the plan object (host memory, released
 *     by craft_plan_destroy) and never allocates or frees device memory.
 *   - `stream` arguments are hipStream_t values passed as void* (NULL = the null stream).
 *     Device entry points only enqueue work: they return after launching, do not
 *     synchronise, and report launch-time errors as CRAFT_EHIP.  Faults inside a kernel
 *     surface at the caller's next synchronisation.  The two exceptions say so below:
 *     craft_moe_rank_forward_result and craft_timing_read wait for what they read.
 *   - Every call returns a craft_status; nothing is thrown across the boundary.
 *   - Router scores must be finite (NaN is not detected; the result is then unspecified).
 *   - Row-major everywhere; [a][b] means b is contiguous.
 */
#ifndef CRAFT_H
#define CRAFT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CRAFT_OK = 0,
    CRAFT_EINVAL = -1,      /* bad argument (NULL, size out of range, misaligned, unknown table) */
    CRAFT_ENOMEM = -2,      /* host allocation failed */
    CRAFT_EHIP = -3,        /* a HIP runtime call or kernel launch failed */
    CRAFT_EWORKSPACE = -4,  /* workspace or table buffer too small */
    CRAFT_EINFEASIBLE = -5  /* the request exceeds a fixed limit of the library (the static scratch of
                               craft_moe_rank_forward_static) */
} craft_status;

const char *craft_status_str(craft_status s);

/* Element types of activations and expert weights. */
enum { CRAFT_F32 = 0, CRAFT_BF16 = 1 };

/* -------------------------------------------------------------- gating network
 * Sec. 2.1 (routing): expert scores per token come from a gating network whose form the paper
 * leaves open; this is the usual linear gate without bias,
 *   logits[t][e] = sum_h x[t][h] * w_router[e][h]   (fp32 accumulation, fp32 result).
 *   dtype     CRAFT_F32 or CRAFT_BF16: element type of x and w_router
 *   x         DEVICE [T][H], 16-byte aligned
 *   w_router  DEVICE [E][H], 16-byte aligned
 *   logits    DEVICE [T][E] fp32, fully overwritten; what craft_route_topk and
 *             craft_moe_rank_forward take as their scores
 *   workspace DEVICE, 16-byte aligned, optional: with at least
 *             craft_router_logits_workspace() bytes the contraction is split over several
 *             workgroups per tile of tokens (partial scores in the workspace, added in a
 *             fixed order by a second kernel), which is what keeps every CU busy at these
 *             shapes; NULL or too small: one workgroup per tile does the whole sum.  Either
 *             way the result depends on the arguments only, never on scheduling; the two
 *             ways round differently.  Calls that share a workspace must be ordered on
 *             one stream.
 * Limits: 1 <= E <= 1024, H >= 1, H % 8 == 0 for bf16.  T may be 0.  Asynchronous on
 * `stream`; CRAFT_EINVAL on a bad size, a NULL or a misaligned pointer.
 */
craft_status craft_router_logits_workspace(int32_t dtype, int64_t T, int32_t H, int32_t E,
                                           size_t *bytes);
craft_status craft_router_logits(int32_t dtype, const void *x, const void *w_router, int64_t T,
                                 int32_t H, int32_t E, float *logits, void *workspace,
                                 size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------ routing
 * Sec. 2.1 (routing): each token activates the K experts it scores highest.
 *   logits  DEVICE [T][E] fp32 router scores, 4-byte aligned (rows are read 16 bytes at a time
 *           when the base is 16-byte aligned and E % 4 == 0, one score at a time otherwise)
 *   ids     DEVICE [T][k] int32: expert with the (j+1)-th largest score (equal scores:
 *           lower expert id first)
 *   w       DEVICE [T][k] fp32: softmax probability of that expert over all E scores;
 *           divided by the sum over the k picked when renormalize != 0
 * Limits: 1 <= k <= E <= 1024, k <= 64.  T may be 0.
 */
craft_status craft_route_topk(const float *logits, int64_t T, int32_t E, int32_t k,
                              int32_t renormalize, int32_t *ids, float *w, void *stream);

/* ------------------------------------------------------------- load profiling
 * Sec. 3.1 "expert load", the W[B][L][E] input of Alg. 1: how many routed assignments name
 * each expert, per profiling batch and layer.
 *   topk_ids      DEVICE [L][T][k] int32 routing trace; every id must lie in [0, E):
 *                 ids outside are not counted and make the call's result unspecified
 *   batch_tokens  tokens per profiling batch; B = ceil(T / batch_tokens)
 *   counts        DEVICE [B][L][E] int64, fully overwritten
 * Limits: E <= 4096.
 */
craft_status craft_expert_load(const int32_t *topk_ids, int32_t L, int64_t T, int32_t k,
                               int32_t E, int64_t batch_tokens, int64_t *counts, void *stream);

/* Sec. 4.3 step 1, between two rebalancing windows: window[i] += counts[i] for the n int32
 * per-expert counts a forward just produced (its `counts` output, or several layers' worth
 * laid side by side).  The window is what craft_plan is fed at the next rebalancing.
 *   counts DEVICE [n] int32;  window DEVICE [n] int64, updated in place. */
craft_status craft_load_accumulate(const int32_t *counts, int64_t n, int64_t *window, void *stream);

/* -------------------------------------------------------------------- planning
 * Host-side.  Decides how many replicas each layer gets under a memory budget, which
 * experts are copied, how many experts each rank holds per layer (Alg. 3) and which rank
 * holds which copy (Sec. 4.2.2 greedy placement).
 *
 * objective 0 (default): one replica at a time to the layer with the largest reduction of
 *   the estimated maximum rank load per byte, until no further replica fits the budget.
 *   The estimate is Alg. 1's model on the aggregated load: a copy of expert e carries
 *   floor(W_s[e] / copies[e]) and a rank's load is the sum over the copies it holds.
 * objective 1: the paper's own pipeline (Sec. 4.2.1).  Alg. 1: for r = 0 and r = 1,2,4,..<=D
 *   every layer is placed on the summed loads with r replicas and every profiling batch is
 *   replayed under that placement (a copy carries floor(W[b][l][e] / copies[e])); the gain
 *   of r is the mean over batches of (average / maximum rank load) minus the same at r = 0.
 *   Alg. 2: one count per layer from {0,1,2,4,..}, summing exactly to the replica total,
 *   with the largest total gain (ties: no replica, then the smaller count).  The total is
 *   budget_bytes / bytes_per_replica, capped at what the counts can hold; a total no
 *   selection reaches falls back to the next lower reachable one.  With auto_r != 0 the
 *   total is R * D for the R >= 1, R * D <= budget, with the highest total gain per replica
 *   (step 2's automatic mode; ties: smaller R).
 * objective 2: the comparison plans of Sec. 5: every layer gets floor(budget / L) replicas
 *   (0 = placement only; budget L * D = uniform replication, one replica per layer per rank).
 * Objectives 1 and 2 count replicas: bytes_per_replica must be NULL or equal in all layers
 * (CRAFT_EINVAL otherwise).
 */
typedef struct craft_plan craft_plan_t;

typedef struct {
    int32_t L;                 /* MoE layers */
    int32_t E;                 /* logical experts per layer */
    int32_t D;                 /* expert-parallel ranks */
    int32_t gpus_per_node;     /* carried in the plan; placement is node-agnostic */
    int64_t B;                 /* profiling batches */
    const int64_t *load;       /* HOST [B][L][E] token counts, all >= 0 */
    const int64_t *bytes_per_replica; /* HOST [L], each > 0; NULL = 1 everywhere */
    int64_t budget_bytes;      /* total over all layers and ranks, >= 0 */
    int32_t objective;         /* 0, 1 or 2, see above */
    int32_t auto_r;            /* objective 1 only: choose the replication factor (see above) */
} craft_plan_params;

craft_status craft_plan(const craft_plan_params *params, craft_plan_t **out);
void craft_plan_destroy(craft_plan_t *plan);

/* Whole-plan summary: total replicas, replication factor R = total / D, and the memory
 * saving against uniform replication, L*D / total (Sec. 5.2; +inf when total is 0). */
craft_status craft_plan_summary(const craft_plan_t *plan, int32_t *L, int32_t *E, int32_t *D,
                                int64_t *total_replicas, double *replication_factor,
                                double *memory_saving_vs_uniform);

/* Per-layer figures.  est_balancedness = average / maximum estimated rank load (Sec. 3.1). */
craft_status craft_plan_layer_info(const craft_plan_t *plan, int32_t layer, int32_t *n_replicas,
                                   int32_t *n_slots, double *est_balancedness,
                                   int64_t *est_max_rank_load);

/* Per-layer tables, copied into caller HOST buffers (any may be NULL):
 *   copies        [E]    copies of each expert (1 + its replicas)
 *   slot_expert   [S]    expert held by each physical slot, S = E + n_replicas; slots are
 *                        numbered rank-major, within a rank by ascending expert id
 *   rank_slot_off [D+1]  first slot of each rank
 *   rank_load     [D]    estimated load of each rank
 */
craft_status craft_plan_layer_tables(const craft_plan_t *plan, int32_t layer, int32_t *copies,
                                     int32_t *slot_expert, int32_t *rank_slot_off,
                                     int64_t *rank_load);

/* The order in which objective 0 handed out replicas: step i gave one replica to
 * layers[i].  Returns the number of steps in *n; copies min(*n, cap) entries. */
craft_status craft_plan_greedy_order(const craft_plan_t *plan, int32_t *layers, int64_t cap,
                                     int64_t *n);

/* Objective 1's benefit matrix (Alg. 1 output) and what the allocation made of it; any
 * pointer may be NULL.  n_counts = K candidate counts; counts HOST [K] (1, 2, 4, ..);
 * base HOST [L] = mean placement-only balancedness; gain HOST [K][L]; total_gain = sum of
 * the gains of the counts Alg. 2 chose; auto_R = the replication factor the automatic
 * mode picked (0 when it was off).  K is 0 for plans of other objectives. */
craft_status craft_plan_benefit(const craft_plan_t *plan, int32_t *n_counts, int32_t *counts,
                                double *base, double *gain, double *total_gain,
                                int32_t *auto_R);

/* Rows each rank would execute for a batch with the given per-expert token counts under
 * the plan's dispatch rule (the i-th token of expert e goes to copy i mod copies[e]).
 *   counts HOST [E];  rows HOST [D];  heaviest = rank with most rows (lowest id on ties). */
craft_status craft_plan_rank_rows(const craft_plan_t *plan, int32_t layer, const int64_t *counts,
                                  int64_t *rows, int32_t *heaviest);

/* Sec. 4.3 step 3: what one rank has to do to its weights of one layer when the plan changes.
 * Slots of a rank are in ascending expert order in both plans.  A new slot whose expert the
 * rank already holds reuses that slot's weights (the j-th copy of an expert on the rank
 * matches the j-th old one); the others must be fetched from wherever the expert lives, and
 * old slots left unmatched are dropped.  Both plans must agree on L, E and D.
 *   reuse   HOST [slots of the rank in new_plan]: local index of the old slot whose weights
 *           the new slot keeps, or -1 when they must be fetched;  may be NULL
 *   n_fetch new slots to fetch;  n_drop old slots dropped;  either may be NULL */
craft_status craft_plan_diff(const craft_plan_t *old_plan, const craft_plan_t *new_plan,
                             int32_t layer, int32_t rank, int32_t *reuse, int32_t *n_fetch,
                             int32_t *n_drop);

/* Device copy of the tables one rank's forward needs.  Query the size, let the caller
 * allocate DEVICE memory (256-byte aligned), upload once, and pass the pointer to every
 * forward of that (plan, layer, rank).  The plan remembers which buffers it filled; a
 * forward given any other pointer returns CRAFT_EINVAL.  The copy is enqueued on `stream`
 * (no synchronisation) from pageable host memory that belongs to the plan, so the plan has to
 * outlive it; a forward enqueued later on the same stream sees the tables.  A buffer may be
 * filled again, also for another (layer, rank): it then counts for the last one only.
 * Uploads belong to set-up: the host memory is pageable, so do not record one into a stream
 * capture. */
craft_status craft_plan_tables_bytes(const craft_plan_t *plan, int32_t layer, int32_t rank,
                                     size_t *bytes);
craft_status craft_plan_tables_upload(craft_plan_t *plan, int32_t layer, int32_t rank,
                                      void *dev_tables, size_t bytes, void *stream);

/* --------------------------------------------------------------- weight packing
 * One-time re-ordering of one expert's bf16 weights into the order the grouped-GEMM
 * kernels stream them in (MFMA operand fragments: 64 lanes x 16 bytes per 16-row x
 * 32-element block; the 16 gate rows of a group of output columns followed by the 16 up
 * rows of the same columns; rows and contraction padded with zeros to whole blocks).  It
 * belongs to model loading,
 * like placing the weights in HBM, and is not part of a forward.
 *   w_gate, w_up  DEVICE [I][H] bf16;  w_down DEVICE [H][I] bf16 (Sec. 2.1: up-projection,
 *                 non-linearity, down-projection)
 *   packed_gateup, packed_down  DEVICE buffers of the sizes craft_pack_weights_bytes
 *                 returns, 16-byte aligned, written in full
 * dtype must be CRAFT_BF16 (fp32 weights are always read row-major); H % 8 == 0, I % 8 == 0.
 */
craft_status craft_pack_weights_bytes(int32_t dtype, int32_t H, int32_t I, size_t *gateup_bytes,
                                      size_t *down_bytes);
craft_status craft_pack_weights(int32_t dtype, int32_t H, int32_t I, const void *w_gate,
                                const void *w_up, const void *w_down, void *packed_gateup,
                                void *packed_down, void *stream);

/* ------------------------------------------------------------- 8-bit expert weights
 * Not in the paper: the bytes of a replica are what its memory budget is spent on, and the
 * slots with few rows are bound by streaming their weights, so the packed FFN can also run
 * on weights stored as OCP FP8 E4M3 codes (1 sign, 4 exponent bits with bias 7, 3 mantissa
 * bits; no infinities; largest finite value 448) with one fp32 scale per weight row.  The
 * codes are widened to bf16 in registers (exactly) in front of the same bf16 MFMA, and the
 * scales are applied to the fp32 accumulators.
 *
 * craft_quantize_e4m3: scale[r] = max_k |w[r][k]| / 448 in fp32 (1 for an all-zero row);
 *   codes[r][k] = the E4M3 value nearest to the fp32 quotient w[r][k] / scale[r], ties to the
 *   even mantissa, the sign bit kept.
 *     w DEVICE [rows][K] bf16;  codes DEVICE [rows][K] uint8;  scale DEVICE [rows] fp32;  K % 8 == 0
 * craft_pack_weights_e4m3: the codes of one expert into the streaming order of
 *   craft_pack_weights (8 bytes per lane instead of 16), the scales appended to the buffers.
 *     gate/up codes DEVICE [I][H], down codes DEVICE [H][I]; scales [I], [I], [H]
 *     packed buffers DEVICE, 16-byte aligned, of craft_pack_weights_e4m3_bytes() bytes
 */
craft_status craft_quantize_e4m3(const void *w, int64_t rows, int32_t K, uint8_t *codes,
                                 float *scale, void *stream);
craft_status craft_pack_weights_e4m3_bytes(int32_t H, int32_t I, size_t *gateup_bytes,
                                           size_t *down_bytes);
craft_status craft_pack_weights_e4m3(int32_t H, int32_t I, const uint8_t *gate_codes,
                                     const uint8_t *up_codes, const uint8_t *down_codes,
                                     const float *gate_scale, const float *up_scale,
                                     const float *down_scale, void *packed_gateup,
                                     void *packed_down, void *stream);

/* ------------------------------------------------------------------- execution
 * One rank's share of one MoE layer (Sec. 2.1) under the plan:
 *   1 route       ids, w = top-k of logits                         (as craft_route_topk)
 *   2 load        counts[e] = assignments naming expert e
 *   3 dispatch    assignment a = t*k+j, the i-th naming expert e, goes to that expert's
 *                 copy (i mod copies[e]); dest[a] = position in the slot-ordered
 *                 permutation, src = inverse of dest
 *   4 expert FFN  for each slot of this rank, rows R of its tokens:
 *                 Y = (silu(R Wg^T) * (R Wu^T)) Wd^T, fp32 accumulation
 *   5 combine     out[t] = sum over this rank's assignments of token t, j ascending, of
 *                 w[t][j] * Y[row of (t,j)]; tokens with none get zeros
 *
 *   x        DEVICE [T][H] activations, dtype
 *   logits   DEVICE [T][E] fp32 router scores (aligned as for craft_route_topk), or NULL: then
 *            the forward computes them first,
 *            as craft_router_logits does (with its workspace), from
 *   w_router DEVICE [E][H] gate weights, dtype (ignored when logits is given)
 *   w_gate, w_up  DEVICE arrays of s device pointers, one per slot of this rank in slot
 *                 order, each to a [I][H] matrix of dtype
 *   w_down        likewise, each [H][I]
 *   w_gateup_packed, w_down_packed  DEVICE arrays of s device pointers to the buffers
 *                 craft_pack_weights filled for each slot's expert.  When both are given
 *                 (bf16 only) the FFN streams these and w_gate / w_up / w_down may be NULL;
 *                 when NULL the FFN reads the row-major matrices.  The streaming kernels
 *                 address token rows and weight fragments by 32-bit byte offsets: x (T * H
 *                 elements) and each packed matrix must stay below 4 GiB, else CRAFT_EINVAL.
 *   weight_format of the packed buffers: CRAFT_W_BF16 (craft_pack_weights) or CRAFT_W_E4M3
 *                 (craft_pack_weights_e4m3)
 *   out      DEVICE [T][H] dtype, fully overwritten
 *   ids, topk_w, dest, src  optional DEVICE outputs [T][k] (int32/fp32/int32/int32);
 *                 NULL = kept in the workspace only
 *   counts   optional DEVICE output [E] int32
 *   slot_cnt, slot_off  optional DEVICE outputs [S] / [S+1] int32 over all slots
 *   max_rows rows the staging buffers are sized for.  0 = the worst case
 *            T * min(k, s).  If the batch routes more rows than this to the rank the
 *            forward does no FFN work, zero-fills out and sets the overflow flag.
 *   tile_rows_gateup, tile_rows_down, riders_gateup, riders_down  tuning knobs of the packed
 *            FFN, normally 0: see craft_moe_rank_forward_tiles for what the library picks by
 *            itself
 *   workspace DEVICE, 256-byte aligned, at least craft_moe_rank_forward_workspace() bytes.
 *            Forwards that share a workspace must be ordered on one stream.
 * Alignment: x, out and all weight matrices 16-byte aligned; H % 8 == 0 and I % 8 == 0
 * for bf16 (H % 4, I % 4 for fp32).
 * Limits: T*k < 2^31, k <= 64, E <= 1024, slots of one rank <= 1024.
 */
enum { CRAFT_W_BF16 = 0, CRAFT_W_E4M3 = 1 };

typedef struct {
    int32_t dtype;
    int64_t T;
    int32_t H, I, k;
    int32_t renormalize;
    const void *x;
    const float *logits;
    const void *w_router;
    const void *const *w_gate;
    const void *const *w_up;
    const void *const *w_down;
    const void *const *w_gateup_packed;
    const void *const *w_down_packed;
    int32_t weight_format;
    void *out;
    int32_t *ids;
    float *topk_w;
    int32_t *dest;
    int32_t *src;
    int32_t *counts;
    int32_t *slot_cnt;
    int32_t *slot_off;
    int64_t max_rows;
    int32_t tile_rows_gateup;  /* packed weights only: rows per row-tile of the gate/up GEMM, */
    int32_t tile_rows_down;    /* of the down GEMM: 128, 160, .., 256; 0 = chosen by the library */
    int32_t riders_gateup;     /* packed weights only: slots with at most 64 rows ride along with the */
    int32_t riders_down;       /* tiles of busy slots: 1 = wherever tiles are at most 224 rows, -1 = never,
                                  0 = chosen by the library */
    const void *tables;        /* from craft_plan_tables_upload */
    void *workspace;
    size_t workspace_bytes;
} craft_fwd_args;

craft_status craft_moe_rank_forward_workspace(const craft_plan_t *plan, int32_t layer,
                                              int32_t rank, const craft_fwd_args *args,
                                              size_t *bytes);
craft_status craft_moe_rank_forward(const craft_plan_t *plan, int32_t layer, int32_t rank,
                                    const craft_fwd_args *args, void *stream);

/* The same forward for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc) and have no workspace to
 * hand in: everything craft_moe_rank_forward keeps in `workspace` lives in a device array of
 * CRAFT_STATIC_SCRATCH_BYTES that is part of the library (each GPU the library runs on holds
 * its own copy until the process ends).  args->workspace and args->workspace_bytes are
 * ignored; every other argument, the kernels and the results are those of
 * craft_moe_rank_forward.  Neither this call nor anything it launches allocates or frees
 * device memory; the first forward of a new (T, k, H, I) on a (layer, rank) notes its tile
 * choice in the plan (a few bytes of host memory), and the first call on a device looks up
 * the array's address there (make that call outside a capture).
 *   CRAFT_EINFEASIBLE when craft_moe_rank_forward_workspace() for these arguments exceeds
 *   CRAFT_STATIC_SCRATCH_BYTES (checked on the host before anything is launched: lower
 *   max_rows or T); the other errors as craft_moe_rank_forward.
 * All calls on one GPU share that GPU's array and the array keeps the last call's contents:
 * forwards through this entry point must be ordered on one stream (calls that overlap on
 * one GPU race), and craft_moe_rank_forward_result has no workspace pointer to read here
 * (rows routed to the rank = slot_off[last slot of the rank + 1] - slot_off[its first slot]
 * from the optional slot_off output; on overflow `out` is all zeros). */
#define CRAFT_STATIC_SCRATCH_BYTES (64u << 20)
craft_status craft_moe_rank_forward_static(const craft_plan_t *plan, int32_t layer, int32_t rank,
                                           const craft_fwd_args *args, void *stream);

/* How forwards with these arguments cut the two grouped GEMMs into tiles: the most rows a
 * row-tile gets (a multiple of 32), and whether the slots with few rows are carried along by
 * the tiles of the busy slots (1) or get tiles of their own (0).  With packed weights both
 * are chosen per (plan, layer, rank, T, k, H, I) from the loads the plan was made from, by
 * playing the launch through against a cost model, so that the tiles of the busy slots fill
 * the CUs in whole rounds; the choice is kept in the plan.  Any output pointer may be NULL.
 * Host-side, no device work. */
craft_status craft_moe_rank_forward_tiles(const craft_plan_t *plan, int32_t layer, int32_t rank,
                                          const craft_fwd_args *args, int32_t *rows_gateup,
                                          int32_t *rows_down, int32_t *riders_gateup,
                                          int32_t *riders_down);

/* After the caller has synchronised the stream: what the last forward on this workspace
 * found.  rows = rows routed to the rank; overflow != 0 when rows > max_rows (nothing was
 * computed).  Copies 16 bytes from the device with a blocking copy on the null stream: this
 * call synchronises, and must not be made while a stream is capturing. */
craft_status craft_moe_rank_forward_result(const void *workspace, int64_t *rows,
                                           int32_t *overflow);

/* ------------------------------------------------------------ kernel timing
 * Optional HIP-event timing of the kernels inside craft_moe_rank_forward, recorded on the
 * stream the kernels run on.  level 0 = off, 1 = the grouped gate/up GEMM only, 2 = every
 * kernel.  Events come from a pool created here (max_forwards forwards can be recorded
 * between two reads).  craft_timing_read synchronises the recorded events, returns the
 * summed milliseconds and the number of launches per kernel, and rewinds the pool.
 */
enum {
    CRAFT_K_ROUTE = 0,     /* top-k + per-block ranks */
    CRAFT_K_SCAN = 1,      /* per-expert scan, slot offsets */
    CRAFT_K_DISPATCH = 2,  /* dest / src, tile tables of the GEMMs */
    CRAFT_K_GATEUP = 3,    /* grouped gate/up GEMM + SwiGLU (gathers its rows) */
    CRAFT_K_DOWN = 4,      /* grouped down GEMM */
    CRAFT_K_COMBINE = 5,   /* weighted combine */
    CRAFT_K_GATE = 6,      /* gating network, when the forward computes the scores itself */
    CRAFT_K_COUNT = 7
};
craft_status craft_timing_enable(int32_t level, int32_t max_forwards);
craft_status craft_timing_read(double ms[CRAFT_K_COUNT], int64_t launches[CRAFT_K_COUNT]);

/* ------------------------------------------------------------ measurement probes
 * Not part of the method: kernels of known work, so that a benchmark can report this
 * machine's own ceilings next to the published ones and scale memory counters.
 * craft_probe_copy: dst[i] = src[i] for `bytes` bytes (a multiple of 16; both DEVICE, 16-byte
 *   aligned, not overlapping): reads `bytes` and writes `bytes`, nothing else.
 * craft_probe_mfma_bf16: blocks x 4 wavefronts each issue iters x 4 independent
 *   v_mfma_f32_32x32x16_bf16 on register operands (no memory traffic but the final store of one
 *   float per thread to sink, DEVICE [blocks * 256]); *flops = the floating-point operations
 *   the launch performs (2 * 32 * 32 * 16 per MFMA).  blocks = 0: two per compute unit.
 * craft_probe_read: each of `blocks` workgroups (0: eight per compute unit) reads all of src
 *   (`bytes`, a multiple of 32 KiB, DEVICE, 16-byte aligned) `passes` times and stores one
 *   word per thread to sink (DEVICE [blocks * 256] uint32); *bytes_read = what the launch
 *   requests in total.  With a buffer of a megabyte or two, which the L2 of every XCD holds
 *   and the L1 of a compute unit does not, this measures what all compute units together
 *   can pull out of L2.
 * craft_probe_mfma_operands: the matrix rate as a function of the operands' contents and of
 *   the instruction's shape (the clock the chip sustains depends on both).  blocks x 4
 *   wavefronts (blocks = 0: one workgroup per compute unit), each with the register shape of
 *   an FFN tile (2 x 8 operand fragments per step, 256 accumulator registers), issue per
 *   iteration the work of 32 products of 32 x 32 x 16 as
 *     shape 0: v_mfma_f32_32x32x16_bf16    shape 1: v_mfma_f32_16x16x32_bf16
 *   on operands holding
 *     data 0: zeros    1: the values 1.0 and 1.5    2: random signs and mantissas, exponents
 *     spread over eight binades below 1
 *   sink DEVICE [blocks * 256] float; *flops as for craft_probe_mfma_bf16.
 * All only enqueue on `stream`; time them with events on that stream. */
craft_status craft_probe_copy(const void *src, void *dst, int64_t bytes, void *stream);
craft_status craft_probe_read(const void *src, int64_t bytes, int32_t passes, int32_t blocks,
                              uint32_t *sink, double *bytes_read, void *stream);
craft_status craft_probe_mfma_bf16(int32_t blocks, int32_t iters, float *sink, double *flops,
                                   void *stream);
craft_status craft_probe_mfma_operands(int32_t shape, int32_t data, int32_t blocks, int32_t iters,
                                       float *sink, double *flops, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CRAFT_H */
