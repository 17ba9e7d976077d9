/*
 * moe_janus.h - C ABI of the MI355X (gfx950) MoE-instance layer step.
 *
 * One MoE instance of a disaggregated MoE deployment runs, per layer and per decode
 * batch (Janus, arXiv 2512.13525, Sec. 3.4, "Scheduling workflow"):
 *
 *   moe_route        gating selection on the MoE side          (Sec. 3.3 "Gating on the MoE side")
 *   moe_schedule     Activated-Expert-Balanced Scheduling       (Sec. 3.4, Alg. 1, Steps 1-3)
 *   moe_permute      this instance's share of the dispatch      (Sec. 3.4, Step 4)
 *   moe_grouped_ffn  expert FFN over the activated experts only (Sec. 2.2, roofline paragraph)
 *   moe_combine      weighted top-k combine, instance-partial   (Sec. 3.3, reverse path)
 *
 * Conventions
 *   - Pointers named *_dev are device pointers owned by the caller; *_host are host
 *     pointers.  The library never frees or reallocates caller memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every
 *     compute call only enqueues work on `stream`: it does not synchronise, does not
 *     allocate and does not read results back to the host, so a whole layer step can be
 *     queued without CPU-GPU synchronisation (Sec. 3.4, "Synchronization-free scheduling").
 *   - All matrices are row-major and densely packed unless stated otherwise.
 *   - Every function returns MOE_OK (0) or a negative error code.  Arguments are checked
 *     on the host before anything is launched; device-resident values (expert ids, replica
 *     ids) are trusted.  moe_strerror() describes a code; moe_last_error() adds the HIP
 *     error text of the calling thread's most recent MOE_EHIP.
 *   - Calls that share output or workspace buffers must be ordered by the caller (same
 *     stream or events).  A placement object is immutable and may be shared.
 *
 * Symbols (paper notation): T tokens, k experts per token, E logical experts, n_inst MoE
 * instances (n_e), C replica slots per instance, d_h hidden size, d_e expert intermediate
 * size.  A request is the pair p = i*k + j (token i, choice j).  The physical replica id
 * (RID) of slot s on instance g is g*C + s.
 */
#ifndef MOE_JANUS_H
#define MOE_JANUS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_OK           0
#define MOE_EINVAL     (-1)   /* null or misaligned pointer, non-positive or inconsistent size */
#define MOE_ESHAPE     (-2)   /* a size the kernels do not support (see each call) */
#define MOE_EPLACEMENT (-3)   /* invalid replica layout */
#define MOE_EHIP       (-4)   /* a HIP runtime call or kernel launch failed */
#define MOE_ENOMEM     (-5)   /* host or device allocation failed (placement create only) */
#define MOE_EWORKSPACE (-6)   /* workspace_bytes smaller than moe_workspace_bytes() */

#define MOE_DTYPE_BF16 0
#define MOE_DTYPE_F32  1

#define MOE_ROUTE_SOFTMAX        0
#define MOE_ROUTE_SIGMOID_GROUP  1

#define MOE_MAX_EXPERTS    1024   /* E */
#define MOE_MAX_INSTANCES    64   /* n_inst */
#define MOE_MAX_SLOTS       256   /* C */
#define MOE_MAX_TOPK         32   /* k */
#define MOE_FFN_BLOCK_ROWS   64   /* most request rows of one slot per entry of the FFN work list */

const char *moe_strerror(int code);
const char *moe_last_error(void);

/* ------------------------------------------------------------------ replica layout
 * The layout is what the MoE controller distributes at reconfiguration time (Sec. 3.4:
 * "replica layout" metadata, updated on the order of hours; Appendix B).  It fixes
 * R(e), G(e) and P(e,g) of Alg. 1's input list.
 *
 * slot_to_expert_host[g*C + s] = logical expert held by slot s of instance g, or -1 for
 * an empty slot.  Rejected with MOE_EPLACEMENT: an expert without any replica, an expert
 * with two replicas on one instance, an id outside [-1, E).  Limits (MOE_ESHAPE):
 * E <= MOE_MAX_EXPERTS, n_inst <= MOE_MAX_INSTANCES, C <= MOE_MAX_SLOTS.
 *
 * The object owns small host and device tables on the device that is current at create
 * time; create and destroy synchronise with the device (they are not on the hot path).
 */
typedef struct moe_placement moe_placement_t;

int  moe_placement_create(moe_placement_t **out, int E, int n_inst, int C,
                          const int32_t *slot_to_expert_host);
void moe_placement_destroy(moe_placement_t *pl);
/* Host-side queries (no device access): replica count R(e), and layout sizes. */
int  moe_placement_replicas(const moe_placement_t *pl, int e);
int  moe_placement_dims(const moe_placement_t *pl, int *E, int *n_inst, int *C);

/* ------------------------------------------------------------------ a0: gating selection
 * Sec. 3.4, first step of the scheduling workflow: the gate yields, per token, the k logical
 * expert ids that the scheduler then maps to replicas.  The score function is a property of
 * the model, not of the paper:
 *   MOE_ROUTE_SOFTMAX        ids = the k largest logits (largest first; equal logits:
 *                            lower id first); w = softmax over all E logits gathered at
 *                            ids, rescaled to sum to 1 when renormalize != 0.
 *   MOE_ROUTE_SIGMOID_GROUP  s = sigmoid(logit); E/n_group contiguous experts per group;
 *                            group score = sum of its two largest s; the topk_group best
 *                            groups survive (lower group id on ties); ids = the k largest
 *                            logits among surviving experts; w = s / sum(selected s) * scale.
 * logits_dev [T,E] float32 -> topk_ids_dev [T,k] int32, topk_w_dev [T,k] float32.
 * Limits: 1 <= k <= min(E, MOE_MAX_TOPK); E <= MOE_MAX_EXPERTS; group mode needs
 * E % n_group == 0, E/n_group >= 2, k <= topk_group*E/n_group, n_group <= 64.  T == 0 is a no-op.
 */
typedef struct moe_route_cfg {
    int   mode;          /* MOE_ROUTE_* */
    int   renormalize;   /* softmax mode only */
    int   n_group;       /* group mode only */
    int   topk_group;    /* group mode only */
    float scale;         /* group mode only */
} moe_route_cfg;

int moe_route(const float *logits_dev, int T, int E, int k, const moe_route_cfg *cfg,
              int32_t *topk_ids_dev, float *topk_w_dev, void *stream);

/* ------------------------------------------------------------------ a1-a3: Alg. 1
 * Step 1 collects the set of activated experts, Step 2 seats every activated
 * single-replica expert on its only host and then every activated multi-replica expert,
 * in ascending expert id, on its least-loaded host (load = activated experts seated on the
 * instance so far in this layer; ties: lowest instance), Step 3 rewrites each request.
 *
 * topk_ids_dev [T,k] int32 (values in [0,E)) ->
 *   rid_dev     [T,k] int32  O(i,j): replica id chosen for request (i,j)
 *   act_rep_dev [E]   int32  actRep[e], -1 for experts not activated
 *   load_dev    [n_inst] int32  activated experts per instance; max = a_max
 * The result depends only on the layout and the set of activated experts, so every
 * instance that runs this call on the same inputs obtains the same schedule.
 * T == 0 yields act_rep = -1, load = 0.  k <= MOE_MAX_TOPK.
 */
int moe_schedule(const moe_placement_t *pl, const int32_t *topk_ids_dev, int T, int k,
                 int32_t *rid_dev, int32_t *act_rep_dev, int32_t *load_dev, void *stream);

/* ------------------------------------------------------------------ baseline policies
 * The two policies AEBS is compared with (Sec. 5, the a_max study): MOE_POLICY_HOME sends every
 * request of expert e to e's first replica (lowest instance: no scheduling at all);
 * MOE_POLICY_RANDOM sends request p to replica number draws[p] mod R(e) of e, replicas counted
 * in ascending instance order (balances tokens, not activated experts; the caller supplies the
 * draws, uint32 [T*k]; NULL for MOE_POLICY_HOME).
 *   rid_dev  [T*k]    int32  replica id per request
 *   load_dev [n_inst] int32  distinct replicas per instance that received a request; max = a_max
 */
#define MOE_POLICY_HOME   0
#define MOE_POLICY_RANDOM 1
int moe_schedule_baseline(const moe_placement_t *pl, const int32_t *topk_ids_dev, int T, int k,
                          int policy, const uint32_t *draws_dev, int32_t *rid_dev, int32_t *load_dev,
                          void *stream);

/* ------------------------------------------------------------------ batched scheduling
 * Sec. 3.5: the scaling model reads a table a_max(n_e, B) estimated by Monte-Carlo sampling:
 * batches of B tokens are drawn, scheduled, and the largest per-instance count is averaged.
 * These two calls schedule n_batches independent batches of T tokens each in ONE launch (one
 * workgroup per batch, the same code as moe_schedule / moe_schedule_baseline, same results bit
 * for bit per batch):
 *   topk_ids_dev [n_batches, T, k] -> load_dev [n_batches, n_inst]   (max over instances = a_max of the batch)
 *   rid_dev [n_batches, T, k] and act_rep_dev [n_batches, E] are optional (NULL = not written);
 *   draws_dev [n_batches, T, k] for MOE_POLICY_RANDOM.
 * n_batches == 0 is a no-op.
 */
int moe_schedule_batched(const moe_placement_t *pl, const int32_t *topk_ids_dev, int n_batches, int T, int k,
                         int32_t *rid_dev, int32_t *act_rep_dev, int32_t *load_dev, void *stream);
int moe_schedule_baseline_batched(const moe_placement_t *pl, const int32_t *topk_ids_dev, int n_batches, int T, int k,
                                  int policy, const uint32_t *draws_dev, int32_t *rid_dev, int32_t *load_dev,
                                  void *stream);

/* ------------------------------------------------------------------ a4: dispatch (Step 4)
 * Keeps the requests whose replica lives on instance g_self and groups them by local slot
 * s = rid - g_self*C, ascending request id inside a slot (a stable grouping: the output is
 * unique).
 *   slot_count_dev [C]    int32  requests per local slot
 *   slot_off_dev   [C+1]  int32  exclusive scan of slot_count; slot_off[C] = n_local
 *   perm_dev       [T*k]  int32  capacity T*k; the first n_local entries are request ids
 *   pos_dev        [T*k]  int32  pos[p] = row of request p in perm, or -1 if p is not local
 *   blocks_dev     [moe_block_list_len(T, k, C)] int32, 16-byte aligned: the work list of
 *                  moe_grouped_ffn.  The rows of every slot are cut into blocks of at most
 *                  R = moe_block_rows(T) rows (32 for small batches, MOE_FFN_BLOCK_ROWS otherwise);
 *                  slots with more than 16 requests come first (their work takes longest),
 *                  ascending slot order otherwise.  Four int32 per entry: entry 0 = {number of
 *                  blocks B, R, number of 64-row blocks and number of 128-row blocks that the slots
 *                  with more than 64 requests make}; entry 1+j = {slot, first row of the block, slot_off[slot+1], slot_off[slot]}.
 *                  Entries past B are left untouched.
 * n_local and B stay on the device; nothing is read back.  The grouped FFN cannot size its
 * launch by them, so it sizes it for moe_max_blocks() and lets the surplus leave at once.
 * rid_dev may hold any values: entries outside [g_self*C, (g_self+1)*C) are simply not local, and
 * a token may name one slot several times (the list never exceeds moe_max_blocks()).
 */
int moe_permute(const moe_placement_t *pl, int g_self, const int32_t *rid_dev, int T, int k,
                int32_t *slot_count_dev, int32_t *slot_off_dev, int32_t *perm_dev,
                int32_t *pos_dev, int32_t *blocks_dev, void *stream);

/* Largest number of blocks a batch of T tokens can produce on an instance with C slots, whatever
 * the request ids are (C + T*k / R: one partly filled block per slot plus the full ones), and
 * the int32 length of blocks_dev. */
int moe_block_rows(int T);
size_t moe_max_blocks(int T, int k, int C);
size_t moe_block_list_len(int T, int k, int C);

/* ------------------------------------------------------------------ a0-a4 in one launch
 * Same results, bit for bit, as moe_route + moe_schedule + moe_permute called one after the
 * other with the same arguments (E is the placement's).  At decode sizes each of those steps is a
 * few microseconds of work behind a launch of similar cost; this entry point pays one launch.
 * sync_dev: moe_front_sync_len() int32 of device memory, zero before the first call; every call
 * leaves its first 33 words zero (the rest is scratch).  Calls that share sync_dev must not overlap
 * in time.  Up to 8192 requests (T*k) the call is one launch and sync_dev is one word; larger
 * batches take three launches: the routing workgroups collect the activated experts in a bitset
 * (Alg. 1, Step 1, token-parallel), the last of them runs Step 2, and Step 3 and the sort run
 * over chunks of 2048 requests, one workgroup each (per-chunk counts, then the scatter; no
 * ordering comes from atomics).
 */
size_t moe_front_sync_len(const moe_placement_t *pl, int T, int k);
int moe_route_schedule_permute(const moe_placement_t *pl, int g_self, const float *logits_dev, int T, int k,
                               const moe_route_cfg *cfg, int32_t *topk_ids_dev, float *topk_w_dev,
                               int32_t *rid_dev, int32_t *act_rep_dev, int32_t *load_dev,
                               int32_t *slot_count_dev, int32_t *slot_off_dev, int32_t *perm_dev,
                               int32_t *pos_dev, int32_t *blocks_dev, int32_t *sync_dev, void *stream);

/* ------------------------------------------------------------------ replica management (host)
 * Appendix B ("Activation-Aware Replica Placement").  Host-only, sequential, no GPU work: they
 * run when the layout is rebuilt, and their result goes to moe_placement_create.  All pointers
 * are HOST pointers.
 *
 * moe_coactivation_counts: window statistics from a trace of batches.  ids_host
 *   [n_batches][batch_pairs] int32 expert ids (the T*k selections of each batch);
 *   c_host_out [E] double = number of batches that activate e; a_host_out [E*E] double,
 *   symmetric, zero diagonal = number of batches that activate both.  MOE_EINVAL on an id
 *   outside [0, E).
 * moe_replica_counts: one replica per expert, then each of the n_inst*C - E spare slots goes to
 *   the expert with the largest c(e)/R(e) that has fewer than n_inst replicas (lower id on
 *   ties).  R_host_out [E] int32.  MOE_EPLACEMENT if n_inst*C < E.
 * moe_place_replicas: Alg. 3.  Replicas in decreasing order of c(e)/R(e) (then expert id); each
 *   goes to the instance with room that does not host its expert and adds the smallest
 *   sum of a(e, e') over the experts already there (lowest instance on ties); if no such
 *   instance exists, the cheapest swap (replica j of an instance g without e moves to an
 *   instance h with room, e takes its slot) by change of summed co-activation load.
 *   a_host [E*E] symmetric; slot_to_expert_host_out [n_inst*C] int32 in placement order, -1 =
 *   empty.  MOE_EPLACEMENT if R(e) < 1, R(e) > n_inst, sum R > n_inst*C, or no swap exists.
 */
int moe_coactivation_counts(const int32_t *ids_host, int n_batches, int batch_pairs, int E,
                            double *c_host_out, double *a_host_out);
int moe_replica_counts(int E, int n_inst, int C, const double *c_host, int32_t *R_host_out);
int moe_place_replicas(int E, int n_inst, int C, const int32_t *R_host, const double *c_host,
                       const double *a_host, int32_t *slot_to_expert_host_out);

/* ------------------------------------------------------------------ resource scaling (host)
 * Sec. 3.5 ("Fine-Grained Scaling under SLOs"), Alg. 2.  Host-only.  For every (n_a, n_e) in
 * {1..n_max} x {ne_min..n_max} whose n_e is on the table's grid: the steady-state batch B* of
 * Eq. 2 (B = lambda * TPOT(B); B* = 1 if the load is too light, candidate dropped if B_max cannot
 * sustain it, else 60 bisections of the residual on [1, B_max]), TPOT by Eq. 1a-1c, the SLO and the
 * attention-side memory check; the feasible candidate with the fewest GPUs wins (first in
 * enumeration order on ties).  All L layers share the coefficients; times in one unit of the
 * caller's choice (lambda in requests per that unit).
 *   TPOT = L * ( max(c_a, alpha*b + c_kv*b*S_ctx) + beta*a_max(n_e, B) + c_e + comm0 + comm1*B ),  b = B/n_a
 *   memory: mem_fixed + mem_per_token * b * S_ctx <= mem_budget
 *   amax_table_host [n_ne][n_B]: a_max on the grid ne_values_host x B_values_host (ascending B);
 *   linear interpolation in B, clamped at the ends.
 * Outputs (host): n_a, n_e, B*, TPOT of the choice; n_a = n_e = 0 if nothing is feasible (still MOE_OK).
 */
typedef struct {
    int L;
    double c_a, alpha, c_kv;       /* attention side, Eq. 1b */
    double beta, c_e;              /* MoE side, Eq. 1c */
    double comm0, comm1;           /* communication per layer: comm0 + comm1 * B */
    double S_ctx;
    double mem_budget, mem_fixed, mem_per_token;
} moe_scaling_model;
int moe_scaling_solve(const moe_scaling_model *m, const double *amax_table_host, const int *ne_values_host, int n_ne,
                      const double *B_values_host, int n_B, double lambda, double slo, int n_max, int ne_min,
                      double B_max, int *n_a_out, int *n_e_out, double *B_star_out, double *tpot_out);

/* ------------------------------------------------------------------ the gate in the same launch
 * Sec. 3.3 ("gating on the MoE side"): the MoE instance receives the complete activations and
 * runs the gate itself.  These two entry points start from the activations instead of from
 * logits: logits[i, e] = sum_c X[i, c] * W_r[e, c] (+ bias[e]), bf16 operands, fp32 products
 * and sums (MFMA), then the selection of moe_route on those fp32 logits, in one launch;
 * moe_gate_route_schedule_permute continues through Alg. 1 and the dispatch exactly like
 * moe_route_schedule_permute.
 *   X_dev      [T, d_h] bf16, row-major, 16-byte aligned
 *   Wr_dev     [E, d_h] bf16, row-major (one row per logical expert), 16-byte aligned
 *   bias_dev   [E] float, or NULL
 *   logits_dev [T, E] float, OUTPUT (the selection reads it back inside the launch)
 *   sync_dev   moe_gate_sync_len(T) int32, zero before the first call; every call leaves them
 *              zero.  Calls that share sync_dev must not overlap in time.
 * Needs d_h % 32 == 0 (MOE_ESHAPE otherwise).  The sum over c is taken in a fixed order
 * (16 contiguous shares of the hidden dimension, added in ascending order), so results are
 * reproducible; it is not the order of a sequential dot product, so a logit can differ from one
 * in the last bits and a selection between logits closer than that can differ too.
 */
size_t moe_gate_sync_len(int T);
int moe_gate_route(const void *X_dev, const void *Wr_dev, const float *bias_dev, int T, int E, int d_h, int k,
                   const moe_route_cfg *cfg, float *logits_dev, int32_t *topk_ids_dev, float *topk_w_dev,
                   int32_t *sync_dev, void *stream);
int moe_gate_route_schedule_permute(const moe_placement_t *pl, int g_self, const void *X_dev, const void *Wr_dev,
                                    const float *bias_dev, int T, int d_h, int k, const moe_route_cfg *cfg,
                                    float *logits_dev, int32_t *topk_ids_dev, float *topk_w_dev,
                                    int32_t *rid_dev, int32_t *act_rep_dev, int32_t *load_dev,
                                    int32_t *slot_count_dev, int32_t *slot_off_dev, int32_t *perm_dev,
                                    int32_t *pos_dev, int32_t *blocks_dev, int32_t *sync_dev, void *stream);

/* ------------------------------------------------------------------ expert weights
 * Canonical layout of one instance's physical experts (what a checkpoint holds):
 *   W13 [C, 2*d_e, d_h]  rows 0..d_e-1 = gate projection, rows d_e..2*d_e-1 = up projection
 *   W2  [C, d_h, d_e]    down projection
 * MOE_DTYPE_F32 consumes the canonical layout directly.  MOE_DTYPE_BF16 consumes a
 * tile-packed copy made once when the replica is pinned (weights are static for hours,
 * Sec. 3.4): every 16-row x 32-column tile is stored as the 1 KiB register image of one
 * wavefront, so that the FFN kernel streams each expert with fully coalesced 128-bit
 * loads.  moe_pack_weights_bf16 converts canonical -> packed on the device
 * (dst and src must not overlap; sizes in elements are equal).
 * The packed W2 groups output channels in pairs of 16-row tiles.
 * Needs d_h % 32 == 0 and d_e % 32 == 0 (MOE_ESHAPE otherwise).
 */
int moe_pack_weights_bf16(const void *W13_dev, const void *W2_dev, int C, int d_h, int d_e,
                          void *W13_packed_dev, void *W2_packed_dev, void *stream);

/* ------------------------------------------------------------------ a5: grouped expert FFN
 * For every local slot s with slot_count[s] > 0 and every request row r in
 * [slot_off[s], slot_off[s+1]), token i = perm[r] / k:
 *     h = Wgate_s x_i, u = Wup_s x_i, a = h/(1+exp(-h)) * u, Yp[r,:] = Wdown_s a.
 * Slots without requests are skipped and their weights are never read, so HBM traffic
 * scales with the number of activated experts (Sec. 2.2, R2).
 *
 *   X_dev  [T, d_h]  bf16 or f32 (dtype)
 *   W13_dev, W2_dev  packed (bf16) or canonical (f32), see above
 *   Yp_dev [T*k, d_h] float32, capacity T*k rows, rows >= n_local are left untouched
 *   blocks_dev       the work list moe_permute wrote for a batch of the same T (bf16 path; a
 *                    list cut for another block size is refused: bit 1 of the status word;
 *                    the f32 path does not read it and accepts NULL).  The bf16 kernels take
 *                    every row range from this list (it repeats what slot_off_dev says); the
 *                    f32 kernels read slot_off_dev.
 *   workspace_dev    at least moe_workspace_bytes() bytes, 256-byte aligned; holds a control
 *                    region of hand-off flags and the intermediate a (bf16 or f32) between
 *                    the two GEMM stages.  The control region must have been cleared with
 *                    moe_workspace_init() once after allocation; every call that runs to
 *                    completion leaves it cleared for the next one.  Calls that share a
 *                    workspace must not overlap in time.
 * bf16 inputs are multiplied on the matrix cores with fp32 accumulation; `a` is rounded
 * to bf16 once.  A slot's rows are cut into blocks of R = moe_block_rows(T) rows, each a streaming
 * item per channel tile (a slot with one block has its weights read from memory exactly once); in
 * batches with many slots of more than 64 requests those slots are computed as tiled GEMMs over
 * larger blocks by workgroups of the same launch (MOE_WS_OPT_WIDE_MIN_WORKGROUPS below).
 * The bf16 path is one launch in which the workgroups of the second stage
 * wait for flags raised by the first.  The wait is bounded: a workgroup whose wait runs out
 * (which means the control region was not cleared, or the GPU was shared with work that starved
 * the kernel) sets bit 0 of the status word, writes quiet NaNs into its rows of Yp instead of
 * results (moe_combine propagates them) and leaves the block's control lines untouched.  After a
 * non-zero status the workspace must be cleared with moe_workspace_init() before its next use.
 * The second-stage workgroups have the higher ids of the launch and rely on the hardware starting
 * workgroups in id order (every first-stage workgroup is started before any second-stage one gets a
 * place); the flags are raised as long as the first-stage workgroups keep running, so only a GPU
 * whose compute units are held by other work for longer than the spin limit (about a second) can
 * overrun.
 * Limits: d_h % 32 == 0, d_e % 32 == 0 (bf16); d_h % 4 == 0, d_e % 4 == 0 (f32; T*k <= 65535);
 * moe_max_blocks(T, k, C) <= 4095 (bf16).
 */
size_t moe_workspace_bytes(int T, int k, int C, int d_h, int d_e, int dtype);

/* Clears the workspace's control region (asynchronous on `stream`). */
int moe_workspace_init(void *workspace_dev, size_t workspace_bytes, void *stream);

/* Synchronous read-back of the header's error word for tests and debugging (not for the hot
 * path): *status_host = 0 if no wait of the bf16 kernel ever overran since the last init. */
int moe_workspace_status(const void *workspace_dev, int *status_host);

int moe_grouped_ffn(const void *X_dev, const void *W13_dev, const void *W2_dev,
                    int T, int k, int C, int d_h, int d_e, int dtype,
                    const int32_t *slot_off_dev, const int32_t *perm_dev, const int32_t *blocks_dev,
                    float *Yp_dev, void *workspace_dev, size_t workspace_bytes, void *stream);

/* The same call for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * workspace is a fixed array of MOE_FFN_STATIC_SCRATCH_BYTES inside the library's device image
 * (one copy per GPU, held until the process ends); the call allocates nothing, on the host or
 * on the device, and uses the copy of the device that is current when it is called.  Shapes
 * whose moe_workspace_bytes() exceeds the array are refused with MOE_EWORKSPACE (the decode
 * decode configurations of the workload list fit; batches of thousands of tokens do not).  Every call first clears the
 * control lines it can use (one small extra launch), so no init call exists and per-workspace
 * options are always at their defaults; a wait overrun still writes NaN rows but cannot be read
 * back through moe_workspace_status.  All calls on one GPU share the array: calls that overlap
 * in time on one GPU (different streams, or several host threads) race on it and must be
 * ordered by the caller.  Results are bit for bit those of moe_grouped_ffn.
 */
#define MOE_FFN_STATIC_SCRATCH_BYTES (32u << 20)
int moe_grouped_ffn_static(const void *X_dev, const void *W13_dev, const void *W2_dev,
                           int T, int k, int C, int d_h, int d_e, int dtype,
                           const int32_t *slot_off_dev, const int32_t *perm_dev, const int32_t *blocks_dev,
                           float *Yp_dev, void *stream);

/* Per-workspace options of the bf16 path: a word in the workspace's header, written by a one-thread
 * kernel on `stream` (so the call is ordered with the FFN calls on that stream and can be captured),
 * read by every later moe_grouped_ffn on this workspace, reset to the default by
 * moe_workspace_init.  value 0 = default; value < 0 is MOE_EINVAL.
 *   MOE_WS_OPT_SPIN_LIMIT            polls a second-stage workgroup spends on its block's flag
 *                                    before it gives up (default 2^20).  For tests of the overrun path.
 *   MOE_WS_OPT_WIDE_MIN_WORKGROUPS   slots with more than 64 requests are computed as tiled GEMMs,
 *                                    but only when the batch has enough blocks of them to fill the
 *                                    chip: over blocks of 64 rows by workgroups of the same launch
 *                                    when (number of 64-row blocks of those slots) x (ceil(d_e / 64)
 *                                    workgroups per block) >= this value (default 256; by default
 *                                    also from 64 such workgroups on when the launch has enough
 *                                    other experts to stream to hide them); in batches
 *                                    of at least 2048 tokens over blocks of 128 rows by two launches
 *                                    of their own when (number of 128-row blocks) x (workgroups per
 *                                    block) >= this value (default 512), which takes precedence.
 *                                    Otherwise they are cut into streaming items like every other
 *                                    slot.  Results do not depend on it beyond rounding order.
 */
#define MOE_WS_OPT_SPIN_LIMIT            0
#define MOE_WS_OPT_WIDE_MIN_WORKGROUPS   1
int moe_workspace_set_option(void *workspace_dev, size_t workspace_bytes, int option, int value, void *stream);

/* ------------------------------------------------------------------ a6: combine
 * Y[i,:] = sum over j with pos[i*k+j] >= 0, in ascending j, of topk_w[i,j] * Yp[pos[i*k+j],:]
 * accumulated in fp32; tokens without a local request get zeros.  This is the instance's
 * partial result that enters the reverse-path reduction across instances (Sec. 3.3).
 *   Y_dev [T, d_h] bf16 or f32 (dtype).  d_h % 4 == 0.
 */
int moe_combine(const float *Yp_dev, const int32_t *pos_dev, const float *topk_w_dev,
                int T, int k, int d_h, int dtype, void *Y_dev, void *stream);

/* ------------------------------------------------------------------ shared expert (option)
 * Some model families add an expert that every token visits with weight 1.  The paper runs it on
 * the attention side, overlapped with the transfer (Sec. 4), so it is not part of the MoE-instance
 * step; these two calls let an instance run it anyway with the same FFN kernel:
 * moe_shared_dispatch writes the dispatch of one slot that holds all T tokens in order
 * (slot_off_dev [2] = {0, T}; perm_dev [T] = identity; blocks_dev [moe_block_list_len(T, 1, 1)],
 * 16-byte aligned), to be passed to moe_grouped_ffn with k = 1, C = 1 and the shared expert's
 * weights; moe_combine_shared is moe_combine plus Ys_dev [T, d_h] f32 (that FFN's output rows)
 * added to each token's routed sum, in fp32, after it.
 */
int moe_shared_dispatch(int T, int32_t *slot_off_dev, int32_t *perm_dev, int32_t *blocks_dev, void *stream);
int moe_combine_shared(const float *Yp_dev, const int32_t *pos_dev, const float *topk_w_dev, const float *Ys_dev,
                       int T, int k, int d_h, int dtype, void *Y_dev, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_JANUS_H */
