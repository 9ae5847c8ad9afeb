/*
 * dynastage — one pipeline stage's forward and backward pass over dynamically planned
 * micro-batches, for AMD MI355X (gfx950).
 *
 * C ABI.  Plain pointers and sizes only.  Every pointer is tagged HOST or DEVICE below.
 * Every call returns a ds_status and never throws or aborts across the boundary.
 *
 * Citations name passages of "DynaPipe: Optimizing Multi-task Training through Dynamic
 * Pipelines" (EuroSys '24): section, equation, algorithm.
 */
#ifndef DYNASTAGE_H
#define DYNASTAGE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DS_OK = 0,
    DS_EINVAL = -1,       /* null pointer, non-positive length / size, unknown enum value, misaligned shape */
    DS_EINFEASIBLE = -2,  /* no partition satisfies the memory cap (some sequence alone exceeds it) */
    DS_ENOMEM = -3,       /* host or device allocation failed */
    DS_EOVERFLOW = -4,    /* a cost or an objective does not fit in int64 */
    DS_EHIP = -5,         /* a HIP runtime call failed (no device, launch error) */
    DS_ELAYOUT = -6,      /* layout does not fit the stage's workspace or does not match its model kind */
    DS_ELIMIT = -7        /* a size beyond the fixed capacity of an entry point that allocates nothing */
} ds_status;

/* ------------------------------------------------------------------------------------------
 * Cost model t(b, L): predicted forward+backward time of a micro-batch of b sequences padded
 * to length L (section "Overview", paragraph "Cost models").  Exact 64-bit integers.
 *   DS_COST_POLY_GPT : fixed + b*L*(lin + L)
 *   DS_COST_POLY_T5  : fixed + b*Lin*(lin + Lin) + b*Ltgt*(lin + Ltgt + Lin)
 *   DS_COST_TABLE    : table[(b-1)*tl + (L-1)]  (HOST, row-major [tb][tl]; decoder-only;
 *                      a slice with b > tb or L > tl makes dp_plan return DS_EINVAL)
 * With fixed = 0, lin = 2048 the polynomial is t = b*L*(1 + L/2048) in units of 1/2048 token.
 */
enum { DS_COST_POLY_GPT = 0, DS_COST_POLY_T5 = 1, DS_COST_TABLE = 2 };

typedef struct {
    int32_t kind;
    int64_t fixed;
    int64_t lin;
    const int64_t* table;   /* HOST; only for DS_COST_TABLE; borrowed for the duration of the call */
    int32_t tb, tl;
} ds_cost_model;

/* ------------------------------------------------------------------------------------------
 * Layout: the micro-batch partition of one global batch and the placement of every sequence
 * in the padded token streams the stage works on.
 *
 * Stream layout (DEVICE tensors handed to stage_fwd_bwd): micro-batches one after another;
 * micro-batch m is a row-major [mb_count[m], mb_lpad[m], d_model] block starting at row
 * mb_row[m]; sequence at sorted position s occupies rows seq_row[s] .. seq_row[s]+seq_len[s]-1;
 * all other rows are padding.  Encoder-decoder layouts have a second ("tgt") stream for the
 * decoder, padded per micro-batch to mb_ltgt[m].
 *
 * All arrays in the view are HOST memory owned by the layout (valid until ds_layout_free).
 */
typedef struct ds_layout ds_layout;

typedef struct {
    int32_t n_seq, n_mb;
    int32_t total_rows, total_rows_tgt;       /* padded rows of each stream (tgt: 0 if none) */
    int64_t total_tokens, total_tokens_tgt;   /* non-pad tokens */
    int64_t objective;                        /* (c-1)*max t + sum t of this partition (Eq1); 0 if no cost model was given */
    int64_t t_max;                            /* max_m t(M_m) */
    const int32_t* perm;                      /* [n_seq] sorted position -> original sample index */
    const int32_t* mb_start;                  /* [n_mb] first sorted position of micro-batch m */
    const int32_t* mb_count;                  /* [n_mb] sequences in micro-batch m */
    const int32_t* mb_lpad;                   /* [n_mb] padded length (packed layouts: the row length) */
    const int32_t* mb_ltgt;                   /* [n_mb] padded target length, or NULL */
    const int64_t* mb_cost;                   /* [n_mb] t(M_m) under the cost model the layout was built with, or NULL */
    const int32_t* mb_row;                    /* [n_mb] first stream row */
    const int32_t* mb_nrows;                  /* [n_mb] stream rows the micro-batch occupies */
    const int32_t* mb_row_tgt;                /* [n_mb] or NULL */
    const int32_t* mb_nrows_tgt;              /* [n_mb] or NULL */
    const int32_t* seq_row;                   /* [n_seq] */
    const int32_t* seq_len;                   /* [n_seq] */
    const int32_t* seq_row_tgt;               /* [n_seq] or NULL */
    const int32_t* seq_len_tgt;               /* [n_seq] or NULL */
} ds_layout_view;

/*
 * ds_cost_table_build — the profiled cost model (section "Overview", paragraph "Cost models"):
 * execution times profiled at a grid of (micro-batch size, sequence length) points, power-of-two
 * spaced in the paper, are bridged by linear interpolation.  Fills the table a DS_COST_TABLE cost
 * model reads: table[(b-1)*tl + (L-1)], b = 1..tb, L = 1..tl.
 *   b_grid HOST int32[nb], l_grid HOST int32[nl]: strictly increasing, >= 1.
 *   t      HOST double[nb*nl], row-major [b][L]: measured time of a micro-batch of b_grid[i]
 *          sequences padded to l_grid[j], any unit; NaN = not profiled.
 *   Value at (b, L): linear along b at the two bracketing lengths, then linear along L between the
 *   two results; a length below l_grid[0] costs what l_grid[0] costs; b or L beyond the grid, b
 *   below b_grid[0], and points whose bracketing grid points (those with non-zero weight) include
 *   an unprofiled one get inf_cost.  Entries are floor(value * scale + 0.5), at least 1.
 *   table HOST int64[tb*tl], written by the call; nothing is retained.
 * Errors: DS_EINVAL (null, empty or unsorted grid, tb/tl < 1, scale <= 0, inf_cost < 1, a
 * negative time), DS_EOVERFLOW (a scaled time reaches inf_cost).
 */
ds_status ds_cost_table_build(const int32_t* b_grid, int32_t nb, const int32_t* l_grid, int32_t nl,
                              const double* t, double scale, int32_t tb, int32_t tl,
                              int64_t inf_cost, int64_t* table);

/*
 * dp_plan — the paper's micro-batch construction (section "Micro-batch Construction").
 *   1. order samples ascending by length (encoder-decoder: by input length, then target
 *      length); equal keys keep their original order;
 *   2. cut the ordered list into consecutive micro-batches minimising
 *         (num_stages-1) * max_m t(M_m) + sum_m t(M_m)                     (Eq1)
 *      with the recurrence over t_max of Eq2, every distinct single-micro-batch cost being a
 *      candidate t_max (no sampling of t_max);
 *   3. only micro-batches with  count * padded_length <= mem_cap_tokens  are admissible
 *      (paragraph "Limit memory consumption"; encoder-decoder: input stream only).
 * Ties: the smallest optimal t_max; among partitions of equal sum the one whose last
 * micro-batch is longest, then whose second-last is longest, and so on.
 *
 * len, len_tgt: HOST int32[n]; len_tgt NULL for decoder-only (required for DS_COST_POLY_T5).
 * *out: new layout owned by the caller (ds_layout_free).  Pure host code, re-entrant,
 * thread-safe.  Errors: DS_EINVAL (null, n <= 0, a length <= 0, num_stages < 1, cap <= 0, bad
 * cost model), DS_EINFEASIBLE, DS_EOVERFLOW, DS_ENOMEM.
 */
ds_status dp_plan(const int32_t* len, const int32_t* len_tgt, int32_t n,
                  const ds_cost_model* cm, int64_t mem_cap_tokens, int32_t num_stages,
                  ds_layout** out);

/*
 * dp_plan_sampled — dp_plan with t_max sampled at fixed intervals (section "Micro-batch
 * Construction", end of "Dynamic programming": the paper only considers t_max values 5 us apart).
 * Candidates are the multiples of t_max_interval (>= 1, in the cost model's unit); for each, Eq2 runs
 * over the slices whose cost does not exceed it, and the candidate minimising
 * (num_stages-1)*candidate + f(N; candidate) wins (ties as dp_plan).  The layout reports the
 * objective and t_max of the partition chosen.  Its objective is at most
 * (num_stages-1)*t_max_interval above dp_plan's; with interval 1 the two calls agree.
 */
ds_status dp_plan_sampled(const int32_t* len, const int32_t* len_tgt, int32_t n,
                          const ds_cost_model* cm, int64_t mem_cap_tokens, int32_t num_stages,
                          int64_t t_max_interval, ds_layout** out);

/*
 * dp_plan_replicas — micro-batch construction under hybrid data + pipeline parallelism (section
 * "Micro-batch Construction", paragraph "Balance data parallel model replicas"): the same
 * dynamic programme with the sum term weighted 1/n_replicas, kept exact by scaling, i.e. minimising
 *       n_replicas * (num_stages-1) * max_m t(M_m) + sum_m t(M_m)
 * (the layout's `objective` is this scaled value), then ds_assign_replicas on the micro-batches'
 * times.  replica_of_mb: HOST int32, capacity n, the first n_mb entries are written;
 * replica_time: HOST int64[n_replicas].  Other arguments and errors as dp_plan; DS_EINVAL also for
 * n_replicas < 1, DS_EOVERFLOW when n_replicas * (num_stages-1) overflows.
 */
ds_status dp_plan_replicas(const int32_t* len, const int32_t* len_tgt, int32_t n,
                           const ds_cost_model* cm, int64_t mem_cap_tokens, int32_t num_stages,
                           int32_t n_replicas, ds_layout** out, int32_t* replica_of_mb,
                           int64_t* replica_time);

/*
 * ds_assign_replicas — Karmarkar-Karp (largest differencing) split of n_items times into
 * n_replicas sets with a small largest sum (same paragraph; the paper names the method only, the
 * rules below make it reproducible).  Every item starts as a partial partition with one non-empty
 * set; the two partial partitions of largest spread (largest set sum - smallest set sum) are merged
 * by joining the first's sets in descending order of sum with the second's in ascending order;
 * repeat until one is left.  Sets inside a partial partition are ordered by (sum descending,
 * smallest member index ascending, empty sets last among equal sums), "ascending" is the exact reverse;
 * partial partitions of equal spread are taken in order of creation (the initial ones by
 * descending time, then ascending index).  Replica r gets the r-th set of the final order, so
 * replica_time is non-increasing.
 * t: HOST int64[n_items], >= 0; replica_of: HOST int32[n_items]; replica_time: HOST int64[n_replicas].
 * Errors: DS_EINVAL (null, n_items < 0, n_replicas < 1, a negative time), DS_EOVERFLOW (sum of t).
 */
ds_status ds_assign_replicas(const int64_t* t, int32_t n_items, int32_t n_replicas,
                             int32_t* replica_of, int64_t* replica_time);

/*
 * ds_layout_from_cuts — layout for a given order and given cut points (the baselines the paper
 * compares against, section "Background", naive padding; and single-sequence micro-batches).
 * perm: HOST int32[n] permutation (NULL = identity); cuts: HOST int32[n_mb+1], cuts[0]=0,
 * cuts[n_mb]=n, strictly increasing.  pad_to / pad_to_tgt: 0 = pad each micro-batch to its own
 * longest sequence; otherwise every micro-batch is padded to that length (>= longest).
 * cm may be NULL (objective, t_max reported as 0).
 */
ds_status ds_layout_from_cuts(const int32_t* len, const int32_t* len_tgt, int32_t n,
                              const int32_t* perm, const int32_t* cuts, int32_t n_mb,
                              int32_t pad_to, int32_t pad_to_tgt,
                              const ds_cost_model* cm, int32_t num_stages, ds_layout** out);

/*
 * ds_layout_token_based — token-based micro-batching, the "TB" baseline (section "Motivation", micro-batching
 * methods: micro-batches of the same token count, fewer samples where they are longer; section "Evaluation",
 * ablation of micro-batching, where the token count per micro-batch is found by search).  Samples are ordered as
 * in dp_plan; the ordered list is cut from the front, a micro-batch taking samples as long as
 *       (samples in it) * (its longest sample)  <=  token_budget
 * (its padded token count; encoder-decoder: of the input stream, the quantity dp_plan's memory cap limits) and
 * closing when one more would exceed it.  Each micro-batch is padded to its own longest sample.
 * len, len_tgt, cm (may be NULL), num_stages, *out as ds_layout_from_cuts.
 * Errors: DS_EINVAL (null, n <= 0, a length <= 0, token_budget <= 0, bad cost model), DS_EINFEASIBLE (a sample
 * longer than token_budget), DS_EOVERFLOW, DS_ENOMEM.
 */
ds_status ds_layout_token_based(const int32_t* len, const int32_t* len_tgt, int32_t n, int64_t token_budget,
                                const ds_cost_model* cm, int32_t num_stages, ds_layout** out);

/*
 * ds_layout_packed — the packing baseline (section "Background", "The current packing
 * solution"): sequences, in their original order, are placed first-fit into rows of row_len
 * tokens; rows_per_mb rows form one micro-batch; attention never crosses a sequence boundary.
 * Decoder-only.  Errors: DS_EINVAL (a length > row_len, ...).
 */
ds_status ds_layout_packed(const int32_t* len, int32_t n, int32_t row_len, int32_t rows_per_mb,
                           ds_layout** out);

ds_status ds_layout_get(const ds_layout* layout, ds_layout_view* view);
void ds_layout_free(ds_layout* layout);

/* ------------------------------------------------------------------------------------------
 * Pipeline execution schedules and communication order (host only; C stages, M micro-batches).
 * Orders are HOST int32 arrays [C][2*M]: order_mb[j*2M + k], order_kind[j*2M + k] = the k-th op
 * of stage j (micro-batch, DS_OP_FWD / DS_OP_BWD).  Per-op data are HOST int64 [M][C]:
 * x[i*C + j] for micro-batch i on stage j.
 */
enum { DS_OP_FWD = 0, DS_OP_BWD = 1 };
enum {
    DS_INSTR_FORWARD = 0, DS_INSTR_BACKWARD = 1,
    DS_INSTR_SEND_ACT_START = 2, DS_INSTR_RECV_ACT_START = 3,
    DS_INSTR_SEND_GRAD_START = 4, DS_INSTR_RECV_GRAD_START = 5,
    DS_INSTR_WAIT_RECV_ACT = 6, DS_INSTR_WAIT_RECV_GRAD = 7
};

/*
 * ds_schedule_adaptive — memory-aware adaptive scheduling (section "Pipeline Execution Schedule",
 * Alg. 1).  Execution proceeds in cycles; in each cycle every stage, in stage order, takes at most
 * one backward op and then at most one forward op from the heads of its buffers of ready ops; a
 * forward op of micro-batch i runs on stage j only if  m_j + act[i][j] < limit[j]  (m_j = activation
 * memory held by the stage), otherwise it stays at the head and the stage skips forward passes
 * until backward passes have freed memory; ops unlocked during a cycle (next stage's forward, the
 * last stage's own backward, previous stage's backward) join the buffers at the end of the cycle.
 * All micro-batches start in the first stage's forward buffer, in index order.
 * Errors: DS_EINVAL (null, C or M < 1, negative act), DS_EINFEASIBLE (some act[i][j] >= limit[j]:
 * that micro-batch can never run; or a cycle in which no op could run).  n_cycles may be NULL.
 */
ds_status ds_schedule_adaptive(int32_t n_stages, int32_t n_mb, const int64_t* act, const int64_t* limit,
                               int32_t* order_mb, int32_t* order_kind, int32_t* n_cycles);

/*
 * ds_schedule_1f1b — the one-forward-one-backward order the paper compares with (same section,
 * "on the n-th device, it executes c + 1 - n forward passes, followed by regular backward-forward
 * cycles"): stage j (0-based) runs min(C - j, M) forwards, then alternates one backward and one
 * forward while forwards are left, then the remaining backwards; micro-batches in index order.
 */
ds_status ds_schedule_1f1b(int32_t n_stages, int32_t n_mb, int32_t* order_mb, int32_t* order_kind);

/*
 * ds_schedule_simulate — device timeline of given per-stage orders under given op times (what
 * section "Communication Planning" simulates with the cost model).  A stage executes its ops in
 * order; an op starts when the stage is free and its predecessor has ended (forward: the same
 * micro-batch's forward on the previous stage; backward: its backward on the next stage, on the
 * last stage its own forward).  Communication takes no time.  Outputs: *makespan; idle[C] =
 * makespan - busy time; peak[C] = largest activation memory held (taken at a forward's start,
 * released at the backward's end, releases first at equal times; needs act); op_start / op_end
 * [C][2*M].  idle, peak, act, op_start, op_end may be NULL.
 * Errors: DS_EINVAL (null, sizes, a negative time, an order that is not a permutation of all 2*M
 * ops of a stage, or orders that deadlock), DS_EOVERFLOW.
 */
ds_status ds_schedule_simulate(int32_t n_stages, int32_t n_mb, const int32_t* order_mb, const int32_t* order_kind,
                               const int64_t* t_fwd, const int64_t* t_bwd, const int64_t* act,
                               int64_t* makespan, int64_t* idle, int64_t* peak, int64_t* op_start, int64_t* op_end);

/*
 * ds_comm_plan — order of communication between adjacent stages and the per-stage instruction
 * stream (section "Communication Planning").  Ops of the simulated timeline are visited in
 * ascending end time (ties: lower stage, then earlier op of that stage); a forward on stage j < C-1
 * queues SEND_ACT_START on j and RECV_ACT_START on j+1, a backward on stage j > 0 queues
 * SEND_GRAD_START on j and RECV_GRAD_START on j-1: both ends of a transfer are queued together, so
 * adjacent stages see their common transfers in the same order.  The stream of a stage lists its
 * compute ops in order; every queued start goes before the first compute op of that stage that
 * starts at or after the start's time; the wait for a received tensor goes immediately before the
 * op that consumes it.  stream_code / stream_mb: HOST int32 [C][8*M] (DS_INSTR_*, micro-batch),
 * stream_len: HOST int32[C].  Errors as ds_schedule_simulate.
 */
ds_status ds_comm_plan(int32_t n_stages, int32_t n_mb, const int32_t* order_mb, const int32_t* order_kind,
                       const int64_t* t_fwd, const int64_t* t_bwd,
                       int32_t* stream_code, int32_t* stream_mb, int32_t* stream_len);

/* ------------------------------------------------------------------------------------------
 * Dynamic recomputation (section "Implementation", paragraph "Dynamic recomputation"; host only).
 * The peak memory of an iteration varies with its micro-batches, so the recomputation scheme is
 * chosen per iteration: micro-batch construction and scheduling are repeated once per scheme, each
 * under that scheme's cost model, and the scheme with the least overhead that stays in memory wins.
 */
typedef struct {
    ds_cost_model cm;           /* t(b, L) of a micro-batch's forward + backward on one stage, INCLUDING what the scheme recomputes */
    int64_t act_per_row;        /* > 0: units of activation memory one padded row (main + target stream) holds on a
                                   stage between the micro-batch's forward and its backward */
    int64_t fwd_num, fwd_den;   /* the forward takes t * fwd_num / fwd_den (integer division), the backward the rest */
} ds_recompute_scheme;

/*
 * ds_plan_recompute — for every scheme r: dp_plan under schemes[r].cm with the token cap
 * (mem_limit - 1) / act_per_row (one micro-batch alone must satisfy Alg. 1's  act < limit); then
 * ds_schedule_adaptive with act = act_per_row * padded rows of the micro-batch and the same
 * mem_limit on each of the num_stages (alike) stages; then ds_schedule_simulate with the times
 * above.  A scheme is feasible if all three succeed.  *chosen = the feasible scheme with the
 * smallest makespan (equal: the one listed first; list schemes in ascending order of
 * recomputation); *out = its layout (caller frees).  makespan / peak: HOST int64[n_schemes] or
 * NULL, -1 for an infeasible scheme (peak = largest memory any stage holds, < mem_limit).
 * Errors: DS_EINVAL, DS_EINFEASIBLE (no scheme fits), DS_EOVERFLOW, DS_ENOMEM.
 */
ds_status ds_plan_recompute(const int32_t* len, const int32_t* len_tgt, int32_t n,
                            const ds_recompute_scheme* schemes, int32_t n_schemes, int64_t mem_limit,
                            int32_t num_stages, int32_t* chosen, ds_layout** out, int64_t* makespan,
                            int64_t* peak);

/* ------------------------------------------------------------------------------------------
 * Stage: the transformer layers of one pipeline stage (what the ForwardPass / BackwardPass
 * pipeline instructions execute, section "Overview", paragraph "Execution plans").
 */
enum { DS_MODEL_GPT = 0, DS_MODEL_T5 = 1 };
enum { DS_DTYPE_F32 = 0, DS_DTYPE_BF16 = 1 };

typedef struct {
    int32_t model;          /* DS_MODEL_* */
    int32_t dtype;          /* storage type of weights and activations; accumulation is always fp32 */
    int32_t n_layers;       /* GPT: decoder layers.  T5: encoder layers */
    int32_t n_dec_layers;   /* T5: decoder layers (0 for GPT) */
    int32_t d_model, n_heads, d_ff;
    int32_t max_rows;       /* workspace capacity: padded rows of the main stream */
    int32_t max_rows_tgt;   /* ... of the target stream (0 for GPT) */
    int32_t max_seqs;
    int32_t recompute;      /* DS_RECOMPUTE_*: what the backward pass recomputes instead of keeping */
} ds_stage_config;

/* Recomputation (activation checkpointing; section "Implementation", paragraph "Dynamic recomputation").
 * NONE: every layer keeps what its backward reads (the attention kernels recompute the probabilities from the saved
 *       log-sum-exp in any case, which is what "selective" recomputation saves elsewhere).
 * FULL: only each layer's input is kept; the layer's forward is run again right before its backward (except for the
 *       layer whose forward ran last).  Results are bit-identical to NONE; the workspace holds one layer's
 *       activations instead of all layers'. */
enum { DS_RECOMPUTE_NONE = 0, DS_RECOMPUTE_FULL = 1 };

/* Per-layer tensors, DEVICE pointers.  The same structs carry weights (element type = the
 * stage dtype) and weight gradients (always float32).  Matrices are row-major
 * [in_features, out_features]: y = x W (+ b).
 *   GPT block (pre-LayerNorm, eps 1e-5):  x1 = x + Attn_causal(LN1(x)) Wo + bo;
 *                                         x2 = x1 + GELU_tanh(LN2(x1) W1 + b1) W2 + b2.
 *   T5 blocks (pre-RMSNorm, eps 1e-6, no biases, gated GELU):
 *     encoder: x += Attn_bidir(RMS1(x)) Wo;  x += (GELU(u Wg) * (u Wu)) W2, u = RMS2(x).
 *     decoder: causal self-attention, cross-attention (queries RMSc(x) Wcq, keys/values
 *              enc_out Wckv), MLP.
 *   Attention scale 1/sqrt(head_dim); heads are consecutive column groups of width head_dim. */
typedef struct {
    void *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o, *ln2_g, *ln2_b, *w_1, *b_1, *w_2, *b_2;
} ds_gpt_layer;

typedef struct {
    void *ln1_g, *w_qkv, *w_o, *ln2_g, *w_g, *w_u, *w_2;
} ds_t5_enc_layer;

typedef struct {
    void *ln1_g, *w_qkv, *w_o, *lnc_g, *w_cq, *w_ckv, *w_co, *ln2_g, *w_g, *w_u, *w_2;
} ds_t5_dec_layer;

/* Activations and gradients of one call, DEVICE pointers, element type = stage dtype, in
 * stream layout ([total_rows, d_model] row-major).  Values at padding rows of the inputs are
 * ignored (they may be NaN); padding rows of the outputs are written as zeros. */
typedef struct {
    const void* act_in;       /* GPT: stage input.  T5: encoder-side input                   */
    const void* act_in_tgt;   /* T5: decoder-side input [total_rows_tgt, d]; NULL for GPT     */
    const void* grad_out;     /* gradient w.r.t. act_out (same shape as act_out)              */
    void* act_out;            /* GPT: [total_rows, d].  T5: decoder output [total_rows_tgt, d] */
    void* grad_in;            /* gradient w.r.t. act_in                                       */
    void* grad_in_tgt;        /* T5: gradient w.r.t. act_in_tgt; NULL for GPT                 */
} ds_stage_io;

typedef struct ds_stage ds_stage;

/* Allocates the stage's device workspace once (saved activations of every layer for max_rows
 * rows, backward temporaries, layout tables).  Uses the current HIP device.
 * Errors: DS_EINVAL (d_model % n_heads, head_dim not in {64,128} for bf16 fast paths is NOT an
 * error: generic kernels take over), DS_ENOMEM, DS_EHIP. */
ds_status ds_stage_create(const ds_stage_config* cfg, ds_stage** out);
void ds_stage_destroy(ds_stage* stage);
/* Bytes of device workspace the stage holds. */
int64_t ds_stage_workspace_bytes(const ds_stage* stage);
/* Bytes of device workspace ds_stage_create would allocate for cfg, without allocating (host only):
 * what a caller compares with its memory limit when it chooses a recomputation scheme.  -1 for an
 * invalid configuration. */
int64_t ds_stage_workspace_need(const ds_stage_config* cfg);

/*
 * stage_fwd_bwd — run forward then backward of every layer of the stage over every
 * micro-batch of the layout (ForwardPass and BackwardPass of all micro-batches; weight
 * gradients summed over micro-batches, section "Background", pipeline-parallel paragraph).
 *
 * weights: HOST array of n_layers ds_gpt_layer (GPT), or n_layers ds_t5_enc_layer followed in
 *          a second array (weights_dec) by n_dec_layers ds_t5_dec_layer (T5); the structs hold
 *          DEVICE pointers.  grads / grads_dec: same shape, DEVICE float32 buffers.
 * accumulate: 0 = overwrite the weight-gradient buffers, 1 = add to them.
 * hip_stream: a hipStream_t (NULL = default stream).  The call enqueues work on that stream and
 * returns; it allocates nothing.  The first call with a new layout uploads the layout's tables
 * (a few KB) and may wait for the stream to drain; later calls with the same layout do not.
 * Calls on the same stage must not overlap in time (they share the workspace).
 * A call with the layout of the previous call only enqueues kernels (no copies, no memsets) and may
 * be captured into a HIP graph; the tables and the attention work lists it relies on stay in the
 * workspace, so a captured call is valid for replay only as long as no call with another layout
 * has been made on the stage in between.
 * Errors: DS_EINVAL, DS_ELAYOUT (layout rows / sequences exceed the workspace, or stream kinds
 * do not match the model), DS_EHIP.
 */
ds_status stage_fwd_bwd(ds_stage* stage, const ds_layout* layout,
                        const void* weights, const void* weights_dec,
                        const ds_stage_io* io,
                        void* grads, void* grads_dec, int32_t accumulate,
                        void* hip_stream);

/* Per-kernel-group timing of stage_fwd_bwd.  When enabled, every kernel group the call enqueues
 * is bracketed by a pair of HIP events on the caller's stream (events are created here, once,
 * never inside stage_fwd_bwd; at most 2048 groups are recorded between two reads).
 * ds_stage_profile_read waits for the recorded events, returns per group kind the summed
 * milliseconds and the number of groups since the last read (HOST arrays of DS_PROF_COUNT
 * entries) and clears the record. */
enum { DS_PROF_GEMM_FWD = 0, DS_PROF_GEMM_DGRAD = 1, DS_PROF_GEMM_WGRAD = 2, DS_PROF_ATTN_FWD = 3,
       DS_PROF_ATTN_BWD = 4, DS_PROF_NORM = 5, DS_PROF_COLSUM = 6, DS_PROF_OTHER = 7, DS_PROF_TRANSPOSE = 8,
       DS_PROF_COUNT = 9 };
ds_status ds_stage_profile_enable(ds_stage* stage, int32_t enable);
ds_status ds_stage_profile_read(ds_stage* stage, float* ms, int32_t* count);

/* Weights that do not change between calls (section "Pipeline Execution Schedule": a stage runs the
 * micro-batches of an iteration one after the other on the same weights).  For bf16 stages
 * stage_fwd_bwd keeps a transposed copy of every weight matrix in its workspace and normally makes
 * it anew in every call.  unchanged = 1 is the caller's promise that the following calls are given
 * the same weight arrays with the same contents as the previous call: the copies are then reused
 * (they are still made when the stage has none yet, or the array of layer structs passed differs
 * in address from the previous call's).  Set it back to 0 after every optimizer step.  Default 0.
 * Errors: DS_EINVAL (null stage). */
ds_status ds_stage_weights_unchanged(ds_stage* stage, int32_t unchanged);

/* Rough count of the kernels one stage_fwd_bwd call launches (diagnostics). */
int32_t ds_stage_last_launch_count(const ds_stage* stage);

/*
 * ds_pack / ds_unpack — move rows between the canonical form (sequences back to back in
 * ORIGINAL sample order, [total_tokens, d] row-major, DEVICE) and a stream of the layout
 * ("padded to the longest in the micro-batch", section "Background").  ds_pack zero-fills
 * padding rows.  which: 0 = main stream, 1 = target stream.  dtype: DS_DTYPE_*.
 */
ds_status ds_pack(const ds_layout* layout, int32_t which, int32_t dtype, int32_t d,
                  const void* canonical, void* stream_rows, void* hip_stream);
ds_status ds_unpack(const ds_layout* layout, int32_t which, int32_t dtype, int32_t d,
                    const void* stream_rows, void* canonical, void* hip_stream);

/* ------------------------------------------------------------------------------------------
 * Building blocks, exported so that each kernel can be checked and profiled alone.  All
 * pointers DEVICE unless said otherwise; dtype = element type of the non-float32 tensors.
 */

/* C[M,N] = op(A) op(B) (+ epilogue).  trans_a = 0: A is [M,K] row-major; 1: A is [K,M].
 * trans_b = 0: B is [K,N]; 1: B is [N,K].  Accumulation in float32.
 * epilogue (DS_EPI_*):
 *   NONE     C = acc (+ bias[n])
 *   GELU     C = acc + bias (pre-activation, stored), C2 = GELU_tanh(C)
 *   RESID    C = acc + bias + R[m,n]; rows with row_valid[m] < 0 are written as 0
 *   DGELU    C = acc * GELU_tanh'(R[m,n])
 *   ACC32    C is float32 [M,N]; C = acc + (accumulate ? C : 0)
 *   GATE     C = acc (stored), C2 = GELU_tanh(R[m,n]) * C            (gated MLP forward)
 *   DGATE    C = acc * R2[m,n] * GELU_tanh'(R[m,n]), C2 = acc * GELU_tanh(R[m,n])   (its backward)
 *   GELU_D   z = acc + bias (not stored); C = GELU_tanh'(z), C2 = GELU_tanh(z).  The stage's MLP forward: it keeps
 *            the derivative instead of the pre-activation (both come from one logistic term), so that the
 *            backward epilogue is one multiplication per element:
 *   MULR     C = acc * R[m,n]                                          (R = the derivative GELU_D stored)
 * N must be a multiple of 8.  force_generic != 0 selects the plain FMA kernel.
 * bias may be NULL.  row_valid may be NULL (all rows valid). */
enum { DS_EPI_NONE = 0, DS_EPI_GELU = 1, DS_EPI_RESID = 2, DS_EPI_DGELU = 3, DS_EPI_ACC32 = 4,
       DS_EPI_GATE = 5, DS_EPI_DGATE = 6, DS_EPI_GELU_D = 7, DS_EPI_MULR = 8 };
ds_status ds_gemm(int32_t dtype, int32_t trans_a, int32_t trans_b, int32_t M, int32_t N, int32_t K,
                  const void* A, const void* B, void* C, int32_t epilogue, const void* bias,
                  const void* R, const void* R2, void* C2, const int32_t* row_valid, int32_t accumulate,
                  int32_t force_generic, void* hip_stream);
/* ds_gemm with a DEVICE float32 workspace of workspace_floats entries (16-byte aligned), which lets the bf16
 * matrix-core kernels split the contraction the way the stage does: weight-gradient launches (ACC32,
 * trans_a = 1, trans_b = 0) into K ranges whose partial sums a second kernel adds up in a fixed order, all other
 * launches for the tiles of their last, partly filled round over the compute units.  The result differs from
 * ds_gemm's only in the order of fp32 additions; a workspace too small for a split is simply not used.
 * Calls sharing a workspace must not overlap. */
ds_status ds_gemm_ws(int32_t dtype, int32_t trans_a, int32_t trans_b, int32_t M, int32_t N, int32_t K,
                     const void* A, const void* B, void* C, int32_t epilogue, const void* bias,
                     const void* R, const void* R2, void* C2, const int32_t* row_valid, int32_t accumulate,
                     int32_t force_generic, float* workspace, int64_t workspace_floats, void* hip_stream);

/* Bytes of DEVICE scratch the bf16 matrix-core attention kernels need: the work lists of the call
 * (sequence, 128-row block), long sequences first and the blocks of one sequence together, and the per-(head, query row)
 * statistics the dQ kernel hands to the dK/dV kernel.  q_total_rows / k_total_rows: rows of the
 * tensors holding the queries / the keys.  Calls that share one scratch buffer must not overlap. */
int64_t ds_attention_scratch_bytes(int32_t n_heads, int32_t head_dim, int32_t q_total_rows, int32_t k_total_rows,
                                   int32_t n_seq);

/* Variable-length attention over a packed QKV-style tensor.
 * q, k, v: row-major with row strides ldq, ldk, ldv (elements); head h uses columns
 * h*head_dim .. of each.  Query sequence s occupies rows q_row[s] .. +q_len[s]-1 of q/o, its
 * keys rows k_row[s] .. +k_len[s]-1 of k/v.  mask: 0 = none (bidirectional / cross), 1 = causal.
 * o: [rows, n_heads*head_dim] with row stride ldo; lse: float32 [n_heads, lse_stride].
 * Rows not covered by any sequence are not touched.  q_row etc. are DEVICE int32 arrays; the
 * sequences must not overlap; a sequence with q_len[s] = 0 is skipped, one with k_len[s] = 0
 * gets zero outputs / gradients.  scratch (DEVICE, 16-byte aligned, at least
 * ds_attention_scratch_bytes) enables the bf16 matrix-core kernels; with scratch = NULL, or a
 * shape they do not take, the generic kernels run.  k_total_rows: rows of the k / v tensors (the
 * q / o tensors have lse_stride rows). */
ds_status ds_attention_fwd(int32_t dtype, int32_t n_seq, int32_t n_heads, int32_t head_dim, int32_t mask,
                           const int32_t* q_row, const int32_t* q_len, const int32_t* k_row, const int32_t* k_len,
                           int32_t max_q_len, int32_t max_k_len,
                           const void* q, int32_t ldq, const void* k, int32_t ldk, const void* v, int32_t ldv,
                           void* o, int32_t ldo, float* lse, int32_t lse_stride,
                           int32_t k_total_rows, void* scratch, int64_t scratch_bytes,
                           int32_t force_generic, void* hip_stream);
/* Backward: given dO, O, LSE produce dQ, dK, dV (same strides as q, k, v).  delta: float32
 * scratch [n_heads, lse_stride]. */
ds_status ds_attention_bwd(int32_t dtype, int32_t n_seq, int32_t n_heads, int32_t head_dim, int32_t mask,
                           const int32_t* q_row, const int32_t* q_len, const int32_t* k_row, const int32_t* k_len,
                           int32_t max_q_len, int32_t max_k_len,
                           const void* q, int32_t ldq, const void* k, int32_t ldk, const void* v, int32_t ldv,
                           const void* o, const void* d_o, int32_t ldo, const float* lse, float* delta, int32_t lse_stride,
                           void* dq, void* dk, void* dv,
                           int32_t k_total_rows, void* scratch, int64_t scratch_bytes,
                           int32_t force_generic, void* hip_stream);

/* Row normalisation.  rms = 0: LayerNorm (gain g, bias b, eps 1e-5, stats = mean and rstd);
 * rms = 1: RMSNorm (gain only, eps 1e-6, stats = rstd).  stats: float32 [2, rows]. */
ds_status ds_norm_fwd(int32_t dtype, int32_t rms, int32_t rows, int32_t d, const void* x,
                      const void* g, const void* b, void* y, float* stats, void* hip_stream);
/* dx = (resid ? resid : 0) + norm_backward(dy); dg, db: float32 [d], overwritten or added to
 * (accumulate).  partial: float32 scratch of at least ds_norm_bwd_scratch_floats(rows, d). */
ds_status ds_norm_bwd(int32_t dtype, int32_t rms, int32_t rows, int32_t d, const void* dy, const void* x,
                      const void* g, const float* stats, const void* resid, void* dx,
                      float* dg, float* db, float* partial, int32_t accumulate, void* hip_stream);
int64_t ds_norm_bwd_scratch_floats(int32_t rows, int32_t d);

/* out[n] (float32) = sum_m x[m,n] (+ out[n] if accumulate).  partial as above (same size rule). */
ds_status ds_colsum(int32_t dtype, int32_t rows, int32_t n, const void* x, float* out, float* partial,
                    int32_t accumulate, void* hip_stream);

/* ds_colsum for callers that cannot allocate or hand over scratch memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same two kernels as ds_colsum, with the partial sums in a
 * 4 MiB array that is part of the library's device image (one copy per GPU, held until the process ends).  The call
 * allocates nothing and frees nothing; it only enqueues the two kernels on hip_stream.  out[n] as ds_colsum.
 * Limits: n <= 65536 (DS_ELIMIT beyond), device ordinal < 64.  All calls on one GPU share that GPU's array: calls
 * that overlap in time on one GPU (different streams, different threads) race; calls on one stream do not.
 * Nothing in the array needs to start at zero (every partial row that is read was written by the same call).
 * Errors: DS_EINVAL (null, rows <= 0, n <= 0, n % 8, dtype), DS_ELIMIT, DS_EHIP. */
ds_status ds_colsum_static(int32_t dtype, int32_t rows, int32_t n, const void* x, float* out, int32_t accumulate,
                           void* hip_stream);

/* Measurement aid (no part of the method): the rate the matrix cores sustain with nothing else going on, the yardstick
 * bench.py prints beside the published peak.  Launches ONE kernel of n_groups work-groups (512 threads each, one per
 * compute unit at a time) on hip_stream; every wavefront issues iters x 64 v_mfma_f32_16x16x32_bf16 on the GEMM
 * kernel's register tile, operands read once.  The caller times it:
 *     flops = n_groups x 8 wavefronts x iters x 64 MFMAs x 2 x 16 x 16 x 32.
 * operands: DEVICE, 24 x 512 x 8 bf16 values (196 608 bytes, 16-byte aligned), read only: fragment f of thread t is
 * the 8 values at (f x 512 + t) x 8; what they hold decides the power the chip draws and with it the result.
 * sink: DEVICE, n_groups x 512 floats, written (one sum per thread, so that the loop cannot be optimised away).
 * Allocates nothing.  Errors: DS_EINVAL (null, alignment, counts <= 0), DS_EHIP. */
ds_status ds_mfma_probe(const void* operands, float* sink, int32_t n_groups, int32_t iters, void* hip_stream);

/* Library identification: returns a static HOST string "dynastage <version> gfx950". */
const char* ds_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DYNASTAGE_H */
