/*
 * gbmw.h -- C ABI of the batched layer-wise strategy search for gfx950 (MI355X).
 *
 * The library solves, for a batch of B independent pipeline-stage searches
 * (the planner calls the search once per stage, PP degree, batch size and
 * partition: Algorithm 1 / Algorithm 2), the dynamic programme of Section
 * 4.1.2, Eq. 3 of "Improving Automatic Parallel Training via Balanced Memory
 * Workload Optimization":
 *
 *   C(l, e, s) = min_{s'} [ C(l-1, e - M(l,s), s') + R(l, s', s) ] + c(l, s)
 *
 * for EVERY forward-memory budget e = 0..E at once, where
 *   c(l, s)      execution time of layer l under strategy s,
 *   M(l, s)      forward memory O_f(l,s) + O_ms(l,s) of that choice, in budget
 *                units (the amount Eq. 3 subtracts from E_fwd),
 *   R(l, s', s)  cost of transforming layer l-1's output laid out for s' into
 *                the layout s needs,
 * and reads optimal plans back from the recorded argmins (Algorithm 3's S_min).
 * Eq. 3 writes its state without the strategy index although R needs it; the
 * state here carries it.  Layer 0 has no predecessor: C(0, e, s) = c(0, s) if
 * e >= M(0, s).  Cells whose memory exceeds the budget are +infinity.
 *
 * Arithmetic: IEEE binary32; each transition is two separately rounded
 * additions in the order (C_prev + R) + c; every minimum keeps the LOWEST index
 * among equal candidates; a minimum over candidates that are all +infinity
 * records index 0.  Results are bit-identical to a sequential evaluation in
 * that order.
 *
 * All computation runs in HIP kernels on the current device; there is no CPU
 * fallback.  Calls are not thread-safe with respect to one context.
 */
#ifndef GBMW_H
#define GBMW_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gbmw_ctx gbmw_ctx; /* opaque; owned by the library */

typedef enum {
  GBMW_OK = 0,
  GBMW_ERR_INVALID_ARG = 1, /* null pointer, size out of range, bad value in c/M/R */
  GBMW_ERR_UNSUPPORTED = 2, /* request needs data the context did not keep */
  GBMW_ERR_OOM = 3,         /* device or host allocation failed */
  GBMW_ERR_DEVICE = 4       /* a HIP call failed; see gbmw_last_error() */
} gbmw_status;

enum { GBMW_PTR_HOST = 0, GBMW_PTR_DEVICE = 1 };

enum {
  GBMW_FLAG_KEEP_ALL_C = 1u,   /* keep every layer's fp32 table (default: last two) */
  GBMW_FLAG_TIME_KERNELS = 2u, /* record a HIP event pair around every min-plus launch
                                  (implies GBMW_FLAG_ONE_STREAM)                       */
  GBMW_FLAG_ONE_STREAM = 4u,   /* enqueue every kernel on p->stream itself.  Default: the
                                  instances are split into groups whose per-layer
                                  launches run on library-owned helper streams of default
                                  priority that fork from and join back into p->stream
                                  with events, so the call is still ordered on p->stream
                                  as a whole                                             */
  GBMW_FLAG_RESOLVE_ALL = 8u,  /* gbmw_partition_search only: solve every stage of every
                                  live pair in every round                               */
  GBMW_FLAG_LAZY_ARGMIN = 16u  /* do not write the argmin records while the tables are
                                  filled; keep every layer's fp32 table instead (implies
                                  GBMW_FLAG_KEEP_ALL_C: 4 bytes per cell instead of 1) and
                                  let gbmw_backtrack and the other plan walkers recompute
                                  the one record they need per layer, with the same
                                  arithmetic and tie rule, so every result is identical.
                                  The fill then costs one add and half a three-input min
                                  per candidate and nothing else                         */,
  GBMW_FLAG_DENSE_ARITHMETIC = 32u /* every lane computes its own cell.  Default: a wave
                                  whose 64 consecutive budgets all read the same column of
                                  the previous layer's table (the tables are step functions
                                  of the budget, so most waves do) computes that column's
                                  cells once, one output strategy per lane.  Every layer
                                  leaves one word per strategy and 64 budgets (1/64 of the
                                  fp32 table bytes of device memory more) that holds such a
                                  group's value: the next layer recognises its runs from
                                  those words without reading the table, and the group's
                                  cells are not written inside the library's own tables
                                  (what gbmw_export_tables and every other call return is
                                  unaffected).  Identical results either way; the flag
                                  exists to time the dense arithmetic                     */,
  GBMW_FLAG_COUNT_WORK = 64u   /* measurement: the min-plus launches also count the waves
                                  that took the shortcut above, for gbmw_last_solve_work
                                  (implies GBMW_FLAG_ONE_STREAM).  The counts depend on the
                                  inputs alone; the counting costs registers, so time the
                                  kernels in a solve without this flag                    */,
  GBMW_FLAG_LAYER_LAUNCHES = 128u /* one launch per layer even for a small problem.
                                  Default: a problem with S <= 64 whose tiles of 64 budgets
                                  (ceil((E+1)/64) per instance) are all resident on the
                                  device at once is filled by a single launch in which the
                                  tiles hand their layers to each other through flags in
                                  device memory.  Its waits are bounded: should one give up
                                  (the device held by other work for seconds), the calls
                                  that wait for the solve return GBMW_ERR_DEVICE and the
                                  context holds no solution.  Identical results either way */,
  GBMW_FLAG_COOPERATIVE_LAUNCH = 512u /* that single launch goes through the cooperative
                                  launch API, which starts a kernel only when all its
                                  workgroups fit on the device at once (about 15 us more per
                                  solve).  For callers that run several solves, or other
                                  kernels, concurrently on one device: with the plain
                                  launch (default) two such kernels that each hold a part of
                                  the device would wait for tiles that cannot start, until
                                  their waits give up                                     */,
  GBMW_FLAG_TEST_WAIT_GIVES_UP = 256u /* testing: the waits of that single launch ask for a
                                  layer that is never published and give up after 1 ms, so
                                  that the error path can be exercised; every workgroup
                                  still ends normally                                     */
};

#define GBMW_MAX_S 256

/*
 * The problem statement.  L is always a host pointer and is read before the call
 * returns.  c, M and R are all host pointers (ptr_space == GBMW_PTR_HOST) or all
 * device pointers (GBMW_PTR_DEVICE).  Lifetime of the three arrays: the solve
 * reads them from work enqueued on `stream` (host arrays through asynchronous
 * copies, device arrays by its first kernel) and nothing reads them after that
 * work has run; they must stay valid and unchanged until a call that waits for
 * the solve has returned (gbmw_synchronize or any of the result calls), or until
 * the caller has itself waited for `stream`, and may be freed or overwritten
 * then.  Every later call on the context (gbmw_backtrack, gbmw_export_tables,
 * gbmw_select_forward_budget, gbmw_pipeline_cost) works from copies the context
 * owns.  Rows of instance b start at off_b = L[0] + ... + L[b-1];
 * sumL = L[0] + ... + L[B-1].
 */
typedef struct {
  int32_t B;        /* number of instances, >= 1                               */
  int32_t S;        /* strategies per layer, 1..GBMW_MAX_S (shared)            */
  int32_t E;        /* forward budget in units, 0..2^28; tables have rows 0..E */
  const int32_t* L; /* [B] layers per instance, each >= 1                      */
  const float* c;   /* [sumL][S]     c[off_b + l][s]  >= 0, +inf = forbidden   */
  const int32_t* M; /* [sumL][S]     M[off_b + l][s]  >= 0                     */
  const float* R;   /* [sumL][S][S]  R[off_b + l][s_prev][s] >= 0, +inf allowed;
                       the l == 0 slab of every instance is ignored           */
  int32_t ptr_space; /* GBMW_PTR_HOST or GBMW_PTR_DEVICE, for c, M and R       */
  void* stream;      /* hipStream_t to enqueue on, or NULL for the null stream */
} gbmw_problem;

/*
 * Fill the tables of all B instances (Eq. 3 for every l, e, s; then
 * best(e) = min_s C(L_b - 1, e, s)).  Work is enqueued on p->stream and the call
 * returns without waiting for it.
 *
 * *ctx is in/out: pass a pointer to NULL to get a new context; pass a context
 * returned earlier to solve again into the same device buffers (they are
 * re-allocated only if the new problem needs more room; a solve that reuses a
 * context enqueues no allocation).  On error a new context is not created and a
 * passed-in one stays valid but holds no solution.
 *
 * Host inputs are validated before anything is enqueued (GBMW_ERR_INVALID_ARG
 * for NaN, negative or -inf in c/R, negative M, L < 1, sizes out of range).
 * Device inputs are validated by a kernel; a violation makes the next
 * gbmw_synchronize / gbmw_get_best / gbmw_backtrack / gbmw_export_tables on
 * the context return GBMW_ERR_INVALID_ARG (the kernels never read or write out
 * of bounds whatever the values are).
 */
gbmw_status gbmw_dp_solve_batched(const gbmw_problem* p, uint32_t flags, gbmw_ctx** ctx);

/*
 * Read plans back (Algorithm 3's strategy list, obtained by walking the argmin
 * records from the last layer down).  Query i asks for instance q_instance[i]
 * at budget q_e[i] (0 <= q_e <= E).  All five arrays are HOST pointers owned by
 * the caller; the call waits for the solve and for its own kernel.
 *   plan     [nq][Lmax] bytes, Lmax = max_b L_b; entries l >= L_b and every
 *            entry of an infeasible query are 0xFF
 *   cost     [nq] best(e_q) (+inf if infeasible)
 *   mem_used [nq] sum_l M(l, s_l) of the plan (-1 if infeasible)
 * An infeasible query is not an error.
 */
gbmw_status gbmw_backtrack(gbmw_ctx* ctx, int32_t nq, const int32_t* q_instance,
                           const int32_t* q_e, uint8_t* plan, float* cost, int32_t* mem_used);

/*
 * gbmw_backtrack for callers that must not allocate device memory (tight serving
 * loops, harnesses that forbid hipMalloc inside a step, code that prepares a HIP
 * graph capture): same arguments, same results, but the staging block for the
 * queries and the plans is a fixed array of GBMW_STATIC_SCRATCH_BYTES bytes
 * inside the library's device image instead of a buffer of the context.  The
 * call allocates nothing and frees nothing, on the device or through any library.
 * Limit: nq * (16 + Lmax) <= GBMW_STATIC_SCRATCH_BYTES, else
 * GBMW_ERR_UNSUPPORTED (nothing is enqueued).  Every GPU the library runs on
 * holds one such array until the process ends, and all contexts on a GPU share
 * it: calls of this function that overlap in time on one GPU race on it
 * (serialise them); each call overwrites what the last one left, nothing in it
 * has to be cleared.  Waits for the solve and for its own kernel, like
 * gbmw_backtrack.
 */
#define GBMW_STATIC_SCRATCH_BYTES (1 << 20)
gbmw_status gbmw_backtrack_static(gbmw_ctx* ctx, int32_t nq, const int32_t* q_instance,
                                  const int32_t* q_e, uint8_t* plan, float* cost,
                                  int32_t* mem_used);

/*
 * The outer loop of Appendix A, Algorithm 3 on top of a solved context: choose
 * the forward budget E_fwd_opt whose plan also respects the OVERALL memory
 * E_all(plan) <= E of Section 4.1.2, Eq. 2,
 *   E_all = max_i { sum_{k<=i} O_f(k,s_k) + O_b(i,s_i) } + sum_k O_ms(k,s_k),
 * where the context was solved with M = O_f + O_ms and E = the device budget.
 * With b_up = max O_b over the instance's layers and strategies, budgets up to
 * E - b_up need no check; the budgets above are visited in increasing order and
 * the walk stops at the first plan that does not fit (a budget without any
 * feasible plan has nothing to check and is passed over; if E - b_up < 0
 * nothing is valid a priori and the walk starts at 0).
 * O_f, O_b, O_ms: HOST pointers, [sumL][S] each, same row order as M, all >= 0;
 * O_f + O_ms must equal the M of the solve (else GBMW_ERR_INVALID_ARG).
 * Outputs (HOST, caller-owned, any may be NULL):
 *   e_opt [B]        chosen E_fwd (-1: none)
 *   cost  [B]        best(e_opt) (+inf if none or infeasible)
 *   plan  [B][Lmax]  strategies of the chosen plan (0xFF padded / if none)
 *   e_all [B]        overall memory of the chosen plan (-1 if none)
 * Waits for the solve and for its own kernels.
 */
gbmw_status gbmw_select_forward_budget(gbmw_ctx* ctx, const int32_t* O_f, const int32_t* O_b,
                                       const int32_t* O_ms, int32_t* e_opt, float* cost,
                                       uint8_t* plan, int32_t* e_all);

/*
 * Pipeline time of Section 4.2.1, Eq. 5 / Appendix C, Eq. 8 for n_pipe
 * pipelines whose stages are instances of a solved context:
 *   cost = (m - 1) * max_i Cns_i + sum_i C_i
 * over the stages i of the pipeline, with C_i = best(e_i) of the stage's
 * instance at the forward budget e_i chosen for it, and Cns_i the same plan's
 * time re-evaluated with c_nosync (layer times without gradient
 * synchronisation; R unchanged): v = c_ns(0,s_0); v = (v + R(l,s_{l-1},s_l)) +
 * c_ns(l,s_l).  c_nosync == NULL means Cns_i = C_i (Eq. 5).  fp32: the sum is a
 * left fold over the stages in the order given; product and final addition are
 * rounded separately.  A stage with e_i < 0 or no feasible plan makes its
 * pipeline +inf.
 * All pointers HOST:
 *   stage_begin     [n_pipe + 1]  stages of pipeline p are stage_begin[p] ..
 *                                 stage_begin[p+1] - 1 (at least one each)
 *   stage_instance  [n_stage]     instance index of each stage
 *   stage_e         [n_stage]     forward budget of each stage (-1..E)
 *   microbatches    [n_pipe]      m >= 1
 *   c_nosync        [sumL][S]     >= 0, or NULL
 *   cost            [n_pipe]      out
 *   stage_cost, stage_cost_nosync [n_stage] out, either may be NULL
 * Waits for the solve and for its own kernels.
 */
gbmw_status gbmw_pipeline_cost(gbmw_ctx* ctx, int32_t n_pipe, const int32_t* stage_begin,
                               const int32_t* stage_instance, const int32_t* stage_e,
                               const int32_t* microbatches, const float* c_nosync, float* cost,
                               float* stage_cost, float* stage_cost_nosync);

/*
 * The inner while-loop of Algorithm 2 (bi-objective optimisation of the pipeline
 * partition, Section 4.2.2 and Appendix B) for n_chain independent
 * (batch size, PP degree) pairs at once.  Pair k cuts its model of Lm_k layers
 * into P_k stages; a partition p is the list of layer counts per stage.  Starting
 * from p0 (the memory-balanced partition), each round
 *   - searches p: every stage's layers are solved under budget E with that
 *     stage's memory table (Eq. 3), the plan at e = E gives the stage time C_i,
 *     its time without gradient synchronisation Cns_i and its memory O_i; the
 *     pipeline time is Eq. 8, the balance degrees are Eq. 6
 *       alpha_t = 1 - max_i C_i / sum_i C_i,  alpha_m = 1 - max_i O_i / sum_i O_i;
 *   - PP_Partition_Adjust: the slowest stage (lowest index among equals) hands
 *     its boundary layer to the adjacent stage with the smaller time (the earlier
 *     one among equals); a stage of one layer hands nothing over;
 *   - Validate: with every layer keeping the strategy just found, each stage of
 *     the new partition must (1) take no longer than the slowest stage did,
 *     (2) need no more than E, (3) need no more than O_t, the largest stage
 *     memory of the searched time-balanced partition p_t (no such limit when p_t
 *     is NULL or its search is infeasible).  A partition searched before is not
 *     searched again.
 * The chain of a pair ends when the new partition is rejected, when a search is
 * infeasible (pipeline time +inf), or after max_iter searches.  Algorithm 2's
 * value for the pair is the cost of its last trace entry.
 * Rounds of all pairs run in lockstep, each as ONE batched table solve of what the
 * accepted moves invalidated: a stage whose layers did not change keeps its
 * result, a stage that gained a layer at its end runs one more layer step on its
 * kept table, a stage that lost its last layer only reduces best(E) again, a stage
 * whose first layer changed is solved again (GBMW_FLAG_RESOLVE_ALL solves every
 * stage of every live pair from scratch each round, with identical results).
 * Device memory: per (pair, stage) argmin rows for Lm_k - P_k + 1 layers.
 *
 * fp32 contract: stage times as in gbmw_dp_solve_batched; re-evaluations under
 * fixed strategies as in gbmw_pipeline_cost (v = c(a, s_a); v = (v + R(l,
 * s_{l-1}, s_l)) + c(l, s_l); the first layer of a stage pays no R); alpha_t is
 * 1 - max / (left fold of C in stage order), all fp32; alpha_m is computed in
 * fp64 from the integer memories and rounded to fp32; both are 0 for a zero sum
 * and for an infeasible search.
 *
 * All pointers are HOST pointers; the call copies the model in, runs every step
 * in kernels on `stream` (one small device-to-host read of the accept flags per
 * round) and returns when the outputs are complete.  Row order: pairs are
 * concatenated; lrow_k = Lm_0 + .. + Lm_{k-1}, prow_k = P_0 + .. + P_{k-1},
 * mrow_k = P_0*Lm_0 + .. + P_{k-1}*Lm_{k-1}.
 */
typedef struct {
  int32_t n_chain;       /* number of pairs, >= 1                                     */
  int32_t S;             /* strategies, 1..GBMW_MAX_S                                 */
  int32_t E;             /* memory budget of every stage, 0..2^28                     */
  int32_t max_iter;      /* searches per pair, 1..4096                                */
  const int32_t* P;      /* [n_chain] stages, 1..64                                   */
  const int32_t* Lm;     /* [n_chain] layers of the pair's model, >= P_k              */
  const int32_t* m;      /* [n_chain] micro-batches, >= 1                             */
  const float* c;        /* [sum Lm][S]      c[lrow_k + l][s]                         */
  const float* c_nosync; /* [sum Lm][S]      or NULL (then Cns = C)                   */
  const float* R;        /* [sum Lm][S][S]   R[lrow_k + l][s_prev][s]; the slab of a
                            stage's first layer is not used                          */
  const int32_t* M;      /* [sum P*Lm][S]    M[mrow_k + i*Lm_k + l][s]: layer l under s
                            when it belongs to stage i                               */
  const int32_t* p0;     /* [sum P]          p0[prow_k + i] >= 1, summing to Lm_k     */
  const int32_t* p_t;    /* [sum P] or NULL  the time-balanced partition              */
  void* stream;          /* hipStream_t or NULL                                       */
  /* Outer loops of Algorithm 1 / 2 (optional, both or neither): the pairs of one batch
   * size form a group (its PP degrees); groups are numbered 0, 1, ... in the order the
   * batch sizes are tried and batch_group is non-decreasing over the pairs.           */
  const float* batch_size;    /* [n_chain] global batch size B of the pair's group, > 0  */
  const int32_t* batch_group; /* [n_chain] group of each pair                            */
  /* Stage searches with the overall-memory check of Appendix A, Algorithm 3 (optional,
   * both or neither; indexed like M).  M is then the forward memory O_f + O_ms of Eq. 2,
   * O_ms its model-state part and O_b the backward activations.  Every stage's plan is
   * read at the largest forward budget e <= E whose plan has E_all <= E (walking up
   * from E - max O_b of the stage's layers; budgets without a plan are passed over, the
   * walk stops at the first plan that does not fit), and the memory of a stage -- the
   * O output, alpha_m, limits 2 and 3, O_t -- is E_all of its plan instead of its
   * forward memory.                                                                   */
  const int32_t* O_b;         /* [sum P*Lm][S] >= 0                                      */
  const int32_t* O_ms;        /* [sum P*Lm][S] 0 <= O_ms <= M                            */
} gbmw_partition_problem;

/* Outputs of gbmw_partition_search; HOST memory owned by the caller.  Pmax = max P_k,
 * Lmmax = max Lm_k.  Entry j of pair k's trace is its j-th searched partition;
 * entries j >= n_iter[k] and stage slots i >= P_k are left untouched.  Any pointer
 * except n_iter may be NULL. */
typedef struct {
  int32_t* n_iter;   /* [n_chain]                    searches done (>= 1)             */
  int32_t* O_t;      /* [n_chain]                    limit 3 (INT32_MAX: none)        */
  int32_t* p;        /* [n_chain][max_iter][Pmax]    partition                        */
  float* cost;       /* [n_chain][max_iter]          Eq. 8 (+inf: infeasible)         */
  float* C;          /* [n_chain][max_iter][Pmax]    stage times (+inf: infeasible)   */
  float* Cns;        /* [n_chain][max_iter][Pmax]                                     */
  int32_t* O;        /* [n_chain][max_iter][Pmax]    stage memories (-1: infeasible)  */
  float* alpha_t;    /* [n_chain][max_iter]                                           */
  float* alpha_m;    /* [n_chain][max_iter]                                           */
  uint8_t* strat;    /* [n_chain][Lmmax]  strategies of the last searched partition
                        (0xFF: layer of an infeasible stage, or l >= Lm_k)           */
  int32_t rounds;        /* out: lockstep rounds, the p_t round included              */
  int32_t stage_solves;  /* out: stage instances solved over all rounds               */
  int64_t cell_updates;  /* out: sum over them of (layers - 1) * (E + 1) * S * S      */
  float device_ms;       /* out: first launch to last kernel, HIP events on `stream`  */
  /* With batch sizes given: per group C_opt = min over its pairs of the pair's value
   * (the cost of its last trace entry); groups are visited in order, the visit ends at
   * the first group whose C_opt is +inf (out of memory), and Tpt = max B / C_opt over
   * the groups visited before it (fp32 division; the first group on a tie).           */
  float tpt;             /* out: Tpt (0 if the first group is already infeasible, or no
                            batch sizes were given)                                   */
  int32_t tpt_group;     /* out: group that gave Tpt (-1: none)                       */
  int32_t tpt_pair;      /* out: its pair with the smallest cost (lowest index among equals) */
} gbmw_partition_result;

/*
 * *ctx is in/out as for gbmw_dp_solve_batched: the context supplies the device
 * buffers of the table solves and of the search state and can be handed to later
 * calls of either kind; after the call it holds no solution.  Inputs are
 * validated on the host first (GBMW_ERR_INVALID_ARG: NaN or negative c / c_nosync
 * / R, negative M, O_b or O_ms, O_ms above M, a partition with an empty stage or
 * the wrong sum, sizes out of range).
 */
gbmw_status gbmw_partition_search(const gbmw_partition_problem* q, uint32_t flags,
                                  gbmw_partition_result* out, gbmw_ctx** ctx);

/*
 * Candidate hybrid-parallelism strategies of one layer on a device group of
 * `group_size` devices (Section 3.2): every decision tree whose levels are
 * distinct paradigms out of DP, SDP and TP (at most three levels), each with a
 * degree from {2, 4, 8, ...}, the degrees multiplying to group_size; the order
 * of the levels matters (level 0 is the outermost, i.e. spans the slowest
 * links).  takeaway3 != 0 drops the trees that hold both DP and SDP; with_ckpt
 * != 0 lists every tree twice, first all without, then all with activation
 * checkpointing.  For 8 devices and PP degrees 1/2/4/8 (groups of 8/4/2/1) this
 * gives 21+9+3+1 = 34 trees, 68 with CKPT, and 11+7+3+1 = 22, 44 with CKPT,
 * after Takeaway #3.
 * Order: fewer levels first, then the degree tuples in lexicographic order, then
 * the paradigm tuples in lexicographic order with DP < SDP < TP.
 * Host-only routine (no device work).  Returns the number of strategies, writing
 * at most `cap` of them to `out` (out may be NULL to ask for the count);
 * -1 if group_size is not a power of two in 1..2^20.
 */
enum { GBMW_DP = 1, GBMW_SDP = 2, GBMW_TP = 3 };
typedef struct {
  int32_t n_levels;   /* 0..3                                   */
  int32_t kind[3];    /* GBMW_DP / GBMW_SDP / GBMW_TP, outer first; 0 beyond n_levels */
  int32_t degree[3];  /* 2, 4, 8, ...; 0 beyond n_levels        */
  int32_t ckpt;       /* 1: activation checkpointing            */
} gbmw_strategy;

int32_t gbmw_enumerate_strategies(int32_t group_size, int32_t with_ckpt, int32_t takeaway3,
                                  gbmw_strategy* out, int32_t cap);

/*
 * A small analytic cost model in the spirit of Section 5 that turns layer
 * shapes into the inputs of the search, evaluated on the device for every
 * (layer, strategy) and (layer, strategy pair).  Fixed by the paper: backward
 * computation is twice the forward; all-reduce moves 2(N-1)/N and SDP 3(N-1)/N
 * of the parameter bytes (Takeaway #3); CKPT adds one forward pass (with TP's
 * all-reduce) to the backward step, keeps only the boundary activations in the
 * forward pass and needs the intermediate ones during backward (Section 3.1);
 * computation and communication that overlap slow each other down by `slow`
 * (1.3 in Section 5); O_f / O_b / O_ms as in Eq. 2.  The rest is this library's
 * modelling choice, stated here in full.  With dp, sdp, tp the degrees of the
 * strategy (1 if absent), span_x = degree_x times the degrees of the levels
 * inside level x, bw(span) = span <= island ? bw_in : bw_out, all in fp64 and in
 * exactly this order of operations:
 *   lb     = Bm / (dp * sdp)                           samples per device
 *   t_f    = lb * flops / tp / rate
 *   tp_ar  = tp > 1 ? 2 (tp-1) / tp * (lb * bnd) / bw(span_tp) : 0
 *   pbytes = params * param_bytes / tp
 *   sdp_ag = sdp > 1 ? (sdp-1) / sdp * pbytes / bw(span_sdp) : 0
 *   dp_ar  = dp > 1 ? 2 (dp-1) / dp * pbytes / bw(span_dp) : 0
 *   fwd    = t_f + tp_ar + sdp_ag
 *   bwd    = 2 t_f + tp_ar, plus (t_f + tp_ar) under CKPT
 *   ov(a,b) = slow * min(a,b) + (max(a,b) - min(a,b))
 *   c      = fwd + ov(bwd, sdp_ag + (dp_ar + sdp_ag))   c_nosync = fwd + ov(bwd, sdp_ag)
 *   ms     = params * state_bytes / (tp * sdp)
 *   act_f  = CKPT ? lb * bnd : lb * (bnd + intm / tp);  act_b = CKPT ? lb * (intm / tp) : 0
 *   O_ms, O_f, O_b = ceil(ms | act_f | act_b / unit_bytes)
 *   M[i]   = O_ms + (P - i) * O_f     stage i of a 1F1B pipeline keeps P - i micro-batches
 *   R(l, s', s) = 0 if the two strategies lay the activations out alike (same
 *            sequence of levels with DP and SDP both counted as batch splits), else
 *            Bm * bnd(l-1) * share / bw_out with b = dp * sdp, share = |1/b - 1/b'| if
 *            b != b' else 1/b; the l == 0 slab is zero.
 * c, c_nosync, R are rounded to fp32 at the end.
 * layers, strategies, hw: HOST pointers.  Outputs: all HOST (out_space ==
 * GBMW_PTR_HOST) or all DEVICE pointers (GBMW_PTR_DEVICE; filled in place, ready to
 * be handed to gbmw_dp_solve_batched); any may be NULL.  The kernels run on `stream`
 * and the call returns when they have finished (it reads back their range check).  Shapes: c, c_nosync [L][S] fp32; O_f, O_b,
 * O_ms [L][S] int32; M [P][L][S] int32; R [L][S][S] fp32.
 * GBMW_ERR_INVALID_ARG: sizes out of range, a strategy that breaks the rules
 * above, non-positive rate / bandwidth / unit, negative shapes, or a memory that
 * does not fit int32.
 */
typedef struct {
  double params; /* parameter count                         */
  double flops;  /* forward FLOPs per sample                */
  double bnd;    /* boundary activation bytes per sample    */
  double intm;   /* intermediate activation bytes per sample */
} gbmw_layer_shape;

typedef struct {
  double rate;        /* device FLOP/s                                      */
  double bw_in;       /* bytes/s inside an island                           */
  double bw_out;      /* bytes/s across islands                             */
  double param_bytes; /* bytes per parameter on the wire                    */
  double state_bytes; /* bytes of model state per parameter (weights, gradients, optimizer) */
  double slow;        /* slowdown of overlapped compute / communication, >= 1 */
  double unit_bytes;  /* bytes per memory unit of the search's budget axis  */
  int32_t island;     /* devices per island                                 */
} gbmw_hardware;

gbmw_status gbmw_cost_model(const gbmw_layer_shape* layers, int32_t L,
                            const gbmw_strategy* strategies, int32_t S, const gbmw_hardware* hw,
                            double Bm, int32_t P, int32_t out_space, float* c, float* c_nosync,
                            int32_t* O_f, int32_t* O_b, int32_t* O_ms, int32_t* M, float* R,
                            void* stream);

/* Lmax of the last solve (row length of `plan` above); 0 if none. */
int32_t gbmw_max_layers(const gbmw_ctx* ctx);

/*
 * best [B][E+1] fp32 and best_s [B][E+1] bytes (lowest-index argmin over s of
 * the last layer; 0 where best is +inf), to HOST memory.  Either may be NULL.
 * Waits for the solve.
 */
gbmw_status gbmw_get_best(gbmw_ctx* ctx, float* best, uint8_t* best_s);

/*
 * Copy the tables of layers [l0, l1) of one instance to HOST memory in the
 * logical layout [l - l0][e][s] (s fastest, e = 0..E), whatever the device
 * layout is.  C (fp32) and A (bytes) may each be NULL.  A[l][e'][s] is the
 * predecessor strategy recorded for layer l (l >= 1) under s when e' units are
 * left for layers < l (i.e. before layer l's own M is added); the l == 0 slab
 * is returned as zeros.  Without GBMW_FLAG_KEEP_ALL_C only the last two layers
 * of C exist: asking for others returns GBMW_ERR_UNSUPPORTED.  Waits for the
 * solve.
 */
gbmw_status gbmw_export_tables(gbmw_ctx* ctx, int32_t instance, int32_t l0, int32_t l1,
                               float* C, uint8_t* A);

/* Wait for everything the context enqueued; reports deferred validation. */
gbmw_status gbmw_synchronize(gbmw_ctx* ctx);

/*
 * Device time of the last solve, in milliseconds, from HIP events recorded on
 * the solve's stream: total_ms spans the first kernel launch to the last
 * kernel's completion; minplus_ms is the sum over the min-plus (Eq. 3 inner
 * minimum, fused with the shift-add) launches and minplus_launches their count
 * (both 0 unless the solve was given GBMW_FLAG_TIME_KERNELS).  Waits for the
 * solve.  Any pointer may be NULL.
 */
gbmw_status gbmw_last_solve_ms(gbmw_ctx* ctx, float* total_ms, float* minplus_ms,
                               int32_t* minplus_launches);

/*
 * What the min-plus launches of the last solve really computed, for roofline
 * accounting (all zero unless the solve was given GBMW_FLAG_COUNT_WORK).  launch
 * selects one min-plus launch of the solve, in the order they were enqueued
 * (0 is the launch of layer 1, whose input is layer 0's closed form and is not
 * read from memory), or -1 for the sum over all of them.  With the run shortcut
 * of Eq. 3's fill (see GBMW_FLAG_DENSE_ARITHMETIC) a group of budgets that reads
 * one and the same column of the previous table is computed once:
 *   work[0]  workgroups (256 budgets) computed once:      S * S candidate updates each
 *   work[1]  waves (64 budgets) computed once, recognised
 *            from the summaries:                          S * S updates each
 *   work[2]  the same, recognised from the loaded table:  S * S updates each
 *   work[3]  (wave, output strategy) rows computed cell
 *            by cell:                                     64 * S updates each
 * Waits for the solve.
 */
gbmw_status gbmw_last_solve_work(gbmw_ctx* ctx, int32_t launch, uint64_t work[4]);

/* Free the context and its device memory (waits first).  NULL is allowed. */
void gbmw_destroy(gbmw_ctx* ctx);

/* Message of the calling thread's most recent failure ("" if none). */
const char* gbmw_last_error(void);

/* Library / kernel variant description, e.g. for benchmark records. */
const char* gbmw_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GBMW_H */
