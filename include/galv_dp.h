/*
 * galv_dp.h — C ABI of the batched plan-search dynamic program for AMD MI355X (gfx950).
 *
 * The library solves, for many independent search instances at once, the
 * layer-by-layer dynamic program that picks one parallelism strategy per model
 * layer under a device memory budget (paper section 3.3, "Dynamic Programming
 * Search", Eq. 1; it is the routine Algorithm 1 calls once per batch size,
 * pipeline degree and stage).  For an instance with L layers, S candidate
 * strategies and budget E it finds the plan p in {0..S-1}^L with
 * sum_l m(l, p_l) <= E that minimises
 *
 *     sum_l c(l, p_l)  +  sum_{l >= 1} R_{r_idx[l]}(p_{l-1}, p_l)
 *
 * through the recurrence  C[l][e][s] = c(l,s) + min_{s'} ( C[l-1][e - m(l,s)][s'] + R(s', s) ),
 * C[0][e][s] = c(0,s) when m(0,s) <= e, followed by an argmin walk over stored
 * back-pointers.  Costs are exact 64-bit integers; every minimum is broken
 * towards the lowest index; "infinity" (no admissible plan: the paper's
 * Out-Of-Memory outcome) is GALV_INF.
 *
 * Conventions
 *  - Pointers named *_dev are DEVICE pointers (HBM of the current HIP device);
 *    everything else is host memory.  `stream` is a hipStream_t passed as void*
 *    (NULL = the default stream).
 *  - The caller owns all device buffers, including the workspace, and keeps the
 *    inputs alive and unchanged until the stream has passed the calls that read
 *    them (m_dev and budget_dev until the last backtrack / export of that solve).
 *  - solve / backtrack / export only enqueue work; they never synchronise the host and
 *    never allocate.  Everything is ordered after the work already in `stream` and
 *    before whatever is enqueued in `stream` afterwards.  Instances are independent,
 *    so a solve may spread their layer sweeps over internal streams of the handle
 *    (forked from and joined back into `stream` with events; see GALV_DP_STREAMS),
 *    which lets sweeps of different instances overlap across layer boundaries.
 *    galv_dp_create touches no device memory (it may create those streams, and 64
 *    bytes of pinned host memory through which a solve tells the next one how many
 *    budget columns the batch really has).
 *  - Errors in host-visible arguments are returned as codes (never exceptions,
 *    never abort); galv_dp_last_error() gives a thread-local message.
 *  - Input VALUES live on the device and cannot be checked synchronously: a
 *    per-instance device status (galv_dp_get_status) reports them instead.
 *    An instance with invalid values yields GALV_INF / -1 like an infeasible one.
 *  - Preconditions on values: c >= 0, R >= 0, m >= 0, 0 <= budget <= max_budget,
 *    0 <= r_idx < n_transition, and  sum_l max_s c(l,s) + sum_{l>=1} max R_{r_idx[l]} < 2^62.
 *  - One handle serves one solve at a time: concurrent calls on one handle race.
 */
#ifndef GALV_DP_H
#define GALV_DP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct galv_dp galv_dp_t; /* opaque handle, host memory, owned by the library */

#define GALV_INF ((int64_t)1 << 62) /* "infinity": infeasible / Out-Of-Memory */

typedef enum {
    GALV_OK = 0,
    GALV_ERR_INVALID_ARG = 1, /* NULL pointer, size out of range, bad instance index     */
    GALV_ERR_WORKSPACE = 2,   /* workspace NULL, misaligned (256 B) or too small         */
    GALV_ERR_RANGE = 3,       /* sizes whose tables cannot be indexed (overflow)         */
    GALV_ERR_HIP = 4,         /* a HIP runtime call failed; see galv_dp_last_error()     */
    GALV_ERR_STATE = 5        /* call order: backtrack / export / status before a solve  */
} galv_status_t;

/* Problem shape, common to all instances of a batch. */
typedef struct {
    int32_t n_instances;  /* B  >= 1 */
    int32_t n_layers;     /* L  >= 1 */
    int32_t n_strategies; /* S  in [1, 1024] */
    int32_t max_budget;   /* E_max >= 0: tables have E_max + 1 budget columns            */
    int32_t n_transition; /* nR >= 1 transition matrices per instance                    */
    uint32_t flags;       /* GALV_DP_* below, 0 for defaults                             */
} galv_dp_desc_t;

/* flags */
#define GALV_DP_FORCE_INT64 1u /* always use the general 64-bit integer kernels, even when
                                  an instance's values would allow the faster exact path */
#define GALV_DP_BP_U8 2u       /* keep back-pointers in one byte instead of four (internal
                                  storage only: results are identical); needs n_strategies <= 255.
                                  Shrinks the largest table of the workspace by 4x.  The sweep
                                  then keeps rolling cost rows (9 bytes per state); where the
                                  single packed table applies (GALV_DP_FORCE_PACK) that form is
                                  the faster one, and this flag buys memory, not time */

#define GALV_DP_NO_U32 4u      /* do not use the 32-bit integer-key kernels (see
                                  GALV_INSTANCE_OK_FAST_U32); the 64-bit-key ones take over   */
#define GALV_DP_NO_PEEK 8u     /* always fetch every usable former-layer row (see below)          */
#define GALV_DP_FORCE_PEEK 16u /* 32-bit-key sweep: look at a row's cells in a tile's first and last
                                  column before fetching the row, and skip the fetch when they show
                                  that the row cannot win any minimum of the tile.  By default this
                                  is done when a layer has enough workgroups to fill the chip (the
                                  sweep is then bound by bytes; below that it is bound by latency
                                  and the extra dependent step costs more than it saves).  Results
                                  are identical either way.                                          */
#define GALV_DP_NO_PACK 32u    /* 32-bit-key instances: always keep the rolling cost rows and plain
                                  back-pointers (see GALV_DP_FORCE_PACK)                            */
#define GALV_DP_FORCE_PACK 64u /* 32-bit-key instances, int32 back-pointers, at most 256 strategies:
                                  keep a SINGLE table, in which the back-pointer word of a state also
                                  carries its cost relative to the smallest former cost of its budget
                                  column, plus one such minimum per column; no cost rows are written.
                                  Half the bytes per state.  By default this is done when a layer has
                                  enough workgroups to fill the chip (as for GALV_DP_FORCE_PEEK).
                                  Results, exported tables included, are identical either way.       */
#define GALV_DP_FORCE_WIDE_TILES 128u   /* sweep workgroups take tiles of 256 budget columns instead of 128
                                           (17 to 256 strategies: the kernel variants that have such a twin).
                                           By default this is done when a layer has enough workgroups to
                                           fill the chip, as for GALV_DP_FORCE_PEEK.  Results are identical. */
#define GALV_DP_NO_WIDE_TILES 0x2000u   /* always 128-column tiles                                           */
#define GALV_DP_STREAMS_SHIFT 8 /* bits 8..12: how many internal streams the layer sweeps are   */
#define GALV_DP_STREAMS_MASK 0x1f00u /* spread over; 1 = none, at most 16; 0 = chosen by the library:
                                        galv_dp_create makes as many as the shape could use with every
                                        budget at max_budget, and each solve takes as many of them as
                                        suit the budgets that the handle's PREVIOUS solve met (its
                                        preparation kernel leaves their tile count in a word of
                                        pinned host memory; no solve waits for it, and before the
                                        first solve max_budget stands in).  Results never depend on it. */
#define GALV_DP_STREAMS(n) ((uint32_t)(n) << GALV_DP_STREAMS_SHIFT)

/* Per-instance status codes written by solve (see galv_dp_get_status). */
#define GALV_INSTANCE_OK_FAST 0      /* packed-key kernels, costs stored in 32 bits (all plan
                                        costs plus the largest R stay below 2^31)          */
#define GALV_INSTANCE_OK_INT64 1     /* general 64-bit integer kernels                      */
#define GALV_INSTANCE_OK_FAST_WIDE 2 /* packed-key kernels, costs stored in 64 bits (cost
                                        times the next power of two >= S stays below 2^52)  */
#define GALV_INSTANCE_OK_FAST_U32 3   /* as OK_FAST and, besides, (2 * largest R + 2) * 2^k <= 2^32
                                        (k = index bits): keys of relative costs in 32-bit
                                        integers, three instructions per two candidates      */
#define GALV_INSTANCE_OK_U32_WIDE 4   /* plan costs beyond 32-bit cells, but (2 * largest R + 2) * 2^k <= 2^32
                                        and n_strategies <= 256: the same 32-bit keys of relative
                                        costs (their width depends on R only), over 64-bit cells  */
#define GALV_INSTANCE_BAD_VALUE (-1) /* a value violates the preconditions above            */

/*
 * Bytes of device workspace a handle for `desc` needs (rolling cost rows,
 * back-pointers for layers 1..L-1, packed transition tables, per-instance
 * state): roughly B * S * (E_max + 1) * (4 * (L - 1) + 32) bytes.
 */
galv_status_t galv_dp_workspace_bytes(const galv_dp_desc_t *desc, size_t *bytes);

/*
 * Create a handle over caller-owned workspace (256-byte aligned device memory
 * of at least galv_dp_workspace_bytes).  The handle keeps the pointer; the
 * workspace must outlive it.  The device that is current at this call is the
 * one every later call on the handle must run on.
 */
galv_status_t galv_dp_create(const galv_dp_desc_t *desc, void *workspace_dev,
                             size_t workspace_bytes, galv_dp_t **out);

/*
 * Run the recurrence of Eq. 1 for all B instances (layers 0..L-1, every budget
 * column 0..budget[b]) and the final minimum at e = budget[b].
 *   c_dev      [B][L][S]      int64  execution time c(l, s)
 *   m_dev      [B][L][S]      int32  memory units m(l, s); m > budget[b] => (l, s) unusable
 *   R_dev      [B][nR][S][S]  int64  R[k][s_prev][s_cur], cost of changing layout between
 *                                    a layer on s_prev and the next layer on s_cur
 *   r_idx_dev  [B][L]         int32  matrix k used between layer l-1 and l (entry 0 unused);
 *                                    NULL => matrix 0 everywhere
 *   budget_dev [B]            int32  budget of each instance
 *   best_cost_dev [B]  out    int64  optimum, GALV_INF when no plan fits
 *   best_last_dev [B]  out    int32  strategy of layer L-1 in the optimal plan, -1 if none
 */
galv_status_t galv_dp_solve_batched(galv_dp_t *h, const int64_t *c_dev, const int32_t *m_dev,
                                    const int64_t *R_dev, const int32_t *r_idx_dev,
                                    const int32_t *budget_dev, int64_t *best_cost_dev,
                                    int32_t *best_last_dev, void *stream);

/*
 * Recover the optimal plan of every instance of the last solve (the per-layer strategies
 * that the search of section 3.3 returns besides the minimum time cost: Algorithm 1's
 * output) by walking the back-pointers from (L-1, budget[b], best_last[b]) to layer 0.
 *   plan_dev [B][L] out int32  strategy index per layer; all -1 when no plan fits.
 * Must be enqueued on the same stream as (or ordered after) the solve.
 */
galv_status_t galv_dp_backtrack(galv_dp_t *h, int32_t *plan_dev, void *stream);

/*
 * Solve and backtrack in one call that ALLOCATES NOTHING, for callers that cannot allocate
 * device memory or create a handle: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same results as galv_dp_create + galv_dp_solve_batched +
 * galv_dp_backtrack, same kernels; the workspace is a fixed array of GALV_DP_STATIC_BYTES
 * inside the library's code object (one copy per GPU, held until the process ends), found
 * once per device through hipGetSymbolAddress.
 *   desc       shape and flags as for galv_dp_create; GALV_DP_STREAMS must be 0 or 1 (all
 *              work runs on `stream`).  A shape whose galv_dp_workspace_bytes exceeds
 *              GALV_DP_STATIC_BYTES is refused with GALV_ERR_WORKSPACE and nothing is enqueued.
 *   inputs and best_cost_dev / best_last_dev as for galv_dp_solve_batched, plan_dev [B][L]
 *              as for galv_dp_backtrack; all must stay alive until `stream` has passed the call.
 * No hipMalloc / hipFree, no stream or event creation, no host synchronisation.  Every call
 * on a GPU uses that GPU's one array, which keeps the previous call's contents (the solve
 * rewrites all it reads): calls that overlap in time on one GPU, on whatever streams, race.
 */
#define GALV_DP_STATIC_BYTES (32u << 20)
galv_status_t galv_dp_solve_static(const galv_dp_desc_t *desc, const int64_t *c_dev,
                                   const int32_t *m_dev, const int64_t *R_dev,
                                   const int32_t *r_idx_dev, const int32_t *budget_dev,
                                   int64_t *best_cost_dev, int32_t *best_last_dev, int32_t *plan_dev,
                                   void *stream);

/*
 * All budgets at once.  The table has "at most e" semantics (the optimal-substructure
 * argument of section 3.3: the optimum of a smaller budget E' <= E is a sub-problem
 * of the same table), so one solve at budget[b] answers every smaller budget, as
 * when one model is planned for several memory limits (Table 1's 8/12/16/20 GB columns).
 *   best_cost_dev [B][E_max+1] out int64  min_s C[L-1][e][s]; GALV_INF if none or e > budget[b]
 *   best_last_dev [B][E_max+1] out int32  lowest minimising s, -1 if none.  May be NULL.
 */
galv_status_t galv_dp_best_per_budget(galv_dp_t *h, int64_t *best_cost_dev, int32_t *best_last_dev,
                                      void *stream);

/*
 * Optimal plans for n_queries (instance, budget) pairs of the last solve, each as
 * if that instance had been solved with that budget (0 <= budget <= budget[b]).
 *   instance_dev [Q] int32, budget_dev [Q] int32
 *   cost_dev     [Q]    out int64  optimum or GALV_INF.  May be NULL.
 *   plan_dev     [Q][L] out int32  all -1 when no plan fits or the query is out of range.
 */
galv_status_t galv_dp_backtrack_queries(galv_dp_t *h, int32_t n_queries, const int32_t *instance_dev,
                                        const int32_t *budget_dev, int64_t *cost_dev,
                                        int32_t *plan_dev, void *stream);

/*
 * Test / debug: write one instance's tables of the last solve in canonical
 * order, as the recurrence defines them.
 *   C_last_dev [E_max+1][S]      int64  C[L-1][e][s]; GALV_INF when unreachable or e > budget
 *   bp_dev     [L][E_max+1][S]   int32  minimising s' of cell (l, e, s); -1 for layer 0,
 *                                       unreachable cells and e > budget.  May be NULL.
 */
galv_status_t galv_dp_export_tables(galv_dp_t *h, int32_t instance, int64_t *C_last_dev,
                                    int32_t *bp_dev, void *stream);

/* Copy the per-instance status codes of the last solve: status_dev [B] int32. */
galv_status_t galv_dp_get_status(galv_dp_t *h, int32_t *status_dev, void *stream);

/*
 * Work statistics of the last solve, for instances on the 32-bit-key path (zeros otherwise):
 *   stats_dev [B][3] int64  [b][0] former-layer rows actually reduced, [b][1] usable rows listed,
 *                           [b][2] rows fetched from the cost table, each summed over the budget
 *                           tiles and the layers 1..L-1.
 * The sweep leaves out rows that cannot win any minimum of a tile (cost above the column minimum
 * by more than the largest transition cost, in every column of the tile), and does not even fetch
 * a row when two of its cells show as much; [b][0] / [b][1] is the share of the min-plus
 * candidates of Eq. 1 that was evaluated, [b][2] / [b][1] the share of the cost cells that was
 * read.  Results do not depend on either.
 */
galv_status_t galv_dp_get_stats(galv_dp_t *h, int64_t *stats_dev, void *stream);

/*
 * What galv_dp_create chose for this handle from the shape and the flags (host call, no GPU work):
 *   config [4] HOST int32  [0] 1 if 32-bit-key instances keep the single packed table (see
 *                              GALV_DP_FORCE_PACK), [1] 1 if the sweep peeks before it fetches a
 *                              row (GALV_DP_FORCE_PEEK), [2] internal streams the last solve used
 *                              (before any solve: what the first will use), [3] budget columns
 *                              per sweep workgroup.
 * For benchmarks and tests that account for bytes moved; results never depend on any of it.
 */
galv_status_t galv_dp_get_config(const galv_dp_t *h, int32_t *config);

/*
 * Outer loop of Algorithm 1 ("Optimization Workflow" of section 3.3) over a window of
 * candidate batch sizes, on the device, from stage optima that galv_dp_solve_batched wrote.
 * For batch size ib and pipeline degree P = pp_degree[ip] the time cost is the sum of its P
 * stage optima (GALV_INF if any stage has no plan that fits); C_opt is the minimum over the
 * degrees (lowest ip on ties); batch sizes are scanned in the order given and the state keeps
 * the one with the largest throughput batch_size / C_opt (compared exactly as integers; the
 * earlier one on ties) until the first batch size whose C_opt is GALV_INF (Out-Of-Memory),
 * where the scan stops for good.
 *   pp_degree      [n_pp]  HOST int32  pipeline degrees, 1 <= n_pp <= 16
 *   stage_cost_dev         int64  for ip = 0..n_pp-1 in turn a block [n_batch][pp_degree[ip]]
 *                                 of stage optima (the best_cost outputs of one solve per degree)
 *   batch_size_dev [n_batch] int64  the batch sizes B > 0 of this window
 *   batch_index_base       added to the window-local index when recording the best batch size
 *   first_window           non-zero: start from an empty state (throughput 0); zero: continue
 *                          from *state_dev as an earlier call left it
 *   c_p_dev  [n_batch][n_pp] out int64  the time costs C_P
 *   state_dev  in/out      see galv_alg1_state_t
 * Precondition: each sum of stage optima stays below 2^62 (a larger sum reads as GALV_INF).
 * Enqueues one small kernel on `stream`; never synchronises or allocates.
 */
typedef struct {
    int64_t batch_size;  /* B of the best throughput so far; 0 while there is none          */
    int64_t cost;        /* its C_opt; throughput = batch_size / cost                        */
    int32_t pp_index;    /* index into pp_degree of the degree that gave C_opt; -1 if none   */
    int32_t batch_index; /* batch_index_base + window index of that batch size; -1 if none   */
    int32_t stopped;     /* 1 once a batch size fitted under no pipeline degree              */
    int32_t n_explored;  /* batch sizes examined before stopping                             */
} galv_alg1_state_t;

galv_status_t galv_alg1_reduce(int32_t n_batch, int32_t n_pp, const int32_t *pp_degree,
                               const int64_t *stage_cost_dev, const int64_t *batch_size_dev,
                               int32_t batch_index_base, int32_t first_window, int64_t *c_p_dev,
                               galv_alg1_state_t *state_dev, void *stream);

/*
 * Coarse-grained exploration (the complexity remark that closes the "Dynamic Programming
 * Search" paragraph of section 3.3: fuse layers, count memory in larger units), as a
 * pre-pass that writes a smaller problem for galv_dp_solve_batched.
 *   fuse >= 1         consecutive layers [j*fuse, min(L, (j+1)*fuse)) become fused layer j and
 *                     run ONE strategy s:  c'(j,s) = sum of c(l,s) + sum over the group's inner
 *                     boundaries of R_{r_idx[l]}(s,s);  the transition into the group keeps the
 *                     selector of its first layer: r_idx'(j) = r_idx[j*fuse].  L' = ceil(L/fuse).
 *   granularity >= 1  memory unit multiplier g:  m'(j,s) = ceil(sum of m(l,s) / g),
 *                     budget'[b] = floor(budget[b] / g).  A (j,s) with a layer that alone exceeds
 *                     budget[b], or whose m' exceeds budget', is marked unusable (m' = budget'+1).
 * Rounding memory up and the budget down keeps every coarse plan feasible for the original
 * problem at the same cost, so the coarse optimum is an upper bound of the fine one; it is
 * exact when fuse = 1 and every m and budget is a multiple of g.
 * Inputs as in galv_dp_solve_batched (r_idx_dev may be NULL); R is used as it is by the coarse solve.
 *   c_out_dev [B][L'][S] int64, m_out_dev [B][L'][S] int32, r_idx_out_dev [B][L'] int32,
 *   budget_out_dev [B] int32.
 */
galv_status_t galv_dp_coarsen(int32_t n_instances, int32_t n_layers, int32_t n_strategies,
                              int32_t n_transition, int32_t fuse, int32_t granularity,
                              const int64_t *c_dev, const int32_t *m_dev, const int64_t *R_dev,
                              const int32_t *r_idx_dev, const int32_t *budget_dev, int64_t *c_out_dev,
                              int32_t *m_out_dev, int32_t *r_idx_out_dev, int32_t *budget_out_dev,
                              void *stream);

/* Plan of the original layers from a plan of fused layers: plan[b][l] = coarse_plan[b][l / fuse].
 *   coarse_plan_dev [B][ceil(L/fuse)] int32, plan_dev [B][L] out int32. */
galv_status_t galv_dp_expand_plan(int32_t n_instances, int32_t n_layers, int32_t fuse,
                                  const int32_t *coarse_plan_dev, int32_t *plan_dev, void *stream);

/* Free the handle: its host memory, its internal streams and events, its word of pinned host memory
 * (the workspace stays the caller's).  Call it once the streams given to this handle's solves have
 * passed that work: a solve still in flight reads the handle's tables and writes that word.  NULL is
 * allowed. */
galv_status_t galv_dp_destroy(galv_dp_t *h);

/* Message of the last error on this thread ("" if none). Never NULL. */
const char *galv_dp_last_error(void);

/*
 * How this binary was built.  The layer sweep prefetches transition costs with scalar loads
 * issued by hand, which is only safe if the compiler did not touch their destination
 * registers while a load was in flight; the package's build step verifies that on the device
 * assembly that goes into the library and then stamps it "isa-checked ..." (source and flag
 * digest, compiler version).  A build made any other way says "unchecked" and must not run
 * on a GPU; the Python binding refuses to load it.  Never NULL.
 */
const char *galv_dp_build_stamp(void);

#ifdef __cplusplus
}
#endif
#endif /* GALV_DP_H */
