/*
 * jsv - allocation search for compound inference serving, on one AMD MI355X.
 *
 * For every task of a compound-inference task graph the search picks one
 * (model variant, spatial-partition size, batch size) tuple, replicated as often
 * as the demand needs, such that the end-to-end latency and accuracy SLOs hold
 * and the number of GPU partition units is minimal.  This is the optimisation of
 * Section 3.2 of the paper (Eq. 1-14) restricted to one tuple per task and to
 * the cost term of the objective, solved by exhaustive enumeration on the GPU.
 * Switches widen it: the paper's full objective (jsv_set_objective), per-variant
 * multiplicative factors (jsv_set_factors), two tuples per task (jsv_set_mixtures),
 * the search spaces of the paper's ablations (jsv_set_search_space); jsv_set_bounds
 * and jsv_set_graph_mode change how the search runs, not what it returns.
 *
 * Conventions
 *   choice id      c = (v*P + p)*B + b            (variant slowest, batch fastest)
 *   candidate      one choice per task; index i = sum_t d_t * prod_{u<t} K_u where
 *                  d_t is the position of task t's choice in its surviving list
 *                  (ascending c) and K_t that list's length; task 0 is the fastest
 *                  digit.  Without pruning K_t = C = V*P*B and d_t = c_t.
 *   demand         integer milli-requests per second (mrps) at the graph's entry
 *   latency        integer microseconds
 *   multipliers    per-task demand multipliers in 1/1000ths (1000 = 1.0)
 *
 * All pointers in the signatures below are HOST pointers unless a comment says
 * "device".  Inputs are copied during the call and stay owned by the caller;
 * outputs are caller-allocated.  Every function returns JSV_OK (0) or a negative
 * error code; none throws or aborts.  "No feasible assignment" is not an error.
 * A context is not thread-safe; distinct contexts are independent.
 */
#ifndef JSV_H
#define JSV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define JSV_API __attribute__((visibility("default")))

#define JSV_MAX_TASKS   16      /* tasks per graph */
#define JSV_MAX_CHOICES 2048    /* V*P*B per task */

enum {
    JSV_OK          =  0,
    JSV_E_NULL      = -1,   /* a required pointer is NULL */
    JSV_E_BADARG    = -2,   /* value out of range (see each call) */
    JSV_E_CYCLE     = -3,   /* the task graph has a cycle */
    JSV_E_OVERFLOW  = -4,   /* latency, cost or search-space size does not fit */
    JSV_E_STATE     = -5,   /* call order: search before profile/graph, T mismatch */
    JSV_E_WORKSPACE = -6,   /* caller-supplied workspace too small */
    JSV_E_DEVICE    = -7,   /* a HIP call failed; see jsv_last_hip_error */
    JSV_E_INTERNAL  = -8    /* the enumeration's winner failed the rescoring of its latency or
                               accuracy test: an inconsistency inside the library, never expected */
};

typedef struct jsv_ctx jsv_ctx;

/*
 * Create a context bound to one GPU.  hip_stream is a hipStream_t borrowed from
 * the caller (NULL = the default stream); all device work of this context is
 * enqueued on it, in order.  No device call is made before the first search, so
 * profile and graph validation work on a machine without a GPU.
 */
JSV_API int  jsv_create(jsv_ctx** out, int device, void* hip_stream);
JSV_API void jsv_destroy(jsv_ctx* ctx);

/* HIP error code (hipError_t as int) of the last failed device call, 0 if none. */
JSV_API int  jsv_last_hip_error(const jsv_ctx* ctx);
JSV_API const char* jsv_error_string(int code);

/*
 * Device scratch memory.  By default the library allocates what a search needs
 * (grow-only, freed by jsv_destroy).  A caller that owns device memory can lend
 * a buffer instead: jsv_workspace_bytes gives the size a search of n_levels
 * demand levels (or a batch of n_levels problems) with the loaded profile needs;
 * jsv_set_workspace lends `bytes` bytes at DEVICE pointer `device_ptr`
 * (256-byte aligned) until the next set call or jsv_destroy; NULL returns to
 * library-owned memory.  A lent buffer that is too small makes the search
 * return JSV_E_WORKSPACE.  The size depends on the modes in force (factors,
 * mixtures): ask after setting them; 0 means the request cannot be served.  The size also
 * depends on the number of compute units of the GPU (per-block partial results): before the
 * context's first device call it is computed for 256 compute units, the MI355X figure, and for
 * the device's own count afterwards.
 */
JSV_API size_t jsv_workspace_bytes(const jsv_ctx* ctx, uint32_t n_levels, uint32_t prune_cap);
JSV_API int    jsv_set_workspace(jsv_ctx* ctx, void* device_ptr, size_t bytes);

/*
 * Profile tables (Table 2 of the paper, "profiled information"): the same V, P,
 * B for every task.
 *   units[P]               cost s_n of each partition size, in GPU slices (> 0)
 *   batch[B]               batch sizes (> 0)
 *   latency_us[T][V][P][B] profiled latency L(t,v,s,b), microseconds, > 0
 *   thr_mrps[T][V][P][B]   profiled throughput H(t,v,s,b), milli-requests/s, > 0;
 *                          NULL derives it as floor(batch * 1e9 / latency_us)
 *   accuracy[T][V]         A(t,v), fp64 in (0, 1]
 * Errors: JSV_E_NULL; JSV_E_BADARG (T = 0, T > JSV_MAX_TASKS, V*P*B = 0 or
 * > JSV_MAX_CHOICES, a zero unit/batch/latency/throughput, accuracy outside
 * (0,1]); JSV_E_OVERFLOW (derived throughput >= 2^32).
 */
JSV_API int jsv_load_profile(jsv_ctx* ctx, uint32_t T, uint32_t V, uint32_t P, uint32_t B,
                     const uint32_t* units, const uint32_t* batch,
                     const uint32_t* latency_us, const uint32_t* thr_mrps,
                     const double* accuracy);

/*
 * Task graph over the same T tasks (Table 2: P, P(t), f_p; Eq. 3, 5, 12).
 *   src[E], dst[E]         edges by task id, any order
 *   demand_mult_milli[T]   demand at task t relative to the entry demand, R(t)/R,
 *                          in 1/1000ths, > 0.  The fraction of requests on a path
 *                          (f_p of Eq. 12) is derived from these: a sink's share of
 *                          all sinks times, per edge, the tail's share of the
 *                          head's predecessors.
 *   capacity_units         S_avail of Eq. 8; 0 = unlimited
 *   queue_factor           the factor on latency for batch-formation queueing;
 *                          Eq. 3 uses 2
 * Errors: JSV_E_NULL; JSV_E_BADARG (T = 0 or > JSV_MAX_TASKS, endpoint >= T, self
 * loop, duplicate edge, zero multiplier, queue_factor = 0); JSV_E_CYCLE;
 * JSV_E_STATE (T differs from the loaded profile).
 */
JSV_API int jsv_set_dag(jsv_ctx* ctx, uint32_t T, uint32_t E, const uint16_t* src, const uint16_t* dst,
                const uint32_t* demand_mult_milli, uint32_t capacity_units, uint32_t queue_factor);

/*
 * What the search optimises (Eq. 14).  mode 0 (default): the cheapest feasible
 * assignment, lowest index on equal cost - the cost term of Eq. 14 alone.  mode 1:
 * the feasible assignment with the largest alpha * A_obj - beta * cost; equal
 * objectives go to the lower cost, then to the lowest index.  The paper's
 * evaluation uses alpha = 1, beta = 0.035 (Section 4.4), which are the defaults
 * used for the `objective` field of the results in mode 0.  Applies to all later
 * searches of the context.  Errors: JSV_E_NULL; JSV_E_BADARG (mode not 0 or 1,
 * alpha or beta negative or not finite).
 */
JSV_API int jsv_set_objective(jsv_ctx* ctx, int mode, double alpha, double beta);

/*
 * Graph mode (off by default): jsv_search and jsv_search_loaded_batch record their
 * copy - kernels - copy sequence into a HIP graph the first time a shape is seen (number
 * of levels, table sizes, workspace, objective) and replay it afterwards, which removes
 * most of the launch overhead of small searches.  New demands and SLOs need no new
 * recording.  In this mode jsv_summary.seconds_enumerate is 0 (the kernels are not timed
 * one by one) and the context's stream must not be under capture by the caller.
 * Needs a context created on a stream of its own: with the default stream (NULL) the call
 * returns JSV_E_STATE.
 */
JSV_API int jsv_set_graph_mode(jsv_ctx* ctx, int on);

/*
 * Search-space restrictions used for the paper's ablations (Section 4.3; Appendix B).
 * All three default to on; switching one off removes choices from every task's list
 * before any pruning, also when prune_cap is 0:
 *   accuracy_scaling = 0      only the most accurate variant of each task (lowest id
 *                             among equally accurate ones)
 *   spatial_partitioning = 0  only the partition with the most units (lowest index among
 *                             equals): every replica takes a whole GPU
 *   graph_informed = 0        static per-task budgets instead of end-to-end ones.  On
 *                             every path the latency SLO is split in the ratio of the
 *                             tasks' highest latencies (most accurate variant, any allowed
 *                             partition and batch); a task keeps its smallest share.
 *                             S_avail (if not 0) is split in the ratio of the expected
 *                             needs mult_t * units / throughput of the allowed tuple of the
 *                             most accurate variant with the highest throughput, floored to
 *                             whole units.  A choice survives only within both budgets.
 * Applies to all later searches of the context (single system or batch).
 */
JSV_API int jsv_set_search_space(jsv_ctx* ctx, int accuracy_scaling, int spatial_partitioning,
                                 int graph_informed);

/*
 * Bounds in the enumeration (on by default).  A group of candidates that share all digits but
 * those of the innermost tasks is excluded as a whole when the digits it shares already break
 * the latency SLO (Eq. 3), when its remaining latency budget is below the fastest choice of
 * the innermost task, or, with S_avail set, when its shared cost plus the cheapest choices of
 * the innermost tasks exceeds S_avail (Eq. 8) or the cost of a candidate already found that
 * meets both SLOs (objective mode: the cost beyond which alpha - beta * cost falls below an
 * objective already reached); the kernel skips the tests of such candidates where a whole
 * 64-lane wave of groups is excluded.  In the cost modes a large level starts from the cost of
 * a candidate that meets Eq. 3, 8 and 13, found by a descent over single-task swaps before
 * the enumeration (the optimum cannot cost more; candidates as cheap stay in).  The result is the same with bounds on or off (an
 * excluded candidate fails a constraint or is worse than one that was found); off makes the kernel issue the tests
 * of every candidate, which is what throughput measurements of the plain enumeration use.
 * jsv_summary.candidates_visited tells how many candidates had their tests issued.  A search
 * with fewer than 8 tiles of 256 lanes per block of the grid runs the plain enumeration even
 * with bounds on: everything is in flight at once there and no bound would arrive in time.
 */
JSV_API int jsv_set_bounds(jsv_ctx* ctx, int on);

/*
 * Launch geometry of the enumeration, for tuning and for tests that the result does not depend
 * on it (the arg-min is a minimum over a total order, so it must not).  blocks_per_cu: resident
 * 256-lane blocks per compute unit, 1..8, capped by what the kernel's registers and LDS allow;
 * 0 = as many as fit (up to 8).  lanes_percent: scales the number of lanes the planner tries to
 * keep busy per demand level, which decides how many leading tasks a lane loops over and how
 * the outermost of those loops is cut into tiles; 1..1600, 0 or 100 = the default.
 * Errors: JSV_E_NULL; JSV_E_BADARG (out of range).
 */
JSV_API int jsv_set_geometry(jsv_ctx* ctx, int blocks_per_cu, int lanes_percent);

/*
 * Mixtures of two tuples per task (Section 3.2: Eq. 2, 6, 7 with two active instance types and
 * the throughput-weighted task accuracy of Eq. 9, 10).  on != 0: besides replicating one tuple
 * a task may run m1 >= 1 replicas of tuple c1 and m2 >= 1 of tuple c2 (c1 < c2), where
 * m1*H1 + m2*H2 covers the task's demand and neither (m1-1, m2) nor (m1, m2-1) does.  Such an
 * option has the latency of its slower tuple, the cost m1*units1 + m2*units2 and the accuracy
 * (m1*H1*A1 + m2*H2*A2) / (m1*H1 + m2*H2), evaluated in fp64 as two products, one sum, one
 * quotient.  Options are ordered by id: c for a single tuple, C + (c1*C + c2)*65536 + m1 for a
 * mixture; an option that alone costs more than S_avail is left out.  jsv_search then prunes
 * the options of every task like single choices (latency filter, exact dominance on
 * (latency, accuracy, cost) with equal triples keeping the lowest id) and, if more than
 * prune_cap remain (flags bit0), thins them over a grid of latency and accuracy: the n
 * survivors in the order (latency, id) are cut into bands = floor(sqrt(prune_cap)) runs (rank
 * r goes to band floor(r*bands/n)), and a band of more than per = floor(prune_cap/bands)
 * options keeps those at ranks floor(j*(size-1)/(per-1)), j < per, of its order by
 * (accuracy, id).  The searched space is the product of the surviving
 * lists, index with task 0 as the fastest digit; full_index is UINT64_MAX; choice2 / replicas2
 * of the result name the second tuple.
 *
 * This narrows the paper's space: Eq. 6 holds with slack too, and Eq. 10 weights accuracy by the
 * provisioned throughput M*H, so a surplus replica of the more accurate tuple can be the
 * cheapest way to meet Eq. 13 (or score higher under Eq. 14).  Splits with surplus replicas and
 * mixtures of more than two tuples are not searched; the result is an upper bound on the cost
 * of the best mixture.
 *
 * In mixture mode jsv_search needs 2 <= prune_cap <= JSV_MAX_CHOICES, 1 <= capacity_units <=
 * 65535 and at most 65536 replicas of any allowed tuple on its own (else JSV_E_BADARG /
 * JSV_E_OVERFLOW); it returns JSV_E_STATE together with per-variant factors, graph_informed =
 * 0 or batch mode, and so do jsv_eval_candidates and jsv_get_pruned.  Objective mode works over
 * the options too (every option has its own accuracy, so every candidate gets its own
 * objective: the general, slower loop of the enumeration).
 */
JSV_API int jsv_set_mixtures(jsv_ctx* ctx, int on);

/*
 * Per-variant multiplicative factors F(t, v, t') (Section 3.2, Eq. 4 and 5) for the system
 * loaded with jsv_load_profile + jsv_set_dag.  factor_milli: host, [E][V] row-major in the
 * edge order given to jsv_set_dag, copied; entry [e][v] is the number of requests variant v
 * of the edge's tail sends along the edge per request it serves, in 1/1000ths, 1 ..
 * JSV_MAX_FACTOR_MILLI.  NULL returns to the fixed per-task multipliers.  A later
 * jsv_load_profile or jsv_set_dag drops the table.
 *
 * With factors set, the demand of a task without predecessors is demand * mult_t as before;
 * the demand of any other task is the sum over its incoming edges of the tail's demand times
 * the factor of the tail's chosen variant, floored per edge to whole micro-requests/s; its
 * mult_t only weighs paths in the accuracy (Eq. 12).  A demand of 2^44 micro-requests/s or more
 * makes the search return JSV_E_OVERFLOW.
 *
 * How a level is searched: every task with an outgoing edge whose factors differ between
 * variants is held to one variant, in all combinations; inside a combination all demands are
 * fixed and cost table, prune and search are the ordinary ones (prune_cap applies per
 * combination).  The level's result is the best over the combinations: cheapest, or in
 * objective mode largest objective then cheapest, then lowest full_index.  In the result,
 * index repeats full_index, evaluated and flags add up over the combinations.
 * levels * combinations may not exceed 65536 (jsv_search: JSV_E_BADARG).
 *
 * Returns JSV_E_STATE without a loaded profile and graph or in batch mode, JSV_E_BADARG for
 * a graph without edges or a factor out of range, JSV_E_OVERFLOW if C^T does not fit 64
 * bits.  While factors are set, jsv_eval_candidates and jsv_get_pruned return JSV_E_STATE,
 * and so does jsv_search with graph_informed = 0.
 */
#define JSV_MAX_FACTOR_MILLI 1000000u
JSV_API int jsv_set_factors(jsv_ctx* ctx, const uint32_t* factor_milli);

typedef struct {
    uint64_t index;        /* winner's index in the searched space; UINT64_MAX if infeasible */
    uint64_t full_index;   /* sum_t c_t * C^t; UINT64_MAX if infeasible or it does not fit */
    uint64_t evaluated;    /* candidates scored at this level = prod_t K_t */
    double   accuracy;     /* A_obj of Eq. 12: normalised to the best achievable */
    uint32_t latency_us;   /* queue_factor * critical path (left side of Eq. 3) */
    int32_t  cost_units;   /* sum of replicas * units (Eq. 7, 8); INT32_MAX if infeasible */
    uint32_t feasible;     /* 0 / 1 */
    uint32_t flags;        /* bit0: the prune cap dropped a non-dominated choice;
                              bit1 (informational): costs were too large for the 32-bit
                              fast path, 64-bit keys were compared instead */
    uint16_t choice[JSV_MAX_TASKS];     /* winner's choice id per task */
    uint32_t replicas[JSV_MAX_TASKS];   /* M of Eq. 6 per task */
    double   objective;    /* alpha * A_obj - beta * cost_units of the winner (Eq. 14) */
    uint16_t choice2[JSV_MAX_TASKS];    /* mixture mode: the task's second tuple; 0xFFFF if the
                                           task runs one tuple (always, outside mixture mode) */
    uint32_t replicas2[JSV_MAX_TASKS];  /* mixture mode: replicas of the second tuple; else 0 */
} jsv_result;

typedef struct {
    int32_t  best_level;       /* position of the feasible level with the largest demand
                                  (first one on equal demands); -1 if none */
    uint32_t max_demand_mrps;  /* its demand: the maximum serviceable demand; 0 if none */
    double   seconds_device;   /* device time of the whole search, HIP events */
    double   seconds_enumerate;/* of which the enumeration kernel */
    uint64_t candidates_visited;   /* candidates whose tests the enumeration kernel issued.  Bounds
                                      on: counted in whole 64-lane waves and whole quads of the
                                      innermost task's stream (padding included), the rest of the
                                      space was excluded in bulk.  Bounds off: the sum of `evaluated`;
                                      in mixture mode, whose stream of options is sorted by latency
                                      and left once no lane can take a later one, counted as with
                                      bounds on */
} jsv_summary;

/*
 * The search (Eq. 2, 3, 5-8, 11-13).  For every demand level: replicas and cost
 * of every (task, choice); optional per-task prune; every candidate of the
 * searched space scored for latency, accuracy and cost and masked against
 * SLO_l, SLO_a and S_avail; the cheapest feasible candidate, lowest index on
 * equal cost.  All levels run in one pass on the context's stream; the call
 * returns after the results are in out[].
 *   demand_mrps[n_levels]  any order, each > 0
 *   slo_accuracy           threshold on A_obj, a fraction of the best achievable.  Eq. 13 is
 *                          tested in fp64 as A_raw >= slo_accuracy * A_max with one fixed
 *                          order of operations for A_raw and A_max, so 1.0 accepts exactly
 *                          the assignments as accurate as the best one.  An assignment
 *                          whose exact A_obj lies within a few ulp of the threshold may
 *                          fall on either side of it
 *   prune_cap              0: exhaustive.  Otherwise >= 2V: each task keeps only
 *                          choices that can meet SLO_l at all and that no other
 *                          choice matches or beats on (latency, accuracy, cost);
 *                          if more than prune_cap remain, each variant is thinned
 *                          to floor(prune_cap/V) of them evenly spaced by latency
 *                          rank (fastest and cheapest always kept; sets flags bit0)
 *   out[n_levels], summary caller-allocated; summary may be NULL
 * Errors: JSV_E_NULL; JSV_E_STATE (no profile or graph, batch loaded; per-variant
 * factors or mixtures together with graph_informed = 0, mixtures together with
 * factors); JSV_E_BADARG (n_levels = 0, a zero demand, NaN threshold, prune_cap in
 * (0, 2V); with factors: levels * combinations > 65536; with mixtures: prune_cap
 * outside [2, JSV_MAX_CHOICES], capacity_units outside [1, 65535]); JSV_E_OVERFLOW
 * (queue_factor * sum of the tasks' largest latencies >= 2^32; a cost >= 2^31;
 * searched space and cost do not fit a 64-bit key together; with factors a demand
 * >= 2^44 micro-requests/s or a winner whose full_index does not fit; with mixtures
 * more than 65535 replicas of one tuple); JSV_E_WORKSPACE (lent buffer too small;
 * with mixtures also a cell grid beyond 2^32 cells); JSV_E_DEVICE; JSV_E_INTERNAL.
 */
JSV_API int jsv_search(jsv_ctx* ctx, const uint32_t* demand_mrps, uint32_t n_levels,
               uint32_t slo_latency_us, double slo_accuracy, uint32_t prune_cap,
               jsv_result* out, jsv_summary* summary);

/*
 * jsv_search for callers that cannot allocate: code that runs where hipMalloc is not allowed
 * (a tight serving loop, a harness that forbids it, a region around which the caller is
 * capturing other work).  Same arguments, same results, record by record, as jsv_search for the
 * loaded single system; but the call allocates nothing - no device memory, no pinned memory,
 * no events: problem tables, workspace and results live in one static device array of
 * JSV_STATIC_SCRATCH_BYTES that the library's code object brings along (one copy per GPU,
 * held until the process ends), instance records are copied straight from and results
 * straight to the caller's host memory, and jsv_summary.seconds_device / seconds_enumerate
 * are 0.  A lent workspace (jsv_set_workspace) is not used.
 *
 * Every context on a GPU shares that GPU's array, which keeps the last call's contents; each
 * call writes everything it reads.  Calls that overlap in time on one GPU - from two threads,
 * or two contexts on different streams - race on it: serialise them.
 *
 * Errors as jsv_search, plus: JSV_E_WORKSPACE if tables and workspace of this search exceed
 * JSV_STATIC_SCRATCH_BYTES (xr8-sized: 8 tasks x 240 choices, 64 levels, prune cap 20 takes
 * 4.2 MB; nothing is launched); JSV_E_STATE with per-variant factors, mixtures, a loaded batch or
 * graph mode, which this entry point does not serve.
 */
#define JSV_STATIC_SCRATCH_BYTES (16u << 20)
JSV_API int jsv_search_static(jsv_ctx* ctx, const uint32_t* demand_mrps, uint32_t n_levels,
                      uint32_t slo_latency_us, double slo_accuracy, uint32_t prune_cap,
                      jsv_result* out, jsv_summary* summary);

/*
 * Parity aid: score n explicit candidates of one level's searched space.
 * index[n] are candidate indices (< prod K_t).  Outputs, each [n] (replicas
 * [n][T]): latency_us, cost, accuracy as in jsv_result; mask bit0 latency SLO
 * met, bit1 accuracy SLO met, bit2 capacity met.  Errors as jsv_search, plus
 * JSV_E_BADARG for an index outside the space.
 */
JSV_API int jsv_eval_candidates(jsv_ctx* ctx, uint32_t demand_mrps, uint32_t slo_latency_us,
                        double slo_accuracy, uint32_t prune_cap,
                        const uint64_t* index, uint32_t n,
                        uint32_t* latency_us, uint32_t* replicas, int32_t* cost,
                        double* accuracy, uint8_t* mask);

/*
 * Parity aid: the surviving choice ids of one task at one level, ascending.
 * choice_ids must hold V*P*B entries; *K receives the count, *truncated whether
 * the cap dropped a non-dominated choice of this task.
 */
JSV_API int jsv_get_pruned(jsv_ctx* ctx, uint32_t demand_mrps, uint32_t slo_latency_us,
                   uint32_t prune_cap, uint32_t task,
                   uint16_t* choice_ids, uint32_t* K, uint32_t* truncated);

/*
 * Many independent systems in one pass: each problem has its own tables, graph,
 * demand, SLOs and prune cap (fields as the arguments of jsv_load_profile,
 * jsv_set_dag and jsv_search).
 */
typedef struct {
    uint32_t T, V, P, B;
    const uint32_t* units;
    const uint32_t* batch;
    const uint32_t* latency_us;
    const uint32_t* thr_mrps;        /* may be NULL */
    const double*   accuracy;
    uint32_t E;
    const uint16_t* src;
    const uint16_t* dst;
    const uint32_t* demand_mult_milli;
    uint32_t capacity_units;
    uint32_t queue_factor;
    uint32_t demand_mrps;
    uint32_t slo_latency_us;
    double   slo_accuracy;
    uint32_t prune_cap;
} jsv_problem;

/*
 * jsv_load_batch validates and stages n problems on the device (replacing any
 * profile/graph or batch loaded before); jsv_search_loaded_batch searches all of
 * them in one pass, out[n].  jsv_search_batch does both.  A problem that fails
 * validation makes the call return its error; *bad (may be NULL) receives its
 * position.
 */
JSV_API int jsv_load_batch(jsv_ctx* ctx, const jsv_problem* problems, uint32_t n, uint32_t* bad);
JSV_API int jsv_search_loaded_batch(jsv_ctx* ctx, jsv_result* out, jsv_summary* summary);
JSV_API int jsv_search_batch(jsv_ctx* ctx, const jsv_problem* problems, uint32_t n, jsv_result* out);

#ifdef __cplusplus
}
#endif
#endif /* JSV_H */
