/*
 * CPU oracle for the one-tuple-per-task allocation search.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  Nothing in the product path may call it,
 * link it or fall back to it; it shares no code, header, table or constant
 * with the HIP sources.
 *
 * What it computes, following the paper's MILP (Section 3.2) restricted to one
 * (variant, partition, batch) tuple per task, replicated as often as needed:
 *
 *   - demand at a task:   R(t) = R * m_t                       (Eq. 5, fixed factors)
 *                         or, with per-variant factors F(t', v, t) given, R(t) = R * m_t at a
 *                         source and sum over predecessors t' of R(t') * F(t', v_t', t)
 *                         elsewhere, v_t' the variant chosen for t'  (Eq. 4, 5)
 *   - replicas:           smallest M >= 1 with M*H >= R(t)     (Eq. 6)
 *   - task cost:          M * s_n of the chosen partition      (Eq. 7)
 *   - total cost:         sum over tasks, <= S_avail           (Eq. 8)
 *   - latency:            q * max over source-to-sink paths of the summed
 *                         per-task latencies, <= SLO_l         (Eq. 2, 3; q = 2)
 *   - path accuracy:      product of the task accuracies       (Eq. 11)
 *   - system accuracy:    sum_p f_p*A_p / A_max, >= SLO_a      (Eq. 12, 13)
 *   - result:             among candidates meeting all three constraints the
 *                         cheapest one; equal costs -> lowest candidate index.
 *                         Optionally instead the paper's objective (Eq. 14): the
 *                         largest alpha*A_obj - beta*cost; equal objectives ->
 *                         lower cost -> lowest candidate index.
 *
 *   - optionally, mixtures (Eq. 2, 6, 7, 9, 10 with up to two active tuples per task): besides
 *                         one tuple replicated M times a task may run M1 >= 1 replicas of one
 *                         tuple and M2 >= 1 of another, just enough of both to carry R(t);
 *                         its latency is the slower tuple's, its cost the sum, its accuracy
 *                         the throughput-weighted mean of the two variants' accuracies.
 *
 * Paths are enumerated explicitly by depth-first search and every candidate is
 * scored from the tables on its own: no dynamic programming over the graph, no
 * sharing between candidates, no blocking.  Integers are exact (64-bit);
 * accuracy is fp64, multiplied along a path from source to sink and summed
 * over paths in depth-first order.
 *
 * Pins (tests/test_oracle_*.py): a hand-worked two-task chain, an independent
 * brute force on tiny inputs, closed forms (one task; separable minimum;
 * multiple-choice knapsack on chains), monotonicity invariants.  The cap-
 * thinning step of the prune is a heuristic of this library with no outside
 * definition: it is checked against hand-worked lists, a second, differently
 * written implementation and its stated properties only ("parity unpinned"
 * beyond that).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_MAX_TASKS 16
#define ORC_MAX_PATHS (1 << 20)

enum { ORC_OK = 0, ORC_E_ARG = -1, ORC_E_CYCLE = -2, ORC_E_RANGE = -3, ORC_E_MEM = -4 };

typedef struct {
    uint64_t index;       /* in the searched space, task 0 = fastest digit */
    uint64_t full_index;  /* sum_t c_t * C^t, UINT64_MAX if that overflows */
    uint64_t evaluated;   /* size of the searched space */
    double accuracy;      /* A_obj of the winner */
    uint32_t latency_us;  /* q * critical path of the winner */
    int32_t cost;         /* INT32_MAX when infeasible */
    uint32_t feasible;
    uint32_t flags;       /* bit0: cap thinning dropped a choice at this level */
    uint16_t choice[ORC_MAX_TASKS];
    uint32_t replicas[ORC_MAX_TASKS];
    double objective;     /* alpha*A_obj - beta*cost of the winner (Eq. 14) */
    uint16_t choice2[ORC_MAX_TASKS];   /* mixtures: the second tuple, 0xFFFF if the task runs one */
    uint32_t replicas2[ORC_MAX_TASKS]; /* mixtures: replicas of the second tuple, 0 if none */
} orc_result;

typedef struct {
    uint32_t T, V, P, B, C, E;
    uint32_t *units, *batch, *lat, *thr, *mult;
    double *acc;
    uint16_t *src, *dst;
    uint32_t *fac;  /* [E][V] per-variant factor of an edge's tail, 1/1000ths; NULL = fixed factors */
    uint32_t capacity, q;
    /* what the search optimises: 0 = cheapest feasible, 1 = Eq. 14 */
    int objective;
    double alpha, beta;
    /* search-space restrictions of the paper's ablations (1 = feature on) */
    int space_a, space_s, space_t;
    int mix;        /* 1: a task may mix two tuples */
    /* graph */
    int npred[ORC_MAX_TASKS], pred[ORC_MAX_TASKS][ORC_MAX_TASKS];
    int nsucc[ORC_MAX_TASKS], succ[ORC_MAX_TASKS][ORC_MAX_TASKS];
    /* explicit paths */
    int npaths;
    int *plen;      /* [npaths] */
    int *pnode;     /* [npaths][T] */
    double *pf;     /* [npaths] fraction of requests on the path */
    double amax;
} orc_model;

/* ---- choice id <-> (variant, partition, batch) ---------------------------- */
static inline uint32_t variant_of(const orc_model *m, uint32_t c) { return c / (m->P * m->B); }
static inline uint32_t part_of(const orc_model *m, uint32_t c) { return (c / m->B) % m->P; }

/* ---- path enumeration ------------------------------------------------------ */
typedef struct { orc_model *m; int stack[ORC_MAX_TASKS]; int depth; int err; int cap; } dfs_t;

static void dfs(dfs_t *d, int node)
{
    orc_model *m = d->m;
    if (d->err) return;
    d->stack[d->depth++] = node;
    if (m->nsucc[node] == 0) {
        if (m->npaths == d->cap) { d->err = ORC_E_RANGE; d->depth--; return; }
        int k = m->npaths++;
        m->plen[k] = d->depth;
        for (int i = 0; i < d->depth; i++) m->pnode[(size_t)k * m->T + i] = d->stack[i];
    } else {
        for (int i = 0; i < m->nsucc[node]; i++) dfs(d, m->succ[node][i]);
    }
    d->depth--;
}

/* 0 if acyclic: repeatedly strip nodes without remaining predecessors */
static int has_cycle(const orc_model *m)
{
    int indeg[ORC_MAX_TASKS], gone[ORC_MAX_TASKS] = {0}, left = (int)m->T;
    for (uint32_t t = 0; t < m->T; t++) indeg[t] = m->npred[t];
    for (;;) {
        int found = -1;
        for (uint32_t t = 0; t < m->T; t++) if (!gone[t] && indeg[t] == 0) { found = (int)t; break; }
        if (found < 0) break;
        gone[found] = 1; left--;
        for (int i = 0; i < m->nsucc[found]; i++) indeg[m->succ[found][i]]--;
    }
    return left != 0;
}

/* system accuracy for given per-task accuracies, before normalisation (Eq. 11, 12) */
static double raw_accuracy_of(const orc_model *m, const double *task_acc)
{
    double total = 0.0;
    for (int k = 0; k < m->npaths; k++) {
        double ap = 1.0;
        for (int i = 0; i < m->plen[k]; i++) ap *= task_acc[m->pnode[(size_t)k * m->T + i]];
        total += m->pf[k] * ap;
    }
    return total;
}

/* the same for one choice of variants */
static double raw_accuracy(const orc_model *m, const uint32_t *variant)
{
    double a[ORC_MAX_TASKS];
    for (uint32_t t = 0; t < m->T; t++) a[t] = m->acc[(size_t)t * m->V + variant[t]];
    return raw_accuracy_of(m, a);
}

void orc_destroy(orc_model *m)
{
    if (!m) return;
    free(m->units); free(m->batch); free(m->lat); free(m->thr); free(m->mult);
    free(m->acc); free(m->src); free(m->dst); free(m->fac); free(m->plen); free(m->pnode); free(m->pf);
    free(m);
}

static void *dup_mem(const void *p, size_t n)
{
    void *q = malloc(n ? n : 1);
    if (q && n) memcpy(q, p, n);
    return q;
}

/*
 * Build a model.  thr_mrps may be NULL: throughput is then batch/latency,
 * floored to whole milli-requests per second.
 */
int orc_create(orc_model **out, uint32_t T, uint32_t V, uint32_t P, uint32_t B,
               const uint32_t *units, const uint32_t *batch, const uint32_t *latency_us,
               const uint32_t *thr_mrps, const double *accuracy,
               uint32_t E, const uint16_t *src, const uint16_t *dst,
               const uint32_t *mult_milli, uint32_t capacity_units, uint32_t queue_factor)
{
    if (!out || !units || !batch || !latency_us || !accuracy || !mult_milli) return ORC_E_ARG;
    if (E && (!src || !dst)) return ORC_E_ARG;
    if (T == 0 || T > ORC_MAX_TASKS || V == 0 || P == 0 || B == 0 || queue_factor == 0) return ORC_E_ARG;
    if ((uint64_t)V * P * B > 65535u) return ORC_E_ARG;
    orc_model *m = (orc_model *)calloc(1, sizeof *m);
    if (!m) return ORC_E_MEM;
    m->T = T; m->V = V; m->P = P; m->B = B; m->C = V * P * B; m->E = E;
    m->capacity = capacity_units; m->q = queue_factor;
    m->objective = 0; m->alpha = 1.0; m->beta = 0.035;     /* the paper's evaluation parameters */
    m->space_a = m->space_s = m->space_t = 1;
    size_t n = (size_t)T * m->C;
    m->units = dup_mem(units, P * sizeof *units);
    m->batch = dup_mem(batch, B * sizeof *batch);
    m->lat = dup_mem(latency_us, n * sizeof *latency_us);
    m->mult = dup_mem(mult_milli, T * sizeof *mult_milli);
    m->acc = dup_mem(accuracy, (size_t)T * V * sizeof *accuracy);
    m->src = dup_mem(src, E * sizeof *src);
    m->dst = dup_mem(dst, E * sizeof *dst);
    m->thr = (uint32_t *)malloc(n * sizeof(uint32_t));
    if (!m->units || !m->batch || !m->lat || !m->mult || !m->acc || !m->src || !m->dst || !m->thr) {
        orc_destroy(m); return ORC_E_MEM;
    }
    for (size_t i = 0; i < n; i++) {
        if (m->lat[i] == 0) { orc_destroy(m); return ORC_E_ARG; }
        if (thr_mrps) m->thr[i] = thr_mrps[i];
        else {
            uint64_t h = (uint64_t)m->batch[i % B] * 1000000000ull / m->lat[i];
            if (h > 0xFFFFFFFFull) { orc_destroy(m); return ORC_E_RANGE; }
            m->thr[i] = (uint32_t)h;
        }
        if (m->thr[i] == 0) { orc_destroy(m); return ORC_E_ARG; }
    }
    for (size_t i = 0; i < (size_t)T * V; i++)
        if (!(m->acc[i] > 0.0 && m->acc[i] <= 1.0)) { orc_destroy(m); return ORC_E_ARG; }
    for (uint32_t t = 0; t < T; t++) if (m->mult[t] == 0) { orc_destroy(m); return ORC_E_ARG; }
    for (uint32_t e = 0; e < E; e++) {
        uint32_t a = src[e], b = dst[e];
        if (a >= T || b >= T || a == b) { orc_destroy(m); return ORC_E_ARG; }
        for (int i = 0; i < m->nsucc[a]; i++)
            if (m->succ[a][i] == (int)b) { orc_destroy(m); return ORC_E_ARG; }
        m->succ[a][m->nsucc[a]++] = (int)b;
        m->pred[b][m->npred[b]++] = (int)a;
    }
    if (has_cycle(m)) { orc_destroy(m); return ORC_E_CYCLE; }

    /* all source-to-sink paths; an isolated task is a path of length one */
    m->plen = (int *)malloc(sizeof(int) * ORC_MAX_PATHS);
    m->pnode = (int *)malloc(sizeof(int) * (size_t)ORC_MAX_PATHS * T);
    if (!m->plen || !m->pnode) { orc_destroy(m); return ORC_E_MEM; }
    dfs_t d; memset(&d, 0, sizeof d); d.m = m; d.cap = ORC_MAX_PATHS;
    for (uint32_t t = 0; t < T; t++) if (m->npred[t] == 0) dfs(&d, (int)t);
    if (d.err) { orc_destroy(m); return d.err; }
    m->plen = (int *)realloc(m->plen, sizeof(int) * (size_t)m->npaths);
    m->pnode = (int *)realloc(m->pnode, sizeof(int) * (size_t)m->npaths * T);
    m->pf = (double *)malloc(sizeof(double) * (size_t)m->npaths);
    if (!m->plen || !m->pnode || !m->pf) { orc_destroy(m); return ORC_E_MEM; }

    /*
     * Fraction of requests on a path (the f_p of Eq. 12), derived from the
     * per-task multipliers: the share of a sink among all sinks, times, for
     * every edge of the path, the share of the edge's tail among all
     * predecessors of its head.
     */
    uint64_t sink_total = 0;
    for (uint32_t t = 0; t < T; t++) if (m->nsucc[t] == 0) sink_total += m->mult[t];
    for (int k = 0; k < m->npaths; k++) {
        const int *nodes = m->pnode + (size_t)k * T;
        int last = nodes[m->plen[k] - 1];
        double f = (double)m->mult[last] / (double)sink_total;
        for (int i = 1; i < m->plen[k]; i++) {
            int head = nodes[i], tail = nodes[i - 1];
            uint64_t in_total = 0;
            for (int j = 0; j < m->npred[head]; j++) in_total += m->mult[m->pred[head][j]];
            f *= (double)m->mult[tail] / (double)in_total;
        }
        m->pf[k] = f;
    }
    /* A_max: every task on its most accurate variant */
    uint32_t best[ORC_MAX_TASKS];
    for (uint32_t t = 0; t < T; t++) {
        uint32_t bv = 0;
        for (uint32_t v = 1; v < V; v++)
            if (m->acc[(size_t)t * V + v] > m->acc[(size_t)t * V + bv]) bv = v;
        best[t] = bv;
    }
    m->amax = raw_accuracy(m, best);
    *out = m;
    return ORC_OK;
}

/* mode 0: cheapest feasible assignment.  mode 1: maximise alpha*A_obj - beta*cost (Eq. 14;
   the paper's evaluation uses alpha = 1, beta = 0.035). */
int orc_set_objective(orc_model *m, int mode, double alpha, double beta)
{
    if (!m || (mode != 0 && mode != 1) || !(alpha >= 0.0) || !(beta >= 0.0)) return ORC_E_ARG;
    m->objective = mode; m->alpha = alpha; m->beta = beta;
    return ORC_OK;
}

int orc_num_paths(const orc_model *m) { return m->npaths; }
double orc_amax(const orc_model *m) { return m->amax; }

/* path k: writes its nodes, returns its length; *f = request fraction */
int orc_get_path(const orc_model *m, int k, int *nodes, double *f)
{
    if (k < 0 || k >= m->npaths) return ORC_E_ARG;
    for (int i = 0; i < m->plen[k]; i++) nodes[i] = m->pnode[(size_t)k * m->T + i];
    *f = m->pf[k];
    return m->plen[k];
}

/* ---- replicas and cost of every (task, choice) at one demand (Eq. 5-7) ---- */
/* replicas (Eq. 6) and cost (Eq. 7) of choice c of task t under a demand of `need` micro-requests/s */
static int replicas_and_cost(const orc_model *m, uint64_t need, uint32_t t, uint32_t c, uint32_t *rep, int32_t *cost)
{
    uint64_t per = 1000ull * m->thr[(size_t)t * m->C + c];   /* one replica, same unit */
    uint64_t r = need / per + (need % per != 0);
    if (r < 1) r = 1;
    uint64_t k = r * m->units[part_of(m, c)];
    if (r > 0xFFFFFFFFull || k > 0x7FFFFFFFull) return ORC_E_RANGE;
    *rep = (uint32_t)r; *cost = (int32_t)k;
    return ORC_OK;
}

static int cost_table_of(const orc_model *m, const uint64_t *need, uint32_t *rep, int32_t *cost)
{
    for (uint32_t t = 0; t < m->T; t++)
        for (uint32_t c = 0; c < m->C; c++) {
            int rc = replicas_and_cost(m, need[t], t, c, &rep[(size_t)t * m->C + c], &cost[(size_t)t * m->C + c]);
            if (rc) return rc;
        }
    return ORC_OK;
}

int orc_cost_table(const orc_model *m, uint32_t demand_mrps, uint32_t *rep, int32_t *cost)
{
    uint64_t need[ORC_MAX_TASKS];
    for (uint32_t t = 0; t < m->T; t++) need[t] = (uint64_t)demand_mrps * m->mult[t];   /* micro-requests/s */
    return cost_table_of(m, need, rep, cost);
}

/* ---- per-variant multiplicative factors (Eq. 4, 5) --------------------------- */
#define ORC_FACTOR_MAX 1000000u             /* a factor of 1000 */
#define ORC_NEED_MAX ((uint64_t)1 << 44)    /* micro-requests/s */

/* fac[e * V + v]: requests sent along edge e per request served by variant v of the edge's
   tail, in 1/1000ths; NULL returns to the fixed per-task multipliers */
int orc_set_factors(orc_model *m, const uint32_t *fac)
{
    if (!m) return ORC_E_ARG;
    free(m->fac); m->fac = NULL;
    if (!fac) return ORC_OK;
    if (m->E == 0) return ORC_E_ARG;
    for (size_t i = 0; i < (size_t)m->E * m->V; i++) if (fac[i] == 0 || fac[i] > ORC_FACTOR_MAX) return ORC_E_ARG;
    m->fac = dup_mem(fac, (size_t)m->E * m->V * sizeof *fac);
    return m->fac ? ORC_OK : ORC_E_MEM;
}

/*
 * Demand at every task for one choice of variants (Eq. 5).  A source sees R * m_t; any
 * other task the sum over its incoming edges of the tail's demand times the factor of the
 * tail's variant, each product rounded down to whole micro-requests/s.
 */
static int demand_flow(const orc_model *m, uint32_t demand_mrps, const uint32_t *variant, uint64_t *need)
{
    int done[ORC_MAX_TASKS] = {0};
    for (uint32_t round = 0; round < m->T; round++)
        for (uint32_t t = 0; t < m->T; t++) {
            if (done[t]) continue;
            int ready = 1;
            for (int i = 0; i < m->npred[t]; i++) if (!done[m->pred[t][i]]) ready = 0;
            if (!ready) continue;
            uint64_t r = 0;
            if (m->npred[t] == 0) r = (uint64_t)demand_mrps * m->mult[t];
            else
                for (uint32_t e = 0; e < m->E; e++)
                    if (m->dst[e] == t) r += need[m->src[e]] * m->fac[(size_t)e * m->V + variant[m->src[e]]] / 1000u;
            if (r >= ORC_NEED_MAX) return ORC_E_RANGE;
            need[t] = r; done[t] = 1;
        }
    return ORC_OK;
}

/* tasks whose variant changes some downstream demand: an outgoing edge with unequal factors */
static uint32_t influencers(const orc_model *m, uint32_t *list)
{
    uint32_t n = 0;
    for (uint32_t t = 0; t < m->T; t++) {
        int varies = 0;
        for (uint32_t e = 0; e < m->E; e++)
            if (m->src[e] == t)
                for (uint32_t v = 1; v < m->V; v++)
                    if (m->fac[(size_t)e * m->V + v] != m->fac[(size_t)e * m->V]) varies = 1;
        if (varies) list[n++] = t;
    }
    return n;
}

/* ---- per-task prune --------------------------------------------------------- */
typedef struct { uint32_t lat; uint32_t c; } lat_c;
static int cmp_lat_c(const void *a, const void *b)
{
    const lat_c *x = (const lat_c *)a, *y = (const lat_c *)b;
    if (x->lat != y->lat) return x->lat < y->lat ? -1 : 1;
    return x->c < y->c ? -1 : (x->c > y->c);
}

/*
 * Search-space restrictions (Section 4.3 and Appendix B of the paper).
 *   accuracy scaling off:      only the most accurate variant of every task
 *   spatial partitioning off:  only the partition with the most units (a whole GPU)
 *   task-graph-informed off:   static per-task budgets.  Latency: on every path the SLO is
 *       split in the ratio of the tasks' highest latencies (most accurate variant, any
 *       allowed partition and batch); a task on several paths gets the smallest share.
 *       Resources: S_avail is split in the ratio of the expected needs m_t * s / H, with
 *       (s, H) the allowed tuple of the most accurate variant with the highest throughput;
 *       the share is floored to whole units.
 */
int orc_set_search_space(orc_model *m, int accuracy_scaling, int spatial_partitioning, int graph_informed)
{
    if (!m) return ORC_E_ARG;
    m->space_a = accuracy_scaling != 0; m->space_s = spatial_partitioning != 0; m->space_t = graph_informed != 0;
    return ORC_OK;
}

static uint32_t best_variant(const orc_model *m, uint32_t t)
{
    uint32_t bv = 0;
    for (uint32_t v = 1; v < m->V; v++)
        if (m->acc[(size_t)t * m->V + v] > m->acc[(size_t)t * m->V + bv]) bv = v;
    return bv;
}

static uint32_t whole_partition(const orc_model *m)
{
    uint32_t bp = 0;
    for (uint32_t p = 1; p < m->P; p++) if (m->units[p] > m->units[bp]) bp = p;
    return bp;
}

/* highest latency and (units, throughput) of the highest-throughput tuple of task u's most
   accurate variant over the allowed partitions and all batches */
static void reference_tuple(const orc_model *m, uint32_t u, uint32_t *lat_max, uint32_t *units, uint32_t *thr)
{
    const uint32_t v = best_variant(m, u), wp = whole_partition(m);
    *lat_max = 0; *thr = 0; *units = 0;
    for (uint32_t p = 0; p < m->P; p++) {
        if (!m->space_s && p != wp) continue;
        for (uint32_t b = 0; b < m->B; b++) {
            const size_t k = (size_t)u * m->C + ((size_t)v * m->P + p) * m->B + b;
            if (m->lat[k] > *lat_max) *lat_max = m->lat[k];
            if (m->thr[k] > *thr) { *thr = m->thr[k]; *units = m->units[p]; }
        }
    }
}

/* may task t use choice c at all under the restrictions?  only[t], if given and not
   UINT32_MAX, is the one variant task t is held to (per-variant factors, below) */
static int allowed(const orc_model *m, const int32_t *cost, uint32_t slo_latency_us, uint32_t t, uint32_t c,
                   const uint32_t *only)
{
    if (only && only[t] != UINT32_MAX && variant_of(m, c) != only[t]) return 0;
    if (!m->space_a && variant_of(m, c) != best_variant(m, t)) return 0;
    if (!m->space_s && part_of(m, c) != whole_partition(m)) return 0;
    if (!m->space_t) {
        uint32_t lmax[ORC_MAX_TASKS], un[ORC_MAX_TASKS], th[ORC_MAX_TASKS];
        for (uint32_t u = 0; u < m->T; u++) reference_tuple(m, u, &lmax[u], &un[u], &th[u]);
        /* latency share on every path through t: q*L <= SLO * lmax_t / sum_path lmax */
        for (int k = 0; k < m->npaths; k++) {
            int on = 0; uint64_t sum = 0;
            for (int i = 0; i < m->plen[k]; i++) {
                uint32_t u = (uint32_t)m->pnode[(size_t)k * m->T + i];
                if (u == t) on = 1;
                sum += lmax[u];
            }
            if (!on) continue;
            unsigned __int128 lhs = (unsigned __int128)m->q * m->lat[(size_t)t * m->C + c] * sum;
            unsigned __int128 rhs = (unsigned __int128)slo_latency_us * lmax[t];
            if (lhs > rhs) return 0;
        }
        if (m->capacity != 0) {
            double total = 0.0, mine = 0.0;
            for (uint32_t u = 0; u < m->T; u++) {
                double e = ((double)m->mult[u] * (double)un[u]) / (double)th[u];
                total += e;
                if (u == t) mine = e;
            }
            double share = (double)m->capacity * (mine / total);
            if ((double)cost[(size_t)t * m->C + c] > __builtin_floor(share)) return 0;
        }
    }
    return 1;
}

/* distance of the nearest resource share to a whole number (tests keep away from 0) */
double orc_budget_margin(const orc_model *m)
{
    if (m->space_t || m->capacity == 0) return 0.5;
    uint32_t lmax, un[ORC_MAX_TASKS], th[ORC_MAX_TASKS];
    double e[ORC_MAX_TASKS], total = 0.0, best = 0.5;
    for (uint32_t u = 0; u < m->T; u++) {
        reference_tuple(m, u, &lmax, &un[u], &th[u]);
        e[u] = ((double)m->mult[u] * (double)un[u]) / (double)th[u];
        total += e[u];
    }
    for (uint32_t u = 0; u < m->T; u++) {
        double share = (double)m->capacity * (e[u] / total);
        double d = share - __builtin_floor(share);
        if (d > 0.5) d = 1.0 - d;
        if (d < best) best = d;
    }
    return best;
}

/*
 * Surviving choices of one task, ascending choice id.  Choices the restrictions above
 * exclude never survive.
 * cap == 0: everything else.  Otherwise: (a) drop what cannot meet the latency SLO
 * even when every other task runs its fastest choice; (b) drop what another
 * choice matches or beats on latency, accuracy and cost; (c) if more than cap
 * remain, thin each variant to floor(cap/V) choices evenly spaced by latency
 * rank, fastest and slowest always kept.
 */
static int prune_task(const orc_model *m, const int32_t *cost, uint32_t slo_latency_us, uint32_t cap,
                      const uint32_t *only, uint32_t t, uint16_t *ids, uint32_t *K, uint32_t *truncated)
{
    const uint32_t C = m->C;
    *truncated = 0;
    if (cap == 0) {
        uint32_t n = 0;
        for (uint32_t c = 0; c < C; c++) if (allowed(m, cost, slo_latency_us, t, c, only)) ids[n++] = (uint16_t)c;
        *K = n;
        return ORC_OK;
    }
    if (cap < 2 * m->V) return ORC_E_ARG;
    uint8_t *alive = (uint8_t *)calloc(C, 1);
    uint8_t *keep = (uint8_t *)calloc(C, 1);
    lat_c *order = (lat_c *)malloc(sizeof(lat_c) * C);
    if (!alive || !keep || !order) { free(alive); free(keep); free(order); return ORC_E_MEM; }

    /* (a) longest path through t with every other task at its fastest choice */
    uint64_t lo[ORC_MAX_TASKS];
    for (uint32_t u = 0; u < m->T; u++) {
        uint32_t best = m->lat[(size_t)u * C];
        for (uint32_t c = 1; c < C; c++) if (m->lat[(size_t)u * C + c] < best) best = m->lat[(size_t)u * C + c];
        lo[u] = best;
    }
    uint64_t through = 0;
    for (int k = 0; k < m->npaths; k++) {
        int on = 0; uint64_t s = 0;
        for (int i = 0; i < m->plen[k]; i++) {
            uint32_t u = (uint32_t)m->pnode[(size_t)k * m->T + i];
            if (u == t) on = 1; else s += lo[u];
        }
        if (on && s > through) through = s;
    }
    for (uint32_t c = 0; c < C; c++)
        alive[c] = allowed(m, cost, slo_latency_us, t, c, only) &&
                   (uint64_t)m->q * ((uint64_t)m->lat[(size_t)t * C + c] + through) <= slo_latency_us;

    /* (b) exact dominance on (latency down, accuracy up, cost down) */
    for (uint32_t c = 0; c < C; c++) {
        if (!alive[c]) continue;
        uint32_t l = m->lat[(size_t)t * C + c];
        double a = m->acc[(size_t)t * m->V + variant_of(m, c)];
        int32_t k = cost[(size_t)t * C + c];
        keep[c] = 1;
        for (uint32_t o = 0; o < C && keep[c]; o++) {
            if (o == c || !alive[o]) continue;
            uint32_t l2 = m->lat[(size_t)t * C + o];
            double a2 = m->acc[(size_t)t * m->V + variant_of(m, o)];
            int32_t k2 = cost[(size_t)t * C + o];
            if (l2 <= l && a2 >= a && k2 <= k) {
                int strict = (l2 < l) || (a2 > a) || (k2 < k);
                if (strict || o < c) keep[c] = 0;
            }
        }
    }
    uint32_t left = 0;
    for (uint32_t c = 0; c < C; c++) left += keep[c];

    /* (c) cap thinning, variant by variant */
    if (left > cap) {
        *truncated = 1;
        uint32_t quota = cap / m->V;
        for (uint32_t v = 0; v < m->V; v++) {
            uint32_t n = 0;
            for (uint32_t c = 0; c < C; c++)
                if (keep[c] && variant_of(m, c) == v) { order[n].lat = m->lat[(size_t)t * C + c]; order[n].c = c; n++; }
            if (n <= quota) continue;
            qsort(order, n, sizeof(lat_c), cmp_lat_c);
            for (uint32_t i = 0; i < n; i++) keep[order[i].c] = 0;
            for (uint32_t j = 0; j < quota; j++) {
                uint32_t rank = (uint32_t)(((uint64_t)j * (n - 1)) / (quota - 1));
                keep[order[rank].c] = 1;
            }
        }
    }
    uint32_t k = 0;
    for (uint32_t c = 0; c < C; c++) if (keep[c]) ids[k++] = (uint16_t)c;
    *K = k;
    free(alive); free(keep); free(order);
    return ORC_OK;
}

int orc_pruned(const orc_model *m, uint32_t demand_mrps, uint32_t slo_latency_us, uint32_t cap,
               uint32_t task, uint16_t *ids, uint32_t *K, uint32_t *truncated)
{
    if (task >= m->T || m->fac || m->mix) return ORC_E_ARG;
    size_t n = (size_t)m->T * m->C;
    uint32_t *rep = (uint32_t *)malloc(n * sizeof *rep);
    int32_t *cost = (int32_t *)malloc(n * sizeof *cost);
    if (!rep || !cost) { free(rep); free(cost); return ORC_E_MEM; }
    int rc = orc_cost_table(m, demand_mrps, rep, cost);
    if (rc == ORC_OK) rc = prune_task(m, cost, slo_latency_us, cap, NULL, task, ids, K, truncated);
    free(rep); free(cost);
    return rc;
}

/* ---- mixtures of two tuples (Eq. 2, 6, 7, 9, 10) ------------------------------ */
#define ORC_MIX_MAX_REPLICAS 65535u

/* One way to run a task: m1 replicas of tuple c1 and, if c2 != 0xFFFF, m2 of tuple c2. */
typedef struct {
    uint16_t c1, c2;
    uint32_t m1, m2;
    uint32_t lat;       /* Eq. 2: the slower of the active tuples */
    int32_t cost;       /* Eq. 7 */
    double acc;         /* Eq. 10 */
    uint64_t id;        /* order of the options: c for a single tuple, C + (c1*C + c2)*65536 + m1 for a mixture */
} option_t;

int orc_set_mixtures(orc_model *m, int on)
{
    if (!m) return ORC_E_ARG;
    m->mix = on != 0;
    return ORC_OK;
}

typedef struct { option_t *v; size_t n, room; } option_list;

static int option_push(option_list *l, const option_t *o)
{
    if (l->n == l->room) {
        size_t room = l->room ? 2 * l->room : 1024;
        option_t *v = (option_t *)realloc(l->v, room * sizeof *v);
        if (!v) return ORC_E_MEM;
        l->v = v; l->room = room;
    }
    l->v[l->n++] = *o;
    return ORC_OK;
}

/*
 * Every option of task t under a demand of `need` micro-requests/s, in ascending id.
 * Single tuples: every allowed choice with its replicas.  Mixtures: allowed c1 < c2 with
 * m1, m2 >= 1 that carry the demand together while neither (m1-1, m2) nor (m1, m2-1) does.
 * An option that alone costs more than S_avail is left out (Eq. 8: it fits no assignment).
 */
static int all_options(const orc_model *m, const int32_t *cost, const uint32_t *rep, uint32_t slo_latency_us,
                       uint64_t need, uint32_t t, option_list *out)
{
    const uint32_t C = m->C;
    for (uint32_t c = 0; c < C; c++) {
        if (!allowed(m, cost, slo_latency_us, t, c, NULL)) continue;
        if (m->capacity != 0 && (uint32_t)cost[(size_t)t * C + c] > m->capacity) continue;
        option_t o;
        o.c1 = (uint16_t)c; o.c2 = 0xFFFF; o.m1 = rep[(size_t)t * C + c]; o.m2 = 0;
        o.lat = m->lat[(size_t)t * C + c]; o.cost = cost[(size_t)t * C + c];
        o.acc = m->acc[(size_t)t * m->V + variant_of(m, c)]; o.id = c;
        int rc = option_push(out, &o);
        if (rc) return rc;
    }
    for (uint32_t c1 = 0; c1 < C; c1++) {
        if (!allowed(m, cost, slo_latency_us, t, c1, NULL)) continue;
        const uint64_t h1 = 1000ull * m->thr[(size_t)t * C + c1];
        const uint64_t alone = need / h1 + (need % h1 != 0);          /* replicas of c1 without help */
        if (alone < 2) continue;
        if (alone - 1 > ORC_MIX_MAX_REPLICAS) return ORC_E_RANGE;
        for (uint32_t c2 = c1 + 1; c2 < C; c2++) {
            if (!allowed(m, cost, slo_latency_us, t, c2, NULL)) continue;
            const uint64_t h2 = 1000ull * m->thr[(size_t)t * C + c2];
            for (uint64_t m1 = 1; m1 < alone; m1++) {
                const uint64_t rest = need - m1 * h1;                  /* > 0 */
                const uint64_t m2 = rest / h2 + (rest % h2 != 0);
                if ((m1 - 1) * h1 + m2 * h2 >= need) continue;         /* one replica of c1 too many */
                const unsigned __int128 k = (unsigned __int128)m1 * m->units[part_of(m, c1)] +
                                            (unsigned __int128)m2 * m->units[part_of(m, c2)];
                if (m->capacity != 0 && k > m->capacity) continue;
                if (m2 > ORC_MIX_MAX_REPLICAS || k > 0x7FFFFFFFull) return ORC_E_RANGE;
                option_t o;
                o.c1 = (uint16_t)c1; o.c2 = (uint16_t)c2; o.m1 = (uint32_t)m1; o.m2 = (uint32_t)m2;
                const uint32_t l1 = m->lat[(size_t)t * C + c1], l2 = m->lat[(size_t)t * C + c2];
                o.lat = l1 > l2 ? l1 : l2;
                o.cost = (int32_t)k;
                /* Eq. 9, 10: weights are the total throughputs of the two instance types */
                const double w1 = (double)(m1 * h1), w2 = (double)(m2 * h2);
                const double a1 = m->acc[(size_t)t * m->V + variant_of(m, c1)];
                const double a2 = m->acc[(size_t)t * m->V + variant_of(m, c2)];
                const double p1 = w1 * a1, p2 = w2 * a2;
                o.acc = (p1 + p2) / (w1 + w2);
                o.id = C + ((uint64_t)c1 * C + c2) * 65536u + m1;
                int rc = option_push(out, &o);
                if (rc) return rc;
            }
        }
    }
    return ORC_OK;
}

typedef struct { uint32_t lat; double acc; uint64_t id; size_t at; } opt_key;
static int cmp_lat_id(const void *a, const void *b)
{
    const opt_key *x = (const opt_key *)a, *y = (const opt_key *)b;
    if (x->lat != y->lat) return x->lat < y->lat ? -1 : 1;
    return x->id < y->id ? -1 : (x->id > y->id);
}
static int cmp_acc_id(const void *a, const void *b)
{
    const opt_key *x = (const opt_key *)a, *y = (const opt_key *)b;
    if (x->acc != y->acc) return x->acc < y->acc ? -1 : 1;
    return x->id < y->id ? -1 : (x->id > y->id);
}

/*
 * Surviving options of one task in mixture mode, ascending id.  cap == 0: all of them.
 * Otherwise the steps of the single-tuple prune on options: (a) latency filter, (b) exact
 * dominance on (latency, accuracy, cost), equal triples keep the lowest id, (c) if more than
 * cap remain, a grid over latency and accuracy: the n survivors, ordered by (latency, id),
 * are cut into bands = floor(sqrt(cap)) runs (the one at rank r goes to band
 * floor(r*bands/n)); a band of more than per = floor(cap/bands) options keeps those at ranks
 * floor(j*(size-1)/(per-1)), j < per, of its order by (accuracy, id): always its least
 * accurate option, which on a front of non-dominated options is a cheap one, and its most
 * accurate one.
 */
static int prune_options(const orc_model *m, uint32_t slo_latency_us, uint32_t cap, uint32_t t,
                         option_list *all, uint32_t *truncated)
{
    *truncated = 0;
    if (cap == 0) return ORC_OK;
    if (cap < 2) return ORC_E_ARG;
    const uint32_t C = m->C;
    uint64_t lo[ORC_MAX_TASKS];
    for (uint32_t u = 0; u < m->T; u++) {
        uint32_t best = m->lat[(size_t)u * C];
        for (uint32_t c = 1; c < C; c++) if (m->lat[(size_t)u * C + c] < best) best = m->lat[(size_t)u * C + c];
        lo[u] = best;
    }
    uint64_t through = 0;
    for (int k = 0; k < m->npaths; k++) {
        int on = 0; uint64_t sum = 0;
        for (int i = 0; i < m->plen[k]; i++) {
            uint32_t u = (uint32_t)m->pnode[(size_t)k * m->T + i];
            if (u == t) on = 1; else sum += lo[u];
        }
        if (on && sum > through) through = sum;
    }
    size_t n = 0;
    for (size_t i = 0; i < all->n; i++)                                 /* (a) */
        if ((uint64_t)m->q * ((uint64_t)all->v[i].lat + through) <= slo_latency_us) all->v[n++] = all->v[i];
    all->n = n;
    uint8_t *keep = (uint8_t *)malloc(n ? n : 1);
    if (!keep) return ORC_E_MEM;
    for (size_t i = 0; i < n; i++) {                                    /* (b) */
        const option_t *x = &all->v[i];
        keep[i] = 1;
        for (size_t j = 0; j < n && keep[i]; j++) {
            if (j == i) continue;
            const option_t *y = &all->v[j];
            if (y->lat <= x->lat && y->acc >= x->acc && y->cost <= x->cost) {
                int strict = (y->lat < x->lat) || (y->acc > x->acc) || (y->cost < x->cost);
                if (strict || y->id < x->id) keep[i] = 0;
            }
        }
    }
    size_t left = 0;
    for (size_t i = 0; i < n; i++) if (keep[i]) all->v[left++] = all->v[i];
    all->n = left;
    free(keep);
    if (left > cap) {                                                   /* (c) */
        *truncated = 1;
        uint32_t bands = 1;
        while ((uint64_t)(bands + 1) * (bands + 1) <= cap) bands++;
        const uint32_t per = cap / bands;
        opt_key *order = (opt_key *)malloc(left * sizeof *order);
        option_t *kept = (option_t *)malloc((size_t)cap * sizeof *kept);
        if (!order || !kept) { free(order); free(kept); return ORC_E_MEM; }
        for (size_t i = 0; i < left; i++) {
            order[i].lat = all->v[i].lat; order[i].acc = all->v[i].acc; order[i].id = all->v[i].id; order[i].at = i;
        }
        qsort(order, left, sizeof *order, cmp_lat_id);
        size_t nk = 0, lo = 0;
        for (uint32_t b = 0; b < bands; b++) {
            size_t hi = lo;                                             /* ranks r with floor(r*bands/left) == b */
            while (hi < left && (uint64_t)hi * bands / left == b) hi++;
            const size_t size = hi - lo;
            qsort(order + lo, size, sizeof *order, cmp_acc_id);
            if (size <= per)
                for (size_t r = 0; r < size; r++) kept[nk++] = all->v[order[lo + r].at];
            else
                for (uint32_t j = 0; j < per; j++) kept[nk++] = all->v[order[lo + ((uint64_t)j * (size - 1)) / (per - 1)].at];
            lo = hi;
        }
        /* back to ascending id (insertion sort, cap is small) */
        for (size_t j = 1; j < nk; j++) {
            option_t x = kept[j]; size_t k = j;
            while (k > 0 && kept[k - 1].id > x.id) { kept[k] = kept[k - 1]; k--; }
            kept[k] = x;
        }
        memcpy(all->v, kept, nk * sizeof *kept);
        all->n = nk;
        free(order); free(kept);
    }
    return ORC_OK;
}

/* ---- one level: tables + lists --------------------------------------------- */
typedef struct {
    const orc_model *m;
    uint32_t *rep; int32_t *cost;
    uint16_t *ids;            /* [T][C] surviving choices */
    option_t *opt[ORC_MAX_TASKS];   /* mixture mode: surviving options per task instead of ids */
    uint32_t K[ORC_MAX_TASKS];
    uint32_t truncated;
    uint64_t space;           /* prod K_t (0 if some K_t = 0) */
    uint32_t slo_l; double slo_a;
    uint32_t demand;
} level_t;

static void level_free(level_t *L)
{
    free(L->rep); free(L->cost); free(L->ids);
    for (int t = 0; t < ORC_MAX_TASKS; t++) free(L->opt[t]);
}

/* only: NULL, or per task the one variant it is held to (UINT32_MAX = free); the demands
   then follow the per-variant factors with every held task on its variant */
static int level_init_held(level_t *L, const orc_model *m, uint32_t demand, uint32_t slo_l, double slo_a,
                           uint32_t cap, const uint32_t *only)
{
    memset(L, 0, sizeof *L);
    size_t n = (size_t)m->T * m->C;
    L->m = m; L->slo_l = slo_l; L->slo_a = slo_a; L->demand = demand;
    L->rep = (uint32_t *)malloc(n * sizeof(uint32_t));
    L->cost = (int32_t *)malloc(n * sizeof(int32_t));
    L->ids = (uint16_t *)malloc(n * sizeof(uint16_t));
    if (!L->rep || !L->cost || !L->ids) { level_free(L); return ORC_E_MEM; }
    int rc;
    if (m->fac) {
        if (!only || !m->space_t) { level_free(L); return ORC_E_ARG; }
        uint32_t v[ORC_MAX_TASKS]; uint64_t need[ORC_MAX_TASKS];
        for (uint32_t t = 0; t < m->T; t++) v[t] = only[t] == UINT32_MAX ? 0 : only[t];
        rc = demand_flow(m, demand, v, need);
        if (!rc) rc = cost_table_of(m, need, L->rep, L->cost);
    } else rc = orc_cost_table(m, demand, L->rep, L->cost);
    if (rc) { level_free(L); return rc; }
    if (m->mix && (m->fac || !m->space_t)) { level_free(L); return ORC_E_ARG; }
    unsigned __int128 space = 1;
    for (uint32_t t = 0; t < m->T; t++) {
        uint32_t tr = 0;
        if (m->mix) {
            option_list all = {0};
            rc = all_options(m, L->cost, L->rep, slo_l, (uint64_t)demand * m->mult[t], t, &all);
            if (!rc) rc = prune_options(m, slo_l, cap, t, &all, &tr);
            if (!rc && all.n > 0xFFFFFFFFull) rc = ORC_E_RANGE;
            L->opt[t] = all.v; L->K[t] = (uint32_t)all.n;
        } else
        rc = prune_task(m, L->cost, slo_l, cap, only, t, L->ids + (size_t)t * m->C, &L->K[t], &tr);
        if (rc) { level_free(L); return rc; }
        L->truncated |= tr;
        space *= L->K[t];
        if (space >> 63) { level_free(L); return ORC_E_RANGE; }
    }
    L->space = (uint64_t)space;
    return ORC_OK;
}

static int level_init(level_t *L, const orc_model *m, uint32_t demand, uint32_t slo_l, double slo_a, uint32_t cap)
{
    if (m->fac) return ORC_E_ARG;     /* with per-variant factors a level is a union of held levels */
    return level_init_held(L, m, demand, slo_l, slo_a, cap, NULL);
}

typedef struct { uint32_t lat; int32_t cost; double acc; uint8_t mask; } score_t;

/* mixture mode: candidate i picks one surviving option per task; c_out[t] = its digits */
static score_t score_options(const level_t *L, uint64_t i, uint32_t *c_out)
{
    const orc_model *m = L->m;
    const option_t *o[ORC_MAX_TASKS];
    double a_task[ORC_MAX_TASKS];
    for (uint32_t t = 0; t < m->T; t++) {
        uint32_t d = (uint32_t)(i % L->K[t]);
        i /= L->K[t];
        o[t] = &L->opt[t][d];
        a_task[t] = o[t]->acc;
        if (c_out) c_out[t] = d;
    }
    uint64_t worst = 0;                                    /* Eq. 2, 3 */
    for (int k = 0; k < m->npaths; k++) {
        uint64_t s = 0;
        for (int j = 0; j < m->plen[k]; j++) s += o[m->pnode[(size_t)k * m->T + j]]->lat;
        if (s > worst) worst = s;
    }
    uint64_t lat = (uint64_t)m->q * worst;
    int64_t cost = 0;                                      /* Eq. 7, 8 */
    for (uint32_t t = 0; t < m->T; t++) cost += o[t]->cost;
    double a = raw_accuracy_of(m, a_task) / m->amax;       /* Eq. 10-13 */
    score_t s;
    s.lat = lat > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)lat;
    s.cost = cost > 0x7FFFFFFF ? 0x7FFFFFFF : (int32_t)cost;
    s.acc = a;
    s.mask = 0;
    if (lat <= L->slo_l) s.mask |= 1;
    if (a >= L->slo_a) s.mask |= 2;
    if (m->capacity == 0 || cost <= (int64_t)m->capacity) s.mask |= 4;
    return s;
}

/* score candidate i of the searched space; c_out[t] = its choice ids */
static score_t score(const level_t *L, uint64_t i, uint32_t *c_out)
{
    const orc_model *m = L->m;
    if (m->mix) return score_options(L, i, c_out);
    uint32_t c[ORC_MAX_TASKS], v[ORC_MAX_TASKS];
    for (uint32_t t = 0; t < m->T; t++) {
        uint32_t d = (uint32_t)(i % L->K[t]);
        i /= L->K[t];
        c[t] = L->ids[(size_t)t * m->C + d];
        v[t] = variant_of(m, c[t]);
        if (c_out) c_out[t] = c[t];
    }
    /* Eq. 3: slowest path, doubled (q) for queueing */
    uint64_t worst = 0;
    for (int k = 0; k < m->npaths; k++) {
        uint64_t s = 0;
        for (int j = 0; j < m->plen[k]; j++) {
            int t = m->pnode[(size_t)k * m->T + j];
            s += m->lat[(size_t)t * m->C + c[t]];
        }
        if (s > worst) worst = s;
    }
    uint64_t lat = (uint64_t)m->q * worst;
    /* Eq. 7, 8; with per-variant factors the demands are those of this candidate's own variants */
    int64_t cost = 0;
    if (m->fac) {
        uint64_t need[ORC_MAX_TASKS];
        if (demand_flow(m, L->demand, v, need)) cost = 0x7FFFFFFF;
        else
            for (uint32_t t = 0; t < m->T; t++) {
                uint32_t r; int32_t k;
                if (replicas_and_cost(m, need[t], t, c[t], &r, &k)) k = 0x7FFFFFFF;
                cost += k;
            }
    } else
        for (uint32_t t = 0; t < m->T; t++) cost += L->cost[(size_t)t * m->C + c[t]];
    /* Eq. 11-13 */
    double a = raw_accuracy(m, v) / m->amax;
    score_t s;
    s.lat = lat > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)lat;
    s.cost = cost > 0x7FFFFFFF ? 0x7FFFFFFF : (int32_t)cost;
    s.acc = a;
    s.mask = 0;
    if (lat <= L->slo_l) s.mask |= 1;
    if (a >= L->slo_a) s.mask |= 2;
    if (m->capacity == 0 || cost <= (int64_t)m->capacity) s.mask |= 4;
    return s;
}

static void result_clear(orc_result *r, const level_t *L)
{
    memset(r, 0, sizeof *r);
    r->index = UINT64_MAX; r->full_index = UINT64_MAX; r->cost = INT32_MAX;
    r->evaluated = L ? L->space : 0;
    r->flags = L ? L->truncated : 0;
}

static void result_fill(orc_result *r, const level_t *L, uint64_t i)
{
    const orc_model *m = L->m;
    uint32_t c[ORC_MAX_TASKS];
    score_t s = score(L, i, c);
    r->index = i; r->feasible = 1;
    r->accuracy = s.acc; r->latency_us = s.lat; r->cost = s.cost;
    r->objective = m->alpha * s.acc - m->beta * (double)s.cost;
    if (m->mix) {                                          /* c[] holds digits */
        for (uint32_t t = 0; t < m->T; t++) {
            const option_t *o = &L->opt[t][c[t]];
            r->choice[t] = o->c1; r->choice2[t] = o->c2;
            r->replicas[t] = o->m1; r->replicas2[t] = o->m2;
        }
        r->full_index = UINT64_MAX;                        /* the options have no fixed-size full space */
        return;
    }
    for (uint32_t t = 0; t < m->T; t++) r->choice2[t] = 0xFFFF;
    uint64_t need[ORC_MAX_TASKS]; uint32_t v[ORC_MAX_TASKS] = {0};
    for (uint32_t t = 0; t < m->T; t++) v[t] = variant_of(m, c[t]);
    int flow_ok = m->fac && demand_flow(m, L->demand, v, need) == ORC_OK;
    for (uint32_t t = 0; t < m->T; t++) {
        r->choice[t] = (uint16_t)c[t];
        r->replicas[t] = L->rep[(size_t)t * m->C + c[t]];
        if (m->fac) {
            int32_t k;
            if (!flow_ok || replicas_and_cost(m, need[t], t, c[t], &r->replicas[t], &k)) r->replicas[t] = 0;
        }
    }
    /* sum_t c_t * C^t by Horner from the last task; it only grows */
    unsigned __int128 full = 0;
    int over = 0;
    for (uint32_t t = m->T; t-- > 0;) {
        full = full * m->C + c[t];
        if (full >= (unsigned __int128)UINT64_MAX) { over = 1; break; }
    }
    r->full_index = over ? UINT64_MAX : (uint64_t)full;
}

/* Is candidate (obj, cost) at a higher index better than the best so far?  Candidates are
   visited in ascending index, so equality never replaces. */
static inline int better(const orc_model *m, double obj, int32_t cost, double bobj, int32_t bcost)
{
    if (m->objective == 0) return cost < bcost;
    return obj > bobj || (obj == bobj && cost < bcost);
}

/* best feasible candidate of [lo, hi): cheapest (mode 0) or largest objective (mode 1);
   remaining ties go to the lowest index */
static void argmin_range(const level_t *L, uint64_t lo, uint64_t hi, int threads,
                         int *found, int32_t *best_cost, uint64_t *best_idx)
{
    const orc_model *m = L->m;
    if (threads < 1) threads = 1;
    int32_t bc[256]; uint64_t bi[256]; int bf[256]; double bo[256];
    if (threads > 256) threads = 256;
    for (int k = 0; k < threads; k++) { bf[k] = 0; bc[k] = INT32_MAX; bi[k] = UINT64_MAX; bo[k] = 0.0; }
    uint64_t span = hi > lo ? hi - lo : 0;
#ifdef _OPENMP
#pragma omp parallel for num_threads(threads) schedule(static, 1)
#endif
    for (int k = 0; k < threads; k++) {
        uint64_t a = lo + (uint64_t)(((unsigned __int128)span * (unsigned)k) / (unsigned)threads);
        uint64_t b = lo + (uint64_t)(((unsigned __int128)span * (unsigned)(k + 1)) / (unsigned)threads);
        for (uint64_t i = a; i < b; i++) {
            score_t s = score(L, i, NULL);
            if (s.mask != 7) continue;
            double obj = m->alpha * s.acc - m->beta * (double)s.cost;
            if (!bf[k] || better(m, obj, s.cost, bo[k], bc[k])) { bf[k] = 1; bc[k] = s.cost; bi[k] = i; bo[k] = obj; }
        }
    }
    *found = 0; *best_cost = INT32_MAX; *best_idx = UINT64_MAX;
    double best_obj = 0.0;
    for (int k = 0; k < threads; k++)   /* chunks are in ascending index order */
        if (bf[k] && (!*found || better(m, bo[k], bc[k], best_obj, *best_cost))) {
            *found = 1; *best_cost = bc[k]; *best_idx = bi[k]; best_obj = bo[k];
        }
}

/*
 * One level with per-variant factors.  The tasks whose variant changes a downstream demand
 * are held to one variant each, in every combination (lowest task id = fastest digit); with
 * them held, every task's demand is fixed, so its cost table, its pruned list and the search
 * of the product of the lists are those of the fixed-factor case.  The level's result is the
 * best over the combinations: cheapest (or largest objective, then cheapest), then lowest
 * full_index; `index` repeats full_index, `evaluated` and `flags` add up over the combinations.
 * If other_obj is given it receives the best objective among feasible candidates whose
 * variants differ from the winner's (-1e300 if none).
 */
static int search_held(const orc_model *m, uint32_t demand, uint32_t slo_l, double slo_a, uint32_t cap,
                       int threads, orc_result *out, double *other_obj)
{
    uint32_t inf[ORC_MAX_TASKS], only[ORC_MAX_TASKS], digit[ORC_MAX_TASKS] = {0};
    const uint32_t n_inf = influencers(m, inf);
    double combos = 1.0;
    for (uint32_t i = 0; i < n_inf; i++) combos *= (double)m->V;
    if (combos > 1048576.0) return ORC_E_RANGE;
    result_clear(out, NULL);
    for (int pass = 0; pass < (other_obj ? 2 : 1); pass++) {
        if (pass == 1) { *other_obj = -1e300; if (!out->feasible) break; }
        memset(digit, 0, sizeof digit);
        for (;;) {
            for (uint32_t t = 0; t < m->T; t++) only[t] = UINT32_MAX;
            for (uint32_t i = 0; i < n_inf; i++) only[inf[i]] = digit[i];
            level_t L;
            int rc = level_init_held(&L, m, demand, slo_l, slo_a, cap, only);
            if (rc) return rc;
            if (pass == 0) {
                out->evaluated += L.space; out->flags |= L.truncated;
                int found; int32_t bc; uint64_t bi;
                argmin_range(&L, 0, L.space, threads, &found, &bc, &bi);
                if (found) {
                    orc_result r;
                    result_clear(&r, &L);
                    result_fill(&r, &L, bi);
                    if (r.full_index == UINT64_MAX) { level_free(&L); return ORC_E_RANGE; }
                    int take = !out->feasible;
                    if (!take) {
                        if (m->objective && r.objective != out->objective) take = r.objective > out->objective;
                        else if (r.cost != out->cost) take = r.cost < out->cost;
                        else take = r.full_index < out->full_index;
                    }
                    if (take) {
                        uint64_t ev = out->evaluated; uint32_t fl = out->flags;
                        *out = r; out->index = r.full_index; out->evaluated = ev; out->flags = fl;
                    }
                }
            } else {
                uint32_t c[ORC_MAX_TASKS];
                for (uint64_t i = 0; i < L.space; i++) {
                    score_t sc = score(&L, i, c);
                    if (sc.mask != 7) continue;
                    int same = 1;
                    for (uint32_t t = 0; t < m->T; t++)
                        if (variant_of(m, c[t]) != variant_of(m, out->choice[t])) same = 0;
                    if (same) continue;
                    double obj = m->alpha * sc.acc - m->beta * (double)sc.cost;
                    if (obj > *other_obj) *other_obj = obj;
                }
            }
            level_free(&L);
            uint32_t i = 0;
            while (i < n_inf && ++digit[i] == m->V) digit[i++] = 0;
            if (i == n_inf) break;
        }
    }
    return ORC_OK;
}

/*
 * Search every demand level.  results[n_levels]; best_level/max_demand: the
 * feasible level with the largest demand (first position on equal demands),
 * -1 / 0 when none is feasible.
 */
int orc_search(const orc_model *m, const uint32_t *demand_mrps, uint32_t n_levels,
               uint32_t slo_latency_us, double slo_accuracy, uint32_t cap, int threads,
               orc_result *results, int32_t *best_level, uint32_t *max_demand)
{
    if (!m || !demand_mrps || !results) return ORC_E_ARG;
    int32_t bl = -1; uint32_t md = 0;
    for (uint32_t l = 0; l < n_levels; l++) {
        if (demand_mrps[l] == 0) return ORC_E_ARG;
        if (m->fac) {
            int rc = search_held(m, demand_mrps[l], slo_latency_us, slo_accuracy, cap, threads, &results[l], NULL);
            if (rc) return rc;
            if (results[l].feasible && (bl < 0 || demand_mrps[l] > md)) { bl = (int32_t)l; md = demand_mrps[l]; }
            continue;
        }
        level_t L;
        int rc = level_init(&L, m, demand_mrps[l], slo_latency_us, slo_accuracy, cap);
        if (rc) return rc;
        result_clear(&results[l], &L);
        int found; int32_t bc; uint64_t bi;
        argmin_range(&L, 0, L.space, threads, &found, &bc, &bi);
        if (found) {
            result_fill(&results[l], &L, bi);
            if (bl < 0 || demand_mrps[l] > md) { bl = (int32_t)l; md = demand_mrps[l]; }
        }
        level_free(&L);
    }
    if (best_level) *best_level = bl;
    if (max_demand) *max_demand = md;
    return ORC_OK;
}

/* arg-min restricted to candidate indices [lo, hi) of one level */
int orc_search_range(const orc_model *m, uint32_t demand_mrps, uint32_t slo_latency_us,
                     double slo_accuracy, uint32_t cap, uint64_t lo, uint64_t hi, int threads,
                     orc_result *result)
{
    level_t L;
    int rc = level_init(&L, m, demand_mrps, slo_latency_us, slo_accuracy, cap);
    if (rc) return rc;
    if (hi > L.space) hi = L.space;
    result_clear(result, &L);
    int found; int32_t bc; uint64_t bi;
    argmin_range(&L, lo, hi, threads, &found, &bc, &bi);
    if (found) result_fill(result, &L, bi);
    level_free(&L);
    return ORC_OK;
}

/* K_t of every task and the size of the searched space at one level */
int orc_space(const orc_model *m, uint32_t demand_mrps, uint32_t slo_latency_us, uint32_t cap,
              uint32_t *K, uint64_t *space, uint32_t *truncated)
{
    level_t L;
    int rc = level_init(&L, m, demand_mrps, slo_latency_us, 0.0, cap);
    if (rc) return rc;
    for (uint32_t t = 0; t < m->T; t++) K[t] = L.K[t];
    *space = L.space; *truncated = L.truncated;
    level_free(&L);
    return ORC_OK;
}

/* score explicit candidates of one level's searched space */
int orc_eval(const orc_model *m, uint32_t demand_mrps, uint32_t slo_latency_us, double slo_accuracy,
             uint32_t cap, const uint64_t *index, uint32_t n,
             uint32_t *latency_us, uint32_t *replicas, int32_t *cost, double *accuracy, uint8_t *mask)
{
    if (m->mix) return ORC_E_ARG;
    level_t L;
    int rc = level_init(&L, m, demand_mrps, slo_latency_us, slo_accuracy, cap);
    if (rc) return rc;
    for (uint32_t k = 0; k < n; k++) {
        if (index[k] >= L.space) { level_free(&L); return ORC_E_RANGE; }
        uint32_t c[ORC_MAX_TASKS];
        score_t s = score(&L, index[k], c);
        latency_us[k] = s.lat; cost[k] = s.cost; accuracy[k] = s.acc; mask[k] = s.mask;
        for (uint32_t t = 0; t < m->T; t++) replicas[(size_t)k * m->T + t] = L.rep[(size_t)t * m->C + c[t]];
    }
    level_free(&L);
    return ORC_OK;
}

/* normalised accuracy of a choice of variants (used by the input guard band) */
double orc_accuracy_of_variants(const orc_model *m, const uint32_t *variant)
{
    return raw_accuracy(m, variant) / m->amax;
}

/* smallest |A_obj - slo_accuracy| over all V^T combinations of variants */
double orc_accuracy_margin(const orc_model *m, double slo_accuracy)
{
    uint32_t v[ORC_MAX_TASKS] = {0};
    double best = 1e300;
    for (;;) {
        double d = raw_accuracy(m, v) / m->amax - slo_accuracy;
        if (d < 0) d = -d;
        if (d < best) best = d;
        uint32_t t = 0;
        while (t < m->T && ++v[t] == m->V) v[t++] = 0;
        if (t == m->T) break;
    }
    return best;
}

/*
 * Objective mode only: gap between the winner's objective and the best objective of any
 * feasible candidate that uses a different combination of variants (mixture mode: of per-task
 * accuracies; 1e300 if there is none, -1 if the level is infeasible).  Candidates with the winner's variants have exactly
 * its accuracy, so their order is decided by integer cost; only this gap is exposed to
 * floating-point rounding, and tests skip inputs where it is tiny.
 */
int orc_objective_margin(const orc_model *m, uint32_t demand_mrps, uint32_t slo_latency_us,
                         double slo_accuracy, uint32_t cap, double *margin)
{
    if (m->fac) {
        orc_result r; double other;
        int rc = search_held(m, demand_mrps, slo_latency_us, slo_accuracy, cap, 1, &r, &other);
        if (rc) return rc;
        *margin = !r.feasible ? -1.0 : other == -1e300 ? 1e300 : r.objective - other;
        return ORC_OK;
    }
    level_t L;
    int rc = level_init(&L, m, demand_mrps, slo_latency_us, slo_accuracy, cap);
    if (rc) return rc;
    int found; int32_t bc; uint64_t bi;
    argmin_range(&L, 0, L.space, 1, &found, &bc, &bi);
    *margin = -1.0;
    if (found) {
        uint32_t cw[ORC_MAX_TASKS], c[ORC_MAX_TASKS];
        score_t w = score(&L, bi, cw);
        double wobj = m->alpha * w.acc - m->beta * (double)w.cost, other = -1e300;
        for (uint64_t i = 0; i < L.space; i++) {
            score_t s = score(&L, i, c);
            if (s.mask != 7) continue;
            int same = 1;
            for (uint32_t t = 0; t < m->T; t++) {
                if (m->mix) {       /* c[] are digits: the same per-task accuracies give exactly the same A_obj */
                    if (L.opt[t][c[t]].acc != L.opt[t][cw[t]].acc) same = 0;
                } else if (variant_of(m, c[t]) != variant_of(m, cw[t])) same = 0;
            }
            if (same) continue;
            double obj = m->alpha * s.acc - m->beta * (double)s.cost;
            if (obj > other) other = obj;
        }
        *margin = other == -1e300 ? 1e300 : wobj - other;
    }
    level_free(&L);
    return ORC_OK;
}

/*
 * Mixture mode: the surviving options of one task at one level, ascending id; at most room
 * are written, *n is their number.
 */
int orc_options(const orc_model *m, uint32_t demand_mrps, uint32_t slo_latency_us, uint32_t cap, uint32_t task,
                uint32_t room, uint16_t *c1, uint16_t *c2, uint32_t *m1, uint32_t *m2,
                uint32_t *latency_us, int32_t *cost, double *accuracy, uint32_t *n, uint32_t *truncated)
{
    if (!m->mix || task >= m->T) return ORC_E_ARG;
    level_t L;
    int rc = level_init(&L, m, demand_mrps, slo_latency_us, 0.0, cap);
    if (rc) return rc;
    *n = L.K[task]; *truncated = L.truncated;
    for (uint32_t i = 0; i < L.K[task] && i < room; i++) {
        const option_t *o = &L.opt[task][i];
        c1[i] = o->c1; c2[i] = o->c2; m1[i] = o->m1; m2[i] = o->m2;
        latency_us[i] = o->lat; cost[i] = o->cost; accuracy[i] = o->acc;
    }
    level_free(&L);
    return ORC_OK;
}

/* Mixture mode: smallest |A_obj - slo_accuracy| over the searched space of one level (tests
   keep away from levels where rounding could flip a candidate's feasibility); 1e300 if empty */
int orc_mixture_margin(const orc_model *m, uint32_t demand_mrps, uint32_t slo_latency_us, double slo_accuracy,
                       uint32_t cap, double *margin)
{
    if (!m->mix) return ORC_E_ARG;
    level_t L;
    int rc = level_init(&L, m, demand_mrps, slo_latency_us, slo_accuracy, cap);
    if (rc) return rc;
    double best = 1e300;
    for (uint64_t i = 0; i < L.space; i++) {
        double d = score(&L, i, NULL).acc - slo_accuracy;
        if (d < 0) d = -d;
        if (d < best) best = d;
    }
    *margin = best;
    level_free(&L);
    return ORC_OK;
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
